// Internal launch interface between the kernel files and the module / C-ABI layer.
// Every function enqueues on `s` and returns without synchronising.  `quota` is the CU
// count the persistent grid is sized for.
#pragma once
#include "common.h"

// ------------------------------------------------------------------------------ GEMM
// C[M,N] = op(A) op(B) (+ bias[N]) (+ R[M,N]), fp32 accumulation in ascending k.
//   a_kc: A is stored [M,K] (K contiguous) else [K,M];  b_kc: B is stored [N,K] else [K,N].
// fprop  Y = X W      : A = X  [T,k] a_kc=1, B = W  [k,n] b_kc=0
// dgrad  dX = dY W^T  : A = dY [T,n] a_kc=1, B = W  [k,n] b_kc=1 (contraction over n)
// wgrad  dW = X^T dY  : A = X  [T,k] a_kc=0, B = dY [T,n] b_kc=0 (contraction over T)
mosaic_status launch_gemm(hipStream_t s, int quota, int dtype, bool a_kc, bool b_kc,
                          int64_t M, int64_t N, int64_t K, const void* A, int64_t lda,
                          const void* B, int64_t ldb, void* C, int64_t ldc,
                          const void* bias, const void* R, void* splitk_scratch = nullptr);
// Z[T,n] = X[T,k] W[k,n] (+ bias[n]) and A = act(Z): GELU / tanh GELU give A[T,n]; SwiGLU reads Z
// as [gate | up] halves and gives A[T,n/2] = silu(gate) * up.  Where the bf16 matrix-core kernel
// takes the product, the activation is applied in its epilogue (same bits as the separate pass);
// otherwise the elementwise kernel follows the product.
mosaic_status launch_linear_act_fwd(hipStream_t s, int quota, int dtype, int act, int64_t T, int64_t k, int64_t n,
                                    const void* X, const void* W, const void* bias, void* Z, void* A);
// Bytes of fp32 scratch the weight-gradient form wants for a deterministic split of a long
// contraction over few output tiles (0 when no split is used for this shape).
size_t gemm_splitk_scratch_bytes(int64_t M, int64_t N, int64_t K);

// ------------------------------------------------------------------------- attention
// packed rows [q (H heads) | k (Hkv heads) | v (Hkv heads)]; Hkv divides H; query head t
// attends to key/value head t / (H/Hkv)
mosaic_status launch_attention_fwd(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv,
                                   int d, int causal, const void* qkv, void* O, float* lse);
mosaic_status launch_attention_bwd(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv,
                                   int d, int causal, const void* qkv, const void* O,
                                   const float* lse, const void* dO, void* dqkv, float* delta);

// ----------------------------------------------------------- norms and elementwise
mosaic_status launch_norm_fwd(hipStream_t s, int quota, int dtype, int norm, int64_t T,
                              int64_t h, float eps, const void* x, const void* gamma,
                              const void* beta, void* y, float* stats);
// scratch of launch_norm_bwd: two slabs of partial sums per row partition, a third when dxsum is asked for
size_t norm_bwd_scratch_bytes(int64_t h, bool with_dxsum = true);
mosaic_status launch_norm_bwd(hipStream_t s, int quota, int dtype, int norm, int64_t T,
                              int64_t h, const void* x, const void* gamma, const float* stats,
                              const void* dy, const void* R, void* dx, void* dgamma,
                              void* dbeta, void* scratch, void* dxsum = nullptr);
// dxsum (may be null): receives the column sums of dx[T,h] as stored, in the fixed two-level
// order of launch_colsum's partitions; formed inside the norm kernel where it has a variant
// for that (LayerNorm rows of up to 2048 bf16 / 1024 fp32 elements), by a pass over dx otherwise.
mosaic_status launch_gelu_fwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, void* a);
mosaic_status launch_gelu_bwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z,
                              const void* da, void* dz);
// dz = da * gelu'(z) and colsum[n] = column sums of dz[T,n] as stored (same bits as launch_colsum
// over dz); scratch: colsum_scratch_bytes(n)
mosaic_status launch_gelu_bwd_colsum(hipStream_t s, int quota, int dtype, int64_t T, int64_t n, const void* z,
                                     const void* da, void* dz, void* colsum, void* scratch);
mosaic_status launch_swiglu_fwd(hipStream_t s, int quota, int dtype, int64_t T, int64_t f,
                                const void* gu, void* a);
mosaic_status launch_swiglu_bwd(hipStream_t s, int quota, int dtype, int64_t T, int64_t f,
                                const void* gu, const void* da, void* dgu);
// ------------------------------------------------------------------- layer variants
mosaic_status launch_gelu_tanh_fwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, void* a);
mosaic_status launch_gelu_tanh_bwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z,
                                   const void* da, void* dz);
// (cos, sin) of n * base^(-2i/d) for n < N, i < d/2, as float2[N][d/2]
size_t rope_table_bytes(int N, int d);
mosaic_status launch_rope_table(hipStream_t s, int quota, int N, int d, float base, void* table);
// rotates the q and k parts of packed [B*N, (H+2*Hkv)*d] rows in place; direction -1 turns back
mosaic_status launch_rope(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d,
                          int direction, void* qkv, const void* table);
// p, m, v (and master, if not null) updated in place; m, v, master are fp32
mosaic_status launch_adamw(hipStream_t s, int quota, int dtype, int64_t n, void* p, const void* g,
                           float* m, float* v, float* master, float lr, float beta1, float beta2,
                           float eps, float weight_decay, int64_t step);
// k=3, pad=1 convolution over frames-major [B, L, C] as gather + GEMM: out [B*Lo, 3*C] with
// column index tap*C + channel; col2im1d is the transposed gather (one owner per element)
mosaic_status launch_im2col1d(hipStream_t s, int quota, int dtype, int64_t B, int L, int Lo, int C,
                              int stride, const void* x, void* out);
mosaic_status launch_col2im1d(hipStream_t s, int quota, int dtype, int64_t B, int L, int Lo, int C,
                              int stride, const void* dP, void* dx);
size_t mse_scratch_bytes();
mosaic_status launch_mse(hipStream_t s, int quota, int dtype, int64_t n, const void* y,
                         const void* target, void* dy, float* loss, void* scratch);
size_t colsum_scratch_bytes(int64_t n);
// out[n] = sum over T rows of X[T,n] in a fixed two-level order.
mosaic_status launch_colsum(hipStream_t s, int quota, int dtype, int64_t T, int64_t n,
                            const void* X, void* out, void* scratch);

// ----------------------------------------------------------------------------- stems
mosaic_status launch_unfold(hipStream_t s, int quota, int dtype, int B, int side, int patch,
                            const void* img, void* out);
// y[b*N+t, :] += pos[t, :]
mosaic_status launch_add_pos(hipStream_t s, int quota, int dtype, int B, int N, int h,
                             const void* pos, void* y);
// dpos[t,:] = sum_b dy[b*N+t,:] in ascending b
mosaic_status launch_pos_grad(hipStream_t s, int quota, int dtype, int B, int N, int h,
                              const void* dy, void* dpos);
// out rows: per sample b, [0,n_b) from img_tok, [n_b,N) from table[ids]; n_b = n_img, or
// counts[b] (clamped to [0,n_img]) when counts is given; ids is [B, N-n_img] without counts and
// one id per sequence position, [B, N], with them
mosaic_status launch_text_stem_fwd(hipStream_t s, int quota, int dtype, int B, int N, int n_img,
                                   int h, int vocab, const void* img_tok, const int32_t* ids,
                                   const int32_t* counts, const void* table, void* out);
// d_img rows from dy (zero for image tokens a sample did not use); dtable[v] = sum over
// occurrences of v (ascending position)
mosaic_status launch_text_stem_bwd(hipStream_t s, int quota, int dtype, int B, int N, int n_img,
                                   int h, int vocab, const void* dy, const int32_t* ids,
                                   const int32_t* counts, void* d_img, void* dtable);
