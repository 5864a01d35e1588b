// C-ABI wrappers of the single operations, and the dispatch between the MFMA attention
// kernels and the plain FMA ones.
#include <mutex>
#include "kernels.h"

mosaic_status launch_attention_fwd_simple(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d,
                                          int causal, const void* qkv, void* O, float* lse);
mosaic_status launch_attention_bwd_simple(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d,
                                          int causal, const void* qkv, const void* O, const float* lse,
                                          const void* dO, void* dqkv, float* delta);

mosaic_status launch_attention_delta(hipStream_t s, int quota, int dtype, int B, int N, int H, int d,
                                     const void* O, const void* dO, float* delta);
bool attention_mfma_supported(int dtype, int d);
mosaic_status launch_attention_fwd_mfma(hipStream_t s, int quota, int B, int N, int H, int Hkv, int d, int causal,
                                        const void* qkv, void* O, float* lse);
mosaic_status launch_attention_bwd_mfma(hipStream_t s, int quota, int B, int N, int H, int Hkv, int d, int causal,
                                        const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv,
                                        float* delta);

static bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

// The MFMA kernels address one sample's packed q|k|v rows with 32-bit byte offsets (buffer
// descriptors); a tile may start up to 63 rows past the end.  Longer slices take the plain
// kernels, which index with 64 bits.
static bool attn_slice_fits32(int N, int H, int Hkv, int d) {
  return ((int64_t)N + 64) * ((int64_t)H + 2 * Hkv) * d * 2 < ((int64_t)1 << 32);
}

static mosaic_status check_attn(int B, int N, int H, int Hkv, int d) {
  if (B <= 0 || N <= 0 || H <= 0 || d <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "attention sizes must be positive");
  if (Hkv <= 0 || H % Hkv) MOSAIC_FAIL(MOSAIC_EINVAL, "key/value heads (%d) must divide the query heads (%d)", Hkv, H);
  if (d > 128) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "head size %d > 128", d);
  return MOSAIC_OK;
}

mosaic_status launch_attention_fwd(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d, int causal,
                                   const void* qkv, void* O, float* lse) {
  MOSAIC_TRY(check_attn(B, N, H, Hkv, d));
  if (attention_mfma_supported(dtype, d) && attn_slice_fits32(N, H, Hkv, d) && aligned16(qkv) && aligned16(O))
    return launch_attention_fwd_mfma(s, quota, B, N, H, Hkv, d, causal, qkv, O, lse);
  return launch_attention_fwd_simple(s, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse);
}

mosaic_status launch_attention_bwd(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d, int causal,
                                   const void* qkv, const void* O, const float* lse, const void* dO, void* dqkv,
                                   float* delta) {
  MOSAIC_TRY(check_attn(B, N, H, Hkv, d));
  if (attention_mfma_supported(dtype, d) && attn_slice_fits32(N, H, Hkv, d) && aligned16(qkv) && aligned16(O) && aligned16(dO) && aligned16(dqkv)) {
    return launch_attention_bwd_mfma(s, quota, B, N, H, Hkv, d, causal, qkv, O, lse, dO, dqkv, delta);
  }
  return launch_attention_bwd_simple(s, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse, dO, dqkv, delta);
}

static mosaic_status check_common(int32_t quota, int32_t dtype) {
  if (dtype != MOSAIC_F32 && dtype != MOSAIC_BF16) MOSAIC_FAIL(MOSAIC_EINVAL, "bad dtype %d", dtype);
  DeviceInfo di;
  MOSAIC_TRY(mosaic_device_info(&di));
  if (quota <= 0 || quota > di.cu_count) MOSAIC_FAIL(MOSAIC_EQUOTA, "quota %d outside [1, %d]", quota, di.cu_count);
  return MOSAIC_OK;
}

#define NONNULL(p) if (!(p)) MOSAIC_FAIL(MOSAIC_EINVAL, "null pointer: " #p)

extern "C" {

mosaic_status mosaic_op_linear_fwd(void* stream, int32_t quota, int32_t dtype, int64_t T, int64_t k, int64_t n,
                                   const void* X, const void* W, const void* bias, const void* R, void* Y) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(X); NONNULL(W); NONNULL(Y);
  if (T < 0 || k <= 0 || n <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad linear sizes");
  return launch_gemm((hipStream_t)stream, quota, dtype, true, false, T, n, k, X, k, W, n, Y, n, bias, R);
}

mosaic_status mosaic_op_linear_dgrad(void* stream, int32_t quota, int32_t dtype, int64_t T, int64_t k, int64_t n,
                                     const void* dY, const void* W, const void* R, void* dX) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(dY); NONNULL(W); NONNULL(dX);
  if (T < 0 || k <= 0 || n <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad linear sizes");
  return launch_gemm((hipStream_t)stream, quota, dtype, true, true, T, k, n, dY, n, W, n, dX, k, nullptr, R);
}

size_t mosaic_op_colsum_scratch_bytes(int64_t n) { return colsum_scratch_bytes(n); }

size_t mosaic_op_linear_wgrad_scratch_bytes(int64_t T, int64_t k, int64_t n) {
  return align_up(gemm_splitk_scratch_bytes(k, n, T), 256) + colsum_scratch_bytes(n);
}

mosaic_status mosaic_op_linear_wgrad(void* stream, int32_t quota, int32_t dtype, int64_t T, int64_t k, int64_t n,
                                     const void* X, const void* dY, void* dW, void* db, void* scratch) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(X); NONNULL(dY); NONNULL(dW);
  if (T < 0 || k <= 0 || n <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad linear sizes");
  NONNULL(scratch);
  if ((uintptr_t)scratch % 16) MOSAIC_FAIL(MOSAIC_EINVAL, "scratch must be 16-byte aligned");
  if (T == 0) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "weight gradient over zero tokens");
  MOSAIC_TRY(launch_gemm((hipStream_t)stream, quota, dtype, false, false, k, n, T, X, k, dY, n, dW, n, nullptr, nullptr, scratch));
  if (db) MOSAIC_TRY(launch_colsum((hipStream_t)stream, quota, dtype, T, n, dY, db,
                                   (char*)scratch + align_up(gemm_splitk_scratch_bytes(k, n, T), 256)));
  return MOSAIC_OK;
}

mosaic_status mosaic_op_attention_fwd(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N, int32_t H,
                                      int32_t d, int32_t causal, const void* qkv, void* O, float* lse) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(qkv); NONNULL(O); NONNULL(lse);
  return launch_attention_fwd((hipStream_t)stream, quota, dtype, B, N, H, H, d, causal, qkv, O, lse);
}

mosaic_status mosaic_op_attention_bwd(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N, int32_t H,
                                      int32_t d, int32_t causal, const void* qkv, const void* O, const float* lse,
                                      const void* dO, void* dqkv, float* delta) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(qkv); NONNULL(O); NONNULL(lse); NONNULL(dO); NONNULL(dqkv); NONNULL(delta);
  return launch_attention_bwd((hipStream_t)stream, quota, dtype, B, N, H, H, d, causal, qkv, O, lse, dO, dqkv, delta);
}

mosaic_status mosaic_op_attention_gqa_fwd(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N, int32_t H,
                                          int32_t Hkv, int32_t d, int32_t causal, const void* qkv, void* O, float* lse) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(qkv); NONNULL(O); NONNULL(lse);
  return launch_attention_fwd((hipStream_t)stream, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse);
}

mosaic_status mosaic_op_attention_gqa_bwd(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N, int32_t H,
                                          int32_t Hkv, int32_t d, int32_t causal, const void* qkv, const void* O,
                                          const float* lse, const void* dO, void* dqkv, float* delta) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(qkv); NONNULL(O); NONNULL(lse); NONNULL(dO); NONNULL(dqkv); NONNULL(delta);
  return launch_attention_bwd((hipStream_t)stream, quota, dtype, B, N, H, Hkv, d, causal, qkv, O, lse, dO, dqkv, delta);
}

mosaic_status mosaic_op_norm_fwd(void* stream, int32_t quota, int32_t dtype, int32_t norm, int64_t T, int64_t h,
                                 float eps, const void* x, const void* gamma, const void* beta, void* y, float* stats) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(x); NONNULL(gamma); NONNULL(y); NONNULL(stats);
  if (norm == MOSAIC_LAYERNORM) NONNULL(beta);
  if (T < 0 || h <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm sizes");
  return launch_norm_fwd((hipStream_t)stream, quota, dtype, norm, T, h, eps, x, gamma, beta, y, stats);
}

size_t mosaic_op_norm_bwd_scratch_bytes(int64_t h) { return norm_bwd_scratch_bytes(h); }

mosaic_status mosaic_op_norm_bwd(void* stream, int32_t quota, int32_t dtype, int32_t norm, int64_t T, int64_t h,
                                 const void* x, const void* gamma, const float* stats, const void* dy, const void* R,
                                 void* dx, void* dgamma, void* dbeta, void* scratch) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(x); NONNULL(gamma); NONNULL(stats); NONNULL(dy); NONNULL(dx); NONNULL(dgamma); NONNULL(scratch);
  if (norm == MOSAIC_LAYERNORM) NONNULL(dbeta);
  if (T < 0 || h <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm sizes");
  return launch_norm_bwd((hipStream_t)stream, quota, dtype, norm, T, h, x, gamma, stats, dy, R, dx, dgamma, dbeta, scratch);
}

// Scratch of the entry point for callers that cannot allocate: the partial column sums of the
// norm backward for rows of up to kStaticNormMaxH elements.  Each GPU holds its own copy of the
// array at its own address; host code never uses the array's name as an address, only the
// pointer that hipGetSymbolAddress returned with that GPU current.
constexpr int64_t kStaticNormMaxH = 5120;
constexpr size_t kStaticScratchBytes = (size_t)512 * 2 * kStaticNormMaxH * sizeof(float);   // 20 MiB
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

static mosaic_status static_scratch_ptr(void** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void* ptr[kMaxDevices] = {};
  int dev = 0;
  MOSAIC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "device index %d beyond the %d this table holds", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    MOSAIC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) MOSAIC_FAIL(MOSAIC_EHIP, "hipGetSymbolAddress returned a null address");
    ptr[dev] = p;
  }
  *out = ptr[dev];
  return MOSAIC_OK;
}

size_t mosaic_op_norm_bwd_static_max_h(void) { return (size_t)kStaticNormMaxH; }

mosaic_status mosaic_op_norm_bwd_static(void* stream, int32_t quota, int32_t dtype, int32_t norm, int64_t T, int64_t h,
                                        const void* x, const void* gamma, const float* stats, const void* dy,
                                        const void* R, void* dx, void* dgamma, void* dbeta) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(x); NONNULL(gamma); NONNULL(stats); NONNULL(dy); NONNULL(dx); NONNULL(dgamma);
  if (norm == MOSAIC_LAYERNORM) NONNULL(dbeta);
  if (T < 0 || h <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm sizes");
  if (h > kStaticNormMaxH || norm_bwd_scratch_bytes(h, false) > kStaticScratchBytes)
    MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "row width %lld exceeds the %lld elements the built-in scratch covers; "
                "use mosaic_op_norm_bwd with a caller-provided scratch", (long long)h, (long long)kStaticNormMaxH);
  void* sc = nullptr;
  MOSAIC_TRY(static_scratch_ptr(&sc));
  return launch_norm_bwd((hipStream_t)stream, quota, dtype, norm, T, h, x, gamma, stats, dy, R, dx, dgamma, dbeta, sc);
}

mosaic_status mosaic_op_gelu_fwd(void* stream, int32_t quota, int32_t dtype, int64_t n, const void* z, void* a) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(z); NONNULL(a);
  return launch_gelu_fwd((hipStream_t)stream, quota, dtype, n, z, a);
}

mosaic_status mosaic_op_gelu_bwd(void* stream, int32_t quota, int32_t dtype, int64_t n, const void* z, const void* da, void* dz) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(z); NONNULL(da); NONNULL(dz);
  return launch_gelu_bwd((hipStream_t)stream, quota, dtype, n, z, da, dz);
}

mosaic_status mosaic_op_swiglu_fwd(void* stream, int32_t quota, int32_t dtype, int64_t T, int64_t f, const void* gu, void* a) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(gu); NONNULL(a);
  return launch_swiglu_fwd((hipStream_t)stream, quota, dtype, T, f, gu, a);
}

mosaic_status mosaic_op_linear_act_fwd(void* stream, int32_t quota, int32_t dtype, int32_t act, int64_t T, int64_t k, int64_t n,
                                       const void* X, const void* W, const void* bias, void* Z, void* A) {
  MOSAIC_TRY(check_common(quota, dtype));
  if (T < 0 || k <= 0 || n < 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad linear shape T=%lld k=%lld n=%lld", (long long)T, (long long)k, (long long)n);
  NONNULL(X); NONNULL(W); NONNULL(Z); NONNULL(A);
  return launch_linear_act_fwd((hipStream_t)stream, quota, dtype, act, T, k, n, X, W, bias, Z, A);
}

mosaic_status mosaic_op_swiglu_bwd(void* stream, int32_t quota, int32_t dtype, int64_t T, int64_t f, const void* gu,
                                   const void* da, void* dgu) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(gu); NONNULL(da); NONNULL(dgu);
  return launch_swiglu_bwd((hipStream_t)stream, quota, dtype, T, f, gu, da, dgu);
}

mosaic_status mosaic_op_gelu_tanh_fwd(void* stream, int32_t quota, int32_t dtype, int64_t n, const void* z, void* a) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(z); NONNULL(a);
  return launch_gelu_tanh_fwd((hipStream_t)stream, quota, dtype, n, z, a);
}

mosaic_status mosaic_op_gelu_tanh_bwd(void* stream, int32_t quota, int32_t dtype, int64_t n, const void* z, const void* da, void* dz) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(z); NONNULL(da); NONNULL(dz);
  return launch_gelu_tanh_bwd((hipStream_t)stream, quota, dtype, n, z, da, dz);
}

size_t mosaic_op_rope_table_bytes(int32_t N, int32_t d) { return (N > 0 && d > 0) ? rope_table_bytes(N, d) : 0; }

mosaic_status mosaic_op_rope_table(void* stream, int32_t quota, int32_t N, int32_t d, float base, void* table) {
  MOSAIC_TRY(check_common(quota, MOSAIC_F32));
  NONNULL(table);
  return launch_rope_table((hipStream_t)stream, quota, N, d, base, table);
}

mosaic_status mosaic_op_rope(void* stream, int32_t quota, int32_t dtype, int32_t B, int32_t N, int32_t H, int32_t d,
                             int32_t direction, void* qkv, const void* table) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(qkv); NONNULL(table);
  return launch_rope((hipStream_t)stream, quota, dtype, B, N, H, H, d, direction, qkv, table);
}

mosaic_status mosaic_op_adamw(void* stream, int32_t quota, int32_t dtype, int64_t n, void* params, const void* grads,
                              float* m, float* v, float* master, float lr, float beta1, float beta2, float eps,
                              float weight_decay, int64_t step) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(params); NONNULL(grads); NONNULL(m); NONNULL(v);
  if (n < 0) MOSAIC_FAIL(MOSAIC_EINVAL, "negative element count");
  return launch_adamw((hipStream_t)stream, quota, dtype, n, params, grads, m, v, master, lr, beta1, beta2, eps, weight_decay, step);
}

size_t mosaic_op_mse_scratch_bytes(void) { return mse_scratch_bytes(); }

mosaic_status mosaic_op_mse(void* stream, int32_t quota, int32_t dtype, int64_t n, const void* y, const void* target,
                            void* dy, float* loss, void* scratch) {
  MOSAIC_TRY(check_common(quota, dtype));
  NONNULL(y); NONNULL(target); NONNULL(dy); NONNULL(loss); NONNULL(scratch);
  return launch_mse((hipStream_t)stream, quota, dtype, n, y, target, dy, loss, scratch);
}

}  // extern "C"
