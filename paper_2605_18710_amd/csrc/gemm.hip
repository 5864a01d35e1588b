// Linear-layer contractions (forward, input gradient, weight gradient) for gfx950.
//
// bf16 path: persistent MFMA kernel.  A workgroup of 4 waves walks output tiles
// tile = blockIdx.x, blockIdx.x + gridDim.x, ...; the grid is sized to the module's CU
// quota.  Each output element is produced by exactly one wave that accumulates k in
// ascending order with v_mfma_f32_32x32x16_bf16, so the bits of the result do not
// depend on the grid, the tile shape or which CU ran the tile.
//
// Operands reach the matrix cores through LDS in "K-contiguous" form [row][BK] (pitch
// BK+8 elements so that 16-lane groups of ds_read_b128 hit 64 distinct banks).  An
// operand that is K-contiguous in HBM is copied with 128-bit loads/stores.  An operand
// whose contraction index is the strided one (the weight in the forward pass, both
// operands of the weight gradient) is transposed on the way in: a thread loads KB rows
// of 8 consecutive elements, transposes the KBx8 block in registers with byte permutes
// and writes 8 K-contiguous pieces.  Global loads for K-tile i+1 are issued before the
// MFMAs of tile i and land in the second LDS buffer afterwards (one barrier per K-tile).
//
// fp32 path (and shapes the MFMA path does not cover): a plain LDS-tiled FMA kernel with
// arbitrary strides; ascending-k accumulation as well.
#include "kernels.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;
constexpr int PITCH = BK + 8;  // bf16 elements per LDS row

__device__ __forceinline__ uint32_t perm_lo(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_perm(hi, lo, 0x05040100u); }
__device__ __forceinline__ uint32_t perm_hi(uint32_t hi, uint32_t lo) { return __builtin_amdgcn_perm(hi, lo, 0x07060302u); }

// Register image of one operand tile (ROWS x BK) in flight from HBM to LDS.
template <int ROWS, bool KC>
struct TileLoader {
  // K-contiguous: thread owns chunk kc = t%8 (8 elements) of rows t/8 + 32*j.
  // K-strided:    thread owns a KB x 8 block: k rows kb*KB.., x chunk c*8.., with
  //               kb = t % (BK/KB), c = t / (BK/KB).
  static constexpr int KB = ROWS * BK / 8 / 256;              // 8 for 256 rows, 4 for 128
  static constexpr int NLOAD = KC ? ROWS / 32 : KB;
  uint4 r[NLOAD];

  __device__ __forceinline__ void load(const bf16* __restrict__ src, int64_t ld, int x0, int k0,
                                       int x_total, int k_total) {
    const int t = threadIdx.x;
    if constexpr (KC) {
      const int kc = t & 7;
      const int k = k0 + kc * 8;
#pragma unroll
      for (int j = 0; j < NLOAD; ++j) {
        const int x = x0 + (t >> 3) + 32 * j;
        if (x < x_total && k < k_total)
          r[j] = *reinterpret_cast<const uint4*>(src + (int64_t)x * ld + k);
        else
          r[j] = make_uint4(0, 0, 0, 0);
      }
    } else {
      constexpr int NKB = BK / KB;
      const int kb = t % NKB, c = t / NKB;
      const int x = x0 + c * 8;
#pragma unroll
      for (int j = 0; j < NLOAD; ++j) {
        const int k = k0 + kb * KB + j;
        if (x < x_total && k < k_total)
          r[j] = *reinterpret_cast<const uint4*>(src + (int64_t)k * ld + x);
        else
          r[j] = make_uint4(0, 0, 0, 0);
      }
    }
  }

  __device__ __forceinline__ void store(bf16* __restrict__ lds) const {
    const int t = threadIdx.x;
    if constexpr (KC) {
      const int kc = t & 7;
#pragma unroll
      for (int j = 0; j < NLOAD; ++j) {
        const int row = (t >> 3) + 32 * j;
        *reinterpret_cast<uint4*>(lds + row * PITCH + kc * 8) = r[j];
      }
    } else {
      constexpr int NKB = BK / KB;
      const int kb = t % NKB, c = t / NKB;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        uint32_t o[KB / 2];
#pragma unroll
        for (int p = 0; p < KB / 2; ++p) {
          const uint32_t lo = (&r[2 * p].x)[i >> 1], hi = (&r[2 * p + 1].x)[i >> 1];
          o[p] = (i & 1) ? perm_hi(hi, lo) : perm_lo(hi, lo);
        }
        bf16* dst = lds + (c * 8 + i) * PITCH + kb * KB;
        if constexpr (KB == 8) *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
        else if constexpr (KB == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
        else *reinterpret_cast<uint32_t*>(dst) = o[0];
      }
    }
  }
};

template <int BM, int BN, bool A_KC, bool B_KC>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(
    const bf16* __restrict__ A, const bf16* __restrict__ B, bf16* __restrict__ C,
    const bf16* __restrict__ bias, const bf16* __restrict__ R, int M, int N, int K,
    int64_t lda, int64_t ldb, int64_t ldc, int tiles_m, int tiles_n) {
  constexpr int WM = BM / 2, WN = BN / 2;   // 2 x 2 waves
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int STAGE = (BM + BN) * PITCH;  // elements per LDS stage
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = (wave >> 1) * WM, wn = (wave & 1) * WN;
  const int lr = lane & 31, lk = (lane >> 5) * 8;
  const int nk = (K + BK - 1) / BK;
  const int ntiles = tiles_m * tiles_n;

  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    // consecutive tiles share the same column block: a wave of workgroups reads few
    // distinct B panels
    const int tn_i = tile / tiles_m, tm_i = tile - tn_i * tiles_m;
    const int m0 = tm_i * BM, n0 = tn_i * BN;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    TileLoader<BM, A_KC> la;
    TileLoader<BN, B_KC> lb;
    la.load(A, lda, m0, 0, M, K);
    lb.load(B, ldb, n0, 0, N, K);
    la.store(smem);
    lb.store(smem + BM * PITCH);
    __syncthreads();

    for (int kt = 0; kt < nk; ++kt) {
      const bf16* sa = smem + (kt & 1) * STAGE;
      const bf16* sb = sa + BM * PITCH;
      if (kt + 1 < nk) {
        la.load(A, lda, m0, (kt + 1) * BK, M, K);
        lb.load(B, ldb, n0, (kt + 1) * BK, N, K);
      }
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8 fa[TM], fb[TN];
#pragma unroll
        for (int i = 0; i < TM; ++i)
          fa[i] = *reinterpret_cast<const bf16x8*>(sa + (wm + i * 32 + lr) * PITCH + ks * 16 + lk);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          fb[j] = *reinterpret_cast<const bf16x8*>(sb + (wn + j * 32 + lr) * PITCH + ks * 16 + lk);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      }
      if (kt + 1 < nk) {
        bf16* da = smem + ((kt + 1) & 1) * STAGE;
        la.store(da);
        lb.store(da + BM * PITCH);
      }
      __syncthreads();
    }

    // epilogue: element (row, col) of a 32x32 block sits in lane col + 32*((row/4)%2),
    // register 4*(row/8) + row%4
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn + j * 32 + lr;
        if (col >= N) continue;
        const float bv = bias ? (float)bias[col] : 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
          if (row < M) {
            float v = acc[i][j][e] + bv;
            if (R) v += (float)R[(int64_t)row * ldc + col];
            C[(int64_t)row * ldc + col] = (bf16)v;
          }
        }
      }
  }
}

// ------------------------------------------------------------------ generic FMA kernel
template <typename T>
__global__ __launch_bounds__(256) void gemm_generic_kernel(
    const T* __restrict__ A, const T* __restrict__ B, T* __restrict__ C, const T* __restrict__ bias,
    const T* __restrict__ R, int M, int N, int K, int64_t sam, int64_t sak, int64_t sbk, int64_t sbn,
    int64_t ldc, int tiles_m, int tiles_n) {
  constexpr int TS = 64, KS = 16;
  __shared__ float As[KS][TS + 1];
  __shared__ float Bs[KS][TS + 1];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int ntiles = tiles_m * tiles_n;
  for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const int tn_i = tile / tiles_m, tm_i = tile - tn_i * tiles_m;
    const int m0 = tm_i * TS, n0 = tn_i * TS;
    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
    for (int k0 = 0; k0 < K; k0 += KS) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int idx = threadIdx.x + 256 * q;     // 0..1023
        // A tile: prefer the contiguous index to vary fastest across threads
        int am, ak;
        if (sak == 1) { ak = idx % KS; am = idx / KS; } else { am = idx % TS; ak = idx / TS; }
        const int gm = m0 + am, gk = k0 + ak;
        As[ak][am] = (gm < M && gk < K) ? to_f32(A[(int64_t)gm * sam + (int64_t)gk * sak]) : 0.f;
        int bn, bk;
        if (sbk == 1) { bk = idx % KS; bn = idx / KS; } else { bn = idx % TS; bk = idx / TS; }
        const int gn = n0 + bn, gk2 = k0 + bk;
        Bs[bk][bn] = (gn < N && gk2 < K) ? to_f32(B[(int64_t)gk2 * sbk + (int64_t)gn * sbn]) : 0.f;
      }
      __syncthreads();
#pragma unroll
      for (int k = 0; k < KS; ++k) {
        float a[4], b[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
        for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
          for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
      }
      __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = m0 + ty * 4 + i;
      if (row >= M) continue;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int col = n0 + tx * 4 + j;
        if (col >= N) continue;
        float v = acc[i][j];
        if (bias) v += to_f32(bias[col]);
        if (R) v += to_f32(R[(int64_t)row * ldc + col]);
        C[(int64_t)row * ldc + col] = from_f32<T>(v);
      }
    }
  }
}

template <int BM, int BN, bool A_KC, bool B_KC>
mosaic_status launch_mfma(hipStream_t s, int quota, int M, int N, int K, const bf16* A, int64_t lda,
                          const bf16* B, int64_t ldb, bf16* C, int64_t ldc, const bf16* bias, const bf16* R) {
  constexpr size_t smem = 2 * (size_t)(BM + BN) * PITCH * sizeof(bf16);
  auto kern = gemm_bf16_kernel<BM, BN, A_KC, B_KC>;
  static bool attr_set = false;   // per instantiation; idempotent, so a race is harmless
  if (!attr_set) {
    MOSAIC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
    attr_set = true;
  }
  const int tiles_m = (int)ceil_div(M, BM), tiles_n = (int)ceil_div(N, BN);
  const int wg_per_cu = (smem > 80 * 1024) ? 1 : 2;
  const int grid = grid_for(quota, wg_per_cu, (int64_t)tiles_m * tiles_n);
  kern<<<grid, 256, smem, s>>>(A, B, C, bias, R, M, N, K, lda, ldb, ldc, tiles_m, tiles_n);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

template <bool A_KC, bool B_KC>
mosaic_status launch_mfma_shape(hipStream_t s, int quota, int M, int N, int K, const bf16* A, int64_t lda,
                                const bf16* B, int64_t ldb, bf16* C, int64_t ldc, const bf16* bias, const bf16* R) {
  // Tile shape is a function of the problem shape only.  Large tiles halve LDS traffic
  // per MFMA; small problems keep 128x128 so that more CUs get a tile.
  const int64_t big_tiles = ceil_div(M, 256) * ceil_div(N, 256);
  if (big_tiles >= 512)
    return launch_mfma<256, 256, A_KC, B_KC>(s, quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R);
  return launch_mfma<128, 128, A_KC, B_KC>(s, quota, M, N, K, A, lda, B, ldb, C, ldc, bias, R);
}

}  // namespace

mosaic_status launch_gemm(hipStream_t s, int quota, int dtype, bool a_kc, bool b_kc, int64_t M, int64_t N,
                          int64_t K, const void* A, int64_t lda, const void* B, int64_t ldb, void* C,
                          int64_t ldc, const void* bias, const void* R) {
  if (M < 0 || N < 0 || K < 0) MOSAIC_FAIL(MOSAIC_EINVAL, "negative GEMM size");
  if (M > INT32_MAX || N > INT32_MAX || K > INT32_MAX) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "GEMM dimension too large");
  if (M == 0 || N == 0) return MOSAIC_OK;
  const bool vec_ok = (lda % 8 == 0) && (ldb % 8 == 0) && (K % 8 == 0 || (!a_kc && !b_kc)) &&
                      (a_kc || M % 8 == 0) && (b_kc || N % 8 == 0) &&
                      ((uintptr_t)A % 16 == 0) && ((uintptr_t)B % 16 == 0) && K > 0;
  if (dtype == MOSAIC_BF16 && vec_ok) {
    const bf16 *a = (const bf16*)A, *b = (const bf16*)B, *bi = (const bf16*)bias, *r = (const bf16*)R;
    bf16* c = (bf16*)C;
    if (a_kc && !b_kc) return launch_mfma_shape<true, false>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r);
    if (a_kc && b_kc) return launch_mfma_shape<true, true>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r);
    if (!a_kc && !b_kc) return launch_mfma_shape<false, false>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r);
    return launch_mfma_shape<false, true>(s, quota, (int)M, (int)N, (int)K, a, lda, b, ldb, c, ldc, bi, r);
  }
  const int64_t sam = a_kc ? lda : 1, sak = a_kc ? 1 : lda;
  const int64_t sbk = b_kc ? 1 : ldb, sbn = b_kc ? ldb : 1;
  const int tiles_m = (int)ceil_div(M, 64), tiles_n = (int)ceil_div(N, 64);
  const int grid = grid_for(quota, 8, (int64_t)tiles_m * tiles_n);
  if (dtype == MOSAIC_BF16)
    gemm_generic_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)A, (const bf16*)B, (bf16*)C, (const bf16*)bias,
                                                   (const bf16*)R, (int)M, (int)N, (int)K, sam, sak, sbk, sbn, ldc, tiles_m, tiles_n);
  else
    gemm_generic_kernel<float><<<grid, 256, 0, s>>>((const float*)A, (const float*)B, (float*)C, (const float*)bias,
                                                    (const float*)R, (int)M, (int)N, (int)K, sam, sak, sbk, sbn, ldc, tiles_m, tiles_n);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}
