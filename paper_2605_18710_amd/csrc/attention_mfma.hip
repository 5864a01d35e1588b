// Flash-style attention for bf16 on the gfx950 matrix cores, head size 64 or 128.
//
// Forward: a workgroup owns 128 queries of one (sample, head), one wave per 32 queries, and
// streams key/value tiles of 64 through LDS with online softmax.  Scores are computed
// transposed, S^T = K Q^T, so that in the 32x32 accumulator layout a lane owns ONE query
// (column lane%32) and 16 keys (its registers): the row maximum and sum are in-lane
// reductions plus one exchange between the two half-waves, and the running rescale is a
// per-lane scalar.  The probabilities feed the second product O^T = V^T P^T straight from
// registers: MFMA's contraction index may be enumerated in any order as long as both
// operands agree, so V^T is read from LDS in the key order the accumulator layout
// dictates (two 4-key runs per 16-key step).  V is transposed on its way into LDS.
//
// Backward is split in two kernels so that every sum has one owner and a fixed order
// (bit-identical for any grid): the dK/dV kernel owns 128 keys and streams query tiles;
// the dQ kernel owns 128 queries and streams key tiles.  Both recompute P from the saved
// row log-sum-exp; D_i = sum_c dO_ic O_ic comes from a small per-row kernel.
#include "kernels.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Position of streamed row r inside a transposed LDS row: each group of 16 keeps its four
// 4-runs in the order 0,2,1,3, so that the 8 indices a half-wave lane owns in registers
// 8*s2 .. 8*s2+7 of an accumulator block (two 4-runs, 8 apart) are 16 contiguous bytes.
__device__ __forceinline__ int tr_pos(int r) {
  const int sub = (r >> 2) & 3;
  return (r & ~15) + ((((sub & 1) << 1) | (sub >> 1)) << 2) + (r & 3);
}

// Cooperative loader of a tile of RS rows x D columns (row stride `rs` elements) by 256
// threads.  A thread owns KB consecutive rows of one 8-column chunk; it can store the
// tile in natural form [row][D+8] and/or transposed form [col][RS+4].
template <int RS, int D>
struct TileLoader {
  static constexpr int KB = RS * D / 2048;
  static_assert(KB >= 1, "tile too small for 256 threads");
  static constexpr int PN = D + 8, PT = RS + 8;
  uint4 r[KB];

  __device__ __forceinline__ void load(const bf16* __restrict__ src, int64_t rs, int row0, int limit) {
    const int t = threadIdx.x, cc = t % (D / 8), rb = t / (D / 8);
#pragma unroll
    for (int j = 0; j < KB; ++j) {
      const int row = row0 + rb * KB + j;
      r[j] = (row < limit) ? *reinterpret_cast<const uint4*>(src + (int64_t)row * rs + cc * 8) : make_uint4(0, 0, 0, 0);
    }
  }
  __device__ __forceinline__ void store_nat(bf16* __restrict__ lds) const {
    const int t = threadIdx.x, cc = t % (D / 8), rb = t / (D / 8);
#pragma unroll
    for (int j = 0; j < KB; ++j) *reinterpret_cast<uint4*>(lds + (rb * KB + j) * PN + cc * 8) = r[j];
  }
  __device__ __forceinline__ void store_tr(bf16* __restrict__ lds) const {
    const int t = threadIdx.x, cc = t % (D / 8), rb = t / (D / 8);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      bf16* dst = lds + (cc * 8 + i) * PT + tr_pos(rb * KB);
      if constexpr (KB == 1) {
        const uint32_t w = (&r[0].x)[i >> 1];
        *reinterpret_cast<uint16_t*>(dst) = (uint16_t)((i & 1) ? (w >> 16) : (w & 0xFFFFu));
      } else {
        uint32_t o[KB / 2];
#pragma unroll
        for (int p = 0; p < KB / 2; ++p) {
          const uint32_t lo = (&r[2 * p].x)[i >> 1], hi = (&r[2 * p + 1].x)[i >> 1];
          o[p] = (i & 1) ? __builtin_amdgcn_perm(hi, lo, 0x07060302u) : __builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
        if constexpr (KB == 2) *reinterpret_cast<uint32_t*>(dst) = o[0];
        else if constexpr (KB == 4) *reinterpret_cast<uint2*>(dst) = make_uint2(o[0], o[1]);
        else *reinterpret_cast<uint4*>(dst) = make_uint4(o[0], o[1], o[2], o[3]);
      }
    }
  }
};

// A-operand fragment from a natural tile: row `row`, columns 16*s + 8*hb .. +7
__device__ __forceinline__ bf16x8 frag_nat(const bf16* lds, int pitch, int row, int s, int hb) {
  return *reinterpret_cast<const bf16x8*>(lds + row * pitch + 16 * s + 8 * hb);
}
// A-operand fragment from a transposed tile [c][tr_pos(r)]: row c, the 8 streamed indices
// that a lane of half hb owns in registers 8*s2 .. 8*s2+7 of a 32x32 accumulator block
// (base + 16*s2 + 4*hb + {0..3} and + 8), one 16-byte read thanks to tr_pos
__device__ __forceinline__ bf16x8 frag_tr(const bf16* lds, int pitch, int c, int base, int s2, int hb) {
  return *reinterpret_cast<const bf16x8*>(lds + c * pitch + base + 16 * s2 + 8 * hb);
}
// registers 8*s2 .. 8*s2+7 of an accumulator block as a bf16 B-operand
__device__ __forceinline__ bf16x8 pack8(const float* v) {
  bf16x8 o;
#pragma unroll
  for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
  return o;
}
// streamed index (within a 32-block) held by register r of a lane of half hb
__device__ __forceinline__ int acc_row(int r, int hb) { return 8 * (r >> 2) + 4 * hb + (r & 3); }

// Work order for tiles of unequal cost (causal masks): items are ranked heaviest first and
// dealt to the persistent workgroups in a snake (even rounds ascending, odd rounds
// descending), so a workgroup that drew a heavy tile next draws a light one.
// Returns the rank of the `round`-th item of workgroup blockIdx.x, or -1.
__device__ __forceinline__ int snake_item(int round, int items) {
  const int G = gridDim.x, b = blockIdx.x;
  const int idx = round * G + ((round & 1) ? (G - 1 - b) : b);
  return idx < items ? idx : -1;
}

// --------------------------------------------------------------------------- forward
template <int D>
__global__ __launch_bounds__(256, 2) void attn_fwd_mfma(const bf16* __restrict__ qkv, bf16* __restrict__ O,
                                                     float* __restrict__ lse, int B, int N, int H, int causal,
                                                     float scale_log2, int qtiles) {
  constexpr int RS = 64, NS = D / 16, NC = D / 32;
  typedef TileLoader<RS, D> L;
  constexpr int KSZ = RS * L::PN, VSZ = D * L::PT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);          // [2][KSZ + VSZ]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  const int h = H * D;
  const int64_t rs = 3 * (int64_t)h;
  const int items = B * H * qtiles;
  for (int round = 0; round * (int)gridDim.x < items; ++round) {
    const int item = snake_item(round, items);
    if (item < 0) continue;
    // late query tiles carry the most keys under a causal mask: rank them first
    const int qt = qtiles - 1 - item / (B * H), hd = item % H, b = (item / H) % B;
    const int q0 = qt * 128, i0 = q0 + 32 * wave, i = i0 + lr;
    const bf16* base = qkv + (int64_t)b * N * rs + hd * D;
    bf16x8 qf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (i < N) qf[s] = *reinterpret_cast<const bf16x8*>(base + (int64_t)i * rs + 16 * s + 8 * hb);
      else { for (int e = 0; e < 8; ++e) qf[s][e] = (bf16)0.f; }
    }
    f32x16 o[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[c][e] = 0.f;
    float m = -INFINITY, lsum = 0.f;
    const int kv_end = causal ? min(N, q0 + 128) : N;
    const int ntiles = (kv_end + RS - 1) / RS;
    L lk, lv;
    lk.load(base + h, rs, 0, N);
    lv.load(base + 2 * h, rs, 0, N);
    __syncthreads();                      // previous item's readers are done with buffer 0
    lk.store_nat(smem);
    lv.store_tr(smem + KSZ);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
      const bf16* ks = smem + (t & 1) * (KSZ + VSZ);
      const bf16* vt = ks + KSZ;
      if (t + 1 < ntiles) {
        lk.load(base + h, rs, (t + 1) * RS, N);
        lv.load(base + 2 * h, rs, (t + 1) * RS, N);
      }
      const int j0 = t * RS;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int jb = j0 + 32 * sub;
        if (jb >= kv_end || (causal && jb > i0 + 31)) continue;     // nothing for this wave
        f32x16 sacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) sacc[e] = 0.f;
#pragma unroll
        for (int s = 0; s < NS; ++s)
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat(ks, L::PN, 32 * sub + lr, s, hb), qf[s], sacc, 0, 0, 0);
        float sv[16];
        float mx = -INFINITY;
        // only blocks that touch the diagonal or the end of the sequence need the mask
        const bool need_mask = (jb + 32 > N) || (causal && jb + 31 > i0);
        if (need_mask) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int j = jb + acc_row(r, hb);
            const bool masked = (j >= N) || (causal && j > i);
            sv[r] = masked ? -INFINITY : sacc[r] * scale_log2;
            mx = fmaxf(mx, sv[r]);
          }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) { sv[r] = sacc[r] * scale_log2; mx = fmaxf(mx, sv[r]); }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float mn = fmaxf(m, mx);
        // rescale the running sums only when some row's maximum moved (exact: the factor is 1 otherwise)
        if (__any(mn > m)) {
          const float mref0 = (mn == -INFINITY) ? 0.f : mn;
          const float corr = fast_exp2(m - mref0);               // m = -inf -> 0
          lsum *= corr;
#pragma unroll
          for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[c][e] *= corr;
          m = mn;
        }
        const float mref = (m == -INFINITY) ? 0.f : m;           // row with nothing visible yet
        float ps = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sv[r] = fast_exp2(sv[r] - mref); ps += sv[r]; }
        lsum += ps;
        const bf16x8 p0 = pack8(sv), p1 = pack8(sv + 8);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(vt, L::PT, 32 * c + lr, 32 * sub, 0, hb), p0, o[c], 0, 0, 0);
          o[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(vt, L::PT, 32 * c + lr, 32 * sub, 1, hb), p1, o[c], 0, 0, 0);
        }
      }
      if (t + 1 < ntiles) {
        bf16* nk = smem + ((t + 1) & 1) * (KSZ + VSZ);
        lk.store_nat(nk);
        lv.store_tr(nk + KSZ);
      }
      __syncthreads();
    }
    const float ltot = lsum + __shfl_xor(lsum, 32, 64);
    if (i < N) {
      const float inv = 1.0f / ltot;
      bf16* orow = O + ((int64_t)b * N + i) * h + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(o[c][4 * g + e] * inv);
          *reinterpret_cast<bf16x4*>(orow + 32 * c + 8 * g + 4 * hb) = v;
        }
      if (hb == 0) lse[((int64_t)b * H + hd) * N + i] = (m + log2f(ltot)) * kLn2;
    }
  }
}

// ------------------------------------------------------------------------------- dQ
template <int D>
__global__ __launch_bounds__(256) void attn_bwd_dq_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                        const float* __restrict__ lse, const float* __restrict__ delta,
                                                        bf16* __restrict__ dqkv, int B, int N, int H, int causal,
                                                        float scale, int qtiles) {
  constexpr int RS = 64, NS = D / 16, NC = D / 32;
  typedef TileLoader<RS, D> L;
  constexpr int NSZ = RS * L::PN, TSZ = D * L::PT;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);          // [2][K nat | V nat | K tr]
  constexpr int STAGE = 2 * NSZ + TSZ;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  const int h = H * D;
  const int64_t rs = 3 * (int64_t)h;
  const float scale_log2 = scale * kLog2e;
  const int items = B * H * qtiles;
  for (int round = 0; round * (int)gridDim.x < items; ++round) {
    const int item = snake_item(round, items);
    if (item < 0) continue;
    const int qt = qtiles - 1 - item / (B * H), hd = item % H, b = (item / H) % B;
    const int q0 = qt * 128, i0 = q0 + 32 * wave, i = i0 + lr;
    const bf16* base = qkv + (int64_t)b * N * rs + hd * D;
    const bf16* dob = dO + (int64_t)b * N * h + hd * D;
    bf16x8 qf[NS], dof[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (i < N) {
        qf[s] = *reinterpret_cast<const bf16x8*>(base + (int64_t)i * rs + 16 * s + 8 * hb);
        dof[s] = *reinterpret_cast<const bf16x8*>(dob + (int64_t)i * h + 16 * s + 8 * hb);
      } else {
        for (int e = 0; e < 8; ++e) { qf[s][e] = (bf16)0.f; dof[s][e] = (bf16)0.f; }
      }
    }
    const float lse2 = (i < N) ? lse[((int64_t)b * H + hd) * N + i] * kLog2e : 0.f;
    const float dlt = (i < N) ? delta[((int64_t)b * H + hd) * N + i] : 0.f;
    f32x16 dq[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) dq[c][e] = 0.f;
    const int kv_end = causal ? min(N, q0 + 128) : N;
    const int ntiles = (kv_end + RS - 1) / RS;
    L lk, lv;
    lk.load(base + h, rs, 0, N);
    lv.load(base + 2 * h, rs, 0, N);
    __syncthreads();
    lk.store_nat(smem); lv.store_nat(smem + NSZ); lk.store_tr(smem + 2 * NSZ);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
      const bf16* ks = smem + (t & 1) * STAGE;
      const bf16* vs = ks + NSZ;
      const bf16* kt = ks + 2 * NSZ;
      if (t + 1 < ntiles) {
        lk.load(base + h, rs, (t + 1) * RS, N);
        lv.load(base + 2 * h, rs, (t + 1) * RS, N);
      }
      const int j0 = t * RS;
#pragma unroll
      for (int sub = 0; sub < 2; ++sub) {
        const int jb = j0 + 32 * sub;
        if (jb >= kv_end || (causal && jb > i0 + 31)) continue;
        f32x16 sacc, pacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat(ks, L::PN, 32 * sub + lr, s, hb), qf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat(vs, L::PN, 32 * sub + lr, s, hb), dof[s], pacc, 0, 0, 0);
        }
        float ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int j = jb + acc_row(r, hb);
          const bool masked = (j >= N) || (i >= N) || (causal && j > i);
          const float p = masked ? 0.f : fast_exp2(sacc[r] * scale_log2 - lse2);
          ds[r] = p * (pacc[r] - dlt);
        }
        const bf16x8 d0 = pack8(ds), d1 = pack8(ds + 8);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          dq[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(kt, L::PT, 32 * c + lr, 32 * sub, 0, hb), d0, dq[c], 0, 0, 0);
          dq[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(kt, L::PT, 32 * c + lr, 32 * sub, 1, hb), d1, dq[c], 0, 0, 0);
        }
      }
      if (t + 1 < ntiles) {
        bf16* nk = smem + ((t + 1) & 1) * STAGE;
        lk.store_nat(nk); lv.store_nat(nk + NSZ); lk.store_tr(nk + 2 * NSZ);
      }
      __syncthreads();
    }
    if (i < N) {
      bf16* out = dqkv + ((int64_t)b * N + i) * rs + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = (bf16)(dq[c][4 * g + e] * scale);
          *reinterpret_cast<bf16x4*>(out + 32 * c + 8 * g + 4 * hb) = v;
        }
    }
  }
}

// --------------------------------------------------------------------------- dK, dV
template <int D>
__global__ __launch_bounds__(256, 2) void attn_bwd_dkv_mfma(const bf16* __restrict__ qkv, const bf16* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         bf16* __restrict__ dqkv, int B, int N, int H, int causal,
                                                         float scale, int ktiles) {
  constexpr int RS = 32, NS = D / 16, NC = D / 32;
  typedef TileLoader<RS, D> L;
  constexpr int NSZ = RS * L::PN, TSZ = D * L::PT;
  constexpr int STAGE = 2 * NSZ + 2 * TSZ;                 // Q nat | dO nat | Q tr | dO tr
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16* smem = reinterpret_cast<bf16*>(smem_raw);
  float* stat = reinterpret_cast<float*>(smem + 2 * STAGE);  // [2][2][RS]: lse*log2e, delta
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int lr = lane & 31, hb = lane >> 5;
  const int h = H * D;
  const int64_t rs = 3 * (int64_t)h;
  const float scale_log2 = scale * kLog2e;
  const int items = B * H * ktiles;
  for (int round = 0; round * (int)gridDim.x < items; ++round) {
    const int item = snake_item(round, items);
    if (item < 0) continue;
    // early key tiles see the most queries under a causal mask: rank them first
    const int kt_i = item / (B * H), hd = item % H, b = (item / H) % B;
    const int k0 = kt_i * 128, j0w = k0 + 32 * wave, j = j0w + lr;
    const bf16* base = qkv + (int64_t)b * N * rs + hd * D;
    const bf16* dob = dO + (int64_t)b * N * h + hd * D;
    const float* lse_b = lse + ((int64_t)b * H + hd) * N;
    const float* del_b = delta + ((int64_t)b * H + hd) * N;
    bf16x8 kf[NS], vf[NS];
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (j < N) {
        kf[s] = *reinterpret_cast<const bf16x8*>(base + h + (int64_t)j * rs + 16 * s + 8 * hb);
        vf[s] = *reinterpret_cast<const bf16x8*>(base + 2 * h + (int64_t)j * rs + 16 * s + 8 * hb);
      } else {
        for (int e = 0; e < 8; ++e) { kf[s][e] = (bf16)0.f; vf[s][e] = (bf16)0.f; }
      }
    }
    f32x16 dk[NC], dv[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int e = 0; e < 16; ++e) { dk[c][e] = 0.f; dv[c][e] = 0.f; }
    const int q_begin = causal ? (k0 / RS) * RS : 0;
    const int ntiles = (N - q_begin + RS - 1) / RS;
    L lq, ld;
    float st_l = 0.f, st_d = 0.f;
    auto load_stats = [&](int row0) {
      if (threadIdx.x < RS) {
        const int gi = row0 + threadIdx.x;
        st_l = (gi < N) ? lse_b[gi] * kLog2e : 0.f;
        st_d = (gi < N) ? del_b[gi] : 0.f;
      }
    };
    auto store_all = [&](int buf) {
      bf16* s0 = smem + buf * STAGE;
      lq.store_nat(s0); ld.store_nat(s0 + NSZ); lq.store_tr(s0 + 2 * NSZ); ld.store_tr(s0 + 2 * NSZ + TSZ);
      if (threadIdx.x < RS) { stat[(buf * 2 + 0) * RS + threadIdx.x] = st_l; stat[(buf * 2 + 1) * RS + threadIdx.x] = st_d; }
    };
    lq.load(base, rs, q_begin, N);
    ld.load(dob, (int64_t)h, q_begin, N);
    load_stats(q_begin);
    __syncthreads();
    store_all(0);
    __syncthreads();
    for (int t = 0; t < ntiles; ++t) {
      const int buf = t & 1;
      const bf16* qs = smem + buf * STAGE;
      const bf16* dos = qs + NSZ;
      const bf16* qt = qs + 2 * NSZ;
      const bf16* dot = qt + TSZ;
      const float* sl = stat + (buf * 2 + 0) * RS;
      const float* sd = stat + (buf * 2 + 1) * RS;
      if (t + 1 < ntiles) {
        lq.load(base, rs, q_begin + (t + 1) * RS, N);
        ld.load(dob, (int64_t)h, q_begin + (t + 1) * RS, N);
        load_stats(q_begin + (t + 1) * RS);
      }
      const int ib = q_begin + t * RS;
      if (!(causal && ib + 31 < j0w) && j0w < N) {            // otherwise every (i, j) here is masked
        f32x16 sacc, pacc;
#pragma unroll
        for (int e = 0; e < 16; ++e) { sacc[e] = 0.f; pacc[e] = 0.f; }
#pragma unroll
        for (int s = 0; s < NS; ++s) {
          sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat(qs, L::PN, lr, s, hb), kf[s], sacc, 0, 0, 0);
          pacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_nat(dos, L::PN, lr, s, hb), vf[s], pacc, 0, 0, 0);
        }
        float pv[16], ds[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int il = acc_row(r, hb), gi = ib + il;
          const bool masked = (gi >= N) || (j >= N) || (causal && j > gi);
          const float p = masked ? 0.f : fast_exp2(sacc[r] * scale_log2 - sl[il]);
          pv[r] = p;
          ds[r] = p * (pacc[r] - sd[il]);
        }
        const bf16x8 p0 = pack8(pv), p1 = pack8(pv + 8), d0 = pack8(ds), d1 = pack8(ds + 8);
#pragma unroll
        for (int c = 0; c < NC; ++c) {
          dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(dot, L::PT, 32 * c + lr, 0, 0, hb), p0, dv[c], 0, 0, 0);
          dv[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(dot, L::PT, 32 * c + lr, 0, 1, hb), p1, dv[c], 0, 0, 0);
          dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(qt, L::PT, 32 * c + lr, 0, 0, hb), d0, dk[c], 0, 0, 0);
          dk[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_tr(qt, L::PT, 32 * c + lr, 0, 1, hb), d1, dk[c], 0, 0, 0);
        }
      }
      if (t + 1 < ntiles) store_all(buf ^ 1);
      __syncthreads();
    }
    if (j < N) {
      bf16* out = dqkv + ((int64_t)b * N + j) * rs + hd * D;
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          bf16x4 vk, vv;
#pragma unroll
          for (int e = 0; e < 4; ++e) { vk[e] = (bf16)(dk[c][4 * g + e] * scale); vv[e] = (bf16)dv[c][4 * g + e]; }
          *reinterpret_cast<bf16x4*>(out + h + 32 * c + 8 * g + 4 * hb) = vk;
          *reinterpret_cast<bf16x4*>(out + 2 * h + 32 * c + 8 * g + 4 * hb) = vv;
        }
    }
  }
}

template <typename K>
mosaic_status set_smem(K kern, size_t bytes) {
  MOSAIC_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
  return MOSAIC_OK;
}

template <int D>
mosaic_status fwd_t(hipStream_t s, int quota, int B, int N, int H, int causal, const bf16* qkv, bf16* O, float* lse) {
  typedef TileLoader<64, D> L;
  constexpr size_t smem = 2 * (size_t)(64 * L::PN + D * L::PT) * sizeof(bf16);
  static bool once = false;
  if (!once) { MOSAIC_TRY(set_smem(attn_fwd_mfma<D>, smem)); once = true; }
  const int qtiles = (int)ceil_div(N, 128);
  const int64_t items = (int64_t)B * H * qtiles;
  const int grid = grid_for(quota, 2, items);
  attn_fwd_mfma<D><<<grid, 256, smem, s>>>(qkv, O, lse, B, N, H, causal, kLog2e / sqrtf((float)D), qtiles);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

template <int D>
mosaic_status bwd_t(hipStream_t s, int quota, int B, int N, int H, int causal, const bf16* qkv, const float* lse,
                    const bf16* dO, bf16* dqkv, const float* delta) {
  const int tiles = (int)ceil_div(N, 128);
  const int64_t items = (int64_t)B * H * tiles;
  const float scale = 1.0f / sqrtf((float)D);
  {
    typedef TileLoader<32, D> L;
    constexpr size_t smem = 2 * (size_t)(2 * 32 * L::PN + 2 * D * L::PT) * sizeof(bf16) + 2 * 2 * 32 * sizeof(float);
    static bool once = false;
    if (!once) { MOSAIC_TRY(set_smem(attn_bwd_dkv_mfma<D>, smem)); once = true; }
    const int grid = grid_for(quota, 2, items);
    attn_bwd_dkv_mfma<D><<<grid, 256, smem, s>>>(qkv, dO, lse, delta, dqkv, B, N, H, causal, scale, tiles);
    MOSAIC_LAUNCH_CHECK();
  }
  {
    typedef TileLoader<64, D> L;
    constexpr size_t smem = 2 * (size_t)(2 * 64 * L::PN + D * L::PT) * sizeof(bf16);
    static bool once = false;
    if (!once) { MOSAIC_TRY(set_smem(attn_bwd_dq_mfma<D>, smem)); once = true; }
    const int grid = grid_for(quota, (smem > 80 * 1024) ? 1 : 2, items);
    attn_bwd_dq_mfma<D><<<grid, 256, smem, s>>>(qkv, dO, lse, delta, dqkv, B, N, H, causal, scale, tiles);
    MOSAIC_LAUNCH_CHECK();
  }
  return MOSAIC_OK;
}

}  // namespace

bool attention_mfma_supported(int dtype, int d) { return dtype == MOSAIC_BF16 && (d == 64 || d == 128); }

mosaic_status launch_attention_fwd_mfma(hipStream_t s, int quota, int B, int N, int H, int d, int causal,
                                        const void* qkv, void* O, float* lse) {
  if (d == 64) return fwd_t<64>(s, quota, B, N, H, causal, (const bf16*)qkv, (bf16*)O, lse);
  return fwd_t<128>(s, quota, B, N, H, causal, (const bf16*)qkv, (bf16*)O, lse);
}

mosaic_status launch_attention_bwd_mfma(hipStream_t s, int quota, int B, int N, int H, int d, int causal,
                                        const void* qkv, const float* lse, const void* dO, void* dqkv,
                                        const float* delta) {
  if (d == 64) return bwd_t<64>(s, quota, B, N, H, causal, (const bf16*)qkv, lse, (const bf16*)dO, (bf16*)dqkv, delta);
  return bwd_t<128>(s, quota, B, N, H, causal, (const bf16*)qkv, lse, (const bf16*)dO, (bf16*)dqkv, delta);
}
