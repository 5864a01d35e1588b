// Reference-grade attention kernels: plain FMA arithmetic in fp32 with online softmax,
// for the fp32 path and for head sizes / dtypes the MFMA kernels do not cover.
//
// Forward: a workgroup owns 16 query rows of one (sample, head) and streams key/value
// blocks of 32.  Backward is split so that no atomics are needed and every sum has a
// fixed order: one kernel owns 16 keys and streams query blocks (dK, dV), the other owns
// 16 queries and streams key blocks (dQ).  P is recomputed from the saved row
// log-sum-exp; D_i = sum_c dO_ic O_ic comes from a small per-row kernel.
#include "kernels.h"

namespace {

constexpr int OWN = 16;     // rows owned by a workgroup
constexpr int STR = 32;     // rows of the streamed block
constexpr int DMAX = 128;

template <typename T>
__device__ __forceinline__ void load_rows(float* dst, int pitch, const T* src, int64_t row_stride,
                                          int first, int count, int limit, int d) {
  // rows [first, first+count) of a [*, d] slice with given row stride; rows >= limit -> 0
  for (int idx = threadIdx.x; idx < count * d; idx += 256) {
    const int r = idx / d, c = idx - r * d;
    const int g = first + r;
    dst[r * pitch + c] = (g < limit) ? to_f32(src[(int64_t)g * row_stride + c]) : 0.f;
  }
}

__device__ __forceinline__ float group16_max(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float group16_sum(float v) {
#pragma unroll
  for (int o = 8; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <typename T>
__global__ __launch_bounds__(256) void attn_fwd_simple(const T* __restrict__ qkv, T* __restrict__ O,
                                                       float* __restrict__ lse, int B, int N, int H, int Hkv, int d,
                                                       int causal, float scale, int qtiles) {
  __shared__ float Qs[OWN * DMAX];
  __shared__ float Ks[STR * (DMAX + 1)];
  __shared__ float Vs[STR * (DMAX + 1)];
  __shared__ float Ss[OWN * STR];
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * d, ko = H * d, vo = (H + Hkv) * d, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * d;
  const int t = threadIdx.x;
  const int i = t >> 4, sub = t & 15;          // query row in tile, position in 16-lane group
  const int items = B * H * qtiles;
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int qt = item % qtiles, hd = (item / qtiles) % H, b = item / (qtiles * H);
    const int q0 = qt * OWN;
    const T* rowb = qkv + (int64_t)b * N * rs;
    const T* base = rowb + hd * d;
    __syncthreads();
    load_rows(Qs, d, base, rs, q0, OWN, N, d);
    float o[DMAX / 16];
#pragma unroll
    for (int c = 0; c < DMAX / 16; ++c) o[c] = 0.f;
    float m = -INFINITY, l = 0.f;
    const int kv_end = causal ? min(N, q0 + OWN) : N;
    for (int k0 = 0; k0 < kv_end; k0 += STR) {
      __syncthreads();
      load_rows(Ks, d + 1, rowb + ko + (hd / GQ) * d, rs, k0, STR, N, d);
      load_rows(Vs, d + 1, rowb + vo + (hd / GQ) * d, rs, k0, STR, N, d);
      __syncthreads();
      float s[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int j = sub * 2 + u;
        float acc = 0.f;
        for (int c = 0; c < d; ++c) acc = fmaf(Qs[i * d + c], Ks[j * (d + 1) + c], acc);
        const int gj = k0 + j, gi = q0 + i;
        const bool masked = (gj >= N) || (causal && gj > gi);
        s[u] = masked ? -INFINITY : acc * scale;
      }
      const float bm = group16_max(fmaxf(s[0], s[1]));
      const float mn = fmaxf(m, bm);
      // a row that has seen no unmasked key yet keeps m = -inf; exp(-inf - -inf) is avoided
      const float corr = (m == -INFINITY) ? 0.f : expf(m - mn);
      float p0 = (s[0] == -INFINITY) ? 0.f : expf(s[0] - mn);
      float p1 = (s[1] == -INFINITY) ? 0.f : expf(s[1] - mn);
      Ss[i * STR + sub * 2] = p0;
      Ss[i * STR + sub * 2 + 1] = p1;
      const float bs = group16_sum(p0 + p1);
      l = l * corr + bs;
      m = mn;
      __syncthreads();
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) {
          float acc = o[cc] * corr;
          for (int j = 0; j < STR; ++j) acc = fmaf(Ss[i * STR + j], Vs[j * (d + 1) + c], acc);
          o[cc] = acc;
        }
      }
    }
    const int gi = q0 + i;
    if (gi < N) {
      const float inv = 1.0f / l;
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) O[((int64_t)b * N + gi) * h + hd * d + c] = from_f32<T>(o[cc] * inv);
      }
      if (sub == 0) lse[((int64_t)b * H + hd) * N + gi] = m + logf(l);
    }
  }
}

// delta[b,hd,i] = sum_c dO[b,i,hd,c] * O[b,i,hd,c]; one 16-lane group per (row, head)
template <typename T>
__global__ __launch_bounds__(256) void attn_delta_kernel(const T* __restrict__ O, const T* __restrict__ dO,
                                                         float* __restrict__ delta, int B, int N, int H, int d) {
  const int64_t items = (int64_t)B * N * H;
  const int sub = threadIdx.x & 15;
  for (int64_t it = (int64_t)blockIdx.x * 16 + (threadIdx.x >> 4); it < items; it += (int64_t)gridDim.x * 16) {
    const int hd = (int)(it % H);
    const int64_t row = it / H;           // b*N + i
    const int64_t off = row * H * d + (int64_t)hd * d;
    float acc = 0.f;
    for (int c = sub; c < d; c += 16) acc = fmaf(to_f32(dO[off + c]), to_f32(O[off + c]), acc);
    acc = group16_sum(acc);
    if (sub == 0) {
      const int b = (int)(row / N), i = (int)(row % N);
      delta[((int64_t)b * H + hd) * N + i] = acc;
    }
  }
}

// dK, dV: workgroup owns OWN keys, streams STR queries at a time in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_kv_simple(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                          const float* __restrict__ lse, const float* __restrict__ delta,
                                                          T* __restrict__ dqkv, int B, int N, int H, int Hkv, int d, int causal,
                                                          float scale, int ktiles) {
  __shared__ float Ks[OWN * DMAX];
  __shared__ float Vs[OWN * DMAX];
  __shared__ float Qs[STR * (DMAX + 1)];
  __shared__ float Ds[STR * (DMAX + 1)];
  __shared__ float Ps[STR * OWN];
  __shared__ float dSs[STR * OWN];
  __shared__ float Ls[STR], Dl[STR];
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * d, ko = H * d, vo = (H + Hkv) * d, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * d;
  const int t = threadIdx.x;
  const int items = B * Hkv * ktiles;
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int kt = item % ktiles, kvh = (item / ktiles) % Hkv, b = item / (ktiles * Hkv);
    const int j0 = kt * OWN;
    const T* rowb = qkv + (int64_t)b * N * rs;
    __syncthreads();
    load_rows(Ks, d, rowb + ko + kvh * d, rs, j0, OWN, N, d);
    load_rows(Vs, d, rowb + vo + kvh * d, rs, j0, OWN, N, d);
    const int jo = t >> 4, sub = t & 15;       // accumulation mapping: key jo, columns sub+16*cc
    float dk[DMAX / 16], dv[DMAX / 16];
#pragma unroll
    for (int c = 0; c < DMAX / 16; ++c) { dk[c] = 0.f; dv[c] = 0.f; }
    const int q_begin = causal ? (j0 / STR) * STR : 0;
    // every query head of the group in turn, query blocks ascending inside a head
    for (int g = 0; g < GQ; ++g)
    for (int i0 = q_begin; i0 < N; i0 += STR) {
      const int hd = kvh * GQ + g;
      const T* base = rowb + hd * d;
      const T* dob = dO + (int64_t)b * N * h + hd * d;
      __syncthreads();
      load_rows(Qs, d + 1, base, rs, i0, STR, N, d);
      load_rows(Ds, d + 1, dob, (int64_t)h, i0, STR, N, d);
      if (t < STR) {
        const int gi = i0 + t;
        Ls[t] = (gi < N) ? lse[((int64_t)b * H + hd) * N + gi] : 0.f;
        Dl[t] = (gi < N) ? delta[((int64_t)b * H + hd) * N + gi] : 0.f;
      }
      __syncthreads();
      // scores: 32 x 16 = 512 entries, two per thread
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int e = t * 2 + u;
        const int i = e / OWN, j = e % OWN;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < d; ++c) {
          s = fmaf(Qs[i * (d + 1) + c], Ks[j * d + c], s);
          dp = fmaf(Ds[i * (d + 1) + c], Vs[j * d + c], dp);
        }
        const int gi = i0 + i, gj = j0 + j;
        const bool masked = (gi >= N) || (gj >= N) || (causal && gj > gi);
        const float p = masked ? 0.f : expf(s * scale - Ls[i]);
        Ps[e] = p;
        dSs[e] = p * (dp - Dl[i]);
      }
      __syncthreads();
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) {
          float av = dv[cc], ak = dk[cc];
          for (int i = 0; i < STR; ++i) {
            av = fmaf(Ps[i * OWN + jo], Ds[i * (d + 1) + c], av);
            ak = fmaf(dSs[i * OWN + jo], Qs[i * (d + 1) + c], ak);
          }
          dv[cc] = av; dk[cc] = ak;
        }
      }
    }
    const int gj = j0 + jo;
    if (gj < N) {
      T* out = dqkv + ((int64_t)b * N + gj) * rs + kvh * d;
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) { out[ko + c] = from_f32<T>(dk[cc] * scale); out[vo + c] = from_f32<T>(dv[cc]); }
      }
    }
  }
}

// dQ: workgroup owns OWN queries, streams STR keys at a time in ascending order.
template <typename T>
__global__ __launch_bounds__(256) void attn_bwd_q_simple(const T* __restrict__ qkv, const T* __restrict__ dO,
                                                         const float* __restrict__ lse, const float* __restrict__ delta,
                                                         T* __restrict__ dqkv, int B, int N, int H, int Hkv, int d, int causal,
                                                         float scale, int qtiles) {
  __shared__ float Qs[OWN * DMAX];
  __shared__ float Ds[OWN * DMAX];
  __shared__ float Ks[STR * (DMAX + 1)];
  __shared__ float Vs[STR * (DMAX + 1)];
  __shared__ float dSs[OWN * STR];
  // rows are [q (H heads) | k (Hkv heads) | v (Hkv heads)]; query head t uses key/value head t / (H/Hkv)
  const int h = H * d, ko = H * d, vo = (H + Hkv) * d, GQ = H / Hkv;
  const int64_t rs = (int64_t)(H + 2 * Hkv) * d;
  const int t = threadIdx.x;
  const int i = t >> 4, sub = t & 15;
  const int items = B * H * qtiles;
  for (int item = blockIdx.x; item < items; item += gridDim.x) {
    const int qt = item % qtiles, hd = (item / qtiles) % H, b = item / (qtiles * H);
    const int q0 = qt * OWN;
    const T* rowb = qkv + (int64_t)b * N * rs;
    const T* base = rowb + hd * d;
    const T* dob = dO + (int64_t)b * N * h + hd * d;
    __syncthreads();
    load_rows(Qs, d, base, rs, q0, OWN, N, d);
    load_rows(Ds, d, dob, (int64_t)h, q0, OWN, N, d);
    const int gi = q0 + i;
    const float li = (gi < N) ? lse[((int64_t)b * H + hd) * N + gi] : 0.f;
    const float di = (gi < N) ? delta[((int64_t)b * H + hd) * N + gi] : 0.f;
    float dq[DMAX / 16];
#pragma unroll
    for (int c = 0; c < DMAX / 16; ++c) dq[c] = 0.f;
    const int kv_end = causal ? min(N, q0 + OWN) : N;
    for (int k0 = 0; k0 < kv_end; k0 += STR) {
      __syncthreads();
      load_rows(Ks, d + 1, rowb + ko + (hd / GQ) * d, rs, k0, STR, N, d);
      load_rows(Vs, d + 1, rowb + vo + (hd / GQ) * d, rs, k0, STR, N, d);
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        const int j = sub * 2 + u;
        float s = 0.f, dp = 0.f;
        for (int c = 0; c < d; ++c) {
          s = fmaf(Qs[i * d + c], Ks[j * (d + 1) + c], s);
          dp = fmaf(Ds[i * d + c], Vs[j * (d + 1) + c], dp);
        }
        const int gj = k0 + j;
        const bool masked = (gi >= N) || (gj >= N) || (causal && gj > gi);
        const float p = masked ? 0.f : expf(s * scale - li);
        dSs[i * STR + j] = p * (dp - di);
      }
      __syncthreads();
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) {
          float a = dq[cc];
          for (int j = 0; j < STR; ++j) a = fmaf(dSs[i * STR + j], Ks[j * (d + 1) + c], a);
          dq[cc] = a;
        }
      }
    }
    if (gi < N) {
      T* out = dqkv + ((int64_t)b * N + gi) * rs + hd * d;
#pragma unroll
      for (int cc = 0; cc < DMAX / 16; ++cc) {
        const int c = sub + 16 * cc;
        if (c < d) out[c] = from_f32<T>(dq[cc] * scale);
      }
    }
  }
}

}  // namespace

mosaic_status launch_attention_fwd_simple(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d,
                                          int causal, const void* qkv, void* O, float* lse) {
  const int qtiles = (int)ceil_div(N, OWN);
  const int64_t items = (int64_t)B * H * qtiles;
  if (items == 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 2, items);
  const float scale = 1.0f / sqrtf((float)d);
  if (dtype == MOSAIC_BF16)
    attn_fwd_simple<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, (bf16*)O, lse, B, N, H, Hkv, d, causal, scale, qtiles);
  else
    attn_fwd_simple<float><<<grid, 256, 0, s>>>((const float*)qkv, (float*)O, lse, B, N, H, Hkv, d, causal, scale, qtiles);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_attention_delta(hipStream_t s, int quota, int dtype, int B, int N, int H, int d,
                                     const void* O, const void* dO, float* delta) {
  const int64_t items = (int64_t)B * N * H;
  if (items == 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 8, ceil_div(items, 16));
  if (dtype == MOSAIC_BF16)
    attn_delta_kernel<bf16><<<grid, 256, 0, s>>>((const bf16*)O, (const bf16*)dO, delta, B, N, H, d);
  else
    attn_delta_kernel<float><<<grid, 256, 0, s>>>((const float*)O, (const float*)dO, delta, B, N, H, d);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_attention_bwd_simple(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d,
                                          int causal, const void* qkv, const void* O, const float* lse,
                                          const void* dO, void* dqkv, float* delta) {
  MOSAIC_TRY(launch_attention_delta(s, quota, dtype, B, N, H, d, O, dO, delta));
  const int tiles = (int)ceil_div(N, OWN);
  const int64_t items = (int64_t)B * H * tiles;
  if (items == 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 1, items);
  const float scale = 1.0f / sqrtf((float)d);
  if (dtype == MOSAIC_BF16) {
    attn_bwd_kv_simple<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, (const bf16*)dO, lse, delta, (bf16*)dqkv, B, N, H, Hkv, d, causal, scale, tiles);
    attn_bwd_q_simple<bf16><<<grid, 256, 0, s>>>((const bf16*)qkv, (const bf16*)dO, lse, delta, (bf16*)dqkv, B, N, H, Hkv, d, causal, scale, tiles);
  } else {
    attn_bwd_kv_simple<float><<<grid, 256, 0, s>>>((const float*)qkv, (const float*)dO, lse, delta, (float*)dqkv, B, N, H, Hkv, d, causal, scale, tiles);
    attn_bwd_q_simple<float><<<grid, 256, 0, s>>>((const float*)qkv, (const float*)dO, lse, delta, (float*)dqkv, B, N, H, Hkv, d, causal, scale, tiles);
  }
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}
