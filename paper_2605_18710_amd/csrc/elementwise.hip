// Bandwidth-bound kernels of the module step: LayerNorm / RMSNorm forward and backward
// (with fused residual add and fixed-order column reductions), GELU / SwiGLU forward and
// backward, MSE loss and gradient, column sums for bias gradients, and the stem kernels
// (patch unfold, position table, embedding gather / owner-computes scatter).
//
// All reductions run in an order fixed by the problem shape alone: persistent grids only
// decide which workgroup handles a work item, so results are bit-identical for any quota.
#include "activations.h"
#include "kernels.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

// ------------------------------------------------------------------------ norm forward
// One wave per row; the row lives in registers (NV 16-byte vectors per lane), so x is
// read from HBM once.  LayerNorm: biased variance around the mean; RMSNorm: mean square.
template <typename T, int NORM, int NV>
__global__ __launch_bounds__(kThreads) void norm_fwd_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const T* __restrict__ beta,
    T* __restrict__ y, float* __restrict__ stats, int64_t rows, int h, float eps) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_h = 1.0f / (float)h;
  for (int64_t row = (int64_t)blockIdx.x * kWaves + wave; row < rows;
       row += (int64_t)gridDim.x * kWaves) {
    Vec16<T> v[NV];
    float s = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VN;
      if (c < h) {
        v[j].load(x + row * h + c);
#pragma unroll
        for (int i = 0; i < VN; ++i) s += (NORM == MOSAIC_LAYERNORM) ? v[j].get(i) : v[j].get(i) * v[j].get(i);
      }
    }
    s = wave_sum(s);
    float mean = 0.f, rstd;
    if (NORM == MOSAIC_LAYERNORM) {
      mean = s * inv_h;
      float q = 0.f;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VN;
        if (c < h) {
#pragma unroll
          for (int i = 0; i < VN; ++i) { const float dlt = v[j].get(i) - mean; q += dlt * dlt; }
        }
      }
      q = wave_sum(q);
      rstd = 1.0f / sqrtf(q * inv_h + eps);
    } else {
      rstd = 1.0f / sqrtf(s * inv_h + eps);
    }
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VN;
      if (c < h) {
        Vec16<T> g, b, o;
        g.load(gamma + c);
        if (NORM == MOSAIC_LAYERNORM) b.load(beta + c);
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          float r = (v[j].get(i) - mean) * rstd * g.get(i);
          if (NORM == MOSAIC_LAYERNORM) r += b.get(i);
          o.set(i, r);
        }
        o.store(y + row * h + c);
      }
    }
    if (lane == 0) { stats[row * 2] = mean; stats[row * 2 + 1] = rstd; }
  }
}

// ----------------------------------------------------------------------- norm backward
// dx: one wave per row, the row of x and dy held in registers (read once), optional
// residual added on the way out.
template <typename T, int NORM, int NV>
__global__ __launch_bounds__(kThreads) void norm_bwd_dx_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const float* __restrict__ stats,
    const T* __restrict__ dy, const T* __restrict__ R, T* __restrict__ dx, int64_t rows, int h) {
  constexpr int VN = Vec16<T>::N;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_h = 1.0f / (float)h;
  Vec16<T> g[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = (j * 64 + lane) * VN;
    if (c < h) g[j].load(gamma + c);
  }
  for (int64_t row = (int64_t)blockIdx.x * kWaves + wave; row < rows; row += (int64_t)gridDim.x * kWaves) {
    const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
    Vec16<T> xv[NV], dv[NV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VN;
      if (c < h) {
        xv[j].load(x + row * h + c);
        dv[j].load(dy + row * h + c);
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          const float t = dv[j].get(i) * g[j].get(i);
          if (NORM == MOSAIC_LAYERNORM) {
            const float xh = (xv[j].get(i) - mean) * rstd;
            s1 += t; s2 += t * xh;
          } else {
            s2 += t * xv[j].get(i);
          }
        }
      }
    }
    if (NORM == MOSAIC_LAYERNORM) s1 = wave_sum(s1) * inv_h;
    s2 = wave_sum(s2) * inv_h;
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const int c = (j * 64 + lane) * VN;
      if (c < h) {
        Vec16<T> o, rv;
        if (R) rv.load(R + row * h + c);
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          const float xr = xv[j].get(i);
          const float t = dv[j].get(i) * g[j].get(i);
          float r;
          if (NORM == MOSAIC_LAYERNORM) r = (t - s1 - (xr - mean) * rstd * s2) * rstd;
          else r = rstd * t - rstd * rstd * rstd * xr * s2;
          if (R) r += rv.get(i);
          o.set(i, r);
        }
        o.store(dx + row * h + c);
      }
    }
  }
}

// dx and the dgamma / dbeta partial sums in one pass over x and dy.  Work item = row
// partition p (rp rows; rp depends on the row count alone).  Wave w of the workgroup takes
// rows r0+w, r0+w+4, ... in ascending order, holds the row of x and dy in registers, writes
// dx and adds dy*xhat (and dy) into per-lane column accumulators.  The four waves'
// accumulators are added in wave order through LDS, one 64-lane column slab at a time, and
// land in scratch[p][2][h]; reduce_partials_kernel adds the partitions in a fixed order.
// CS: the column sums of the values written to dx (as stored, after rounding) are formed the
// same way in a third slab, scratch[p][3][h]: dx is the output gradient of the linear layer in
// front of the residual branch, so this is that layer's bias gradient, without another pass.
template <typename T, int NORM, int NV, bool CS = false>
__global__ __launch_bounds__(kThreads) void norm_bwd_fused_kernel(
    const T* __restrict__ x, const T* __restrict__ gamma, const float* __restrict__ stats,
    const T* __restrict__ dy, const T* __restrict__ R, T* __restrict__ dx, float* __restrict__ scratch,
    int64_t rows, int h, int rp, int np) {
  constexpr int VN = Vec16<T>::N;
  constexpr int NSUM = (NORM == MOSAIC_LAYERNORM) ? 2 : 1;
  constexpr int NSLAB = CS ? 3 : 2;                    // slabs per partition in scratch
  __shared__ float red[kWaves - 1][NSUM + (CS ? 1 : 0)][64 * VN];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float inv_h = 1.0f / (float)h;
  Vec16<T> g[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    const int c = (j * 64 + lane) * VN;
    if (c < h) g[j].load(gamma + c);
  }
  for (int p = blockIdx.x; p < np; p += gridDim.x) {
    float ag[NV][VN], ab[NSUM == 2 ? NV : 1][VN], ax[CS ? NV : 1][VN];
#pragma unroll
    for (int j = 0; j < NV; ++j)
#pragma unroll
      for (int i = 0; i < VN; ++i) { ag[j][i] = 0.f; if (NSUM == 2) ab[j][i] = 0.f; if (CS) ax[j][i] = 0.f; }
    const int64_t r0 = (int64_t)p * rp;
    const int64_t r1 = (r0 + rp < rows) ? r0 + rp : rows;
    for (int64_t row = r0 + wave; row < r1; row += kWaves) {
      const float mean = stats[row * 2], rstd = stats[row * 2 + 1];
      Vec16<T> xv[NV], dv[NV];
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VN;
        if (c < h) {
          xv[j].load(x + row * h + c);
          dv[j].load(dy + row * h + c);
        }
      }
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VN;
        if (c < h) {
#pragma unroll
          for (int i = 0; i < VN; ++i) {
            const float d = dv[j].get(i);
            const float t = d * g[j].get(i);
            if (NORM == MOSAIC_LAYERNORM) {
              const float xh = (xv[j].get(i) - mean) * rstd;
              s1 += t; s2 += t * xh;
              ag[j][i] += d * xh; ab[NSUM == 2 ? j : 0][i] += d;
            } else {
              s2 += t * xv[j].get(i);
              ag[j][i] += d * xv[j].get(i) * rstd;
            }
          }
        }
      }
      if (NORM == MOSAIC_LAYERNORM) s1 = wave_sum(s1) * inv_h;
      s2 = wave_sum(s2) * inv_h;
#pragma unroll
      for (int j = 0; j < NV; ++j) {
        const int c = (j * 64 + lane) * VN;
        if (c < h) {
          Vec16<T> o, rv;
          if (R) rv.load(R + row * h + c);
#pragma unroll
          for (int i = 0; i < VN; ++i) {
            const float xr = xv[j].get(i);
            const float t = dv[j].get(i) * g[j].get(i);
            float r;
            if (NORM == MOSAIC_LAYERNORM) r = (t - s1 - (xr - mean) * rstd * s2) * rstd;
            else r = rstd * t - rstd * rstd * rstd * xr * s2;
            if (R) r += rv.get(i);
            o.set(i, r);
            if (CS) ax[CS ? j : 0][i] += o.get(i);
          }
          o.store(dx + row * h + c);
        }
      }
    }
    // waves 1..3 hand their sums to wave 0, slab by slab; every wave passes every barrier
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      if (wave > 0) {
#pragma unroll
        for (int i = 0; i < VN; ++i) {
          red[wave - 1][0][i * 64 + lane] = ag[j][i];
          if (NSUM == 2) red[wave - 1][NSUM - 1][i * 64 + lane] = ab[NSUM == 2 ? j : 0][i];
          if (CS) red[wave - 1][NSUM][i * 64 + lane] = ax[CS ? j : 0][i];
        }
      }
      __syncthreads();
      if (wave == 0) {
        const int c = (j * 64 + lane) * VN;
        if (c < h) {
#pragma unroll
          for (int i = 0; i < VN; ++i) {
            float a = ag[j][i], b = (NSUM == 2) ? ab[NSUM == 2 ? j : 0][i] : 0.f, xs = CS ? ax[CS ? j : 0][i] : 0.f;
#pragma unroll
            for (int w = 0; w < kWaves - 1; ++w) {
              a += red[w][0][i * 64 + lane];
              if (NSUM == 2) b += red[w][NSUM - 1][i * 64 + lane];
              if (CS) xs += red[w][NSUM][i * 64 + lane];
            }
            scratch[((int64_t)p * NSLAB + 0) * h + c + i] = a;
            if (NSUM == 2) scratch[((int64_t)p * NSLAB + 1) * h + c + i] = b;
            if (CS) scratch[((int64_t)p * NSLAB + 2) * h + c + i] = xs;
          }
        }
      }
      __syncthreads();
    }
  }
}

// dgamma / dbeta partial column sums: work item = (row partition p, tile of 256 column
// vectors); a thread owns VN columns and walks the partition's rows in ascending order.
// scratch[p][2][h]; the partitions are added in a fixed order by reduce_partials_kernel.
template <typename T, int NORM>
__global__ __launch_bounds__(kThreads) void norm_colgrad_partial_kernel(
    const T* __restrict__ x, const float* __restrict__ stats, const T* __restrict__ dy,
    float* __restrict__ scratch, int64_t rows, int h, int rp, int np, int ctiles) {
  constexpr int VN = Vec16<T>::N;
  const int64_t items = (int64_t)np * ctiles;
  for (int64_t it = blockIdx.x; it < items; it += gridDim.x) {
    const int p = (int)(it / ctiles), ct = (int)(it - (int64_t)p * ctiles);
    const int c = (ct * kThreads + threadIdx.x) * VN;
    if (c >= h) continue;
    float ag[VN], ab[VN];
#pragma unroll
    for (int i = 0; i < VN; ++i) { ag[i] = 0.f; ab[i] = 0.f; }
    const int64_t r0 = (int64_t)p * rp;
    const int64_t r1 = (r0 + rp < rows) ? r0 + rp : rows;
    auto add_row = [&](const Vec16<T>& xv, const Vec16<T>& dv, float mean, float rstd) {
#pragma unroll
      for (int i = 0; i < VN; ++i) {
        const float d = dv.get(i);
        if (NORM == MOSAIC_LAYERNORM) { ag[i] += d * ((xv.get(i) - mean) * rstd); ab[i] += d; }
        else ag[i] += d * xv.get(i) * rstd;
      }
    };
    int64_t row = r0;
    // four rows requested together, added in ascending row order
    for (; row + 4 <= r1; row += 4) {
      Vec16<T> xv[4], dv[4];
      float mean[4], rstd[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        xv[u].load(x + (row + u) * h + c);
        dv[u].load(dy + (row + u) * h + c);
        mean[u] = stats[(row + u) * 2]; rstd[u] = stats[(row + u) * 2 + 1];
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) add_row(xv[u], dv[u], mean[u], rstd[u]);
    }
    for (; row < r1; ++row) {
      Vec16<T> xv, dv;
      xv.load(x + row * h + c);
      dv.load(dy + row * h + c);
      add_row(xv, dv, stats[row * 2], stats[row * 2 + 1]);
    }
#pragma unroll
    for (int i = 0; i < VN; ++i) {
      scratch[((int64_t)p * 2 + 0) * h + c + i] = ag[i];
      scratch[((int64_t)p * 2 + 1) * h + c + i] = ab[i];
    }
  }
}

// out[col] = sum_p partial[p*ld + col], partitions taken in 8 contiguous slices that are
// added in slice order: a fixed tree that depends on np only.  Columns [0, split) go to
// out0, columns [split, split2) to out1, columns [split2, ncols) to out2; a null destination
// skips its columns.
template <typename T>
__global__ __launch_bounds__(kThreads) void reduce_partials_kernel(
    const float* __restrict__ partial, int np, int64_t ld, int64_t ncols, int64_t split,
    T* __restrict__ out0, T* __restrict__ out1, int64_t split2 = INT64_MAX, T* __restrict__ out2 = nullptr) {
  __shared__ float red[8][32];
  const int cl = threadIdx.x & 31, sl = threadIdx.x >> 5;
  const int per = (np + 7) / 8;
  const int64_t groups = (ncols + 31) / 32;
  for (int64_t gidx = blockIdx.x; gidx < groups; gidx += gridDim.x) {
    const int64_t col = gidx * 32 + cl;
    float acc = 0.f;
    T* dst = nullptr;
    if (col < ncols) dst = col < split ? out0 + col : col < split2 ? (out1 ? out1 + (col - split) : nullptr) : (out2 ? out2 + (col - split2) : nullptr);
    if (dst) {
      const int p1 = (sl + 1) * per < np ? (sl + 1) * per : np;
      int p = sl * per;
      // eight independent requests in flight, added in ascending p as before
      for (; p + 8 <= p1; p += 8) {
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partial[(int64_t)(p + u) * ld + col];
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
      }
      for (; p < p1; ++p) acc += partial[(int64_t)p * ld + col];
    }
    red[sl][cl] = acc;
    __syncthreads();
    if (sl == 0 && dst) {
      float t = 0.f;
#pragma unroll
      for (int q = 0; q < 8; ++q) t += red[q][cl];
      *dst = from_f32<T>(t);
    }
    __syncthreads();
  }
}

// -------------------------------------------------------------------------- activations
// gelu_f, gelu_grad_f, sigmoid_f, swiglu_f: activations.h

template <typename T>
__global__ __launch_bounds__(kThreads) void gelu_fwd_kernel(const T* __restrict__ z, T* __restrict__ a, int64_t nvec) {
  constexpr int VN = Vec16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    Vec16<T> v, o;
    v.load(z + i * VN);
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, gelu_f(v.get(k)));
    o.store(a + i * VN);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gelu_bwd_kernel(const T* __restrict__ z, const T* __restrict__ da,
                                                            T* __restrict__ dz, int64_t nvec) {
  constexpr int VN = Vec16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    Vec16<T> v, d, o;
    v.load(z + i * VN);
    d.load(da + i * VN);
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, d.get(k) * gelu_grad_f(v.get(k)));
    o.store(dz + i * VN);
  }
}

// dz = da * gelu'(z) and, in the same pass, the partial column sums of dz as stored (the bias
// gradient of the linear layer that produced z): work item = (row partition p, tile of 256
// column vectors); a thread owns VN columns and walks the partition's rows in ascending order,
// exactly as colsum_partial_kernel does over the stored dz, so the sums have the same bits.
template <typename T>
__global__ __launch_bounds__(kThreads) void gelu_bwd_colsum_kernel(const T* __restrict__ z, const T* __restrict__ da,
                                                                   T* __restrict__ dz, float* __restrict__ partial,
                                                                   int64_t rows, int64_t n, int rp, int np, int ctiles) {
  constexpr int VN = Vec16<T>::N;
  const int64_t items = (int64_t)np * ctiles;
  for (int64_t it = blockIdx.x; it < items; it += gridDim.x) {
    const int p = (int)(it / ctiles), ct = (int)(it - (int64_t)p * ctiles);
    const int64_t c = ((int64_t)ct * kThreads + threadIdx.x) * VN;
    if (c >= n) continue;
    float acc[VN];
#pragma unroll
    for (int k = 0; k < VN; ++k) acc[k] = 0.f;
    const int64_t r0 = (int64_t)p * rp;
    const int64_t r1 = (r0 + rp < rows) ? r0 + rp : rows;
    auto one = [&](const Vec16<T>& zv, const Vec16<T>& dv, int64_t r) {
      Vec16<T> o;
#pragma unroll
      for (int k = 0; k < VN; ++k) { o.set(k, dv.get(k) * gelu_grad_f(zv.get(k))); acc[k] += o.get(k); }
      o.store(dz + r * n + c);
    };
    int64_t r = r0;
    for (; r + 4 <= r1; r += 4) {          // four rows requested together, taken in ascending order
      Vec16<T> zv[4], dv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) { zv[u].load(z + (r + u) * n + c); dv[u].load(da + (r + u) * n + c); }
#pragma unroll
      for (int u = 0; u < 4; ++u) one(zv[u], dv[u], r + u);
    }
    for (; r < r1; ++r) {
      Vec16<T> zv, dv;
      zv.load(z + r * n + c); dv.load(da + r * n + c);
      one(zv, dv, r);
    }
#pragma unroll
    for (int k = 0; k < VN; ++k) partial[(int64_t)p * n + c + k] = acc[k];
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void swiglu_fwd_kernel(const T* __restrict__ gu, T* __restrict__ a,
                                                              int64_t rows, int fv) {
  constexpr int VN = Vec16<T>::N;
  const int64_t nvec = rows * fv;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / fv;
    const int64_t c = (i - r * fv) * VN;
    const int64_t f = (int64_t)fv * VN;
    Vec16<T> g, u, o;
    g.load(gu + r * 2 * f + c);
    u.load(gu + r * 2 * f + f + c);
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, swiglu_f(g.get(k), u.get(k)));
    o.store(a + r * f + c);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void swiglu_bwd_kernel(const T* __restrict__ gu, const T* __restrict__ da,
                                                              T* __restrict__ dgu, int64_t rows, int fv) {
  constexpr int VN = Vec16<T>::N;
  const int64_t nvec = rows * fv;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    const int64_t r = i / fv;
    const int64_t c = (i - r * fv) * VN;
    const int64_t f = (int64_t)fv * VN;
    Vec16<T> g, u, d, og, ou;
    g.load(gu + r * 2 * f + c);
    u.load(gu + r * 2 * f + f + c);
    d.load(da + r * f + c);
#pragma unroll
    for (int k = 0; k < VN; ++k) {
      const float z = g.get(k), s = sigmoid_f(z);
      og.set(k, d.get(k) * u.get(k) * (s * (1.0f + z * (1.0f - s))));
      ou.set(k, d.get(k) * (z * s));
    }
    og.store(dgu + r * 2 * f + c);
    ou.store(dgu + r * 2 * f + f + c);
  }
}

// ---------------------------------------------------------------------------------- MSE
constexpr int kMsePartials = 1024;

__device__ __forceinline__ float block_sum_fixed(float v, float* red) {
  // fixed-shape reduction: butterfly inside each wave, then waves added in index order
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (lane == 0) red[wave] = v;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < kWaves; ++w) t += red[w];
  __syncthreads();
  return t;
}

template <typename T>
__global__ __launch_bounds__(kThreads) void mse_kernel(const T* __restrict__ y, const T* __restrict__ tg,
                                                       T* __restrict__ dy, float* __restrict__ partial,
                                                       int64_t nvec, int64_t chunk, float scale) {
  constexpr int VN = Vec16<T>::N;
  __shared__ float red[kWaves];
  for (int p = blockIdx.x; p < kMsePartials; p += gridDim.x) {
    const int64_t v0 = (int64_t)p * chunk;
    const int64_t v1 = (v0 + chunk < nvec) ? v0 + chunk : nvec;
    float acc = 0.f;
    for (int64_t i = v0 + threadIdx.x; i < v1; i += kThreads) {
      Vec16<T> a, b, o;
      a.load(y + i * VN);
      b.load(tg + i * VN);
#pragma unroll
      for (int k = 0; k < VN; ++k) {
        const float dlt = a.get(k) - b.get(k);
        acc += dlt * dlt;
        o.set(k, dlt * scale);
      }
      o.store(dy + i * VN);
    }
    const float t = block_sum_fixed(acc, red);
    if (threadIdx.x == 0) partial[p] = t;
  }
}

__global__ __launch_bounds__(kThreads) void mse_final_kernel(const float* __restrict__ partial,
                                                             float* __restrict__ loss, float inv_n) {
  __shared__ float red[kWaves];
  float acc = 0.f;
  for (int p = threadIdx.x; p < kMsePartials; p += kThreads) acc += partial[p];
  const float t = block_sum_fixed(acc, red);
  if (threadIdx.x == 0) *loss = t * inv_n;
}

// ------------------------------------------------------------------------------ colsum
// row partitions of a column reduction (a function of the row count alone).  512: two
// workgroups per CU for the one-pass norm backward (5.1 TB/s at the decoder shape against 4.8
// with 256; 1024 partitions make the partial sums too much traffic: 4.1)
constexpr int kColsumMaxParts = 512;
// widest row (in 16-byte vectors per lane) whose column accumulators the fused norm backward keeps in registers
constexpr int kNormFusedMaxNV = 8;   // LayerNorm; RMSNorm (one sum per column) also fits at 10

template <typename T>
__global__ __launch_bounds__(kThreads) void colsum_partial_kernel(const T* __restrict__ X, float* __restrict__ partial,
                                                                  int64_t rows, int64_t n, int rp, int np, int ctiles) {
  constexpr int VN = Vec16<T>::N;
  const int64_t items = (int64_t)np * ctiles;
  for (int64_t it = blockIdx.x; it < items; it += gridDim.x) {
    const int p = (int)(it / ctiles), ct = (int)(it - (int64_t)p * ctiles);
    const int64_t c = ((int64_t)ct * kThreads + threadIdx.x) * VN;
    if (c >= n) continue;
    float acc[VN];
#pragma unroll
    for (int k = 0; k < VN; ++k) acc[k] = 0.f;
    const int64_t r0 = (int64_t)p * rp;
    const int64_t r1 = (r0 + rp < rows) ? r0 + rp : rows;
    int64_t r = r0;
    // four rows requested together, added in ascending row order
    for (; r + 4 <= r1; r += 4) {
      Vec16<T> v[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) v[u].load(X + (r + u) * n + c);
#pragma unroll
      for (int u = 0; u < 4; ++u)
#pragma unroll
        for (int k = 0; k < VN; ++k) acc[k] += v[u].get(k);
    }
    for (; r < r1; ++r) {
      Vec16<T> v;
      v.load(X + r * n + c);
#pragma unroll
      for (int k = 0; k < VN; ++k) acc[k] += v.get(k);
    }
#pragma unroll
    for (int k = 0; k < VN; ++k) partial[(int64_t)p * n + c + k] = acc[k];
  }
}

// ------------------------------------------------------------------------------- stems
// Patch vector index = (c*p + i)*p + j; patches row-major over the image.
template <typename T>
__global__ __launch_bounds__(kThreads) void unfold_kernel(const T* __restrict__ img, T* __restrict__ out,
                                                          int B, int side, int patch) {
  const int g = side / patch, pd = 3 * patch * patch;
  const int64_t total = (int64_t)B * g * g * pd;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    const int e = (int)(i % pd);
    const int64_t tok = i / pd;
    const int px = (int)(tok % g), py = (int)((tok / g) % g), b = (int)(tok / ((int64_t)g * g));
    const int jj = e % patch, ii = (e / patch) % patch, c = e / (patch * patch);
    out[i] = img[(((int64_t)b * 3 + c) * side + (py * patch + ii)) * side + (px * patch + jj)];
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void add_pos_kernel(const T* __restrict__ pos, T* __restrict__ y,
                                                           int B, int N, int h) {
  const int64_t total = (int64_t)B * N * h, per = (int64_t)N * h;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads)
    y[i] = from_f32<T>(to_f32(y[i]) + to_f32(pos[i % per]));
}

template <typename T>
__global__ __launch_bounds__(kThreads) void pos_grad_kernel(const T* __restrict__ dy, T* __restrict__ dpos,
                                                            int B, int N, int h) {
  const int64_t per = (int64_t)N * h;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < per; i += (int64_t)gridDim.x * kThreads) {
    float acc = 0.f;
    for (int b = 0; b < B; ++b) acc += to_f32(dy[(int64_t)b * per + i]);
    dpos[i] = from_f32<T>(acc);
  }
}

// Token ids and image-token counts.  Without per-sample counts every sample has n_img image
// tokens and ids holds the N - n_img text ids of a sample, [B, N - n_img].  With counts
// (int32 [B], clamped to [0, n_img]) sample b takes its first counts[b] image tokens and ids
// holds one id per sequence position, [B, N], read at positions counts[b] .. N-1.
__device__ __forceinline__ int stem_n_img(const int32_t* counts, int b, int n_img) {
  if (!counts) return n_img;
  const int c = counts[b];
  return c < 0 ? 0 : (c > n_img ? n_img : c);
}
__device__ __forceinline__ int stem_id(const int32_t* ids, const int32_t* counts, int b, int t, int N, int n_img, int vocab) {
  // an id outside the table is clamped rather than followed out of bounds (forward and backward alike)
  const int id = counts ? ids[(int64_t)b * N + t] : ids[(int64_t)b * (N - n_img) + (t - n_img)];
  return id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void text_stem_fwd_kernel(const T* __restrict__ img_tok, const int32_t* __restrict__ ids,
                                                                 const int32_t* __restrict__ counts,
                                                                 const T* __restrict__ table, T* __restrict__ out,
                                                                 int B, int N, int n_img, int h, int vocab) {
  const int64_t total = (int64_t)B * N * h;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    const int c = (int)(i % h);
    const int64_t row = i / h;
    const int t = (int)(row % N), b = (int)(row / N);
    if (t < stem_n_img(counts, b, n_img)) out[i] = img_tok[((int64_t)b * n_img + t) * h + c];
    else out[i] = table[(int64_t)stem_id(ids, counts, b, t, N, n_img, vocab) * h + c];
  }
}

// gradient of the image tokens: rows the sample did not use get zero
template <typename T>
__global__ __launch_bounds__(kThreads) void split_img_kernel(const T* __restrict__ dy, const int32_t* __restrict__ counts,
                                                             T* __restrict__ d_img, int B, int N, int n_img, int h) {
  const int64_t total = (int64_t)B * n_img * h;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total; i += (int64_t)gridDim.x * kThreads) {
    const int c = (int)(i % h);
    const int64_t row = i / h;
    const int t = (int)(row % n_img), b = (int)(row / n_img);
    d_img[i] = t < stem_n_img(counts, b, n_img) ? dy[((int64_t)b * N + t) * h + c] : from_f32<T>(0.f);
  }
}

// Embedding gradient, owner computes: the workgroup that owns table row v walks all token
// positions once, 256 at a time, and gathers the positions that hold v into a list in LDS in
// ascending order (waves in order, lanes in order, by ballot and prefix count); whenever the
// list is nearly full, and at the end, every thread adds the listed rows of dy to the column
// sums it keeps in registers, in list order.  The sum of a row is therefore taken over its
// occurrences in ascending position whatever the grid, repeated ids need no atomics, and a
// row nobody uses costs one pass over the ids and a zero fill.
constexpr int kEmbedList = 1024;                     // positions gathered before they are summed
constexpr int kEmbedMaxCols = 32;                    // columns per thread: rows of up to 8192 elements
template <typename T>
__global__ __launch_bounds__(kThreads) void embed_grad_kernel(const T* __restrict__ dy, const int32_t* __restrict__ ids,
                                                              const int32_t* __restrict__ counts,
                                                              T* __restrict__ dtable, int B, int N, int n_img, int h, int vocab) {
  __shared__ int list[kEmbedList];
  __shared__ int wave_hits[kWaves];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int total = B * N;
  for (int v = blockIdx.x; v < vocab; v += gridDim.x) {
    float acc[kEmbedMaxCols];
#pragma unroll
    for (int j = 0; j < kEmbedMaxCols; ++j) acc[j] = 0.f;
    int n_list = 0;                                  // the same in every thread
    auto add_listed = [&]() {
      for (int e = 0; e < n_list; ++e) {
        const T* row = dy + (int64_t)list[e] * h;
#pragma unroll
        for (int j = 0; j < kEmbedMaxCols; ++j) {
          const int c = j * kThreads + threadIdx.x;
          if (c < h) acc[j] += to_f32(row[c]);
        }
      }
      __syncthreads();                               // everybody is done with the list
      n_list = 0;
    };
    for (int p0 = 0; p0 < total; p0 += kThreads) {
      const int p = p0 + threadIdx.x;
      bool hit = false;
      if (p < total) {
        const int b = p / N, t = p - b * N;
        hit = t >= stem_n_img(counts, b, n_img) && stem_id(ids, counts, b, t, N, n_img, vocab) == v;
      }
      const unsigned long long m = __ballot(hit);
      if (lane == 0) wave_hits[wave] = __popcll(m);
      __syncthreads();
      int before = n_list, all = 0;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) { if (w < wave) before += wave_hits[w]; all += wave_hits[w]; }
      if (hit) list[before + __popcll(m & ((1ull << lane) - 1ull))] = p;
      n_list += all;
      __syncthreads();                               // list entries visible; wave_hits free for the next chunk
      if (n_list > kEmbedList - kThreads) add_listed();
    }
    if (n_list > 0) add_listed();
#pragma unroll
    for (int j = 0; j < kEmbedMaxCols; ++j) {
      const int c = j * kThreads + threadIdx.x;
      if (c < h) dtable[(int64_t)v * h + c] = from_f32<T>(acc[j]);
    }
  }
}

int pick_nv(int need) {
  const int opts[] = {1, 2, 3, 4, 5, 6, 8, 10};
  for (int o : opts) if (o >= need) return o;
  return -1;
}

}  // namespace

// =================================================================== host launchers
#define DISPATCH_NV(NVV, MACRO) \
  switch (NVV) {                \
    case 1: MACRO(1); break;    \
    case 2: MACRO(2); break;    \
    case 3: MACRO(3); break;    \
    case 4: MACRO(4); break;    \
    case 5: MACRO(5); break;    \
    case 6: MACRO(6); break;    \
    case 8: MACRO(8); break;    \
    default: MACRO(10); break;  \
  }

template <typename T>
static mosaic_status norm_fwd_t(hipStream_t s, int quota, int norm, int64_t rows, int64_t h, float eps,
                                const T* x, const T* gamma, const T* beta, T* y, float* stats) {
  constexpr int VN = Vec16<T>::N;
  if (h % VN) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "norm width %lld is not a multiple of %d", (long long)h, VN);
  const int nv = pick_nv((int)ceil_div(h, 64 * VN));
  if (nv < 0) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "norm width %lld too large", (long long)h);
  if (rows == 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 8, ceil_div(rows, kWaves));
#define L(NVC)                                                                                         \
  if (norm == MOSAIC_LAYERNORM)                                                                        \
    norm_fwd_kernel<T, MOSAIC_LAYERNORM, NVC><<<grid, kThreads, 0, s>>>(x, gamma, beta, y, stats, rows, (int)h, eps); \
  else                                                                                                 \
    norm_fwd_kernel<T, MOSAIC_RMSNORM, NVC><<<grid, kThreads, 0, s>>>(x, gamma, beta, y, stats, rows, (int)h, eps)
  DISPATCH_NV(nv, L);
#undef L
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_norm_fwd(hipStream_t s, int quota, int dtype, int norm, int64_t T, int64_t h, float eps,
                              const void* x, const void* gamma, const void* beta, void* y, float* stats) {
  if (norm != MOSAIC_LAYERNORM && norm != MOSAIC_RMSNORM) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm kind %d", norm);
  if (dtype == MOSAIC_BF16)
    return norm_fwd_t<bf16>(s, quota, norm, T, h, eps, (const bf16*)x, (const bf16*)gamma, (const bf16*)beta, (bf16*)y, stats);
  return norm_fwd_t<float>(s, quota, norm, T, h, eps, (const float*)x, (const float*)gamma, (const float*)beta, (float*)y, stats);
}

static inline void col_partition(int64_t T, int* rp, int* np) {
  int64_t r = ceil_div(T, kColsumMaxParts);
  if (r < 8) r = 8;
  *rp = (int)r;
  *np = (int)ceil_div(T, r);
}

size_t norm_bwd_scratch_bytes(int64_t h, bool with_dxsum) { return (size_t)kColsumMaxParts * (with_dxsum ? 3 : 2) * (size_t)h * sizeof(float); }
// widest row (16-byte vectors per lane) for which the one-pass kernel also keeps the column sums of dx
constexpr int kNormDxSumMaxNV = 4;

template <typename T>
static mosaic_status norm_bwd_t(hipStream_t s, int quota, int norm, int64_t rows, int64_t h, const T* x,
                                const T* gamma, const float* stats, const T* dy, const T* R, T* dx,
                                T* dgamma, T* dbeta, float* scratch, T* dxsum, int dtype) {
  constexpr int VN = Vec16<T>::N;
  if (h % VN) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "norm width %lld is not a multiple of %d", (long long)h, VN);
  const int nv = pick_nv((int)ceil_div(h, 64 * VN));
  if (nv < 0) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "norm width %lld too large", (long long)h);
  if (rows == 0) return MOSAIC_OK;
  int rp, np;
  col_partition(rows, &rp, &np);
  const int g2 = grid_for(quota, 8, ceil_div(2 * h, 32));
  if (dxsum && norm == MOSAIC_LAYERNORM && nv <= kNormDxSumMaxNV) {
    // one pass that also sums the columns of dx
    const int gf = grid_for(quota, 8, np);
#define LC(NVC) norm_bwd_fused_kernel<T, MOSAIC_LAYERNORM, NVC, true><<<gf, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, scratch, rows, (int)h, rp, np)
    switch (nv) {
      case 1: LC(1); break;
      case 2: LC(2); break;
      case 3: LC(3); break;
      default: LC(4); break;
    }
#undef LC
    MOSAIC_LAUNCH_CHECK();
    const int g3 = grid_for(quota, 8, ceil_div(3 * h, 32));
    reduce_partials_kernel<T><<<g3, kThreads, 0, s>>>(scratch, np, 3 * h, 3 * h, h, dgamma, dbeta, 2 * h, dxsum);
    MOSAIC_LAUNCH_CHECK();
    return MOSAIC_OK;
  }
  // no kernel that sums dx on the way for this norm or width: the sums take a pass of their own, afterwards
  auto sum_dx = [&]() -> mosaic_status { return dxsum ? launch_colsum(s, quota, dtype, rows, h, dx, dxsum, scratch) : MOSAIC_OK; };
  if (nv <= kNormFusedMaxNV || norm == MOSAIC_RMSNORM) {
    // one pass: x and dy are read once for dx and for the column sums
    const int gf = grid_for(quota, 8, np);
#define LF(NVC)                                                                                       \
    if (norm == MOSAIC_LAYERNORM)                                                                     \
      norm_bwd_fused_kernel<T, MOSAIC_LAYERNORM, NVC><<<gf, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, scratch, rows, (int)h, rp, np); \
    else                                                                                              \
      norm_bwd_fused_kernel<T, MOSAIC_RMSNORM, NVC><<<gf, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, scratch, rows, (int)h, rp, np)
    switch (nv) {
      case 1: LF(1); break;
      case 2: LF(2); break;
      case 3: LF(3); break;
      case 4: LF(4); break;
      case 5: LF(5); break;
      case 6: LF(6); break;
      case 8: LF(8); break;
      default:
        norm_bwd_fused_kernel<T, MOSAIC_RMSNORM, 10><<<gf, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, scratch, rows, (int)h, rp, np);
        break;
    }
#undef LF
    MOSAIC_LAUNCH_CHECK();
    reduce_partials_kernel<T><<<g2, kThreads, 0, s>>>(scratch, np, 2 * h, 2 * h, h, dgamma,
                                                      norm == MOSAIC_LAYERNORM ? dbeta : (T*)nullptr);
    MOSAIC_LAUNCH_CHECK();
    return sum_dx();
  }
  const int grid = grid_for(quota, 8, ceil_div(rows, kWaves));
#define L(NVC)                                                                                        \
  if (norm == MOSAIC_LAYERNORM)                                                                       \
    norm_bwd_dx_kernel<T, MOSAIC_LAYERNORM, NVC><<<grid, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, rows, (int)h); \
  else                                                                                                \
    norm_bwd_dx_kernel<T, MOSAIC_RMSNORM, NVC><<<grid, kThreads, 0, s>>>(x, gamma, stats, dy, R, dx, rows, (int)h)
  DISPATCH_NV(nv, L);
#undef L
  MOSAIC_LAUNCH_CHECK();
  const int ctiles = (int)ceil_div(h, (int64_t)kThreads * VN);
  const int g1 = grid_for(quota, 8, (int64_t)np * ctiles);
  if (norm == MOSAIC_LAYERNORM)
    norm_colgrad_partial_kernel<T, MOSAIC_LAYERNORM><<<g1, kThreads, 0, s>>>(x, stats, dy, scratch, rows, (int)h, rp, np, ctiles);
  else
    norm_colgrad_partial_kernel<T, MOSAIC_RMSNORM><<<g1, kThreads, 0, s>>>(x, stats, dy, scratch, rows, (int)h, rp, np, ctiles);
  MOSAIC_LAUNCH_CHECK();
  reduce_partials_kernel<T><<<g2, kThreads, 0, s>>>(scratch, np, 2 * h, 2 * h, h, dgamma,
                                                    norm == MOSAIC_LAYERNORM ? dbeta : (T*)nullptr);
  MOSAIC_LAUNCH_CHECK();
  return sum_dx();
}

mosaic_status launch_norm_bwd(hipStream_t s, int quota, int dtype, int norm, int64_t T, int64_t h, const void* x,
                              const void* gamma, const float* stats, const void* dy, const void* R, void* dx,
                              void* dgamma, void* dbeta, void* scratch, void* dxsum) {
  if (norm != MOSAIC_LAYERNORM && norm != MOSAIC_RMSNORM) MOSAIC_FAIL(MOSAIC_EINVAL, "bad norm kind %d", norm);
  if (dtype == MOSAIC_BF16)
    return norm_bwd_t<bf16>(s, quota, norm, T, h, (const bf16*)x, (const bf16*)gamma, stats, (const bf16*)dy,
                            (const bf16*)R, (bf16*)dx, (bf16*)dgamma, (bf16*)dbeta, (float*)scratch, (bf16*)dxsum, dtype);
  return norm_bwd_t<float>(s, quota, norm, T, h, (const float*)x, (const float*)gamma, stats, (const float*)dy,
                           (const float*)R, (float*)dx, (float*)dgamma, (float*)dbeta, (float*)scratch, (float*)dxsum, dtype);
}

#define EW_CHECK_VEC(n, dtype)                                                               \
  const int vn__ = (dtype == MOSAIC_BF16) ? 8 : 4;                                           \
  if ((n) % vn__) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "element count %lld is not a multiple of %d", (long long)(n), vn__)

mosaic_status launch_gelu_fwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, void* a) {
  EW_CHECK_VEC(n, dtype);
  if (n == 0) return MOSAIC_OK;
  const int64_t nvec = n / vn__;
  const int grid = grid_for(quota, 8, ceil_div(nvec, kThreads));
  if (dtype == MOSAIC_BF16) gelu_fwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)z, (bf16*)a, nvec);
  else gelu_fwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)z, (float*)a, nvec);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_gelu_bwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, const void* da, void* dz) {
  EW_CHECK_VEC(n, dtype);
  if (n == 0) return MOSAIC_OK;
  const int64_t nvec = n / vn__;
  const int grid = grid_for(quota, 8, ceil_div(nvec, kThreads));
  if (dtype == MOSAIC_BF16) gelu_bwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)z, (const bf16*)da, (bf16*)dz, nvec);
  else gelu_bwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)z, (const float*)da, (float*)dz, nvec);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_swiglu_fwd(hipStream_t s, int quota, int dtype, int64_t T, int64_t f, const void* gu, void* a) {
  EW_CHECK_VEC(f, dtype);
  if (T * f == 0) return MOSAIC_OK;
  const int fv = (int)(f / vn__);
  const int grid = grid_for(quota, 8, ceil_div(T * fv, kThreads));
  if (dtype == MOSAIC_BF16) swiglu_fwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)gu, (bf16*)a, T, fv);
  else swiglu_fwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)gu, (float*)a, T, fv);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_swiglu_bwd(hipStream_t s, int quota, int dtype, int64_t T, int64_t f, const void* gu,
                                const void* da, void* dgu) {
  EW_CHECK_VEC(f, dtype);
  if (T * f == 0) return MOSAIC_OK;
  const int fv = (int)(f / vn__);
  const int grid = grid_for(quota, 8, ceil_div(T * fv, kThreads));
  if (dtype == MOSAIC_BF16) swiglu_bwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)gu, (const bf16*)da, (bf16*)dgu, T, fv);
  else swiglu_bwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)gu, (const float*)da, (float*)dgu, T, fv);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

size_t mse_scratch_bytes() { return kMsePartials * sizeof(float); }

mosaic_status launch_mse(hipStream_t s, int quota, int dtype, int64_t n, const void* y, const void* target,
                         void* dy, float* loss, void* scratch) {
  EW_CHECK_VEC(n, dtype);
  if (n == 0) MOSAIC_FAIL(MOSAIC_EINVAL, "mse over zero elements");
  const int64_t nvec = n / vn__;
  const int64_t chunk = ceil_div(nvec, kMsePartials);
  const int grid = grid_for(quota, 8, kMsePartials);
  const float scale = (float)(2.0 / (double)n);
  if (dtype == MOSAIC_BF16)
    mse_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)y, (const bf16*)target, (bf16*)dy, (float*)scratch, nvec, chunk, scale);
  else
    mse_kernel<float><<<grid, kThreads, 0, s>>>((const float*)y, (const float*)target, (float*)dy, (float*)scratch, nvec, chunk, scale);
  MOSAIC_LAUNCH_CHECK();
  mse_final_kernel<<<1, kThreads, 0, s>>>((const float*)scratch, loss, (float)(1.0 / (double)n));
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

size_t colsum_scratch_bytes(int64_t n) { return (size_t)kColsumMaxParts * (size_t)n * sizeof(float); }

mosaic_status launch_colsum(hipStream_t s, int quota, int dtype, int64_t T, int64_t n, const void* X, void* out,
                            void* scratch) {
  EW_CHECK_VEC(n, dtype);
  if (n == 0) return MOSAIC_OK;
  int rp, np;
  col_partition(T, &rp, &np);
  const int ctiles = (int)ceil_div(n, (int64_t)kThreads * vn__);
  if (np > 0) {
    const int grid = grid_for(quota, 8, (int64_t)np * ctiles);
    if (dtype == MOSAIC_BF16)
      colsum_partial_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)X, (float*)scratch, T, n, rp, np, ctiles);
    else
      colsum_partial_kernel<float><<<grid, kThreads, 0, s>>>((const float*)X, (float*)scratch, T, n, rp, np, ctiles);
    MOSAIC_LAUNCH_CHECK();
  }
  const int g2 = grid_for(quota, 8, ceil_div(n, 32));
  if (dtype == MOSAIC_BF16)
    reduce_partials_kernel<bf16><<<g2, kThreads, 0, s>>>((const float*)scratch, np, n, n, n, (bf16*)out, (bf16*)nullptr);
  else
    reduce_partials_kernel<float><<<g2, kThreads, 0, s>>>((const float*)scratch, np, n, n, n, (float*)out, (float*)nullptr);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_gelu_bwd_colsum(hipStream_t s, int quota, int dtype, int64_t T, int64_t n, const void* z,
                                     const void* da, void* dz, void* colsum, void* scratch) {
  EW_CHECK_VEC(n, dtype);
  if (n == 0) return MOSAIC_OK;
  int rp, np;
  col_partition(T, &rp, &np);
  const int ctiles = (int)ceil_div(n, (int64_t)kThreads * vn__);
  if (np > 0) {
    const int grid = grid_for(quota, 8, (int64_t)np * ctiles);
    if (dtype == MOSAIC_BF16)
      gelu_bwd_colsum_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)z, (const bf16*)da, (bf16*)dz, (float*)scratch, T, n, rp, np, ctiles);
    else
      gelu_bwd_colsum_kernel<float><<<grid, kThreads, 0, s>>>((const float*)z, (const float*)da, (float*)dz, (float*)scratch, T, n, rp, np, ctiles);
    MOSAIC_LAUNCH_CHECK();
  }
  const int g2 = grid_for(quota, 8, ceil_div(n, 32));
  if (dtype == MOSAIC_BF16)
    reduce_partials_kernel<bf16><<<g2, kThreads, 0, s>>>((const float*)scratch, np, n, n, n, (bf16*)colsum, (bf16*)nullptr);
  else
    reduce_partials_kernel<float><<<g2, kThreads, 0, s>>>((const float*)scratch, np, n, n, n, (float*)colsum, (float*)nullptr);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

#define EW_LAUNCH(KERNEL, total, ...)                                                        \
  do {                                                                                       \
    if ((total) == 0) return MOSAIC_OK;                                                      \
    const int grid = grid_for(quota, 8, ceil_div((total), kThreads));                        \
    if (dtype == MOSAIC_BF16) KERNEL<bf16><<<grid, kThreads, 0, s>>> __VA_ARGS__(bf16);      \
    else KERNEL<float><<<grid, kThreads, 0, s>>> __VA_ARGS__(float);                         \
    MOSAIC_LAUNCH_CHECK();                                                                   \
    return MOSAIC_OK;                                                                        \
  } while (0)

mosaic_status launch_unfold(hipStream_t s, int quota, int dtype, int B, int side, int patch, const void* img, void* out) {
  if (patch <= 0 || side % patch) MOSAIC_FAIL(MOSAIC_EINVAL, "image side %d is not a multiple of patch %d", side, patch);
  const int64_t total = (int64_t)B * 3 * side * side;
#define ARGS(TT) ((const TT*)img, (TT*)out, B, side, patch)
  EW_LAUNCH(unfold_kernel, total, ARGS);
#undef ARGS
}

mosaic_status launch_add_pos(hipStream_t s, int quota, int dtype, int B, int N, int h, const void* pos, void* y) {
  const int64_t total = (int64_t)B * N * h;
#define ARGS(TT) ((const TT*)pos, (TT*)y, B, N, h)
  EW_LAUNCH(add_pos_kernel, total, ARGS);
#undef ARGS
}

mosaic_status launch_pos_grad(hipStream_t s, int quota, int dtype, int B, int N, int h, const void* dy, void* dpos) {
  const int64_t total = (int64_t)N * h;
#define ARGS(TT) ((const TT*)dy, (TT*)dpos, B, N, h)
  EW_LAUNCH(pos_grad_kernel, total, ARGS);
#undef ARGS
}

mosaic_status launch_text_stem_fwd(hipStream_t s, int quota, int dtype, int B, int N, int n_img, int h, int vocab,
                                   const void* img_tok, const int32_t* ids, const int32_t* counts, const void* table, void* out) {
  const int64_t total = (int64_t)B * N * h;
#define ARGS(TT) ((const TT*)img_tok, ids, counts, (const TT*)table, (TT*)out, B, N, n_img, h, vocab)
  EW_LAUNCH(text_stem_fwd_kernel, total, ARGS);
#undef ARGS
}

mosaic_status launch_text_stem_bwd(hipStream_t s, int quota, int dtype, int B, int N, int n_img, int h, int vocab,
                                   const void* dy, const int32_t* ids, const int32_t* counts, void* d_img, void* dtable) {
  if (d_img != nullptr && n_img > 0) {
    const int64_t total = (int64_t)B * n_img * h;
    const int grid = grid_for(quota, 8, ceil_div(total, kThreads));
    if (dtype == MOSAIC_BF16) split_img_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)dy, counts, (bf16*)d_img, B, N, n_img, h);
    else split_img_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dy, counts, (float*)d_img, B, N, n_img, h);
    MOSAIC_LAUNCH_CHECK();
  }
  if (vocab > 0) {
    if (h > kEmbedMaxCols * kThreads) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "embedding rows of %d elements; the gradient kernel holds up to %d", h, kEmbedMaxCols * kThreads);
    const int grid = grid_for(quota, 8, vocab);
    if (dtype == MOSAIC_BF16)
      embed_grad_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)dy, ids, counts, (bf16*)dtable, B, N, n_img, h, vocab);
    else
      embed_grad_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dy, ids, counts, (float*)dtable, B, N, n_img, h, vocab);
    MOSAIC_LAUNCH_CHECK();
  }
  return MOSAIC_OK;
}
