// Layer variants beyond the workloads' kernel list, all bandwidth-bound: the tanh form of
// GELU, rotary position embedding on the q and k parts of packed q|k|v rows, and the AdamW
// update over a module's flat parameter buffer.  Grid-stride kernels over 16-byte vectors;
// every output element has one owner, so results do not depend on the grid.
#include "kernels.h"

namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float tanh_gelu_f(float z) {
  const float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
  return 0.5f * z * (1.0f + tanhf(u));
}
__device__ __forceinline__ float tanh_gelu_grad_f(float z) {
  const float u = 0.7978845608028654f * (z + 0.044715f * z * z * z);
  const float t = tanhf(u);
  return 0.5f * (1.0f + t) + 0.5f * z * (1.0f - t * t) * 0.7978845608028654f * (1.0f + 3.0f * 0.044715f * z * z);
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gelu_tanh_fwd_kernel(const T* __restrict__ z, T* __restrict__ a, int64_t nvec) {
  constexpr int VN = Vec16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    Vec16<T> v, o;
    v.load(z + i * VN);
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, tanh_gelu_f(v.get(k)));
    o.store(a + i * VN);
  }
}

template <typename T>
__global__ __launch_bounds__(kThreads) void gelu_tanh_bwd_kernel(const T* __restrict__ z, const T* __restrict__ da,
                                                                 T* __restrict__ dz, int64_t nvec) {
  constexpr int VN = Vec16<T>::N;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    Vec16<T> v, d, o;
    v.load(z + i * VN);
    d.load(da + i * VN);
#pragma unroll
    for (int k = 0; k < VN; ++k) o.set(k, d.get(k) * tanh_gelu_grad_f(v.get(k)));
    o.store(dz + i * VN);
  }
}

// table[n][i] = (cos, sin)(n * base^(-2i/d)), n < N, i < d/2.  Angles reach thousands of
// radians, where a float argument alone is off by 1e-4; they are formed and reduced in double.
__global__ __launch_bounds__(kThreads) void rope_table_kernel(float2* __restrict__ table, int N, int half, double base) {
  const int64_t total = (int64_t)N * half;
  for (int64_t e = (int64_t)blockIdx.x * kThreads + threadIdx.x; e < total; e += (int64_t)gridDim.x * kThreads) {
    const int n = (int)(e / half), i = (int)(e - (int64_t)n * half);
    const double ang = (double)n * pow(base, -2.0 * (double)i / (double)(2 * half));
    table[e] = make_float2((float)cos(ang), (float)sin(ang));
  }
}

// In place on the q and k parts (the first `rot` columns) of rows [q | k | v] of width `width`:
// pair (x[2i], x[2i+1]) of a head turns by the tabulated angle of (row's position, i);
// sign = -1 turns back.
template <typename T>
__global__ __launch_bounds__(kThreads) void rope_kernel(T* __restrict__ qkv, const float2* __restrict__ table, int64_t rows,
                                                        int N, int rot, int width, int d, float sign) {
  constexpr int VN = Vec16<T>::N;
  const int vpr = rot / VN;                         // vectors of the q|k part of a row
  const int64_t nvec = rows * vpr;
  const int half = d / 2;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * kThreads) {
    const int64_t row = v / vpr;
    const int col = (int)(v - row * vpr) * VN;      // first column inside [q | k]
    const int n = (int)(row % N);
    const int i0 = (col % d) / 2;                   // first pair index inside the head (VN divides d)
    T* p = qkv + row * (int64_t)width + col;
    Vec16<T> x, o;
    x.load(p);
#pragma unroll
    for (int k = 0; k < VN / 2; ++k) {
      const float2 cs = table[(int64_t)n * half + i0 + k];
      const float xe = x.get(2 * k), xo = x.get(2 * k + 1), s = sign * cs.y;
      o.set(2 * k, xe * cs.x - xo * s);
      o.set(2 * k + 1, xe * s + xo * cs.x);
    }
    o.store(p);
  }
}

// AdamW with decoupled weight decay and bias-corrected moments; moments (and the optional
// master copy of the parameters) are fp32 whatever the parameter dtype.
template <typename T>
__global__ __launch_bounds__(kThreads) void adamw_kernel(T* __restrict__ p, const T* __restrict__ g, float* __restrict__ m,
                                                         float* __restrict__ v, float* __restrict__ master, int64_t nvec,
                                                         float lr, float b1, float b2, float eps, float wd,
                                                         float inv_bc1, float inv_bc2) {
  // Four elements per thread for either type: the fp32 state moves as one 16-byte vector, a
  // bf16 parameter and gradient as one 8-byte vector, so that every instruction of a wave
  // covers one contiguous run (1 KB, or 512 bytes) and each line is written whole by one
  // instruction.
  typedef __attribute__((ext_vector_type(4))) T vec4;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < nvec; i += (int64_t)gridDim.x * kThreads) {
    vec4 pv = *reinterpret_cast<const vec4*>(p + i * 4);
    const vec4 gv = *reinterpret_cast<const vec4*>(g + i * 4);
    float4 mv = *reinterpret_cast<const float4*>(m + i * 4);
    float4 vv = *reinterpret_cast<const float4*>(v + i * 4);
    float4 ms = make_float4(0.f, 0.f, 0.f, 0.f);
    if (master) ms = *reinterpret_cast<const float4*>(master + i * 4);
    float* mp = &mv.x; float* vp = &vv.x; float* sp = &ms.x;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float gk = (float)gv[k];
      const float pk = master ? sp[k] : (float)pv[k];
      const float mk = b1 * mp[k] + (1.0f - b1) * gk;
      const float vk = b2 * vp[k] + (1.0f - b2) * gk * gk;
      mp[k] = mk; vp[k] = vk;
      const float upd = (mk * inv_bc1) / (sqrtf(vk * inv_bc2) + eps) + wd * pk;
      const float np_ = pk - lr * upd;
      sp[k] = np_;
      pv[k] = (T)np_;
    }
    *reinterpret_cast<float4*>(m + i * 4) = mv;
    *reinterpret_cast<float4*>(v + i * 4) = vv;
    if (master) *reinterpret_cast<float4*>(master + i * 4) = ms;
    *reinterpret_cast<vec4*>(p + i * 4) = pv;
  }
}

// Gathers the three taps of a k=3, pad=1 convolution over frames-major x [B, L, C]:
// out[(b*Lo + t), k*C + c] = x[b, t*stride - 1 + k, c], zero outside [0, L).
template <typename T>
__global__ __launch_bounds__(kThreads) void im2col1d_kernel(const T* __restrict__ x, T* __restrict__ out, int64_t B, int L,
                                                            int Lo, int C, int stride) {
  constexpr int VN = Vec16<T>::N;
  const int cv = C / VN;
  const int64_t nvec = B * Lo * 3 * cv;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * kThreads) {
    const int c = (int)(v % cv) * VN;
    const int k = (int)((v / cv) % 3);
    const int64_t row = v / (3 * cv);
    const int t = (int)(row % Lo);
    const int64_t b = row / Lo;
    const int src = t * stride - 1 + k;
    Vec16<T> val;
    if (src >= 0 && src < L) val.load(x + (b * L + src) * C + c);
    else {
#pragma unroll
      for (int e = 0; e < VN; ++e) val.set(e, 0.f);
    }
    val.store(out + row * 3 * (int64_t)C + (int64_t)k * C + c);
  }
}

// The transpose of the gather: dx[b, s, c] = sum over taps k (ascending) of
// dP[(b*Lo + t), k*C + c] with t*stride - 1 + k == s; one owner per element, fixed order.
template <typename T>
__global__ __launch_bounds__(kThreads) void col2im1d_kernel(const T* __restrict__ dP, T* __restrict__ dx, int64_t B, int L,
                                                            int Lo, int C, int stride) {
  constexpr int VN = Vec16<T>::N;
  const int cv = C / VN;
  const int64_t nvec = B * L * cv;
  for (int64_t v = (int64_t)blockIdx.x * kThreads + threadIdx.x; v < nvec; v += (int64_t)gridDim.x * kThreads) {
    const int c = (int)(v % cv) * VN;
    const int64_t fr = v / cv;
    const int s_ = (int)(fr % L);
    const int64_t b = fr / L;
    float acc[VN];
#pragma unroll
    for (int e = 0; e < VN; ++e) acc[e] = 0.f;
    for (int k = 0; k < 3; ++k) {
      const int num = s_ + 1 - k;
      if (num < 0 || num % stride) continue;
      const int t = num / stride;
      if (t >= Lo) continue;
      Vec16<T> val;
      val.load(dP + (b * Lo + t) * 3 * (int64_t)C + (int64_t)k * C + c);
#pragma unroll
      for (int e = 0; e < VN; ++e) acc[e] += val.get(e);
    }
    Vec16<T> o;
#pragma unroll
    for (int e = 0; e < VN; ++e) o.set(e, acc[e]);
    o.store(dx + fr * C + c);
  }
}

}  // namespace

mosaic_status launch_im2col1d(hipStream_t s, int quota, int dtype, int64_t B, int L, int Lo, int C, int stride,
                              const void* x, void* out) {
  const int vn = dtype == MOSAIC_BF16 ? 8 : 4;
  if (C % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "channel count %d is not a multiple of %d", C, vn);
  if (B <= 0 || L <= 0 || Lo <= 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 8, ceil_div(B * Lo * 3 * (C / vn), kThreads));
  if (dtype == MOSAIC_BF16) im2col1d_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)x, (bf16*)out, B, L, Lo, C, stride);
  else im2col1d_kernel<float><<<grid, kThreads, 0, s>>>((const float*)x, (float*)out, B, L, Lo, C, stride);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_col2im1d(hipStream_t s, int quota, int dtype, int64_t B, int L, int Lo, int C, int stride,
                              const void* dP, void* dx) {
  const int vn = dtype == MOSAIC_BF16 ? 8 : 4;
  if (C % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "channel count %d is not a multiple of %d", C, vn);
  if (B <= 0 || L <= 0 || Lo <= 0) return MOSAIC_OK;
  const int grid = grid_for(quota, 8, ceil_div(B * L * (C / vn), kThreads));
  if (dtype == MOSAIC_BF16) col2im1d_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)dP, (bf16*)dx, B, L, Lo, C, stride);
  else col2im1d_kernel<float><<<grid, kThreads, 0, s>>>((const float*)dP, (float*)dx, B, L, Lo, C, stride);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_gelu_tanh_fwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, void* a) {
  const int vn = dtype == MOSAIC_BF16 ? 8 : 4;
  if (n % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "element count %lld is not a multiple of %d", (long long)n, vn);
  if (n == 0) return MOSAIC_OK;
  const int64_t nvec = n / vn;
  const int grid = grid_for(quota, 8, ceil_div(nvec, kThreads));
  if (dtype == MOSAIC_BF16) gelu_tanh_fwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)z, (bf16*)a, nvec);
  else gelu_tanh_fwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)z, (float*)a, nvec);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_gelu_tanh_bwd(hipStream_t s, int quota, int dtype, int64_t n, const void* z, const void* da, void* dz) {
  const int vn = dtype == MOSAIC_BF16 ? 8 : 4;
  if (n % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "element count %lld is not a multiple of %d", (long long)n, vn);
  if (n == 0) return MOSAIC_OK;
  const int64_t nvec = n / vn;
  const int grid = grid_for(quota, 8, ceil_div(nvec, kThreads));
  if (dtype == MOSAIC_BF16) gelu_tanh_bwd_kernel<bf16><<<grid, kThreads, 0, s>>>((const bf16*)z, (const bf16*)da, (bf16*)dz, nvec);
  else gelu_tanh_bwd_kernel<float><<<grid, kThreads, 0, s>>>((const float*)z, (const float*)da, (float*)dz, nvec);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

size_t rope_table_bytes(int N, int d) { return (size_t)N * (size_t)(d / 2) * sizeof(float2); }

mosaic_status launch_rope_table(hipStream_t s, int quota, int N, int d, float base, void* table) {
  if (N <= 0 || d <= 0 || (d & 1) || !(base > 0.f)) MOSAIC_FAIL(MOSAIC_EINVAL, "rotary table needs N > 0, even d > 0 and base > 0");
  const int grid = grid_for(quota, 8, ceil_div((int64_t)N * (d / 2), kThreads));
  rope_table_kernel<<<grid, kThreads, 0, s>>>((float2*)table, N, d / 2, (double)base);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_rope(hipStream_t s, int quota, int dtype, int B, int N, int H, int Hkv, int d, int direction,
                          void* qkv, const void* table) {
  const int vn = dtype == MOSAIC_BF16 ? 8 : 4;
  if (B < 0 || N <= 0 || H <= 0 || Hkv <= 0 || d <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad rotary sizes");
  if (d % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "head size %d is not a multiple of %d", d, vn);
  if (direction != 1 && direction != -1) MOSAIC_FAIL(MOSAIC_EINVAL, "direction must be +1 or -1");
  const int64_t rows = (int64_t)B * N;
  if (rows == 0) return MOSAIC_OK;
  const int rot = (H + Hkv) * d, width = (H + 2 * Hkv) * d;
  const int grid = grid_for(quota, 8, ceil_div(rows * (rot / vn), kThreads));
  if (dtype == MOSAIC_BF16) rope_kernel<bf16><<<grid, kThreads, 0, s>>>((bf16*)qkv, (const float2*)table, rows, N, rot, width, d, (float)direction);
  else rope_kernel<float><<<grid, kThreads, 0, s>>>((float*)qkv, (const float2*)table, rows, N, rot, width, d, (float)direction);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

mosaic_status launch_adamw(hipStream_t s, int quota, int dtype, int64_t n, void* p, const void* g, float* m, float* v,
                           float* master, float lr, float beta1, float beta2, float eps, float weight_decay, int64_t step) {
  const int vn = 4;
  if (n % vn) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "element count %lld is not a multiple of %d", (long long)n, vn);
  if (step < 1) MOSAIC_FAIL(MOSAIC_EINVAL, "step counts from 1");
  if (((uintptr_t)p | (uintptr_t)g | (uintptr_t)m | (uintptr_t)v | (uintptr_t)master) & 15) MOSAIC_FAIL(MOSAIC_EINVAL, "AdamW buffers must be 16-byte aligned");
  if (!(beta1 >= 0.f && beta1 < 1.f && beta2 >= 0.f && beta2 < 1.f)) MOSAIC_FAIL(MOSAIC_EINVAL, "betas must lie in [0,1)");
  if (n == 0) return MOSAIC_OK;
  // bias corrections in double on the host: 1 - beta^t loses digits in float for small t
  const float inv_bc1 = (float)(1.0 / (1.0 - pow((double)beta1, (double)step)));
  const float inv_bc2 = (float)(1.0 / (1.0 - pow((double)beta2, (double)step)));
  const int64_t nvec = n / vn;
  const int grid = grid_for(quota, 8, ceil_div(nvec, kThreads));
  if (dtype == MOSAIC_BF16)
    adamw_kernel<bf16><<<grid, kThreads, 0, s>>>((bf16*)p, (const bf16*)g, m, v, master, nvec, lr, beta1, beta2, eps, weight_decay, inv_bc1, inv_bc2);
  else
    adamw_kernel<float><<<grid, kThreads, 0, s>>>((float*)p, (const float*)g, m, v, master, nvec, lr, beta1, beta2, eps, weight_decay, inv_bc1, inv_bc2);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}
