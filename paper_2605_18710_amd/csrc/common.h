// Shared host/device helpers for the gfx950 kernels and the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <stdarg.h>
#include "../../include/mosaic.h"

typedef __bf16 bf16;

// ---------------------------------------------------------------------------- errors
void mosaic_set_error(const char* fmt, ...);

#define MOSAIC_FAIL(code, ...)            \
  do {                                    \
    mosaic_set_error(__VA_ARGS__);        \
    return (code);                        \
  } while (0)

#define MOSAIC_HIP(expr)                                                          \
  do {                                                                            \
    hipError_t e__ = (expr);                                                      \
    if (e__ != hipSuccess) {                                                      \
      mosaic_set_error("%s failed: %s", #expr, hipGetErrorString(e__));           \
      return MOSAIC_EHIP;                                                         \
    }                                                                             \
  } while (0)

#define MOSAIC_TRY(expr)                  \
  do {                                    \
    mosaic_status s__ = (expr);           \
    if (s__ != MOSAIC_OK) return s__;     \
  } while (0)

// Launch check: kernel launches report configuration errors through hipGetLastError.
#define MOSAIC_LAUNCH_CHECK()                                                     \
  do {                                                                            \
    hipError_t e__ = hipGetLastError();                                           \
    if (e__ != hipSuccess) {                                                      \
      mosaic_set_error("kernel launch failed: %s", hipGetErrorString(e__));       \
      return MOSAIC_EHIP;                                                         \
    }                                                                             \
  } while (0)

static inline size_t dtype_size(int32_t dtype) { return dtype == MOSAIC_BF16 ? 2 : 4; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Device properties cached per process.
struct DeviceInfo {
  int cu_count;
  int xcd_count;
  bool ok;
};
mosaic_status mosaic_device_info(DeviceInfo* out);

// Persistent-grid sizing: `quota` CUs times the number of workgroups that fit on a CU,
// capped by the number of work items.  The grid only decides WHICH workgroup computes a
// work item, never how, so results do not depend on it.
static inline int grid_for(int quota, int wg_per_cu, int64_t items) {
  int64_t g = (int64_t)quota * wg_per_cu;
  if (g > items) g = items;
  if (g < 1) g = 1;
  return (int)g;
}

// --------------------------------------------------------------- device-side helpers
#ifdef __HIPCC__
__device__ __forceinline__ float to_f32(float x) { return x; }
__device__ __forceinline__ float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ __forceinline__ T from_f32(float x);
template <> __device__ __forceinline__ float from_f32<float>(float x) { return x; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float x) { return (bf16)x; }

// 16-byte vector of T: 4 floats or 8 bf16.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  float4 v;
  __device__ __forceinline__ void load(const float* p) { v = *reinterpret_cast<const float4*>(p); }
  __device__ __forceinline__ void store(float* p) const { *reinterpret_cast<float4*>(p) = v; }
  __device__ __forceinline__ float get(int i) const { return (&v.x)[i]; }
  __device__ __forceinline__ void set(int i, float f) { (&v.x)[i] = f; }
};
template <> struct Vec16<bf16> {
  static constexpr int N = 8;
  typedef __attribute__((ext_vector_type(8))) __bf16 v8;
  v8 v;
  __device__ __forceinline__ void load(const bf16* p) { v = *reinterpret_cast<const v8*>(p); }
  __device__ __forceinline__ void store(bf16* p) const { *reinterpret_cast<v8*>(p) = v; }
  __device__ __forceinline__ float get(int i) const { return (float)v[i]; }
  __device__ __forceinline__ void set(int i, float f) { v[i] = (bf16)f; }
};

__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x += __shfl_xor(x, o, 64);
  return x;
}
__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) x = fmaxf(x, __shfl_xor(x, o, 64));
  return x;
}
#endif
