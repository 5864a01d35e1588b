// Activation formulas shared by the elementwise kernels and the GEMM epilogues that apply them
// in place of a separate pass: one definition, so both roads give the same bits.
#pragma once
#include <hip/hip_runtime.h>

__device__ __forceinline__ float gelu_f(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float gelu_grad_f(float z) {
  return 0.5f * (1.0f + erff(z * 0.70710678118654752f)) + z * expf(-0.5f * z * z) * 0.39894228040143268f;
}
__device__ __forceinline__ float sigmoid_f(float z) { return 1.0f / (1.0f + expf(-z)); }
// SwiGLU: silu(gate) * up
__device__ __forceinline__ float swiglu_f(float gate, float up) { return gate * sigmoid_f(gate) * up; }
