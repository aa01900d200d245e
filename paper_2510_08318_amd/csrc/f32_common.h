// Building blocks of the fp32-arithmetic kernels: plain FMA on LDS tiles.  The tensors they read and write
// are fp32 (no bf16/fp16 anywhere: the fp32 mode) or bf16 bit patterns widened exactly on load and rounded
// to nearest even on store (the bf16-storage, fp32-arithmetic mode); the arithmetic is the same.
#pragma once
#include <hip/hip_runtime.h>
#include "kernels.h"

namespace linattn {
namespace f32 {

constexpr int NT = 256;       // threads per workgroup

// Element i of a stored tensor as fp32, and the store of an fp32 value: T = float or uint16_t (bf16 bits).
__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const uint16_t* p, size_t i) { return __builtin_bit_cast(float, (uint32_t)p[i] << 16); }
__device__ __forceinline__ void stf(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(uint16_t* p, size_t i, float v) { p[i] = __builtin_bit_cast(uint16_t, (__bf16)v); }

__device__ __forceinline__ float wave_max(float x) {
  for (int m = 32; m >= 1; m >>= 1) x = fmaxf(x, __shfl_xor(x, m, 64));
  return x;
}
__device__ __forceinline__ float wave_sum(float x) {
  for (int m = 32; m >= 1; m >>= 1) x += __shfl_xor(x, m, 64);
  return x;
}

// Eq. 5 on a tile of TT tokens (TT = 16 or 32): sX [TT][D+1] holds the tokens, sW [D][D/2] the map; on return
// sPhi [TT][D] holds softmax(u) then softmax(-u) per token, rows >= n_valid are zero.
// KIND = kPhiRelu: sPhi = max(sX, 0) instead, sW is not read.
// Contains __syncthreads(); every thread of the workgroup must call it.
template <int D, int TT, int KIND>
__device__ __forceinline__ void phi_tile(const float* sX, const float* sW, float* sPhi, int tid, int n_valid) {
  constexpr int HALF = D / 2;
  if constexpr (KIND == kPhiRelu) {
    for (int i = tid; i < TT * D; i += NT) {
      const int tt = i / D, c = i % D;
      sPhi[i] = tt < n_valid ? fmaxf(sX[tt * (D + 1) + c], 0.f) : 0.f;
    }
    __syncthreads();
    return;
  }
  {
    constexpr int FB = NT / TT;                  // feature groups
    const int tt = tid % TT, fb = tid / TT;
    float u[HALF / FB];
#pragma unroll
    for (int j = 0; j < HALF / FB; ++j) u[j] = 0.f;
    for (int c = 0; c < D; ++c) {
      const float x = sX[tt * (D + 1) + c];
#pragma unroll
      for (int j = 0; j < HALF / FB; ++j) u[j] = fmaf(x, sW[c * HALF + fb + FB * j], u[j]);
    }
#pragma unroll
    for (int j = 0; j < HALF / FB; ++j) sPhi[tt * D + fb + FB * j] = u[j];
  }
  __syncthreads();
  {
    const int w = tid / 64, lane = tid % 64;
    for (int i = 0; i < TT / 4; ++i) {
      const int tt = w * (TT / 4) + i;
      const float x = sPhi[tt * D + (lane % HALF)];
      const float mx = wave_max(x);
      const float mn = -wave_max(-x);
      const float ep = expf(x - mx);
      const float em = expf(mn - x);
      float sp = wave_sum(ep), sm = wave_sum(em);
      if (HALF == 32) { sp *= 0.5f; sm *= 0.5f; }   // both half-waves hold the same 32 features
      const bool valid = tt < n_valid;
      if (lane < HALF) {
        sPhi[tt * D + lane] = valid ? ep / sp : 0.f;
        sPhi[tt * D + HALF + lane] = valid ? em / sm : 0.f;
      }
    }
  }
  __syncthreads();
}

}  // namespace f32
}  // namespace linattn
