// Cross-workgroup reduction of the split-n partial states, in a fixed order (no atomics, so
// the result is bitwise reproducible).
#include "kernels.h"

namespace linattn {
namespace {

// state[bh][e] = sum_{p=0..P-1} partials[bh][p][e], p ascending.
__global__ __launch_bounds__(256) void state_reduce_kernel(const float* __restrict__ partials, float* __restrict__ state,
                                                           int P, int elems) {
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int bh = blockIdx.y;
  if (e >= elems) return;
  const float* src = partials + (size_t)bh * P * elems + e;
  float acc = 0.f;
  int p = 0;
  // eight independent loads in flight, added in ascending p
  for (; p + 8 <= P; p += 8) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = src[(size_t)(p + i) * elems];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += t[i];
  }
  for (; p < P; ++p) acc += src[(size_t)p * elems];
  state[(size_t)bh * elems + e] = acc;
}

}  // namespace

hipError_t launch_state_reduce(const float* partials, float* state, const Plan& p, hipStream_t s) {
  const int elems = (int)p.state_elems;
  state_reduce_kernel<<<dim3((elems + 255) / 256, p.BH), 256, 0, s>>>(partials, state, p.P, elems);
  return hipGetLastError();
}

}  // namespace linattn
