// Cross-workgroup reduction of the split-n partial states, in a fixed order (no atomics, so
// the result is bitwise reproducible), and the packing of the reduced state into the fp16
// MFMA operand image the query pass consumes.
#include "kernels.h"
#include "mfma_layout.h"

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
  for (int p = 0; p < P; ++p) acc += src[(size_t)p * elems];
  state[(size_t)bh * elems + e] = acc;
}

// One thread builds the 8 fp16 values lane `lane` feeds to MFMA as the A operand of
// out^T = S^T phi(q)^T for k-step `ks` and row block `mb` (see mfma_layout.h).  S and z of one
// (b,h) are scaled by a common power of two that brings their largest magnitude into
// [2^13, 2^14): the output is a ratio, so the scale cancels, and fp16 cannot overflow.
template <int D>
__global__ __launch_bounds__(256) void state_pack_kernel(const float* __restrict__ state, uint4* __restrict__ sa) {
  using L = ApplyLayout<D>;
  const int idx = blockIdx.x * 256 + threadIdx.x;        // (ks, mb, lane)
  const int bh = blockIdx.y;
  __shared__ float s_red[4];
  float scale;
  {
    const float* S0 = state + (size_t)bh * (D + 1) * D;
    float amax = 0.f;
    for (int i = threadIdx.x; i < (D + 1) * D; i += 256) amax = fmaxf(amax, fabsf(S0[i]));
    for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
    if (threadIdx.x % 64 == 0) s_red[threadIdx.x / 64] = amax;
    __syncthreads();
    amax = fmaxf(fmaxf(s_red[0], s_red[1]), fmaxf(s_red[2], s_red[3]));
    scale = (amax > 0.f && amax < 3.0e38f) ? ldexpf(1.0f, 13 - ilogbf(amax)) : 1.0f;
  }
  if (idx >= L::KS * L::MBZ * 64) return;
  const int lane = idx % 64;
  const int mb = (idx / 64) % L::MBZ;
  const int ks = idx / (64 * L::MBZ);
  const int m = lane % 32, g = lane / 32;
  const float* S = state + (size_t)bh * (D + 1) * D;
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int f = L::feature(ks, g, e);
    if (mb < L::MB) x[e] = scale * S[f * D + L::channel(mb, m)];
    else x[e] = (m == 0 || m == 4) ? scale * S[D * D + f] : 0.f;
  }
  uint4 r;
  r.x = pack_f16x2(x[0], x[1]);
  r.y = pack_f16x2(x[2], x[3]);
  r.z = pack_f16x2(x[4], x[5]);
  r.w = pack_f16x2(x[6], x[7]);
  sa[(size_t)bh * (L::KS * L::MBZ * 64) + idx] = r;
}

}  // namespace

hipError_t launch_state_reduce(const float* partials, float* state, void* sa, const Plan& p, hipStream_t s) {
  const int elems = (int)p.state_elems;
  state_reduce_kernel<<<dim3((elems + 255) / 256, p.BH), 256, 0, s>>>(partials, state, p.P, elems);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || !sa) return e;
  if (p.d == 128) {
    using L = ApplyLayout<128>;
    state_pack_kernel<128><<<dim3((L::KS * L::MBZ * 64 + 255) / 256, p.BH), 256, 0, s>>>(state, (uint4*)sa);
  } else {
    using L = ApplyLayout<64>;
    state_pack_kernel<64><<<dim3((L::KS * L::MBZ * 64 + 255) / 256, p.BH), 256, 0, s>>>(state, (uint4*)sa);
  }
  return hipGetLastError();
}

}  // namespace linattn
