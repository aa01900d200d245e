// Cross-workgroup reductions in a fixed order (no atomics, so the results are bitwise
// reproducible): the split-n partial states, and the weight gradient dW~ = sum x^T du.
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

// The same for the flattened split of the bf16 forward: head bh owns the slots of the workgroups
// whose tile ranges touch it, in ascending workgroup order.
__global__ __launch_bounds__(256) void state_reduce_split_kernel(const float* __restrict__ partials, float* __restrict__ state,
                                                                 Split sp, int elems) {
  __shared__ int s_cnt;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int bh = blockIdx.y;
  if (threadIdx.x == 0)
    s_cnt = split_owner(sp, (long long)(bh + 1) * sp.ntile - 1) - split_owner(sp, (long long)bh * sp.ntile) + 1;
  __syncthreads();
  if (e >= elems) return;
  const int cnt = s_cnt;
  const float* src = partials + (size_t)bh * sp.PS * elems + e;
  float acc = 0.f;
  int p = 0;
  for (; p + 8 <= cnt; p += 8) {
    float t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = src[(size_t)(p + i) * elems];
#pragma unroll
    for (int i = 0; i < 8; ++i) acc += t[i];
  }
  if (p + 4 <= cnt) {
    float t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = src[(size_t)(p + i) * elems];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc += t[i];
    p += 4;
  }
  for (; p < cnt; ++p) acc += src[(size_t)p * elems];
  state[(size_t)bh * elems + e] = acc;
}

// The same, four adjacent elements per thread (elems % 4 == 0, both pointers 16-byte aligned): a quarter
// of the load instructions for the same bytes.  Each element is still the sum of its slots in
// ascending order, so the result is bitwise that of state_reduce_split_kernel.
__global__ __launch_bounds__(256) void state_reduce_split4_kernel(const float4* __restrict__ partials, float4* __restrict__ state,
                                                                  Split sp, int elems4) {
  __shared__ int s_cnt;
  const int e = blockIdx.x * 256 + threadIdx.x;
  const int bh = blockIdx.y;
  if (threadIdx.x == 0)
    s_cnt = split_owner(sp, (long long)(bh + 1) * sp.ntile - 1) - split_owner(sp, (long long)bh * sp.ntile) + 1;
  __syncthreads();
  if (e >= elems4) return;
  const int cnt = s_cnt;
  const float4* src = partials + (size_t)bh * sp.PS * elems4 + e;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  int p = 0;
  for (; p + 8 <= cnt; p += 8) {
    float4 t[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) t[i] = src[(size_t)(p + i) * elems4];
#pragma unroll
    for (int i = 0; i < 8; ++i) { acc.x += t[i].x; acc.y += t[i].y; acc.z += t[i].z; acc.w += t[i].w; }
  }
  if (p + 4 <= cnt) {
    float4 t[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) t[i] = src[(size_t)(p + i) * elems4];
#pragma unroll
    for (int i = 0; i < 4; ++i) { acc.x += t[i].x; acc.y += t[i].y; acc.z += t[i].z; acc.w += t[i].w; }
    p += 4;
  }
  for (; p < cnt; ++p) {
    const float4 t = src[(size_t)p * elems4];
    acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
  }
  state[(size_t)bh * elems4 + e] = acc;
}

// ---- dW~ = sum_{b, i} x_i^T du_i ------------------------------------------------------------
// Partial sums per (b,h) and token split (fp32 FMA, LDS tiles), then a fixed-order reduction over
// splits and batch items.
template <int D, typename XT>
__global__ __launch_bounds__(256) void dw_partial_kernel(const XT* __restrict__ x, const float* __restrict__ du,
                                                         float* __restrict__ part, int H, int n, int P, int chunk, Rows rw) {
  constexpr int HALF = D / 2;
  constexpr int TT = 32;
  __shared__ float sX[TT][D + 1];
  __shared__ float sU[TT][HALF];
  const int tid = threadIdx.x, bh = blockIdx.y, p = blockIdx.x;
  const int t_begin = p * chunk, t_end = min(n, t_begin + chunk);
  const XT* xb = x + head_base(rw, bh, H);
  const float* ub = du + (size_t)bh * n * HALF;
  constexpr int BC = D / 16, BF = HALF / 16;        // each thread owns BC x BF entries
  const int c0 = (tid / 16) * BC, f0 = (tid % 16) * BF;
  float acc[BC][BF];
#pragma unroll
  for (int i = 0; i < BC; ++i)
#pragma unroll
    for (int j = 0; j < BF; ++j) acc[i][j] = 0.f;
  for (int t0 = t_begin; t0 < t_end; t0 += TT) {
    __syncthreads();
    for (int i = tid; i < TT * D; i += 256) {
      const int r = i / D, c = i % D, t = t0 + r;
      float val = 0.f;
      if (t < t_end) {
        if constexpr (sizeof(XT) == 2) val = __builtin_bit_cast(float, (uint32_t)xb[(size_t)t * rw.sn + c] << 16);
        else val = xb[(size_t)t * rw.sn + c];
      }
      sX[r][c] = val;
    }
    for (int i = tid; i < TT * HALF; i += 256) {
      const int r = i / HALF, f = i % HALF, t = t0 + r;
      sU[r][f] = t < t_end ? ub[(size_t)t * HALF + f] : 0.f;
    }
    __syncthreads();
    for (int r = 0; r < TT; ++r) {
      float a[BC], b[BF];
#pragma unroll
      for (int i = 0; i < BC; ++i) a[i] = sX[r][c0 + i];
#pragma unroll
      for (int j = 0; j < BF; ++j) b[j] = sU[r][f0 + j];
#pragma unroll
      for (int i = 0; i < BC; ++i)
#pragma unroll
        for (int j = 0; j < BF; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
  }
  float* dst = part + ((size_t)bh * P + p) * (size_t)D * HALF;
#pragma unroll
  for (int i = 0; i < BC; ++i)
#pragma unroll
    for (int j = 0; j < BF; ++j) dst[(c0 + i) * HALF + f0 + j] = acc[i][j];
}

// dw[h][e] = sum_b sum_p part[(b*H + h)][p][e], b then p ascending.
// blockIdx.z picks one of up to two (partials, output, partials per (b,h)) triples; a triple without output is skipped.
__global__ __launch_bounds__(256) void dw_reduce_kernel(const float* __restrict__ part0, float* __restrict__ dw0, int P0,
                                                        const float* __restrict__ part1, float* __restrict__ dw1, int P1,
                                                        int B, int H, int elems) {
  const float* part = blockIdx.z ? part1 : part0;
  float* dw = blockIdx.z ? dw1 : dw0;
  const int P = blockIdx.z ? P1 : P0;
  const int e = blockIdx.x * 256 + threadIdx.x, h = blockIdx.y;
  if (e >= elems || dw == nullptr) return;
  // eight partials are requested together and then added in ascending order (a missing one adds 0): one memory
  // latency per eight terms instead of one per term, the order of the sum unchanged
  float acc = 0.f;
  for (int b = 0; b < B; ++b) {
    const float* src = part + ((size_t)(b * H + h) * P) * elems + e;
    for (int p0 = 0; p0 < P; p0 += 8) {
      float v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = p0 + j < P ? src[(size_t)(p0 + j) * elems] : 0.f;
#pragma unroll
      for (int j = 0; j < 8; ++j) acc += v[j];
    }
  }
  dw[(size_t)h * elems + e] = acc;
}

// dL/dr of the mixed attention (Eq. 6): the per-workgroup parts summed in a fixed order by one
// workgroup; zero outside the clip's range [0, 1].
__global__ __launch_bounds__(256) void dr_reduce_kernel(const float* __restrict__ part, int count,
                                                        const float* __restrict__ r, float* __restrict__ dr) {
  __shared__ float red[256];
  float acc = 0.f;
  for (int i = threadIdx.x; i < count; i += 256) acc += part[i];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int m = 128; m >= 1; m >>= 1) {
    if ((int)threadIdx.x < m) red[threadIdx.x] += red[threadIdx.x + m];
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    const float rv = *r;
    *dr = (rv >= 0.f && rv <= 1.f) ? red[0] : 0.f;
  }
}

__device__ __forceinline__ uint4 ld_nt16(const uint4* p) {
  typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}

// part[blockIdx.x] = sum over this workgroup's share of a[i] * b[i], both bf16 arrays of n16 16-byte
// pieces; fixed grid and fixed order inside a workgroup, so the result is reproducible.
__global__ __launch_bounds__(256) void dot_bf16_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                       size_t n16, float* __restrict__ part) {
  __shared__ float red[4];
  float acc = 0.f;
  auto term = [&](uint4 x, uint4 y) {
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc = fmaf(__builtin_bit_cast(float, xs[j] << 16), __builtin_bit_cast(float, ys[j] << 16), acc);
      acc = fmaf(__builtin_bit_cast(float, xs[j] & 0xffff0000u), __builtin_bit_cast(float, ys[j] & 0xffff0000u), acc);
    }
  };
  // four pieces of each array in flight per thread; the tail one piece at a time
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) { x[u] = ld_nt16(a + i + u * stride); y[u] = ld_nt16(b + i + u * stride); }
#pragma unroll
    for (int u = 0; u < 4; ++u) term(x[u], y[u]);
  }
  for (; i < n16; i += stride) term(a[i], b[i]);
  for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = acc;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The same with the head's mean value row taken off b: part = sum a[i] * (b[i] - vbar[bh(i)][ch(i)]), for a, b
// in the layout `rw` of the token tensors (d a power of two).  The query-side backward works with the output
// minus vbar; this is the matching form of the sum dout . s of the mixed attention's dL/dr.
__global__ __launch_bounds__(256) void dot_centred_bf16_kernel(const uint4* __restrict__ a, const uint4* __restrict__ b,
                                                               const float* __restrict__ vbar, size_t n16,
                                                               float* __restrict__ part, int n, int H, int d, int bnhd) {
  __shared__ float red[4];
  float acc = 0.f;
  const int dshift = d == 128 ? 7 : 6;
  auto term = [&](uint4 x, uint4 y, size_t i) {
    const size_t e0 = i * 8, row = e0 >> dshift;
    const int ch = (int)(e0 & (size_t)(d - 1));
    size_t bh;
    if (bnhd) { const size_t bt = row / (size_t)H; bh = (bt / (size_t)n) * H + (row - bt * H); }
    else bh = row / (size_t)n;
    const float* vb = vbar + bh * d + ch;
    const uint32_t xs[4] = {x.x, x.y, x.z, x.w}, ys[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      acc = fmaf(__builtin_bit_cast(float, xs[j] << 16), __builtin_bit_cast(float, ys[j] << 16) - vb[2 * j], acc);
      acc = fmaf(__builtin_bit_cast(float, xs[j] & 0xffff0000u), __builtin_bit_cast(float, ys[j] & 0xffff0000u) - vb[2 * j + 1], acc);
    }
  };
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 x[4], y[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) { x[u] = ld_nt16(a + i + u * stride); y[u] = ld_nt16(b + i + u * stride); }
#pragma unroll
    for (int u = 0; u < 4; ++u) term(x[u], y[u], i + u * stride);
  }
  for (; i < n16; i += stride) term(a[i], b[i], i);
  for (int m = 32; m >= 1; m >>= 1) acc += __shfl_xor(acc, m, 64);
  if (threadIdx.x % 64 == 0) red[threadIdx.x / 64] = acc;
  __syncthreads();
  if (threadIdx.x == 0) part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace

hipError_t launch_dot_centred_bf16(const void* a, const void* b, const float* vbar, float* part, const Plan& p, hipStream_t s) {
  const size_t elems = (size_t)p.BH * p.n * p.d;
  dot_centred_bf16_kernel<<<kDotParts, 256, 0, s>>>((const uint4*)a, (const uint4*)b, vbar, elems / 8, part, p.n, p.H, p.d,
                                                    p.rows.sn != (size_t)p.d);
  return hipGetLastError();
}

hipError_t launch_dot_bf16(const void* a, const void* b, size_t elems, float* part, hipStream_t s) {
  dot_bf16_kernel<<<kDotParts, 256, 0, s>>>((const uint4*)a, (const uint4*)b, elems / 8, part);
  return hipGetLastError();
}

hipError_t launch_dr_reduce(const float* part, int count, const float* r, float* dr, hipStream_t s) {
  dr_reduce_kernel<<<1, 256, 0, s>>>(part, count, r, dr);
  return hipGetLastError();
}

hipError_t launch_state_reduce(const float* partials, float* state, const Plan& p, hipStream_t s) {
  const int elems = (int)p.state_elems;
  state_reduce_kernel<<<dim3((elems + 255) / 256, p.BH), 256, 0, s>>>(partials, state, p.P, elems);
  return hipGetLastError();
}

hipError_t launch_state_reduce_split(const float* partials, float* state, const Plan& p, hipStream_t s) {
  const int elems = (int)p.state_elems;
  if (elems % 4 == 0 && ((reinterpret_cast<uintptr_t>(partials) | reinterpret_cast<uintptr_t>(state)) & 15u) == 0) {
    const int elems4 = elems / 4;
    state_reduce_split4_kernel<<<dim3((elems4 + 255) / 256, p.BH), 256, 0, s>>>(
        reinterpret_cast<const float4*>(partials), reinterpret_cast<float4*>(state), p.split, elems4);
  } else {
    state_reduce_split_kernel<<<dim3((elems + 255) / 256, p.BH), 256, 0, s>>>(partials, state, p.split, elems);
  }
  return hipGetLastError();
}

hipError_t launch_dw(const void* x, bool x_is_bf16, const float* du, float* part, float* dw, const Plan& p, hipStream_t s) {
  const int elems = p.d * (p.d / 2);
  const dim3 grid(p.P, p.BH);
  if (p.d == 128) {
    if (x_is_bf16) dw_partial_kernel<128, uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)x, du, part, p.H, p.n, p.P, p.chunk, p.rows);
    else dw_partial_kernel<128, float><<<grid, 256, 0, s>>>((const float*)x, du, part, p.H, p.n, p.P, p.chunk, p.rows);
  } else {
    if (x_is_bf16) dw_partial_kernel<64, uint16_t><<<grid, 256, 0, s>>>((const uint16_t*)x, du, part, p.H, p.n, p.P, p.chunk, p.rows);
    else dw_partial_kernel<64, float><<<grid, 256, 0, s>>>((const float*)x, du, part, p.H, p.n, p.P, p.chunk, p.rows);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_dw_reduce(part, dw, p, s);
}

hipError_t launch_dw_reduce(const float* part, float* dw, const Plan& p, hipStream_t s) {
  const int elems = p.d * (p.d / 2);
  dw_reduce_kernel<<<dim3((elems + 255) / 256, p.H), 256, 0, s>>>(part, dw, p.P, nullptr, nullptr, 0, p.B, p.H, elems);
  return hipGetLastError();
}

hipError_t launch_dw_reduce2(const float* part0, float* dw0, int P0, const float* part1, float* dw1, int P1, const Plan& p, hipStream_t s) {
  const int elems = p.d * (p.d / 2);
  dw_reduce_kernel<<<dim3((elems + 255) / 256, p.H, 2), 256, 0, s>>>(part0, dw0, P0, part1, dw1, P1, p.B, p.H, elems);
  return hipGetLastError();
}

}  // namespace linattn
