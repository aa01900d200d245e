// Memory-rate probe for the benchmark's roofline context: what a kernel that does nothing but stream
// reaches on this GPU, to set beside the published 8 TB/s.  Not part of the linear-attention library
// (it is built into a library of its own and only bench.py loads it).
//
//   kind 0: read `bytes` from src, every workgroup striding over the whole range, 8 non-temporal
//           16-byte loads in flight per thread; nothing is written (the xor of the data decides a
//           store that never happens).
//   kind 1: copy `bytes` from src to dst with non-temporal loads and stores, 4 in flight per thread.
//
// src, dst: device pointers, 16-byte aligned; bytes a multiple of 16.  Returns the hipError_t of the launch.
#include <hip/hip_runtime.h>
#include <cstddef>
#include <cstdint>

namespace {

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int U>
__global__ __launch_bounds__(256) void read_kernel(const u32x4* __restrict__ x, size_t n16, unsigned* sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  unsigned acc = 0;
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(x + i + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) acc ^= v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) {
    const u32x4 v = __builtin_nontemporal_load(x + i);
    acc ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (acc == 0x9E3779B9u && sink) sink[0] = acc;      // keeps the loads alive
}

template <int U>
__global__ __launch_bounds__(256) void copy_kernel(const u32x4* __restrict__ x, u32x4* __restrict__ y, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + (U - 1) * stride < n16; i += U * stride) {
    u32x4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(x + i + u * stride);
#pragma unroll
    for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], y + i + u * stride);
  }
  for (; i < n16; i += stride) __builtin_nontemporal_store(__builtin_nontemporal_load(x + i), y + i);
}

}  // namespace

extern "C" int membw_probe(int kind, const void* src, void* dst, size_t bytes, int workgroups, void* stream) {
  if (!src || (kind == 1 && !dst) || bytes % 16 || workgroups < 1 || (kind != 0 && kind != 1)) return (int)hipErrorInvalidValue;
  if (((uintptr_t)src | (uintptr_t)dst) % 16) return (int)hipErrorInvalidValue;
  hipStream_t s = (hipStream_t)stream;
  const size_t n16 = bytes / 16;
  if (kind == 0)
    read_kernel<8><<<workgroups, 256, 0, s>>>((const u32x4*)src, n16, (unsigned*)dst);
  else
    copy_kernel<4><<<workgroups, 256, 0, s>>>((const u32x4*)src, (u32x4*)dst, n16);
  return (int)hipGetLastError();
}
