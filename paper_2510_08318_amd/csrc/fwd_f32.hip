// fp32-arithmetic forward path: plain-FMA, LDS-tiled kernels, on fp32 tensors (no bf16 anywhere; the 1e-5
// accuracy contract) or on bf16 tensors widened on load (LINATTN_BF16_F32MATH: bf16 storage with none of
// the fp16 operands of the MFMA path).  The bandwidth-tuned path is the bf16 one in fwd_bf16.hip.
#include "kernels.h"
#include "f32_common.h"

namespace linattn {
namespace {

using namespace f32;
constexpr int TT = 32;        // tokens per tile

template <int D, int KIND, typename T>
__global__ __launch_bounds__(NT) void state_partials_f32_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                                const T* __restrict__ wk, float* __restrict__ partials,
                                                                int H, int n, int P, int chunk, Rows rw) {
  constexpr int HALF = D / 2;
  constexpr int BLK = D / 16;
  extern __shared__ float smem[];
  float* sW = smem;
  float* sX = sW + D * HALF;
  float* sV = sX + TT * (D + 1);
  float* sPhi = sV + TT * D;

  const int tid = threadIdx.x;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk;
  const int t_end = min(n, t_begin + chunk);
  const T* kb = k + head_base(rw, bh, H);
  const T* vb = v + head_base(rw, bh, H);
  const T* wb = wk + (size_t)h * D * HALF;
  if constexpr (KIND == kPhiHedgehog)
    for (int i = tid; i < D * HALF; i += NT) sW[i] = ldf(wb, i);

  float acc[BLK][BLK];
#pragma unroll
  for (int i = 0; i < BLK; ++i)
#pragma unroll
    for (int j = 0; j < BLK; ++j) acc[i][j] = 0.f;
  float zacc = 0.f;
  const int f0 = (tid / 16) * BLK, c0 = (tid % 16) * BLK;

  for (int t0 = t_begin; t0 < t_end; t0 += TT) {
    __syncthreads();
    for (int i = tid; i < TT * D; i += NT) {
      const int tt = i / D, c = i % D;
      const int t = t0 + tt;
      const bool valid = t < t_end;
      sX[tt * (D + 1) + c] = valid ? ldf(kb, (size_t)t * rw.sn + c) : 0.f;
      sV[tt * D + c] = valid ? ldf(vb, (size_t)t * rw.sn + c) : 0.f;
    }
    __syncthreads();
    phi_tile<D, TT, KIND>(sX, sW, sPhi, tid, t_end - t0);
    for (int tt = 0; tt < TT; ++tt) {
      float a[BLK], b[BLK];
#pragma unroll
      for (int i = 0; i < BLK; ++i) a[i] = sPhi[tt * D + f0 + i];
#pragma unroll
      for (int j = 0; j < BLK; ++j) b[j] = sV[tt * D + c0 + j];
#pragma unroll
      for (int i = 0; i < BLK; ++i)
#pragma unroll
        for (int j = 0; j < BLK; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    if (tid < D)
      for (int tt = 0; tt < TT; ++tt) zacc += sPhi[tt * D + tid];
  }

  float* dst = partials + ((size_t)bh * P + p) * (size_t)(D + 1) * D;
#pragma unroll
  for (int i = 0; i < BLK; ++i)
#pragma unroll
    for (int j = 0; j < BLK; ++j) dst[(f0 + i) * D + c0 + j] = acc[i][j];
  if (tid < D) dst[D * D + tid] = zacc;
}

template <int D, int KIND, typename T>
__global__ __launch_bounds__(NT) void apply_f32_kernel(const T* __restrict__ q, const T* __restrict__ wq,
                                                       const float* __restrict__ state, T* __restrict__ out,
                                                       const T* __restrict__ blend, const float* __restrict__ rptr,
                                                       int H, int n, int chunk, Rows rw) {
  constexpr int HALF = D / 2;
  extern __shared__ float smem[];
  float* sW = smem;
  float* sS = sW + D * HALF;            // [(D+1)][D]
  float* sX = sS + (D + 1) * D;
  float* sPhi = sX + TT * (D + 1);

  const int tid = threadIdx.x;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk;
  const int t_end = min(n, t_begin + chunk);
  const T* qb = q + head_base(rw, bh, H);
  T* ob = out + head_base(rw, bh, H);
  // mixed attention (Eq. 6): out = r' s + (1 - r') o with r' = clip(r, 0, 1); off when blend is null
  const T* bb = blend ? blend + head_base(rw, bh, H) : nullptr;
  const float rb = blend ? fminf(fmaxf(*rptr, 0.f), 1.f) : 0.f;
  const T* wb = wq + (size_t)h * D * HALF;
  const float* sb = state + (size_t)bh * (D + 1) * D;
  if constexpr (KIND == kPhiHedgehog)
    for (int i = tid; i < D * HALF; i += NT) sW[i] = ldf(wb, i);
  for (int i = tid; i < (D + 1) * D; i += NT) sS[i] = sb[i];

  const int tt = tid / 8, cb = tid % 8;
  for (int t0 = t_begin; t0 < t_end; t0 += TT) {
    __syncthreads();
    for (int i = tid; i < TT * D; i += NT) {
      const int r = i / D, c = i % D;
      const int t = t0 + r;
      sX[r * (D + 1) + c] = (t < t_end) ? ldf(qb, (size_t)t * rw.sn + c) : 0.f;
    }
    __syncthreads();
    phi_tile<D, TT, KIND>(sX, sW, sPhi, tid, t_end - t0);
    float acc[D / 8];
#pragma unroll
    for (int j = 0; j < D / 8; ++j) acc[j] = 0.f;
    float den = 0.f;
    for (int f = 0; f < D; ++f) {
      const float a = sPhi[tt * D + f];
      den = fmaf(a, sS[D * D + f], den);
#pragma unroll
      for (int j = 0; j < D / 8; ++j) acc[j] = fmaf(a, sS[f * D + cb + 8 * j], acc[j]);
    }
    const int t = t0 + tt;
    if (t < t_end) {
      const float inv = 1.0f / (KIND == kPhiRelu ? den + kReluEps : den);
#pragma unroll
      for (int j = 0; j < D / 8; ++j) {
        float val = acc[j] * inv;
        if (bb) val = fmaf(rb, ldf(bb, (size_t)t * rw.sn + cb + 8 * j) - val, val);
        stf(ob, (size_t)t * rw.sn + cb + 8 * j, val);
      }
    }
  }
}

template <int D>
constexpr size_t state_smem() { return sizeof(float) * (D * (D / 2) + TT * (D + 1) + TT * D + TT * D); }
template <int D>
constexpr size_t apply_smem() { return sizeof(float) * (D * (D / 2) + (D + 1) * D + TT * (D + 1) + TT * D); }

template <int D, int KIND, typename T>
hipError_t run_state(const void* k, const void* v, const void* wk, float* partials, const Plan& p, hipStream_t s) {
  hipError_t e = set_smem_once<state_partials_f32_kernel<D, KIND, T>>(state_smem<D>());
  if (e != hipSuccess) return e;
  state_partials_f32_kernel<D, KIND, T><<<dim3(p.P, p.BH), NT, state_smem<D>(), s>>>(
      (const T*)k, (const T*)v, (const T*)wk, partials, p.H, p.n, p.P, p.chunk, p.rows);
  return hipGetLastError();
}
template <int D, int KIND, typename T>
hipError_t run_apply(const void* q, const void* wq, const float* state, void* out,
                     const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s) {
  hipError_t e = set_smem_once<apply_f32_kernel<D, KIND, T>>(apply_smem<D>());
  if (e != hipSuccess) return e;
  apply_f32_kernel<D, KIND, T><<<dim3(p.QP, p.BH), NT, apply_smem<D>(), s>>>(
      (const T*)q, (const T*)wq, state, (T*)out, (const T*)blend_in, blend_r, p.H, p.n, p.qchunk, p.rows);
  return hipGetLastError();
}

template <typename T>
hipError_t state_any(const void* k, const void* v, const void* wk, float* partials, const Plan& p, hipStream_t s) {
  if (p.kind == kPhiRelu)
    return p.d == 128 ? run_state<128, kPhiRelu, T>(k, v, wk, partials, p, s) : run_state<64, kPhiRelu, T>(k, v, wk, partials, p, s);
  return p.d == 128 ? run_state<128, kPhiHedgehog, T>(k, v, wk, partials, p, s) : run_state<64, kPhiHedgehog, T>(k, v, wk, partials, p, s);
}
template <typename T>
hipError_t apply_any(const void* q, const void* wq, const float* state, void* out,
                     const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s) {
  if (p.kind == kPhiRelu)
    return p.d == 128 ? run_apply<128, kPhiRelu, T>(q, wq, state, out, blend_in, blend_r, p, s)
                      : run_apply<64, kPhiRelu, T>(q, wq, state, out, blend_in, blend_r, p, s);
  return p.d == 128 ? run_apply<128, kPhiHedgehog, T>(q, wq, state, out, blend_in, blend_r, p, s)
                    : run_apply<64, kPhiHedgehog, T>(q, wq, state, out, blend_in, blend_r, p, s);
}

}  // namespace

hipError_t launch_state_partials_f32(const void* k, const void* v, const void* wk, float* partials,
                                     const Plan& p, hipStream_t s) {
  return p.bf16_storage ? state_any<uint16_t>(k, v, wk, partials, p, s) : state_any<float>(k, v, wk, partials, p, s);
}

hipError_t launch_apply_f32(const void* q, const void* wq, const float* state, void* out,
                            const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s) {
  return p.bf16_storage ? apply_any<uint16_t>(q, wq, state, out, blend_in, blend_r, p, s)
                        : apply_any<float>(q, wq, state, out, blend_in, blend_r, p, s);
}

}  // namespace linattn
