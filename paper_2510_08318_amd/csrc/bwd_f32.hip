// fp32-arithmetic backward path: plain FMA on LDS tiles of 16 tokens, on fp32 tensors (no bf16/fp16
// anywhere: the 1e-5 accuracy contract) or on bf16 tensors widened on load and rounded on store
// (LINATTN_BF16_F32MATH).  Same mathematics as bwd_bf16.hip (chain rule through Eq. 3 and Eq. 5); not
// tuned for bandwidth.
#include "kernels.h"
#include "f32_common.h"

namespace linattn {
namespace {

using namespace f32;
constexpr int TB = 16;        // tokens per tile
constexpr int TPT = NT / TB;  // threads per token (16)

// du for a tile: sG [TB][D] = dL/dphi, sPhi [TB][D] = phi; writes sDU [TB][D/2].
// Contains __syncthreads(); sC: [TB][2] scratch.
template <int D>
__device__ __forceinline__ void jacobian_tile(const float* sG, const float* sPhi, float* sDU, float* sC, int tid) {
  constexpr int HALF = D / 2;
  if (tid < 2 * TB) {
    const int tt = tid / 2, half = tid % 2;
    float c = 0.f;
    for (int a = 0; a < HALF; ++a) c = fmaf(sG[tt * D + half * HALF + a], sPhi[tt * D + half * HALF + a], c);
    sC[tt * 2 + half] = c;
  }
  __syncthreads();
  for (int i = tid; i < TB * HALF; i += NT) {
    const int tt = i / HALF, a = i % HALF;
    sDU[tt * HALF + a] = sPhi[tt * D + a] * (sG[tt * D + a] - sC[tt * 2])
                       - sPhi[tt * D + HALF + a] * (sG[tt * D + HALF + a] - sC[tt * 2 + 1]);
  }
  __syncthreads();
}

// dx[tt][c] = sum_a du[tt][a] W[c][a], stored for valid tokens; optional copy of du to the workspace.
template <int D, typename T>
__device__ __forceinline__ void dx_tile(const float* sDU, const float* sW, T* xout, size_t sn, float* du_ws,
                                        int t0, int n_valid, int tid) {
  constexpr int HALF = D / 2;
  const int tt = tid / TPT, cb = tid % TPT;
  if (tt < n_valid) {
#pragma unroll 1
    for (int j = 0; j < D / TPT; ++j) {
      const int c = cb + TPT * j;
      float acc = 0.f;
      for (int a = 0; a < HALF; ++a) acc = fmaf(sDU[tt * HALF + a], sW[c * HALF + a], acc);
      stf(xout, (size_t)(t0 + tt) * sn + c, acc);
    }
    if (du_ws)
      for (int a = cb; a < HALF; a += TPT) du_ws[(size_t)(t0 + tt) * HALF + a] = sDU[tt * HALF + a];
  }
}

template <int D, int KIND, typename T>
__global__ __launch_bounds__(NT) void bwd_q_f32_kernel(const T* __restrict__ q, const T* __restrict__ dout,
                                                       const T* __restrict__ wq, const float* __restrict__ state,
                                                       T* __restrict__ dq, float* __restrict__ partials,
                                                       float* __restrict__ du_ws,
                                                       const T* __restrict__ blend, const float* __restrict__ rptr,
                                                       float* __restrict__ dr_part,
                                                       int H, int n, int P, int chunk, Rows rw) {
  constexpr int HALF = D / 2;
  constexpr int BLK = D / 16;
  constexpr int SS = D + 1;                 // row stride of the state copy (bank spread)
  extern __shared__ float smem[];
  float* sW = smem;                         // [D][HALF]
  float* sS = sW + D * HALF;                // [D+1][SS]
  float* sX = sS + (D + 1) * SS;            // [TB][D+1]
  float* sPhi = sX + TB * (D + 1);          // [TB][D]
  float* sDO = sPhi + TB * D;               // [TB][D]   dO, later dO / den
  float* sG = sDO + TB * D;                 // [TB][D]   o, then g
  float* sDU = sG + TB * D;                 // [TB][HALF]
  float* sDen = sDU + TB * HALF;            // [TB]
  float* sDel = sDen + TB;                  // [TB]
  float* sC = sDel + TB;                    // [TB][2]

  const int tid = threadIdx.x;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk, t_end = min(n, t_begin + chunk);
  const T* qb = q + head_base(rw, bh, H);
  const T* dob = dout + head_base(rw, bh, H);
  T* dqb = dq + head_base(rw, bh, H);
  // mixed attention (Eq. 6), off when blend is null: dout is the gradient of the mixed output
  const T* bb = blend ? blend + head_base(rw, bh, H) : nullptr;
  const float om = blend ? 1.f - fminf(fmaxf(*rptr, 0.f), 1.f) : 1.f;
  float dr_acc = 0.f;
  const T* wb = wq + (size_t)h * D * HALF;
  const float* sb = state + (size_t)bh * (D + 1) * D;
  if constexpr (KIND == kPhiHedgehog)
    for (int i = tid; i < D * HALF; i += NT) sW[i] = ldf(wb, i);
  for (int i = tid; i < (D + 1) * D; i += NT) sS[(i / D) * SS + (i % D)] = sb[i];

  float acc[BLK][BLK];
#pragma unroll
  for (int i = 0; i < BLK; ++i)
#pragma unroll
    for (int j = 0; j < BLK; ++j) acc[i][j] = 0.f;
  float zacc = 0.f;
  const int f0 = (tid / 16) * BLK, c0 = (tid % 16) * BLK;
  const int tt = tid / TPT, cb = tid % TPT;

  for (int t0 = t_begin; t0 < t_end; t0 += TB) {
    const int n_valid = min(TB, t_end - t0);
    __syncthreads();
    for (int i = tid; i < TB * D; i += NT) {
      const int r = i / D, c = i % D;
      const bool valid = r < n_valid;
      sX[r * (D + 1) + c] = valid ? ldf(qb, (size_t)(t0 + r) * rw.sn + c) : 0.f;
      sDO[r * D + c] = valid ? ldf(dob, (size_t)(t0 + r) * rw.sn + c) : 0.f;
    }
    __syncthreads();
    phi_tile<D, TB, KIND>(sX, sW, sPhi, tid, n_valid);     // rows >= n_valid are zero
    // o = phi S / den  -> sG, den -> sDen
    {
      float den = 0.f;
      for (int f = 0; f < D; ++f) den = fmaf(sPhi[tt * D + f], sS[D * SS + f], den);
      if constexpr (KIND == kPhiRelu) den += kReluEps;
      const float inv = tt < n_valid ? 1.0f / den : 0.f;
#pragma unroll 1
      for (int j = 0; j < D / TPT; ++j) {
        const int c = cb + TPT * j;
        float a = 0.f;
        for (int f = 0; f < D; ++f) a = fmaf(sPhi[tt * D + f], sS[f * SS + c], a);
        sG[tt * D + c] = a * inv;
      }
      if (cb == 0) sDen[tt] = tt < n_valid ? den : 1.f;
    }
    __syncthreads();
    if (tid < TB) {
      float dl = 0.f;
      for (int c = 0; c < D; ++c) dl = fmaf(sDO[tid * D + c], sG[tid * D + c], dl);
      if (bb) {
        if (tid < n_valid) {
          float ds = 0.f;
          for (int c = 0; c < D; ++c) ds = fmaf(sDO[tid * D + c], ldf(bb, (size_t)(t0 + tid) * rw.sn + c), ds);
          dr_acc += ds - dl;
        }
        for (int c = 0; c < D; ++c) sDO[tid * D + c] *= om;
        dl *= om;
      }
      sDel[tid] = dl;
    }
    __syncthreads();
    // g = (dO S^T - delta z) / den  -> sG (o is dead)
    {
      const float inv = 1.0f / sDen[tt];
      const float dl = sDel[tt];
      float gv[D / TPT];
#pragma unroll 1
      for (int j = 0; j < D / TPT; ++j) {
        const int f = cb + TPT * j;
        float a = 0.f;
        for (int c = 0; c < D; ++c) a = fmaf(sDO[tt * D + c], sS[f * SS + c], a);
        gv[j] = (a - dl * sS[D * SS + f]) * inv;
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < D / TPT; ++j) sG[tt * D + cb + TPT * j] = gv[j];
      // dO / den in place (operand of dS); delta / den
#pragma unroll 1
      for (int j = 0; j < D / TPT; ++j) sDO[tt * D + cb + TPT * j] *= inv;
      if (cb == 0) sDel[tt] = dl * inv;
    }
    __syncthreads();
    if constexpr (KIND == kPhiRelu) {
      // dq = g where q > 0 (this thread wrote these entries of sG itself)
      if (tt < n_valid)
        for (int j = 0; j < D / TPT; ++j) {
          const int c = cb + TPT * j;
          stf(dqb, (size_t)(t0 + tt) * rw.sn + c, sX[tt * (D + 1) + c] > 0.f ? sG[tt * D + c] : 0.f);
        }
    } else {
      jacobian_tile<D>(sG, sPhi, sDU, sC, tid);
      dx_tile<D, T>(sDU, sW, dqb, rw.sn, du_ws ? du_ws + (size_t)bh * n * HALF : nullptr, t0, n_valid, tid);
    }
    // dS += phi^T (dO / den), dz -= phi * (delta / den)
    for (int r = 0; r < TB; ++r) {
      float a[BLK], b[BLK];
#pragma unroll
      for (int i = 0; i < BLK; ++i) a[i] = sPhi[r * D + f0 + i];
#pragma unroll
      for (int j = 0; j < BLK; ++j) b[j] = sDO[r * D + c0 + j];
#pragma unroll
      for (int i = 0; i < BLK; ++i)
#pragma unroll
        for (int j = 0; j < BLK; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    if (tid < D)
      for (int r = 0; r < TB; ++r) zacc = fmaf(-sPhi[r * D + tid], sDel[r], zacc);
  }

  float* dst = partials + ((size_t)bh * P + p) * (size_t)(D + 1) * D;
#pragma unroll
  for (int i = 0; i < BLK; ++i)
#pragma unroll
    for (int j = 0; j < BLK; ++j) dst[(f0 + i) * D + c0 + j] = acc[i][j];
  if (tid < D) dst[D * D + tid] = zacc;
  if (bb) {
    __syncthreads();
    if (tid < TB) sC[tid] = dr_acc;
    __syncthreads();
    if (tid == 0) {
      float t = 0.f;
      for (int i = 0; i < TB; ++i) t += sC[i];
      dr_part[(size_t)bh * P + p] = t;
    }
  }
}

template <int D, int KIND, typename T>
__global__ __launch_bounds__(NT) void bwd_k_f32_kernel(const T* __restrict__ k, const T* __restrict__ v,
                                                       const T* __restrict__ wk, const float* __restrict__ dstate,
                                                       T* __restrict__ dk, T* __restrict__ dv,
                                                       float* __restrict__ du_ws, int H, int n, int chunk, Rows rw) {
  constexpr int HALF = D / 2;
  constexpr int SS = D + 1;
  extern __shared__ float smem[];
  float* sW = smem;
  float* sS = sW + D * HALF;                // dS, dz  [D+1][SS]
  float* sX = sS + (D + 1) * SS;            // [TB][D+1]
  float* sPhi = sX + TB * (D + 1);
  float* sV = sPhi + TB * D;
  float* sG = sV + TB * D;
  float* sDU = sG + TB * D;
  float* sC = sDU + TB * HALF;

  const int tid = threadIdx.x;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk, t_end = min(n, t_begin + chunk);
  const T* kb = k + head_base(rw, bh, H);
  const T* vb = v + head_base(rw, bh, H);
  T* dkb = dk + head_base(rw, bh, H);
  T* dvb = dv + head_base(rw, bh, H);
  const T* wb = wk + (size_t)h * D * HALF;
  const float* sb = dstate + (size_t)bh * (D + 1) * D;
  if constexpr (KIND == kPhiHedgehog)
    for (int i = tid; i < D * HALF; i += NT) sW[i] = ldf(wb, i);
  for (int i = tid; i < (D + 1) * D; i += NT) sS[(i / D) * SS + (i % D)] = sb[i];
  const int tt = tid / TPT, cb = tid % TPT;

  for (int t0 = t_begin; t0 < t_end; t0 += TB) {
    const int n_valid = min(TB, t_end - t0);
    __syncthreads();
    for (int i = tid; i < TB * D; i += NT) {
      const int r = i / D, c = i % D;
      const bool valid = r < n_valid;
      sX[r * (D + 1) + c] = valid ? ldf(kb, (size_t)(t0 + r) * rw.sn + c) : 0.f;
      sV[r * D + c] = valid ? ldf(vb, (size_t)(t0 + r) * rw.sn + c) : 0.f;
    }
    __syncthreads();
    phi_tile<D, TB, KIND>(sX, sW, sPhi, tid, n_valid);
    // dv = phi dS ; g = v dS^T + dz
#pragma unroll 1
    for (int j = 0; j < D / TPT; ++j) {
      const int c = cb + TPT * j;
      float a = 0.f, gsum = 0.f;
      for (int f = 0; f < D; ++f) a = fmaf(sPhi[tt * D + f], sS[f * SS + c], a);
      if (tt < n_valid) stf(dvb, (size_t)(t0 + tt) * rw.sn + c, a);
      const int f = c;
      for (int cc = 0; cc < D; ++cc) gsum = fmaf(sV[tt * D + cc], sS[f * SS + cc], gsum);
      sG[tt * D + f] = gsum + sS[D * SS + f];
    }
    __syncthreads();
    if constexpr (KIND == kPhiRelu) {
      if (tt < n_valid)
        for (int j = 0; j < D / TPT; ++j) {
          const int c = cb + TPT * j;
          stf(dkb, (size_t)(t0 + tt) * rw.sn + c, sX[tt * (D + 1) + c] > 0.f ? sG[tt * D + c] : 0.f);
        }
    } else {
      jacobian_tile<D>(sG, sPhi, sDU, sC, tid);
      dx_tile<D, T>(sDU, sW, dkb, rw.sn, du_ws ? du_ws + (size_t)bh * n * HALF : nullptr, t0, n_valid, tid);
    }
  }
}

template <int D>
constexpr size_t q_smem() {
  return sizeof(float) * (D * (D / 2) + (D + 1) * (D + 1) + TB * (D + 1) + 3 * TB * D + TB * (D / 2) + 4 * TB);
}
template <int D>
constexpr size_t k_smem() {
  return sizeof(float) * (D * (D / 2) + (D + 1) * (D + 1) + TB * (D + 1) + 3 * TB * D + TB * (D / 2) + 2 * TB);
}

template <int D, int KIND, typename T>
hipError_t run_bwd(const BwdArgs& a, const Plan& p, hipStream_t s) {
  hipError_t e;
  const dim3 grid(p.P, p.BH);
  constexpr bool kBf16 = sizeof(T) == 2;
  if ((e = set_smem_once<bwd_q_f32_kernel<D, KIND, T>>(q_smem<D>())) != hipSuccess) return e;
  bwd_q_f32_kernel<D, KIND, T><<<grid, NT, q_smem<D>(), s>>>((const T*)a.q, (const T*)a.dout, (const T*)a.wq, a.state,
                                                    (T*)a.dq, a.partials, a.dwq ? a.du_q : nullptr,
                                                    (const T*)a.blend_in, a.blend_r, a.dr_part, p.H, p.n, p.P, p.chunk, p.rows);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if (a.blend_in && a.blend_dr && (e = launch_dr_reduce(a.dr_part, p.BH * p.P, a.blend_r, a.blend_dr, s)) != hipSuccess) return e;
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = launch_state_reduce(a.partials, a.dstate, p, s)) != hipSuccess) return e;
  if ((e = set_smem_once<bwd_k_f32_kernel<D, KIND, T>>(k_smem<D>())) != hipSuccess) return e;
  bwd_k_f32_kernel<D, KIND, T><<<grid, NT, k_smem<D>(), s>>>((const T*)a.k, (const T*)a.v, (const T*)a.wk, a.dstate,
                                                    (T*)a.dk, (T*)a.dv, a.dwk ? a.du_k : nullptr, p.H, p.n, p.chunk, p.rows);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if constexpr (KIND == kPhiHedgehog) {
    if (a.dwq && (e = launch_dw(a.q, kBf16, a.du_q, a.dw_part, a.dwq, p, s)) != hipSuccess) return e;
    if (a.dwk && (e = launch_dw(a.k, kBf16, a.du_k, a.dw_part, a.dwk, p, s)) != hipSuccess) return e;
  }
  return hipSuccess;
}

template <typename T>
hipError_t bwd_any(const BwdArgs& a, const Plan& p, hipStream_t s) {
  if (p.kind == kPhiRelu) return p.d == 128 ? run_bwd<128, kPhiRelu, T>(a, p, s) : run_bwd<64, kPhiRelu, T>(a, p, s);
  return p.d == 128 ? run_bwd<128, kPhiHedgehog, T>(a, p, s) : run_bwd<64, kPhiHedgehog, T>(a, p, s);
}

}  // namespace

hipError_t launch_bwd_f32(const BwdArgs& a, const Plan& p, hipStream_t s) {
  return p.bf16_storage ? bwd_any<uint16_t>(a, p, s) : bwd_any<float>(a, p, s);
}

}  // namespace linattn
