// bf16-I/O backward path on gfx950 MFMA.  The paper trains through the converted layers
// (Sec. 5.1) but prints no gradient formula; these kernels apply the chain rule to Eq. 3 and Eq. 5.
// With S, z from the forward, den_i = phi(q_i).z, o_i = phi(q_i) S / den_i, delta_i = dO_i.o_i:
//
//   query side   g_i  = dL/dphi(q_i) = (dO_i S^T - delta_i z) / den_i
//                dS   = sum_i phi(q_i)^T dO_i / den_i          dz = -sum_i phi(q_i) delta_i / den_i
//   key side     g_j  = dL/dphi(k_j) = v_j dS^T + dz           dv_j = phi(k_j) dS
//   through phi  du = p+ (g+ - <g+,p+>) - p- (g- - <g-,p->),   dx = du W~^T,   dW~ = sum x^T du
//
// bwd_prep_kernel : fp16 operand image of S for g (rows = features, contraction over channels)
// bwd_q_kernel    : per 128-token tile: phi(Q), o, delta, g, du, dq; dS, dz partials (split-n); dW~_q partials
// bwd_k_kernel    : per 32-token block: phi(K), g, du, dk, dv; dW~_k partials
// (the partials are reduced in state_reduce.hip)
//
// Precision: every 16-bit MFMA operand except the stored bf16 q, k (projection) is fp16.
// Operands that belong to one token only (dO_i for g_i, du_i for dx_i) are scaled by a per-token
// power of two taken from their largest magnitude, so any gradient scale is safe.  Operands of
// the sums over tokens (dO_i/den_i, delta_i/den_i, du for dW~) are scaled by one power of two per
// workgroup that follows the running maximum over its tiles (largest magnitude so far in [16, 32));
// when a tile raises the maximum the fp32 accumulators are rescaled by the exact ratio, so neither a
// late large tile nor leading all-zero tiles can overflow or flush fp16; within a tile values down
// to 2^-18 of the running maximum keep full precision.  Accumulation is fp32 everywhere; partial
// sums are combined in a fixed order.
#include "kernels.h"
#include "mfma_common.h"

namespace linattn {
namespace {

// ---- operand images, built once per head ---------------------------------------------------
// The two main kernels need, per (b,h), MFMA operand images of S (resp. dS) in two index orders
// and, per head, two images of W~.  Building them costs scattered reads; done by every workgroup
// of a head it dominated the kernels' fixed cost, so they are built once here and the main
// kernels copy them into LDS with coalesced 16-byte loads.
//   grid (B*H, 8): slice blockIdx.y of the entries of (b,h); the workgroups of batch item 0 also
//   build the W~ images of their head (WQK = true: both W~_q and W~_k images into wimg).
//   WQK = true is the pass over S (image simg in the A-operand order of the query pass: the query
//   side wants o on the lane's own token); WQK = false is the pass over dS, whose image is in the
//   B-operand order of dv = phi(k) dS with the tokens on the accumulator rows.
// 512 threads: staging the state is latency, not bandwidth (256 threads: 16.8 + 10.8 us for the two
// passes at config 5, 512: 11.9 + 8.3 us, 1024 the same; more slices per head change nothing).
constexpr int PT = 512, PREP_Y = 8;
// Both passes centre the state before it is rounded to fp16 operands (exact in real arithmetic; the roundings
// then act on what the gradients are made of instead of on a common part that cancels):
//   pass over S:  S^c = S - z vbar^T with vbar = sum_j v_j / n (the + half of S sums to sum_j v_j, the + half
//                 of z to n).  The query-side kernel then works with o - vbar and delta^c = delta - dO . vbar, g is
//                 unchanged, and its dz comes out as dz^c = dz + dS vbar.
//   pass over dS: the key-side dz is completed against the ROUNDED image: dzc[f] = dz^c[f] - vbar . r(dS[f]), so
//                 that v_j . r(dS[f]) + dzc[f] = (v_j - vbar) . r(dS[f]) + dz^c[f] holds exactly and the rounding
//                 of the image acts on v_j - vbar, not on v_j (values with a common offset cost nothing).
//   CENTRE (LINATTN_FLAG_CENTRED): the query-side kernel accumulated dS' = sum (phi - 2/D)^T dO/den and dz' likewise;
//                 (2/D) x its column sums (cs_part) complete them: dS = dS' + (2/D) 1 colsum^T (constant over the
//                 features: it only enters the row that dv gets back), dz^c = dz' + (2/D) wsum.  In addition the
//                 mean over each half's features is taken out of dS' and of dz^c: the softmax Jacobian drops what
//                 is constant over a half, and dv gets the constant row mean_+ + mean_- back.  (Without the flag
//                 this last step is left out: where phi is spiky the rows of dS differ by orders of magnitude and
//                 a common shift only adds rounding error to the small ones.)
template <int D, bool WQK, bool CENTRE>
__global__ __launch_bounds__(PT) void bwd_prep_kernel(const float* __restrict__ state, uint4* __restrict__ gimg,
                                                       uint4* __restrict__ simg, float* __restrict__ scale_out,
                                                       const uint16_t* __restrict__ wq, const uint16_t* __restrict__ wk,
                                                       uint4* __restrict__ wimg, int H,
                                                       float* __restrict__ vbar, float* __restrict__ dv_row, float* __restrict__ dzc,
                                                       const float* __restrict__ cs_part, int P) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  using G = GradLayout<D>;
  constexpr int SIMG = L::KS * L::MBZ * 64;
  constexpr int WB_IMG = (C::LOC / 8) * L::MB * 64;
  // the state (and W~) is staged in LDS with coalesced loads; the scattered reads of the image
  // entries then hit LDS
  extern __shared__ uint4 prep_smem[];
  float* S = reinterpret_cast<float*>(prep_smem);                         // [(D+1)*D]
  uint16_t* sWq = reinterpret_cast<uint16_t*>(S + (D + 1) * D);          // [D*HALF], then W~_k
  uint16_t* sWk = sWq + D * C::HALF;
  __shared__ float red[PT / 64];
  const int bh = blockIdx.x, tid = threadIdx.x;
  {
    const uint4* g = reinterpret_cast<const uint4*>(state + (size_t)bh * (D + 1) * D);
    for (int i = tid; i < (D + 1) * D / 4; i += PT) reinterpret_cast<uint4*>(S)[i] = g[i];
    if constexpr (WQK) {
      if (bh < H) {
        const uint4* gq = reinterpret_cast<const uint4*>(wq + (size_t)bh * D * C::HALF);
        const uint4* gk = reinterpret_cast<const uint4*>(wk + (size_t)bh * D * C::HALF);
        for (int i = tid; i < D * C::HALF / 8; i += PT) {
          reinterpret_cast<uint4*>(sWq)[i] = gq[i];
          reinterpret_cast<uint4*>(sWk)[i] = gk[i];
        }
      }
    }
  }
  __syncthreads();
  __shared__ float cA[D], cB[D], cC[D];
  constexpr int HF = D / 2;
  constexpr int PARTS = PT / D;                    // threads per channel (or feature) in the sums below
  __shared__ float part[PT];
  if constexpr (WQK) {
    {
      // column sums of the + half of S, PARTS threads per channel over HF / PARTS rows each; the + half of z sums to n
      const int ch = tid % D, q = tid / D;
      float sv = 0.f;
      for (int f = q * (HF / PARTS); f < (q + 1) * (HF / PARTS); ++f) sv += S[f * D + ch];
      part[tid] = sv;
    }
    __syncthreads();
    if (tid < D) {
      float sv = 0.f, nt = 0.f;
      for (int q = 0; q < PARTS; ++q) sv += part[q * D + tid];
      for (int f = 0; f < HF; ++f) nt += S[D * D + f];
      const float vb = sv / nt;
      cA[tid] = vb;
      if (blockIdx.y == 0) vbar[(size_t)bh * D + tid] = vb;
    }
    __syncthreads();
    for (int i = tid; i < D * D; i += PT) S[i] -= S[D * D + i / D] * cA[i % D];
    __syncthreads();
  } else {
    // colsum (cA) and wsum of the query-side workgroups, in a fixed order (CENTRE only); vbar (cC)
    if (tid < D) {
      float t = 0.f;
      if constexpr (CENTRE)
        for (int p = 0; p < P; ++p) t += cs_part[((size_t)bh * P + p) * (D + 8) + tid];
      cA[tid] = t;
      cC[tid] = vbar[(size_t)bh * D + tid];
    } else if (tid == D) {
      float t = 0.f;
      if constexpr (CENTRE)
        for (int p = 0; p < P; ++p) t += cs_part[((size_t)bh * P + p) * (D + 8) + D];
      red[0] = t;
    }
    __syncthreads();
    const float wsum = red[0];
    // means over each half: of dS per channel (thread = channel); dz^c (cB)
    float m0 = 0.f, m1 = 0.f;
    if (tid < D) {
      for (int f = 0; f < HF; ++f) { m0 += S[f * D + tid]; m1 += S[(HF + f) * D + tid]; }
      m0 *= 1.0f / HF; m1 *= 1.0f / HF;
      if constexpr (!CENTRE) { m0 = 0.f; m1 = 0.f; }
      if (blockIdx.y == 0) dv_row[(size_t)bh * D + tid] = (m0 + m1) + (4.0f / D) * cA[tid];
      cB[tid] = S[D * D + tid] + (2.0f / D) * wsum;
    }
    __syncthreads();
    if (tid < D) cA[tid] = m0;
    __syncthreads();
    for (int i = tid; i < HF * D; i += PT) S[i] -= cA[i % D];
    __syncthreads();
    if (tid < D) cA[tid] = m1;
    if (tid == D) {
      float a = 0.f, b = 0.f;
      for (int f = 0; f < HF; ++f) { a += cB[f]; b += cB[HF + f]; }
      red[0] = CENTRE ? a * (1.0f / HF) : 0.f; red[1] = CENTRE ? b * (1.0f / HF) : 0.f;
    }
    __syncthreads();
    for (int i = HF * D + tid; i < D * D; i += PT) S[i] -= cA[i % D];
    if (tid < D) {
      cB[tid] -= tid < HF ? red[0] : red[1];
      S[D * D + tid] = 0.f;            // the image's z block is not used on the key side and stays out of the scale
    }
    __syncthreads();
  }
  const float scale = head_scale<D, PT>(S, red, tid);      // every block of a head computes the same value
  if (blockIdx.y == 0 && tid == 0) scale_out[2 * bh] = scale;
  if constexpr (!WQK) {
    if (blockIdx.y == 0) {
      // PARTS adjacent threads per feature, D / PARTS channels each, combined inside the wavefront
      const int f = tid / PARTS, q = tid % PARTS;
      const float inv = __builtin_amdgcn_rcpf(scale);       // exact: a power of two
      float dot = 0.f;
      for (int ch = q * (D / PARTS); ch < (q + 1) * (D / PARTS); ++ch)
        dot = fmaf((float)(_Float16)(scale * S[f * D + ch]), cC[ch], dot);
      for (int m = 1; m < PARTS; m <<= 1) dot += __shfl_xor(dot, m, 64);
      if (q == 0) dzc[(size_t)bh * D + f] = cB[f] - dot * inv;
    }
  }
  const int first = blockIdx.y * PT + tid, step = PT * gridDim.y;
  if constexpr (WQK) {
    // one tile for both products of the query side, then the z block (together as large as an image of S)
    constexpr int TILE = D * D / 8;
    static_assert(TILE + L::KS * 64 == SIMG, "tile + z block fill the image region");
    for (int idx = first; idx < TILE; idx += step) simg[(size_t)bh * SIMG + idx] = state_tile_entry<D>(S, scale, idx);
    for (int idx = first; idx < L::KS * 64; idx += step) simg[(size_t)bh * SIMG + TILE + idx] = state_z_entry<D>(S, scale, idx);
  } else {
    for (int idx = first; idx < G::IMG; idx += step) gimg[(size_t)bh * G::IMG + idx] = grad_image_entry<D>(S, scale, idx);
    for (int idx = first; idx < SIMG; idx += step) simg[(size_t)bh * SIMG + idx] = state_image_entry<D, true>(S, scale, idx);
  }
  if constexpr (WQK) {
    if (bh < H) {
      static_assert(C::W_IMG == WB_IMG, "the four W~ images have one size");
      uint4* dst = wimg + (size_t)bh * 4 * C::W_IMG;
      for (int idx = first; idx < C::W_IMG; idx += step) {
        dst[idx] = w_image_entry<D>(sWq, idx);
        dst[C::W_IMG + idx] = w_image_t_entry<D>(sWq, idx);
        dst[2 * C::W_IMG + idx] = w_image_entry<D>(sWk, idx);
        dst[3 * C::W_IMG + idx] = w_image_t_entry<D>(sWk, idx);
      }
    }
  }
}

template <int D>
constexpr size_t prep_smem_bytes() { return (size_t)(D + 1) * D * sizeof(float) + 2 * (size_t)D * (D / 2) * 2; }

// Softmax Jacobian of Eq. 5 for one token spread over a lane pair: gacc holds g in the GradLayout
// row order (first GM/2 blocks the softmax(+u) half, then the softmax(-u) half), already scaled.
template <int D>
__device__ __forceinline__ void phi_jacobian(const float (&gp)[Cfg<D>::LOC], const float (&gm)[Cfg<D>::LOC],
                                             const float (&pp)[Cfg<D>::LOC], const float (&pm)[Cfg<D>::LOC],
                                             float (&du)[Cfg<D>::LOC]) {
  using C = Cfg<D>;
  float cp = 0.f, cm = 0.f;
#pragma unroll
  for (int j = 0; j < C::LOC; ++j) { cp = fmaf(gp[j], pp[j], cp); cm = fmaf(gm[j], pm[j], cm); }
  float lo, hi;
  pair32(cp, lo, hi); cp = lo + hi;
  pair32(cm, lo, hi); cm = lo + hi;
#pragma unroll
  for (int j = 0; j < C::LOC; ++j) du[j] = pp[j] * (gp[j] - cp) - pm[j] * (gm[j] - cm);
}

// dx = du W~^T for one block of 32 tokens, tokens on the accumulator rows: du is scaled by one power
// of two per block (its largest magnitude lands in [1,2)), cast to fp16 and fed as the A operand
// (lane (t,g) holds features g*LOC + 8ks + e of token t); the B operands are the W~ image.
// acc[mb][r] of lane (c,g) is its * dx[token 8*(r/4) + 4g + r%4][channel MB*c + mb].
//
// dub receives the scaled fp16 du as packed (lane (t,g): features g*LOC .. g*LOC + LOC-1 of token t; zero for tokens
// that do not exist), blk_its the inverse scale (0 for an all-zero block): what the dW~ contraction parks.
// AHEAD: lookahead of the W~ operand reads of dx (pipelined_operands).
template <int D, int AHEAD>
__device__ __forceinline__ void du_to_dx(const float (&du)[Cfg<D>::LOC], const uint4* sWB, int lane, bool valid,
                                         f32x16 (&acc)[D / 32], float& its, uint32_t (&dub)[Cfg<D>::LOC / 2], float& blk_its) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  constexpr int DK = C::LOC / 8;
  float m = 0.f;
#pragma unroll
  for (int j = 0; j < C::LOC; ++j) m = fmaxf(m, fabsf(du[j]));
  if (!valid) m = 0.f;
  float lo, hi;
  pair32(m, lo, hi); m = fmaxf(lo, hi);
  m = wave_max_paired(m);
  const float ts = valid ? pow2_normaliser(m) : 0.f;
#pragma unroll
  for (int j = 0; j < C::LOC / 2; ++j) dub[j] = pack_f16x2(du[2 * j] * ts, du[2 * j + 1] * ts);
  its = __builtin_amdgcn_rcpf(pow2_normaliser(m));     // exact: a power of two
  blk_its = m > 0.f ? its : 0.f;
#pragma unroll
  for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[mb][r] = 0.f;
  const uint4* wb = sWB + lane + opaque_zero();
  pipelined_operands<DK * L::MB, AHEAD>(
      [&](int i) { return wb[i * 64]; },
      [&](int i, uint4 b) {
        const int ks = i / L::MB, mb = i % L::MB;
        uint4 aq; aq.x = dub[4 * ks]; aq.y = dub[4 * ks + 1]; aq.z = dub[4 * ks + 2]; aq.w = dub[4 * ks + 3];
        acc[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(aq), as_f16x8(b), acc[mb], 0, 0, 0);
      });
}

// ---- dW~ = sum_i x_i^T du_i, accumulated inside the kernels that make du ---------------------
// The workgroup parks 128 tokens in LDS as two fp16 tiles, x [kTile][D] and du [kTile][D/2] (rows swizzled
// like the phi tile; a 32-token block of du carries the power-of-two scale du_to_dx gave it, with the
// inverse scales beside the tile).  Its NW wavefronts then contract over the tokens with transposing
// reads of both tiles: wavefront w owns the feature block w % NB and RB 32-channel row blocks and brings
// the blocks to one common power-of-two scale that follows the running maximum of the workgroup
// (gamma_step; the accumulators are rescaled by the exact ratio when a tile raises it).  Partials per
// workgroup are reduced in a fixed order afterwards.
template <int D, int NW>
struct DwTile {
  static constexpr int HALF = D / 2;
  static constexpr int LOC = D / 4;
  static constexpr int RSX = D * 2;                        // bytes per row of the x tile
  static constexpr int RSU = HALF * 2;                     // bytes per row of the du tile
  static constexpr int NB = HALF / 32;                     // 32-column blocks of du
  static constexpr int RB = (D / 32) * NB >= NW ? (D / 32) * NB / NW : 1;   // row blocks per wavefront
  static constexpr int BPT = kTile / 32;                   // du blocks per parked tile
  static constexpr int KSN = kTile / 16;
  static constexpr int KBATCH = NW > 4 ? KSN / 2 : KSN;     // k-steps whose operands are in flight together
  static constexpr int DU_BYTES = kTile * RSU;
  f32x16 acc[RB];
  float gamma;
  int fb, row0;
  bool active;

  __device__ __forceinline__ void init(int w) {
    fb = w % NB; row0 = (w / NB) * RB;
    active = row0 < D / 32;
    gamma = kGammaUnset;
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
  }
  // The x rows of block slot (0..3) as the projection holds them: lane (t,g) has the 16-byte chunks 2ks + g of token t.
  static __device__ __forceinline__ void park_x(const uint4 (&xr)[D / 16], char* sX, int slot, int lane) {
    const int row = 32 * slot + lane % 32, g = lane / 32;
    char* rowp = sX + row * RSX;
#pragma unroll
    for (int ks = 0; ks < D / 16; ++ks) {
      uint4 hv;
      hv.x = bf16x2_to_f16x2(xr[ks].x); hv.y = bf16x2_to_f16x2(xr[ks].y);
      hv.z = bf16x2_to_f16x2(xr[ks].z); hv.w = bf16x2_to_f16x2(xr[ks].w);
      *reinterpret_cast<uint4*>(rowp + (((2 * ks + g) ^ swz<D>(row)) * 16)) = hv;
    }
  }
  // The scaled fp16 du of block slot (0..3) of the parked tile, as du_to_dx packs it: lane (t,g) holds features
  // g*LOC .. g*LOC + LOC-1 of token t.
  static __device__ __forceinline__ void park_du(const uint32_t (&dub)[LOC / 2], float blk_its, char* sU, float* sIts, int slot, int lane) {
    const int row = 32 * slot + lane % 32, g = lane / 32;
    char* rowp = sU + row * RSU;
#pragma unroll
    for (int c = 0; c < LOC / 8; ++c) {
      uint4 v; v.x = dub[4 * c]; v.y = dub[4 * c + 1]; v.z = dub[4 * c + 2]; v.w = dub[4 * c + 3];
      *reinterpret_cast<uint4*>(rowp + (((g * (LOC / 8) + c) ^ swz<HALF>(row)) * 16)) = v;
    }
    if (lane == 0) sIts[slot] = blk_its;
  }
  // lane: pass lane + opaque_zero() from inside the tile loop: the read offsets are then worked out per tile (a few
  // integer operations) instead of being held in registers, or spilled, across the whole loop
  __device__ __forceinline__ void contract(const char* sX, const char* sU, const float* sIts, int lane) {
    float its[BPT];
    float m = 0.f;
#pragma unroll
    for (int i = 0; i < BPT; ++i) { its[i] = sIts[i]; m = fmaxf(m, its[i]); }
    float gnext = gamma;
    float ratio = gamma_step(gnext, gamma_for(m));
    // the same in every lane: kept in scalar registers
    gamma = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, gnext)));
    ratio = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, ratio)));
    if (ratio != 1.f) {
#pragma unroll
      for (int j = 0; j < RB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] *= ratio;
    }
    if (!active) return;
    int offA[RB][2], offB[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      offB[j] = tr_offset_g4<HALF>(32 * fb, lane, j);
#pragma unroll
      for (int i = 0; i < RB; ++i) offA[i][j] = tr_offset_g4<D>(32 * (row0 + i), lane, j);
    }
    // the operands of KBATCH k-steps are requested before their first MFMA: one LDS latency per batch instead of one
    // per k-step (the whole tile at once where the wavefront has 512 registers, half of it where it has 256)
#pragma unroll
    for (int k0 = 0; k0 < KSN; k0 += KBATCH) {
      f16x8 a[KBATCH][RB], b[KBATCH];
#pragma unroll
      for (int ks = 0; ks < KBATCH; ++ks) {
        b[ks] = read_tr(sU + (k0 + ks) * 16 * RSU, offB[0], offB[1]);
#pragma unroll
        for (int i = 0; i < RB; ++i) a[ks][i] = read_tr(sX + (k0 + ks) * 16 * RSX, offA[i][0], offA[i][1]);
      }
#pragma unroll
      for (int ks = 0; ks < KBATCH; ++ks) {
        const _Float16 f = (_Float16)(gamma * its[(k0 + ks) / 2]);   // a power of two, or 0 for an all-zero block
        const f16x8 bo = b[ks] * f;
#pragma unroll
        for (int i = 0; i < RB; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ks][i], bo, acc[i], 0, 0, 0);
      }
    }
  }
  // part: this workgroup's [D][HALF] partial
  __device__ __forceinline__ void store(float* part, int lane) const {
    if (!active) return;
    const float ig = __builtin_amdgcn_rcpf(gamma);
    const int c = lane % 32, g = lane / 32;
#pragma unroll
    for (int i = 0; i < RB; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        part[(32 * (row0 + i) + 8 * (r / 4) + 4 * g + (r % 4)) * HALF + 32 * fb + c] = acc[i][r] * ig;
  }
};

// ---- query side --------------------------------------------------------------------------
// LDS operands of the query-side kernel's MFMA phases are requested QAHEAD MFMAs before their use (one more for g):
// with one wavefront per SIMD nothing else hides an LDS latency.  3 (4 for g) against 5 (6): 296 -> 293 us per
// backward call at the training shape; 8 measures between the two.
constexpr int QAHEAD = 5;
// BLEND: dout is the gradient of the mixed output of Eq. 6; the linear branch receives
// (1 - r') dout, and the workgroup's part of -sum dout . o goes to dr_part (dL/dr = sum dout . (s - o);
// the sum dout . s is a separate streaming dot product, taken only when dL/dr is asked for).
// DW: dW~_q is accumulated here as well (DwTile): after the tile's dS contraction the phi and dO tiles in LDS
// are dead, and the tile's q rows (read again: the registers that held them are long reused) and du images
// take their place.
template <int D, bool BLEND, bool CENTRE, bool DW>
__global__ __launch_bounds__(NT) void bwd_q_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ dout,
                                                   const uint16_t* __restrict__ wq, const float* __restrict__ state,
                                                   const uint4* __restrict__ simg,
                                                   const uint4* __restrict__ wimg, const float* __restrict__ scales,
                                                   uint16_t* __restrict__ dq,
                                                   float* __restrict__ partials, float* __restrict__ dw_part,
                                                   const uint16_t* __restrict__ blend, const float* __restrict__ rptr,
                                                   float* __restrict__ dr_part,
                                                   float* __restrict__ cs_part,
                                                   int H, int n, int P, Rows rw) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  using G = GradLayout<D>;
  constexpr int RS = D * 2;
  constexpr int WMN = D / 64;
  constexpr int SA_IMG = L::KS * L::MBZ * 64;
  constexpr int WB_IMG = (C::LOC / 8) * L::MB * 64;
  constexpr float kMean = 2.0f / D;                        // mean of phi over its features
  using DWT = DwTile<D, NT / 64>;
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  uint4* sSA = sWA + C::W_IMG;                             // the state tile (state_tile_entry), then its z block
  const char* sT = reinterpret_cast<const char*>(sSA);
  uint4* sWB = sSA + SA_IMG;
  char* sPhi = reinterpret_cast<char*>(sWB + WB_IMG);      // [kTile][D] fp16: phi(q) (CENTRE: phi(q) - 2/D)
  char* sDO = sPhi + kTile * RS;                           // [kTile][D] fp16: gamma * dO / den
  uint16_t* sW16 = reinterpret_cast<uint16_t*>(sDO + kTile * RS);   // [kTile] fp16: -gamma * delta / den
  float* sZ = reinterpret_cast<float*>(sW16 + kTile);      // [D] z, unscaled
  float* sRed = sZ + D;                                    // [8]: 0..3 the tile's operand maxima, 4..7 the du blocks' inverse scales
  char* sDU = reinterpret_cast<char*>(sRed + 8);           // DW: the tile's du, [kTile][D/2] fp16

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32;
  const int mi = w / 2, ni = w % 2;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const uint16_t* qb = q + head_base(rw, bh, H);
  const uint16_t* dob = dout + head_base(rw, bh, H);
  uint16_t* dqb = dq + head_base(rw, bh, H);
  const float om = BLEND ? 1.f - fminf(fmaxf(*rptr, 0.f), 1.f) : 1.f;      // 1 - r'
  float dr_acc = 0.f;
  const float* sb = state + (size_t)bh * (D + 1) * D;
  const int ntile = (n + kTile - 1) / kTile;
  const int nblk = (n + 31) / 32;

  copy_image<NT>(wimg + (size_t)h * 4 * C::W_IMG, sWA, C::W_IMG, tid);
  copy_image<NT>(wimg + (size_t)h * 4 * C::W_IMG + C::W_IMG, sWB, WB_IMG, tid);
  copy_image<NT>(simg + (size_t)bh * SA_IMG, sSA, SA_IMG, tid);
  const float scale = scales[2 * bh];
  for (int i = tid; i < D; i += NT) sZ[i] = sb[D * D + i];
  __syncthreads();

  float csum[WMN], wsum = 0.f;                     // column sums of the dO/den operand, sum of the -delta/den operand
#pragma unroll
  for (int j = 0; j < WMN; ++j) csum[j] = 0.f;
  f32x16 s[WMN][WMN], zacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zacc[r] = 0.f;
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < WMN; ++j) s[i][j][r] = 0.f;
  }
  const int zmb = (WMN == 2) ? (2 * mi + ni) : mi;
  const bool do_z = (WMN == 2) || (ni == 0);
  // read offsets of the dS contraction; DW: worked out again in every tile (registers are what is short there)
  int offA[WMN][2], offB[WMN][2];
  auto set_offsets = [&](int ln) {
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        offA[i][j] = tr_offset<D>(32 * (mi * WMN + i), ln, j);
        offB[i][j] = tr_offset<D>(32 * (ni * WMN + i), ln, j);
      }
  };
  if constexpr (!DW) set_offsets(lane);
  const int prow = 32 * w + (lane % 32);
  const int psw = swz<D>(prow);
  float gamma = kGammaUnset;
  DWT dwt;
  if constexpr (DW) dwt.init(w);

  // the lane's q rows of the next tile are requested late in this tile, behind the softmax Jacobian: the
  // middle of the chain is where registers are short (never behind a branch: after the last tile the rows
  // are simply read again); its dO rows are requested at the top of the tile and first needed after the
  // projection, the softmaxes and o
  uint4 xq[C::UK];
  auto load_rows = [&](uint4 (&x)[C::UK], int tile) {
    const int t = tile * kTile + prow;
    const uint4* row = reinterpret_cast<const uint4*>(qb + (size_t)(t < n ? t : n - 1) * rw.sn);
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) x[ks] = row[2 * ks + g];
  };
  auto load_q = [&](int tile) { load_rows(xq, tile); };
  load_q(p < ntile ? p : 0);
  for (int tile = p; tile < ntile; tile += P) {
    const int t = tile * kTile + prow;
    const bool valid = t < n;
    const int tc = valid ? t : (n - 1);
    uint4 dor[D / 16];
    {
      const uint4* drow = reinterpret_cast<const uint4*>(dob + (size_t)tc * rw.sn + g * (D / 2));
#pragma unroll
      for (int i = 0; i < D / 16; ++i) dor[i] = drow[i];
    }
    // dL/dr gets dout . (s - o) = dout . s - delta, from the unscaled dout; everything downstream is
    // linear in dout, so the factor 1 - r' is applied to the scalars that carry it (om below).
    // dout . s is taken here, while few registers are live.
    f32x16 u[C::UM];
    project<D, QAHEAD>(xq, sWA, lane, u);
    uint4 xr[C::UK];                              // this tile's rows once more, for dW~ (rows past n repeat row n - 1: their du is zero)
    if constexpr (DW) {
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) xr[ks] = xq[ks];
    }
    float pp[C::LOC], pm[C::LOC];
    uint32_t pk[C::NPK];
    softmax_full<D>(u, pp, pm, pk);

    // o = phi(q) S / den on the lane's channels g*D/2 + 16*mb + r
    float o[D / 2];
    float den_s;                                   // scale * den
    {
      f32x16 oa[L::MB], dn;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dn[r] = 0.f;
#pragma unroll
        for (int mb = 0; mb < L::MB; ++mb) oa[mb][r] = 0.f;
      }
      const int lz = lane + opaque_zero();
      const uint4* szi = sSA + D * D / 8 + lz;     // the z block behind the tile
      int offT[L::MB][2];
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int j = 0; j < 2; ++j) offT[mb][j] = tr_offset<D>(32 * mb, lz, j);
      pipelined_operands<L::KS * L::MBZ, QAHEAD>(
          [&](int i) {
            const int ks = i / L::MBZ, mb = i % L::MBZ;
            if (mb == L::MB) return szi[ks * 64];
            return __builtin_bit_cast(uint4, read_tr(sT + ks * 16 * RS, offT[mb < L::MB ? mb : 0][0], offT[mb < L::MB ? mb : 0][1]));
          },
          [&](int i, uint4 a) {
            const int ks = i / L::MBZ, mb = i % L::MBZ;
            uint4 bq; bq.x = pk[4 * ks]; bq.y = pk[4 * ks + 1]; bq.z = pk[4 * ks + 2]; bq.w = pk[4 * ks + 3];
            if (mb < L::MB) oa[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), as_f16x8(bq), oa[mb], 0, 0, 0);
            else dn = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), as_f16x8(bq), dn, 0, 0, 0);
          });
      den_s = dn[0];
      const float inv = __builtin_amdgcn_rcpf(den_s);
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[16 * mb + r] = oa[mb][r] * inv;
    }
    const float inv_den = scale * __builtin_amdgcn_rcpf(den_s);     // 1 / den

    // dO on the same channels, delta = dO . o
    float dof[D / 2];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) unpack_bf16x8(dor[i], dof + 8 * i);
    float delta = 0.f, dmax = 0.f;
#pragma unroll
    for (int c = 0; c < D / 2; ++c) { delta = fmaf(dof[c], o[c], delta); dmax = fmaxf(dmax, fabsf(dof[c])); }
    if constexpr (BLEND) {
      // the -dout . o part of dout . (s - o), on this lane's channels; the images are centred, so o here is
      // o - vbar: the other part of the sum is taken as dout . (s - vbar) to match
      if (valid) dr_acc -= delta;
    }
    float lo, hi;
    pair32(delta, lo, hi); delta = lo + hi;
    pair32(dmax, lo, hi); dmax = fmaxf(lo, hi);
    const float stok = pow2_normaliser(dmax);

    // operands of the sums over tokens, parked now so that phi and dO need not stay in registers
    // through the rest of the block
    {
      // the tile's largest operand of the two sums, |dO_i| / den_i or |delta_i| / den_i
      float m = valid ? fmaxf(dmax, fabsf(delta)) * inv_den * om : 0.f;
      m = wave_max_paired(m);
      if (lane == 0) sRed[w] = m;
    }
    __syncthreads();                             // previous tile's operand reads are done
    {
      const float m = fmaxf(fmaxf(sRed[0], sRed[1]), fmaxf(sRed[2], sRed[3]));
      float gnext = gamma;
      float ratio = gamma_step(gnext, gamma_for(m));
      // the same in every lane: kept in scalar registers
      gamma = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, gnext)));
      ratio = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, ratio)));
      if (ratio != 1.f) {                        // this tile is larger than every earlier one
        if constexpr (CENTRE) {
          wsum *= ratio;
#pragma unroll
          for (int j = 0; j < WMN; ++j) csum[j] *= ratio;
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          zacc[r] *= ratio;
#pragma unroll
          for (int i = 0; i < WMN; ++i)
#pragma unroll
            for (int j = 0; j < WMN; ++j) s[i][j][r] *= ratio;
        }
      }
    }
    {
      char* rowp = sPhi + prow * RS;
      constexpr int CPH = C::LOC / 8;
#pragma unroll
      for (int c = 0; c < CPH; ++c) {
        // CENTRE: phi minus its mean over the features, rounded after the subtraction: the fp16 rounding then acts
        // on the deviation from the uniform map; (2/D) x the column sums are added back by the prep kernel
        uint4 a, b;
        if constexpr (CENTRE) {
          a.x = pack_f16x2(pp[8 * c] - kMean, pp[8 * c + 1] - kMean);     a.y = pack_f16x2(pp[8 * c + 2] - kMean, pp[8 * c + 3] - kMean);
          a.z = pack_f16x2(pp[8 * c + 4] - kMean, pp[8 * c + 5] - kMean); a.w = pack_f16x2(pp[8 * c + 6] - kMean, pp[8 * c + 7] - kMean);
          b.x = pack_f16x2(pm[8 * c] - kMean, pm[8 * c + 1] - kMean);     b.y = pack_f16x2(pm[8 * c + 2] - kMean, pm[8 * c + 3] - kMean);
          b.z = pack_f16x2(pm[8 * c + 4] - kMean, pm[8 * c + 5] - kMean); b.w = pack_f16x2(pm[8 * c + 6] - kMean, pm[8 * c + 7] - kMean);
        } else {
          a.x = pk[4 * c]; a.y = pk[4 * c + 1]; a.z = pk[4 * c + 2]; a.w = pk[4 * c + 3];
          b.x = pk[C::LOC / 2 + 4 * c]; b.y = pk[C::LOC / 2 + 4 * c + 1];
          b.z = pk[C::LOC / 2 + 4 * c + 2]; b.w = pk[C::LOC / 2 + 4 * c + 3];
        }
        if (!valid) { a = make_uint4(0, 0, 0, 0); b = a; }
        *reinterpret_cast<uint4*>(rowp + (((g * CPH + c) ^ psw) * 16)) = a;
        *reinterpret_cast<uint4*>(rowp + (((C::CH / 2 + g * CPH + c) ^ psw) * 16)) = b;
      }
      const float sc = valid ? inv_den * gamma * om : 0.f;
      char* drowp = sDO + prow * RS;
#pragma unroll
      for (int c = 0; c < D / 16; ++c) {
        uint4 a;
        a.x = pack_f16x2(dof[8 * c] * sc, dof[8 * c + 1] * sc);     a.y = pack_f16x2(dof[8 * c + 2] * sc, dof[8 * c + 3] * sc);
        a.z = pack_f16x2(dof[8 * c + 4] * sc, dof[8 * c + 5] * sc); a.w = pack_f16x2(dof[8 * c + 6] * sc, dof[8 * c + 7] * sc);
        *reinterpret_cast<uint4*>(drowp + (((g * (C::CH / 2) + c) ^ psw) * 16)) = a;
      }
      if (g == 0) sW16[prow] = (uint16_t)(pack_f16x2(valid ? -delta * sc : 0.f, 0.f) & 0xffffu);
    }

    // g = (dO S^T - delta z) / den, rows laid out like phi
    float gp[C::LOC], gm[C::LOC];
    {
      f32x16 ga[G::GM];
#pragma unroll
      for (int mb = 0; mb < G::GM; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) ga[mb][r] = 0.f;
      // A operand (ks, mb): the lane's feature row of block mb, channels g*D/2 + 8ks .. +7 = chunks 2ks and 2ks+1
      // of that row, the lane group's 8 bytes of each (state_tile_entry)
      const int lz = lane + opaque_zero();
      const char* grow = sT + state_tile_grad_row<D>(lz);
      const int sw16 = swz<D>((state_tile_grad_row<D>(lz) / RS) % 16) * 16;
      pipelined_operands<G::KS * G::GM, QAHEAD + 1>(
          [&](int i) {
            const int ks = i / G::GM, mb = i % G::GM;
            const char* rowp = grow + 32 * mb * RS;
            const uint2 lo = *reinterpret_cast<const uint2*>(rowp + ((32 * ks) ^ sw16));
            const uint2 hi = *reinterpret_cast<const uint2*>(rowp + ((32 * ks + 16) ^ sw16));
            return make_uint4(lo.x, lo.y, hi.x, hi.y);
          },
          [&](int i, uint4 a) {
            const int ks = i / G::GM, mb = i % G::GM;
            uint4 bq;
            bq.x = pack_f16x2(dof[8 * ks] * stok, dof[8 * ks + 1] * stok);     bq.y = pack_f16x2(dof[8 * ks + 2] * stok, dof[8 * ks + 3] * stok);
            bq.z = pack_f16x2(dof[8 * ks + 4] * stok, dof[8 * ks + 5] * stok); bq.w = pack_f16x2(dof[8 * ks + 6] * stok, dof[8 * ks + 7] * stok);
            ga[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), as_f16x8(bq), ga[mb], 0, 0, 0);
          });
      const float r1 = om * __builtin_amdgcn_rcpf(den_s * stok);     // (1 - r') / (scale * stok * den)
      const float r2 = om * delta * inv_den;
#pragma unroll
      for (int mb = 0; mb < G::GM; ++mb) {
        const int f0 = (mb < G::GM / 2 ? 0 : C::HALF) + g * C::LOC + 16 * (mb % (G::GM / 2));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float val = ga[mb][r] * r1 - r2 * sZ[f0 + r];
          if (mb < G::GM / 2) gp[16 * mb + r] = val; else gm[16 * (mb - G::GM / 2) + r] = val;
        }
      }
    }
    float du[C::LOC];
    phi_jacobian<D>(gp, gm, pp, pm, du);

    // The next tile's q rows, and (DW) this tile's rows once more for dW~, wanted after the dS contraction.  Both go
    // out before the dq stores: loads and stores retire in order, and a wait for a load issued behind the
    // stores would wait for the stores as well.
    load_q(tile + P < ntile ? tile + P : tile);

    {
      f32x16 xa[L::MB];
      float its;
      const int blk = tile * (kTile / 32) + w;
      uint32_t dub[C::LOC / 2];
      float blk_its = 0.f;
      du_to_dx<D, QAHEAD>(du, sWB, lane, valid, xa, its, dub, blk_its);
      // the previous tile's dW~ contraction has read its du tile: every wavefront has passed this tile's first barrier since
      if constexpr (DW) DWT::park_du(dub, blk_its, sDU, sRed + 4, w, lane);
      store_token_rows<D>(dqb, rw.sn, blk * 32, n, lane, xa, its);
    }

    __syncthreads();
    if constexpr (DW) set_offsets(lane + opaque_zero());
    contract_tile<D, false, CENTRE>(sPhi, sDO, offA, offB, s, zacc, ni != 0, do_z,
                     [&](int ks) { return as_f16x8(*reinterpret_cast<const uint4*>(sW16 + 16 * ks + 8 * g)); }, csum, &wsum);
    if constexpr (DW) {
      __syncthreads();                           // every wavefront is done with the phi and dO tiles
      DWT::park_x(xr, sPhi, w, lane);
      __syncthreads();
      dwt.contract(sPhi, sDU, sRed + 4, lane + opaque_zero());
      // the next tile's barrier before it parks phi and dO covers these reads
    }
  }
  if constexpr (DW) dwt.store(dw_part + ((size_t)bh * P + p) * (size_t)D * C::HALF, lane);

  const float ig = __builtin_amdgcn_rcpf(gamma);    // exact: gamma is a power of two
  if constexpr (CENTRE) {
    // column sums of dO/den (the wavefronts mi = 0 hold every channel block once) and the sum of -delta/den
    float* cs = cs_part + ((size_t)bh * P + p) * (D + 8);
#pragma unroll
    for (int j = 0; j < WMN; ++j) {
      float lo, hi;
      pair32(csum[j], lo, hi);
      if (mi == 0 && g == 0) cs[32 * (ni * WMN + j) + (lane % 32)] = (lo + hi) * ig;
    }
    float lo, hi;
    pair32(wsum, lo, hi);
    if (w == 0 && lane == 0) cs[D] = (lo + hi) * ig;
  }
  float* dst = partials + ((size_t)bh * P + p) * (size_t)(D + 1) * D;
  const int c = lane % 32;
#pragma unroll
  for (int i = 0; i < WMN; ++i)
#pragma unroll
    for (int j = 0; j < WMN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int f = 32 * (mi * WMN + i) + 8 * (r / 4) + 4 * g + (r % 4);
        dst[f * D + 32 * (ni * WMN + j) + c] = s[i][j][r] * ig;
      }
  if (do_z && c == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) dst[D * D + 32 * zmb + 8 * (r / 4) + 4 * g + (r % 4)] = zacc[r] * ig;
  }
  if constexpr (BLEND) {
    for (int k = 32; k >= 1; k >>= 1) dr_acc += __shfl_xor(dr_acc, k, 64);
    __syncthreads();
    if (lane == 0) sRed[w] = dr_acc;
    __syncthreads();
    if (tid == 0) dr_part[(size_t)bh * P + p] = (sRed[0] + sRed[1]) + (sRed[2] + sRed[3]);
  }
}

// ---- key side ----------------------------------------------------------------------------
constexpr int NTK = 512;     // 8 wavefronts, one workgroup per compute unit
// Operand lookahead of the key-side MFMA phases.  With two wavefronts per SIMD the other wavefront
// hides the LDS latency and registers are what is short: reading each operand right before its
// MFMA (0) measured 101.5 us, one ahead 102.9, three ahead 106.7, the compiler's own order 105.
constexpr int KAHEAD = 0;

// DW: dW~_k is accumulated here as well (DwTile).  The eight wavefronts then walk their blocks in step: after each
// round of eight blocks the wavefronts 0-3 park their k rows (read again) and du, all eight contract over those
// 128 tokens (one 32 x 32 block of dW~_k each), then the same for the blocks of the wavefronts 4-7.
template <int D, bool DW>
__global__ __launch_bounds__(NTK) void bwd_k_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                    const uint16_t* __restrict__ wk, const float* __restrict__ dstate,
                                                    const uint4* __restrict__ dsimg, const uint4* __restrict__ dgimg,
                                                    const uint4* __restrict__ wimg, const float* __restrict__ scales,
                                                    uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                                    float* __restrict__ dw_part,
                                                    const float* __restrict__ dzc, const float* __restrict__ dv_row,
                                                    int H, int n, Rows rw) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  using G = GradLayout<D>;
  constexpr int NW = NTK / 64;
  constexpr int SA_IMG = L::KS * L::MBZ * 64;
  constexpr int WB_IMG = (C::LOC / 8) * L::MB * 64;
  using DWT = DwTile<D, NW>;
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  uint4* sVA = sWA + C::W_IMG;             // image of dS^T for dv (contraction over features)
  uint4* sGA = sVA + SA_IMG;               // image of dS for g (contraction over channels)
  uint4* sWB = sGA + G::IMG;
  float* sZ = reinterpret_cast<float*>(sWB + WB_IMG);   // [D] dz, unscaled
  float* sRed = sZ + D;                                 // [8]: DW: 0..3 the parked du blocks' inverse scales
  char* sX = reinterpret_cast<char*>(sRed + 8);         // DW: [kTile][D] fp16, k rows of four blocks
  char* sU = sX + kTile * D * 2;                        // DW: [kTile][D/2] fp16, their du

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32;
  const int bh = blockIdx.y, h = bh % H;
  const uint16_t* kb = k + head_base(rw, bh, H);
  const uint16_t* vb = v + head_base(rw, bh, H);
  uint16_t* dkb = dk + head_base(rw, bh, H);
  uint16_t* dvb = dv + head_base(rw, bh, H);
  const float* ds = dstate + (size_t)bh * (D + 1) * D;

  copy_image<NTK>(wimg + (size_t)h * 4 * C::W_IMG + 2 * C::W_IMG, sWA, C::W_IMG, tid);
  copy_image<NTK>(wimg + (size_t)h * 4 * C::W_IMG + 3 * C::W_IMG, sWB, WB_IMG, tid);
  copy_image<NTK>(dsimg + (size_t)bh * SA_IMG, sVA, SA_IMG, tid);
  copy_image<NTK>(dgimg + (size_t)bh * G::IMG, sGA, G::IMG, tid);
  const float scale = scales[2 * bh + 1];
  // dzc is dz matched to the rounded image of dS (and, with LINATTN_FLAG_CENTRED, to its centring over the
  // features, for which dv gets a constant row back): see bwd_prep_kernel
  for (int i = tid; i < D; i += NTK) sZ[i] = dzc[(size_t)bh * D + i];
  __syncthreads();
  const float inv_scale = __builtin_amdgcn_rcpf(scale);    // exact: power of two
  float dv_add[L::MB];
#pragma unroll
  for (int mb = 0; mb < L::MB; ++mb) dv_add[mb] = dv_row[(size_t)bh * D + L::MB * (lane % 32) + mb];

  const int nblk = (n + 31) / 32;
  const int stride = gridDim.x * NW;
  uint4 xk[C::UK], vr[D / 16];
  auto load_rows = [&](uint4 (&x)[C::UK], int b) {
    const int t = b * 32 + (lane % 32);
    const int tc = t < n ? t : (n - 1);
    const uint4* row = reinterpret_cast<const uint4*>(kb + (size_t)tc * rw.sn);
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) x[ks] = row[2 * ks + g];
  };
  auto load_k = [&](int b) { load_rows(xk, b); };
  auto load_v = [&](int b) {
    const int t = b * 32 + (lane % 32);
    const int tc = t < n ? t : (n - 1);
    const uint4* vrow = reinterpret_cast<const uint4*>(vb + (size_t)tc * rw.sn + g * (D / 2));
#pragma unroll
    for (int i = 0; i < D / 16; ++i) vr[i] = vrow[i];
  };
  DWT dwt;
  if constexpr (DW) dwt.init(w);
  // DW: every wavefront of the workgroup makes the same number of rounds (there are barriers inside); a wavefront
  // whose block does not exist works on tokens past n: its loads repeat row n - 1, its du is zero, its stores go
  // to the sink
  int b = blockIdx.x * NW + w;
  if (DW || b < nblk) load_k(b);
  for (int b0 = blockIdx.x * NW; DW ? b0 < nblk : b < nblk; b0 += stride, b += stride) {
    const int t = b * 32 + (lane % 32);
    const bool valid = t < n;
    load_v(b);                                        // wanted after the projection, the softmax and dv
    f32x16 u[C::UM];
    project<D>(xk, sWA, lane, u);
    if constexpr (!DW) {
      if (b + stride < nblk) load_k(b + stride);      // next block's k flies during this one
    }
    float pp[C::LOC], pm[C::LOC];
    uint32_t pk[C::NPK];
    softmax_full<D>(u, pp, pm, pk);

    // dv = phi(k) dS, tokens on the accumulator rows
    {
      f32x16 va[L::MB];
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) va[mb][r] = 0.f;
      const uint4* sva = sVA + lane + opaque_zero();
      pipelined_operands<L::KS * L::MB, KAHEAD>(
          [&](int i) { return sva[((i / L::MB) * L::MBZ + i % L::MB) * 64]; },
          [&](int i, uint4 b) {
            const int ks = i / L::MB, mb = i % L::MB;
            uint4 aq; aq.x = pk[4 * ks]; aq.y = pk[4 * ks + 1]; aq.z = pk[4 * ks + 2]; aq.w = pk[4 * ks + 3];
            va[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(aq), as_f16x8(b), va[mb], 0, 0, 0);
          });
      store_token_rows<D>(dvb, rw.sn, b * 32, n, lane, va, inv_scale, dv_add);
    }

    // g = v dS^T + dz, rows laid out like phi
    float gp[C::LOC], gm[C::LOC];
    {
      f32x16 ga[G::GM];
#pragma unroll
      for (int mb = 0; mb < G::GM; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) ga[mb][r] = 0.f;
      const uint4* sga = sGA + lane + opaque_zero();
      pipelined_operands<G::KS * G::GM, KAHEAD>(
          [&](int i) { return sga[i * 64]; },
          [&](int i, uint4 a) {
            const int ks = i / G::GM, mb = i % G::GM;
            uint4 bq;
            bq.x = bf16x2_to_f16x2(vr[ks].x); bq.y = bf16x2_to_f16x2(vr[ks].y);
            bq.z = bf16x2_to_f16x2(vr[ks].z); bq.w = bf16x2_to_f16x2(vr[ks].w);
            ga[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), as_f16x8(bq), ga[mb], 0, 0, 0);
          });
#pragma unroll
      for (int mb = 0; mb < G::GM; ++mb) {
        const int f0 = (mb < G::GM / 2 ? 0 : C::HALF) + g * C::LOC + 16 * (mb % (G::GM / 2));
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float val = fmaf(ga[mb][r], inv_scale, sZ[f0 + r]);
          if (mb < G::GM / 2) gp[16 * mb + r] = val; else gm[16 * (mb - G::GM / 2) + r] = val;
        }
      }
    }
    float du[C::LOC];
    phi_jacobian<D>(gp, gm, pp, pm, du);
    {
      f32x16 xa[L::MB];
      float its;
      uint32_t dub[C::LOC / 2];
      float blk_its = 0.f;
      du_to_dx<D, KAHEAD>(du, sWB, lane, valid, xa, its, dub, blk_its);
      uint4 xr[C::UK];
      if constexpr (DW) {
        // the next block's k rows (with the dW~ accumulator resident they do not fit beside the middle of the chain) and
        // this block's rows once more; both before the dk stores: a wait for them must not wait for the stores
        load_k(b + stride);
        load_rows(xr, b);
      }
      store_token_rows<D>(dkb, rw.sn, b * 32, n, lane, xa, its);
      if constexpr (DW) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          __syncthreads();                             // the tiles' previous readers are done
          if (w / 4 == half) {
            // (addresses worked out here, from a lane index the optimiser cannot hoist: held across the loop they end up
            // in scratch memory, and a wait for a scratch load also waits for the dk stores just issued)
            const int lz = lane + opaque_zero();
            DWT::park_x(xr, sX, w % 4, lz);
            DWT::park_du(dub, blk_its, sU, sRed, w % 4, lz);
          }
          __syncthreads();
          dwt.contract(sX, sU, sRed, lane + opaque_zero());
        }
      }
    }
  }
  if constexpr (DW) dwt.store(dw_part + ((size_t)bh * gridDim.x + blockIdx.x) * (size_t)D * C::HALF, lane);
}

template <int D, bool DW>
constexpr size_t q_smem() {
  return sizeof(uint4) * (Cfg<D>::W_IMG + ApplyLayout<D>::KS * ApplyLayout<D>::MBZ * 64 + (Cfg<D>::LOC / 8) * ApplyLayout<D>::MB * 64)
       + 2 * (size_t)kTile * D * 2 + kTile * 2 + (D + 8) * sizeof(float) + (DW ? DwTile<D, NT / 64>::DU_BYTES : 0);
}
template <int D, bool DW>
constexpr size_t k_smem() {
  return sizeof(uint4) * (Cfg<D>::W_IMG + ApplyLayout<D>::KS * ApplyLayout<D>::MBZ * 64 + GradLayout<D>::IMG
                          + (Cfg<D>::LOC / 8) * ApplyLayout<D>::MB * 64) + (D + 8) * sizeof(float)
       + (DW ? (size_t)kTile * D * 2 + DwTile<D, NTK / 64>::DU_BYTES : 0);
}
template <auto Kernel>
struct KernelTag {
  static constexpr auto value = Kernel;
};
template <int D, bool CENTRE>
hipError_t run_bwd(const BwdArgs& a, const Plan& p, hipStream_t s) {
  hipError_t e;
  if ((e = set_smem_once<bwd_prep_kernel<D, true, CENTRE>>(prep_smem_bytes<D>())) != hipSuccess) return e;
  if ((e = set_smem_once<bwd_prep_kernel<D, false, CENTRE>>(prep_smem_bytes<D>())) != hipSuccess) return e;
  bwd_prep_kernel<D, true, CENTRE><<<dim3(p.BH, PREP_Y), PT, prep_smem_bytes<D>(), s>>>(a.state, nullptr, (uint4*)a.simg, a.scales,
                                                       (const uint16_t*)a.wq, (const uint16_t*)a.wk, (uint4*)a.wimg, p.H,
                                                       a.vbar, nullptr, nullptr, nullptr, p.P);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  // dW~ partials: [BH][P] blocks of the query side, then [BH][KP] of the key side
  const size_t side_elems = (size_t)p.BH * p.P * D * (D / 2);
  auto launch_q = [&](auto kernel) -> hipError_t {
    const size_t smem = a.dwq ? q_smem<D, true>() : q_smem<D, false>();
    hipError_t e2 = set_smem_once<decltype(kernel)::value>(smem);
    if (e2 != hipSuccess) return e2;
    decltype(kernel)::value<<<dim3(p.P, p.BH), NT, smem, s>>>(
        (const uint16_t*)a.q, (const uint16_t*)a.dout, (const uint16_t*)a.wq, a.state,
        (const uint4*)a.simg, (const uint4*)a.wimg, a.scales,
        (uint16_t*)a.dq, a.partials, a.dw_part,
        (const uint16_t*)a.blend_in, a.blend_r, a.blend_in ? a.dr_part : nullptr, a.cs_part, p.H, p.n, p.P, p.rows);
    return hipGetLastError();
  };
  if (a.blend_in) {
    e = a.dwq ? launch_q(KernelTag<bwd_q_kernel<D, true, CENTRE, true>>{}) : launch_q(KernelTag<bwd_q_kernel<D, true, CENTRE, false>>{});
    if (e != hipSuccess) return e;
    if (a.blend_dr) {
      if ((e = launch_dot_centred_bf16(a.dout, a.blend_in, a.vbar, a.dr_part + (size_t)p.BH * p.P, p, s)) != hipSuccess) return e;
      if ((e = launch_dr_reduce(a.dr_part, p.BH * p.P + kDotParts, a.blend_r, a.blend_dr, s)) != hipSuccess) return e;
    }
  } else {
    e = a.dwq ? launch_q(KernelTag<bwd_q_kernel<D, false, CENTRE, true>>{}) : launch_q(KernelTag<bwd_q_kernel<D, false, CENTRE, false>>{});
    if (e != hipSuccess) return e;
  }
  if ((e = launch_state_reduce(a.partials, a.dstate, p, s)) != hipSuccess) return e;
  // images of dS: the second half of the scales array, no W~ images
  bwd_prep_kernel<D, false, CENTRE><<<dim3(p.BH, PREP_Y), PT, prep_smem_bytes<D>(), s>>>(a.dstate, (uint4*)a.dgimg, (uint4*)a.dsimg, a.scales + 1,
                                                        nullptr, nullptr, nullptr, p.H, a.vbar, a.dv_row, a.dzc, a.cs_part, p.P);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  auto launch_k = [&](auto kernel, size_t smem) -> hipError_t {
    hipError_t e2 = set_smem_once<decltype(kernel)::value>(smem);
    if (e2 != hipSuccess) return e2;
    decltype(kernel)::value<<<dim3(p.KP, p.BH), NTK, smem, s>>>(
        (const uint16_t*)a.k, (const uint16_t*)a.v, (const uint16_t*)a.wk, a.dstate,
        (const uint4*)a.dsimg, (const uint4*)a.dgimg, (const uint4*)a.wimg, a.scales,
        (uint16_t*)a.dk, (uint16_t*)a.dv, a.dw_part + side_elems, a.dzc, a.dv_row, p.H, p.n, p.rows);
    return hipGetLastError();
  };
  e = a.dwk ? launch_k(KernelTag<bwd_k_kernel<D, true>>{}, k_smem<D, true>()) : launch_k(KernelTag<bwd_k_kernel<D, false>>{}, k_smem<D, false>());
  if (e != hipSuccess) return e;
  if (a.dwq || a.dwk) {
    if ((e = launch_dw_reduce2(a.dwq ? a.dw_part : nullptr, a.dwq, p.P, a.dwk ? a.dw_part + side_elems : nullptr, a.dwk, p.KP, p, s)) != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_bwd_bf16(const BwdArgs& a, const Plan& p, hipStream_t s) {
  if (p.centred) return p.d == 128 ? run_bwd<128, true>(a, p, s) : run_bwd<64, true>(a, p, s);
  return p.d == 128 ? run_bwd<128, false>(a, p, s) : run_bwd<64, false>(a, p, s);
}

}  // namespace linattn
