// Device-side building blocks shared by the bf16-I/O forward and backward kernels (gfx950 MFMA,
// tokens along the N dimension): operand images in LDS, the two halves of Eq. 5, transposing
// LDS reads.  Header-only; include after kernels.h.
#pragma once
#include "mfma_layout.h"

namespace linattn {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int NT = 256;          // 4 wavefronts (tile-synchronised kernels)

template <int D>
struct Cfg {
  static constexpr int HALF = D / 2;     // pre-softmax features u = x W~
  static constexpr int UM = HALF / 32;   // row blocks of U^T
  static constexpr int UK = D / 16;      // k-steps over the d input channels
  static constexpr int LOC = HALF / 2;   // pre-softmax features a lane owns
  static constexpr int NPK = D / 4;      // packed fp16 pairs of phi a lane owns (d/2 values)
  static constexpr int CH = D / 8;       // 16-byte chunks per tile row
  static constexpr int W_IMG = UK * UM * 64;   // uint4 entries of the W~^T operand image
};

// XOR swizzle of the 16-byte chunk index inside a tile row: makes the transposing 8-byte reads
// (4 consecutive rows x 32 bytes per 16 lanes) and the 16-byte row writes hit distinct banks.
// Depends on r % 16 only, so it is the same for every 16-row k-step of a tile.
template <int D>
__device__ __forceinline__ int swz(int r) {
  if (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  if (D == 32) return r & 3;                               // 4 chunks per row
  return (((r & 3) << 1) ^ ((r >> 2) & 3)) & 7;
}

// A zero the optimiser cannot see through: added to an LDS index it keeps loop-invariant
// operand reads inside the loop (hoisted, they would not fit the register file and spill).
__device__ __forceinline__ int opaque_zero() {
  int z = 0;
  asm volatile("" : "+v"(z));
  return z;
}

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
// Streaming (non-temporal) 16-byte global load / store, for fully coalesced accesses only: with
// the operand-layout loads (two 16-byte pieces of a row per instruction, four instructions per
// 128-byte line) the hint makes the line be fetched again and costs 20 % of the bandwidth.
__device__ __forceinline__ uint4 ld_nt(const uint4* p) {
  return __builtin_bit_cast(uint4, __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p)));
}
__device__ __forceinline__ void st_nt(uint4* p, uint4 v) {
  __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(p));
}

// Exchange with lane^32: returns (value of the low-half lane, value of the high-half lane),
// identical in both lanes of a pair.
__device__ __forceinline__ void pair32(float x, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  lo = __builtin_bit_cast(float, (uint32_t)r[0]);
  hi = __builtin_bit_cast(float, (uint32_t)r[1]);
}

// W~ [D][D/2] bf16 (one head) -> LDS image of the A operands of U^T = W~^T X^T:
// entry (ks, mb, lane=(m,g)) holds W~[16ks + 8g + e][owned_row<HALF>(mb, m)], e = 0..7.
template <int D>
__device__ __forceinline__ uint4 w_image_entry(const uint16_t* __restrict__ w, int idx) {
  using C = Cfg<D>;
  const int lane = idx % 64, mb = (idx / 64) % C::UM, ks = idx / (64 * C::UM);
  const int m = lane % 32, g = lane / 32;
  const int uf = owned_row<C::HALF>(mb, m);
  uint32_t x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = w[(16 * ks + 8 * g + e) * C::HALF + uf];
  uint4 r;
  r.x = x[0] | (x[1] << 16); r.y = x[2] | (x[3] << 16);
  r.z = x[4] | (x[5] << 16); r.w = x[6] | (x[7] << 16);
  return r;
}
template <int D, int NTHREADS>
__device__ __forceinline__ void build_w_image(const uint16_t* __restrict__ w, uint4* sWA, int tid) {
  for (int idx = tid; idx < Cfg<D>::W_IMG; idx += NTHREADS) sWA[idx] = w_image_entry<D>(w, idx);
}

// N uses (MFMAs) of 16-byte operands that come from LDS or global memory, each requested AHEAD uses
// before it is needed.  Left to itself the compiler, short of registers, issues read, wait, MFMA,
// read, wait, MFMA: with one wavefront per SIMD nothing hides those waits.  AHEAD = 0 keeps that
// order but fences it, so that a single operand is live at a time.
template <int N, int AHEAD, typename Load, typename Use>
__device__ __forceinline__ void pipelined_operands(Load load, Use use) {
  uint4 op[N];
#pragma unroll
  for (int i = 0; i < AHEAD && i < N; ++i) op[i] = load(i);
#pragma unroll
  for (int i = 0; i < N; ++i) {
    if (i + AHEAD < N) op[i + AHEAD] = load(i + AHEAD);
    __builtin_amdgcn_sched_barrier(0);
    use(i, op[i]);
    __builtin_amdgcn_sched_barrier(0);
  }
}

// First half of Eq. 5 for the 32 tokens of one wavefront: U^T = W~^T X^T on bf16 MFMA.
// xb[ks] is this lane's B operand (8 channels of its token per k-step).  On return the lane holds
// u[mb][r] = pre-softmax feature g*LOC + 16*mb + r of its token.  xb is dead afterwards, so the
// caller can refill it with the next block while the softmax runs.
// AHEAD > 0: the W~ operands are requested that many MFMAs ahead (pipelined_operands).
template <int D, int AHEAD = 0>
__device__ __forceinline__ void project(const uint4 (&xb)[Cfg<D>::UK], const uint4* sWA, int lane,
                                        f32x16 (&u)[Cfg<D>::UM]) {
  using C = Cfg<D>;
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) u[mb][r] = 0.f;
  const uint4* wa = sWA + lane + opaque_zero();
  if constexpr (AHEAD > 0) {
    pipelined_operands<C::UK * C::UM, AHEAD>(
        [&](int i) { return wa[i * 64]; },
        [&](int i, uint4 a) {
          u[i % C::UM] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(xb[i / C::UM]), u[i % C::UM], 0, 0, 0);
        });
    return;
  }
#pragma unroll
  for (int ks = 0; ks < C::UK; ++ks) {
    const bf16x8 b = as_bf16x8(xb[ks]);
#pragma unroll
    for (int mb = 0; mb < C::UM; ++mb) {
      const bf16x8 a = as_bf16x8(wa[(ks * C::UM + mb) * 64]);
      u[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, u[mb], 0, 0, 0);
    }
  }
}

// Sum of the two fp16 halves of a packed pair, added to an fp32 accumulator (v_dot2_f32_f16 against (1, 1):
// exact products, fp32 sum).
__device__ __forceinline__ float add_pair_f16(uint32_t p, float acc) {
  const f16x2 one = {(_Float16)1.0f, (_Float16)1.0f};
  return __builtin_amdgcn_fdot2(__builtin_bit_cast(f16x2, p), one, acc, false);
}

// Second half of Eq. 5: the two softmaxes over the d/2 features (in-lane, plus one exchange with
// lane^32).  pk[] receives the lane's d/2 values of phi as fp16 pairs: first LOC values
// softmax(+u) for features g*LOC .. g*LOC+LOC-1, then LOC values softmax(-u) for the same
// features.  valid == false zeroes the token (tail masking happens after phi: phi(0) is the
// uniform vector, not zero).
// CENTRE: the values are phi - 2/D (phi minus its mean over the features), so that the fp16 rounding
// acts on the deviation from the uniform map; the caller adds (2/D) x the column sums back.
template <int D, bool CENTRE = false>
__device__ __forceinline__ void softmax_pair(const f32x16 (&u)[Cfg<D>::UM], bool valid, uint32_t (&pk)[Cfg<D>::NPK]) {
  using C = Cfg<D>;
  float mx = u[0][0], mn = u[0][0];
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx = fmaxf(mx, u[mb][r]); mn = fminf(mn, u[mb][r]); }
  float lo, hi;
  pair32(mx, lo, hi); mx = fmaxf(lo, hi);
  pair32(mn, lo, hi); mn = fminf(lo, hi);
  // one softmax half at a time keeps only LOC exponentials live
#pragma unroll
  for (int half = 0; half < 2; ++half) {
    const float sl = half ? -kLog2e : kLog2e;
    const float c0 = half ? mn * kLog2e : -mx * kLog2e;
    float e[C::LOC];
    float s = 0.f;
#pragma unroll
    for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float a = __builtin_amdgcn_exp2f(fmaf(u[mb][r], sl, c0));
        e[16 * mb + r] = a;
        s += a;
      }
    pair32(s, lo, hi); s = lo + hi;
    const float inv = valid ? __builtin_amdgcn_rcpf(s) : 0.f;
    if constexpr (CENTRE) {
      const float mc = valid ? -2.0f / D : 0.f;
#pragma unroll
      for (int j = 0; j < C::LOC / 2; ++j)
        pk[half * (C::LOC / 2) + j] = pack_f16x2(fmaf(e[2 * j], inv, mc), fmaf(e[2 * j + 1], inv, mc));
    } else {
#pragma unroll
    for (int j = 0; j < C::LOC / 2; ++j) pk[half * (C::LOC / 2) + j] = pack_f16x2(e[2 * j] * inv, e[2 * j + 1] * inv);
    }
  }
}

// Eq. 5 with the normalised values kept in fp32 as well (the backward needs them for the softmax
// Jacobian): pp[j], pm[j] = softmax(+u), softmax(-u) of feature g*LOC + j; pk as in softmax_pair.
template <int D>
__device__ __forceinline__ void softmax_full(const f32x16 (&u)[Cfg<D>::UM], float (&pp)[Cfg<D>::LOC],
                                             float (&pm)[Cfg<D>::LOC], uint32_t (&pk)[Cfg<D>::NPK]) {
  using C = Cfg<D>;
  float mx = u[0][0], mn = u[0][0];
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx = fmaxf(mx, u[mb][r]); mn = fminf(mn, u[mb][r]); }
  float lo, hi;
  pair32(mx, lo, hi); mx = fmaxf(lo, hi);
  pair32(mn, lo, hi); mn = fminf(lo, hi);
  float sp = 0.f, sm = 0.f;
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float a = __builtin_amdgcn_exp2f(fmaf(u[mb][r], kLog2e, -mx * kLog2e));
      const float b = __builtin_amdgcn_exp2f(fmaf(u[mb][r], -kLog2e, mn * kLog2e));
      pp[16 * mb + r] = a; pm[16 * mb + r] = b;
      sp += a; sm += b;
    }
  pair32(sp, lo, hi); sp = lo + hi;
  pair32(sm, lo, hi); sm = lo + hi;
  const float ip = __builtin_amdgcn_rcpf(sp), im = __builtin_amdgcn_rcpf(sm);
#pragma unroll
  for (int j = 0; j < C::LOC; ++j) { pp[j] *= ip; pm[j] *= im; }
#pragma unroll
  for (int j = 0; j < C::LOC / 2; ++j) {
    pk[j] = pack_f16x2(pp[2 * j], pp[2 * j + 1]);
    pk[C::LOC / 2 + j] = pack_f16x2(pm[2 * j], pm[2 * j + 1]);
  }
}

// Eq. 5 up to a per-token positive factor, for the query side only: the output of Eq. 3 is a ratio
// that is linear in phi(q_i) above and below, so phi(q_i) may be scaled by any positive number.
// Scaling by the softmax(+u) denominator s+ leaves exp(u - max u) as the first half and
// (s+/s-) exp(min u - u) as the second: one multiply per token-half saved, values stay in (0, 64].
template <int D>
__device__ __forceinline__ void softmax_pair_ratio(const f32x16 (&u)[Cfg<D>::UM], uint32_t (&pk)[Cfg<D>::NPK]) {
  using C = Cfg<D>;
  float mx = u[0][0], mn = u[0][0];
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx = fmaxf(mx, u[mb][r]); mn = fminf(mn, u[mb][r]); }
  float lo, hi;
  pair32(mx, lo, hi); mx = fmaxf(lo, hi);
  pair32(mn, lo, hi); mn = fminf(lo, hi);
  float sp = 0.f;
  {
    const float c0 = -mx * kLog2e;
    float e[C::LOC];
#pragma unroll
    for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float a = __builtin_amdgcn_exp2f(fmaf(u[mb][r], kLog2e, c0));
        e[16 * mb + r] = a;
        sp += a;
      }
#pragma unroll
    for (int j = 0; j < C::LOC / 2; ++j) pk[j] = pack_f16x2(e[2 * j], e[2 * j + 1]);
    pair32(sp, lo, hi); sp = lo + hi;
  }
  {
    const float c0 = mn * kLog2e;
    float e[C::LOC];
    float sm = 0.f;
#pragma unroll
    for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float a = __builtin_amdgcn_exp2f(fmaf(u[mb][r], -kLog2e, c0));
        e[16 * mb + r] = a;
        sm += a;
      }
    pair32(sm, lo, hi); sm = lo + hi;
    const float ratio = sp * __builtin_amdgcn_rcpf(sm);
#pragma unroll
    for (int j = 0; j < C::LOC / 2; ++j) pk[C::LOC / 2 + j] = pack_f16x2(e[2 * j] * ratio, e[2 * j + 1] * ratio);
  }
}

// Power of two that brings the largest magnitude of a (b,h) state [D+1][D] (S rows, then z) into
// [2^13, 2^14): fp16 operand images of the state are scaled by it.  Every consumer forms a ratio
// or divides the scale out again.  red: >= NTHREADS/64 floats of LDS.  Contains __syncthreads().
template <int D, int NTHREADS>
__device__ __forceinline__ float head_scale(const float* __restrict__ S, float* red, int tid) {
  constexpr int N = (D + 1) * D;
  float amax = 0.f;
  for (int i0 = tid; i0 < N; i0 += 8 * NTHREADS) {
    float t[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { const int i = i0 + j * NTHREADS; t[j] = i < N ? fabsf(S[i]) : 0.f; }
#pragma unroll
    for (int j = 0; j < 8; ++j) amax = fmaxf(amax, t[j]);
  }
  for (int m = 32; m >= 1; m >>= 1) amax = fmaxf(amax, __shfl_xor(amax, m, 64));
  if (tid % 64 == 0) red[tid / 64] = amax;
  __syncthreads();
  amax = red[0];
#pragma unroll
  for (int i = 1; i < NTHREADS / 64; ++i) amax = fmaxf(amax, red[i]);
  __syncthreads();                       // red may be reused by the caller
  return (amax >= 0x1p-100f && amax < 3.0e38f) ? ldexpf(1.0f, 13 - ilogbf(amax)) : 1.0f;   // the scale itself stays finite
}

// fp32 state [D+1][D] of one (b,h) -> LDS image of the fp16 A operands of Y^T = S^T phi^T
// (contraction over the features of phi): entry (ks, mb, lane=(m,g)) holds
// scale * S[feature(ks,g,e)][channel(mb,m)], e = 0..7; the extra row block mb = MB holds
// scale * z[feature] in rows 0 and 4 (one per lane group) and zeros elsewhere.
// COLS: the same registers read as B operands of Y = phi S (lane (c,g) holds column c), with the
// channels dealt out by ApplyLayout::channel_cols; the extra block then holds scale * z[feature] in
// every column, so each lane of the product receives phi . z of its own token rows.
// KIND = kPhiRelu: the features are the d channels in their plain order, 16ks + 8g + e.
template <int D, bool COLS = false, int KIND = kPhiHedgehog>
__device__ __forceinline__ uint4 state_image_entry(const float* __restrict__ S, float scale, int idx) {
  using L = ApplyLayout<D>;
  const int lane = idx % 64, mb = (idx / 64) % L::MBZ, ks = idx / (64 * L::MBZ);
  const int m = lane % 32, g = lane / 32;
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int f = KIND == kPhiRelu ? 16 * ks + 8 * g + e : L::feature(ks, g, e);
    if (mb < L::MB) x[e] = scale * S[f * D + (COLS ? L::channel_cols(mb, m) : L::channel(mb, m))];
    else x[e] = (COLS || m == 0 || m == 4) ? scale * S[D * D + f] : 0.f;
  }
  uint4 r;
  r.x = pack_f16x2(x[0], x[1]); r.y = pack_f16x2(x[2], x[3]);
  r.z = pack_f16x2(x[4], x[5]); r.w = pack_f16x2(x[6], x[7]);
  return r;
}
template <int D, int NTHREADS, bool COLS = false, int KIND = kPhiHedgehog>
__device__ __forceinline__ void build_state_image(const float* __restrict__ S, uint4* sSA, float scale, int tid) {
  using L = ApplyLayout<D>;
  for (int idx = tid; idx < L::KS * L::MBZ * 64; idx += NTHREADS) sSA[idx] = state_image_entry<D, COLS, KIND>(S, scale, idx);
}

// Index maps of G^T = S Y^T (contraction over the d channels; rows = features of phi), used by the
// backward kernels.  The B operand is a token's half row: lane (t, g) feeds channels
// g*D/2 + 8*ks + e in k-step ks.  The accumulator rows are laid out like phi itself: lane (t, g),
// row block mb, register r holds the softmax(+u) feature g*LOC + 16*mb + r for mb < GM/2 and
// the softmax(-u) feature HALF + g*LOC + 16*(mb - GM/2) + r otherwise.
template <int D>
struct GradLayout {
  static constexpr int HALF = D / 2;
  static constexpr int LOC = D / 4;
  static constexpr int KS = D / 16;       // k-steps over the channels
  static constexpr int GM = D / 32;       // row blocks over the D features
  static constexpr int IMG = KS * GM * 64;
  __device__ static constexpr int channel(int ks, int g, int e) { return g * (D / 2) + 8 * ks + e; }
  __device__ static constexpr int feature(int mb, int m) {
    const int gg = (m / 4) % 2, r = 4 * (m / 8) + (m % 4);
    return (mb < GM / 2 ? 0 : HALF) + gg * LOC + 16 * (mb % (GM / 2)) + r;
  }
};

// One A-operand entry (ks, mb, lane) of the image of G^T = S Y^T: scale * S[feature][channel .. +7].
template <int D>
__device__ __forceinline__ uint4 grad_image_entry(const float* __restrict__ S, float scale, int idx) {
  using G = GradLayout<D>;
  const int lane = idx % 64, mb = (idx / 64) % G::GM, ks = idx / (64 * G::GM);
  const int m = lane % 32, g = lane / 32;
  const float* row = S + G::feature(mb, m) * D + G::channel(ks, g, 0);
  uint4 r;
  r.x = pack_f16x2(scale * row[0], scale * row[1]); r.y = pack_f16x2(scale * row[2], scale * row[3]);
  r.z = pack_f16x2(scale * row[4], scale * row[5]); r.w = pack_f16x2(scale * row[6], scale * row[7]);
  return r;
}

// One fp16 tile of the state that serves both products of the query-side backward, o = phi S (contraction over
// the features) and g = dO S^T (contraction over the channels).  Row rho = 16ks + 8g + e holds the feature
// that lane group g feeds as element e of k-step ks of phi (ApplyLayout::feature), column position
// p = 32mb + i holds the channel behind accumulator row i of row block mb (ApplyLayout::channel): a
// transposing read of rows 16ks .. 16ks+15, columns 32mb .. 32mb+31 is then the A operand (ks, mb) of o, and
// the 8 channels g*D/2 + 8ks' .. +7 that a lane group feeds to g in k-step ks' sit in one row as two runs of
// four positions, 16*ks' + 4g .. +3 and 8 further on: two 8-byte reads.  The 16-byte chunks of a row are
// XOR-swizzled with swz<D>(rho), like every tile that is read with transposing reads.
// idx = rho * (D/8) + (chunk as stored).
template <int D>
__device__ __forceinline__ uint4 state_tile_entry(const float* __restrict__ S, float scale, int idx) {
  using L = ApplyLayout<D>;
  const int rho = idx / (D / 8), c = (idx % (D / 8)) ^ swz<D>(rho);
  const int f = L::feature(rho / 16, (rho / 8) % 2, rho % 8);
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int pos = 8 * c + e;
    x[e] = scale * S[f * D + L::channel(pos / 32, pos % 32)];
  }
  uint4 r;
  r.x = pack_f16x2(x[0], x[1]); r.y = pack_f16x2(x[2], x[3]);
  r.z = pack_f16x2(x[4], x[5]); r.w = pack_f16x2(x[6], x[7]);
  return r;
}
// The z block of the image built by state_image_entry alone: entry (ks, lane).
template <int D>
__device__ __forceinline__ uint4 state_z_entry(const float* __restrict__ S, float scale, int idx) {
  using L = ApplyLayout<D>;
  return state_image_entry<D>(S, scale, ((idx / 64) * L::MBZ + L::MB) * 64 + idx % 64);
}
// Byte offset, inside the tile, of the row that holds feature GradLayout::feature(0, m) for this lane
// (m = lane % 32), plus the lane group's 8 bytes inside a chunk; row block mb of g is 32*mb rows further on.
template <int D>
__device__ __forceinline__ int state_tile_grad_row(int lane) {
  const int m = lane % 32, gg = (m / 4) % 2, r = 4 * (m / 8) + (m % 4);
  return (16 * (r / 8) + 8 * gg + (r % 8)) * (D * 2) + 8 * (lane / 32);
}

// W~ [D][D/2] bf16 (one head) -> LDS image (fp16, exact) of the B operands of dX = dU W~^T
// (contraction over the d/2 pre-softmax features, tokens on the accumulator rows): entry
// (ks, mb, lane=(c,g)) holds W~[channel_cols(mb,c)][g*LOC + 8ks + e], e = 0..7; ks < LOC/8, mb < D/32.
template <int D>
__device__ __forceinline__ uint4 w_image_t_entry(const uint16_t* __restrict__ w, int idx) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  const int lane = idx % 64, mb = (idx / 64) % L::MB, ks = idx / (64 * L::MB);
  const int m = lane % 32, g = lane / 32;
  const uint16_t* row = w + L::channel_cols(mb, m) * C::HALF + g * C::LOC + 8 * ks;
  float x[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) x[e] = __builtin_bit_cast(float, (uint32_t)row[e] << 16);
  uint4 r;
  r.x = pack_f16x2(x[0], x[1]); r.y = pack_f16x2(x[2], x[3]);
  r.z = pack_f16x2(x[4], x[5]); r.w = pack_f16x2(x[6], x[7]);
  return r;
}
template <int D, int NTHREADS>
__device__ __forceinline__ void build_w_image_t(const uint16_t* __restrict__ w, uint4* sWB, int tid) {
  constexpr int N = (Cfg<D>::LOC / 8) * ApplyLayout<D>::MB * 64;
  for (int idx = tid; idx < N; idx += NTHREADS) sWB[idx] = w_image_t_entry<D>(w, idx);
}

template <int D>
__device__ __forceinline__ int swz_out(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }

// Transposing LDS read: from a [row][column] fp16 tile, lane l of a wavefront receives
// tile[row0 + 8*(l/32) + 0..7][col0 + l%32] -- an MFMA A or B operand whose contraction index
// is the tile row.  Two ds_read_b64_tr_b16: within each group of 16 lanes, lane s supplies the
// address of row s/4, columns 4*(s%4)..+3, and receives column s of the four rows.
// tr_offset() is the lane's byte offset for row0 = 0 and the first (j = 0) or second (j = 1)
// group of four rows; row0 = 16*ks adds 16*ks*RS bytes (the swizzle repeats every 16 rows).
template <int D>
__device__ __forceinline__ int tr_offset(int col0, int lane, int j) {
  constexpr int RS = D * 2;
  const int r = 8 * (lane / 32) + ((lane % 16) / 4) + 4 * j;
  const int col = col0 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);    // element column, multiple of 4
  return r * RS + (((col / 8) ^ swz<D>(r)) * 16) + (col % 8) * 2;
}

// Byte offset of this lane's address for a transposing read of an operand of k-step 0 in the
// token order of a turned operand (the 16 tokens behind a lane's accumulator registers):
// j = 0: tile rows 4g .. 4g+3, j = 1: rows 8+4g .. 8+4g+3 (g = lane/32); columns col0 + lane%32.
template <int D>
__device__ __forceinline__ int tr_offset_g4(int col0, int lane, int j) {
  constexpr int RS = D * 2;
  const int r = 4 * (lane / 32) + ((lane % 16) / 4) + 8 * j;
  const int col = col0 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);
  return r * RS + (((col / 8) ^ swz<D>(r)) * 16) + (col % 8) * 2;
}

__device__ __forceinline__ f16x8 read_tr(const char* tile, int off0, int off1) {
  struct { s16x4 lo, hi; } v;
  v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + off0));
  v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(tile + off1));
  return __builtin_bit_cast(f16x8, v);
}

// power of two p with p * m in [1, 2) for 2^-100 <= m < 3e38; 1 for smaller m (zero included) and
// for non-finite m.  The lower limit keeps p itself finite: for m below 2^-127 (fp32 subnormals, which
// a saturated softmax leaves in du) the exact normaliser is not representable, and such values are
// zero against anything they are added to, so they may flush in the fp16 operand.
__device__ __forceinline__ float pow2_normaliser(float m) {
  return (m >= 0x1p-100f && m < 3.0e38f) ? ldexpf(1.0f, -ilogbf(m)) : 1.0f;
}

// Running power-of-two scale of a workgroup's sums over tokens (fp16 MFMA operands, fp32
// accumulators).  A tile whose largest operand magnitude is m wants the scale gamma_for(m), which
// puts m into [16, 32).  The workgroup keeps the smallest scale any of its tiles has asked for and,
// when a tile lowers it, multiplies its accumulators by the exact ratio (gamma_step), so a tile far
// larger than every earlier one cannot overflow fp16, and tiles that are all zero (kGammaUnset) leave
// the choice to the first tile that is not.
constexpr float kGammaUnset = 0x1p60f;
__device__ __forceinline__ float gamma_for(float m) {
  return m >= 0x1p-56f && m < 3.0e38f ? 16.f * pow2_normaliser(m) : kGammaUnset;
}
// Returns the factor (a power of two <= 1) the accumulators must be multiplied by; updates gamma.
__device__ __forceinline__ float gamma_step(float& gamma, float wanted) {
  const float next = fminf(gamma, wanted);
  const float ratio = next * __builtin_amdgcn_rcpf(gamma);      // exact: both are powers of two
  gamma = next;
  return ratio;
}

__device__ __forceinline__ void unpack_bf16x8(uint4 v, float* f) {
  f[0] = __builtin_bit_cast(float, v.x << 16); f[1] = __builtin_bit_cast(float, v.x & 0xffff0000u);
  f[2] = __builtin_bit_cast(float, v.y << 16); f[3] = __builtin_bit_cast(float, v.y & 0xffff0000u);
  f[4] = __builtin_bit_cast(float, v.z << 16); f[5] = __builtin_bit_cast(float, v.z & 0xffff0000u);
  f[6] = __builtin_bit_cast(float, v.w << 16); f[7] = __builtin_bit_cast(float, v.w & 0xffff0000u);
}

// max(x, 0) on a packed pair of bf16 (-0 becomes +0).
// As 16-bit integers the negative bf16 values are exactly the negative numbers, so one packed
// signed maximum with 0 does it.
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t u) {
  typedef short s16x2 __attribute__((ext_vector_type(2)));
  const s16x2 z = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2, u), z));
}
// Eight bf16 of a row -> fp16 of max(x, 0): an MFMA operand piece of the ReLU map.
__device__ __forceinline__ uint4 relu_f16x8(uint4 x) {
  uint4 r;
  r.x = bf16x2_to_f16x2(relu_bf16x2(x.x)); r.y = bf16x2_to_f16x2(relu_bf16x2(x.y));
  r.z = bf16x2_to_f16x2(relu_bf16x2(x.z)); r.w = bf16x2_to_f16x2(relu_bf16x2(x.w));
  return r;
}

// Copy n16 16-byte entries from global memory into LDS (all threads of the workgroup).
template <int NTHREADS>
__device__ __forceinline__ void copy_image(const uint4* __restrict__ src, uint4* dst, int n16, int tid) {
  for (int i = tid; i < n16; i += NTHREADS) dst[i] = src[i];
}

// Maximum of x over the wavefront, given x already equal in lanes l and l^32: DPP steps inside each
// row of 16 lanes, then the two rows of the low half are combined through scalar registers.
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}
__device__ __forceinline__ float wave_max_paired(float x) {
  x = fmaxf(x, dpp_move<0xB1>(x));      // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp_move<0x4E>(x));      // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp_move<0x124>(x));     // row_ror 4
  x = fmaxf(x, dpp_move<0x128>(x));     // row_ror 8
  const float a = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 0));
  const float b = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 16));
  return fmaxf(a, b);
}

// Where the stores of token rows past the end of a head go (8 bytes per lane; the contents mean nothing).
static __device__ __attribute__((aligned(256))) unsigned char g_store_sink[64 * 8];

// Accumulators with tokens on the rows (lane (c,g), register r: token t0 + 8*(r/4) + 4g + r%4,
// channels MB*c .. MB*c + MB-1 in acc[0..MB-1]) -> mul * acc as bf16 rows of base.  Every store
// instruction writes two whole rows of d channels.
template <int D>
__device__ __forceinline__ void store_token_rows(uint16_t* base, size_t sn, int t0, int n, int lane,
                                                 const f32x16 (&acc)[D / 32], float mul, const float (&add)[D / 32]) {
  constexpr int MB = D / 32;
  static_assert(MB == 2 || MB == 4, "head width 64 or 128");
  const int c = lane % 32, g = lane / 32;
  char* ub = reinterpret_cast<char*>(base + (size_t)t0 * sn);
  const uint32_t lo = ((uint32_t)(4 * g) * (uint32_t)sn + (uint32_t)(MB * c)) * 2u;
  // No branch around any of the stores: rows past n go to a sink instead (a select).  Behind branches the
  // compiler cannot count the stores in flight, and a later wait for a load that was requested before them
  // (the next block's rows) turns into a wait for the stores as well.
  const bool full = t0 + 32 <= n;
  char* sink = reinterpret_cast<char*>(g_store_sink) + lane * 8;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int row = 8 * (r / 4) + (r % 4);
    const bool there = full || t0 + row + 4 * g < n;
    char* dst = there ? ub + (size_t)row * sn * 2 + lo : sink;
    if constexpr (MB == 4) {
      uint2 v;
      v.x = pack_bf16x2(fmaf(acc[0][r], mul, add[0]), fmaf(acc[1][r], mul, add[1]));
      v.y = pack_bf16x2(fmaf(acc[2][r], mul, add[2]), fmaf(acc[3][r], mul, add[3]));
      *reinterpret_cast<uint2*>(dst) = v;
    } else {
      *reinterpret_cast<uint32_t*>(dst) = pack_bf16x2(fmaf(acc[0][r], mul, add[0]), fmaf(acc[1][r], mul, add[1]));
    }
  }
}

template <int D>
__device__ __forceinline__ void store_token_rows(uint16_t* base, size_t sn, int t0, int n, int lane,
                                                 const f32x16 (&acc)[D / 32], float mul) {
  float zero[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; ++i) zero[i] = 0.f;
  store_token_rows<D>(base, sn, t0, n, lane, acc, mul, zero);
}

// 32x32x16 MFMA on operands carried as f16x8 registers whose bits are fp16 or (BF16) bf16.
template <bool BF16>
__device__ __forceinline__ f32x16 mfma16(f16x8 a, f16x8 b, f32x16 c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

// One 128-token tile of a split-n sum over tokens: s[i][j] += A_i^T B_j and zacc += A_z^T w, with A
// and B fp16 tiles [kTile][D] in LDS (swizzled 16-byte chunks) read by transposing reads, the
// operands of k-step ks+1 requested before the MFMAs of k-step ks.  wop(ks) returns the B operand
// of the z sum for that k-step (per-token weights, the same in every column); z_hi picks which of
// the wavefront's A blocks feeds it, do_z whether this wavefront owns a z block at all.
// BF16: the tiles and wop's operands hold bf16 instead of fp16 (same bits per element, bf16 MFMA).
// SUMS: also accumulate csum[j] += the sum over the tile's tokens of the B operand's column of this lane
// (a lane holds 8 tokens of one channel per k-step) and *wsum += the sum of wop's operand (fp16 tiles only).
template <int D, bool BF16 = false, bool SUMS = false, typename WOp>
__device__ __forceinline__ void contract_tile(const char* sA, const char* sB, const int (&offA)[D / 64][2],
                                              const int (&offB)[D / 64][2], f32x16 (&s)[D / 64][D / 64],
                                              f32x16& zacc, bool z_hi, bool do_z, WOp wop,
                                              float* csum = nullptr, float* wsum = nullptr) {
  constexpr int RS = D * 2, WMN = D / 64, KSN = kTile / 16;
  f16x8 a[KSN][WMN], b[KSN][WMN], wv[KSN];
  auto request = [&](int kn) {
#pragma unroll
    for (int i = 0; i < WMN; ++i) a[kn][i] = read_tr(sA + kn * 16 * RS, offA[i][0], offA[i][1]);
#pragma unroll
    for (int j = 0; j < WMN; ++j) b[kn][j] = read_tr(sB + kn * 16 * RS, offB[j][0], offB[j][1]);
    wv[kn] = wop(kn);
  };
  request(0);
#pragma unroll
  for (int ks = 0; ks < KSN; ++ks) {
    if (ks + 1 < KSN) request(ks + 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < WMN; ++j) s[i][j] = mfma16<BF16>(a[ks][i], b[ks][j], s[i][j]);
    if (WMN == 2) {
      // a select, not a branch: branches inside the loop make the compiler's waits conservative
      const f16x8 az = z_hi ? a[ks][WMN - 1] : a[ks][0];
      zacc = mfma16<BF16>(az, wv[ks], zacc);
    } else if (do_z) {
      zacc = mfma16<BF16>(a[ks][0], wv[ks], zacc);
    }
    if constexpr (SUMS) {
#pragma unroll
      for (int j = 0; j < WMN; ++j) {
        const uint4 q = __builtin_bit_cast(uint4, b[ks][j]);
        csum[j] = add_pair_f16(q.x, csum[j]); csum[j] = add_pair_f16(q.y, csum[j]);
        csum[j] = add_pair_f16(q.z, csum[j]); csum[j] = add_pair_f16(q.w, csum[j]);
      }
      const uint4 q = __builtin_bit_cast(uint4, wv[ks]);
      float t = *wsum;
      t = add_pair_f16(q.x, t); t = add_pair_f16(q.y, t); t = add_pair_f16(q.z, t); t = add_pair_f16(q.w, t);
      *wsum = t;
    }
    __builtin_amdgcn_sched_barrier(0);
  }
}

}  // namespace linattn
