// bf16-I/O forward path on gfx950 MFMA (fp32 accumulation), tokens along the N dimension.
//
// Precision: the projections u = x W~ multiply the stored bf16 values exactly (bf16 MFMA).
// phi, and the state it is contracted with, are carried as fp16 (11-bit significand): phi lies
// in [0,1] and a few entries near 1 (sharp softmaxes of large-magnitude tokens) dominate sums
// that otherwise cancel, so 8-bit significands miss the 1e-2 accuracy contract by 2-4x while
// fp16 operands leave the bf16 rounding of the output as the largest error.  V is widened
// bf16 -> fp16 on its way into LDS (exact for 2^-14 <= |v| < 65520).
//
// state_partials_ws_kernel   : phi(K) (Eq. 5) fused with the split-n partial state
//                              S_p = sum_j phi(k_j)^T v_j, z_p = sum_j phi(k_j)  (Eq. 3)
// apply_bf16_kernel          : phi(Q), out = phi(Q) S / (phi(Q) . z), bf16 store (Eq. 3)
//
// Both start from U^T = W~^T X^T with X rows loaded straight into the MFMA B operand
// (16 bytes per lane), so a lane owns one token and d/4 of its d/2 pre-softmax features; the
// softmax reductions are in-lane plus one exchange with lane^32.
#include "kernels.h"
#include "mfma_common.h"

namespace linattn {
namespace {

// ------------------------------------------------------------------------------------------
// Query pass.  A wavefront owns 32-token blocks b = p*NW + w, stepping by (gridDim.x * NW), so
// the workgroups of a head sweep its tokens together.  Per block: load Q rows straight into the
// B operand of the projection (a lane owns a token), phi; phi then is the A operand of
// out = phi S, which puts the tokens on the accumulator rows and the channels on the lanes: a lane
// holds MB adjacent channels of 16 tokens and every store instruction writes two whole rows.  One
// more column block of the S image carries z in every column, so the same lanes get phi . z.
template <int MB> struct RowPiece;
template <> struct RowPiece<4> { typedef uint2 type; };
template <> struct RowPiece<2> { typedef uint32_t type; };
__device__ __forceinline__ uint32_t piece_word(const uint2& p, int i) { return i ? p.y : p.x; }
__device__ __forceinline__ uint32_t piece_word(const uint32_t& p, int) { return p; }
__device__ __forceinline__ void set_piece_word(uint2& p, int i, uint32_t v) { if (i) p.y = v; else p.x = v; }
__device__ __forceinline__ void set_piece_word(uint32_t& p, int, uint32_t v) { p = v; }
__device__ __forceinline__ void st_nt(uint2* p, uint2 v) {
  typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
  __builtin_nontemporal_store(__builtin_bit_cast(u32x2, v), reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void st_nt(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }

constexpr int NT3 = 768;         // 12 wavefronts, one workgroup per compute unit

// BLEND: mixed attention (Sec. 4.1, Eq. 6): out = r' s + (1 - r') o with the softmax-branch output
// s read in the same pieces as out is stored, and r' = clip(*rptr, 0, 1).
// KIND = kPhiRelu: phi(q) = max(q, 0) straight from the loaded rows (no projection, no W~), features
// in channel order, kReluEps in the denominator.
template <int D, bool BLEND, int KIND>
__global__ __launch_bounds__(NT3) void apply_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ wq,
                                                         const float* __restrict__ state, uint16_t* __restrict__ out,
                                                         const uint16_t* __restrict__ blend, const float* __restrict__ rptr,
                                                         int H, int n, Rows rw) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  constexpr int NW = NT3 / 64;
  constexpr int SA_IMG = L::KS * L::MBZ * 64;
  constexpr int HB = L::MB / 2;             // channel column blocks per accumulation pass (two passes)
  using Piece = typename RowPiece<L::MB>::type;   // a lane's MB adjacent bf16 channels of one token
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  uint4* sSA = sWA + C::W_IMG;
  char* sStage = reinterpret_cast<char*>(sSA + SA_IMG); // staging area of the prologue

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32;
  const int bh = blockIdx.y, h = bh % H;
  const uint16_t* qb = q + head_base(rw, bh, H);
  uint16_t* ob = out + head_base(rw, bh, H);
  const uint16_t* bb = BLEND ? blend + head_base(rw, bh, H) : nullptr;
  const float rb = BLEND ? fminf(fmaxf(*rptr, 0.f), 1.f) : 0.f;

  const int nblk = (n + 31) / 32;
  const int stride = gridDim.x * NW;
  const int c = lane % 32;
  const uint32_t lane_off = ((uint32_t)(4 * g) * (uint32_t)rw.sn + (uint32_t)(L::MB * c)) * 2u;   // bytes

  uint4 x[C::UK];
  auto load_block = [&](int b) {
    const int t = b * 32 + (lane % 32);
    const int tc = t < n ? t : (n - 1);
    const uint4* row = reinterpret_cast<const uint4*>(qb + (size_t)tc * rw.sn);
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) x[ks] = row[2 * ks + g];
  };
  // the first block's rows are requested before the prologue, so that they arrive under it
  int b = blockIdx.x * NW + w;
  if (b < nblk) load_block(b);

  float scale;
  {
    // The state and W~ of this (b,h) are first copied into LDS with coalesced 16-byte loads,
    // then turned into the operand images from there: the scattered reads the images need would cost tens of microseconds from global memory.
    float* stS = reinterpret_cast<float*>(sStage);
    uint16_t* stW = reinterpret_cast<uint16_t*>(stS + (D + 1) * D);
    float* red = reinterpret_cast<float*>(stW + D * C::HALF);
    const uint4* gS = reinterpret_cast<const uint4*>(state + (size_t)bh * (D + 1) * D);
    const uint4* gW = reinterpret_cast<const uint4*>(wq + (size_t)h * D * C::HALF);
    for (int i = tid; i < (D + 1) * D / 4; i += NT3) reinterpret_cast<uint4*>(stS)[i] = gS[i];
    if constexpr (KIND == kPhiHedgehog)
      for (int i = tid; i < D * C::HALF / 8; i += NT3) reinterpret_cast<uint4*>(stW)[i] = gW[i];
    __syncthreads();
    scale = head_scale<D, NT3>(stS, red, tid);
    if constexpr (KIND == kPhiHedgehog) build_w_image<D, NT3>(stW, sWA, tid);
    build_state_image<D, NT3, true, KIND>(stS, sSA, scale, tid);
  }
  __syncthreads();
  const float den_eps = KIND == kPhiRelu ? scale * kReluEps : 0.f;    // the image carries scale * z

  for (; b < nblk; b += stride) {
    uint32_t pk[C::NPK];
    if constexpr (KIND == kPhiRelu) {
      static_assert(C::NPK == 4 * C::UK, "one 16-byte piece of phi per piece of the row");
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) {
        const uint4 f = relu_f16x8(x[ks]);
        pk[4 * ks] = f.x; pk[4 * ks + 1] = f.y; pk[4 * ks + 2] = f.z; pk[4 * ks + 3] = f.w;
      }
      if constexpr (!BLEND) load_block(b + stride < nblk ? b + stride : b);
    } else {
      f32x16 u[C::UM];
      project<D>(x, sWA, lane, u);
      // next block's rows fly during the rest of this one (BLEND: the pieces of s take their
      // registers, so each 16-byte piece of the next rows is requested in the second pass as the
      // k-step that frees a piece of phi has been issued)
      if constexpr (!BLEND) load_block(b + stride < nblk ? b + stride : b);
      softmax_pair_ratio<D>(u, pk);
    }
    // register r of an accumulator is token b*32 + 8*(r/4) + 4g + r%4; the lane's MB channels of it
    // are MB*c .. MB*c + MB-1, two bytes each
    const bool full = b * 32 + 32 <= n;
    Piece sv[BLEND ? 16 : 1];               // the same pieces of the softmax branch
    if constexpr (BLEND) {
      const char* sb = reinterpret_cast<const char*>(bb + (size_t)(b * 32) * rw.sn) + lane_off;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + (r % 4);
        const bool there = full || b * 32 + row + 4 * g < n;
        sv[r] = there ? *reinterpret_cast<const Piece*>(sb + (size_t)row * rw.sn * 2) : Piece{};
      }
    }

    const uint4* next_row = nullptr;
    if constexpr (BLEND) {
      const int bn = b + stride < nblk ? b + stride : b;
      const int t = bn * 32 + (lane % 32);
      next_row = reinterpret_cast<const uint4*>(qb + (size_t)(t < n ? t : n - 1) * rw.sn);
    }
    // out = phi S in two passes over the lane's channels; the first also carries the block whose
    // every column is z, so each lane gets the normalisers of its 16 tokens
    const uint4* ssa = sSA + lane + opaque_zero();
    float inv[16], keep[16];
    Piece word[16];
#pragma unroll
    for (int pass = 0; pass < 2; ++pass) {
      f32x16 o[HB], dn;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        dn[r] = 0.f;
#pragma unroll
        for (int i = 0; i < HB; ++i) o[i][r] = 0.f;
      }
#pragma unroll
      for (int ks = 0; ks < L::KS; ++ks) {
        uint4 aq; aq.x = pk[4 * ks]; aq.y = pk[4 * ks + 1]; aq.z = pk[4 * ks + 2]; aq.w = pk[4 * ks + 3];
        const f16x8 aop = as_f16x8(aq);
#pragma unroll
        for (int i = 0; i < HB; ++i)
          o[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop, as_f16x8(ssa[(ks * L::MBZ + pass * HB + i) * 64]), o[i], 0, 0, 0);
        if (pass == 0) dn = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop, as_f16x8(ssa[(ks * L::MBZ + L::MB) * 64]), dn, 0, 0, 0);
        if constexpr (BLEND) {
          static_assert(C::UK == L::KS, "one piece of x per k-step");
          if (pass == 1) x[ks] = next_row[2 * ks + g];
        }
      }
      if (pass == 0) {
#pragma unroll
        for (int r = 0; r < 16; ++r) inv[r] = __builtin_amdgcn_rcpf(KIND == kPhiRelu ? dn[r] + den_eps : dn[r]);
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float y[HB];
#pragma unroll
        for (int i = 0; i < HB; ++i) {
          y[i] = o[i][r] * inv[r];
          if constexpr (BLEND) {
            const int ch = pass * HB + i;                         // which of the lane's MB channels
            const uint32_t sw = piece_word(sv[r], ch / 2);
            const float sf = (ch % 2) ? __builtin_bit_cast(float, sw & 0xffff0000u) : __builtin_bit_cast(float, sw << 16);
            y[i] = fmaf(rb, sf - y[i], y[i]);
          }
        }
        if constexpr (HB == 2) {
          set_piece_word(word[r], pass, pack_bf16x2(y[0], y[1]));
        } else {
          if (pass == 0) keep[r] = y[0];
          else set_piece_word(word[r], 0, pack_bf16x2(keep[r], y[0]));
        }
      }
    }
    {
      // Every store instruction writes two whole rows.  The stores are non-temporal: with ordinary
      // stores the tail of out stays dirty in the last-level cache and is written back under
      // whatever kernel runs next (measured: the next call's state pass loses 30 us, this pass
      // gains 20 us)
      // No branch around any of them: rows past n go to a sink instead (a select), see store_token_rows.
      char* ub = reinterpret_cast<char*>(ob + (size_t)(b * 32) * rw.sn) + lane_off;
      char* sink = reinterpret_cast<char*>(g_store_sink) + lane * 8;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + (r % 4);
        const bool there = full || b * 32 + row + 4 * g < n;
        st_nt(reinterpret_cast<Piece*>(there ? ub + (size_t)row * rw.sn * 2 : sink), word[r]);
      }
    }
  }
}

// State pass, wavefront-specialised: 8 wavefronts, one workgroup per compute unit.  Wavefronts
// 0-3 ("phi") turn the K rows of tile i+1 into phi and park it in one of two LDS buffers;
// wavefronts 4-7 ("acc") park the V tile there and meanwhile accumulate S = phi^T V, z = phi^T 1
// from the other buffer (tile i).  Each SIMD hosts one wavefront of each kind, so the softmax
// arithmetic of one tile overlaps the MFMA phase of the previous one; a single barrier per tile
// swaps the buffers.
constexpr int NT1 = 512;
constexpr int OPA = 1;           // k-steps of operand read-ahead in the accumulate phase (1, 2, 3 measured alike)

// Feature of phi (order of Eq. 5) behind feature slot n (0..31) of 32-row block fb of the turned
// phi (see state_partials_ws_kernel): fb = half*(D/64) + b, jj = n/16, g' = (n%16)/8, e = n%8
//   feature = half*D/2 + g'*D/4 + 8*(2b + jj) + e.
template <int D>
__device__ __forceinline__ int turned_feature(int fb, int n) {
  const int half = fb / (D / 64), b = fb % (D / 64);
  return half * (D / 2) + ((n % 16) / 8) * (D / 4) + 8 * (2 * b + n / 16) + (n % 8);
}

// One segment of a workgroup's tile range: tiles tile0 .. tile0+nt-1 of one (b,h), whose K and V
// rows start at kb, vb and whose W~_k is wkh; the partial state goes to dst.  Every thread of the
// workgroup calls it (it contains workgroup barriers).
// CENTRE (LINATTN_FLAG_CENTRED): the phi wavefronts produce phi - 2/D, so that the fp16 rounding acts on the
// deviation from the uniform map; the accumulate wavefronts sum the columns of V from the operands they read
// anyway (a lane of a transposed V operand holds 8 tokens of one channel) and the segment's partial state is
// completed in fp32: S += (2/D) 1 (sum v)^T, z += (2/D) x the number of tokens.
template <int D, bool CENTRE>
__device__ __forceinline__ void state_segment(const uint16_t* __restrict__ kb, const uint16_t* __restrict__ vb,
                                              const uint16_t* __restrict__ wkh, float* __restrict__ dst,
                                              int tile0, int nt, int n, Rows rw) {
  using C = Cfg<D>;
  constexpr int RS = D * 2;
  constexpr int WMN = D / 64;
  constexpr int VPT = (kTile * C::CH) / 256;     // 16-byte chunks of the V tile per acc thread
  constexpr int BUF = 2 * kTile * RS;            // one buffer: turned-phi operand image, then V tile
  constexpr int FB = D / 32;                     // 32-row blocks of S over the features
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  char* sBuf = reinterpret_cast<char*>(sWA + C::W_IMG);
  float* zred = reinterpret_cast<float*>(sBuf + 2 * BUF);      // [4][D] z of the four phi wavefronts

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int role = w / 4, pw = w % 4;            // role 0: phi, role 1: acc
  const int g = lane / 32;

  build_w_image<D, NT1>(wkh, sWA, tid);
  __syncthreads();

  if (role == 0) {
    // ---- phi wavefronts ------------------------------------------------------------------
    const int prow = 32 * pw + (lane % 32);
    // selection operands: B[k = 8g+e][n] = 1 iff n == 16*jj + 8g + e
    f16x8 sel[2];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
      uint32_t q[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int e0 = 16 * jj + 8 * g + 2 * i;
        q[i] = ((lane % 32) == e0 ? 0x3C00u : 0u) | ((lane % 32) == e0 + 1 ? 0x3C000000u : 0u);
      }
      uint4 t; t.x = q[0]; t.y = q[1]; t.z = q[2]; t.w = q[3];
      sel[jj] = as_f16x8(t);
    }
    float zs[FB];
#pragma unroll
    for (int i = 0; i < FB; ++i) zs[i] = 0.f;
    auto load_k = [&](uint4 (&x)[C::UK], int tile) {
      const int t = tile * kTile + prow;
      const int tc = t < n ? t : (n - 1);
      const uint4* row = reinterpret_cast<const uint4*>(kb + (size_t)tc * rw.sn);
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) x[ks] = row[2 * ks + g];
    };
    // one tile: x holds its K rows and is refilled with the tile two steps ahead as soon as the
    // projection has consumed it
    auto phi_step = [&](uint4 (&x)[C::UK], int it) {
      if (it < nt) {
        const int tile = tile0 + it;
        const bool valid = (tile * kTile + prow) < n;
        f32x16 u[C::UM];
        project<D>(x, sWA, lane, u);
        if (it + 2 < nt) load_k(x, tile + 2);
        uint32_t pk[C::NPK];
        softmax_pair<D, CENTRE>(u, valid, pk);
        // turn phi from "token per lane" to "feature slot per lane" with an MFMA against the 0/1
        // selection operands: the accumulator is then (after an exact repack to fp16) the A operand
        // of S = phi^T V with the tokens of a 16-token k-step in the order {4g..4g+3, 8+4g..8+4g+3};
        // z is the in-lane sum.  The operands go to LDS ready-made: entry (pw, fb, kb, lane).
        uint4* img = reinterpret_cast<uint4*>(sBuf + (it & 1) * BUF) + (pw * FB * 2) * 64 + lane;
#pragma unroll
        for (int fb = 0; fb < FB; ++fb) {
          const int half = fb / (D / 64), b = fb % (D / 64);
          f32x16 t;
#pragma unroll
          for (int r = 0; r < 16; ++r) t[r] = 0.f;
#pragma unroll
          for (int jj = 0; jj < 2; ++jj) {
            const int base = half * (C::LOC / 2) + 4 * (2 * b + jj);
            uint4 a; a.x = pk[base]; a.y = pk[base + 1]; a.z = pk[base + 2]; a.w = pk[base + 3];
            t = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(a), sel[jj], t, 0, 0, 0);
          }
          float zsum = 0.f;
#pragma unroll
          for (int r = 0; r < 16; ++r) zsum += t[r];
          zs[fb] += zsum;
#pragma unroll
          for (int kb = 0; kb < 2; ++kb) {
            uint4 a;
            a.x = pack_f16x2(t[8 * kb], t[8 * kb + 1]);     a.y = pack_f16x2(t[8 * kb + 2], t[8 * kb + 3]);
            a.z = pack_f16x2(t[8 * kb + 4], t[8 * kb + 5]); a.w = pack_f16x2(t[8 * kb + 6], t[8 * kb + 7]);
            img[(fb * 2 + kb) * 64] = a;
          }
        }
      }
      __syncthreads();
    };
    uint4 xa[C::UK], xc[C::UK];
    load_k(xa, tile0);
    if (nt > 1) load_k(xc, tile0 + 1);
    for (int it = 0; it <= nt; it += 2) {       // nt + 1 barriers in total, as in the acc branch
      phi_step(xa, it);
      if (it + 1 <= nt) phi_step(xc, it + 1);
    }
    // z of this wavefront's tokens: both lane groups of a slot
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {
      float lo, hi;
      pair32(zs[fb], lo, hi);
      if (g == 0) zred[pw * D + 32 * fb + lane] = lo + hi;
    }
    if constexpr (CENTRE) {
      __syncthreads();      // the two barriers of the accumulate branch's column-sum reduction
      __syncthreads();
    }
  } else {
    // ---- acc wavefronts ------------------------------------------------------------------
    const int mi = pw / 2, ni = pw % 2;
    const int atid = tid - 256;
    f32x16 s[WMN][WMN];
#pragma unroll
    for (int r = 0; r < 16; ++r)
#pragma unroll
      for (int i = 0; i < WMN; ++i)
#pragma unroll
        for (int j = 0; j < WMN; ++j) s[i][j][r] = 0.f;
    auto fblk = [&](int i) { return mi * WMN + ((WMN == 2) ? (i ^ ni) : i); };
    int offB[WMN][2];
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) offB[i][j] = tr_offset_g4<D>(32 * (ni * WMN + i), lane, j) + kTile * RS;
    auto load_v = [&](uint4 (&vr)[VPT], int tile) {
      const int t0 = tile * kTile;
#pragma unroll
      for (int i = 0; i < VPT; ++i) {
        const int idx = atid + 256 * i;
        const int r = idx / C::CH, c = idx % C::CH;
        const int tv = (t0 + r) < n ? (t0 + r) : (n - 1);
        vr[i] = ld_nt(reinterpret_cast<const uint4*>(vb + (size_t)tv * rw.sn) + c);
      }
    };
    float csum[WMN];                                 // CENTRE: column sums of V over the lane's tokens
#pragma unroll
    for (int j = 0; j < WMN; ++j) csum[j] = 0.f;
    // one step: park V tile `it` (held in vr, refilled with the tile two steps ahead), then
    // accumulate tile it-1 from the other buffer
    auto acc_step = [&](uint4 (&vr)[VPT], int it) {
      if (it < nt) {
        char* sV = sBuf + (it & 1) * BUF + kTile * RS;
#pragma unroll
        for (int i = 0; i < VPT; ++i) {
          const int idx = atid + 256 * i;
          const int rv = idx / C::CH, c = idx % C::CH;
          uint4 hv;
          hv.x = bf16x2_to_f16x2(vr[i].x); hv.y = bf16x2_to_f16x2(vr[i].y);
          hv.z = bf16x2_to_f16x2(vr[i].z); hv.w = bf16x2_to_f16x2(vr[i].w);
          *reinterpret_cast<uint4*>(sV + rv * RS + ((c ^ swz<D>(rv)) * 16)) = hv;
        }
        if (it + 2 < nt) load_v(vr, tile0 + it + 2);
      }
      if (it >= 1) {
        // operands are requested OPA k-steps before the MFMAs that use them.
        // k-step ks = tokens 16ks .. 16ks+15 = phi wavefront ks/2, half kb = ks%2 of its block.
        const char* buf = sBuf + ((it - 1) & 1) * BUF;
        const uint4* img = reinterpret_cast<const uint4*>(buf) + lane + opaque_zero();
        constexpr int KSN = kTile / 16;
        f16x8 a[KSN][WMN], b[KSN][WMN];
        auto request = [&](int kn) {
#pragma unroll
          for (int i = 0; i < WMN; ++i) a[kn][i] = as_f16x8(img[(((kn / 2) * FB + fblk(i)) * 2 + (kn % 2)) * 64]);
#pragma unroll
          for (int j = 0; j < WMN; ++j) b[kn][j] = read_tr(buf + kn * 16 * RS, offB[j][0], offB[j][1]);
        };
#pragma unroll
        for (int ks = 0; ks < OPA; ++ks) request(ks);
#pragma unroll
        for (int ks = 0; ks < KSN; ++ks) {
          if (ks + OPA < KSN) request(ks + OPA);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int i = 0; i < WMN; ++i)
#pragma unroll
            for (int j = 0; j < WMN; ++j)
              s[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[ks][i], b[ks][j], s[i][j], 0, 0, 0);
          if constexpr (CENTRE) {
#pragma unroll
            for (int j = 0; j < WMN; ++j) {
              const uint4 q = __builtin_bit_cast(uint4, b[ks][j]);
              csum[j] = add_pair_f16(q.x, csum[j]); csum[j] = add_pair_f16(q.y, csum[j]);
              csum[j] = add_pair_f16(q.z, csum[j]); csum[j] = add_pair_f16(q.w, csum[j]);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      __syncthreads();
    };
    uint4 va[VPT], vc[VPT];
    load_v(va, tile0);
    if (nt > 1) load_v(vc, tile0 + 1);
    for (int it = 0; it <= nt; it += 2) {
      acc_step(va, it);
      if (it + 1 <= nt) acc_step(vc, it + 1);
    }
    const int c = lane % 32;
    float corr[WMN];
#pragma unroll
    for (int j = 0; j < WMN; ++j) corr[j] = 0.f;
    if constexpr (CENTRE) {
      // column sums of v: the two lane groups of the wavefronts mi = 0 (mi = 1 holds the same sums), in a
      // fixed order; every step has ended with a barrier, so the tile buffers are free.  Rows past n
      // were parked as copies of row n - 1: their share is taken out again.
      float* svp = reinterpret_cast<float*>(sBuf);            // [D] sums, then [D] (2/D) x sums
#pragma unroll
      for (int j = 0; j < WMN; ++j) {
        float lo, hi;
        pair32(csum[j], lo, hi);
        if (mi == 0 && g == 0) svp[32 * (ni * WMN + j) + c] = lo + hi;
      }
      __syncthreads();
      float* svs = svp + D;
      if (atid < D) {
        const int t_hi = (tile0 + nt) * kTile;
        const int dup = t_hi > n ? t_hi - n : 0;
        float t = svp[atid];
        if (dup > 0) {
          const uint32_t last = bf16x2_to_f16x2((uint32_t)vb[(size_t)(n - 1) * rw.sn + atid]) & 0xffffu;
          t -= (float)dup * (float)__builtin_bit_cast(_Float16, (uint16_t)last);
        }
        svs[atid] = t * (2.0f / D);
      }
      __syncthreads();
#pragma unroll
      for (int j = 0; j < WMN; ++j) corr[j] = svs[32 * (ni * WMN + j) + c];
    }
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < WMN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int f = turned_feature<D>(fblk(i), 8 * (r / 4) + 4 * g + (r % 4));
          dst[f * D + 32 * (ni * WMN + j) + c] = CENTRE ? s[i][j][r] + corr[j] : s[i][j][r];
        }
  }
  // z: the four phi wavefronts, in a fixed order (CENTRE: plus 2/D per token of the segment)
  __syncthreads();
  if (tid < D) {
    float zv = (zred[tid] + zred[2 * D + tid]) + (zred[D + tid] + zred[3 * D + tid]);
    if constexpr (CENTRE) {
      const int t_lo = tile0 * kTile, t_hi = (tile0 + nt) * kTile < n ? (tile0 + nt) * kTile : n;
      zv += (2.0f / D) * (float)(t_hi - t_lo);
    }
    dst[D * D + turned_feature<D>(tid / 32, tid % 32)] = zv;
  }
  __syncthreads();                               // the next segment reuses every LDS region
}

// Grid: Split::G workgroups; workgroup g takes the tiles [lo(g), lo(g+1)) of the call's (b,h)-major
// tile sequence, one segment per head it touches (at most two).
template <int D, bool CENTRE>
__global__ __launch_bounds__(NT1) void state_partials_ws_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                                const uint16_t* __restrict__ wk, float* __restrict__ partials,
                                                                int H, int n, Split sp, Rows rw) {
  const int g = blockIdx.x;
  long long lo = split_lo(sp, g);
  const long long hi = split_lo(sp, g + 1);
  while (lo < hi) {
    const int bh = (int)(lo / sp.ntile);
    const long long head0 = (long long)bh * sp.ntile;
    const long long seg_hi = hi < head0 + sp.ntile ? hi : head0 + sp.ntile;
    const int slot = g - split_owner(sp, head0);
    state_segment<D, CENTRE>(k + head_base(rw, bh, H), v + head_base(rw, bh, H), wk + (size_t)(bh % H) * D * (D / 2),
                     partials + ((size_t)bh * sp.PS + slot) * (size_t)(D + 1) * D,
                     (int)(lo - head0), (int)(seg_hi - lo), n, rw);
    lo = seg_hi;
  }
}

template <int D>
constexpr size_t state_ws_smem() { return sizeof(uint4) * Cfg<D>::W_IMG + 4 * (size_t)kTile * D * 2 + 4 * D * sizeof(float); }

template <int D>
constexpr size_t apply_smem() {
  // the images, then the prologue's staging of the fp32 state, W~ and a few reduction slots
  return sizeof(uint4) * (Cfg<D>::W_IMG + ApplyLayout<D>::KS * ApplyLayout<D>::MBZ * 64)
       + (size_t)(D + 1) * D * sizeof(float) + (size_t)D * (D / 2) * 2 + 64 * sizeof(float);
}

}  // namespace

namespace {
template <int D, bool CENTRE>
hipError_t run_state_ws(const void* k, const void* v, const void* wk, float* partials, const Plan& p, hipStream_t s) {
  hipError_t e;
  if ((e = set_smem_once<state_partials_ws_kernel<D, CENTRE>>(state_ws_smem<D>())) != hipSuccess) return e;
  state_partials_ws_kernel<D, CENTRE><<<dim3(p.split.G), dim3(NT1), state_ws_smem<D>(), s>>>(
      (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)wk, partials, p.H, p.n, p.split, p.rows);
  return hipGetLastError();
}
}  // namespace

hipError_t launch_state_partials_bf16(const void* k, const void* v, const void* wk, float* partials,
                                      const Plan& p, hipStream_t s) {
  if (p.d == 128)
    return p.centred ? run_state_ws<128, true>(k, v, wk, partials, p, s) : run_state_ws<128, false>(k, v, wk, partials, p, s);
  return p.centred ? run_state_ws<64, true>(k, v, wk, partials, p, s) : run_state_ws<64, false>(k, v, wk, partials, p, s);
}

namespace {

template <int D, bool BLEND, int KIND>
hipError_t run_apply(const void* q, const void* wq, const float* state, void* out, const void* blend_in,
                     const float* blend_r, const Plan& p, hipStream_t s) {
  hipError_t e;
  if ((e = set_smem_once<apply_bf16_kernel<D, BLEND, KIND>>(apply_smem<D>())) != hipSuccess) return e;
  apply_bf16_kernel<D, BLEND, KIND><<<dim3(p.QP, p.BH), NT3, apply_smem<D>(), s>>>(
      (const uint16_t*)q, (const uint16_t*)wq, state, (uint16_t*)out, (const uint16_t*)blend_in, blend_r, p.H, p.n, p.rows);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_apply_bf16(const void* q, const void* wq, const float* state, void* out,
                             const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s) {
  if (p.kind == kPhiRelu)      // the dispatch has refused a blend with this map
    return p.d == 128 ? run_apply<128, false, kPhiRelu>(q, nullptr, state, out, nullptr, nullptr, p, s)
                      : run_apply<64, false, kPhiRelu>(q, nullptr, state, out, nullptr, nullptr, p, s);
  if (p.d == 128)
    return blend_in ? run_apply<128, true, kPhiHedgehog>(q, wq, state, out, blend_in, blend_r, p, s)
                    : run_apply<128, false, kPhiHedgehog>(q, wq, state, out, nullptr, nullptr, p, s);
  return blend_in ? run_apply<64, true, kPhiHedgehog>(q, wq, state, out, blend_in, blend_r, p, s)
                  : run_apply<64, false, kPhiHedgehog>(q, wq, state, out, nullptr, nullptr, p, s);
}

}  // namespace linattn
