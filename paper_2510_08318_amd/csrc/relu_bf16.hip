// ReLU feature map, bf16 I/O: phi(x) = max(x, 0) on the d channels of a head (the "ReLU" row of
// the paper's ablation of kernel functions), put into Eq. 3 with kReluEps in the denominator.
// This file holds the state pass and the backward; the query pass is apply_bf16_kernel<.., kPhiRelu>
// in fwd_bf16.hip.
//
// With no projection and no softmax the map costs a sign test, so every kernel here is the plain
// contraction of Eq. 3 (or of its chain rule) on MFMA with fp32 accumulation -- bf16 operands in
// the state pass (K and V as stored: exact products, no conversion), fp16 where a state or a
// gradient is an operand (the query pass and the backward):
//   relu_state_kernel  : S_p = sum_j phi(k_j)^T v_j, z_p = sum_j phi(k_j) over the tiles of a split
//   relu_prep_kernel   : MFMA operand images of a state (S or dS), built once per head
//   relu_bwd_q_kernel  : den, G = dO S^T, delta, dq; split-n partials of dS, dz
//   relu_bwd_k_kernel  : dv = phi(k) dS, dk = (v dS^T + dz) where k > 0
// Gradients (chain rule through Eq. 3, then the mask of max(x, 0), whose derivative at 0 is taken as 0):
//   den_i = phi(q_i).z + eps, o_i = phi(q_i) S / den_i, delta_i = dO_i . o_i
//   dphi(q_i) = (S dO_i - delta_i z) / den_i;  dS = sum_i phi(q_i)^T dO_i / den_i;  dz = -sum_i phi(q_i) delta_i / den_i
//   dphi(k_j) = dS v_j + dz;  dv_j = dS^T phi(k_j)
// Operands that are gradients are scaled by powers of two before the cast to fp16, as in bwd_bf16.hip.
#include "kernels.h"
#include "mfma_common.h"

namespace linattn {
namespace {

// ---- state pass -------------------------------------------------------------------------------
// 4 wavefronts.  One segment = the 128-token tiles tile0 .. tile0+nt-1 of one (b,h): K (through
// max(.,0)) and V are parked in LDS as they are, bf16 (no conversion: the kernel's time is its own
// instruction stream, not HBM), and contracted over the tokens with transposing reads on bf16 MFMA;
// wavefront (mi, ni) owns the feature rows 32*WMN*mi .. and the channel columns 32*WMN*ni .. of S.
// z = phi(K)^T 1 rides along as one more MFMA per k-step against an operand of ones.  Every thread
// of the workgroup calls it (it contains workgroup barriers).
template <int D>
__device__ __forceinline__ void relu_state_segment(const uint16_t* __restrict__ kb, const uint16_t* __restrict__ vb,
                                                   float* __restrict__ dst, int tile0, int nt, int n, Rows rw) {
  constexpr int RS = D * 2;
  constexpr int WMN = D / 64;
  constexpr int XPT = (kTile * (D / 8)) / NT;   // 16-byte chunks of a tile per thread
  extern __shared__ uint4 smem[];
  char* sK = reinterpret_cast<char*>(smem);      // [kTile][D] bf16, swizzled chunks
  char* sV = sK + kTile * RS;

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32;
  const int mi = w / 2, ni = w % 2;
  const int tile_end = tile0 + nt;

  f32x16 s[WMN][WMN], zacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zacc[r] = 0.f;
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < WMN; ++j) s[i][j][r] = 0.f;
  }
  const int zmb = (WMN == 2) ? (2 * mi + ni) : mi;      // the 32-feature block whose z this wavefront sums
  const bool do_z = (WMN == 2) || (ni == 0);
  int offA[WMN][2], offB[WMN][2];
#pragma unroll
  for (int i = 0; i < WMN; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      offA[i][j] = tr_offset<D>(32 * (mi * WMN + i), lane, j);
      offB[i][j] = tr_offset<D>(32 * (ni * WMN + i), lane, j);
    }
  uint4 ones;
  ones.x = ones.y = ones.z = ones.w = 0x3F803F80u;      // bf16 1.0
  const f16x8 one_op = as_f16x8(ones);

  // Loads are branch-free (rows past n read row n-1 and are zeroed on their way into LDS; after the
  // last tile of a segment that tile is requested once more and ignored): a load behind a branch
  // makes the compiler wait for every outstanding load at the join.
  // Tiles kept in flight per workgroup, and how often the loop body repeats them.  Measured at the
  // Wan-14B 720p shape: one tile 287 us, two 276 us, three 295 us, four 290 us.  The compiler waits
  // for every outstanding load at the top of the loop, so only an unrolled body overlaps them.
  constexpr int DEPTH = 2, UNROLL = 2;
  uint4 kr[DEPTH][XPT], vr[DEPTH][XPT];
  // Addresses: a wavefront-uniform tile pointer (scalar registers) plus a 32-bit byte offset per
  // thread and piece that is computed once (15 vector instructions per load otherwise, a quarter
  // of this kernel's instruction stream).  Rows past n are redirected to row n-1 with one minimum
  // per load.
  static_assert(NT % (D / 8) == 0, "a thread keeps its chunk column");
  uint32_t voff[XPT];
#pragma unroll
  for (int i = 0; i < XPT; ++i)
    voff[i] = (uint32_t)(((tid + NT * i) / (D / 8)) * rw.sn + (tid % (D / 8)) * 8) * 2u;
  int loff[XPT];                                   // LDS byte offsets of the thread's pieces
#pragma unroll
  for (int i = 0; i < XPT; ++i) {
    const int r = (tid + NT * i) / (D / 8), c = tid % (D / 8);
    loff[i] = r * RS + ((c ^ swz<D>(r)) * 16);
  }
  auto load_tile = [&](uint4 (&kx)[XPT], uint4 (&vx)[XPT], int tile) {
    tile = tile < tile_end ? tile : tile_end - 1;
    const int t0 = tile * kTile;
    const char* kt = reinterpret_cast<const char*>(kb + (size_t)t0 * rw.sn);
    const char* vt = reinterpret_cast<const char*>(vb + (size_t)t0 * rw.sn);
    const int last = n - 1 - t0;                  // last row of the tile that exists (>= kTile-1: all do)
    const uint32_t last_off = (uint32_t)(last * rw.sn + (tid % (D / 8)) * 8) * 2u;
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      const uint32_t off = voff[i] < last_off ? voff[i] : last_off;      // same column: offsets grow with the row
      kx[i] = ld_nt(reinterpret_cast<const uint4*>(kt + off));
      vx[i] = ld_nt(reinterpret_cast<const uint4*>(vt + off));
    }
  };
  auto consume = [&](uint4 (&kx)[XPT], uint4 (&vx)[XPT], int tile, bool real) {
    __syncthreads();                              // previous tile's operand reads are done
    // the tiles stay bf16 (the products of a bf16 MFMA are exact): K through the sign test, V as it
    // is.  Rows that do not exist hold copies of row n-1: zeroing their K is enough (phi = 0 adds
    // nothing to S or z); only a head's last tile and padding steps pay for that.
    const bool full = real && (tile + 1) * kTile <= n;      // uniform
#pragma unroll
    for (int i = 0; i < XPT; ++i) {
      uint4 hk;
      hk.x = relu_bf16x2(kx[i].x); hk.y = relu_bf16x2(kx[i].y); hk.z = relu_bf16x2(kx[i].z); hk.w = relu_bf16x2(kx[i].w);
      if (!full) {
        const int r = (tid + NT * i) / (D / 8);
        if (!(real && tile * kTile + r < n)) hk = make_uint4(0, 0, 0, 0);
      }
      *reinterpret_cast<uint4*>(sK + loff[i]) = hk;
      *reinterpret_cast<uint4*>(sV + loff[i]) = vx[i];
    }
    load_tile(kx, vx, tile + DEPTH);
    __syncthreads();
    contract_tile<D, true>(sK, sV, offA, offB, s, zacc, ni != 0, do_z, [&](int) { return one_op; });
  };
#pragma unroll
  for (int j = 0; j < DEPTH; ++j) load_tile(kr[j], vr[j], tile0 + j);
  for (int tile = tile0; tile < tile_end; tile += UNROLL * DEPTH) {
#pragma unroll
    for (int u = 0; u < UNROLL; ++u)
#pragma unroll
      for (int j = 0; j < DEPTH; ++j) {
        const int tl = tile + u * DEPTH + j;
        consume(kr[j], vr[j], tl, tl < tile_end);     // a padding step adds zeros
      }
  }
  const int c = lane % 32;
#pragma unroll
  for (int i = 0; i < WMN; ++i)
#pragma unroll
    for (int j = 0; j < WMN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int f = 32 * (mi * WMN + i) + 8 * (r / 4) + 4 * g + (r % 4);
        dst[f * D + 32 * (ni * WMN + j) + c] = s[i][j][r];
      }
  if (do_z && c == 0) {
#pragma unroll
    for (int r = 0; r < 16; ++r) dst[D * D + 32 * zmb + 8 * (r / 4) + 4 * g + (r % 4)] = zacc[r];
  }
  __syncthreads();                               // the next segment reuses the LDS tiles
}

// Grid: Split::G workgroups; workgroup g takes the tiles [lo(g), lo(g+1)) of the call's (b,h)-major
// tile sequence, one segment per head it touches (at most two), so every compute unit gets the same
// share whatever B*H is.  Partials: [BH][Split::PS][(d+1)*d], summed by the split reduction.
template <int D>
__global__ __launch_bounds__(NT) void relu_state_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                        float* __restrict__ partials, int H, int n, Split sp, Rows rw) {
  const int gi = blockIdx.x;
  long long lo = split_lo(sp, gi);
  const long long hi = split_lo(sp, gi + 1);
  while (lo < hi) {
    const int bh = (int)(lo / sp.ntile);
    const long long head0 = (long long)bh * sp.ntile;
    const long long seg_hi = hi < head0 + sp.ntile ? hi : head0 + sp.ntile;
    const int slot = gi - split_owner(sp, head0);
    relu_state_segment<D>(k + head_base(rw, bh, H), v + head_base(rw, bh, H),
                          partials + ((size_t)bh * sp.PS + slot) * (size_t)(D + 1) * D,
                          (int)(lo - head0), (int)(seg_hi - lo), n, rw);
    lo = seg_hi;
  }
}

// ---- operand images of a state, built once per head ------------------------------------------------
// For M = S or dS ([D+1][D] fp32, row D = z or dz), both scaled by one power of two per head:
//   cimg: B operands of Y = phi M (contraction over the features): state_image_entry<D, true, kPhiRelu>
//   timg: B operands of G = X M^T (contraction over the channels, columns = features):
//         entry (ks, mb, lane=(c,g)) holds M[channel_cols(mb,c)][16ks + 8g + e], e = 0..7
// grid (BH, 8): slice blockIdx.y of the entries.
constexpr int PT = 512;      // threads of the image builder (staging the state is latency-bound)
// The images are built with the head's mean value row taken out, as in the Eq. 5 path (exact in real
// arithmetic; values with a common offset then cost the gradients nothing):
//   pass over S (DS = false): S^c = S - z c^T with c = sum_f S[f] / sum_f z[f], the phi-weighted mean of v (any
//     row c would do: the query side then works with o - c and delta - dO . c, dq is unchanged up to
//     eps / den, and its dz comes out as dz + dS c); c is written to `mean_row`;
//   pass over dS (DS = true): dzc[f] = dz[f] - c . r(dS[f]) with r the fp16 rounding of the image, so that
//     v_j . r(dS[f]) + dzc[f] = (v_j - c) . r(dS[f]) + (dz + dS c)[f] holds exactly on the key side.
template <int D, bool DS>
__global__ __launch_bounds__(PT) void relu_prep_kernel(const float* __restrict__ state, uint4* __restrict__ cimg,
                                                        uint4* __restrict__ timg, float* __restrict__ scale_out,
                                                        float* __restrict__ mean_row, float* __restrict__ dzc) {
  using L = ApplyLayout<D>;
  constexpr int CIMG = L::KS * L::MBZ * 64, TIMG = L::KS * L::MB * 64;
  extern __shared__ uint4 prep_stage[];
  float* S = reinterpret_cast<float*>(prep_stage);                        // [(D+1)*D]
  __shared__ float red[PT / 64];
  const int bh = blockIdx.x, tid = threadIdx.x;
  {
    const uint4* gsrc = reinterpret_cast<const uint4*>(state + (size_t)bh * (D + 1) * D);
    for (int i = tid; i < (D + 1) * D / 4; i += PT) reinterpret_cast<uint4*>(S)[i] = gsrc[i];
  }
  __syncthreads();
  __shared__ float cM[D];
  if constexpr (!DS) {
    if (tid < D) {
      float sv = 0.f, zt = 0.f;
      for (int f = 0; f < D; ++f) { sv += S[f * D + tid]; zt += S[D * D + f]; }
      const float c = zt > 0.f ? sv / zt : 0.f;
      cM[tid] = c;
      if (blockIdx.y == 0) mean_row[(size_t)bh * D + tid] = c;
    }
    __syncthreads();
    for (int i = tid; i < D * D; i += PT) S[i] -= S[D * D + i / D] * cM[i % D];
    __syncthreads();
  } else {
    if (tid < D) cM[tid] = mean_row[(size_t)bh * D + tid];
    __syncthreads();
  }
  const float scale = head_scale<D, PT>(S, red, tid);      // every block of a head computes the same value
  if (blockIdx.y == 0 && tid == 0) scale_out[2 * bh] = scale;      // [BH][2]: S, dS
  if constexpr (DS) {
    if (blockIdx.y == 0 && tid < D) {
      const float inv = __builtin_amdgcn_rcpf(scale);       // exact: a power of two
      float dot = 0.f;
      for (int ch = 0; ch < D; ++ch) dot = fmaf((float)(_Float16)(scale * S[tid * D + ch]), cM[ch], dot);
      dzc[(size_t)bh * D + tid] = S[D * D + tid] - dot * inv;
    }
  }
  const int first = blockIdx.y * PT + tid, step = PT * gridDim.y;
  for (int idx = first; idx < CIMG; idx += step) cimg[(size_t)bh * CIMG + idx] = state_image_entry<D, true, kPhiRelu>(S, scale, idx);
  for (int idx = first; idx < TIMG; idx += step) {
    const int lane = idx % 64, mb = (idx / 64) % L::MB, ks = idx / (64 * L::MB);
    const int c = lane % 32, g = lane / 32;
    const float* row = S + L::channel_cols(mb, c) * D + 16 * ks + 8 * g;
    uint4 r;
    r.x = pack_f16x2(scale * row[0], scale * row[1]); r.y = pack_f16x2(scale * row[2], scale * row[3]);
    r.z = pack_f16x2(scale * row[4], scale * row[5]); r.w = pack_f16x2(scale * row[6], scale * row[7]);
    timg[(size_t)bh * TIMG + idx] = r;
  }
}

// Sum of x over the 32 lanes that share lane/32 (every one of them receives it): DPP inside each
// row of 16 lanes, then the two rows of a half are exchanged with one permlane16 swap.
__device__ __forceinline__ float half_wave_sum(float x) {
  x += dpp_move<0xB1>(x);      // quad_perm [1,0,3,2]
  x += dpp_move<0x4E>(x);      // quad_perm [2,3,0,1]
  x += dpp_move<0x124>(x);     // row_ror 4
  x += dpp_move<0x128>(x);     // row_ror 8
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);   // rows 1, 3 of the first <-> rows 0, 2 of the second
  return __builtin_bit_cast(float, (uint32_t)r[0]) + __builtin_bit_cast(float, (uint32_t)r[1]);
}

// One channel (0..3, or 0..1 for d = 64) of a lane's piece of a row, as float.
__device__ __forceinline__ float piece_elem(const uint2& p, int i) {
  const uint32_t wv = i < 2 ? p.x : p.y;
  return (i % 2) ? __builtin_bit_cast(float, wv & 0xffff0000u) : __builtin_bit_cast(float, wv << 16);
}
__device__ __forceinline__ float piece_elem(const uint32_t& p, int i) {
  return i ? __builtin_bit_cast(float, p & 0xffff0000u) : __builtin_bit_cast(float, p << 16);
}
template <int MB> struct RowPieceT;
template <> struct RowPieceT<4> { typedef uint2 type; };
template <> struct RowPieceT<2> { typedef uint32_t type; };

// Rows of x (bf16) in the layout of an accumulator with the tokens on its rows: piece r of lane (c,g)
// is token t0 + 8*(r/4) + 4g + r%4, channels MB*c .. MB*c + MB-1.  Rows past n read as row n-1.
template <int D, typename Piece>
__device__ __forceinline__ void load_row_pieces(const uint16_t* base, size_t sn, int t0, int n, int lane, Piece (&out)[16]) {
  constexpr int MB = D / 32;
  const int c = lane % 32, g = lane / 32;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    int t = t0 + 8 * (r / 4) + 4 * g + (r % 4);
    t = t < n ? t : n - 1;
    out[r] = *reinterpret_cast<const Piece*>(base + (size_t)t * sn + MB * c);
  }
}

// ---- query side of the backward -------------------------------------------------------------------
// grid (P, BH), 4 wavefronts; wavefront w of a tile owns its tokens 32w .. 32w+31.  Per block:
//   A operands straight from the loaded rows (a lane owns a token): phi(q) and ts * dO (ts: one power
//   of two per block);  dn = phi(q) . (scale z) on the accumulator rows (one MFMA column block of z),
//   ga = ts * scale * dO S^T with the tokens on the rows and the features on the lanes; q once more in
//   that layout for the mask and for delta = sum_f G_f phi_f / den (a sum over the 32 lanes); dq rows
//   are stored from the accumulators.  Then phi(q) and gamma * dO / den go to LDS as fp16 and the
//   four wavefronts contract them over the tile's tokens into dS (dz: one more MFMA per k-step).
template <int D>
__global__ __launch_bounds__(NT) void relu_bwd_q_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ dout,
                                                        const float* __restrict__ state, const uint4* __restrict__ cimg,
                                                        const uint4* __restrict__ timg, const float* __restrict__ scale_ptr,
                                                        uint16_t* __restrict__ dq, float* __restrict__ partials,
                                                        int H, int n, int P, Rows rw) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  using Piece = typename RowPieceT<L::MB>::type;
  constexpr int RS = D * 2;
  constexpr int WMN = D / 64;
  constexpr int CIMG = L::KS * L::MBZ * 64, TIMG = L::KS * L::MB * 64;
  extern __shared__ uint4 smem[];
  uint4* sZB = smem;                                       // [KS][64] the z column block of cimg
  uint4* sT = sZB + L::KS * 64;                            // [KS][MB][64] timg
  char* sPhi = reinterpret_cast<char*>(sT + TIMG);         // [kTile][D] fp16: phi(q)
  char* sDO = sPhi + kTile * RS;                           // [kTile][D] fp16: gamma * dO / den
  uint16_t* sW16 = reinterpret_cast<uint16_t*>(sDO + kTile * RS);   // [kTile] fp16: -gamma * delta / den
  float* sRow = reinterpret_cast<float*>(sW16 + kTile);    // [4 wavefronts][2][32] per-token scalars
  float* sRed = sRow + 4 * 64;                             // [8]

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32, c = lane % 32;
  const int mi = w / 2, ni = w % 2;
  const int bh = blockIdx.y, p = blockIdx.x;
  const uint16_t* qb = q + head_base(rw, bh, H);
  const uint16_t* dob = dout + head_base(rw, bh, H);
  uint16_t* dqb = dq + head_base(rw, bh, H);
  const float* sb = state + (size_t)bh * (D + 1) * D;
  const int ntile = (n + kTile - 1) / kTile;

  for (int i = tid; i < L::KS * 64; i += NT)
    sZB[i] = cimg[(size_t)bh * CIMG + ((i / 64) * L::MBZ + L::MB) * 64 + (i % 64)];
  copy_image<NT>(timg + (size_t)bh * TIMG, sT, TIMG, tid);
  const float scale = scale_ptr[2 * bh];
  float zl[L::MB];                                         // z of the lane's features
#pragma unroll
  for (int mb = 0; mb < L::MB; ++mb) zl[mb] = sb[D * D + L::channel_cols(mb, c)];
  __syncthreads();

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
  int offA[WMN][2], offB[WMN][2];
#pragma unroll
  for (int i = 0; i < WMN; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      offA[i][j] = tr_offset<D>(32 * (mi * WMN + i), lane, j);
      offB[i][j] = tr_offset<D>(32 * (ni * WMN + i), lane, j);
    }
  const int prow = 32 * w + (lane % 32);
  const int psw = swz<D>(prow);
  float* myRow = sRow + w * 64;
  float gamma = kGammaUnset;

  // The rows of a tile are requested inside the tile before it, each set as soon as its registers are free (the
  // accumulator-layout q rows before the dq stores, the operand-layout q and dO rows behind the parking of phi
  // and dO): with one wavefront per SIMD nothing else hides the latency of a load at the top of a tile.  Never
  // behind a branch: after the last tile its rows are simply read again.
  uint4 xq[C::UK], dor[C::UK];
  Piece qrow[16];
  auto load_operand_rows = [&](int tile) {
    const int t = tile * kTile + prow;
    const int tc = t < n ? t : (n - 1);
    const uint4* row = reinterpret_cast<const uint4*>(qb + (size_t)tc * rw.sn);
    const uint4* drow = reinterpret_cast<const uint4*>(dob + (size_t)tc * rw.sn);
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) { xq[ks] = row[2 * ks + g]; dor[ks] = drow[2 * ks + g]; }
  };
  load_operand_rows(p < ntile ? p : 0);
  load_row_pieces<D>(qb, rw.sn, (p < ntile ? p : 0) * kTile + 32 * w, n, lane, qrow);
  for (int tile = p; tile < ntile; tile += P) {
    const int t0 = tile * kTile + 32 * w;
    const int t = tile * kTile + prow;
    const bool valid = t < n;
    const int next = tile + P < ntile ? tile + P : tile;

    // block scale of dO
    float dmax = 0.f;
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) {
      float f[8];
      unpack_bf16x8(dor[ks], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) dmax = fmaxf(dmax, fabsf(f[e]));
    }
    if (!valid) dmax = 0.f;
    float lo, hi;
    pair32(dmax, lo, hi); dmax = fmaxf(lo, hi);              // the token's largest |dO|
    const float ts = pow2_normaliser(wave_max_paired(dmax));

    // den and G on the accumulator rows
    f32x16 ga[L::MB], dn;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dn[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) ga[mb][r] = 0.f;
    }
    const uint4* szb = sZB + lane + opaque_zero();
    const uint4* st = sT + lane + opaque_zero();
    pipelined_operands<L::KS, 3>(
        [&](int ks) { return szb[ks * 64]; },
        [&](int ks, uint4 b) {
          dn = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(relu_f16x8(xq[ks])), as_f16x8(b), dn, 0, 0, 0);
        });
    pipelined_operands<L::KS * L::MB, 3>(
        [&](int i) { return st[i * 64]; },
        [&](int i, uint4 b) {
          const int ks = i / L::MB, mb = i % L::MB;
          float f[8];
          unpack_bf16x8(dor[ks], f);
          uint4 aq;
          aq.x = pack_f16x2(f[0] * ts, f[1] * ts); aq.y = pack_f16x2(f[2] * ts, f[3] * ts);
          aq.z = pack_f16x2(f[4] * ts, f[5] * ts); aq.w = pack_f16x2(f[6] * ts, f[7] * ts);
          ga[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_f16x8(aq), as_f16x8(b), ga[mb], 0, 0, 0);
        });
    // per row: a = 1 / (scale * den), delta = (sum_f G_f phi_f) / den; dq = (G - delta z) / den where q > 0
    const float its = __builtin_amdgcn_rcpf(ts);                // exact: a power of two
    const float den_eps = scale * kReluEps;
    float arow[16], drow_[16];
    f32x16 dqa[L::MB];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float part = 0.f;
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) part = fmaf(ga[mb][r], fmaxf(piece_elem(qrow[r], mb), 0.f), part);
      const float sum = half_wave_sum(part);                    // ts * scale * dO . (phi S)
      const float a = __builtin_amdgcn_rcpf(dn[r] + den_eps);   // 1 / (scale * den)
      const float delta = sum * a * its;
      arow[r] = a;
      drow_[r] = delta;
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) {
        const float val = ga[mb][r] * (a * its) - delta * (scale * a) * zl[mb];
        dqa[mb][r] = piece_elem(qrow[r], mb) > 0.f ? val : 0.f;
      }
    }
    load_row_pieces<D>(qb, rw.sn, next * kTile + 32 * w, n, lane, qrow);
    store_token_rows<D>(dqb, rw.sn, t0, n, lane, dqa, 1.f);

    // the per-token scalars back onto the lanes that own the tokens
    if (c == 0) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = 8 * (r / 4) + 4 * g + (r % 4);
        myRow[row] = arow[r];
        myRow[32 + row] = drow_[r];
      }
    }
    __builtin_amdgcn_wave_barrier();
    const float a_t = myRow[lane % 32];
    const float delta_t = myRow[32 + (lane % 32)];
    __builtin_amdgcn_wave_barrier();
    const float inv_den = scale * a_t;                          // 1 / den
    // a query with phi(q) = 0 adds nothing to dS and dz, but its 1 / den = 1 / eps would set the
    // common scale gamma and push every other token's operand into the fp16 subnormals
    bool live;
    {
      uint32_t any = 0;
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) {
        const uint4 f = relu_f16x8(xq[ks]);
        any |= f.x | f.y | f.z | f.w;
      }
      auto r2 = __builtin_amdgcn_permlane32_swap(any, any, false, false);
      live = valid && (((uint32_t)r2[0] | (uint32_t)r2[1]) != 0);
    }

    // operands of the sums over tokens
    {
      float m = live ? fmaxf(dmax, fabsf(delta_t)) * inv_den : 0.f;
      m = wave_max_paired(m);
      if (lane == 0) sRed[w] = m;
    }
    __syncthreads();                             // previous tile's operand reads are done
    {
      // running power-of-two scale of the two sums over tokens (see gamma_for)
      const float m = fmaxf(fmaxf(sRed[0], sRed[1]), fmaxf(sRed[2], sRed[3]));
      const float ratio = gamma_step(gamma, gamma_for(m));
      if (ratio != 1.f) {
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
      char* drowp = sDO + prow * RS;
      const float sc = live ? inv_den * gamma : 0.f;
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) {
        uint4 a = relu_f16x8(xq[ks]);
        if (!live) a = make_uint4(0, 0, 0, 0);
        *reinterpret_cast<uint4*>(rowp + (((2 * ks + g) ^ psw) * 16)) = a;
        float f[8];
        unpack_bf16x8(dor[ks], f);
        uint4 b;
        b.x = pack_f16x2(f[0] * sc, f[1] * sc); b.y = pack_f16x2(f[2] * sc, f[3] * sc);
        b.z = pack_f16x2(f[4] * sc, f[5] * sc); b.w = pack_f16x2(f[6] * sc, f[7] * sc);
        *reinterpret_cast<uint4*>(drowp + (((2 * ks + g) ^ psw) * 16)) = b;
      }
      if (g == 0) sW16[prow] = (uint16_t)(pack_f16x2(live ? -delta_t * sc : 0.f, 0.f) & 0xffffu);
    }
    load_operand_rows(next);
    __syncthreads();
    contract_tile<D>(sPhi, sDO, offA, offB, s, zacc, ni != 0, do_z,
                     [&](int ks) { return as_f16x8(*reinterpret_cast<const uint4*>(sW16 + 16 * ks + 8 * g)); });
  }

  const float ig = __builtin_amdgcn_rcpf(gamma);    // exact: gamma is a power of two
  float* dst = partials + ((size_t)bh * P + p) * (size_t)(D + 1) * D;
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
}

// ---- key side of the backward ---------------------------------------------------------------------
// grid (KP, BH), 8 wavefronts, each on its own 32-token blocks.  Both products have the tokens on
// the accumulator rows: dv = phi(k) dS (B operands: cimg of dS) and g = v dS^T + dz (timg of dS);
// dk = g where k > 0, with k read once more in the accumulator layout for the mask.
constexpr int NTK = 512;
template <int D>
__global__ __launch_bounds__(NTK) void relu_bwd_k_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                         const float* __restrict__ dstate, const uint4* __restrict__ cimg,
                                                         const uint4* __restrict__ timg, const float* __restrict__ scale_ptr,
                                                         uint16_t* __restrict__ dk, uint16_t* __restrict__ dv,
                                                         const float* __restrict__ dzc, int H, int n, Rows rw) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  using Piece = typename RowPieceT<L::MB>::type;
  constexpr int NW = NTK / 64;
  constexpr int CIMG = L::KS * L::MBZ * 64, TIMG = L::KS * L::MB * 64;
  extern __shared__ uint4 smem[];
  uint4* sC = smem;
  uint4* sT = sC + CIMG;

  const int tid = threadIdx.x, lane = tid % 64;
  const int w = __builtin_amdgcn_readfirstlane(tid / 64);
  const int g = lane / 32, c = lane % 32;
  const int bh = blockIdx.y;
  const uint16_t* kb = k + head_base(rw, bh, H);
  const uint16_t* vb = v + head_base(rw, bh, H);
  uint16_t* dkb = dk + head_base(rw, bh, H);
  uint16_t* dvb = dv + head_base(rw, bh, H);
  copy_image<NTK>(cimg + (size_t)bh * CIMG, sC, CIMG, tid);
  copy_image<NTK>(timg + (size_t)bh * TIMG, sT, TIMG, tid);
  const float inv_scale = __builtin_amdgcn_rcpf(scale_ptr[2 * bh]);    // exact: power of two
  float dzl[L::MB];
#pragma unroll
  for (int mb = 0; mb < L::MB; ++mb) dzl[mb] = dzc[(size_t)bh * D + L::channel_cols(mb, c)];   // dz matched to the image (relu_prep_kernel)
  __syncthreads();

  const int nblk = (n + 31) / 32;
  const int stride = gridDim.x * NW;
  for (int b = blockIdx.x * NW + w; b < nblk; b += stride) {
    const int t = b * 32 + (lane % 32);
    const int tc = t < n ? t : (n - 1);
    uint4 xk[C::UK], xv[C::UK];
    {
      const uint4* row = reinterpret_cast<const uint4*>(kb + (size_t)tc * rw.sn);
      const uint4* vrow = reinterpret_cast<const uint4*>(vb + (size_t)tc * rw.sn);
#pragma unroll
      for (int ks = 0; ks < C::UK; ++ks) { xk[ks] = row[2 * ks + g]; xv[ks] = vrow[2 * ks + g]; }
    }
    Piece krow[16];
    load_row_pieces<D>(kb, rw.sn, b * 32, n, lane, krow);
    {
      f32x16 va[L::MB];
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) va[mb][r] = 0.f;
      const uint4* sc = sC + lane + opaque_zero();
#pragma unroll
      for (int ks = 0; ks < L::KS; ++ks) {
        const f16x8 aop = as_f16x8(relu_f16x8(xk[ks]));
#pragma unroll
        for (int mb = 0; mb < L::MB; ++mb)
          va[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop, as_f16x8(sc[(ks * L::MBZ + mb) * 64]), va[mb], 0, 0, 0);
      }
      store_token_rows<D>(dvb, rw.sn, b * 32, n, lane, va, inv_scale);
    }
    {
      f32x16 ga[L::MB];
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) ga[mb][r] = 0.f;
      const uint4* st = sT + lane + opaque_zero();
#pragma unroll
      for (int ks = 0; ks < L::KS; ++ks) {
        uint4 aq;
        aq.x = bf16x2_to_f16x2(xv[ks].x); aq.y = bf16x2_to_f16x2(xv[ks].y);
        aq.z = bf16x2_to_f16x2(xv[ks].z); aq.w = bf16x2_to_f16x2(xv[ks].w);
        const f16x8 aop = as_f16x8(aq);
#pragma unroll
        for (int mb = 0; mb < L::MB; ++mb)
          ga[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(aop, as_f16x8(st[(ks * L::MB + mb) * 64]), ga[mb], 0, 0, 0);
      }
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          ga[mb][r] = piece_elem(krow[r], mb) > 0.f ? fmaf(ga[mb][r], inv_scale, dzl[mb]) : 0.f;
      store_token_rows<D>(dkb, rw.sn, b * 32, n, lane, ga, 1.f);
    }
  }
}

template <int D>
constexpr size_t state_smem() { return 2 * (size_t)kTile * D * 2; }
template <int D>
constexpr size_t prep_smem() { return (size_t)(D + 1) * D * sizeof(float); }
template <int D>
constexpr size_t q_smem() {
  return sizeof(uint4) * (ApplyLayout<D>::KS * 64 + ApplyLayout<D>::KS * ApplyLayout<D>::MB * 64)
       + 2 * (size_t)kTile * D * 2 + kTile * 2 + (4 * 64 + 8) * sizeof(float);
}
template <int D>
constexpr size_t k_smem() {
  return sizeof(uint4) * (ApplyLayout<D>::KS * ApplyLayout<D>::MBZ * 64 + ApplyLayout<D>::KS * ApplyLayout<D>::MB * 64);
}

template <int D>
hipError_t run_state(const void* k, const void* v, float* partials, const Plan& p, hipStream_t s) {
  hipError_t e;
  if ((e = set_smem_once<relu_state_kernel<D>>(state_smem<D>())) != hipSuccess) return e;
  relu_state_kernel<D><<<dim3(p.split.G), NT, state_smem<D>(), s>>>((const uint16_t*)k, (const uint16_t*)v, partials,
                                                                   p.H, p.n, p.split, p.rows);
  return hipGetLastError();
}

template <int D>
hipError_t run_bwd(const BwdArgs& a, const Plan& p, hipStream_t s) {
  hipError_t e;
  if ((e = set_smem_once<relu_prep_kernel<D, false>>(prep_smem<D>())) != hipSuccess) return e;
  if ((e = set_smem_once<relu_prep_kernel<D, true>>(prep_smem<D>())) != hipSuccess) return e;
  relu_prep_kernel<D, false><<<dim3(p.BH, 8), PT, prep_smem<D>(), s>>>(a.state, (uint4*)a.simg, (uint4*)a.gimg, a.scales, a.vbar, nullptr);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = set_smem_once<relu_bwd_q_kernel<D>>(q_smem<D>())) != hipSuccess) return e;
  relu_bwd_q_kernel<D><<<dim3(p.P, p.BH), NT, q_smem<D>(), s>>>(
      (const uint16_t*)a.q, (const uint16_t*)a.dout, a.state, (const uint4*)a.simg, (const uint4*)a.gimg, a.scales,
      (uint16_t*)a.dq, a.partials, p.H, p.n, p.P, p.rows);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = launch_state_reduce(a.partials, a.dstate, p, s)) != hipSuccess) return e;
  relu_prep_kernel<D, true><<<dim3(p.BH, 8), PT, prep_smem<D>(), s>>>(a.dstate, (uint4*)a.dsimg, (uint4*)a.dgimg, a.scales + 1, a.vbar, a.dzc);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = set_smem_once<relu_bwd_k_kernel<D>>(k_smem<D>())) != hipSuccess) return e;
  relu_bwd_k_kernel<D><<<dim3(p.KP, p.BH), NTK, k_smem<D>(), s>>>(
      (const uint16_t*)a.k, (const uint16_t*)a.v, a.dstate, (const uint4*)a.dsimg, (const uint4*)a.dgimg, a.scales + 1,
      (uint16_t*)a.dk, (uint16_t*)a.dv, a.dzc, p.H, p.n, p.rows);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_relu_state_bf16(const void* k, const void* v, float* partials, const Plan& p, hipStream_t s) {
  return p.d == 128 ? run_state<128>(k, v, partials, p, s) : run_state<64>(k, v, partials, p, s);
}

hipError_t launch_relu_bwd_bf16(const BwdArgs& a, const Plan& p, hipStream_t s) {
  return p.d == 128 ? run_bwd<128>(a, p, s) : run_bwd<64>(a, p, s);
}

}  // namespace linattn
