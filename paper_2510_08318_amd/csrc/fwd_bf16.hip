// bf16-I/O forward path on gfx950 MFMA (fp32 accumulation), tokens along the N dimension.
//
// Precision: the projections u = x W~ multiply the stored bf16 values exactly (bf16 MFMA).
// phi, and the state it is contracted with, are carried as fp16 (11-bit significand): phi lies
// in [0,1] and a few entries near 1 (sharp softmaxes of large-magnitude tokens) dominate sums
// that otherwise cancel, so 8-bit significands miss the 1e-2 accuracy contract by 2-4x while
// fp16 operands leave the bf16 rounding of the output as the largest error.  V is widened
// bf16 -> fp16 on its way into LDS (exact for 2^-14 <= |v| < 65520).
//
// state_partials_bf16_kernel : phi(K) (Eq. 5) fused with the split-n partial state
//                              S_p = sum_j phi(k_j)^T v_j, z_p = sum_j phi(k_j)  (Eq. 3)
// apply_bf16_kernel          : phi(Q), out = phi(Q) S / (phi(Q) . z), bf16 store (Eq. 3)
//
// Both start from U^T = W~^T X^T with X rows loaded straight into the MFMA B operand
// (16 bytes per lane), so a lane owns one token and d/4 of its d/2 pre-softmax features; the
// softmax reductions are in-lane plus one exchange with lane^32.
#include "kernels.h"
#include "mfma_layout.h"

namespace linattn {
namespace {

constexpr float kLog2e = 1.4426950408889634f;
constexpr int NT = 256;          // 4 wavefronts

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
template <int D>
__device__ __forceinline__ int swz(int r) {
  if (D == 128) return ((r & 3) << 2) | ((r >> 2) & 3);
  return (((r & 3) << 1) ^ (r >> 2)) & 7;
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
__device__ __forceinline__ void build_w_image(const uint16_t* __restrict__ w, uint4* sWA, int tid) {
  using C = Cfg<D>;
  for (int idx = tid; idx < C::W_IMG; idx += NT) {
    const int lane = idx % 64, mb = (idx / 64) % C::UM, ks = idx / (64 * C::UM);
    const int m = lane % 32, g = lane / 32;
    const int uf = owned_row<C::HALF>(mb, m);
    uint32_t x[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) x[e] = w[(16 * ks + 8 * g + e) * C::HALF + uf];
    uint4 r;
    r.x = x[0] | (x[1] << 16); r.y = x[2] | (x[3] << 16);
    r.z = x[4] | (x[5] << 16); r.w = x[6] | (x[7] << 16);
    sWA[idx] = r;
  }
}

// Eq. 5 for the 32 tokens of one wavefront.  xb[ks] is this lane's B operand (8 channels of its
// token per k-step).  On return pk[] holds the lane's d/2 values of phi as fp16 pairs:
// first LOC values softmax(+u) for features g*LOC .. g*LOC+LOC-1, then LOC values softmax(-u)
// for the same features.  valid == false zeroes the token (tail masking happens after phi:
// phi(0) is the uniform vector, not zero).
template <int D>
__device__ __forceinline__ void phi_block(const uint4 (&xb)[Cfg<D>::UK], const uint4* sWA, int lane, bool valid,
                                          uint32_t (&pk)[Cfg<D>::NPK]) {
  using C = Cfg<D>;
  f32x16 u[C::UM];
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) u[mb][r] = 0.f;
#pragma unroll
  for (int ks = 0; ks < C::UK; ++ks) {
    const bf16x8 b = as_bf16x8(xb[ks]);
#pragma unroll
    for (int mb = 0; mb < C::UM; ++mb) {
      const bf16x8 a = as_bf16x8(sWA[(ks * C::UM + mb) * 64 + lane]);
      u[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, u[mb], 0, 0, 0);
    }
  }
  float mx = u[0][0], mn = u[0][0];
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) { mx = fmaxf(mx, u[mb][r]); mn = fminf(mn, u[mb][r]); }
  float lo, hi;
  pair32(mx, lo, hi); mx = fmaxf(lo, hi);
  pair32(mn, lo, hi); mn = fminf(lo, hi);
  const float cpos = -mx * kLog2e, cneg = mn * kLog2e;
  float ep[C::LOC], em[C::LOC];
  float sp = 0.f, sm = 0.f;
#pragma unroll
  for (int mb = 0; mb < C::UM; ++mb)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float x = u[mb][r];
      const float a = __builtin_amdgcn_exp2f(fmaf(x, kLog2e, cpos));
      const float b = __builtin_amdgcn_exp2f(fmaf(x, -kLog2e, cneg));
      ep[16 * mb + r] = a; em[16 * mb + r] = b;
      sp += a; sm += b;
    }
  pair32(sp, lo, hi); sp = lo + hi;
  pair32(sm, lo, hi); sm = lo + hi;
  const float ip = valid ? __builtin_amdgcn_rcpf(sp) : 0.f;
  const float im = valid ? __builtin_amdgcn_rcpf(sm) : 0.f;
#pragma unroll
  for (int j = 0; j < C::LOC / 2; ++j) {
    pk[j] = pack_f16x2(ep[2 * j] * ip, ep[2 * j + 1] * ip);
    pk[C::LOC / 2 + j] = pack_f16x2(em[2 * j] * im, em[2 * j + 1] * im);
  }
}

// ------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(NT, 2) void apply_bf16_kernel(const uint16_t* __restrict__ q, const uint16_t* __restrict__ wq,
                                                           const uint4* __restrict__ sa, uint16_t* __restrict__ out,
                                                           int H, int n, int chunk) {
  using C = Cfg<D>;
  using L = ApplyLayout<D>;
  constexpr int SA_IMG = L::KS * L::MBZ * 64;
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  uint4* sSA = sWA + C::W_IMG;

  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int g = lane / 32;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk;
  const int t_end = min(n, t_begin + chunk);
  const uint16_t* qb = q + (size_t)bh * n * D;
  uint16_t* ob = out + (size_t)bh * n * D;

  build_w_image<D>(wq + (size_t)h * D * C::HALF, sWA, tid);
  const uint4* sab = sa + (size_t)bh * SA_IMG;
  for (int i = tid; i < SA_IMG; i += NT) sSA[i] = sab[i];
  __syncthreads();

  for (int t0 = t_begin + 32 * w; t0 < t_end; t0 += 32 * (NT / 64)) {
    const int t = t0 + (lane % 32);
    const bool valid = t < t_end;
    const int tc = valid ? t : (t_end - 1);
    const uint4* row = reinterpret_cast<const uint4*>(qb + (size_t)tc * D);
    uint4 xb[C::UK];
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) xb[ks] = row[2 * ks + g];
    uint32_t pk[C::NPK];
    phi_block<D>(xb, sWA, lane, valid, pk);

    f32x16 o[L::MB], dn;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      dn[r] = 0.f;
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) o[mb][r] = 0.f;
    }
#pragma unroll
    for (int ks = 0; ks < L::KS; ++ks) {
      uint4 bq; bq.x = pk[4 * ks]; bq.y = pk[4 * ks + 1]; bq.z = pk[4 * ks + 2]; bq.w = pk[4 * ks + 3];
      const f16x8 b = as_f16x8(bq);
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) {
        const f16x8 a = as_f16x8(sSA[(ks * L::MBZ + mb) * 64 + lane]);
        o[mb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, o[mb], 0, 0, 0);
      }
      const f16x8 az = as_f16x8(sSA[(ks * L::MBZ + L::MB) * 64 + lane]);
      dn = __builtin_amdgcn_mfma_f32_32x32x16_f16(az, b, dn, 0, 0, 0);
    }
    if (valid) {
      const float inv = 1.0f / dn[0];
      uint4* orow = reinterpret_cast<uint4*>(ob + (size_t)t * D + g * (D / 2));
#pragma unroll
      for (int mb = 0; mb < L::MB; ++mb) {
        uint4 a, b;
        a.x = pack_bf16x2(o[mb][0] * inv, o[mb][1] * inv);   a.y = pack_bf16x2(o[mb][2] * inv, o[mb][3] * inv);
        a.z = pack_bf16x2(o[mb][4] * inv, o[mb][5] * inv);   a.w = pack_bf16x2(o[mb][6] * inv, o[mb][7] * inv);
        b.x = pack_bf16x2(o[mb][8] * inv, o[mb][9] * inv);   b.y = pack_bf16x2(o[mb][10] * inv, o[mb][11] * inv);
        b.z = pack_bf16x2(o[mb][12] * inv, o[mb][13] * inv); b.w = pack_bf16x2(o[mb][14] * inv, o[mb][15] * inv);
        orow[2 * mb] = a;
        orow[2 * mb + 1] = b;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------
// Transposing LDS read: from a [row][column] fp16 tile, lane l of a wavefront receives
// tile[row0 + 8*(l/32) + 0..7][col0 + l%32] -- an MFMA A or B operand whose contraction index
// is the tile row.  Two ds_read_b64_tr_b16: within each group of 16 lanes, lane s supplies the
// address of row s/4, columns 4*(s%4)..+3, and receives column s of the four rows.
template <int D>
__device__ __forceinline__ f16x8 read_tr(const char* tile, int row0, int col0, int lane) {
  constexpr int RS = D * 2;   // row stride in bytes
  const int r = row0 + 8 * (lane / 32) + ((lane % 16) / 4);
  const int col = col0 + 16 * ((lane / 16) % 2) + 4 * (lane % 4);    // element column, multiple of 4
  const int chunk = col / 8, within = (col % 8) * 2;
  struct { s16x4 lo, hi; } v;
  {
    const char* p = tile + r * RS + ((chunk ^ swz<D>(r)) * 16) + within;
    v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  }
  {
    const int r2 = r + 4;
    const char* p = tile + r2 * RS + ((chunk ^ swz<D>(r2)) * 16) + within;
    v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(p));
  }
  return __builtin_bit_cast(f16x8, v);
}

template <int D>
__global__ __launch_bounds__(NT, 2) void state_partials_bf16_kernel(const uint16_t* __restrict__ k, const uint16_t* __restrict__ v,
                                                                    const uint16_t* __restrict__ wk, float* __restrict__ partials,
                                                                    int H, int n, int P, int chunk) {
  using C = Cfg<D>;
  constexpr int RS = D * 2;            // tile row stride, bytes
  constexpr int WMN = D / 64;          // 32x32 blocks per wavefront along each side of S
  constexpr int VPT = (kTile * C::CH) / NT;   // 16-byte chunks of the V tile per thread
  extern __shared__ uint4 smem[];
  uint4* sWA = smem;
  char* sPhi = reinterpret_cast<char*>(sWA + C::W_IMG);   // [kTile][D] fp16, swizzled chunks
  char* sV = sPhi + kTile * RS;                           // [kTile][D] fp16, swizzled chunks

  const int tid = threadIdx.x, lane = tid % 64, w = tid / 64;
  const int g = lane / 32;
  const int mi = w / 2, ni = w % 2;
  const int bh = blockIdx.y, p = blockIdx.x, h = bh % H;
  const int t_begin = p * chunk;
  const int t_end = min(n, t_begin + chunk);
  const uint16_t* kb = k + (size_t)bh * n * D;
  const uint16_t* vb = v + (size_t)bh * n * D;

  build_w_image<D>(wk + (size_t)h * D * C::HALF, sWA, tid);

  f32x16 s[WMN][WMN], zacc;
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    zacc[r] = 0.f;
#pragma unroll
    for (int i = 0; i < WMN; ++i)
#pragma unroll
      for (int j = 0; j < WMN; ++j) s[i][j][r] = 0.f;
  }
  const int zmb = (WMN == 2) ? (2 * mi + ni) : mi;      // row block of z this wavefront sums
  const bool do_z = (WMN == 2) || (ni == 0);
  uint4 ones;
  ones.x = ones.y = ones.z = ones.w = 0x3C003C00u;      // fp16 1.0 pairs

  uint4 xb[C::UK], vreg[VPT];
  auto load_tile = [&](int t0) {
    const int t = t0 + 32 * w + (lane % 32);
    const int tc = t < t_end ? t : (t_end - 1);
    const uint4* row = reinterpret_cast<const uint4*>(kb + (size_t)tc * D);
#pragma unroll
    for (int ks = 0; ks < C::UK; ++ks) xb[ks] = row[2 * ks + g];
#pragma unroll
    for (int i = 0; i < VPT; ++i) {
      const int idx = tid + NT * i;
      const int r = idx / C::CH, c = idx % C::CH;
      const int tv = (t0 + r) < t_end ? (t0 + r) : (t_end - 1);
      vreg[i] = reinterpret_cast<const uint4*>(vb + (size_t)tv * D)[c];
    }
  };

  load_tile(t_begin);
  __syncthreads();                               // W image complete
  for (int t0 = t_begin; t0 < t_end; t0 += kTile) {
    const bool valid = (t0 + 32 * w + (lane % 32)) < t_end;
    uint32_t pk[C::NPK];
    phi_block<D>(xb, sWA, lane, valid, pk);
    __syncthreads();                             // previous tile's operand reads are done
    {
      const int r = 32 * w + (lane % 32);
      char* rowp = sPhi + r * RS;
      const int sw = swz<D>(r);
      constexpr int CPH = C::LOC / 8;            // 16-byte chunks per softmax half a lane owns
#pragma unroll
      for (int c = 0; c < CPH; ++c) {
        uint4 a, b;
        a.x = pk[4 * c]; a.y = pk[4 * c + 1]; a.z = pk[4 * c + 2]; a.w = pk[4 * c + 3];
        b.x = pk[C::LOC / 2 + 4 * c]; b.y = pk[C::LOC / 2 + 4 * c + 1];
        b.z = pk[C::LOC / 2 + 4 * c + 2]; b.w = pk[C::LOC / 2 + 4 * c + 3];
        *reinterpret_cast<uint4*>(rowp + (((g * CPH + c) ^ sw) * 16)) = a;                 // softmax(+u) half
        *reinterpret_cast<uint4*>(rowp + (((C::CH / 2 + g * CPH + c) ^ sw) * 16)) = b;     // softmax(-u) half
      }
#pragma unroll
      for (int i = 0; i < VPT; ++i) {
        const int idx = tid + NT * i;
        const int rv = idx / C::CH, c = idx % C::CH;
        uint4 h;
        h.x = bf16x2_to_f16x2(vreg[i].x); h.y = bf16x2_to_f16x2(vreg[i].y);
        h.z = bf16x2_to_f16x2(vreg[i].z); h.w = bf16x2_to_f16x2(vreg[i].w);
        *reinterpret_cast<uint4*>(sV + rv * RS + ((c ^ swz<D>(rv)) * 16)) = h;
      }
    }
    __syncthreads();
    if (t0 + kTile < t_end) load_tile(t0 + kTile);   // in flight during the MFMA phase below

#pragma unroll
    for (int ks = 0; ks < kTile / 16; ++ks) {
      f16x8 a[WMN], b[WMN];
#pragma unroll
      for (int i = 0; i < WMN; ++i) a[i] = read_tr<D>(sPhi, 16 * ks, 32 * (mi * WMN + i), lane);
#pragma unroll
      for (int j = 0; j < WMN; ++j) b[j] = read_tr<D>(sV, 16 * ks, 32 * (ni * WMN + j), lane);
#pragma unroll
      for (int i = 0; i < WMN; ++i)
#pragma unroll
        for (int j = 0; j < WMN; ++j) s[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], s[i][j], 0, 0, 0);
      if (do_z) {
        const f16x8 az = (WMN == 2) ? a[ni] : a[0];
        zacc = __builtin_amdgcn_mfma_f32_32x32x16_f16(az, as_f16x8(ones), zacc, 0, 0, 0);
      }
    }
  }

  // partial state in the exported layout: S [D][D] (feature rows in the order of Eq. 5), then z [D]
  float* dst = partials + ((size_t)bh * P + p) * (size_t)(D + 1) * D;
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
}

template <int D>
constexpr size_t state_smem() { return sizeof(uint4) * Cfg<D>::W_IMG + 2 * (size_t)kTile * D * 2; }
template <int D>
constexpr size_t apply_smem() { return sizeof(uint4) * (Cfg<D>::W_IMG + ApplyLayout<D>::KS * ApplyLayout<D>::MBZ * 64); }

template <typename K>
hipError_t set_smem(K kernel, size_t bytes) {
  return hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

}  // namespace

hipError_t launch_state_partials_bf16(const void* k, const void* v, const void* wk, float* partials,
                                      const Plan& p, hipStream_t s) {
  dim3 grid(p.P, p.BH), block(NT);
  hipError_t e;
  if (p.d == 128) {
    if ((e = set_smem(state_partials_bf16_kernel<128>, state_smem<128>())) != hipSuccess) return e;
    state_partials_bf16_kernel<128><<<grid, block, state_smem<128>(), s>>>(
        (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)wk, partials, p.H, p.n, p.P, p.chunk);
  } else {
    if ((e = set_smem(state_partials_bf16_kernel<64>, state_smem<64>())) != hipSuccess) return e;
    state_partials_bf16_kernel<64><<<grid, block, state_smem<64>(), s>>>(
        (const uint16_t*)k, (const uint16_t*)v, (const uint16_t*)wk, partials, p.H, p.n, p.P, p.chunk);
  }
  return hipGetLastError();
}

hipError_t launch_apply_bf16(const void* q, const void* wq, const void* sa, void* out,
                             const Plan& p, hipStream_t s) {
  dim3 grid(p.QP, p.BH), block(NT);
  hipError_t e;
  if (p.d == 128) {
    if ((e = set_smem(apply_bf16_kernel<128>, apply_smem<128>())) != hipSuccess) return e;
    apply_bf16_kernel<128><<<grid, block, apply_smem<128>(), s>>>(
        (const uint16_t*)q, (const uint16_t*)wq, (const uint4*)sa, (uint16_t*)out, p.H, p.n, p.qchunk);
  } else {
    if ((e = set_smem(apply_bf16_kernel<64>, apply_smem<64>())) != hipSuccess) return e;
    apply_bf16_kernel<64><<<grid, block, apply_smem<64>(), s>>>(
        (const uint16_t*)q, (const uint16_t*)wq, (const uint4*)sa, (uint16_t*)out, p.H, p.n, p.qchunk);
  }
  return hipGetLastError();
}

}  // namespace linattn
