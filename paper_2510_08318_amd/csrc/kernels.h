// Internal interface between the host dispatch (api.cpp) and the gfx950 kernels.
// Nothing here is exported from the shared library.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <atomic>

namespace linattn {

// Tokens a workgroup of the bf16 kernels consumes per iteration (4 waves x 32 tokens).
constexpr int kTile = 128;
// Workgroup slots the split-n plan aims to fill: one resident workgroup per compute unit.
constexpr int kSlots = 256;
// Compute units of the gfx950 parts this library targets (MI355X / MI350X).
constexpr int kCUs = 256;
// Feature maps (the values of LINATTN_PHI_*): Eq. 5, and the weight-free phi(x) = max(x, 0) of the
// kernel-function ablation.  The ReLU map can give phi(q) . z = 0, so its denominator carries
// kReluEps.
constexpr int kPhiHedgehog = 1, kPhiRelu = 2;
constexpr float kReluEps = 1e-6f;
// Workgroups (= partial sums) of the streaming dot product sum(dout * s) of the mixed attention's dL/dr.
constexpr int kDotParts = 1024;

// Where the rows of q, k, v, out (and dout, dq, dk, dv) sit in memory, in elements: element
// (b, h, t, c) is at b*sb + h*sh + t*sn + c.  [B,H,n,d]: sb = H*n*d, sh = n*d, sn = d;
// [B,n,H,d] (heads interleaved per token, what a transformer block's projection emits):
// sb = n*H*d, sh = d, sn = H*d.
struct Rows {
  size_t sb, sh, sn;
};
__host__ __device__ inline size_t head_base(const Rows& r, int bh, int H) {
  return (size_t)(bh / H) * r.sb + (size_t)(bh % H) * r.sh;
}

// Split of the bf16 state pass: the T = B*H*ntile 128-token tiles of a call, in (b,h)-major order,
// are dealt to G workgroups in contiguous ranges [lo(g), lo(g+1)), lo(g) = floor(g*T/G), so that
// every compute unit gets the same share whatever B*H is (a per-head split leaves
// 256 mod B*H units idle).  T/G <= ntile, so a range touches at most two heads; a workgroup
// writes one partial state per head it touches, into slot g - owner(first tile of the head).
struct Split {
  int G;            // workgroups
  int ntile;        // tiles per (b,h)
  long long T;      // tiles in all
  int PS;           // partial slots per (b,h) (the largest number of workgroups touching one head)
};
__host__ __device__ inline long long split_lo(const Split& s, int g) { return (long long)g * s.T / s.G; }
// the workgroup whose range holds tile x
__host__ __device__ inline int split_owner(const Split& s, long long x) {
  int g = (int)(x * s.G / s.T);
  while (g + 1 < s.G && split_lo(s, g + 1) <= x) ++g;
  while (g > 0 && split_lo(s, g) > x) --g;
  return g;
}

// How one call is cut into workgroups and where its scratch regions sit in the workspace.
struct Plan {
  int B, H, n, d;
  int kind;         // kPhiHedgehog or kPhiRelu (set by the dispatch, not by make_plan)
  bool bf16_storage; // the fp32-arithmetic kernels read and write bf16 tensors (LINATTN_BF16_F32MATH)
  bool centred;      // LINATTN_FLAG_CENTRED (set by the dispatch): phi minus its mean in the sums over tokens, centred operand images
  int BH;
  Rows rows;        // memory layout of the token tensors
  Split split;      // bf16 forward state pass
  int P;            // split-n factor (partials per (b,h)) of the fp32 state pass and of the backward
  int chunk;        // tokens per split, a multiple of kTile (fp32 kernels; the bf16 ones deal tiles round-robin)
  int QP;           // workgroups per (b,h) of the query pass
  int qchunk;       // tokens per workgroup of the fp32 query pass
  size_t state_elems;     // (d+1)*d
  size_t off_partials;    // fp32 [BH][max(P, split.PS)][(d+1)*d]
  size_t off_state;       // fp32 [BH][(d+1)*d]   (used when the caller gave no state buffer)
  size_t fwd_bytes;       // end of the two regions above: all the scratch a forward call touches
  // backward only
  int KP;                 // workgroups per (b,h) of the key-side backward pass
  size_t off_dstate;      // fp32 [BH][(d+1)*d]   dS, dz
  size_t off_gimg;        // fp16 [BH][d*d]       operand image of S for dL/dphi(q) (bf16 mode)
  // operand images built once per head by the backward's prep kernels (bf16 mode)
  size_t img_state_bytes; // bytes of one query-pass-style image of a (d+1) x d state
  size_t off_simg;        // [BH] image of S (as in the query pass), for the recomputed o
  size_t off_dsimg;       // [BH] the same image of dS, for dv
  size_t off_dgimg;       // fp16 [BH][d*d]       operand image of dS for dL/dphi(k)
  size_t off_wimg;        // [H][4][d*d bytes]    W~_q image, W~_q transposed image, then the same for W~_k
  size_t off_scales;      // fp32 [BH][2]         power-of-two scales of the S and dS images
  size_t off_centre;      // centred backward: fp32 [BH][3][d] (mean value row vbar, constant row of dv, centred dz), then
                          // [BH][P][d+8] per-workgroup column sums of dO/den (d) and the sum of -delta/den (1)
  size_t off_drpart;      // fp32 [BH][P] + [kDotParts]: per-workgroup parts of dL/dr (mixed attention, Eq. 6)
  size_t off_dwpart;      // fp32 [BH][P][d*d/2] partial dW~_q, then [BH][max(P, KP)][d*d/2] partial dW~_k (weight gradients only)
  size_t du_bytes;        // bytes of one dL/du region (0 in bf16 mode: dW~ is accumulated where du is made)
  size_t off_du_q;        // dL/du of the query side (weight gradients, fp32 arithmetic only): fp32 [BH][n][d/2]
  size_t off_du_k;        // the same for the key side
  size_t bytes_no_wgrads; // workspace needed by forward and by backward without dW~
  size_t total_bytes;
};

// Pure host arithmetic; returns false if the shape is unsupported or overflows.
// total_bytes includes the weight-gradient regions, bytes_no_wgrads does not.
bool make_plan(int B, int H, int n, int d, int dtype, int layout, Plan* p);

// Everything one backward call touches (device pointers; workspace regions already resolved).
struct BwdArgs {
  const void *q, *k, *v, *dout, *wq, *wk;
  void *dq, *dk, *dv;
  const float* state;     // [BH][d+1][d] from the forward
  float *dwq, *dwk;       // nullable
  float *partials, *dstate, *dw_part, *du_q, *du_k;
  void* gimg;
  void *simg, *dsimg, *dgimg, *wimg;
  float* scales;
  float *vbar, *dv_row, *dzc, *cs_part;   // centred backward (Plan::off_centre)
  // mixed attention (Eq. 6): softmax-branch output, the layer's r, dL/dr; all null when off
  const void* blend_in;
  const float* blend_r;
  float* blend_dr;
  float* dr_part;
};

// Raises a kernel's dynamic-LDS limit to `bytes`, once per kernel instantiation and device: the
// attribute call is a driver call, and the launchers sit on the enqueue path of every step.
template <auto Kernel>
hipError_t set_smem_once(size_t bytes) {
  static std::atomic<uint64_t> done{0};
  int dev = -1;
  const bool tracked = hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < 64;
  if (tracked && (done.load(std::memory_order_acquire) >> dev & 1)) return hipSuccess;
  const hipError_t e = hipFuncSetAttribute((const void*)Kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && tracked) done.fetch_or(uint64_t(1) << dev, std::memory_order_release);
  return e;
}

// ---- forward launchers (enqueue only) ---------------------------------------------------
// phi(K) fused with the split-n partial state (Eq. 5 + the two sums of Eq. 3).
hipError_t launch_state_partials_f32(const void* k, const void* v, const void* wk, float* partials,
                                     const Plan& p, hipStream_t s);
hipError_t launch_state_partials_bf16(const void* k, const void* v, const void* wk, float* partials,
                                      const Plan& p, hipStream_t s);
// The same for the ReLU map (bf16); partial slots per head follow Plan::split as well.
hipError_t launch_relu_state_bf16(const void* k, const void* v, float* partials, const Plan& p, hipStream_t s);
// Fixed-order sum of the partials into the exported state layout [BH][d+1][d] fp32.
hipError_t launch_state_reduce(const float* partials, float* state, const Plan& p, hipStream_t s);
// The same for the partials of the bf16 forward state pass (slots per head follow Plan::split).
hipError_t launch_state_reduce_split(const float* partials, float* state, const Plan& p, hipStream_t s);
// phi(Q) S / (phi(Q) . z) and the store of out (Eq. 3, right-hand side).
hipError_t launch_apply_f32(const void* q, const void* wq, const float* state, void* out,
                            const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s);
hipError_t launch_apply_bf16(const void* q, const void* wq, const float* state, void* out,
                             const void* blend_in, const float* blend_r, const Plan& p, hipStream_t s);

// ---- backward launchers (enqueue only) --------------------------------------------------
// dw[H][d][d/2] = sum over batch and tokens of x^T du; x is [B,H,n,d] bf16 or fp32, du fp32 [B,H,n,d/2].
// dw[h][e] = sum over b, then over the P splits, of part[(b*H+h)][p][e].
hipError_t launch_dw_reduce(const float* part, float* dw, const Plan& p, hipStream_t s);
// The same for two (partials, output, partials per (b,h)) triples in one launch; a triple whose output is null is skipped.
hipError_t launch_dw_reduce2(const float* part0, float* dw0, int P0, const float* part1, float* dw1, int P1, const Plan& p, hipStream_t s);
hipError_t launch_dw(const void* x, bool x_is_bf16, const float* du, float* part, float* dw, const Plan& p, hipStream_t s);
hipError_t launch_bwd_bf16(const BwdArgs& a, const Plan& p, hipStream_t s);
hipError_t launch_bwd_f32(const BwdArgs& a, const Plan& p, hipStream_t s);
hipError_t launch_relu_bwd_bf16(const BwdArgs& a, const Plan& p, hipStream_t s);
// part[0 .. kDotParts-1] = partial sums of sum_i a[i] * b[i] over two contiguous bf16 arrays (elems % 8 == 0).
hipError_t launch_dot_bf16(const void* a, const void* b, size_t elems, float* part, hipStream_t s);
// part[0 .. kDotParts-1] = partial sums of sum_i a[i] * (b[i] - vbar[bh(i)][channel(i)]) over two bf16 token tensors in the
// plan's layout; vbar fp32 [BH][d].
hipError_t launch_dot_centred_bf16(const void* a, const void* b, const float* vbar, float* part, const Plan& p, hipStream_t s);
// dr = sum of the count parts in a fixed order if 0 <= *r <= 1, else 0 (Eq. 6, clipped r).
hipError_t launch_dr_reduce(const float* part, int count, const float* r, float* dr, hipStream_t s);

}  // namespace linattn
