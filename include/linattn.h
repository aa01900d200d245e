/*
 * linattn.h -- C ABI of the MI355X (gfx950) linear-attention library.
 *
 * The operator is the non-causal linear attention that LinVideo puts in place of
 * softmax attention in a video diffusion transformer (paper Sec. 3):
 *
 *   Eq. 3:  o_i = phi(q_i) S / (phi(q_i) . z),   S = sum_j phi(k_j)^T v_j,  z = sum_j phi(k_j)
 *   Eq. 5:  phi(x) = softmax(x W~) (+) softmax(-x W~),  W~ in R^{d x d/2}, one W~ for q, one for k
 *
 * evaluated independently for every (batch, head) pair over all n tokens (no mask, no
 * scaling of q.k, no epsilon: every entry of phi is positive so the denominator is too).
 *
 * Conventions shared by every entry point
 *   - q, k, v, out, dout, dq, dk, dv: DEVICE pointers, 16-byte aligned, d innermost and
 *     contiguous, all eight in the descriptor's layout: [B, H, n, d] (LINATTN_LAYOUT_BHND, the
 *     default) or [B, n, H, d] (LINATTN_LAYOUT_BNHD: heads interleaved per token, the form in
 *     which a transformer block's projection q = x W_q (Sec. 3) leaves them, so no transpose
 *     copy is needed around the operator).  d in {64, 128}, n >= 1 arbitrary, B, H >= 1,
 *     64-bit indexing inside.
 *   - element type of those tensors and of W~ is the descriptor's dtype: bf16 (LINATTN_BF16 and
 *     LINATTN_BF16_F32MATH) or fp32 (LINATTN_F32).  All accumulation is fp32.  The fp32 mode never
 *     rounds through bf16.
 *   - all pointers are borrowed: the caller keeps them alive until the stream work is done.
 *   - calls only enqueue work on `stream` (a hipStream_t passed as void*, NULL = default
 *     stream).  They never synchronise and never allocate.
 *   - every argument error is detected on the host before any HIP call and returned as a
 *     negative status; nothing is enqueued in that case.
 *   - results are bitwise reproducible run to run (no floating-point atomics).
 *   - out must not alias q, k or v; dq, dk, dv must not alias any input.
 *   - calls that share a descriptor share its workspace: do not overlap them on
 *     different streams.
 *
 * Numeric domain of the bf16 mode (the fp32 mode computes in fp32 throughout)
 *   - q, k enter the projection of Eq. 5 as stored; phi, v, dout and the states S, dS enter the
 *     matrix cores as fp16 (11-bit significand) with fp32 accumulation.  phi, the states, dout and
 *     every gradient operand are rescaled by exact powers of two first (per token, per 32-token
 *     block, per head, or per workgroup following the running maximum), so their magnitude does
 *     not matter: any finite bf16 q, k, dout is in the domain.
 *   - v is widened to fp16 unscaled: |v| must be below 65504 (fp16's largest finite value).  Larger
 *     entries become infinite inside the kernels and the call returns LINATTN_OK with Inf/NaN in
 *     out, state and the gradients; the library does not scan for them.  Entries with
 *     0 < |v| < 2^-14 lose their low bits (absolute error below 2^-25).
 *   - Accuracy: out, dq, dk, dv, dW~ agree with exact arithmetic on the stored inputs to 1e-2 of
 *     max(|value|, RMS of the tensor over its (b,h) slice).  Known exception (11-bit operands):
 *     dL/dphi(k_j) = v_j dS^T + dz inherits an absolute error of about 2e-4 |v_j| |dS| from the
 *     fp16 operands behind dS, so the dk row of a key whose v_j is far larger than the other
 *     tokens' carries |v_j| / rms|v| times the error of an ordinary row.  For the rows at 20x
 *     magnitude of the Wan-14B-shaped test recipe (0.1 % of the tokens) this reads up to 1e-1 of the
 *     slice RMS, and dW~_k, which weights those rows by |k_j| once more, up to 2e-2; all other rows of
 *     dk, and dq, dv, dW~_q everywhere, meet 1e-2.  (A common offset of v, however large, is not an
 *     exception: the backward's operand images are built with the head's mean value row taken out.)  Second exception: where phi is within a few per
 *     cent of uniform (the spread of x W~ over the features far below 1), dq, dk and dW~ are
 *     differences of nearly equal rows of S and dS and come out up to 0.2 off; out and dv keep 1e-2.
 *     LINATTN_FLAG_CENTRED removes this exception (not the first) at a cost of 3-5 %.
 *   - LINATTN_BF16_F32MATH reads and writes the same bf16 tensors but does all arithmetic in fp32
 *     (the kernels of the fp32 mode, no matrix cores, no fp16 operands): none of the limits above
 *     applies, |v| may be any finite bf16 value, and the only rounding that matters is the bf16
 *     store of the results.  It is about 50x slower than LINATTN_BF16 (5.5 ms against 0.11 ms for the
 *     forward at the Wan-1.3B 480p shape): a device-side reference and a mode for numerically
 *     delicate inputs, not the fast path.
 */
#ifndef LINATTN_H
#define LINATTN_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* status codes */
#define LINATTN_OK            0
#define LINATTN_E_NULL       -1   /* a required pointer is NULL */
#define LINATTN_E_SHAPE      -2   /* B, H, n <= 0, unsupported d, shape differs from the descriptor, or too large */
#define LINATTN_E_DTYPE      -3   /* unknown dtype */
#define LINATTN_E_ALIGN      -4   /* a tensor pointer is not 16-byte aligned */
#define LINATTN_E_PHI        -5   /* unknown phi_id / unsupported kind / table full */
#define LINATTN_E_WORKSPACE  -6   /* workspace missing or smaller than linattn_workspace_bytes() */
#define LINATTN_E_HIP        -7   /* a HIP launch reported an error */
#define LINATTN_E_STATE      -8   /* linattn_bwd without a state buffer, or a state buffer too small for this B */
#define LINATTN_E_ALIAS      -9   /* an output aliases an input */

/* feature-map kinds */
#define LINATTN_PHI_HEDGEHOG  1   /* Eq. 5 */
#define LINATTN_PHI_RELU      2   /* phi(x) = max(x, 0) on the d channels, no weights: the "ReLU" row of the
                                     paper's ablation of kernel functions (appendix "Ablation for Kernel
                                     Function").  The paper gives the name only; this library's reading:
                                     o_i = phi(q_i) S / (phi(q_i) . z + 1e-6), because a row of q or k can be
                                     all non-positive (such a query gets o_i = 0); the derivative of max(x, 0)
                                     at 0 is 0.  Descriptor: wq, wk, dwq, dwk and the three blend pointers
                                     must be NULL (E_PHI otherwise); state rows are the d channels of k. */

/* dtypes */
#define LINATTN_BF16  1          /* bf16 tensors, matrix-core kernels (bf16 / fp16 operands, fp32 accumulation) */
#define LINATTN_F32   2          /* fp32 tensors, fp32 arithmetic */
#define LINATTN_BF16_F32MATH 3   /* bf16 tensors, fp32 arithmetic (see "Numeric domain" above) */

/* descriptor flags */
#define LINATTN_FLAG_CENTRED 1u  /* LINATTN_BF16 with the map of Eq. 5: every fp16 operand that carries phi or a state is
                                    rounded after its mean has been taken out -- phi - 2/d in the two sums over tokens
                                    (state pass: S, z; query-side backward: dS, dz), with (2/d) x the column sums of v
                                    resp. of dout/den added back in fp32; operand images of S - z vbar^T (vbar the
                                    head's mean value row) and of dS, dz minus their means over each half's features,
                                    which the softmax Jacobian drops (dv gets the constant row back).  Exact in real
                                    arithmetic; the roundings then act on the deviation of phi from the uniform map, so
                                    the regime where phi is within a few per cent of uniform meets the 1e-2 contract
                                    for all five gradients.  Costs about 3 % of the forward (8 % of its state pass) and
                                    4 % of the backward.  A layer uses one setting for its forward and backward calls. */

/* memory layouts of q, k, v, out, dout, dq, dk, dv */
#define LINATTN_LAYOUT_BHND  0   /* element (b,h,t,c) at ((b*H + h)*n + t)*d + c */
#define LINATTN_LAYOUT_BNHD  1   /* element (b,h,t,c) at ((b*n + t)*H + h)*d + c */

/*
 * Description of a feature map plus the buffers a layer owns.  Eq. 3 takes q, k, v only;
 * Eq. 5 adds the two learnable matrices, which live here so that linattn_fwd keeps the
 * paper's argument list.  The struct is copied by linattn_phi_create.
 */
typedef struct linattn_phi_desc {
  int kind;               /* LINATTN_PHI_HEDGEHOG or LINATTN_PHI_RELU */
  int dtype;              /* LINATTN_BF16, LINATTN_F32 or LINATTN_BF16_F32MATH: type of q,k,v,out,dout,dq,dk,dv,wq,wk */
  int H, d;               /* wq, wk: device, [H, d, d/2] contiguous, one map per head (Eq. 5) */
  const void *wq, *wk;
  void *dwq, *dwk;        /* optional device fp32 [H, d, d/2]: linattn_bwd OVERWRITES them with the
                             gradient summed over batch and tokens; NULL = not computed */
  void *state;            /* optional device fp32 [B, H, d+1, d]: rows 0..d-1 = S with rows indexed by
                             the feature of phi in the order of Eq. 5 (softmax(+) half first),
                             row d = z.  linattn_fwd writes it when non-NULL; linattn_bwd reads it.
                             Its size is state_bytes (last field). */
  void *workspace;        /* device scratch, 256-byte aligned, >= linattn_workspace_bytes(...) */
  size_t workspace_bytes;
  int layout;             /* LINATTN_LAYOUT_BHND (0) or LINATTN_LAYOUT_BNHD; the state, dW~ and the
                             workspace do not depend on it */
  /* Mixed attention of the selective-transfer stage (Sec. 4.1, Eq. 6), active when blend_in and
   * blend_r are both non-NULL (set only one: E_NULL):
   *     out = r' * blend_in + (1 - r') * (Eq. 3),   r' = clip(*blend_r, 0, 1)  (footnote to Eq. 6)
   * blend_in is the softmax-attention output of the same layer, computed by the caller: device,
   * dtype and layout of out, must not overlap out.  blend_r: device, one fp32, read by the
   * kernels (no host copy).  linattn_bwd then treats dout as the gradient of the blended output:
   * dq, dk, dv, dW~ receive (1 - r') times the gradients of Eq. 3, and blend_dr (optional, device,
   * one fp32) is OVERWRITTEN with dL/dr = sum(dout * (blend_in - o)) for 0 <= r <= 1 and 0 outside
   * (the closed ends let r move from its initial value 1).  The gradient with respect to blend_in
   * is r' * dout, an elementwise product left to the caller. */
  const void *blend_in;
  const float *blend_r;
  float *blend_dr;
  size_t state_bytes;     /* bytes behind `state` (ignored when state is NULL).  A call with batch size B
                             touches B * H * (d+1) * d * 4 of them: linattn_phi_create returns E_STATE if
                             not even B = 1 fits, linattn_fwd / linattn_bwd return E_STATE for a B that
                             does not fit. */
  unsigned flags;         /* 0, or LINATTN_FLAG_CENTRED (Eq. 5 map with LINATTN_BF16 only: E_PHI otherwise) */
} linattn_phi_desc;

/* Register a descriptor; *phi_id_out receives a handle >= 16.  Host-only, no HIP call.
 * Errors: E_NULL (desc, out, wq, wk), E_PHI (kind, table full, flags that do not fit kind or dtype), E_DTYPE, E_SHAPE (H, d, layout),
 * E_ALIGN, E_STATE (state given with state_bytes < H * (d+1) * d * 4). */
int linattn_phi_create(const linattn_phi_desc* desc, int* phi_id_out);

/* Forget a handle.  E_PHI if it is not live.  Buffers stay the caller's. */
int linattn_phi_destroy(int phi_id);

/* Replace the three mixed-attention pointers of a live handle (blend_in changes every step).
 * All NULL switches the blend off.  Host-only.  Errors: E_PHI, E_NULL (exactly one of blend_in,
 * blend_r given, or blend_dr without them), E_ALIGN (blend_in not 16-byte aligned). */
int linattn_phi_set_blend(int phi_id, const void* blend_in, const float* blend_r, float* blend_dr);

/* Scratch bytes linattn_fwd, and linattn_bwd without weight gradients (dwq == dwk == NULL), need
 * for this problem (pure function of its arguments, no HIP call).  Returns 0 for an invalid
 * argument. */
size_t linattn_workspace_bytes(int B, int H, int n, int d, int kind, int dtype);

/* Scratch bytes linattn_bwd needs when the descriptor asks for dwq or dwk (W~ is learnable, Eq. 5):
 * the above plus the partial sums of dW~ (one [d][d/2] fp32 block per workgroup of the two main kernels) and, in
 * the fp32-arithmetic modes only, two fp32 buffers [B,H,n,d/2] for dL/du (the bf16 kernels accumulate dW~ where
 * du is made).  For LINATTN_PHI_RELU (no weights) it equals linattn_workspace_bytes. */
size_t linattn_workspace_bytes_wgrads(int B, int H, int n, int d, int kind, int dtype);

/*
 * Forward, Eq. 3 with the descriptor's phi (Eq. 5, or the ReLU map).  Three stages on `stream`: phi(K) fused with a split-n
 * partial state, a fixed-order reduction of the partials, phi(Q) S / (phi(Q) . z) with the
 * store of out.  Writes out [B,H,n,d] and, if the descriptor has one, state.
 * Errors: E_PHI, E_NULL, E_SHAPE (also H or d different from the descriptor), E_ALIGN,
 * E_WORKSPACE, E_STATE (state buffer smaller than this B needs), E_ALIAS, E_HIP.
 */
int linattn_fwd(const void* q, const void* k, const void* v, void* out,
                int B, int H, int n, int d, int phi_id, void* stream);

/*
 * linattn_fwd for callers that cannot allocate device memory or size a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels and bit-identical results, but the split-n partials (and the state, when the descriptor
 * has no state buffer) live in a static device array of LINATTN_NOALLOC_SCRATCH_BYTES that is part
 * of the library's code object on each GPU; the descriptor's workspace is ignored and may be NULL.
 * The call allocates nothing and frees nothing.
 *   - Limit: the forward scratch of the problem (what linattn_workspace_bytes counts up to the
 *     state region: partials of at most 256 workgroups plus B*H states) must fit the array;
 *     E_WORKSPACE otherwise.  All five task configurations fit (config 4 needs 31.7 MB).
 *   - Every call on one GPU shares that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race.  Nothing needs clearing between calls: a call overwrites every
 *     scratch word before reading it.
 *   - The first call on a device looks the array's address up (hipGetSymbolAddress); make that
 *     call outside stream capture.
 * Errors: as linattn_fwd; E_HIP also if the array's address cannot be found.
 */
#define LINATTN_NOALLOC_SCRATCH_BYTES (32u << 20)
int linattn_fwd_noalloc(const void* q, const void* k, const void* v, void* out,
                        int B, int H, int n, int d, int phi_id, void* stream);

/*
 * Backward of linattn_fwd for L with dL/dout = dout: writes dq, dk, dv [B,H,n,d] and, if the
 * descriptor has them, dwq and dwk (Eq. 5 only; the ReLU map has no weights).  Needs the state a
 * forward call with the same q-independent inputs (k, v, wk) left in the descriptor's state buffer.
 * Errors: as linattn_fwd, plus E_STATE.
 */
int linattn_bwd(const void* q, const void* k, const void* v, const void* dout,
                void* dq, void* dk, void* dv,
                int B, int H, int n, int d, int phi_id, void* stream);

/* Static description of a status code. */
const char* linattn_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* LINATTN_H */
