// Host side of the C ABI: descriptor table, argument validation, launch plan, dispatch.
// Every check happens before the first HIP call, so the error paths run on a machine
// with no GPU.
#include "../../include/linattn.h"
#include "../../include/linattn_bench.h"
#include "kernels.h"

#include <mutex>
#include <cstring>

namespace linattn {

bool make_plan(int B, int H, int n, int d, int dtype, int layout, Plan* p) {
  if (B <= 0 || H <= 0 || n <= 0) return false;
  if (d != 64 && d != 128) return false;
  if (dtype != LINATTN_BF16 && dtype != LINATTN_F32 && dtype != LINATTN_BF16_F32MATH) return false;
  if (layout != LINATTN_LAYOUT_BHND && layout != LINATTN_LAYOUT_BNHD) return false;
  const long long BH = (long long)B * H;
  if (BH > 65535) return false;                       // grid.y
  if ((long long)n > (1LL << 30)) return false;
  Plan r{};
  r.B = B; r.H = H; r.n = n; r.d = d; r.BH = (int)BH;
  r.bf16_storage = dtype == LINATTN_BF16_F32MATH;
  if (layout == LINATTN_LAYOUT_BHND) r.rows = Rows{(size_t)H * n * d, (size_t)n * d, (size_t)d};
  else r.rows = Rows{(size_t)n * H * d, (size_t)d, (size_t)H * d};
  const int tiles = (n + kTile - 1) / kTile;
  int P = kSlots / (int)BH;
  if (P < 1) P = 1;
  if (P > tiles) P = tiles;
  int tiles_per = (tiles + P - 1) / P;
  r.chunk = tiles_per * kTile;
  r.P = (n + r.chunk - 1) / r.chunk;
  r.QP = r.P;
  r.qchunk = r.chunk;
  if (dtype == LINATTN_BF16) {
    // query pass: 12-wavefront workgroups, one per compute unit, 32-token blocks dealt round-robin
    const int nblk = (n + 31) / 32;
    int QP = kCUs / (int)BH;
    if (QP < 1) QP = 1;
    if (QP > (nblk + 11) / 12) QP = (nblk + 11) / 12;
    r.QP = QP;
  }
  r.state_elems = (size_t)(d + 1) * d;
  {
    Split sp{};
    sp.ntile = tiles;
    sp.T = (long long)BH * tiles;
    sp.G = BH > kSlots ? (int)BH : (int)(sp.T < kSlots ? sp.T : kSlots);
    sp.PS = 1;
    for (long long bh = 0; bh < BH; ++bh) {
      const int cnt = split_owner(sp, (bh + 1) * tiles - 1) - split_owner(sp, bh * tiles) + 1;
      if (cnt > sp.PS) sp.PS = cnt;
    }
    r.split = sp;
  }
  auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
  size_t off = 0;
  const int slots = r.P > r.split.PS ? r.P : r.split.PS;
  r.off_partials = off; off = up(off + (size_t)BH * slots * r.state_elems * sizeof(float));
  r.off_state = off;    off = up(off + (size_t)BH * r.state_elems * sizeof(float));
  r.fwd_bytes = off;
  {
    const int nblk = (n + 31) / 32;
    int KP = kCUs / (int)BH;
    if (KP < 1) KP = 1;
    if (KP > (nblk + 7) / 8) KP = (nblk + 7) / 8;
    r.KP = KP;
  }
  r.off_dstate = off;   off = up(off + (size_t)BH * r.state_elems * sizeof(float));
  r.off_gimg = off;     off = up(off + (size_t)BH * d * d * 2);
  r.img_state_bytes = (size_t)(d / 16) * (d / 32 + 1) * 64 * 16;
  r.off_simg = off;     off = up(off + (size_t)BH * r.img_state_bytes);
  r.off_dsimg = off;    off = up(off + (size_t)BH * r.img_state_bytes);
  r.off_dgimg = off;    off = up(off + (size_t)BH * d * d * 2);
  r.off_wimg = off;     off = up(off + (size_t)H * 4 * d * d);
  r.off_scales = off;   off = up(off + (size_t)BH * 2 * sizeof(float));
  r.off_centre = off;   off = up(off + ((size_t)BH * 3 * d + (size_t)BH * r.P * (d + 8)) * sizeof(float));
  r.off_drpart = off;   off = up(off + ((size_t)BH * r.P + kDotParts) * sizeof(float));
  r.bytes_no_wgrads = off;
  r.off_dwpart = off;   off = up(off + (size_t)BH * (r.P + (r.P > r.KP ? r.P : r.KP)) * d * (d / 2) * sizeof(float));
  // the fp32-arithmetic modes keep dL/du as fp32 rows for a separate dW~ pass; the bf16 kernels accumulate dW~ where du is made
  r.du_bytes = dtype == LINATTN_BF16 ? 0 : (size_t)BH * n * (d / 2) * sizeof(float);
  r.off_du_q = off;     off = up(off + r.du_bytes);
  r.off_du_k = off;     off = up(off + r.du_bytes);
  r.total_bytes = off;
  *p = r;
  return true;
}

namespace {

constexpr int kFirstId = 16;
constexpr int kMaxDesc = 1024;

struct Slot {
  bool live = false;
  linattn_phi_desc d{};
};

Slot g_slots[kMaxDesc];
std::mutex g_mu;
hipEvent_t g_stage_events[4];
bool g_stage_events_on = false;

// The four events of the call in flight, copied under the lock by the entry point (null = off).
struct StageEvents {
  bool on = false;
  hipEvent_t ev[4];
  void mark(int i, hipStream_t s) const {
    if (on) (void)hipEventRecord(ev[i], s);
  }
};
StageEvents stage_events() {
  std::lock_guard<std::mutex> lk(g_mu);
  StageEvents r;
  r.on = g_stage_events_on;
  for (int i = 0; i < 4; ++i) r.ev[i] = g_stage_events[i];
  return r;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_blend(const void* blend_in, const float* blend_r, const float* blend_dr) {
  if ((blend_in == nullptr) != (blend_r == nullptr)) return LINATTN_E_NULL;
  if (blend_dr && !blend_in) return LINATTN_E_NULL;
  if (blend_in && (reinterpret_cast<uintptr_t>(blend_in) & 15u)) return LINATTN_E_ALIGN;
  return LINATTN_OK;
}

bool overlaps(const void* a, const void* b, size_t bytes) {
  const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
  return x < y + bytes && y < x + bytes;
}

int fetch(int phi_id, linattn_phi_desc* out) {
  std::lock_guard<std::mutex> lk(g_mu);
  const int i = phi_id - kFirstId;
  if (i < 0 || i >= kMaxDesc || !g_slots[i].live) return LINATTN_E_PHI;
  *out = g_slots[i].d;
  return LINATTN_OK;
}

// Checks common to forward and backward.  Fills desc and plan.  own_scratch: the call brings its own
// scratch memory, so the descriptor's workspace is neither needed nor looked at.
int check_call(const void* const* tensors, int n_tensors, int B, int H, int n, int d, int phi_id,
               bool want_wgrads, linattn_phi_desc* desc, Plan* plan, bool own_scratch = false) {
  int st = fetch(phi_id, desc);
  if (st != LINATTN_OK) return st;
  for (int i = 0; i < n_tensors; ++i)
    if (!tensors[i]) return LINATTN_E_NULL;
  if (H != desc->H || d != desc->d) return LINATTN_E_SHAPE;
  if (!make_plan(B, H, n, d, desc->dtype, desc->layout, plan)) return LINATTN_E_SHAPE;
  plan->kind = desc->kind;
  plan->centred = (desc->flags & LINATTN_FLAG_CENTRED) != 0;
  for (int i = 0; i < n_tensors; ++i)
    if (!aligned16(tensors[i])) return LINATTN_E_ALIGN;
  const size_t need = (want_wgrads && (desc->dwq || desc->dwk)) ? plan->total_bytes : plan->bytes_no_wgrads;
  if (!own_scratch && (!desc->workspace || desc->workspace_bytes < need)) return LINATTN_E_WORKSPACE;
  if (desc->state && (size_t)plan->BH * plan->state_elems * sizeof(float) > desc->state_bytes) return LINATTN_E_STATE;
  return LINATTN_OK;
}

// ---- scratch of linattn_fwd_noalloc ---------------------------------------------------------
// One array per GPU, part of the loaded code object, alive until the process ends.  Its name is a
// host-side handle only: device code is given the address hipGetSymbolAddress returns for the
// current device, looked up once per device.
constexpr size_t kStaticScratchBytes = LINATTN_NOALLOC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
char* g_scratch_ptr[kMaxDevices] = {};

int static_scratch(char** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LINATTN_E_HIP;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return LINATTN_E_HIP;
    g_scratch_ptr[dev] = static_cast<char*>(p);
  }
  *out = g_scratch_ptr[dev];
  return LINATTN_OK;
}

// The forward path on scratch memory `ws` (the descriptor's workspace, or the static array).
int run_fwd(const linattn_phi_desc& desc, const Plan& plan, const void* q, const void* k, const void* v, void* out,
            char* ws, hipStream_t s) {
  float* partials = reinterpret_cast<float*>(ws + plan.off_partials);
  float* state = desc.state ? static_cast<float*>(desc.state) : reinterpret_cast<float*>(ws + plan.off_state);
  hipError_t e;
  const StageEvents ev = stage_events();
  ev.mark(0, s);
  if (desc.dtype != LINATTN_BF16) {
    e = launch_state_partials_f32(k, v, desc.wk, partials, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
    ev.mark(1, s);
    e = launch_state_reduce(partials, state, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
    ev.mark(2, s);
    e = launch_apply_f32(q, desc.wq, state, out, desc.blend_in, desc.blend_r, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
  } else {
    const bool relu = desc.kind == LINATTN_PHI_RELU;
    e = relu ? launch_relu_state_bf16(k, v, partials, plan, s) : launch_state_partials_bf16(k, v, desc.wk, partials, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
    ev.mark(1, s);
    e = launch_state_reduce_split(partials, state, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
    ev.mark(2, s);
    e = launch_apply_bf16(q, desc.wq, state, out, desc.blend_in, desc.blend_r, plan, s);
    if (e != hipSuccess) return LINATTN_E_HIP;
  }
  ev.mark(3, s);
  return LINATTN_OK;
}

// Argument checks of a forward call (everything but the scratch memory).
int check_fwd(const void* q, const void* k, const void* v, void* out, int B, int H, int n, int d, int phi_id,
              bool own_scratch, linattn_phi_desc* desc, Plan* plan) {
  const void* tensors[4] = {q, k, v, out};
  int st = check_call(tensors, 4, B, H, n, d, phi_id, false, desc, plan, own_scratch);
  if (st != LINATTN_OK) return st;
  const size_t esz = desc->dtype == LINATTN_F32 ? 4 : 2;
  const size_t bytes = (size_t)plan->BH * n * d * esz;
  if (overlaps(out, q, bytes) || overlaps(out, k, bytes) || overlaps(out, v, bytes)) return LINATTN_E_ALIAS;
  if (desc->blend_in && overlaps(out, desc->blend_in, bytes)) return LINATTN_E_ALIAS;
  return LINATTN_OK;
}

}  // namespace
}  // namespace linattn

using namespace linattn;

extern "C" {

const char* linattn_strerror(int status) {
  switch (status) {
    case LINATTN_OK: return "ok";
    case LINATTN_E_NULL: return "a required pointer is NULL";
    case LINATTN_E_SHAPE: return "unsupported or inconsistent shape (B,H,n >= 1; d in {64,128}; H,d as in the descriptor)";
    case LINATTN_E_DTYPE: return "unknown dtype";
    case LINATTN_E_ALIGN: return "tensor pointer is not 16-byte aligned (workspace: 256)";
    case LINATTN_E_PHI: return "unknown phi_id, unsupported feature-map kind, or descriptor table full";
    case LINATTN_E_WORKSPACE: return "workspace missing or smaller than linattn_workspace_bytes()";
    case LINATTN_E_HIP: return "a HIP launch failed";
    case LINATTN_E_STATE: return "linattn_bwd needs the descriptor's state buffer, or the state buffer is too small for this batch size";
    case LINATTN_E_ALIAS: return "an output aliases an input";
    default: return "unknown status";
  }
}

int linattn_set_stage_events(void* const* events) {
  std::lock_guard<std::mutex> lk(g_mu);
  g_stage_events_on = events != nullptr;
  if (events)
    for (int i = 0; i < 4; ++i) g_stage_events[i] = static_cast<hipEvent_t>(events[i]);
  return LINATTN_OK;
}

size_t linattn_workspace_bytes(int B, int H, int n, int d, int kind, int dtype) {
  if (kind != LINATTN_PHI_HEDGEHOG && kind != LINATTN_PHI_RELU) return 0;
  Plan p;
  if (!make_plan(B, H, n, d, dtype, LINATTN_LAYOUT_BHND, &p)) return 0;
  return p.bytes_no_wgrads;
}

size_t linattn_workspace_bytes_wgrads(int B, int H, int n, int d, int kind, int dtype) {
  if (kind == LINATTN_PHI_RELU) return linattn_workspace_bytes(B, H, n, d, kind, dtype);    // no weights
  if (kind != LINATTN_PHI_HEDGEHOG) return 0;
  Plan p;
  if (!make_plan(B, H, n, d, dtype, LINATTN_LAYOUT_BHND, &p)) return 0;
  return p.total_bytes;
}

int linattn_phi_create(const linattn_phi_desc* desc, int* phi_id_out) {
  if (!desc || !phi_id_out) return LINATTN_E_NULL;
  if (desc->kind != LINATTN_PHI_HEDGEHOG && desc->kind != LINATTN_PHI_RELU) return LINATTN_E_PHI;
  if (desc->dtype != LINATTN_BF16 && desc->dtype != LINATTN_F32 && desc->dtype != LINATTN_BF16_F32MATH) return LINATTN_E_DTYPE;
  if (desc->H <= 0 || (desc->d != 64 && desc->d != 128)) return LINATTN_E_SHAPE;
  if (desc->layout != LINATTN_LAYOUT_BHND && desc->layout != LINATTN_LAYOUT_BNHD) return LINATTN_E_SHAPE;
  if (desc->kind == LINATTN_PHI_RELU) {
    // weight-free: nothing to point at, and no mixed attention with this map
    if (desc->wq || desc->wk || desc->dwq || desc->dwk || desc->blend_in || desc->blend_r || desc->blend_dr) return LINATTN_E_PHI;
  } else {
    if (!desc->wq || !desc->wk) return LINATTN_E_NULL;
    if (!aligned16(desc->wq) || !aligned16(desc->wk)) return LINATTN_E_ALIGN;
    if (desc->dwq && !aligned16(desc->dwq)) return LINATTN_E_ALIGN;
    if (desc->dwk && !aligned16(desc->dwk)) return LINATTN_E_ALIGN;
  }
  if (desc->flags & ~LINATTN_FLAG_CENTRED) return LINATTN_E_PHI;
  if ((desc->flags & LINATTN_FLAG_CENTRED) && (desc->kind != LINATTN_PHI_HEDGEHOG || desc->dtype != LINATTN_BF16)) return LINATTN_E_PHI;
  if (desc->state && !aligned16(desc->state)) return LINATTN_E_ALIGN;
  if (desc->state && desc->state_bytes < (size_t)desc->H * (desc->d + 1) * desc->d * sizeof(float)) return LINATTN_E_STATE;
  if (desc->workspace && (reinterpret_cast<uintptr_t>(desc->workspace) & 255u)) return LINATTN_E_ALIGN;
  if (int st = check_blend(desc->blend_in, desc->blend_r, desc->blend_dr)) return st;
  std::lock_guard<std::mutex> lk(g_mu);
  for (int i = 0; i < kMaxDesc; ++i) {
    if (!g_slots[i].live) {
      g_slots[i].live = true;
      g_slots[i].d = *desc;
      *phi_id_out = kFirstId + i;
      return LINATTN_OK;
    }
  }
  return LINATTN_E_PHI;
}

int linattn_phi_set_blend(int phi_id, const void* blend_in, const float* blend_r, float* blend_dr) {
  if (int st = check_blend(blend_in, blend_r, blend_dr)) return st;
  std::lock_guard<std::mutex> lk(g_mu);
  const int i = phi_id - kFirstId;
  if (i < 0 || i >= kMaxDesc || !g_slots[i].live) return LINATTN_E_PHI;
  if (g_slots[i].d.kind == LINATTN_PHI_RELU && blend_in) return LINATTN_E_PHI;
  g_slots[i].d.blend_in = blend_in;
  g_slots[i].d.blend_r = blend_r;
  g_slots[i].d.blend_dr = blend_dr;
  return LINATTN_OK;
}

int linattn_phi_destroy(int phi_id) {
  std::lock_guard<std::mutex> lk(g_mu);
  const int i = phi_id - kFirstId;
  if (i < 0 || i >= kMaxDesc || !g_slots[i].live) return LINATTN_E_PHI;
  g_slots[i].live = false;
  return LINATTN_OK;
}

int linattn_fwd(const void* q, const void* k, const void* v, void* out,
                int B, int H, int n, int d, int phi_id, void* stream) {
  linattn_phi_desc desc;
  Plan plan;
  const int st = check_fwd(q, k, v, out, B, H, n, d, phi_id, false, &desc, &plan);
  if (st != LINATTN_OK) return st;
  return run_fwd(desc, plan, q, k, v, out, static_cast<char*>(desc.workspace), static_cast<hipStream_t>(stream));
}

int linattn_fwd_noalloc(const void* q, const void* k, const void* v, void* out,
                        int B, int H, int n, int d, int phi_id, void* stream) {
  linattn_phi_desc desc;
  Plan plan;
  int st = check_fwd(q, k, v, out, B, H, n, d, phi_id, true, &desc, &plan);
  if (st != LINATTN_OK) return st;
  if (plan.fwd_bytes > kStaticScratchBytes) return LINATTN_E_WORKSPACE;
  char* ws = nullptr;
  if ((st = static_scratch(&ws)) != LINATTN_OK) return st;
  return run_fwd(desc, plan, q, k, v, out, ws, static_cast<hipStream_t>(stream));
}

int linattn_bwd(const void* q, const void* k, const void* v, const void* dout,
                void* dq, void* dk, void* dv,
                int B, int H, int n, int d, int phi_id, void* stream) {
  linattn_phi_desc desc;
  Plan plan;
  const void* tensors[7] = {q, k, v, dout, dq, dk, dv};
  int st = check_call(tensors, 7, B, H, n, d, phi_id, true, &desc, &plan);
  if (st != LINATTN_OK) return st;
  if (!desc.state) return LINATTN_E_STATE;
  const size_t esz = desc.dtype == LINATTN_F32 ? 4 : 2;
  const size_t bytes = (size_t)plan.BH * n * d * esz;
  const void* ins[4] = {q, k, v, dout};
  void* outs[3] = {dq, dk, dv};
  for (int i = 0; i < 3; ++i) {
    for (int j = 0; j < 4; ++j)
      if (overlaps(outs[i], ins[j], bytes)) return LINATTN_E_ALIAS;
    for (int j = i + 1; j < 3; ++j)
      if (overlaps(outs[i], outs[j], bytes)) return LINATTN_E_ALIAS;
    if (desc.blend_in && overlaps(outs[i], desc.blend_in, bytes)) return LINATTN_E_ALIAS;
  }
  char* ws = static_cast<char*>(desc.workspace);
  BwdArgs a{};
  a.q = q; a.k = k; a.v = v; a.dout = dout; a.wq = desc.wq; a.wk = desc.wk;
  a.dq = dq; a.dk = dk; a.dv = dv;
  a.state = static_cast<const float*>(desc.state);
  a.dwq = static_cast<float*>(desc.dwq);
  a.dwk = static_cast<float*>(desc.dwk);
  a.partials = reinterpret_cast<float*>(ws + plan.off_partials);
  a.dstate = reinterpret_cast<float*>(ws + plan.off_dstate);
  a.gimg = ws + plan.off_gimg;
  a.simg = ws + plan.off_simg;
  a.dsimg = ws + plan.off_dsimg;
  a.dgimg = ws + plan.off_dgimg;
  a.wimg = ws + plan.off_wimg;
  a.scales = reinterpret_cast<float*>(ws + plan.off_scales);
  a.vbar = reinterpret_cast<float*>(ws + plan.off_centre);
  a.dv_row = a.vbar + (size_t)plan.BH * d;
  a.dzc = a.dv_row + (size_t)plan.BH * d;
  a.cs_part = a.dzc + (size_t)plan.BH * d;
  a.blend_in = desc.blend_in; a.blend_r = desc.blend_r; a.blend_dr = desc.blend_dr;
  a.dr_part = reinterpret_cast<float*>(ws + plan.off_drpart);
  a.dw_part = reinterpret_cast<float*>(ws + plan.off_dwpart);
  a.du_q = reinterpret_cast<float*>(ws + plan.off_du_q);
  a.du_k = reinterpret_cast<float*>(ws + plan.off_du_k);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (desc.kind == LINATTN_PHI_RELU) { a.dwq = nullptr; a.dwk = nullptr; }
  const hipError_t e = desc.dtype != LINATTN_BF16 ? launch_bwd_f32(a, plan, s)
                     : desc.kind == LINATTN_PHI_RELU ? launch_relu_bwd_bf16(a, plan, s) : launch_bwd_bf16(a, plan, s);
  return e == hipSuccess ? LINATTN_OK : LINATTN_E_HIP;
}

}  // extern "C"
