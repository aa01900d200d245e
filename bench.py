#!/usr/bin/env python3
"""Benchmark of the linear-attention forward path on one MI355X.

A step is one linattn_fwd call (state pass, reduction, query pass) over one batch of synthetic
Wan-14B/720p-shaped tensors (B=1, H=40, n=75600, d=128, bf16) already resident in HBM.
Prints one JSON line: whole-path tokens/s, the HBM roofline of the dominant kernel measured with
HIP events between the stages, and the CPU fp64 oracle timed on a bounded sample beside it.

`--pass bwd` times linattn_bwd instead (default workload: the config-5 training shape, with the
weight gradients unless --no-wgrads); its roofline object covers the whole call against the seven
compulsory tensor passes.  The headline metric is the forward one.
"""
from __future__ import annotations

import argparse
import ctypes
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published peak
MFMA_PEAK_TFLOPS = 2500.0      # dense bf16 / fp16 matrix-core peak
CONFIG_HEADS = {"C2": 12}
PREWARM_SECONDS = 0.25         # forward calls before --warmup, so that short runs do not time the clock ramp
# HBM bytes per launch (read + written) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# command with --calib-copy, scaled by the readings of the 1 GiB copy kernel (FETCH x2 KiB,
# WRITE x1 KiB); keyed by (workload, stage).  The committed summary with the commands is
# profiles/fwd_wan14b_720p_pmc.md.  None for workloads that have not been measured.
MEASURED_TRAFFIC = {("C3", 0): 1_553_370_522 + 19_021_824, ("C3", 2): 794_324_787 + 774_176_666}
# The same for one linattn_bwd call (all its kernels), weight gradients on: profiles/bwd_wan1p3b_480p_pmc.md.
MEASURED_TRAFFIC_BWD = {"C5": 560_400_000 + 338_100_000}


def _hip():
    lib = ctypes.CDLL("libamdhip64.so")
    lib.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
    lib.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
    lib.hipEventDestroy.argtypes = [ctypes.c_void_p]
    return lib


def streaming_rates(nbytes: int, stream: int, reps: int = 20):
    """What plain streaming kernels reach on this GPU, measured now: GB/s of a read-only kernel over
    nbytes and of a copy kernel (nbytes read + nbytes written), HIP events on `stream`.  Context for
    `frac`, which stays relative to the published peak."""
    import torch
    from paper_2510_08318_amd import build as B
    if not os.path.exists(B.PROBE_LIB):
        raise RuntimeError(f"{B.PROBE_LIB} is missing: run `python paper_2510_08318_amd/build.py`")
    lib = ctypes.CDLL(B.PROBE_LIB)
    lib.membw_probe.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int, ctypes.c_void_p]
    lib.membw_probe.restype = ctypes.c_int
    hip = _hip()
    nbytes -= nbytes % 16
    src = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    ev = [ctypes.c_void_p() for _ in range(2)]
    for e in ev:
        assert hip.hipEventCreate(ctypes.byref(e)) == 0
    hip.hipEventRecord.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    out = {}
    # each rate is the best of a few launch shapes
    for name, kind, moved in (("read_GBps", 0, nbytes), ("copy_GBps", 1, 2 * nbytes)):
        best = 0.0
        for groups in (256, 512, 2048, 8192):
            def run():
                rc = lib.membw_probe(kind, src.data_ptr(), dst.data_ptr(), nbytes, groups, stream)
                assert rc == 0, f"membw_probe: hip error {rc}"
            for _ in range(3):
                run()
            assert hip.hipEventRecord(ev[0], stream) == 0
            for _ in range(reps):
                run()
            assert hip.hipEventRecord(ev[1], stream) == 0
            torch.cuda.synchronize()
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), ev[0], ev[1]) == 0
            best = max(best, moved / (ms.value / reps * 1e-3) / 1e9)
        out[name] = round(best, 1)
    for e in ev:
        hip.hipEventDestroy(e)
    del src, dst
    return out


def cpu_baseline(x, budget_s: float = 12.0, relu: bool = False):
    """The oracle as it stands, on a bounded sample: whole heads of the same workload."""
    from oracle import linattn_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    done = 0
    t0 = time.perf_counter()
    for h in range(x.H):
        if relu:
            from oracle import relu_oracle as R
            R.relu_fwd(O.to_f64(x.q[0, h]), O.to_f64(x.k[0, h]), O.to_f64(x.v[0, h]))
        else:
            O.fwd(O.to_f64(x.q[0, h]), O.to_f64(x.k[0, h]), O.to_f64(x.v[0, h]), O.to_f64(x.wq[h]), O.to_f64(x.wk[h]))
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    head_tokens_per_s = done * x.n / dt
    res = {"value": head_tokens_per_s / x.H, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": f"{done} of {x.H} heads of batch item 0, all {x.n} tokens, fp64 numpy, {dt:.1f} s"}
    if not relu:
        res["single_thread"] = cpu_single_thread()
    return res


def cpu_single_thread():
    """Per-core figure: the oracle on one head of the Wan-1.3B 480p shape (config 2) with one BLAS thread."""
    from oracle import linattn_oracle as O
    from paper_2510_08318_amd import synth
    from threadpoolctl import threadpool_limits
    y = synth.generate("C2", H=1)
    args = [O.to_f64(t) for t in (y.q[0, 0], y.k[0, 0], y.v[0, 0], y.wq[0], y.wk[0])]
    with threadpool_limits(limits=1):
        t0 = time.perf_counter()
        O.fwd(*args)
        dt = time.perf_counter() - t0
    heads = CONFIG_HEADS["C2"]
    return {"value": round(y.n / dt / heads, 1), "unit": "tokens/s", "cores": 1,
            "sample": f"1 of {heads} heads of config 2 (n={y.n}, d={y.d}), {dt:.2f} s; tokens/s = n / (time x {heads} heads)"}


def cpu_baseline_bwd(x, budget_s: float = 12.0, relu: bool = False):
    """The oracle's backward (forward recomputed inside it), whole heads of the same workload."""
    from oracle import linattn_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    done = 0
    t0 = time.perf_counter()
    for h in range(x.H):
        if relu:
            from oracle import relu_oracle as R
            R.relu_bwd(O.to_f64(x.q[0, h]), O.to_f64(x.k[0, h]), O.to_f64(x.v[0, h]), O.to_f64(x.dout[0, h]))
        else:
            O.bwd(O.to_f64(x.q[0, h]), O.to_f64(x.k[0, h]), O.to_f64(x.v[0, h]), O.to_f64(x.wq[h]), O.to_f64(x.wk[h]),
                  O.to_f64(x.dout[0, h]))
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": done * x.n / dt / x.H, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{done} of {x.H} heads of batch item 0, all {x.n} tokens, fp64 numpy backward, {dt:.1f} s"}


def check_timed_output(x, sets, calls, lay, relu, args, blend_s):
    """Sampled rows of the buffer the last timed step wrote, against the oracle (Eq. 3 from the fp64
    state of the head): four heads, 1024 rows each plus the first and last 64.  Not part of the timing."""
    import numpy as np
    import torch
    from oracle import linattn_oracle as O
    from paper_2510_08318_amd import torch_glue as G
    out = sets[(calls - 1) % len(sets)][3]
    if args.layout == "bnhd":
        out = out.permute(0, 2, 1, 3)
    rng = np.random.default_rng(0)
    heads = sorted(set([(0, 0), (x.B - 1, x.H - 1), (0, x.H // 2), (x.B - 1, x.H // 3)]))
    worst = 0.0
    for b, h in heads:
        rows = np.unique(np.concatenate([rng.choice(x.n, min(1024, x.n), replace=False), np.arange(min(64, x.n)),
                                         np.arange(max(0, x.n - 64), x.n)])).astype(np.int64)
        kk, vv, qq = O.to_f64(x.k[b, h]), O.to_f64(x.v[b, h]), O.to_f64(x.q[b, h][rows])
        if relu:
            from oracle import relu_oracle as R
            S, z = R.relu_state(kk, vv)
            fq = R.phi_relu(qq)
            ref = (fq @ S) / ((fq @ z) + R.RELU_EPS)[:, None]
        else:
            S, z = O.state(kk, vv, O.to_f64(x.wk[h]))
            fq = O.phi(qq, O.to_f64(x.wq[h]))
            ref = (fq @ S) / (fq @ z)[:, None]
        idx = torch.from_numpy(rows).cuda()
        if blend_s is not None:
            sb = blend_s.permute(0, 2, 1, 3) if args.layout == "bnhd" else blend_s
            ref = 0.5 * G.to_host_f64(sb[b, h][idx]) + 0.5 * ref
        worst = max(worst, O.err_metric(G.to_host_f64(out[b, h][idx]), ref)[0])
    tol = 1e-2 if x.dtype == "bf16" else 1e-5
    return {"value": float(f"{worst:.3e}"), "tolerance": tol, "ok": bool(worst <= tol),
            "sample": f"{len(heads)} heads x ~1150 sampled rows of the last timed step's output vs the fp64 oracle, "
                      "max |diff| / max(|ref|, rms of the sampled rows of the head)"}


SECONDARY = (
    # label, workload, pass, options
    ("fwd C2 (Wan-1.3B 480p)", "C2", "fwd", {}),
    ("fwd C4 (CFG batch, B=2)", "C4", "fwd", {}),
    ("fwd C6 (CogVideoX-2B shape)", "C6", "fwd", {}),
    ("fwd C3 [B,n,H,d] layout", "C3", "fwd", {"layout": "bnhd"}),
    ("fwd C3 mixed attention (Eq. 6)", "C3", "fwd", {"blend": True}),
    ("fwd C3 ReLU map", "C3", "fwd", {"relu": True}),
    ("bwd C5 with weight gradients", "C5", "bwd", {}),
    ("bwd C5 without weight gradients", "C5", "bwd", {"wgrads": False}),
    ("bwd C5 ReLU map", "C5", "bwd", {"relu": True}),
    ("bwd C3 shape with weight gradients", "C3", "bwd", {}),
    ("fwd C3 with LINATTN_FLAG_CENTRED", "C3", "fwd", {"centred": True}),
    ("bwd C5 with weight gradients and LINATTN_FLAG_CENTRED", "C5", "bwd", {"centred": True}),
    ("fwd C2, bf16 tensors with fp32 arithmetic (LINATTN_BF16_F32MATH)", "C2", "fwd", {"f32math": True, "steps": 20}),
    ("bwd C5, bf16 tensors with fp32 arithmetic (LINATTN_BF16_F32MATH)", "C5", "bwd", {"f32math": True, "steps": 10}),
)


def quick_time(workload, which, *, layout="bhnd", blend=False, relu=False, wgrads=True, f32math=False, centred=False, steps=200):
    """One secondary workload, timed like the headline one (pre-warm, then `steps` calls by the wall
    clock, inputs resident in HBM, buffer sets rotated below the cache scale)."""
    import torch
    from paper_2510_08318_amd import binding as L, synth, torch_glue as G
    x = synth.generate(workload, with_dout=(which == "bwd"))
    names = ("q", "k", "v") + (("dout",) if which == "bwd" else ())
    t = {nm: G.to_device(getattr(x, nm)) for nm in names}
    if layout == "bnhd":
        t = {nm: a.permute(0, 2, 1, 3).contiguous() for nm, a in t.items()}
    wq, wk = G.to_device(x.wq), G.to_device(x.wk)
    if relu:
        lay = G.ReluLayer(x.H, x.d, x.B, x.n, t["q"].dtype, layout=layout, f32_math=f32math)
    else:
        lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=(which == "bwd" and wgrads), layout=layout, f32_math=f32math, centred=centred)
    if blend:
        lay.set_blend((torch.randn(t["q"].shape, device="cuda") * 0.1).to(t["q"].dtype), torch.tensor([0.5], device="cuda"))
    outs = ("out",) if which == "fwd" else ("dq", "dk", "dv")
    ntens = len(names) + len(outs) + (1 if blend else 0)
    set_bytes = ntens * t["q"].numel() * t["q"].element_size()
    nsets = 1 if set_bytes >= 1_000_000_000 or which == "bwd" else min(16, max(3, -(-1_500_000_000 // set_bytes)))
    sets = []
    for i in range(nsets):
        ins = [t[nm] if i == 0 else t[nm].clone() for nm in names]
        sets.append(ins + [torch.empty_like(t["q"]) for _ in outs])
    stream = torch.cuda.current_stream().cuda_stream
    calls = [0]
    if which == "bwd":
        lay.forward(t["q"], t["k"], t["v"])          # the state the backward needs

    def step():
        a = sets[calls[0] % nsets]
        calls[0] += 1
        if which == "fwd":
            L.linattn_fwd(a[0], a[1], a[2], a[3], x.B, x.H, x.n, x.d, lay.phi_id, stream)
        else:
            L.linattn_bwd(a[0], a[1], a[2], a[3], a[4], a[5], a[6], x.B, x.H, x.n, x.d, lay.phi_id, stream)

    t0 = time.perf_counter()
    while time.perf_counter() - t0 < PREWARM_SECONDS:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    lay.close()
    esz = 2 if x.dtype == "bf16" else 4
    # forward: read K, V, Q (and the softmax-branch tensor when blending), write out; backward: read q, k, v, dO, write dq, dk, dv
    algo = ((5 if blend else 4) if which == "fwd" else 7) * x.d * esz * x.B * x.H * x.n
    return {"ms_per_step": round(dt * 1e3, 4), "tokens_per_s": round(x.B * x.n / dt, 1),
            "path_frac": round(algo / dt / 1e9 / HBM_PEAK_GBS, 4), "buffer_sets": nsets, "steps": steps}


def secondary_measurements():
    """The other workloads of the benchmark spec, timed in this same process after the headline measurement
    (context for the one JSON line; none of them is `value`)."""
    import gc
    import torch
    res = {}
    for label, workload, which, opt in SECONDARY:
        try:
            res[label] = quick_time(workload, which, **opt)
        except Exception as exc:                     # context only: report and go on
            res[label] = {"error": f"{type(exc).__name__}: {exc}"}
        gc.collect()
        torch.cuda.empty_cache()
    return res


def _calib_copy():
    """One 1 GiB device-to-device copy: the reference reading for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE."""
    import torch
    src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)                      # reads 1 GiB, writes 1 GiB
    torch.cuda.synchronize()
    del src, dst


def bench_bwd(args):
    """linattn_bwd on one batch (state from one forward call made before the timed region)."""
    import torch
    from paper_2510_08318_amd import synth, torch_glue as G
    x = synth.generate(args.workload, with_dout=True)
    q, k, v, wq, wk, dout = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    if args.layout == "bnhd":
        q, k, v, dout = [t.permute(0, 2, 1, 3).contiguous() for t in (q, k, v, dout)]
    relu = args.phi == "relu"
    if relu:
        lay = G.ReluLayer(x.H, x.d, x.B, x.n, q.dtype, layout=args.layout)
    else:
        lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=not args.no_wgrads, layout=args.layout)
    if args.blend:
        lay.set_blend((torch.randn(q.shape, device="cuda") * 0.1).to(q.dtype), torch.tensor([0.5], device="cuda"),
                      torch.zeros(1, device="cuda"))
    lay.forward(q, k, v)
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)

    def step():
        lay.backward(q, k, v, dout, dq, dk, dv)

    t0 = time.perf_counter()
    prewarm_calls = 0
    while time.perf_counter() - t0 < PREWARM_SECONDS:      # as in the forward benchmark
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        prewarm_calls += 8
    prewarm_s = time.perf_counter() - t0
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps
    esz = 2 if x.dtype == "bf16" else 4
    head_tokens = x.B * x.H * x.n
    algo = 7 * x.d * esz * head_tokens          # read q, k, v, dO; write dq, dk, dv
    achieved = algo / dt / 1e9
    res = {
        "metric": f"linear-attn bwd tokens/s ({args.workload})", "value": round(x.B * x.n / dt, 1), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": x.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={x.B} H={x.H} n={x.n} d={x.d} {x.dtype}, "
                               + ("backward of Eq. 3 with the ReLU map, state saved by the forward" if relu else
                                  f"backward of Eq. 3 + Eq. 5, state saved by the forward, weight gradients {'off' if args.no_wgrads else 'on'}")
                               + (", [B,n,H,d] layout" if args.layout == "bnhd" else "")
                               + (", mixed attention (Eq. 6, r = 0.5) with dL/dr" if args.blend else "")},
        "roofline": {"bound": "hbm", "kernel": "linattn_bwd (all kernels of one call)", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": None if (relu or args.blend or args.no_wgrads or args.layout != "bhnd")
                                else MEASURED_TRAFFIC_BWD.get(args.workload)},
        "prewarm": {"seconds": round(prewarm_s, 3), "calls": prewarm_calls},
    }
    if args.calib_copy:
        _calib_copy()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline_bwd(x, relu=relu)
    lay.close()
    print(json.dumps(res), flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default=None, help="configuration name in paper_2510_08318_amd.synth (default C3; C5 for --pass bwd)")
    ap.add_argument("--pass", dest="which", choices=("fwd", "bwd"), default="fwd")
    ap.add_argument("--no-wgrads", action="store_true", help="--pass bwd: skip the weight gradients")
    ap.add_argument("--blend", action="store_true",
                    help="mixed attention of Eq. 6: also read a softmax-branch tensor s and blend it with r = 0.5")
    ap.add_argument("--layout", choices=("bhnd", "bnhd"), default="bhnd",
                    help="memory layout of q, k, v, out: [B,H,n,d] (default, the headline configuration) or [B,n,H,d]")
    ap.add_argument("--phi", choices=("hedgehog", "relu"), default="hedgehog",
                    help="feature map: Eq. 5 (default, the headline configuration) or the weight-free max(x, 0) of the kernel-function ablation")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-secondary", action="store_true",
                    help="skip the secondary workloads (other configurations, layouts, maps and the backward) timed after the headline one; --no-cpu-baseline and --calib-copy skip them as well")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy kernel (reference reading for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU (one MI355X); --gpus must be 1")

    import torch
    from paper_2510_08318_amd import binding as L, synth, torch_glue as G
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.workload is None:
        args.workload = "C5" if args.which == "bwd" else "C3"
    if args.which == "bwd":
        return bench_bwd(args)

    x = synth.generate(args.workload)
    q, k, v, wq, wk = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk)]
    if args.layout == "bnhd":
        q, k, v = [t.permute(0, 2, 1, 3).contiguous() for t in (q, k, v)]
    relu = args.phi == "relu"
    lay = G.ReluLayer(x.H, x.d, x.B, x.n, q.dtype, layout=args.layout) if relu else G.Layer(wq, wk, x.B, x.n, layout=args.layout)
    blend_s = None
    if args.blend:
        blend_s = (torch.randn(q.shape, device="cuda") * 0.1).to(q.dtype)
        lay.set_blend(blend_s, torch.tensor([0.5], device="cuda"))
    out = torch.empty_like(q)
    stream = torch.cuda.current_stream().cuda_stream
    # A buffer set below the last-level cache scale (256 MB) would be served from cache on the next
    # step: such workloads rotate over several distinct sets (copies of the same values), so that a
    # step never re-reads what the previous steps left behind.  Set 0 is the one that is checked.
    set_bytes = 4 * q.numel() * q.element_size()
    nsets = 1 if set_bytes >= 1_000_000_000 else min(16, max(3, -(-1_500_000_000 // set_bytes)))
    sets = [(q, k, v, out)] + [tuple(t.clone() for t in (q, k, v, out)) for _ in range(nsets - 1)]
    calls = [0]

    def step():
        a, b_, c, o = sets[calls[0] % nsets]
        calls[0] += 1
        L.linattn_fwd(a, b_, c, o, x.B, x.H, x.n, x.d, lay.phi_id, stream)

    # pre-warm: a fixed, reported phase of forward calls (clocks ramp over the first ~0.2 s)
    t0 = time.perf_counter()
    prewarm_calls = 0
    while time.perf_counter() - t0 < PREWARM_SECONDS:
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        prewarm_calls += 8
    prewarm_s = time.perf_counter() - t0
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    tokens_per_s = x.B * x.n / (dt / args.steps)

    # per-stage durations: the same K steps again, right away (the clocks are still up), with HIP events
    # between the stages
    hip = _hip()
    evs = []
    for _ in range(args.steps):
        four = []
        for _ in range(4):
            e = ctypes.c_void_p()
            assert hip.hipEventCreate(ctypes.byref(e)) == 0
            four.append(e.value)
        evs.append(four)
    for four in evs:
        L.linattn_set_stage_events(four)
        step()
    L.linattn_set_stage_events(None)
    torch.cuda.synchronize()
    stage_ms = [0.0, 0.0, 0.0]
    per_call = []
    for four in evs:
        tot = 0.0
        for i in range(3):
            ms = ctypes.c_float()
            assert hip.hipEventElapsedTime(ctypes.byref(ms), four[i], four[i + 1]) == 0
            stage_ms[i] += ms.value / args.steps
            tot += ms.value
        per_call.append(tot)
    per_call.sort()
    for four in evs:
        for e in four:
            hip.hipEventDestroy(e)
    # every step writes the same values (the path is deterministic), so the buffer the last call wrote is
    # what the timed steps wrote
    max_err = None if args.no_cpu_baseline else check_timed_output(x, sets, calls[0], lay, relu, args, blend_s)

    esz = 2 if x.dtype == "bf16" else 4
    head_tokens = x.B * x.H * x.n
    # read K, V | - | read Q (and the softmax-branch tensor of Eq. 6 when blending), write out
    stage_bytes = [2 * x.d * esz * head_tokens, 0, (3 if args.blend else 2) * x.d * esz * head_tokens]
    names = ["state_partials (phi(K)^T V, split-n)", "state_reduce", "apply (phi(Q) S / phi(Q).z)"]
    dom = 0 if stage_ms[0] >= stage_ms[2] else 2
    achieved = stage_bytes[dom] / (stage_ms[dom] * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": names[dom], "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": None if (relu or args.blend or args.layout != "bhnd") else MEASURED_TRAFFIC.get((args.workload, dom)),
                "stage_ms": [round(t, 4) for t in stage_ms],
                "path_GBps": round(sum(stage_bytes) / (sum(stage_ms) * 1e-3) / 1e9, 1),
                "path_frac": round(sum(stage_bytes) / (sum(stage_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                # one call = first to last stage event; distribution over the K event-bracketed calls
                "call_ms_median": round(per_call[len(per_call) // 2], 4), "call_ms_min": round(per_call[0], 4)}
    if x.dtype == "bf16":
        # matrix-core use, reported beside the HBM bound: each pass issues 56 v_mfma_f32_32x32x16 (32768 FLOP
        # each) per 32 head-tokens -- state pass 16 projection + 8 turning + 32 contraction, query pass
        # 16 + 40; the ReLU map 32 + 8 and 40 -- which SQ_INSTS_MFMA confirms (profiles/fwd_wan14b_720p_pmc.md)
        blocks = x.B * x.H * -(-x.n // 32)
        per_block = ([40, 0, 40] if relu else [56, 0, 56]) if x.d == 128 else (None if relu else [16, 0, 16])
        if per_block:
            tf = [per_block[i] * blocks * 32768 / (stage_ms[i] * 1e-3) / 1e12 if stage_ms[i] > 0 else 0.0 for i in (0, 2)]
            roofline["mfma"] = {"state_pass_TFLOPs": round(tf[0], 1), "query_pass_TFLOPs": round(tf[1], 1),
                                "peak_TFLOPs": MFMA_PEAK_TFLOPS, "state_pass_frac": round(tf[0] / MFMA_PEAK_TFLOPS, 4),
                                "query_pass_frac": round(tf[1] / MFMA_PEAK_TFLOPS, 4),
                                "source": "MFMA instructions per 32-token block x blocks x 32768 FLOP / stage duration (HIP events)"}

    # the same bytes through plain streaming kernels, measured now (the state pass only reads, the
    # query pass reads and writes the same amount)
    try:
        rates = streaming_rates(stage_bytes[0], stream)
        floor_ms = stage_bytes[0] / rates["read_GBps"] / 1e6 + stage_bytes[2] / rates["copy_GBps"] / 1e6
        roofline["streaming"] = {**rates, "path_ms_at_streaming_rates": round(floor_ms, 4),
                                 "path_frac_of_streaming": round(floor_ms / sum(stage_ms), 4)}
    except (RuntimeError, OSError) as exc:        # the probe is context, not the product: report and go on
        print(f"bench.py: streaming-rate probe skipped: {exc}", file=sys.stderr)
        roofline["streaming"] = None

    res = {
        "metric": "linear-attn fwd tokens/s (Wan-14B 720p shape)" if args.workload == "C3" and not relu
                  else f"linear-attn fwd tokens/s ({args.workload}{', ReLU map' if relu else ''})",
        "value": round(tokens_per_s, 1), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": x.dtype, "data": "synthetic",
        "config": {"workload": f"{args.workload}: B={x.B} H={x.H} n={x.n} d={x.d} {x.dtype}, {'ReLU' if relu else 'Hedgehog'} phi, non-causal"
                               + (", [B,n,H,d] layout" if args.layout == "bnhd" else "")
                               + (", mixed with a softmax-branch input (Eq. 6, r = 0.5)" if args.blend else ""),
                   "head_tokens_per_s": round(tokens_per_s * x.H, 1)},
        "roofline": roofline,
        "prewarm": {"seconds": round(prewarm_s, 3), "calls": prewarm_calls,
                    "note": "untimed forward calls before --warmup; steps and warmup echo the arguments"},
        "buffer_sets": nsets,
        "max_err": max_err,
    }
    if args.calib_copy:
        _calib_copy()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(x, relu=relu)
    lay.close()
    headline = args.workload == "C3" and not relu and not args.blend and args.layout == "bhnd"
    if headline and not (args.no_secondary or args.no_cpu_baseline or args.calib_copy):
        del sets, q, k, v, out
        torch.cuda.empty_cache()
        res["secondary"] = secondary_measurements()
    print(json.dumps(res), flush=True)


if __name__ == "__main__":
    main()
