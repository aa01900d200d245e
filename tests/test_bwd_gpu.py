"""Parity of the HIP backward path with the CPU fp64 oracle, through the C ABI.

dq, dk, dv are compared element by element with the RMS-floored relative error (1e-2 for bf16
tensors, 1e-5 for fp32); the weight gradients dW~_q, dW~_k (fp32 outputs) with the same metric.
"""
import numpy as np
import pytest

from oracle import linattn_oracle as O
from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}
WTOL = {"f32": 2e-5, "bf16": 1e-2}


def _gpu_fwd_bwd(x, want_wgrads=True):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    q, k, v, wq, wk, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=want_wgrads)
    lay.forward(q, k, v)
    dq, dk, dv = lay.backward(q, k, v, do)
    torch.cuda.synchronize()
    res = [G.to_host_f64(t) for t in (dq, dk, dv)]
    if want_wgrads:
        res += [G.to_host_f64(lay.dwq), G.to_host_f64(lay.dwk)]
    lay.close()
    return res


def _check(x, want_wgrads=True):
    got = _gpu_fwd_bwd(x, want_wgrads)
    ref = O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)
    names = ["dq", "dk", "dv", "dwq", "dwk"]
    errs = {}
    dv_scale = np.abs(ref[2]).max()
    for i, g in enumerate(got):
        assert np.isfinite(g).all(), names[i]
        if np.sqrt(np.mean(ref[i] ** 2)) < 1e-6 * dv_scale:
            # a gradient that is identically zero (n = 1: the output is v whatever q and k are):
            # relative error is undefined, compare against the size of the non-zero gradients
            errs[names[i]] = np.abs(g - ref[i]).max() / dv_scale
        else:
            errs[names[i]] = O.err_metric(g, ref[i])[0]
    for name, e in errs.items():
        tol = WTOL[x.dtype] if name.startswith("dw") else TOL[x.dtype]
        assert e <= tol, errs
    return errs


@pytest.mark.parametrize("n,d,H,B", [(1, 64, 1, 1), (17, 64, 2, 1), (33, 128, 1, 2), (100, 128, 3, 1), (515, 64, 2, 2)])
def test_fp32_backward(n, d, H, B):
    _check(synth.generate("C1", n=n, d=d, H=H, B=B, with_dout=True))


def test_config1_fp32_backward_full():
    _check(synth.generate("C1", with_dout=True))


@pytest.mark.parametrize("n", [1, 2, 31, 33, 127, 128, 129, 300, 1000, 4133])
def test_bf16_backward_ragged_lengths(n):
    _check(synth.generate("C5", n=n, H=2))


@pytest.mark.parametrize("name,n,H,B,d", [
    ("C5", 777, 2, 1, 64),
    ("C5", 2049, 3, 2, 64),
    ("C5", 6000, 13, 1, 128),
    ("C5", 20000, 2, 2, 128),
])
def test_bf16_backward_shapes(name, n, H, B, d):
    _check(synth.generate(name, n=n, H=H, B=B, d=d))


def test_backward_without_weight_grads_and_small_dout():
    # gradients are linear in dO: a 2^-20 smaller dO must give 2^-20 smaller gradients (the
    # per-token and per-workgroup power-of-two scalings make this exact up to underflow)
    x = synth.generate("C5", n=1500, H=2)
    a = _gpu_fwd_bwd(x, want_wgrads=False)
    y = synth.generate("C5", n=1500, H=2)
    d32 = synth.bf16_bits_to_f32(y.dout) * np.float32(2.0 ** -20)
    y.dout = synth.f32_to_bf16_bits(d32)
    b = _gpu_fwd_bwd(y, want_wgrads=False)
    for u, w in zip(a, b):
        np.testing.assert_allclose(w * 2.0 ** 20, u, rtol=0, atol=1e-3 * np.abs(u).max())
    ref = O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)
    for u, r in zip(a, ref[:3]):
        assert O.err_metric(u, r)[0] <= 1e-2


@pytest.mark.parametrize("cfg,n,d", [("C5", 1000, 128), ("C5", 333, 64), ("C1", 300, 64)])
@pytest.mark.parametrize("side", ["q", "k"])
def test_one_weight_gradient_only(cfg, n, d, side):
    """dwq or dwk alone may be requested: the one asked for matches the oracle, dq, dk, dv are unchanged."""
    import torch
    from paper_2510_08318_amd import torch_glue as G
    x = synth.generate(cfg, n=n, d=d, H=2, B=2, with_dout=True)
    q, k, v, wq, wk, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=side)
    lay.forward(q, k, v)
    grads = lay.backward(q, k, v, do)
    torch.cuda.synchronize()
    got = [G.to_host_f64(t) for t in grads] + [G.to_host_f64(lay.dwq if side == "q" else lay.dwk)]
    assert (lay.dwk if side == "q" else lay.dwq) is None
    lay.close()
    ref = O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)
    ref = list(ref[:3]) + [ref[3] if side == "q" else ref[4]]
    for name, g, r in zip(["dq", "dk", "dv", "dw"], got, ref):
        tol = WTOL[x.dtype] if name == "dw" else TOL[x.dtype]
        assert O.err_metric(g, r)[0] <= tol, (name, side)


def test_one_descriptor_serves_smaller_calls():
    """A descriptor whose workspace and state were sized for (B=2, n=1000) also serves a (B=1, n=300) call,
    between two full-size calls: every call is planned from its own arguments."""
    import torch
    from paper_2510_08318_amd import binding as L, torch_glue as G
    big = synth.generate("C5", n=1000, H=2, B=2)
    small = synth.generate("C5", n=300, H=2, B=1)
    small.wq, small.wk = big.wq, big.wk                  # the layer's maps
    wq, wk = G.to_device(big.wq), G.to_device(big.wk)
    lay = G.Layer(wq, wk, big.B, big.n, want_wgrads=True)
    stream = torch.cuda.current_stream().cuda_stream
    for x in (big, small, big):
        q, k, v, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.dout)]
        out, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
        L.linattn_fwd(q, k, v, out, x.B, x.H, x.n, x.d, lay.phi_id, stream)
        L.linattn_bwd(q, k, v, do, dq, dk, dv, x.B, x.H, x.n, x.d, lay.phi_id, stream)
        torch.cuda.synchronize()
        got = [G.to_host_f64(t) for t in (out, dq, dk, dv, lay.dwq, lay.dwk)]
        ref = [O.fwd_bh(x.q, x.k, x.v, x.wq, x.wk)] + list(O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout))
        for name, g, r in zip(["out", "dq", "dk", "dv", "dwq", "dwk"], got, ref):
            assert O.err_metric(g, r)[0] <= 1e-2, (name, x.B, x.n)
    lay.close()


def test_two_layers_on_two_streams():
    """Two descriptors, each with its own workspace, driven from two streams at once (default priority):
    calls share no state, so both results are those of the oracle."""
    import torch
    from paper_2510_08318_amd import binding as L, torch_glue as G
    xs = [synth.generate("C5", n=3000, H=3, B=1), synth.generate("C5", n=2049, H=2, B=2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    work = []
    for x in xs:
        q, k, v, do, wq, wk = [G.to_device(t) for t in (x.q, x.k, x.v, x.dout, x.wq, x.wk)]
        lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=True)
        outs = [torch.empty_like(q) for _ in range(4)]
        work.append((x, lay, (q, k, v, do), outs))
    torch.cuda.synchronize()
    for _ in range(4):
        for (x, lay, (q, k, v, do), (out, dq, dk, dv)), st in zip(work, streams):
            L.linattn_fwd(q, k, v, out, x.B, x.H, x.n, x.d, lay.phi_id, st.cuda_stream)
            L.linattn_bwd(q, k, v, do, dq, dk, dv, x.B, x.H, x.n, x.d, lay.phi_id, st.cuda_stream)
    for st in streams:
        st.synchronize()
    for x, lay, _, (out, dq, dk, dv) in work:
        got = [G.to_host_f64(t) for t in (out, dq, dk, dv, lay.dwq, lay.dwk)]
        ref = [O.fwd_bh(x.q, x.k, x.v, x.wq, x.wk)] + list(O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout))
        for name, g, r in zip(["out", "dq", "dk", "dv", "dwq", "dwk"], got, ref):
            assert O.err_metric(g, r)[0] <= 1e-2, (name, x.n)
        lay.close()


def test_backward_bitwise_deterministic():
    import torch
    from paper_2510_08318_amd import torch_glue as G
    x = synth.generate("C5", n=5000, H=3)
    q, k, v, wq, wk, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=True)
    lay.forward(q, k, v)
    first = [t.clone() for t in lay.backward(q, k, v, do)] + [lay.dwq.clone(), lay.dwk.clone()]
    for _ in range(2):
        again = list(lay.backward(q, k, v, do)) + [lay.dwq, lay.dwk]
        torch.cuda.synchronize()
        for a, b in zip(first, again):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b)
    lay.close()


def test_backward_closed_forms_on_device():
    # the attention weights of each query sum to one: sum_j dv_j = sum_i dO_i
    x = synth.generate("C5", n=3000, H=2)
    dq, dk, dv = _gpu_fwd_bwd(x, want_wgrads=False)
    do = synth.bf16_bits_to_f32(x.dout).astype(np.float64)
    lhs, rhs = dv.sum(axis=2), do.sum(axis=2)
    assert np.abs(lhs - rhs).max() <= 2e-2 * np.abs(rhs).max()
    # constant v: the output does not depend on q or k, so dq = dk = 0 (up to rounding noise
    # far below the size of the gradients of the unconstrained problem)
    # (the constant row has the spread of the random v, so the rounding noise is comparable)
    c = synth.generate("C5", n=3000, H=2)
    amp = float(np.sqrt(3.0) * synth.bf16_bits_to_f32(x.v).std())
    c.v[:] = synth.f32_to_bf16_bits(np.linspace(-amp, amp, 128, dtype=np.float32))
    dq0, dk0, _ = _gpu_fwd_bwd(c, want_wgrads=False)
    assert np.abs(dq0).max() <= 2e-2 * np.abs(dq).max()
    assert np.abs(dk0).max() <= 2e-2 * np.abs(dk).max()
