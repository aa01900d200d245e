"""Parity of the HIP path with the ReLU feature map (LINATTN_PHI_RELU) against the CPU fp64 oracle,
through the C ABI: forward, exported state and backward, fp32 (1e-5) and bf16 (1e-2), both layouts.

The inputs are the q, k, v, dout of the usual synthetic configs; the learnable maps are not used.
"""
import numpy as np
import pytest

from oracle import linattn_oracle as O
from oracle import relu_oracle as R
from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}


def _run(x, layout="bhnd", backward=True):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    ts = [G.to_device(t) for t in ((x.q, x.k, x.v, x.dout) if backward else (x.q, x.k, x.v))]
    if layout == "bnhd":
        ts = [t.permute(0, 2, 1, 3).contiguous() for t in ts]
    lay = G.ReluLayer(x.H, x.d, x.B, x.n, ts[0].dtype, layout=layout)
    out = lay.forward(*ts[:3])
    res = [out]
    if backward:
        res += list(lay.backward(*ts))
    torch.cuda.synchronize()
    state = G.to_host_f64(lay.state)
    if layout == "bnhd":
        res = [t.permute(0, 2, 1, 3) for t in res]
    res = [G.to_host_f64(t) for t in res]
    lay.close()
    return res, state


def _check(x, layout="bhnd", backward=True):
    got, state = _run(x, layout, backward)
    ref = [R.relu_fwd_bh(x.q, x.k, x.v)]
    if backward:
        ref += list(R.relu_bwd_bh(x.q, x.k, x.v, x.dout))
    names = ["out", "dq", "dk", "dv"]
    errs = {}
    scale = max(np.abs(r).max() for r in ref[1:]) if backward else 1.0
    for i, g in enumerate(got):
        assert np.isfinite(g).all(), names[i]
        if i > 0 and np.sqrt(np.mean(ref[i] ** 2)) < 1e-6 * scale:
            errs[names[i]] = np.abs(g - ref[i]).max() / scale       # identically zero gradient (n = 1)
        else:
            errs[names[i]] = O.err_metric(g, ref[i])[0]
    st_ref = R.relu_state_bh(x.k, x.v)
    errs["state"] = O.err_metric(state, st_ref)[0]
    for name, e in errs.items():
        assert e <= (1e-5 if name == "state" and x.dtype == "f32" else TOL[x.dtype]), errs
    return errs


@pytest.mark.parametrize("n,d,H,B", [(1, 64, 1, 1), (17, 64, 2, 1), (33, 128, 1, 2), (100, 128, 3, 1), (515, 64, 2, 2)])
def test_fp32(n, d, H, B):
    _check(synth.generate("C1", n=n, d=d, H=H, B=B, with_dout=True))


@pytest.mark.parametrize("n", [1, 2, 31, 33, 127, 128, 129, 300, 1000, 4133])
def test_bf16_ragged_lengths(n):
    _check(synth.generate("C5", n=n, H=2))


@pytest.mark.parametrize("n,H,B,d", [(777, 2, 1, 64), (2049, 3, 2, 64), (6000, 13, 1, 128), (20000, 2, 2, 128)])
def test_bf16_shapes(n, H, B, d):
    _check(synth.generate("C5", n=n, H=H, B=B, d=d))


@pytest.mark.parametrize("dtype_cfg,n,d", [("C1", 300, 64), ("C5", 1000, 128), ("C5", 333, 64)])
def test_heads_interleaved_layout(dtype_cfg, n, d):
    _check(synth.generate(dtype_cfg, n=n, d=d, H=3, B=2, with_dout=True), layout="bnhd")


def test_dead_rows_and_small_dout():
    # a query and a key with no positive entry: out = 0 for that query, dq = 0, dk = 0 for that key;
    # gradients are linear in dO, so a 2^-20 smaller dO gives 2^-20 smaller gradients
    x = synth.generate("C5", n=700, H=2)
    neg = lambda a: (a | np.uint16(0x8000))              # bf16 sign bit
    x.q[0, 1, 5] = neg(x.q[0, 1, 5])
    x.k[0, 0, 9] = neg(x.k[0, 0, 9])
    errs = _check(x)
    got, _ = _run(x)
    assert not got[0][0, 1, 5].any() and not got[1][0, 1, 5].any() and not got[2][0, 0, 9].any()
    import copy
    y = copy.copy(x)
    f = O.to_f64(x.dout) * 2.0 ** -20
    y.dout = (f.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)     # exact: a power of two
    got_small, _ = _run(y)
    for a, b in zip(got[1:], got_small[1:]):
        assert O.err_metric(b * 2.0 ** 20, a)[0] <= 2e-2


def test_deterministic():
    x = synth.generate("C5", n=3000, H=3)
    a, sa = _run(x)
    b, sb = _run(x)
    for u, w in zip(a, b):
        assert np.array_equal(u, w)
    assert np.array_equal(sa, sb)


def test_premapped_nonnegative_features_reduce_to_textbook_gemms():
    """q, k that already are non-negative features pass through max(x, 0) unchanged, so the path must
    return plain kernel attention: (q k^T) v divided by the row sums of q k^T, written here with
    numpy matmuls only (no oracle code), fp32 and bf16."""
    for cfg, n, d, tol in (("C1", 300, 64, 1e-5), ("C5", 1000, 128, 1e-2)):
        x = synth.generate(cfg, n=n, d=d, H=2, B=1, with_dout=True)
        if x.dtype == "bf16":
            x.q = x.q & np.uint16(0x7FFF)                    # clear the sign bit: |q|, |k|
            x.k = x.k & np.uint16(0x7FFF)
        else:
            x.q, x.k = np.abs(x.q), np.abs(x.k)
        got, _ = _run(x, backward=False)
        q, k, v = (O.to_f64(t) for t in (x.q, x.k, x.v))
        for h in range(x.H):
            w = q[0, h] @ k[0, h].T
            ref = (w @ v[0, h]) / (w.sum(-1, keepdims=True) + 1e-6)
            assert O.err_metric(got[0][0, h], ref)[0] <= tol
