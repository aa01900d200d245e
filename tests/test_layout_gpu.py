"""The [B, n, H, d] layout (heads interleaved per token) through the C ABI: same numbers as the
oracle computes for the [B, H, n, d] tensors, forward and backward, both dtypes.

The oracle is layout-free (it works per head); the test hands the library the transposed
tensors and transposes the results back.
"""
import numpy as np
import pytest

from oracle import linattn_oracle as O
from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 1e-2}
WTOL = {"f32": 2e-5, "bf16": 1e-2}


def _bnhd(a):
    return np.ascontiguousarray(np.transpose(a, (0, 2, 1, 3)))


def _run(x, backward):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    q, k, v = [G.to_device(_bnhd(t)) for t in (x.q, x.k, x.v)]
    wq, wk = G.to_device(x.wq), G.to_device(x.wk)
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=backward, layout="bnhd")
    out = lay.forward(q, k, v)
    res = {"out": np.transpose(G.to_host_f64(out), (0, 2, 1, 3)), "state": G.to_host_f64(lay.state)}
    if backward:
        dq, dk, dv = lay.backward(q, k, v, G.to_device(_bnhd(x.dout)))
        torch.cuda.synchronize()
        for name, t in (("dq", dq), ("dk", dk), ("dv", dv)):
            res[name] = np.transpose(G.to_host_f64(t), (0, 2, 1, 3))
        res["dwq"], res["dwk"] = G.to_host_f64(lay.dwq), G.to_host_f64(lay.dwk)
    torch.cuda.synchronize()
    lay.close()
    return res


def _check(x, backward):
    got = _run(x, backward)
    ref_out = O.fwd_bh(x.q, x.k, x.v, x.wq, x.wk)
    assert np.isfinite(got["out"]).all()
    assert O.err_metric(got["out"], ref_out)[0] <= TOL[x.dtype]
    st_ref = O.state_bh(x.k, x.v, x.wk)
    assert np.abs(got["state"] - st_ref).max() / np.abs(st_ref).max() <= 2e-3
    if backward:
        ref = dict(zip(("dq", "dk", "dv", "dwq", "dwk"), O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)))
        for name, r in ref.items():
            tol = WTOL[x.dtype] if name.startswith("dw") else TOL[x.dtype]
            assert O.err_metric(got[name], r)[0] <= tol, name


@pytest.mark.parametrize("n,H,B,d", [(33, 3, 2, 128), (300, 2, 1, 64), (1000, 5, 2, 128), (4133, 3, 1, 128)])
def test_bf16_interleaved_heads_forward(n, H, B, d):
    _check(synth.generate("C3", n=n, H=H, B=B, d=d), backward=False)


@pytest.mark.parametrize("n,H,B,d", [(31, 2, 1, 64), (515, 3, 2, 128)])
def test_fp32_interleaved_heads_forward(n, H, B, d):
    _check(synth.generate("C1", n=n, H=H, B=B, d=d), backward=False)


@pytest.mark.parametrize("n,H,B,d", [(129, 2, 2, 128), (777, 3, 1, 64), (2049, 4, 1, 128)])
def test_bf16_interleaved_heads_backward(n, H, B, d):
    _check(synth.generate("C5", n=n, H=H, B=B, d=d), backward=True)


@pytest.mark.parametrize("n,H,B,d", [(100, 3, 1, 128), (515, 2, 2, 64)])
def test_fp32_interleaved_heads_backward(n, H, B, d):
    _check(synth.generate("C1", n=n, H=H, B=B, d=d, with_dout=True), backward=True)


def test_layouts_agree_bitwise():
    """The same problem in both layouts gives identical bits (same arithmetic, other addresses)."""
    import torch
    from paper_2510_08318_amd import torch_glue as G
    x = synth.generate("C2", n=2500, H=4)
    wq, wk = G.to_device(x.wq), G.to_device(x.wk)
    a = G.Layer(wq, wk, x.B, x.n)
    b = G.Layer(wq, wk, x.B, x.n, layout="bnhd")
    oa = a.forward(*[G.to_device(t) for t in (x.q, x.k, x.v)])
    ob = b.forward(*[G.to_device(_bnhd(t)) for t in (x.q, x.k, x.v)])
    torch.cuda.synchronize()
    assert torch.equal(oa, ob.permute(0, 2, 1, 3))
    assert torch.equal(a.state, b.state)
    a.close(); b.close()
