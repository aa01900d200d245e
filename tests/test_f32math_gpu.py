"""LINATTN_BF16_F32MATH: bf16 tensors, fp32 arithmetic (the kernels of the fp32 mode reading and writing
bf16).  It has none of the fp16 operands of the matrix-core path, so the cases that path documents as
outside its 1e-2 contract -- phi within a few per cent of uniform, the dk rows of keys at 20x magnitude,
dW~ of a saturated map -- must meet 1e-2 here, as must everything else; the fp32 outputs (state, dW~)
are held to the fp32 mode's bars."""
import numpy as np
import pytest

from oracle import linattn_oracle as O
from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu
NAMES = ["dq", "dk", "dv", "dwq", "dwk"]
TOL = 1e-2            # bf16 tensors: the store rounds to 8 significant bits (2^-9 = 2e-3 relative, worst case 3.9e-3)
F32_TOL = 2e-5        # fp32 outputs of sums over all tokens (dW~), as in the fp32 mode
STATE_TOL = 1e-5      # exported fp32 state, normwise


def _run(x, layout="bhnd", blend=None):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    q, k, v, wq, wk, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    perm = (lambda t: t.permute(0, 2, 1, 3).contiguous()) if layout == "bnhd" else (lambda t: t)
    back = (lambda t: t.permute(0, 2, 1, 3)) if layout == "bnhd" else (lambda t: t)
    q, k, v, do = [perm(t) for t in (q, k, v, do)]
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=True, layout=layout, f32_math=True)
    dr = None
    if blend is not None:
        s, r = blend
        dr = torch.zeros(1, device="cuda")
        lay.set_blend(perm(G.to_device(s)), torch.tensor([r], device="cuda"), dr)
    out = lay.forward(q, k, v)
    dq, dk, dv = lay.backward(q, k, v, do)
    torch.cuda.synchronize()
    res = {"out": G.to_host_f64(back(out)), "state": G.to_host_f64(lay.state),
           "grads": [G.to_host_f64(back(t)) for t in (dq, dk, dv)] + [G.to_host_f64(lay.dwq), G.to_host_f64(lay.dwk)],
           "dr": None if dr is None else float(dr.item())}
    lay.close()
    return res


def _check(x, label=""):
    got = _run(x)
    errs = {"out": O.err_metric(got["out"], O.fwd_bh(x.q, x.k, x.v, x.wq, x.wk))[0]}
    st_ref = O.state_bh(x.k, x.v, x.wk)
    errs["state"] = float(np.linalg.norm(got["state"] - st_ref) / np.linalg.norm(st_ref))
    ref = O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)
    dv_scale = np.abs(ref[2]).max()
    for name, g, r in zip(NAMES, got["grads"], ref):
        assert np.isfinite(g).all(), name
        if np.sqrt(np.mean(r ** 2)) < 1e-6 * dv_scale:
            # identically zero in exact arithmetic (n = 1: the output is v whatever q and k are): a relative
            # error is undefined, the result is measured against the size of the gradients that are not zero
            errs[name] = float(np.abs(g - r).max() / dv_scale)
        else:
            errs[name] = O.err_metric(g, r)[0]
    print(f"[f32math {label}] " + ", ".join(f"{k} {v:.2e}" for k, v in errs.items()))
    return errs


def _assert_contract(errs, dw_tol=F32_TOL):
    for name in ("out", "dq", "dk", "dv"):
        assert errs[name] <= TOL, errs
    assert errs["state"] <= STATE_TOL, errs
    assert errs["dwq"] <= dw_tol and errs["dwk"] <= dw_tol, errs


@pytest.mark.parametrize("n,H,d", [(1, 2, 128), (33, 2, 128), (1000, 3, 128), (2049, 2, 64)])
def test_recipe_inputs(n, H, d):
    _assert_contract(_check(synth.generate("C5", n=n, H=H, d=d), f"C5 n={n} d={d}"))


@pytest.mark.parametrize("d", [64, 128])
def test_near_uniform_phi_meets_the_contract(d):
    """q, k scaled by 0.01: phi within a few per cent of uniform, the regime in which the matrix-core path
    is documented (and pinned) at 0.2 for dq, dk, dW~."""
    from tests.test_range_gpu import _scaled
    errs = _check(_scaled(d, sq=0.01, sk=0.01), f"near-uniform d={d}")
    _assert_contract(errs, dw_tol=1e-3)      # dW~ is a difference of nearly equal terms here: fp32 conditioning


def test_outlier_rows_meet_the_contract():
    """Config-3 recipe (0.1 % of the tokens at 20x): every row of dk, the 20x keys included."""
    x = synth.generate("C3", n=3000, H=2, with_dout=True)
    assert len(x.outlier_rows[0]) > 0
    _assert_contract(_check(x, "outliers"), dw_tol=1e-4)


@pytest.mark.parametrize("steps", [dict(q=(1.0, 2.0 ** 12)), dict(k=(1.0, 2.0 ** 12)), dict(dout=(0.0, 1e-6))],
                         ids=lambda s: ",".join(f"{k}={v[0]:g}->{v[1]:g}" for k, v in s.items()))
def test_saturated_maps_and_stepped_gradients(steps):
    from tests.test_range_gpu import _stepped
    x = _stepped(64, H=4, n=3000, **steps)
    errs = _check(x, str(steps))
    # dW~ of a saturated side is ill-conditioned in u = x W~ itself: fp32 rounding of u moves it by 0.5e-3 .. 2e-3
    _assert_contract(errs, dw_tol=1e-2 if "dout" not in steps else F32_TOL)


def test_heads_interleaved_layout_is_bitwise_the_same():
    x = synth.generate("C5", n=517, H=3, d=128)
    a, b = _run(x), _run(x, layout="bnhd")
    assert np.array_equal(a["out"], b["out"]) and np.array_equal(a["state"], b["state"])
    for g, h in zip(a["grads"], b["grads"]):
        assert np.array_equal(g, h)


def test_mixed_attention():
    x = synth.generate("C5", n=700, H=2, d=128)
    rng = np.random.default_rng(5)
    s = synth._pack((rng.standard_normal(x.q.shape) * 0.1).astype(np.float32), x.dtype)
    r = 0.37
    got = _run(x, blend=(s, r))
    out_ref = O.blend_fwd_bh(x.q, x.k, x.v, x.wq, x.wk, s, r)
    assert O.err_metric(got["out"], out_ref)[0] <= TOL
    ref = O.blend_bwd_bh(x.q, x.k, x.v, x.wq, x.wk, s, r, x.dout)
    for name, g, rr in zip(NAMES, got["grads"], ref[:5]):
        assert O.err_metric(g, rr)[0] <= (TOL if name in ("dq", "dk", "dv") else F32_TOL), name
    assert abs(got["dr"] - ref[6]) <= 1e-4 * max(1.0, abs(ref[6]))


def test_relu_map():
    import torch
    from oracle import relu_oracle as R
    from paper_2510_08318_amd import torch_glue as G
    x = synth.generate("C5", n=900, H=2, d=128)
    q, k, v, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.dout)]
    lay = G.ReluLayer(x.H, x.d, x.B, x.n, q.dtype, f32_math=True)
    got = [lay.forward(q, k, v)] + list(lay.backward(q, k, v, do))
    torch.cuda.synchronize()
    got = [G.to_host_f64(t) for t in got]
    lay.close()
    ref = [R.relu_fwd_bh(x.q, x.k, x.v)] + list(R.relu_bwd_bh(x.q, x.k, x.v, x.dout))
    for name, g, r in zip(["out", "dq", "dk", "dv"], got, ref):
        assert O.err_metric(g, r)[0] <= TOL, name
