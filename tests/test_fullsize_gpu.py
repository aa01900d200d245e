"""Full-size parity: every configuration of the task at its real shape, in the launch configuration
the benchmark times, with EVERY head and EVERY token row compared with the CPU fp64 oracle.

Forward: out of each (b,h) against the oracle's Eq. 3 (right-hand form) with the RMS-floored relative
error (1e-2, bf16 tensors), the exported state normwise (2e-3).  Backward: dq, dk, dv of every head
and dW~_q, dW~_k against the oracle's chain rule, on the config-5 recipe and on the config-3 recipe
(0.1 % of the token rows at 20x magnitude), the latter at n = 20000 and at the full 40-head,
75600-token shape.  The oracle works one head at a time, so no full fp64 copy of a tensor is held.
"""
import numpy as np
import pytest

from oracle import linattn_oracle as O
from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu

TOL = 1e-2           # bf16 tensors, RMS-floored max relative error
STATE_TOL = 2e-3     # exported fp32 state, normwise
# dk of the key rows at 20x magnitude (outlier recipe).  dL/dphi(k_j) = v_j dS^T + dz scales with |v_j|, and so does
# the absolute error it inherits from the fp16 operands behind dS (phi(q) and dO/den in the sum over tokens, the dS
# operand image) and from the fp16 du: about 2e-4 of |g_j|.  Where phi(k_j) is peaked but not saturated, du_j is a
# p-weighted difference of two close entries of g_j, no larger than for an ordinary row, while its absolute error is
# 20 times an ordinary row's.  Kernels at the full 40-head shape: up to 1e-1 of the head's RMS on the worst such row
# of the worst head, 4.6e-2 on head 1
# (a CPU emulation of the kernel's roundings: 3.2e-2; phi(q) alone 4.6e-2, the dS image 2.8e-2, du 1.4e-2,
# dO/den 1.1e-2; at n = 20000: 1.35e-2).  Every other row meets 1e-2.
# Observed over all heads: 8.2e-2 of the head's RMS, 9.8e-2 against max(own RMS, RMS of the other rows).
# dW~_k on this recipe: 2.0e-2 (B = 2, n = 9000: few outlier rows, each dominant in the sum), 5.2e-3 at n = 75600.
OUTLIER_ROW_BOUND = 0.25
OUTLIER_OWN_RMS_BOUND = 0.25
OUTLIER_DWK_BOUND = 5e-2


def _forward_all_heads(name, relu=False):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    x = synth.generate(name)
    q, k, v, wq, wk = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk)]
    lay = G.ReluLayer(x.H, x.d, x.B, x.n, q.dtype) if relu else G.Layer(wq, wk, x.B, x.n)
    out = lay.forward(q, k, v)
    torch.cuda.synchronize()
    worst, worst_state = 0.0, 0.0
    for b in range(x.B):
        for h in range(x.H):
            kk, vv, qq = O.to_f64(x.k[b, h]), O.to_f64(x.v[b, h]), O.to_f64(x.q[b, h])
            if relu:
                from oracle import relu_oracle as R
                S, z = R.relu_state(kk, vv)
                ref = R.relu_fwd(qq, kk, vv)
            else:
                S, z = O.state(kk, vv, O.to_f64(x.wk[h]))
                fq = O.phi(qq, O.to_f64(x.wq[h]))
                ref = (fq @ S) / (fq @ z)[:, None]            # Eq. 3, right-hand form, from the fp64 state
            st = G.to_host_f64(lay.state[b, h])
            e_state = max(np.abs(st[:x.d] - S).max() / np.abs(S).max(), np.abs(st[x.d] - z).max() / np.abs(z).max())
            err = O.err_metric(G.to_host_f64(out[b, h]), ref)[0]
            assert e_state <= STATE_TOL and err <= TOL, (name, b, h, err, e_state)
            worst, worst_state = max(worst, err), max(worst_state, e_state)
    # convexity holds at any size: every output lies between the smallest and largest v of its channel
    if not relu:
        vmin = v.float().amin(dim=2, keepdim=True)
        vmax = v.float().amax(dim=2, keepdim=True)
        o32 = out.float()
        assert bool(((o32 <= vmax + 1e-6) & (o32 >= vmin - 1e-6)).all())
    lay.close()
    print(f"[{name}{' relu' if relu else ''}] all {x.B * x.H} heads, all {x.n} rows: worst error {worst:.2e}, state {worst_state:.2e}")
    return worst


def test_config2_wan_1p3b_480p_every_head_and_row():
    _forward_all_heads("C2")


def test_config3_wan_14b_720p_every_head_and_row():
    _forward_all_heads("C3")


def test_config4_cfg_batch_every_head_and_row():
    _forward_all_heads("C4")


def test_cogvideox_2b_shape_every_head_and_row():
    """Second architecture (30 heads of width 64, 17550 tokens): the d = 64 kernels at a real shape."""
    _forward_all_heads("C6")


def test_relu_map_config3_shape_every_head_and_row():
    _forward_all_heads("C3", relu=True)


def _backward_all_heads(x, relu=False, wgrads=True):
    import torch
    from paper_2510_08318_amd import torch_glue as G
    q, k, v, wq, wk, do = [G.to_device(t) for t in (x.q, x.k, x.v, x.wq, x.wk, x.dout)]
    lay = G.ReluLayer(x.H, x.d, x.B, x.n, q.dtype) if relu else G.Layer(wq, wk, x.B, x.n, want_wgrads=wgrads)
    lay.forward(q, k, v)
    dq, dk, dv = lay.backward(q, k, v, do)
    torch.cuda.synchronize()
    worst = {}
    dwq_ref = np.zeros((x.H, x.d, x.d // 2))
    dwk_ref = np.zeros_like(dwq_ref)
    for b in range(x.B):
        for h in range(x.H):
            args = [O.to_f64(t) for t in (x.q[b, h], x.k[b, h], x.v[b, h])]
            if relu:
                from oracle import relu_oracle as R
                ref = R.relu_bwd(*args, O.to_f64(x.dout[b, h]))
            else:
                ref = O.bwd(*args, O.to_f64(x.wq[h]), O.to_f64(x.wk[h]), O.to_f64(x.dout[b, h]))
                dwq_ref[h] += ref[3]
                dwk_ref[h] += ref[4]
            rows = x.outlier_rows[b] if len(x.outlier_rows) > b else np.zeros(0, np.int64)
            for name, t, r in zip(("dq", "dk", "dv"), (dq, dk, dv), ref):
                g = G.to_host_f64(t[b, h])
                err = O.err_metric(g, r)[0]
                if name == "dk" and len(rows):
                    # The key rows at 20x magnitude are outside the 1e-2 contract (see OUTLIER_ROW_BOUND and the
                    # numeric-domain note in include/linattn.h).  Checked: every other row against the RMS floor of
                    # those rows (1e-2); each outlier row against the larger of its own RMS and that floor, and
                    # the head-wide number, against the documented bound.
                    keep = np.ones(x.n, bool); keep[rows] = False
                    err_rest = O.err_metric(g[keep], r[keep])[0]
                    rms_rest = np.sqrt(np.mean(r[keep] ** 2))
                    err_rows = max(float((np.abs(g[i] - r[i]) / np.maximum(np.abs(r[i]), max(np.sqrt(np.mean(r[i] ** 2)), rms_rest))).max())
                                   for i in rows)          # floor: the row's own RMS, or that of the other rows if larger
                    assert err_rest <= TOL and err_rows <= OUTLIER_OWN_RMS_BOUND and err <= OUTLIER_ROW_BOUND, (name, b, h, err_rest, err_rows, err)
                    worst["dk outlier rows, own RMS"] = max(worst.get("dk outlier rows, own RMS", 0.0), err_rows)
                    worst["dk head-wide"] = max(worst.get("dk head-wide", 0.0), err)
                    err = err_rest
                else:
                    assert err <= TOL, (name, b, h, err)
                worst[name] = max(worst.get(name, 0.0), err)
    if not relu and wgrads:
        has_outliers = any(len(r_) for r_ in x.outlier_rows)
        for name, t, r in (("dwq", lay.dwq, dwq_ref), ("dwk", lay.dwk, dwk_ref)):
            err = O.err_metric(G.to_host_f64(t), r)[0]
            # dW~_k = sum_j k_j^T du_j weights the du error of a 20x key row by another factor 20
            assert err <= (OUTLIER_DWK_BOUND if name == "dwk" and has_outliers else TOL), (name, err)
            worst[name] = err
    lay.close()
    print(f"[backward{' relu' if relu else ''} B={x.B} H={x.H} n={x.n} d={x.d}] every head and row: "
          + ", ".join(f"{k_} {e:.2e}" for k_, e in worst.items()))
    return worst


def test_config5_post_training_step_every_head_and_row():
    """Config 5 at full size (B=1, H=12, n=32760, d=128), forward then backward, weight gradients on."""
    _backward_all_heads(synth.generate("C5"))


def test_relu_map_config5_every_head_and_row():
    _backward_all_heads(synth.generate("C5"), relu=True)


def test_backward_on_the_outlier_recipe():
    """Config-3 recipe (outlier token rows at 20x in q, k, v), n = 20000: per-token and per-workgroup fp16
    scales of the backward meet rows whose magnitude jumps by 20 within a tile."""
    _backward_all_heads(synth.generate("C3", n=20000, H=3, with_dout=True))


def test_backward_at_the_config3_shape_every_head_and_row():
    """Backward at the Wan-14B 720p shape (B=1, H=40, n=75600, d=128) on its outlier recipe: all 40 heads."""
    _backward_all_heads(synth.generate("C3", with_dout=True))


def test_backward_cfg_batch_shape_two_items():
    """B = 2 with 40 heads (B*H = 80 launch rows, dW~ summed over the batch) at a reduced length."""
    _backward_all_heads(synth.generate("C4", n=9000, with_dout=True))
