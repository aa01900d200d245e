"""Pins for the ReLU-map oracle (oracle/relu_oracle.py): fixed by Eq. 3, by the definition of
max(x, 0) and by mathematics, never by the oracle's own output.

  * Eq. 3's O(n^2) weighted average, query by query with scalar loops, is the definition.
  * torch's relu is the library form of the map; torch's automatic differentiation of a forward
    written here from Eq. 3's left-hand side pins every gradient, central differences pin them again.
  * Invariants and closed forms: negative entries do not matter, non-negative inputs give plain
    dot-product kernel attention, a constant v is reproduced, an all-non-positive query gives 0,
    one token gives v.
  * Planted mistakes in copies of the arithmetic must make the pins fail.

The eps rule for a zero denominator is this build's reading (the paper gives none): the tests state
it, nothing external pins it.
"""
import numpy as np
import pytest
import torch

from oracle import relu_oracle as R


def _rand(n, d, seed, scale=1.0):
    g = np.random.default_rng(seed)
    q = g.standard_normal((n, d)) * scale
    k = g.standard_normal((n, d)) * scale
    v = g.standard_normal((n, d))
    return q, k, v


def test_phi_is_library_relu():
    x = np.random.default_rng(0).standard_normal((33, 16))
    x[3, 4] = 0.0
    np.testing.assert_array_equal(R.phi_relu(x), torch.relu(torch.from_numpy(x)).numpy())


def test_state_form_equals_quadratic_form():
    q, k, v = _rand(23, 8, 1)
    np.testing.assert_allclose(R.relu_fwd(q, k, v), R.relu_fwd_bruteforce(q, k, v), rtol=1e-12, atol=1e-14)


def test_state_entries_by_hand():
    # two keys, d = 2:  phi(k) = [[1, 0], [0.5, 2]],  v = [[1, 2], [3, 4]]
    k = np.array([[1.0, -3.0], [0.5, 2.0]])
    v = np.array([[1.0, 2.0], [3.0, 4.0]])
    S, z = R.relu_state(k, v)
    np.testing.assert_allclose(S, [[1 * 1 + 0.5 * 3, 1 * 2 + 0.5 * 4], [2 * 3, 2 * 4]], rtol=0, atol=1e-15)
    np.testing.assert_allclose(z, [1.5, 2.0], rtol=0, atol=1e-15)
    # one query q = [2, -1]: phi = [2, 0]; num = 2 * S[0], den = 2 * 1.5
    o = R.relu_fwd(np.array([[2.0, -1.0]]), k, v)
    np.testing.assert_allclose(o[0], np.array([5.0, 8.0]) / (3.0 + R.RELU_EPS), rtol=1e-15)


def test_negative_entries_do_not_matter():
    q, k, v = _rand(19, 8, 2)
    q2, k2 = q.copy(), k.copy()
    q2[q2 < 0] *= 7.0
    k2[k2 < 0] -= 3.0
    np.testing.assert_array_equal(R.relu_fwd(q, k, v), R.relu_fwd(q2, k2, v))


def test_nonnegative_inputs_give_dot_product_attention():
    q, k, v = _rand(17, 8, 3)
    q, k = np.abs(q), np.abs(k)
    w = q @ k.T
    ref = (w @ v) / (w.sum(-1) + R.RELU_EPS)[:, None]
    np.testing.assert_allclose(R.relu_fwd(q, k, v), ref, rtol=1e-12)


def test_constant_v_is_reproduced_and_outputs_are_averages():
    q, k, v = _rand(29, 8, 4)
    c = np.linspace(-1, 1, 8)
    o = R.relu_fwd(q, k, np.tile(c, (29, 1)))
    S, z = R.relu_state(k, v)
    den = R.phi_relu(q) @ z
    np.testing.assert_allclose(o, np.outer(den / (den + R.RELU_EPS), c), rtol=1e-12, atol=1e-15)
    o = R.relu_fwd(q, k, v)
    assert (o <= v.max(0) + 1e-12).all() and (o >= v.min(0) - 1e-12).all()      # weights are >= 0


def test_dead_query_and_one_token():
    q, k, v = _rand(11, 8, 5)
    q[4] = -np.abs(q[4])
    o = R.relu_fwd(q, k, v)
    np.testing.assert_array_equal(o[4], np.zeros(8))
    dq, dk, dv = R.relu_bwd(q, k, v, np.ones_like(v))
    np.testing.assert_array_equal(dq[4], np.zeros(8))
    # a single key: every live query returns v_0 (up to eps)
    o1 = R.relu_fwd(np.abs(q), np.abs(k[:1]), v[:1])
    np.testing.assert_allclose(o1, np.tile(v[0], (11, 1)), rtol=1e-4)


def _torch_forward(q, k, v):
    """Eq. 3, left-hand side, written with torch ops for automatic differentiation."""
    w = torch.relu(q) @ torch.relu(k).T
    return (w @ v) / (w.sum(-1, keepdim=True) + R.RELU_EPS)


def test_gradients_match_automatic_differentiation():
    q, k, v = _rand(21, 8, 6)
    dout = np.random.default_rng(7).standard_normal(v.shape)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    (_torch_forward(tq, tk, tv) * torch.from_numpy(dout)).sum().backward()
    dq, dk, dv = R.relu_bwd(q, k, v, dout)
    np.testing.assert_allclose(dq, tq.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dk, tk.grad.numpy(), rtol=1e-10, atol=1e-13)
    np.testing.assert_allclose(dv, tv.grad.numpy(), rtol=1e-10, atol=1e-13)


@pytest.mark.parametrize("which", ["q", "k", "v"])
def test_gradients_match_finite_differences(which):
    q, k, v = _rand(9, 4, 8)
    dout = np.random.default_rng(9).standard_normal(v.shape)
    grads = dict(zip("qkv", R.relu_bwd(q, k, v, dout)))
    args = {"q": q, "k": k, "v": v}
    for idx in [(0, 0), (3, 2), (8, 3)]:
        a = args[which]
        h = 1e-6
        assert abs(a[idx]) > 10 * h          # away from the kink
        ap, am = a.copy(), a.copy()
        ap[idx] += h
        am[idx] -= h
        fd = (R.relu_loss(**{**args, which: ap}, dout=dout) - R.relu_loss(**{**args, which: am}, dout=dout)) / (2 * h)
        assert abs(fd - grads[which][idx]) <= 1e-6 * max(1.0, abs(fd))


def test_bh_wrappers_loop_over_heads_and_widen_bf16():
    g = np.random.default_rng(10)
    x = g.standard_normal((2, 3, 7, 8)).astype(np.float32)
    bits = (x.view(np.uint32) >> 16).astype(np.uint16)                      # truncation: some bf16 values
    exact = (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    out = R.relu_fwd_bh(bits, bits, bits)
    for b in range(2):
        for h in range(3):
            np.testing.assert_array_equal(out[b, h], R.relu_fwd(exact[b, h], exact[b, h], exact[b, h]))
    st = R.relu_state_bh(bits, bits)
    assert st.shape == (2, 3, 9, 8)
    np.testing.assert_array_equal(st[1, 2, 8], np.maximum(exact[1, 2], 0).sum(0))


# ---- the pins have teeth: planted mistakes in copies of the arithmetic ----------------------

def _fwd_variant(q, k, v, mistake):
    fk = np.maximum(k, 0.0)
    fq = np.maximum(q, 0.0)
    if mistake == "abs":
        fk, fq = np.abs(k), np.abs(q)
    S = fk.T @ v if mistake != "transposed" else v.T @ fk
    z = fk.sum(0) if mistake != "z_from_q" else fq.sum(0)
    den = fq @ z + (R.RELU_EPS if mistake != "no_eps" else 0.0)
    return (fq @ S) / den[:, None]


@pytest.mark.parametrize("mistake", ["abs", "transposed", "z_from_q"])
def test_planted_forward_mistakes_are_caught(mistake):
    q, k, v = _rand(23, 8, 1)
    ref = R.relu_fwd_bruteforce(q, k, v)
    assert np.abs(_fwd_variant(q, k, v, None) - ref).max() < 1e-12
    assert np.abs(_fwd_variant(q, k, v, mistake) - ref).max() > 1e-3


def test_planted_backward_mistake_is_caught():
    q, k, v = _rand(21, 8, 6)
    dout = np.random.default_rng(7).standard_normal(v.shape)
    tq, tk, tv = (torch.tensor(a, dtype=torch.float64, requires_grad=True) for a in (q, k, v))
    (_torch_forward(tq, tk, tv) * torch.from_numpy(dout)).sum().backward()
    dq, dk, dv = R.relu_bwd(q, k, v, dout)
    # dropping the mask, or the dz term, must show
    fk, fq = np.maximum(k, 0), np.maximum(q, 0)
    S, z = fk.T @ v, fk.sum(0)
    den = fq @ z + R.RELU_EPS
    dS = fq.T @ (dout / den[:, None])
    dk_no_dz = (v @ dS.T) * (k > 0)
    assert np.abs(dk_no_dz - tk.grad.numpy()).max() > 1e-3
    assert np.abs(dk - tk.grad.numpy()).max() < 1e-12
