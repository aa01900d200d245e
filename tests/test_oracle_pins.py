"""Pins for the CPU oracle: everything here is fixed by the paper's equations or by
mathematics, never by the oracle's own output.

  * Eq. 3 states that the O(n^2) weighted average and the O(n) state form are the
    same function: the brute-force evaluation is the definition itself.
  * Eq. 5 makes phi two softmaxes: closed forms and scipy's softmax pin it.
  * Closed-form special cases of the whole operator (mean pooling, constant v,
    one token, equal keys), invariants (convexity, permutations), and central
    finite differences for every gradient.
  * Each pin is also shown to have teeth: a planted mistake in a copy of the
    oracle's arithmetic must make it fail.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

from oracle import linattn_oracle as O
from paper_2510_08318_amd import synth


def _rand(n, d, seed, scale=1.0, dv=None):
    g = np.random.default_rng(seed)
    q = g.standard_normal((n, d)) * scale / np.sqrt(d)
    k = g.standard_normal((n, d)) * scale / np.sqrt(d)
    v = g.standard_normal((n, dv or d)) / np.sqrt(d)
    Wq = g.standard_normal((d, d // 2))
    Wk = g.standard_normal((d, d // 2))
    return q, k, v, Wq, Wk


# ---------------------------------------------------------------- phi (Eq. 5)

def test_phi_matches_library_softmax():
    q, _, _, Wq, _ = _rand(37, 16, 0, scale=5.0)
    f = O.phi(q, Wq)
    u = q @ Wq
    np.testing.assert_allclose(f[:, :8], scipy_softmax(u, axis=-1), rtol=1e-13, atol=0)
    np.testing.assert_allclose(f[:, 8:], scipy_softmax(-u, axis=-1), rtol=1e-13, atol=0)


def test_phi_closed_forms():
    q, _, _, Wq, _ = _rand(50, 32, 1, scale=3.0)
    f = O.phi(q, Wq)
    assert f.shape == (50, 32)
    assert (f > 0).all() and (f < 1).all()
    np.testing.assert_allclose(f[:, :16].sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(f[:, 16:].sum(-1), 1.0, rtol=1e-14)
    # d = 2: each half is a softmax over a single feature, so phi == [1, 1]
    f2 = O.phi(np.random.default_rng(2).standard_normal((9, 2)), np.array([[0.7], [-1.3]]))
    np.testing.assert_array_equal(f2, np.ones((9, 2)))
    # W~ = 0 gives the uniform vector 2/d
    np.testing.assert_allclose(O.phi(q, np.zeros_like(Wq)), 1.0 / 16, rtol=1e-15)
    # ratio of two entries in the + half is exp(u_a - u_b); in the - half exp(u_b - u_a)
    u = q @ Wq
    np.testing.assert_allclose(f[:, 3] / f[:, 5], np.exp(u[:, 3] - u[:, 5]), rtol=1e-12)
    np.testing.assert_allclose(f[:, 16 + 3] / f[:, 16 + 5], np.exp(u[:, 5] - u[:, 3]), rtol=1e-12)


def test_phi_extreme_inputs_stay_finite():
    # |u| in the hundreds (outlier tokens): a softmax without max-subtraction overflows
    g = np.random.default_rng(3)
    x = g.standard_normal((5, 8)) * 300
    W = g.standard_normal((8, 4))
    f = O.phi(x, W)
    assert np.isfinite(f).all()
    np.testing.assert_allclose(f[:, :4].sum(-1), 1.0, rtol=1e-14)
    np.testing.assert_allclose(f[:, 4:].sum(-1), 1.0, rtol=1e-14)


# ------------------------------------------------------- forward (Eq. 3)

@pytest.mark.parametrize("n,d,seed,scale", [(1, 4, 0, 1.0), (7, 4, 1, 1.0), (33, 8, 2, 4.0),
                                             (130, 16, 3, 1.0), (257, 64, 4, 8.0)])
def test_fwd_equals_bruteforce(n, d, seed, scale):
    q, k, v, Wq, Wk = _rand(n, d, seed, scale)
    a = O.fwd(q, k, v, Wq, Wk)
    b = O.fwd_bruteforce(q, k, v, Wq, Wk)
    np.testing.assert_allclose(a, b, rtol=1e-11, atol=1e-13)


def test_fwd_equals_independent_weights_matrix():
    """Left side of Eq. 3 via an explicit n x n weight matrix built from scipy's softmax."""
    q, k, v, Wq, Wk = _rand(61, 8, 5, 2.0)
    fq = np.concatenate([scipy_softmax(q @ Wq, axis=1), scipy_softmax(-(q @ Wq), axis=1)], 1)
    fk = np.concatenate([scipy_softmax(k @ Wk, axis=1), scipy_softmax(-(k @ Wk), axis=1)], 1)
    w = np.einsum("if,jf->ij", fq, fk)
    ref = (w / w.sum(1, keepdims=True)) @ v
    np.testing.assert_allclose(O.fwd(q, k, v, Wq, Wk), ref, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(O.fwd_bruteforce(q, k, v, Wq, Wk), ref, rtol=1e-11, atol=1e-14)


def test_config1_full_bruteforce():
    """The tiny configuration (B=1, H=2, n=1024, d=64, fp32 storage), all of it."""
    x = synth.generate("C1")
    for h in range(x.H):
        args = [O.to_f64(t) for t in (x.q[0, h], x.k[0, h], x.v[0, h], x.wq[h], x.wk[h])]
        a = O.fwd(*args)
        b = O.fwd_bruteforce(*args)
        assert O.err_metric(a, b)[0] < 1e-12


def test_closed_form_mean_pool_when_W_is_zero():
    q, k, v, Wq, Wk = _rand(40, 8, 6)
    mean = v.mean(0, keepdims=True).repeat(40, 0)
    np.testing.assert_allclose(O.fwd(q, k, v, np.zeros_like(Wq), Wk), mean, rtol=1e-12, atol=1e-15)
    np.testing.assert_allclose(O.fwd(q, k, v, Wq, np.zeros_like(Wk)), mean, rtol=1e-12, atol=1e-15)


def test_closed_form_constant_v_one_token_equal_keys():
    q, k, v, Wq, Wk = _rand(25, 8, 7, 3.0)
    c = np.linspace(-1, 2, 8)
    np.testing.assert_allclose(O.fwd(q, k, np.tile(c, (25, 1)), Wq, Wk), np.tile(c, (25, 1)), rtol=1e-12)
    # n_k = 1: the only value comes back for every query
    np.testing.assert_allclose(O.fwd(q, k[:1], v[:1], Wq, Wk), np.tile(v[0], (25, 1)), rtol=1e-12)
    # equal keys: uniform weights
    keq = np.tile(k[3], (25, 1))
    np.testing.assert_allclose(O.fwd(q, keq, v, Wq, Wk), np.tile(v.mean(0), (25, 1)), rtol=1e-12, atol=1e-15)


def test_two_token_hand_computation():
    """n = 2, d = 2 (phi == [1,1]) and d = 4 worked by hand."""
    q = np.array([[0.3, -0.2], [1.0, 2.0]])
    k = np.array([[0.5, 0.1], [-0.4, 0.9]])
    v = np.array([[1.0, 0.0], [0.0, 2.0]])
    W = np.array([[1.0], [1.0]])
    np.testing.assert_allclose(O.fwd(q, k, v, W, W), [[0.5, 1.0], [0.5, 1.0]], rtol=1e-15)
    # d = 4, W~ = first two unit vectors: u = x[:2]
    W4 = np.zeros((4, 2)); W4[0, 0] = W4[1, 1] = 1.0
    q4 = np.array([[np.log(3.0), 0.0, 9.0, 9.0]])
    k4 = np.array([[0.0, 0.0, 1.0, 1.0], [np.log(2.0), 0.0, -5.0, 5.0]])
    v4 = np.array([[1.0, 0, 0, 0], [0, 1.0, 0, 0]])
    # phi(q) = [3/4, 1/4, 1/4, 3/4]; phi(k1) = [1/2]*4; phi(k2) = [2/3, 1/3, 1/3, 2/3]
    w1 = 0.5 * (0.75 + 0.25 + 0.25 + 0.75)
    w2 = 0.75 * 2 / 3 + 0.25 / 3 + 0.25 / 3 + 0.75 * 2 / 3
    expect = np.array([[w1 / (w1 + w2), w2 / (w1 + w2), 0, 0]])
    np.testing.assert_allclose(O.fwd(q4, k4, v4, W4, W4), expect, rtol=1e-14, atol=1e-16)


def test_invariants():
    n, d = 96, 16
    q, k, v, Wq, Wk = _rand(n, d, 8, 2.0)
    out = O.fwd(q, k, v, Wq, Wk)
    # convex combination of the values, channel by channel
    assert (out <= v.max(0) + 1e-13).all() and (out >= v.min(0) - 1e-13).all()
    # normaliser positive and at most 2n (each phi half sums to one)
    S, z = O.state(k, v, Wk)
    den = O.phi(q, Wq) @ z
    assert (den > 0).all() and (den <= 2 * n).all()
    np.testing.assert_allclose(z.sum(), 2 * n, rtol=1e-13)
    # permuting (k, v) jointly changes nothing; permuting q permutes the output rows
    p = np.random.default_rng(9).permutation(n)
    np.testing.assert_allclose(O.fwd(q, k[p], v[p], Wq, Wk), out, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(O.fwd(q[p], k, v, Wq, Wk), out[p], rtol=1e-12, atol=1e-15)
    # a common permutation of the feature columns of W~q and W~k is unobservable
    c = np.random.default_rng(10).permutation(d // 2)
    np.testing.assert_allclose(O.fwd(q, k, v, Wq[:, c], Wk[:, c]), out, rtol=1e-11, atol=1e-14)
    # associativity: (phi(Q) phi(K)^T) V == phi(Q) (phi(K)^T V)
    fq, fk = O.phi(q, Wq), O.phi(k, Wk)
    np.testing.assert_allclose((fq @ fk.T) @ v, fq @ S, rtol=1e-11, atol=1e-14)
    # state of a concatenation is the sum of the states (what split-n relies on)
    S1, z1 = O.state(k[:40], v[:40], Wk)
    S2, z2 = O.state(k[40:], v[40:], Wk)
    np.testing.assert_allclose(S1 + S2, S, rtol=1e-11, atol=1e-14)
    np.testing.assert_allclose(z1 + z2, z, rtol=1e-12)


def test_state_layout_and_bf16_widening():
    x = synth.generate("C2", n=48, H=2)
    st = O.state_bh(x.k, x.v, x.wk)
    assert st.shape == (1, 2, 129, 128)
    k0 = synth.bf16_bits_to_f32(x.k[0, 1]).astype(np.float64)
    np.testing.assert_array_equal(O.to_f64(x.k[0, 1]), k0)
    S, z = O.state(k0, O.to_f64(x.v[0, 1]), O.to_f64(x.wk[1]))
    np.testing.assert_array_equal(st[0, 1, :128], S)
    np.testing.assert_array_equal(st[0, 1, 128], z)
    # widening is exact: 1.0 and a value with a full 8-bit significand
    np.testing.assert_array_equal(O.to_f64(np.array([0x3F80, 0xC0FF], np.uint16)), [1.0, -7.96875])


# ------------------------------------------------------------- backward

def _fd_check(n, d, seed, scale, n_probe=12):
    q, k, v, Wq, Wk = _rand(n, d, seed, scale)
    dout = np.random.default_rng(seed + 100).standard_normal((n, d)) * 0.1
    dq, dk, dv, dWq, dWk = O.bwd(q, k, v, Wq, Wk, dout)
    g = np.random.default_rng(seed + 200)
    grads = {"q": dq, "k": dk, "v": dv, "Wq": dWq, "Wk": dWk}
    for name, G in grads.items():
        scale_ref = np.abs(G).max()
        for _ in range(n_probe):
            idx = tuple(int(g.integers(s)) for s in G.shape)
            fd = O.finite_difference(q, k, v, Wq, Wk, dout, name, idx)
            assert abs(fd - G[idx]) <= 1e-6 * max(abs(G[idx]), 1e-3 * scale_ref) + 1e-12, (name, idx, fd, G[idx])


def test_bwd_matches_finite_differences_small():
    _fd_check(19, 8, 11, 2.0)


def test_bwd_matches_finite_differences_n256_slice():
    """Config 5's check: the gradients against fp64 central differences at n = 256."""
    x = synth.generate("C5", n=256, H=1)
    q, k, v, Wq, Wk, dout = [O.to_f64(t) for t in (x.q[0, 0], x.k[0, 0], x.v[0, 0], x.wq[0], x.wk[0], x.dout[0, 0])]
    dq, dk, dv, dWq, dWk = O.bwd(q, k, v, Wq, Wk, dout)
    grads = {"q": dq, "k": dk, "v": dv, "Wq": dWq, "Wk": dWk}
    g = np.random.default_rng(77)
    for name, G in grads.items():
        scale_ref = np.abs(G).max()
        for _ in range(8):
            idx = tuple(int(g.integers(s)) for s in G.shape)
            fd = O.finite_difference(q, k, v, Wq, Wk, dout, name, idx)
            assert abs(fd - G[idx]) <= 1e-6 * max(abs(G[idx]), 1e-2 * scale_ref) + 1e-13, (name, idx, fd, G[idx])


def test_bwd_closed_forms():
    n, d = 30, 8
    q, k, v, Wq, Wk = _rand(n, d, 12, 2.0)
    dout = np.random.default_rng(13).standard_normal((n, d))
    dq, dk, dv, dWq, dWk = O.bwd(q, k, v, Wq, Wk, dout)
    # the attention weights of each query sum to one, so sum_j dv_j = sum_i dO_i
    np.testing.assert_allclose(dv.sum(0), dout.sum(0), rtol=1e-11, atol=1e-13)
    # gradients are linear in dO
    r = O.bwd(q, k, v, Wq, Wk, -2.5 * dout)
    for a, b in zip(r, (dq, dk, dv, dWq, dWk)):
        np.testing.assert_allclose(a, -2.5 * b, rtol=1e-11, atol=1e-14)
    # constant v: the output does not depend on q, k or W~ at all
    vc = np.tile(np.linspace(1, 2, d), (n, 1))
    dq0, dk0, _, dWq0, dWk0 = O.bwd(q, k, vc, Wq, Wk, dout)
    for a in (dq0, dk0, dWq0, dWk0):
        assert np.abs(a).max() < 1e-12
    # adding a constant to every row of v shifts out by it: gradients wrt q, k unchanged
    dq1, dk1, _, _, _ = O.bwd(q, k, v + 3.0, Wq, Wk, dout)
    np.testing.assert_allclose(dq1, dq, rtol=1e-9, atol=1e-12)
    np.testing.assert_allclose(dk1, dk, rtol=1e-9, atol=1e-12)


def test_bwd_batch_wrapper_sums_weight_grads_over_batch():
    x = synth.generate("C5", n=40, H=2, B=2)
    dq, dk, dv, dwq, dwk = O.bwd_bh(x.q, x.k, x.v, x.wq, x.wk, x.dout)
    acc = np.zeros_like(dwq)
    for b in range(2):
        for h in range(2):
            r = O.bwd(*[O.to_f64(t) for t in (x.q[b, h], x.k[b, h], x.v[b, h], x.wq[h], x.wk[h], x.dout[b, h])])
            np.testing.assert_array_equal(dq[b, h], r[0])
            acc[h] += r[3]
    np.testing.assert_allclose(dwq, acc, rtol=1e-14)


# ----------------------------------------- the pins have teeth (planted mistakes, CPU only)

def _mutants():
    """Copies of the O(n) forward with one plausible mistake each."""
    def sm(u):
        e = np.exp(u - u.max(-1, keepdims=True)); return e / e.sum(-1, keepdims=True)

    def make(phi_fn, combine):
        def f(q, k, v, Wq, Wk):
            fq, fk = phi_fn(q, Wq), phi_fn(k, Wk)
            return combine(fq, fk, v)
        return f

    good_phi = lambda x, W: np.concatenate([sm(x @ W), sm(-(x @ W))], -1)
    good_comb = lambda fq, fk, v: (fq @ (fk.T @ v)) / (fq @ fk.sum(0))[:, None]
    yield "dropped minus half", make(lambda x, W: np.concatenate([sm(x @ W), sm(x @ W)], -1), good_comb)
    yield "transposed W", make(lambda x, W: np.concatenate([sm(x[:, : W.shape[1]] @ W.T[:, : W.shape[1]]), sm(-(x @ W))], -1), good_comb)
    yield "softmax over tokens", make(lambda x, W: np.concatenate([np.exp(x @ W) / np.exp(x @ W).sum(0), sm(-(x @ W))], -1), good_comb)
    yield "no normaliser", make(good_phi, lambda fq, fk, v: fq @ (fk.T @ v))
    yield "normaliser from q", make(good_phi, lambda fq, fk, v: (fq @ (fk.T @ v)) / (fk @ fq.sum(0))[: fq.shape[0], None])
    yield "swapped Wq/Wk", (lambda q, k, v, Wq, Wk: good_comb(good_phi(q, Wk), good_phi(k, Wq), v))


def test_planted_mistakes_are_caught_by_bruteforce_pin():
    q, k, v, Wq, Wk = _rand(24, 8, 21, 2.0)
    ref = O.fwd_bruteforce(q, k, v, Wq, Wk)
    for name, f in _mutants():
        assert np.abs(f(q, k, v, Wq, Wk) - ref).max() > 1e-6, name


def test_planted_gradient_mistakes_are_caught_by_fd():
    """Three plausible slips in the chain rule of Eq. 3 + Eq. 5 -- the dz term dropped, the sign of the
    softmax(-u) half of the Jacobian flipped, the 1/den of dL/dphi(q) left out -- each planted in a copy
    of the oracle's arithmetic: the finite difference sides with the oracle and against the copy."""
    q, k, v, Wq, Wk = _rand(12, 8, 22, 2.0)
    dout = np.random.default_rng(23).standard_normal((12, 8))
    dq, dk, dv, dWq, dWk = O.bwd(q, k, v, Wq, Wk, dout)
    fk, fq = O.phi(k, Wk), O.phi(q, Wq)
    S, z = fk.T @ v, fk.sum(0)
    den = fq @ z
    o = (fq @ S) / den[:, None]
    delta = (dout * o).sum(-1)
    dS = fq.T @ (dout / den[:, None])
    dz = -(fq * (delta / den)[:, None]).sum(0)

    def vjp_wrong_sign(x, W, g):
        h = W.shape[1]
        u = x @ W
        pp, pm = scipy_softmax(u, axis=-1), scipy_softmax(-u, axis=-1)
        gp, gm = g[:, :h], g[:, h:]
        du = pp * (gp - (gp * pp).sum(-1, keepdims=True)) + pm * (gm - (gm * pm).sum(-1, keepdims=True))
        return du @ W.T

    planted = {
        "dropped dz": ("k", dk, O._phi_vjp(k, Wk, v @ dS.T)[0]),
        "plus sign on the minus half": ("k", dk, vjp_wrong_sign(k, Wk, v @ dS.T + dz[None, :])),
        "missing 1/den": ("q", dq, O._phi_vjp(q, Wq, dout @ S.T - delta[:, None] * z[None, :])[0]),
    }
    for name, (which, good, bad) in planted.items():
        idx = tuple(int(i) for i in np.unravel_index(np.abs(bad - good).argmax(), good.shape))
        fd = O.finite_difference(q, k, v, Wq, Wk, dout, which, idx)
        assert abs(fd - good[idx]) < 1e-6 * max(1e-3, abs(good[idx])), name
        assert abs(fd - bad[idx]) > 1e-4 * abs(good[idx]), name


# ---------------------------------------------------------------- the error metric of the parity tests

def _metric_case():
    """Two (b,h) slices [2 x 3] with very different magnitudes and three planted errors.
    Slice 0: ref = [[3, 4, 0], [0, 0, 0]]  -> rms = sqrt(25/6) = 2.0412...
      got differs by 0.3 at the entry 4  (|ref| > rms: 0.3/4 = 0.075)
      and by 0.1 at an entry 0           (|ref| < rms: 0.1/rms = 0.04899)
    Slice 1: ref = 1e-3 * [[1, 1, 1], [1, 1, 1]] -> rms = 1e-3
      got differs by 2e-4 at one entry   (2e-4/1e-3 = 0.2)   <- the worst
    """
    ref = np.zeros((1, 2, 2, 3))
    ref[0, 0] = [[3.0, 4.0, 0.0], [0.0, 0.0, 0.0]]
    ref[0, 1] = 1e-3
    got = ref.copy()
    got[0, 0, 0, 1] += 0.3
    got[0, 0, 1, 2] -= 0.1
    got[0, 1, 1, 0] += 2e-4
    return got, ref


def test_err_metric_hand_values():
    """max |got - ref| / max(|ref|, rms of ref over the element's own (b,h) slice), and the normwise
    max |diff| / max |ref| per slice: values worked out by hand."""
    got, ref = _metric_case()
    rms0 = np.sqrt(25.0 / 6.0)
    # each error alone
    one = ref.copy(); one[0, 0, 0, 1] += 0.3
    assert O.err_metric(one, ref) == (pytest.approx(0.3 / 4.0, rel=1e-12), pytest.approx(0.3 / 4.0, rel=1e-12))
    one = ref.copy(); one[0, 0, 1, 2] -= 0.1
    assert O.err_metric(one, ref) == (pytest.approx(0.1 / rms0, rel=1e-12), pytest.approx(0.1 / 4.0, rel=1e-12))
    one = ref.copy(); one[0, 1, 1, 0] += 2e-4
    assert O.err_metric(one, ref) == (pytest.approx(0.2, rel=1e-9), pytest.approx(0.2, rel=1e-9))
    # all three: the small slice decides both numbers; a floor or a norm taken over the whole tensor
    # would hide it behind the large slice
    worst, norm = O.err_metric(got, ref)
    assert worst == pytest.approx(0.2, rel=1e-9) and norm == pytest.approx(0.2, rel=1e-9)
    # exact agreement, an all-zero reference (floor 1: absolute error), symmetric in sign
    assert O.err_metric(ref, ref) == (0.0, 0.0)
    zero = np.zeros((1, 1, 2, 2)); off = zero.copy(); off[0, 0, 1, 1] = -0.25
    assert O.err_metric(off, zero) == (0.25, 0.25)
    # 2-D input is one slice
    assert O.err_metric(got[0, 0], ref[0, 0])[0] == pytest.approx(0.3 / 4.0, rel=1e-12)
    # a non-finite value never passes
    for poison in (np.nan, np.inf, -np.inf):
        for where in ((0, 0, 0, 0), (0, 1, 1, 2)):
            bad = got.copy(); bad[where] = poison
            assert O.err_metric(bad, ref) == (np.inf, np.inf)


def test_err_metric_lenient_variants_give_other_numbers():
    """Plausible lenient versions of the metric -- one floor for the whole tensor, max |ref| in place of
    the RMS, the mean in place of the max, no per-slice norm -- all disagree with the hand values."""
    got, ref = _metric_case()
    diff = np.abs(got - ref)
    want = 0.2
    global_floor = (diff / np.maximum(np.abs(ref), np.sqrt(np.mean(ref ** 2)))).max()
    per_slice_max_floor = max((diff[0, s] / np.abs(ref[0, s]).max()).max() for s in range(2))
    mean_not_max = max((diff[0, s] / np.maximum(np.abs(ref[0, s]), np.sqrt(np.mean(ref[0, s] ** 2)))).mean() for s in range(2))
    global_norm = diff.max() / np.abs(ref).max()
    for name, val in (("global floor", global_floor), ("mean instead of max", mean_not_max), ("global norm", global_norm)):
        assert abs(val - want) > 0.05, name
    # max |ref| of the slice as the floor: the error at a zero entry of the large slice reads 0.1/4 with
    # it, 0.1/rms = 0.049 with the RMS floor
    one = ref.copy(); one[0, 0, 1, 2] -= 0.1
    with_max_floor = max((np.abs(one - ref)[0, s] / np.abs(ref[0, s]).max()).max() for s in range(2))
    assert with_max_floor == pytest.approx(0.025) and O.err_metric(one, ref)[0] == pytest.approx(0.1 / np.sqrt(25.0 / 6.0))
    assert per_slice_max_floor == pytest.approx(0.2, rel=1e-9)      # (on the full case that variant agrees)


# ---- mixed attention (Eq. 6) -------------------------------------------------------------

def _blend_problem(seed=5, B=1, H=2, n=23, d=8):
    g = np.random.default_rng(seed)
    mk = lambda: g.standard_normal((B, H, n, d)) / np.sqrt(d)
    q, k, v, s, dout = mk(), mk(), mk(), mk(), mk()
    wq, wk = g.standard_normal((H, d, d // 2)), g.standard_normal((H, d, d // 2))
    return q, k, v, wq, wk, s, dout


def _blend_loss(q, k, v, wq, wk, s, r, dout):
    return float(np.sum(dout * O.blend_fwd_bh(q, k, v, wq, wk, s, r)))


def test_blend_is_eq6_written_out():
    """Eq. 6 term by term, with the quadratic-cost forms of both branches on a tiny problem: the
    second term is the left-hand side of Eq. 3, the first is handed in as s."""
    q, k, v, wq, wk, s, _ = _blend_problem()
    r = 0.37
    got = O.blend_fwd_bh(q, k, v, wq, wk, s, r)
    for h in range(q.shape[1]):
        fq, fk = O.phi(q[0, h], wq[h]), O.phi(k[0, h], wk[h])
        w = fq @ fk.T
        lin = (w @ v[0, h]) / w.sum(axis=1, keepdims=True)
        np.testing.assert_allclose(got[0, h], r * s[0, h] + (1 - r) * lin, rtol=1e-12, atol=1e-14)


def test_blend_clipping_and_end_points():
    q, k, v, wq, wk, s, dout = _blend_problem()
    lin = O.fwd_bh(q, k, v, wq, wk)
    np.testing.assert_array_equal(O.blend_fwd_bh(q, k, v, wq, wk, s, 0.0), lin)
    np.testing.assert_array_equal(O.blend_fwd_bh(q, k, v, wq, wk, s, 1.0), s)
    np.testing.assert_array_equal(O.blend_fwd_bh(q, k, v, wq, wk, s, 1.7), s)       # clipped (footnote to Eq. 6)
    np.testing.assert_array_equal(O.blend_fwd_bh(q, k, v, wq, wk, s, -0.2), lin)
    # r = 1 (the paper's initial value): the linear branch gets no gradient, s gets all of it, and r
    # still moves (closed end of the clip)
    dq, dk, dv, dwq, dwk, ds, dr = O.blend_bwd_bh(q, k, v, wq, wk, s, 1.0, dout)
    assert not dq.any() and not dk.any() and not dv.any() and not dwq.any() and not dwk.any()
    np.testing.assert_array_equal(ds, dout)
    assert dr == pytest.approx(float(np.sum(dout * (s - lin))), rel=1e-12)
    assert O.blend_bwd_bh(q, k, v, wq, wk, s, 1.7, dout)[6] == 0.0
    assert O.blend_bwd_bh(q, k, v, wq, wk, s, -0.2, dout)[6] == 0.0
    # r = 0: the plain backward
    ref = O.bwd_bh(q, k, v, wq, wk, dout)
    got = O.blend_bwd_bh(q, k, v, wq, wk, s, 0.0, dout)
    for a, b in zip(got[:5], ref):
        np.testing.assert_array_equal(a, b)
    assert not got[5].any()


def test_blend_gradients_match_finite_differences():
    q, k, v, wq, wk, s, dout = _blend_problem(seed=9)
    r = 0.3
    dq, dk, dv, dwq, dwk, ds, dr = O.blend_bwd_bh(q, k, v, wq, wk, s, r, dout)
    h = 1e-6
    fd_r = (_blend_loss(q, k, v, wq, wk, s, r + h, dout) - _blend_loss(q, k, v, wq, wk, s, r - h, dout)) / (2 * h)
    assert dr == pytest.approx(fd_r, rel=1e-7)
    g = np.random.default_rng(3)
    args = {"q": q, "k": k, "v": v, "wq": wq, "wk": wk, "s": s}
    grads = {"q": dq, "k": dk, "v": dv, "wq": dwq, "wk": dwk, "s": ds}
    for name, G in grads.items():
        for _ in range(4):
            idx = tuple(int(g.integers(n_)) for n_ in G.shape)
            plus = {k_: a.copy() for k_, a in args.items()}
            minus = {k_: a.copy() for k_, a in args.items()}
            step = 1e-6 * max(1.0, abs(args[name][idx]))
            plus[name][idx] += step
            minus[name][idx] -= step
            fd = (_blend_loss(plus["q"], plus["k"], plus["v"], plus["wq"], plus["wk"], plus["s"], r, dout)
                  - _blend_loss(minus["q"], minus["k"], minus["v"], minus["wq"], minus["wk"], minus["s"], r, dout)) / (2 * step)
            assert abs(fd - G[idx]) <= 1e-6 * max(abs(G[idx]), 1e-2 * np.abs(G).max()) + 1e-12, (name, idx, fd, G[idx])


def test_blend_planted_mistakes_are_caught():
    """dr with the branches swapped, or the linear branch not scaled by 1 - r, fail the FD pin."""
    q, k, v, wq, wk, s, dout = _blend_problem(seed=9)
    r, h = 0.3, 1e-6
    fd_r = (_blend_loss(q, k, v, wq, wk, s, r + h, dout) - _blend_loss(q, k, v, wq, wk, s, r - h, dout)) / (2 * h)
    lin = O.fwd_bh(q, k, v, wq, wk)
    wrong_dr = float(np.sum(dout * (lin - s)))
    assert abs(wrong_dr - fd_r) > 1e-3 * abs(fd_r)
    unscaled = O.bwd_bh(q, k, v, wq, wk, dout)[0]
    right = O.blend_bwd_bh(q, k, v, wq, wk, s, r, dout)[0]
    assert np.abs(unscaled - right).max() > 0.1 * np.abs(right).max()


def test_hand_computed_two_token_fixture():
    """tests/golden/two_tokens_d4_by_hand.txt: Eq. 3 + Eq. 5 worked out by hand in exact rationals."""
    import os
    rows = {}
    with open(os.path.join(os.path.dirname(__file__), "golden", "two_tokens_d4_by_hand.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *vals = line.split()
                rows[name] = np.array([float(t) for t in vals])
    ln3 = np.log(3.0)
    W = np.zeros((4, 2)); W[0, 0] = 1.0
    q = np.array([[ln3, 0, 0, 0], [0, 0, 0, 0.0]])
    k = np.array([[ln3, 0, 0, 0], [-ln3, 0, 0, 0.0]])
    v = np.stack([rows["v_1"], rows["v_2"]])
    out = O.fwd(q, k, v, W, W)
    np.testing.assert_allclose(out, np.stack([rows["o_1"], rows["o_2"]]), rtol=0, atol=1e-14)
    np.testing.assert_allclose(O.fwd_bruteforce(q, k, v, W, W), out, rtol=0, atol=1e-14)
    S, z = O.state(k, v, W)
    np.testing.assert_allclose(z, rows["z"], atol=1e-15)
    np.testing.assert_allclose(S, np.stack([rows[f"S_row_{i}"] for i in range(4)]), atol=1e-14)
    np.testing.assert_allclose(O.phi(q, W) @ z, [rows["den_1"][0], rows["den_2"][0]], atol=1e-15)
