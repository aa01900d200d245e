"""CPU fp64 oracle for non-causal linear attention with the Hedgehog feature map.

THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path (the HIP library
and its Python binding) never does, and shares no code with it.

What it computes, written from the paper (LinVideo, Sec. 3):

  * feature map, Eq. 5:      phi(x) = softmax(x W~) (+) softmax(-x W~),
                             W~ in R^{d x d/2}, softmax and concat over the
                             feature axis, one W~ for q and another for k;
  * operator, Eq. 3 (left):  o_i = sum_j w_ij v_j / sum_j w_ij,
                             w_ij = phi(q_i) . phi(k_j)            -- O(n^2)
  * operator, Eq. 3 (right): o_i = phi(q_i) S / (phi(q_i) . z),
                             S = sum_j phi(k_j)^T v_j, z = sum_j phi(k_j)
                                                                  -- O(n)
  * backward of the right-hand form (the paper fine-tunes through the layer,
    Sec. 5.1, but prints no gradient formula; the expressions below are the
    chain rule applied to Eq. 3 and Eq. 5).

Everything is per head: 2-D arrays q, k, v [n, d], W~ [d, d/2].  The *_bh
wrappers loop over [B, H, n, d] tensors.  Inputs may be float arrays or bf16 bit
patterns (uint16); they are widened exactly to fp64 first, so the oracle sees
the same rounded inputs as the device does.  No tiling, fusion or reordering:
matmul is used as a library step and nothing else is clever.

Readings where the paper is silent: d is the head width and each head has its
own W~; no bias, temperature, 1/sqrt(d) or epsilon (every entry of phi is
positive, so the denominator is positive); the sum runs over all n tokens.

Mixed attention of the selective-transfer stage (Sec. 4.1, Eq. 6): the layer's output is
r' * s + (1 - r') * o, where o is the linear attention above, s is the softmax
attention of the same q, k, v -- an INPUT here, it is never computed -- and
r' = clip(r, 0, 1) (footnote to Eq. 6), one learnable scalar r per layer.  Reading of
the clip's derivative: 1 for 0 <= r <= 1, 0 outside; the closed ends are needed
because the paper initialises every r to exactly 1 and trains it from there.

Pins: tests/test_oracle_pins.py (brute force, closed forms, invariants,
scipy's softmax, finite differences).  No function here is unpinned.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "to_f64", "phi", "state", "fwd", "fwd_bruteforce", "bwd", "fwd_bh", "bwd_bh",
    "state_bh", "finite_difference", "loss", "err_metric",
    "clip01", "blend_fwd_bh", "blend_bwd_bh",
]


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor to fp64 (uint16 is read as bf16 bits)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _softmax_rows(u: np.ndarray) -> np.ndarray:
    e = np.exp(u - u.max(axis=-1, keepdims=True))   # shift leaves softmax unchanged
    return e / e.sum(axis=-1, keepdims=True)


def phi(x: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Eq. 5: [n, d] -> [n, d]; first d/2 columns softmax(xW~), last d/2 softmax(-xW~)."""
    u = x @ W
    return np.concatenate([_softmax_rows(u), _softmax_rows(-u)], axis=-1)


def state(k: np.ndarray, v: np.ndarray, Wk: np.ndarray):
    """The two bracketed sums of Eq. 3 (right): S [d, d] and z [d]."""
    fk = phi(k, Wk)
    return fk.T @ v, fk.sum(axis=0)


def fwd(q, k, v, Wq, Wk) -> np.ndarray:
    """Eq. 3, right-hand (O(n)) form."""
    S, z = state(k, v, Wk)
    fq = phi(q, Wq)
    return (fq @ S) / (fq @ z)[:, None]


def fwd_bruteforce(q, k, v, Wq, Wk) -> np.ndarray:
    """Eq. 3, left-hand (O(n^2)) form, one query at a time."""
    n, d = q.shape
    h = d // 2
    out = np.empty((n, v.shape[1]), np.float64)
    uq = q @ Wq
    uk = k @ Wk
    # feature maps by the definition of softmax, token by token
    fk = np.empty((k.shape[0], d), np.float64)
    for j in range(k.shape[0]):
        ep = np.exp(uk[j] - uk[j].max())
        em = np.exp(-uk[j] - (-uk[j]).max())
        fk[j, :h] = ep / ep.sum()
        fk[j, h:] = em / em.sum()
    for i in range(n):
        ep = np.exp(uq[i] - uq[i].max())
        em = np.exp(-uq[i] - (-uq[i]).max())
        fq = np.concatenate([ep / ep.sum(), em / em.sum()])
        w = fk @ fq                      # w_ij for all j
        out[i] = (w[:, None] * v).sum(axis=0) / w.sum()
    return out


def _phi_vjp(x, W, g):
    """Pull a cotangent g = dL/dphi(x) [n, d] back through Eq. 5.

    With p+ = softmax(u), p- = softmax(-u), u = x W~:
      du = p+ (g+ - <g+, p+>) - p- (g- - <g-, p->),  dx = du W~^T,  dW~ = x^T du.
    """
    h = W.shape[1]
    u = x @ W
    pp, pm = _softmax_rows(u), _softmax_rows(-u)
    gp, gm = g[:, :h], g[:, h:]
    du = pp * (gp - (gp * pp).sum(-1, keepdims=True)) - pm * (gm - (gm * pm).sum(-1, keepdims=True))
    return du @ W.T, x.T @ du


def bwd(q, k, v, Wq, Wk, dout):
    """Gradients of L = sum(dout * fwd(...)) w.r.t. q, k, v, W~_q, W~_k (one head)."""
    fk = phi(k, Wk)
    fq = phi(q, Wq)
    S = fk.T @ v
    z = fk.sum(axis=0)
    den = fq @ z
    o = (fq @ S) / den[:, None]
    delta = (dout * o).sum(-1)                         # dO_i . o_i
    dfq = (dout @ S.T - delta[:, None] * z[None, :]) / den[:, None]
    dS = fq.T @ (dout / den[:, None])
    dz = -(fq * (delta / den)[:, None]).sum(axis=0)
    dfk = v @ dS.T + dz[None, :]
    dv = fk @ dS
    dq, dWq = _phi_vjp(q, Wq, dfq)
    dk, dWk = _phi_vjp(k, Wk, dfk)
    return dq, dk, dv, dWq, dWk


def loss(q, k, v, Wq, Wk, dout) -> float:
    return float((dout * fwd(q, k, v, Wq, Wk)).sum())


def finite_difference(q, k, v, Wq, Wk, dout, which: str, idx, rel_step: float = 1e-6) -> float:
    """Central difference of `loss` w.r.t. one entry of the tensor named `which`."""
    args = {"q": q, "k": k, "v": v, "Wq": Wq, "Wk": Wk}
    a = args[which]
    x0 = a[idx]
    h = rel_step * max(1.0, abs(x0))
    ap = a.copy(); ap[idx] = x0 + h
    am = a.copy(); am[idx] = x0 - h
    lp = loss(**{**args, which: ap}, dout=dout)
    lm = loss(**{**args, which: am}, dout=dout)
    return (lp - lm) / (2 * h)


# ---- [B, H, n, d] wrappers ------------------------------------------------------------

def state_bh(k, v, wk):
    """fp64 state in the exported layout [B, H, d+1, d]: rows 0..d-1 = S, row d = z."""
    B, H, n, d = k.shape
    out = np.empty((B, H, d + 1, d), np.float64)
    for b in range(B):
        for h in range(H):
            S, z = state(to_f64(k[b, h]), to_f64(v[b, h]), to_f64(wk[h]))
            out[b, h, :d] = S
            out[b, h, d] = z
    return out


def fwd_bh(q, k, v, wq, wk) -> np.ndarray:
    B, H, n, d = q.shape
    out = np.empty((B, H, n, d), np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h] = fwd(to_f64(q[b, h]), to_f64(k[b, h]), to_f64(v[b, h]),
                            to_f64(wq[h]), to_f64(wk[h]))
    return out


def bwd_bh(q, k, v, wq, wk, dout):
    """dq, dk, dv [B,H,n,d]; dWq, dWk [H,d,d/2] summed over the batch."""
    B, H, n, d = q.shape
    dq = np.empty((B, H, n, d), np.float64)
    dk = np.empty_like(dq)
    dv = np.empty_like(dq)
    dwq = np.zeros((H, d, d // 2), np.float64)
    dwk = np.zeros_like(dwq)
    for b in range(B):
        for h in range(H):
            r = bwd(to_f64(q[b, h]), to_f64(k[b, h]), to_f64(v[b, h]),
                    to_f64(wq[h]), to_f64(wk[h]), to_f64(dout[b, h]))
            dq[b, h], dk[b, h], dv[b, h] = r[0], r[1], r[2]
            dwq[h] += r[3]
            dwk[h] += r[4]
    return dq, dk, dv, dwq, dwk


def err_metric(got: np.ndarray, ref: np.ndarray):
    """Max relative error per (b, h) slice with an RMS floor, and the normwise error.

    The outputs are heavily cancelling averages of zero-mean values, so a plain
    element-wise relative error is unbounded near zeros; each element's error is
    therefore divided by max(|ref|, rms of ref over its (b, h) slice).
    Returns (max floored relative error, max |diff| / max |ref|); both are +inf if any
    element of got (or of ref) is NaN or infinite, so that `err <= tol` can never pass on one.
    """
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    lead = ref.shape[:-2]
    g2 = got.reshape((-1,) + ref.shape[-2:])
    r2 = ref.reshape((-1,) + ref.shape[-2:])
    if not (np.isfinite(g2).all() and np.isfinite(r2).all()):
        return float("inf"), float("inf")
    worst, worst_norm = 0.0, 0.0
    for s in range(r2.shape[0]):
        diff = np.abs(g2[s] - r2[s])
        rms = np.sqrt(np.mean(r2[s] ** 2))
        floor = np.maximum(np.abs(r2[s]), rms)
        floor = np.where(floor > 0, floor, 1.0)
        worst = max(worst, float((diff / floor).max()))
        m = float(np.abs(r2[s]).max())
        worst_norm = max(worst_norm, float(diff.max()) / (m if m > 0 else 1.0))
    return worst, worst_norm


# ---- mixed attention (Eq. 6) -------------------------------------------------------------

def clip01(r: float) -> float:
    """r clipped into [0, 1] (footnote to Eq. 6)."""
    return min(max(float(r), 0.0), 1.0)


def blend_fwd_bh(q, k, v, wq, wk, s, r: float) -> np.ndarray:
    """Eq. 6 with the softmax branch given: clip(r) * s + (1 - clip(r)) * linear attention."""
    rb = clip01(r)
    return rb * to_f64(s) + (1.0 - rb) * fwd_bh(q, k, v, wq, wk)


def blend_bwd_bh(q, k, v, wq, wk, s, r: float, dout):
    """Gradients of L = sum(dout * blend_fwd_bh(...)): dq, dk, dv, dWq, dWk, ds, dr.

    The linear branch receives (1 - clip(r)) * dout; the softmax branch output s receives
    clip(r) * dout; dr = sum(dout * (s - o)) inside the clip's range, 0 outside."""
    rb = clip01(r)
    do = to_f64(dout)
    dq, dk, dv, dwq, dwk = bwd_bh(q, k, v, wq, wk, (1.0 - rb) * do)
    o = fwd_bh(q, k, v, wq, wk)
    inside = 0.0 <= float(r) <= 1.0
    dr = float(np.sum(do * (to_f64(s) - o))) if inside else 0.0
    return dq, dk, dv, dwq, dwk, rb * do, dr

