"""CPU fp64 oracle for non-causal linear attention with the ReLU feature map.

THIS IS TEST INFRASTRUCTURE.  Only the tests, the smoke check and the
benchmark's cpu_baseline leg may import it; the product path (the HIP library
and its Python binding) never does, and shares no code with it.

What it computes: the operator of LinVideo's Eq. 3,

    o_i = phi(q_i) S / (phi(q_i) . z + eps),   S = sum_j phi(k_j)^T v_j,   z = sum_j phi(k_j),

with the kernel function the paper's ablation of kernel functions names "ReLU" (table "Comparison
across kernel functions", appendix "Ablation for Kernel Function").  The paper gives the name
only.  Readings taken here:

  * phi(x) = max(x, 0) element by element on the d channels of a head, no weights, no bias
    (the plainest map of that name; feature width d, so the state has the same shape as with
    the map of Eq. 5);
  * a row of q or k can be all non-positive, so phi(q_i) . z can be 0, which cannot happen with
    Eq. 5.  eps = 1e-6 is added to the denominator (the usual guard of kernel-feature linear
    attention); such a query then gets o_i = 0.  PARITY UNPINNED for this rule: nothing in the
    paper fixes it;
  * derivative of max(x, 0) at x = 0 is taken as 0.

Everything else (per head, fp64, no tiling or reordering, matmul as a library step, inputs
widened exactly from their stored type) is as in linattn_oracle.py, which this file does not
import.

Pins: tests/test_relu_oracle_pins.py -- the O(n^2) form of Eq. 3 query by query, automatic
differentiation of a separately written forward, finite differences, invariants (negative
entries of q, k do not matter; non-negative inputs reduce to plain dot-product kernel
attention; a constant v is reproduced; an all-non-positive query gives 0).
"""
from __future__ import annotations

import numpy as np

__all__ = ["RELU_EPS", "to_f64", "phi_relu", "relu_state", "relu_fwd", "relu_fwd_bruteforce", "relu_bwd",
           "relu_loss", "relu_state_bh", "relu_fwd_bh", "relu_bwd_bh"]

RELU_EPS = 1e-6


def to_f64(a: np.ndarray) -> np.ndarray:
    """Exact widening of a stored tensor to fp64 (uint16 is read as bf16 bits)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def phi_relu(x: np.ndarray) -> np.ndarray:
    return np.maximum(x, 0.0)


def relu_state(k: np.ndarray, v: np.ndarray):
    """The two bracketed sums of Eq. 3 (right): S [d, d] and z [d]."""
    fk = phi_relu(k)
    return fk.T @ v, fk.sum(axis=0)


def relu_fwd(q, k, v) -> np.ndarray:
    """Eq. 3, right-hand (O(n)) form, eps in the denominator."""
    S, z = relu_state(k, v)
    fq = phi_relu(q)
    return (fq @ S) / ((fq @ z) + RELU_EPS)[:, None]


def relu_fwd_bruteforce(q, k, v) -> np.ndarray:
    """Eq. 3, left-hand (O(n^2)) form: one query at a time, weights w_ij = phi(q_i) . phi(k_j)."""
    n = q.shape[0]
    out = np.empty((n, v.shape[1]), np.float64)
    for i in range(n):
        fq = np.where(q[i] > 0, q[i], 0.0)
        w = np.empty(k.shape[0], np.float64)
        for j in range(k.shape[0]):
            w[j] = sum(fq[c] * k[j, c] for c in range(k.shape[1]) if k[j, c] > 0)
        out[i] = (w[:, None] * v).sum(axis=0) / (w.sum() + RELU_EPS)
    return out


def relu_bwd(q, k, v, dout):
    """Gradients of L = sum(dout * relu_fwd(q, k, v)) w.r.t. q, k, v (one head): the chain rule
    through Eq. 3, then the mask of max(x, 0)."""
    fk = phi_relu(k)
    fq = phi_relu(q)
    S = fk.T @ v
    z = fk.sum(axis=0)
    den = fq @ z + RELU_EPS
    o = (fq @ S) / den[:, None]
    delta = (dout * o).sum(-1)                         # dO_i . o_i
    dfq = (dout @ S.T - delta[:, None] * z[None, :]) / den[:, None]
    dS = fq.T @ (dout / den[:, None])
    dz = -(fq * (delta / den)[:, None]).sum(axis=0)
    dfk = v @ dS.T + dz[None, :]
    dv = fk @ dS
    return dfq * (q > 0), dfk * (k > 0), dv


def relu_loss(q, k, v, dout) -> float:
    return float((dout * relu_fwd(q, k, v)).sum())


# ---- [B, H, n, d] wrappers ------------------------------------------------------------

def relu_state_bh(k, v):
    """fp64 state in the exported layout [B, H, d+1, d]: rows 0..d-1 = S, row d = z."""
    B, H, n, d = k.shape
    out = np.empty((B, H, d + 1, d), np.float64)
    for b in range(B):
        for h in range(H):
            S, z = relu_state(to_f64(k[b, h]), to_f64(v[b, h]))
            out[b, h, :d] = S
            out[b, h, d] = z
    return out


def relu_fwd_bh(q, k, v) -> np.ndarray:
    B, H, n, d = q.shape
    out = np.empty((B, H, n, d), np.float64)
    for b in range(B):
        for h in range(H):
            out[b, h] = relu_fwd(to_f64(q[b, h]), to_f64(k[b, h]), to_f64(v[b, h]))
    return out


def relu_bwd_bh(q, k, v, dout):
    B, H, n, d = q.shape
    dq = np.empty((B, H, n, d), np.float64)
    dk = np.empty_like(dq)
    dv = np.empty_like(dq)
    for b in range(B):
        for h in range(H):
            dq[b, h], dk[b, h], dv[b, h] = relu_bwd(to_f64(q[b, h]), to_f64(k[b, h]), to_f64(v[b, h]),
                                                    to_f64(dout[b, h]))
    return dq, dk, dv
