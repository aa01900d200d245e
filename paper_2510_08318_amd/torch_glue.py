"""PyTorch as plumbing: device buffers and the current stream for the C-ABI calls.

Nothing of the operator is computed here; `Layer` owns the buffers a converted attention layer
needs (W~_q, W~_k, state, workspace), registers them as a phi descriptor and forwards to
linattn_fwd / linattn_bwd.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B_


def to_device(stored: np.ndarray, device="cuda") -> torch.Tensor:
    """Stored numpy tensor (float32, or uint16 bf16 bit patterns) -> device tensor of that dtype."""
    if stored.dtype == np.uint16:
        return torch.from_numpy(stored.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(stored, dtype=np.float32)).to(device)


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> fp64 numpy (exact widening)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


class ReluLayer:
    """Buffers + descriptor of one linear-attention layer with the weight-free map phi(x) = max(x, 0)
    (the "ReLU" row of the paper's ablation of kernel functions)."""

    def __init__(self, H: int, d: int, B: int, n: int, dtype: torch.dtype, *, layout: str = "bhnd", device="cuda",
                 f32_math: bool = False):
        assert layout in ("bhnd", "bnhd") and dtype in (torch.bfloat16, torch.float32)
        self.layout, self.H, self.d, self.B, self.n, self.tdtype = layout, H, d, B, n, dtype
        self.dtype = (B_.BF16_F32MATH if f32_math else B_.BF16) if dtype == torch.bfloat16 else B_.F32
        self.state = torch.empty((B, H, d + 1, d), dtype=torch.float32, device=device)
        self.workspace_bytes = B_.linattn_workspace_bytes(B, H, n, d, B_.PHI_RELU, self.dtype)
        if self.workspace_bytes == 0:
            raise ValueError("unsupported shape")
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)
        assert self.workspace.data_ptr() % 256 == 0
        self.phi_id = B_.linattn_phi_create(B_.PHI_RELU, self.dtype, H, d, None, None, None, None, self.state,
                                            self.workspace, self.workspace_bytes,
                                            B_.LAYOUT_BNHD if layout == "bnhd" else B_.LAYOUT_BHND)

    def close(self):
        if self.phi_id is not None:
            B_.linattn_phi_destroy(self.phi_id)
            self.phi_id = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, *ts):
        shape = (self.B, self.n, self.H, self.d) if self.layout == "bnhd" else (self.B, self.H, self.n, self.d)
        for t in ts:
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype and tuple(t.shape) == shape

    def forward(self, q, k, v, out=None):
        self._check(q, k, v)
        out = torch.empty_like(q) if out is None else out
        B_.linattn_fwd(q, k, v, out, self.B, self.H, self.n, self.d, self.phi_id, torch.cuda.current_stream().cuda_stream)
        return out

    def backward(self, q, k, v, dout, dq=None, dk=None, dv=None):
        self._check(q, k, v, dout)
        dq = torch.empty_like(q) if dq is None else dq
        dk = torch.empty_like(q) if dk is None else dk
        dv = torch.empty_like(q) if dv is None else dv
        B_.linattn_bwd(q, k, v, dout, dq, dk, dv, self.B, self.H, self.n, self.d, self.phi_id,
                       torch.cuda.current_stream().cuda_stream)
        return dq, dk, dv


class Layer:
    """Buffers + descriptor of one linear-attention layer (Eq. 3 with the map of Eq. 5)."""

    def __init__(self, wq: torch.Tensor, wk: torch.Tensor, B: int, n: int, *, keep_state: bool = True,
                 want_wgrads: bool = False, layout: str = "bhnd", f32_math: bool = False, centred: bool = False):
        """layout "bhnd": q, k, v, out are [B, H, n, d]; "bnhd": [B, n, H, d] (heads interleaved per token).
        want_wgrads: False, True (both dW~_q and dW~_k), or "q" / "k" for one of them.
        f32_math (bf16 tensors only): fp32 arithmetic on the bf16 tensors (LINATTN_BF16_F32MATH).
        centred (bf16 matrix-core path only): LINATTN_FLAG_CENTRED."""
        assert layout in ("bhnd", "bnhd")
        self.layout = layout
        assert wq.is_cuda and wk.is_cuda and wq.dtype == wk.dtype and wq.shape == wk.shape
        self.H, self.d, half = wq.shape
        assert half * 2 == self.d
        self.dtype = (B_.BF16_F32MATH if f32_math else B_.BF16) if wq.dtype == torch.bfloat16 else B_.F32
        assert wq.dtype in (torch.bfloat16, torch.float32)
        self.wq, self.wk = wq.contiguous(), wk.contiguous()
        self.B, self.n = B, n
        dev = wq.device
        self.state = torch.empty((B, self.H, self.d + 1, self.d), dtype=torch.float32, device=dev) if keep_state else None
        assert want_wgrads in (False, True, "q", "k")
        self.dwq = torch.empty((self.H, self.d, half), dtype=torch.float32, device=dev) if want_wgrads in (True, "q") else None
        self.dwk = torch.empty((self.H, self.d, half), dtype=torch.float32, device=dev) if want_wgrads in (True, "k") else None
        size_fn = B_.linattn_workspace_bytes_wgrads if want_wgrads else B_.linattn_workspace_bytes
        self.workspace_bytes = size_fn(B, self.H, n, self.d, B_.PHI_HEDGEHOG, self.dtype)
        if self.workspace_bytes == 0:
            raise ValueError("unsupported shape")
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        self.phi_id = B_.linattn_phi_create(B_.PHI_HEDGEHOG, self.dtype, self.H, self.d, self.wq, self.wk,
                                            self.dwq, self.dwk, self.state, self.workspace, self.workspace_bytes,
                                            B_.LAYOUT_BNHD if layout == "bnhd" else B_.LAYOUT_BHND,
                                            flags=B_.FLAG_CENTRED if centred else 0)

    def set_blend(self, s=None, r=None, dr=None):
        """Mixed attention (Eq. 6): s = softmax-branch output (dtype and layout of out), r = device fp32[1],
        dr = optional device fp32[1] receiving dL/dr in backward.  All None switches it off."""
        if s is not None:
            assert s.is_cuda and s.is_contiguous() and s.dtype == self.wq.dtype
            assert r.is_cuda and r.dtype == torch.float32 and r.numel() == 1
            assert dr is None or (dr.is_cuda and dr.dtype == torch.float32 and dr.numel() == 1)
        self._blend = (s, r, dr)          # keep the buffers alive
        B_.linattn_phi_set_blend(self.phi_id, s, r, dr)

    def close(self):
        if self.phi_id is not None:
            B_.linattn_phi_destroy(self.phi_id)
            self.phi_id = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _stream(self):
        return torch.cuda.current_stream().cuda_stream

    def _dims(self, t):
        if self.layout == "bnhd":
            Bq, n, H, d = t.shape
        else:
            Bq, H, n, d = t.shape
        assert (Bq, H, n, d) == (self.B, self.H, self.n, self.d)
        return Bq, H, n, d

    def forward(self, q, k, v, out=None):
        Bq, H, n, d = self._dims(q)
        for t in (q, k, v):
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.wq.dtype and t.shape == q.shape
        if out is None:
            out = torch.empty_like(q)
        B_.linattn_fwd(q, k, v, out, Bq, H, n, d, self.phi_id, self._stream())
        return out

    def backward(self, q, k, v, dout, dq=None, dk=None, dv=None):
        Bq, H, n, d = self._dims(q)
        for t in (q, k, v, dout):
            assert t.is_cuda and t.is_contiguous() and t.dtype == self.wq.dtype and t.shape == q.shape
        dq = torch.empty_like(q) if dq is None else dq
        dk = torch.empty_like(q) if dk is None else dk
        dv = torch.empty_like(q) if dv is None else dv
        B_.linattn_bwd(q, k, v, dout, dq, dk, dv, Bq, H, n, d, self.phi_id, self._stream())
        return dq, dk, dv
