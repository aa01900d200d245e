"""The entry points only enqueue kernels on the caller's stream (no allocation, no synchronisation, no
memset), so a forward + backward pair can be captured into a HIP graph.  The graph is replayed several
times with the program's own eager work and synchronisations between the replays, on new input values
written into the captured buffers, and every replay must equal the eager result bit for bit.
"""
import numpy as np
import pytest

from paper_2510_08318_amd import synth

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("blend", [False, True])
def test_captured_forward_backward_replays_bitwise(blend):
    import torch
    from paper_2510_08318_amd import binding as L, torch_glue as G
    xs = [synth.generate("C5", n=2049, H=3, B=1), synth.generate("C2", n=2049, H=3, B=1, with_dout=True)]
    x = xs[0]
    wq, wk = G.to_device(x.wq), G.to_device(x.wk)
    lay = G.Layer(wq, wk, x.B, x.n, want_wgrads=True)
    bufs = [G.to_device(t) for t in (x.q, x.k, x.v, x.dout)]
    if blend:
        s_in = (torch.randn(bufs[0].shape, device="cuda") * 0.1).to(bufs[0].dtype)
        lay.set_blend(s_in, torch.tensor([0.4], device="cuda"), torch.zeros(1, device="cuda"))
    outs = [torch.empty_like(bufs[0]) for _ in range(4)]

    def run(stream):
        q, k, v, do = bufs
        out, dq, dk, dv = outs
        L.linattn_fwd(q, k, v, out, x.B, x.H, x.n, x.d, lay.phi_id, stream)
        L.linattn_bwd(q, k, v, do, dq, dk, dv, x.B, x.H, x.n, x.d, lay.phi_id, stream)

    def snapshot():
        torch.cuda.synchronize()
        extra = [lay.dwq, lay.dwk] + ([lay._blend[2]] if blend else [])
        return [t.clone() for t in outs + extra]

    run(torch.cuda.current_stream().cuda_stream)          # warm-up outside the capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(torch.cuda.current_stream().cuda_stream)
    for rep in range(4):
        src = xs[rep % 2]
        for dst, t in zip(bufs, (src.q, src.k, src.v, src.dout)):
            dst.copy_(G.to_device(t))                      # eager work between the replays
        run(torch.cuda.current_stream().cuda_stream)
        eager = snapshot()
        for t in outs:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        replayed = snapshot()
        for a, b in zip(eager, replayed):
            assert torch.equal(a, b), rep
        assert all(torch.isfinite(t.float()).all() for t in replayed)
    lay.close()
