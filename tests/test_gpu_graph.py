"""The whole step (compaction, forward, backward) captured in a HIP graph: the library
allocates nothing, never synchronises and uses only kernels (no memset nodes), so a caller may
capture it.  Replays are interleaved with eager work and every replay is compared with the
eager result."""
import pytest
import torch

from paper_2503_21817_amd import binding as B
from paper_2503_21817_amd import workloads as W
from helpers import Problem

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("r_host", [True, False], ids=["R-host", "R-device"])
def test_graph_replays_match_eager(r_host):
    w = W.small(C=512, I=1368, visual=(300, 411), text=(20, 35), keep=(130, 212), seed=61, name="graph")
    p = Problem(w)
    T, R, C, I = w.T, w.R, w.C, w.I
    bufs = B.SkipFFNBuffers(T, R if r_host else T, C, I, training=True)
    dws = [torch.zeros((I, C), dtype=torch.bfloat16, device="cuda"),
           torch.zeros((I, C), dtype=torch.bfloat16, device="cuda"),
           torch.zeros((C, I), dtype=torch.bfloat16, device="cuda")]
    dgain = torch.zeros(C, dtype=torch.float32, device="cuda")
    hidden = p.d_hidden.clone()
    grad = p.d_grad.clone()
    out = torch.empty_like(hidden)
    gh = torch.empty_like(grad)

    def step():
        B.skipffn_compact(p.d_mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
        B.skipffn_forward(hidden, out, bufs.idx, R if r_host else None, p.d_wg, p.d_wu, p.d_wd,
                          eps=w.eps, num_retained=bufs.num_retained, saved=bufs.saved,
                          workspace=bufs.fwd_ws)
        B.skipffn_backward(grad, gh, bufs.idx, R if r_host else None, p.d_wg, p.d_wu, p.d_wd,
                           bufs.saved, *dws, eps=w.eps, num_retained=bufs.num_retained,
                           workspace=bufs.bwd_ws, d_rms_gain=dgain)

    step()                                   # eager reference (also the one-time kernel set-up)
    torch.cuda.synchronize()
    ref = [t.clone() for t in (out, gh, *dws, dgain)]

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step()                               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(g, stream=side):
            step()
    torch.cuda.synchronize()

    for rep in range(4):
        for t in (out, gh, *dws, dgain):     # eager work between replays: poison the outputs
            t.fill_(float("nan") if t.is_floating_point() else 0)
        bufs.idx.fill_(-1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for a, b in zip((out, gh, *dws, dgain), ref):
            assert torch.equal(a.view(torch.int16) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.int16) if b.dtype == torch.bfloat16 else b), f"replay {rep}"
