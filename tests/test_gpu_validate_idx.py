"""The index-list check of the forward / backward calls (a debugging flag) and its asynchronous
form: a list that is not strictly ascending inside [0, T) is reported and nothing is written."""
import numpy as np
import pytest
import torch

from paper_2503_21817_amd import binding as B
from paper_2503_21817_amd import workloads as W
from helpers import Problem

pytestmark = pytest.mark.gpu


def _setup():
    w = W.config(1)
    p = Problem(w)
    bufs = B.SkipFFNBuffers(w.T, w.R, w.C, w.I)
    B.skipffn_compact(p.d_mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
    torch.cuda.synchronize()
    return w, p, bufs


def _bad_lists(idx, R, T):
    a = idx.clone(); a[3] = T                      # past the last token
    b = idx.clone(); b[5] = b[4]                   # repeated entry
    c = idx.clone(); c[0] = -1                     # negative
    d = idx.clone(); d[R - 1], d[R - 2] = idx[R - 2].item(), idx[R - 1].item()   # last two swapped
    return [(a, 3), (b, 5), (c, 0), (d, R - 1)]


def test_asynchronous_check_reports_the_first_offending_position():
    w, p, bufs = _setup()
    st = torch.full((2,), 7, dtype=torch.int32, device="cuda")
    B.skipffn_validate_idx(bufs.idx, w.R, w.T, st)
    assert st.tolist() == [0, 2**31 - 1]
    B.skipffn_validate_idx(bufs.idx, None, w.T, st, num_retained=bufs.num_retained)   # count read on the device
    assert st.tolist() == [0, 2**31 - 1]
    for bad, where in _bad_lists(bufs.idx, w.R, w.T):
        B.skipffn_validate_idx(bad, w.R, w.T, st)
        assert st.tolist() == [1, where]
    two = bufs.idx.clone(); two[10] = two[9]; two[20] = -4
    B.skipffn_validate_idx(two, w.R, w.T, st)
    assert st.tolist() == [1, 10]
    B.skipffn_validate_idx(bufs.idx, 0, w.T, st)              # nothing to check
    assert st.tolist() == [0, 2**31 - 1]


def test_flag_rejects_a_bad_list_before_anything_is_written():
    w, p, bufs = _setup()
    ref = p.d_hidden.clone()
    B.skipffn_forward(ref, ref, bufs.idx, w.R, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, saved=bufs.saved,
                      workspace=bufs.fwd_ws)
    h = p.d_hidden.clone()
    B.skipffn_forward(h, h, bufs.idx, w.R, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, saved=bufs.saved,
                      workspace=bufs.fwd_ws, flags=B.FLAG_VALIDATE_IDX)
    assert torch.equal(h.view(torch.int16), ref.view(torch.int16))       # a good list: the same result
    dws = [torch.zeros(s, dtype=torch.bfloat16, device="cuda") for s in ((w.I, w.C), (w.I, w.C), (w.C, w.I))]
    for bad, _ in _bad_lists(bufs.idx, w.R, w.T):
        h = p.d_hidden.clone()
        out = torch.full_like(h, 3.0)
        with pytest.raises(B.SkipFFNError) as ei:
            B.skipffn_forward(h, out, bad, w.R, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, saved=bufs.saved,
                              workspace=bufs.fwd_ws, flags=B.FLAG_VALIDATE_IDX)
        assert ei.value.status == B.EIDX
        torch.cuda.synchronize()
        assert bool((out == 3.0).all()) and torch.equal(h.view(torch.int16), p.d_hidden.view(torch.int16))
        g = p.d_grad.clone()
        with pytest.raises(B.SkipFFNError) as ei:
            B.skipffn_backward(g, g, bad, w.R, p.d_wg, p.d_wu, p.d_wd, bufs.saved, *dws, eps=w.eps,
                               workspace=bufs.bwd_ws, flags=B.FLAG_VALIDATE_IDX)
        assert ei.value.status == B.EIDX
        torch.cuda.synchronize()
        assert torch.equal(g.view(torch.int16), p.d_grad.view(torch.int16))
        assert all(bool((d == 0).all()) for d in dws)
    # the device-side count is honoured: entries past it are not looked at
    junk = bufs.idx.clone()
    junk[w.R:] = -9
    ws_t = torch.empty(B.skipffn_forward_workspace_bytes(w.T, w.C, w.I, False), dtype=torch.uint8, device="cuda")
    outs = []
    for flags in (0, B.FLAG_VALIDATE_IDX):
        h = p.d_hidden.clone()
        B.skipffn_forward(h, h, junk, None, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, num_retained=bufs.num_retained,
                          workspace=ws_t, flags=flags)
        outs.append(h)
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))
