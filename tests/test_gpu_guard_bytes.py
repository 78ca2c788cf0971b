"""No kernel writes outside the buffers the caller hands over: every workspace, saved-activation
buffer and output is carved out of a larger allocation whose surrounding bytes hold a pattern, at
exactly the size the *_bytes query reports, and the pattern must survive the call."""
import numpy as np
import pytest
import torch

from paper_2503_21817_amd import binding as B
from paper_2503_21817_amd import workloads as W
from helpers import Problem

pytestmark = pytest.mark.gpu

GUARD = 1 << 16
PATTERN = 0xA5


class Guarded:
    """A byte range of exactly `nbytes` (256-byte aligned) between two guard zones."""

    def __init__(self, nbytes, name):
        self.name = name
        self.nbytes = nbytes
        body = (nbytes + 255) // 256 * 256
        self.raw = torch.full((GUARD + body + GUARD,), PATTERN, dtype=torch.uint8, device="cuda")
        assert self.raw.data_ptr() % 256 == 0
        self.view = self.raw[GUARD:GUARD + nbytes]

    def typed(self, dtype, shape):
        return self.view.view(dtype).view(shape)

    def check(self):
        head = self.raw[:GUARD]
        tail = self.raw[GUARD + self.nbytes:]
        assert bool((head == PATTERN).all()), f"{self.name}: bytes before the buffer were written"
        assert bool((tail == PATTERN).all()), f"{self.name}: bytes after the buffer were written"


SHAPES = [
    W.config(1),
    W.small(C=512, I=1368, visual=(300, 411), text=(20, 35), keep=(130, 212), seed=11, name="ragged-2tiles"),
    W.small(C=264, I=520, visual=(700,), text=(9,), keep=(600,), seed=12, name="odd-dims-3tiles"),
    W.small(C=1024, I=2048, visual=(64,), text=(1,), keep=(0,), seed=13, name="one-row"),
    W.small(C=2048, I=5632, visual=(1100, 900), text=(30, 41), keep=(513, 300), seed=14, name="mid"),
    W.small(C=2048, I=2816, visual=(200,), text=(9,), keep=(100,), seed=15, name="few-rows-split-gate-up"),
    W.small(C=1024, I=1368, visual=(300,), text=(20,), keep=(180,), seed=16, name="two-128-row-tiles"),
]
FLAGS = [0, B.FLAG_BALANCED_SPLIT, B.FLAG_DW_FP32 | B.FLAG_BALANCED_SPLIT]


@pytest.mark.parametrize("w", SHAPES, ids=lambda w: w.name)
@pytest.mark.parametrize("flags", FLAGS)
def test_forward_backward_stay_inside_their_buffers(w, flags):
    print(f"guard bytes {w.name} T={w.T} R={w.R} C={w.C} I={w.I} flags={flags}", flush=True)
    p = Problem(w, unit_gain=False, with_gain_tensor=True)
    T, R, C, I = w.T, w.R, w.C, w.I
    g = {
        "idx": Guarded(4 * T, "idx"),
        "nr": Guarded(4, "num_retained"),
        "compact_ws": Guarded(max(B.skipffn_compact_workspace_bytes(T), 16), "compact workspace"),
        "saved": Guarded(B.skipffn_saved_bytes(R, C, I), "saved activations"),
        "fwd_ws": Guarded(B.skipffn_forward_workspace_bytes(R, C, I, True), "forward workspace"),
        "bwd_ws": Guarded(B.skipffn_backward_workspace_bytes(R, C, I), "backward workspace"),
        "out": Guarded(2 * T * C, "out"),
        "gh": Guarded(2 * T * C, "grad_hidden"),
        "dgain": Guarded(4 * C, "d_rms_gain"),
    }
    wbytes = 4 if flags & B.FLAG_DW_FP32 else 2
    wdt = torch.float32 if flags & B.FLAG_DW_FP32 else torch.bfloat16
    for k in ("dwg", "dwu", "dwd"):
        g[k] = Guarded(wbytes * I * C, k)
    idx = g["idx"].typed(torch.int32, (T,))
    nr = g["nr"].typed(torch.int32, (1,))
    B.skipffn_compact(p.d_mask, idx, nr, None, g["compact_ws"].view)
    out = g["out"].typed(torch.bfloat16, (T, C))
    B.skipffn_forward(p.d_hidden, out, idx, R, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, rms_gain=p.d_gain,
                      num_retained=nr, saved=g["saved"].view, workspace=g["fwd_ws"].view,
                      flags=flags & B.FLAG_BALANCED_SPLIT)
    gh = g["gh"].typed(torch.bfloat16, (T, C))
    B.skipffn_backward(p.d_grad, gh, idx, R, p.d_wg, p.d_wu, p.d_wd, g["saved"].view,
                       g["dwg"].typed(wdt, (I, C)), g["dwu"].typed(wdt, (I, C)),
                       g["dwd"].typed(wdt, (C, I)), eps=w.eps, rms_gain=p.d_gain, num_retained=nr,
                       workspace=g["bwd_ws"].view, flags=flags,
                       d_rms_gain=g["dgain"].typed(torch.float32, (C,)))
    torch.cuda.synchronize()
    assert int(nr.item()) == R
    for v in g.values():
        v.check()
    # the outputs themselves were produced (finite), so the run was a real one
    assert torch.isfinite(out.float()).all() and torch.isfinite(gh.float()).all()


@pytest.mark.parametrize("S,n_lo,n_hi,C", [(5, 0, 70, 264), (33, 1, 300, 1024), (3, 500, 2100, 4096)])
def test_summary_stays_inside_its_buffers(S, n_lo, n_hi, C):
    print(f"guard bytes summary S={S} n in [{n_lo},{n_hi}] C={C}", flush=True)
    rng = np.random.default_rng(S * 7 + C)
    sizes = rng.integers(n_lo, n_hi + 1, S)
    sizes[0] = n_lo
    n_tok = int(sizes.sum())
    T = n_tok + 17
    seg = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    tok = rng.permutation(T)[:n_tok].astype(np.int32)
    hidden = (torch.randn(T, C, device="cuda") * 0.5).to(torch.bfloat16)
    wv = (torch.randn(C, device="cuda") * 0.05).to(torch.bfloat16)
    d_tok = torch.from_numpy(tok).cuda() if n_tok else torch.empty(0, dtype=torch.int32, device="cuda")
    d_seg = torch.from_numpy(seg).cuda()
    g = {
        "out": Guarded(2 * S * C, "summary out"),
        "saved": Guarded(max(B.skipffn_summary_saved_bytes(n_tok, S, C), 1), "summary saved"),
        "ws": Guarded(max(B.skipffn_summary_workspace_bytes(n_tok, S, C), 1), "summary workspace"),
        "gh": Guarded(2 * T * C, "grad_hidden"),
        "dw": Guarded(4 * C, "dw"),
    }
    out = g["out"].typed(torch.bfloat16, (S, C))
    B.skipffn_summary_forward(hidden, d_tok, d_seg, wv, out, saved=g["saved"].view, workspace=g["ws"].view)
    go = (torch.randn(S, C, device="cuda")).to(torch.bfloat16)
    gh = g["gh"].typed(torch.bfloat16, (T, C))
    gh.zero_()
    B.skipffn_summary_backward(hidden, d_tok, d_seg, wv, g["saved"].view, go, gh,
                               g["dw"].typed(torch.float32, (C,)), workspace=g["ws"].view)
    torch.cuda.synchronize()
    for v in g.values():
        v.check()


@pytest.mark.parametrize("sizes,C,k", [((1, 2, 77, 300), 264, 36), ((1500, 40), 1024, 144),
                                      ((4096,), 512, 64), ((0, 5), 256, 1)])
def test_token_merge_stays_inside_its_buffers(sizes, C, k):
    print(f"guard bytes merge sizes={sizes} C={C} k={k}", flush=True)
    n_tok, n_max, S = sum(sizes), max(sizes), len(sizes)
    seg = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int64)
    x = (torch.randn(n_tok, C, device="cuda")).to(torch.bfloat16)
    g = {
        "out": Guarded(2 * S * k * C, "merge out"),
        "kept": Guarded(4 * S * k, "kept_idx"),
        "assign": Guarded(4 * n_tok, "assign"),
        "avg": Guarded(4 * n_tok, "avg_sim"),
        "ws": Guarded(B.skipffn_token_merge_workspace_bytes(n_tok, n_max, C), "merge workspace"),
    }
    B.skipffn_token_merge(x, seg, k, g["out"].typed(torch.bfloat16, (S, k, C)),
                          g["kept"].typed(torch.int32, (S, k)), g["assign"].typed(torch.int32, (n_tok,)),
                          g["avg"].typed(torch.float32, (n_tok,)), workspace=g["ws"].view)
    gout = torch.randn(S, k, C, device="cuda").to(torch.bfloat16)
    g["gx"] = Guarded(2 * n_tok * C, "merge grad_x")
    B.skipffn_token_merge_backward(gout, seg, g["assign"].typed(torch.int32, (n_tok,)),
                                   g["gx"].typed(torch.bfloat16, (n_tok, C)))
    torch.cuda.synchronize()
    for v in g.values():
        v.check()


@pytest.mark.parametrize("lens,Cv,keep", [((576, 577, 0, 3), 1024, 144), ((20000, 17), 72, 5000)])
def test_selection_stays_inside_its_buffers(lens, Cv, keep):
    print(f"guard bytes select lens={lens} Cv={Cv} keep={keep}", flush=True)
    n, nb = sum(lens), len(lens)
    T = n + 2 * nb
    feat = torch.randn(n, Cv, device="cuda").to(torch.bfloat16)
    cls = torch.randn(nb, Cv, device="cuda").to(torch.bfloat16)
    off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
    pos = torch.from_numpy(np.sort(np.random.default_rng(n).permutation(T)[:n]).astype(np.int32)).cuda()
    g = {"mask": Guarded(n, "mask"), "sim": Guarded(4 * n, "sim"), "skip": Guarded(T, "skip_mask")}
    B.skipffn_select_retained(feat, cls, off, keep, g["mask"].view, g["sim"].typed(torch.float32, (n,)),
                              token_pos=pos, skip_mask=g["skip"].view)
    torch.cuda.synchronize()
    for v in g.values():
        v.check()
    assert int((g["mask"].view == 0).sum()) == sum(min(keep, l) for l in lens)


@pytest.mark.parametrize("slabs,T,R,D,dt", [(6, 1000, 333, 128, torch.bfloat16), (3, 257, 257, 40, torch.float16),
                                            (2, 4099, 1, 128, torch.bfloat16)])
def test_row_gathers_stay_inside_their_buffers(slabs, T, R, D, dt):
    print(f"guard bytes kv slabs={slabs} T={T} R={R} D={D}", flush=True)
    rng = np.random.default_rng(T + R)
    idx = torch.from_numpy(np.sort(rng.permutation(T)[:R]).astype(np.int32)).cuda()
    src = torch.randn(slabs, T, D, device="cuda").to(dt)
    gk = Guarded(2 * slabs * R * D, "kv dst")
    dst = gk.typed(dt, (slabs, R, D))
    B.skipffn_kv_compact(src, dst, idx, R)
    gr = Guarded(2 * R * D, "gathered rows")
    rows = gr.typed(dt, (R, D))
    B.skipffn_gather_rows(src[0], rows, idx, R)
    torch.cuda.synchronize()
    gk.check(); gr.check()
    assert torch.equal(dst, src[:, idx.long()]) and torch.equal(rows, src[0][idx.long()])
