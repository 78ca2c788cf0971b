"""The pieces composed the way Skip-Vision uses them for one prefill (Sections 4.1-4.3): pick the
retained visual tokens by similarity to the CLS token, write one summary token per image from all
of its visual tokens, compact the mask once, run a stack of Skip-FFN blocks in place on the
retained rows with the row count read on the device (no host round trip anywhere), and drop the
skipped tokens from a KV cache.  Checked against the same composition of the oracle; the one
floating-point decision (the selection) is compared in the kernel's precision, everything after
it follows the mask the GPU produced."""
import numpy as np
import pytest
import torch

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import binding as B
from helpers import REL_L2_TOL, bits_of, rel_l2, to_dev_bf16

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("visual,text,keep,C,I,Cv,layers", [((300, 411), (20, 35), (75, 103), 512, 1368, 256, 3),
                                                            ((576,) * 3, (40,) * 3, (144,) * 3, 1024, 2816, 1024, 2)],
                         ids=["ragged", "llava-like"])
def test_prefill_pipeline(visual, text, keep, C, I, Cv, layers):
    print(f"pipeline visual={visual} text={text} keep={keep} C={C} I={I} layers={layers}", flush=True)
    rng = np.random.default_rng(sum(visual) + C)
    nb = len(visual)
    # sequence b: [visual tokens][one summary token][text tokens]
    starts, vis_pos, sum_pos = [], [], []
    t = 0
    for b in range(nb):
        starts.append(t)
        vis_pos.append(np.arange(t, t + visual[b]))
        sum_pos.append(t + visual[b])
        t += visual[b] + 1 + text[b]
    T = t
    n_feat = sum(visual)
    seq_off = np.concatenate([[0], np.cumsum(visual)]).astype(np.int32)
    token_pos = np.concatenate(vis_pos).astype(np.int32)
    feat = O.f64_to_bf16_bits(rng.standard_normal((n_feat, Cv)))
    cls = O.f64_to_bf16_bits(rng.standard_normal((nb, Cv)))
    hidden = O.f64_to_bf16_bits(rng.standard_normal((T, C)))
    w_sum = O.f64_to_bf16_bits(rng.standard_normal(C) * 0.05)
    weights = [tuple(O.f64_to_bf16_bits(rng.standard_normal(shape) * 0.02)
                     for shape in ((I, C), (I, C), (C, I))) for _ in range(layers)]
    heads, D = 4, 64
    cache = O.f64_to_bf16_bits(rng.standard_normal((layers, 2, heads, T, D)))

    # ---- GPU ----
    d_hidden = to_dev_bf16(hidden)
    d_keep = torch.from_numpy(np.asarray(keep, dtype=np.int32)).cuda()
    d_off = torch.from_numpy(seq_off).cuda()
    d_pos = torch.from_numpy(token_pos).cuda()
    mask = torch.empty(n_feat, dtype=torch.uint8, device="cuda")
    sim = torch.empty(n_feat, dtype=torch.float32, device="cuda")
    skip = torch.zeros(T, dtype=torch.uint8, device="cuda")            # summary and text: retained
    B.skipffn_select_retained(to_dev_bf16(feat), to_dev_bf16(cls), d_off, d_keep, mask, sim,
                              token_pos=d_pos, skip_mask=skip)
    d_sum = torch.empty((nb, C), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(max(B.skipffn_summary_workspace_bytes(n_feat, nb, C), 16), dtype=torch.uint8, device="cuda")
    B.skipffn_summary_forward(d_hidden, d_pos, d_off, to_dev_bf16(w_sum), d_sum, workspace=ws)
    d_hidden[torch.tensor(sum_pos, device="cuda")] = d_sum            # placing the rows is the caller's job
    R_cap = T
    bufs = B.SkipFFNBuffers(T, R_cap, C, I, training=False)
    B.skipffn_compact(skip, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
    hidden0 = d_hidden.clone()
    for wg, wu, wd in weights:
        B.skipffn_forward(d_hidden, d_hidden, bufs.idx, None, to_dev_bf16(wg), to_dev_bf16(wu), to_dev_bf16(wd),
                          num_retained=bufs.num_retained, workspace=bufs.fwd_ws)
    d_cache = to_dev_bf16(cache)
    R_want = sum(keep) + nb + sum(text)
    # the row count lives on the device, so the compacted cache keeps the prefill capacity T
    d_small = torch.full((layers, 2, heads, T, D), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.skipffn_kv_compact(d_cache, d_small, bufs.idx, None, num_retained=bufs.num_retained)
    torch.cuda.synchronize()

    # ---- the selection, in the kernel's precision, and against fp64 where the margin is clear ----
    g_mask, g_sim, g_skip = mask.cpu().numpy(), sim.cpu().numpy(), skip.cpu().numpy()
    ref_sel = O.select_retained(feat, cls, seq_off, np.asarray(keep))
    assert np.allclose(g_sim, ref_sel["sim"], rtol=0, atol=2e-5)
    for b in range(nb):
        lo, hi = seq_off[b], seq_off[b + 1]
        assert np.array_equal(g_mask[lo:hi], O.select_top_n(g_sim[lo:hi], keep[b]))
        s64 = np.sort(ref_sel["sim"][lo:hi])[::-1]
        if s64[keep[b] - 1] - s64[keep[b]] > 1e-4:
            assert np.array_equal(g_mask[lo:hi], ref_sel["mask"][lo:hi])
    want_skip = np.zeros(T, np.uint8)
    want_skip[token_pos] = g_mask
    assert np.array_equal(g_skip, want_skip)
    idx, R, _ = O.compact(g_skip)
    assert int(bufs.num_retained.item()) == R == R_want
    assert np.array_equal(bufs.idx[:R].cpu().numpy(), idx)

    # ---- the summary rows ----
    ref_sum = O.summary_forward(hidden, token_pos, seq_off, w_sum)
    assert rel_l2(O.bf16_bits_to_f64(bits_of(d_sum)), ref_sum["xs"]) < REL_L2_TOL

    # ---- the stack: the oracle starts from the hidden states the GPU stack started from ----
    h = bits_of(hidden0)
    for wg, wu, wd in weights:
        h = O.skipffn_forward(h, g_skip, wg, wu, wd)["out_bits"]
    got = bits_of(d_hidden)
    skipped = g_skip != 0
    assert np.array_equal(got[skipped], bits_of(hidden0)[skipped])      # never touched
    assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(h[idx])) < REL_L2_TOL

    # ---- the cache without the skipped tokens ----
    assert np.array_equal(bits_of(d_small[..., :R, :]), O.kv_skip_cache_all(cache, g_skip))
    assert bool(torch.isnan(d_small[..., R:, :]).all())                 # rows past R untouched


def test_training_step_pipeline():
    """One training step through the same pieces: summary token written into the sequence, two
    Skip-FFN blocks forward with saved activations, backward through both, and the gradient at the
    summary position sent back through the summary layer into the visual tokens and its weight."""
    visual, text, keep, C, I, layers = (300, 411), (20, 35), (75, 103), 512, 1368, 2
    print(f"training pipeline visual={visual} text={text} keep={keep} C={C} I={I} layers={layers}", flush=True)
    rng = np.random.default_rng(77)
    nb = len(visual)
    vis_pos, sum_pos, skip_np = [], [], []
    t = 0
    for b in range(nb):
        vis_pos.append(np.arange(t, t + visual[b]))
        m = np.ones(visual[b], np.uint8)
        m[rng.permutation(visual[b])[:keep[b]]] = 0
        skip_np += [m, np.zeros(1 + text[b], np.uint8)]
        sum_pos.append(t + visual[b])
        t += visual[b] + 1 + text[b]
    T = t
    skip_np = np.concatenate(skip_np)
    seg = np.concatenate([[0], np.cumsum(visual)]).astype(np.int32)
    tok = np.concatenate(vis_pos).astype(np.int32)
    hidden = O.f64_to_bf16_bits(rng.standard_normal((T, C)))
    grad_top = O.f64_to_bf16_bits(rng.standard_normal((T, C)))
    w_sum = O.f64_to_bf16_bits(rng.standard_normal(C) * 0.05)
    weights = [tuple(O.f64_to_bf16_bits(rng.standard_normal(shape) * 0.02)
                     for shape in ((I, C), (I, C), (C, I))) for _ in range(layers)]
    d_sum_pos = torch.tensor(sum_pos, device="cuda")

    # ---- GPU ----
    d_h0 = to_dev_bf16(hidden)
    d_tok, d_seg, d_wsum = torch.from_numpy(tok).cuda(), torch.from_numpy(seg).cuda(), to_dev_bf16(w_sum)
    n_tok = len(tok)
    sv_sum = torch.empty(B.skipffn_summary_saved_bytes(n_tok, nb, C), dtype=torch.uint8, device="cuda")
    ws_sum = torch.empty(B.skipffn_summary_workspace_bytes(n_tok, nb, C), dtype=torch.uint8, device="cuda")
    d_s = torch.empty((nb, C), dtype=torch.bfloat16, device="cuda")
    B.skipffn_summary_forward(d_h0, d_tok, d_seg, d_wsum, d_s, saved=sv_sum, workspace=ws_sum)
    d_h = d_h0.clone()
    d_h[d_sum_pos] = d_s
    d_skip = torch.from_numpy(skip_np).cuda()
    R = int((skip_np == 0).sum())
    bufs = [B.SkipFFNBuffers(T, R, C, I, training=True) for _ in range(layers)]
    B.skipffn_compact(d_skip, bufs[0].idx, bufs[0].num_retained, None, bufs[0].compact_ws)
    idx = bufs[0].idx
    dws = []
    d_w = [tuple(to_dev_bf16(a) for a in wl) for wl in weights]
    for l in range(layers):
        B.skipffn_forward(d_h, d_h, idx, R, *d_w[l], saved=bufs[l].saved, workspace=bufs[l].fwd_ws)
    d_g = to_dev_bf16(grad_top)
    for l in reversed(range(layers)):
        dw = [torch.empty((I, C), dtype=torch.float32, device="cuda"), torch.empty((I, C), dtype=torch.float32, device="cuda"),
              torch.empty((C, I), dtype=torch.float32, device="cuda")]
        B.skipffn_backward(d_g, d_g, idx, R, *d_w[l], bufs[l].saved, *dw, workspace=bufs[l].bwd_ws,
                           flags=B.FLAG_DW_FP32)
        dws.append(dw)
    dws.reverse()
    d_gs = d_g[d_sum_pos].contiguous()
    d_g[d_sum_pos] = 0                                  # the rows the summary replaced get no gradient
    d_dwsum = torch.empty(C, dtype=torch.float32, device="cuda")
    B.skipffn_summary_backward(d_h0, d_tok, d_seg, d_wsum, sv_sum, d_gs, d_g, d_dwsum, workspace=ws_sum)
    torch.cuda.synchronize()

    # ---- the same composition of the oracle ----
    s = O.summary_forward(hidden, tok, seg, w_sum)
    h = hidden.copy()
    h[sum_pos] = s["out_bits"]
    hs = [h]
    for wl in weights:
        hs.append(O.skipffn_forward(hs[-1], skip_np, *wl)["out_bits"])
    g = grad_top
    ref_dw = []
    for l in reversed(range(layers)):
        b = O.skipffn_backward(hs[l], skip_np, *weights[l], g)
        ref_dw.append(b)
        g = b["dx_bits"]
    ref_dw.reverse()
    gs = g[sum_pos].copy()
    g = g.copy()
    g[sum_pos] = 0
    sb = O.summary_backward(hidden, tok, seg, w_sum, gs, g)

    assert rel_l2(O.bf16_bits_to_f64(bits_of(d_h)), O.bf16_bits_to_f64(hs[-1])) < REL_L2_TOL
    got_g = bits_of(d_g)
    assert rel_l2(O.bf16_bits_to_f64(got_g), O.bf16_bits_to_f64(sb["gh_bits"])) < REL_L2_TOL
    # the rows the summary tokens replaced carry exactly zero
    assert np.all(got_g[sum_pos] == 0)
    for l in range(layers):
        for name, got in zip(("dw_gate", "dw_up", "dw_down"), dws[l]):
            assert rel_l2(got.cpu().numpy().astype(np.float64), ref_dw[l][name]) < REL_L2_TOL, (l, name)
    assert rel_l2(d_dwsum.cpu().numpy().astype(np.float64), sb["dw"]) < 2 * REL_L2_TOL
