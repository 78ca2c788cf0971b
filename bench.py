#!/usr/bin/env python3
"""Benchmark of the Skip-FFN block on one MI355X.

A step is one pass of the whole hot path over one synthetic batch: mask
compaction, gather + RMSNorm, gate/up GEMM + SiLU*mul, down GEMM + residual
scatter, and the backward over retained rows (dX, dW_gate, dW_up, dW_down).
Inputs are resident in HBM before the timed region starts.  One JSON line is
printed: metric / value / unit / ms_per_step, the workload in `config`, `roofline` for the
kernel class with the largest share of the step (algorithmic FLOPs or bytes over its average
HIP-event duration, against the published peak), `kernels` (every class the same way) and
`cpu_baseline` (the fp64 numpy oracle timed on the host cores).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 5] [--passes fwd+bwd]

The default workload is the largest single-GPU forward+backward configuration: 32 stacked
layers at C=4096, I=14336 over 16 sequences of 576 visual + 40 text tokens, 25 % of the visual
tokens retained (--config 1..4 select the others).
"""

from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# What the box itself reaches (profiles/bench_cfg2_fwd_bwd_hbm_traffic_and_mfma_counters.md): a
# register-only MFMA loop on random bf16 operands (the clock drops under the power cap), and a
# 1 GiB device copy (bench.py --sweep copy).  Context next to the published peaks, never `peak`.
MEASURED_MFMA_RANDOM_TFLOPS = 1900.0
MEASURED_COPY_GBS = 5000.0

# Bytes per launch that the L2s exchanged with the fabric / HBM come from the tracked profile of
# the same launch configuration: rocprofv3 --pmc FETCH_SIZE (x 2.0, calibrated with a copy kernel)
# + WRITE_SIZE, summarised per kernel class in profiles/bench_cfg<N>_<passes>_hbm_traffic_and_mfma_counters.md.
# Counters cannot be read from inside this process, so the figure is the profiled one.


def profiled_traffic(cfg, passes):
    """{kernel class: bytes per launch} from the tracked counter summary of this workload, or
    {} when there is none.  Table rows read  | kernel | class | fetched MB | written MB | ..."""
    name = f"bench_cfg{cfg}_{passes.replace('+', '_')}_hbm_traffic_and_mfma_counters.md"
    path = os.path.join(ROOT, "profiles", name)
    out = {}
    if not os.path.exists(path):
        return out
    with open(path) as f:
        for line in f:
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) < 4 or not line.lstrip().startswith("|"):
                continue
            if cells[1] in out:          # the traffic table comes first; later tables repeat the class column
                continue
            try:
                float(cells[1])
                continue                 # a table without the class column
            except ValueError:
                pass
            try:
                out[cells[1]] = (float(cells[2]) + float(cells[3])) * 1e6
            except ValueError:
                continue
    return out


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5,
                    help="workload 1..5 (token mix and layer shape); the default, 5, is the largest "
                         "forward+backward configuration: 32 layers, forward 1..32 then backward 32..1")
    ap.add_argument("--sweep", default=None, choices=["retention", "rows", "compact", "kv", "summary", "select", "merge", "copy", "mfma", "prefill"],
                    help="retention: time the step at retained fractions 0, 1/8, 1/4, 1/2, 1 of the visual "
                         "tokens at the configuration's fixed T; rows: the step (one layer) at retained counts "
                         "around multiples of the 256-row tile height, T = 16384; compact: the mask compaction alone at "
                         "T = 2^16 .. 2^26; kv: the skip KV-cache compaction of a whole LLaMA-3-8B cache "
                         "(32 layers x key/value x 8 heads x 128) for the token mixes of configurations "
                         "2, 3 and 5; summary: the adaptive summary layer, forward and backward, on "
                         "the visual token sets of the same mixes.  The JSON line then carries a 'sweep' array")
    ap.add_argument("--passes", default="fwd+bwd", choices=["fwd", "fwd+bwd"])
    ap.add_argument("--structured", action="store_true",
                    help="configuration 3 only: retain the leading 576 visual tokens of every sequence (the "
                         "global view of a high-resolution image) instead of seeded-random positions")
    ap.add_argument("--out-of-place", action="store_true",
                    help="write to separate output / gradient tensors: skipped rows are then byte-copied "
                         "by the passthrough kernel (in place they cost nothing)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays (the per-kernel events "
                         "still come from eager launches)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle leg")
    return ap.parse_args()


def kernel_work(name, R, T, C, I, dw_bytes):
    """(kind, algorithmic amount per launch): flops for the MFMA kernels, bytes for
    the HBM-bound ones."""
    rc, ri = R * C, R * I
    table = {
        "gemm_gate_up_swiglu": ("mfma", 4 * R * C * I),
        "gemm_down": ("mfma", 2 * R * C * I),
        "gemm_dh_swiglu_bwd+dw_down": ("mfma", 4 * R * C * I),    # two GEMMs in one grid
        "gemm_dw_gate_up": ("mfma", 4 * R * C * I),               # dW_gate and dW_up in one grid
        "gemm_dxn": ("mfma", 4 * R * C * I),
        "compact": ("hbm", T + 4 * R),
        "gather_rmsnorm": ("hbm", 2 * rc * 2 + 4 * R),
        "resid_scatter": ("hbm", 2 * rc * 2),
        "gather_rows": ("hbm", 2.5 * rc * 2),                     # row gather + transposed copy
        "rmsnorm_bwd_scatter": ("hbm", rc * (2 + 2 + 4 + 2)),
        "passthrough_copy": ("hbm", 2 * (T - R) * C * 2),
    }
    return table.get(name, ("hbm", 0))


def cpu_baseline(w, passes, target_s):
    """The oracle, as it stands, on a bounded sample of the same workload: the
    first sequences of the batch (all of their tokens), sized for ~target_s."""
    from oracle import skipffn_oracle as O
    from paper_2503_21817_amd import workloads as W
    from paper_2503_21817_amd.flopmodel import skipffn_flops
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    mask, hidden, grad = W.make_mask(w), W.make_hidden(w), W.make_grad(w)
    wg, wu, wd = W.make_weights(w)
    lens = [v + t for v, t in zip(w.visual, w.text)]

    def run(nseq):
        n = sum(lens[:nseq])
        t0 = time.perf_counter()
        O.skipffn_forward(hidden[:n], mask[:n], wg, wu, wd, None, w.eps)
        if passes == "fwd+bwd":
            O.skipffn_backward(hidden[:n], mask[:n], wg, wu, wd, grad[:n], None, w.eps)
        dt = time.perf_counter() - t0
        R = int((mask[:n] == 0).sum())
        return dt, n, R

    dt1, n1, R1 = run(1)
    nseq = 1
    if len(lens) > 1 and dt1 < target_s / 2:
        nseq = int(min(len(lens), max(1, target_s // max(dt1, 1e-3))))
    dt, n, R = (dt1, n1, R1) if nseq == 1 else run(nseq)
    reps = 1
    if nseq == len(lens) and dt < target_s / 2:
        # the whole batch is quicker than the target: repeat it
        extra = int(min(10, target_s // max(dt, 1e-3)))
        for _ in range(extra):
            dt += run(nseq)[0]
        reps += extra
    flops = reps * skipffn_flops(R, w.C, w.I, passes == "fwd+bwd")
    rec = {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
           "cpu_model": cpu_model(),
           "sample": f"first {nseq} of {len(lens)} sequences ({n} tokens, {R} retained), "
                     f"{'one layer of ' + str(w.layers) + ', ' if w.layers > 1 else ''}{passes}, fp64 numpy, {reps} pass(es), {dt:.1f} s",
           "seconds": dt, "retained_tokens_per_s": reps * R / dt}
    # the whole step at that rate (all sequences, all layers): extrapolated, not run
    full = w.layers * skipffn_flops(w.R, w.C, w.I, passes == "fwd+bwd")
    rec["extrapolated_step_seconds"] = full / (flops / dt)
    return rec


def _time_steps(torch, fn, warmup, steps):
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        fn(warmup + i)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def retention_sweep(torch, B, W, w, bwd, args):
    """Step time against the retained share of the visual tokens at fixed T (Section 5.2's
    cost model is linear in the retained count): one entry per fraction and a least-squares
    line  ms = intercept + slope * R."""
    from dataclasses import replace
    from paper_2503_21817_amd.flopmodel import skipffn_flops

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    T, C, I = w.T, w.C, w.I
    hidden0 = dev_bf16(W.make_hidden(w))
    grad0 = dev_bf16(W.make_grad(w))
    wg, wu, wd = (dev_bf16(a) for a in W.make_weights(w))
    dws = [torch.empty(shape, dtype=torch.bfloat16, device="cuda") for shape in ((I, C), (I, C), (C, I))]
    bufs = B.SkipFFNBuffers(T, T, C, I, training=bwd)
    ncopy = 8
    hiddens = [hidden0.clone() for _ in range(ncopy)]
    grads = [grad0.clone() for _ in range(ncopy)]
    rows = []
    for frac in (0.0, 0.125, 0.25, 0.5, 1.0):
        wf = replace(w, keep=[int(round(frac * v)) for v in w.visual], text=list(w.text))
        # fraction 0 also drops the text tokens from the FFN: the empty-set path of the block
        mask_np = W.make_mask(wf)
        if frac == 0.0:
            mask_np[:] = 1
        mask = torch.from_numpy(mask_np).cuda()
        R = int((mask_np == 0).sum())

        def step(i):
            h = hiddens[i % ncopy]
            B.skipffn_compact(mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
            B.skipffn_forward(h, h, bufs.idx, R, wg, wu, wd, eps=w.eps, saved=bufs.saved,
                              workspace=bufs.fwd_ws)
            if bwd:
                g = grads[i % ncopy]
                B.skipffn_backward(g, g, bufs.idx, R, wg, wu, wd, bufs.saved, *dws, eps=w.eps,
                                   workspace=bufs.bwd_ws)

        ms = _time_steps(torch, step, args.warmup, args.steps)
        fl = skipffn_flops(R, C, I, bwd)
        rows.append({"retained_fraction_of_visual": frac, "R": R, "ms_per_step": round(ms, 4),
                     "tflops": round(fl / (ms * 1e-3) / 1e12, 1)})
    Rs = np.array([r["R"] for r in rows], dtype=np.float64)
    ms = np.array([r["ms_per_step"] for r in rows])
    slope, intercept = np.polyfit(Rs, ms, 1)
    return {"metric": "Skip-FFN step time against retained count", "unit": "ms", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"{w.name}: T={T} fixed, C={C}, I={I}, 1 layer, {args.passes}, "
                                   "in place"},
            "sweep": rows, "fit_ms": {"intercept": round(float(intercept), 4),
                                      "per_1000_retained": round(float(slope) * 1e3, 4)}}


def rows_sweep(torch, B, bwd, args):
    """One layer at C=4096, I=14336, T=16384 over retained counts just below, at and just above
    multiples of the 256-row tile height (and the configurations' own counts): how much a nearly
    empty last row of tiles costs."""
    from paper_2503_21817_amd.flopmodel import skipffn_flops
    C, I, T = 4096, 14336, 16384
    g = torch.Generator(device="cuda")
    g.manual_seed(4200)
    hid = torch.randn((T, C), generator=g, device="cuda").to(torch.bfloat16)
    grad = torch.randn((T, C), generator=g, device="cuda").to(torch.bfloat16)
    ws = [(torch.randn(shape, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
          for shape in ((I, C), (I, C), (C, I))]
    dws = [torch.empty_like(w) for w in ws]
    rows = []
    for R in (1280, 1288, 1344, 1408, 1472, 1536, 2560, 2568, 2624, 2688, 2752, 2816, 2944, 3072, 3080, 4096, 4104,
              4224, 8192, 8200, 9623):
        mask = torch.ones(T, dtype=torch.uint8, device="cuda")
        mask[torch.randperm(T, generator=g, device="cuda")[:R]] = 0
        bufs = B.SkipFFNBuffers(T, R, C, I, training=bwd)
        h, gg = hid.clone(), grad.clone()

        def step(i):
            B.skipffn_compact(mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
            B.skipffn_forward(h, h, bufs.idx, R, *ws, saved=bufs.saved, workspace=bufs.fwd_ws)
            if bwd:
                B.skipffn_backward(gg, gg, bufs.idx, R, *ws, bufs.saved, *dws, workspace=bufs.bwd_ws)

        ms = _time_steps(torch, step, args.warmup, args.steps)
        rows.append({"R": R, "tile_rows": round(R / 256, 3), "ms_per_step": round(ms, 4),
                     "tflops": round(skipffn_flops(R, C, I, bwd) / (ms * 1e-3) / 1e12, 1),
                     "us_per_retained_row": round(ms * 1e3 / R, 4)})
        del bufs
    return {"metric": "Skip-FFN step time against retained count around tile-row multiples", "unit": "ms",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": f"T={T} fixed, C={C}, I={I}, 1 layer, {args.passes}, in place"}, "sweep": rows}


def prefill_sweep(torch, B, args):
    """Inference prefill of one Skip-FFN block (forward only, nothing saved, in place) at small
    batches: LLaVA-shaped sequences of 576 visual + 40 text tokens with 144 visual tokens
    retained, and one LLaVA-HD sequence (2880 + 64 tokens, 576 retained).  With few rows the
    block is bound by streaming the 352 MB of weights once, so the rate at which it does that is
    reported next to the time."""
    C, I = 4096, 14336
    g = torch.Generator(device="cuda")
    g.manual_seed(4100)
    ws = [(torch.randn(shape, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
          for shape in ((I, C), (I, C), (C, I))]
    rows = []
    for name, nseq, V, Tx, keep in (("llava-b1-keep64", 1, 576, 40, 64), ("llava-b1", 1, 576, 40, 144),
                                    ("llava-b2", 2, 576, 40, 144),
                                    ("llava-b4", 4, 576, 40, 144), ("llava-b8", 8, 576, 40, 144),
                                    ("llava-hd-b1", 1, 2880, 64, 576)):
        T, R = nseq * (V + Tx), nseq * (keep + Tx)
        mask_np = np.ones(T, np.uint8)
        rng = np.random.default_rng(4100 + T)
        for b in range(nseq):
            base = b * (V + Tx)
            mask_np[base + rng.choice(V, size=keep, replace=False)] = 0
            mask_np[base + V:base + V + Tx] = 0
        mask = torch.from_numpy(mask_np).cuda()
        hidden = torch.randn((T, C), generator=g, device="cuda").to(torch.bfloat16)
        copies = [hidden.clone() for _ in range(4)]
        bufs = B.SkipFFNBuffers(T, R, C, I, training=False)

        def step(i):
            h = copies[i % 4]
            B.skipffn_compact(mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
            B.skipffn_forward(h, h, bufs.idx, R, *ws, workspace=bufs.fwd_ws)

        ms = _time_steps(torch, step, args.warmup, args.steps)
        rows.append({"workload": name, "T": T, "R": R, "us": round(ms * 1e3, 1),
                     "tflops": round(6.0 * R * C * I / (ms * 1e-3) / 1e12, 1),
                     "weights_tbs": round(3.0 * C * I * 2 / (ms * 1e-3) / 1e12, 2)})
    return {"metric": "Skip-FFN prefill (forward only) time", "unit": "us", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "C=4096, I=14336, 1 layer, forward only, in place, nothing saved"},
            "sweep": rows}


def compact_sweep(torch, B, args):
    """The mask compaction alone, 25 % retained at seeded-uniform positions: algorithmic
    bytes T (mask) + 4 R (index list) per launch against HIP-event time."""
    rows = []
    for lg in (13, 16, 20, 24, 26):
        T = 1 << lg
        g = torch.Generator(device="cuda")
        g.manual_seed(77 + lg)
        mask = (torch.rand(T, generator=g, device="cuda") >= 0.25).to(torch.uint8)
        idx = torch.empty(T, dtype=torch.int32, device="cuda")
        nret = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(max(B.skipffn_compact_workspace_bytes(T), 16), dtype=torch.uint8, device="cuda")
        for _ in range(args.warmup):
            B.skipffn_compact(mask, idx, nret, None, ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            B.skipffn_compact(mask, idx, nret, None, ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        R = int(nret.item())
        assert R == int((mask == 0).sum().item())
        gbs = (T + 4 * R) / (ms * 1e-3) / 1e9
        rows.append({"T": T, "R": R, "us": round(ms * 1e3, 2), "gbs": round(gbs, 1),
                     "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)})
    return {"metric": "mask compaction bandwidth", "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "mask compaction, 25 % retained, T = 2^13 .. 2^26"}, "sweep": rows}


def summary_sweep(torch, B, W, args):
    """Adaptive summary layer (Section 4.2): per sequence one summary of the retained and one
    of the skipped visual tokens.  Algorithmic bytes: forward reads the listed rows once
    (n_tok * C * 2); backward reads them and reads + writes their gradient rows (3x)."""
    rows = []
    for cfg in (2, 3, 5):
        w = W.config(cfg)
        T, C = w.T, w.C
        tok_np, seg_np = W.make_summary_sets(w)
        n_tok, S = len(tok_np), len(seg_np) - 1
        g = torch.Generator(device="cuda")
        g.manual_seed(600 + cfg)
        hid = torch.randn((T, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        gh = torch.randn((T, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        gout = torch.randn((S, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        wv = torch.from_numpy(W.make_summary_weight(w).view(np.int16)).cuda().view(torch.bfloat16)
        tok = torch.from_numpy(tok_np).cuda()
        seg = torch.from_numpy(seg_np).cuda()
        out = torch.empty((S, C), dtype=torch.bfloat16, device="cuda")
        dw = torch.empty(C, dtype=torch.float32, device="cuda")
        sv = torch.empty(B.skipffn_summary_saved_bytes(n_tok, S, C), dtype=torch.uint8, device="cuda")
        ws = torch.empty(B.skipffn_summary_workspace_bytes(n_tok, S, C), dtype=torch.uint8, device="cuda")

        def timed(fn):
            for _ in range(args.warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(args.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / args.steps

        ms_f = timed(lambda: B.skipffn_summary_forward(hid, tok, seg, wv, out, saved=sv, workspace=ws))
        ms_b = timed(lambda: B.skipffn_summary_backward(hid, tok, seg, wv, sv, gout, gh, dw, workspace=ws))
        bf, bb = n_tok * C * 2, 3 * n_tok * C * 2
        rows.append({"workload": w.name, "n_tok": n_tok, "sets": S,
                     "fwd_us": round(ms_f * 1e3, 1), "fwd_gbs": round(bf / (ms_f * 1e-3) / 1e9, 1),
                     "bwd_us": round(ms_b * 1e3, 1), "bwd_gbs": round(bb / (ms_b * 1e-3) / 1e9, 1),
                     "fwd_frac_hbm_peak": round(bf / (ms_f * 1e-3) / 1e9 / PEAK_HBM_GBS, 4),
                     "bwd_frac_hbm_peak": round(bb / (ms_b * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)})
    return {"metric": "adaptive summary layer bandwidth", "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "dtype": "bf16 in, f32 arithmetic",
            "data": "synthetic",
            "config": {"workload": "retained and skipped visual token sets of configurations 2, 3, 5, C=4096"},
            "sweep": rows}


def select_sweep(torch, B, W, args):
    """Retained-token selection (Section 4.1): cosine similarity of every visual token to its
    sequence's CLS token, then the top-n rank count.  Vision width 1024 (the paper's ViT-L
    class encoders); algorithmic bytes = one read of the features, n_feat * Cv * 2."""
    rows = []
    Cv = 1024
    for cfg in (2, 3, 5):
        w = W.config(cfg)
        lens = list(w.visual)
        n = sum(lens)
        g = torch.Generator(device="cuda")
        g.manual_seed(700 + cfg)
        feat = torch.randn((n, Cv), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        cls = torch.randn((len(lens), Cv), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        off = torch.from_numpy(np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)).cuda()
        keep = torch.from_numpy(np.asarray(w.keep, dtype=np.int32)).cuda()
        mask = torch.empty(n, dtype=torch.uint8, device="cuda")
        sim = torch.empty(n, dtype=torch.float32, device="cuda")
        for _ in range(args.warmup):
            B.skipffn_select_retained(feat, cls, off, keep, mask, sim)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            B.skipffn_select_retained(feat, cls, off, keep, mask, sim)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        assert int((mask == 0).sum().item()) == sum(w.keep)
        gbs = n * Cv * 2 / (ms * 1e-3) / 1e9
        rows.append({"workload": w.name, "n_feat": n, "sequences": len(lens), "us": round(ms * 1e3, 1),
                     "gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)})
    return {"metric": "retained-token selection", "unit": "us", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "dtype": "bf16 in, f32 similarities", "data": "synthetic",
            "config": {"workload": "visual tokens of configurations 2, 3, 5, vision width 1024"},
            "sweep": rows}


def merge_sweep(torch, B, args):
    """Token merge (Section 4.1): sets of 1024 local tokens reduced to 256 (the paper's ablation
    setting), 8 and 32 sets, vision width 1024 and backbone width 4096.  The similarity GEMMs
    are 2 * n^2 * C FLOP per set; the rest is memory-bound."""
    rows = []
    n, k = 1024, 256
    for S, C in ((8, 1024), (32, 1024), (8, 4096)):
        g = torch.Generator(device="cuda")
        g.manual_seed(800 + S + C)
        x = torch.randn((S * n, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        seg = [i * n for i in range(S + 1)]
        out = torch.empty((S, k, C), dtype=torch.bfloat16, device="cuda")
        kept = torch.empty((S, k), dtype=torch.int32, device="cuda")
        assign = torch.empty(S * n, dtype=torch.int32, device="cuda")
        avg = torch.empty(S * n, dtype=torch.float32, device="cuda")
        ws = torch.empty(B.skipffn_token_merge_workspace_bytes(S * n, n, C), dtype=torch.uint8, device="cuda")
        for _ in range(args.warmup):
            B.skipffn_token_merge(x, seg, k, out, kept, assign, avg, workspace=ws)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            B.skipffn_token_merge(x, seg, k, out, kept, assign, avg, workspace=ws)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        assert int((kept >= 0).sum().item()) == S * k
        gout = torch.randn((S, k, C), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        gx = torch.empty_like(x)
        for _ in range(args.warmup):
            B.skipffn_token_merge_backward(gout, seg, assign, gx)
        e0.record()
        for _ in range(args.steps):
            B.skipffn_token_merge_backward(gout, seg, assign, gx)
        e1.record()
        torch.cuda.synchronize()
        ms_b = e0.elapsed_time(e1) / args.steps
        bwd_bytes = (S * k + S * n) * C * 2.0          # read each slot gradient once, write every row
        rows.append({"sets": S, "tokens_per_set": n, "kept": k, "C": C, "us": round(ms * 1e3, 1),
                     "us_per_set": round(ms * 1e3 / S, 1),
                     "similarity_gemm_gflop": round(2 * n * n * C * S / 1e9, 1),
                     "bwd_us": round(ms_b * 1e3, 1), "bwd_gbs": round(bwd_bytes / (ms_b * 1e-3) / 1e9, 1)})
    return {"metric": "token merge", "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "dtype": "bf16 in, f32 similarities", "data": "synthetic",
            "config": {"workload": "1024 -> 256 tokens per set"}, "sweep": rows}


def mfma_probe(torch, B, random_operands, iters, steps, warmup, blocks=512):
    """One figure of the register-only MFMA loop: 2 workgroups of 4 wavefronts per CU, operands in
    registers, no memory traffic."""
    out = torch.empty(blocks * 256, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(2 * blocks, dtype=torch.int64, device="cuda")
    for _ in range(max(warmup, 1)):
        B.skipffn_probe_mfma(blocks, iters, random_operands, out, clocks)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(steps):
        B.skipffn_probe_mfma(blocks, iters, random_operands, out, clocks)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / steps
    flops = blocks * 4 * iters * 32 * 16384.0
    c = clocks.view(blocks, 2).double()
    ghz = float((c[:, 0].sum() / c[:, 1].sum()).item()) * 0.1       # cycles per 10 ns tick
    return {"operands": "random bf16" if random_operands else "constant 1.0",
            "ms": round(ms, 3), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
            "frac_published_peak": round(flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "shader_clock_ghz": round(ghz, 3)}


def mfma_sweep(torch, B, args):
    """What the matrix cores of this machine sustain with operands in registers (no memory traffic):
    constant operands, then pseudo-random bf16 operands."""
    rows = [mfma_probe(torch, B, r, 20000, args.steps, args.warmup) for r in (0, 1)]
    return {"metric": "register-only MFMA loop", "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": "512 workgroups x 4 wavefronts x 640000 v_mfma_f32_16x16x32_bf16"},
            "sweep": rows}


def copy_sweep(torch, args):
    """A plain device copy of 1 GiB (read 1 GiB, write 1 GiB): the HBM rate this machine reaches,
    next to the published 8 TB/s, and the kernel of known size that the FETCH_SIZE / WRITE_SIZE
    counters are calibrated with."""
    n = 1 << 30
    src = torch.full((n,), 1, dtype=torch.uint8, device="cuda")
    dst = torch.full((n,), 2, dtype=torch.uint8, device="cuda")
    for _ in range(args.warmup):
        dst.copy_(src)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.steps):
        dst.copy_(src)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.steps
    gbs = 2 * n / (ms * 1e-3) / 1e9
    return {"metric": "device copy bandwidth (read + write)", "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "dtype": "u8", "data": "synthetic",
            "config": {"workload": "1 GiB device-to-device copy"}, "us": round(ms * 1e3, 1),
            "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)}


def kv_sweep(torch, B, W, args):
    """Skip KV-cache (Section 4.3) on a packed cache [layers, 2, kv heads, T, head dim] of the
    backbone (32 x 2 x 8 x T x 128, bf16): algorithmic bytes = read + write of the retained
    rows, 2 * slabs * R * 256 B, against HIP-event time."""
    rows = []
    L, H, D = 32, 8, 128
    for cfg in (2, 3, 5):
        w = W.config(cfg)
        T, R = w.T, w.R
        mask = torch.from_numpy(W.make_mask(w)).cuda()
        idx = torch.empty(T, dtype=torch.int32, device="cuda")
        nret = torch.zeros(1, dtype=torch.int32, device="cuda")
        ws = torch.empty(max(B.skipffn_compact_workspace_bytes(T), 16), dtype=torch.uint8, device="cuda")
        B.skipffn_compact(mask, idx, nret, None, ws)
        g = torch.Generator(device="cuda")
        g.manual_seed(500 + cfg)
        src = torch.randn((L, 2, H, T, D), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
        dst = torch.empty((L, 2, H, R, D), dtype=torch.bfloat16, device="cuda")
        for _ in range(args.warmup):
            B.skipffn_kv_compact(src, dst, idx, R)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            B.skipffn_kv_compact(src, dst, idx, R)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / args.steps
        assert torch.equal(dst[3, 1, 5], src[3, 1, 5][idx[:R].long()])
        nbytes = 2 * L * 2 * H * R * D * 2
        gbs = nbytes / (ms * 1e-3) / 1e9
        rows.append({"workload": w.name, "T": T, "R": R, "cache_MB": round(src.numel() * 2 / 1e6, 1),
                     "us": round(ms * 1e3, 1), "gbs": round(gbs, 1), "frac_hbm_peak": round(gbs / PEAK_HBM_GBS, 4)})
        del src, dst
    return {"metric": "skip KV-cache compaction bandwidth", "unit": "GB/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "dtype": "bf16 (bit copy)", "data": "synthetic",
            "config": {"workload": "LLaMA-3-8B cache, packed batch, token mixes of configurations 2, 3, 5"},
            "sweep": rows}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the Skip-FFN block of one data-parallel rank); "
              "--gpus N with N > 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2503_21817_amd import binding as B
    from paper_2503_21817_amd import workloads as W
    from paper_2503_21817_amd.flopmodel import skipffn_flops

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()   # fail loudly if the HIP library is missing

    w = W.config(args.config, structured=args.structured) if args.config == 3 else W.config(args.config)
    bwd = args.passes == "fwd+bwd"
    if args.sweep == "rows":
        print(json.dumps(rows_sweep(torch, B, bwd, args)))
        return
    if args.sweep == "compact":
        print(json.dumps(compact_sweep(torch, B, args)))
        return
    if args.sweep == "mfma":
        print(json.dumps(mfma_sweep(torch, B, args)))
        return
    if args.sweep == "prefill":
        print(json.dumps(prefill_sweep(torch, B, args)))
        return
    if args.sweep == "copy":
        print(json.dumps(copy_sweep(torch, args)))
        return
    if args.sweep == "merge":
        print(json.dumps(merge_sweep(torch, B, args)))
        return
    if args.sweep == "select":
        print(json.dumps(select_sweep(torch, B, W, args)))
        return
    if args.sweep == "summary":
        print(json.dumps(summary_sweep(torch, B, W, args)))
        return
    if args.sweep == "kv":
        print(json.dumps(kv_sweep(torch, B, W, args)))
        return
    if args.sweep == "retention":
        print(json.dumps(retention_sweep(torch, B, W, w, bwd, args)))
        return
    T, R, C, I = w.T, w.R, w.C, w.I
    L = w.layers

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    mask = torch.from_numpy(W.make_mask(w)).cuda()
    hidden0 = dev_bf16(W.make_hidden(w))
    grad0 = dev_bf16(W.make_grad(w))
    if L == 1:
        weights = [tuple(dev_bf16(a) for a in W.make_weights(w))]
        data = "synthetic"
    else:
        # 32 layers of independent N(0, 0.02) weights, drawn on the device (seeded): the host
        # generator of the parity tests would hold the GPU idle for minutes
        gen = torch.Generator(device="cuda")
        weights = []
        for l in range(L):
            gen.manual_seed(2000 + w.cfg * 100 + l)
            weights.append(tuple(
                (torch.randn(shape, generator=gen, device="cuda", dtype=torch.float32) * 0.02)
                .to(torch.bfloat16) for shape in ((I, C), (I, C), (C, I))))
        data = "synthetic (weights drawn on the device)"
    bufs = B.SkipFFNBuffers(T, R, C, I, training=bwd)
    saved = [bufs.saved] + [torch.empty_like(bufs.saved) for _ in range(L - 1)] if bwd else [None] * L
    dws = [tuple(torch.empty(shape, dtype=torch.bfloat16, device="cuda")
                 for shape in ((I, C), (I, C), (C, I))) for _ in range(L)] if bwd else []

    # The block runs in place (skipped rows are never touched); rotate through
    # fresh copies of the input so values do not drift from step to step.
    ncopy = min(args.steps + args.warmup, 32)
    hiddens = [hidden0.clone() for _ in range(ncopy)]
    grads = [grad0.clone() for _ in range(ncopy)] if bwd else []

    oop = args.out_of_place
    out_buf = torch.empty_like(hidden0) if oop else None
    gout_buf = torch.empty_like(grad0) if (oop and bwd) else None

    def step(i):
        h = hiddens[i % ncopy]
        B.skipffn_compact(mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
        for l in range(L):
            wg, wu, wd = weights[l]
            B.skipffn_forward(h, out_buf if oop else h, bufs.idx, R, wg, wu, wd, eps=w.eps, saved=saved[l],
                              workspace=bufs.fwd_ws)
        if bwd:
            g = grads[i % ncopy]
            for l in reversed(range(L)):
                wg, wu, wd = weights[l]
                B.skipffn_backward(g, gout_buf if oop else g, bufs.idx, R, wg, wu, wd, saved[l], *dws[l],
                                   eps=w.eps, workspace=bufs.bwd_ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph:
        # one graph per input copy would be needed to rotate inputs; replaying on one copy lets
        # values drift in place, which does not change the work done
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step(0)
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step(0)
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_step = dt / args.steps * 1e3

    # Per-kernel durations: HIP events recorded by the library around every
    # launch, on the stream the kernels run on, over the same K steps.
    for i in range(ncopy):
        hiddens[i].copy_(hidden0)
        if bwd:
            grads[i].copy_(grad0)
    torch.cuda.synchronize()
    B.skipffn_profile_begin()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    ms_step_prof = (time.perf_counter() - t0) / args.steps * 1e3
    prof = B.skipffn_profile_end()

    kernels = {}
    for name, (ms, n) in prof.items():
        kind, amount = kernel_work(name, R, T, C, I, 2)
        avg = ms / n
        e = {"avg_ms": round(avg, 5), "launches_per_step": n / args.steps}
        if amount and avg > 0:
            if kind == "mfma":
                e["tflops"] = round(amount / (avg * 1e-3) / 1e12, 1)
                e["frac_peak"] = round(e["tflops"] / PEAK_BF16_TFLOPS, 4)
            else:
                e["gbs"] = round(amount / (avg * 1e-3) / 1e9, 1)
                e["frac_peak"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
        e["ms_per_step"] = round(ms / args.steps, 5)
        kernels[name] = e
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    kind, amount = kernel_work(dom, R, T, C, I, 2)
    dom_avg_s = kernels[dom]["avg_ms"] * 1e-3
    if kind == "mfma":
        achieved, peak, unit = amount / dom_avg_s / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
    else:
        achieved, peak, unit = amount / dom_avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
    roofline = {"kernel": dom, "bound": kind, "achieved": round(achieved, 2), "peak": peak,
                "unit": unit, "frac": round(achieved / peak, 4),
                "traffic": (None if oop or args.graph else profiled_traffic(args.config, args.passes).get(dom)),
                "avg_launch_ms": kernels[dom]["avg_ms"],
                "frac_of_measured_ceiling": round(achieved / (MEASURED_MFMA_RANDOM_TFLOPS if kind == "mfma"
                                                              else MEASURED_COPY_GBS), 4)}
    if kind == "mfma":
        # the ceiling of THIS box, measured right after the timed region while the chip is warm:
        # a register-only MFMA loop on random bf16 operands (no memory traffic at all)
        live = mfma_probe(torch, B, 1, 8000, steps=3, warmup=1)
        roofline["measured_ceiling"] = live["tflops"]
        roofline["measured_ceiling_clock_ghz"] = live["shader_clock_ghz"]
        roofline["frac_of_measured_ceiling"] = round(achieved / live["tflops"], 4)
    gemm_ms = sum(v["ms_per_step"] for k, v in kernels.items() if k.startswith("gemm_"))

    flops = L * skipffn_flops(R, C, I, bwd)
    tflops = flops / (ms_step * 1e-3) / 1e12
    rec = {
        "metric": "retained-token FFN fwd+bwd TFLOP/s" if bwd else "retained-token FFN fwd TFLOP/s",
        "value": round(tflops, 2), "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": data,
        "config": {"workload": f"{w.name}: T={T} tokens, R={R} retained, C={C}, I={I}, "
                               f"{L} layer{'s' if L > 1 else ''}, {args.passes}, {'out of place' if oop else 'in place'}",
                   "T": T, "R": R, "C": C, "I": I, "layers": L, "passes": args.passes,
                   "launch": "hip graph replay" if args.graph else "eager"},
        "pct_bf16_mfma_peak": round(100 * tflops / PEAK_BF16_TFLOPS, 2),
        "gemm_only_tflops": round(flops / (gemm_ms * 1e-3) / 1e12, 2) if gemm_ms > 0 else None,
        "effective_tokens_per_s": round(T / (ms_step * 1e-3)),
        "retained_tokens_per_s": round(R / (ms_step * 1e-3)),
        "ms_per_step_with_events": round(ms_step_prof, 4),
        "roofline": roofline,
        "kernels": kernels,
    }
    if not args.no_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(w, args.passes, args.cpu_seconds)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
