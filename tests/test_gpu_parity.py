"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer / byte results are compared bit for bit;
floating-point results by relative L2 error over retained rows, bound 1e-2
(bf16 inputs, fp32 accumulation, bf16 intermediates)."""
import numpy as np
import pytest
import torch

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import binding as B
from paper_2503_21817_amd import workloads as W
from helpers import REL_L2_TOL, Problem, bits_of, f64_of, rel_l2, to_dev_bf16

pytestmark = pytest.mark.gpu


def run_compact(mask_np, want_pos=True):
    T = mask_np.shape[0]
    d_mask = torch.from_numpy(mask_np).cuda() if T else torch.empty(0, dtype=torch.uint8, device="cuda")
    idx = torch.full((max(T, 1),), -7, dtype=torch.int32, device="cuda")
    nr = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    pos = torch.full((max(T, 1),), -7, dtype=torch.int32, device="cuda") if want_pos else None
    ws = torch.empty(max(B.skipffn_compact_workspace_bytes(T), 16), dtype=torch.uint8, device="cuda")
    B.skipffn_compact(d_mask, idx, nr, pos, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), int(nr.item()), None if pos is None else pos.cpu().numpy()


@pytest.mark.parametrize("T", [0, 1, 3, 64, 255, 256, 257, 1000, 4097, 16384, 29411, 262144,
                               262145, 300001, (1 << 20) + 37])
@pytest.mark.parametrize("kind", ["rand", "all0", "all1", "alt", "ends", "bytes"])
def test_compact_bit_exact(T, kind):
    rng = np.random.default_rng(T + len(kind))
    if kind == "rand":
        m = (rng.random(T) < 0.7).astype(np.uint8)
    elif kind == "all0":
        m = np.zeros(T, np.uint8)
    elif kind == "all1":
        m = np.ones(T, np.uint8)
    elif kind == "alt":
        m = (np.arange(T) % 2).astype(np.uint8)
    elif kind == "ends":
        m = np.ones(T, np.uint8); m[:1] = 0; m[-1:] = 0
    else:
        m = (rng.integers(0, 256, T) * (rng.random(T) < 0.5)).astype(np.uint8)
    print(f"compact T={T} kind={kind}", flush=True)
    idx, R, pos = run_compact(m)
    oidx, oR, opos = O.compact(m)
    assert R == oR
    assert np.array_equal(idx[:R], oidx)
    if T:
        assert np.all(idx[R:T] == -7)          # entries beyond R untouched
        assert np.array_equal(pos[:T], opos)


@pytest.mark.parametrize("cfg", [2, 3, 4])
def test_compact_on_workload_masks(cfg):
    w = W.config(cfg)
    m = W.make_mask(w)
    idx, R, pos = run_compact(m, want_pos=False)
    oidx, oR, _ = O.compact(m)
    assert R == oR == w.R and np.array_equal(idx[:R], oidx)


def gpu_forward(p, R_host=True, inplace=False, saved=True, flags=0):
    w = p.w
    bufs = B.SkipFFNBuffers(w.T, w.T if not R_host else w.R, w.C, w.I, training=saved)
    B.skipffn_compact(p.d_mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
    hidden = p.d_hidden.clone()
    out = hidden if inplace else torch.full_like(hidden, float("nan"))
    B.skipffn_forward(hidden, out, bufs.idx, w.R if R_host else None, p.d_wg, p.d_wu, p.d_wd,
                      eps=w.eps, rms_gain=p.d_gain, num_retained=bufs.num_retained,
                      saved=bufs.saved, workspace=bufs.fwd_ws, flags=flags)
    torch.cuda.synchronize()
    return out, bufs


def gpu_backward(p, bufs, R_host=True, inplace=False, flags=0, dw=None, dgain=None):
    w = p.w
    grad = p.d_grad.clone()
    gh = grad if inplace else torch.full_like(grad, float("nan"))
    dt = torch.float32 if flags & B.FLAG_DW_FP32 else torch.bfloat16
    if dw is None:
        dw = [torch.full((w.I, w.C), float("nan"), dtype=dt, device="cuda"),
              torch.full((w.I, w.C), float("nan"), dtype=dt, device="cuda"),
              torch.full((w.C, w.I), float("nan"), dtype=dt, device="cuda")]
    B.skipffn_backward(grad, gh, bufs.idx, w.R if R_host else None, p.d_wg, p.d_wu, p.d_wd,
                       bufs.saved, dw[0], dw[1], dw[2], eps=w.eps, rms_gain=p.d_gain,
                       num_retained=bufs.num_retained, workspace=bufs.bwd_ws, flags=flags,
                       d_rms_gain=dgain)
    torch.cuda.synchronize()
    return gh, dw


SMALL = [
    W.config(1),
    W.small(C=512, I=1368, visual=(300, 411), text=(20, 35), keep=(130, 212), seed=11, name="ragged-2tiles"),
    W.small(C=264, I=520, visual=(700,), text=(9,), keep=(600,), seed=12, name="odd-dims-3tiles"),
    W.small(C=1024, I=2048, visual=(64,), text=(1,), keep=(0,), seed=13, name="one-row"),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("gain", [False, True])
def test_forward_stage_by_stage(w, gain):
    print(f"forward stages {w.name} T={w.T} R={w.R} C={w.C} I={w.I} gain={gain}", flush=True)
    p = Problem(w, unit_gain=not gain, with_gain_tensor=gain)
    ref = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    out, bufs = gpu_forward(p)
    R = w.R
    idx = bufs.idx[:R].cpu().numpy()
    assert np.array_equal(idx, ref["idx"])
    sv = bufs.saved_views(R)
    # gathered input rows are bit copies
    assert np.array_equal(bits_of(sv["xrows"]), p.hidden[idx])
    assert rel_l2(f64_of(sv["rstd"]), ref["rstd"]) < 1e-6
    assert rel_l2(f64_of(sv["xn"]), ref["xn"]) < 3e-3          # one bf16 rounding: 2^-9 rms
    for k in ("G", "U", "H"):
        assert rel_l2(f64_of(sv[k]), ref[k]) < REL_L2_TOL, k
    # the transposed copy of the normalised rows is exact, its padding columns are zero
    xnT = bits_of(sv["xnT"])
    assert np.array_equal(xnT[:, :R], bits_of(sv["xn"]).T)
    assert not xnT[:, R:].any()
    # so is the transposed copy of silu(gate) * up that the gate/up epilogue (or, with few rows, a copy kernel) leaves
    HT = bits_of(sv["HT"])
    assert np.array_equal(HT[:, :R], bits_of(sv["H"]).T)
    assert not HT[:, R:].any()
    got = bits_of(out)
    skipped = p.mask != 0
    assert np.array_equal(got[skipped], p.hidden[skipped])      # bitwise passthrough
    e = rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(ref["out_bits"][idx]))
    assert e < REL_L2_TOL, e
    # the FFN update on its own (the residual can hide it when |y| << |x|)
    y_out, _ = gpu_forward(p, flags=B.FLAG_NO_RESIDUAL)
    yb = bits_of(y_out)
    assert np.array_equal(yb[skipped], p.hidden[skipped])
    ey = rel_l2(O.bf16_bits_to_f64(yb[idx]), ref["Y"])
    assert ey < REL_L2_TOL, ey


@pytest.mark.parametrize("w", SMALL, ids=lambda w: w.name)
@pytest.mark.parametrize("gain", [False, True])
def test_backward_against_oracle(w, gain):
    print(f"backward {w.name} T={w.T} R={w.R} C={w.C} I={w.I} gain={gain}", flush=True)
    p = Problem(w, unit_gain=not gain, with_gain_tensor=gain)
    ref = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    _, bufs = gpu_forward(p)
    gh, dw = gpu_backward(p, bufs)
    idx = ref["idx"]
    got = bits_of(gh)
    skipped = p.mask != 0
    assert np.array_equal(got[skipped], p.grad[skipped])
    e = rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(ref["dx_bits"][idx]))
    assert e < REL_L2_TOL, ("dx", e)
    for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
        e = rel_l2(f64_of(t), ref[k])
        assert e < REL_L2_TOL, (k, e)
    # fp32 weight gradients, then accumulation on top of them: 2x
    gh32, dw32 = gpu_backward(p, bufs, flags=B.FLAG_DW_FP32)
    assert np.array_equal(bits_of(gh32), got)
    for t, k in zip(dw32, ("dw_gate", "dw_up", "dw_down")):
        assert rel_l2(f64_of(t), ref[k]) < REL_L2_TOL, k
    first = [t.clone() for t in dw32]
    gpu_backward(p, bufs, flags=B.FLAG_DW_FP32 | B.FLAG_DW_ACCUMULATE, dw=dw32)
    for t, f in zip(dw32, first):
        assert torch.equal(t, 2 * f)
    # bf16 accumulate onto zeros equals overwrite
    z = [torch.zeros_like(t) for t in dw]
    gpu_backward(p, bufs, flags=B.FLAG_DW_ACCUMULATE, dw=z)
    for t, f in zip(z, dw):
        assert torch.equal(t, f)


def test_invariants_on_gpu():
    w = W.small(C=512, I=1024, visual=(300,), text=(30,), keep=(77,), seed=21)
    p = Problem(w)
    out1, bufs = gpu_forward(p)
    # run twice: bitwise equal (deterministic reduction order)
    out2, _ = gpu_forward(p)
    assert torch.equal(out1.view(torch.int16), out2.view(torch.int16))
    # in place == out of place
    out3, _ = gpu_forward(p, inplace=True)
    assert torch.equal(out1.view(torch.int16), out3.view(torch.int16))
    # device-side R == host R
    out4, bufs4 = gpu_forward(p, R_host=False)
    assert torch.equal(out1.view(torch.int16), out4.view(torch.int16))
    gh1, dw1 = gpu_backward(p, bufs)
    gh2, dw2 = gpu_backward(p, bufs, inplace=True)
    gh4, dw4 = gpu_backward(p, bufs4, R_host=False)
    assert torch.equal(gh1.view(torch.int16), gh2.view(torch.int16))
    assert torch.equal(gh1.view(torch.int16), gh4.view(torch.int16))
    for a, b, c in zip(dw1, dw2, dw4):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
        assert torch.equal(a.view(torch.int16), c.view(torch.int16))


def test_retain_all_and_retain_none():
    base = W.small(C=256, I=512, visual=(150,), text=(10,), keep=(150,), seed=31)
    p = Problem(base)
    assert not p.mask.any()
    out, bufs = gpu_forward(p)
    wide = [O.bf16_bits_to_f64(a) for a in (p.hidden, p.wg, p.wu, p.wd)]
    dense = O.dense_swiglu_layer(wide[0], wide[1], wide[2], wide[3], None, base.eps)
    assert rel_l2(f64_of(out), dense) < REL_L2_TOL
    none = W.small(C=256, I=512, visual=(150,), text=(0,), keep=(0,), seed=32)
    q = Problem(none)
    q.hidden[3, :4] = [0x7FC1, 0xFF80, 0x8000, 0x0001]
    q.d_hidden = to_dev_bf16(q.hidden)
    assert q.mask.all()
    out, bufs = gpu_forward(q)
    assert np.array_equal(bits_of(out), q.hidden)
    assert int(bufs.num_retained.item()) == 0
    gh, dw = gpu_backward(q, bufs)
    assert np.array_equal(bits_of(gh), q.grad)
    for t in dw:
        assert not t.view(torch.int16).any()
    # accumulate with R == 0 leaves dW alone
    keep = [torch.ones_like(t) for t in dw]
    gpu_backward(q, bufs, flags=B.FLAG_DW_ACCUMULATE, dw=keep)
    for t in keep:
        assert torch.equal(t, torch.ones_like(t))


def test_inference_forward_without_saved_buffer():
    w = W.small(C=512, I=1024, visual=(300,), text=(30,), keep=(77,), seed=21)
    p = Problem(w)
    a, _ = gpu_forward(p, saved=True)
    b, _ = gpu_forward(p, saved=False)
    assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_skip_kv_cache_row_gather():
    rng = np.random.default_rng(5)
    T, D = 777, 1024
    cache = rng.integers(0, 65536, (T, D)).astype(np.uint16)
    m = (rng.random(T) < 0.75).astype(np.uint8)
    idx, R, _ = O.compact(m)
    src = to_dev_bf16(cache)
    dst = torch.zeros((R, D), dtype=torch.bfloat16, device="cuda")
    B.skipffn_gather_rows(src, dst, torch.from_numpy(idx).cuda(), R)
    torch.cuda.synchronize()
    assert np.array_equal(bits_of(dst), O.kv_skip_cache(cache, m))


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_forward_backward(seed):
    """Seeded random shapes: odd multiples of 8 for C and I, ragged R, one to three
    sequences; both R given by the host and R read on the device."""
    rng = np.random.default_rng(1000 + seed)
    C = 8 * int(rng.integers(8, 90))
    I = 8 * int(rng.integers(8, 200))
    nseq = int(rng.integers(1, 4))
    vis = [int(rng.integers(1, 400)) for _ in range(nseq)]
    txt = [int(rng.integers(0, 30)) for _ in range(nseq)]
    keep = [int(rng.integers(0, v + 1)) for v in vis]
    w = W.small(C=C, I=I, visual=vis, text=txt, keep=keep, seed=50 + seed, name=f"rand{seed}")
    print(f"random shape {seed}: T={w.T} R={w.R} C={C} I={I}", flush=True)
    if w.R == 0:
        pytest.skip("empty retained set is covered elsewhere")
    p = Problem(w, unit_gain=False, with_gain_tensor=bool(seed & 1))
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    idx = fo["idx"]
    sk = p.mask != 0
    for r_host in (True, False):
        out, bufs = gpu_forward(p, R_host=r_host, inplace=bool(seed & 2))
        got = bits_of(out)
        assert np.array_equal(got[sk], p.hidden[sk])
        assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
        gh, dw = gpu_backward(p, bufs, R_host=r_host, inplace=bool(seed & 2))
        gb = bits_of(gh)
        assert np.array_equal(gb[sk], p.grad[sk])
        assert rel_l2(O.bf16_bits_to_f64(gb[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
        for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
            assert rel_l2(f64_of(t), bo[k]) < REL_L2_TOL, (k, r_host)


@pytest.mark.parametrize("C,I", [(264, 200), (1096, 456), (456, 1096), (2056, 136), (192, 2056)],
                         ids=lambda v: str(v))
def test_k_ranges_that_end_inside_a_slab(C, I):
    """256-row tiles (R > 256) with contraction lengths that are no multiple of the 64-deep K slab, from
    3 to 33 slabs: the main loop runs its steady state (unmasked loads, offsets stepped per slab) up to
    the slabs at the end of the K range - and, in the dXn GEMM, of each of its two operand pairs - which
    take the guarded, masked path.  R = 300 is no multiple of 64 either (the weight-gradient GEMMs
    contract over it)."""
    w = W.small(C=C, I=I, visual=(330,), text=(12,), keep=(288,), seed=70 + C % 7, name=f"ktail-{C}-{I}")
    assert w.R == 300
    p = Problem(w, unit_gain=False, with_gain_tensor=True)
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    idx, sk = fo["idx"], p.mask != 0
    for r_host in (True, False):
        out, bufs = gpu_forward(p, R_host=r_host)
        got = bits_of(out)
        assert np.array_equal(got[sk], p.hidden[sk])
        assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
        sv = bufs.saved_views(w.R)
        for k in ("G", "U", "H"):
            assert rel_l2(f64_of(sv[k]), fo[k]) < REL_L2_TOL, k
        gh, dw = gpu_backward(p, bufs, R_host=r_host)
        gb = bits_of(gh)
        assert np.array_equal(gb[sk], p.grad[sk])
        assert rel_l2(O.bf16_bits_to_f64(gb[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
        for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
            assert rel_l2(f64_of(t), bo[k]) < REL_L2_TOL, (k, r_host)


BALANCED = [
    # (workload, what it exercises)
    W.small(C=512, I=1368, visual=(300, 411), text=(20, 35), keep=(130, 212), seed=21,
            name="bal-2groups-2tiles"),           # 2 m-tiles, K tail, aligned chunks + remainder pieces
    W.small(C=264, I=520, visual=(700,), text=(9,), keep=(600,), seed=22,
            name="bal-3tiles-short-k"),           # ragged C, few K slabs: q from the slab budget
    W.small(C=1024, I=2048, visual=(64,), text=(1,), keep=(0,), seed=23, name="bal-one-row"),
    W.small(C=256, I=9000, visual=(900, 600), text=(30, 12), keep=(450, 333), seed=24,
            name="bal-long-k-4tiles"),            # long K, remainder pieces spanning tiles
    W.small(C=4096, I=320, visual=(4400,), text=(30,), keep=(4100,), seed=25,
            name="bal-17-mtiles-16-workgroups"),  # more m-tiles than workgroups per group: a whole
                                                  # tile per workgroup first, the 17th split 5 ways
]


@pytest.mark.parametrize("w", BALANCED, ids=lambda w: w.name)
@pytest.mark.parametrize("r_host", [True, False], ids=["R-host", "R-device"])
def test_balanced_split_forward_backward(w, r_host):
    """The balanced K split of the down and dXn GEMMs (forced by flag: the cost model would
    not pick it at these sizes) against the oracle, with R known on the host and R read on
    the device (the plan is then recomputed in the kernels from the device-side count)."""
    p = Problem(w, unit_gain=False)
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    idx = fo["idx"]
    sk = p.mask != 0
    out, bufs = gpu_forward(p, R_host=r_host, flags=B.FLAG_BALANCED_SPLIT)
    got = bits_of(out)
    assert np.array_equal(got[sk], p.hidden[sk])
    assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
    gh, dw = gpu_backward(p, bufs, R_host=r_host, flags=B.FLAG_BALANCED_SPLIT)
    gb = bits_of(gh)
    assert np.array_equal(gb[sk], p.grad[sk])
    assert rel_l2(O.bf16_bits_to_f64(gb[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
    # the split only changes the order of fp32 additions: results agree with the default path
    out2, bufs2 = gpu_forward(p, R_host=r_host)
    gh2, _ = gpu_backward(p, bufs2, R_host=r_host)
    a, b = f64_of(out)[idx], f64_of(out2)[idx]
    assert rel_l2(a, b) < 1e-2
    assert rel_l2(f64_of(gh)[idx], f64_of(gh2)[idx]) < 1e-2


KV_CASES = [
    # (leading dims, T, D, keep probability, destination capacity: "packed" or "prefill")
    ((3, 2, 4), 777, 128, 0.25, "packed"),      # layers x key/value x heads, LLaMA head size
    ((2, 2, 8), 616, 128, 0.30, "prefill"),     # compacted cache keeps the prefill capacity
    ((5,), 1000, 8, 0.5, "packed"),             # 16-byte rows
    ((70000,), 6, 8, 0.5, "packed"),            # more slabs than one grid dimension holds
    ((1, 1), 300, 1024, 1.0, "packed"),         # nothing skipped
]


@pytest.mark.parametrize("lead,T,D,keep,cap", KV_CASES, ids=lambda v: str(v).replace(" ", ""))
@pytest.mark.parametrize("r_host", [True, False], ids=["R-host", "R-device"])
def test_skip_kv_cache_whole_cache(lead, T, D, keep, cap, r_host):
    """Section 4.3 on a whole cache in one launch, bit for bit against the oracle."""
    rng = np.random.default_rng(31 + T)
    cache = rng.integers(0, 65536, lead + (T, D)).astype(np.uint16)
    m = (rng.random(T) >= keep).astype(np.uint8)
    want = O.kv_skip_cache_all(cache, m)
    R = want.shape[-2]
    mask = torch.from_numpy(m).cuda()
    idx = torch.empty(T, dtype=torch.int32, device="cuda")
    nret = torch.zeros(1, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(B.skipffn_compact_workspace_bytes(T), 16), dtype=torch.uint8, device="cuda")
    B.skipffn_compact(mask, idx, nret, None, ws)
    src = to_dev_bf16(cache)
    rcap = T if (cap == "prefill" or not r_host) else R
    dst = torch.full(lead + (rcap, D), -1.0, dtype=torch.bfloat16, device="cuda")
    B.skipffn_kv_compact(src, dst, idx, R if r_host else None, num_retained=nret)
    torch.cuda.synchronize()
    got = bits_of(dst)
    assert np.array_equal(got[..., :R, :], want)
    # rows past R are left as they were
    assert np.all(got[..., R:, :] == bits_of(torch.full((1,), -1.0, dtype=torch.bfloat16))[0])


GAIN_CASES = [
    W.small(C=512, I=1368, visual=(300, 411), text=(20, 35), keep=(130, 212), seed=41, name="gain-2tiles"),
    W.small(C=264, I=520, visual=(700,), text=(9,), keep=(600,), seed=42, name="gain-odd-dims"),
    W.small(C=1024, I=256, visual=(64,), text=(1,), keep=(0,), seed=43, name="gain-one-row"),
    W.small(C=4104, I=128, visual=(40,), text=(3,), keep=(19,), seed=44, name="gain-wide-row"),   # C > 4096: streaming path
]


@pytest.mark.parametrize("w", GAIN_CASES, ids=lambda w: w.name)
@pytest.mark.parametrize("with_gain", [True, False], ids=["gain", "unit-gain"])
def test_rmsnorm_gain_gradient(w, with_gain):
    """d_rms_gain against the oracle (the gradient at g = 1 when no gain tensor is given);
    asking for it must not change dX; accumulate adds to what is there; R on the device."""
    p = Problem(w, unit_gain=not with_gain, with_gain_tensor=with_gain)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    idx = bo["idx"]
    _, bufs = gpu_forward(p)
    gh0, _ = gpu_backward(p, bufs)
    dgain = torch.full((w.C,), float("nan"), dtype=torch.float32, device="cuda")
    gh1, _ = gpu_backward(p, bufs, dgain=dgain)
    got = dgain.double().cpu().numpy()
    assert rel_l2(got, bo["dgain"]) < REL_L2_TOL
    assert rel_l2(f64_of(gh1)[idx], f64_of(gh0)[idx]) < 1e-6      # same sums, same order
    # deterministic: a second run gives the same bits
    dgain2 = torch.zeros_like(dgain)
    gpu_backward(p, bufs, dgain=dgain2)
    assert torch.equal(dgain, dgain2)
    # accumulate
    acc = torch.ones_like(dgain)
    dwa = [torch.zeros((w.I, w.C), dtype=torch.bfloat16, device="cuda"),
           torch.zeros((w.I, w.C), dtype=torch.bfloat16, device="cuda"),
           torch.zeros((w.C, w.I), dtype=torch.bfloat16, device="cuda")]
    gpu_backward(p, bufs, flags=B.FLAG_DW_ACCUMULATE, dw=dwa, dgain=acc)
    assert rel_l2(acc.double().cpu().numpy() - 1.0, bo["dgain"]) < REL_L2_TOL
    # R read on the device
    _, bufs_d = gpu_forward(p, R_host=False)
    dgain_d = torch.full((w.C,), float("nan"), dtype=torch.float32, device="cuda")
    gpu_backward(p, bufs_d, R_host=False, dgain=dgain_d)
    assert rel_l2(dgain_d.double().cpu().numpy(), bo["dgain"]) < REL_L2_TOL


def test_gain_gradient_with_nothing_retained_is_zero():
    w = W.small(C=256, I=512, visual=(50,), text=(0,), keep=(0,), seed=45, name="gain-empty")
    p = Problem(w)
    _, bufs = gpu_forward(p)
    dgain = torch.full((w.C,), 7.0, dtype=torch.float32, device="cuda")
    gpu_backward(p, bufs, dgain=dgain)
    assert torch.count_nonzero(dgain).item() == 0


TINY = [
    W.small(C=8, I=8, visual=(2,), text=(1,), keep=(0,), seed=71, name="tiny-8-8-one-row"),
    W.small(C=8, I=16, visual=(5,), text=(0,), keep=(5,), seed=72, name="tiny-8-16-all-kept"),
    W.small(C=24, I=8, visual=(70,), text=(3,), keep=(33,), seed=73, name="tiny-24-8"),
    W.small(C=8200, I=16, visual=(9,), text=(0,), keep=(4,), seed=74, name="wide-8200-16"),   # C beyond the register-resident row paths
]


@pytest.mark.parametrize("w", TINY, ids=lambda w: w.name)
def test_smallest_and_widest_shapes(w):
    """The minimum widths the interface allows (8), a single retained row, and a hidden size
    beyond the register-resident row kernels (streaming paths of RMSNorm forward/backward)."""
    p = Problem(w, unit_gain=False, with_gain_tensor=True)
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    idx = fo["idx"]
    sk = p.mask != 0
    out, bufs = gpu_forward(p, flags=B.FLAG_NO_RESIDUAL)
    got = bits_of(out)
    assert np.array_equal(got[sk], p.hidden[sk])
    fo_nr = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps, no_residual=True)
    assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo_nr["out_bits"][idx])) < REL_L2_TOL
    out, bufs = gpu_forward(p)
    assert rel_l2(O.bf16_bits_to_f64(bits_of(out)[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
    dgain = torch.zeros(w.C, dtype=torch.float32, device="cuda")
    gh, dw = gpu_backward(p, bufs, flags=B.FLAG_DW_FP32, dgain=dgain)
    gb = bits_of(gh)
    assert np.array_equal(gb[sk], p.grad[sk])
    assert rel_l2(O.bf16_bits_to_f64(gb[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
    for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
        assert rel_l2(t.double().cpu().numpy(), bo[k]) < REL_L2_TOL, k
    assert rel_l2(dgain.double().cpu().numpy(), bo["dgain"]) < REL_L2_TOL



@pytest.mark.parametrize("R", [1, 63, 64, 65, 127, 128, 129, 191, 255, 256, 257])
@pytest.mark.parametrize("r_host", [True, False], ids=["R-host", "R-device"])
@pytest.mark.parametrize("C,I", [(520, 1368), (1024, 1368), (2048, 2816)],
                         ids=["fused-gate-up", "gate-up-2-splits", "gate-up-4-splits"])
def test_row_counts_around_the_128_row_tiles(R, r_host, C, I):
    """Up to 256 retained rows the forward GEMMs run on 128-row tiles (one or two rows of tiles,
    split-K partial sums for the down projection); 257 is the first count on 256-row tiles.  Up
    to 128 rows the gate/up GEMM is split along K as well when K is long enough (C = 520 is not:
    fused epilogue; C = 1024 gives 2 splits, C = 2048 with 22 column tiles 4) and the SwiGLU runs
    in the reducing kernel.  With the count on the device the row bound is T, which selects the
    variant."""
    visual = R - 7 if R > 7 else R
    text = R - visual
    T_pad = 40 if r_host else 0          # R-device: keep T (the bound) within the same variant
    w = W.small(C=C, I=I, visual=(visual + T_pad,), text=(text,), keep=(visual,), seed=300 + R,
                name=f"rows-{R}")
    assert w.R == R
    print(f"narrow tiles R={R} T={w.T} r_host={r_host}", flush=True)
    p = Problem(w, unit_gain=False, with_gain_tensor=True)
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps)
    fo_nr = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.gain, w.eps, no_residual=True)
    idx, sk = fo["idx"], p.mask != 0
    for saved in (False, True):
        out, bufs = gpu_forward(p, R_host=r_host, saved=saved, flags=B.FLAG_NO_RESIDUAL)
        got = bits_of(out)
        assert np.array_equal(got[sk], p.hidden[sk])
        assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo_nr["out_bits"][idx])) < REL_L2_TOL
        out, bufs = gpu_forward(p, R_host=r_host, saved=saved, inplace=True)
        got = bits_of(out)
        assert np.array_equal(got[sk], p.hidden[sk])
        assert rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
    sv = bufs.saved_views(R)
    for k in ("G", "U", "H"):
        assert rel_l2(f64_of(sv[k]), fo[k]) < REL_L2_TOL, k
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, p.gain, w.eps)
    gh, dw = gpu_backward(p, bufs, R_host=r_host)
    assert rel_l2(O.bf16_bits_to_f64(bits_of(gh)[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
    for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
        assert rel_l2(f64_of(t), bo[k]) < REL_L2_TOL, k


@pytest.mark.parametrize("R_max", [300, 2000])
def test_buffers_sized_for_a_larger_row_bound(R_max):
    """Buffers sized once for R_max rows serve a call with fewer rows (here a count that takes the
    128-row tiles and more K splits than the bound's own configuration would)."""
    w = W.small(C=520, I=1368, visual=(200,), text=(13,), keep=(87,), seed=55, name="bound")
    p = Problem(w)
    bufs = B.SkipFFNBuffers(w.T, R_max, w.C, w.I, training=True)
    B.skipffn_compact(p.d_mask, bufs.idx, bufs.num_retained, None, bufs.compact_ws)
    out = p.d_hidden.clone()
    B.skipffn_forward(out, out, bufs.idx, w.R, p.d_wg, p.d_wu, p.d_wd, eps=w.eps, saved=bufs.saved,
                      workspace=bufs.fwd_ws)
    gh = p.d_grad.clone()
    dw = [torch.empty((w.I, w.C), dtype=torch.bfloat16, device="cuda"),
          torch.empty((w.I, w.C), dtype=torch.bfloat16, device="cuda"),
          torch.empty((w.C, w.I), dtype=torch.bfloat16, device="cuda")]
    B.skipffn_backward(gh, gh, bufs.idx, w.R, p.d_wg, p.d_wu, p.d_wd, bufs.saved, *dw, eps=w.eps,
                       workspace=bufs.bwd_ws)
    torch.cuda.synchronize()
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, None, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, None, w.eps)
    idx = fo["idx"]
    assert rel_l2(O.bf16_bits_to_f64(bits_of(out)[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx])) < REL_L2_TOL
    assert rel_l2(O.bf16_bits_to_f64(bits_of(gh)[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx])) < REL_L2_TOL
    for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
        assert rel_l2(f64_of(t), bo[k]) < REL_L2_TOL, k


@pytest.mark.parametrize("R", [257, 300, 384, 385, 512 + 1, 512 + 128, 768 + 100])
def test_last_tile_row_of_at_most_128_rows(R):
    """A row count that leaves at most 128 rows for the last row of tiles runs that row on
    128-row tiles in the gate/up GEMM (257, 300, 384, 513, 640, 868; 385 leaves 129 rows
    and keeps a full-height tile).  Every row is checked on its own: the tail rows sit in
    different tiles from the rest.  The intermediate width leaves a ragged column tile too."""
    from helpers import max_slice_rel_l2
    w = W.small(C=520, I=1368, visual=(R + 30,), text=(9,), keep=(R - 9,), seed=900 + R, name=f"tail-{R}")
    assert w.R == R
    print(f"tail row R={R} T={w.T}", flush=True)
    p = Problem(w)
    fo = O.skipffn_forward(p.hidden, p.mask, p.wg, p.wu, p.wd, None, w.eps)
    bo = O.skipffn_backward(p.hidden, p.mask, p.wg, p.wu, p.wd, p.grad, None, w.eps)
    idx, sk = fo["idx"], p.mask != 0
    out, bufs = gpu_forward(p, saved=True, inplace=True)
    got = bits_of(out)
    assert np.array_equal(got[sk], p.hidden[sk])
    assert max_slice_rel_l2(O.bf16_bits_to_f64(got[idx]), O.bf16_bits_to_f64(fo["out_bits"][idx]), axis=1) < REL_L2_TOL
    sv = bufs.saved_views(R)
    for k in ("G", "U", "H"):
        assert max_slice_rel_l2(f64_of(sv[k]), fo[k], axis=1) < REL_L2_TOL, k
    gh, dw = gpu_backward(p, bufs)
    gb = bits_of(gh)
    assert np.array_equal(gb[sk], p.grad[sk])
    assert max_slice_rel_l2(O.bf16_bits_to_f64(gb[idx]), O.bf16_bits_to_f64(bo["dx_bits"][idx]), axis=1) < REL_L2_TOL
    for t, k in zip(dw, ("dw_gate", "dw_up", "dw_down")):
        assert rel_l2(f64_of(t), bo[k]) < REL_L2_TOL, k
