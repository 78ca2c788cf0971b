"""GPU parity of the token merge (Section 4.1) through the C ABI.  Which tokens are kept and
where a token goes are integers decided by floating-point similarities, so those decisions are
checked in the kernel's precision (the oracle's rule applied to the averages the GPU returns
must give the GPU's kept set; every assignment must be optimal up to the rounding of the
similarities, and equal to the fp64 choice wherever that choice has a clear margin); the merged
rows are then compared with the oracle's merge of the same groups."""
import numpy as np
import pytest
import torch

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import binding as B
from helpers import REL_L2_TOL, bits_of, rel_l2, to_dev_bf16

pytestmark = pytest.mark.gpu

SIM_TOL = 6e-3        # bf16 rounding of the normalised rows: about 2^-8 on a cosine similarity


def run_gpu(xb, seg, k):
    n_tok, C = xb.shape
    S = len(seg) - 1
    n_max = max([seg[i + 1] - seg[i] for i in range(S)] + [0])
    d_x = to_dev_bf16(xb)
    out = torch.full((S, k, C), float("nan"), dtype=torch.bfloat16, device="cuda")
    kept = torch.full((S, k), -7, dtype=torch.int32, device="cuda")
    assign = torch.full((n_tok,), -7, dtype=torch.int32, device="cuda")
    avg = torch.full((n_tok,), float("nan"), dtype=torch.float32, device="cuda")
    ws = torch.empty(B.skipffn_token_merge_workspace_bytes(n_tok, n_max, C), dtype=torch.uint8, device="cuda")
    B.skipffn_token_merge(d_x, seg, k, out, kept, assign, avg, workspace=ws)
    torch.cuda.synchronize()
    return bits_of(out), kept.cpu().numpy(), assign.cpu().numpy(), avg.cpu().numpy()


def check(xb, seg, k, expect_exact=False):
    out, kept, assign, avg = run_gpu(xb, seg, k)
    ref = O.token_merge(xb, seg, k)
    for s in range(len(seg) - 1):
        lo, hi = seg[s], seg[s + 1]
        n = hi - lo
        kk = min(k, n)
        if n == 0:
            assert np.all(kept[s] == -1) and np.all(out[s] == 0)
            continue
        X = O.bf16_bits_to_f64(xb[lo:hi])
        S64 = O.cosine_matrix(X)
        assert np.allclose(avg[lo:hi], ref["avg"][lo:hi], rtol=0, atol=SIM_TOL)
        # kept set: the oracle's rule on the GPU's own averages
        order = np.argsort(avg[lo:hi], kind="stable")
        want_kept = np.sort(order[:kk]) + lo
        assert np.array_equal(kept[s, :kk], want_kept) and np.all(kept[s, kk:] == -1)
        kloc = kept[s, :kk] - lo
        a = assign[lo:hi]
        assert np.array_equal(a[kloc], np.arange(kk))
        assert np.all((a >= 0) & (a < kk))
        # every merged token went to a kept token that is (nearly) its most similar one
        for i in range(n):
            if i in set(kloc.tolist()):
                continue
            best = S64[i, kloc].max()
            assert S64[i, kloc[a[i]]] >= best - 2 * SIM_TOL, (s, i)
            top2 = np.sort(S64[i, kloc])[-2:] if kk > 1 else [None, None]
            if kk == 1 or top2[1] - top2[0] > 2 * SIM_TOL:
                assert a[i] == int(np.argmax(S64[i, kloc])), (s, i)
        # merged rows: the oracle's mean over the GPU's groups
        merged = O.merge_rows(X, a, kk)
        assert rel_l2(O.bf16_bits_to_f64(out[s, :kk]), merged) < REL_L2_TOL
        assert np.all(out[s, kk:] == 0)
    if expect_exact:
        assert np.array_equal(kept, ref["kept"]) and np.array_equal(assign, ref["assign"])
        assert rel_l2(O.bf16_bits_to_f64(out), O.bf16_bits_to_f64(ref["out_bits"])) < REL_L2_TOL


def clustered(n, C, centers, noise, seed):
    """Tokens scattered around a few directions: large margins in every decision."""
    rng = np.random.default_rng(seed)
    ctr = rng.standard_normal((centers, C))
    lab = rng.integers(0, centers, n)
    return O.f64_to_bf16_bits(ctr[lab] * rng.uniform(0.5, 2.0, (n, 1)) + noise * rng.standard_normal((n, C)))


@pytest.mark.parametrize("lens,C,k", [((1024,), 1024, 256), ((300, 77, 512), 256, 64), ((40, 0, 9), 264, 16),
                                      ((600,), 4096, 150)],
                         ids=["paper-1024-to-256", "three-sets", "empty-and-short-sets", "backbone-width"])
def test_merge_random_tokens(lens, C, k):
    rng = np.random.default_rng(sum(lens) + C)
    xb = O.f64_to_bf16_bits(rng.standard_normal((sum(lens), C)))
    seg = [0] + np.cumsum(lens).tolist()
    check(xb, seg, k)


def test_merge_clustered_tokens_small_margins_inside_clusters():
    xb = clustered(500, 512, centers=40, noise=0.05, seed=3)
    check(xb, [0, 200, 500], 60)


def test_duplicates_single_token_and_k_extremes():
    rng = np.random.default_rng(9)
    base = O.f64_to_bf16_bits(rng.standard_normal((5, 128)))
    xb = base[[0, 1, 2, 1, 3, 0, 4, 2]]                      # exact duplicates: similarity ties
    check(xb, [0, 8], 3)
    check(xb, [0, 8], 8)                                     # k = n: nothing merged
    out, kept, assign, _ = run_gpu(xb, [0, 8], 8)
    assert np.array_equal(out[0], xb) and kept[0].tolist() == list(range(8))
    check(xb, [0, 8], 1)                                     # k = 1: the mean of all
    check(xb[:1], [0, 1], 4)                                 # a single token
    out, kept, assign, _ = run_gpu(xb, [0, 8], 12)           # k > n: zero rows after the 8 tokens
    assert np.array_equal(out[0, :8], xb) and np.all(out[0, 8:] == 0) and kept[0, 8:].tolist() == [-1] * 4


# ---- gradient ------------------------------------------------------------------------------------
def run_gpu_backward(gb, seg, assign, n_tok, C):
    d_g = to_dev_bf16(gb)
    d_a = torch.from_numpy(np.asarray(assign, dtype=np.int32)).cuda()
    gx = torch.full((max(n_tok, 1), C), float("nan"), dtype=torch.bfloat16, device="cuda")[:n_tok]
    B.skipffn_token_merge_backward(d_g, seg, d_a, gx)
    torch.cuda.synchronize()
    return bits_of(gx)


@pytest.mark.parametrize("lens,C,k", [((1024,), 1024, 256), ((300, 77, 512), 256, 64), ((40, 0, 9), 264, 16),
                                      ((600,), 4096, 150), ((3,) * 70, 128, 2)],
                         ids=["paper-1024-to-256", "three-sets", "empty-and-short-sets", "backbone-width",
                              "more-sets-than-one-launch-takes"])
def test_merge_gradient(lens, C, k):
    """The gradient for the groups the GPU's own forward formed, against the oracle's gradient
    for those groups: one division and one rounding per element."""
    rng = np.random.default_rng(sum(lens) + C + 1)
    n_tok = sum(lens)
    xb = O.f64_to_bf16_bits(rng.standard_normal((n_tok, C)))
    seg = [0] + np.cumsum(lens).tolist()
    _, _, assign, _ = run_gpu(xb, seg, k)
    gb = O.f64_to_bf16_bits(rng.standard_normal((len(lens), k, C)))
    got = run_gpu_backward(gb, seg, assign, n_tok, C)
    ref = O.token_merge_backward(gb, seg, k, assign)
    g64 = O.bf16_bits_to_f64(got)
    assert rel_l2(g64, ref["dx"]) < REL_L2_TOL
    # element by element: float32 quotient rounded to bf16 against the exact quotient rounded to
    # bf16 - equal except where the exact quotient sits within 2^-24 of a rounding boundary
    same = got == ref["dx_bits"]
    assert same.mean() > 0.9999
    assert np.all(np.abs(g64 - ref["dx"]) <= np.abs(ref["dx"]) * 2.0 ** -8 + 1e-30)
    # the members of a slot share its gradient: they add up to it (up to their roundings)
    for s in range(len(lens)):
        lo, hi = seg[s], seg[s + 1]
        kk = min(k, hi - lo)
        for j in range(min(kk, 5)):
            mem = np.flatnonzero(assign[lo:hi] == j) + lo
            tot = g64[mem].sum(0)
            assert np.allclose(tot, O.bf16_bits_to_f64(gb[s, j]), rtol=2.0 ** -7, atol=1e-6)


def test_merge_gradient_passes_through_a_set_kept_whole_and_zeroes_invalid_slots():
    rng = np.random.default_rng(21)
    gb = O.f64_to_bf16_bits(rng.standard_normal((2, 8, 64)))
    assign = np.array([0, 1, 2, 3, 4,   2, -1, 0, 9, 0, 2], dtype=np.int32)     # sets of 5 and 6 rows
    got = run_gpu_backward(gb, [0, 5, 11], assign, 11, 64)
    assert np.array_equal(got[:5], gb[0, :5])                                   # identity, bit for bit
    assert np.all(got[6] == 0) and np.all(got[8] == 0)                          # -1 and an index >= min(k, n)
    ref = O.token_merge_backward(gb, [0, 5, 11], 8, np.where((assign < 0) | (assign > 5), -1, assign))
    assert np.array_equal(got, ref["dx_bits"])


def test_non_finite_tokens_keep_exactly_k_and_stay_inside_the_outputs():
    """One Inf / NaN row per set turns similarities and averages into NaN.  The rank order is
    total (NaN after every number, then by index), so exactly min(k, n) tokens are kept per set and
    nothing is written outside kept_idx / out: both are carved out of larger buffers whose
    surrounding bytes must survive."""
    rng = np.random.default_rng(31)
    lens, C, k = (96, 130, 40), 256, 24
    x = rng.standard_normal((sum(lens), C))
    x[5, 17] = np.inf
    x[96 + 129, :] = np.nan
    x[96 + 130 + 1, 0] = -np.inf
    xb = O.f64_to_bf16_bits(x)
    seg = [0] + np.cumsum(lens).tolist()
    S, n_tok = len(lens), sum(lens)
    pad = 64
    d_x = to_dev_bf16(xb)
    out_big = torch.full((pad + S * k * C + pad,), 1.5, dtype=torch.bfloat16, device="cuda")
    kept_big = torch.full((pad + S * k + pad,), -77, dtype=torch.int32, device="cuda")
    assign_big = torch.full((pad + n_tok + pad,), -77, dtype=torch.int32, device="cuda")
    avg_big = torch.full((pad + n_tok + pad,), 3.25, dtype=torch.float32, device="cuda")
    out = out_big[pad:pad + S * k * C].view(S, k, C)
    kept = kept_big[pad:pad + S * k].view(S, k)
    assign = assign_big[pad:pad + n_tok]
    avg = avg_big[pad:pad + n_tok]
    ws = torch.empty(B.skipffn_token_merge_workspace_bytes(n_tok, max(lens), C), dtype=torch.uint8, device="cuda")
    B.skipffn_token_merge(d_x, seg, k, out, kept, assign, avg, workspace=ws)
    torch.cuda.synchronize()
    for big, fill in ((out_big, 1.5), (kept_big, -77), (assign_big, -77), (avg_big, 3.25)):
        assert bool((big[:pad] == fill).all()) and bool((big[-pad:] == fill).all())
    kept_h, assign_h, avg_h = kept.cpu().numpy(), assign.cpu().numpy(), avg.cpu().numpy()
    for s in range(S):
        lo, hi = seg[s], seg[s + 1]
        kk = min(k, hi - lo)
        # the oracle's rule (a stable sort, NaN last) on the GPU's own averages
        want = np.sort(np.argsort(avg_h[lo:hi], kind="stable")[:kk]) + lo
        assert np.array_equal(kept_h[s, :kk], want)
        assert np.all((assign_h[lo:hi] >= -1) & (assign_h[lo:hi] < kk))
        assert np.array_equal(assign_h[kept_h[s, :kk]], np.arange(kk))
