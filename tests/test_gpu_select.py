"""GPU parity of the retained-token selection (Section 4.1) through the C ABI.  The mask is an
integer decided by floating-point similarities, so the decision is compared in the kernel's
precision: the oracle's selection rule applied to the float32 similarities the GPU returns must
give the GPU's mask bit for bit, and those similarities must match the fp64 ones."""
import numpy as np
import pytest
import torch

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import binding as B
from helpers import to_dev_bf16

pytestmark = pytest.mark.gpu


def run_gpu(feat, cls, seq_off, n_keep, token_pos=None, T=0):
    d_f, d_c = to_dev_bf16(feat), to_dev_bf16(cls)
    d_off = torch.from_numpy(np.asarray(seq_off, dtype=np.int32)).cuda()
    n = feat.shape[0]
    mask = torch.full((n,), 9, dtype=torch.uint8, device="cuda")
    sim = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    nk = n_keep if np.isscalar(n_keep) else torch.from_numpy(np.asarray(n_keep, dtype=np.int32)).cuda()
    pos = None if token_pos is None else torch.from_numpy(np.asarray(token_pos, dtype=np.int32)).cuda()
    sk = None if token_pos is None else torch.full((T,), 7, dtype=torch.uint8, device="cuda")
    B.skipffn_select_retained(d_f, d_c, d_off, nk, mask, sim, token_pos=pos, skip_mask=sk)
    torch.cuda.synchronize()
    return mask.cpu().numpy(), sim.cpu().numpy(), None if sk is None else sk.cpu().numpy()


def check(feat, cls, seq_off, n_keep):
    mask, sim, _ = run_gpu(feat, cls, seq_off, n_keep)
    ref = O.select_retained(feat, cls, seq_off, n_keep)
    assert np.allclose(sim, ref["sim"], rtol=0, atol=2e-5)
    nb = len(seq_off) - 1
    nk = np.broadcast_to(np.asarray(n_keep), (nb,))
    for b in range(nb):
        lo, hi = seq_off[b], seq_off[b + 1]
        # the decision, in the kernel's precision
        assert np.array_equal(mask[lo:hi], O.select_top_n(sim[lo:hi], nk[b])), b
        assert int((mask[lo:hi] == 0).sum()) == min(int(nk[b]), hi - lo)
        # where the fp64 similarities are separated at the threshold by more than the fp32
        # error, the fp64 decision must be the same
        s64 = np.sort(ref["sim"][lo:hi])[::-1]
        k = min(int(nk[b]), hi - lo)
        if 0 < k < hi - lo and s64[k - 1] - s64[k] > 1e-4:
            assert np.array_equal(mask[lo:hi], ref["mask"][lo:hi]), b
    return mask, sim


@pytest.mark.parametrize("lens,Cv,keep", [((576,) * 4, 1024, 144), ((2880, 100, 1, 17), 1024, [576, 30, 1, 0]),
                                          ((33, 0, 64), 264, 10), ((20000,), 64, 5000)],
                         ids=["llava-576", "hd-and-ragged", "empty-seq-odd-width", "longer-than-lds"])
def test_selection_against_oracle(lens, Cv, keep):
    rng = np.random.default_rng(len(lens) + Cv)
    n = sum(lens)
    feat = O.f64_to_bf16_bits(rng.standard_normal((n, Cv)))
    cls = O.f64_to_bf16_bits(rng.standard_normal((len(lens), Cv)))
    seq_off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    check(feat, cls, seq_off, keep)


def test_equal_similarities_go_to_the_lower_index_and_keep_all_or_none():
    rng = np.random.default_rng(4)
    base = O.f64_to_bf16_bits(rng.standard_normal((6, 128)))
    feat = base[[0, 1, 0, 2, 0, 3, 1, 4, 5, 0]]            # repeated rows: exactly equal similarities
    cls = O.f64_to_bf16_bits(rng.standard_normal((1, 128)))
    off = np.array([0, 10], dtype=np.int32)
    for k in (0, 1, 3, 4, 10, 50):
        mask, sim = check(feat, cls, off, k)
        assert sim[0] == sim[2] == sim[4] == sim[9]
    # parallel vectors have similarity 1, opposite -1, a zero row 0
    c = O.bf16_bits_to_f64(cls[0])
    feat2 = O.f64_to_bf16_bits(np.stack([c, 4 * c, -c, np.zeros(128)]))
    _, sim2, _ = run_gpu(feat2, cls, np.array([0, 4], np.int32), 1)
    assert np.allclose(sim2, [1, 1, -1, 0], atol=1e-6)


def test_mask_scattered_to_token_positions_feeds_the_compaction():
    rng = np.random.default_rng(8)
    lens, txt = (40, 25), (5, 3)
    n = sum(lens)
    feat = O.f64_to_bf16_bits(rng.standard_normal((n, 256)))
    cls = O.f64_to_bf16_bits(rng.standard_normal((2, 256)))
    off = np.array([0, 40, 65], dtype=np.int32)
    # flat token order: [visual 40][text 5][visual 25][text 3]
    pos = np.concatenate([np.arange(0, 40), np.arange(45, 70)]).astype(np.int32)
    T = 73
    pos_bad = pos.copy(); pos_bad[3] = -5; pos_bad[50] = 10_000           # ignored
    mask, sim, sk = run_gpu(feat, cls, off, [10, 5], token_pos=pos_bad, T=T)
    want = np.full(T, 7, np.uint8)
    good = np.ones(n, bool); good[[3, 50]] = False
    want[pos[good]] = mask[good]
    assert np.array_equal(sk, want)


def test_non_finite_features_still_retain_exactly_n():
    """A feature row holding Inf has a NaN similarity (Inf / Inf); a row that is NaN throughout has
    no length at all and gets similarity 0, like a zero row.  NaN loses to every number (the
    oracle's sort puts it last as well), so exactly n tokens are retained whatever the input."""
    rng = np.random.default_rng(15)
    f = rng.standard_normal((300, 128))
    f[7, 3] = np.inf
    f[100, :] = np.nan
    f[299, 0] = -np.inf
    feat = O.f64_to_bf16_bits(f)
    cls = O.f64_to_bf16_bits(rng.standard_normal((2, 128)))
    off = np.array([0, 120, 300], dtype=np.int32)
    for keep in (1, 50, 119, 120, 179, 180):
        mask, sim, _ = run_gpu(feat, cls, off, keep)
        assert np.isnan(sim[[7, 299]]).all() and sim[100] == 0.0
        assert np.isfinite(np.delete(sim, [7, 299])).all()
        for b in range(2):
            lo, hi = off[b], off[b + 1]
            assert int((mask[lo:hi] == 0).sum()) == min(keep, hi - lo)
            assert np.array_equal(mask[lo:hi], O.select_top_n(sim[lo:hi], keep))
