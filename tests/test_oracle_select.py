"""Pins for the oracle's retained-token selection (Section 4.1: the n visual tokens most
similar to the CLS token are retained)."""
import numpy as np
import pytest

from oracle import skipffn_oracle as O


def test_cosine_closed_forms():
    c = np.array([3.0, 4.0, 0.0])
    F = np.array([[3.0, 4.0, 0.0],        # same direction
                  [6.0, 8.0, 0.0],        # same direction, other length
                  [-3.0, -4.0, 0.0],      # opposite
                  [0.0, 0.0, 5.0],        # orthogonal
                  [4.0, 3.0, 0.0],        # cos = 24/25
                  [0.0, 0.0, 0.0]])       # zero vector
    assert np.allclose(O.cls_similarity(F, c), [1, 1, -1, 0, 24 / 25, 0], rtol=0, atol=1e-15)
    assert np.all(O.cls_similarity(F, np.zeros(3)) == 0)


def test_cosine_against_a_plain_loop_and_scale_invariance():
    rng = np.random.default_rng(0)
    F, c = rng.standard_normal((17, 9)), rng.standard_normal(9)
    want = []
    for t in range(17):
        dot = sum(F[t, j] * c[j] for j in range(9))
        want.append(dot / (sum(x * x for x in F[t]) ** 0.5 * sum(x * x for x in c) ** 0.5))
    got = O.cls_similarity(F, c)
    assert np.allclose(got, want, rtol=1e-13)
    assert np.allclose(O.cls_similarity(F * 7.5, c * 0.01), got, rtol=1e-13)
    assert np.all(np.abs(got) <= 1 + 1e-15)


@pytest.mark.parametrize("n,k", [(10, 3), (10, 0), (10, 10), (10, 25), (1, 1), (57, 20)])
def test_selection_against_sorting_by_hand(n, k):
    rng = np.random.default_rng(n + k)
    sim = rng.standard_normal(n)
    mask = O.select_top_n(sim, k)
    kk = min(k, n)
    assert mask.dtype == np.uint8 and int((mask == 0).sum()) == kk
    if 0 < kk < n:
        assert sim[mask == 0].min() >= sim[mask == 1].max()
    # brute force: a token is retained iff fewer than k tokens beat it
    for t in range(n):
        beats = sum(1 for u in range(n) if sim[u] > sim[t] or (sim[u] == sim[t] and u < t))
        assert mask[t] == (0 if beats < kk else 1)


def test_ties_go_to_the_lower_index():
    sim = np.array([0.5, 0.9, 0.5, 0.5, 0.1])
    assert O.select_top_n(sim, 2).tolist() == [0, 0, 1, 1, 1]
    assert O.select_top_n(sim, 3).tolist() == [0, 0, 0, 1, 1]


def test_bf16_interface_per_sequence():
    rng = np.random.default_rng(3)
    fb = O.f64_to_bf16_bits(rng.standard_normal((30, 8)))
    cb = O.f64_to_bf16_bits(rng.standard_normal((2, 8)))
    r = O.select_retained(fb, cb, [0, 12, 30], [4, 5])
    assert int((r["mask"][:12] == 0).sum()) == 4 and int((r["mask"][12:] == 0).sum()) == 5
    one = O.cls_similarity(O.bf16_bits_to_f64(fb[12:]), O.bf16_bits_to_f64(cb[1]))
    assert np.array_equal(r["sim"][12:], one)
    assert np.array_equal(r["mask"][12:], O.select_top_n(one, 5))
