"""Pins for the oracle's adaptive summary layer (Section 4.2, the summary-token equation):
closed forms, the library softmax, fp64 autograd and finite differences."""
import numpy as np
import pytest
import torch

from oracle import skipffn_oracle as O


def case(n, C, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal((n, C)), rng.standard_normal(C) * 0.3, rng.standard_normal(C)


def test_closed_forms():
    X, w, _ = case(7, 5, 0)
    # zero weight: every token scores 0, the summary is the plain mean
    f = O.summary_forward_real(X, np.zeros(5))
    assert np.allclose(f["xs"], X.mean(axis=0), rtol=0, atol=1e-15)
    assert np.allclose(f["p"], 1 / 7)
    # one token: the summary is that token, whatever the weight
    f = O.summary_forward_real(X[:1], w)
    assert np.array_equal(f["xs"], X[0])
    # a token whose score dominates takes all the weight
    Xd = X.copy(); Xd[3] = 50.0 * w / np.dot(w, w)          # score 50, the others O(1)
    f = O.summary_forward_real(Xd, w)
    assert f["p"][3] > 1 - 1e-15 and np.allclose(f["xs"], Xd[3], atol=1e-12)
    # two tokens: p0 = sigmoid(s0 - s1)
    f = O.summary_forward_real(X[:2], w)
    s = X[:2] @ w
    assert np.isclose(f["p"][0], 1 / (1 + np.exp(s[1] - s[0])), rtol=1e-14)


def test_weights_are_a_distribution_and_the_summary_a_convex_combination():
    X, w, _ = case(40, 9, 1)
    f = O.summary_forward_real(X, w)
    assert np.isclose(f["p"].sum(), 1.0, rtol=1e-14) and np.all(f["p"] > 0)
    assert np.all(f["xs"] <= X.max(axis=0) + 1e-12) and np.all(f["xs"] >= X.min(axis=0) - 1e-12)
    assert np.isclose(f["lse"], np.log(np.exp(f["s"]).sum()), rtol=1e-13)
    # order of the tokens does not matter
    perm = np.random.default_rng(2).permutation(40)
    assert np.allclose(O.summary_forward_real(X[perm], w)["xs"], f["xs"], rtol=1e-13, atol=1e-15)


def test_against_library_softmax_and_autograd():
    X, w, g = case(23, 11, 3)
    f = O.summary_forward_real(X, w)
    b = O.summary_backward_real(X, w, g)
    Xt = torch.tensor(X, requires_grad=True)
    wt = torch.tensor(w, requires_grad=True)
    xs = torch.softmax(Xt @ wt, dim=0) @ Xt
    assert np.allclose(f["xs"], xs.detach().numpy(), rtol=1e-13, atol=1e-15)
    (xs * torch.tensor(g)).sum().backward()
    assert np.allclose(b["dX"], Xt.grad.numpy(), rtol=1e-11, atol=1e-13)
    assert np.allclose(b["dw"], wt.grad.numpy(), rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("seed", [4, 5])
def test_finite_differences(seed):
    X, w, g = case(6, 4, seed)
    b = O.summary_backward_real(X, w, g)
    h = 1e-6

    def L():
        return float(np.dot(O.summary_forward_real(X, w)["xs"], g))

    for arr, name in ((X, "dX"), (w, "dw")):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h; lp = L()
            arr[i] = old - h; lm = L()
            arr[i] = old
            num[i] = (lp - lm) / (2 * h)
        assert np.linalg.norm(num - b[name]) / np.linalg.norm(b[name]) < 1e-8, name


def test_large_scores_do_not_overflow():
    X, w, _ = case(5, 3, 6)
    f = O.summary_forward_real(X * 1e3, w * 1e3)
    assert np.all(np.isfinite(f["xs"])) and np.isclose(f["p"].sum(), 1.0)


def test_bf16_interface_segments():
    rng = np.random.default_rng(7)
    T, C = 50, 16
    hid = O.f64_to_bf16_bits(rng.standard_normal((T, C)))
    wb = O.f64_to_bf16_bits(rng.standard_normal(C) * 0.3)
    tok = np.array([3, 4, 9, 20, 21, 22, 23, 40, 41], dtype=np.int32)
    seg = np.array([0, 3, 7, 9], dtype=np.int32)
    f = O.summary_forward(hid, tok, seg, wb)
    assert f["out_bits"].shape == (3, C)
    for i in range(3):
        rows = tok[seg[i]:seg[i + 1]]
        one = O.summary_forward_real(O.bf16_bits_to_f64(hid[rows]), O.bf16_bits_to_f64(wb))
        assert np.array_equal(f["out_bits"][i], O.f64_to_bf16_bits(one["xs"]))
    gout = O.f64_to_bf16_bits(rng.standard_normal((3, C)))
    gh0 = O.f64_to_bf16_bits(rng.standard_normal((T, C)))
    b = O.summary_backward(hid, tok, seg, wb, gout, gh0)
    untouched = np.setdiff1d(np.arange(T), tok)
    assert np.array_equal(b["gh_bits"][untouched], gh0[untouched])
    # dw is the sum of the per-set gradients
    tot = np.zeros(C)
    for i in range(3):
        rows = tok[seg[i]:seg[i + 1]]
        tot += O.summary_backward_real(O.bf16_bits_to_f64(hid[rows]), O.bf16_bits_to_f64(wb),
                                       O.bf16_bits_to_f64(gout[i]))["dw"]
    assert np.allclose(b["dw"], tot, rtol=1e-14)


def test_empty_set_gives_a_zero_row_and_no_gradient():
    rng = np.random.default_rng(8)
    hid = O.f64_to_bf16_bits(rng.standard_normal((10, 8)))
    wb = O.f64_to_bf16_bits(rng.standard_normal(8))
    tok = np.array([1, 2, 5], dtype=np.int32)
    seg = np.array([0, 2, 2, 3], dtype=np.int32)            # the middle set is empty
    f = O.summary_forward(hid, tok, seg, wb)
    assert np.all(f["out_bits"][1] == 0) and f["lse"][1] == -np.inf
    gout = O.f64_to_bf16_bits(rng.standard_normal((3, 8)))
    gh0 = O.f64_to_bf16_bits(rng.standard_normal((10, 8)))
    with_empty = O.summary_backward(hid, tok, seg, wb, gout, gh0)
    without = O.summary_backward(hid, tok, np.array([0, 2, 3], dtype=np.int32), wb, gout[[0, 2]], gh0)
    assert np.array_equal(with_empty["gh_bits"], without["gh_bits"])
    assert np.array_equal(with_empty["dw"], without["dw"])

