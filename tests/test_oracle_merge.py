"""Pins for the oracle's token merge (Section 4.1): library cosine similarities, plain loops,
closed forms and structural invariants."""
import numpy as np
import pytest
from sklearn.metrics.pairwise import cosine_similarity

from oracle import skipffn_oracle as O


def test_cosine_matrix_against_the_library_and_a_loop():
    rng = np.random.default_rng(0)
    X = rng.standard_normal((13, 7))
    S = O.cosine_matrix(X)
    assert np.allclose(S, cosine_similarity(X), rtol=1e-13, atol=1e-15)
    for i in range(13):
        for j in range(13):
            want = float(X[i] @ X[j]) / (np.linalg.norm(X[i]) * np.linalg.norm(X[j]))
            assert abs(S[i, j] - want) < 1e-14
    assert np.allclose(np.diag(S), 1.0) and np.allclose(S, S.T)
    Z = X.copy(); Z[4] = 0
    assert np.all(O.cosine_matrix(Z)[4] == 0)


def test_average_excludes_the_token_itself():
    S = np.array([[1.0, 0.5, -0.5], [0.5, 1.0, 0.0], [-0.5, 0.0, 1.0]])
    assert np.allclose(O.average_similarity(S), [0.0, 0.25, -0.25])
    assert np.all(O.average_similarity(np.ones((1, 1))) == 0)


def brute(X, k):
    """The three steps written as plain loops."""
    n = len(X)
    S = [[float(X[i] @ X[j]) / (np.linalg.norm(X[i]) * np.linalg.norm(X[j])) for j in range(n)] for i in range(n)]
    avg = [sum(S[i][j] for j in range(n) if j != i) / (n - 1) for i in range(n)]
    kept = []
    for t in range(n):
        lower = sum(1 for u in range(n) if avg[u] < avg[t] or (avg[u] == avg[t] and u < t))
        if lower < k:
            kept.append(t)
    groups = {j: [j] for j in kept}
    for i in range(n):
        if i not in groups:
            best = max(kept, key=lambda j: (S[i][j], -j))
            groups[best].append(i)
    merged = np.stack([np.mean([X[i] for i in sorted(groups[j])], axis=0) for j in kept])
    return kept, groups, merged


@pytest.mark.parametrize("n,k,seed", [(12, 4, 1), (9, 1, 2), (9, 9, 3), (30, 7, 4)])
def test_against_plain_loops(n, k, seed):
    X = np.random.default_rng(seed).standard_normal((n, 6))
    r = O.token_merge_real(X, k)
    kept, groups, merged = brute(X, k)
    assert r["kept"].tolist() == kept
    for slot, j in enumerate(kept):
        assert sorted(np.flatnonzero(r["assign"] == slot).tolist()) == sorted(groups[j])
    assert np.allclose(r["merged"], merged, rtol=1e-13, atol=1e-15)


def test_closed_forms():
    rng = np.random.default_rng(5)
    X = rng.standard_normal((8, 5))
    # k = n: nothing is merged;  k = 1: one token, the mean of all
    assert np.array_equal(O.token_merge_real(X, 8)["merged"], X)
    assert np.allclose(O.token_merge_real(X, 1)["merged"][0], X.mean(axis=0))
    assert np.array_equal(O.token_merge_real(X, 20)["merged"], X)          # k > n
    # a tight cluster plus one outlier orthogonal to it: the outlier has the lowest average
    # similarity, so it is kept first; with k = 2 the cluster collapses onto its own kept member
    a, b = np.array([1.0, 0, 0, 0, 0]), np.array([0, 1.0, 0, 0, 0])
    Y = np.stack([a + 0.01 * rng.standard_normal(5) for _ in range(3)] + [b] +
                 [a + 0.01 * rng.standard_normal(5) for _ in range(2)])
    assert O.token_merge_real(Y, 1)["kept"].tolist() == [3]
    r = O.token_merge_real(Y, 2)
    assert 3 in r["kept"].tolist()
    slot_out = r["kept"].tolist().index(3)
    assert np.flatnonzero(r["assign"] == slot_out).tolist() == [3]          # nobody merges into the outlier
    assert np.allclose(r["merged"][1 - slot_out], Y[[0, 1, 2, 4, 5]].mean(axis=0))
    # a duplicated token goes to its twin (similarity exactly 1) when only the twin is kept
    D = np.stack([X[0], X[1], X[2], X[1]])
    S = O.cosine_matrix(D)
    kept, assign = O.merge_decisions(S, np.array([0.0, 0.1, 0.2, 0.3]), 3)   # keep 0, 1, 2
    assert kept.tolist() == [0, 1, 2] and assign.tolist() == [0, 1, 2, 1]


def test_structure_every_token_lands_in_exactly_one_kept_slot():
    X = np.random.default_rng(6).standard_normal((40, 8))
    r = O.token_merge_real(X, 11)
    assert len(r["kept"]) == 11 and np.all(np.diff(r["kept"]) > 0)
    assert np.all((r["assign"] >= 0) & (r["assign"] < 11))
    assert np.all(r["assign"][r["kept"]] == np.arange(11))
    # the merge preserves the token sum weighted by group size
    cnt = np.bincount(r["assign"], minlength=11)
    assert np.allclose((r["merged"] * cnt[:, None]).sum(axis=0), X.sum(axis=0), rtol=1e-12)
    # the kept tokens are the least similar on average
    assert r["avg"][r["kept"]].max() <= np.delete(r["avg"], r["kept"]).min()


def test_bf16_interface():
    rng = np.random.default_rng(7)
    xb = O.f64_to_bf16_bits(rng.standard_normal((25, 8)))
    r = O.token_merge(xb, [0, 10, 10, 25], 6)
    assert r["out_bits"].shape == (3, 6, 8) and np.all(r["out_bits"][1] == 0) and np.all(r["kept"][1] == -1)
    one = O.token_merge_real(O.bf16_bits_to_f64(xb[10:25]), 6)
    assert np.array_equal(r["kept"][2], one["kept"] + 10)
    assert np.array_equal(r["out_bits"][2], O.f64_to_bf16_bits(one["merged"]))


# ---- gradient of the merge (decisions held fixed) -----------------------------------------------
def test_merge_gradient_against_central_differences_of_the_whole_merge():
    """At a generic point the kept set and the assignment do not change under a small step, so
    the difference quotient of the COMPLETE merge (similarities, selection, assignment, mean)
    must equal the gradient that treats the decisions as constants."""
    rng = np.random.default_rng(5)
    n, C, k = 9, 5, 3
    X = rng.standard_normal((n, C))
    r = O.token_merge_real(X, k)
    Wt = rng.standard_normal(r["merged"].shape)          # loss = sum(merged * Wt)
    dX = O.merge_rows_backward(Wt, r["assign"], n)
    h = 1e-6
    for i in range(n):
        for c in range(C):
            Xp = X.copy(); Xp[i, c] += h
            Xm = X.copy(); Xm[i, c] -= h
            rp, rm = O.token_merge_real(Xp, k), O.token_merge_real(Xm, k)
            assert np.array_equal(rp["assign"], r["assign"]) and np.array_equal(rm["assign"], r["assign"])
            fd = (np.sum(rp["merged"] * Wt) - np.sum(rm["merged"] * Wt)) / (2 * h)
            assert abs(fd - dX[i, c]) < 1e-8, (i, c)


def test_merge_gradient_against_autograd_and_the_adjoint_identity():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(6)
    n, C, kk = 40, 6, 7
    assign = rng.integers(-1, kk, n)
    assign[:kk] = np.arange(kk)                          # every slot has a member
    X = rng.standard_normal((n, C))
    G = rng.standard_normal((kk, C))
    dX = O.merge_rows_backward(G, assign, n)
    # <merge_rows(X), G> == <X, backward(G)>: the backward is the transpose of the forward
    assert abs(np.sum(O.merge_rows(X, assign, kk) * G) - np.sum(X * dX)) < 1e-12
    # library witness: a scatter-mean built from index_add, differentiated by autograd
    xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    sel = torch.tensor(np.flatnonzero(assign >= 0))
    slot = torch.tensor(assign[assign >= 0])
    sums = torch.zeros(kk, C, dtype=torch.float64).index_add(0, slot, xt[sel])
    cnt = torch.zeros(kk, dtype=torch.float64).index_add(0, slot, torch.ones(len(sel), dtype=torch.float64))
    (sums / cnt[:, None] * torch.tensor(G)).sum().backward()
    assert np.allclose(dX, xt.grad.numpy(), rtol=0, atol=1e-14)
    assert np.all(dX[assign < 0] == 0)


def test_merge_gradient_closed_forms_and_bf16_interface():
    # a set kept whole: every token is its own slot, the gradient passes through unchanged
    rng = np.random.default_rng(7)
    xb = O.f64_to_bf16_bits(rng.standard_normal((11, 8)))
    seg = [0, 4, 4, 11]
    k = 7
    fwd = O.token_merge(xb, seg, k)
    gb = O.f64_to_bf16_bits(rng.standard_normal((3, k, 8)))
    bwd = O.token_merge_backward(gb, seg, k, fwd["assign"])
    assert np.array_equal(bwd["dx_bits"][0:4], gb[0, :4])
    assert np.array_equal(bwd["dx_bits"][4:11], gb[2, :7])
    # k = 1: one slot holding the mean of all n tokens: every row gets grad / n
    fwd1 = O.token_merge(xb, [0, 11], 1)
    g1 = O.f64_to_bf16_bits(rng.standard_normal((1, 1, 8)))
    b1 = O.token_merge_backward(g1, [0, 11], 1, fwd1["assign"])
    assert np.allclose(b1["dx"], O.bf16_bits_to_f64(g1[0, 0])[None, :] / 11, rtol=0, atol=1e-16)
    # column sums: the gradients handed to the members of a slot add up to the slot's gradient
    fwd2 = O.token_merge(xb, [0, 11], 3)
    g2 = O.f64_to_bf16_bits(rng.standard_normal((1, 3, 8)))
    b2 = O.token_merge_backward(g2, [0, 11], 3, fwd2["assign"])
    for j in range(3):
        assert np.allclose(b2["dx"][fwd2["assign"] == j].sum(0), O.bf16_bits_to_f64(g2[0, j]), atol=1e-14)
