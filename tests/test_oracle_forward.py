"""Pins for the oracle's forward pass (Eq. 4 / Eq. 5 of Section 4.2)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import workloads as W


def real_case(T=7, C=8, I=12, seed=0, frac_skip=0.5, gain=True):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, C))
    wg = rng.standard_normal((I, C)) * 0.4
    wu = rng.standard_normal((I, C)) * 0.4
    wd = rng.standard_normal((C, I)) * 0.4
    g = 1.0 + 0.2 * rng.standard_normal(C) if gain else None
    skip = (rng.random(T) < frac_skip).astype(np.uint8)
    return x, skip, wg, wu, wd, g


def torch_layer(x, wg, wu, wd, g, eps):
    """Second witness: PyTorch CPU float64 library ops."""
    xt = torch.tensor(x, dtype=torch.float64)
    gt = None if g is None else torch.tensor(g, dtype=torch.float64)
    n = F.rms_norm(xt, (x.shape[1],), gt, eps)
    h = F.silu(F.linear(n, torch.tensor(wg))) * F.linear(n, torch.tensor(wu))
    return (xt + F.linear(h, torch.tensor(wd))).numpy()


@pytest.mark.parametrize("gain", [True, False])
def test_retain_all_equals_plain_layer(gain):
    x, _, wg, wu, wd, g = real_case(T=9, C=16, I=24, seed=1, gain=gain)
    skip = np.zeros(9, np.uint8)
    out = O.skipffn_forward_real(x, skip, wg, wu, wd, g, 1e-5)["out"]
    dense = O.dense_swiglu_layer(x, wg, wu, wd, g, 1e-5)
    lib = torch_layer(x, wg, wu, wd, g, 1e-5)
    assert np.allclose(out, dense, rtol=1e-12, atol=1e-13)
    assert np.allclose(out, lib, rtol=1e-12, atol=1e-13)


def test_retained_rows_match_library_layer_under_a_mask():
    x, skip, wg, wu, wd, g = real_case(T=11, C=16, I=20, seed=2)
    res = O.skipffn_forward_real(x, skip, wg, wu, wd, g, 1e-5)
    lib = torch_layer(x, wg, wu, wd, g, 1e-5)
    keep = skip == 0
    assert keep.any() and (~keep).any()
    assert np.allclose(res["out"][keep], lib[keep], rtol=1e-12, atol=1e-13)
    assert np.array_equal(res["out"][~keep], x[~keep])


def test_retain_none_is_identity():
    w = W.small(C=32, I=48, visual=(10,), text=(0,), keep=(0,))
    h = W.make_hidden(w)
    wg, wu, wd = W.make_weights(w)
    res = O.skipffn_forward(h, np.ones(w.T, np.uint8), wg, wu, wd)
    assert res["R"] == 0 and res["idx"].shape == (0,)
    assert np.array_equal(res["out_bits"], h)


def test_skipped_rows_bitwise_including_special_values():
    w = W.small(C=32, I=48, visual=(20,), text=(4,), keep=(5,))
    h = W.make_hidden(w).copy()
    m = W.make_mask(w)
    sk = np.flatnonzero(m)
    # NaN payloads (quiet and signalling), infinities, negative zero, subnormals
    h[sk[0], :8] = [0x7FC1, 0xFFC0, 0x7F81, 0xFF85, 0x7F80, 0xFF80, 0x8000, 0x0001]
    h[sk[1], :] = 0x8000
    wg, wu, wd = W.make_weights(w)
    res = O.skipffn_forward(h, m, wg, wu, wd)
    assert np.array_equal(res["out_bits"][sk], h[sk])
    # and retained rows did change
    assert not np.array_equal(res["out_bits"][res["idx"]], h[res["idx"]])


def test_zero_down_or_gate_projection_leaves_input():
    w = W.small(C=32, I=48, visual=(12,), text=(3,), keep=(6,))
    h = W.make_hidden(w); m = W.make_mask(w)
    wg, wu, wd = W.make_weights(w)
    z = np.zeros_like(wd)
    assert np.array_equal(O.skipffn_forward(h, m, wg, wu, z)["out_bits"], h)
    zg = np.zeros_like(wg)
    assert np.array_equal(O.skipffn_forward(h, m, zg, wu, wd)["out_bits"], h)   # silu(0) = 0


def test_constant_row_closed_form():
    # x = a * ones  =>  n(x) = sign(a) / sqrt(1 + eps / a^2) in every channel
    C, eps = 16, 1e-5
    for a in (3.0, -0.25):
        xn, rstd = O.rmsnorm_rows(np.full((1, C), a), None, eps)
        assert np.allclose(xn, math.copysign(1.0, a) / math.sqrt(1 + eps / a**2), rtol=1e-14)
        assert np.isclose(rstd[0], 1 / math.sqrt(a * a + eps), rtol=1e-14)


def test_power_of_two_scale_invariance():
    # FFN(2x) = FFN(x) when eps = 0 (RMSNorm removes the scale); with eps > 0 the
    # difference is of relative size eps / mean(x^2)
    x, skip, wg, wu, wd, g = real_case(T=6, C=16, I=20, seed=4)
    z = np.zeros(6, np.uint8)
    y1 = O.skipffn_forward_real(x, z, wg, wu, wd, g, 0.0)["Y"]
    y2 = O.skipffn_forward_real(2 * x, z, wg, wu, wd, g, 0.0)["Y"]
    assert np.allclose(y1, y2, rtol=1e-13, atol=1e-14)
    y3 = O.skipffn_forward_real(x, z, wg, wu, wd, g, 1e-5)["Y"]
    assert 0 < np.abs(y3 - y1).max() < 1e-4 * np.abs(y1).max()


def test_hand_worked_example():
    # C = 2, I = 1, eps = 0: x = (3, 4): mean square 12.5, xn = x / sqrt(12.5).
    # W_gate = (1, 0) -> G = 3/sqrt(12.5); W_up = (0, 1) -> U = 4/sqrt(12.5);
    # H = G * U / (1 + e^-G) ; W_down = (2, -1)^T -> Y = (2H, -H).
    x = np.array([[3.0, 4.0]])
    r = math.sqrt(12.5)
    G, U = 3 / r, 4 / r
    H = G * U / (1 + math.exp(-G))
    res = O.skipffn_forward_real(x, np.zeros(1, np.uint8), np.array([[1.0, 0.0]]),
                                 np.array([[0.0, 1.0]]), np.array([[2.0], [-1.0]]), None, 0.0)
    assert np.allclose(res["out"], [[3 + 2 * H, 4 - H]], rtol=1e-14)
    # numerically: G = 0.848528..., sigmoid(G) = 0.700268..., H = 0.672229...
    assert abs(H - 0.6722) < 1e-4 and abs(res["out"][0, 0] - 4.3445) < 1e-4
    # transposed-operand check: non-square, asymmetric weights, one token, by loops
    rng = np.random.default_rng(5)
    C, I = 3, 5
    xx = rng.standard_normal(C); wg = rng.standard_normal((I, C)); wu = rng.standard_normal((I, C))
    wd = rng.standard_normal((C, I)); g = rng.standard_normal(C); eps = 1e-5
    ms = sum(v * v for v in xx) / C
    xn = [xx[c] / math.sqrt(ms + eps) * g[c] for c in range(C)]
    Gs = [sum(xn[c] * wg[i, c] for c in range(C)) for i in range(I)]
    Us = [sum(xn[c] * wu[i, c] for c in range(C)) for i in range(I)]
    Hs = [Gs[i] / (1 + math.exp(-Gs[i])) * Us[i] for i in range(I)]
    outs = [xx[c] + sum(Hs[i] * wd[c, i] for i in range(I)) for c in range(C)]
    got = O.skipffn_forward_real(xx[None], np.zeros(1, np.uint8), wg, wu, wd, g, eps)["out"][0]
    assert np.allclose(got, outs, rtol=1e-13)


def test_skip_error_identity_and_token_independence():
    # Section 5 (per-layer skipping error): for a token skipped under mask A and
    # retained under mask B, out_B - out_A = FFN(h) and its norm is the error.
    x, skip, wg, wu, wd, g = real_case(T=10, C=16, I=20, seed=6)
    A = skip.copy(); A[3] = 1
    B = A.copy(); B[3] = 0
    ra = O.skipffn_forward_real(x, A, wg, wu, wd, g)
    rb = O.skipffn_forward_real(x, B, wg, wu, wd, g)
    ffn3 = O.ffn_rows(x[3:4], wg, wu, wd, g, 1e-5)["Y"][0]
    assert np.allclose(rb["out"][3] - ra["out"][3], ffn3, rtol=1e-13, atol=1e-14)
    eps_l = np.linalg.norm(rb["out"][3] - ra["out"][3])
    assert np.isclose(eps_l, np.linalg.norm(ffn3))
    others = np.arange(10) != 3
    assert np.array_equal(ra["out"][others], rb["out"][others])
    # changing another token's value does not touch this token's output
    x2 = x.copy(); x2[5] += 1.0
    rc = O.skipffn_forward_real(x2, B, wg, wu, wd, g)
    assert np.array_equal(rc["out"][others & (np.arange(10) != 5)],
                          rb["out"][others & (np.arange(10) != 5)])
    assert np.array_equal(rc["out"][3], rb["out"][3])


def test_bf16_interface_is_real_path_rounded_once():
    w = W.small(C=64, I=96, visual=(30, 17), text=(5, 4), keep=(9, 3))
    h = W.make_hidden(w); m = W.make_mask(w)
    wg, wu, wd = W.make_weights(w); gn = W.make_gain(w, unit=False)
    res = O.skipffn_forward(h, m, wg, wu, wd, gn, 1e-5)
    real = O.skipffn_forward_real(O.bf16_bits_to_f64(h), m, *(O.bf16_bits_to_f64(a) for a in (wg, wu, wd)),
                                  O.bf16_bits_to_f64(gn), 1e-5)
    assert np.array_equal(res["idx"], real["idx"])
    assert np.array_equal(res["out_bits"][res["idx"]], O.f64_to_bf16_bits(real["out"][res["idx"]]))
    # witness on the widened values: torch library layer, within one bf16 ulp
    lib = torch_layer(O.bf16_bits_to_f64(h), *(O.bf16_bits_to_f64(a) for a in (wg, wu, wd)),
                      O.bf16_bits_to_f64(gn), 1e-5)
    got = O.bf16_bits_to_f64(res["out_bits"])
    keep = m == 0
    assert np.all(np.abs(got[keep] - lib[keep]) <= 2.0**-8 * np.abs(lib[keep]) + 1e-30)
    nr = O.skipffn_forward(h, m, wg, wu, wd, gn, 1e-5, no_residual=True)
    assert np.array_equal(nr["out_bits"][nr["idx"]], O.f64_to_bf16_bits(real["Y"]))
    assert np.array_equal(nr["out_bits"][m != 0], h[m != 0])
