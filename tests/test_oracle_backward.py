"""Pins for the oracle's backward pass: central finite differences, PyTorch
CPU float64 autograd (library), and the skip invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import workloads as W
from test_oracle_forward import real_case


def loss(x, skip, wg, wu, wd, g, wloss, eps=1e-5):
    return float(np.sum(O.skipffn_forward_real(x, skip, wg, wu, wd, g, eps)["out"] * wloss))


@pytest.mark.parametrize("seed,gain", [(0, True), (1, False), (2, True)])
def test_finite_differences(seed, gain):
    T, C, I = 6, 8, 12
    x, skip, wg, wu, wd, g = real_case(T, C, I, seed=seed, gain=gain)
    skip[0] = 0; skip[1] = 1
    rng = np.random.default_rng(100 + seed)
    wl = rng.standard_normal((T, C))
    grads = O.skipffn_backward_real(x, skip, wg, wu, wd, wl, g, 1e-5)
    h = 1e-5

    def fd(arr, name):
        num = np.zeros_like(arr)
        it = np.nditer(arr, flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            old = arr[i]
            arr[i] = old + h; lp = loss(x, skip, wg, wu, wd, g, wl)
            arr[i] = old - h; lm = loss(x, skip, wg, wu, wd, g, wl)
            arr[i] = old
            num[i] = (lp - lm) / (2 * h)
        ana = grads[name]
        err = np.linalg.norm(num - ana) / max(np.linalg.norm(ana), 1e-30)
        assert err < 1e-7, (name, err)

    fd(x, "dx"); fd(wg, "dw_gate"); fd(wu, "dw_up"); fd(wd, "dw_down")
    if g is not None:
        fd(g, "dgain")


@pytest.mark.parametrize("gain", [True, False])
def test_against_torch_autograd(gain):
    T, C, I = 9, 16, 24
    x, skip, wg, wu, wd, g = real_case(T, C, I, seed=11, gain=gain)
    rng = np.random.default_rng(12)
    gout = rng.standard_normal((T, C))
    mine = O.skipffn_backward_real(x, skip, wg, wu, wd, gout, g, 1e-5)

    xt = torch.tensor(x, requires_grad=True)
    tg, tu, td = (torch.tensor(a, requires_grad=True) for a in (wg, wu, wd))
    # without a gain the oracle reports the gradient at g = 1
    gt = torch.tensor(np.ones(C) if g is None else g, requires_grad=True)
    keep = torch.tensor(skip == 0)
    xr = xt[keep]
    n = F.rms_norm(xr, (C,), gt, 1e-5)
    y = F.linear(F.silu(F.linear(n, tg)) * F.linear(n, tu), td)
    out = xt.clone()
    out[keep] = xr + y
    (out * torch.tensor(gout)).sum().backward()
    for name, t in (("dx", xt), ("dw_gate", tg), ("dw_up", tu), ("dw_down", td), ("dgain", gt)):
        assert np.allclose(mine[name], t.grad.numpy(), rtol=1e-11, atol=1e-12), name


def test_skipped_gradient_is_bit_copy_and_retain_none_gives_zero_dw():
    w = W.small(C=32, I=48, visual=(20,), text=(4,), keep=(5,))
    h = W.make_hidden(w); m = W.make_mask(w); go = W.make_grad(w).copy()
    sk = np.flatnonzero(m)
    go[sk[0], :6] = [0x7FC1, 0xFF81, 0x7F80, 0xFF80, 0x8000, 0x0001]
    wg, wu, wd = W.make_weights(w)
    res = O.skipffn_backward(h, m, wg, wu, wd, go)
    assert np.array_equal(res["dx_bits"][sk], go[sk])
    none = O.skipffn_backward(h, np.ones(w.T, np.uint8), wg, wu, wd, go)
    assert np.array_equal(none["dx_bits"], go)
    for k in ("dw_gate", "dw_up", "dw_down"):
        assert none[k].shape == res[k].shape and not none[k].any()


def test_bf16_interface_matches_real_path():
    w = W.small(C=64, I=96, visual=(30, 17), text=(5, 4), keep=(9, 3))
    h = W.make_hidden(w); m = W.make_mask(w); go = W.make_grad(w)
    wg, wu, wd = W.make_weights(w); gn = W.make_gain(w, unit=False)
    res = O.skipffn_backward(h, m, wg, wu, wd, go, gn, 1e-5)
    wide = [O.bf16_bits_to_f64(a) for a in (wg, wu, wd)]
    real = O.skipffn_backward_real(O.bf16_bits_to_f64(h), m, *wide, O.bf16_bits_to_f64(go),
                                   O.bf16_bits_to_f64(gn), 1e-5)
    idx = res["idx"]
    assert np.array_equal(res["dx_bits"][idx], O.f64_to_bf16_bits(real["dx"][idx]))
    for k in ("dw_gate", "dw_up", "dw_down"):
        assert np.allclose(res[k], real[k], rtol=1e-12, atol=1e-14)


def test_weight_gradients_sum_over_tokens():
    # dW is a sum of per-token outer products: two halves of the retained set
    # add up to the whole
    x, skip, wg, wu, wd, g = real_case(10, 8, 12, seed=21)
    skip[:] = 0
    gout = np.random.default_rng(22).standard_normal((10, 8))
    full = O.skipffn_backward_real(x, skip, wg, wu, wd, gout, g)
    a = skip.copy(); a[5:] = 1
    b = skip.copy(); b[:5] = 1
    ga = O.skipffn_backward_real(x, a, wg, wu, wd, gout, g)
    gb = O.skipffn_backward_real(x, b, wg, wu, wd, gout, g)
    for k in ("dw_gate", "dw_up", "dw_down"):
        assert np.allclose(full[k], ga[k] + gb[k], rtol=1e-12, atol=1e-14)
