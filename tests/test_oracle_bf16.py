"""Pins for the oracle's bf16 conversions: torch's converter (a library
routine written independently), exhaustive round trips and closed-form tie
cases."""
import numpy as np
import torch

from oracle import skipffn_oracle as O


def torch_bits(a32):
    return torch.from_numpy(np.asarray(a32, dtype=np.float32)).to(torch.bfloat16) \
        .view(torch.int16).numpy().view(np.uint16)


def test_round_trip_all_patterns():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    wide = O.bf16_bits_to_f64(bits)
    back = O.f64_to_bf16_bits(wide)
    nan = np.isnan(wide)
    assert np.array_equal(back[~nan], bits[~nan])
    # NaNs stay NaNs with their sign
    assert np.all((back[nan] & 0x7F80) == 0x7F80) and np.all((back[nan] & 0x7F) != 0)
    assert np.array_equal(back[nan] >> 15, bits[nan] >> 15)


def test_widen_matches_torch():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float64).numpy()
    w = O.bf16_bits_to_f64(bits)
    ok = np.isnan(t) == np.isnan(w)
    assert ok.all()
    m = ~np.isnan(t)
    assert np.array_equal(t[m], w[m])
    assert np.array_equal(np.signbit(t[m]), np.signbit(w[m]))


def test_rounding_matches_torch_on_float32_inputs():
    rng = np.random.default_rng(0)
    a = np.concatenate([
        rng.standard_normal(200000).astype(np.float32),
        (rng.standard_normal(50000) * 1e-38).astype(np.float32),   # subnormal bf16 range
        (rng.standard_normal(50000) * 1e38).astype(np.float32),    # near overflow
        rng.integers(0, 2**32, 200000, dtype=np.uint64).astype(np.uint32).view(np.float32),
    ])
    a = a[~np.isnan(a)]
    assert np.array_equal(O.f64_to_bf16_bits(a.astype(np.float64)), torch_bits(a))


def test_ties_to_even_closed_form():
    # 1 + 2^-8 is half way between 1 (even) and 1 + 2^-7 (odd)
    one = 0x3F80
    assert O.f64_to_bf16_bits(np.array([1.0 + 2.0**-8]))[0] == one
    assert O.f64_to_bf16_bits(np.array([1.0 + 3 * 2.0**-8]))[0] == one + 2
    # anything above the tie goes up - this needs the single rounding from
    # float64 (a value below float32 resolution above the tie)
    assert O.f64_to_bf16_bits(np.array([1.0 + 2.0**-8 + 2.0**-40]))[0] == one + 1
    assert O.f64_to_bf16_bits(np.array([1.0 + 2.0**-8 - 2.0**-40]))[0] == one
    assert O.f64_to_bf16_bits(np.array([-0.0]))[0] == 0x8000
    assert O.f64_to_bf16_bits(np.array([np.inf, -np.inf])).tolist() == [0x7F80, 0xFF80]
    # largest finite bf16 is (2 - 2^-7) * 2^127; half a step above rounds to inf
    big = (2.0 - 2.0**-7) * 2.0**127
    assert O.f64_to_bf16_bits(np.array([big]))[0] == 0x7F7F
    assert O.f64_to_bf16_bits(np.array([big + 2.0**119]))[0] == 0x7F80
    assert O.f64_to_bf16_bits(np.array([big + 2.0**119 - 2.0**80]))[0] == 0x7F7F
    # smallest subnormal 2^-133; half of it ties to zero (even), a bit more goes up
    assert O.f64_to_bf16_bits(np.array([2.0**-133]))[0] == 1
    assert O.f64_to_bf16_bits(np.array([2.0**-134]))[0] == 0
    assert O.f64_to_bf16_bits(np.array([2.0**-134 * 1.0000001]))[0] == 1


def test_generator_bf16_bits_are_torch_bits():
    from paper_2503_21817_amd import workloads as W
    w = W.small()
    h = W.make_hidden(w)
    assert h.dtype == np.uint16 and h.shape == (w.T, w.C)
    # deterministic
    assert np.array_equal(h, W.make_hidden(w))
    v = O.bf16_bits_to_f64(h)
    assert abs(v.mean()) < 0.02 and abs(v.std() - 1.0) < 0.02
