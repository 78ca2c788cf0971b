"""The register-only MFMA loop used as the measured ceiling does the arithmetic it is priced for."""
import pytest

pytestmark = pytest.mark.gpu


def test_probe_counts_every_mfma():
    import torch
    from paper_2503_21817_amd import binding as B

    blocks, iters = 8, 10
    out = torch.zeros(blocks * 256, dtype=torch.float32, device="cuda")
    clocks = torch.zeros(2 * blocks, dtype=torch.int64, device="cuda")
    B.skipffn_probe_mfma(blocks, iters, 0, out, clocks)
    torch.cuda.synchronize()
    # operands all 1.0: one 16x16x32 MFMA adds 32 to each accumulator element; a lane holds 4
    # elements of each of its 32 accumulator tiles and writes their sum
    assert torch.all(out == float(iters * 32 * 4 * 32))
    c = clocks.view(blocks, 2)
    assert torch.all(c > 0)
    # random operands: finite, and not all equal
    B.skipffn_probe_mfma(blocks, iters, 1, out, clocks)
    torch.cuda.synchronize()
    assert torch.isfinite(out).all() and out.unique().numel() > 1


def test_probe_rejects_bad_arguments():
    from paper_2503_21817_amd import binding as B

    rc = B.lib().skipffn_probe_mfma(4, 4, 0, None, None, None)
    assert rc != 0
    assert B.lib().skipffn_probe_mfma(0, 0, 0, None, None, None) == 0
