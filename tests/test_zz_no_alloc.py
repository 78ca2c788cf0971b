"""The workspace-free compaction entry point (for callers that cannot allocate) against the
ordinary one, through the C ABI: bit-exact indices, count and positions, on two calls in a row of
which the second is smaller (the built-in scratch keeps the first call's contents)."""
import numpy as np
import pytest
import torch

from paper_2503_21817_amd import binding as B

pytestmark = pytest.mark.gpu


def _both(mask_np):
    T = mask_np.shape[0]
    mask = torch.from_numpy(mask_np).cuda()
    ref_idx = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    ref_n = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    ref_pos = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    ws = torch.empty(max(B.skipffn_compact_workspace_bytes(T), 16), dtype=torch.uint8, device="cuda")
    B.skipffn_compact(mask, ref_idx, ref_n, ref_pos, ws)
    idx = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    n = torch.full((1,), -5, dtype=torch.int32, device="cuda")
    pos = torch.full((T,), -5, dtype=torch.int32, device="cuda")
    B.skipffn_compact_static(mask, idx, n, pos)
    torch.cuda.synchronize()
    return (ref_idx, ref_n, ref_pos), (idx, n, pos)


def test_static_scratch_compaction_matches_the_workspace_one_twice_in_a_row():
    rng = np.random.default_rng(2024)
    # sizes beyond one block (262144 tokens), where the scratch is in use; the second call is
    # smaller and its mask differs; then a one-block size that does not touch the scratch
    for T, keep in ((2**20 + 37, 0.25), (300_001, 0.6), (5_000, 0.1)):
        mask_np = (rng.random(T) >= keep).astype(np.uint8)
        ref, got = _both(mask_np)
        R = int(ref[1].item())
        assert R == int((mask_np == 0).sum()) == int(got[1].item())
        assert torch.equal(got[0], ref[0])                     # idx[0..R) and the untouched tail
        assert np.array_equal(got[0][:R].cpu().numpy(), np.flatnonzero(mask_np == 0))
        assert torch.equal(got[2], ref[2])


def test_static_scratch_compaction_rejects_sizes_beyond_its_scratch():
    lim = B.skipffn_compact_static_max_tokens()
    assert lim == 2**28
    fake = 0x7f0000001000
    assert B.lib().skipffn_compact_static(fake, lim + 1, fake, fake, None, None) == B.ESHAPE
    assert B.lib().skipffn_compact_static(fake, -1, fake, fake, None, None) == B.EINVAL
