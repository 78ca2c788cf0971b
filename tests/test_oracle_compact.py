"""Pins for the retained-index compaction: brute force on small masks."""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle import skipffn_oracle as O
from paper_2503_21817_amd import workloads as W


def brute(mask):
    idx = [t for t in range(len(mask)) if mask[t] == 0]
    pos = [-1] * len(mask)
    for r, t in enumerate(idx):
        pos[t] = r
    return idx, pos


@pytest.mark.parametrize("T", [0, 1, 2, 63, 64, 65, 255, 256, 257, 1023, 1025, 3001])
@pytest.mark.parametrize("kind", ["all0", "all1", "alt", "first", "last", "rand", "bytes"])
def test_compact_brute_force(T, kind):
    rng = np.random.default_rng(T * 7 + len(kind))
    if kind == "all0":
        m = np.zeros(T, np.uint8)
    elif kind == "all1":
        m = np.ones(T, np.uint8)
    elif kind == "alt":
        m = (np.arange(T) % 2).astype(np.uint8)
    elif kind == "first":
        m = np.ones(T, np.uint8); m[:1] = 0
    elif kind == "last":
        m = np.ones(T, np.uint8); m[-1:] = 0
    elif kind == "rand":
        m = (rng.random(T) < 0.7).astype(np.uint8)
    else:  # any non-zero byte means skip
        m = rng.integers(0, 256, T).astype(np.uint8) * (rng.random(T) < 0.5)
        m = m.astype(np.uint8)
    idx, R, pos = O.compact(m)
    bidx, bpos = brute(m.tolist())
    assert R == len(bidx)
    assert idx.dtype == np.int32 and idx.tolist() == bidx
    assert pos.tolist() == bpos


@settings(max_examples=200, deadline=None)
@given(st.lists(st.integers(0, 255), max_size=300))
def test_compact_property(bytes_):
    m = np.array(bytes_, dtype=np.uint8)
    idx, R, pos = O.compact(m)
    assert np.all(np.diff(idx) > 0)
    assert R == int(np.sum(m == 0))
    assert np.all(m[idx] == 0)
    assert np.array_equal(np.flatnonzero(pos >= 0), idx)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5])
def test_workload_masks_have_declared_counts(cfg):
    w = W.config(cfg)
    m = W.make_mask(w)
    assert m.shape == (w.T,)
    idx, R, _ = O.compact(m)
    assert R == w.R
    # per sequence: text always retained, exactly keep visual retained
    off = 0
    for v, t, k in zip(w.visual, w.text, w.keep):
        assert int(np.sum(m[off:off + v] == 0)) == k
        assert np.all(m[off + v:off + v + t] == 0)
        off += v + t
    if cfg == 2:
        assert (w.T, w.R) == (4928, 1472)
    if cfg == 3:
        assert (w.T, w.R) == (11776, 2560)
        ws = W.config(3, structured=True)
        ms = W.make_mask(ws)
        assert np.all(ms[:576] == 0) and np.all(ms[576:2880] == 1)
    if cfg == 5:
        assert (w.T, w.R, w.layers) == (9856, 2944, 32)


def test_kv_skip_cache_is_row_selection():
    rng = np.random.default_rng(3)
    cache = rng.integers(0, 65536, (50, 16)).astype(np.uint16)
    m = (rng.random(50) < 0.6).astype(np.uint8)
    kept = O.kv_skip_cache(cache, m)
    rows = [cache[t] for t in range(50) if m[t] == 0]
    assert kept.shape[0] == len(rows)
    for a, b in zip(kept, rows):
        assert np.array_equal(a, b)


def test_kv_skip_cache_all_is_the_set_difference_of_every_slab():
    """Section 4.3: the compacted cache is the cache minus the rows of skipped tokens.  The
    oracle gathers retained rows; deleting the skipped rows (numpy.delete) is the same set
    difference written the other way round, and a plain loop checks one slab row by row."""
    rng = np.random.default_rng(9)
    L, H, T, D = 3, 4, 57, 8
    cache = rng.integers(0, 65536, (L, 2, H, T, D)).astype(np.uint16)
    skip = (rng.random(T) < 0.6).astype(np.uint8)
    got = O.kv_skip_cache_all(cache, skip)
    skipped_positions = np.flatnonzero(skip != 0)
    want = np.delete(cache, skipped_positions, axis=-2)
    assert got.shape == want.shape == (L, 2, H, T - len(skipped_positions), D)
    assert np.array_equal(got, want)
    rows = [cache[2, 1, 3, t] for t in range(T) if skip[t] == 0]
    assert np.array_equal(got[2, 1, 3], np.stack(rows))
    # nothing skipped / everything skipped
    assert np.array_equal(O.kv_skip_cache_all(cache, np.zeros(T, np.uint8)), cache)
    assert O.kv_skip_cache_all(cache, np.ones(T, np.uint8)).shape == (L, 2, H, 0, D)

