"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every declared symbol, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from paper_2503_21817_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "skipffn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(skipffn_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.lib()
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.exported_symbols()) == names
    assert B.skipffn_version() >= 100


def test_status_strings():
    lib = B.lib()
    seen = {lib.skipffn_status_string(i).decode() for i in range(7)}
    assert len(seen) == 7
    assert "unknown" in lib.skipffn_status_string(99).decode()


def test_size_queries_are_monotone_and_cover_their_sections():
    C, I = 4096, 14336
    for R in (0, 1, 255, 1472, 2560):
        sv = B.skipffn_saved_bytes(R, C, I)
        off = B.skipffn_saved_layout(R, C, I)
        assert off == sorted(off) and off[0] == 0
        assert len(off) == 8 and sv >= off[7] + I * ((R + 63) // 64 * 64) * 2
        assert off[7] - off[6] >= C * ((R + 63) // 64 * 64) * 2
        assert off[6] - off[5] >= R * I * 2
        assert off[1] - off[0] >= R * C * 2 and off[3] - off[2] >= R * 4
        fw_inf = B.skipffn_forward_workspace_bytes(R, C, I, False)
        fw_tr = B.skipffn_forward_workspace_bytes(R, C, I, True)
        assert fw_inf >= fw_tr >= R * C * 4
        assert B.skipffn_backward_workspace_bytes(R, C, I) >= R * C * 2 + 2 * R * I * 2
    assert B.skipffn_saved_bytes(2560, C, I) > B.skipffn_saved_bytes(1472, C, I)
    assert B.skipffn_compact_workspace_bytes(0) > 0
    assert B.skipffn_compact_workspace_bytes(1 << 26) >= 2 * 4 * ((1 << 26) // 65536)


FAKE = 0x7f0000001000      # aligned, never dereferenced: validation fails first
ODD = FAKE + 2


def fwd(T=8, C=64, I=128, eps=1e-5, hidden=FAKE, out=FAKE, idx=FAKE, R=4, nr=None, gain=None,
        wg=FAKE, wu=FAKE, wd=FAKE, saved=None, ws=FAKE, ws_bytes=1 << 40, flags=0):
    return B.lib().skipffn_forward(T, C, I, eps, hidden, out, idx, R, nr, gain, wg, wu, wd, saved,
                                   ws, ws_bytes, flags, None)


def bwd(T=8, C=64, I=128, go=FAKE, gh=FAKE, idx=FAKE, R=4, nr=None, wg=FAKE, wu=FAKE, wd=FAKE,
        saved=FAKE, dwg=FAKE, dwu=FAKE, dwd=FAKE, dgain=None, ws=FAKE, ws_bytes=1 << 40, flags=0):
    return B.lib().skipffn_backward(T, C, I, 1e-5, go, gh, idx, R, nr, None, wg, wu, wd, saved,
                                    dwg, dwu, dwd, dgain, ws, ws_bytes, flags, None)


def test_forward_rejects_bad_arguments_on_the_host():
    assert fwd(T=-1) == B.EINVAL
    assert fwd(R=9) == B.EINVAL                 # R > T
    assert fwd(R=-1, nr=None) == B.EINVAL       # device count requested, no pointer
    assert fwd(R=-2) == B.EINVAL
    assert fwd(C=60) == B.ESHAPE
    assert fwd(I=100) == B.ESHAPE
    assert fwd(T=1 << 20, C=4096, R=4) == B.ESHAPE      # hidden >= 2 GiB
    assert fwd(hidden=None) == B.EINVAL
    assert fwd(hidden=ODD) == B.EINVAL
    assert fwd(out=FAKE + 16) == B.EINVAL       # partial overlap
    assert fwd(idx=None) == B.EINVAL
    assert fwd(wg=None) == B.EINVAL
    assert fwd(wd=ODD) == B.EINVAL
    assert fwd(gain=ODD) == B.EINVAL
    assert fwd(flags=0x100) == B.EUNSUPPORTED
    assert fwd(ws=None) == B.EWORKSPACE
    assert fwd(ws_bytes=16) == B.EWORKSPACE
    assert fwd(eps=float("nan")) == B.EINVAL
    # T == 0 and R == 0 in place are valid no-ops that enqueue nothing
    assert fwd(T=0, R=0, hidden=None, out=None, idx=None, ws=None, ws_bytes=0) == B.OK
    assert fwd(R=0, idx=None, ws=None, ws_bytes=0) == B.OK
    # the index check is a known flag bit; with nothing retained (or no tokens) nothing is enqueued
    assert fwd(R=0, idx=None, ws=None, ws_bytes=0, flags=B.FLAG_VALIDATE_IDX) == B.OK
    assert fwd(T=0, R=0, hidden=None, out=None, idx=None, ws=None, ws_bytes=0, flags=B.FLAG_VALIDATE_IDX) == B.OK
    assert fwd(flags=0x20) == B.EUNSUPPORTED


def test_compact_static_rejects_bad_arguments_on_the_host():
    c = B.lib().skipffn_compact_static        # skip_mask, T, idx, num_retained, pos, stream
    lim = B.skipffn_compact_static_max_tokens()
    assert lim == 2 ** 28
    assert c(FAKE, lim + 1, FAKE, FAKE, None, None) == B.ESHAPE       # beyond the built-in scratch
    assert c(FAKE, -1, FAKE, FAKE, None, None) == B.EINVAL
    assert c(FAKE, 10, FAKE, None, None, None) == B.EINVAL           # no count output
    assert c(ODD, 10, FAKE, FAKE, None, None) == B.EINVAL
    assert c(FAKE, 10, None, FAKE, None, None) == B.EINVAL


def test_validate_idx_rejects_bad_arguments_on_the_host():
    v = B.lib().skipffn_validate_idx          # idx, R, num_retained, T, status, stream
    assert v(FAKE, 4, None, -1, FAKE, None) == B.EINVAL
    assert v(FAKE, 9, None, 8, FAKE, None) == B.EINVAL          # R > T
    assert v(FAKE, -1, None, 8, FAKE, None) == B.EINVAL         # device count requested, no pointer
    assert v(FAKE, 4, None, 8, None, None) == B.EINVAL          # no status words
    assert v(FAKE, 4, None, 8, ODD, None) == B.EINVAL
    assert v(None, 4, None, 8, FAKE, None) == B.EINVAL
    assert v(ODD, 4, None, 8, FAKE, None) == B.EINVAL


def test_backward_rejects_bad_arguments_on_the_host():
    assert bwd(T=-1) == B.EINVAL
    assert bwd(R=9) == B.EINVAL
    assert bwd(C=60) == B.ESHAPE
    assert bwd(go=None) == B.EINVAL
    assert bwd(gh=FAKE + 32) == B.EINVAL
    assert bwd(saved=None) == B.EINVAL
    assert bwd(dwg=None) == B.EINVAL
    assert bwd(dwd=ODD) == B.EINVAL
    assert bwd(flags=0x20) == B.EUNSUPPORTED
    # the index check is a known flag: with nothing retained it has nothing to look at
    assert bwd(flags=B.FLAG_VALIDATE_IDX, ws_bytes=0) == B.EWORKSPACE
    assert bwd(ws_bytes=0) == B.EWORKSPACE
    assert bwd(dgain=ODD) == B.EINVAL


def test_compact_and_gather_reject_bad_arguments_on_the_host():
    lib = B.lib()
    assert lib.skipffn_compact(FAKE, -1, FAKE, FAKE, None, FAKE, 1 << 20, None) == B.EINVAL
    assert lib.skipffn_compact(FAKE, 10, FAKE, None, None, FAKE, 1 << 20, None) == B.EINVAL
    assert lib.skipffn_compact(ODD, 10, FAKE, FAKE, None, FAKE, 1 << 20, None) == B.EINVAL
    assert lib.skipffn_compact(FAKE, 10, FAKE, FAKE, None, FAKE, 0, None) == B.EWORKSPACE
    assert lib.skipffn_gather_rows(FAKE, FAKE, 10, 24, FAKE, 3, None, None) == B.ESHAPE
    assert lib.skipffn_gather_rows(FAKE, FAKE, 10, 32, FAKE, 11, None, None) == B.EINVAL
    assert lib.skipffn_gather_rows(None, FAKE, 10, 32, FAKE, 3, None, None) == B.EINVAL
    assert lib.skipffn_gather_rows(FAKE, FAKE, 10, 32, FAKE, 0, None, None) == B.OK
    # whole-cache form: src, dst, n_slabs, T, row_bytes, slab strides, idx, R, num_retained, stream;
    # only calls that are rejected (or are no-ops) before anything is enqueued
    kv = lib.skipffn_kv_compact
    FAR = ctypes.c_void_p(0x7000_0000_0000)
    assert kv(FAKE, FAR, 4, 10, 24, 240, 240, FAKE, 3, None, None) == B.ESHAPE      # row not 16-byte
    assert kv(FAKE, FAR, 4, 10, 32, 328, 320, FAKE, 3, None, None) == B.ESHAPE      # stride not 16-byte
    assert kv(FAKE, FAR, 4, 10, 32, 160, 320, FAKE, 3, None, None) == B.EINVAL      # source slab shorter than T rows
    assert kv(FAKE, FAR, 4, 10, 32, 320, 64, FAKE, 3, None, None) == B.EINVAL       # destination slab shorter than R rows
    assert kv(FAKE, FAR, 4, 10, 32, 320, 320, FAKE, 11, None, None) == B.EINVAL     # R > T
    assert kv(FAKE, FAR, 4, 10, 32, 320, 320, None, 3, None, None) == B.EINVAL      # no index list
    assert kv(FAKE, FAKE, 4, 10, 32, 320, 320, FAKE, 3, None, None) == B.EINVAL     # in place
    assert kv(FAKE, FAR, 4, 10, 32, 320, 320, FAKE, -1, None, None) == B.EINVAL     # device count missing
    assert kv(FAKE, FAR, 0, 10, 32, 320, 320, FAKE, 3, None, None) == B.OK          # empty cache
    assert kv(FAKE, FAR, 4, 10, 32, 320, 320, FAKE, 0, None, None) == B.OK          # nothing retained


def test_summary_layer_rejects_bad_arguments_on_the_host():
    lib = B.lib()
    f, b = lib.skipffn_summary_forward, lib.skipffn_summary_backward
    BIG = 1 << 40
    # T, C, hidden, tok, seg, n_tok, S, w, out, saved, workspace, workspace_bytes, stream
    assert f(10, 60, FAKE, FAKE, FAKE, 5, 1, FAKE, FAKE, None, FAKE, BIG, None) == B.ESHAPE
    assert f(10, 64, FAKE, FAKE, FAKE, -1, 1, FAKE, FAKE, None, FAKE, BIG, None) == B.EINVAL
    assert f(10, 64, FAKE, FAKE, None, 5, 1, FAKE, FAKE, None, FAKE, BIG, None) == B.EINVAL
    assert f(10, 64, FAKE, None, FAKE, 5, 1, FAKE, FAKE, None, FAKE, BIG, None) == B.EINVAL
    assert f(10, 64, FAKE, FAKE, FAKE, 5, 1, ODD, FAKE, None, FAKE, BIG, None) == B.EINVAL
    assert f(10, 64, FAKE, FAKE, FAKE, 5, 1, FAKE, FAKE, None, FAKE, 16, None) == B.EWORKSPACE
    assert f(10, 64, FAKE, FAKE, FAKE, 5, 0, FAKE, FAKE, None, FAKE, BIG, None) == B.OK      # no sets
    assert lib.skipffn_summary_workspace_bytes(1000, 4, 4096) >= (1000 // 16 + 4) * 4096 * 4
    assert lib.skipffn_summary_saved_bytes(1000, 4, 4096) >= 1000 * 4 + 4 * 4 + 4 * 4096 * 4
    # ..., w, saved, grad_out, grad_hidden, dw, workspace, workspace_bytes, flags, stream
    assert b(10, 64, FAKE, FAKE, FAKE, 5, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, 0x1, None) == B.EUNSUPPORTED
    assert b(10, 64, FAKE, FAKE, FAKE, 5, 1, FAKE, FAKE, FAKE, FAKE, None, FAKE, BIG, 0, None) == B.EINVAL
    assert b(10, 64, FAKE, FAKE, FAKE, 5, 1, FAKE, None, FAKE, FAKE, FAKE, FAKE, BIG, 0, None) == B.EINVAL
    assert b(10, 64, FAKE, FAKE, FAKE, 5, 1, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 16, 0, None) == B.EWORKSPACE


def test_select_retained_rejects_bad_arguments_on_the_host():
    f = B.lib().skipffn_select_retained
    # features, cls, seq_off, n_feat, B, Cv, n_keep, n_keep_dev, mask, sim, token_pos, skip_mask, T, stream
    assert f(FAKE, FAKE, FAKE, 10, 1, 60, 3, None, FAKE, FAKE, None, None, 0, None) == B.ESHAPE
    assert f(FAKE, FAKE, FAKE, -1, 1, 64, 3, None, FAKE, FAKE, None, None, 0, None) == B.EINVAL
    assert f(FAKE, FAKE, None, 10, 1, 64, 3, None, FAKE, FAKE, None, None, 0, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, 10, 1, 64, 3, None, None, FAKE, None, None, 0, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, 10, 1, 64, 3, None, FAKE, None, None, None, 0, None) == B.EINVAL
    assert f(ODD, FAKE, FAKE, 10, 1, 64, 3, None, FAKE, FAKE, None, None, 0, None) == B.EINVAL
    assert f(FAKE, FAKE, FAKE, 10, 1, 64, 3, None, FAKE, FAKE, FAKE, None, 5, None) == B.EINVAL   # half a pair
    assert f(FAKE, FAKE, FAKE, 10, 0, 64, 3, None, FAKE, FAKE, None, None, 0, None) == B.OK       # no sequences


def test_token_merge_rejects_bad_arguments_on_the_host():
    lib = B.lib()
    f = lib.skipffn_token_merge
    seg = (ctypes.c_int32 * 3)(0, 10, 30)
    bad = (ctypes.c_int32 * 3)(0, 10, 5)
    big = (ctypes.c_int32 * 2)(0, 5000)
    BIG = 1 << 40
    # x, seg_host, S, C, k, out, kept_idx, assign, avg_sim, workspace, workspace_bytes, stream
    assert f(FAKE, seg, 2, 60, 4, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.ESHAPE
    assert f(FAKE, bad, 2, 64, 4, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.EINVAL      # not ascending
    assert f(FAKE, big, 1, 64, 4, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.ESHAPE      # set too large
    assert f(FAKE, seg, 2, 64, -1, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.EINVAL
    assert f(FAKE, None, 2, 64, 4, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.EINVAL
    assert f(FAKE, seg, 2, 64, 4, None, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.EINVAL
    assert f(FAKE, seg, 2, 64, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 64, None) == B.EWORKSPACE
    assert f(FAKE, seg, 0, 64, 4, FAKE, FAKE, FAKE, FAKE, FAKE, BIG, None) == B.OK           # no sets
    assert lib.skipffn_token_merge_workspace_bytes(2048, 1024, 4096) >= 2048 * 4096 * 2 + 1024 * 1024 * 4


def test_token_merge_backward_rejects_bad_arguments_on_the_host():
    f = B.lib().skipffn_token_merge_backward
    seg = (ctypes.c_int32 * 3)(0, 10, 30)
    bad = (ctypes.c_int32 * 3)(0, 10, 5)
    big = (ctypes.c_int32 * 2)(0, 5000)
    empty = (ctypes.c_int32 * 3)(4, 4, 4)
    # grad_out, seg_host, S, C, k, assign, grad_x, stream
    assert f(FAKE, seg, 2, 60, 4, FAKE, FAKE, None) == B.ESHAPE
    assert f(FAKE, bad, 2, 64, 4, FAKE, FAKE, None) == B.EINVAL
    assert f(FAKE, big, 1, 64, 4, FAKE, FAKE, None) == B.ESHAPE
    assert f(FAKE, seg, 2, 64, -1, FAKE, FAKE, None) == B.EINVAL
    assert f(FAKE, None, 2, 64, 4, FAKE, FAKE, None) == B.EINVAL
    assert f(FAKE, seg, 2, 64, 4, None, FAKE, None) == B.EINVAL
    assert f(FAKE, seg, 2, 64, 4, FAKE, None, None) == B.EINVAL
    assert f(None, seg, 2, 64, 4, FAKE, FAKE, None) == B.EINVAL
    assert f(None, seg, 0, 64, 4, None, None, None) == B.OK           # no sets
    assert f(None, empty, 2, 64, 4, None, None, None) == B.OK         # only empty sets


def test_header_is_plain_c_and_links_against_the_library(tmp_path):
    """include/skipffn.h compiles as C99 with warnings as errors, and a C object that takes the
    address of every declared function links against libskipffn.so (no GPU call is made)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    src = os.path.join(ROOT, "tests", "cpp", "header_is_c.c")
    obj = str(tmp_path / "h.o")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-c", src, "-o", obj],
                   check=True)
    so = str(tmp_path / "h.so")
    subprocess.run(["gcc", "-shared", "-o", so, obj, B.LIB_PATH, "-Wl,--no-undefined",
                    "-Wl,-rpath," + os.path.dirname(B.LIB_PATH)], check=True)


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        B.lib()


def test_buffer_sizes_grow_with_the_row_bound():
    """A buffer sized for R_max rows is accepted for every smaller row count: the size queries
    never decrease as R_max grows (the tile variant and the K split change with the row count)."""
    lib = B.lib()
    C, I = 4096, 14336
    prev = (0, 0, 0, 0)
    for R in list(range(0, 600)) + [1000, 1472, 4096, 16384]:
        cur = (lib.skipffn_forward_workspace_bytes(R, C, I, 0), lib.skipffn_forward_workspace_bytes(R, C, I, 1),
               lib.skipffn_backward_workspace_bytes(R, C, I), lib.skipffn_saved_bytes(R, C, I))
        assert all(c >= p for c, p in zip(cur, prev)), (R, cur, prev)
        prev = cur
