"""ctypes binding of libskipffn.so - argument marshalling only.

Every function here has the name of the C entry point it calls
(include/skipffn.h) and does no arithmetic: PyTorch tensors provide device
memory and the current HIP stream, nothing else.  A missing library or a
non-zero status raises; there is no fallback path.
"""

from __future__ import annotations

import ctypes
import os
from ctypes import (POINTER, c_char_p, c_double, c_float, c_int, c_int32, c_int64,
                    c_size_t, c_uint32, c_void_p)

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libskipffn.so")

FLAG_DW_FP32 = 0x1
FLAG_DW_ACCUMULATE = 0x2
FLAG_NO_RESIDUAL = 0x4
FLAG_BALANCED_SPLIT = 0x8
FLAG_VALIDATE_IDX = 0x10

OK, EINVAL, ESHAPE, EWORKSPACE, EHIP, EUNSUPPORTED, EIDX = range(7)

# every symbol include/skipffn.h declares: (restype, argtypes)
_SIGNATURES = {
    "skipffn_compact_workspace_bytes": (c_size_t, [c_int64]),
    "skipffn_compact": (c_int, [c_void_p, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                c_size_t, c_void_p]),
    "skipffn_compact_static_max_tokens": (c_int64, []),
    "skipffn_compact_static": (c_int, [c_void_p, c_int64, c_void_p, c_void_p, c_void_p, c_void_p]),
    "skipffn_validate_idx": (c_int, [c_void_p, c_int64, c_void_p, c_int64, c_void_p, c_void_p]),
    "skipffn_saved_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "skipffn_forward_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int64, c_int]),
    "skipffn_forward": (c_int, [c_int64, c_int64, c_int64, c_float, c_void_p, c_void_p,
                                c_void_p, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                c_void_p, c_void_p, c_void_p, c_size_t, c_uint32, c_void_p]),
    "skipffn_backward_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "skipffn_backward": (c_int, [c_int64, c_int64, c_int64, c_float, c_void_p, c_void_p,
                                 c_void_p, c_int64, c_void_p, c_void_p, c_void_p, c_void_p,
                                 c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                 c_size_t, c_uint32, c_void_p]),
    "skipffn_gather_rows": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_void_p, c_int64,
                                    c_void_p, c_void_p]),
    "skipffn_kv_compact": (c_int, [c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int64, c_int64,
                                   c_void_p, c_int64, c_void_p, c_void_p]),
    "skipffn_summary_saved_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "skipffn_summary_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "skipffn_summary_forward": (c_int, [c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_int64, c_int64,
                                        c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "skipffn_summary_backward": (c_int, [c_int64, c_int64, c_void_p, c_void_p, c_void_p, c_int64, c_int64,
                                         c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p,
                                         c_size_t, c_uint32, c_void_p]),
    "skipffn_select_retained": (c_int, [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_int64,
                                        c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int64, c_void_p]),
    "skipffn_token_merge_workspace_bytes": (c_size_t, [c_int64, c_int64, c_int64]),
    "skipffn_token_merge": (c_int, [c_void_p, POINTER(c_int32), c_int64, c_int64, c_int64, c_void_p, c_void_p,
                                    c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]),
    "skipffn_token_merge_backward": (c_int, [c_void_p, POINTER(c_int32), c_int64, c_int64, c_int64, c_void_p,
                                             c_void_p, c_void_p]),
    "skipffn_probe_mfma": (c_int, [c_int64, c_int64, c_int, c_void_p, c_void_p, c_void_p]),
    "skipffn_saved_layout": (c_int, [c_int64, c_int64, c_int64, POINTER(c_size_t)]),
    "skipffn_status_string": (c_char_p, [c_int]),
    "skipffn_last_hip_error": (c_int, []),
    "skipffn_version": (c_int, []),
    "skipffn_profile_begin": (c_int, []),
    "skipffn_profile_end": (c_int, [POINTER(c_char_p), POINTER(c_double), POINTER(c_int64), c_int]),
}

_lib = None


class SkipFFNError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().skipffn_status_string(status).decode()
        if status == EHIP:
            msg += f" (hipError {lib().skipffn_last_hip_error()})"
        super().__init__(f"{where}: status {status}: {msg}")


def lib() -> ctypes.CDLL:
    """Load the C-ABI library (built by paper_2503_21817_amd.build)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2503_21817_amd.build` "
                "(there is no CPU or PyTorch fallback for the Skip-FFN path)")
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype = res
            fn.argtypes = args
        _lib = l
    return _lib


def exported_symbols():
    return sorted(_SIGNATURES)


def _check(status: int, where: str):
    if status != OK:
        raise SkipFFNError(status, where)


def _ptr(t):
    return None if t is None else c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _rargs(R, num_retained):
    """(R, num_retained pointer): R is a host int, or None to use the device count."""
    if R is None:
        if num_retained is None:
            raise ValueError("pass R or num_retained")
        return -1, _ptr(num_retained)
    return int(R), _ptr(num_retained)


# --------------------------------------------------------------------------------------
def skipffn_compact_workspace_bytes(T: int) -> int:
    return lib().skipffn_compact_workspace_bytes(T)


def skipffn_compact(skip_mask, idx, num_retained, pos=None, workspace=None):
    """skip_mask u8 [T] -> idx i32 [T] (first R entries), num_retained i32 [1], pos i32 [T]."""
    T = skip_mask.numel()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().skipffn_compact(_ptr(skip_mask), T, _ptr(idx), _ptr(num_retained), _ptr(pos),
                                 _ptr(workspace), ws_bytes, _stream()), "skipffn_compact")


def skipffn_compact_static_max_tokens() -> int:
    return lib().skipffn_compact_static_max_tokens()


def skipffn_compact_static(skip_mask, idx, num_retained, pos=None):
    """skipffn_compact without a workspace: the library's own per-GPU scratch is used."""
    T = skip_mask.numel()
    _check(lib().skipffn_compact_static(_ptr(skip_mask), T, _ptr(idx), _ptr(num_retained), _ptr(pos), _stream()),
           "skipffn_compact_static")


def skipffn_validate_idx(idx, R, T, status, *, num_retained=None):
    """status i32 [2] on the device: {0 ok / 1 bad, first offending position}; asynchronous."""
    Rv, nr = _rargs(R, num_retained)
    _check(lib().skipffn_validate_idx(_ptr(idx), Rv, nr, T, _ptr(status), _stream()), "skipffn_validate_idx")


def skipffn_saved_bytes(R_max, C, I) -> int:
    return lib().skipffn_saved_bytes(R_max, C, I)


def skipffn_forward_workspace_bytes(R_max, C, I, has_saved) -> int:
    return lib().skipffn_forward_workspace_bytes(R_max, C, I, int(bool(has_saved)))


def skipffn_backward_workspace_bytes(R_max, C, I) -> int:
    return lib().skipffn_backward_workspace_bytes(R_max, C, I)


def skipffn_saved_layout(R_max, C, I):
    arr = (c_size_t * 8)()
    _check(lib().skipffn_saved_layout(R_max, C, I, arr), "skipffn_saved_layout")
    return list(arr)


def skipffn_forward(hidden, out, idx, R, w_gate, w_up, w_down, *, eps=1e-5, rms_gain=None,
                    num_retained=None, saved=None, workspace=None, flags=0):
    T, C = hidden.shape
    I = w_gate.shape[0]
    Rv, nr = _rargs(R, num_retained)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().skipffn_forward(T, C, I, eps, _ptr(hidden), _ptr(out), _ptr(idx), Rv, nr,
                                 _ptr(rms_gain), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                 _ptr(saved), _ptr(workspace), ws_bytes, flags, _stream()),
           "skipffn_forward")


def skipffn_backward(grad_out, grad_hidden, idx, R, w_gate, w_up, w_down, saved, dw_gate, dw_up,
                     dw_down, *, eps=1e-5, rms_gain=None, num_retained=None, workspace=None,
                     flags=0, d_rms_gain=None):
    T, C = grad_out.shape
    I = w_gate.shape[0]
    Rv, nr = _rargs(R, num_retained)
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    _check(lib().skipffn_backward(T, C, I, eps, _ptr(grad_out), _ptr(grad_hidden), _ptr(idx), Rv,
                                  nr, _ptr(rms_gain), _ptr(w_gate), _ptr(w_up), _ptr(w_down),
                                  _ptr(saved), _ptr(dw_gate), _ptr(dw_up), _ptr(dw_down),
                                  _ptr(d_rms_gain), _ptr(workspace), ws_bytes, flags, _stream()),
           "skipffn_backward")


def skipffn_gather_rows(src, dst, idx, R, *, num_retained=None):
    T = src.shape[0]
    row_bytes = (src.numel() // max(T, 1)) * src.element_size()
    Rv, nr = _rargs(R, num_retained)
    _check(lib().skipffn_gather_rows(_ptr(src), _ptr(dst), T, row_bytes, _ptr(idx), Rv, nr,
                                     _stream()), "skipffn_gather_rows")


def skipffn_kv_compact(src, dst, idx, R, *, num_retained=None):
    """src [..., T, D] -> dst [..., R_cap, D] (same leading dims, any R_cap >= R): every
    leading index is one slab.  Both tensors are contiguous."""
    T, D = src.shape[-2], src.shape[-1]
    n_slabs = src.numel() // max(T * D, 1)
    row_bytes = D * src.element_size()
    Rv, nr = _rargs(R, num_retained)
    _check(lib().skipffn_kv_compact(_ptr(src), _ptr(dst), n_slabs, T, row_bytes, T * row_bytes,
                                    dst.shape[-2] * row_bytes, _ptr(idx), Rv, nr, _stream()),
           "skipffn_kv_compact")


def skipffn_summary_saved_bytes(n_tok, S, C) -> int:
    return lib().skipffn_summary_saved_bytes(n_tok, S, C)


def skipffn_summary_workspace_bytes(n_tok, S, C) -> int:
    return lib().skipffn_summary_workspace_bytes(n_tok, S, C)


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def skipffn_summary_forward(hidden, tok, seg, w, out, *, saved=None, workspace=None):
    """hidden bf16 [T, C]; tok i32 [n_tok]; seg i32 [S + 1]; w bf16 [C]; out bf16 [S, C]."""
    T, C = hidden.shape
    _check(lib().skipffn_summary_forward(T, C, _ptr(hidden), _ptr(tok), _ptr(seg), tok.numel(),
                                         seg.numel() - 1, _ptr(w), _ptr(out), _ptr(saved),
                                         _ptr(workspace), _nbytes(workspace), _stream()),
           "skipffn_summary_forward")


def skipffn_summary_backward(hidden, tok, seg, w, saved, grad_out, grad_hidden, dw, *, workspace=None,
                             flags=0):
    T, C = hidden.shape
    _check(lib().skipffn_summary_backward(T, C, _ptr(hidden), _ptr(tok), _ptr(seg), tok.numel(),
                                          seg.numel() - 1, _ptr(w), _ptr(saved), _ptr(grad_out),
                                          _ptr(grad_hidden), _ptr(dw), _ptr(workspace),
                                          _nbytes(workspace), flags, _stream()),
           "skipffn_summary_backward")


def skipffn_select_retained(features, cls, seq_off, n_keep, mask, sim, *, token_pos=None, skip_mask=None):
    """features bf16 [n_feat, Cv]; cls bf16 [B, Cv]; seq_off i32 [B + 1]; n_keep: int, or an
    i32 [B] device tensor; mask u8 [n_feat]; sim f32 [n_feat]."""
    n_feat, Cv = features.shape
    nb = seq_off.numel() - 1
    if isinstance(n_keep, torch.Tensor):
        nk, nkd = 0, _ptr(n_keep)
    else:
        nk, nkd = int(n_keep), None
    T = 0 if skip_mask is None else skip_mask.numel()
    _check(lib().skipffn_select_retained(_ptr(features), _ptr(cls), _ptr(seq_off), n_feat, nb, Cv, nk, nkd,
                                         _ptr(mask), _ptr(sim), _ptr(token_pos), _ptr(skip_mask), T,
                                         _stream()), "skipffn_select_retained")


def skipffn_token_merge_workspace_bytes(n_tok, n_max, C) -> int:
    return lib().skipffn_token_merge_workspace_bytes(n_tok, n_max, C)


def skipffn_token_merge(x, seg, k, out, kept_idx, assign, avg_sim, *, workspace=None):
    """x bf16 [n_tok, C]; seg: host sequence of S + 1 offsets; out bf16 [S, k, C];
    kept_idx i32 [S, k]; assign i32 [n_tok]; avg_sim f32 [n_tok]."""
    seg = [int(v) for v in seg]
    arr = (c_int32 * len(seg))(*seg)
    _check(lib().skipffn_token_merge(_ptr(x), arr, len(seg) - 1, x.shape[1], int(k), _ptr(out),
                                     _ptr(kept_idx), _ptr(assign), _ptr(avg_sim), _ptr(workspace),
                                     _nbytes(workspace), _stream()), "skipffn_token_merge")


def skipffn_token_merge_backward(grad_out, seg, assign, grad_x):
    """grad_out bf16 [S, k, C]; seg: host sequence of S + 1 offsets; assign i32 [n_tok] from the
    forward call; grad_x bf16 [n_tok, C]."""
    seg = [int(v) for v in seg]
    arr = (c_int32 * len(seg))(*seg)
    _check(lib().skipffn_token_merge_backward(_ptr(grad_out), arr, len(seg) - 1, grad_out.shape[2],
                                              grad_out.shape[1], _ptr(assign), _ptr(grad_x), _stream()),
           "skipffn_token_merge_backward")


def skipffn_probe_mfma(blocks, iters, random_operands, out, clocks):
    """out f32 [blocks * 256]; clocks i64 [2 * blocks] (shader cycles, 100 MHz ticks per workgroup)."""
    _check(lib().skipffn_probe_mfma(blocks, iters, int(bool(random_operands)), _ptr(out), _ptr(clocks),
                                    _stream()), "skipffn_probe_mfma")


def skipffn_version() -> int:
    return lib().skipffn_version()


def skipffn_profile_begin():
    _check(lib().skipffn_profile_begin(), "skipffn_profile_begin")


def skipffn_profile_end():
    """-> {kernel class: (total ms, launches)} for classes that ran."""
    cap = 32
    names = (c_char_p * cap)()
    ms = (c_double * cap)()
    cnt = (c_int64 * cap)()
    n = lib().skipffn_profile_end(names, ms, cnt, cap)
    return {names[i].decode(): (ms[i], cnt[i]) for i in range(min(n, cap)) if cnt[i] > 0}


# --------------------------------------------------------------------------------------
class SkipFFNBuffers:
    """Device buffers for one (T, R_max, C, I) problem: index list, saved
    activations and workspaces, allocated once through PyTorch."""

    def __init__(self, T, R_max, C, I, device="cuda", training=True):
        self.T, self.R_max, self.C, self.I = T, R_max, C, I
        u8 = dict(dtype=torch.uint8, device=device)
        self.idx = torch.empty(max(T, 1), dtype=torch.int32, device=device)
        self.num_retained = torch.zeros(1, dtype=torch.int32, device=device)
        self.compact_ws = torch.empty(max(skipffn_compact_workspace_bytes(T), 16), **u8)
        self.saved = torch.empty(skipffn_saved_bytes(R_max, C, I), **u8) if training else None
        self.fwd_ws = torch.empty(skipffn_forward_workspace_bytes(R_max, C, I, training), **u8)
        self.bwd_ws = torch.empty(skipffn_backward_workspace_bytes(R_max, C, I), **u8) \
            if training else None

    def saved_views(self, R):
        """bf16 / f32 tensor views of the saved sections, for stage-wise checks."""
        off = skipffn_saved_layout(self.R_max, self.C, self.I)
        C, I = self.C, self.I
        s = self.saved

        def sect(o, nbytes, dtype, shape):
            return s[o:o + nbytes].view(dtype).view(shape)
        return {
            "xrows": sect(off[0], R * C * 2, torch.bfloat16, (R, C)),
            "xn": sect(off[1], R * C * 2, torch.bfloat16, (R, C)),
            "rstd": sect(off[2], R * 4, torch.float32, (R,)),
            "G": sect(off[3], R * I * 2, torch.bfloat16, (R, I)),
            "U": sect(off[4], R * I * 2, torch.bfloat16, (R, I)),
            "H": sect(off[5], R * I * 2, torch.bfloat16, (R, I)),
            "xnT": sect(off[6], C * ((self.R_max + 63) // 64 * 64) * 2, torch.bfloat16,
                        (C, (self.R_max + 63) // 64 * 64)),
            "HT": sect(off[7], I * ((self.R_max + 63) // 64 * 64) * 2, torch.bfloat16,
                       (I, (self.R_max + 63) // 64 * 64)),
        }
