"""CPU oracle for the Skip-FFN decoder-layer block (Skip-Vision, Section 4.2) and for the
operations around it: skip KV-cache (Section 4.3), adaptive summary layer (Section 4.2),
retained-token selection and token merge (Section 4.1).

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
GPU library is checked against.  It may be imported by tests, by the smoke
check and by the benchmark's CPU-baseline leg, and by nothing else; the product
path never routes through it.  It shares no code with the HIP path.

What the block computes (Section 4.2, the two un-numbered-in-text equations for
retained and skipped tokens, here "Eq. 4" and "Eq. 5" counting displayed
equations from the start of the paper):

    retained token :  h_out = h_attn + FFN(h_attn)          (Eq. 4)
    skipped  token :  h_out = h_attn                        (Eq. 5)

The paper's backbone is LLaMA-3-8B (Section 5.4, training setup) and its cost
model counts three C x M matrices per FFN (Section 5.2, the term 3*N2*C*M; and
Table 1, 10.5*L*N*C^2 = 3*(3.5C)*C per token per layer), so FFN is the
pre-norm SwiGLU block with no biases:

    n(x)   = x * rsqrt(mean_c(x_c^2) + eps) * g             (RMSNorm)
    FFN(x) = W_down ( silu(W_gate n(x)) * (W_up n(x)) )

Readings taken where the paper is silent are listed in the design notes of the
repository; the ones that matter here: the norm is part of FFN and the residual
uses the un-normalised x; eps is added to the mean square inside the root;
weights use the [out_features, in_features] row-major layout; the skip mask is
one byte per token, non-zero = skipped; retained indices are listed in
ascending token order; skipped rows are copied bit for bit (no arithmetic);
every output is rounded once, round-to-nearest-even, from the exactly
accumulated value.

All arithmetic is float64 with no intermediate rounding.  A matrix product
(numpy matmul) is used as a step; nothing is blocked, fused or reordered.

Pins (tests/test_oracle_*.py, all run without a GPU): bf16 conversion against
torch's converter and exhaustive round trips; compaction against brute force;
retain-all against an independently written dense layer and against PyTorch CPU
float64 ops with autograd; retain-none identity; bitwise passthrough with
NaN/Inf/-0 payloads; central finite differences for every gradient; closed
forms (zero down-projection, constant rows, power-of-two scale invariance, a
hand-worked C=2, I=1 example); the per-layer skip error identity of Section 5
(Eq. 8); per-token independence; the RMSNorm-gain gradient against finite
differences and autograd.  The functions further down carry their own section
comments and pins: kv_skip_cache* (numpy.delete, row loops), summary_* (closed
forms, library softmax, fp64 autograd, finite differences), cls_similarity /
select_top_n (closed forms, plain loops, brute-force ranking), token_merge*
(library cosine matrix, the three steps as plain loops, closed forms, invariants;
the merge gradient against central differences of the whole merge, fp64 autograd
of an index_add mean and the adjoint identity).
No function here is "parity unpinned".
"""

from __future__ import annotations

import numpy as np

__all__ = [
    "kv_skip_cache", "kv_skip_cache_all",
    "summary_forward_real", "summary_backward_real", "summary_forward", "summary_backward",
    "cls_similarity", "select_top_n", "select_retained",
    "cosine_matrix", "average_similarity", "merge_decisions", "merge_rows", "token_merge_real", "token_merge",
    "merge_rows_backward", "token_merge_backward",
    "bf16_bits_to_f64",
    "f64_to_bf16_bits",
    "f64_to_f32",
    "compact",
    "rmsnorm_rows",
    "ffn_rows",
    "dense_swiglu_layer",
    "skipffn_forward_real",
    "skipffn_backward_real",
    "skipffn_forward",
    "skipffn_backward",
    "kv_skip_cache",
]


# --------------------------------------------------------------------------
# bfloat16 <-> float64.  bf16 = sign, 8 exponent bits, 7 fraction bits: the top
# half of an IEEE binary32.
# --------------------------------------------------------------------------

def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns (uint16) to float64, exactly."""
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    as32 = (b.astype(np.uint32) << np.uint32(16)).view(np.float32)
    with np.errstate(invalid="ignore"):                  # signalling NaN payloads
        return as32.astype(np.float64)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float64 to the nearest bf16 (ties to even), one rounding.

    The spacing of bf16 numbers around x = m * 2**e (0.5 <= |m| < 1) is
    2**(e-8) in the normal range and 2**-133 in the subnormal range; x is
    divided by that spacing (exact), rounded to an integer with ties to even,
    and multiplied back (exact).  Magnitudes that round to 2**128 or more
    become infinity.  NaN maps to the quiet NaN 0x7FC0 with the sign kept.
    """
    x = np.asarray(x, dtype=np.float64)
    out = np.empty(x.shape, dtype=np.uint16)
    flat_x = x.reshape(-1)
    flat_o = out.reshape(-1)

    nan = np.isnan(flat_x)
    inf = np.isinf(flat_x)
    fin = ~(nan | inf)

    xf = np.where(fin, flat_x, 0.0)
    _, e = np.frexp(xf)
    qexp = np.maximum(e.astype(np.int64) - 8, -133)
    scaled = np.ldexp(xf, (-qexp).astype(np.int32))      # exact: power of two
    r = np.ldexp(np.rint(scaled), qexp.astype(np.int32))  # rint = ties to even
    with np.errstate(over="ignore"):
        r32 = r.astype(np.float32)                        # exact or -> inf
    big = np.abs(r) >= 2.0 ** 128
    r32 = np.where(big, np.copysign(np.float32(np.inf), r).astype(np.float32), r32)
    # keep the sign of a negative zero / of values that rounded to zero
    r32 = np.copysign(r32, np.where(fin, flat_x, 1.0)).astype(np.float32)
    bits = (r32.view(np.uint32) >> np.uint32(16)).astype(np.uint16)

    sign = np.signbit(flat_x).astype(np.uint16) << np.uint16(15)
    bits = np.where(inf, sign | np.uint16(0x7F80), bits)
    bits = np.where(nan, sign | np.uint16(0x7FC0), bits)
    flat_o[:] = bits
    return out


def f64_to_f32(x: np.ndarray) -> np.ndarray:
    """Round float64 to binary32 (ties to even) - numpy's own conversion."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float64).astype(np.float32)


# --------------------------------------------------------------------------
# Step 1: which tokens go through the FFN (Section 4.1 decides the partition;
# the block only consumes it).
# --------------------------------------------------------------------------

def compact(skip: np.ndarray):
    """Indices of retained tokens in ascending order.

    skip: one byte per token, non-zero = skipped (bypasses the FFN).
    Returns (idx int32[R], R, pos int32[T]) where pos[t] is the compacted row
    of token t, or -1 for a skipped token.
    """
    skip = np.asarray(skip).reshape(-1)
    T = skip.shape[0]
    idx = np.flatnonzero(skip == 0).astype(np.int32)
    R = int(idx.shape[0])
    pos = np.full(T, -1, dtype=np.int32)
    pos[idx] = np.arange(R, dtype=np.int32)
    return idx, R, pos


# --------------------------------------------------------------------------
# The FFN of one LLaMA-style decoder layer on a stack of rows, float64.
# --------------------------------------------------------------------------

def rmsnorm_rows(x: np.ndarray, gain: np.ndarray | None, eps: float):
    """n(x) for each row.  Returns (xn, rstd)."""
    C = x.shape[1]
    ms = np.sum(x * x, axis=1) / C
    rstd = 1.0 / np.sqrt(ms + eps)
    xn = x * rstd[:, None]
    if gain is not None:
        xn = xn * gain[None, :]
    return xn, rstd


def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def ffn_rows(x, w_gate, w_up, w_down, gain, eps):
    """FFN(x) for each row of x [R, C]; weights are [out, in].

    Returns a dict with every intermediate: xn, rstd, G, U, H, Y.
    """
    xn, rstd = rmsnorm_rows(x, gain, eps)
    G = xn @ w_gate.T                       # [R, I]
    U = xn @ w_up.T                         # [R, I]
    with np.errstate(over="ignore"):
        H = G * _sigmoid(G) * U             # silu(G) * U
    Y = H @ w_down.T                        # [R, C]
    return {"xn": xn, "rstd": rstd, "G": G, "U": U, "H": H, "Y": Y}


def dense_swiglu_layer(x, w_gate, w_up, w_down, gain, eps):
    """An ordinary decoder-layer FFN half, x + FFN(x), written with no
    indexing and no call into the functions above: one row at a time, the
    textbook LLaMA MLP.  It exists so that the retain-everything case of the
    skip path has something separately written to agree with (Eq. 4 applied to
    every token)."""
    T, C = x.shape
    out = np.empty_like(x)
    for t in range(T):
        row = x[t]
        mean_sq = float(np.dot(row, row)) / C
        normed = row / np.sqrt(mean_sq + eps)
        if gain is not None:
            normed = normed * gain
        g = w_gate @ normed
        u = w_up @ normed
        act = g / (1.0 + np.exp(-g))
        out[t] = row + w_down @ (act * u)
    return out


# --------------------------------------------------------------------------
# Skip-FFN on real (float64) inputs: used by the finite-difference pins and as
# the core of the bf16-interface functions below.
# --------------------------------------------------------------------------

def skipffn_forward_real(hidden, skip, w_gate, w_up, w_down, gain=None, eps=1e-5):
    """Eq. 4 / Eq. 5 on float64 arrays, no rounding anywhere.

    Returns dict: out [T, C], idx, R, and the FFN intermediates on retained
    rows (xn, rstd, G, U, H, Y).
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    idx, R, _ = compact(skip)
    out = hidden.copy()                                  # Eq. 5 for everybody
    inter = ffn_rows(hidden[idx], w_gate, w_up, w_down, gain, eps)
    out[idx] = hidden[idx] + inter["Y"]                  # Eq. 4 for retained
    res = {"out": out, "idx": idx, "R": R}
    res.update(inter)
    return res


def skipffn_backward_real(hidden, skip, w_gate, w_up, w_down, grad_out,
                          gain=None, eps=1e-5):
    """Gradients of L = sum(out * grad_out) for the block above.

    Skipped tokens have an identity Jacobian: dX = dOut.  For retained tokens
    the chain rule is applied stage by stage in reverse order:
      dH = dY W_down ; dW_down = dY^T H
      s = sigmoid(G) ; dG = dH * U * s * (1 + G (1 - s)) ; dU = dH * G * s
      dW_gate = dG^T xn ; dW_up = dU^T xn ; dxn = dG W_gate + dU W_up
      with xh = x * rstd, dxh = dxn * g :
      dx = rstd * (dxh - xh * mean_c(dxh * xh)) ; dX = dY + dx
      dgain = sum_r dxn * xh   (n(x) = xh * g is linear in the gain; with gain=None
      this is the gradient at g = 1)
    Returns dict: dx [T, C], dw_gate [I, C], dw_up [I, C], dw_down [C, I],
    dgain [C] and the intermediates dH, dG, dU, dxn on retained rows.
    """
    hidden = np.asarray(hidden, dtype=np.float64)
    grad_out = np.asarray(grad_out, dtype=np.float64)
    idx, R, _ = compact(skip)
    C = hidden.shape[1]
    x = hidden[idx]
    f = ffn_rows(x, w_gate, w_up, w_down, gain, eps)
    dY = grad_out[idx]

    dH = dY @ w_down                                     # [R, I]
    dw_down = dY.T @ f["H"]                              # [C, I]
    s = _sigmoid(f["G"])
    dG = dH * f["U"] * s * (1.0 + f["G"] * (1.0 - s))
    dU = dH * f["G"] * s
    dw_gate = dG.T @ f["xn"]                             # [I, C]
    dw_up = dU.T @ f["xn"]                               # [I, C]
    dxn = dG @ w_gate + dU @ w_up                        # [R, C]

    xh = x * f["rstd"][:, None]
    dxh = dxn if gain is None else dxn * gain[None, :]
    proj = np.sum(dxh * xh, axis=1) / C
    dx_norm = f["rstd"][:, None] * (dxh - xh * proj[:, None])
    dgain = np.sum(dxn * xh, axis=0)                     # [C]

    dx = grad_out.copy()                                 # skipped: identity
    dx[idx] = dY + dx_norm
    return {"dx": dx, "dw_gate": dw_gate, "dw_up": dw_up, "dw_down": dw_down,
            "dgain": dgain, "dH": dH, "dG": dG, "dU": dU, "dxn": dxn, "idx": idx, "R": R}


# --------------------------------------------------------------------------
# The interface the GPU library has: bf16 bit patterns in, bf16 (or fp32 for
# weight gradients) out, each output rounded once.
# --------------------------------------------------------------------------

def _widen_opt(bits):
    return None if bits is None else bf16_bits_to_f64(bits)


def skipffn_forward(hidden_bits, skip, w_gate_bits, w_up_bits, w_down_bits,
                    gain_bits=None, eps=1e-5, no_residual=False):
    """Forward of one Skip-FFN block on bf16 data.

    hidden_bits uint16 [T, C]; skip uint8 [T]; weights uint16 [I, C], [I, C],
    [C, I]; gain uint16 [C] or None (= 1).
    Returns dict: out_bits uint16 [T, C] (skipped rows are byte copies of the
    input), idx, R, and float64 intermediates xn, rstd, G, U, H, Y for
    stage-by-stage comparison.  no_residual=True writes bf16(Y) instead of
    bf16(x + Y) on retained rows (a debugging view of the FFN update alone).
    """
    hidden_bits = np.ascontiguousarray(hidden_bits, dtype=np.uint16)
    wg, wu, wd = (bf16_bits_to_f64(w) for w in (w_gate_bits, w_up_bits, w_down_bits))
    g = _widen_opt(gain_bits)
    idx, R, _ = compact(skip)
    x = bf16_bits_to_f64(hidden_bits[idx])
    inter = ffn_rows(x, wg, wu, wd, g, eps)
    out_bits = hidden_bits.copy()
    val = inter["Y"] if no_residual else x + inter["Y"]
    out_bits[idx] = f64_to_bf16_bits(val)
    res = {"out_bits": out_bits, "idx": idx, "R": R}
    res.update(inter)
    return res


def skipffn_backward(hidden_bits, skip, w_gate_bits, w_up_bits, w_down_bits,
                     grad_out_bits, gain_bits=None, eps=1e-5):
    """Backward of one Skip-FFN block on bf16 data.

    Returns dict: dx_bits uint16 [T, C] (skipped rows are byte copies of
    grad_out), float64 dw_gate / dw_up / dw_down / dgain (round them with
    f64_to_bf16_bits or f64_to_f32 to the dtype being compared), and the
    float64 intermediates dH, dG, dU, dxn.
    """
    hidden_bits = np.ascontiguousarray(hidden_bits, dtype=np.uint16)
    grad_out_bits = np.ascontiguousarray(grad_out_bits, dtype=np.uint16)
    wg, wu, wd = (bf16_bits_to_f64(w) for w in (w_gate_bits, w_up_bits, w_down_bits))
    g = _widen_opt(gain_bits)
    idx, R, _ = compact(skip)

    # Only retained rows enter the arithmetic; widen just those.
    sub_hidden = bf16_bits_to_f64(hidden_bits[idx])
    sub_grad = bf16_bits_to_f64(grad_out_bits[idx])
    sub = skipffn_backward_real(sub_hidden, np.zeros(R, dtype=np.uint8),
                                wg, wu, wd, sub_grad, g, eps)
    dx_bits = grad_out_bits.copy()
    dx_bits[idx] = f64_to_bf16_bits(sub["dx"])
    return {"dx_bits": dx_bits, "dw_gate": sub["dw_gate"], "dw_up": sub["dw_up"],
            "dw_down": sub["dw_down"], "dgain": sub["dgain"], "dH": sub["dH"], "dG": sub["dG"],
            "dU": sub["dU"], "dxn": sub["dxn"], "idx": idx, "R": R}


# --------------------------------------------------------------------------
# Skip KV-cache (Section 4.3, the set-difference equation): after prefill the
# key/value rows of FFN-skipped tokens are removed from the cache.
# --------------------------------------------------------------------------

def kv_skip_cache(cache_bits, skip):
    """cache_bits uint16 [T, D] (one head's keys or values, any D): returns
    the rows of retained tokens, in token order - K_cache minus K_skip."""
    idx, _, _ = compact(skip)
    return np.ascontiguousarray(np.asarray(cache_bits)[idx])


def kv_skip_cache_all(cache_bits, skip):
    """cache_bits uint16 [..., T, D] (every leading index is one slab: layer, key/value,
    head ...): the same set difference applied to every slab, one after the other."""
    c = np.asarray(cache_bits)
    lead = c.shape[:-2]
    flat = c.reshape((-1,) + c.shape[-2:])
    out = [kv_skip_cache(flat[s], skip) for s in range(flat.shape[0])]
    R = out[0].shape[0] if out else int((np.asarray(skip) == 0).sum())
    return np.stack(out).reshape(lead + (R, c.shape[-1])) if out else np.zeros(lead + (R, c.shape[-1]), c.dtype)


# --------------------------------------------------------------------------
# Adaptive summary layer (Section 4.2, the summary-token equation):
#   x^s = softmax(X W^T)^T X,   X [n, C] a set of visual tokens, W [1, C],
# the softmax taken over the n tokens.  One summary row per token set.
# --------------------------------------------------------------------------

def summary_forward_real(X, w):
    """X float64 [n, C], w float64 [C] -> dict: xs [C], p [n] (softmax weights),
    s [n] (scores X w) and lse (log-sum-exp of s).  n >= 1."""
    X = np.asarray(X, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    s = X @ w                                   # [n] : X W^T
    m = np.max(s)
    e = np.exp(s - m)
    p = e / np.sum(e)                           # softmax over tokens
    xs = p @ X                                  # (softmax)^T X
    return {"xs": xs, "p": p, "s": s, "lse": m + np.log(np.sum(e))}


def summary_backward_real(X, w, g):
    """Gradients of L = sum(x^s * g): with dp = X g and ds = p * (dp - p . dp)
    (softmax Jacobian),  dX = p g^T + ds w^T,  dw = X^T ds."""
    X = np.asarray(X, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    f = summary_forward_real(X, w)
    p = f["p"]
    dp = X @ g                                  # [n]
    ds = p * (dp - np.dot(p, dp))
    dX = np.outer(p, g) + np.outer(ds, w)
    dw = X.T @ ds
    return {"dX": dX, "dw": dw, "ds": ds, "dp": dp}


def summary_forward(hidden_bits, tok, seg, w_bits):
    """bf16 interface over S token sets: set i is the rows tok[seg[i]:seg[i+1]] of
    hidden_bits [T, C].  Returns out_bits uint16 [S, C] (each summary rounded once),
    float64 xs [S, C], scores [n_tok] and lse [S]."""
    tok = np.asarray(tok, dtype=np.int64)
    seg = np.asarray(seg, dtype=np.int64)
    w = bf16_bits_to_f64(w_bits)
    S = len(seg) - 1
    C = np.asarray(hidden_bits).shape[1]
    xs = np.zeros((S, C))
    scores = np.zeros(len(tok))
    lse = np.zeros(S)
    for i in range(S):
        rows = tok[seg[i]:seg[i + 1]]
        if len(rows) == 0:          # the paper does not define an empty set: zero row, lse = -inf
            lse[i] = -np.inf
            continue
        f = summary_forward_real(bf16_bits_to_f64(np.asarray(hidden_bits)[rows]), w)
        xs[i] = f["xs"]
        scores[seg[i]:seg[i + 1]] = f["s"]
        lse[i] = f["lse"]
    return {"out_bits": f64_to_bf16_bits(xs), "xs": xs, "scores": scores, "lse": lse}


def summary_backward(hidden_bits, tok, seg, w_bits, grad_out_bits, grad_hidden_bits):
    """Backward over S disjoint token sets: returns gh_bits uint16 [T, C] =
    bf16(grad_hidden + dX) on the listed rows (other rows are byte copies) and
    float64 dw [C] summed over the sets."""
    tok = np.asarray(tok, dtype=np.int64)
    seg = np.asarray(seg, dtype=np.int64)
    w = bf16_bits_to_f64(w_bits)
    hb = np.asarray(hidden_bits)
    gh_bits = np.array(grad_hidden_bits, dtype=np.uint16, copy=True)
    dw = np.zeros(hb.shape[1])
    for i in range(len(seg) - 1):
        rows = tok[seg[i]:seg[i + 1]]
        if len(rows) == 0:
            continue
        b = summary_backward_real(bf16_bits_to_f64(hb[rows]), w, bf16_bits_to_f64(np.asarray(grad_out_bits)[i]))
        gh_bits[rows] = f64_to_bf16_bits(bf16_bits_to_f64(gh_bits[rows]) + b["dX"])
        dw += b["dw"]
    return {"gh_bits": gh_bits, "dw": dw}


# --------------------------------------------------------------------------
# Retained-token selection for a backbone without global / local views
# (Section 4.1): the n visual tokens most similar to the CLS token are
# retained, the rest are skipped.  Similarity = cosine similarity.
# --------------------------------------------------------------------------

def cls_similarity(features, cls):
    """features float64 [n, Cv], cls float64 [Cv] -> cosine similarity [n]
    (0 where a vector has zero length)."""
    F = np.asarray(features, dtype=np.float64)
    c = np.asarray(cls, dtype=np.float64)
    num = F @ c
    den = np.sqrt(np.sum(F * F, axis=1)) * np.sqrt(np.sum(c * c))
    out = np.zeros(F.shape[0])
    nz = den > 0
    out[nz] = num[nz] / den[nz]
    return out


def select_top_n(sim, n_keep):
    """sim [n] -> skip mask uint8 [n]: 0 for the n_keep tokens of highest similarity
    (equal similarities: the lower index first), 1 for the rest."""
    sim = np.asarray(sim)
    n = sim.shape[0]
    k = max(0, min(int(n_keep), n))
    order = np.argsort(-sim, kind="stable")        # descending, ties by index
    mask = np.ones(n, dtype=np.uint8)
    mask[order[:k]] = 0
    return mask


def select_retained(features_bits, cls_bits, seq_off, n_keep):
    """bf16 interface over B sequences: features uint16 [n_feat, Cv], cls uint16 [B, Cv],
    seq_off [B + 1] (rows of sequence b: seq_off[b] .. seq_off[b+1]), n_keep int or [B].
    Returns dict: mask uint8 [n_feat] (0 = retained) and sim float64 [n_feat]."""
    seq_off = np.asarray(seq_off, dtype=np.int64)
    B = len(seq_off) - 1
    nk = np.broadcast_to(np.asarray(n_keep, dtype=np.int64), (B,))
    fb = np.asarray(features_bits)
    sim = np.zeros(fb.shape[0])
    mask = np.ones(fb.shape[0], dtype=np.uint8)
    for b in range(B):
        lo, hi = seq_off[b], seq_off[b + 1]
        sim[lo:hi] = cls_similarity(bf16_bits_to_f64(fb[lo:hi]), bf16_bits_to_f64(np.asarray(cls_bits)[b]))
        mask[lo:hi] = select_top_n(sim[lo:hi], nk[b])
    return {"mask": mask, "sim": sim}


# --------------------------------------------------------------------------
# Token merge of the skipped (local) visual tokens (Section 4.1, the three
# bullet points): pairwise cosine similarities and their per-token average;
# the k tokens of lowest average similarity are kept; every other token is
# merged with the most similar kept token.  The paper does not spell out the
# merge: here (as in the token-merging work it cites) a kept token becomes the
# plain mean of itself and the tokens merged into it.
# --------------------------------------------------------------------------

def cosine_matrix(X):
    """X float64 [n, C] -> [n, n] cosine similarities (a zero row has similarity 0 to
    everything, itself included)."""
    X = np.asarray(X, dtype=np.float64)
    norm = np.sqrt(np.sum(X * X, axis=1))
    Xn = np.zeros_like(X)
    nz = norm > 0
    Xn[nz] = X[nz] / norm[nz, None]
    return Xn @ Xn.T


def average_similarity(S):
    """Mean similarity of every token to the OTHER tokens of its set (0 for a single token)."""
    S = np.asarray(S, dtype=np.float64)
    n = S.shape[0]
    if n <= 1:
        return np.zeros(n)
    return (np.sum(S, axis=1) - np.diag(S)) / (n - 1)


def merge_decisions(S, avg, k):
    """-> (kept, assign): kept = ascending indices of the min(k, n) tokens of lowest average
    similarity (equal averages: the lower index first); assign[i] = slot (position in kept)
    of the kept token that token i ends up in: its own slot if kept, else the kept token of
    highest similarity to it (equal similarities: the lower index)."""
    S = np.asarray(S)
    n = S.shape[0]
    kk = max(0, min(int(k), n))
    order = np.argsort(np.asarray(avg), kind="stable")          # ascending, ties by index
    kept = np.sort(order[:kk])
    slot_of = -np.ones(n, dtype=np.int64)
    slot_of[kept] = np.arange(kk)
    assign = slot_of.copy()
    if kk > 0:
        for i in range(n):
            if slot_of[i] < 0:
                assign[i] = int(np.argmax(S[i, kept]))          # first maximum = lowest index
    return kept, assign


def merge_rows(X, assign, kk):
    """Plain mean of the rows assigned to every slot, rows added in index order."""
    X = np.asarray(X, dtype=np.float64)
    out = np.zeros((kk, X.shape[1]))
    cnt = np.zeros(kk)
    for i in range(X.shape[0]):
        if assign[i] >= 0:
            out[assign[i]] += X[i]
            cnt[assign[i]] += 1
    return out / np.maximum(cnt, 1)[:, None]


def token_merge_real(X, k):
    X = np.asarray(X, dtype=np.float64)
    S = cosine_matrix(X)
    avg = average_similarity(S)
    kept, assign = merge_decisions(S, avg, k)
    return {"merged": merge_rows(X, assign, len(kept)), "kept": kept, "assign": assign,
            "S": S, "avg": avg}


def merge_rows_backward(dM, assign, n):
    """Gradient of merge_rows with the assignment held fixed (the choice of kept tokens and the
    arg-max assignment are piecewise constant in X, so they carry no gradient): slot j is the
    mean of its c_j member rows, hence every member row receives dM[j] / c_j."""
    dM = np.asarray(dM, dtype=np.float64)
    cnt = np.zeros(dM.shape[0])
    for i in range(n):
        if assign[i] >= 0:
            cnt[assign[i]] += 1
    dX = np.zeros((n, dM.shape[1]))
    for i in range(n):
        if assign[i] >= 0:
            dX[i] = dM[assign[i]] / cnt[assign[i]]
    return dX


def token_merge_backward(grad_out_bits, seg, k, assign):
    """bf16 interface of the merge gradient over several sets: grad_out_bits uint16 [S, k, C],
    assign int [n_tok] as returned by token_merge -> dx float64 [n_tok, C] and its bf16 bits."""
    gb = np.asarray(grad_out_bits)
    seg = np.asarray(seg, dtype=np.int64)
    n_tok = int(seg[-1]) if len(seg) else 0
    C = gb.shape[2]
    dx = np.zeros((n_tok, C))
    for s in range(len(seg) - 1):
        lo, hi = seg[s], seg[s + 1]
        if hi > lo:
            dx[lo:hi] = merge_rows_backward(bf16_bits_to_f64(gb[s]), np.asarray(assign)[lo:hi], hi - lo)
    return {"dx": dx, "dx_bits": f64_to_bf16_bits(dx)}


def token_merge(x_bits, seg, k):
    """bf16 interface over several sets (set s = rows seg[s]:seg[s+1] of x_bits [n_tok, C]):
    out_bits uint16 [S, k, C] (rows past a set's kept count are zero), kept int64 [S, k] (row
    index in x_bits, -1 padding), assign int64 [n_tok] (slot), avg float64 [n_tok]."""
    xb = np.asarray(x_bits)
    seg = np.asarray(seg, dtype=np.int64)
    S_sets = len(seg) - 1
    C = xb.shape[1]
    out = np.zeros((S_sets, k, C))
    kept = -np.ones((S_sets, k), dtype=np.int64)
    assign = -np.ones(xb.shape[0], dtype=np.int64)
    avg = np.zeros(xb.shape[0])
    for s in range(S_sets):
        lo, hi = seg[s], seg[s + 1]
        if hi <= lo:
            continue
        r = token_merge_real(bf16_bits_to_f64(xb[lo:hi]), k)
        kk = len(r["kept"])
        out[s, :kk] = r["merged"]
        kept[s, :kk] = r["kept"] + lo
        assign[lo:hi] = r["assign"]
        avg[lo:hi] = r["avg"]
    return {"out_bits": f64_to_bf16_bits(out), "merged": out, "kept": kept, "assign": assign, "avg": avg}

