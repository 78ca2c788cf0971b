/*
 * skipffn.h - C ABI of the MI355X (gfx950) Skip-FFN block.
 *
 * The block is the feed-forward half of one decoder layer under Skip-Vision
 * (Section 4.2 of the paper):
 *
 *     retained token :  h_out = h_attn + FFN(h_attn)
 *     skipped  token :  h_out = h_attn
 *
 * with FFN the pre-norm SwiGLU MLP of the paper's LLaMA-3-8B backbone
 * (Section 5.4; three C x M matrices, cf. the 3*N2*C*M term of Section 5.2 and
 * Table 1):  FFN(x) = W_down( silu(W_gate n(x)) * (W_up n(x)) ),
 * n(x) = x * rsqrt(mean(x^2) + eps) * gain.
 *
 * Conventions common to every call
 * --------------------------------
 *  - All tensor pointers are DEVICE pointers (HBM of the current HIP device)
 *    unless a parameter says "host".  Tensors are dense row-major.
 *  - bf16 tensors are passed as `const void*` / `void*` to 16-bit elements
 *    (the upper half of an IEEE binary32).  Accumulation is fp32.
 *  - T = tokens in the flattened (packed, unpadded) batch, R = retained rows,
 *    C = hidden size, I = intermediate size (the paper's M).
 *    C % 8 == 0, I % 8 == 0; every tensor pointer is 16-byte aligned.
 *  - Weights use the [out_features, in_features] layout: w_gate, w_up [I, C],
 *    w_down [C, I]  (y = x W^T).  No pre-packing.
 *  - skip_mask: one byte per token, non-zero = the token skips the FFN.
 *  - idx: ascending token indices of the retained rows (what skipffn_compact
 *    writes).  `R` is given by the host (R >= 0); or R = -1 and `num_retained`
 *    points at the device-side count written by skipffn_compact, in which case
 *    no host synchronisation happens and buffers must be sized for R = T.
 *  - Ownership: the caller owns every buffer.  The library allocates no
 *    device memory, keeps no pointer after a call returns, never synchronises
 *    the device and enqueues work only on `stream` (a hipStream_t passed as
 *    void*; NULL = the default stream).  Results are complete when the stream
 *    reaches the end of the enqueued work.
 *  - Every function returns a skipffn_status; 0 is success.  Argument errors
 *    are detected on the host before anything is enqueued.  Nothing aborts,
 *    throws or prints.
 */
#ifndef SKIPFFN_H
#define SKIPFFN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum skipffn_status {
    SKIPFFN_OK = 0,
    SKIPFFN_EINVAL = 1,       /* null / misaligned pointer, negative size, R > T */
    SKIPFFN_ESHAPE = 2,       /* C or I not a multiple of 8, or a tensor >= 2 GiB */
    SKIPFFN_EWORKSPACE = 3,   /* workspace (or saved buffer) too small */
    SKIPFFN_EHIP = 4,         /* a HIP call failed; see skipffn_last_hip_error */
    SKIPFFN_EUNSUPPORTED = 5, /* unknown flag bit */
    SKIPFFN_EIDX = 6          /* SKIPFFN_FLAG_VALIDATE_IDX: idx is not strictly ascending inside [0, T) */
} skipffn_status;

/* flags (bitwise or) */
#define SKIPFFN_FLAG_DW_FP32        0x1u  /* backward: dw_* are float32, not bf16 */
#define SKIPFFN_FLAG_DW_ACCUMULATE  0x2u  /* backward: dw_* += instead of = */
#define SKIPFFN_FLAG_NO_RESIDUAL    0x4u  /* forward: retained rows get bf16(FFN(x)), not bf16(x + FFN(x)) - a debugging view */
#define SKIPFFN_FLAG_BALANCED_SPLIT  0x8u  /* use the balanced K split of the down / dXn GEMMs whenever it applies
                                             (by default a cost model picks between it, plain split-K and no split) */
#define SKIPFFN_FLAG_VALIDATE_IDX    0x10u /* forward / backward, debugging: check idx[0..R) on the device first (strictly
                                             ascending, inside [0, T)) and return SKIPFFN_EIDX, with nothing else
                                             enqueued, when it is not.  The ONE case in which a call waits for the
                                             stream (it reads the verdict back), so not for use under graph capture.
                                             Without the flag idx is trusted: a wrong entry is an out-of-bounds write. */
#define SKIPFFN_FLAG_ALL            0x1Fu

/* ---- step 1: mask -> ascending retained indices -------------------------
 * Section 4.1 decides which visual tokens are retained; the block consumes
 * that partition.  Writes idx[0..R) = positions t with skip_mask[t] == 0 in
 * increasing t (entries beyond R are left untouched), *num_retained = R and,
 * if pos != NULL, pos[t] = compacted row of token t or -1 if skipped.
 *   skip_mask  u8  [T]  device, 16-byte aligned
 *   idx        i32 [T]  device OUT (capacity T)
 *   num_retained i32 [1] device OUT
 *   pos        i32 [T]  device OUT or NULL
 *   workspace  device scratch of at least skipffn_compact_workspace_bytes(T)
 * T == 0 is valid (writes *num_retained = 0).  Deterministic. */
size_t skipffn_compact_workspace_bytes(int64_t T);
int skipffn_compact(const uint8_t* skip_mask, int64_t T, int32_t* idx,
                    int32_t* num_retained, int32_t* pos,
                    void* workspace, size_t workspace_bytes, void* stream);

/* skipffn_compact for callers that cannot allocate device memory and so have no workspace to
 * hand over: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments, outputs and guarantees as skipffn_compact minus the workspace: the
 * few kilobytes of scratch the multi-block path needs (T above 262144) live in a 32 KB array
 * inside the library, one copy per GPU, held until the process ends.  The call allocates and
 * frees nothing.  T may be at most skipffn_compact_static_max_tokens() (2^28); a larger T returns
 * SKIPFFN_ESHAPE with nothing enqueued.  Every call on a GPU uses that GPU's one array: calls
 * that may overlap in time on the same GPU (different streams without ordering) race - give
 * those skipffn_compact with a workspace each. */
int64_t skipffn_compact_static_max_tokens(void);
int skipffn_compact_static(const uint8_t* skip_mask, int64_t T, int32_t* idx,
                           int32_t* num_retained, int32_t* pos, void* stream);

/* The same check as SKIPFFN_FLAG_VALIDATE_IDX, asynchronous (Section 4.2's retained set must be
 * a set of token positions: the block scatters through it).  Enqueues two small kernels that
 * write status[0] = 0 if idx[0..R) is strictly ascending and inside [0, T), else 1, and
 * status[1] = the first offending position (INT32_MAX if none).
 *   status  i32 [2] device OUT;  idx, R, num_retained as in the conventions.  No host wait. */
int skipffn_validate_idx(const int32_t* idx, int64_t R, const int32_t* num_retained, int64_t T,
                         int32_t* status, void* stream);

/* ---- steps 2-4: forward of the block (Section 4.2, both equations) --------
 *   hidden  bf16 [T, C]  input (h_attn)
 *   out     bf16 [T, C]  output; may be the same pointer as hidden (in place:
 *                        skipped rows are then not touched at all).  When
 *                        out != hidden, skipped rows are copied bit for bit.
 *                        Partial overlap is not allowed.
 *   idx, R, num_retained : see conventions
 *   rms_gain bf16 [C] or NULL (= all ones)
 *   w_gate, w_up bf16 [I, C]; w_down bf16 [C, I]
 *   saved   NULL, or a buffer of skipffn_saved_bytes(R_max, C, I) bytes that
 *           receives what backward needs (gathered input rows, normalised
 *           rows, 1/rms, gate, up and hidden activations, and row-contiguous copies of the
 *           normalised rows and of the hidden activations); required for
 *           training because an in-place forward overwrites its input.
 *   workspace: at least skipffn_forward_workspace_bytes(R_max, C, I, saved != NULL)
 * where R_max = R if R >= 0 else T.  The size queries never decrease as R_max grows, so
 * buffers sized once for a bound serve every call with fewer rows.
 * R == 0 or T == 0: no arithmetic (out-of-place: plain copy).
 * Results are deterministic: every reduction has a fixed order.  The GEMMs pick their tile
 * height and K split from the row bound of the call (R, or T when R = -1), C and I, so the
 * same data may round differently in the last bit under a different bound. */
size_t skipffn_saved_bytes(int64_t R_max, int64_t C, int64_t I);
size_t skipffn_forward_workspace_bytes(int64_t R_max, int64_t C, int64_t I, int has_saved);
int skipffn_forward(int64_t T, int64_t C, int64_t I, float eps,
                    const void* hidden, void* out,
                    const int32_t* idx, int64_t R, const int32_t* num_retained,
                    const void* rms_gain,
                    const void* w_gate, const void* w_up, const void* w_down,
                    void* saved, void* workspace, size_t workspace_bytes,
                    uint32_t flags, void* stream);

/* ---- step 5: backward over retained rows only -----------------------------
 * The paper applies the skip during supervised fine-tuning (Section 4.2), so
 * gradients flow through the FFN for retained tokens only; a skipped token has
 * an identity Jacobian through this block.
 *   grad_out    bf16 [T, C]  upstream gradient
 *   grad_hidden bf16 [T, C]  OUT; may alias grad_out (skipped rows untouched);
 *                            otherwise skipped rows are bit copies of grad_out
 *   saved       what the matching forward wrote (same R, C, I)
 *   dw_gate, dw_up [I, C]; dw_down [C, I]: bf16, overwritten, unless
 *       SKIPFFN_FLAG_DW_FP32 (float32) / SKIPFFN_FLAG_DW_ACCUMULATE (+=).
 *       With R == 0 they are zero-filled (or left as they are when
 *       accumulating).
 *   d_rms_gain  NULL, or float32 [C] OUT: gradient of the RMSNorm gain (of an all-ones gain
 *       when rms_gain is NULL), overwritten or += like dw_*; always float32.  It is summed
 *       over rows in a fixed order (deterministic).
 *   workspace: at least skipffn_backward_workspace_bytes(R_max, C, I) */
size_t skipffn_backward_workspace_bytes(int64_t R_max, int64_t C, int64_t I);
int skipffn_backward(int64_t T, int64_t C, int64_t I, float eps,
                     const void* grad_out, void* grad_hidden,
                     const int32_t* idx, int64_t R, const int32_t* num_retained,
                     const void* rms_gain,
                     const void* w_gate, const void* w_up, const void* w_down,
                     const void* saved,
                     void* dw_gate, void* dw_up, void* dw_down, void* d_rms_gain,
                     void* workspace, size_t workspace_bytes,
                     uint32_t flags, void* stream);

/* ---- skip KV-cache (Section 4.3, the set-difference equation) -------------
 * After prefill the key / value rows of FFN-skipped tokens are dropped:
 * dst[r, :] = src[idx[r], :] for r < R.  row_bytes % 16 == 0.
 *   src  [T, row_bytes] device;  dst [R, row_bytes] device OUT (no overlap) */
int skipffn_gather_rows(const void* src, void* dst, int64_t T, int64_t row_bytes,
                        const int32_t* idx, int64_t R, const int32_t* num_retained,
                        void* stream);

/* Whole-cache form of the same set difference: a cache holds n_slabs slabs (one per layer,
 * key/value, batch entry and head - whatever precedes the token axis in the caller's
 * layout), each [T, row_bytes]; slab s starts at src + s * src_slab_bytes.  For every slab
 *     dst[s][r, :] = src[s][idx[r], :]   for r < R,
 * slab s of dst starting at dst + s * dst_slab_bytes (dst_slab_bytes >= R_max * row_bytes,
 * so the compacted cache may keep the prefill capacity or be packed).  One launch for the
 * whole cache.  row_bytes, src_slab_bytes, dst_slab_bytes are multiples of 16; src and dst
 * must not overlap (compacting in place would race: row r is a source for an earlier
 * destination).  n_slabs == 0 or R == 0: nothing is done. */
int skipffn_kv_compact(const void* src, void* dst, int64_t n_slabs, int64_t T, int64_t row_bytes,
                       int64_t src_slab_bytes, int64_t dst_slab_bytes,
                       const int32_t* idx, int64_t R, const int32_t* num_retained, void* stream);

/* ---- adaptive summary layer (Section 4.2, the summary-token equation) ------------------
 *     x^s = softmax(X w^T)^T X
 * X [n, C] a set of visual tokens, w [1, C] the layer's weight, the softmax taken over the
 * n tokens: one summary row per token set.  A call handles S sets at once:
 *   hidden  bf16 [T, C]          token features
 *   tok     i32 [n_tok] device   token indices, the sets laid one after the other
 *   seg     i32 [S + 1] device   set s is tok[seg[s] .. seg[s+1]); sizes need not be known
 *                                on the host.  Entries of tok outside [0, T) and segment
 *                                bounds outside [0, n_tok] are ignored, never dereferenced.
 *   w       bf16 [C]
 *   out     bf16 [S, C] OUT      the summary tokens (an empty set gives a zero row)
 *   saved   NULL (inference) or skipffn_summary_saved_bytes(n_tok, S, C) bytes OUT:
 *           scores f32 [n_tok], log-sum-exp f32 [S], x^s in f32 [S, C]
 *   workspace: at least skipffn_summary_workspace_bytes(n_tok, S, C)
 * Backward, for L with dL/dx^s = grad_out bf16 [S, C]:
 *   grad_hidden bf16 [T, C] IN/OUT: row t of every listed token becomes
 *       bf16(grad_hidden[t] + p_t * grad_out[s] + ds_t * w), ds_t = p_t (grad_out[s] . X_t -
 *       grad_out[s] . x^s); rows not listed are not touched.  The sets must be disjoint.
 *   dw  f32 [C] OUT: sum_t ds_t X_t over all sets, overwritten, or += with
 *       SKIPFFN_FLAG_DW_ACCUMULATE (the only flag accepted); summed in a fixed order.
 * C % 8 == 0; pointers 16-byte aligned (tok, seg: 4-byte).  S == 0 or n_tok == 0: only the
 * zero rows / zero dw are written. */
size_t skipffn_summary_saved_bytes(int64_t n_tok, int64_t S, int64_t C);
size_t skipffn_summary_workspace_bytes(int64_t n_tok, int64_t S, int64_t C);
int skipffn_summary_forward(int64_t T, int64_t C, const void* hidden,
                            const int32_t* tok, const int32_t* seg, int64_t n_tok, int64_t S,
                            const void* w, void* out, void* saved,
                            void* workspace, size_t workspace_bytes, void* stream);
int skipffn_summary_backward(int64_t T, int64_t C, const void* hidden,
                             const int32_t* tok, const int32_t* seg, int64_t n_tok, int64_t S,
                             const void* w, const void* saved, const void* grad_out,
                             void* grad_hidden, void* dw,
                             void* workspace, size_t workspace_bytes, uint32_t flags, void* stream);

/* ---- retained-token selection (Section 4.1) --------------------------------------------
 * For a backbone without global / local views the paper retains, per sequence, the n visual
 * tokens most similar to the CLS token and skips the rest.  Similarity is the cosine of the
 * vision features; a token is retained iff fewer than n tokens of its sequence have a larger
 * similarity (equal similarities: the lower index first), so the mask is unique for the
 * float32 similarities computed, which are returned.
 *   features  bf16 [n_feat, Cv]  visual tokens of all sequences, packed
 *   cls       bf16 [B, Cv]       one CLS row per sequence
 *   seq_off   i32 [B + 1] device rows of sequence b: seq_off[b] .. seq_off[b+1]) (clamped to n_feat)
 *   n_keep / n_keep_dev          retained count n: one host value, or i32 [B] on the device
 *   mask      u8 [n_feat] OUT    0 = retained, 1 = skipped, in feature order
 *   sim       f32 [n_feat] OUT   the similarities (also the kernels' scratch: required)
 *   token_pos, skip_mask, T      optional pair: token_pos i32 [n_feat] gives each visual token's
 *       position in a flat token sequence of length T and skip_mask u8 [T] receives the same
 *       value there (other entries, e.g. text tokens, are not touched; positions outside
 *       [0, T) are ignored) - the mask skipffn_compact consumes, without a host round trip.
 * Cv % 8 == 0; features, cls 16-byte aligned. */
int skipffn_select_retained(const void* features, const void* cls, const int32_t* seq_off,
                            int64_t n_feat, int64_t B, int64_t Cv, int64_t n_keep,
                            const int32_t* n_keep_dev, uint8_t* mask, float* sim,
                            const int32_t* token_pos, uint8_t* skip_mask, int64_t T, void* stream);

/* ---- token merge (Section 4.1, the three steps) ----------------------------------------
 * Reduces each set of (local, skipped) visual tokens to k tokens: pairwise cosine
 * similarities and their average per token (over the other tokens of the set); the k tokens
 * of lowest average similarity are kept; every other token is merged into the kept token it
 * is most similar to.  A kept token becomes the plain mean of itself and the tokens merged
 * into it (the paper leaves the merge itself open).  Equal averages / similarities go to the
 * lower index; decisions are taken on the float32 values computed, which are returned.
 *   x         bf16 [n_tok, C]     tokens of all sets, set s = rows seg_host[s] .. seg_host[s+1])
 *   seg_host  i32 [S + 1] HOST    ascending, seg_host[0] >= 0; at most 4096 rows per set
 *   k                             tokens kept per set (<= 4096); a set of n <= k rows is kept whole
 *   out       bf16 [S, k, C] OUT  merged tokens in the index order of the kept tokens; rows past
 *                                 a set's kept count are zero
 *   kept_idx  i32 [S, k] OUT      row index (in x) of every kept token, -1 padding
 *   assign    i32 [n_tok] OUT     slot (0 .. k-1 within its set) each token ends up in
 *   avg_sim   f32 [n_tok] OUT     the average similarities
 *   workspace: at least skipffn_token_merge_workspace_bytes(n_tok, n_max, C), n_max = rows of
 *              the largest set
 * Sets are processed in groups of up to 64 per launch, in order on the stream. */
size_t skipffn_token_merge_workspace_bytes(int64_t n_tok, int64_t n_max, int64_t C);
int skipffn_token_merge(const void* x, const int32_t* seg_host, int64_t S, int64_t C, int64_t k,
                        void* out, int32_t* kept_idx, int32_t* assign, float* avg_sim,
                        void* workspace, size_t workspace_bytes, void* stream);

/* Gradient of the token merge with respect to x (Section 4.1; the merged tokens feed the
 * language model during training).  Which tokens are kept and where a token goes are piecewise
 * constant in x and carry no gradient; a kept slot is the mean of its m members, so every
 * member receives grad_out[slot] / m, rounded once to bf16.
 *   grad_out  bf16 [S, k, C]      gradient of `out` (rows past a set's kept count are ignored)
 *   seg_host, S, C, k             as in the forward call
 *   assign    i32 [n_tok]         the forward call's output; a value outside 0 .. min(k, n)-1
 *                                 gives a zero row
 *   grad_x    bf16 [n_tok, C] OUT every row is written
 * No workspace. */
int skipffn_token_merge_backward(const void* grad_out, const int32_t* seg_host, int64_t S, int64_t C,
                                 int64_t k, const int32_t* assign, void* grad_x, void* stream);

/* ---- layout of `saved`, for tests that compare stage by stage -------------
 * Byte offsets of the sections inside a saved buffer for (R_max, C, I):
 * offsets[0] x rows bf16 [R, C]; [1] normalised rows bf16 [R, C];
 * [2] 1/rms f32 [R]; [3] gate bf16 [R, I]; [4] up bf16 [R, I];
 * [5] silu(gate)*up bf16 [R, I]; [6] normalised rows transposed, bf16 [C, ld];
 * [7] silu(gate)*up transposed, bf16 [I, ld]; ld = R_max rounded up to a multiple of 64
 * (the weight-gradient GEMMs contract over the rows and read the copies in which the row
 * index is contiguous; columns >= R are not read).
 * `offsets` is a HOST array of 8. */
int skipffn_saved_layout(int64_t R_max, int64_t C, int64_t I, size_t* offsets);

/* ---- diagnostics ---------------------------------------------------------- */
const char* skipffn_status_string(int status);
int skipffn_last_hip_error(void);     /* hipError_t of the last SKIPFFN_EHIP on this thread */
int skipffn_version(void);            /* major * 10000 + minor * 100 + patch */

/* Measurement aid, not part of the method: a register-only loop of independent
 * v_mfma_f32_16x16x32_bf16 (no memory traffic), i.e. what the matrix cores of the chip in hand
 * sustain - the ceiling bench.py quotes next to the published peak.  `blocks` workgroups of 4
 * wavefronts issue iters * 32 MFMAs per wavefront (16384 FLOP each); operands are the constant
 * 1.0 or, with random_operands != 0, pseudo-random bf16 values (the clock a power-capped chip
 * holds depends on the data).
 *   out     f32 [blocks * 256] device OUT (keeps the arithmetic alive)
 *   clocks  i64 [2 * blocks]  device OUT: per workgroup, shader cycles and 100 MHz wall-clock
 *           ticks spent in the loop (their ratio is the shader clock) */
int skipffn_probe_mfma(int64_t blocks, int64_t iters, int random_operands, float* out, int64_t* clocks,
                       void* stream);

/* Duration in milliseconds, measured with HIP events on `stream`, of the most
 * recent launch of each hot-path kernel class since the last
 * skipffn_profile_begin.  Profiling mode records events around every kernel
 * launch (it never synchronises inside a forward/backward call);
 * skipffn_profile_end synchronises those events and fills host arrays.
 *   names: host array of `cap` const char* (kernel class names, static storage)
 *   ms, launches: host arrays of `cap`;  returns the number of classes. */
int skipffn_profile_begin(void);
int skipffn_profile_end(const char** names, double* ms, int64_t* launches, int cap);

#ifdef __cplusplus
}
#endif
#endif /* SKIPFFN_H */
