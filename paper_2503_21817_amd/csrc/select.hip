// Retained-token selection for a backbone without global / local views (Section 4.1): per
// sequence, the n visual tokens whose features are most similar (cosine) to the CLS token
// are retained (mask 0), the rest are skipped (mask 1).  Two kernels: similarities (memory-
// bound, features read once), then a rank count per sequence (a token is retained iff fewer
// than n tokens beat it; equal similarities: the lower index wins; a NaN similarity loses to
// every number), which needs no sort and gives the unique answer for the similarities computed.
#include "kernels.hpp"
#include "segments.hpp"

namespace skipffn {

constexpr int SEL_THREADS = 256;
constexpr int SEL_LDS_SIMS = 16384;      // similarities of one sequence kept in LDS (64 KB)

// ---- cosine similarity to the sequence's CLS row, four tokens per wavefront ----------------
__global__ __launch_bounds__(SEL_THREADS) void cls_sim_kernel(
    const bf16_t* __restrict__ feat, const bf16_t* __restrict__ cls, const int32_t* __restrict__ seq_off,
    int B, int n_feat, int Cv, float* __restrict__ sim) {
    __shared__ float red[4];
    int b, t0, nt;
    if (!locate_chunk<SEL_CH>(seq_off, B, n_feat, (int)blockIdx.x, b, t0, nt)) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int chunks = Cv >> 3;
    const u32x4* pc = reinterpret_cast<const u32x4*>(cls + (int64_t)b * Cv);
    // |cls|^2 by the whole workgroup
    float cc = 0.0f;
    for (int c = tid; c < chunks; c += SEL_THREADS) {
        float y[8];
        unpack8s(pc[c], y);
#pragma unroll
        for (int j = 0; j < 8; ++j) cc += y[j] * y[j];
    }
    const float cls_sq = block_sum256(cc, red);
    // tokens 4 wv .. 4 wv + 3 of the chunk: dot and squared norm, rows loaded together
    const u32x4* rows[4];
    bool ok[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const int i = wv * 4 + k;
        ok[k] = i < nt;
        rows[k] = reinterpret_cast<const u32x4*>(feat + (int64_t)(t0 + (ok[k] ? i : 0)) * Cv);
    }
    float dot[4] = {0.f, 0.f, 0.f, 0.f}, sq[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c = lane; c < chunks; c += 64) {
        u32x4 xr[4];
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (ok[k]) xr[k] = rows[k][c];
        float y[8];
        unpack8s(pc[c], y);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (ok[k]) {
                float x[8];
                unpack8s(xr[k], x);
#pragma unroll
                for (int j = 0; j < 8; ++j) {
                    dot[k] += x[j] * y[j];
                    sq[k] += x[j] * x[j];
                }
            }
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const float d = wave_sum(dot[k]), q = wave_sum(sq[k]);
        if (lane == 0 && ok[k]) {
            const float den = sqrtf(q) * sqrtf(cls_sq);
            sim[t0 + wv * 4 + k] = den > 0.0f ? d / den : 0.0f;
        }
    }
}

// ---- rank count and mask: a workgroup takes SEL_RANK_CH tokens of one sequence ----------------
// Every workgroup stages the similarities of the whole sequence in LDS (up to SEL_LDS_SIMS;
// longer sequences are read from global memory) and counts, for each of its tokens, how many
// tokens beat it.
constexpr int SEL_RANK_CH = SEL_THREADS;
__global__ __launch_bounds__(SEL_THREADS) void select_topn_kernel(
    const float* __restrict__ sim, const int32_t* __restrict__ seq_off, int B, int n_feat, int n_keep,
    const int32_t* __restrict__ n_keep_dev, uint8_t* __restrict__ mask,
    const int32_t* __restrict__ token_pos, uint8_t* __restrict__ skip_mask, int64_t T) {
    __shared__ __align__(16) uint32_t ssim[SEL_LDS_SIMS];     // rank keys of the similarities
    int b, t0, nt;
    if (!locate_chunk<SEL_RANK_CH>(seq_off, B, n_feat, (int)blockIdx.x, b, t0, nt)) return;
    int lo, hi;
    seg_bounds(seq_off, b, n_feat, lo, hi);
    const int n = hi - lo;
    const int keep = n_keep_dev != nullptr ? n_keep_dev[b] : n_keep;
    const bool in_lds = n <= SEL_LDS_SIMS;
    if (in_lds) {
        for (int u = threadIdx.x; u < n; u += SEL_THREADS) ssim[u] = rank_key<true>(sim[lo + u]);
        __syncthreads();
    }
    const int t = (t0 - lo) + threadIdx.x;           // index inside the sequence
    if ((int)threadIdx.x >= nt) return;
    int beats = 0;
    if (in_lds) {
        beats = rank_in_lds(ssim, n, t);
    } else {
        const uint64_t mine = rank_pair(rank_key<true>(sim[lo + t]), t);
        for (int u = 0; u < n; ++u) beats += rank_pair(rank_key<true>(sim[lo + u]), u) < mine ? 1 : 0;
    }
    const uint8_t m = beats < keep ? 0 : 1;
    mask[lo + t] = m;
    if (skip_mask != nullptr && token_pos != nullptr) {
        const int pos = token_pos[lo + t];
        if ((int64_t)pos >= 0 && (int64_t)pos < T) skip_mask[pos] = m;
    }
}

hipError_t launch_select_retained(const bf16_t* feat, const bf16_t* cls, const int32_t* seq_off,
                                  int64_t n_feat, int B, int Cv, int n_keep, const int32_t* n_keep_dev,
                                  uint8_t* mask, float* sim, const int32_t* token_pos,
                                  uint8_t* skip_mask, int64_t T, hipStream_t s) {
    if (B <= 0 || n_feat <= 0) return hipSuccess;
    const unsigned nq = (unsigned)((n_feat + SEL_CH - 1) / SEL_CH + B);
    profile_mark_begin(KC_SELECT, s);
    hipLaunchKernelGGL(cls_sim_kernel, dim3(nq), dim3(SEL_THREADS), 0, s, feat, cls, seq_off, B,
                       (int)n_feat, Cv, sim);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        const unsigned nr = (unsigned)((n_feat + SEL_RANK_CH - 1) / SEL_RANK_CH + B);
        hipLaunchKernelGGL(select_topn_kernel, dim3(nr), dim3(SEL_THREADS), 0, s, sim, seq_off, B,
                           (int)n_feat, n_keep, n_keep_dev, mask, token_pos, skip_mask, T);
        e = hipGetLastError();
    }
    profile_mark_end(KC_SELECT, s);
    return e;
}

}  // namespace skipffn
