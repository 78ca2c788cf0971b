// Adaptive summary layer (Section 4.2, the summary-token equation):
//     x^s = softmax(X w^T)^T X        X = a set of visual tokens [n, C], w [C]
// one summary row per token set, forward and backward.  Memory-bound: X is read once from
// HBM per pass (a second read of the same rows inside a workgroup hits L2).
//
// A token set s is the rows tok[seg[s] .. seg[s+1]) of the hidden states; tok and seg live
// on the device, so set sizes need not be known on the host.  Every set is cut into chunks
// of SUM_CH tokens, one workgroup per chunk ("flash" style): a chunk produces its own
// maximum m, denominator d = sum exp(s_t - m) and unnormalised weighted row sum; a second
// small kernel merges the chunks of a set.  The launch covers the upper bound
// ceil(n_tok / SUM_CH) + S chunks; workgroups past the real count exit.
#include "kernels.hpp"
#include "segments.hpp"

namespace skipffn {

constexpr int SUM_THREADS = 256;
static_assert(SUM_CH == 16, "four wavefronts of four tokens");
constexpr float kNoScore = -3.0e38f;      // score of an out-of-range token index: weight 0

// dots of four rows of `hidden` (row index < 0: skipped, result 0) with the row `b`, by one
// wavefront.  Loads are issued for two column steps of all four rows before any arithmetic, so
// that ten 16-byte loads per lane are in flight (a skipped row reads row 0: always in bounds).
__device__ __forceinline__ void wave_dot4(const bf16_t* __restrict__ hidden, int C, const int* rows,
                                          const bf16_t* __restrict__ b, int chunks, int lane, float* out) {
    const u32x4* pb = reinterpret_cast<const u32x4*>(b);
    const u32x4* pr[4];
    float scale[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        pr[k] = reinterpret_cast<const u32x4*>(hidden + (int64_t)(rows[k] >= 0 ? rows[k] : 0) * C);
        scale[k] = rows[k] >= 0 ? 1.0f : 0.0f;
    }
    float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int c = lane;
    for (; c + 64 < chunks; c += 128) {
        u32x4 x0[4], x1[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) { x0[k] = pr[k][c]; x1[k] = pr[k][c + 64]; }
        const u32x4 w0 = pb[c], w1 = pb[c + 64];
        float y0[8], y1[8];
        unpack8s(w0, y0);
        unpack8s(w1, y1);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float a[8], d[8];
            unpack8s(x0[k], a);
            unpack8s(x1[k], d);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k] += a[j] * y0[j] + d[j] * y1[j];
        }
    }
    if (c < chunks) {
        u32x4 x0[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) x0[k] = pr[k][c];
        float y0[8];
        unpack8s(pb[c], y0);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float a[8];
            unpack8s(x0[k], a);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[k] += a[j] * y0[j];
        }
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) out[k] = wave_sum(acc[k]) * scale[k];
}

// ---- forward, per chunk ---------------------------------------------------------------------
__global__ __launch_bounds__(SUM_THREADS) void summary_chunk_fwd_kernel(
    const bf16_t* __restrict__ hidden, int64_t T, int C, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ seg, int S, int n_tok, const bf16_t* __restrict__ w,
    float* __restrict__ scores, float* __restrict__ part_acc, float* __restrict__ part_md) {
    __shared__ float sc[SUM_CH];
    __shared__ int rowid[SUM_CH];
    int s, t0, nt;
    if (!locate_chunk<SUM_CH>(seg, S, n_tok, (int)blockIdx.x, s, t0, nt)) return;   // uniform over the workgroup
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int chunks = C >> 3;
    // phase A: scores s_t = X_t . w, four tokens per wavefront (SUM_CH = 16 = 4 waves x 4)
    {
        int rows[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = wv * 4 + k;
            int row = -1;
            if (i < nt) {
                row = tok[t0 + i];
                if ((uint32_t)row >= (uint32_t)T) row = -1;
            }
            rows[k] = row;
        }
        float v[4];
        wave_dot4(hidden, C, rows, w, chunks, lane, v);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = wv * 4 + k;
                if (i < nt) {
                    const float sv = rows[k] >= 0 ? v[k] : kNoScore;
                    sc[i] = sv;
                    rowid[i] = rows[k];
                    if (scores != nullptr) scores[t0 + i] = sv;
                }
            }
        }
    }
    __syncthreads();
    float m = kNoScore;
    for (int i = 0; i < nt; ++i) m = fmaxf(m, sc[i]);
    float e[SUM_CH];
    float d = 0.0f;
#pragma unroll
    for (int i = 0; i < SUM_CH; ++i) {
        e[i] = (i < nt && rowid[i] >= 0) ? __expf(sc[i] - m) : 0.0f;
        d += e[i];
    }
    // phase B: every thread owns 16-byte column chunks: sum_t e_t X_t.  The sixteen row loads of
    // a chunk are unconditional (an absent token reads row 0 with weight 0) and issued together.
    const bf16_t* rp[SUM_CH];
#pragma unroll
    for (int i = 0; i < SUM_CH; ++i)
        rp[i] = hidden + (int64_t)((i < nt && rowid[i] >= 0) ? rowid[i] : 0) * C;
    float* pa = part_acc + (int64_t)blockIdx.x * C;
    for (int c = tid; c < chunks; c += SUM_THREADS) {
        u32x4 xr[SUM_CH];
#pragma unroll
        for (int i = 0; i < SUM_CH; ++i) xr[i] = *reinterpret_cast<const u32x4*>(rp[i] + c * 8);
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
#pragma unroll
        for (int i = 0; i < SUM_CH; ++i) {
            float x[8];
            unpack8s(xr[i], x);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += e[i] * x[j];
        }
        f32x4 lo = {acc[0], acc[1], acc[2], acc[3]}, hi = {acc[4], acc[5], acc[6], acc[7]};
        *reinterpret_cast<f32x4*>(pa + c * 8) = lo;
        *reinterpret_cast<f32x4*>(pa + c * 8 + 4) = hi;
    }
    if (tid == 0) {
        part_md[2 * blockIdx.x] = m;
        part_md[2 * blockIdx.x + 1] = d;
    }
}

// ---- forward, merge the chunks of a set -------------------------------------------------------
// grid (S, ceil(C / 8 / 64)): 64 column chunks x 4 interleaved chunk lanes per workgroup.
// out bf16 [S, C]; xs_f32 [S, C] and lse [S] for the backward.
constexpr int MERGE_Q = 256;              // chunk scales staged in LDS per pass
__global__ __launch_bounds__(SUM_THREADS) void summary_merge_fwd_kernel(
    int C, const int32_t* __restrict__ seg, int n_tok, int nq_max, const float* __restrict__ part_acc,
    const float* __restrict__ part_md, bf16_t* __restrict__ out, float* __restrict__ xs_f32,
    float* __restrict__ lse) {
    __shared__ float scale[MERGE_Q];
    __shared__ float red[4];
    __shared__ float part4[4][64][8];
    const int s = blockIdx.x;
    const int tid = threadIdx.x;
    int q0, q1;
    chunk_range<SUM_CH>(seg, s, n_tok, nq_max, q0, q1);
    // global maximum and denominator of the set
    float M = kNoScore;
    for (int q = q0 + tid; q < q1; q += SUM_THREADS) M = fmaxf(M, part_md[2 * q]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off, 64));
    if ((tid & 63) == 0) red[tid >> 6] = M;
    __syncthreads();
    M = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    float dpart = 0.0f;
    for (int q = q0 + tid; q < q1; q += SUM_THREADS) dpart += part_md[2 * q + 1] * __expf(part_md[2 * q] - M);
    const float D = block_sum256(dpart, red);
    const float inv = D > 0.0f ? 1.0f / D : 0.0f;     // empty set: zero row
    const int cx = tid & 63, sy = tid >> 6;
    const int c = blockIdx.y * 64 + cx;
    const bool cok = c < (C >> 3);
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    for (int qb = q0; qb < q1; qb += MERGE_Q) {
        const int nqb = q1 - qb < MERGE_Q ? q1 - qb : MERGE_Q;
        __syncthreads();
        if (tid < nqb) scale[tid] = __expf(part_md[2 * (qb + tid)] - M);
        __syncthreads();
        if (cok)
            for (int k = sy; k < nqb; k += 4) {
                const float sc = scale[k];
                const float* pa = part_acc + (int64_t)(qb + k) * C + c * 8;
                f32x4 lo = *reinterpret_cast<const f32x4*>(pa), hi = *reinterpret_cast<const f32x4*>(pa + 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[j] += sc * lo[j];
                    acc[4 + j] += sc * hi[j];
                }
            }
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) part4[sy][cx][j] = acc[j];
    __syncthreads();
    if (sy == 0 && cok) {
#pragma unroll
        for (int j = 0; j < 8; ++j)
            acc[j] = ((part4[0][cx][j] + part4[1][cx][j]) + (part4[2][cx][j] + part4[3][cx][j])) * inv;
        u32x4 pk;
#pragma unroll
        for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(acc[2 * j], acc[2 * j + 1]);
        *reinterpret_cast<u32x4*>(out + (int64_t)s * C + c * 8) = pk;
        if (xs_f32 != nullptr) {
            f32x4 lo = {acc[0], acc[1], acc[2], acc[3]}, hi = {acc[4], acc[5], acc[6], acc[7]};
            *reinterpret_cast<f32x4*>(xs_f32 + (int64_t)s * C + c * 8) = lo;
            *reinterpret_cast<f32x4*>(xs_f32 + (int64_t)s * C + c * 8 + 4) = hi;
        }
    }
    if (lse != nullptr && blockIdx.y == 0 && tid == 0) lse[s] = D > 0.0f ? M + __logf(D) : kNoScore;
}

// ---- backward, per chunk ------------------------------------------------------------------------
// With p_t = exp(s_t - lse), dp_t = g . X_t and delta = g . x^s (= sum_u p_u dp_u):
//   ds_t = p_t (dp_t - delta);  dX_t = p_t g + ds_t w  (added to grad_hidden row t);
//   dw = sum_t ds_t X_t  (per chunk into part_dw, summed by summary_dw_reduce_kernel)
__global__ __launch_bounds__(SUM_THREADS) void summary_chunk_bwd_kernel(
    const bf16_t* __restrict__ hidden, int64_t T, int C, const int32_t* __restrict__ tok,
    const int32_t* __restrict__ seg, int S, int n_tok, const bf16_t* __restrict__ w,
    const float* __restrict__ xs_f32, const float* __restrict__ scores, const float* __restrict__ lse,
    const bf16_t* __restrict__ gout, bf16_t* grad_hidden, float* __restrict__ part_dw) {
    __shared__ float pp[SUM_CH], dss[SUM_CH];
    __shared__ int rowid[SUM_CH];
    __shared__ float red[4];
    int s, t0, nt;
    if (!locate_chunk<SUM_CH>(seg, S, n_tok, (int)blockIdx.x, s, t0, nt)) return;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int chunks = C >> 3;
    const bf16_t* g = gout + (int64_t)s * C;
    // delta = g . x^s
    float dl = 0.0f;
    for (int c = tid; c < chunks; c += SUM_THREADS) {
        float gg[8];
        unpack8s(*reinterpret_cast<const u32x4*>(g + c * 8), gg);
        const float* xp = xs_f32 + (int64_t)s * C + c * 8;
        f32x4 lo = *reinterpret_cast<const f32x4*>(xp), hi = *reinterpret_cast<const f32x4*>(xp + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) dl += gg[j] * lo[j] + gg[4 + j] * hi[j];
    }
    const float delta = block_sum256(dl, red);
    const float L = lse[s];
    {
        int rows[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = wv * 4 + k;
            int row = -1;
            if (i < nt) {
                row = tok[t0 + i];
                if ((uint32_t)row >= (uint32_t)T) row = -1;
            }
            rows[k] = row;
        }
        float dp[4];
        wave_dot4(hidden, C, rows, g, chunks, lane, dp);
        if (lane == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int i = wv * 4 + k;
                if (i < nt) {
                    const float p = rows[k] >= 0 ? __expf(scores[t0 + i] - L) : 0.0f;
                    pp[i] = p;
                    dss[i] = p * (dp[k] - delta);
                    rowid[i] = rows[k];
                }
            }
        }
    }
    __syncthreads();
    float* pd = part_dw + (int64_t)blockIdx.x * C;
    for (int c = tid; c < chunks; c += SUM_THREADS) {
        float gg[8], ww[8], dw[8];
        unpack8s(*reinterpret_cast<const u32x4*>(g + c * 8), gg);
        unpack8s(*reinterpret_cast<const u32x4*>(w + c * 8), ww);
#pragma unroll
        for (int j = 0; j < 8; ++j) dw[j] = 0.0f;
        // eight tokens at a time: all loads first (the rows are distinct, which the compiler
        // cannot know, so a plain read-modify-write loop would serialise on memory latency)
#pragma unroll
        for (int i0 = 0; i0 < SUM_CH; i0 += 8) {
            u32x4 xr[8], gr[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k;
                if (i < nt && rowid[i] >= 0) {
                    const int64_t o = (int64_t)rowid[i] * C + c * 8;
                    xr[k] = *reinterpret_cast<const u32x4*>(hidden + o);
                    gr[k] = *reinterpret_cast<const u32x4*>(grad_hidden + o);
                }
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int i = i0 + k;
                if (i < nt && rowid[i] >= 0) {
                    float x[8], gh[8];
                    unpack8s(xr[k], x);
                    unpack8s(gr[k], gh);
                    const float p = pp[i], ds = dss[i];
#pragma unroll
                    for (int j = 0; j < 8; ++j) {
                        gh[j] += p * gg[j] + ds * ww[j];
                        dw[j] += ds * x[j];
                    }
                    u32x4 pk;
#pragma unroll
                    for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(gh[2 * j], gh[2 * j + 1]);
                    *reinterpret_cast<u32x4*>(grad_hidden + (int64_t)rowid[i] * C + c * 8) = pk;
                }
            }
        }
        f32x4 lo = {dw[0], dw[1], dw[2], dw[3]}, hi = {dw[4], dw[5], dw[6], dw[7]};
        *reinterpret_cast<f32x4*>(pd + c * 8) = lo;
        *reinterpret_cast<f32x4*>(pd + c * 8 + 4) = hi;
    }
}

// dw[c] (+)= sum over all chunks of part_dw[q][c]: eight interleaved partial sums per column,
// added in a fixed order (deterministic).  32 columns per workgroup.
__global__ __launch_bounds__(SUM_THREADS) void summary_dw_reduce_kernel(
    const float* __restrict__ part_dw, const int32_t* __restrict__ seg, int S, int n_tok, int nq_max,
    int C, float* __restrict__ dw, int accumulate) {
    __shared__ float part8[8][32];
    int q0, q1;
    chunk_range<SUM_CH>(seg, S - 1, n_tok, nq_max, q0, q1);           // q1 = total number of chunks
    const int cx = threadIdx.x & 31, sy = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + cx;
    float a0 = 0.0f, a1 = 0.0f;
    if (c < C) {
        int q = sy;
        for (; q + 8 < q1; q += 16) {                  // two loads in flight per thread
            a0 += part_dw[(int64_t)q * C + c];
            a1 += part_dw[(int64_t)(q + 8) * C + c];
        }
        if (q < q1) a0 += part_dw[(int64_t)q * C + c];
    }
    part8[sy][cx] = a0 + a1;
    __syncthreads();
    if (sy == 0 && c < C) {
        float v = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) v += part8[k][cx];
        dw[c] = accumulate ? dw[c] + v : v;
    }
}

// ---- launchers -----------------------------------------------------------------------------------
int64_t summary_max_chunks(int64_t n_tok, int64_t S) { return (n_tok + SUM_CH - 1) / SUM_CH + S; }

hipError_t launch_summary_forward(const bf16_t* hidden, int64_t T, int C, const int32_t* tok,
                                  const int32_t* seg, int64_t n_tok, int S, const bf16_t* w,
                                  bf16_t* out, float* scores, float* lse, float* xs_f32,
                                  float* part_acc, float* part_md, hipStream_t s) {
    if (S <= 0) return hipSuccess;
    const unsigned nq = (unsigned)summary_max_chunks(n_tok, S);
    profile_mark_begin(KC_SUMMARY_FWD, s);
    hipLaunchKernelGGL(summary_chunk_fwd_kernel, dim3(nq), dim3(SUM_THREADS), 0, s, hidden, T, C, tok, seg,
                       S, (int)n_tok, w, scores, part_acc, part_md);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        dim3 grid((unsigned)S, (unsigned)(((C >> 3) + 63) / 64));
        hipLaunchKernelGGL(summary_merge_fwd_kernel, grid, dim3(SUM_THREADS), 0, s, C, seg, (int)n_tok, (int)nq,
                           part_acc, part_md, out, xs_f32, lse);
        e = hipGetLastError();
    }
    profile_mark_end(KC_SUMMARY_FWD, s);
    return e;
}

hipError_t launch_summary_backward(const bf16_t* hidden, int64_t T, int C, const int32_t* tok,
                                   const int32_t* seg, int64_t n_tok, int S, const bf16_t* w,
                                   const float* xs_f32, const float* scores, const float* lse,
                                   const bf16_t* gout, bf16_t* grad_hidden, float* part_dw, float* dw,
                                   int accumulate, hipStream_t s) {
    if (S <= 0) return hipSuccess;
    const unsigned nq = (unsigned)summary_max_chunks(n_tok, S);
    profile_mark_begin(KC_SUMMARY_BWD, s);
    hipLaunchKernelGGL(summary_chunk_bwd_kernel, dim3(nq), dim3(SUM_THREADS), 0, s, hidden, T, C, tok, seg,
                       S, (int)n_tok, w, xs_f32, scores, lse, gout, grad_hidden, part_dw);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) {
        hipLaunchKernelGGL(summary_dw_reduce_kernel, dim3((unsigned)((C + 31) / 32)), dim3(SUM_THREADS), 0,
                           s, part_dw, seg, S, (int)n_tok, (int)nq, C, dw, accumulate);
        e = hipGetLastError();
    }
    profile_mark_end(KC_SUMMARY_BWD, s);
    return e;
}

}  // namespace skipffn
