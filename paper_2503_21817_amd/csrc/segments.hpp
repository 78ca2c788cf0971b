// Token sets described by a device-side offset table: set i is positions [seg[i], seg[i+1]) of
// a token list of n_tok entries.  Sets are cut into chunks of CH positions, one workgroup per
// chunk; a launch covers the upper bound ceil(n_tok / CH) + S chunks and workgroups past the
// real count exit.  Bounds are clamped so that a malformed table cannot send a read outside
// the list.
#pragma once

#include "common.hpp"

namespace skipffn {

__device__ __forceinline__ void seg_bounds(const int32_t* __restrict__ seg, int i, int n_tok, int& b, int& e) {
    e = seg[i + 1];
    e = e < 0 ? 0 : (e > n_tok ? n_tok : e);
    b = seg[i];
    b = b < 0 ? 0 : (b > e ? e : b);
}
// chunk q -> (set s, first position t0, count nt); false past the last chunk
template <int CH>
__device__ __forceinline__ bool locate_chunk(const int32_t* __restrict__ seg, int S, int n_tok, int q,
                                             int& s, int& t0, int& nt) {
    int cc = 0;
    for (int i = 0; i < S; ++i) {
        int b, e;
        seg_bounds(seg, i, n_tok, b, e);
        const int nc = (e - b + CH - 1) / CH;
        if (q < cc + nc) {
            s = i;
            t0 = b + (q - cc) * CH;
            nt = e - t0 < CH ? e - t0 : CH;
            return true;
        }
        cc += nc;
    }
    return false;
}
// chunks [q0, q1) of set s, clamped to the nq_max chunks the launch covers
template <int CH>
__device__ __forceinline__ void chunk_range(const int32_t* __restrict__ seg, int s, int n_tok, int nq_max,
                                            int& q0, int& q1) {
    int cc = 0;
    for (int i = 0; i < s; ++i) {
        int b, e;
        seg_bounds(seg, i, n_tok, b, e);
        cc += (e - b + CH - 1) / CH;
    }
    int b, e;
    seg_bounds(seg, s, n_tok, b, e);
    q0 = cc < nq_max ? cc : nq_max;
    q1 = cc + (e - b + CH - 1) / CH;
    q1 = q1 < nq_max ? q1 : nq_max;
}

__device__ __forceinline__ void unpack8s(const u32x4& v, float* f) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = bf16lo_to_f32(v[j]);
        f[2 * j + 1] = bf16hi_to_f32(v[j]);
    }
}

// The order of the rank counts: "DESCENDING ? larger first : smaller first", equal values (+0 and
// -0 are equal) ordered by index.  The order is total: a NaN comes after every number (NaNs among
// themselves by index), so exactly min(k, n) entries have rank < k whatever the values are.
// rank_key maps a value to an unsigned key that increases along that order, so that "entry (v, u)
// comes before entry (vt, t)" is one 64-bit comparison of (key, index) pairs: the rank loops do a
// compare and an add per entry instead of the five float comparisons of the direct form (which
// took the rank kernels from 28 to 82 us at 1024-token sets).
template <bool DESCENDING>
__device__ __forceinline__ uint32_t rank_key(float v) {
    if (v != v) return 0xFFFFFFFFu;
    uint32_t b = __float_as_uint(v);
    if (b == 0x80000000u) b = 0u;                               // -0 == +0
    // increasing with v; numbers (infinities included) map into [0x007FFFFF, 0xFF800000], and so does the
    // complement of that range, so 0xFFFFFFFF is left to the NaNs in both orders
    const uint32_t asc = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
    return DESCENDING ? ~asc : asc;
}
__device__ __forceinline__ uint64_t rank_pair(uint32_t key, int index) {
    return ((uint64_t)key << 32) | (uint32_t)index;
}
// Number of entries u of keys[0..n) (an LDS array of rank_key values) that come before entry t.
// (One value per LDS read: a four-wide version was measured twice as slow.)
__device__ __forceinline__ int rank_in_lds(const uint32_t* keys, int n, int t) {
    const uint64_t mine = rank_pair(keys[t], t);
    int before = 0;
    for (int u = 0; u < n; ++u) before += rank_pair(keys[u], u) < mine ? 1 : 0;
    return before;
}

__device__ __forceinline__ float block_sum256(float v, float* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace skipffn
