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

// Whether entry (v, u) comes before entry (vt, t) in the order "DESCENDING ? larger first :
// smaller first", equal values ordered by index.  The order is total: a NaN comes after every
// number (NaNs among themselves by index), so exactly min(k, n) entries have rank < k whatever
// the values are.
template <bool DESCENDING>
__device__ __forceinline__ bool ranks_before(float v, int u, float vt, int t) {
    const bool vn = v != v, tn = vt != vt;
    const bool first = DESCENDING ? v > vt : v < vt;           // false when either is NaN
    const bool same = (v == vt) || (vn && tn);
    return first || (!vn && tn) || (same && u < t);
}
// Number of entries u of vals[0..n) (an LDS array) that come before entry t in that order.
// (One value per LDS read: a four-wide version was measured twice as slow.)
template <bool DESCENDING>
__device__ __forceinline__ int rank_in_lds(const float* vals, int n, int t, float vt) {
    int before = 0;
    for (int u = 0; u < n; ++u) before += ranks_before<DESCENDING>(vals[u], u, vt, t) ? 1 : 0;
    return before;
}

__device__ __forceinline__ float block_sum256(float v, float* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace skipffn
