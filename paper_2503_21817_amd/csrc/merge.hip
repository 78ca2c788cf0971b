// Token merge of the skipped (local) visual tokens (Section 4.1, the three bullet points):
//   1. cosine similarity between every pair of tokens of a set, averaged per token;
//   2. the k tokens of lowest average similarity are kept;
//   3. every other token is merged into the kept token it is most similar to (plain mean).
// The similarity matrices are dense contractions and run on the MFMA GEMM core (normalised
// rows times their transpose, fp32 out, all sets of a group in one grid); everything else is
// small and memory-bound and also runs for a whole group of sets per launch (blockIdx.y = set;
// the sets' row offsets travel in the kernel arguments, so nothing is copied to the device).
// Decisions that depend on floating point (which tokens are kept, where a token goes) are
// taken on the float32 averages / similarities computed here, with ties to the lower index,
// so they are unique for those values.  A token with a non-finite feature has NaN similarities:
// its average ranks after every number, so exactly min(k, n) tokens are kept whatever the input;
// a token whose similarities are all NaN goes to no slot (assign = -1) and gets a zero gradient.
#include "kernels.hpp"
#include "segments.hpp"

namespace skipffn {

constexpr int MG_THREADS = 256;

// ---- Xn = X / |X| (a zero row stays zero), one workgroup per row ------------------------------
__global__ __launch_bounds__(MG_THREADS) void row_normalize_kernel(const bf16_t* __restrict__ x, int C,
                                                                   bf16_t* __restrict__ xn) {
    __shared__ float red[4];
    const int64_t r = blockIdx.x;
    const int tid = threadIdx.x, chunks = C >> 3;
    const u32x4* src = reinterpret_cast<const u32x4*>(x + r * C);
    u32x4* dst = reinterpret_cast<u32x4*>(xn + r * C);
    float ss = 0.0f;
    for (int c = tid; c < chunks; c += MG_THREADS) {
        float f[8];
        unpack8s(src[c], f);
#pragma unroll
        for (int j = 0; j < 8; ++j) ss += f[j] * f[j];
    }
    ss = block_sum256(ss, red);
    const float inv = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;
    for (int c = tid; c < chunks; c += MG_THREADS) {
        float f[8];
        unpack8s(src[c], f);
        u32x4 pk;
#pragma unroll
        for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(f[2 * j] * inv, f[2 * j + 1] * inv);
        dst[c] = pk;
    }
}

// In the kernels below: set = blockIdx.y, rows [lo, lo + n) of the token list; S_set is its
// similarity matrix [n][ld] inside the group's buffer (stride sim_stride floats per set).

// ---- avg_i = (sum_j S_ij - S_ii) / (n - 1), one wavefront per row ------------------------------
__global__ __launch_bounds__(MG_THREADS) void sim_rowmean_kernel(const float* __restrict__ sim, SegTable st,
                                                                 int ld, int64_t sim_stride,
                                                                 float* __restrict__ avg) {
    const int set = blockIdx.y;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const float* row = sim + set * sim_stride + (int64_t)i * ld;
    float acc = 0.0f;
    for (int j = lane; j < n; j += 64) acc += (j == i) ? 0.0f : row[j];
    acc = wave_sum(acc);
    if (lane == 0) avg[lo + i] = n > 1 ? acc / (float)(n - 1) : 0.0f;
}

// ---- kept[t] = 1 iff fewer than k tokens of the set have a lower average -----------------------
__global__ __launch_bounds__(MG_THREADS) void merge_rank_kernel(const float* __restrict__ avg, SegTable st,
                                                                int k, uint8_t* __restrict__ kept) {
    __shared__ __align__(16) uint32_t sav[MERGE_MAX_N];       // rank keys of the averages
    const int set = blockIdx.y;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    if ((int)blockIdx.x * MG_THREADS >= n) return;          // uniform over the workgroup
    for (int u = threadIdx.x; u < n; u += MG_THREADS) sav[u] = rank_key<false>(avg[lo + u]);
    __syncthreads();
    const int t = blockIdx.x * MG_THREADS + threadIdx.x;
    if (t >= n) return;
    const int lower = rank_in_lds(sav, n, t);
    kept[lo + t] = lower < k ? 1 : 0;
}

// ---- slots: position of every kept token among the kept tokens, in index order ----------------
// one workgroup per set; slot_of[t] = slot or -1; kept_idx[set][slot] = lo + t, -1 padding
__global__ __launch_bounds__(MG_THREADS) void merge_slot_kernel(const uint8_t* __restrict__ kept, SegTable st,
                                                                int k, int set_base,
                                                                int32_t* __restrict__ slot_of,
                                                                int32_t* __restrict__ kept_idx) {
    __shared__ int cnt[MG_THREADS];
    const int set = blockIdx.x;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    const int tid = threadIdx.x;
    const int per = (n + MG_THREADS - 1) / MG_THREADS;       // consecutive tokens per thread
    const int b = tid * per, e = b + per < n ? b + per : n;
    int c = 0;
    for (int t = b; t < e; ++t) c += kept[lo + t];
    cnt[tid] = c;
    __syncthreads();
    int slot = 0;
    for (int u = 0; u < tid; ++u) slot += cnt[u];
    int32_t* kout = kept_idx + (int64_t)(set_base + set) * k;
    for (int t = b; t < e; ++t) {
        if (kept[lo + t] && slot < k) {      // the rank order is total, so slot < k always holds: belt and braces
            slot_of[lo + t] = slot;
            kout[slot] = lo + t;
            ++slot;
        } else {
            slot_of[lo + t] = -1;
        }
    }
    const int kk = k < n ? k : n;
    for (int sidx = kk + tid; sidx < k; sidx += MG_THREADS) kout[sidx] = -1;
}

// ---- destination of every token: own slot if kept, else the most similar kept token ----------
__global__ __launch_bounds__(MG_THREADS) void merge_assign_kernel(const float* __restrict__ sim, SegTable st,
                                                                  int ld, int64_t sim_stride,
                                                                  const int32_t* __restrict__ slot_of,
                                                                  int32_t* __restrict__ assign) {
    const int set = blockIdx.y;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (i >= n) return;
    const int own = slot_of[lo + i];
    if (own >= 0) {
        if (lane == 0) assign[lo + i] = own;
        return;
    }
    const float* row = sim + set * sim_stride + (int64_t)i * ld;
    float best = -3.0e38f;
    int bj = 0x7fffffff;
    for (int j = lane; j < n; j += 64) {
        if (slot_of[lo + j] >= 0) {
            const float v = row[j];
            if (v > best) { best = v; bj = j; }      // j ascending per lane: a tie keeps the lower index
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        const float ov = __shfl_xor(best, off, 64);
        const int oj = __shfl_xor(bj, off, 64);
        if (ov > best || (ov == best && oj < bj)) { best = ov; bj = oj; }
    }
    if (lane == 0) assign[lo + i] = bj != 0x7fffffff ? slot_of[lo + bj] : -1;
}

// ---- out[set][slot] = mean of the rows assigned to the slot, added in index order --------------
__global__ __launch_bounds__(MG_THREADS) void merge_mean_kernel(const bf16_t* __restrict__ x, SegTable st, int C,
                                                                int k, int set_base,
                                                                const int32_t* __restrict__ assign,
                                                                bf16_t* __restrict__ out) {
    __shared__ int members[MERGE_MAX_N];
    __shared__ int nmem;
    const int set = blockIdx.y, slot = blockIdx.x;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    const int kk = k < n ? k : n;
    const int tid = threadIdx.x, chunks = C >> 3;
    u32x4* dst = reinterpret_cast<u32x4*>(out + ((int64_t)(set_base + set) * k + slot) * C);
    if (slot >= kk) {                       // fewer tokens than slots: zero rows
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int c = tid; c < chunks; c += MG_THREADS) dst[c] = z;
        return;
    }
    // the slot's member list, in index order (one wavefront compacts with ballots)
    if (tid < 64) {
        int count = 0;
        for (int base = 0; base < n; base += 64) {
            const int i = base + tid;
            const bool mine = i < n && assign[lo + i] == slot;
            const unsigned long long bal = __ballot(mine);
            if (mine) members[count + __popcll(bal & ((1ull << tid) - 1ull))] = i;
            count += __popcll(bal);
        }
        if (tid == 0) nmem = count;
    }
    __syncthreads();
    const int m = nmem;
    const float inv = 1.0f / (float)(m > 0 ? m : 1);
    for (int c = tid; c < chunks; c += MG_THREADS) {
        float acc[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
        for (int q = 0; q < m; ++q) {
            float f[8];
            unpack8s(*reinterpret_cast<const u32x4*>(x + (int64_t)(lo + members[q]) * C + c * 8), f);
#pragma unroll
            for (int j = 0; j < 8; ++j) acc[j] += f[j];
        }
        u32x4 pk;
#pragma unroll
        for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(acc[2 * j] * inv, acc[2 * j + 1] * inv);
        dst[c] = pk;
    }
}

// ---- gradient of the mean: dx[t] = dout[set][assign[t]] / (members of that slot) ---------------
// The kept set and the assignment are piecewise constant in x and carry no gradient.  Every
// workgroup recounts the members per slot of its set in LDS (integer adds: order-free), then
// its wavefronts write MB_ROWS rows.
constexpr int MB_ROWS = 16;

__global__ __launch_bounds__(MG_THREADS) void merge_bwd_kernel(const bf16_t* __restrict__ dout, SegTable st,
                                                               int C, int k, int set_base,
                                                               const int32_t* __restrict__ assign,
                                                               bf16_t* __restrict__ dx) {
    __shared__ int cnt[MERGE_MAX_N];
    const int set = blockIdx.y;
    const int lo = st.off[set], n = st.off[set + 1] - lo;
    const int r0 = blockIdx.x * MB_ROWS;
    if (r0 >= n) return;
    const int kk = k < n ? k : n;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, chunks = C >> 3;
    for (int j = tid; j < kk; j += MG_THREADS) cnt[j] = 0;
    __syncthreads();
    for (int i = tid; i < n; i += MG_THREADS) {
        const int a = assign[lo + i];
        if (a >= 0 && a < kk) atomicAdd(&cnt[a], 1);
    }
    __syncthreads();
    for (int r = r0 + wave; r < r0 + MB_ROWS && r < n; r += 4) {
        const int a = assign[lo + r];
        u32x4* dst = reinterpret_cast<u32x4*>(dx + (int64_t)(lo + r) * C);
        if (a < 0 || a >= kk) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int c = lane; c < chunks; c += 64) dst[c] = z;
            continue;
        }
        const float m = (float)cnt[a];
        const u32x4* src = reinterpret_cast<const u32x4*>(dout + ((int64_t)(set_base + set) * k + a) * C);
        for (int c = lane; c < chunks; c += 64) {
            float f[8];
            unpack8s(src[c], f);
            u32x4 pk;
#pragma unroll
            for (int j = 0; j < 4; ++j) pk[j] = pack_bf16x2(f[2 * j] / m, f[2 * j + 1] / m);
            dst[c] = pk;
        }
    }
}

// ---- launchers ---------------------------------------------------------------------------------------
hipError_t launch_merge_bwd_group(const bf16_t* dout, const SegTable& st, int n_max, int C, int k, int set_base,
                                  const int32_t* assign, bf16_t* dx, hipStream_t s) {
    if (st.count == 0 || n_max <= 0) return hipSuccess;
    hipLaunchKernelGGL(merge_bwd_kernel, dim3((unsigned)((n_max + MB_ROWS - 1) / MB_ROWS), (unsigned)st.count),
                       dim3(MG_THREADS), 0, s, dout, st, C, k, set_base, assign, dx);
    return hipGetLastError();
}

hipError_t launch_row_normalize(const bf16_t* x, int64_t rows, int C, bf16_t* xn, hipStream_t s) {
    if (rows <= 0) return hipSuccess;
    hipLaunchKernelGGL(row_normalize_kernel, dim3((unsigned)rows), dim3(MG_THREADS), 0, s, x, C, xn);
    return hipGetLastError();
}

// steps after the similarity GEMMs for the sets of one table (set_base = index of its first set)
hipError_t launch_merge_group(const bf16_t* x, const SegTable& st, int n_max, int C, int k, int set_base,
                              const float* sim, int ld, int64_t sim_stride, float* avg, uint8_t* kept,
                              int32_t* slot_of, int32_t* kept_idx, int32_t* assign, bf16_t* out,
                              hipStream_t s) {
    hipError_t e = hipSuccess;
    const unsigned sets = (unsigned)st.count;
    if (sets == 0) return e;
    if (n_max > 0) {
        hipLaunchKernelGGL(sim_rowmean_kernel, dim3((unsigned)((n_max + 3) / 4), sets), dim3(MG_THREADS), 0, s,
                           sim, st, ld, sim_stride, avg);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(merge_rank_kernel, dim3((unsigned)((n_max + MG_THREADS - 1) / MG_THREADS), sets),
                           dim3(MG_THREADS), 0, s, avg, st, k, kept);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(merge_slot_kernel, dim3(sets), dim3(MG_THREADS), 0, s, kept, st, k, set_base, slot_of,
                       kept_idx);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    if (n_max > 0) {
        hipLaunchKernelGGL(merge_assign_kernel, dim3((unsigned)((n_max + 3) / 4), sets), dim3(MG_THREADS), 0, s,
                           sim, st, ld, sim_stride, slot_of, assign);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (k > 0) {
        hipLaunchKernelGGL(merge_mean_kernel, dim3((unsigned)k, sets), dim3(MG_THREADS), 0, s, x, st, C, k,
                           set_base, assign, out);
        e = hipGetLastError();
    }
    return e;
}

}  // namespace skipffn
