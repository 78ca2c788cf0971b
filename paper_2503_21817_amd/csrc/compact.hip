// Mask -> ascending retained-token indices (stream compaction).
//
// The retained / skipped partition of Section 4.1 arrives as one byte per token
// (non-zero = the token skips the FFN).  Each wavefront walks a contiguous token
// range 256 tokens at a time: a lane loads 4 mask bytes, four wave ballots give
// the keep-bits of the whole 256-token slab, and mbcnt (popcount of the ballot
// below the lane) gives every lane its exclusive rank - no shared-memory scan in
// the inner loop.  Ranges are ordered wave-major inside a block and block-major
// across blocks, so ranks are ascending in token order and the result is unique
// and deterministic.  Small inputs (every configuration of the block itself) use
// one block and one launch; large masks use count / scan / write launches with
// no spinning between blocks.
#include <mutex>

#include "kernels.hpp"

namespace skipffn {

constexpr int CP_THREADS = 1024;
constexpr int CP_WAVES = CP_THREADS / 64;
constexpr int64_t CP_SINGLE_MAX = 262144;   // one block up to this many tokens
constexpr int64_t CP_BLOCK_SPAN = 65536;    // tokens per block beyond that

__device__ __forceinline__ uint32_t load_mask4(const uint8_t* mask, int64_t tok, int64_t end) {
    // bytes past `end` read as 1 (skipped)
    if (tok + 4 <= end) return *reinterpret_cast<const uint32_t*>(mask + tok);
    uint32_t w = 0x01010101u;
    for (int j = 0; j < 4; ++j)
        if (tok + j < end) w = (w & ~(0xffu << (8 * j))) | ((uint32_t)mask[tok + j] << (8 * j));
    return w;
}

__device__ __forceinline__ int lanes_below(uint64_t m) {
    return __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0));
}

// A wave walks its range 1024 tokens at a time: the four 4-byte mask loads of a lane are issued
// together (the walk is bound by load latency, not by the ballots), then the four 256-token
// slabs are ranked one after the other.
constexpr int CP_UNROLL = 4;

// number of retained tokens in [begin, end) - one wave
__device__ int wave_count(const uint8_t* mask, int64_t begin, int64_t end, int lane) {
    int total = 0;
    for (int64_t base = begin; base < end; base += 256 * CP_UNROLL) {
        uint32_t w[CP_UNROLL];
#pragma unroll
        for (int q = 0; q < CP_UNROLL; ++q) {
            const int64_t tok = base + 256 * q + 4 * lane;
            w[q] = tok < end ? load_mask4(mask, tok, end) : 0x01010101u;
        }
#pragma unroll
        for (int q = 0; q < CP_UNROLL; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                bool keep = ((w[q] >> (8 * j)) & 0xffu) == 0u;
                total += __popcll(__ballot(keep));
            }
    }
    return total;   // uniform over the wave
}

__device__ void wave_write(const uint8_t* mask, int64_t begin, int64_t end, int lane,
                           int out_base, int32_t* idx, int32_t* pos) {
    for (int64_t base = begin; base < end; base += 256 * CP_UNROLL) {
        uint32_t wq[CP_UNROLL];
#pragma unroll
        for (int q = 0; q < CP_UNROLL; ++q) {
            const int64_t tok = base + 256 * q + 4 * lane;
            wq[q] = tok < end ? load_mask4(mask, tok, end) : 0x01010101u;
        }
#pragma unroll
        for (int q = 0; q < CP_UNROLL; ++q) {
            const int64_t tok = base + 256 * q + 4 * lane;
            const uint32_t w = wq[q];
            bool keep[4];
            int rank = 0, slab = 0;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                keep[j] = ((w >> (8 * j)) & 0xffu) == 0u;
                uint64_t m = __ballot(keep[j]);
                rank += lanes_below(m);       // kept tokens of lower lanes at byte j
                slab += __popcll(m);
            }
            // tokens of lower lanes at ANY byte position precede this lane's tokens
            int r = out_base + rank;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (tok + j < end) {
                    if (keep[j]) {
                        idx[r] = (int32_t)(tok + j);
                        if (pos) pos[tok + j] = r;
                        ++r;
                    } else if (pos) {
                        pos[tok + j] = -1;
                    }
                }
            }
            out_base += slab;
        }
    }
}

// MODE 0: single block does everything.  MODE 1: count only -> block_count.
// MODE 2: write, starting at block_offset[block].
template <int MODE>
__global__ __launch_bounds__(CP_THREADS) void compact_kernel(
    const uint8_t* __restrict__ mask, int64_t T, int64_t span, int32_t* __restrict__ idx,
    int32_t* __restrict__ num_retained, int32_t* __restrict__ pos,
    int32_t* __restrict__ block_count, const int32_t* __restrict__ block_offset) {
    __shared__ int wcount[CP_WAVES];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t bbegin = (int64_t)blockIdx.x * span;
    int64_t bend = bbegin + span < T ? bbegin + span : T;
    int64_t wspan = span / CP_WAVES;              // multiple of 256 by construction
    int64_t wbegin = bbegin + wave * wspan;
    int64_t wend = wbegin + wspan < bend ? wbegin + wspan : bend;
    if (wbegin > bend) wbegin = bend;

    int c = wave_count(mask, wbegin, wend, lane);
    if (lane == 0) wcount[wave] = c;
    __syncthreads();
    int before = 0, total = 0;
#pragma unroll
    for (int w = 0; w < CP_WAVES; ++w) {
        int v = wcount[w];
        before += w < wave ? v : 0;
        total += v;
    }
    if (MODE == 1) {
        if (threadIdx.x == 0) block_count[blockIdx.x] = total;
        return;
    }
    int base = MODE == 2 ? block_offset[blockIdx.x] : 0;
    if (MODE == 0 && threadIdx.x == 0) *num_retained = total;
    wave_write(mask, wbegin, wend, lane, base + before, idx, pos);
}

// exclusive scan of nb block counts by one block; also writes the grand total
__global__ __launch_bounds__(CP_THREADS) void compact_scan_kernel(
    const int32_t* __restrict__ block_count, int nb, int32_t* __restrict__ block_offset,
    int32_t* __restrict__ num_retained) {
    __shared__ int part[CP_THREADS];
    const int t = threadIdx.x;
    const int per = (nb + CP_THREADS - 1) / CP_THREADS;
    int lo = t * per, hi = lo + per < nb ? lo + per : nb;
    int s = 0;
    for (int i = lo; i < hi; ++i) s += block_count[i];
    part[t] = s;
    __syncthreads();
    // Hillis-Steele inclusive scan over 1024 partial sums
    for (int off = 1; off < CP_THREADS; off <<= 1) {
        int v = t >= off ? part[t - off] : 0;
        __syncthreads();
        part[t] += v;
        __syncthreads();
    }
    int run = part[t] - s;    // exclusive prefix of this thread's slice
    for (int i = lo; i < hi; ++i) {
        block_offset[i] = run;
        run += block_count[i];
    }
    if (t == CP_THREADS - 1) *num_retained = part[t];
}

static int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }

static int compact_blocks(int64_t T) {
    if (T <= CP_SINGLE_MAX) return 1;
    return (int)((T + CP_BLOCK_SPAN - 1) / CP_BLOCK_SPAN);
}

size_t compact_workspace_bytes(int64_t T) {
    int nb = compact_blocks(T < 0 ? 0 : T);
    return round_up((size_t)nb * 2 * sizeof(int32_t), 256);
}

hipError_t launch_compact(const uint8_t* mask, int64_t T, int32_t* idx, int32_t* num_retained,
                          int32_t* pos, void* ws, hipStream_t s) {
    const int nb = compact_blocks(T);
    if (nb == 1) {
        int64_t span = round_up(T > 0 ? T : 1, 256 * CP_WAVES);
        profile_mark_begin(KC_COMPACT, s);
        hipLaunchKernelGGL(compact_kernel<0>, dim3(1), dim3(CP_THREADS), 0, s, mask, T, span, idx,
                           num_retained, pos, (int32_t*)nullptr, (const int32_t*)nullptr);
        profile_mark_end(KC_COMPACT, s);
        return hipGetLastError();
    }
    int32_t* count = static_cast<int32_t*>(ws);
    int32_t* offset = count + nb;
    const int64_t span = CP_BLOCK_SPAN;
    profile_mark_begin(KC_COMPACT, s);
    hipLaunchKernelGGL(compact_kernel<1>, dim3(nb), dim3(CP_THREADS), 0, s, mask, T, span, idx,
                       num_retained, pos, count, (const int32_t*)nullptr);
    hipLaunchKernelGGL(compact_scan_kernel, dim3(1), dim3(CP_THREADS), 0, s, count, nb, offset,
                       num_retained);
    hipLaunchKernelGGL(compact_kernel<2>, dim3(nb), dim3(CP_THREADS), 0, s, mask, T, span, idx,
                       num_retained, pos, (int32_t*)nullptr, offset);
    profile_mark_end(KC_COMPACT, s);
    return hipGetLastError();
}

// ---- compaction with the library's own scratch (callers that cannot allocate) ---------------------
// The count / offset arrays of the multi-block path live in a file-scope device array instead of
// a caller workspace.  Each GPU the library runs on holds its own copy of the array at its own
// address; the address is looked up once per device, with that device current, and host code
// uses that pointer only (the array's name is a host-side stand-in, not a device address).
// Nothing in the array has to start at zero: every launch writes the counts and offsets of the
// blocks it uses before reading them.  Calls that overlap in time on one GPU share the array
// and race; calls on one stream (or otherwise ordered) do not.
constexpr int CP_STATIC_MAX_BLOCKS = 4096;                       // 32 KB of scratch per GPU
static __device__ __align__(256) int32_t scratch[2 * CP_STATIC_MAX_BLOCKS];

int64_t compact_static_max_tokens() { return (int64_t)CP_STATIC_MAX_BLOCKS * CP_BLOCK_SPAN; }

constexpr int CP_MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static int32_t* g_scratch_ptr[CP_MAX_DEVICES];

hipError_t launch_compact_static(const uint8_t* mask, int64_t T, int32_t* idx, int32_t* num_retained,
                                 int32_t* pos, hipStream_t s) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= CP_MAX_DEVICES) return hipErrorInvalidDevice;
    int32_t* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lk(g_scratch_mu);
        if (g_scratch_ptr[dev] == nullptr) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (p == nullptr) return hipErrorInvalidSymbol;
            g_scratch_ptr[dev] = static_cast<int32_t*>(p);
        }
        ptr = g_scratch_ptr[dev];
    }
    return launch_compact(mask, T, idx, num_retained, pos, ptr, s);
}

// ---- index-list check (debugging aid of the forward / backward calls) ---------------------------
// status[0] = 0 when idx[0..R) is strictly ascending and inside [0, T), else 1; status[1] = the
// first offending position (INT_MAX when there is none).  Two launches: the first resets the
// two words (a kernel, so that the sequence can be captured in a HIP graph).
__global__ void idx_status_reset_kernel(int32_t* __restrict__ status) {
    if (threadIdx.x == 0) { status[0] = 0; status[1] = 0x7fffffff; }
}
__global__ __launch_bounds__(256) void validate_idx_kernel(const int32_t* __restrict__ idx, int Rbound,
                                                           const int32_t* __restrict__ r_dev, int64_t T,
                                                           int32_t* __restrict__ status) {
    const int R = effective_rows(Rbound, r_dev);
    for (int r = blockIdx.x * 256 + threadIdx.x; r < R; r += gridDim.x * 256) {
        const int v = idx[r];
        const bool bad = v < 0 || (int64_t)v >= T || (r > 0 && idx[r - 1] >= v);
        if (bad) {
            atomicMin(&status[1], r);
            status[0] = 1;
        }
    }
}

hipError_t launch_validate_idx(const int32_t* idx, int R, const int32_t* r_dev, int64_t T, int32_t* status,
                               hipStream_t s) {
    hipLaunchKernelGGL(idx_status_reset_kernel, dim3(1), dim3(64), 0, s, status);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || R <= 0) return e;
    int blocks = (R + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    hipLaunchKernelGGL(validate_idx_kernel, dim3(blocks), dim3(256), 0, s, idx, R, r_dev, T, status);
    return hipGetLastError();
}

}  // namespace skipffn
