// Memory-bound row kernels of the Skip-FFN block: 16-byte accesses, fp32 arithmetic.
// Rows are addressed through the retained index list, so only the R retained rows are
// touched (Section 4.2: skipped tokens keep their residual and see no FFN work).
// Kernels that reduce over a row give the row to one 256-thread workgroup (R is a few
// thousand at most, so a wavefront per row would leave most of the chip without work in
// flight); purely elementwise ones run one thread per 16-byte chunk.
#include "kernels.hpp"

namespace skipffn {

constexpr int ROW_THREADS = 256;
constexpr int RMS_MAXV = 4;                   // register-resident row up to C = 256*8*4 = 8192

__device__ __forceinline__ void unpack8(const u32x4& v, float* f) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f[2 * j] = bf16lo_to_f32(v[j]);
        f[2 * j + 1] = bf16hi_to_f32(v[j]);
    }
}
__device__ __forceinline__ u32x4 pack8(const float* f) {
    u32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = pack_bf16x2(f[2 * j], f[2 * j + 1]);
    return v;
}
// sum over the 256 threads of a workgroup (one call per kernel: `red` is not reused)
__device__ __forceinline__ float block_sum(float v, float* red) {
    v = wave_sum(v);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return (red[0] + red[1]) + (red[2] + red[3]);
}

// ---- gather + RMSNorm -------------------------------------------------------------
// n(x) = x * rsqrt(mean(x^2) + eps) * gain for the rows idx[r]; x is read once
// (held in registers), the un-normalised row is optionally copied for backward.
template <bool IN_REGS>
__global__ __launch_bounds__(ROW_THREADS) void gather_rmsnorm_kernel(
    const bf16_t* __restrict__ hidden, const int32_t* __restrict__ idx, int Rbound,
    const int32_t* __restrict__ r_dev, int C, float eps, const bf16_t* __restrict__ gain,
    bf16_t* __restrict__ xrows, bf16_t* __restrict__ xn, float* __restrict__ rstd_out) {
    __shared__ float red[4];
    const int R = effective_rows(Rbound, r_dev);
    const int tid = threadIdx.x;
    const int r = blockIdx.x;
    if (r >= R) return;                       // the whole workgroup leaves together
    const int chunks = C >> 3;
    const u32x4* src = reinterpret_cast<const u32x4*>(hidden + (int64_t)idx[r] * C);
    const u32x4* gsrc = reinterpret_cast<const u32x4*>(gain);
    u32x4* dxn = reinterpret_cast<u32x4*>(xn + (int64_t)r * C);
    u32x4* dxr = xrows ? reinterpret_cast<u32x4*>(xrows + (int64_t)r * C) : nullptr;

    u32x4 held[IN_REGS ? RMS_MAXV : 1];
    float ss = 0.0f;
    if (IN_REGS) {
#pragma unroll
        for (int v = 0; v < RMS_MAXV; ++v) {
            int c = tid + ROW_THREADS * v;
            if (c < chunks) {
                held[v] = src[c];
                float f[8];
                unpack8(held[v], f);
#pragma unroll
                for (int j = 0; j < 8; ++j) ss += f[j] * f[j];
            }
        }
    } else {
        for (int c = tid; c < chunks; c += ROW_THREADS) {
            float f[8];
            unpack8(src[c], f);
#pragma unroll
            for (int j = 0; j < 8; ++j) ss += f[j] * f[j];
        }
    }
    ss = block_sum(ss, red);
    const float rstd = 1.0f / sqrtf(ss / (float)C + eps);
    if (tid == 0) rstd_out[r] = rstd;

    auto emit = [&](int c, const u32x4& raw) {
        float f[8];
        unpack8(raw, f);
        if (gain != nullptr) {
            float g[8];
            unpack8(gsrc[c], g);
#pragma unroll
            for (int j = 0; j < 8; ++j) f[j] = f[j] * rstd * g[j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) f[j] = f[j] * rstd;
        }
        dxn[c] = pack8(f);
        if (dxr) dxr[c] = raw;
    };
    if (IN_REGS) {
#pragma unroll
        for (int v = 0; v < RMS_MAXV; ++v) {
            int c = tid + ROW_THREADS * v;
            if (c < chunks) emit(c, held[v]);
        }
    } else {
        for (int c = tid; c < chunks; c += ROW_THREADS) emit(c, src[c]);
    }
}

hipError_t launch_gather_rmsnorm(const bf16_t* hidden, const int32_t* idx, int R,
                                 const int32_t* r_dev, int C, float eps, const bf16_t* gain,
                                 bf16_t* xrows, bf16_t* xn, float* rstd, hipStream_t s) {
    if (R <= 0) return hipSuccess;
    dim3 grid(R), block(ROW_THREADS);
    profile_mark_begin(KC_GATHER_RMSNORM, s);
    if (C <= ROW_THREADS * 8 * RMS_MAXV)
        hipLaunchKernelGGL(gather_rmsnorm_kernel<true>, grid, block, 0, s, hidden, idx, R, r_dev, C,
                           eps, gain, xrows, xn, rstd);
    else
        hipLaunchKernelGGL(gather_rmsnorm_kernel<false>, grid, block, 0, s, hidden, idx, R, r_dev, C,
                           eps, gain, xrows, xn, rstd);
    profile_mark_end(KC_GATHER_RMSNORM, s);
    return hipGetLastError();
}

// ---- split-K reduce + residual + scatter ----------------------------------------------
// out[idx[r]][c] = bf16( res[idx[r]][c] + sum_z partial[z][r][c] ), summed in z order.
// One thread per 16-byte chunk of the output.
// number of partial slabs to add for row r, column col
__device__ __forceinline__ int partial_count(const PartialLayout& pl, int R, int r, int col) {
    if (pl.sk_nbg == 0) return pl.splits;
    const StreamKPlan p = streamk_plan((R + BM - 1) / BM, pl.sk_kt, pl.sk_nbg);
    (void)col;                       // the count depends on the m-tile only
    return streamk_count(p, r / BM);
}

__global__ __launch_bounds__(ROW_THREADS) void resid_scatter_kernel(
    const float* __restrict__ partial, PartialLayout pl, int Rbound, const int32_t* __restrict__ r_dev,
    int C, const int32_t* __restrict__ idx, const bf16_t* res, bf16_t* out, int no_residual) {
    const int R = effective_rows(Rbound, r_dev);
    const int chunks = C >> 3;
    const int64_t g = (int64_t)blockIdx.x * ROW_THREADS + threadIdx.x;
    const int r = (int)(g / chunks), c = (int)(g - (int64_t)r * chunks);
    if (r >= R) return;
    const int64_t orow = (int64_t)idx[r] * C;
    const int64_t zstride = (int64_t)Rbound * C;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    const float* p = partial + (int64_t)r * C + c * 8;
    const int splits = partial_count(pl, R, r, c * 8);
    for (int z = 0; z < splits; ++z) {
        f32x4 a = *reinterpret_cast<const f32x4*>(p + z * zstride);
        f32x4 b = *reinterpret_cast<const f32x4*>(p + z * zstride + 4);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[j] += a[j];
            acc[4 + j] += b[j];
        }
    }
    if (!no_residual) {
        float x[8];
        unpack8(*reinterpret_cast<const u32x4*>(res + orow + c * 8), x);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += x[j];
    }
    *reinterpret_cast<u32x4*>(out + orow + c * 8) = pack8(acc);
}

hipError_t launch_resid_scatter(const float* partial, PartialLayout pl, int R, const int32_t* r_dev,
                                int C, const int32_t* idx, const bf16_t* res, bf16_t* out,
                                int no_residual, hipStream_t s) {
    if (R <= 0) return hipSuccess;
    const int64_t total = (int64_t)R * (C >> 3);
    dim3 grid((unsigned)((total + ROW_THREADS - 1) / ROW_THREADS)), block(ROW_THREADS);
    profile_mark_begin(KC_RESID_SCATTER, s);
    hipLaunchKernelGGL(resid_scatter_kernel, grid, block, 0, s, partial, pl, R, r_dev, C, idx,
                       res, out, no_residual);
    profile_mark_end(KC_RESID_SCATTER, s);
    return hipGetLastError();
}

// ---- SwiGLU over split-K partial sums of the gate/up GEMM (few rows) ------------------------------
// partial[z][Rbound][ldp] fp32, ldp = tiles_n * 256: tile tn holds gate columns tn*128 .. +127 at
// tn*256 and the same up columns at tn*256 + 128.  One thread per 8 columns of I:
// H = silu(sum_z gate) * sum_z up (and G, U when they are saved), splits summed in order.
__global__ __launch_bounds__(ROW_THREADS) void swiglu_reduce_kernel(
    const float* __restrict__ partial, int splits, int Rbound, const int32_t* __restrict__ r_dev, int I,
    int ldp, bf16_t* __restrict__ H, bf16_t* __restrict__ G, bf16_t* __restrict__ U) {
    const int R = effective_rows(Rbound, r_dev);
    const int chunks = I >> 3;
    const int64_t gid = (int64_t)blockIdx.x * ROW_THREADS + threadIdx.x;
    const int r = (int)(gid / chunks), c = (int)(gid - (int64_t)r * chunks);
    if (r >= R) return;
    const int i0 = c * 8;
    const float* p = partial + (int64_t)r * ldp + (i0 >> 7) * 256 + (i0 & 127);
    const int64_t zstride = (int64_t)Rbound * ldp;
    float g[8], u[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { g[j] = 0.0f; u[j] = 0.0f; }
    for (int z = 0; z < splits; ++z) {
        const f32x4 g0 = *reinterpret_cast<const f32x4*>(p + z * zstride);
        const f32x4 g1 = *reinterpret_cast<const f32x4*>(p + z * zstride + 4);
        const f32x4 u0 = *reinterpret_cast<const f32x4*>(p + z * zstride + 128);
        const f32x4 u1 = *reinterpret_cast<const f32x4*>(p + z * zstride + 132);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            g[j] += g0[j]; g[4 + j] += g1[j];
            u[j] += u0[j]; u[4 + j] += u1[j];
        }
    }
    float h[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) h[j] = g[j] * __builtin_amdgcn_rcpf(1.0f + __expf(-g[j])) * u[j];
    const int64_t o = (int64_t)r * I + i0;
    *reinterpret_cast<u32x4*>(H + o) = pack8(h);
    if (G != nullptr) {
        *reinterpret_cast<u32x4*>(G + o) = pack8(g);
        *reinterpret_cast<u32x4*>(U + o) = pack8(u);
    }
}

hipError_t launch_swiglu_reduce(const float* partial, int splits, int R, const int32_t* r_dev, int I, int ldp,
                                bf16_t* H, bf16_t* G, bf16_t* U, hipStream_t s) {
    if (R <= 0) return hipSuccess;
    const int64_t total = (int64_t)R * (I >> 3);
    dim3 grid((unsigned)((total + ROW_THREADS - 1) / ROW_THREADS)), block(ROW_THREADS);
    hipLaunchKernelGGL(swiglu_reduce_kernel, grid, block, 0, s, partial, splits, R, r_dev, I, ldp, H, G, U);
    return hipGetLastError();
}

// ---- row gather (upstream gradient rows; skip KV-cache of Section 4.3) -----------------
constexpr int ROWS_PER_BLOCK = ROW_THREADS / 64;   // copy kernels: one wavefront per row
__global__ __launch_bounds__(ROW_THREADS) void gather_rows_kernel(
    const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t row_chunks,
    const int32_t* __restrict__ idx, int Rbound, const int32_t* __restrict__ r_dev) {
    const int R = effective_rows(Rbound, r_dev);
    const int lane = threadIdx.x & 63;
    const int r = blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (r >= R) return;
    const u32x4* s = src + (int64_t)idx[r] * row_chunks;
    u32x4* d = dst + (int64_t)r * row_chunks;
    for (int64_t c = lane; c < row_chunks; c += 64) d[c] = s[c];
}

hipError_t launch_gather_rows(const void* src, void* dst, int64_t row_bytes, const int32_t* idx,
                              int R, const int32_t* r_dev, hipStream_t s) {
    if (R <= 0 || row_bytes <= 0) return hipSuccess;
    dim3 grid((R + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK), block(ROW_THREADS);
    profile_mark_begin(KC_GATHER_ROWS, s);
    hipLaunchKernelGGL(gather_rows_kernel, grid, block, 0, s, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), row_bytes / 16, idx, R, r_dev);
    profile_mark_end(KC_GATHER_ROWS, s);
    return hipGetLastError();
}

// ---- skip KV-cache over a whole cache (Section 4.3) --------------------------------------------
// One thread per 16-byte chunk of the compacted cache; blockIdx.y walks the slabs.  Cache rows
// are short (one head of one token: 256 bytes for d = 128), so a wavefront per row would
// leave three quarters of its lanes idle.
__global__ __launch_bounds__(ROW_THREADS) void kv_compact_kernel(
    const char* __restrict__ src, char* __restrict__ dst, int64_t n_slabs, int row_chunks,
    int64_t src_slab_bytes, int64_t dst_slab_bytes, const int32_t* __restrict__ idx, int Rbound,
    const int32_t* __restrict__ r_dev) {
    const int R = effective_rows(Rbound, r_dev);
    const int64_t g = (int64_t)blockIdx.x * ROW_THREADS + threadIdx.x;
    const int r = (int)(g / row_chunks), c = (int)(g - (int64_t)r * row_chunks);
    if (r >= R) return;
    const int64_t so = (int64_t)idx[r] * row_chunks + c, d_o = (int64_t)r * row_chunks + c;
    for (int64_t sl = blockIdx.y; sl < n_slabs; sl += gridDim.y) {
        const u32x4* s = reinterpret_cast<const u32x4*>(src + sl * src_slab_bytes);
        u32x4* d = reinterpret_cast<u32x4*>(dst + sl * dst_slab_bytes);
        d[d_o] = s[so];
    }
}

hipError_t launch_kv_compact(const void* src, void* dst, int64_t n_slabs, int64_t row_bytes,
                             int64_t src_slab_bytes, int64_t dst_slab_bytes, const int32_t* idx,
                             int R, const int32_t* r_dev, hipStream_t s) {
    if (R <= 0 || row_bytes <= 0 || n_slabs <= 0) return hipSuccess;
    const int row_chunks = (int)(row_bytes / 16);
    const int64_t per_slab = (int64_t)R * row_chunks;
    dim3 grid((unsigned)((per_slab + ROW_THREADS - 1) / ROW_THREADS),
              (unsigned)(n_slabs < 65535 ? n_slabs : 65535)), block(ROW_THREADS);
    profile_mark_begin(KC_KV_COMPACT, s);
    hipLaunchKernelGGL(kv_compact_kernel, grid, block, 0, s, static_cast<const char*>(src),
                       static_cast<char*>(dst), n_slabs, row_chunks, src_slab_bytes, dst_slab_bytes,
                       idx, R, r_dev);
    profile_mark_end(KC_KV_COMPACT, s);
    return hipGetLastError();
}

// ---- row gather with a transposed copy ------------------------------------------------------
// dst[r][:] = src[row(r)][:] (optional) and dstT[c][r] = src[row(r)][c], where row(r) = idx[r]
// (or r when idx is null).  dstT has leading dimension ldT (a multiple of 8 >= the row
// bound); columns r >= R of dstT are written as zeros so that K-slabs reading past R see
// zeros.  The weight-gradient GEMMs contract over R: a copy with R contiguous lets them read
// this operand with plain 16-byte LDS reads instead of transposing ones.
constexpr int TR_TILE = 64;
__global__ __launch_bounds__(256) void gather_transpose_kernel(
    const bf16_t* __restrict__ src, int C, const int32_t* __restrict__ idx, int Rbound,
    const int32_t* __restrict__ r_dev, bf16_t* __restrict__ dst, bf16_t* __restrict__ dstT, int ldT) {
    __shared__ bf16_t tile[TR_TILE][TR_TILE + 2];
    const int R = effective_rows(Rbound, r_dev);
    const int r0 = blockIdx.x * TR_TILE, c0 = blockIdx.y * TR_TILE;
    const int t = threadIdx.x;
    // phase 1: 64 rows x 64 columns, 16 bytes per access
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = t + 256 * i;
        const int rr = q >> 3, ch = q & 7;
        const int r = r0 + rr, c = c0 + ch * 8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (r < R && c < C) {
            const int64_t srow = idx ? (int64_t)idx[r] : (int64_t)r;
            v = *reinterpret_cast<const u32x4*>(src + srow * C + c);
            if (dst) *reinterpret_cast<u32x4*>(dst + (int64_t)r * C + c) = v;
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            tile[rr][ch * 8 + 2 * k] = (bf16_t)(v[k] & 0xffffu);
            tile[rr][ch * 8 + 2 * k + 1] = (bf16_t)(v[k] >> 16);
        }
    }
    __syncthreads();
    // phase 2: 64 output rows (columns of src) x 64 r values = 8 chunks of 16 bytes each
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = t + 256 * i;
        const int cc = q >> 3, ch = q & 7;
        const int c = c0 + cc, r = r0 + ch * 8;
        if (c < C && r < ldT) {
            u32x4 v;
#pragma unroll
            for (int k = 0; k < 4; ++k)
                v[k] = (uint32_t)tile[ch * 8 + 2 * k][cc] | ((uint32_t)tile[ch * 8 + 2 * k + 1][cc] << 16);
            *reinterpret_cast<u32x4*>(dstT + (int64_t)c * ldT + r) = v;
        }
    }
}

hipError_t launch_gather_transpose(const bf16_t* src, int C, const int32_t* idx, int R,
                                   const int32_t* r_dev, bf16_t* dst, bf16_t* dstT, int ldT,
                                   hipStream_t s) {
    if (R <= 0 || C <= 0) return hipSuccess;
    dim3 grid((ldT + TR_TILE - 1) / TR_TILE, (C + TR_TILE - 1) / TR_TILE), block(256);
    profile_mark_begin(KC_GATHER_ROWS, s);
    hipLaunchKernelGGL(gather_transpose_kernel, grid, block, 0, s, src, C, idx, R, r_dev, dst, dstT, ldT);
    profile_mark_end(KC_GATHER_ROWS, s);
    return hipGetLastError();
}

// ---- bit copy of skipped rows (out-of-place calls) ---------------------------------------
// A row t is copied unless a binary search finds it in the ascending list idx.
__global__ __launch_bounds__(ROW_THREADS) void passthrough_kernel(
    const u32x4* __restrict__ src, u32x4* __restrict__ dst, int64_t T, int64_t row_chunks,
    const int32_t* __restrict__ idx, int Rbound, const int32_t* __restrict__ r_dev) {
    const int R = effective_rows(Rbound, r_dev);
    const int lane = threadIdx.x & 63;
    const int64_t t = (int64_t)blockIdx.x * ROWS_PER_BLOCK + (threadIdx.x >> 6);
    if (t >= T) return;
    int lo = 0, hi = R;              // first position with idx[pos] >= t
    while (lo < hi) {
        int mid = (lo + hi) >> 1;
        if (idx[mid] < t) lo = mid + 1; else hi = mid;
    }
    if (lo < R && idx[lo] == t) return;   // retained: written by the scatter epilogue
    const u32x4* s = src + t * row_chunks;
    u32x4* d = dst + t * row_chunks;
    for (int64_t c = lane; c < row_chunks; c += 64) d[c] = s[c];
}

hipError_t launch_passthrough(const void* src, void* dst, int64_t T, int64_t row_bytes,
                              const int32_t* idx, int R, const int32_t* r_dev, hipStream_t s) {
    if (T <= 0 || row_bytes <= 0) return hipSuccess;
    dim3 grid((unsigned)((T + ROWS_PER_BLOCK - 1) / ROWS_PER_BLOCK)), block(ROW_THREADS);
    profile_mark_begin(KC_PASSTHROUGH, s);
    hipLaunchKernelGGL(passthrough_kernel, grid, block, 0, s, static_cast<const u32x4*>(src),
                       static_cast<u32x4*>(dst), T, row_bytes / 16, idx, R < 0 ? 0 : R, r_dev);
    profile_mark_end(KC_PASSTHROUGH, s);
    return hipGetLastError();
}

// ---- RMSNorm backward + residual gradient + scatter ----------------------------------------
// With xh = x * rstd and dxh = dxn * gain:
//   dx = rstd * (dxh - xh * mean_c(dxh * xh));  dX[idx[r]] = bf16(dY[r] + dx)
// dxn arrives as `splits` fp32 partial sums [z][r][c] (the split-K slabs of the
// dG*W_gate + dU*W_up GEMM), added here in z order.
// With GAIN_GRAD a workgroup walks a strip of GAIN_STRIP rows and also accumulates the
// gradient of the gain, dgain[c] = sum_r dxn[r][c] * x[r][c] * rstd[r], over its strip into
// gpart[strip][c]; gain_grad_reduce_kernel adds the strips in order (deterministic).
template <bool IN_REGS, bool GAIN_GRAD>
__global__ __launch_bounds__(ROW_THREADS) void rmsnorm_bwd_scatter_kernel(
    const float* __restrict__ part, PartialLayout pl, int Rbound, const int32_t* __restrict__ r_dev,
    int C, const bf16_t* __restrict__ xrows, const float* __restrict__ rstd_in,
    const bf16_t* __restrict__ gain, const bf16_t* __restrict__ dY,
    const int32_t* __restrict__ idx, bf16_t* dX, float* __restrict__ gpart) {
    __shared__ float red[4];
    const int R = effective_rows(Rbound, r_dev);
    const int tid = threadIdx.x;
    constexpr int STRIP = GAIN_GRAD ? GAIN_STRIP : 1;
    const int r_begin = blockIdx.x * STRIP;
    if (r_begin >= R) return;                 // the whole workgroup leaves together
    const int r_end = r_begin + STRIP < R ? r_begin + STRIP : R;
    const int chunks = C >> 3;
    const int64_t zstride = (int64_t)Rbound * C;
    const u32x4* gs = reinterpret_cast<const u32x4*>(gain);
    constexpr int MAXV = 2;                   // register-resident row: C <= 256 * 8 * 2 = 4096
    float gacc[IN_REGS ? MAXV : 1][8];
    if (IN_REGS && GAIN_GRAD) {
#pragma unroll
        for (int v = 0; v < MAXV; ++v)
#pragma unroll
            for (int j = 0; j < 8; ++j) gacc[v][j] = 0.0f;
    }
    float* gp = GAIN_GRAD ? gpart + (int64_t)blockIdx.x * C : nullptr;

    for (int r = r_begin; r < r_end; ++r) {
        const float rstd = rstd_in[r];
        const float* p = part + (int64_t)r * C;
        const u32x4* xs = reinterpret_cast<const u32x4*>(xrows + (int64_t)r * C);
        const int splits = partial_count(pl, R, r, 0);
        // d = dxn (sum of the split-K slabs)
        auto load_dxn = [&](int c, float* d) {
#pragma unroll
            for (int j = 0; j < 8; ++j) d[j] = 0.0f;
            for (int z = 0; z < splits; ++z) {
                f32x4 a = *reinterpret_cast<const f32x4*>(p + z * zstride + c * 8);
                f32x4 b = *reinterpret_cast<const f32x4*>(p + z * zstride + c * 8 + 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    d[j] += a[j];
                    d[4 + j] += b[j];
                }
            }
        };
        auto apply_gain = [&](int c, float* d) {
            if (gain != nullptr) {
                float g[8];
                unpack8(gs[c], g);
#pragma unroll
                for (int j = 0; j < 8; ++j) d[j] *= g[j];
            }
        };
        const u32x4* dys = reinterpret_cast<const u32x4*>(dY + (int64_t)r * C);
        u32x4* out = reinterpret_cast<u32x4*>(dX + (int64_t)idx[r] * C);
        auto emit = [&](int c, const float* d, const float* x, const u32x4& dyraw, float dot) {
            float gy[8], o[8];
            unpack8(dyraw, gy);
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = gy[j] + rstd * (d[j] - (x[j] * rstd) * dot);
            out[c] = pack8(o);
        };

        if (IN_REGS) {
            // the row (sum of the split-K slabs, x and dY) is read once and kept in registers
            float d[MAXV][8], x[MAXV][8];
            u32x4 dyraw[MAXV];
            float dot = 0.0f;
#pragma unroll
            for (int v = 0; v < MAXV; ++v) {
                int c = tid + ROW_THREADS * v;
                if (c < chunks) {
                    load_dxn(c, d[v]);
                    unpack8(xs[c], x[v]);
                    dyraw[v] = dys[c];
                    if (GAIN_GRAD) {
#pragma unroll
                        for (int j = 0; j < 8; ++j) gacc[v][j] += d[v][j] * (x[v][j] * rstd);
                    }
                    apply_gain(c, d[v]);
#pragma unroll
                    for (int j = 0; j < 8; ++j) dot += d[v][j] * (x[v][j] * rstd);
                }
            }
            dot = block_sum(dot, red) / (float)C;
#pragma unroll
            for (int v = 0; v < MAXV; ++v) {
                int c = tid + ROW_THREADS * v;
                if (c < chunks) emit(c, d[v], x[v], dyraw[v], dot);
            }
        } else {
            float dot = 0.0f;
            for (int c = tid; c < chunks; c += ROW_THREADS) {
                float d[8], x[8];
                load_dxn(c, d);
                unpack8(xs[c], x);
                if (GAIN_GRAD) {
                    // the strip's partial lives in global memory: each thread owns its chunks
                    f32x4* g0 = reinterpret_cast<f32x4*>(gp + c * 8);
                    f32x4 lo = {0.f, 0.f, 0.f, 0.f}, hi = lo;
                    if (r > r_begin) { lo = g0[0]; hi = g0[1]; }
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        lo[j] += d[j] * (x[j] * rstd);
                        hi[j] += d[4 + j] * (x[4 + j] * rstd);
                    }
                    g0[0] = lo; g0[1] = hi;
                }
                apply_gain(c, d);
#pragma unroll
                for (int j = 0; j < 8; ++j) dot += d[j] * (x[j] * rstd);
            }
            dot = block_sum(dot, red) / (float)C;
            for (int c = tid; c < chunks; c += ROW_THREADS) {
                float d[8], x[8];
                load_dxn(c, d);
                apply_gain(c, d);
                unpack8(xs[c], x);
                emit(c, d, x, dys[c], dot);
            }
        }
        if (STRIP > 1) __syncthreads();       // `red` is reused by the next row
    }
    if (IN_REGS && GAIN_GRAD) {
#pragma unroll
        for (int v = 0; v < MAXV; ++v) {
            int c = tid + ROW_THREADS * v;
            if (c < chunks) {
                f32x4* g0 = reinterpret_cast<f32x4*>(gp + c * 8);
                f32x4 lo = {gacc[v][0], gacc[v][1], gacc[v][2], gacc[v][3]};
                f32x4 hi = {gacc[v][4], gacc[v][5], gacc[v][6], gacc[v][7]};
                g0[0] = lo; g0[1] = hi;
            }
        }
    }
}

// dgain[c] (+)= sum over strips of gpart[strip][c]: eight interleaved partial sums per column,
// added in a fixed order (deterministic).  32 columns per workgroup.
__global__ __launch_bounds__(ROW_THREADS) void gain_grad_reduce_kernel(
    const float* __restrict__ gpart, int Rbound, const int32_t* __restrict__ r_dev, int C,
    float* __restrict__ dgain, int accumulate) {
    __shared__ float part8[8][32];
    const int R = effective_rows(Rbound, r_dev);
    const int nstrips = (R + GAIN_STRIP - 1) / GAIN_STRIP;
    const int cx = threadIdx.x & 31, sy = threadIdx.x >> 5;
    const int c = blockIdx.x * 32 + cx;
    float a0 = 0.0f, a1 = 0.0f;
    if (c < C) {
        int q = sy;
        for (; q + 8 < nstrips; q += 16) {             // two loads in flight per thread
            a0 += gpart[(int64_t)q * C + c];
            a1 += gpart[(int64_t)(q + 8) * C + c];
        }
        if (q < nstrips) a0 += gpart[(int64_t)q * C + c];
    }
    part8[sy][cx] = a0 + a1;
    __syncthreads();
    if (sy == 0 && c < C) {
        float v = 0.0f;
#pragma unroll
        for (int k = 0; k < 8; ++k) v += part8[k][cx];
        dgain[c] = accumulate ? dgain[c] + v : v;
    }
}

hipError_t launch_rmsnorm_bwd_scatter(const float* dxn_partial, PartialLayout pl, int R,
                                      const int32_t* r_dev, int C, const bf16_t* xrows,
                                      const float* rstd, const bf16_t* gain, const bf16_t* dY,
                                      const int32_t* idx, bf16_t* dX, float* gain_partial,
                                      float* dgain, int accumulate, hipStream_t s) {
    if (R <= 0) return hipSuccess;
    const bool gg = dgain != nullptr;
    dim3 grid(gg ? (R + GAIN_STRIP - 1) / GAIN_STRIP : R), block(ROW_THREADS);
    profile_mark_begin(KC_RMSNORM_BWD, s);
    if (C <= 4096) {
        if (gg)
            hipLaunchKernelGGL((rmsnorm_bwd_scatter_kernel<true, true>), grid, block, 0, s, dxn_partial,
                               pl, R, r_dev, C, xrows, rstd, gain, dY, idx, dX, gain_partial);
        else
            hipLaunchKernelGGL((rmsnorm_bwd_scatter_kernel<true, false>), grid, block, 0, s, dxn_partial,
                               pl, R, r_dev, C, xrows, rstd, gain, dY, idx, dX, gain_partial);
    } else {
        if (gg)
            hipLaunchKernelGGL((rmsnorm_bwd_scatter_kernel<false, true>), grid, block, 0, s, dxn_partial,
                               pl, R, r_dev, C, xrows, rstd, gain, dY, idx, dX, gain_partial);
        else
            hipLaunchKernelGGL((rmsnorm_bwd_scatter_kernel<false, false>), grid, block, 0, s, dxn_partial,
                               pl, R, r_dev, C, xrows, rstd, gain, dY, idx, dX, gain_partial);
    }
    hipError_t e = hipGetLastError();
    if (e == hipSuccess && gg) {
        hipLaunchKernelGGL(gain_grad_reduce_kernel, dim3((C + 31) / 32), block, 0, s, gain_partial, R,
                           r_dev, C, dgain, accumulate);
        e = hipGetLastError();
    }
    profile_mark_end(KC_RMSNORM_BWD, s);
    return e;
}

// ---- zero fill (a kernel, so that it can be captured in a HIP graph) -----------------------
__global__ __launch_bounds__(256) void fill_zero_kernel(u32x4* p, size_t chunks) {
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    size_t stride = (size_t)gridDim.x * 256;
    u32x4 z = {0u, 0u, 0u, 0u};
    for (; i < chunks; i += stride) p[i] = z;
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t s) {
    if (bytes == 0) return hipSuccess;
    size_t chunks = bytes / 16;     // callers pass multiples of 16
    size_t blocks = (chunks + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    profile_mark_begin(KC_FILL, s);
    hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, s,
                       static_cast<u32x4*>(p), chunks);
    profile_mark_end(KC_FILL, s);
    return hipGetLastError();
}

}  // namespace skipffn
