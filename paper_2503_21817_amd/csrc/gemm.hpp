// bf16 MFMA GEMM core for gfx950 with the fused epilogues of the Skip-FFN block.
//
// One workgroup = 512 threads = 8 wavefronts (2 per SIMD) computes a 256 x 256
// tile of C = A * B with fp32 accumulation, stepping K in slabs of 64.  Waves
// are arranged 2 (M) x 4 (N); each owns 128 x 64 = 4 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16 (128 accumulator registers).
//
// Operand layouts in global memory (all row-major, as PyTorch stores them):
//   "KC"  : [rows][K]   - the contraction index is contiguous
//   "MNC" : [K][rows]   - the M (or N) index is contiguous
// Both are staged through LDS with 16-byte loads/stores and no transposition:
// KC tiles are read back with ds_read_b128 (8 consecutive k per lane), MNC
// tiles with the transposing ds_read_b64_tr_b16 of gfx950, which hands each
// lane 4 consecutive k for its own column.  XOR swizzles keep both read
// patterns free of LDS bank conflicts.  LDS is double buffered (2 x 64 KB).
//
// Global loads are raw buffer loads: lanes outside the matrix (ragged M, K or N
// tails) read zeros, so no shape restriction beyond "dimensions are multiples
// of 8 elements where they are contiguous" is needed.
#pragma once

#include "common.hpp"

namespace skipffn {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int GEMM_THREADS = 512;
constexpr int TILE_BYTES = BM * BK * 2;           // 32 KB per operand per stage
constexpr int GEMM_LDS_BYTES = 4 * TILE_BYTES;    // A,B x 2 stages = 128 KB

enum EpiKind : int {
    EPI_SWIGLU = 0,        // B = {W_gate, W_up} interleaved per tile; out0=H, out1=G, out2=U (bf16)
    EPI_STORE = 1,         // out0 [M,N] bf16 or fp32, overwrite or accumulate
    EPI_PARTIAL = 2,       // fp32 partial[z][M][N]
    EPI_RESID_SCATTER = 3, // out0[idx[m]][n] = bf16(res[idx[m]][n] + acc)
    EPI_SWIGLU_BWD = 4     // acc = dH; e0=G, e1=U -> out0 = dG, out1 = dU (bf16)
};

struct GemmArgs {
    int M, N, K;                 // C is M x N; contraction length K (per pair)
    const int32_t* m_dev;        // optional device row count replacing M (M is then the bound)
    const int32_t* k_dev;        // optional device count replacing K
    const bf16_t* A0; const bf16_t* A1; int lda; uint32_t a_bytes;
    const bf16_t* B0; const bf16_t* B1; int ldb; uint32_t b_bytes;
    int pairs;                   // 1, or 2: K runs over (A0,B0) then (A1,B1)
    int splits;                  // split-K factor
    int tiles_m, tiles_n;
    void* out0; void* out1; void* out2; int ldo;
    const bf16_t* e0; const bf16_t* e1; int lde;
    const int32_t* idx;
    float* partial;              // [splits][M][N]
    int out_f32;                 // EPI_STORE: 1 = fp32 output
    int accumulate;              // EPI_STORE: 1 = +=
    int no_residual;             // EPI_RESID_SCATTER: 1 = do not add the residual
};

// ---- LDS addressing ----------------------------------------------------------
// KC tile: 256 rows x 64 k, 128 B per row, 16-byte chunk c stored at c ^ (row & 7)
__device__ __forceinline__ uint32_t kc_off(int row, int chunk) {
    return (uint32_t)(row * 128 + (((chunk) ^ (row & 7)) << 4));
}
// MNC tile: 64 k-rows x 256 columns, 512 B per k-row, 32-byte chunk c stored at c ^ (krow & 3)
__device__ __forceinline__ uint32_t mnc_off(int krow, int c32, int within) {
    return (uint32_t)(krow * 512 + (((c32) ^ (krow & 3)) << 5) + within);
}

__device__ __forceinline__ bf16x8 lds_frag_kc(const char* tile, int row_base, int s, int lane) {
    int row = row_base + (lane & 31);
    int chunk = 2 * s + (lane >> 5);
    u32x4 v = *reinterpret_cast<const u32x4*>(tile + kc_off(row, chunk));
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ bf16x8 lds_frag_mnc(const char* tile, int col_base, int s, int lane) {
    int b = lane >> 4, i = lane & 15;
    int krow = 16 * s + 8 * (b >> 1) + (i >> 2);
    int c32 = (col_base >> 4) + (b & 1);
    int within = 8 * (i & 3);
    typedef __attribute__((address_space(3))) short4v* lds_ptr;
    short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + mnc_off(krow, c32, within)));
    short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(tile + mnc_off(krow + 4, c32, within)));
    typedef __attribute__((ext_vector_type(8))) short short8v;
    short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

__device__ __forceinline__ float silu_f(float g) { return g / (1.0f + __expf(-g)); }

// blockIdx.x -> logical id such that each XCD (blocks are dealt round-robin to
// the 8 XCDs) walks a contiguous range of the logical order and so re-uses
// operand tiles in its own L2.
__device__ __forceinline__ int xcd_remap(int b, int nb) {
    int xcd = b & 7, j = b >> 3;
    int q = nb >> 3, rem = nb & 7;
    int start = xcd * q + (xcd < rem ? xcd : rem);
    return start + j;
}

template <bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs P) {
    extern __shared__ __align__(16) char smem[];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wm = wave >> 2;      // 0..1
    const int wn = wave & 3;       // 0..3

    // ---- which tile / split --------------------------------------------------
    const int nb = gridDim.x;
    int L = xcd_remap(blockIdx.x, nb);
    const int tm = L % P.tiles_m;
    L /= P.tiles_m;
    const int tn = L % P.tiles_n;
    const int z = L / P.tiles_n;

    const int Meff = effective_rows(P.M, P.m_dev);
    const int Keff = effective_rows(P.K, P.k_dev);
    const int m0 = tm * BM;
    const int n0 = (EPI == EPI_SWIGLU) ? tn * (BN / 2) : tn * BN;
    if (m0 >= Meff) return;    // whole block leaves together: no barrier was reached yet

    const int ktiles_pair = (Keff + BK - 1) / BK;
    const int ktotal = ktiles_pair * P.pairs;
    const int per_split = (ktotal + P.splits - 1) / P.splits;
    const int kt_begin = z * per_split;
    int kt_end = kt_begin + per_split;
    if (kt_end > ktotal) kt_end = ktotal;

    __amdgpu_buffer_rsrc_t rA0 = make_rsrc(P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rA1 = make_rsrc(P.A1 ? P.A1 : P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rB0 = make_rsrc(P.B0, P.b_bytes);
    __amdgpu_buffer_rsrc_t rB1 = make_rsrc(P.B1 ? P.B1 : P.B0, P.b_bytes);

    // ---- per-thread global/LDS staging addresses -----------------------------
    // KC : 4 chunks per thread: row = t/8 + 64 i, 16-byte chunk c = t%8
    // MNC: 4 chunks per thread: krow = t/32 + 16 i, 16-byte chunk c = t%32
    uint32_t a_goff[4], b_goff[4];     // byte offset of the chunk at k-tile 0 (or OOB)
    uint32_t a_loff[4], b_loff[4];     // LDS byte offset inside the operand tile
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        if (A_KC) {
            int row = (t >> 3) + 64 * i, c = t & 7;
            int gr = m0 + row;
            a_goff[i] = gr < Meff ? (uint32_t)(((int64_t)gr * P.lda + c * 8) * 2) : kOobOffset;
            a_loff[i] = kc_off(row, c);
        } else {
            int krow = (t >> 5) + 16 * i, c = t & 31;
            int gc = m0 + c * 8;
            a_goff[i] = gc < Meff ? (uint32_t)(((int64_t)krow * P.lda + gc) * 2) : kOobOffset;
            a_loff[i] = mnc_off(krow, c >> 1, (c & 1) * 16);
        }
        if (B_KC) {
            int row = (t >> 3) + 64 * i, c = t & 7;
            // SWIGLU: tile rows 0..127 are W_gate rows, 128..255 the same rows of W_up
            int gr = (EPI == EPI_SWIGLU) ? n0 + (row & 127) : n0 + row;
            b_goff[i] = gr < P.N ? (uint32_t)(((int64_t)gr * P.ldb + c * 8) * 2) : kOobOffset;
            b_loff[i] = kc_off(row, c);
        } else {
            int krow = (t >> 5) + 16 * i, c = t & 31;
            int gc = n0 + c * 8;
            b_goff[i] = gc < P.N ? (uint32_t)(((int64_t)krow * P.ldb + gc) * 2) : kOobOffset;
            b_loff[i] = mnc_off(krow, c >> 1, (c & 1) * 16);
        }
    }
    const int a_kchunk = A_KC ? (t & 7) * 8 : 0;       // k offset of this thread's chunk (KC)
    const int b_kchunk = B_KC ? (t & 7) * 8 : 0;
    const int a_krow = A_KC ? 0 : (t >> 5);            // k row of chunk i = a_krow + 16 i (MNC)
    const int b_krow = B_KC ? 0 : (t >> 5);

    u32x4 ra[4], rb[4];
    auto gload = [&](int kt) {
        const int pair = kt >= ktiles_pair ? 1 : 0;
        const int kg = (kt - pair * ktiles_pair) * BK;  // k offset inside the pair
        __amdgpu_buffer_rsrc_t ra_src = pair ? rA1 : rA0;
        __amdgpu_buffer_rsrc_t rb_src = pair ? rB1 : rB0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t off;
            if (A_KC) {
                off = (kg + a_kchunk) < Keff ? a_goff[i] + (uint32_t)kg * 2u : kOobOffset;
            } else {
                off = (kg + a_krow + 16 * i) < Keff
                          ? a_goff[i] + (uint32_t)(((int64_t)kg * P.lda) * 2) : kOobOffset;
            }
            if (a_goff[i] == kOobOffset) off = kOobOffset;
            ra[i] = buf_load16(ra_src, off);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t off;
            if (B_KC) {
                off = (kg + b_kchunk) < Keff ? b_goff[i] + (uint32_t)kg * 2u : kOobOffset;
            } else {
                off = (kg + b_krow + 16 * i) < Keff
                          ? b_goff[i] + (uint32_t)(((int64_t)kg * P.ldb) * 2) : kOobOffset;
            }
            if (b_goff[i] == kOobOffset) off = kOobOffset;
            if (EPI == EPI_SWIGLU)   // chunks i = 2, 3 are tile rows 128..255 (compile-time choice)
                rb[i] = buf_load16(i >= 2 ? rB1 : rB0, off);
            else
                rb[i] = buf_load16(rb_src, off);
        }
    };
    auto lstore = [&](int stage) {
        char* sa = smem + stage * 2 * TILE_BYTES;
        char* sb = sa + TILE_BYTES;
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(sa + a_loff[i]) = ra[i];
#pragma unroll
        for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(sb + b_loff[i]) = rb[i];
    };

    f32x16 acc[4][2];
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    // rows of the B tile read by this wave's two n-tiles
    int b_rowbase[2];
    if (EPI == EPI_SWIGLU) {
        b_rowbase[0] = wn * 32;          // gate columns
        b_rowbase[1] = 128 + wn * 32;    // the same columns of up
    } else {
        b_rowbase[0] = wn * 64;
        b_rowbase[1] = wn * 64 + 32;
    }

    if (kt_begin < kt_end) {
        gload(kt_begin);
        lstore(0);
        __syncthreads();
        for (int kt = kt_begin; kt < kt_end; ++kt) {
            const int stage = (kt - kt_begin) & 1;
            const char* sa = smem + stage * 2 * TILE_BYTES;
            const char* sb = sa + TILE_BYTES;
            const bool more = (kt + 1) < kt_end;
            if (more) gload(kt + 1);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                bf16x8 af[4], bfr[2];
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
                    af[mt] = A_KC ? lds_frag_kc(sa, wm * 128 + mt * 32, s, lane)
                                  : lds_frag_mnc(sa, wm * 128 + mt * 32, s, lane);
#pragma unroll
                for (int nt = 0; nt < 2; ++nt)
                    bfr[nt] = B_KC ? lds_frag_kc(sb, b_rowbase[nt], s, lane)
                                   : lds_frag_mnc(sb, b_rowbase[nt], s, lane);
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            af[mt], bfr[nt], acc[mt][nt], 0, 0, 0);
            }
            if (more) lstore(stage ^ 1);
            __syncthreads();
        }
    }

    // ---- epilogue --------------------------------------------------------------
    // acc[mt][nt][r] is C[row][col] with
    //   row = m0 + wm*128 + mt*32 + 8*(r/4) + 4*(lane/32) + r%4
    //   col = (tile column base) + lane%32
    const int lrow = wm * 128 + 4 * (lane >> 5);
    const int lcol = lane & 31;

    if (EPI == EPI_SWIGLU) {
        bf16_t* H = static_cast<bf16_t*>(P.out0);
        bf16_t* G = static_cast<bf16_t*>(P.out1);
        bf16_t* U = static_cast<bf16_t*>(P.out2);
        const int col = n0 + wn * 32 + lcol;
        if (col < P.N) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    int row = m0 + lrow + mt * 32 + 8 * (r >> 2) + (r & 3);
                    if (row < Meff) {
                        float g = acc[mt][0][r], u = acc[mt][1][r];
                        int64_t o = (int64_t)row * P.ldo + col;
                        H[o] = f32_to_bf16(silu_f(g) * u);
                        if (G != nullptr) {
                            G[o] = f32_to_bf16(g);
                            U[o] = f32_to_bf16(u);
                        }
                    }
                }
        }
        return;
    }

#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
        for (int nt = 0; nt < 2; ++nt) {
            const int col = n0 + wn * 64 + nt * 32 + lcol;
            if (col >= P.N) continue;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                int row = m0 + lrow + mt * 32 + 8 * (r >> 2) + (r & 3);
                if (row >= Meff) continue;
                float v = acc[mt][nt][r];
                if (EPI == EPI_STORE) {
                    int64_t o = (int64_t)row * P.ldo + col;
                    if (P.out_f32) {
                        float* O = static_cast<float*>(P.out0);
                        O[o] = P.accumulate ? O[o] + v : v;
                    } else {
                        bf16_t* O = static_cast<bf16_t*>(P.out0);
                        O[o] = f32_to_bf16(P.accumulate ? bf16_to_f32(O[o]) + v : v);
                    }
                } else if (EPI == EPI_PARTIAL) {
                    P.partial[((int64_t)z * P.M + row) * P.N + col] = v;
                } else if (EPI == EPI_RESID_SCATTER) {
                    int64_t o = (int64_t)P.idx[row] * P.ldo + col;
                    bf16_t* O = static_cast<bf16_t*>(P.out0);
                    float res = P.no_residual ? 0.0f : bf16_to_f32(P.e0[o]);
                    O[o] = f32_to_bf16(res + v);
                } else if (EPI == EPI_SWIGLU_BWD) {
                    int64_t o = (int64_t)row * P.ldo + col;
                    float g = bf16_to_f32(P.e0[o]), u = bf16_to_f32(P.e1[o]);
                    float sg = 1.0f / (1.0f + __expf(-g));
                    float dg = v * u * sg * (1.0f + g * (1.0f - sg));
                    float du = v * g * sg;
                    static_cast<bf16_t*>(P.out0)[o] = f32_to_bf16(dg);
                    static_cast<bf16_t*>(P.out1)[o] = f32_to_bf16(du);
                }
            }
        }
}

}  // namespace skipffn
