// bf16 MFMA GEMM core for gfx950 with the fused epilogues of the Skip-FFN block.
//
// One workgroup = 512 threads = 8 wavefronts (2 per SIMD) computes a 256 x 256
// tile of C = A * B with fp32 accumulation, stepping K in slabs of 32.  Waves
// are arranged 2 (M) x 4 (N); each owns 128 x 64 = 4 x 2 MFMA tiles of
// v_mfma_f32_32x32x16_bf16 (128 accumulator registers).
//
// Operand layouts in global memory (all row-major, as PyTorch stores them):
//   "KC"  : [rows][K]   - the contraction index is contiguous
//   "MNC" : [K][rows]   - the M (or N) index is contiguous
// Both are staged through LDS by 16-byte direct-to-LDS buffer loads (no VGPR
// staging, no ds_write) and with no transposition: KC tiles are read back with
// ds_read_b128 (8 consecutive k per lane), MNC tiles with the transposing
// ds_read_b64_tr_b16 of gfx950, which hands each lane 4 consecutive k for its own
// column.  XOR swizzles, applied on the global-address side of the direct loads,
// keep both read patterns free of LDS bank conflicts.
//
// LDS holds a ring of NSTAGE = 5 slabs (5 x 32 KB = all 160 KB of the CU), up to
// four of them in flight from memory, so memory latency of about three slab times
// is covered.  The two waves of each SIMD alternate between a memory phase and a
// compute phase half a slab apart (see the main loop), which keeps the matrix
// pipe fed while fragments are read and loads are issued.
//
// Global loads are raw buffer loads: lanes outside the matrix (ragged M, K or N
// tails) read zeros, so no shape restriction beyond "dimensions are multiples
// of 8 elements where they are contiguous" is needed.
#pragma once

#include "common.hpp"

namespace skipffn {

constexpr int BM = 256, BN = 256, BK = 32;
constexpr int GEMM_THREADS = 512;
constexpr int NSTAGE = 5;
constexpr int OPER_BYTES = BM * BK * 2;             // 16 KB per operand per stage
constexpr int STAGE_BYTES = 2 * OPER_BYTES;         // 32 KB
constexpr int GEMM_LDS_BYTES = NSTAGE * STAGE_BYTES;  // 160 KB
constexpr int PANEL_M = 8;                          // tile-order panel width (L2 locality)

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
// The LDS of gfx950 serves 256 B per clock (64 banks of 4 B): a 16-byte read is
// processed 16 lanes at a time, an 8-byte read 32 lanes at a time, and is free of
// bank conflicts when those lanes cover 256 distinct bytes modulo 256.
// KC tile: 256 rows x 32 k, 64 B per row, 16-byte chunk c stored at c ^ ((row/4) & 3):
// sixteen consecutive rows reading the same logical chunk touch every bank once.
__device__ __forceinline__ uint32_t kc_off(int row, int chunk) {
    return (uint32_t)(row * 64 + (((chunk) ^ ((row >> 2) & 3)) << 4));
}
// MNC tile: 32 k-rows x 256 columns, 512 B per k-row, 32-byte chunk c stored at
// c ^ (2 * (krow & 3)): the 4 k-rows x 64 B that 32 lanes of a transposing read
// touch land in 8 distinct 32-byte slots of the 256-byte bank window.
__device__ __forceinline__ uint32_t mnc_off(int krow, int c32, int within) {
    return (uint32_t)(krow * 512 + (((c32) ^ ((krow & 3) << 1)) << 5) + within);
}

// s = 0, 1: the two k-steps of 16 inside a slab
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

__device__ __forceinline__ float sigmoid_f(float g) {
    return __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at their maxima), gfx9 encoding
#define SKIPFFN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// s_waitcnt lgkmcnt(0) only
#define SKIPFFN_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)

// blockIdx.x -> (tile m, tile n, split).  Workgroups are dealt round-robin to the
// 8 XCDs, each with its own L2: the remap gives every XCD a contiguous range of a
// logical order in which 32 consecutive tiles form a PANEL_M x (32 / PANEL_M)
// rectangle, so the tiles an XCD runs at one time share A and B slabs in its L2.
__device__ __forceinline__ void tile_of_block(int b, int nb, int tiles_m, int tiles_n,
                                              int& tm, int& tn, int& z) {
    int xcd = b & 7, j = b >> 3;
    int q = nb >> 3, rem = nb & 7;
    int L = xcd * q + (xcd < rem ? xcd : rem) + j;
    const int per_split = tiles_m * tiles_n;
    z = L / per_split;
    L -= z * per_split;
    const int panel_tiles = PANEL_M * tiles_n;
    const int p = L / panel_tiles;
    const int in_panel = L - p * panel_tiles;
    int pm = tiles_m - p * PANEL_M;
    pm = pm < PANEL_M ? pm : PANEL_M;          // width of this (possibly last, narrower) panel
    tn = in_panel / pm;
    tm = p * PANEL_M + (in_panel - tn * pm);
}

template <bool A_KC, bool B_KC, int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs P) {
    extern __shared__ __align__(16) char smem[];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 2;      // 0..1
    const int wn = wave & 3;       // 0..3

    int tm, tn, z;
    tile_of_block(blockIdx.x, gridDim.x, P.tiles_m, P.tiles_n, tm, tn, z);

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
    const int nk = kt_end > kt_begin ? kt_end - kt_begin : 0;

    __amdgpu_buffer_rsrc_t rA0 = make_rsrc(P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rA1 = make_rsrc(P.A1 ? P.A1 : P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rB0 = make_rsrc(P.B0, P.b_bytes);
    __amdgpu_buffer_rsrc_t rB1 = make_rsrc(P.B1 ? P.B1 : P.B0, P.b_bytes);

    // ---- global -> LDS staging (direct-to-LDS buffer loads) ----------------------
    // A wave-wide 16-byte load deposits lane l at LDS base + 16*l, so each load
    // fills one contiguous 1 KB region q of the operand slab (16 regions; wave w
    // owns regions 2w, 2w+1).  The swizzle is applied on the global side: a lane
    // fetches the chunk whose swizzled home is its own 16-byte slot.
    //   KC : region q = rows 16q..16q+15;  lane -> row 16q + l/4, chunk (l%4) ^ ((l/16)%4)
    //   MNC: region q = k-rows 2q, 2q+1;   lane -> krow 2q + l/32, slot p = l%32:
    //        32-byte chunk (p/2) ^ (2 * (krow & 3)), half p & 1
    uint32_t a_goff[2], b_goff[2];     // byte offset of the lane's chunk at slab 0 (or OOB)
    int a_kk[2], b_kk[2];              // k index (inside the slab) the validity test uses
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int q = wave * 2 + i;
        if (A_KC) {
            int row = 16 * q + (lane >> 2), c = (lane & 3) ^ ((lane >> 4) & 3);
            int gr = m0 + row;
            a_goff[i] = gr < Meff ? (uint32_t)(((int64_t)gr * P.lda + c * 8) * 2) : kOobOffset;
            a_kk[i] = c * 8;
        } else {
            int krow = 2 * q + (lane >> 5), pslot = lane & 31;
            int c16 = 2 * ((pslot >> 1) ^ ((krow & 3) << 1)) + (pslot & 1);
            int gc = m0 + c16 * 8;
            a_goff[i] = gc < Meff ? (uint32_t)(((int64_t)krow * P.lda + gc) * 2) : kOobOffset;
            a_kk[i] = krow;
        }
        if (B_KC) {
            int row = 16 * q + (lane >> 2), c = (lane & 3) ^ ((lane >> 4) & 3);
            // SWIGLU: tile rows 0..127 are W_gate rows, 128..255 the same rows of W_up
            int gr = (EPI == EPI_SWIGLU) ? n0 + (row & 127) : n0 + row;
            b_goff[i] = gr < P.N ? (uint32_t)(((int64_t)gr * P.ldb + c * 8) * 2) : kOobOffset;
            b_kk[i] = c * 8;
        } else {
            int krow = 2 * q + (lane >> 5), pslot = lane & 31;
            int c16 = 2 * ((pslot >> 1) ^ ((krow & 3) << 1)) + (pslot & 1);
            int gc = n0 + c16 * 8;
            b_goff[i] = gc < P.N ? (uint32_t)(((int64_t)krow * P.ldb + gc) * 2) : kOobOffset;
            b_kk[i] = krow;
        }
    }
    typedef __attribute__((address_space(3))) void* lds_void_ptr;
    // issue the 4 loads of this wave for slab j (0-based inside this block's K range)
    auto gload = [&](int j) {
        const int kt = kt_begin + j;
        const int pair = kt >= ktiles_pair ? 1 : 0;
        const int kg = (kt - pair * ktiles_pair) * BK;  // k offset inside the pair
        __amdgpu_buffer_rsrc_t ra_src = pair ? rA1 : rA0;
        __amdgpu_buffer_rsrc_t rb_src = pair ? rB1 : rB0;
        if (EPI == EPI_SWIGLU) rb_src = wave >= 4 ? rB1 : rB0;   // regions 8.. = rows 128..
        char* sa = smem + (j % NSTAGE) * STAGE_BYTES + wave * 2048;
        char* sb = sa + OPER_BYTES;
        const uint32_t a_step = A_KC ? (uint32_t)kg * 2u : (uint32_t)(((int64_t)kg * P.lda) * 2);
        const uint32_t b_step = B_KC ? (uint32_t)kg * 2u : (uint32_t)(((int64_t)kg * P.ldb) * 2);
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            uint32_t off = (a_goff[i] != kOobOffset && (kg + a_kk[i]) < Keff) ? a_goff[i] + a_step
                                                                              : kOobOffset;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(ra_src, (lds_void_ptr)(sa + i * 1024), 16,
                                                     (int)off, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            uint32_t off = (b_goff[i] != kOobOffset && (kg + b_kk[i]) < Keff) ? b_goff[i] + b_step
                                                                              : kOobOffset;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rb_src, (lds_void_ptr)(sb + i * 1024), 16,
                                                     (int)off, 0, 0, 0);
        }
    };
    // wait until at most `newer` slabs issued after the wanted one are still in flight
    auto wait_slab = [&](int newer) {
        if (newer >= 3) SKIPFFN_WAIT_VMCNT(12);
        else if (newer == 2) SKIPFFN_WAIT_VMCNT(8);
        else if (newer == 1) SKIPFFN_WAIT_VMCNT(4);
        else SKIPFFN_WAIT_VMCNT(0);
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

    if (nk > 0) {
        // Ping-pong schedule.  The two waves that share a SIMD (wave w and w + 4, i.e.
        // the two row groups wm = 0, 1) run half a slab apart: while one issues its
        // 16 MFMAs of slab j ("compute phase"), the other reads the fragments of its
        // next slab from LDS, issues its share of the global loads and waits for
        // them ("memory phase").  Phases are delimited by workgroup barriers; group 1
        // takes one extra barrier before the loop and group 0 one after it, so the
        // groups stay exactly one phase apart and every wave executes the same number
        // of barriers.  The matrix pipe of each SIMD always has one wave in its
        // compute phase.
        bf16x8 af[2][4], bfr[2][2];
        auto load_frags = [&](int j, int s) {
            const char* sa = smem + (j % NSTAGE) * STAGE_BYTES;
            const char* sb = sa + OPER_BYTES;
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
                af[s][mt] = A_KC ? lds_frag_kc(sa, wm * 128 + mt * 32, s, lane)
                                 : lds_frag_mnc(sa, wm * 128 + mt * 32, s, lane);
#pragma unroll
            for (int nt = 0; nt < 2; ++nt)
                bfr[s][nt] = B_KC ? lds_frag_kc(sb, b_rowbase[nt], s, lane)
                                  : lds_frag_mnc(sb, b_rowbase[nt], s, lane);
        };

        // prologue: slabs 0 .. NSTAGE-2 in flight, slab 0 landed and visible
#pragma unroll
        for (int p = 0; p < NSTAGE - 1; ++p)
            if (p < nk) gload(p);
        wait_slab(nk - 1 < NSTAGE - 2 ? nk - 1 : NSTAGE - 2);
        __builtin_amdgcn_s_barrier();
        if (wm == 1) __builtin_amdgcn_s_barrier();       // group 1 starts one phase later

        for (int j = 0; j < nk; ++j) {
            // ---- memory phase of slab j.  Slab j is visible (prologue, or the waits of
            // both groups in their memory phase j-1 followed by a barrier); the stage of
            // slab j-1 has been read by both groups and can be refilled.
            load_frags(j, 0);
            load_frags(j, 1);
            if (j + NSTAGE - 1 < nk) gload(j + NSTAGE - 1);
            if (j + 1 < nk) {
                const int newer = nk - (j + 2);           // slabs issued after j+1
                wait_slab(newer < NSTAGE - 2 ? newer : NSTAGE - 2);
            }
            SKIPFFN_WAIT_LGKMCNT0();                       // fragments are in registers
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            // ---- compute phase of slab j
#pragma unroll
            for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
                for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                    for (int nt = 0; nt < 2; ++nt)
                        acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            af[s2][mt], bfr[s2][nt], acc[mt][nt], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        }
        if (wm == 0) __builtin_amdgcn_s_barrier();       // balances group 1's extra barrier
    }

    // ---- epilogue --------------------------------------------------------------
    // acc[mt][nt][r] is C[row][col] with
    //   row = m0 + wm*128 + mt*32 + 8*(r/4) + 4*(lane/32) + r%4
    //   col = (tile column base) + lane%32
    const int lrow = m0 + wm * 128 + 4 * (lane >> 5);
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
                    int row = lrow + mt * 32 + 8 * (r >> 2) + (r & 3);
                    if (row < Meff) {
                        float g = acc[mt][0][r], u = acc[mt][1][r];
                        uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
                        H[o] = f32_to_bf16(g * sigmoid_f(g) * u);
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
                int row = lrow + mt * 32 + 8 * (r >> 2) + (r & 3);
                if (row >= Meff) continue;
                float v = acc[mt][nt][r];
                if (EPI == EPI_STORE) {
                    uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
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
                    uint32_t o = (uint32_t)P.idx[row] * (uint32_t)P.ldo + (uint32_t)col;
                    bf16_t* O = static_cast<bf16_t*>(P.out0);
                    float res = P.no_residual ? 0.0f : bf16_to_f32(P.e0[o]);
                    O[o] = f32_to_bf16(res + v);
                } else if (EPI == EPI_SWIGLU_BWD) {
                    uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
                    float g = bf16_to_f32(P.e0[o]), u = bf16_to_f32(P.e1[o]);
                    float sg = sigmoid_f(g);
                    float dg = v * u * sg * (1.0f + g * (1.0f - sg));
                    float du = v * g * sg;
                    static_cast<bf16_t*>(P.out0)[o] = f32_to_bf16(dg);
                    static_cast<bf16_t*>(P.out1)[o] = f32_to_bf16(du);
                }
            }
        }
}

}  // namespace skipffn
