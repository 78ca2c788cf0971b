// bf16 MFMA GEMM core for gfx950 with the fused epilogues of the Skip-FFN block.
//
// One workgroup = 512 threads = 8 wavefronts (2 per SIMD) computes a 256 x 256
// tile of C = A * B with fp32 accumulation, stepping K in slabs of 64.  Waves
// are arranged 2 (M) x 4 (N); each owns 128 x 64 = 8 x 4 MFMA tiles of
// v_mfma_f32_16x16x32_bf16 (128 accumulator registers).  The chip runs these loops at
// its power limit, and the 16x16x32 form spends less energy per FLOP than 32x32x16 (half
// the accumulator traffic): a register-only loop of it sustains 15-19 % more FLOP/s.
//
// Operand layouts in global memory (all row-major, as PyTorch stores them):
//   "KC"  : [rows][K]   - the contraction index is contiguous
//   "MNC" : [K][rows]   - the M (or N) index is contiguous
// Both are staged through LDS by 16-byte direct-to-LDS buffer loads (no VGPR
// staging, no ds_write) and with no transposition: KC tiles are read back with
// ds_read_b128 (8 consecutive k per lane), MNC tiles with the transposing
// ds_read_b64_tr_b16 of gfx950, which hands each lane 4 consecutive k for its own
// column (two of them make the 8 consecutive k of an MFMA operand register set).  XOR swizzles, applied on the global-address side of the direct loads,
// keep both read patterns free of LDS bank conflicts.
//
// LDS (160 KB) holds a ring of 2 A slabs and 3 B slabs of 256 x 64 (32 KB each):
// B is the operand that streams from HBM in every GEMM of the block (weights, or
// the long activation matrix), so it is fetched two slabs ahead, A one slab ahead.
// A slab row of a KC operand is one full 128-byte line, which keeps the address
// unit at one line per 8 lanes.  The two waves of each SIMD alternate between a
// memory phase and a compute phase half a slab apart (see the main loop), which
// keeps the matrix pipe fed while fragments are read and loads are issued.
//
// Global loads are raw buffer loads: lanes outside the matrix (ragged M, K or N
// tails) read zeros, so no shape restriction beyond "dimensions are multiples
// of 8 elements where they are contiguous" is needed.
#pragma once

#include <utility>

#include "common.hpp"
#include "layout.hpp"
#include "streamk.hpp"

namespace skipffn {

constexpr int GEMM_THREADS = 512;
constexpr int NSTAGE_A = 2, NSTAGE_B = 3;
constexpr int OPER_BYTES = BM * BK * 2;             // 32 KB per operand slab
constexpr int LDS_B_BASE = NSTAGE_A * OPER_BYTES;
constexpr int GEMM_LDS_BYTES = (NSTAGE_A + NSTAGE_B) * OPER_BYTES;  // 160 KB
constexpr int EPI_ROWS = 32;                         // rows of C staged per epilogue pass and row group
constexpr int PANEL_M = 8;                          // tile-order panel width (L2 locality)

enum EpiKind : int {
    EPI_SWIGLU = 0,        // B = {W_gate, W_up} interleaved per tile; out0=H, out1=G, out2=U (bf16)
    EPI_STORE = 1,         // out0 [M,N] bf16 or fp32, overwrite or accumulate
    EPI_PARTIAL = 2,       // fp32 partial[z][M][N]
    EPI_RESID_SCATTER = 3, // out0[idx[m]][n] = bf16(res[idx[m]][n] + acc)
    EPI_SWIGLU_BWD = 4,    // acc = dH; e0=G, e1=U -> out0 = dG, out1 = dU (bf16)
    EPI_PARTIAL_GU = 6     // B as for EPI_SWIGLU, fp32 partial[z][M][tiles_n * 256]: tile tn owns columns
                           // tn*256 .. +127 (gate) and +128 .. +255 (up); the SwiGLU is applied by the reducing kernel
};

struct GemmArgs {
    int M, N, K;                 // C is M x N; contraction length K (per pair)
    const int32_t* m_dev;        // optional device row count replacing M (M is then the bound)
    const int32_t* k_dev;        // optional device count replacing K
    const bf16_t* A0; const bf16_t* A1; int lda; uint32_t a_bytes;
    const bf16_t* B0; const bf16_t* B1; int ldb; uint32_t b_bytes;
    int pairs;                   // 1, or 2: K runs over (A0,B0) then (A1,B1)
    int splits;                  // split-K factor
    int batch;                   // 1, or 2 independent problems: (A0 -> out0), (A1 -> out1) sharing B.  pairs == 1
    int tiles_m, tiles_n;
    void* out0; void* out1; void* out2; int ldo;
    void* outT0; void* outT1; int ldt;   // SwiGLU epilogues: transposed copies [N][ldt] of out0 (H^T), or of out0 and
                                         // out1 (dG^T, dU^T); ldt a multiple of 8 >= the row bound; null = none
    const bf16_t* e0; const bf16_t* e1; int lde;
    const int32_t* idx;
    float* partial;              // [splits][M][N]
    int out_f32;                 // EPI_STORE: 1 = fp32 output
    int accumulate;              // EPI_STORE: 1 = +=
    int no_residual;             // EPI_RESID_SCATTER: 1 = do not add the residual
    int narrow;                  // host side: 1 = launch the 128-row tile variant (tiles_m counts 128-row tiles)
    int tail_narrow;             // 1 = the rows past tiles_m * 256 (at most 128 of them) form one extra row of
                                 // 128-row tiles, run by the last tiles_n workgroups of the grid
};

// Row offsets of up to SEG_TABLE_MAX token sets, passed by value in the kernel arguments
// (set i = rows [off[i], off[i+1]) of a token list).
constexpr int SEG_TABLE_MAX = 64;
struct SegTable { int count; int off[SEG_TABLE_MAX + 1]; };

// ---- LDS addressing ----------------------------------------------------------
// The LDS of gfx950 serves 256 B per clock (64 banks of 4 B): a 16-byte read is
// processed 16 lanes at a time, an 8-byte read 32 lanes at a time, and is free of
// bank conflicts when those lanes cover 256 distinct bytes modulo 256.
// KC tile: 256 rows x 64 k, 128 B per row, 16-byte chunk c stored at c ^ ((row/2) & 7):
// sixteen consecutive rows reading the same logical chunk touch every bank once.
__device__ __forceinline__ uint32_t kc_off(int row, int chunk) {
    return (uint32_t)(row * 128 + (((chunk) ^ ((row >> 1) & 7)) << 4));
}
// MNC tile: 64 k-rows x 256 columns, 512 B per k-row, 32-byte chunk c stored at
// c ^ mnc_swz(krow).  The 32 lanes a transposing read processes at a time are two groups of
// 16, each touching 4 consecutive k-rows x 32 B of the same logical chunk, the groups 8 k-rows
// apart: bits 0-1 and bit 3 of the k-row put those eight pieces into the eight distinct
// 32-byte slots of the 256-byte bank window.
__device__ __forceinline__ int mnc_swz(int krow) { return ((krow & 3) << 1) | ((krow >> 3) & 1); }
__device__ __forceinline__ uint32_t mnc_off(int krow, int c32, int within) {
    return (uint32_t)(krow * 512 + (((c32) ^ mnc_swz(krow)) << 5) + within);
}

// One operand register set of v_mfma_f32_16x16x32_bf16: lane l holds row (or column) l % 16 of
// the 16-row fragment and the 8 consecutive k starting at 8 * (l / 16).  With ks = 0, 1 the two
// k-steps of 32 inside a slab, a KC fragment is the 16 bytes at kc_off(row_base + l % 16,
// 4 * ks + l / 16); an MNC fragment two transposing reads at mnc_off(32 * ks + 8 * (l / 16) +
// (l % 16) / 4 {+ 4}, col_base / 16, 8 * (l % 4)).  Fragments 16 rows (columns) apart differ by a
// constant in the KC tile (+2048 bytes) and by an XOR of bits 5-6 in the MNC tile; the two k-steps
// differ by a per-lane amount in the KC tile (the swizzle) and by +16384 bytes in the MNC tile.

// The fragment reads of the main loop are issued through inline assembly, with the address
// split into one per-lane register and an immediate offset.  Two reasons: while a wave issues
// v_mfma_f32_16x16x32 back to back, every vector ALU instruction of the other wave on its SIMD
// takes about twice as long to issue (measured: 48 dependent VALU operations 264 cycles next to
// an idle wave, 343 next to 32x32x16 MFMAs, 478 next to 16x16x32 MFMAs; LDS reads and buffer
// loads are not slowed), so a memory phase must spend as few VALU instructions on addresses as
// possible; and for the builtin form of the transposing read the compiler cannot tell that it
// does not alias the direct-to-LDS loads in flight and puts s_waitcnt vmcnt(0) in front of it,
// which would serialise the whole load pipeline.  The assembly form is invisible to the
// compiler's wait-count insertion, so the CALLER must wait for lgkmcnt(0) before the returned
// registers are consumed (the main loop does, at the end of every memory phase).
template <int IMM>
__device__ __forceinline__ bf16x8 ds_read_b128_imm(uint32_t lds_addr) {
    static_assert(IMM >= 0 && IMM < 65536, "16-bit offset field");
    u32x4 v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(IMM));
    return __builtin_bit_cast(bf16x8, v);
}
// A group of 16 lanes addresses a 4 (k-rows) x 16 (columns) block, lane i the 8 bytes at k-row
// i / 4, columns 4 * (i % 4) .. +3, and receives column i of it: 4 consecutive k.
template <int IMM>
__device__ __forceinline__ u32x2 ds_read_tr16_b64_imm(uint32_t lds_addr) {
    static_assert(IMM >= 0 && IMM < 65536, "16-bit offset field");
    u32x2 v;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(lds_addr), "n"(IMM));
    return v;
}
__device__ __forceinline__ uint32_t lds_addr_of(const char* p) {
    typedef __attribute__((address_space(3))) const char* lds_cptr;
    return (uint32_t)(uintptr_t)(lds_cptr)p;
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N-1>): loop indices usable as immediates
template <class F, int... I>
__device__ __forceinline__ void static_for_impl(F&& f, std::integer_sequence<int, I...>) {
    (f(std::integral_constant<int, I>{}), ...);
}
template <int N, class F>
__device__ __forceinline__ void static_for(F&& f) {
    static_for_impl(static_cast<F&&>(f), std::make_integer_sequence<int, N>{});
}

__device__ __forceinline__ float sigmoid_f(float g) {
    return __builtin_amdgcn_rcpf(1.0f + __expf(-g));
}

// s_waitcnt vmcnt(n) only (expcnt / lgkmcnt left at their maxima), gfx9 encoding
#define SKIPFFN_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt(0x0F70 | ((n) & 15) | (((n) >> 4) << 14))
// s_waitcnt lgkmcnt(0) only
#define SKIPFFN_WAIT_LGKMCNT0() __builtin_amdgcn_s_waitcnt(0xC07F)

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for vmcnt(0),
// i.e. until every global store this wave has issued is acknowledged (microseconds per
// epilogue pass); the epilogues hand data from wave to wave through LDS alone, so their
// stores may stay in flight across the barrier.
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_sched_barrier(0);
    SKIPFFN_WAIT_LGKMCNT0();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
}

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

// One output tile (tm, tn) over the K slabs [kt_begin, kt_end) of the concatenated pairs;
// z selects the fp32 slab an EPI_PARTIAL result goes to.
//
// NARROW: the tile is 128 rows tall (for GEMMs with few rows: twice the workgroups per row of
// tiles, half the MFMA work per slab, so that the loop is bound by streaming B).  The eight
// waves keep their 2 x 4 arrangement, each owning 64 x 64 = 4 x 4 MFMA tiles; only the first
// 16 KB of an A stage are used.  KC A operands only.
template <bool A_KC, bool B_KC, int EPI, bool NARROW = false>
__device__ __forceinline__ void gemm_tile(const GemmArgs& P, const int tm, const int tn, const int z,
                                          const int kt_begin, const int kt_end, const int Meff,
                                          const int Keff) {
    static_assert(A_KC, "the A operand of every GEMM of the block is K-contiguous");
    constexpr int TM = NARROW ? BM / 2 : BM;        // tile rows
    constexpr int WROWS = TM / 2;                   // rows per wave row group
    constexpr int MT = WROWS / 32;                  // epilogue passes (32 rows per row group each)
    constexpr int MI = WROWS / 16;                  // MFMA tiles per wave along M (4 along N)
    constexpr int A_LOADS = TM / 64;                // 1 KB regions of an A slab each wave fills
    constexpr bool GU = (EPI == EPI_SWIGLU || EPI == EPI_PARTIAL_GU);   // B tile = 128 rows of W_gate + 128 of W_up
    // The A ring: 2 stages of 32 KB, fetched one slab ahead - or, for the 128-row tile, 3 stages
    // of 16 KB fetched two slabs ahead, in the same phase as B.  The 128-row tile streams its B
    // operand from HBM (few or no other tiles of the grid share it in L2); issuing everything in
    // the first phase of slab j lets a load stay in flight for 2 slab times instead of 1 (A) and
    // 1.4 (B): measured 4-6 % faster on the gate/up GEMM up to 256 rows.
    constexpr int NSA = NARROW ? 3 : NSTAGE_A;
    constexpr int A_STAGE = NARROW ? OPER_BYTES / 2 : OPER_BYTES;
    constexpr int A_AHEAD = NARROW ? 2 : 1;
    constexpr int B_BASE = NSA * A_STAGE;
    static_assert(B_BASE + NSTAGE_B * OPER_BYTES <= GEMM_LDS_BYTES, "operand rings must fit in LDS");
    extern __shared__ __align__(16) char smem[];
    const int t = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wm = wave >> 2;      // 0..1
    const int wn = wave & 3;       // 0..3

    const int m0 = tm * TM;
    const int n0 = GU ? tn * (BN / 2) : tn * BN;
    const int ktiles_pair = (Keff + BK - 1) / BK;
    const int nk = kt_end > kt_begin ? kt_end - kt_begin : 0;

    __amdgpu_buffer_rsrc_t rA0 = make_rsrc(P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rA1 = make_rsrc(P.A1 ? P.A1 : P.A0, P.a_bytes);
    __amdgpu_buffer_rsrc_t rB0 = make_rsrc(P.B0, P.b_bytes);
    __amdgpu_buffer_rsrc_t rB1 = make_rsrc(P.B1 ? P.B1 : P.B0, P.b_bytes);

    // ---- global -> LDS staging (direct-to-LDS buffer loads) ----------------------
    // A wave-wide 16-byte load deposits lane l at LDS base + 16*l, so each load
    // fills one contiguous 1 KB region q of the operand slab (32 regions; wave w
    // owns regions 4w..4w+3).  The swizzle is applied on the global side: a lane
    // fetches the chunk whose swizzled home is its own 16-byte slot.
    //   KC : region q = rows 8q..8q+7;   lane -> row 8q + l/8, chunk (l%8) ^ ((row/2)%8)
    //   MNC: region q = k-rows 2q, 2q+1; lane -> krow 2q + l/32, slot p = l%32:
    //        32-byte chunk (p/2) ^ mnc_swz(krow), half p & 1
    uint32_t a_goff[4], b_goff[4];     // byte offset of the lane's chunk at slab 0 (or OOB)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int q = wave * 4 + i;
        {
            const int qa = wave * A_LOADS + i;      // regions of A: wave w owns A_LOADS consecutive ones
            int row = 8 * qa + (lane >> 3), c = (lane & 7) ^ ((row >> 1) & 7);
            int gr = m0 + row;
            a_goff[i] = gr < Meff ? (uint32_t)(((int64_t)gr * P.lda + c * 8) * 2) : kOobOffset;
        }
        if (B_KC) {
            int row = 8 * q + (lane >> 3), c = (lane & 7) ^ ((row >> 1) & 7);
            // SWIGLU: tile rows 0..127 are W_gate rows, 128..255 the same rows of W_up
            int gr = GU ? n0 + (row & 127) : n0 + row;
            b_goff[i] = gr < P.N ? (uint32_t)(((int64_t)gr * P.ldb + c * 8) * 2) : kOobOffset;
        } else {
            int krow = 2 * q + (lane >> 5), pslot = lane & 31;
            int c16 = 2 * ((pslot >> 1) ^ mnc_swz(krow)) + (pslot & 1);
            int gc = n0 + c16 * 8;
            b_goff[i] = gc < P.N ? (uint32_t)(((int64_t)krow * P.ldb + gc) * 2) : kOobOffset;
        }
    }
    typedef __attribute__((address_space(3))) void* lds_void_ptr;
    // Issue this wave's share of A slab j / B slab j (0-based inside this block's K range).
    // The slab step is uniform and travels in the scalar offset of the buffer load; the per-lane
    // offset stays the loop-invariant a_goff / b_goff (an invalid row keeps kOobOffset: the range
    // check looks at the per-lane offset alone), so a slab that lies inside K costs no vector ALU
    // instruction at all.  Only a slab that reaches past K (the last one of a K that is no
    // multiple of 64) masks lanes individually; the empty assembly statements keep the compiler
    // from merging the two forms into one load with selected operands.
    auto gload_a = [&](int j) {
        const int kt = kt_begin + j;
        const int pair = kt >= ktiles_pair ? 1 : 0;
        const int kg = (kt - pair * ktiles_pair) * BK;  // k offset inside the pair
        __amdgpu_buffer_rsrc_t src = pair ? rA1 : rA0;
        char* dst = smem + (j % NSA) * A_STAGE + wave * (A_LOADS * 1024);
        const uint32_t step = (uint32_t)kg * 2u;
        if (kg + BK <= Keff) {
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (lds_void_ptr)(dst + i * 1024), 16, (int)a_goff[i], (int)step, 0, 0);
        } else {
            asm volatile("; K tail" ::: "memory");
#pragma unroll
            for (int i = 0; i < A_LOADS; ++i) {
                const int row = 8 * (wave * A_LOADS + i) + (lane >> 3);
                const int kk = ((lane & 7) ^ ((row >> 1) & 7)) * 8;
                const uint32_t off = (a_goff[i] != kOobOffset && kg + kk < Keff) ? a_goff[i] + step : kOobOffset;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (lds_void_ptr)(dst + i * 1024), 16, (int)off, 0, 0, 0);
            }
            asm volatile("; K tail end" ::: "memory");
        }
    };
    auto gload_b = [&](int j) {
        const int kt = kt_begin + j;
        const int pair = kt >= ktiles_pair ? 1 : 0;
        const int kg = (kt - pair * ktiles_pair) * BK;
        __amdgpu_buffer_rsrc_t src = pair ? rB1 : rB0;
        if (GU) src = wave >= 4 ? rB1 : rB0;   // regions 16.. = rows 128..
        char* dst = smem + B_BASE + (j % NSTAGE_B) * OPER_BYTES + wave * 4096;
        const uint32_t step = B_KC ? (uint32_t)kg * 2u : (uint32_t)(((int64_t)kg * P.ldb) * 2);
        if (kg + BK <= Keff) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (lds_void_ptr)(dst + i * 1024), 16, (int)b_goff[i], (int)step, 0, 0);
        } else {
            asm volatile("; K tail" ::: "memory");
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int kk;
                if (B_KC) {
                    const int row = 8 * (wave * 4 + i) + (lane >> 3);
                    kk = ((lane & 7) ^ ((row >> 1) & 7)) * 8;
                } else {
                    kk = 2 * (wave * 4 + i) + (lane >> 5);
                }
                const uint32_t off = (b_goff[i] != kOobOffset && kg + kk < Keff) ? b_goff[i] + step : kOobOffset;
                __builtin_amdgcn_raw_ptr_buffer_load_lds(src, (lds_void_ptr)(dst + i * 1024), 16, (int)off, 0, 0, 0);
            }
            asm volatile("; K tail end" ::: "memory");
        }
    };

    f32x4 acc[MI][4];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[mi][ni][r] = 0.0f;

    // Per-lane LDS offsets of this wave's fragments inside an operand stage (see the fragment
    // layouts above): the A fragment of MFMA tile mi lies mi * 2048 bytes after a_rd[ks]; B tile
    // ni of a KC stage b_tile_imm(ni) bytes after b_rd[ks], of an MNC stage at b_rd[ni] plus
    // ks * 16384 (and + 2048 for its second half).
    uint32_t a_rd[2], b_rd[B_KC ? 2 : 4];
    // SWIGLU: 32 gate columns (n-tiles 0, 1) and the same 32 columns of up (n-tiles 2, 3), 128 tile rows on
    const int b_row0 = GU ? wn * 32 : wn * 64;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
        a_rd[ks] = kc_off(wm * WROWS + (lane & 15), 4 * ks + (lane >> 4));
        if (B_KC) b_rd[ks] = kc_off(b_row0 + (lane & 15), 4 * ks + (lane >> 4));
    }
    if (!B_KC) {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni)
            b_rd[ni] = mnc_off(8 * (lane >> 4) + ((lane & 15) >> 2), (b_row0 >> 4) + ni, 8 * (lane & 3));
    }

    if (nk > 0) {
        // Ping-pong schedule.  The two waves that share a SIMD (wave w and w + 4, i.e.
        // the two row groups wm = 0, 1) run one phase apart: while one issues the 32
        // MFMAs of a half slab ("compute phase"), the other reads the fragments of
        // its next half slab from LDS ("memory phase").  Phases are delimited by
        // workgroup barriers; group 1 takes one extra barrier before the loop and
        // group 0 one after it, so the groups stay exactly one phase apart and every
        // wave executes the same number of barriers.  Per slab j a group runs
        // M(j,0) C(j,0) M(j,1) C(j,1); with p = 4j:
        //     phase      p        p+1      p+2      p+3
        //     group 0    M(j,0)   C(j,0)   M(j,1)   C(j,1)
        //     group 1    C(j-1,1) M(j,0)   C(j,0)   M(j,1)
        // Global loads are issued in the memory phases, where a wave has nothing else
        // to do while the address unit accepts them (about 16 clocks per wave-wide
        // 16-byte load, during which the issuing wave is blocked): A(j+1) in M(j,0)
        // and B(j+2) in M(j,1), four loads per wave and phase, so the address unit
        // sees an even stream of 16 loads per phase.  Their target stages (those of
        // A(j-1), B(j-1)) were last read in phase p-1.  Before the barrier that ends
        // phase p+3 every wave waits until only its B(j+2) loads may still be in
        // flight, so A(j+1) and B(j+1) are visible to all waves from phase p+4 on.
        bf16x8 af[MI], bfr[4];
        const uint32_t lds0 = lds_addr_of(smem);
        auto load_frags = [&](int j, auto ks) {
            const uint32_t sa = lds0 + (uint32_t)((j % NSA) * A_STAGE);
            const uint32_t sb = lds0 + (uint32_t)(B_BASE + (j % NSTAGE_B) * OPER_BYTES);
            const uint32_t aa = a_rd[ks] + sa;
            static_for<MI>([&](auto mi) { af[mi] = ds_read_b128_imm<mi * 2048>(aa); });
            if constexpr (B_KC) {
                const uint32_t ba = b_rd[ks] + sb;
                static_for<4>([&](auto ni) {
                    bfr[ni] = ds_read_b128_imm<GU ? (ni >> 1) * 16384 + (ni & 1) * 2048 : ni * 2048>(ba);
                });
            } else {
                static_for<4>([&](auto ni) {
                    const uint32_t ba = b_rd[ni] + sb;
                    const u32x2 lo = ds_read_tr16_b64_imm<ks * 16384>(ba);
                    const u32x2 hi = ds_read_tr16_b64_imm<ks * 16384 + 2048>(ba);
                    const u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
                    bfr[ni] = __builtin_bit_cast(bf16x8, both);
                });
            }
        };
        // The memory phase of the steady state: the loads of this phase (slabs that exist and lie
        // inside K: no test, no mask) spread evenly between the fragment reads.  A direct-to-LDS load
        // holds the issuing wave until the address unit takes it (about 64 cycles with four waves
        // loading at once); reads issued before it return meanwhile.  While the other wave of the
        // SIMD issues MFMAs back to back, EVERY instruction of this wave - scalar ones included -
        // takes two to three times as long to issue (a wait of 32 cycles inserted here costs 90), so
        // the phase carries as few instructions as possible: everything uniform about it (ring
        // stages, the scalar offsets of the loads, the operand descriptors) is kept in registers
        // and stepped once per slab instead of being derived from the slab index.
        uint32_t st_rd_a = 0, st_rd_b = 0;       // LDS address of the stages slab j is read from
        uint32_t st_ld_a = 0, st_ld_b = 0;       // LDS offset this wave loads slab j + A_AHEAD of A / slab j + 2 of B to
        uint32_t st_step_a = 0, st_step_b = 0;   // scalar offsets of those loads
        __amdgpu_buffer_rsrc_t st_src_a = rA0, st_src_b = rB0;
        auto memory_phase_fast = [&](auto ks) {
            constexpr int KS = decltype(ks)::value;
            constexpr int NLA = KS == 0 ? A_LOADS : 0;
            constexpr int NLB = (NARROW ? KS == 0 : KS == 1) ? 4 : 0;
            constexpr int NL = NLA + NLB, NR = MI + 4;
            const uint32_t aa = a_rd[KS] + st_rd_a;
            const uint32_t ba = B_KC ? b_rd[KS] + st_rd_b : st_rd_b;
            const uint32_t stepa = st_step_a, stepb = st_step_b;
            const __amdgpu_buffer_rsrc_t srca = st_src_a, srcb = st_src_b;
            char* dsta = smem + st_ld_a;
            char* dstb = smem + st_ld_b;
            static_for<NR>([&](auto r) {
                static_for<NL>([&](auto l) {
                    if constexpr (l * NR / NL == r) {
                        if constexpr (l < NLA)
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(srca, (lds_void_ptr)(dsta + l * 1024), 16,
                                                                     (int)a_goff[l], (int)stepa, 0, 0);
                        else
                            __builtin_amdgcn_raw_ptr_buffer_load_lds(srcb, (lds_void_ptr)(dstb + (l - NLA) * 1024), 16,
                                                                     (int)b_goff[l - NLA], (int)stepb, 0, 0);
                    }
                });
                if constexpr (r < MI) {
                    af[r] = ds_read_b128_imm<r * 2048>(aa);
                } else if constexpr (B_KC) {
                    constexpr int ni = r - MI;
                    bfr[ni] = ds_read_b128_imm<GU ? (ni >> 1) * 16384 + (ni & 1) * 2048 : ni * 2048>(ba);
                } else {
                    constexpr int ni = r - MI;
                    const uint32_t bn = b_rd[ni] + ba;
                    const u32x2 lo = ds_read_tr16_b64_imm<KS * 16384>(bn);
                    const u32x2 hi = ds_read_tr16_b64_imm<KS * 16384 + 2048>(bn);
                    const u32x4 both = {lo[0], lo[1], hi[0], hi[1]};
                    bfr[ni] = __builtin_bit_cast(bf16x8, both);
                }
            });
        };
        auto compute_phase = [&]() {
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int nj = 0; nj < 4; ++nj) {
                    // B fragment first: the accumulator then holds, per lane, one row m of
                    // C and four consecutive columns n (see the epilogue).  Boustrophedon order:
                    // consecutive MFMAs always share one operand register set.
                    const int ni = (mi & 1) ? 3 - nj : nj;
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[ni], af[mi], acc[mi][ni], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        };
        auto phase_barrier = [&]() {
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
        };
        // slab j+1 of both operands has landed; what slab j issued for slab j+2 (B, and A when it
        // is fetched two ahead) may still fly
        constexpr int FLYING = 4 + (A_AHEAD == 2 ? A_LOADS : 0);
        auto wait_next_slab = [&](int j) {
            if (j + 2 < nk) SKIPFFN_WAIT_VMCNT(FLYING); else SKIPFFN_WAIT_VMCNT(0);
        };

        // prologue: slabs 0 and 1 issued (A(1) only when A is fetched two ahead); A(0) and B(0)
        // landed and visible
        gload_a(0);
        gload_b(0);
        if (nk > 1) {
            if (A_AHEAD == 2) gload_a(1);
            gload_b(1);
            SKIPFFN_WAIT_VMCNT(FLYING);
        } else {
            SKIPFFN_WAIT_VMCNT(0);
        }
        phase_barrier();
        if (wm == 1) phase_barrier();                     // group 1 starts one phase later

        // slabs [0, kfull) of a pair lie inside K
        const int kfull = Keff / BK;
        const uint32_t dstep_b = B_KC ? (uint32_t)BK * 2u : (uint32_t)BK * (uint32_t)P.ldb * 2u;
        const uint32_t rd_a_end = lds0 + NSA * A_STAGE, rd_b_end = lds0 + B_BASE + NSTAGE_B * OPER_BYTES;
        const uint32_t ld_a_end = NSA * A_STAGE + wave * (A_LOADS * 1024);
        const uint32_t ld_b_end = B_BASE + NSTAGE_B * OPER_BYTES + wave * 4096;
        int fast_end = 0;                  // iterations [j, fast_end) are steady state
        for (int j = 0; j < nk; ++j) {
            bool fast = j < fast_end;
            if (!fast) {
                // does a steady-state run start at slab j?  For `run` iterations the slabs to load
                // (j + A_AHEAD of A, j + 2 of B) exist, lie inside K and stay in the operand pair they
                // are in now.
                // (the empty assembly statements pin this rarely executed arithmetic to this place and to
                // scalar registers: derived from the loop counter, it would otherwise be hoisted to the
                // top of every iteration)
                int js = j;
                asm volatile("" : "+s"(js));
                const int kta = kt_begin + js + A_AHEAD, ktb = kt_begin + js + 2;
                const int paira = kta >= ktiles_pair ? 1 : 0, pairb = ktb >= ktiles_pair ? 1 : 0;
                const int ia = kta - paira * ktiles_pair, ib = ktb - pairb * ktiles_pair;
                int run = nk - 2 - js;
                run = run < kfull - ia ? run : kfull - ia;
                asm volatile("" : "+s"(run));
                run = run < kfull - ib ? run : kfull - ib;
                asm volatile("" : "+s"(run));
                if (run > 0) {
                    fast = true;
                    fast_end = js + run;
                    st_rd_a = lds0 + (uint32_t)((js % NSA) * A_STAGE);
                    st_rd_b = lds0 + (uint32_t)(B_BASE + (js % NSTAGE_B) * OPER_BYTES);
                    st_ld_a = (uint32_t)(((js + A_AHEAD) % NSA) * A_STAGE + wave * (A_LOADS * 1024));
                    st_ld_b = (uint32_t)(B_BASE + ((js + 2) % NSTAGE_B) * OPER_BYTES + wave * 4096);
                    st_step_a = (uint32_t)(ia * BK) * 2u;
                    st_step_b = (uint32_t)ib * dstep_b;
                    st_src_a = paira ? rA1 : rA0;
                    st_src_b = GU ? (wave >= 4 ? rB1 : rB0) : (pairb ? rB1 : rB0);
                }
            }
            // M(j,0)
            if (fast) {
                memory_phase_fast(std::integral_constant<int, 0>{});
            } else {
                // a slab at the end of the K range (or of a pair): loads guarded and masked
                int js = j;
                asm volatile("" : "+s"(js));
                load_frags(js, std::integral_constant<int, 0>{});
                if (js + A_AHEAD < nk) gload_a(js + A_AHEAD);
                if (NARROW && js + 2 < nk) gload_b(js + 2);
            }
            SKIPFFN_WAIT_LGKMCNT0();
            phase_barrier();
            // C(j,0)
            compute_phase();
            phase_barrier();
            // M(j,1)
            if (fast) {
                memory_phase_fast(std::integral_constant<int, 1>{});
            } else {
                int js = j;
                asm volatile("" : "+s"(js));
                load_frags(js, std::integral_constant<int, 1>{});
                if (!NARROW && js + 2 < nk) gload_b(js + 2);
            }
            if (wm == 1) wait_next_slab(j);
            SKIPFFN_WAIT_LGKMCNT0();
            phase_barrier();
            // C(j,1)
            compute_phase();
            if (wm == 0) wait_next_slab(j);
            if (fast) {
                // next slab: rotate the ring stages, step the load offsets
                st_rd_a += A_STAGE; if (st_rd_a == rd_a_end) st_rd_a -= NSA * A_STAGE;
                st_rd_b += OPER_BYTES; if (st_rd_b == rd_b_end) st_rd_b -= NSTAGE_B * OPER_BYTES;
                st_ld_a += A_STAGE; if (st_ld_a == ld_a_end) st_ld_a -= NSA * A_STAGE;
                st_ld_b += OPER_BYTES; if (st_ld_b == ld_b_end) st_ld_b -= NSTAGE_B * OPER_BYTES;
                st_step_a += (uint32_t)BK * 2u;
                st_step_b += dstep_b;
            }
            phase_barrier();
        }
        if (wm == 0) phase_barrier();                     // balances group 1's extra barrier
    }

    // ---- epilogue --------------------------------------------------------------
    // With the B fragment as first MFMA operand, acc[mi][ni][r] is C[row][col] with
    //   row = m0 + wm*WROWS + mi*16 + lane%16        (WROWS = 128, or 64 in the 128-row variant)
    //   col = (tile column base) + ni*16 + 4*(lane/16) + r
    // i.e. the four registers of an MFMA tile are four consecutive columns of one row.
    // The tile leaves through LDS (free after the main loop): per pass mt, every
    // row group (wm) dumps its 32 x 256 fp32 slice (MFMA tile rows 2mt, 2mt+1) as 16-byte vectors, and after a
    // barrier each thread takes row-contiguous chunks of 8 columns, applies the epilogue
    // arithmetic and moves 16 bytes per global access.  The barriers order LDS traffic only, so the stores of one pass overlap
    // the staging of the next.
    //
    // The SwiGLU epilogues also leave TRANSPOSED copies of their results (H^T; dG^T and dU^T:
    // [columns][rows], leading dimension ldt) for the weight-gradient GEMMs, which contract
    // over the rows and read both operands with plain 16-byte LDS reads when the row index is
    // contiguous.  A thread's packed results (pairs of columns, adjacent rows) go to an LDS
    // buffer T[column pair][row] with one 8- or 16-byte write per column pair; after a second
    // barrier each thread picks up 8 consecutive rows of a column pair (two 16-byte reads),
    // separates the two columns with byte permutes and stores 16 bytes per column.
    constexpr bool HAS_T = (EPI == EPI_SWIGLU || EPI == EPI_SWIGLU_BWD);
    constexpr int SLICE_COLS = (EPI == EPI_SWIGLU) ? 128 : 256;       // per staged matrix
    constexpr int SLICE_STRIDE = SLICE_COLS * 4 + 16;                   // bytes; +16 spreads rows over banks
    constexpr int SLICE_MATS = (EPI == EPI_SWIGLU) ? 2 : 1;             // G and U
    constexpr int SLICE_BYTES = SLICE_MATS * EPI_ROWS * SLICE_STRIDE;   // per row group
    // Staging buffers: two per row group, alternating between passes, so that one barrier per
    // pass suffices - except for the SwiGLU backward, whose two transposition buffers leave
    // room for one per row group only (it takes a second barrier per pass anyway).
    constexpr int NSTAGING = (EPI == EPI_SWIGLU_BWD) ? 1 : 2;
    constexpr int T_MATS = (EPI == EPI_SWIGLU_BWD) ? 2 : 1;
    constexpr int T_PAIRS = SLICE_COLS / 2;                             // column pairs per row group
    constexpr int T_ROWB = EPI_ROWS * 4 + 16;                           // bytes per column pair: 32 rows + pad
    constexpr int T_BYTES = T_PAIRS * T_ROWB + (T_PAIRS / 4) * 16;      // per matrix and row group (skewed, see t_off)
    constexpr int T_BASE = 2 * NSTAGING * SLICE_BYTES;
    static_assert(T_BASE + (HAS_T ? 2 * T_MATS * T_BYTES : 0) <= GEMM_LDS_BYTES, "staging must fit in LDS");
    const int cq = lane >> 4;                     // column quad of this lane inside an MFMA tile
    const int tg = t & 255;                       // thread index inside the row group
    constexpr int CHUNKS_PER_ROW = SLICE_COLS / 8;
    constexpr int CHUNKS_PER_THREAD = EPI_ROWS * CHUNKS_PER_ROW / 256;
    // chunk i of this thread: column chunk cc, row rbase + i * RSTEP - adjacent rows where the
    // transposed copies want them (one wide LDS write per column pair), else rows spread over the slice
    const int cc = tg % CHUNKS_PER_ROW;
    constexpr int RSTEP = HAS_T ? 1 : 256 / CHUNKS_PER_ROW;
    const int rbase = HAS_T ? (tg / CHUNKS_PER_ROW) * CHUNKS_PER_THREAD : tg / CHUNKS_PER_ROW;
    // byte offset of (column pair cp, row r) in a transposition buffer: 16 extra bytes per four
    // column pairs (= per chunk of 8 columns) make the writes of a wave tile all 64 banks
    auto t_off = [&](int cp, int r) { return cp * T_ROWB + (cp >> 2) * 16 + r * 4; };
    const bool want_t = HAS_T && P.outT0 != nullptr;

    // EPI_SWIGLU_BWD reads G and U next to the accumulator: those 16-byte loads are issued one
    // pass ahead (and ahead of the previous pass's stores in the in-order vmcnt queue), so
    // their latency hides behind the staging of the pass before.
    u32x4 pre_g[2][CHUNKS_PER_THREAD], pre_u[2][CHUNKS_PER_THREAD];
    auto prefetch_gu = [&](int mt) {
        if (EPI != EPI_SWIGLU_BWD) return;
#pragma unroll
        for (int i = 0; i < CHUNKS_PER_THREAD; ++i) {
            const int row = m0 + wm * WROWS + mt * 32 + rbase + i * RSTEP;
            const int col = n0 + cc * 8;
            if (row >= Meff || col >= P.N) continue;
            const uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
            pre_g[mt & 1][i] = *reinterpret_cast<const u32x4*>(P.e0 + o);
            pre_u[mt & 1][i] = *reinterpret_cast<const u32x4*>(P.e1 + o);
        }
    };
    prefetch_gu(0);

#pragma unroll
    for (int mt = 0; mt < MT; ++mt) {
        char* sbuf = smem + ((NSTAGING == 2 ? (mt & 1) * 2 : 0) + wm) * SLICE_BYTES;
        // ---- dump this wave's part of the slice
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni) {
                const f32x4 v = acc[2 * mt + s2][ni];
                int col, mat;
                if (EPI == EPI_SWIGLU)          { mat = ni >> 1; col = wn * 32 + (ni & 1) * 16 + 4 * cq; }
                else if (EPI == EPI_PARTIAL_GU) { mat = 0;  col = (ni >> 1) * 128 + wn * 32 + (ni & 1) * 16 + 4 * cq; }
                else                            { mat = 0;  col = wn * 64 + ni * 16 + 4 * cq; }
                *reinterpret_cast<f32x4*>(sbuf + mat * EPI_ROWS * SLICE_STRIDE +
                                          (s2 * 16 + (lane & 15)) * SLICE_STRIDE + col * 4) = v;
            }
        lds_barrier();
        if (mt + 1 < MT) prefetch_gu(mt + 1);
        // packed results of this thread's chunks, kept for the transposed copies: [matrix][column pair k][row i]
        uint32_t tpk[T_MATS][4][CHUNKS_PER_THREAD];
        // ---- row-contiguous chunks of 8 columns
#pragma unroll
        for (int i = 0; i < CHUNKS_PER_THREAD; ++i) {
            const int r = rbase + i * RSTEP, c = cc;
            const int row = m0 + wm * WROWS + mt * 32 + r;
            const int col = n0 + c * 8;
            const bool live = row < Meff && (EPI == EPI_PARTIAL_GU || col < P.N);
            if (HAS_T) {
#pragma unroll
                for (int m = 0; m < T_MATS; ++m)
#pragma unroll
                    for (int k = 0; k < 4; ++k) tpk[m][k][i] = 0u;     // rows past the end: zeros in the copies
            }
            if (!live) continue;
            // lanes c >= 8 (mod 16) read their second half first: conflict-free 16-byte reads
            const int swap = (c >> 3) & 1;
            float v[8], w[8];
            {
                const char* src = sbuf + r * SLICE_STRIDE + c * 32;
                f32x4 a = *reinterpret_cast<const f32x4*>(src + (swap ? 16 : 0));
                f32x4 b = *reinterpret_cast<const f32x4*>(src + (swap ? 0 : 16));
                f32x4 lo = swap ? b : a, hi = swap ? a : b;
#pragma unroll
                for (int k = 0; k < 4; ++k) { v[k] = lo[k]; v[4 + k] = hi[k]; }
            }
            if (EPI == EPI_SWIGLU) {
                const char* src = sbuf + EPI_ROWS * SLICE_STRIDE + r * SLICE_STRIDE + c * 32;
                f32x4 a = *reinterpret_cast<const f32x4*>(src + (swap ? 16 : 0));
                f32x4 b = *reinterpret_cast<const f32x4*>(src + (swap ? 0 : 16));
                f32x4 lo = swap ? b : a, hi = swap ? a : b;
#pragma unroll
                for (int k = 0; k < 4; ++k) { w[k] = lo[k]; w[4 + k] = hi[k]; }
                const uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
                u32x4 ph, pg, pu;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float g0 = v[2 * k], g1 = v[2 * k + 1], u0 = w[2 * k], u1 = w[2 * k + 1];
                    ph[k] = pack_bf16x2(g0 * sigmoid_f(g0) * u0, g1 * sigmoid_f(g1) * u1);
                    pg[k] = pack_bf16x2(g0, g1);
                    pu[k] = pack_bf16x2(u0, u1);
                    if (HAS_T) tpk[0][k][i] = ph[k];
                }
                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out0) + o) = ph;
                if (P.out1 != nullptr) {
                    *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out1) + o) = pg;
                    *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out2) + o) = pu;
                }
            } else if (EPI == EPI_STORE) {
                const uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
                if (P.out_f32) {
                    f32x4* O = reinterpret_cast<f32x4*>(static_cast<float*>(P.out0) + o);
                    f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
                    if (P.accumulate) { lo += O[0]; hi += O[1]; }
                    O[0] = lo;
                    O[1] = hi;
                } else {
                    u32x4* O = reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out0) + o);
                    if (P.accumulate) {
                        u32x4 old = *O;
#pragma unroll
                        for (int k = 0; k < 4; ++k) {
                            v[2 * k] += bf16lo_to_f32(old[k]);
                            v[2 * k + 1] += bf16hi_to_f32(old[k]);
                        }
                    }
                    u32x4 pk;
#pragma unroll
                    for (int k = 0; k < 4; ++k) pk[k] = pack_bf16x2(v[2 * k], v[2 * k + 1]);
                    *O = pk;
                }
            } else if (EPI == EPI_PARTIAL_GU) {
                // every column of the tile is written (rows of W beyond N read as zeros)
                f32x4* O = reinterpret_cast<f32x4*>(P.partial + ((int64_t)z * P.M + row) * ((int64_t)P.tiles_n * BN) +
                                                    (int64_t)tn * BN + c * 8);
                f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
                O[0] = lo;
                O[1] = hi;
            } else if (EPI == EPI_PARTIAL) {
                f32x4* O = reinterpret_cast<f32x4*>(P.partial + ((int64_t)z * P.M + row) * P.N + col);
                f32x4 lo = {v[0], v[1], v[2], v[3]}, hi = {v[4], v[5], v[6], v[7]};
                O[0] = lo;
                O[1] = hi;
            } else if (EPI == EPI_RESID_SCATTER) {
                const uint32_t o = (uint32_t)P.idx[row] * (uint32_t)P.ldo + (uint32_t)col;
                if (!P.no_residual) {
                    u32x4 x = *reinterpret_cast<const u32x4*>(P.e0 + o);
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        v[2 * k] += bf16lo_to_f32(x[k]);
                        v[2 * k + 1] += bf16hi_to_f32(x[k]);
                    }
                }
                u32x4 pk;
#pragma unroll
                for (int k = 0; k < 4; ++k) pk[k] = pack_bf16x2(v[2 * k], v[2 * k + 1]);
                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out0) + o) = pk;
            } else if (EPI == EPI_SWIGLU_BWD) {
                const uint32_t o = (uint32_t)row * (uint32_t)P.ldo + (uint32_t)col;
                const u32x4 gq = pre_g[mt & 1][i];
                const u32x4 uq = pre_u[mt & 1][i];
                u32x4 dgq, duq;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    float gg[2] = {bf16lo_to_f32(gq[k]), bf16hi_to_f32(gq[k])};
                    float uu[2] = {bf16lo_to_f32(uq[k]), bf16hi_to_f32(uq[k])};
                    float dg[2], du[2];
#pragma unroll
                    for (int e = 0; e < 2; ++e) {
                        float sg = sigmoid_f(gg[e]);
                        float dh = v[2 * k + e];
                        dg[e] = dh * uu[e] * sg * (1.0f + gg[e] * (1.0f - sg));
                        du[e] = dh * gg[e] * sg;
                    }
                    dgq[k] = pack_bf16x2(dg[0], dg[1]);
                    duq[k] = pack_bf16x2(du[0], du[1]);
                    if (HAS_T) { tpk[0][k][i] = dgq[k]; tpk[T_MATS - 1][k][i] = duq[k]; }
                }
                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out0) + o) = dgq;
                *reinterpret_cast<u32x4*>(static_cast<bf16_t*>(P.out1) + o) = duq;
            }
        }
        if constexpr (HAS_T) {
            if (want_t) {
                // ---- transposed copies: T[matrix][row group][column pair][row]
                static_assert(CHUNKS_PER_THREAD == 2 || CHUNKS_PER_THREAD == 4, "one 8- or 16-byte write per column pair");
#pragma unroll
                for (int m = 0; m < T_MATS; ++m) {
                    char* tb = smem + T_BASE + (m * 2 + wm) * T_BYTES;
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        char* dst = tb + t_off(cc * 4 + k, rbase);
                        if (CHUNKS_PER_THREAD == 4) {
                            u32x4 q = {tpk[m][k][0], tpk[m][k][1], tpk[m][k][2], tpk[m][k][3]};
                            *reinterpret_cast<u32x4*>(dst) = q;
                        } else {
                            u32x2 q = {tpk[m][k][0], tpk[m][k][1]};
                            *reinterpret_cast<u32x2*>(dst) = q;
                        }
                    }
                }
                lds_barrier();
                // items: (matrix, column pair, block of 8 rows); 4 row blocks per column pair
                constexpr int ITEMS = T_MATS * T_PAIRS * 4 / 256;       // per thread
#pragma unroll
                for (int it = 0; it < ITEMS; ++it) {
                    const int id = tg + 256 * it;
                    const int m = id / (T_PAIRS * 4);
                    const int rem = id - m * (T_PAIRS * 4);
                    const int rb = rem & 3, cp = rem >> 2;     // four consecutive lanes: 64 contiguous bytes of one column
                    const char* tb = smem + T_BASE + (m * 2 + wm) * T_BYTES + t_off(cp, rb * 8);
                    const u32x4 a = *reinterpret_cast<const u32x4*>(tb);
                    const u32x4 b = *reinterpret_cast<const u32x4*>(tb + 16);
                    // a, b: rows rb*8 .. +7 of the column pair, low half = even column
                    u32x4 even, odd;
                    even[0] = __builtin_amdgcn_perm(a[1], a[0], 0x05040100u); odd[0] = __builtin_amdgcn_perm(a[1], a[0], 0x07060302u);
                    even[1] = __builtin_amdgcn_perm(a[3], a[2], 0x05040100u); odd[1] = __builtin_amdgcn_perm(a[3], a[2], 0x07060302u);
                    even[2] = __builtin_amdgcn_perm(b[1], b[0], 0x05040100u); odd[2] = __builtin_amdgcn_perm(b[1], b[0], 0x07060302u);
                    even[3] = __builtin_amdgcn_perm(b[3], b[2], 0x05040100u); odd[3] = __builtin_amdgcn_perm(b[3], b[2], 0x07060302u);
                    const int colT = n0 + 2 * cp;
                    const int rowT = m0 + wm * WROWS + mt * 32 + rb * 8;
                    if (rowT >= P.ldt || colT >= P.N) continue;        // ldt is a multiple of 8 >= the row bound
                    bf16_t* base = static_cast<bf16_t*>(m == 0 ? P.outT0 : P.outT1);
                    *reinterpret_cast<u32x4*>(base + (int64_t)colT * P.ldt + rowT) = even;
                    if (colT + 1 < P.N) *reinterpret_cast<u32x4*>(base + (int64_t)(colT + 1) * P.ldt + rowT) = odd;
                }
            }
        }
        // a single staging buffer is dumped into again by the next pass: its readers must be done (with the
        // transposed copies the barrier before the read-back has seen to that)
        if (NSTAGING == 1 && !want_t && mt + 1 < MT) lds_barrier();
    }
}

// The gate/up GEMM may end in a row of 128-row tiles: a row count just above a multiple of 256
// then costs half a tile row instead of a whole one (R = 2944 = 11.5 tile rows: 1288 tile units
// of work instead of 1344), and the half-height tiles, dispatched last, even out the end of the
// grid (measured 635 -> 597 us).  The dH GEMM does not get it: its 128-row tiles are bound by the
// memory phases of the N-contiguous weight operand and take as long as full ones, and the extra
// code path cost the shared dH + dW_down kernel 2 % (713 -> 730 us with the path unused).
template <bool A_KC, int EPI>
constexpr bool kTailNarrowOk = A_KC && EPI == EPI_SWIGLU;

// One workgroup's share of a plain (optionally split-K, optionally batched) GEMM: `block` of
// `nblocks` in the launch order of this problem.
template <bool A_KC, bool B_KC, int EPI, bool NARROW = false>
__device__ __forceinline__ void gemm_block(GemmArgs P, const int block, const int nblocks) {
    const int Meff = effective_rows(P.M, P.m_dev);
    const int Keff = effective_rows(P.K, P.k_dev);
    if constexpr (!NARROW && kTailNarrowOk<A_KC, EPI>) {
        // host contract: tail_narrow comes with splits == 1, batch == 1 and a host-side row count
        const int full = P.tiles_m * P.tiles_n;
        if (P.tail_narrow && block >= full) {
            const int ktotal = ((Keff + BK - 1) / BK) * P.pairs;
            gemm_tile<A_KC, B_KC, EPI, true>(P, 2 * P.tiles_m, block - full, 0, 0, ktotal, Meff, Keff);
            return;
        }
        if (P.tail_narrow) {
            int tm, tn, z;
            tile_of_block(block, full, P.tiles_m, P.tiles_n, tm, tn, z);
            const int ktotal = ((Keff + BK - 1) / BK) * P.pairs;
            gemm_tile<A_KC, B_KC, EPI, false>(P, tm, tn, 0, 0, ktotal, Meff, Keff);
            return;
        }
    }
    int tm, tn, z;
    tile_of_block(block, nblocks, P.tiles_m, P.tiles_n, tm, tn, z);
    // batched launch (two problems in one grid, used for dW_gate / dW_up): the upper half of
    // the z range is problem 1
    const bool second = P.batch == 2 && z >= P.splits;
    if (second) {
        z -= P.splits;
        P.A0 = P.A1;
        P.out0 = P.out1;
    }
    if (tm * (NARROW ? BM / 2 : BM) >= Meff) return;    // whole block leaves together: no barrier was reached yet
    const int ktotal = ((Keff + BK - 1) / BK) * P.pairs;
    const int per_split = (ktotal + P.splits - 1) / P.splits;
    const int kt_begin = z * per_split;
    int kt_end = kt_begin + per_split;
    if (kt_end > ktotal) kt_end = ktotal;
    gemm_tile<A_KC, B_KC, EPI, NARROW>(P, tm, tn, z, kt_begin, kt_end, Meff, Keff);
}

template <bool A_KC, bool B_KC, int EPI, bool NARROW = false>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_kernel(GemmArgs P) {
    gemm_block<A_KC, B_KC, EPI, NARROW>(P, (int)blockIdx.x, (int)gridDim.x);
}

// Two independent GEMMs in one grid: workgroups [0, nblocks0) run problem 0 (launched
// first: give it the longer tiles), the rest problem 1, so the last round of one fills
// with tiles of the other instead of leaving CUs idle.  nblocks0 is a multiple of 8 (the
// host pads with workgroups that exit at once) so that both problems see the round-robin
// XCD assignment from its start.
template <bool A0_KC, bool B0_KC, int EPI0, bool A1_KC, bool B1_KC, int EPI1>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_dual_kernel(GemmArgs P0, GemmArgs P1,
                                                                      int nblocks0, int real0) {
    const int b = (int)blockIdx.x;
    if (b < nblocks0) {
        if (b < real0) gemm_block<A0_KC, B0_KC, EPI0>(P0, b, real0);
    } else {
        gemm_block<A1_KC, B1_KC, EPI1>(P1, b - nblocks0, (int)gridDim.x - nblocks0);
    }
}

// ---- balanced split-K for GEMMs that leave through fp32 partial slabs (see streamk.hpp) ------
// grid = tiles_n * nbg workgroups (P.splits carries nbg); EPI_PARTIAL only
template <bool A_KC, bool B_KC>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_streamk_kernel(GemmArgs P) {
    const int nbg = P.splits;
    const int nb = (int)gridDim.x;
    const int tiles_n = nb / nbg;
    int b = (int)blockIdx.x;
    // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous range of the
    // logical order below
    if ((nb & 7) == 0) b = (b & 7) * (nb >> 3) + (b >> 3);
    const int Meff = effective_rows(P.M, P.m_dev);
    const int Keff = effective_rows(P.K, P.k_dev);
    const int g = (Meff + BM - 1) / BM;
    const int kt = ((Keff + BK - 1) / BK) * P.pairs;
    if (g == 0 || kt == 0) return;
    const StreamKPlan p = streamk_plan(g, kt, nbg);
    // Logical order: aligned chunks first, chunk-major, then n-tile, then m-tile - so an XCD
    // works on ONE K range of many n-tiles (the m-tiles of an n-tile share the weight slabs,
    // the n-tiles share the activation slabs, and no XCD streams the whole K extent of the
    // activations); the remainder pieces follow.  (tn, j) = n-tile and workgroup index in its group.
    // (With more tiles than workgroups in a group every workgroup starts with whole tiles of its own,
    // see streamk.hpp; the order below is that of the gr tiles that are split.)
    int tn, j;
    const int gr = p.gr;
    const int aligned_total = p.a * gr * tiles_n;
    if (b < aligned_total) {
        const int c = b / (tiles_n * gr);
        const int r = b - c * (tiles_n * gr);
        tn = r / gr;
        j = c * gr + (r - tn * gr);
    } else {
        const int per = nbg - p.a * gr;           // workgroups per group left for the remainder
        const int r = b - aligned_total;
        tn = r / per;
        j = p.a * gr + (r - tn * per);
    }
    StreamKIter it = streamk_begin(p, j);
    StreamKSeg sg;
    bool first = true;
    while (streamk_next(p, it, sg)) {      // uniform over the workgroup
        if (!first) lds_barrier();          // the staging buffers of the previous epilogue are free again
        first = false;
        gemm_tile<A_KC, B_KC, EPI_PARTIAL>(P, sg.i, tn, sg.slot, sg.kb, sg.ke, Meff, Keff);
    }
}

// ---- self-similarity of several row sets in one grid: S_i = X_i X_i^T (fp32) -------------------
// P describes the whole row list (A0 = first row, lda = row length, K = row length); item i uses
// rows st.off[i] .. st.off[i+1]) and writes [n_i][P.ldo] floats at out0 + i * out_stride.  The
// grid covers tiles_1d x tiles_1d tiles per item (tiles_1d from the largest set).
template <int EPI>
__global__ __launch_bounds__(GEMM_THREADS) void gemm_bf16_selfsim_kernel(GemmArgs P, SegTable st, int tiles_1d,
                                                                         int64_t out_stride) {
    const int b = (int)blockIdx.x;
    const int per_item = tiles_1d * tiles_1d;
    const int item = b / per_item;
    const int r = b - item * per_item;
    const int tn = r / tiles_1d, tm = r - tn * tiles_1d;
    const int lo = st.off[item], n = st.off[item + 1] - lo;
    if (tm * BM >= n || tn * BN >= n) return;        // whole block leaves together
    P.A0 += (int64_t)lo * P.lda;
    P.B0 = P.A0;
    P.a_bytes = P.b_bytes = (uint32_t)((int64_t)n * P.lda * 2);
    P.M = P.N = n;
    P.out0 = static_cast<float*>(P.out0) + item * out_stride;
    const int ktotal = (P.K + BK - 1) / BK;
    gemm_tile<true, true, EPI>(P, tm, tn, 0, 0, ktotal, n, P.K);
}

}  // namespace skipffn
