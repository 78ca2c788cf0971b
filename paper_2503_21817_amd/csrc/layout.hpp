// Host-side planning of the Skip-FFN block: how the `saved` buffer and the workspaces are carved
// into sections, and how the K range of a GEMM is cut over the compute units.  Plain C++ (no HIP
// constructs), shared by the library's entry points and by a host checker that is built with the
// address and undefined-behaviour sanitizers.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include <algorithm>

#include "streamk.hpp"

namespace skipffn {

constexpr int BM = 256, BN = 256, BK = 64;          // output tile and K slab of the GEMM core
constexpr int GAIN_STRIP = 4;                        // rows per workgroup of the gain-gradient pass

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
// bytes of the gain-gradient scratch (one fp32 row of C per strip of rows)
inline size_t gain_partial_bytes(int64_t R, int64_t C) {
    return (size_t)((R + GAIN_STRIP - 1) / GAIN_STRIP) * (size_t)C * 4;
}

constexpr int kMaxSplits = 8;
constexpr int kMaxSplitsNarrow = 16;     // few rows: small fp32 slabs, and every CU has to stream weights

// How the K range of a GEMM with tiles_m x tiles_n output tiles and `ktiles` K slabs is cut
// on `ncu` CUs (one workgroup per CU).  Costs are in units of one K slab of one tile: every
// round of `ncu` workgroups costs its slab count plus a fixed prologue/epilogue, partial tiles
// cost a write now and a read in the reducing kernel.
//   splits == 1, sk_nbg == 0 : one workgroup per tile, epilogue fused
//   splits  > 1, sk_nbg == 0 : plain split-K into `splits` fp32 slabs
//   sk_nbg  > 0              : balanced split (gemm_bf16_streamk_kernel), sk_nbg workgroups per
//                              n-tile group (with more m-tiles than workgroups in a group, every
//                              workgroup first runs whole tiles of its own; the rest is split)
struct KPartition { int splits; int sk_nbg; };
inline KPartition choose_k_partition(int tiles_m, int tiles_n, int ktiles, bool force_balanced, int ncu) {
    const int tiles = tiles_m * tiles_n;
    KPartition best{1, 0};
    double best_cost = 1e30;
    for (int s = 1; s <= kMaxSplits; ++s) {
        int per = (ktiles + s - 1) / s;
        if (s > 1 && per < 8) break;
        int rounds = (tiles * s + ncu - 1) / ncu;
        double cost = rounds * (per + 8.0 + (s > 1 ? 8.0 : 0.0)) + (s > 1 ? 0.04 * s * tiles : 0.0);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = KPartition{s, 0}; }
    }
    const int nbg = tiles_n > 0 ? ncu / tiles_n : 0;
    if (nbg >= 1 && tiles > 0) {
        const StreamKPlan p = streamk_plan(tiles_m, ktiles, nbg);
        if (force_balanced) return KPartition{1, nbg};
        if (p.gr > 0 && p.q >= 8) {
            double slabs = 0.0;
            for (int i = 0; i < tiles_m; ++i) slabs += streamk_count(p, i);
            // an aligned chunk is one segment; a remainder piece runs one segment (with its own
            // prologue and epilogue: about 5 slabs' worth, measured) per tile it touches; with more
            // tiles than workgroups in a group, whole tiles come first
            const double aligned = p.a > 0 ? p.q + 16.0 : 0.0;
            const double pieces = p.nr > 0 ? p.qr + 16.0 + 5.0 * (p.qr / p.rem) : 0.0;
            double cost = p.full * (ktiles + 16.0) + std::max(aligned, pieces) + 0.04 * slabs * tiles_n;
            if (cost < best_cost - 1e-9) { best_cost = cost; best = KPartition{1, nbg}; }
        }
    }
    return best;
}

// Few rows: the GEMMs of the forward pass run on 128-row tiles (twice the workgroups per row of
// tiles, a loop bound by streaming the weights instead of by MFMA work on empty rows).
// Measured at C=4096, I=14336: gate/up 86 -> 75 us and down 44 -> 38 us up to 128 rows, a few
// per cent up to 256 rows, slower beyond (the half-height tiles are bound by the load / barrier
// skeleton of the loop, not by MFMA work).
inline bool narrow_rows(int64_t rows) { return rows <= 256; }
// plain split-K for the 128-row tiles: fill the CUs, keep at least 8 slabs per workgroup
inline KPartition choose_k_split_narrow(int tiles_m, int tiles_n, int ktiles, int ncu) {
    const int tiles = tiles_m * tiles_n;
    KPartition best{1, 0};
    double best_cost = 1e30;
    for (int s = 1; s <= kMaxSplitsNarrow; ++s) {
        const int per = (ktiles + s - 1) / s;
        if (s > 1 && per < 8) break;
        const int rounds = (tiles * s + ncu - 1) / ncu;
        const double cost = rounds * (per + 8.0 + (s > 1 ? 8.0 : 0.0)) + (s > 1 ? 0.02 * s * tiles : 0.0);
        if (cost < best_cost - 1e-9) { best_cost = cost; best = KPartition{s, 0}; }
    }
    return best;
}

// Gate/up GEMM with few rows: one row of tiles has only I / 128 workgroups (112 for I = 14336), and a
// workgroup cannot keep enough weight bytes in flight to make up for the idle CUs.  Up to 128 rows
// the K range is therefore split over 2..4 workgroups per tile, which write fp32 partial sums of
// gate and up; the SwiGLU moves to the reducing kernel.  0 = not used (fused epilogue instead).
// Measured at C=4096, I=14336 (GEMM + reduction against the fused 128-row GEMM): 53 / 72 us at 16
// rows, 57 / 71 at 64, 65 / 73 at 128; at 184 and 256 rows the partial sums (229 KB per row, written
// and read) cost what the split gains.
constexpr int64_t kGateUpSplitMaxRows = BM / 2;
inline int gate_up_splits(int64_t rows, int64_t C, int64_t I, int ncu) {
    if (rows > kGateUpSplitMaxRows) return 0;
    const int64_t tiles_n = (I + BN / 2 - 1) / (BN / 2), ktiles = (C + BK - 1) / BK;
    int64_t s = std::min<int64_t>(4, ncu / std::max<int64_t>(tiles_n, 1));
    while (s > 1 && ktiles / s < 8) --s;
    return s >= 2 ? (int)s : 0;
}
inline size_t gate_up_partial_bytes(int64_t R, int64_t C, int64_t I, int ncu) {
    // sized for the largest row count that takes this path, so that a bound covers every smaller count
    const int64_t rows = std::min<int64_t>(R, kGateUpSplitMaxRows);
    const int s = gate_up_splits(rows, C, I, ncu);
    const int64_t tiles_n = (I + BN / 2 - 1) / (BN / 2);
    return s ? (size_t)s * (size_t)rows * (size_t)tiles_n * BN * 4 : 0;
}

// Leading dimension of the transposed copies ([columns][rows]): rows rounded up to 64 elements, so that every
// row of a copy starts on a 128-byte line (with a multiple of 8 only, each 128-byte piece the GEMMs load
// straddles two lines: the weight-gradient GEMMs ran 11-23 % slower at such row counts).
inline int64_t ld_transposed(int64_t R) { return (R + 63) / 64 * 64; }

struct SavedLayout { size_t off[8]; size_t total; };
inline SavedLayout saved_layout(int64_t R, int64_t C, int64_t I) {
    SavedLayout L;
    size_t o = 0;
    L.off[0] = o; o += align_up((size_t)R * C * 2);
    L.off[1] = o; o += align_up((size_t)R * C * 2);
    L.off[2] = o; o += align_up((size_t)R * 4);
    L.off[3] = o; o += align_up((size_t)R * I * 2);
    L.off[4] = o; o += align_up((size_t)R * I * 2);
    L.off[5] = o; o += align_up((size_t)R * I * 2);
    L.off[6] = o; o += align_up((size_t)C * ld_transposed(R) * 2);
    L.off[7] = o; o += align_up((size_t)I * ld_transposed(R) * 2);
    L.total = o;
    return L;
}

struct FwdWs { size_t xn, rstd, h, partial, gu_partial, status, total; };
inline FwdWs fwd_ws(int64_t R, int64_t C, int64_t I, bool has_saved, int ncu) {
    FwdWs w; size_t o = 0;
    w.xn = o;   if (!has_saved) o += align_up((size_t)R * C * 2);
    w.rstd = o; if (!has_saved) o += align_up((size_t)R * 4);
    w.h = o;    if (!has_saved) o += align_up((size_t)R * I * 2);
    // a buffer sized for R_max rows must do for every smaller count: the 128-row variant (up to
    // 256 rows) may use more slabs than the 256-row tiles
    const size_t slab_rows = std::max<size_t>((size_t)kMaxSplits * R, (size_t)kMaxSplitsNarrow * std::min<int64_t>(R, 256));
    w.partial = o; o += align_up(slab_rows * C * 4);
    w.gu_partial = o; o += align_up(gate_up_partial_bytes(R, C, I, ncu));
    w.status = o; o += 256;              // verdict of SKIPFFN_FLAG_VALIDATE_IDX
    w.total = o;
    return w;
}

struct BwdWs { size_t dy, dyT, dg, du, dgT, duT, partial, gainp, status, total; };
inline BwdWs bwd_ws(int64_t R, int64_t C, int64_t I) {
    BwdWs w; size_t o = 0;
    w.dy = o; o += align_up((size_t)R * C * 2);
    w.dyT = o; o += align_up((size_t)C * ld_transposed(R) * 2);
    w.dg = o; o += align_up((size_t)R * I * 2);
    w.du = o; o += align_up((size_t)R * I * 2);
    w.dgT = o; o += align_up((size_t)I * ld_transposed(R) * 2);
    w.duT = o; o += align_up((size_t)I * ld_transposed(R) * 2);
    w.partial = o; o += align_up((size_t)kMaxSplits * R * C * 4);
    w.gainp = o; o += align_up(gain_partial_bytes(R, C));
    w.status = o; o += 256;              // verdict of SKIPFFN_FLAG_VALIDATE_IDX
    w.total = o;
    return w;
}

}  // namespace skipffn
