// Host check of the buffer carving and K-split planning (csrc/layout.hpp), meant to be built with
// -fsanitize=address,undefined: every section of `saved` and of the two workspaces is 256-byte
// aligned, the sections are disjoint, in order and large enough for what the kernels put there,
// totals never decrease as the row bound grows, and every K partition the planner picks stays
// within the partial-slab budget the workspaces are sized for.  A byte map of each buffer is
// painted section by section, so an overlap or an overrun is also a sanitizer report.
// Prints "ok <cases>" or the first violation.
#include <cstdio>
#include <cstdlib>
#include <vector>
#include "../../paper_2503_21817_amd/csrc/layout.hpp"
using namespace skipffn;

static int fail(const char* what, long R, long C, long I, int ncu) {
    printf("%s at R=%ld C=%ld I=%ld ncu=%d\n", what, R, C, I, ncu);
    return 1;
}

// paint [off, off + bytes) of a map scaled down by `unit` bytes per cell; returns false on overlap
static bool paint(std::vector<unsigned char>& map, size_t off, size_t bytes, size_t unit) {
    if (bytes == 0) return true;
    const size_t a = off / unit, b = (off + bytes - 1) / unit;
    for (size_t i = a; i <= b; ++i) {
        if (map.at(i)) return false;
        map[i] = 1;
    }
    return true;
}

int main() {
    long cases = 0;
    const long Cs[] = {8, 256, 264, 4096}, Is[] = {8, 688, 14336};
    const long Rs[] = {0, 1, 7, 8, 31, 128, 129, 184, 256, 257, 1000, 1472, 2560, 2944, 9623, 16384};
    const int ncus[] = {256, 304, 64, 1};
    for (int ncu : ncus)
        for (long C : Cs)
            for (long I : Is) {
                size_t prev_sv = 0, prev_fw[2] = {0, 0}, prev_bw = 0;
                for (long R : Rs) {
                    const size_t unit = 256;
                    // ---- saved
                    const SavedLayout L = saved_layout(R, C, I);
                    const size_t need[8] = {(size_t)R * C * 2, (size_t)R * C * 2, (size_t)R * 4, (size_t)R * I * 2,
                                            (size_t)R * I * 2, (size_t)R * I * 2, (size_t)C * ld_transposed(R) * 2,
                                            (size_t)I * ld_transposed(R) * 2};
                    std::vector<unsigned char> map(L.total / unit + 2, 0);
                    for (int k = 0; k < 8; ++k) {
                        if (L.off[k] % 256) return fail("saved section not aligned", R, C, I, ncu);
                        if (L.off[k] + need[k] > L.total) return fail("saved section past the end", R, C, I, ncu);
                        if (!paint(map, L.off[k], need[k], unit)) return fail("saved sections overlap", R, C, I, ncu);
                    }
                    if (ld_transposed(R) % 64 || ld_transposed(R) < R) return fail("transposed leading dimension", R, C, I, ncu);
                    if (L.total < prev_sv) return fail("saved size decreases", R, C, I, ncu);
                    prev_sv = L.total;
                    // ---- forward workspace, with and without a saved buffer
                    for (int hs = 0; hs < 2; ++hs) {
                        const FwdWs W = fwd_ws(R, C, I, hs != 0, ncu);
                        std::vector<unsigned char> m2(W.total / unit + 2, 0);
                        const size_t slab_rows = std::max<size_t>((size_t)kMaxSplits * R, (size_t)kMaxSplitsNarrow * std::min<long>(R, 256));
                        const size_t offs[6] = {W.xn, W.rstd, W.h, W.partial, W.gu_partial, W.status};
                        const size_t sz[6] = {hs ? 0 : (size_t)R * C * 2, hs ? 0 : (size_t)R * 4, hs ? 0 : (size_t)R * I * 2,
                                              slab_rows * C * 4, gate_up_partial_bytes(R, C, I, ncu), 8};
                        for (int k = 0; k < 6; ++k) {
                            if (offs[k] % 256) return fail("forward workspace section not aligned", R, C, I, ncu);
                            if (offs[k] + sz[k] > W.total) return fail("forward workspace section past the end", R, C, I, ncu);
                            if (!paint(m2, offs[k], sz[k], unit)) return fail("forward workspace sections overlap", R, C, I, ncu);
                        }
                        if (W.total < prev_fw[hs]) return fail("forward workspace size decreases", R, C, I, ncu);
                        prev_fw[hs] = W.total;
                    }
                    // ---- backward workspace
                    {
                        const BwdWs W = bwd_ws(R, C, I);
                        std::vector<unsigned char> m3(W.total / unit + 2, 0);
                        const size_t offs[9] = {W.dy, W.dyT, W.dg, W.du, W.dgT, W.duT, W.partial, W.gainp, W.status};
                        const size_t sz[9] = {(size_t)R * C * 2, (size_t)C * ld_transposed(R) * 2, (size_t)R * I * 2, (size_t)R * I * 2,
                                              (size_t)I * ld_transposed(R) * 2, (size_t)I * ld_transposed(R) * 2,
                                              (size_t)kMaxSplits * R * C * 4, gain_partial_bytes(R, C), 8};
                        for (int k = 0; k < 9; ++k) {
                            if (offs[k] % 256) return fail("backward workspace section not aligned", R, C, I, ncu);
                            if (offs[k] + sz[k] > W.total) return fail("backward workspace section past the end", R, C, I, ncu);
                            if (!paint(m3, offs[k], sz[k], unit)) return fail("backward workspace sections overlap", R, C, I, ncu);
                        }
                        if (W.total < prev_bw) return fail("backward workspace size decreases", R, C, I, ncu);
                        prev_bw = W.total;
                    }
                    // ---- K partitions of the down GEMM (K = I) and of the dXn GEMM (K = 2 I)
                    if (R > 0) {
                        const int tiles_n = (int)((C + BN - 1) / BN);
                        for (int pairs = 1; pairs <= 2; ++pairs)
                            for (int forced = 0; forced < 2; ++forced) {
                                const int tiles_m = (int)((R + BM - 1) / BM), ktiles = pairs * (int)((I + BK - 1) / BK);
                                const KPartition kp = choose_k_partition(tiles_m, tiles_n, ktiles, forced != 0, ncu);
                                if (kp.splits < 1 || kp.splits > kMaxSplits) return fail("split factor out of range", R, C, I, ncu);
                                if (kp.sk_nbg > 0) {
                                    if (kp.sk_nbg * tiles_n > ncu) return fail("balanced split larger than the chip", R, C, I, ncu);
                                    const StreamKPlan p = streamk_plan(tiles_m, ktiles, kp.sk_nbg);
                                    for (int i = 0; i < tiles_m; ++i)
                                        if (streamk_count(p, i) > kMaxSplits) return fail("more partial slabs than the workspace holds", R, C, I, ncu);
                                }
                            }
                        if (R <= 256) {
                            const int tiles_m = (int)((R + BM / 2 - 1) / (BM / 2)), ktiles = (int)((I + BK - 1) / BK);
                            const KPartition kp = choose_k_split_narrow(tiles_m, tiles_n, ktiles, ncu);
                            if (kp.splits < 1 || kp.splits > kMaxSplitsNarrow || kp.sk_nbg != 0) return fail("narrow split out of range", R, C, I, ncu);
                        }
                        const int gs = gate_up_splits(R, C, I, ncu);
                        if (gs < 0 || gs == 1 || gs > 4 || (R > BM / 2 && gs != 0)) return fail("gate/up split out of range", R, C, I, ncu);
                    }
                    ++cases;
                }
            }
    printf("ok %ld\n", cases);
    return 0;
}
