// Balanced split of the K range of a GEMM whose result leaves through fp32 partial slabs.
// Plain C++ (no HIP constructs): shared by the GEMM kernel, the reducing kernels and the host.
//
// When a GEMM has fewer output tiles than the chip has CUs, the K range of its tiles is cut so
// that every workgroup gets the same number of slabs, instead of an integer split factor that
// leaves CUs idle.  All m-tiles of one n-tile form a group served by `nbg` workgroups; a group
// of g tiles with kt slabs each is cut into
//   * `a` aligned chunks of q slabs per tile (workgroups 0 .. a*g-1 of the group: the g tiles of
//     a chunk walk the same K range at the same time, so they share the streamed operand in
//     L2), and
//   * the rest [a*q, kt) of every tile, laid end to end (g * rem slabs) and cut into nr pieces
//     of qr >= rem slabs (workgroups a*g .. a*g+nr-1); a piece runs one segment per tile it
//     touches.
// Tile i of a group receives streamk_count() partial slabs: slots 0..a-1 from the aligned
// chunks, then one or two from the remainder pieces.  The reducing kernels add exactly those.
//
// A group with more tiles than workgroups (g > nbg) first gives every workgroup `full` = g / nbg
// whole tiles (workgroup j: tiles j, j + nbg, ...: one partial slab each, and the nbg tiles of a
// round walk the K range together); the scheme above then applies to the gr = g - full * nbg tiles
// that are left.  (Letting every workgroup walk an equal share of all g tiles end to end balances
// just as well, but puts the workgroups of a group at different K positions: the streamed operand
// is then fetched once per workgroup instead of once per group - measured 13-20 % slower on the
// down and dXn GEMMs at 17 and 33 tile rows.)
#pragma once

#if defined(__HIPCC__)
#define SKIPFFN_HD __host__ __device__
#else
#define SKIPFFN_HD
#endif

namespace skipffn {

struct StreamKPlan { int g, kt, nbg, q, a, rem, nr, qr, full, base, gr; };
constexpr int kStreamKMaxAligned = 6;            // at most 6 + 2 partial slabs per tile

SKIPFFN_HD inline StreamKPlan streamk_plan(int g, int kt, int nbg) {
    StreamKPlan p;
    p.g = g; p.kt = kt; p.nbg = nbg;
    p.full = g > nbg ? g / nbg : 0;
    p.base = p.full * nbg;
    p.gr = g - p.base;
    g = p.gr;                                                // the split applies to these tiles
    if (g == 0) { p.q = kt > 0 ? kt : 1; p.a = 0; p.rem = 0; p.nr = 0; p.qr = 1; return p; }
    const int q_bal = (g * kt + nbg - 1) / nbg;
    const int q_min = (kt + kStreamKMaxAligned - 1) / kStreamKMaxAligned;
    p.q = q_bal > q_min ? q_bal : q_min;
    if (p.q < 1) p.q = 1;
    p.a = kt / p.q;                                          // a * g <= nbg
    p.rem = kt - p.a * p.q;
    if (p.rem > 0) {
        const int want = (g * p.rem + p.q - 1) / p.q;       // <= g
        const int have = nbg - p.a * g;                      // >= 1 when rem > 0
        p.nr = want < have ? want : have;
        p.qr = (g * p.rem + p.nr - 1) / p.nr;                // rem <= qr <= q
    } else {
        p.nr = 0; p.qr = 1;
    }
    return p;
}

// number of partial slabs tile i (0 <= i < g) of a group receives
SKIPFFN_HD inline int streamk_count(const StreamKPlan& p, int i) {
    if (i < p.base) return 1;
    i -= p.base;
    int c = p.a;
    if (p.rem > 0) c += ((i + 1) * p.rem - 1) / p.qr - (i * p.rem) / p.qr + 1;
    return c;
}

// The work of workgroup j (0 <= j < nbg) of a group, one segment at a time:
//   StreamKIter it = streamk_begin(p, j);  StreamKSeg s;  while (streamk_next(p, it, s)) ...
// A segment is K slabs [kb, ke) of tile i, accumulated into partial slab `slot` of that tile.
struct StreamKSeg { int i, kb, ke, slot; };
struct StreamKIter { int j, u, u_end, f; };
SKIPFFN_HD inline StreamKIter streamk_begin(const StreamKPlan& p, int j) {
    StreamKIter it;
    it.j = j;
    it.f = 0;                            // whole tiles done so far
    if (j < p.a * p.gr) {                // aligned chunk: one pseudo-unit
        it.u = 0; it.u_end = 1;
    } else {
        const int rj = j - p.a * p.gr;
        if (rj >= p.nr) { it.u = 0; it.u_end = 0; return it; }
        it.u = rj * p.qr;
        it.u_end = it.u + p.qr;
        if (it.u_end > p.gr * p.rem) it.u_end = p.gr * p.rem;
    }
    return it;
}
SKIPFFN_HD inline bool streamk_next(const StreamKPlan& p, StreamKIter& it, StreamKSeg& s) {
    if (it.f < p.full) {                 // a whole tile of this workgroup's own
        s.i = it.f * p.nbg + it.j;
        s.kb = 0; s.ke = p.kt; s.slot = 0;
        ++it.f;
        return true;
    }
    if (it.u >= it.u_end) return false;
    if (it.j < p.a * p.gr) {
        const int c = it.j / p.gr;
        s.i = p.base + it.j - c * p.gr;
        s.kb = c * p.q;
        s.ke = s.kb + p.q;
        s.slot = c;
        it.u = it.u_end;
        return true;
    }
    const int rj = it.j - p.a * p.gr;
    const int ir = it.u / p.rem;         // index among the tiles that are split
    s.i = p.base + ir;
    const int k0 = it.u - ir * p.rem;
    int len = p.rem - k0;
    if (len > it.u_end - it.u) len = it.u_end - it.u;
    s.slot = p.a + rj - (ir * p.rem) / p.qr;
    s.kb = p.a * p.q + k0;
    s.ke = s.kb + len;
    it.u += len;
    return true;
}

}  // namespace skipffn
