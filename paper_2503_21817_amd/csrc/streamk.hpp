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
#pragma once

#if defined(__HIPCC__)
#define SKIPFFN_HD __host__ __device__
#else
#define SKIPFFN_HD
#endif

namespace skipffn {

struct StreamKPlan { int g, kt, nbg, q, a, rem, nr, qr; };
constexpr int kStreamKMaxAligned = 6;            // at most 6 + 2 partial slabs per tile

SKIPFFN_HD inline StreamKPlan streamk_plan(int g, int kt, int nbg) {
    StreamKPlan p;
    p.g = g; p.kt = kt; p.nbg = nbg;
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
    int c = p.a;
    if (p.rem > 0) c += ((i + 1) * p.rem - 1) / p.qr - (i * p.rem) / p.qr + 1;
    return c;
}

// The work of workgroup j (0 <= j < nbg) of a group, one segment at a time:
//   StreamKIter it = streamk_begin(p, j);  StreamKSeg s;  while (streamk_next(p, it, s)) ...
// A segment is K slabs [kb, ke) of tile i, accumulated into partial slab `slot` of that tile.
struct StreamKSeg { int i, kb, ke, slot; };
struct StreamKIter { int j, u, u_end; };
SKIPFFN_HD inline StreamKIter streamk_begin(const StreamKPlan& p, int j) {
    StreamKIter it;
    it.j = j;
    if (j < p.a * p.g) {                 // aligned chunk: one pseudo-unit
        it.u = 0; it.u_end = 1;
    } else {
        const int rj = j - p.a * p.g;
        if (rj >= p.nr) { it.u = 0; it.u_end = 0; return it; }
        it.u = rj * p.qr;
        it.u_end = it.u + p.qr;
        if (it.u_end > p.g * p.rem) it.u_end = p.g * p.rem;
    }
    return it;
}
SKIPFFN_HD inline bool streamk_next(const StreamKPlan& p, StreamKIter& it, StreamKSeg& s) {
    if (it.u >= it.u_end) return false;
    if (it.j < p.a * p.g) {
        const int c = it.j / p.g;
        s.i = it.j - c * p.g;
        s.kb = c * p.q;
        s.ke = s.kb + p.q;
        s.slot = c;
        it.u = it.u_end;
        return true;
    }
    const int rj = it.j - p.a * p.g;
    s.i = it.u / p.rem;
    const int k0 = it.u - s.i * p.rem;
    int len = p.rem - k0;
    if (len > it.u_end - it.u) len = it.u_end - it.u;
    s.slot = p.a + rj - (s.i * p.rem) / p.qr;
    s.kb = p.a * p.q + k0;
    s.ke = s.kb + len;
    it.u += len;
    return true;
}

}  // namespace skipffn
