// Brute-force check of the balanced K split (csrc/streamk.hpp): for every (g, kt, nbg) in a
// range, every K slab of every tile is covered exactly once, slot numbers of a tile are
// 0..count-1 without repeats, counts stay within the partial-slab budget, and no workgroup
// gets more than q slabs beyond its whole tiles.  Prints "ok <cases>" or the first violation.
#include <cstdio>
#include <vector>
#include "../../paper_2503_21817_amd/csrc/streamk.hpp"
using namespace skipffn;

int main() {
    long cases = 0;
    for (int g = 1; g <= 40; ++g)
        for (int nbg = 1; nbg <= 40; ++nbg)
            for (int kt = 1; kt <= 300; kt += (kt < 70 ? 1 : 7)) {
                const StreamKPlan p = streamk_plan(g, kt, nbg);
                if (p.base + p.gr != g || p.gr < 0 || (g > nbg && p.gr >= nbg) || (g <= nbg && p.full != 0) ||
                    p.a * p.gr > nbg || p.a > kStreamKMaxAligned || (p.rem > 0 && (p.nr < 1 || p.a * p.gr + p.nr > nbg)) ||
                    (p.rem > 0 && p.qr < p.rem)) {
                    printf("bad plan g=%d kt=%d nbg=%d: q=%d a=%d rem=%d nr=%d qr=%d\n", g, kt, nbg, p.q, p.a, p.rem, p.nr, p.qr);
                    return 1;
                }
                std::vector<int> cover(g * kt, 0);
                std::vector<std::vector<int>> slots(g);
                for (int j = 0; j < nbg; ++j) {
                    StreamKIter it = streamk_begin(p, j);
                    StreamKSeg s;
                    int work = 0;
                    while (streamk_next(p, it, s)) {
                        if (s.i < 0 || s.i >= g || s.kb < 0 || s.ke > kt || s.kb >= s.ke) {
                            printf("bad segment g=%d kt=%d nbg=%d j=%d: i=%d [%d,%d)\n", g, kt, nbg, j, s.i, s.kb, s.ke);
                            return 1;
                        }
                        for (int k = s.kb; k < s.ke; ++k) cover[s.i * kt + k]++;
                        slots[s.i].push_back(s.slot);
                        work += s.ke - s.kb;
                    }
                    if (work > p.full * kt + (p.gr > 0 ? p.q : 0)) { printf("overload g=%d kt=%d nbg=%d j=%d: %d > q=%d\n", g, kt, nbg, j, work, p.q); return 1; }
                }
                for (int x = 0; x < g * kt; ++x)
                    if (cover[x] != 1) { printf("coverage g=%d kt=%d nbg=%d tile %d slab %d: %d\n", g, kt, nbg, x / kt, x % kt, cover[x]); return 1; }
                for (int i = 0; i < g; ++i) {
                    const int c = streamk_count(p, i);
                    if (c > kStreamKMaxAligned + 2 || (int)slots[i].size() != c) { printf("count g=%d kt=%d nbg=%d tile %d: count %d, segments %zu\n", g, kt, nbg, i, c, slots[i].size()); return 1; }
                    std::vector<int> seen(c, 0);
                    for (int sl : slots[i]) {
                        if (sl < 0 || sl >= c || seen[sl]) { printf("slot g=%d kt=%d nbg=%d tile %d: slot %d of %d\n", g, kt, nbg, i, sl, c); return 1; }
                        seen[sl] = 1;
                    }
                }
                ++cases;
            }
    printf("ok %ld\n", cases);
    return 0;
}
