// Host-side walk of the work-item space of the LDS-patch kernels: for every grid size 1..40 (a
// partition of that many CUs) and a range of tile counts, the workgroups of a launch, each
// stepping through its items the way the kernels do, must visit every (split, channel block, row
// tile) exactly once.  Prints "ok <cases>" or the first failure.
#include <cstdio>
#include <vector>

#include "patch_items.h"

using namespace sgprs;

struct Space { int n_mtiles, n_ntiles, splits, xcd_groups, n_slots; };

int main()
{
    long cases = 0;
    for (int n_ntiles : {1, 2, 3, 4, 8})
        for (int splits : {1, 2})
            for (int n_mtiles = 1; n_mtiles <= 70; ++n_mtiles) {
                Space a{n_mtiles, n_ntiles, splits, 0, 0};
                patch_index_space(n_mtiles, n_ntiles, splits, &a.xcd_groups, &a.n_slots);
                for (int grid = 1; grid <= 40; ++grid) {
                    int g = grid < a.n_slots ? grid : a.n_slots;
                    if (a.xcd_groups && g >= 8) g -= g % 8;  // as the launchers do
                    std::vector<int> seen((size_t)n_mtiles * n_ntiles * splits, 0);
                    for (int b = 0; b < g; ++b) {
                        int item = b;
                        PatchItem cur = next_item(a, item, g);
                        int guard = 0;
                        while (cur.valid) {
                            if (cur.mtile < 0 || cur.mtile >= n_mtiles || cur.ntile < 0 || cur.ntile >= n_ntiles || cur.split < 0 ||
                                cur.split >= splits) {
                                printf("FAIL out of range: ntiles %d splits %d mtiles %d grid %d item %d\n", n_ntiles, splits, n_mtiles, g, item);
                                return 1;
                            }
                            ++seen[((size_t)cur.mtile * n_ntiles + cur.ntile) * splits + cur.split];
                            int nxt_index = item + g;
                            const PatchItem nxt = next_item(a, nxt_index, g);
                            if (!nxt.valid) break;
                            item = nxt_index;
                            cur = nxt;
                            if (++guard > 100000) { printf("FAIL endless walk\n"); return 1; }
                        }
                    }
                    for (size_t i = 0; i < seen.size(); ++i)
                        if (seen[i] != 1) {
                            printf("FAIL ntiles %d splits %d mtiles %d grid %d: tile %zu visited %d times\n", n_ntiles, splits, n_mtiles, g, i,
                                   seen[i]);
                            return 1;
                        }
                    ++cases;
                }
            }
    printf("ok %ld\n", cases);
    return 0;
}
