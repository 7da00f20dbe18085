// Prints optimistic_keep(K, prefix, n_items) of the planner for the triples given on the command
// line (K prefix n_items ...), one value per line.  With "levels" as the first argument: for every
// triple (n_items K small_first) the number of levels and the end of the first one, as make_levels
// plans them for 1024 workgroups, regions of 64 entries and no seed pass.
// Host-only: the planner header has no HIP in it.
#include <cstdio>
#include <cstdlib>
#include <cstring>

#include "st_plan.h"

int main(int argc, char** argv)
{
    if (argc > 1 && strcmp(argv[1], "levels") == 0) {
        for (int i = 2; i + 2 < argc; i += 3) {
            st::Plan p;
            const int rc = st::make_levels(atoll(argv[i]), atoi(argv[i + 1]), 64, 1024, 512, 0, 2048, &p, true, atoi(argv[i + 2]) != 0);
            printf("%d %lld\n", rc == 0 ? p.n_levels : -1, rc == 0 ? (long long)p.level[0].end : -1LL);
        }
        return 0;
    }
    for (int i = 1; i + 2 < argc; i += 3)
        printf("%d\n", st::optimistic_keep(atoi(argv[i]), atoll(argv[i + 1]), atoll(argv[i + 2])));
    return 0;
}
