// Prints optimistic_keep(K, prefix, n_items) of the planner for the triples given on the command
// line (K prefix n_items ...), one value per line.  Host-only: the planner header has no HIP in it.
#include <cstdio>
#include <cstdlib>

#include "st_plan.h"

int main(int argc, char** argv)
{
    for (int i = 1; i + 2 < argc; i += 3)
        printf("%d\n", st::optimistic_keep(atoi(argv[i]), atoll(argv[i + 1]), atoll(argv[i + 2])));
    return 0;
}
