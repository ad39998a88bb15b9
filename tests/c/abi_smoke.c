/* Plain C99 caller of the host-side entry points: packs the fully connected
 * 4-rank graph, builds the AllReduce schedule of configuration 1 and prints
 * what a test then checks.  No GPU call is made. */
#include <stdio.h>
#include <stdlib.h>

#include "blink.h"

int main(void) {
    int32_t src[12], dst[12];
    double cap[12];
    int m = 0;
    for (int u = 0; u < 4; ++u)
        for (int v = 0; v < 4; ++v)
            if (u != v) {
                src[m] = u;
                dst[m] = v;
                cap[m] = 1.0;
                ++m;
            }
    blink_trees_t* trees = NULL;
    blink_status_t st = blink_pack_trees(4, m, src, dst, cap, 0, 0.05, 0.05, &trees);
    if (st != BLINK_OK) {
        fprintf(stderr, "pack: %s\n", blink_strerror(st));
        return 1;
    }
    blink_schedule_t* sched = NULL;
    st = blink_make_schedule(trees, BLINK_OP_ALLREDUCE, (size_t)1 << 20, (size_t)1 << 16, BLINK_FUSE_EDGE, &sched);
    if (st != BLINK_OK) {
        fprintf(stderr, "schedule: %s\n", blink_strerror(st));
        return 1;
    }
    uint64_t bounds[17];
    blink_schedule_get_bounds(sched, bounds);
    size_t n_steps = blink_schedule_num_steps(sched);
    blink_step_t* steps = (blink_step_t*)malloc(n_steps * sizeof *steps);
    blink_schedule_get_steps(sched, steps);
    unsigned long long covered = 0;
    for (size_t i = 0; i < n_steps; ++i)
        if (steps[i].kind == BLINK_STEP_COPY && steps[i].dst == 3) covered += steps[i].len;
    double slow, fast;
    st = blink_hybrid_split(700.0, 10.0, 25.0, 0.0, &slow, &fast);
    blink_schedule_t* none = NULL;
    const int bad = (int)blink_make_schedule(trees, BLINK_OP_ALLREDUCE, 16, 0, BLINK_FUSE_EDGE, &none);
    printf("trees %d rate %.1f steps %zu bounds %llu %llu %llu %llu copied_into_rank3 %llu split %.1f %.1f bad %d\n",
           blink_trees_count(trees), blink_trees_rate(trees), n_steps, (unsigned long long)bounds[0],
           (unsigned long long)bounds[1], (unsigned long long)bounds[2], (unsigned long long)bounds[3], covered,
           slow, fast, bad);
    free(steps);
    blink_schedule_free(sched);
    blink_trees_free(trees);
    return st == BLINK_OK ? 0 : 1;
}
