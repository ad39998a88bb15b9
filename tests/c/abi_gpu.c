/* Plain C99 caller of the execution half of the C ABI: device buffers from the
 * HIP runtime's C interface, blink_pack_trees -> blink_make_schedule ->
 * blink_allreduce (every fusion level, and the entry point that allocates
 * nothing) -> copy back, compared with the closed form of an integer sum; then
 * blink_broadcast.  Needs a GPU.  Prints "ok <checked elements>" on success. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "blink.h"

/* the few entry points of the HIP runtime's C interface used here */
int hipSetDevice(int device);
int hipMalloc(void** ptr, size_t size);
int hipFree(void* ptr);
int hipMemcpy(void* dst, const void* src, size_t bytes, int kind);
int hipDeviceSynchronize(void);
enum { kHostToDevice = 1, kDeviceToHost = 2 };

#define K 4
#define N 1000003u

static int check(int hip_status, const char* what) {
    if (hip_status != 0) fprintf(stderr, "%s failed with HIP status %d\n", what, hip_status);
    return hip_status != 0;
}

int main(void) {
    int32_t src[K * (K - 1)], dst[K * (K - 1)];
    double cap[K * (K - 1)];
    int m = 0;
    for (int u = 0; u < K; ++u)
        for (int v = 0; v < K; ++v)
            if (u != v) {
                src[m] = u;
                dst[m] = v;
                cap[m] = 1.0;
                ++m;
            }
    blink_trees_t* trees = NULL;
    blink_status_t st = blink_pack_trees(K, m, src, dst, cap, 1, 0.05, 0.05, &trees);
    if (st != BLINK_OK) {
        fprintf(stderr, "pack: %s\n", blink_strerror(st));
        return 1;
    }
    if (check(hipSetDevice(0), "hipSetDevice")) return 1;
    int32_t* host = (int32_t*)malloc(N * sizeof *host);
    void* bufs[K];
    for (int r = 0; r < K; ++r)
        if (check(hipMalloc(&bufs[r], N * sizeof *host), "hipMalloc")) return 1;
    unsigned long long checked = 0;
    /* pass 0..2: blink_allreduce with fusion EDGE, NODE, TREE; pass 3: blink_allreduce_noalloc (TREE); pass 4: broadcast */
    for (int pass = 0; pass < 5; ++pass) {
        for (int r = 0; r < K; ++r) {
            for (unsigned j = 0; j < N; ++j) host[j] = (int32_t)((r + 1) * (int)(j % 1000u + 1u));
            if (check(hipMemcpy(bufs[r], host, N * sizeof *host, kHostToDevice), "hipMemcpy")) return 1;
        }
        const blink_fusion_t fusion = pass == 0 ? BLINK_FUSE_EDGE : (pass == 1 ? BLINK_FUSE_NODE : BLINK_FUSE_TREE);
        const blink_op_t op = pass == 4 ? BLINK_OP_BROADCAST : BLINK_OP_ALLREDUCE;
        blink_schedule_t* sched = NULL;
        st = blink_make_schedule(trees, op, N, 65536, fusion, &sched);
        if (st != BLINK_OK) {
            fprintf(stderr, "schedule: %s\n", blink_strerror(st));
            return 1;
        }
        if (pass < 3)
            st = blink_allreduce(bufs, K, N, BLINK_INT32, sched, NULL);
        else if (pass == 3)
            st = blink_allreduce_noalloc(bufs, K, N, BLINK_INT32, sched, NULL);
        else
            st = blink_broadcast(bufs, K, N, BLINK_INT32, sched, NULL);
        if (st != BLINK_OK) {
            fprintf(stderr, "pass %d: %s\n", pass, blink_strerror(st));
            return 1;
        }
        if (check(hipDeviceSynchronize(), "hipDeviceSynchronize")) return 1;
        blink_progress_t progress;
        if (blink_schedule_status(sched, &progress) != BLINK_OK || progress.state != 0) {
            fprintf(stderr, "pass %d: a wait was abandoned\n", pass);
            return 1;
        }
        for (int r = 0; r < K; ++r) {
            if (check(hipMemcpy(host, bufs[r], N * sizeof *host, kDeviceToHost), "hipMemcpy")) return 1;
            for (unsigned j = 0; j < N; ++j) {
                /* allreduce: (1+2+3+4) * v; broadcast from rank 1: 2 * v */
                const int32_t want = (int32_t)((pass == 4 ? 2 : K * (K + 1) / 2) * (int)(j % 1000u + 1u));
                if (host[j] != want) {
                    fprintf(stderr, "pass %d rank %d element %u: %d, expected %d\n", pass, r, j, host[j], want);
                    return 1;
                }
            }
            checked += N;
        }
        blink_schedule_free(sched);
    }
    for (int r = 0; r < K; ++r) hipFree(bufs[r]);
    free(host);
    blink_trees_free(trees);
    printf("ok %llu\n", checked);
    return 0;
}
