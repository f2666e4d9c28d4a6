/* The C ABI used from plain C99: includes the header, prints the struct sizes the Python binding
 * mirrors, and calls host-only entry points (no GPU needed). */
#include <stdio.h>
#include <stdlib.h>

#include "tgemm.h"

int main(void)
{
    int64_t ids[12];
    int32_t popped[1000];
    int i, rc;
    tgemm_balance bal;
    tgemm_segment segs[512];
    printf("sizes %zu %zu %zu %zu %zu %zu %zu\n", sizeof(tgemm_opts), sizeof(tgemm_task), sizeof(tgemm_stats), sizeof(tgemm_trace_rec),
           sizeof(tgemm_mlp_trace_rec), sizeof(tgemm_balance), sizeof(tgemm_segment));
    rc = tgemm_task_order(3, 4, TGEMM_ORDER_SERPENTINE, 1, ids);
    if (rc != TGEMM_OK) { printf("task_order failed: %s\n", tgemm_last_error()); return 1; }
    printf("order");
    for (i = 0; i < 12; ++i) printf(" %lld", (long long)ids[i]);
    printf("\n");
    rc = tgemm_queue_selftest(1000, 2, 2, popped);
    if (rc != TGEMM_OK) { printf("queue selftest failed: %s\n", tgemm_last_error()); return 1; }
    for (i = 0; i < 1000; ++i)
        if (popped[i] != 1) { printf("id %d popped %d times\n", i, popped[i]); return 1; }
    rc = tgemm_balance_plan(8000, 8000, 8000, 1024, TGEMM_F32, 256, 0, &bal, segs, 512);
    if (rc != TGEMM_OK) { printf("balance plan failed: %s\n", tgemm_last_error()); return 1; }
    printf("balance %d %d %d %d\n", (int)bal.applies, (int)bal.whole_round_tiles, (int)bal.tail_tiles, (int)bal.n_segments);
    rc = tgemm_task_order(3, 4, 99, 1, ids);
    printf("bad order -> %d (%s)\n", rc, tgemm_strerror(rc));
    return rc == TGEMM_OK;
}
