// Tile plan: pure integer host code (section 3.1 of the paper: T x T tiles with clamped edge tiles,
// one task per output tile, ceil(K/T) steps per task; Algorithm 1 "decode": id = i * n_j + j).
#include "common.h"

extern "C" {

int tgemm_plan(int64_t M, int64_t N, int64_t K, int32_t T, tgemm_task* out, int64_t cap, int64_t* n_tasks)
{
    if (M < 0 || N < 0 || K < 0 || T <= 0) return tg::fail(TGEMM_EARG, "tgemm_plan: bad sizes");
    if (!n_tasks || cap < 0 || (cap > 0 && !out)) return tg::fail(TGEMM_EARG, "tgemm_plan: bad output arguments");
    const int64_t n_i = (M + T - 1) / T, n_j = (N + T - 1) / T, n_k = (K + T - 1) / T;
    *n_tasks = n_i * n_j;
    for (int64_t id = 0; id < n_i * n_j && id < cap; ++id) {
        tgemm_task& t = out[id];
        t.id = id;
        t.i = id / n_j;
        t.j = id % n_j;
        t.r0 = t.i * T;
        t.r1 = t.r0 + T < M ? t.r0 + T : M;
        t.c0 = t.j * T;
        t.c1 = t.c0 + T < N ? t.c0 + T : N;
        t.n_k = n_k;
    }
    return TGEMM_OK;
}

int tgemm_task_order(int64_t n_i, int64_t n_j, int32_t order, int64_t strip, int64_t* out_ids)
{
    if (n_i < 0 || n_j < 0 || (n_i * n_j > 0 && !out_ids)) return tg::fail(TGEMM_EARG, "tgemm_task_order: bad argument");
    if (order != TGEMM_ORDER_SERPENTINE && order != TGEMM_ORDER_ROW_MAJOR && order != TGEMM_ORDER_STRIPS)
        return tg::fail(TGEMM_EARG, "tgemm_task_order: unknown order %d", order);
    int64_t w = 0;
    if (order == TGEMM_ORDER_STRIPS) {
        if (strip < 1) return tg::fail(TGEMM_EARG, "tgemm_task_order: strip width %lld", (long long)strip);
        int64_t s = 0;
        for (int64_t j0 = 0; j0 < n_j; j0 += strip, ++s) {
            const int64_t j1 = j0 + strip < n_j ? j0 + strip : n_j;
            for (int64_t ii = 0; ii < n_i; ++ii) {
                const int64_t i = (s & 1) ? n_i - 1 - ii : ii;
                for (int64_t j = j0; j < j1; ++j) out_ids[w++] = i * n_j + j;
            }
        }
        return TGEMM_OK;
    }
    for (int64_t i = 0; i < n_i; ++i) {
        const bool back = (order == TGEMM_ORDER_SERPENTINE) && (i & 1);
        for (int64_t jj = 0; jj < n_j; ++jj) {
            const int64_t j = back ? n_j - 1 - jj : jj;
            out_ids[w++] = i * n_j + j;
        }
    }
    return TGEMM_OK;
}

}  // extern "C"
