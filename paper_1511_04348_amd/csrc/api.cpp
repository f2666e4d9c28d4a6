// C-ABI entry points: argument checks, pointer classification, dispatch to the in-core launch or
// the out-of-core tile engine.  See include/tgemm.h for the contract of every function.
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <mutex>
#include <thread>

#include "common.h"
#include "gemm_kernel.h"
#include "ms_queue.h"

namespace tg {

static thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

PtrKind classify_pointer(const void* p, int device)
{
    hipPointerAttribute_t at;
    memset(&at, 0, sizeof at);
    hipError_t e = hipPointerGetAttributes(&at, p);
    if (e != hipSuccess) {
        (void)hipGetLastError();   // unknown to HIP: ordinary pageable memory
        return PTR_PAGEABLE;
    }
    if (at.type == hipMemoryTypeDevice) return PTR_DEVICE;
    if (at.type == hipMemoryTypeHost) return PTR_PINNED;
    if (at.type == hipMemoryTypeManaged) return PTR_DEVICE;
    (void)device;
    return PTR_PAGEABLE;
}

// The library's own streams, four per device, created when a context first needs one and kept until
// the process ends: contexts that bring no streams of their own borrow these.  (Streams that are
// created and destroyed with every context end up sharing hardware queues after a few contexts --
// measured: an out-of-core step ran 1.5 times slower in a process that had destroyed a used
// context before -- because fetch, compute and write-back then queue behind each other.)  Contexts
// on one device therefore share streams; that adds ordering between them, never removes any.
static std::mutex g_stream_mu;
static hipStream_t g_streams[64][4] = {};
static hipError_t pooled_stream(int device, int s, hipStream_t* out)
{
    std::lock_guard<std::mutex> lock(g_stream_mu);
    if (!g_streams[device][s]) {
        hipError_t e = hipStreamCreateWithFlags(&g_streams[device][s], hipStreamNonBlocking);
        if (e != hipSuccess) { g_streams[device][s] = nullptr; return e; }
    }
    *out = g_streams[device][s];
    return hipSuccess;
}

// TGEMM_LOG=1 in the environment: one line per tgemm_run / mlp_* call on stderr.
void log_call(const char* what, const tgemm_ctx* ctx, int rc)
{
    static const bool on = [] { const char* v = getenv("TGEMM_LOG"); return v && *v && *v != '0'; }();
    if (!on) return;
    const tgemm_stats& s = ctx->stats;
    fprintf(stderr, "[tgemm] %s rc=%d %s wall %.3f ms kernel %.3f ms tasks %lld tile products %lld launches %lld slots %lld "
            "hits %lld misses %lld evictions %lld h2d %lld B d2h %lld B\n", what, rc, s.in_core ? "in-core" : "out-of-core",
            s.wall_ms, s.kernel_ms, (long long)s.n_tasks, (long long)s.n_tile_gemms, (long long)s.kernel_launches,
            (long long)s.n_slots, (long long)s.hits, (long long)s.misses, (long long)s.evictions, (long long)s.h2d_bytes,
            (long long)s.d2h_bytes);
}

static double now_ms()
{
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

static bool overlap(const void* a, size_t na, const void* b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

}  // namespace tg

using namespace tg;

extern "C" {

const char* tgemm_strerror(int code)
{
    switch (code) {
        case TGEMM_OK: return "ok";
        case TGEMM_EARG: return "invalid argument";
        case TGEMM_ENOMEM: return "out of memory";
        case TGEMM_EUNPINNED: return "host pointer is not page-locked";
        case TGEMM_EBUDGET: return "hbm_budget below the minimum working set";
        case TGEMM_EHIP: return "HIP runtime error";
        case TGEMM_ESTATE: return "call order violated";
        default: return "unknown error";
    }
}

const char* tgemm_last_error(void) { return g_err; }

int tgemm_create(tgemm_ctx** out, int device, void* const* streams, const tgemm_opts* opts)
{
    if (!out) return fail(TGEMM_EARG, "tgemm_create: out is NULL");
    *out = nullptr;
    int n_dev = 0;
    if (hipGetDeviceCount(&n_dev) != hipSuccess || n_dev <= 0) {
        (void)hipGetLastError();
        return fail(TGEMM_EHIP, "tgemm_create: no HIP device is visible");
    }
    if (device < 0 || device >= n_dev || device >= 64) return fail(TGEMM_EARG, "tgemm_create: device %d of %d", device, n_dev);
    tgemm_opts o;
    memset(&o, 0, sizeof o);
    o.affinity_core = -1;
    o.order = TGEMM_ORDER_STRIPS;
    if (opts) o = *opts;
    if (o.order != TGEMM_ORDER_SERPENTINE && o.order != TGEMM_ORDER_ROW_MAJOR && o.order != TGEMM_ORDER_STRIPS)
        return fail(TGEMM_EARG, "tgemm_create: unknown task order %d", o.order);
    if (o.strip_width < 0) return fail(TGEMM_EARG, "tgemm_create: strip_width %d", o.strip_width);
    if (o.kernel_config < 0 || o.kernel_config > 4)
        return fail(TGEMM_EARG, "tgemm_create: kernel_config %d", o.kernel_config);
    if (o.incore_schedule < 0 || o.incore_schedule > 2)
        return fail(TGEMM_EARG, "tgemm_create: incore_schedule %d", o.incore_schedule);
    if (o.rs_depth < 0 || o.rs_depth > 64) return fail(TGEMM_EARG, "tgemm_create: rs_depth %d (0 .. 64)", o.rs_depth);
    TG_HIP(hipSetDevice(device));
    {   // the static scratch array's address on this device, for the entry points that allocate nothing
        const int rc = static_scratch_resolve(device, nullptr);
        if (rc != TGEMM_OK) return rc;
    }
    tgemm_ctx* c = new (std::nothrow) tgemm_ctx();
    if (!c) return fail(TGEMM_ENOMEM, "tgemm_create: host allocation failed");
    c->device = device;
    c->opts = o;
    for (int s = 0; s < 4; ++s) {
        if (streams && streams[s]) {
            c->streams[s] = (hipStream_t)streams[s];
        } else {
            hipError_t e = pooled_stream(device, s, &c->streams[s]);
            if (e != hipSuccess) {
                tgemm_destroy(c);
                return fail(TGEMM_EHIP, "hipStreamCreate: %s", hipGetErrorString(e));
            }
        }
    }
    if (hipEventCreate(&c->ev_start) != hipSuccess || hipEventCreate(&c->ev_stop) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_fork, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming) != hipSuccess) {
        tgemm_destroy(c);
        return fail(TGEMM_EHIP, "hipEventCreate failed");
    }
    if (hipDeviceGetAttribute(&c->n_cus, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess) c->n_cus = 0;
    *out = c;
    return TGEMM_OK;
}

int tgemm_destroy(tgemm_ctx* ctx)
{
    if (!ctx) return TGEMM_OK;
    (void)hipSetDevice(ctx->device);
    for (int s = 0; s < 4; ++s)
        if (ctx->streams[s]) (void)hipStreamSynchronize(ctx->streams[s]);
    destroy_engine(ctx);
    if (ctx->ev_start) (void)hipEventDestroy(ctx->ev_start);
    if (ctx->ev_stop) (void)hipEventDestroy(ctx->ev_stop);
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
    sk_destroy(ctx->sk);
    delete ctx;
    return TGEMM_OK;
}

int tgemm_invalidate(tgemm_ctx* ctx, const void* host_base)
{
    if (!ctx) return fail(TGEMM_EARG, "tgemm_invalidate: ctx is NULL");
    if (!host_base) return fail(TGEMM_EARG, "tgemm_invalidate: host_base is NULL");
    // only tgemm_opts.keep_tiles lets tiles outlive a call; without it there is never anything to drop
    TG_HIP(hipSetDevice(ctx->device));
    for (int s = 0; s < 4; ++s) TG_HIP(hipStreamSynchronize(ctx->streams[s]));
    (void)invalidate_tiles(ctx, host_base);
    return TGEMM_OK;
}

int tgemm_sync(tgemm_ctx* ctx)
{
    if (!ctx) return fail(TGEMM_EARG, "tgemm_sync: ctx is NULL");
    TG_HIP(hipSetDevice(ctx->device));
    for (int s = 0; s < 4; ++s) TG_HIP(hipStreamSynchronize(ctx->streams[s]));
    if (ctx->kernel_timing_pending) {
        float ms = 0.f;
        TG_HIP(hipEventElapsedTime(&ms, ctx->ev_start, ctx->ev_stop));
        ctx->stats.kernel_ms = ms;
        ctx->kernel_timing_pending = false;
    }
    return TGEMM_OK;
}

int tgemm_run(tgemm_ctx* ctx, const void* A, const void* B, void* C,
              int64_t M, int64_t N, int64_t K, int32_t T, int32_t dtype, size_t hbm_budget)
{
    if (!ctx) return fail(TGEMM_EARG, "tgemm_run: ctx is NULL");
    if (M < 0 || N < 0 || K < 0) return fail(TGEMM_EARG, "tgemm_run: negative size (%lld,%lld,%lld)", (long long)M, (long long)N, (long long)K);
    if (T <= 0) return fail(TGEMM_EARG, "tgemm_run: tile size %d", T);
    if (dtype != TGEMM_F32 && dtype != TGEMM_BF16) return fail(TGEMM_EARG, "tgemm_run: unknown dtype %d", dtype);
    const int64_t LIM = (int64_t)1 << 30;
    if (M > LIM || N > LIM || K > LIM) return fail(TGEMM_EARG, "tgemm_run: dimension above 2^30");
    const double t0 = now_ms();
    memset(&ctx->stats, 0, sizeof ctx->stats);
    ctx->trace.clear();
    if (M == 0 || N == 0) return TGEMM_OK;
    if (!C) return fail(TGEMM_EARG, "tgemm_run: C is NULL");
    if (K > 0 && (!A || !B)) return fail(TGEMM_EARG, "tgemm_run: A or B is NULL");
    TG_HIP(hipSetDevice(ctx->device));
    const size_t es = dtype == TGEMM_F32 ? 4 : 2;
    const size_t bytes_a = (size_t)M * K * es, bytes_b = (size_t)K * N * es, bytes_c = (size_t)M * N * 4;
    if (K > 0 && (overlap(A, bytes_a, C, bytes_c) || overlap(B, bytes_b, C, bytes_c)))
        return fail(TGEMM_EARG, "tgemm_run: C overlaps an input");
    const PtrKind kc = classify_pointer(C, ctx->device);
    if (K == 0) {   // nothing to add; C keeps its value, wherever it lives
        if (kc == PTR_PAGEABLE) return fail(TGEMM_EUNPINNED, "tgemm_run: C is pageable host memory");
        return TGEMM_OK;
    }
    const PtrKind ka = classify_pointer(A, ctx->device), kb = classify_pointer(B, ctx->device);
    if (ka == PTR_PAGEABLE || kb == PTR_PAGEABLE || kc == PTR_PAGEABLE)
        return fail(TGEMM_EUNPINNED, "tgemm_run: %s%s%s not page-locked (use hipHostMalloc / pin_memory)",
                    ka == PTR_PAGEABLE ? "A " : "", kb == PTR_PAGEABLE ? "B " : "", kc == PTR_PAGEABLE ? "C " : "");
    if (ka != kb || ka != kc)
        return fail(TGEMM_EARG, "tgemm_run: A, B, C must be all device or all pinned host pointers");

    const int64_t n_i = (M + T - 1) / T, n_j = (N + T - 1) / T, n_k = (K + T - 1) / T;
    // task ids, the task queue and the launch grid are sized by the task count
    if (n_i * n_j > ((int64_t)1 << 31) || n_i * n_j * n_k > ((int64_t)1 << 40))
        return fail(TGEMM_EARG, "tgemm_run: %lld x %lld x %lld tiles: more than 2^31 tasks (or 2^40 tile products); use a larger T",
                    (long long)n_i, (long long)n_j, (long long)n_k);
    ctx->stats.n_tasks = n_i * n_j;
    ctx->stats.n_tile_gemms = n_i * n_j * n_k;

    if (ka == PTR_PINNED) {
        const int rc = run_out_of_core(ctx, A, B, (float*)C, M, N, K, T, dtype, hbm_budget);
        ctx->stats.wall_ms = now_ms() - t0;
        log_call("tgemm_run", ctx, rc);
        return rc;
    }

    // ---- in-core: one launch covers every task (Algorithm 1 with every tile an L1 hit)
    GemmDesc d;
    memset(&d, 0, sizeof d);
    d.A = A; d.B = B; d.C = (float*)C;
    d.lda = K; d.ldb = N; d.ldc = N;
    d.M = M; d.N = N; d.K = K; d.T = T;
    d.a_kcontig = 1; d.b_kcontig = 0;
    d.epilogue = EPI_AXPBY; d.alpha = 1.f; d.beta = 1.f;
    d.config = ctx->opts.kernel_config;
    hipStream_t st = ctx->streams[0];
    TG_HIP(hipEventRecord(ctx->ev_start, st));
    // fp32 with the automatic shape: the balanced schedule where the macro tiles leave a partial round
    // (it declines, having launched nothing, wherever it does not apply or would not gain)
    hipError_t e = hipErrorNotSupported;
    int launches = 1;
    if (ctx->opts.incore_schedule != TGEMM_SCHEDULE_ONE_LAUNCH) {
        e = launch_gemm_balanced(d, dtype == TGEMM_BF16, &ctx->sk, ctx->n_cus, ctx->opts.incore_schedule == TGEMM_SCHEDULE_BALANCED, st,
                                 ctx->streams[1], ctx->ev_fork, ctx->ev_join, &launches);
    }
    if (e == hipErrorNotSupported) {
        launches = 1;
        e = launch_tile_gemm(d, dtype == TGEMM_BF16, st);
    }
    if (e != hipSuccess) return fail(TGEMM_EHIP, "tile GEMM launch failed: %s", hipGetErrorString(e));
    TG_HIP(hipEventRecord(ctx->ev_stop, st));
    ctx->kernel_timing_pending = true;
    ctx->stats.in_core = 1;
    ctx->stats.kernel_launches = launches;
    if (!ctx->opts.async_incore) {
        TG_HIP(hipStreamSynchronize(st));
        float ms = 0.f;
        TG_HIP(hipEventElapsedTime(&ms, ctx->ev_start, ctx->ev_stop));
        ctx->stats.kernel_ms = ms;
        ctx->kernel_timing_pending = false;
    }
    ctx->stats.wall_ms = now_ms() - t0;
    log_call("tgemm_run", ctx, TGEMM_OK);
    return TGEMM_OK;
}

int tgemm_last_stats(tgemm_ctx* ctx, tgemm_stats* out)
{
    if (!ctx || !out) return fail(TGEMM_EARG, "tgemm_last_stats: NULL argument");
    *out = ctx->stats;
    return TGEMM_OK;
}

int tgemm_trace(tgemm_ctx* ctx, tgemm_trace_rec* out, int64_t cap, int64_t* n)
{
    if (!ctx || !n || cap < 0 || (cap > 0 && !out)) return fail(TGEMM_EARG, "tgemm_trace: bad argument");
    *n = (int64_t)ctx->trace.size();
    const int64_t m = cap < *n ? cap : *n;
    if (m > 0) memcpy(out, ctx->trace.data(), (size_t)m * sizeof(tgemm_trace_rec));
    return TGEMM_OK;
}

int tgemm_balance_plan(int64_t M, int64_t N, int64_t K, int32_t T, int32_t dtype, int32_t n_cus,
                       int32_t whatever_the_estimate, tgemm_balance* out, tgemm_segment* segments, int64_t cap)
{
    if (!out || cap < 0 || (cap > 0 && !segments)) return fail(TGEMM_EARG, "tgemm_balance_plan: bad argument");
    if (dtype != TGEMM_F32 && dtype != TGEMM_BF16) return fail(TGEMM_EARG, "tgemm_balance_plan: dtype %d", dtype);
    if (M < 0 || N < 0 || K < 0 || T <= 0 || n_cus <= 0) return fail(TGEMM_EARG, "tgemm_balance_plan: bad size");
    try {
        return sk_inspect(M, N, K, T, dtype == TGEMM_BF16, n_cus, whatever_the_estimate != 0, out, segments, cap);
    } catch (...) {
        return fail(TGEMM_ENOMEM, "tgemm_balance_plan: host allocation failed");
    }
}

int tgemm_queue_selftest(int64_t n, int32_t producers, int32_t consumers, int32_t* popped_count)
{
    if (n < 0 || n > 0x7ffffff0 || producers < 1 || consumers < 1 || producers > 64 || consumers > 64 || (n > 0 && !popped_count))
        return fail(TGEMM_EARG, "tgemm_queue_selftest: bad argument");
    for (int64_t i = 0; i < n; ++i) popped_count[i] = 0;
    // a pool much smaller than n forces node reuse (the ABA case the counted pointers guard)
    const uint32_t cap = (uint32_t)(n < 64 ? (n > 0 ? n : 1) : 64);
    TaskQueue q(cap);
    std::atomic<int64_t> next_id{0}, n_popped{0};
    std::vector<std::atomic<int32_t>> counts(n > 0 ? n : 1);
    for (auto& c : counts) c.store(0);
    std::vector<std::thread> th;
    for (int p = 0; p < producers; ++p)
        th.emplace_back([&] {
            for (;;) {
                const int64_t id = next_id.fetch_add(1);
                if (id >= n) return;
                while (!q.enqueue(id)) std::this_thread::yield();   // pool full: wait for a consumer
            }
        });
    for (int c = 0; c < consumers; ++c)
        th.emplace_back([&] {
            int64_t v;
            while (n_popped.load() < n) {
                if (q.dequeue(&v)) {
                    if (v >= 0 && v < n) counts[v].fetch_add(1);
                    n_popped.fetch_add(1);
                } else {
                    std::this_thread::yield();
                }
            }
        });
    for (auto& t : th) t.join();
    for (int64_t i = 0; i < n; ++i) popped_count[i] = counts[i].load();
    return TGEMM_OK;
}

}  // extern "C"
