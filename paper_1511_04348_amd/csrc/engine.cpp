// Out-of-core tile engine: the one-GPU form of the paper's scheduling runtime and tile cache.
//
//   section 3.2  GPU computation thread  -> one submit thread per run (optionally bound to a core)
//                4 concurrent tasks      -> 4 reservation-station slots (each owns a C tile buffer);
//                                           4 HIP streams with fixed roles, see below
//                non-blocking task queue -> TaskQueue (ms_queue.h), filled by the caller thread
//   section 3.4  L1 tile cache           -> slots in one HBM pool, directory keyed (matrix, ti, tj),
//                                           strict LRU; there is no second-level (peer) cache on
//                                           one GPU, a miss goes to host memory
//   Algorithm 1  lines 5-17              -> submit_loop(): dequeue, decode, k loop {lookup A_ik,
//                                           lookup B_kj, fetch on miss, asynchronous tile GEMM},
//                                           asynchronous harvest of C_ij
//
// What differs from Algorithm 1:
//   - No per-round "synchronize all streams" (line 8): a reservation-station slot takes the next
//     task as soon as its previous one has been harvested.
//   - Stream roles.  The paper runs each task's fetches, products and harvest on the task's own
//     stream and relies on four such chains to overlap.  On this GPU concurrent kernels share the
//     CUs evenly, so four copy->product chains fall into lock step (all fetch, then all multiply)
//     and the host link and the MFMA pipes take turns instead of overlapping.  The four streams
//     therefore form a pipeline: stream 0 fetches (every A/B tile and C_ij upload, in issue order,
//     running ahead of the products as far as the cache allows), streams 1 and 2 multiply (tasks
//     alternate between them), stream 3 harvests.  Four tasks are still in flight at a time.
//   - Every cross-stream hazard is an event edge, never a host-side wait: a product waits for
//     the `ready` events of its two tiles and of its C buffer; a fetch into an evicted slot waits
//     for the `read` events of the products that still use the old tile; the harvest waits for
//     the task's last product; the next upload into a C buffer waits for its harvest.
// Cache decisions are taken in issue order on the host, so hits, misses and evictions are a pure
// function of (sizes, T, slot count, task order), independent of timing.
#include <pthread.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <exception>
#include <new>
#include <thread>
#include <unordered_map>
#include <vector>

#include "common.h"
#include "copy_kernel.h"
#include "gemm_kernel.h"
#include "ms_queue.h"

namespace tg {

namespace {

// Identity of a cached tile: which host matrix (index into Engine::mats) and which tile of it.
struct TileKey {
    int32_t mat = -1;
    int32_t ti = 0, tj = 0;
    bool operator==(const TileKey& o) const { return mat == o.mat && ti == o.ti && tj == o.tj; }
};
struct TileKeyHash {
    size_t operator()(const TileKey& k) const
    {
        uint64_t h = ((uint64_t)(uint32_t)k.ti << 32) | (uint32_t)k.tj;
        h ^= (uint64_t)(uint32_t)k.mat * 0x9E3779B97F4A7C15ull;
        h ^= h >> 29; h *= 0xBF58476D1CE4E5B9ull; h ^= h >> 32;
        return (size_t)h;
    }
};
// A host matrix as the cache knows it.  Two calls mean the same matrix when base pointer, shape,
// element size and tile size agree (the same matrix may be the left operand of one product and the
// right operand of another: a tile's layout in its slot depends on the matrix alone).
struct HostMatrix {
    const void* base;
    int64_t rows, cols;
    size_t es;
    int64_t T;
};

struct Slot {
    TileKey key;
    hipEvent_t ready = nullptr;
    hipEvent_t read_ev[2] = {nullptr, nullptr};     // last product on compute stream 0 / 1 that read the slot
    bool read_pending[2] = {false, false};
    int prev = -1, next = -1;
};

inline TileKey tile_key(int mat, int64_t ti, int64_t tj)
{
    TileKey k;
    k.mat = mat; k.ti = (int32_t)ti; k.tj = (int32_t)tj;
    return k;
}

}  // namespace

class Engine {
public:
    char* pool = nullptr;
    size_t pool_bytes = 0;
    std::vector<Slot> slots;
    // per reservation-station slot
    hipEvent_t c_ready[4] = {nullptr, nullptr, nullptr, nullptr};       // C_ij uploaded
    hipEvent_t products_done[4] = {nullptr, nullptr, nullptr, nullptr}; // last k-step finished
    hipEvent_t task_done[4] = {nullptr, nullptr, nullptr, nullptr};     // C_ij harvested
    bool task_pending[4] = {false, false, false, false};
    // directory + LRU list (head = least recently used)
    std::unordered_map<TileKey, int, TileKeyHash> dir;
    int lru_head = -1, lru_tail = -1;
    int n_used = 0;                 // slots handed out so far (slots below it are in use or on the free list)
    std::vector<int> free_slots;    // slots emptied by tgemm_invalidate
    std::vector<HostMatrix> mats;   // the matrices whose tiles the directory may hold
    size_t geom_slot_ab = 0, geom_slot_c = 0;   // slot geometry the cached tiles were laid out for
    int geom_n_ab = 0;

    ~Engine()
    {
        for (auto& s : slots) {
            if (s.ready) (void)hipEventDestroy(s.ready);
            for (auto& e : s.read_ev)
                if (e) (void)hipEventDestroy(e);
        }
        for (int i = 0; i < 4; ++i) {
            if (task_done[i]) (void)hipEventDestroy(task_done[i]);
            if (c_ready[i]) (void)hipEventDestroy(c_ready[i]);
            if (products_done[i]) (void)hipEventDestroy(products_done[i]);
        }
        if (pool) (void)hipFree(pool);
    }

    // The pool is exactly what the call's budget allows: a larger one left by an earlier call with a
    // larger budget is given back first, so the device bytes held never exceed the current budget.
    int ensure_pool(size_t bytes)
    {
        if (pool && pool_bytes == bytes) return TGEMM_OK;
        if (pool) {
            (void)hipFree(pool);
            pool = nullptr;
            pool_bytes = 0;
        }
        hipError_t e = hipMalloc((void**)&pool, bytes);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            pool = nullptr;
            return fail(TGEMM_ENOMEM, "tile cache: hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
        }
        pool_bytes = bytes;
        return TGEMM_OK;
    }

    int ensure_events(int n_slots)
    {
        for (int i = 0; i < 4; ++i) {
            if (!task_done[i]) TG_HIP(hipEventCreateWithFlags(&task_done[i], hipEventDisableTiming));
            if (!c_ready[i]) TG_HIP(hipEventCreateWithFlags(&c_ready[i], hipEventDisableTiming));
            if (!products_done[i]) TG_HIP(hipEventCreateWithFlags(&products_done[i], hipEventDisableTiming));
        }
        const size_t old = slots.size();
        if ((size_t)n_slots > old) slots.resize(n_slots);
        for (size_t i = old; i < slots.size(); ++i) {
            TG_HIP(hipEventCreateWithFlags(&slots[i].ready, hipEventDisableTiming));
            for (auto& e : slots[i].read_ev) TG_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        }
        return TGEMM_OK;
    }

    void reset_directory()
    {
        dir.clear();
        mats.clear();
        free_slots.clear();
        lru_head = lru_tail = -1;
        n_used = 0;
        for (auto& s : slots) {
            s.key = TileKey();
            s.prev = s.next = -1;
            for (auto& p : s.read_pending) p = false;
        }
        for (auto& p : task_pending) p = false;
    }

    int matrix_id(const void* base, int64_t rows, int64_t cols, size_t es, int64_t T)
    {
        for (size_t i = 0; i < mats.size(); ++i)
            if (mats[i].base == base && mats[i].rows == rows && mats[i].cols == cols && mats[i].es == es && mats[i].T == T)
                return (int)i;
        mats.push_back(HostMatrix{base, rows, cols, es, T});
        return (int)mats.size() - 1;
    }

    // Drops every cached tile of the matrices that start at `base`; their slots become free.
    // Called between runs only (all streams idle), so nothing reads the slots any more.
    int64_t invalidate(const void* base)
    {
        int64_t dropped = 0;
        for (int i = 0; i < n_used; ++i) {
            Slot& s = slots[i];
            if (s.key.mat < 0 || mats[(size_t)s.key.mat].base != base) continue;
            dir.erase(s.key);
            lru_unlink(i);
            s.key = TileKey();
            free_slots.push_back(i);
            ++dropped;
        }
        return dropped;
    }

    void lru_unlink(int i)
    {
        Slot& s = slots[i];
        if (s.prev >= 0) slots[s.prev].next = s.next; else lru_head = s.next;
        if (s.next >= 0) slots[s.next].prev = s.prev; else lru_tail = s.prev;
        s.prev = s.next = -1;
    }
    void lru_push_mru(int i)
    {
        Slot& s = slots[i];
        s.prev = lru_tail;
        s.next = -1;
        if (lru_tail >= 0) slots[lru_tail].next = i; else lru_head = i;
        lru_tail = i;
    }
};

int64_t invalidate_tiles(tgemm_ctx* ctx, const void* host_base)
{
    return ctx->engine ? ctx->engine->invalidate(host_base) : 0;
}

void destroy_engine(tgemm_ctx* ctx)
{
    delete ctx->engine;
    ctx->engine = nullptr;
}

namespace {

struct Run {
    tgemm_ctx* ctx;
    Engine* eng;
    const char* A;
    const char* B;
    float* C;
    int64_t M, N, K, T;
    int64_t n_i, n_j, n_k;
    int64_t tm, tn, tk;        // slot extents (rows of A/C tiles, cols of B/C tiles, k extent)
    size_t es;                 // bytes per A/B element
    size_t slot_ab, slot_c;    // bytes per slot
    int n_ab;                  // A/B slots available
    TaskQueue* queue;
    std::atomic<bool> producer_done{false};
    std::atomic<bool> failed{false};
    int rc = TGEMM_OK;
    char err[256] = "";
    int rr = 0;                // round-robin start of the slot search
    int64_t n_issued = 0;      // tasks issued so far (alternates the compute stream)
    int copy_mode = 1;
    bool bf16 = false;
    int mat_a = 0, mat_b = 1;  // directory ids of the two operand matrices

    char* ab_slot_ptr(int slot) const { return eng->pool + 4 * slot_c + (size_t)slot * slot_ab; }
    float* c_slot_ptr(int s) const { return (float*)(eng->pool + (size_t)s * slot_c); }

    bool check(hipError_t e, const char* what)
    {
        if (e == hipSuccess) return true;
        if (rc == TGEMM_OK) {
            rc = TGEMM_EHIP;
            snprintf(err, sizeof err, "%s failed: %s", what, hipGetErrorString(e));
            failed.store(true, std::memory_order_release);
        }
        return false;
    }

    // One tile transfer.  copy_mode 1 (default): hipMemcpy2DAsync, i.e. the DMA engines -- they take
    // no CU resources, so tile products running meanwhile keep their speed.  copy_mode 0
    // (TGEMM_COPY=kernel): the library's strided copy kernel reading page-locked host memory
    // directly; measured slower end to end because its long-latency host reads share the CUs'
    // memory pipelines with the products.
    hipError_t copy2d(void* dst, size_t dpitch, const void* src, size_t spitch, size_t width, size_t height,
                      hipMemcpyKind kind, hipStream_t st)
    {
        if (copy_mode == 1) return hipMemcpy2DAsync(dst, dpitch, src, spitch, width, height, kind, st);
        return launch_copy_2d(dst, dpitch, src, spitch, width, height, st);
    }

    // Algorithm 1 lines 6-7: the next free reservation-station slot.
    int pick_slot()
    {
        for (;;) {
            for (int t = 0; t < 4; ++t) {
                const int s = (rr + t) & 3;
                if (!eng->task_pending[s]) { rr = s + 1; return s; }
                const hipError_t q = hipEventQuery(eng->task_done[s]);
                if (q == hipSuccess) {
                    eng->task_pending[s] = false;
                    rr = s + 1;
                    return s;
                }
                if (q != hipErrorNotReady) {
                    check(q, "hipEventQuery");
                    return -1;
                }
                (void)hipGetLastError();
            }
            std::this_thread::sleep_for(std::chrono::microseconds(20));
        }
    }

    // Algorithm 1 lines 12-15: look the tile up in the L1 tile cache; on a miss take a free slot
    // or evict the least recently used one and fetch the tile from host memory (fetch stream).
    int acquire(int mat, int64_t ti, int64_t tj, const char* src, size_t src_pitch,
                size_t width_bytes, size_t height, size_t slot_pitch, int* hit, int* evicted)
    {
        Engine& e = *eng;
        hipStream_t fetch = ctx->streams[0];
        const TileKey key = tile_key(mat, ti, tj);
        auto it = e.dir.find(key);
        *evicted = 0;
        if (it != e.dir.end()) {
            const int slot = it->second;
            e.lru_unlink(slot);
            e.lru_push_mru(slot);
            *hit = 1;
            ctx->stats.hits++;
            return slot;
        }
        *hit = 0;
        ctx->stats.misses++;
        int slot;
        if (!e.free_slots.empty()) {
            slot = e.free_slots.back();
            e.free_slots.pop_back();
        } else if (e.n_used < n_ab) {
            slot = e.n_used++;
        } else {
            slot = e.lru_head;
            e.lru_unlink(slot);
            e.dir.erase(e.slots[slot].key);
            *evicted = 1;
            ctx->stats.evictions++;
            Slot& sl = e.slots[slot];
            for (int c = 0; c < 2; ++c) {
                if (sl.read_pending[c])
                    check(hipStreamWaitEvent(fetch, sl.read_ev[c], 0), "hipStreamWaitEvent(read)");
                sl.read_pending[c] = false;
            }
        }
        Slot& sl = e.slots[slot];
        sl.key = key;
        e.dir[key] = slot;
        e.lru_push_mru(slot);
        check(copy2d(ab_slot_ptr(slot), slot_pitch, src, src_pitch, width_bytes, height,
                     hipMemcpyHostToDevice, fetch), "H2D tile copy");
        ctx->stats.h2d_bytes += (int64_t)(width_bytes * height);
        check(hipEventRecord(sl.ready, fetch), "hipEventRecord(ready)");
        return slot;
    }

    // Algorithm 1 lines 9-17 for one task in reservation-station slot s.
    void issue_task(int64_t id, int s)
    {
        hipStream_t fetch = ctx->streams[0], harvest = ctx->streams[3];
        const int cs_idx = (int)(n_issued++ & 1);
        hipStream_t comp = ctx->streams[1 + cs_idx];
        const int64_t i = id / n_j, j = id % n_j;              // decode
        const int64_t r0 = i * T, rows = std::min(T, M - r0);
        const int64_t c0 = j * T, cols = std::min(T, N - c0);
        float* cs = c_slot_ptr(s);
        // C_ij enters with its current value: the product accumulates into C.  The buffer is free:
        // pick_slot() saw the harvest of its previous task complete.
        check(copy2d(cs, tn * 4, C + r0 * N + c0, N * 4, cols * 4, rows, hipMemcpyHostToDevice, fetch),
              "H2D C tile copy");
        ctx->stats.h2d_bytes += rows * cols * 4;
        check(hipEventRecord(eng->c_ready[s], fetch), "hipEventRecord(C ready)");
        check(hipStreamWaitEvent(comp, eng->c_ready[s], 0), "hipStreamWaitEvent(C ready)");
        for (int64_t k = 0; k < n_k && rc == TGEMM_OK; ++k) {
            const int64_t k0 = k * T, klen = std::min(T, K - k0);
            int a_hit, b_hit, a_ev, b_ev;
            const int sa = acquire(mat_a, i, k, A + (r0 * K + k0) * es, K * es, klen * es, rows, tk * es, &a_hit, &a_ev);
            const int sb = acquire(mat_b, k, j, B + (k0 * N + c0) * es, N * es, cols * es, klen, tn * es, &b_hit, &b_ev);
            Slot& la = eng->slots[sa];
            Slot& lb = eng->slots[sb];
            check(hipStreamWaitEvent(comp, la.ready, 0), "hipStreamWaitEvent(A ready)");
            check(hipStreamWaitEvent(comp, lb.ready, 0), "hipStreamWaitEvent(B ready)");
            GemmDesc d;
            memset(&d, 0, sizeof d);
            d.A = ab_slot_ptr(sa); d.B = ab_slot_ptr(sb); d.C = cs;
            d.lda = tk; d.ldb = tn; d.ldc = tn;
            d.M = rows; d.N = cols; d.K = klen;
            d.T = (int32_t)std::max(std::max(rows, cols), klen);   // the tile product is one task, one step
            d.a_kcontig = 1; d.b_kcontig = 0;
            d.epilogue = EPI_AXPBY; d.alpha = 1.f; d.beta = 1.f;
            d.config = ctx->opts.kernel_config;
            check(launch_tile_gemm(d, bf16, comp), "tile GEMM launch");
            ctx->stats.kernel_launches++;
            check(hipEventRecord(la.read_ev[cs_idx], comp), "hipEventRecord(read A)");
            la.read_pending[cs_idx] = true;
            check(hipEventRecord(lb.read_ev[cs_idx], comp), "hipEventRecord(read B)");
            lb.read_pending[cs_idx] = true;
            if (ctx->opts.trace) {
                tgemm_trace_rec r;
                r.task_id = id; r.i = (int32_t)i; r.j = (int32_t)j; r.k = (int32_t)k; r.stream = s;
                r.a_hit = a_hit; r.b_hit = b_hit; r.a_slot = sa; r.b_slot = sb; r.a_evicted = a_ev; r.b_evicted = b_ev;
                ctx->trace.push_back(r);
            }
        }
        // harvest
        check(hipEventRecord(eng->products_done[s], comp), "hipEventRecord(products done)");
        check(hipStreamWaitEvent(harvest, eng->products_done[s], 0), "hipStreamWaitEvent(products done)");
        check(copy2d(C + r0 * N + c0, N * 4, cs, tn * 4, cols * 4, rows, hipMemcpyDeviceToHost, harvest),
              "D2H C tile copy");
        ctx->stats.d2h_bytes += rows * cols * 4;
        check(hipEventRecord(eng->task_done[s], harvest), "hipEventRecord(task done)");
        eng->task_pending[s] = true;
    }

    void submit_loop()
    {
        if (!check(hipSetDevice(ctx->device), "hipSetDevice")) return;
        if (ctx->opts.affinity_core >= 0) {
            cpu_set_t set;
            CPU_ZERO(&set);
            CPU_SET(ctx->opts.affinity_core, &set);
            (void)pthread_setaffinity_np(pthread_self(), sizeof set, &set);   // best effort
        }
        // Algorithm 1 line 5: run until the task queue has drained (and the producer has finished).
        // Tasks pass through the reservation station (section 3.2): it is topped up from the queue to
        // `depth` tasks -- waiting for the producer, so that its content does not depend on thread
        // timing -- and when a slot is free the task with the most input tiles in the tile cache
        // leaves first, ties going to the one that entered first.  depth 1 is plain queue order.
        const size_t depth = (size_t)std::min(std::max(ctx->opts.rs_depth, 1), 64);
        std::vector<int64_t> station;
        station.reserve(depth);
        bool drained = false;
        while (rc == TGEMM_OK) {
            while (!drained && station.size() < depth) {
                int64_t id;
                if (queue->dequeue(&id)) { station.push_back(id); continue; }
                if (!producer_done.load(std::memory_order_acquire)) { std::this_thread::yield(); continue; }
                if (queue->dequeue(&id)) station.push_back(id);      // enqueued just before the flag
                else drained = true;
            }
            if (station.empty()) break;
            const int s = pick_slot();
            if (s < 0) break;
            size_t best = 0;
            if (depth > 1) {
                int64_t best_score = -1;
                for (size_t q = 0; q < station.size(); ++q) {
                    const int64_t i = station[q] / n_j, j = station[q] % n_j;
                    int64_t score = 0;
                    for (int64_t k = 0; k < n_k; ++k)
                        score += (int64_t)eng->dir.count(tile_key(mat_a, i, k)) + (int64_t)eng->dir.count(tile_key(mat_b, k, j));
                    if (score > best_score) { best_score = score; best = q; }
                }
            }
            const int64_t id = station[best];
            station.erase(station.begin() + (std::ptrdiff_t)best);
            issue_task(id, s);
        }
        for (int s = 0; s < 4; ++s) check(hipStreamSynchronize(ctx->streams[s]), "hipStreamSynchronize");
        for (auto& p : eng->task_pending) p = false;
    }
};

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

}  // namespace

static int run_out_of_core_body(tgemm_ctx* ctx, const void* A, const void* B, float* C, int64_t M, int64_t N,
                                int64_t K, int32_t T, int32_t dtype, size_t hbm_budget);

int run_out_of_core(tgemm_ctx* ctx, const void* A, const void* B, float* C, int64_t M, int64_t N,
                    int64_t K, int32_t T, int32_t dtype, size_t hbm_budget)
{
    // nothing thrown by the host containers or by std::thread may cross the C boundary
    try {
        return run_out_of_core_body(ctx, A, B, C, M, N, K, T, dtype, hbm_budget);
    } catch (const std::bad_alloc&) {
        return fail(TGEMM_ENOMEM, "tgemm_run: host allocation failed");
    } catch (const std::exception& e) {
        return fail(TGEMM_ENOMEM, "tgemm_run: %s", e.what());
    } catch (...) {
        return fail(TGEMM_ENOMEM, "tgemm_run: unexpected exception");
    }
}

static int run_out_of_core_body(tgemm_ctx* ctx, const void* A, const void* B, float* C, int64_t M, int64_t N,
                                int64_t K, int32_t T, int32_t dtype, size_t hbm_budget)
{
    Run r;
    r.ctx = ctx;
    r.A = (const char*)A; r.B = (const char*)B; r.C = C;
    r.M = M; r.N = N; r.K = K; r.T = T;
    r.n_i = (M + T - 1) / T; r.n_j = (N + T - 1) / T; r.n_k = (K + T - 1) / T;
    r.tm = std::min<int64_t>(T, M); r.tn = std::min<int64_t>(T, N); r.tk = std::min<int64_t>(T, K);
    r.es = dtype == TGEMM_BF16 ? 2 : 4;
    r.bf16 = dtype == TGEMM_BF16;
    if (const char* cm = getenv("TGEMM_COPY")) r.copy_mode = (strcmp(cm, "kernel") == 0) ? 0 : 1;
    r.slot_ab = round_up(std::max(r.tm * r.tk, r.tk * r.tn) * r.es, 256);
    r.slot_c = round_up((size_t)(r.tm * r.tn) * 4, 256);
    const size_t min_bytes = 4 * r.slot_c + 8 * r.slot_ab;
    if (hbm_budget < min_bytes)
        return fail(TGEMM_EBUDGET, "tgemm_run: hbm_budget %zu is below the minimum working set %zu "
                    "(4 C slots of %zu bytes + 8 A/B slots of %zu bytes)", hbm_budget, min_bytes, r.slot_c, r.slot_ab);
    int64_t n_ab = (int64_t)((hbm_budget - 4 * r.slot_c) / r.slot_ab);
    n_ab = std::min<int64_t>(n_ab, r.n_i * r.n_k + r.n_k * r.n_j);   // never more than the distinct tiles
    n_ab = std::max<int64_t>(n_ab, 8);
    r.n_ab = (int)n_ab;

    if (!ctx->engine) {
        ctx->engine = new (std::nothrow) Engine();
        if (!ctx->engine) return fail(TGEMM_ENOMEM, "tgemm_run: host allocation failed");
    }
    r.eng = ctx->engine;
    int rc = r.eng->ensure_pool(4 * r.slot_c + (size_t)r.n_ab * r.slot_ab);
    if (rc != TGEMM_OK) return rc;
    rc = r.eng->ensure_events(r.n_ab);
    if (rc != TGEMM_OK) return rc;
    // Section 3.4 keeps tiles in GPU memory for reuse.  Across calls that is opt-in (tgemm_opts.keep_tiles):
    // the directory, the recency order and the tiles survive as long as the slot geometry does; otherwise
    // every call starts with an empty directory and a changed host matrix can never be seen stale.
    Engine& e = *r.eng;
    if (!ctx->opts.keep_tiles || e.geom_slot_ab != r.slot_ab || e.geom_slot_c != r.slot_c || e.geom_n_ab != r.n_ab ||
        e.mats.size() > 4096)
        e.reset_directory();
    for (auto& sl : e.slots)          // the previous run ended with every stream idle
        for (auto& p : sl.read_pending) p = false;
    for (auto& p : e.task_pending) p = false;
    e.geom_slot_ab = r.slot_ab; e.geom_slot_c = r.slot_c; e.geom_n_ab = r.n_ab;
    r.mat_a = e.matrix_id(A, M, K, r.es, T);
    r.mat_b = e.matrix_id(B, K, N, r.es, T);
    ctx->stats.n_slots = r.n_ab;

    // Algorithm 1 line 1: the task queue receives every task id in issue order
    const int64_t n_tasks = r.n_i * r.n_j;
    std::vector<int64_t> order((size_t)n_tasks);
    // strips: as many tile columns of B as fit in the cache beside two row panels of A (under
    // strict LRU the previous row panel is still younger than the strip's first B column when the
    // next one arrives, so it needs room too or the strip's B tiles get evicted in a cascade)
    // That is the widest strip; the columns are then shared out evenly over as few strips as that
    // allows, so that no narrow strip is left over at the end (in a strip of one column every task
    // fetches a whole row panel of A for a single column of products: more link time than MFMA time).
    int64_t strip = ctx->opts.strip_width;
    if (strip <= 0) {
        const int64_t widest = std::min(std::max<int64_t>(1, r.n_ab / r.n_k - 2), std::max<int64_t>(1, r.n_j));
        const int64_t n_strips = (r.n_j + widest - 1) / widest;
        strip = n_strips > 0 ? (r.n_j + n_strips - 1) / n_strips : 1;
    }
    strip = std::min(strip, r.n_j);
    rc = tgemm_task_order(r.n_i, r.n_j, ctx->opts.order, strip, order.data());
    if (rc != TGEMM_OK) return rc;
    TaskQueue queue((uint32_t)std::min<int64_t>(n_tasks, 1 << 20));
    r.queue = &queue;
    if (ctx->opts.trace) ctx->trace.reserve((size_t)(n_tasks * r.n_k));

    // Algorithm 1 lines 3-4: the GPU computation thread; the caller thread is the producer
    std::thread submit([&r] {
        try {
            r.submit_loop();
        } catch (...) {     // host allocation inside the loop: report it, let the producer stop
            if (r.rc == TGEMM_OK) {
                r.rc = TGEMM_ENOMEM;
                snprintf(r.err, sizeof r.err, "host allocation failed in the submit thread");
            }
            r.failed.store(true, std::memory_order_release);
            for (int s = 0; s < 4; ++s) (void)hipStreamSynchronize(r.ctx->streams[s]);
        }
    });
    for (int64_t t = 0; t < n_tasks && !r.failed.load(std::memory_order_acquire); ++t)
        while (!queue.enqueue(order[(size_t)t]) && !r.failed.load(std::memory_order_acquire))
            std::this_thread::yield();   // pool full: the consumer is behind
    r.producer_done.store(true, std::memory_order_release);
    submit.join();
    if (r.rc != TGEMM_OK) return fail(r.rc, "%s", r.err);
    return TGEMM_OK;
}

}  // namespace tg
