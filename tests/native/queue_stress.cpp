// Stress of the non-blocking task queue (section 3.2 of the paper) for sanitizer builds on the host:
// P producers push disjoint id ranges, C consumers pop until every id has been seen; the queue is
// sized well below the id count so that nodes are recycled through the free list many times over
// (the ABA-prone part).  Checks: every id exactly once, per-producer FIFO order at each consumer.
// Exit code 0 on success; prints what failed otherwise.
#include <atomic>
#include <cstdio>
#include <cstdlib>
#include <thread>
#include <vector>

#include "ms_queue.h"

int main(int argc, char** argv)
{
    const int64_t n = argc > 1 ? atoll(argv[1]) : 200000;
    const int P = argc > 2 ? atoi(argv[2]) : 3, C = argc > 3 ? atoi(argv[3]) : 3;
    const uint32_t capacity = argc > 4 ? (uint32_t)atoi(argv[4]) : 64;
    tg::TaskQueue q(capacity);
    std::vector<std::atomic<int>> seen((size_t)n);
    for (auto& s : seen) s.store(0, std::memory_order_relaxed);
    std::atomic<int64_t> popped{0};
    std::atomic<int> order_errors{0};
    std::vector<std::thread> th;
    for (int p = 0; p < P; ++p)
        th.emplace_back([&, p] {
            const int64_t lo = n * p / P, hi = n * (p + 1) / P;
            for (int64_t id = lo; id < hi; ++id)
                while (!q.enqueue(id)) std::this_thread::yield();   // pool exhausted: consumers will free nodes
        });
    for (int c = 0; c < C; ++c)
        th.emplace_back([&] {
            std::vector<int64_t> last((size_t)P, -1);
            int64_t id;
            while (popped.load(std::memory_order_acquire) < n) {
                if (!q.dequeue(&id)) { std::this_thread::yield(); continue; }
                popped.fetch_add(1, std::memory_order_acq_rel);
                if (id < 0 || id >= n) { order_errors.fetch_add(1); continue; }
                seen[(size_t)id].fetch_add(1, std::memory_order_relaxed);
                int p = 0;
                while (p + 1 < P && id >= n * (p + 1) / P) ++p;
                if (id <= last[(size_t)p]) order_errors.fetch_add(1);   // one producer's ids arrive in its order
                last[(size_t)p] = id;
            }
        });
    for (auto& t : th) t.join();
    int64_t bad = 0;
    for (int64_t i = 0; i < n; ++i) bad += seen[(size_t)i].load() != 1;
    int64_t dummy;
    const bool empty = !q.dequeue(&dummy);
    if (bad || order_errors.load() || !empty) {
        printf("FAILED: %lld ids not seen exactly once, %d order errors, queue empty at the end: %d\n",
               (long long)bad, order_errors.load(), (int)empty);
        return 1;
    }
    printf("ok: %lld ids, %d producers, %d consumers, capacity %u\n", (long long)n, P, C, capacity);
    return 0;
}
