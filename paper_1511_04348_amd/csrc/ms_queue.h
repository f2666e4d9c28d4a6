// Non-blocking FIFO of task ids (section 3.2 of the paper, "Non-blocking Task Queue"; Algorithm 1
// lines 1, 5-7), after Michael & Scott, "Simple, fast, and practical non-blocking and blocking
// concurrent queue algorithms", PODC 1996: a singly linked list with a dummy node, head and tail
// advanced by compare-and-swap, and counted pointers against the ABA problem.  Nodes live in a
// fixed pool and are recycled through a counted-pointer free list, so no memory is ever returned
// to the allocator while the queue is in use.
//
// A "pointer" is a 64-bit word: low 32 bits = node index (NIL = 0xffffffff), high 32 bits = a
// modification count bumped by every successful CAS on that word.
#pragma once
#include <atomic>
#include <cstdint>
#include <memory>

namespace tg {

class TaskQueue {
public:
    // capacity = the largest number of ids that are inside the queue at one time
    explicit TaskQueue(uint32_t capacity)
        : n_nodes_(capacity + 1), nodes_(new Node[capacity + 1])
    {
        for (uint32_t i = 0; i < n_nodes_; ++i) {
            nodes_[i].value.store(0, std::memory_order_relaxed);
            nodes_[i].next.store(pack(i + 1 < n_nodes_ ? i + 1 : NIL, 0), std::memory_order_relaxed);
        }
        // node 0 becomes the dummy; the rest form the free list
        free_.store(pack(n_nodes_ > 1 ? 1 : NIL, 0), std::memory_order_relaxed);
        nodes_[0].next.store(pack(NIL, 0), std::memory_order_relaxed);
        head_.store(pack(0, 0), std::memory_order_relaxed);
        tail_.store(pack(0, 0), std::memory_order_release);
    }

    // false when the pool is exhausted (more than `capacity` ids inside)
    bool enqueue(int64_t v)
    {
        const uint32_t n = alloc_node();
        if (n == NIL) return false;
        nodes_[n].value.store(v, std::memory_order_relaxed);
        // keep the count of the node's own next word moving forward across reuses
        uint64_t old_next = nodes_[n].next.load(std::memory_order_relaxed);
        nodes_[n].next.store(pack(NIL, cnt(old_next) + 1), std::memory_order_release);
        for (;;) {
            const uint64_t tail = tail_.load(std::memory_order_acquire);
            const uint64_t next = nodes_[idx(tail)].next.load(std::memory_order_acquire);
            if (tail != tail_.load(std::memory_order_acquire)) continue;
            if (idx(next) == NIL) {
                uint64_t expect = next;
                if (nodes_[idx(tail)].next.compare_exchange_weak(expect, pack(n, cnt(next) + 1),
                                                                 std::memory_order_acq_rel)) {
                    uint64_t t = tail;
                    tail_.compare_exchange_strong(t, pack(n, cnt(tail) + 1), std::memory_order_acq_rel);
                    return true;
                }
            } else {   // tail is lagging: help it forward
                uint64_t t = tail;
                tail_.compare_exchange_strong(t, pack(idx(next), cnt(tail) + 1), std::memory_order_acq_rel);
            }
        }
    }

    // false when the queue is empty
    bool dequeue(int64_t* out)
    {
        for (;;) {
            const uint64_t head = head_.load(std::memory_order_acquire);
            const uint64_t tail = tail_.load(std::memory_order_acquire);
            const uint64_t next = nodes_[idx(head)].next.load(std::memory_order_acquire);
            if (head != head_.load(std::memory_order_acquire)) continue;
            if (idx(head) == idx(tail)) {
                if (idx(next) == NIL) return false;
                uint64_t t = tail;
                tail_.compare_exchange_strong(t, pack(idx(next), cnt(tail) + 1), std::memory_order_acq_rel);
            } else {
                if (idx(next) == NIL) continue;   // stale snapshot
                const int64_t v = nodes_[idx(next)].value.load(std::memory_order_relaxed);
                uint64_t h = head;
                if (head_.compare_exchange_weak(h, pack(idx(next), cnt(head) + 1), std::memory_order_acq_rel)) {
                    *out = v;
                    free_node(idx(head));
                    return true;
                }
            }
        }
    }

private:
    static constexpr uint32_t NIL = 0xffffffffu;
    struct Node {
        std::atomic<int64_t> value;
        std::atomic<uint64_t> next;
    };
    static uint64_t pack(uint32_t i, uint32_t c) { return ((uint64_t)c << 32) | i; }
    static uint32_t idx(uint64_t p) { return (uint32_t)p; }
    static uint32_t cnt(uint64_t p) { return (uint32_t)(p >> 32); }

    uint32_t alloc_node()
    {
        for (;;) {
            const uint64_t top = free_.load(std::memory_order_acquire);
            if (idx(top) == NIL) return NIL;
            const uint64_t nxt = nodes_[idx(top)].next.load(std::memory_order_acquire);
            uint64_t t = top;
            if (free_.compare_exchange_weak(t, pack(idx(nxt), cnt(top) + 1), std::memory_order_acq_rel))
                return idx(top);
        }
    }
    void free_node(uint32_t n)
    {
        for (;;) {
            const uint64_t top = free_.load(std::memory_order_acquire);
            const uint64_t old = nodes_[n].next.load(std::memory_order_relaxed);
            nodes_[n].next.store(pack(idx(top), cnt(old) + 1), std::memory_order_release);
            uint64_t t = top;
            if (free_.compare_exchange_weak(t, pack(n, cnt(top) + 1), std::memory_order_acq_rel)) return;
        }
    }

    const uint32_t n_nodes_;
    std::unique_ptr<Node[]> nodes_;
    alignas(64) std::atomic<uint64_t> head_;
    alignas(64) std::atomic<uint64_t> tail_;
    alignas(64) std::atomic<uint64_t> free_;
};

}  // namespace tg
