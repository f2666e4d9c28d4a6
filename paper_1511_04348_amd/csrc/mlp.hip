// MLP passes reduced to tiled matrix products (section 2 of the paper):
//   forward  (equation 1)  Z_l = A_{l-1} W_l,  A_l = sigmoid(Z_l)  (sigmoid fused into the product's epilogue)
//   backward (equation 4)  D_{l-1} = (D_l W_l^T) * A_{l-1} * (1 - A_{l-1})   (derivative fused likewise)
//            (equation 3)  dW_l = A_{l-1}^T D_l
//   update                 W_l <- W_l - lr dW_l   (the dW product's epilogue writes straight into W_l)
// plus one row-wise kernel for softmax, cross-entropy and the output error D_L.
// Every product goes through the same tile GEMM kernels as tgemm_run, with tile size T.
//
// Two residency modes.  In-core: the weights are device matrices and every product is one launch
// on stream 0.  Out-of-core: the weights stay in pinned host memory and are staged, T x T tile by
// tile, through an HBM tile cache (section 3.4 of the paper; the victim is the tile whose next use
// in the step's fixed sweep lies furthest ahead, see WeightCache) -- the kernels then take
// the weight operand as a table of tile pointers.  Streams form the same pipeline as in
// tgemm_run: stream 0 fetches weight tiles (running ahead of the products), stream 1 computes,
// stream 3 writes updated tiles back.  The forward pass walks W_l by tile columns (a column of
// tiles is one launch over the whole batch, so every weight tile is fetched once per pass); the
// backward pass walks W_l by tile rows (the row's tiles serve the D W^T product, then receive the
// update, then are written back), so each tile crosses the link at most twice per step in each
// direction.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <chrono>
#include <deque>
#include <new>
#include <mutex>
#include <unordered_map>
#include <vector>

#include "common.h"
#include "gemm_kernel.h"

// ---- static scratch for mlp_forward_static ------------------------------------------------------
// Device memory that exists from the moment the code object is loaded: the hidden activations and
// the logits of a forward pass for callers that must not allocate.  Every GPU that loads the library
// holds its own copy at its own address; host code never uses the array's name as an address (it is
// only a host-side stand-in for the symbol) but the per-device address that hipGetSymbolAddress
// returned for it.
static __device__ __align__(256) unsigned char tgemm_static_scratch[TGEMM_STATIC_SCRATCH_BYTES];

namespace tg {

namespace {
constexpr int MAX_DEVICES = 64;
void* g_static_scratch[MAX_DEVICES] = {};     // per device: address of that device's copy of the array
std::mutex g_static_scratch_mu;
}  // namespace

// Looks the array's address up on `device` (which must be the current device); once per device.
int static_scratch_resolve(int device, void** out)
{
    if (device < 0 || device >= MAX_DEVICES) return fail(TGEMM_EARG, "static scratch: device %d", device);
    std::lock_guard<std::mutex> lock(g_static_scratch_mu);
    if (!g_static_scratch[device]) {
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(tgemm_static_scratch));
        if (e != hipSuccess || !p) {
            (void)hipGetLastError();
            return fail(TGEMM_EHIP, "static scratch: hipGetSymbolAddress failed on device %d: %s", device, hipGetErrorString(e));
        }
        g_static_scratch[device] = p;
    }
    if (out) *out = g_static_scratch[device];
    return TGEMM_OK;
}

namespace {

// ---- weight tile cache (out-of-core mode) -------------------------------------------------------
struct WSlot {
    int64_t key = -1;
    hipEvent_t ready = nullptr;      // fetch finished (stream 0); owned by the slot
    // Events of whole launches / whole write-back groups (not owned, recycled by their owners): a
    // recycled event stands for newer work, so waiting on it waits at least long enough.
    hipEvent_t read = nullptr;       // the last product using the tile finished (stream 1)
    hipEvent_t flushed = nullptr;    // its write-back finished (stream 3)
    bool read_pending = false, flush_pending = false;
    int64_t pos_f = -1, pos_b = -1;  // the tile's place in the forward / backward sweep of a training step
    int64_t last_launch = -1;        // launch group that used the slot last
    int64_t fetch_seq = 0, read_seq = 0, flush_seq = 0;   // sequence numbers of its fetch / pending read / write-back
};

// Replacement: a training step sweeps every weight tile twice in a fixed order (forward: layer by
// layer, tile column by tile column; backward: layers in reverse, tile row by tile row), so the
// next use of every cached tile is known.  The victim is the tile whose next use lies farthest
// ahead (for a cyclic sweep over more tiles than slots, LRU evicts exactly the tiles needed next
// and misses about twice as often).  Tiles of the launch being assembled are never evicted, and
// tiles that a launch still reads or whose write-back is still in flight are passed over while
// any settled slot is left, so that fetches keep running ahead of the products instead of
// queueing behind the write-back stream.
struct WeightCache {
    char* pool = nullptr;
    size_t slot_bytes = 0;
    int n_slots = 0, n_used = 0;
    std::vector<WSlot> slots;
    std::unordered_map<int64_t, int> dir;
    bool exact = false;                      // tgemm_opts.exact_replacement: the furthest next use, whatever is in flight
    int64_t period = 0;                      // accesses per training step (two per tile)
    int64_t launch_id = 0;                   // current launch group (one tile column / tile row)
    std::vector<int64_t> base_f, base_b;     // first sweep position of layer l, forward / backward
    // Reads finish in launch order and write-backs in issue order (one stream each), so "has this
    // slot's last read / write-back finished" is a comparison with the newest finished sequence
    // number; the queues hold (sequence number, event) of what is still in flight.
    struct InFlight { int64_t seq; hipEvent_t ev; };
    std::deque<InFlight> reads, flushes;
    int64_t read_issue = 0, read_done = 0, flush_issue = 0, flush_done = 0;
    int64_t fetch_issue = 0, fetch_waited = 0;   // fetches issued; newest one the compute stream waits for
    std::vector<hipEvent_t> flush_pool;      // one event per write-back group, reused round robin
    size_t flush_next = 0;

    ~WeightCache() { release(); }
    void release()
    {
        for (auto& s : slots)
            if (s.ready) (void)hipEventDestroy(s.ready);
        slots.clear();
        for (auto& e : flush_pool)
            if (e) (void)hipEventDestroy(e);
        flush_pool.clear();
        flush_next = 0;
        fetch_issue = fetch_waited = 0;
        if (pool) (void)hipFree(pool);
        pool = nullptr;
        dir.clear();
        n_slots = n_used = 0;
        launch_id = 0;
        reads.clear(); flushes.clear();
        read_issue = read_done = flush_issue = flush_done = 0;
    }
    char* ptr(int slot) const { return pool + (size_t)slot * slot_bytes; }
    void all_reads_done() { reads.clear(); read_done = read_issue; }
    void reads_done_upto(int64_t seq)
    {
        while (!reads.empty() && reads.front().seq <= seq) reads.pop_front();
        read_done = std::max(read_done, seq);
    }
    // An event for the next write-back group: the pool's next one, once it is out of the queue.
    int next_flush_event(hipEvent_t* out)
    {
        hipEvent_t e = flush_pool[flush_next];
        flush_next = (flush_next + 1) % flush_pool.size();
        while (!flushes.empty() && flushes.size() >= flush_pool.size()) {
            TG_HIP(hipEventSynchronize(flushes.front().ev));
            flush_done = flushes.front().seq;
            flushes.pop_front();
        }
        *out = e;
        return TGEMM_OK;
    }
    void all_flushes_done() { flushes.clear(); flush_done = flush_issue; }
    static void advance(std::deque<InFlight>& q, int64_t& done)
    {
        while (!q.empty() && hipEventQuery(q.front().ev) == hipSuccess) {
            done = q.front().seq;
            q.pop_front();
        }
        (void)hipGetLastError();    // hipErrorNotReady from the query is not an error
    }
    bool settled(WSlot& s)
    {
        if (s.read_pending && s.read_seq <= read_done) s.read_pending = false;
        if (s.flush_pending && s.flush_seq <= flush_done) s.flush_pending = false;
        return !s.read_pending && !s.flush_pending;
    }
    // accesses from sweep position `cur` until the slot's tile is wanted again
    int64_t next_use(const WSlot& s, int64_t cur) const
    {
        const int64_t df = ((s.pos_f - cur - 1) % period + period) % period;
        const int64_t db = ((s.pos_b - cur - 1) % period + period) % period;
        return std::min(df, db);
    }
    // Victim for a fetch at sweep position `cur`; -1 if every slot belongs to the current launch.
    // Candidates are the slots whose next use is at least half as far away as the farthest one.
    // Among them a settled slot (no read or write-back in flight) with the farthest next use wins.
    // If none is settled -- the host queues launches well ahead of the GPU, so every cached tile may
    // still have work queued -- the one whose pending work finishes first: a slot that only waits
    // for reads (the one used longest ago) before any slot with a write-back queued (write-backs
    // trail the products by a long queue, and a fetch waiting for one holds up every later fetch).
    int pick_victim(int64_t cur)
    {
        if (exact) {     // two tiles never share a sweep position, so there are no ties
            int far = -1;
            int64_t d_far = -1;
            for (int i = 0; i < n_slots; ++i) {
                if (slots[i].last_launch == launch_id) continue;
                const int64_t d = next_use(slots[i], cur);
                if (d > d_far) { d_far = d; far = i; }
            }
            return far;
        }
        advance(reads, read_done);
        advance(flushes, flush_done);
        int64_t dmax = -1;
        for (int i = 0; i < n_slots; ++i)
            if (slots[i].last_launch != launch_id) dmax = std::max(dmax, next_use(slots[i], cur));
        if (dmax < 0) return -1;
        int best_settled = -1, oldest = -1;
        int64_t bsd = -1;
        for (int i = 0; i < n_slots; ++i) {
            WSlot& s = slots[i];
            if (s.last_launch == launch_id) continue;
            const int64_t d = next_use(s, cur);
            if (2 * d < dmax) continue;
            const bool is_settled = settled(s);     // also refreshes the pending flags
            if (d > bsd && is_settled) { bsd = d; best_settled = i; }
            if (oldest < 0) { oldest = i; continue; }
            const WSlot& o = slots[oldest];
            if (s.flush_pending != o.flush_pending) { if (!s.flush_pending) oldest = i; }
            else if (s.flush_pending ? s.flush_seq < o.flush_seq : s.last_launch < o.last_launch) oldest = i;
        }
        return best_settled >= 0 ? best_settled : oldest;
    }
};

struct TableRing {
    static constexpr int N = 96;
    void** dev[N] = {};
    void** host[N] = {};
    hipEvent_t done[N] = {};
    hipEvent_t table_ready[N] = {};   // the entry's table has arrived on the device (fetch stream)
    bool used[N] = {};
    int64_t seq[N] = {};     // read sequence number of the launch that used the entry last
    int next = 0;
    int cap = 0;   // pointers per entry
};

// Out-of-core velocity / master-copy matrices (pinned host, fp32): the T rows that one launch of the
// dW product updates pass through one of two device buffers -- fetched whole (the rows are contiguous
// in the host matrix), updated in place by the epilogue, written back whole.
struct RowStream {
    float* buf[2] = {};
    hipEvent_t ready[2] = {}, freed[2] = {};
    bool in_use[2] = {};          // `freed` has been recorded for the buffer's last use
    hipEvent_t last_freed = nullptr;   // the newest write-back (all earlier ones precede it on the flush stream)
    size_t bytes = 0;             // capacity of one buffer
    int next = 0;
    void release()
    {
        for (int i = 0; i < 2; ++i) {
            if (buf[i]) (void)hipFree(buf[i]);
            if (ready[i]) (void)hipEventDestroy(ready[i]);
            if (freed[i]) (void)hipEventDestroy(freed[i]);
            buf[i] = nullptr; ready[i] = freed[i] = nullptr; in_use[i] = false;
        }
        last_freed = nullptr; bytes = 0; next = 0;
    }
};

inline int64_t wkey(int layer, int64_t r, int64_t c) { return ((int64_t)layer << 56) | (r << 28) | c; }

}  // namespace
}  // namespace tg

struct tgemm_mlp {
    tgemm_ctx* ctx = nullptr;
    int n_layers = 0;
    std::vector<int64_t> dims;
    std::vector<char*> W;         // caller-owned weights (device or pinned host)
    std::vector<float*> bias;     // caller-owned bias rows b_l (device, float), empty: no bias terms
    std::vector<float*> dbias;    // caller-owned destinations of mlp_backward's bias gradients, may hold NULLs
    std::vector<float*> vel;      // caller-owned velocity matrices V_l (float; device, or pinned host for out-of-core weights), empty: plain SGD
    std::vector<float*> vel_bias; // velocity rows of the bias terms (may be empty)
    std::vector<float*> master;   // caller-owned fp32 copies of bf16 weights (device, or pinned host for out-of-core weights), empty: none
    float mu = 0.f;               // momentum coefficient
    float* colsum_part = nullptr; // partial column sums of an error matrix: COLSUM_CHUNKS x max n_l floats
    int32_t dtype = TGEMM_F32;
    int32_t act_kind = TGEMM_ACT_SIGMOID;   // hidden-layer activation
    int32_t round_mode = TGEMM_ROUND_NEAREST;   // how mlp_step rounds updated bf16 weights
    uint64_t sr_seed = 0;
    uint32_t sr_step = 0;         // mlp_step calls since mlp_set_rounding
    size_t es = 4;                // bytes per weight / activation / error element
    int32_t T = 0;
    size_t budget = 0;
    bool ooc = false;
    int64_t cap_batch = 0;        // batch the workspaces were sized for
    int64_t batch = 0;            // batch of the last forward (0: none yet)
    const char* X = nullptr;      // input of the last forward (caller owned)
    std::vector<char*> act;       // act[l], l = 1..L-1 : batch x dims[l], dtype
    std::vector<char*> delta;     // delta[l], l = 1..L : batch x dims[l], dtype
    float* logits = nullptr;      // batch x dims[L], float
    float* row_loss = nullptr;    // batch
    bool have_delta = false;
    tg::WeightCache cache;
    tg::TableRing ring;
    tg::RowStream vel_rows, master_rows;   // out-of-core networks with velocities / master copies
    std::vector<tgemm_mlp_trace_rec> trace; // weight-tile lookups of the last call (tgemm_opts.trace)
};

namespace tg {
namespace {

__device__ inline uint16_t to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// One workgroup per row of the logits.  P = softmax(z) with the row maximum subtracted;
// row_loss = -log P[label]; delta = (P - onehot(label)) * inv_batch (float, or bf16 rounded to
// nearest even).  probs / delta / labels may be NULL (no labels: no loss, no delta).
// The row is read twice: once for the maximum and the sum together (each thread keeps a running
// maximum m and the sum of exp(z - m), rescaled whenever m grows; threads, then waves, are merged the
// same way), once to write the results.  VEC: four adjacent columns per access (n % 4 == 0, aligned).
__device__ inline void softmax_merge(float& m, float& s, float m2, float s2)
{
    const float mn = fmaxf(m, m2);
    if (mn == -INFINITY) return;                         // nothing but -inf so far on both sides
    s = s * expf(m - mn) + s2 * expf(m2 - mn);
    m = mn;
}
template <bool DELTA_BF16, bool VEC>
__global__ __launch_bounds__(256) void softmax_xent_rows(const float* __restrict__ logits, int64_t ld, int n,
                                                         const int32_t* __restrict__ labels, float inv_batch,
                                                         void* __restrict__ delta, float* __restrict__ probs,
                                                         float* __restrict__ row_loss)
{
    __shared__ float red_m[4], red_s[4];
    const int row = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const float* z = logits + (int64_t)row * ld;
    float m = -INFINITY, s = 0.f;
    if (VEC) {
        for (int c = 4 * tid; c < n; c += 1024) {
            const float4 x = *reinterpret_cast<const float4*>(z + c);
            const float mn = fmaxf(m, fmaxf(fmaxf(x.x, x.y), fmaxf(x.z, x.w)));
            if (mn > -INFINITY) {
                s = s * expf(m - mn) + ((expf(x.x - mn) + expf(x.y - mn)) + (expf(x.z - mn) + expf(x.w - mn)));
                m = mn;
            }
        }
    } else {
        for (int c = tid; c < n; c += 256) softmax_merge(m, s, z[c], 1.f);
    }
    for (int o = 32; o > 0; o >>= 1) softmax_merge(m, s, __shfl_xor(m, o, 64), __shfl_xor(s, o, 64));
    if (lane == 0) { red_m[wave] = m; red_s[wave] = s; }
    __syncthreads();
    m = red_m[0]; s = red_s[0];
    for (int w = 1; w < 4; ++w) softmax_merge(m, s, red_m[w], red_s[w]);
    const int y = labels ? labels[row] : -1;
    const float inv = 1.f / s;
    if (probs || delta) {
        if (VEC) {
            for (int c = 4 * tid; c < n; c += 1024) {
                const float4 x = *reinterpret_cast<const float4*>(z + c);
                float4 p;
                p.x = expf(x.x - m) * inv; p.y = expf(x.y - m) * inv;
                p.z = expf(x.z - m) * inv; p.w = expf(x.w - m) * inv;
                if (probs) *reinterpret_cast<float4*>(probs + (int64_t)row * ld + c) = p;
                if (delta) {
                    float4 d;
                    d.x = (p.x - (c == y ? 1.f : 0.f)) * inv_batch; d.y = (p.y - (c + 1 == y ? 1.f : 0.f)) * inv_batch;
                    d.z = (p.z - (c + 2 == y ? 1.f : 0.f)) * inv_batch; d.w = (p.w - (c + 3 == y ? 1.f : 0.f)) * inv_batch;
                    if (DELTA_BF16) {
                        uint2 w;
                        w.x = (uint32_t)to_bf16_rne(d.x) | ((uint32_t)to_bf16_rne(d.y) << 16);
                        w.y = (uint32_t)to_bf16_rne(d.z) | ((uint32_t)to_bf16_rne(d.w) << 16);
                        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(delta) + (int64_t)row * ld + c) = w;
                    } else {
                        *reinterpret_cast<float4*>(reinterpret_cast<float*>(delta) + (int64_t)row * ld + c) = d;
                    }
                }
            }
        } else {
            for (int c = tid; c < n; c += 256) {
                const float p = expf(z[c] - m) * inv;
                if (probs) probs[(int64_t)row * ld + c] = p;
                if (delta) {
                    const float d = (p - (c == y ? 1.f : 0.f)) * inv_batch;
                    if (DELTA_BF16) reinterpret_cast<uint16_t*>(delta)[(int64_t)row * ld + c] = to_bf16_rne(d);
                    else reinterpret_cast<float*>(delta)[(int64_t)row * ld + c] = d;
                }
            }
        }
    }
    if (tid == 0 && labels) row_loss[row] = (y >= 0 && y < n) ? (logf(s) + m - z[y]) : NAN;
}

// Bias gradient db = 1^T D (column sums of the batch x n error matrix), in two deterministic passes:
// partial sums over bands of COLSUM_ROWS rows, then the bands in ascending order.  The second pass
// stores the sum (db != NULL) and / or applies b <- b - lr * sum (b != NULL).
constexpr int COLSUM_ROWS = 512;
// VEC = 4: a thread owns four adjacent columns (one 8- or 16-byte load per row; needs n % 4 == 0 and a
// 16-byte aligned matrix); VEC = 1: one column per thread.  Rows are added in ascending order either way.
template <bool BF16, int VEC>
__global__ __launch_bounds__(256) void colsum_partial(const void* __restrict__ D, int64_t ld, int64_t rows, int n,
                                                      float* __restrict__ part)
{
    const int col = (blockIdx.x * 256 + threadIdx.x) * VEC;
    if (col >= n) return;
    const int64_t r0 = (int64_t)blockIdx.y * COLSUM_ROWS, r1 = min(rows, r0 + COLSUM_ROWS);
    float s[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) s[e] = 0.f;
    if (BF16) {
        const uint16_t* d = reinterpret_cast<const uint16_t*>(D) + col;
#pragma unroll 4
        for (int64_t r = r0; r < r1; ++r) {
            if (VEC == 4) {
                const uint2 w = *reinterpret_cast<const uint2*>(d + r * ld);
                s[0] += __uint_as_float(w.x << 16); s[1 % VEC] += __uint_as_float(w.x & 0xffff0000u);
                s[2 % VEC] += __uint_as_float(w.y << 16); s[3 % VEC] += __uint_as_float(w.y & 0xffff0000u);
            } else {
                s[0] += __uint_as_float((uint32_t)d[r * ld] << 16);
            }
        }
    } else {
        const float* d = reinterpret_cast<const float*>(D) + col;
#pragma unroll 4
        for (int64_t r = r0; r < r1; ++r) {
            if (VEC == 4) {
                const float4 w = *reinterpret_cast<const float4*>(d + r * ld);
                s[0] += w.x; s[1 % VEC] += w.y; s[2 % VEC] += w.z; s[3 % VEC] += w.w;
            } else {
                s[0] += d[r * ld];
            }
        }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) part[(int64_t)blockIdx.y * n + col + e] = s[e];
}
// With a velocity row vb (momentum): vb <- mu vb + sum; b <- b - lr vb.
__global__ __launch_bounds__(256) void colsum_finish(const float* __restrict__ part, int bands, int n, float lr,
                                                     float* __restrict__ b, float* __restrict__ db, float mu,
                                                     float* __restrict__ vb)
{
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col >= n) return;
    float s = 0.f;
    for (int k = 0; k < bands; ++k) s += part[(int64_t)k * n + col];
    if (db) db[col] = s;
    if (b) {
        if (vb) {
            s = fmaf(mu, vb[col], s);
            vb[col] = s;
        }
        b[col] = fmaf(-lr, s, b[col]);
    }
}

double now_ms()
{
    return std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now().time_since_epoch()).count();
}

inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

void free_workspaces(tgemm_mlp* m)
{
    for (auto& p : m->act) { if (p) (void)hipFree(p); p = nullptr; }
    for (auto& p : m->delta) { if (p) (void)hipFree(p); p = nullptr; }
    if (m->logits) (void)hipFree(m->logits);
    if (m->row_loss) (void)hipFree(m->row_loss);
    if (m->colsum_part) (void)hipFree(m->colsum_part);
    m->logits = nullptr; m->row_loss = nullptr; m->colsum_part = nullptr;
    m->cap_batch = 0; m->batch = 0; m->have_delta = false;
    m->cache.release();
    m->vel_rows.release();
    m->master_rows.release();
    TableRing& r = m->ring;
    for (int i = 0; i < TableRing::N; ++i) {
        if (r.dev[i]) (void)hipFree(r.dev[i]);
        if (r.host[i]) (void)hipHostFree(r.host[i]);
        if (r.done[i]) (void)hipEventDestroy(r.done[i]);
        if (r.table_ready[i]) (void)hipEventDestroy(r.table_ready[i]);
        r.dev[i] = nullptr; r.host[i] = nullptr; r.done[i] = nullptr; r.table_ready[i] = nullptr; r.used[i] = false;
    }
    r.next = 0; r.cap = 0;
}

int64_t total_tiles(const tgemm_mlp* m)
{
    int64_t n = 0;
    for (int l = 1; l <= m->n_layers; ++l) n += cdiv(m->dims[l - 1], m->T) * cdiv(m->dims[l], m->T);
    return n;
}

int ensure_workspaces(tgemm_mlp* m, int64_t batch)
{
    if (batch <= m->cap_batch) return TGEMM_OK;
    free_workspaces(m);
    const int L = m->n_layers;
    size_t total = (size_t)batch * 4 + (size_t)batch * m->dims[L] * 4;
    for (int l = 1; l <= L; ++l) total += (size_t)batch * m->dims[l] * m->es * (l < L ? 2 : 1);
    size_t colsum_bytes = 0;
    if (!m->bias.empty()) {
        int64_t widest = 0;
        for (int l = 1; l <= L; ++l) widest = std::max(widest, m->dims[l]);
        colsum_bytes = (size_t)cdiv(batch, COLSUM_ROWS) * widest * 4;
        total += colsum_bytes;
    }
    // out-of-core velocities / master copies: two buffers of T rows of the widest weight matrix each
    size_t row_bytes = 0;
    if (m->ooc && (!m->vel.empty() || !m->master.empty())) {
        int64_t widest = 0;
        for (int l = 1; l <= L; ++l) widest = std::max(widest, m->dims[l]);
        row_bytes = (size_t)m->T * widest * 4;
        total += 2 * row_bytes * ((m->vel.empty() ? 0 : 1) + (m->master.empty() ? 0 : 1));
    }
    // out-of-core: the rest of the budget is the weight tile cache
    int64_t max_tiles = 0, n_slots = 0;
    const size_t slot_bytes = (size_t)m->T * m->T * m->es;
    if (m->ooc) {
        for (int l = 0; l <= L; ++l) max_tiles = std::max(max_tiles, cdiv(m->dims[l], m->T));
        const size_t ring_bytes = (size_t)TableRing::N * max_tiles * sizeof(void*);
        const size_t need = total + ring_bytes + (size_t)(2 * max_tiles + 2) * slot_bytes;
        if (m->budget < need)
            return fail(TGEMM_EBUDGET, "mlp: batch %lld needs %zu bytes of activations and at least %lld weight-tile "
                        "slots of %zu bytes; hbm_budget is %zu", (long long)batch, total, (long long)(2 * max_tiles + 2),
                        slot_bytes, m->budget);
        n_slots = (int64_t)((m->budget - total - ring_bytes) / slot_bytes);
        n_slots = std::min(n_slots, total_tiles(m));
        total += ring_bytes;
    } else if (m->budget && total > m->budget) {
        return fail(TGEMM_EBUDGET, "mlp: activations and errors for batch %lld need %zu bytes, hbm_budget is %zu",
                    (long long)batch, total, m->budget);
    }
    auto alloc = [&](void** p, size_t bytes) -> bool {
        if (hipMalloc(p, bytes) != hipSuccess) { (void)hipGetLastError(); *p = nullptr; return false; }
        return true;
    };
    bool ok = alloc((void**)&m->row_loss, (size_t)batch * 4) && alloc((void**)&m->logits, (size_t)batch * m->dims[L] * 4);
    if (colsum_bytes) ok = ok && alloc((void**)&m->colsum_part, colsum_bytes);
    for (int l = 1; l <= L && ok; ++l) {
        if (l < L) ok = ok && alloc((void**)&m->act[l], (size_t)batch * m->dims[l] * m->es);
        ok = ok && alloc((void**)&m->delta[l], (size_t)batch * m->dims[l] * m->es);
    }
    auto alloc_rows = [&](RowStream& rs) {
        rs.bytes = row_bytes;
        for (int i = 0; i < 2 && ok; ++i)
            ok = alloc((void**)&rs.buf[i], row_bytes) &&
                 hipEventCreateWithFlags(&rs.ready[i], hipEventDisableTiming) == hipSuccess &&
                 hipEventCreateWithFlags(&rs.freed[i], hipEventDisableTiming) == hipSuccess;
    };
    if (ok && row_bytes && !m->vel.empty()) alloc_rows(m->vel_rows);
    if (ok && row_bytes && !m->master.empty()) alloc_rows(m->master_rows);
    if (ok && m->ooc) {
        WeightCache& c = m->cache;
        c.slot_bytes = slot_bytes;
        c.base_f.assign((size_t)L + 2, 0);
        c.base_b.assign((size_t)L + 2, 0);
        const int64_t all = total_tiles(m);
        c.period = 2 * all;
        int64_t at = 0;
        for (int l = 1; l <= L; ++l) { c.base_f[(size_t)l] = at; at += cdiv(m->dims[l - 1], m->T) * cdiv(m->dims[l], m->T); }
        for (int l = L; l >= 1; --l) { c.base_b[(size_t)l] = at; at += cdiv(m->dims[l - 1], m->T) * cdiv(m->dims[l], m->T); }
        ok = alloc((void**)&c.pool, (size_t)n_slots * slot_bytes);
        if (ok) {
            c.n_slots = (int)n_slots;
            c.slots.resize((size_t)n_slots);
            for (auto& s : c.slots) ok = ok && hipEventCreateWithFlags(&s.ready, hipEventDisableTiming) == hipSuccess;
            c.flush_pool.assign(256, nullptr);
            for (auto& e : c.flush_pool) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
        }
        TableRing& r = m->ring;
        r.cap = (int)max_tiles;
        for (int i = 0; i < TableRing::N && ok; ++i) {
            ok = alloc((void**)&r.dev[i], (size_t)max_tiles * sizeof(void*)) &&
                 hipHostMalloc((void**)&r.host[i], (size_t)max_tiles * sizeof(void*), hipHostMallocDefault) == hipSuccess &&
                 hipEventCreateWithFlags(&r.done[i], hipEventDisableTiming) == hipSuccess &&
                 hipEventCreateWithFlags(&r.table_ready[i], hipEventDisableTiming) == hipSuccess;
        }
    }
    if (!ok) {
        (void)hipGetLastError();
        free_workspaces(m);
        return fail(TGEMM_ENOMEM, "mlp: device allocation of %zu workspace bytes failed", total);
    }
    m->cap_batch = batch;
    return TGEMM_OK;
}

// ---- out-of-core helpers ------------------------------------------------------------------------

// Tile (r, c) of W_l into the cache (section 3.4: hit -> use it, miss -> fetch from host memory).
// bwd: the access belongs to the backward sweep.
int acquire_tile(tgemm_mlp* m, int l, int64_t r, int64_t c, bool bwd, int* slot_out)
{
    WeightCache& wc = m->cache;
    tgemm_ctx* ctx = m->ctx;
    hipStream_t fetch = ctx->streams[0];
    const int64_t key = wkey(l, r, c);
    const int64_t T = m->T, nc = m->dims[l];
    const int64_t n_r = cdiv(m->dims[l - 1], T), n_c = cdiv(nc, T);
    const int64_t pos_f = wc.base_f[(size_t)l] + c * n_r + r, pos_b = wc.base_b[(size_t)l] + r * n_c + c;
    auto it = wc.dir.find(key);
    tgemm_mlp_trace_rec rec;
    rec.group = wc.launch_id;
    rec.layer = l; rec.r = (int32_t)r; rec.c = (int32_t)c; rec.backward = bwd ? 1 : 0;
    rec.ev_layer = rec.ev_r = rec.ev_c = -1;
    if (it != wc.dir.end()) {
        wc.slots[it->second].last_launch = wc.launch_id;
        ctx->stats.hits++;
        *slot_out = it->second;
        if (ctx->opts.trace) { rec.hit = 1; rec.slot = it->second; m->trace.push_back(rec); }
        return TGEMM_OK;
    }
    ctx->stats.misses++;
    int slot;
    if (wc.n_used < wc.n_slots) {
        slot = wc.n_used++;
    } else {
        slot = wc.pick_victim(bwd ? pos_b : pos_f);
        if (slot < 0) return fail(TGEMM_EBUDGET, "mlp: the weight-tile cache cannot hold the tiles of one launch");
        WSlot& s = wc.slots[slot];
        wc.dir.erase(s.key);
        rec.ev_layer = (int32_t)(s.key >> 56); rec.ev_r = (int32_t)((s.key >> 28) & 0xfffffff); rec.ev_c = (int32_t)(s.key & 0xfffffff);
        ctx->stats.evictions++;
        (void)wc.settled(s);      // the flags are fresh: a pending one's event has not been recycled
        if (s.read_pending) TG_HIP(hipStreamWaitEvent(fetch, s.read, 0));
        if (s.flush_pending) TG_HIP(hipStreamWaitEvent(fetch, s.flushed, 0));
        s.read_pending = s.flush_pending = false;
    }
    WSlot& s = wc.slots[slot];
    s.key = key;
    s.pos_f = pos_f;
    s.pos_b = pos_b;
    s.last_launch = wc.launch_id;
    wc.dir[key] = slot;
    const int64_t rows = std::min(T, m->dims[l - 1] - r * T), cols = std::min(T, nc - c * T);
    const char* src = m->W[l - 1] + ((size_t)(r * T) * nc + (size_t)c * T) * m->es;
    TG_HIP(hipMemcpy2DAsync(wc.ptr(slot), (size_t)T * m->es, src, (size_t)nc * m->es, (size_t)cols * m->es, (size_t)rows,
                            hipMemcpyHostToDevice, fetch));
    ctx->stats.h2d_bytes += rows * cols * (int64_t)m->es;
    TG_HIP(hipEventRecord(s.ready, fetch));
    s.fetch_seq = ++wc.fetch_issue;
    *slot_out = slot;
    if (ctx->opts.trace) { rec.hit = 0; rec.slot = slot; m->trace.push_back(rec); }
    return TGEMM_OK;
}

// Claims the next table-ring entry (waits on the host until the launch that last used it is done,
// which also bounds how far the host runs ahead of the GPU).
int ring_claim(tgemm_mlp* m, int* entry)
{
    TableRing& r = m->ring;
    const int e = r.next;
    r.next = (r.next + 1) % TableRing::N;
    if (r.used[e]) {
        TG_HIP(hipEventSynchronize(r.done[e]));
        m->cache.reads_done_upto(r.seq[e]);      // launches finish in order
    }
    r.used[e] = false;
    *entry = e;
    return TGEMM_OK;
}

// Uploads the table of `n` slot pointers for the next launch and makes the compute stream wait for it.
// The table travels on the fetch stream, behind the launch's own tile fetches: the compute stream then
// holds nothing but kernels (a small copy between two kernels on one stream cost 12 of the 18 us that
// lay between launches), and since fetches complete in issue order the one wait covers the tiles too.
int ring_publish(tgemm_mlp* m, int entry, const int* tile_slots, int n)
{
    TableRing& r = m->ring;
    WeightCache& wc = m->cache;
    hipStream_t comp = m->ctx->streams[1], fetch = m->ctx->streams[0];
    for (int i = 0; i < n; ++i) r.host[entry][i] = wc.ptr(tile_slots[i]);
    TG_HIP(hipMemcpyAsync(r.dev[entry], r.host[entry], (size_t)n * sizeof(void*), hipMemcpyHostToDevice, fetch));
    TG_HIP(hipEventRecord(r.table_ready[entry], fetch));
    TG_HIP(hipStreamWaitEvent(comp, r.table_ready[entry], 0));
    wc.fetch_waited = wc.fetch_issue;
    return TGEMM_OK;
}

int ring_finish(tgemm_mlp* m, int entry, const int* tile_slots, int n)
{
    TableRing& r = m->ring;
    hipStream_t comp = m->ctx->streams[1];
    TG_HIP(hipEventRecord(r.done[entry], comp));
    r.used[entry] = true;
    WeightCache& wc = m->cache;
    const int64_t seq = ++wc.read_issue;
    r.seq[entry] = seq;
    for (int i = 0; i < n; ++i) {
        WSlot& s = wc.slots[tile_slots[i]];
        s.read = r.done[entry];
        s.read_pending = true;
        s.read_seq = seq;
    }
    wc.reads.push_back({seq, r.done[entry]});
    return TGEMM_OK;
}

int launch(tgemm_mlp* m, GemmDesc& d, hipStream_t st)
{
    d.T = m->T;
    d.config = m->ctx->opts.kernel_config;
    hipError_t e = launch_tile_gemm(d, m->dtype == TGEMM_BF16, st);
    if (e != hipSuccess) return fail(TGEMM_EHIP, "mlp: tile GEMM launch failed: %s", hipGetErrorString(e));
    m->ctx->stats.kernel_launches++;
    m->ctx->stats.n_tile_gemms += cdiv(d.M, d.T) * cdiv(d.N, d.T) * cdiv(d.K, d.T);
    return TGEMM_OK;
}

hipStream_t compute_stream(tgemm_mlp* m) { return m->ctx->streams[m->ooc ? 1 : 0]; }

// equation 1 for layer l: out = epilogue(A_{l-1} W_l); out: batch x n_l (the layer's activation
// matrix in the network's element type, or the float logits for the last layer)
int forward_layer(tgemm_mlp* m, int l, const char* in, int64_t batch, char* out)
{
    const int L = m->n_layers;
    const bool bf = m->dtype == TGEMM_BF16;
    GemmDesc d;
    memset(&d, 0, sizeof d);
    d.A = in; d.lda = m->dims[l - 1]; d.a_kcontig = 1;                  // A_{l-1}: batch x n_{l-1}
    d.b_kcontig = 0;                                                     // W_l: n_{l-1} x n_l
    d.M = batch; d.K = m->dims[l - 1];
    d.epilogue = (l < L) ? EPI_ACT : EPI_AXPBY;
    d.act = m->act_kind;
    d.alpha = 1.f; d.beta = 0.f;
    d.out_bf16 = (bf && l < L) ? 1 : 0;                                  // logits stay float
    const size_t out_es = (l < L) ? m->es : 4;
    d.ldc = m->dims[l];
    const float* b = m->bias.empty() ? nullptr : m->bias[(size_t)l - 1];
    if (!m->ooc) {
        d.B = m->W[l - 1]; d.ldb = m->dims[l];
        d.C = (float*)out; d.N = m->dims[l];
        d.bias = b;
        return launch(m, d, compute_stream(m));
    }
    // out-of-core: one launch per tile column j of W_l, over the whole batch and all k-steps
    const int64_t T = m->T, n_k = cdiv(m->dims[l - 1], T), n_j = cdiv(m->dims[l], T);
    std::vector<int> tiles((size_t)n_k);
    for (int64_t j = 0; j < n_j; ++j) {
        int entry, rc;
        if ((rc = ring_claim(m, &entry)) != TGEMM_OK) return rc;
        for (int64_t k = 0; k < n_k; ++k)
            if ((rc = acquire_tile(m, l, k, j, false, &tiles[(size_t)k])) != TGEMM_OK) return rc;
        if ((rc = ring_publish(m, entry, tiles.data(), (int)n_k)) != TGEMM_OK) return rc;
        d.b_tiles = (const void* const*)m->ring.dev[entry];
        d.B = m->cache.ptr(tiles[0]); d.ldb = T;
        d.C = (float*)(out + (size_t)(j * T) * out_es);
        d.N = std::min(T, m->dims[l] - j * T);
        d.bias = b ? b + j * T : nullptr;
        if ((rc = launch(m, d, compute_stream(m))) != TGEMM_OK) return rc;
        if ((rc = ring_finish(m, entry, tiles.data(), (int)n_k)) != TGEMM_OK) return rc;
        ++m->cache.launch_id;
    }
    return TGEMM_OK;
}

int forward(tgemm_mlp* m, const char* X, int64_t batch)
{
    const char* in = X;
    for (int l = 1; l <= m->n_layers; ++l) {
        const int rc = forward_layer(m, l, in, batch, (l < m->n_layers) ? m->act[l] : (char*)m->logits);
        if (rc != TGEMM_OK) return rc;
        in = (l < m->n_layers) ? m->act[l] : nullptr;
    }
    m->X = X;
    m->batch = batch;
    m->have_delta = false;
    return TGEMM_OK;
}

// Row-wise softmax of `logits` (batch x n_L floats, 16-byte aligned): probabilities to `probs`, and
// with labels the error matrix to `delta` and the row losses to `row_loss` (any of them may be NULL).
int softmax_rows(tgemm_mlp* m, const float* logits, int64_t batch, const int32_t* labels, float* probs, void* delta,
                 float* row_loss)
{
    const int L = m->n_layers;
    const int64_t n = m->dims[L];
    const bool vec = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(probs) & 15) == 0);   // the workspaces are aligned
    const dim3 grid((unsigned)batch), block(256);
    const float inv_batch = 1.f / (float)batch;
    hipStream_t st = compute_stream(m);
#define TG_SOFTMAX(BF, V) \
    hipLaunchKernelGGL((softmax_xent_rows<BF, V>), grid, block, 0, st, logits, n, (int)n, labels, inv_batch, delta, probs, row_loss)
    if (m->dtype == TGEMM_BF16) { if (vec) TG_SOFTMAX(true, true); else TG_SOFTMAX(true, false); }
    else { if (vec) TG_SOFTMAX(false, true); else TG_SOFTMAX(false, false); }
#undef TG_SOFTMAX
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(TGEMM_EHIP, "mlp: softmax launch failed: %s", hipGetErrorString(e));
    return TGEMM_OK;
}

int softmax(tgemm_mlp* m, const int32_t* labels, float* probs, bool want_delta)
{
    return softmax_rows(m, m->logits, m->batch, labels, probs, want_delta ? (void*)m->delta[m->n_layers] : nullptr, m->row_loss);
}

int sync_all(tgemm_mlp* m)
{
    for (int s = 0; s < 4; ++s) TG_HIP(hipStreamSynchronize(m->ctx->streams[s]));
    for (auto& s : m->cache.slots) s.read_pending = s.flush_pending = false;
    m->cache.all_reads_done();
    m->cache.all_flushes_done();
    m->cache.fetch_waited = m->cache.fetch_issue;
    for (auto& u : m->ring.used) u = false;
    return TGEMM_OK;
}

// End of a step with deferred write-back: fetches and kernels are complete, the write-backs queued on
// the flush stream are not.  A slot keeps flush_pending; whoever overwrites it next (an eviction's
// fetch, the next update) waits for its `flushed` event first.
int sync_compute(tgemm_mlp* m)
{
    for (int s = 0; s < 3; ++s) TG_HIP(hipStreamSynchronize(m->ctx->streams[s]));
    for (auto& s : m->cache.slots) s.read_pending = false;
    m->cache.all_reads_done();
    m->cache.fetch_waited = m->cache.fetch_issue;
    WeightCache::advance(m->cache.flushes, m->cache.flush_done);     // keeps the queue to what is in flight
    for (auto& u : m->ring.used) u = false;
    return TGEMM_OK;
}

int read_loss(tgemm_mlp* m, float* loss)
{
    hipStream_t st = compute_stream(m);
    std::vector<float> rows((size_t)m->batch);
    TG_HIP(hipMemcpyAsync(rows.data(), m->row_loss, (size_t)m->batch * 4, hipMemcpyDeviceToHost, st));
    TG_HIP(hipStreamSynchronize(st));
    double s = 0.0;
    for (float v : rows) s += v;
    if (loss) *loss = (float)(s / (double)m->batch);
    return TGEMM_OK;
}

// T rows of an out-of-core fp32 matrix into the next device buffer (fetch stream); the compute stream
// waits for them.  The buffer's previous contents have been written back.
int rows_fetch(tgemm_mlp* m, RowStream& rs, const float* host_rows, size_t bytes, hipStream_t comp, int* which)
{
    hipStream_t fetch = m->ctx->streams[0];
    const int b = rs.next;
    rs.next ^= 1;
    if (rs.in_use[b]) TG_HIP(hipStreamWaitEvent(fetch, rs.freed[b], 0));
    TG_HIP(hipMemcpyAsync(rs.buf[b], host_rows, bytes, hipMemcpyHostToDevice, fetch));
    TG_HIP(hipEventRecord(rs.ready[b], fetch));
    TG_HIP(hipStreamWaitEvent(comp, rs.ready[b], 0));
    m->ctx->stats.h2d_bytes += (int64_t)bytes;
    *which = b;
    return TGEMM_OK;
}
// ... and back to the host matrix (flush stream, which already waits for the launch that updated them)
int rows_writeback(tgemm_mlp* m, RowStream& rs, int b, float* host_rows, size_t bytes)
{
    hipStream_t flush = m->ctx->streams[3];
    TG_HIP(hipMemcpyAsync(host_rows, rs.buf[b], bytes, hipMemcpyDeviceToHost, flush));
    TG_HIP(hipEventRecord(rs.freed[b], flush));
    rs.in_use[b] = true;
    rs.last_freed = rs.freed[b];
    m->ctx->stats.d2h_bytes += (int64_t)bytes;
    return TGEMM_OK;
}


// equations 4 and 3 for layer l.  update: W_l <- W_l - lr dW_l in place of storing dW_l; dW_out:
// optional dense float destination for the plain gradient.
int backward_layer(tgemm_mlp* m, int l, float* dW_out, bool update, float lr)
{
    const bool bf = m->dtype == TGEMM_BF16;
    const int64_t batch = m->batch, T = m->T;
    const char* a_prev = (l == 1) ? m->X : m->act[l - 1];
    hipStream_t comp = compute_stream(m);

    if (!m->bias.empty()) {   // db_l = 1^T D_l; D_l is complete on the compute stream at this point
        float* db = m->dbias.empty() ? nullptr : m->dbias[(size_t)l - 1];
        float* b = update ? m->bias[(size_t)l - 1] : nullptr;
        if (db || b) {
            const int n = (int)m->dims[l], bands = (int)cdiv(batch, COLSUM_ROWS);
            const bool vec = (n % 4 == 0) && ((reinterpret_cast<uintptr_t>(m->delta[l]) & 15) == 0);
            const dim3 grid((unsigned)cdiv(n, vec ? 1024 : 256), (unsigned)bands);
            const void* D = m->delta[l];
            if (bf && vec) hipLaunchKernelGGL((colsum_partial<true, 4>), grid, dim3(256), 0, comp, D, (int64_t)n, batch, n, m->colsum_part);
            else if (bf) hipLaunchKernelGGL((colsum_partial<true, 1>), grid, dim3(256), 0, comp, D, (int64_t)n, batch, n, m->colsum_part);
            else if (vec) hipLaunchKernelGGL((colsum_partial<false, 4>), grid, dim3(256), 0, comp, D, (int64_t)n, batch, n, m->colsum_part);
            else hipLaunchKernelGGL((colsum_partial<false, 1>), grid, dim3(256), 0, comp, D, (int64_t)n, batch, n, m->colsum_part);
            hipLaunchKernelGGL(colsum_finish, dim3((unsigned)cdiv(n, 256)), dim3(256), 0, comp,
                               (const float*)m->colsum_part, bands, n, lr, b, db, m->mu,
                               (b && !m->vel_bias.empty()) ? m->vel_bias[(size_t)l - 1] : (float*)nullptr);
            TG_HIP(hipGetLastError());
        }
    }

    GemmDesc da;   // D_{l-1} = (D_l W_l^T) * A_{l-1} * (1 - A_{l-1})
    memset(&da, 0, sizeof da);
    da.A = m->delta[l]; da.lda = m->dims[l]; da.a_kcontig = 1;             // D_l: batch x n_l
    da.b_kcontig = 1;                                                      // W_l stored n_{l-1} x n_l = N x K
    da.M = batch; da.K = m->dims[l];
    da.ldc = m->dims[l - 1]; da.ldaux = m->dims[l - 1];
    da.epilogue = EPI_DACT; da.alpha = 1.f; da.beta = 0.f;
    da.act = m->act_kind;
    da.out_bf16 = bf ? 1 : 0;

    GemmDesc dw;   // dW_l = A_{l-1}^T D_l
    memset(&dw, 0, sizeof dw);
    dw.lda = m->dims[l - 1]; dw.a_kcontig = 0;                             // A_{l-1} stored K x M (batch x n_{l-1})
    dw.B = m->delta[l]; dw.ldb = m->dims[l]; dw.b_kcontig = 0;             // D_l: batch x n_l
    dw.N = m->dims[l]; dw.K = batch;
    dw.epilogue = EPI_AXPBY;

    if (!m->ooc) {
        if (l > 1) {   // reads W_l before it is updated below
            da.B = m->W[l - 1]; da.ldb = m->dims[l];
            da.C = (float*)m->delta[l - 1]; da.aux = a_prev; da.N = m->dims[l - 1];
            const int rc = launch(m, da, comp);
            if (rc != TGEMM_OK) return rc;
        }
        if (update || dW_out) {
            dw.A = a_prev; dw.M = m->dims[l - 1]; dw.ldc = m->dims[l];
            if (update) {
                dw.C = (float*)m->W[l - 1]; dw.alpha = -lr; dw.beta = 1.f; dw.out_bf16 = bf ? 1 : 0;
                if (!m->vel.empty()) {   // V <- mu V + dW; W <- W - lr V
                    dw.epilogue = EPI_MOMENTUM;
                    dw.state = m->vel[(size_t)l - 1]; dw.ldstate = m->dims[l]; dw.mu = m->mu;
                }
                if (!m->master.empty()) {   // the step goes to the fp32 copy; W becomes its rounded image
                    dw.master = m->master[(size_t)l - 1]; dw.ldmaster = m->dims[l];
                }
                dw.sr = (bf && m->round_mode == TGEMM_ROUND_STOCHASTIC) ? 1 : 0;
                dw.sr_key = sr_step_key(m->sr_seed, (uint32_t)l, m->sr_step); dw.sr_row0 = 0;
            }
            else { dw.C = dW_out; dw.alpha = 1.f; dw.beta = 0.f; dw.out_bf16 = 0; }
            const int rc = launch(m, dw, comp);
            if (rc != TGEMM_OK) return rc;
        }
        return TGEMM_OK;
    }

    // out-of-core: walk W_l by tile rows r.  The row's tiles serve D W^T (pre-update values), then
    // take the update, then are written back to the host weights.
    if (l == 1 && !update && !dW_out) return TGEMM_OK;   // nothing needs W_1
    const int64_t n_r = cdiv(m->dims[l - 1], T), n_c = cdiv(m->dims[l], T);
    hipStream_t flush = m->ctx->streams[3];
    std::vector<int> tiles((size_t)n_c);
    for (int64_t r = 0; r < n_r; ++r) {
        const int64_t rows = std::min(T, m->dims[l - 1] - r * T);
        int rc, entry;
        const bool need_tiles = (l > 1) || update;
        if (need_tiles)
            for (int64_t c = 0; c < n_c; ++c)
                if ((rc = acquire_tile(m, l, r, c, true, &tiles[(size_t)c])) != TGEMM_OK) return rc;
        if (l > 1) {
            if ((rc = ring_claim(m, &entry)) != TGEMM_OK) return rc;
            if ((rc = ring_publish(m, entry, tiles.data(), (int)n_c)) != TGEMM_OK) return rc;
            da.b_tiles = (const void* const*)m->ring.dev[entry];
            da.B = m->cache.ptr(tiles[0]); da.ldb = T;
            da.C = (float*)(m->delta[l - 1] + (size_t)(r * T) * m->es);
            da.aux = a_prev + (size_t)(r * T) * m->es;
            da.N = rows;
            if ((rc = launch(m, da, comp)) != TGEMM_OK) return rc;
            if ((rc = ring_finish(m, entry, tiles.data(), (int)n_c)) != TGEMM_OK) return rc;
        }
        dw.A = a_prev + (size_t)(r * T) * m->es;
        dw.M = rows;
        if (update) {
            // a write-back of the previous step may still be reading these tiles
            WeightCache::advance(m->cache.flushes, m->cache.flush_done);
            hipEvent_t waited = nullptr;
            for (int64_t c = 0; c < n_c; ++c) {
                WSlot& s = m->cache.slots[tiles[(size_t)c]];
                (void)m->cache.settled(s);
                if (s.flush_pending && s.flushed != waited) {
                    TG_HIP(hipStreamWaitEvent(comp, s.flushed, 0));
                    waited = s.flushed;
                }
            }
            if ((rc = ring_claim(m, &entry)) != TGEMM_OK) return rc;
            if ((rc = ring_publish(m, entry, tiles.data(), (int)n_c)) != TGEMM_OK) return rc;
            dw.c_tiles = (void* const*)m->ring.dev[entry];
            dw.C = (float*)m->cache.ptr(tiles[0]); dw.ldc = T;
            dw.alpha = -lr; dw.beta = 1.f; dw.out_bf16 = bf ? 1 : 0;
            dw.sr = (bf && m->round_mode == TGEMM_ROUND_STOCHASTIC) ? 1 : 0;
            dw.sr_key = sr_step_key(m->sr_seed, (uint32_t)l, m->sr_step); dw.sr_row0 = r * T;
            // velocities / master copies of these rows: host -> device buffer -> epilogue -> host
            const size_t band_bytes = (size_t)rows * m->dims[l] * 4, band_at = (size_t)(r * T) * m->dims[l];
            int vb = -1, mb = -1;
            if (!m->vel.empty()) {
                if ((rc = rows_fetch(m, m->vel_rows, m->vel[(size_t)l - 1] + band_at, band_bytes, comp, &vb)) != TGEMM_OK) return rc;
                dw.epilogue = EPI_MOMENTUM;
                dw.state = m->vel_rows.buf[vb]; dw.ldstate = m->dims[l]; dw.mu = m->mu;
            }
            if (!m->master.empty()) {
                if ((rc = rows_fetch(m, m->master_rows, m->master[(size_t)l - 1] + band_at, band_bytes, comp, &mb)) != TGEMM_OK) return rc;
                dw.master = m->master_rows.buf[mb]; dw.ldmaster = m->dims[l];
            }
            if ((rc = launch(m, dw, comp)) != TGEMM_OK) return rc;
            if ((rc = ring_finish(m, entry, tiles.data(), (int)n_c)) != TGEMM_OK) return rc;
            // write the updated row of tiles back (stream 3) once the launch has finished
            TG_HIP(hipStreamWaitEvent(flush, m->ring.done[entry], 0));
            if (vb >= 0 && (rc = rows_writeback(m, m->vel_rows, vb, m->vel[(size_t)l - 1] + band_at, band_bytes)) != TGEMM_OK) return rc;
            if (mb >= 0 && (rc = rows_writeback(m, m->master_rows, mb, m->master[(size_t)l - 1] + band_at, band_bytes)) != TGEMM_OK) return rc;
            hipEvent_t group;
            if ((rc = m->cache.next_flush_event(&group)) != TGEMM_OK) return rc;
            const int64_t flush_seq = ++m->cache.flush_issue;
            for (int64_t c = 0; c < n_c; ++c) {
                const int64_t cols = std::min(T, m->dims[l] - c * T);
                char* dst = m->W[l - 1] + ((size_t)(r * T) * m->dims[l] + (size_t)c * T) * m->es;
                TG_HIP(hipMemcpy2DAsync(dst, (size_t)m->dims[l] * m->es, m->cache.ptr(tiles[(size_t)c]), (size_t)T * m->es,
                                        (size_t)cols * m->es, (size_t)rows, hipMemcpyDeviceToHost, flush));
                m->ctx->stats.d2h_bytes += rows * cols * (int64_t)m->es;
                WSlot& s = m->cache.slots[tiles[(size_t)c]];
                s.flushed = group;
                s.flush_pending = true;
                s.flush_seq = flush_seq;
            }
            TG_HIP(hipEventRecord(group, flush));
            m->cache.flushes.push_back({flush_seq, group});
        } else if (dW_out) {
            dw.c_tiles = nullptr;
            dw.C = dW_out + (size_t)(r * T) * m->dims[l]; dw.ldc = m->dims[l];
            dw.alpha = 1.f; dw.beta = 0.f; dw.out_bf16 = 0;
            if ((rc = launch(m, dw, comp)) != TGEMM_OK) return rc;
        }
        ++m->cache.launch_id;
    }
    return TGEMM_OK;
}

int backward(tgemm_mlp* m, void* const* dW, bool update, float lr)
{
    // rows written back by an earlier step (deferred write-back) are on the host before this step
    // fetches any of them again
    for (RowStream* rs : {&m->vel_rows, &m->master_rows})
        if (update && rs->last_freed) TG_HIP(hipStreamWaitEvent(m->ctx->streams[0], rs->last_freed, 0));
    for (int l = m->n_layers; l >= 1; --l) {
        const int rc = backward_layer(m, l, dW ? (float*)dW[l - 1] : nullptr, update, lr);
        if (rc != TGEMM_OK) return rc;
    }
    return TGEMM_OK;
}

int check_batch(tgemm_mlp* m, const void* X, int64_t batch)
{
    if (!m) return fail(TGEMM_EARG, "mlp: object is NULL");
    if (!X || batch <= 0 || batch > ((int64_t)1 << 28)) return fail(TGEMM_EARG, "mlp: bad input or batch %lld", (long long)batch);
    if (classify_pointer(X, m->ctx->device) != PTR_DEVICE) return fail(TGEMM_EARG, "mlp: X must be a device pointer");
    return TGEMM_OK;
}

// After a pass that failed part-way: wait for whatever was enqueued (ignoring further errors) and
// forget the pass, so that nothing runs on half-overwritten activations afterwards.
void abandon_pass(tgemm_mlp* m)
{
    (void)hipSetDevice(m->ctx->device);
    for (int s = 0; s < 4; ++s) (void)hipStreamSynchronize(m->ctx->streams[s]);
    (void)hipGetLastError();
    for (auto& s : m->cache.slots) s.read_pending = s.flush_pending = false;
    m->cache.all_reads_done();
    m->cache.all_flushes_done();
    m->cache.fetch_waited = m->cache.fetch_issue;
    for (auto& u : m->ring.used) u = false;
    m->batch = 0;
    m->have_delta = false;
}

void begin_call(tgemm_mlp* m)
{
    memset(&m->ctx->stats, 0, sizeof m->ctx->stats);
    m->trace.clear();
    m->ctx->stats.in_core = m->ooc ? 0 : 1;
    m->ctx->stats.n_slots = m->cache.n_slots;
}

}  // namespace
}  // namespace tg

using namespace tg;

extern "C" {

int mlp_create(tgemm_ctx* ctx, tgemm_mlp** out, int32_t n_layers, const int64_t* dims, void* const* W,
               int32_t dtype, int32_t T, size_t hbm_budget)
{
    if (!out) return fail(TGEMM_EARG, "mlp_create: out is NULL");
    *out = nullptr;
    if (!ctx || !dims || !W || n_layers < 1 || n_layers > 64 || T <= 0)
        return fail(TGEMM_EARG, "mlp_create: bad argument");
    if (dtype != TGEMM_F32 && dtype != TGEMM_BF16) return fail(TGEMM_EARG, "mlp_create: unknown dtype %d", dtype);
    for (int l = 0; l <= n_layers; ++l)
        if (dims[l] <= 0 || dims[l] > ((int64_t)1 << 28)) return fail(TGEMM_EARG, "mlp_create: dims[%d] = %lld", l, (long long)dims[l]);
    TG_HIP(hipSetDevice(ctx->device));
    int n_dev = 0, n_host = 0;
    for (int l = 0; l < n_layers; ++l) {
        if (!W[l]) return fail(TGEMM_EARG, "mlp_create: W[%d] is NULL", l);
        const PtrKind k = classify_pointer(W[l], ctx->device);
        if (k == PTR_PAGEABLE) return fail(TGEMM_EUNPINNED, "mlp_create: W[%d] is pageable host memory", l);
        if (k == PTR_DEVICE) ++n_dev; else ++n_host;
    }
    if (n_dev && n_host) return fail(TGEMM_EARG, "mlp_create: weights must be all device or all pinned host pointers");
    if (n_host && hbm_budget == 0) return fail(TGEMM_EBUDGET, "mlp_create: host-resident weights need an hbm_budget");
    tgemm_mlp* m = new (std::nothrow) tgemm_mlp();
    if (!m) return fail(TGEMM_ENOMEM, "mlp_create: host allocation failed");
    m->ctx = ctx;
    m->n_layers = n_layers;
    m->dims.assign(dims, dims + n_layers + 1);
    for (int l = 0; l < n_layers; ++l) m->W.push_back((char*)W[l]);
    m->dtype = dtype;
    m->es = dtype == TGEMM_BF16 ? 2 : 4;
    m->T = T;
    m->budget = hbm_budget;
    m->ooc = n_host > 0;
    m->cache.exact = ctx->opts.exact_replacement != 0;
    m->act.assign(n_layers + 1, nullptr);
    m->delta.assign(n_layers + 1, nullptr);
    *out = m;
    return TGEMM_OK;
}

int mlp_set_activation(tgemm_mlp* m, int32_t act)
{
    if (!m) return fail(TGEMM_EARG, "mlp_set_activation: object is NULL");
    if (act != TGEMM_ACT_SIGMOID && act != TGEMM_ACT_TANH && act != TGEMM_ACT_RELU)
        return fail(TGEMM_EARG, "mlp_set_activation: unknown activation %d", act);
    static_assert(TGEMM_ACT_SIGMOID == ACT_SIGMOID && TGEMM_ACT_TANH == ACT_TANH && TGEMM_ACT_RELU == ACT_RELU,
                  "activation codes of the ABI and of the kernels");
    m->act_kind = act;
    m->batch = 0;          // activations of an earlier forward pass belong to the old function
    m->have_delta = false;
    return TGEMM_OK;
}

int mlp_set_bias(tgemm_mlp* m, void* const* b, void* const* db)
{
    if (!m) return fail(TGEMM_EARG, "mlp_set_bias: object is NULL");
    TG_HIP(hipSetDevice(m->ctx->device));
    if (!b) {
        if (db) return fail(TGEMM_EARG, "mlp_set_bias: gradient destinations without bias rows");
    } else {
        for (int l = 0; l < m->n_layers; ++l) {
            if (!b[l]) return fail(TGEMM_EARG, "mlp_set_bias: b[%d] is NULL", l);
            hipPointerAttribute_t at;
            if (hipPointerGetAttributes(&at, b[l]) != hipSuccess || at.type != hipMemoryTypeDevice) {
                (void)hipGetLastError();
                return fail(TGEMM_EARG, "mlp_set_bias: b[%d] is not device memory", l);
            }
            if (db && db[l] && (hipPointerGetAttributes(&at, db[l]) != hipSuccess || at.type != hipMemoryTypeDevice)) {
                (void)hipGetLastError();
                return fail(TGEMM_EARG, "mlp_set_bias: db[%d] is not device memory", l);
            }
        }
    }
    int rc = sync_all(m);
    if (rc != TGEMM_OK) return rc;
    const bool had = !m->bias.empty();
    m->bias.clear();
    m->dbias.clear();
    if (b) {
        for (int l = 0; l < m->n_layers; ++l) m->bias.push_back((float*)b[l]);
        if (db) for (int l = 0; l < m->n_layers; ++l) m->dbias.push_back((float*)db[l]);
    }
    if (had != !m->bias.empty()) free_workspaces(m);   // the column-sum scratch comes or goes with the bias terms
    m->batch = 0;            // a pending forward pass belongs to the old function
    m->have_delta = false;
    return TGEMM_OK;
}

int mlp_set_momentum(tgemm_mlp* m, float mu, void* const* V, void* const* Vb)
{
    if (!m) return fail(TGEMM_EARG, "mlp_set_momentum: object is NULL");
    TG_HIP(hipSetDevice(m->ctx->device));
    if (!V) {
        if (Vb) return fail(TGEMM_EARG, "mlp_set_momentum: bias velocities without weight velocities");
    } else {
        if (!(mu >= 0.f && mu < 1.f)) return fail(TGEMM_EARG, "mlp_set_momentum: mu = %g is outside [0, 1)", (double)mu);
        for (int l = 0; l < m->n_layers; ++l) {
            hipPointerAttribute_t at;
            // the velocities live where the weights live
            if (!V[l] || classify_pointer(V[l], m->ctx->device) != (m->ooc ? PTR_PINNED : PTR_DEVICE))
                return fail(TGEMM_EARG, "mlp_set_momentum: V[%d] is not %s", l,
                            m->ooc ? "page-locked host memory (the weights are out-of-core)" : "device memory");
            if (Vb && (!Vb[l] || hipPointerGetAttributes(&at, Vb[l]) != hipSuccess || at.type != hipMemoryTypeDevice)) {
                (void)hipGetLastError();
                return fail(TGEMM_EARG, "mlp_set_momentum: Vb[%d] is not device memory", l);
            }
        }
    }
    int rc = sync_all(m);
    if (rc != TGEMM_OK) return rc;
    if (m->ooc && (V != nullptr) != !m->vel.empty()) free_workspaces(m);   // the row buffers come or go
    m->vel.clear();
    m->vel_bias.clear();
    m->mu = 0.f;
    if (V) {
        for (int l = 0; l < m->n_layers; ++l) m->vel.push_back((float*)V[l]);
        if (Vb) for (int l = 0; l < m->n_layers; ++l) m->vel_bias.push_back((float*)Vb[l]);
        m->mu = mu;
    }
    return TGEMM_OK;
}

int mlp_set_master_weights(tgemm_mlp* m, void* const* Wm)
{
    if (!m) return fail(TGEMM_EARG, "mlp_set_master_weights: object is NULL");
    TG_HIP(hipSetDevice(m->ctx->device));
    if (Wm) {
        if (m->dtype != TGEMM_BF16) return fail(TGEMM_EARG, "mlp_set_master_weights: fp32 weights need no master copy");
        for (int l = 0; l < m->n_layers; ++l)
            if (!Wm[l] || classify_pointer(Wm[l], m->ctx->device) != (m->ooc ? PTR_PINNED : PTR_DEVICE))
                return fail(TGEMM_EARG, "mlp_set_master_weights: Wm[%d] is not %s", l,
                            m->ooc ? "page-locked host memory (the weights are out-of-core)" : "device memory");
    }
    int rc = sync_all(m);
    if (rc != TGEMM_OK) return rc;
    if (m->ooc && (Wm != nullptr) != !m->master.empty()) free_workspaces(m);   // the row buffers come or go
    m->master.clear();
    if (Wm) for (int l = 0; l < m->n_layers; ++l) m->master.push_back((float*)Wm[l]);
    return TGEMM_OK;
}

int mlp_set_rounding(tgemm_mlp* m, int32_t mode, uint64_t seed)
{
    if (!m) return fail(TGEMM_EARG, "mlp_set_rounding: object is NULL");
    if (mode != TGEMM_ROUND_NEAREST && mode != TGEMM_ROUND_STOCHASTIC)
        return fail(TGEMM_EARG, "mlp_set_rounding: unknown mode %d", mode);
    if (mode == TGEMM_ROUND_STOCHASTIC && m->dtype != TGEMM_BF16)
        return fail(TGEMM_EARG, "mlp_set_rounding: stochastic rounding applies to bf16 weights only");
    m->round_mode = mode;
    m->sr_seed = seed;
    m->sr_step = 0;
    return TGEMM_OK;
}

int mlp_destroy(tgemm_mlp* m)
{
    if (!m) return TGEMM_OK;
    (void)hipSetDevice(m->ctx->device);
    for (int s = 0; s < 4; ++s) (void)hipStreamSynchronize(m->ctx->streams[s]);
    free_workspaces(m);
    delete m;
    return TGEMM_OK;
}

static int mlp_forward_body(tgemm_mlp* m, const void* X, int64_t batch, float* probs)
{
    int rc = check_batch(m, X, batch);
    if (rc != TGEMM_OK) return rc;
    const double t0 = now_ms();
    TG_HIP(hipSetDevice(m->ctx->device));
    if ((rc = ensure_workspaces(m, batch)) != TGEMM_OK) return rc;
    begin_call(m);
    if ((rc = forward(m, (const char*)X, batch)) != TGEMM_OK) return rc;
    if (probs && (rc = softmax(m, nullptr, probs, false)) != TGEMM_OK) return rc;
    if ((rc = sync_all(m)) != TGEMM_OK) return rc;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

static int mlp_forward_static_body(tgemm_mlp* m, const void* X, int64_t batch, float* probs)
{
    int rc = check_batch(m, X, batch);
    if (rc != TGEMM_OK) return rc;
    if (!probs) return fail(TGEMM_EARG, "mlp_forward_static: probs is NULL (the logits do not outlive the call)");
    if (m->ooc) return fail(TGEMM_EARG, "mlp_forward_static: the weights must be device-resident");
    const int L = m->n_layers;
    // layout of the scratch array: A_1 .. A_{L-1}, then the logits, each rounded up to 256 bytes
    size_t need = 0;
    for (int l = 1; l < L; ++l) need += ((size_t)batch * m->dims[l] * m->es + 255) / 256 * 256;
    const size_t logits_at = need;
    need += (size_t)batch * m->dims[L] * 4;
    if (need > (size_t)TGEMM_STATIC_SCRATCH_BYTES)
        return fail(TGEMM_EBUDGET, "mlp_forward_static: batch %lld needs %zu bytes of activations and logits, the static "
                    "scratch holds %zu; use mlp_forward", (long long)batch, need, (size_t)TGEMM_STATIC_SCRATCH_BYTES);
    const double t0 = now_ms();
    TG_HIP(hipSetDevice(m->ctx->device));
    void* base = nullptr;
    if ((rc = static_scratch_resolve(m->ctx->device, &base)) != TGEMM_OK) return rc;
    begin_call(m);
    char* at = (char*)base;
    const char* in = (const char*)X;
    for (int l = 1; l <= L; ++l) {
        char* out = (l < L) ? at : (char*)base + logits_at;
        if ((rc = forward_layer(m, l, in, batch, out)) != TGEMM_OK) break;
        in = out;
        if (l < L) at += ((size_t)batch * m->dims[l] * m->es + 255) / 256 * 256;
    }
    if (rc == TGEMM_OK)
        rc = softmax_rows(m, (const float*)((char*)base + logits_at), batch, nullptr, probs, nullptr, nullptr);
    // whatever was launched has finished before the call returns, also after an error
    const hipError_t e = hipStreamSynchronize(compute_stream(m));
    if (rc != TGEMM_OK) return rc;
    if (e != hipSuccess) return fail(TGEMM_EHIP, "mlp_forward_static: %s", hipGetErrorString(e));
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

static int mlp_backward_body(tgemm_mlp* m, const int32_t* labels, void* const* dW, float* loss)
{
    if (!m || !labels) return fail(TGEMM_EARG, "mlp_backward: NULL argument");
    if (m->batch <= 0) return fail(TGEMM_ESTATE, "mlp_backward: no forward pass precedes");
    const double t0 = now_ms();
    TG_HIP(hipSetDevice(m->ctx->device));
    begin_call(m);
    int rc;
    if ((rc = softmax(m, labels, nullptr, true)) != TGEMM_OK) return rc;
    if ((rc = backward(m, dW, false, 0.f)) != TGEMM_OK) return rc;
    if ((rc = read_loss(m, loss)) != TGEMM_OK) return rc;
    if ((rc = sync_all(m)) != TGEMM_OK) return rc;
    m->have_delta = true;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

static int mlp_step_body(tgemm_mlp* m, const void* X, const int32_t* labels, int64_t batch, float lr, float* loss)
{
    int rc = check_batch(m, X, batch);
    if (rc != TGEMM_OK) return rc;
    if (!labels) return fail(TGEMM_EARG, "mlp_step: labels is NULL");
    const double t0 = now_ms();
    TG_HIP(hipSetDevice(m->ctx->device));
    if ((rc = ensure_workspaces(m, batch)) != TGEMM_OK) return rc;
    begin_call(m);
    m->ctx->kernel_timing_pending = false;     // the two events now belong to this step
    TG_HIP(hipEventRecord(m->ctx->ev_start, compute_stream(m)));
    if ((rc = forward(m, (const char*)X, batch)) != TGEMM_OK) return rc;
    if ((rc = softmax(m, labels, nullptr, true)) != TGEMM_OK) return rc;
    if ((rc = backward(m, nullptr, true, lr)) != TGEMM_OK) return rc;
    TG_HIP(hipEventRecord(m->ctx->ev_stop, compute_stream(m)));
    if ((rc = read_loss(m, loss)) != TGEMM_OK) return rc;
    if ((rc = (m->ooc && m->ctx->opts.deferred_writeback) ? sync_compute(m) : sync_all(m)) != TGEMM_OK) return rc;
    {   // time on the compute stream from the step's first launch to its last
        float ms = 0.f;
        TG_HIP(hipEventElapsedTime(&ms, m->ctx->ev_start, m->ctx->ev_stop));
        m->ctx->stats.kernel_ms = ms;
    }
    m->have_delta = true;
    ++m->sr_step;
    m->ctx->stats.wall_ms = now_ms() - t0;
    return TGEMM_OK;
}

int mlp_trace(tgemm_mlp* m, tgemm_mlp_trace_rec* out, int64_t cap, int64_t* n)
{
    if (!m || !n || cap < 0 || (cap > 0 && !out)) return fail(TGEMM_EARG, "mlp_trace: bad argument");
    *n = (int64_t)m->trace.size();
    const int64_t k = cap < *n ? cap : *n;
    if (k > 0) memcpy(out, m->trace.data(), (size_t)k * sizeof(tgemm_mlp_trace_rec));
    return TGEMM_OK;
}

int mlp_read(tgemm_mlp* m, int32_t what, int32_t layer, void* dst, size_t offset, size_t bytes)
{
    if (!m || !dst) return fail(TGEMM_EARG, "mlp_read: NULL argument");
    if (m->batch <= 0) return fail(TGEMM_ESTATE, "mlp_read: no forward pass precedes");
    const int L = m->n_layers;
    const void* src = nullptr;
    size_t have = 0;
    if (what == 0 && layer >= 1 && layer < L) { src = m->act[layer]; have = (size_t)m->batch * m->dims[layer] * m->es; }
    else if (what == 1) { src = m->logits; have = (size_t)m->batch * m->dims[L] * 4; }
    else if (what == 2 && layer >= 1 && layer <= L) {
        if (!m->have_delta) return fail(TGEMM_ESTATE, "mlp_read: no backward pass precedes");
        src = m->delta[layer]; have = (size_t)m->batch * m->dims[layer] * m->es;
    }
    if (!src) return fail(TGEMM_EARG, "mlp_read: what=%d layer=%d", what, layer);
    if (offset > have || bytes > have - offset)
        return fail(TGEMM_EARG, "mlp_read: %zu bytes at offset %zu requested, matrix has %zu", bytes, offset, have);
    TG_HIP(hipSetDevice(m->ctx->device));
    TG_HIP(hipMemcpy(dst, (const char*)src + offset, bytes, hipMemcpyDeviceToHost));
    return TGEMM_OK;
}

// The public forms: no exception crosses the C boundary, and after any error everything that was
// enqueued has finished and the object holds no half-made pass (the next call starts from a clean
// state; mlp_backward then reports TGEMM_ESTATE until a forward pass has succeeded).
#define TG_GUARDED(m, call)                                                                   \
    int rc_;                                                                                  \
    try { rc_ = (call); }                                                                     \
    catch (const std::bad_alloc&) { rc_ = fail(TGEMM_ENOMEM, "mlp: host allocation failed"); } \
    catch (...) { rc_ = fail(TGEMM_EHIP, "mlp: unexpected exception"); }                      \
    /* argument and call-order errors are reported before any work: a pending pass stays usable */ \
    if (rc_ != TGEMM_OK && rc_ != TGEMM_EARG && rc_ != TGEMM_ESTATE && (m)) abandon_pass(m);  \
    if (m) log_call(__func__, (m)->ctx, rc_);                                                 \
    return rc_

int mlp_forward(tgemm_mlp* m, const void* X, int64_t batch, float* probs) { TG_GUARDED(m, mlp_forward_body(m, X, batch, probs)); }
int mlp_forward_static(tgemm_mlp* m, const void* X, int64_t batch, float* probs)
{
    // leaves the object's own pass state alone, also on error (it has drained its stream itself)
    try { return mlp_forward_static_body(m, X, batch, probs); }
    catch (...) { return fail(TGEMM_EHIP, "mlp_forward_static: unexpected exception"); }
}
int mlp_backward(tgemm_mlp* m, const int32_t* labels, void* const* dW, float* loss) { TG_GUARDED(m, mlp_backward_body(m, labels, dW, loss)); }
int mlp_step(tgemm_mlp* m, const void* X, const int32_t* labels, int64_t batch, float lr, float* loss)
{
    TG_GUARDED(m, mlp_step_body(m, X, labels, batch, lr, loss));
}
#undef TG_GUARDED

}  // extern "C"
