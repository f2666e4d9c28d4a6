/*
 * tgemm -- tiled in-core / out-of-core matrix multiplication and the MLP
 * training passes reduced to it, for one MI355X (gfx950).
 *
 * C ABI.  Plain pointers and sizes only.  Every function returns an int
 * status (TGEMM_OK == 0, negative == error) and never throws; the text of the
 * last error on the calling thread is available from tgemm_last_error().
 *
 * Conventions shared by all entry points
 *   - Matrices are dense, row-major, contiguous (leading dimension == number
 *     of columns).
 *   - dtype TGEMM_F32: A, B are float.  dtype TGEMM_BF16: A, B are uint16_t
 *     holding bfloat16 bit patterns.  C and every accumulation are float.
 *   - "device pointer" = memory of the context's GPU (hipMalloc, torch cuda
 *     tensor).  "pinned host pointer" = page-locked host memory
 *     (hipHostMalloc, torch pin_memory).  Pageable host memory is rejected
 *     with TGEMM_EUNPINNED.
 *   - The caller owns every matrix, weight, input and label buffer and keeps
 *     it alive and unmodified for the duration of a call.  The library owns
 *     contexts, its tile cache, workspaces and any stream it created itself.
 *   - Calls are synchronous: on return the result is complete and visible
 *     (unless tgemm_opts.async_incore is set, see tgemm_sync).  After an
 *     error the context stays usable; outputs are unspecified only for
 *     TGEMM_EHIP, which is reported after work has started.
 *   - The library's streams do not synchronise with any other stream: work that produces an input
 *     on another stream (including the null stream) must have completed before a call.
 *   - A context is used by one caller thread at a time.
 *   - TGEMM_LOG=1 in the environment prints one line per tgemm_run / mlp_* call on stderr (status,
 *     wall and kernel time, tasks, launches, cache hits / misses / evictions, host-link bytes).
 */
#ifndef TGEMM_H
#define TGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tgemm_ctx tgemm_ctx;
typedef struct tgemm_mlp tgemm_mlp;

enum { TGEMM_F32 = 0, TGEMM_BF16 = 1 };

enum {
    TGEMM_OK = 0,
    TGEMM_EARG = -1,      /* null / aliasing / non-positive size / unknown enum / mixed pointer kinds */
    TGEMM_ENOMEM = -2,    /* host or device allocation failed */
    TGEMM_EUNPINNED = -3, /* a host pointer is not page-locked */
    TGEMM_EBUDGET = -4,   /* hbm_budget below the minimum working set */
    TGEMM_EHIP = -5,      /* a HIP call failed after work started */
    TGEMM_ESTATE = -6     /* call order violated (e.g. backward before forward) */
};

/* Order in which output-tile tasks are issued (the result does not depend on it, the tile-cache
 * traffic does).
 *   ROW_MAJOR   tile rows top to bottom, columns left to right.
 *   SERPENTINE  as ROW_MAJOR, but odd tile rows run right to left.
 *   STRIPS      column strips of `strip` tile columns, left to right; inside a strip the tile rows
 *               ascend (even strips) or descend (odd strips), and inside a tile row the strip's
 *               columns ascend.  With strip <= slots / k-steps - 2 the strip's B tiles and two row
 *               panels of A fit in the cache together, so under strict LRU B is fetched once and
 *               A once per strip; the automatic width shares the tile columns out evenly over the
 *               fewest strips of at most that width. */
enum { TGEMM_ORDER_SERPENTINE = 0, TGEMM_ORDER_ROW_MAJOR = 1, TGEMM_ORDER_STRIPS = 2 };

enum { TGEMM_SCHEDULE_AUTO = 0, TGEMM_SCHEDULE_ONE_LAUNCH = 1, TGEMM_SCHEDULE_BALANCED = 2 };

typedef struct tgemm_opts {
    int32_t trace;         /* 1: record one tgemm_trace_rec per tile product of out-of-core runs */
    int32_t order;         /* TGEMM_ORDER_* */
    int32_t affinity_core; /* >= 0: bind the submit thread to this CPU core (section 3.2, "GPU
                              computation thread"); -1: leave it to the OS */
    int32_t async_incore;  /* 1: in-core tgemm_run returns after enqueueing; see tgemm_sync */
    int32_t kernel_config; /* 0: automatic; 1..3 force a macro-tile shape (small, medium, large);
                              4: large, bf16 register-staged kernel even where the direct-to-LDS one applies */
    int32_t strip_width;   /* TGEMM_ORDER_STRIPS: tile columns per strip; 0 = from the slot count */
    int32_t deferred_writeback; /* 1: an out-of-core mlp_step returns once its kernels are done and lets
                              the write-back of updated weight tiles run on into the next call; the
                              host weights are complete after tgemm_sync, mlp_forward, mlp_backward
                              or mlp_destroy */
    int32_t rs_depth;      /* out-of-core tgemm_run, the reservation station of section 3.2: 0 or 1: tasks go
                              to the streams in queue order; n > 1 (at most 64): the station holds the next
                              n tasks of the queue, and whenever a stream is free the one with the most
                              input tiles (A_ik and B_kj over all k) in the tile cache leaves first, ties
                              going to the one that entered first */
    int32_t exact_replacement; /* out-of-core MLP weight cache: 1: the victim of a miss is always the cached
                              tile (outside the launch being assembled) whose next use in the step's
                              sweep lies furthest ahead -- a pure function of sizes, T and slot count.
                              0 (default): among the tiles whose next use is at least half as far as
                              that, one with no read or write-back in flight is preferred, so that
                              fetches keep running ahead of the products; which tile that is depends
                              on timing, the number of misses need not */
    int32_t keep_tiles;    /* out-of-core tgemm_run: 1: A/B tiles stay in the tile cache from one call on the
                              context to the next (section 3.4: tiles are cached for reuse), with their
                              recency order, as long as tile size, slot sizes and slot count of the calls
                              agree (a call with another geometry starts with an empty cache).  A cached
                              tile is recognised by its host matrix (base pointer, shape, element size,
                              T) and its tile indices.  The caller then owns coherence: after changing a
                              host matrix that earlier calls have read (or reusing its memory for
                              another matrix), call tgemm_invalidate before the next tgemm_run, or stale
                              tiles are used.  0 (default): every call starts with an empty cache */
    int32_t incore_schedule; /* in-core tgemm_run with the automatic kernel shape (bf16: only products whose M
                              and N are multiples of 256, so there is no remainder launch).
                              TGEMM_SCHEDULE_AUTO (0, default): where the 256 x 256 macro tiles do not fill
                              whole rounds of one tile per compute unit (and T is a multiple of 256, K of
                              32, rows 16-byte aligned) and a cost estimate promises a gain, the tiles of
                              the last, partial round are cut along k into segments that run on all units
                              and leave partial sums in a 128 MiB device workspace (allocated by the
                              context at the first such call); a second kernel adds a tile's sums in
                              ascending order of k, and then C.  Rows and columns beyond the last
                              multiple of 256 run as a launch of their own.  Elements of those tiles are
                              then sums of several chains over consecutive parts of the k range (about
                              compute units / tiles of the partial round of them, at least two) instead
                              of one chain; which parts depends on the sizes and the number of compute
                              units only (tgemm_balance_plan shows them).
                              TGEMM_SCHEDULE_ONE_LAUNCH (1): always one launch, one chain per element (also
                              the mode for callers that may not allocate or copy inside tgemm_run: the
                              balanced schedule allocates its workspace at the first qualifying call and
                              uploads its tables whenever the sizes change).
                              TGEMM_SCHEDULE_BALANCED (2): the balanced schedule wherever it applies,
                              whatever the estimate says */
} tgemm_opts;

/* One output tile C_ij = one task (section 3.1; Algorithm 1, "decode").
 * id = i * n_j + j.  Row range [r0, r1), column range [c0, c1); n_k = number of k-steps. */
typedef struct tgemm_task {
    int64_t id, i, j, r0, r1, c0, c1, n_k;
} tgemm_task;

typedef struct tgemm_stats {
    double wall_ms;        /* host wall clock of the last tgemm_run / mlp_* call                  */
    double kernel_ms;      /* HIP-event time on the launch stream around the GEMM kernel(s) of the
                              last in-core tgemm_run, or from the first to the last launch of the
                              last mlp_step on its compute stream (0 for out-of-core tgemm_run,
                              mlp_forward and mlp_backward)                                        */
    int64_t in_core;       /* 1 if the last run was in-core                                       */
    int64_t n_tasks;       /* output tiles                                                        */
    int64_t n_tile_gemms;  /* tile products C_ij += A_ik B_kj                                      */
    int64_t n_slots;       /* A/B tile-cache slots the budget allowed (out-of-core)               */
    int64_t hits, misses, evictions; /* tile-cache lookups (out-of-core)                          */
    int64_t h2d_bytes, d2h_bytes;    /* bytes moved over the host link (out-of-core)              */
    int64_t kernel_launches;
} tgemm_stats;

/* One tile product of an out-of-core run, in issue order (Algorithm 1, the k loop). */
typedef struct tgemm_trace_rec {
    int64_t task_id;
    int32_t i, j, k;       /* C tile (i,j), step k: uses A tile (i,k) and B tile (k,j)            */
    int32_t stream;        /* 0..3: the reservation-station slot (C tile buffer) the task used    */
    int32_t a_hit, b_hit;  /* 1: tile was in the cache, 0: fetched from host memory               */
    int32_t a_slot, b_slot;
    int32_t a_evicted, b_evicted; /* 1: the fetch displaced another tile                          */
} tgemm_trace_rec;

const char* tgemm_strerror(int code);
const char* tgemm_last_error(void);

/* Section 3.5, Algorithm 1 lines 1-4: creates the runtime of one GPU -- 4 streams and 4 task slots
 * (section 3.2: four concurrent tasks per GPU), the task queue, the tile cache directory and the
 * submit thread.  Out-of-core runs use the streams as a pipeline: streams[0] fetches tiles from host
 * memory, streams[1] and streams[2] run the tile products, streams[3] harvests finished C tiles;
 * in-core runs and the MLP passes launch on streams[0].
 *   device   HIP device ordinal.
 *   streams  NULL, or 4 hipStream_t values (as void*) borrowed from the caller for the lifetime of
 *            the context; entries that are NULL are taken from the library's own set of four streams
 *            for that device, which is created at first need and kept until the process ends, so
 *            contexts on one device that bring no streams share them (work of two such contexts is
 *            ordered per stream; results never depend on it).  All streams must have default priority.
 *   opts     NULL for defaults (no trace, strips order with automatic width, no core binding,
 *            synchronous, queue order).
 * Errors: TGEMM_EARG (out == NULL, bad device, bad enum), TGEMM_EHIP, TGEMM_ENOMEM. */
int tgemm_create(tgemm_ctx** out, int device, void* const* streams, const tgemm_opts* opts);

/* Frees everything the context owns.  NULL is accepted.  All work has completed on return. */
int tgemm_destroy(tgemm_ctx* ctx);

/* Section 3.1 + Algorithm 1: C <- C + A B computed tile by tile.
 *   A  M x K, B  K x N (dtype elements), C  M x N float, all row-major contiguous; C is read and
 *      written; A, B, C must not overlap.
 *   T  tile size (> 0).  Output tile (i,j) is one task; it accumulates A_ik B_kj for k ascending;
 *      edge tiles are clamped to the matrix.
 *   All three pointers device pointers  -> in-core: one kernel launch covers every task, hbm_budget
 *      is ignored (possibly a few launches with a workspace, see tgemm_opts.incore_schedule).
 *   All three pointers pinned host      -> out-of-core: A/B tiles are staged into an HBM tile cache
 *      (LRU, section 3.4); C tiles are uploaded, accumulated and harvested; fetch, products and
 *      harvest overlap on the 4 streams with 4 tasks in flight.  Every
 *      device byte allocated for the call (A/B slots + 4 C slots) stays within hbm_budget bytes;
 *      the minimum is 4 C slots + 8 A/B slots (TGEMM_EBUDGET otherwise, before any work).
 *      Unless tgemm_opts.keep_tiles is set, the cache directory starts empty at every call: no tile
 *      survives from one call to the next, so the caller may change A and B between calls freely.
 *      With keep_tiles see tgemm_invalidate.  C tiles are never kept: on return no tile of C remains
 *      on the device only.  The slot pool is exactly what the call's budget allows (a larger one left
 *      by an earlier call is given back first).
 *   At most 2^31 tasks and 2^40 tile products (TGEMM_EARG above that: use a larger T).
 *   M, N or K == 0 is legal (C unchanged).
 * Errors: TGEMM_EARG, TGEMM_EUNPINNED, TGEMM_EBUDGET, TGEMM_ENOMEM, TGEMM_EHIP. */
int tgemm_run(tgemm_ctx* ctx, const void* A, const void* B, void* C,
              int64_t M, int64_t N, int64_t K, int32_t T, int32_t dtype, size_t hbm_budget);

/* Section 3.4 keeps tiles in GPU memory for later reuse.  With tgemm_opts.keep_tiles that holds across
 * calls, and a caller who has changed a host matrix (or reused its memory) must have its cached tiles
 * dropped: this call waits for the context's streams, then removes every cached tile of every matrix
 * whose base pointer is host_base; their slots are free for the next fetches.  Without keep_tiles no
 * tile outlives a call and there is nothing to drop (the call still succeeds).  Out-of-core MLP
 * weights are not touched (see mlp_create).
 * TGEMM_EARG if ctx or host_base is NULL. */
int tgemm_invalidate(tgemm_ctx* ctx, const void* host_base);

/* Waits for everything enqueued on the context's streams (only needed with opts.async_incore). */
int tgemm_sync(tgemm_ctx* ctx);

/* Section 3.1 / Algorithm 1 "decode": the task list of an M x N x K product with tile size T, in id
 * order.  Pure host code, no context needed.  Writes min(cap, n) records to out (out may be NULL
 * when cap == 0) and the total number of tasks to *n_tasks. */
int tgemm_plan(int64_t M, int64_t N, int64_t K, int32_t T, tgemm_task* out, int64_t cap, int64_t* n_tasks);

/* Issue order of the task ids for an n_i x n_j task grid under `order` (`strip` >= 1 is the strip
 * width of TGEMM_ORDER_STRIPS and ignored otherwise); writes n_i * n_j ids. */
int tgemm_task_order(int64_t n_i, int64_t n_j, int32_t order, int64_t strip, int64_t* out_ids);

/* One weight-tile lookup of an out-of-core mlp_forward / mlp_backward / mlp_step, in issue order
 * (section 3.4: a hit uses the cached copy, a miss fetches the tile from host memory).
 * A training step looks tiles up in a fixed sweep: forward, layers ascending, one launch group per
 * tile column of W_l with its tiles by ascending tile row; backward, layers descending, one group per
 * tile row of W_l with its tiles by ascending tile column (without an update the first layer has no
 * backward lookups). */
typedef struct tgemm_mlp_trace_rec {
    int64_t group;          /* running number of the launch group since the object was created */
    int32_t layer, r, c;    /* tile (r, c) of W_layer, layer = 1 .. n_layers                     */
    int32_t backward;       /* 1: the lookup belongs to the backward sweep                        */
    int32_t hit;            /* 1: found in the cache                                              */
    int32_t slot;           /* cache slot that holds the tile from now on                         */
    int32_t ev_layer, ev_r, ev_c; /* the tile the fetch displaced, or -1, -1, -1                  */
} tgemm_mlp_trace_rec;

/* Statistics of the last tgemm_run / mlp_* call on the context. */
int tgemm_last_stats(tgemm_ctx* ctx, tgemm_stats* out);

/* Trace of the last out-of-core run (requires opts.trace).  Copies min(cap, n) records. */
int tgemm_trace(tgemm_ctx* ctx, tgemm_trace_rec* out, int64_t cap, int64_t* n);

/* Section 3.2, non-blocking task queue: pushes n ids from `producers` threads and pops them from
 * `consumers` threads through the library's lock-free queue; writes to popped_count[id] how many
 * times each id came out.  Host-only self test used by the CPU test-suite. */
int tgemm_queue_selftest(int64_t n, int32_t producers, int32_t consumers, int32_t* popped_count);

/* The balanced schedule of an in-core product (tgemm_opts.incore_schedule), for inspection and for the
 * CPU test-suite; host only, no GPU needed.  For C (M x N) += A (M x K) B (K x N) with tile size T on a
 * device of n_cus compute units (at most 256), operands assumed 16-byte aligned with rows of M, N, K
 * elements: whether the schedule applies (whatever_the_estimate != 0: wherever it can run, else only where
 * its cost estimate promises a gain), the interior it covers with 256 x 256 macro tiles, how many of
 * them run as whole rounds, and the k segments of the others in launch order.
 *   segment.tile         macro tile, numbered task by task over the interior (tiles below
 *                        whole_round_tiles belong to the whole rounds)
 *   segment.first_chunk  first 32-k chunk of the segment, n_chunks of them
 *   segment.slot         where its partial sum goes; the slots of one tile are consecutive and ascend with k
 * Copies min(cap, n_segments) segments; segments may be NULL when cap is 0.  dtype as in tgemm_run. */
typedef struct tgemm_segment {
    int32_t tile, first_chunk, n_chunks, slot;
} tgemm_segment;
typedef struct tgemm_balance {
    int32_t applies;            /* 0: tgemm_run takes one launch for this product; the other fields are 0 */
    int32_t whole_round_tiles;  /* macro tiles of the whole rounds (a multiple of n_cus)              */
    int32_t tail_tiles;         /* macro tiles of the partial round, cut into segments                */
    int32_t n_segments;
    int32_t chunks_per_tile;    /* K / 32                                                             */
    int32_t even_parts;         /* > 0: every tile of the partial round is cut into this many pieces at the
                                   same depths (bf16); 0: equal ranges of the (tile, chunk) pairs laid end
                                   to end, longest segment first                                      */
    int64_t interior_rows, interior_cols; /* multiples of 256; the rest of C is computed by a launch of its own */
} tgemm_balance;
int tgemm_balance_plan(int64_t M, int64_t N, int64_t K, int32_t T, int32_t dtype, int32_t n_cus,
                       int32_t whatever_the_estimate, tgemm_balance* out, tgemm_segment* segments, int64_t cap);

/* ---- MLP passes (section 2: forward pass = equation 1, backward pass = equations 3 and 4) ----
 *
 * Network: n_layers weight matrices W_l of shape dims[l] x dims[l+1], no bias; sigmoid after every
 * layer but the last; softmax + mean cross-entropy on the last.
 *   W        n_layers caller-owned matrices (dtype elements), all of one kind.
 *            Device pointers: in-core, every product is one launch.
 *            Pinned host pointers: out-of-core.  T x T weight tiles are staged through an HBM tile
 *            cache (section 3.4; the tile evicted is the one whose next use in the fixed sweep of a
 *            training step lies furthest ahead); the forward pass fetches each tile once, the
 *            backward pass uses a tile for D W^T, updates it and writes it back.  Tiles stay cached
 *            from one call to the next: while the object exists only the library may write to
 *            out-of-core weights.  On return of every call the
 *            host weights are complete and no modified tile remains only on the device (with
 *            opts.deferred_writeback an mlp_step leaves its last write-backs in flight; they are
 *            ordered before any later use of the tile and complete by tgemm_sync).
 *   dtype    TGEMM_F32, or TGEMM_BF16: weights, X, activations and errors are bf16, logits,
 *            probabilities, dW outputs and all accumulation float; the updated weights are
 *            bf16_round_to_nearest_even(float(W) - lr * dW).
 *   T        tile size of every product.
 *   hbm_budget  upper bound on device bytes the object may allocate: activations, errors, logits and
 *            (out-of-core) the weight-tile cache, which takes what the workspaces leave.  0 = no
 *            bound (in-core only; out-of-core needs a budget).  TGEMM_EBUDGET is reported by the
 *            first forward / step whose batch makes the workspaces plus the minimum cache
 *            (2 * max_l ceil(dims[l] / T) + 2 tiles) exceed it.
 * The object allocates its workspaces on the first forward for a batch size and reuses them while
 * the batch size does not grow. */
int mlp_create(tgemm_ctx* ctx, tgemm_mlp** out, int32_t n_layers, const int64_t* dims,
               void* const* W, int32_t dtype, int32_t T, size_t hbm_budget);
int mlp_destroy(tgemm_mlp* mlp);

/* Hidden-layer activation (section 2 leaves the function open: the passes stay matrix products
 * whatever it is).  A_l = act(Z_l) in the forward product's epilogue; the backward pass multiplies
 * by the slope written in terms of the stored activation a = act(z):
 *   TGEMM_ACT_SIGMOID  1 / (1 + exp(-z)),  slope a (1 - a)     (default)
 *   TGEMM_ACT_TANH     tanh(z),            slope 1 - a^2
 *   TGEMM_ACT_RELU     max(0, z),          slope 1 where a > 0, else 0
 * Takes effect from the next mlp_forward / mlp_step; a pending forward pass is discarded
 * (mlp_backward then reports TGEMM_ESTATE).  TGEMM_EARG for an unknown code. */
enum { TGEMM_ACT_SIGMOID = 0, TGEMM_ACT_TANH = 1, TGEMM_ACT_RELU = 2 };
int mlp_set_activation(tgemm_mlp* mlp, int32_t act);

/* Bias terms (section 2 writes each layer as a matrix product; a bias row is the usual extension,
 * equivalent to a constant-one input column): Z_l = A_{l-1} W_l + 1 b_l^T, added in the forward
 * product's epilogue before the activation / before the logits are stored.  The backward pass gets
 * db_l = 1^T D_l (column sums of the error matrix over the batch, summed in a fixed order: bands of
 * 512 rows, then the bands in ascending order); mlp_step applies b_l <- b_l - lr db_l.
 *   b   array of n_layers device pointers, b[l-1] -> dims[l] floats (fp32 also for bf16 networks),
 *       caller-owned like the weights and updated in place by mlp_step; always device memory, also
 *       when the weights are out-of-core.  NULL removes the bias terms (the default).
 *   db  NULL, or array of n_layers device pointers (entries may be NULL): mlp_backward and mlp_step
 *       store db_l there.
 * Waits for outstanding work, discards a pending forward pass and, when bias terms come or go,
 * releases the workspaces (the next pass sizes them again; the column-sum scratch of
 * ceil(batch / 512) x max_l dims[l] floats counts against hbm_budget).
 * TGEMM_EARG for a NULL entry of b, a pointer that is not device memory, or db without b. */
int mlp_set_bias(tgemm_mlp* mlp, void* const* b, void* const* db);

/* Momentum for mlp_step (section 2 only says that the parameters are updated after the two passes;
 * this is the classical heavy-ball rule):  V_l <- mu V_l + dW_l;  W_l <- W_l - lr V_l, both inside
 * the dW product's epilogue (the gradient is never stored).  With mu = 0 the weights move exactly as
 * without momentum (and V_l receives dW_l).
 *   mu  in [0, 1).
 *   V   array of n_layers pointers, V[l-1] -> dims[l-1] x dims[l] floats, row-major (fp32 also
 *       for bf16 networks), caller-owned and caller-initialised (zeros for a fresh run); NULL
 *       switches momentum off (the default).  The velocities live where the weights live: device
 *       memory for device-resident weights, pinned host memory for out-of-core weights.  Out-of-core,
 *       the T rows of V_l that one launch of the dW product updates are fetched into one of two
 *       device buffers (T x max_l dims[l] floats each, counted against hbm_budget), updated there and
 *       written back, 8 bytes per weight and step over the host link; like the weights they are
 *       complete in host memory when the call returns (with opts.deferred_writeback: after
 *       tgemm_sync), and while momentum is set only the library may write to them.
 *   Vb  NULL, or array of n_layers device pointers to dims[l] floats: velocities of the bias rows
 *       (used when bias rows are set; without Vb the bias rows take plain SGD steps).
 * TGEMM_EARG for mu outside [0, 1), for a V[l] of the wrong kind of memory, for a Vb[l] that is not
 * device memory, or for Vb without V.  Waits for outstanding work; on an out-of-core network a change
 * between with and without momentum releases the workspaces (the next pass sizes them again). */
int mlp_set_momentum(tgemm_mlp* mlp, float mu, void* const* V, void* const* Vb);

/* Rounding of the updated weights in mlp_step for bf16 networks (section 2's update, W_l - lr dW_l,
 * is formed in fp32 in the product's epilogue and then stored as bf16).
 *   TGEMM_ROUND_NEAREST     round to nearest even (default).  An update below half an ulp of the
 *                           weight (2^-9 relative) is lost entirely.
 *   TGEMM_ROUND_STOCHASTIC  add 16 uniform random bits below the bf16 cut and truncate: the stored
 *                           value is one of the two bf16 neighbours of the fp32 result, the upper one
 *                           (in magnitude) with probability equal to the dropped fraction, so its
 *                           expectation is the fp32 result; exactly representable results never move.
 * The random bits are a pure function of (seed, layer l = 1..n_layers, step, row, col) with
 * mix32 = the 32-bit finalizer of MurmurHash3 (x ^= x >> 16; x *= 0x85ebca6b; x ^= x >> 13;
 * x *= 0xc2b2ae35; x ^= x >> 16) and arithmetic modulo 2^32:
 *   key  = mix32(mix32(mix32(mix32(seed mod 2^32) ^ (seed >> 32)) ^ l) ^ step)
 *   bits = mix32(mix32(row + key) + (col / 2) * 0x9E3779B9);  even col takes bits mod 2^16, odd col bits >> 16
 * (row, col index W_l; step counts the mlp_step calls since this function was last called), so a
 * run is reproducible whatever the tile size, kernel or residency mode.
 * TGEMM_EARG for an unknown mode, or for the stochastic mode on an fp32 network. */
enum { TGEMM_ROUND_NEAREST = 0, TGEMM_ROUND_STOCHASTIC = 1 };
int mlp_set_rounding(tgemm_mlp* mlp, int32_t mode, uint64_t seed);

/* fp32 master copies of bf16 weights for mlp_step (section 2's update leaves the storage precision
 * open; bf16 storage alone loses every step below half an ulp of the weight, see mlp_set_rounding).
 * With master copies the two passes still read the bf16 W_l, while the step is applied in fp32 to
 * the copy inside the dW product's epilogue:
 *   M_l <- M_l - lr dW_l   (with momentum: M_l <- M_l - lr V_l);   W_l <- bf16(M_l)
 * where bf16() rounds as mlp_set_rounding says (to nearest even by default).
 *   Wm  array of n_layers pointers, Wm[l-1] -> dims[l-1] x dims[l] floats, row-major,
 *       caller-owned and caller-initialised (normally float(W_l)); the library never reads W_l to
 *       form the step, so a copy that disagrees with W_l wins at the first step.  NULL removes the
 *       master copies (the default).  Device memory for device-resident weights, pinned host memory
 *       for out-of-core weights (then streamed through two device row buffers like the velocities
 *       of mlp_set_momentum, with the same cost and the same rules).
 * bf16 networks only: TGEMM_EARG for an fp32 network or a pointer of the wrong kind of memory.
 * Waits for outstanding work; on an out-of-core network a change between with and without master
 * copies releases the workspaces. */
int mlp_set_master_weights(tgemm_mlp* mlp, void* const* Wm);

/* Equation 1 for every layer: Z_l = A_{l-1} W_l, A_l = sigmoid(Z_l); last layer: logits.
 *   X      device pointer, batch x dims[0], dtype elements.
 *   probs  NULL, or device pointer to batch x dims[n_layers] floats receiving softmax(logits). */
int mlp_forward(tgemm_mlp* mlp, const void* X, int64_t batch, float* probs);

/* mlp_forward for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and same results as
 * mlp_forward, but the hidden activations and the logits live in a static device array of
 * TGEMM_STATIC_SCRATCH_BYTES that every GPU running the library holds from load time to process end
 * (its address on the context's device is looked up once, in tgemm_create).  The call allocates and
 * frees nothing, on the device or through any library.
 *   mlp    a network with device-resident weights (TGEMM_EARG for out-of-core weights).  Its own
 *          workspaces and pass state are left alone: a pending mlp_forward stays pending, and
 *          mlp_backward / mlp_read never see this call's activations.
 *   X      device pointer, batch x dims[0], dtype elements.
 *   probs  device pointer to batch x dims[n_layers] floats (16-byte aligned) receiving
 *          softmax(logits); required.
 * The activations (batch x dims[l] elements for l = 1..n_layers-1, each rounded up to 256 bytes)
 * plus batch x dims[n_layers] floats of logits must fit the array: TGEMM_EBUDGET otherwise, before
 * any work.  Nothing in the array has to start at zero (every product overwrites its destination),
 * so it keeps the previous call's contents.  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (from several contexts or threads) race. */
#define TGEMM_STATIC_SCRATCH_BYTES (32u << 20)
int mlp_forward_static(tgemm_mlp* mlp, const void* X, int64_t batch, float* probs);

/* Equations 3 and 4 for every layer, from the activations of the preceding mlp_forward:
 *   D_L = (softmax(Z_L) - onehot(labels)) / batch;  dW_l = A_{l-1}^T D_l;
 *   D_{l-1} = (D_l W_l^T) * A_{l-1} * (1 - A_{l-1}).
 *   labels  device pointer, batch int32 values in [0, dims[n_layers]).
 *   dW      NULL, or n_layers device pointers (dims[l] x dims[l+1] floats, also for TGEMM_BF16)
 *           receiving dW_l; single entries may be NULL.
 *   loss    host pointer receiving the mean cross-entropy (may be NULL).
 * The weights are not changed.  TGEMM_ESTATE if no forward preceded. */
int mlp_backward(tgemm_mlp* mlp, const int32_t* labels, void* const* dW, float* loss);

/* One training step: forward, backward and W_l <- W_l - lr * dW_l fused into the dW product's
 * epilogue (dW is never stored); every error D_{l-1} is formed from the pre-update W_l.
 *   loss  host pointer receiving the loss before the update (may be NULL). */
int mlp_step(tgemm_mlp* mlp, const void* X, const int32_t* labels, int64_t batch, float lr, float* loss);

/* Weight-tile lookups of the last mlp_forward / mlp_backward / mlp_step on an out-of-core network
 * (requires opts.trace).  Copies min(cap, n) records; out may be NULL when cap == 0. */
int mlp_trace(tgemm_mlp* mlp, tgemm_mlp_trace_rec* out, int64_t cap, int64_t* n);

/* Test access to the object's device workspaces after a forward / backward:
 *   what 0: activation A_l (l = 1..n_layers-1; batch x dims[l], dtype elements)
 *        1: logits Z_L (batch x dims[n_layers] floats; layer ignored)
 *        2: error D_l  (l = 1..n_layers; batch x dims[l], dtype elements)
 * Copies `bytes` bytes starting `offset` bytes into the matrix to the host buffer dst.  TGEMM_EARG
 * if offset + bytes exceeds the matrix. */
int mlp_read(tgemm_mlp* mlp, int32_t what, int32_t layer, void* dst, size_t offset, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* TGEMM_H */
