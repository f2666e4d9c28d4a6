// Balanced schedule of the in-core product C += A B (tgemm_opts.incore_schedule; see gemm_kernel.h):
// host-side plan (which macro tiles run as whole rounds, how the partial round is cut along k, in what
// order the pieces are launched), the launches, and the kernel that adds the pieces' sums to C.
// The tile kernels themselves (whole rounds by a grid limit, the segments' EPI_PARTIAL epilogue, the
// strips' instance of the small fp32 shape) are in gemm_f32.hip and gemm_bf16_dl.hip.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/tgemm.h"
#include "gemm_kernel.h"

namespace tg {

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct SkTile {
    int32_t row0, col0, first_slot, n_slots;   // a tile of the partial round and its slots of the workspace
};
constexpr int SK_MAX_SLOTS = 512;              // segments <= units + tiles of the partial round < 2 * 256
constexpr size_t SK_SLOT_FLOATS = 256 * 256;
constexpr size_t SK_TABLE_BYTES = 16384;       // segment table, then tile table (8 KiB each)

struct SkWorkspace {
    int64_t M = 0, N = 0, K = 0, ldc = 0;      // the product the tables were made for
    int32_t T = 0, n_cus = 0;
    bool forced = false, bf16 = false;
    bool use = false;
    int even_parts = 0;                         // see tgemm_balance
    int64_t Mi = 0, Ni = 0;
    int grid_full = 0;                          // macro tiles of the whole rounds
    std::vector<SkSegment> segments;            // in launch order
    std::vector<SkTile> tiles;
    bool uploaded = false;
    char* dev = nullptr;                        // SK_TABLE_BYTES of tables, then SK_MAX_SLOTS slots
};

void sk_destroy(SkWorkspace* ws)
{
    if (!ws) return;
    if (ws->dev) (void)hipFree(ws->dev);
    delete ws;
}

// Adds a tile's segment sums (ascending k) and then C: 16 workgroups per tile, 16 rows each.
__global__ __launch_bounds__(256) void sk_fixup(float* __restrict__ C, int64_t ldc, const float* __restrict__ partial,
                                                 const SkTile* __restrict__ tiles)
{
    const SkTile t = tiles[blockIdx.x >> 4];
    const int rg = blockIdx.x & 15;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int u = threadIdx.x + 256 * i;            // 16-byte unit of the row group: 16 rows x 64 units
        const int r = rg * 16 + (u >> 6), c4 = (u & 63) << 2;
        const float* src = partial + (size_t)t.first_slot * SK_SLOT_FLOATS + r * 256 + c4;
        f32x4 sum = gload<f32x4>(src);
        for (int s = 1; s < t.n_slots; ++s) {
            const f32x4 q = gload<f32x4>(src + (size_t)s * SK_SLOT_FLOATS);
#pragma unroll
            for (int e = 0; e < 4; ++e) sum[e] += q[e];
        }
        float* dst = C + (int64_t)(t.row0 + r) * ldc + t.col0 + c4;
        const f32x4 c = gload<f32x4>(dst);
#pragma unroll
        for (int e = 0; e < 4; ++e) sum[e] += c[e];
        gstore<f32x4>(dst, sum);
    }
}

// The plan for one product: whether the balanced schedule applies and is expected to win, and its tables.
static void sk_make_plan(SkWorkspace& w, const GemmDesc& d, bool bf16, int n_cus, bool forced)
{
    w.M = d.M; w.N = d.N; w.K = d.K; w.T = d.T; w.ldc = d.ldc; w.n_cus = n_cus; w.forced = forced; w.bf16 = bf16;
    w.use = false; w.uploaded = false;
    w.segments.clear(); w.tiles.clear();
    constexpr int64_t B = 256, BK = 32;
    if (n_cus < 8 || n_cus > 256 || d.K % BK != 0 || d.K < 16 * BK || d.M < B || d.N < B) return;
    if (d.M > 0x7fffffff || d.N > 0x7fffffff || d.K > 0x7fffffff) return;
    const int64_t Mi = d.M / B * B, Ni = d.N / B * B;
    // the tile size as the launcher clamps it for the interior product; tasks must be whole macro tiles
    int64_t T = d.T;
    const int64_t big = (Mi > Ni ? Mi : Ni) > d.K ? (Mi > Ni ? Mi : Ni) : d.K;
    if (T > big) T = big;
    if (T % B != 0) return;
    const int64_t n_tiles = (Mi / B) * (Ni / B), n_ch = d.K / BK;
    const int64_t rounds = n_tiles / n_cus, n_tail = n_tiles % n_cus;
    if (n_tail == 0 || n_tiles > 0x7fffffff) return;
    int uniform_parts = 0;      // > 0: every tile of the partial round in this many even pieces (bf16)
    if (bf16) {
        // the direct-to-LDS kernel alone has the segment epilogue; strips are not offered
        if (Mi != d.M || Ni != d.N) return;
        GemmDesc in = d;
        in.T = (int32_t)T;
        if (!bf::bf16_dl_applicable(in)) return;
        // The bf16 loop takes a chunk in under a microsecond: segments at different depths of k, which
        // share no panel piece in the L2 at any moment, ask for more than HBM delivers and run at about
        // half pace.  So the tiles are cut evenly instead, each into units / tiles pieces (of at least 4
        // chunks) at the same depths, in one wave of workgroups that walk k together like a round of
        // whole tiles; with more than half as many tiles as units that is no cut at all, and the
        // ranges of the fp32 schedule are used, priced at half pace.
        uniform_parts = (int)(n_cus / n_tail);
        if (uniform_parts > n_ch / 4) uniform_parts = (int)(n_ch / 4);
        // Estimate in rounds of 256 x 256 tiles (0.0284 us per unit of K), as the bf16 launcher compares
        // its shapes: one launch takes whole rounds of the large shape, or of the 128 x 128 one (512 to a
        // round, 0.95 of a large round); balanced, the partial round costs its longest piece, plus 8
        // chunks of starts and 45 us of fix-up.
        const double round_us = 0.0284 * (double)d.K;
        const double c3 = (double)((n_tiles + n_cus - 1) / n_cus);
        const double c2 = 0.95 * (double)((4 * n_tiles + 2 * n_cus - 1) / (2 * n_cus));
        const double plain_rounds = c3 < c2 ? c3 : c2;
        const double tail_rounds = uniform_parts >= 2 ? (double)((n_ch + uniform_parts - 1) / uniform_parts) / (double)n_ch
                                                      : 2.0 * (double)n_tail / n_cus;
        const double bal_rounds = (double)rounds + tail_rounds + (0.0284 * BK * 8 + 45.0) / round_us;
        if (bal_rounds > 0.985 * plain_rounds && !forced) return;
        if (uniform_parts < 2) uniform_parts = 0;
    } else {
        // Estimate in microseconds, fitted to square products of 2048 .. 10240: whole rounds at 0.227 per
        // tile and unit of K; the partial round's share 7 % slower (its segments share no panel pieces in
        // L2) plus 10 for their starts; the fix-up 8 + 0.19 per tile; the strips by the cost model of
        // pick_config, or, with at most one 64 x 64 tile per unit between them, one chain of K / 2 MFMAs
        // per SIMD.  Against the one launch's best shape by the same cost model, which is rough for
        // small products: below 140 tiles they are left alone.
        double plain = 0.0, strips = 0.0, e = 0.0;
        pick_config_est(d, &plain);
        plain *= (double)d.K;
        GemmDesc s = d;
        if (d.N > Ni) { s.M = d.M; s.N = d.N - Ni; pick_config_est(s, &e); strips += e * (double)d.K; }
        if (d.M > Mi) { s.M = d.M - Mi; s.N = Ni; pick_config_est(s, &e); strips += e * (double)d.K; }
        const int64_t small = ((d.M + 63) / 64) * ((d.N - Ni + 63) / 64) + ((d.M - Mi + 63) / 64) * (Ni / 64);
        if (small <= n_cus) strips = small > 0 ? 0.0166 * (double)d.K + 12.0 : 0.0;
        const double balanced = 0.227 * (double)d.K * ((double)rounds + 1.07 * (double)n_tail / n_cus) + 10.0 +
                                (8.0 + 0.19 * (double)n_tail) + strips;
        if ((balanced > 0.975 * plain || n_tiles < 140) && !forced) return;
    }

    // macro tile number (task by task, as the kernel numbers them) -> origin, for the interior product
    const int64_t n_i = (Mi + T - 1) / T, n_j = (Ni + T - 1) / T;
    const int64_t tpm = (n_i > 1 ? T : Mi) / B, tpn = (n_j > 1 ? T : Ni) / B;
    const int64_t tpm_last = (Mi - (n_i - 1) * T) / B, tpn_last = (Ni - (n_j - 1) * T) / B;
    const int64_t macro_cols = (n_j - 1) * tpn + tpn_last, band = tpm * macro_cols;
    auto origin = [&](int64_t lid, int32_t* row0, int32_t* col0) {
        const int64_t ti = lid / band, in_band = lid - ti * band;
        const int64_t h = (ti == n_i - 1) ? tpm_last : tpm;
        int64_t tj = in_band / (h * tpn);
        if (tj > n_j - 1) tj = n_j - 1;
        const int64_t in_task = in_band - tj * h * tpn;
        const int64_t wcols = (tj == n_j - 1) ? tpn_last : tpn;
        const int64_t si = in_task / wcols, sj = in_task - si * wcols;
        *row0 = (int32_t)(ti * T + si * B);
        *col0 = (int32_t)(tj * T + sj * B);
    };
    // the (tile, chunk) pairs of the partial round laid end to end, cut into n_cus equal ranges, each
    // range cut again where it crosses into the next tile; slots are numbered in that order, so a
    // tile's slots are consecutive and ascend with k
    const int64_t U = n_tail * n_ch;
    w.tiles.resize((size_t)n_tail);
    for (int64_t t = 0; t < n_tail; ++t) {
        origin(rounds * n_cus + t, &w.tiles[t].row0, &w.tiles[t].col0);
        w.tiles[t].first_slot = -1;
        w.tiles[t].n_slots = 0;
    }
    if (uniform_parts > 0) {
        // slot = tile * parts + part; workgroups by part, then by tile (neighbours in the task order share
        // panels), numbered so that consecutive ones land on the same XCD like the whole rounds' workgroups
        const int64_t n = n_tail * uniform_parts;
        std::vector<SkSegment> list((size_t)n);
        for (int64_t j = 0; j < uniform_parts; ++j)
            for (int64_t t = 0; t < n_tail; ++t) {
                const int64_t b = j * n_ch / uniform_parts, e2 = (j + 1) * n_ch / uniform_parts;
                list[(size_t)(j * n_tail + t)] = SkSegment{(int32_t)(rounds * n_cus + t), (int32_t)b, (int32_t)(e2 - b),
                                                           (int32_t)(t * uniform_parts + j)};
            }
        for (int64_t t = 0; t < n_tail; ++t) {
            w.tiles[t].first_slot = (int32_t)(t * uniform_parts);
            w.tiles[t].n_slots = uniform_parts;
        }
        w.segments.resize((size_t)n);
        const int64_t q = n >> 3, r = n & 7;
        for (int64_t blk = 0; blk < n; ++blk) {
            const int64_t xcd = blk & 7, local = blk >> 3;
            w.segments[(size_t)blk] = list[(size_t)(xcd * q + (xcd < r ? xcd : r) + local)];
        }
    } else {
        std::vector<int> first_of_range((size_t)n_cus + 1);     // a range's pieces: segments first_of_range[g] .. [g + 1]
        for (int64_t g = 0; g < n_cus; ++g) {
            first_of_range[(size_t)g] = (int)w.segments.size();
            int64_t b = g * U / n_cus;
            const int64_t e2 = (g + 1) * U / n_cus;
            while (b < e2) {
                const int64_t t = b / n_ch, te = (t + 1) * n_ch;
                const int64_t n = (e2 < te ? e2 : te) - b;
                const int32_t slot = (int32_t)w.segments.size();
                w.segments.push_back(SkSegment{(int32_t)(rounds * n_cus + t), (int32_t)(b - t * n_ch), (int32_t)n, slot});
                if (w.tiles[t].first_slot < 0) w.tiles[t].first_slot = slot;
                w.tiles[t].n_slots += 1;
                b += n;
            }
        }
        first_of_range[(size_t)n_cus] = (int)w.segments.size();
        // Launch order.  The hardware deals workgroup b to XCD b % 8, and inside an XCD the next workgroup goes to
        // the first unit that falls free.  Every range is a unit's fair share, in one piece or two (t < units, so a
        // range crosses at most one tile boundary).  Each XCD gets as many ranges as it has units, the two-piece
        // ones dealt round, which is exactly the number of workgroups the hardware will hand it; its list is its
        // ranges' longer pieces, longest first, then the shorter ones, longest first: the unit with the shortest
        // long piece falls free first and takes the longest short piece, its own range's other half or one as long.
        const int64_t n = (int64_t)w.segments.size();
        if (n_cus % 8 == 0 && n <= SK_MAX_SLOTS) {
            std::vector<SkSegment> head[8], tail[8];
            int64_t cut = 0, whole = 0;
            for (int64_t g = 0; g < n_cus; ++g)
                if (first_of_range[(size_t)g + 1] - first_of_range[(size_t)g] == 2) {
                    const SkSegment& a = w.segments[(size_t)first_of_range[(size_t)g]];
                    const SkSegment& b = w.segments[(size_t)first_of_range[(size_t)g] + 1];
                    const int x = (int)(cut++ % 8);
                    head[x].push_back(a.n_chunks >= b.n_chunks ? a : b);
                    tail[x].push_back(a.n_chunks >= b.n_chunks ? b : a);
                }
            for (int64_t g = 0; g < n_cus; ++g)
                if (first_of_range[(size_t)g + 1] - first_of_range[(size_t)g] == 1) {
                    int x = (int)(whole++ % 8);
                    while ((int64_t)head[x].size() >= n_cus / 8) x = (x + 1) % 8;     // the XCD's ranges are complete
                    head[x].push_back(w.segments[(size_t)first_of_range[(size_t)g]]);
                }
            auto longer = [](const SkSegment& a, const SkSegment& b) { return a.n_chunks > b.n_chunks; };
            std::vector<SkSegment> order((size_t)n);
            bool ok = true;
            for (int x = 0; x < 8 && ok; ++x) {
                std::stable_sort(head[x].begin(), head[x].end(), longer);
                std::stable_sort(tail[x].begin(), tail[x].end(), longer);
                head[x].insert(head[x].end(), tail[x].begin(), tail[x].end());
                ok = (int64_t)head[x].size() == n / 8 + (x < n % 8 ? 1 : 0);
                for (size_t i = 0; ok && i < head[x].size(); ++i) order[8 * i + (size_t)x] = head[x][i];
            }
            if (ok) w.segments.swap(order);
            else std::stable_sort(w.segments.begin(), w.segments.end(), longer);
        } else {
            std::stable_sort(w.segments.begin(), w.segments.end(),
                             [](const SkSegment& a, const SkSegment& b2) { return a.n_chunks > b2.n_chunks; });
        }
    }
    if (w.segments.size() > (size_t)SK_MAX_SLOTS || w.segments.size() * sizeof(SkSegment) > SK_TABLE_BYTES / 2 ||
        w.tiles.size() * sizeof(SkTile) > SK_TABLE_BYTES / 2) {
        w.segments.clear(); w.tiles.clear();
        return;
    }
    w.Mi = Mi; w.Ni = Ni;
    w.grid_full = (int)(rounds * n_cus);
    w.even_parts = uniform_parts;
    w.use = true;
}

// The plan alone, for tgemm_balance_plan: operands taken as aligned, dense, with rows of M, N, K elements.
int sk_inspect(int64_t M, int64_t N, int64_t K, int32_t T, bool bf16, int n_cus, bool forced, tgemm_balance* out,
               tgemm_segment* segments, int64_t cap)
{
    static_assert(sizeof(tgemm_segment) == sizeof(SkSegment), "the table is handed out as it is");
    memset(out, 0, sizeof *out);
    if (M <= 0 || N <= 0 || K <= 0 || T <= 0) return 0;
    GemmDesc d;
    memset(&d, 0, sizeof d);
    alignas(16) static const char aligned_dummy[16] = {0};
    d.A = aligned_dummy; d.B = aligned_dummy; d.C = nullptr;      // only their alignment is looked at
    d.lda = K; d.ldb = N; d.ldc = N;
    d.M = M; d.N = N; d.K = K; d.T = T;
    d.a_kcontig = 1; d.b_kcontig = 0;
    d.epilogue = EPI_AXPBY; d.alpha = 1.f; d.beta = 1.f;
    const int row_unit = bf16 ? 8 : 4;
    auto off32 = [](int64_t ld) { return 256 * ld * 4 + 4096 < ((int64_t)1 << 31); };
    if (d.lda % row_unit || d.ldb % row_unit || d.ldc % 4 || !off32(d.lda) || !off32(d.ldb)) return 0;
    SkWorkspace w;
    sk_make_plan(w, d, bf16, n_cus, forced);
    if (!w.use) return 0;
    out->applies = 1;
    out->whole_round_tiles = w.grid_full;
    out->tail_tiles = (int32_t)w.tiles.size();
    out->n_segments = (int32_t)w.segments.size();
    out->chunks_per_tile = (int32_t)(K / 32);
    out->even_parts = w.even_parts;
    out->interior_rows = w.Mi;
    out->interior_cols = w.Ni;
    const int64_t n = cap < (int64_t)w.segments.size() ? cap : (int64_t)w.segments.size();
    if (n > 0) memcpy(segments, w.segments.data(), (size_t)n * sizeof(SkSegment));
    return 0;
}

hipError_t launch_gemm_balanced(const GemmDesc& d, bool bf16, SkWorkspace** wsp, int n_cus, bool forced, hipStream_t stream,
                                hipStream_t side, hipEvent_t fork, hipEvent_t join, int* launches)
{
    if (launches) *launches = 0;
    if (!wsp || d.config != 0 || d.epilogue != EPI_AXPBY || d.alpha != 1.f || d.beta != 1.f || !d.a_kcontig || d.b_kcontig ||
        d.bias || d.b_tiles || d.c_tiles || d.M <= 0 || d.N <= 0 || d.K <= 0 || d.T <= 0)
        return hipErrorNotSupported;
    // what the unpredicated, vector paths of the kernels ask of the operands
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    auto off32 = [](int64_t ld) { return 256 * ld * 4 + 4096 < ((int64_t)1 << 31); };
    const int row_unit = bf16 ? 8 : 4;       // elements of A and B in 16 bytes
    if (!al16(d.A) || !al16(d.B) || !al16(d.C) || d.lda % row_unit || d.ldb % row_unit || d.ldc % 4 || !off32(d.lda) || !off32(d.ldb))
        return hipErrorNotSupported;
    SkWorkspace* w = *wsp;
    if (!w) {
        w = new (std::nothrow) SkWorkspace();
        if (!w) return hipErrorNotSupported;
        *wsp = w;
    }
    if (w->M != d.M || w->N != d.N || w->K != d.K || w->T != d.T || w->ldc != d.ldc || w->n_cus != n_cus || w->forced != forced ||
        w->bf16 != bf16) {
        // an earlier call's table copies may still be reading the vectors that the new plan rewrites
        if (w->uploaded && hipStreamSynchronize(stream) != hipSuccess) return hipErrorNotSupported;
        try {
            sk_make_plan(*w, d, bf16, n_cus, forced);
        } catch (...) {
            w->use = false;
            w->M = 0;
        }
    }
    if (!w->use) return hipErrorNotSupported;
    if (!w->dev) {
        if (hipMalloc((void**)&w->dev, SK_TABLE_BYTES + SK_MAX_SLOTS * SK_SLOT_FLOATS * sizeof(float)) != hipSuccess) {
            (void)hipGetLastError();
            w->dev = nullptr;
            return hipErrorNotSupported;
        }
    }
    hipError_t e;
    if (!w->uploaded) {     // the vectors live as long as the plan: the copies may read them any time
        e = hipMemcpyAsync(w->dev, w->segments.data(), w->segments.size() * sizeof(SkSegment), hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return e;
        e = hipMemcpyAsync(w->dev + SK_TABLE_BYTES / 2, w->tiles.data(), w->tiles.size() * sizeof(SkTile), hipMemcpyHostToDevice, stream);
        if (e != hipSuccess) return e;
        w->uploaded = true;
    }
    int n = 0;
    GemmDesc in = d;
    in.M = w->Mi; in.N = w->Ni; in.config = 3;
    if (w->grid_full > 0) {
        in.sk_grid_limit = w->grid_full;
        if ((e = launch_tile_gemm(in, bf16, stream)) != hipSuccess) return e;
        ++n;
    }
    in.sk_grid_limit = 0;
    in.epilogue = EPI_PARTIAL;
    in.sk_segments = reinterpret_cast<const SkSegment*>(w->dev);
    in.sk_n_segments = (int32_t)w->segments.size();
    in.sk_partial = reinterpret_cast<float*>(w->dev + SK_TABLE_BYTES);
    if ((e = launch_tile_gemm(in, bf16, stream)) != hipSuccess) return e;
    ++n;
    // The strips start when the segments are done, next to the fix-up, as one launch.  (Started with the
    // whole rounds they took compute units from them -- a large workgroup and a small one do not fit a
    // unit together; as two launches side by side their workgroups landed two to a unit, on half of
    // the units, and took twice their time.)
    const bool right = d.N > w->Ni, bottom = d.M > w->Mi;      // (fp32 only)
    if (right || bottom) {
        e = hipEventRecord(fork, stream);
        if (e != hipSuccess) return e;
    }
    if (right || bottom) {  // both strips in one launch (see GemmDesc::l_shape)
        GemmDesc s = d;
        s.l_shape = 1; s.l_row0 = w->Mi; s.l_col0 = w->Ni;
        if ((e = hipStreamWaitEvent(side, fork, 0)) != hipSuccess) return e;
        if ((e = launch_tile_gemm_f32(s, side)) != hipSuccess) return e;
        if ((e = hipEventRecord(join, side)) != hipSuccess) return e;
        ++n;
    }
    hipLaunchKernelGGL(sk_fixup, dim3((unsigned)w->tiles.size() * 16), dim3(256), 0, stream, d.C, d.ldc,
                       reinterpret_cast<const float*>(w->dev + SK_TABLE_BYTES),
                       reinterpret_cast<const SkTile*>(w->dev + SK_TABLE_BYTES / 2));
    if ((e = hipGetLastError()) != hipSuccess) return e;
    ++n;
    if ((right || bottom) && (e = hipStreamWaitEvent(stream, join, 0)) != hipSuccess) return e;
    if (launches) *launches = n;
    return hipSuccess;
}

}  // namespace tg
