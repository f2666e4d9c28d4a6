// bf16 -> fp32 tile GEMM kernel for gfx950 (CDNA4): the tile product of Algorithm 1 of the paper
// for bf16 operands with fp32 accumulation (v_mfma_f32_32x32x16_bf16).
//
// Same structure as the fp32 kernel: one launch covers a whole tiled product, a workgroup owns one
// macro tile of one task's output tile and walks the k-steps in ascending order; workgroups are
// numbered task by task and XCD by XCD.
//
// The MFMA wants, per lane, 8 consecutive-k elements of one row of A and of one column of B, so
// both operands sit in LDS k-contiguous: As[m][k], Bs[n][k], 64 k per stage, rows padded to 144 B
// (conflict-free 16-byte reads).  A k-contiguous source (row-major A; W in the D W^T product) is
// copied with 16-byte loads and 16-byte LDS writes.  An m/n-contiguous source (row-major B; A^T
// and D in the A^T D product) is transposed in registers on the way: a thread loads 8 k-rows x 4
// columns (eight 8-byte loads), regroups the 16-bit halves into four 8-k vectors and writes four
// 16-byte LDS rows.  Which k lands in which MFMA slot is irrelevant as long as A and B agree.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "gemm_bf16_common.h"

namespace tg {
namespace bf {

constexpr int BK = 64;            // k per LDS stage
constexpr int ROW_W = 36;         // LDS row stride in 32-bit words: 128 B of data + 16 B pad

// ---- k-contiguous source: rows are mn, 64 contiguous k per stage -------------------------------
// unit u -> (mn = u / 8, kq = u % 8): 16 bytes = 8 k.
template <int BMN, int NT>
struct LoaderKC {
    static constexpr int UP = BMN * 8 / NT;
    static constexpr int N_LOADS = UP;        // global load instructions per chunk (fast path)
    static_assert((BMN * 8) % NT == 0, "tile must divide evenly over the threads");
    u32x4 reg[UP];
    uint32_t off[UP];     // byte offset of unit p from the chunk origin (interior fast path)

    // `valid` (>= 4) of the BMN rows exist on an edge tile: rows beyond them are clamped onto the
    // last valid one, so every address stays inside the matrix; what they load only reaches rows /
    // columns of the product that the epilogue never stores.
    __device__ inline void init(int64_t ld, int valid, int tid)
    {
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            off[p] = (uint32_t)(((int64_t)min(u >> 3, valid - 1) * ld + ((u & 7) << 3)) * 2);
        }
    }
    // full chunk: no predicates, origin = element (mn0, kk)
    __device__ inline void load_fast(const uint16_t* __restrict__ origin)
    {
        const char* base = reinterpret_cast<const char*>(origin);
#pragma unroll
        for (int p = 0; p < UP; ++p) reg[p] = gload<u32x4>(base + off[p]);
    }

    __device__ inline void load(const uint16_t* __restrict__ X, int64_t ld, int mn0, int mn_end, int kk,
                                int klim, bool vec_ok, int tid)
    {
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            const int mn = mn0 + (u >> 3);
            const int k = kk + ((u & 7) << 3);
            u32x4 v = {0u, 0u, 0u, 0u};
            if (mn < mn_end && k < klim) {
                const uint16_t* src = X + (int64_t)mn * ld + k;
                if (vec_ok && k + 7 < klim) {
                    v = gload<u32x4>(src);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        if (k + e < klim) v[e >> 1] |= (uint32_t)gload<uint16_t>(src + e) << ((e & 1) * 16);
                }
            }
            reg[p] = v;
        }
    }
    __device__ inline void store(uint32_t* __restrict__ S, int tid) const
    {
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            *reinterpret_cast<u32x4*>(&S[(u >> 3) * ROW_W + ((u & 7) << 2)]) = reg[p];
        }
    }
};

// ---- mn-contiguous source: rows are k, BMN contiguous mn ---------------------------------------
// A unit is 8 k-rows (8 kg .. 8 kg + 7) x 4 mn (4 q .. 4 q + 3); a thread owns UP units that differ
// in kg.  Thread bits 0-1 and 4.. select q, bits 2-3 (then the bits above q, then the unit index)
// select kg: any 16 consecutive lanes hold 4 values of q and 4 of kg, which makes the four 16-byte
// LDS row stores below bank-conflict free (row stride 9 bank quads), while the lanes of a wave
// still cover 128 contiguous bytes of each k-row.
template <int BMN, int NT>
struct LoaderMC {
    static constexpr int Q = BMN / 4;
    static constexpr int QH = Q / 4;          // values of the high part of q
    static constexpr int UP = Q * 8 / NT;     // units per thread
    static constexpr int KG_T = 8 / UP;       // kg values covered by the thread index
    static constexpr int N_LOADS = UP * 8;    // global load instructions per chunk (fast path)
    static_assert(Q * 8 % NT == 0 && UP >= 1 && KG_T >= 4 && NT == 16 * QH * (KG_T / 4), "thread/unit mapping");
    u32x2 reg[UP][8];
    uint32_t off0;        // byte offset of unit 0's first row from the chunk origin
    int q, kg0;

    // `valid` (>= 4, a multiple of 4) of the BMN columns exist on an edge tile: units beyond them
    // are clamped onto the last valid four.
    __device__ inline void init(int64_t ld, int valid, int tid)
    {
        q = (tid & 3) | (((tid >> 4) & (QH - 1)) << 2);
        kg0 = ((tid >> 2) & 3) | ((tid / (16 * QH)) << 2);
        off0 = (uint32_t)(((int64_t)(kg0 << 3) * ld + min(q << 2, valid - 4)) * 2);
    }
    // full chunk: origin = element (k = kk, mn = mn0)
    __device__ inline void load_fast(const uint16_t* __restrict__ origin, int64_t ld)
    {
        const char* base = reinterpret_cast<const char*>(origin);
#pragma unroll
        for (int p = 0; p < UP; ++p)
#pragma unroll
            for (int r = 0; r < 8; ++r)
                reg[p][r] = gload<u32x2>(base + (size_t)(p * KG_T * 8 + r) * (size_t)ld * 2 + off0);
    }

    __device__ inline void load(const uint16_t* __restrict__ X, int64_t ld, int mn0, int mn_end, int kk,
                                int klim, bool vec_ok, int tid)
    {
        const int mn = mn0 + (q << 2);
        const bool full = vec_ok && (mn + 3 < mn_end);
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int kb = kk + ((kg0 + p * KG_T) << 3);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                u32x2 v = {0u, 0u};
                const int k = kb + r;
                if (k < klim && mn < mn_end) {
                    const uint16_t* src = X + (int64_t)k * ld + mn;
                    if (full) {
                        v = gload<u32x2>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (mn + e < mn_end) v[e >> 1] |= (uint32_t)gload<uint16_t>(src + e) << ((e & 1) * 16);
                    }
                }
                reg[p][r] = v;
            }
        }
    }
    // 8 x 4 block of 16-bit elements -> four rows of 8 k
    __device__ inline void store(uint32_t* __restrict__ S, int tid) const
    {
        const int mn = q << 2;
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int kg = kg0 + p * KG_T;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                u32x4 o;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t x = reg[p][2 * w][e >> 1], y = reg[p][2 * w + 1][e >> 1];
                    o[w] = (e & 1) ? ((x >> 16) | (y & 0xffff0000u)) : ((x & 0xffffu) | (y << 16));
                }
                *reinterpret_cast<u32x4*>(&S[(mn + e) * ROW_W + (kg << 2)]) = o;
            }
        }
    }
};

template <int BMN, int NT>
__device__ inline void fast_load(LoaderKC<BMN, NT>& l, const uint16_t* X, int64_t ld, int mn0, int kk)
{
    l.load_fast(X + (int64_t)mn0 * ld + kk);
}
template <int BMN, int NT>
__device__ inline void fast_load(LoaderMC<BMN, NT>& l, const uint16_t* X, int64_t ld, int mn0, int kk)
{
    l.load_fast(X + (int64_t)kk * ld + mn0, ld);
}

template <int BMN, int NT, bool KC> struct PickLoader { typedef LoaderKC<BMN, NT> type; };
template <int BMN, int NT> struct PickLoader<BMN, NT, false> { typedef LoaderMC<BMN, NT> type; };

// ---- the kernel ---------------------------------------------------------------------------------
// DEPTH = chunks in flight in registers in the interior (fast) k loop.
template <int RA, int RB, int WM, int WN, int DEPTH, bool A_KC, bool B_KC, int EPI, bool OUT_BF16>
__global__ __launch_bounds__(WM * WN * 64) void tile_gemm_bf16(const GemmParams p)
{
    constexpr int WTM = 32 * RA, WTN = 32 * RB;
    constexpr int BM = WM * WTM, BN = WN * WTN;
    constexpr int NT = WM * WN * 64;
    constexpr int STAGE_A = BM * ROW_W, STAGE_B = BN * ROW_W;   // words
    typedef typename PickLoader<BM, NT, A_KC>::type LA;
    typedef typename PickLoader<BN, NT, B_KC>::type LB;

    extern __shared__ __attribute__((aligned(16))) uint32_t smem_w[];
    uint32_t* As = smem_w;                    // [2][BM][ROW_W]
    uint32_t* Bs = smem_w + 2 * STAGE_A;      // [2][BN][ROW_W]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lh = lane >> 5;

    const TileCoord tc = decode_tile<BM, BN>(p);
    const int ti = tc.ti, tj = tc.tj, row0 = tc.row0, col0 = tc.col0, row_end = tc.row_end, col_end = tc.col_end;
    (void)ti;

    const uint16_t* __restrict__ A = reinterpret_cast<const uint16_t*>(p.A);
    const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(p.B);

    f32x16 acc[RA][RB];
#pragma unroll
    for (int r = 0; r < RA; ++r)
#pragma unroll
        for (int c = 0; c < RB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    LA la[DEPTH];
    LB lb[DEPTH];
    const int a_valid = min(BM, row_end - row0), b_valid = min(BN, col_end - col0);
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
        la[d].init(p.lda, max(a_valid, 4), tid);
        lb[d].init(p.ldb, max(b_valid, 4), tid);
    }
    const int n_chunks = p.n_chunks;
    const int cps = p.chunks_per_step;

    // lane's LDS read base: row (wave tile row / col + li), k offset 8 * lh elements = 4 * lh words
    const int a_off = (wm * WTM + li) * ROW_W + lh * 4;
    const int b_off = (wn * WTN + li) * ROW_W + lh * 4;

    // one 64-k chunk from LDS stage st
    auto compute = [&](int st) {
        const uint32_t* as = As + st * STAGE_A + a_off;
        const uint32_t* bs = Bs + st * STAGE_B + b_off;
#pragma unroll
        for (int s = 0; s < BK / 16; ++s) {
            bf16x8 af[RA], bfr[RB];
#pragma unroll
            for (int r = 0; r < RA; ++r)
                af[r] = *reinterpret_cast<const bf16x8*>(as + r * 32 * ROW_W + s * 8);
#pragma unroll
            for (int cc = 0; cc < RB; ++cc)
                bfr[cc] = *reinterpret_cast<const bf16x8*>(bs + cc * 32 * ROW_W + s * 8);
#pragma unroll
            for (int r = 0; r < RA; ++r)
#pragma unroll
                for (int cc = 0; cc < RB; ++cc)
                    acc[r][cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cc], af[r], acc[r][cc], 0, 0, 0);   // transposed block
        }
    };

    int ld_step = 0, ld_within = 0;      // chunk the next issue fetches
    const int bcol = col0 - tj * p.T;    // column inside the task's tile column (tile tables)

    if (p.fast_a && p.fast_b && p.fast_k && a_valid >= 4 && b_valid >= 4 && (A_KC || a_valid % 4 == 0) &&
        (B_KC || b_valid % 4 == 0)) {
        // ---- every chunk a full 64 k: unpredicated loads from a running origin plus fixed
        // per-thread offsets (clamped into the tile's valid extent on edge tiles); DEPTH chunks in
        // flight in registers.
        const uint16_t* a_org = A + (A_KC ? (int64_t)row0 * p.lda : (int64_t)row0);
        const uint16_t* b_org = B + (B_KC ? (int64_t)col0 * p.ldb : (int64_t)col0);
        const int64_t a_adv = A_KC ? (int64_t)BK : (int64_t)BK * p.lda;
        const int64_t b_adv = B_KC ? (int64_t)BK : (int64_t)BK * p.ldb;
        // The origin of the next B chunk changes tile at a k-step boundary when B is a tile table;
        // that (uniform) branch is kept apart from the loads so that loads, MFMAs and LDS traffic
        // of one iteration form a single scheduling region.
        auto next_b_origin = [&]() {
            if (p.b_tiles && ld_within == 0) {
                const uint16_t* t = reinterpret_cast<const uint16_t*>(p.b_tiles[(int64_t)ld_step * p.n_j + tj]);
                b_org = t + (B_KC ? (int64_t)bcol * p.ldb : (int64_t)bcol);
            }
        };
        auto issue = [&](LA& sa, LB& sb) {
            fast_load(sa, a_org, p.lda, 0, 0);
            a_org += a_adv;
            fast_load(sb, b_org, p.ldb, 0, 0);
            b_org += b_adv;
            ld_within = (ld_within + 1 == cps) ? 0 : ld_within + 1;
            ld_step += (ld_within == 0);
        };
        constexpr int N_VMEM = LA::N_LOADS + LB::N_LOADS;     // global load instructions per chunk
        constexpr int N_MFMA = RA * RB * (BK / 16);
        constexpr bool SPREAD_LOADS = (NT == 512);            // measured: helps the 8-wave shape only
#pragma unroll
        for (int d = 0; d < DEPTH; ++d)
            if (d < n_chunks) {
                next_b_origin();
                issue(la[d], lb[d]);
            }
        if (n_chunks > 0) {
            la[0].store(As, tid);
            lb[0].store(Bs, tid);
        }
        __syncthreads();
        // Steady state: iteration c refills the register set that held chunk c with chunk c + DEPTH,
        // multiplies chunk c, and moves chunk c + 1 (issued DEPTH - 1 iterations ago) into the other
        // LDS stage.  Nothing in the body is conditional, and the global loads are spread between
        // the MFMAs: the vector-memory unit takes a wave's loads at a limited rate, and a wave that
        // issues all of them up front sits in that queue while its MFMAs wait behind them.
        int c0 = 0;
        for (; c0 + 2 * DEPTH <= n_chunks; c0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const int c = c0 + d;
                next_b_origin();
                issue(la[d], lb[d]);
                compute(c & 1);
                la[(d + 1) % DEPTH].store(As + ((c + 1) & 1) * STAGE_A, tid);
                lb[(d + 1) % DEPTH].store(Bs + ((c + 1) & 1) * STAGE_B, tid);
                if (SPREAD_LOADS) {
#pragma unroll
                    for (int i = 0; i < N_VMEM; ++i) {
                        __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA / N_VMEM, 0);   // MFMA
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);                 // one global load
                    }
                }
                __syncthreads();
            }
        }
        // the last chunks: nothing left to issue
        for (; c0 < n_chunks; c0 += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                const int c = c0 + d;
                if (c < n_chunks) {
                    if (c + DEPTH < n_chunks) {
                        next_b_origin();
                        issue(la[d], lb[d]);
                    }
                    compute(c & 1);
                    if (c + 1 < n_chunks) {
                        la[(d + 1) % DEPTH].store(As + ((c + 1) & 1) * STAGE_A, tid);
                        lb[(d + 1) % DEPTH].store(Bs + ((c + 1) & 1) * STAGE_B, tid);
                    }
                    __syncthreads();
                }
            }
        }
    } else {
        // ---- edge tiles and ragged k-steps: predicated, zero-filling loaders, one chunk in flight
        LA& sa = la[0];
        LB& sb = lb[0];
        auto issue = [&]() {
            const int kk = ld_step * p.T + ld_within * BK;
            const int klim = min(p.K, (ld_step + 1) * p.T);
            sa.load(A, p.lda, row0, row_end, kk, klim, p.vec_a, tid);
            const uint16_t* bsrc = B;
            int bm0 = col0, bm1 = col_end, bk0 = kk, bk1 = klim;
            if (p.b_tiles) {
                bsrc = reinterpret_cast<const uint16_t*>(p.b_tiles[(int64_t)ld_step * p.n_j + tj]);
                bm0 = bcol; bm1 = col_end - tj * p.T;
                bk0 = kk - ld_step * p.T; bk1 = klim - ld_step * p.T;
            }
            sb.load(bsrc, p.ldb, bm0, bm1, bk0, bk1, p.vec_b, tid);
            if (++ld_within == cps) { ld_within = 0; ++ld_step; }
        };
        if (n_chunks > 0) {
            issue();
            sa.store(As, tid);
            sb.store(Bs, tid);
        }
        __syncthreads();
        for (int c = 0; c < n_chunks; ++c) {
            const bool more = (c + 1 < n_chunks);
            if (more) issue();
            compute(c & 1);
            if (more) {
                sa.store(As + ((c + 1) & 1) * STAGE_A, tid);
                sb.store(Bs + ((c + 1) & 1) * STAGE_B, tid);
            }
            __syncthreads();
        }
    }

    epilogue<RA, RB, EPI, OUT_BF16>(p, tc, acc, row0 + wm * WTM, col0 + wn * WTN, li, lh);
}

// ---- host-side launcher -------------------------------------------------------------------------
template <int RA, int RB, int WM, int WN>
struct Cfg {
    static constexpr int BM = WM * 32 * RA, BN = WN * 32 * RB, NT = WM * WN * 64;
    static constexpr size_t LDS = 2 * (size_t)(BM + BN) * ROW_W * 4;
};

template <int RA, int RB, int WM, int WN, int DEPTH, bool A_KC, bool B_KC, int EPI, bool OB>
static hipError_t launch_one(const GemmParams& p, int grid, hipStream_t stream)
{
    typedef Cfg<RA, RB, WM, WN> C;
    auto kern = tile_gemm_bf16<RA, RB, WM, WN, DEPTH, A_KC, B_KC, EPI, OB>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS, stream, p);
    return hipGetLastError();
}

template <int RA, int RB, int WM, int WN, int DEPTH>
static hipError_t launch_cfg(GemmParams& p, const GemmDesc& d, hipStream_t stream)
{
    typedef Cfg<RA, RB, WM, WN> C;
    const int64_t grid = fill_grid(p, d, C::BM, C::BN, BK);
    if (grid == 0) return hipErrorInvalidValue;

#define TGB_LAUNCH(AK, BKC, E, OB) return launch_one<RA, RB, WM, WN, DEPTH, AK, BKC, E, OB>(p, (int)grid, stream)
#define TGB_EPI(AK, BKC)                                                            \
    if (d.epilogue == EPI_AXPBY && !d.out_bf16) { TGB_LAUNCH(AK, BKC, EPI_AXPBY, false); }    \
    if (d.epilogue == EPI_AXPBY && d.out_bf16) { TGB_LAUNCH(AK, BKC, EPI_AXPBY, true); }      \
    if (d.epilogue == EPI_ACT && d.out_bf16) { TGB_LAUNCH(AK, BKC, EPI_ACT, true); }  \
    if (d.epilogue == EPI_DACT && d.out_bf16) { TGB_LAUNCH(AK, BKC, EPI_DACT, true); } \
    return hipErrorInvalidValue;
    if (d.a_kcontig && !d.b_kcontig) { TGB_EPI(true, false) }
    if (!d.a_kcontig && !d.b_kcontig) {
        if (d.epilogue == EPI_MOMENTUM && d.out_bf16) { TGB_LAUNCH(false, false, EPI_MOMENTUM, true); }
        TGB_EPI(false, false)
    }
    if (d.a_kcontig && d.b_kcontig) { TGB_EPI(true, true) }
    return hipErrorInvalidValue;
#undef TGB_EPI
#undef TGB_LAUNCH
}

}  // namespace bf

hipError_t launch_tile_gemm_bf16(const GemmDesc& d, hipStream_t stream)
{
    if (d.M <= 0 || d.N <= 0 || d.K < 0 || d.T <= 0) return hipErrorInvalidValue;
    if (d.M > 0x3fffffff || d.N > 0x3fffffff || d.K > 0x3fffffff) return hipErrorInvalidValue;
    // a bias row goes with the forward products only: activation, or plain fp32 result
    if (d.bias && !(d.epilogue == EPI_ACT || (d.epilogue == EPI_AXPBY && !d.out_bf16))) return hipErrorInvalidValue;
    GemmParams p;
    p.A = d.A; p.B = d.B; p.C = d.C; p.aux = d.aux;
    p.lda = d.lda; p.ldb = d.ldb; p.ldc = d.ldc; p.ldaux = d.ldaux;
    p.M = (int)d.M; p.N = (int)d.N; p.K = (int)d.K;
    int64_t T = d.T;
    const int64_t big = (d.M > d.N ? d.M : d.N) > d.K ? (d.M > d.N ? d.M : d.N) : d.K;
    if (T > big) T = big > 0 ? big : 1;
    p.T = (int)T;
    p.alpha = d.alpha; p.beta = d.beta; p.act = d.act;
    p.sr = (d.sr && d.out_bf16 && (d.epilogue == EPI_AXPBY || d.epilogue == EPI_MOMENTUM)) ? 1 : 0;
    p.state = d.state; p.ldstate = d.ldstate; p.mu = d.mu;
    if (d.epilogue == EPI_MOMENTUM && (!d.state || d.a_kcontig || d.b_kcontig)) return hipErrorInvalidValue;
    p.sr_key = d.sr_key; p.sr_row0 = (uint32_t)d.sr_row0;
    // an fp32 master copy goes with the updates of a bf16 C only (C dense or in tiles; the copy is dense)
    p.master = d.master; p.ldmaster = d.ldmaster;
    if (d.master && (!d.out_bf16 || !(d.epilogue == EPI_MOMENTUM || (d.epilogue == EPI_AXPBY && d.beta != 0.f))))
        return hipErrorInvalidValue;
    p.bias = d.bias;
    p.vec_bias = d.bias && ((reinterpret_cast<uintptr_t>(d.bias) & 15) == 0) && (T % 4 == 0);
    p.b_tiles = d.b_tiles; p.c_tiles = d.c_tiles;
    p.segments = nullptr; p.partial = nullptr;
    p.l_split = 0; p.l_row0 = 0; p.l_col0 = 0; p.l_rcols = 1; p.l_bcols = 1;
    // k-contiguous operands use 16-byte loads (8 elements), m/n-contiguous ones 8-byte loads (4)
    auto ok = [&](const void* q, int64_t ld, bool kc) {
        const int e = kc ? 8 : 4;
        return (T % e == 0) && ((reinterpret_cast<uintptr_t>(q) & (uintptr_t)(2 * e - 1)) == 0) && (ld % e == 0);
    };
    p.vec_a = ok(d.A, d.lda, d.a_kcontig != 0);
    p.vec_b = ok(d.B, d.ldb, d.b_kcontig != 0);
    // epilogue: 4 consecutive columns per access (16 bytes of fp32, 8 bytes of bf16); the tile table's
    // slots are aligned by the cache
    {
        const uintptr_t need = d.out_bf16 ? 7 : 15;
        p.vec_c = (d.ldc % 4 == 0) && ((reinterpret_cast<uintptr_t>(d.C) & need) == 0) && (T % 4 == 0);
        if (d.master) p.vec_c = p.vec_c && (d.ldmaster % 4 == 0) && ((reinterpret_cast<uintptr_t>(d.master) & 15) == 0);
        p.vec_aux = d.aux && (d.ldaux % 4 == 0) && ((reinterpret_cast<uintptr_t>(d.aux) & 7) == 0) && (T % 4 == 0);
    }
    // the unpredicated load path keeps per-thread byte offsets in 32 bits
    auto off32 = [](int64_t ld) { return 256 * ld * 2 + 4096 < ((int64_t)1 << 31); };
    p.fast_a = p.vec_a && off32(d.lda);
    p.fast_b = p.vec_b && off32(d.ldb);
    p.fast_k = (d.K % bf::BK == 0) && (T % bf::BK == 0 || T >= d.K);   // every chunk is a full 64 k
    GemmDesc dd = d;
    dd.T = (int32_t)T;
    // config: 1, 2 = 128 x 128 macro tiles; 3 = 256 x 256 (direct-to-LDS kernel when the operands
    // allow it, else register-staged); 4 = 256 x 256 register-staged; 0 = pick by a cost model
    const bool dl_ok = bf::bf16_dl_applicable(dd);
    int cfg = d.config;
    if (cfg < 1 || cfg > 4) {
        auto tiles = [&](int64_t bm, int64_t bn) {
            const int64_t n_i = (d.M + T - 1) / T, n_j = (d.N + T - 1) / T;
            const int64_t lm = d.M - (n_i - 1) * T, ln = d.N - (n_j - 1) * T;
            const int64_t fm = n_i > 1 ? T : lm, fn = n_j > 1 ? T : ln;
            return ((n_i - 1) * ((fm + bm - 1) / bm) + (lm + bm - 1) / bm) *
                   ((n_j - 1) * ((fn + bn - 1) / bn) + (ln + bn - 1) / bn);
        };
        auto cost = [&](int64_t n_tiles, int64_t per_round, double round_time) {
            return (double)((n_tiles + per_round - 1) / per_round) * round_time;
        };
        // time of one round of workgroups over the chip, relative to a 256 x 256 round of the kernel
        // that will run (measured)
        const double c3 = cost(tiles(256, 256), 256, 1.0);
        const double c2 = cost(tiles(128, 128), 512, dl_ok ? 0.95 : 0.6);
        cfg = c3 <= c2 ? 3 : 2;
    }
    // the balanced schedule's launches exist in the direct-to-LDS kernel only
    if (d.epilogue == EPI_PARTIAL || d.sk_grid_limit > 0) return dl_ok ? bf::launch_tile_gemm_bf16_dl(p, dd, stream) : hipErrorInvalidValue;
    if (d.l_shape) return hipErrorInvalidValue;
    if (cfg == 3 && dl_ok) return bf::launch_tile_gemm_bf16_dl(p, dd, stream);
    if (d.master) cfg = 2;   // of the register-staged shapes only the smaller one carries a master copy
    if (cfg >= 3) return bf::launch_cfg<2, 4, 4, 2, 1>(p, dd, stream);   // 256 x 256, 8 waves of 64 x 128
    return bf::launch_cfg<2, 2, 2, 2, 1>(p, dd, stream);                  // 128 x 128, 4 waves of 64 x 64
}

}  // namespace tg
