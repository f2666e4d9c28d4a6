// fp32 tile GEMM kernel for gfx950 (CDNA4): the "Asynchronous GEMM(A[i,k], B[k,j])" of
// Algorithm 1 of the paper, for every k-step of every output tile C_ij (section 3.1).
//
// One launch covers a whole tiled product.  A workgroup owns one macro tile (BM x BN) of one
// task's output tile and walks that task's k-steps in ascending order, so the summation order of
// every C element is fixed.  Workgroups are numbered task by task, which makes the T x T task
// grid the L2 blocking: the workgroups resident on one XCD at a time belong to one or two tasks
// and share their A row panel and B column panel.
//
// Data path: global -> registers (prefetch of chunk c+1 while chunk c is multiplied) -> LDS
// (double buffered, [k][m] and [k][n] layouts, row padded by 4 floats) -> v_mfma_f32_32x32x2_f32.
// A wave reads RA consecutive rows (RB consecutive columns) per lane with one wide LDS read, so the
// 32x32 MFMA block r of a wave covers rows {RA*i + r}: a permutation of the wave tile that costs
// nothing and gives each lane RB contiguous output columns for vector stores.
//
// Operand storage: A is "k-contiguous" (row-major M x K) or "m-contiguous" (stored K x M, the
// transposed-A product of the backward pass); likewise B.  Edge tiles and ragged k-steps are
// zero-filled on the way into LDS and masked on the way out.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>
#include <utility>

#include "gemm_kernel.h"

namespace tg {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int PAD = 4;       // floats of row padding in LDS
constexpr int SMALL_BK = 32; // k extent of an LDS stage of the small macro tile (the same as the others: four
                             // of its workgroups fit a CU; with 64-k stages, two, and it was slower up to 2048^3)

template <int R> struct Vec;
template <> struct Vec<1> { typedef float type; };
template <> struct Vec<2> { typedef f32x2 type; };
template <> struct Vec<4> { typedef f32x4 type; };

template <int R> __device__ inline float vget(const typename Vec<R>::type& v, int i) { return v[i]; }
template <> __device__ inline float vget<1>(const float& v, int) { return v; }

// ---- global -> register staging of one operand tile chunk -------------------------------------
// BK = k extent of one LDS stage (a "chunk").
// KC = true : source rows are mn, BK contiguous k each.   unit u -> (mn = u / KQ, kq = u % KQ)
// KC = false: source rows are k, BMN contiguous mn each.  unit u -> (k = u / (BMN/4), q = u % (BMN/4))
template <int BMN, int NT, bool KC, int BK, int PADX = PAD>
struct TileLoader {
    static constexpr int KQ = BK / 4;                  // 16-byte units per k-contiguous row of a stage
    static constexpr int UNITS = BMN * BK / 4;
    static constexpr int UP = (UNITS + NT - 1) / NT;   // units per thread
    static_assert(UNITS % NT == 0, "tile must divide evenly over the threads");

    __device__ static inline void load(f32x4 (&reg)[UP], const float* __restrict__ X, int64_t ld,
                                       int mn0, int mn_end, int kk, int klim, bool vec_ok, int tid)
    {
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (KC) {
                const int mn = mn0 + (u / KQ);
                const int k = kk + ((u % KQ) << 2);
                if (mn < mn_end) {
                    const float* src = X + (int64_t)mn * ld + k;
                    if (vec_ok && k + 3 < klim) {
                        v = gload<f32x4>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (k + e < klim) v[e] = gload<float>(src + e);
                    }
                }
            } else {
                constexpr int Q = BMN / 4;
                const int k = kk + u / Q;
                const int mn = mn0 + ((u % Q) << 2);
                if (k < klim) {
                    const float* src = X + (int64_t)k * ld + mn;
                    if (vec_ok && mn + 3 < mn_end) {
                        v = gload<f32x4>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (mn + e < mn_end) v[e] = gload<float>(src + e);
                    }
                }
            }
            reg[p] = v;
        }
    }

    // Full-chunk fast path: per-thread byte offsets from the chunk origin (element (mn0, kk)),
    // computed once, and unpredicated 16-byte loads.  On an edge tile only `valid` (>= 4) of the
    // BMN rows / columns exist: units beyond them are clamped onto the last valid ones, so every
    // address stays inside the matrix.  What they load lands in rows / columns of the product
    // that the epilogue never stores, and cannot reach any other element.
    __device__ static inline void init_offsets(uint32_t (&off)[UP], int64_t ld, int valid, int tid)
    {
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            if (KC) off[p] = (uint32_t)(((int64_t)min(u / KQ, valid - 1) * ld + ((u % KQ) << 2)) * 4);
            else off[p] = (uint32_t)(((int64_t)(u / (BMN / 4)) * ld + min((u % (BMN / 4)) << 2, valid - 4)) * 4);
        }
    }
    __device__ static inline void load_fast(f32x4 (&reg)[UP], const uint32_t (&off)[UP], const float* __restrict__ origin)
    {
        const char* base = reinterpret_cast<const char*>(origin);
#pragma unroll
        for (int p = 0; p < UP; ++p) reg[p] = gload<f32x4>(base + off[p]);
    }

    static constexpr int STORE_INSTS = KC ? 4 : 1;     // LDS store instructions per register of a thread
    // one of the thread's registers -> LDS stage
    __device__ static inline void store_one(const f32x4& r, float* __restrict__ S, int tid, int p)
    {
        constexpr int LD = BMN + PADX;
        const int u = tid + p * NT;
        if (KC) {
            const int mn = u / KQ;
            const int k = (u % KQ) << 2;
#pragma unroll
            for (int e = 0; e < 4; ++e) S[(k + e) * LD + mn] = r[e];
        } else {
            constexpr int Q = BMN / 4;
            const int k = u / Q;
            const int mn = (u % Q) << 2;
            *reinterpret_cast<f32x4*>(&S[k * LD + mn]) = r;
        }
    }
    // registers -> LDS stage (layout [BK][BMN + PAD])
    __device__ static inline void store(const f32x4 (&reg)[UP], float* __restrict__ S, int tid)
    {
        constexpr int LD = BMN + PADX;
#pragma unroll
        for (int p = 0; p < UP; ++p) {
            const int u = tid + p * NT;
            if (KC) {
                const int mn = u / KQ;
                const int k = (u % KQ) << 2;
#pragma unroll
                for (int e = 0; e < 4; ++e) S[(k + e) * LD + mn] = reg[p][e];
            } else {
                constexpr int Q = BMN / 4;
                const int k = u / Q;
                const int mn = (u % Q) << 2;
                *reinterpret_cast<f32x4*>(&S[k * LD + mn]) = reg[p];
            }
        }
    }
};

// One direct global -> LDS load (gfx950 global_load_lds_dwordx4): lane l moves 16 bytes from
// sbase + voff(l) to LDS byte address lds_addr + 16 l, without passing through registers.  The
// compiler does not see the LDS write, so it inserts no waits for it: the consumer waits with an
// explicit vmcnt(0) before the barrier that publishes the stage.
__device__ inline void dma16(uint32_t lds_addr, uint32_t voff, const void* sbase)
{
    const uint64_t b = reinterpret_cast<uint64_t>(sbase);
    const uint32_t blo = __builtin_amdgcn_readfirstlane((uint32_t)b), bhi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    sbase = reinterpret_cast<const void*>(((uint64_t)bhi << 32) | blo);
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

// ---- instruction order of the steady k loop ------------------------------------------------------
// A chunk's LDS reads and the LDS stores of the next chunk may alias as far as the compiler can tell,
// so it keeps them in source order; the loop body is therefore written in the order it should run:
// for every k pair but the last, the fragment reads of the following pair, the pair's MFMAs, and --
// in the first half of the pairs -- a share of the next chunk's global loads, in the second half the
// stores of a share of the staged registers ("pieces": one f32x4 register of the thread each).
// __builtin_amdgcn_sched_group_barrier(mask, n, 0) then asks the scheduler for n instructions of a
// class next (0x008 MFMA, 0x020 global load, 0x100 LDS read, 0x200 LDS write), which spreads a pair's
// loads or stores between its MFMAs.
struct ChunkPlan {
    // pairs 0 .. NKP-1 run before the barrier; H = first pair that takes stores
    template <int NKP> static constexpr int first_store_pair() { return (NKP + 1) / 2; }
    // the pair that stores piece q of NS
    template <int NKP, int NS> static constexpr int pair_of_piece(int q)
    {
        constexpr int H = first_store_pair<NKP>();
        return H + (q * (NKP - H)) / NS;
    }
    // LDS store instructions of pair kp: pieces 0 .. UPA-1 are A registers (IA instructions each),
    // the others B registers (IB each)
    template <int NKP, int UPA, int UPB, int IA, int IB> static constexpr int stores_of_pair(int kp)
    {
        int n = 0;
        for (int q = 0; q < UPA + UPB; ++q)
            if (pair_of_piece<NKP, UPA + UPB>(q) == kp) n += (q < UPA) ? IA : IB;
        return n;
    }
    // global loads of pair kp (NV over the first H pairs)
    template <int NKP, int NV> static constexpr int loads_of_pair(int kp)
    {
        constexpr int H = first_store_pair<NKP>();
        return kp < H ? NV * (kp + 1) / H - NV * kp / H : 0;
    }
};
template <class F, int... I>
__device__ __attribute__((always_inline)) inline void for_each_index(std::integer_sequence<int, I...>, F&& f)
{
    (f(std::integral_constant<int, I>{}), ...);
}
template <int MASK, int N>
__device__ __attribute__((always_inline)) inline void sched_group()
{
    if constexpr (N > 0) __builtin_amdgcn_sched_group_barrier(MASK, N, 0);
}
// MF MFMAs with X instructions of class MASK spread between them
template <int MF, int X, int MASK, int J = 0>
__device__ __attribute__((always_inline)) inline void sched_mix()
{
    if constexpr (X == 0) {
        sched_group<0x008, MF>();
    } else if constexpr (J < X) {
        sched_group<0x008, MF * (J + 1) / X - MF * J / X>();
        sched_group<MASK, 1>();
        sched_mix<MF, X, MASK, J + 1>();
    }
}

// ---- the kernel ---------------------------------------------------------------------------------
// TAIL: the instance for products whose last k chunk is ragged (K % BK != 0); its loop over full chunks
// ends with one predicated, zero-filling chunk.  A separate kernel so that the plain instance's loop
// is compiled exactly as if the tail did not exist.
// LSH: the launch covers the strips right of column p.l_col0 (all rows) and below row p.l_row0 (the
// columns left of l_col0) of the product instead of the whole of it: macro tiles 0 .. l_split - 1
// cover the right strip (l_rcols to a row), the others the bottom strip (l_bcols to a row).
template <int RA, int RB, int WM, int WN, int BK, bool A_KC, bool B_KC, int EPI, bool TAIL, bool LSH = false>
__global__ __launch_bounds__(WM * WN * 64) void tile_gemm_f32(const GemmParams p)
{
    constexpr int WTM = 32 * RA, WTN = 32 * RB;
    constexpr int BM = WM * WTM, BN = WN * WTN;
    constexpr int NT = WM * WN * 64;
    // Row padding of a stage.  A k-contiguous operand is stored transposed, four k rows per register:
    // with a row pitch = 4 mod 64 banks the 16 k quads of a wave's store fall on 4 bank groups (a
    // 4-way conflict), with an odd pitch on 16.  Scalar fragments (one 32 x 32 block per wave) need no
    // alignment, so that shape takes the odd pitch for such operands.
    constexpr int PAD_A = (A_KC && RA == 1) ? 1 : PAD, PAD_B = (B_KC && RB == 1) ? 1 : PAD;
    constexpr int LDA_S = BM + PAD_A, LDB_S = BN + PAD_B;
    constexpr int STAGE_A = BK * LDA_S, STAGE_B = BK * LDB_S;
    typedef TileLoader<BM, NT, A_KC, BK, PAD_A> LA;
    typedef TileLoader<BN, NT, B_KC, BK, PAD_B> LB;
    typedef typename Vec<RA>::type VA;
    typedef typename Vec<RB>::type VB;

    extern __shared__ __attribute__((aligned(16))) float smem[];
    float* As = smem;                    // [2][BK][LDA_S]
    float* Bs = smem + 2 * STAGE_A;      // [2][BK][LDB_S]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int li = lane & 31, lh = lane >> 5;

    // -- workgroup -> (task i,j ; macro tile si,sj).  Consecutive logical ids stay on one XCD.
    int lid;
    {
        const int n = gridDim.x, b = blockIdx.x;
        const int q = n >> 3, r = n & 7, xcd = b & 7, local = b >> 3;
        lid = xcd * q + (xcd < r ? xcd : r) + local;
    }
    // EPI_PARTIAL: this workgroup's segment (macro tile, first chunk, chunks, workspace slot) comes from
    // a table whose order is the plan's: the dispatcher hands workgroups to compute units in that order as
    // the units fall free
    int c_begin = 0, c_count = p.n_chunks, ws_slot = 0;
    if constexpr (EPI == EPI_PARTIAL) {
        const SkSegment sg = p.segments[blockIdx.x];
        lid = sg.tile; c_begin = sg.first_chunk; c_count = sg.n_chunks; ws_slot = sg.slot;
    }
    const int band = p.tpm * p.macro_cols;            // macro tiles in a full band of tasks
    int ti = lid / band;
    const int in_band = lid - ti * band;
    const int h = (ti == p.n_i - 1) ? p.tpm_last : p.tpm;
    int tj = in_band / (h * p.tpn);
    if (tj > p.n_j - 1) tj = p.n_j - 1;
    const int in_task = in_band - tj * h * p.tpn;
    const int wcols = (tj == p.n_j - 1) ? p.tpn_last : p.tpn;
    const int si = in_task / wcols, sj = in_task - si * wcols;

    int row0 = ti * p.T + si * BM;
    int col0 = tj * p.T + sj * BN;
    int row_end = min(p.M, (ti + 1) * p.T);
    int col_end = min(p.N, (tj + 1) * p.T);
    if constexpr (LSH) {     // dense operands; ti, tj are not used then
        if (lid < p.l_split) {
            row0 = (lid / p.l_rcols) * BM; col0 = p.l_col0 + (lid % p.l_rcols) * BN; row_end = p.M; col_end = p.N;
        } else {
            const int b = lid - p.l_split;
            row0 = p.l_row0 + (b / p.l_bcols) * BM; col0 = (b % p.l_bcols) * BN; row_end = p.M; col_end = p.l_col0;
        }
    }

    const float* __restrict__ A = reinterpret_cast<const float*>(p.A);
    const float* __restrict__ B = reinterpret_cast<const float*>(p.B);

    f32x16 acc[RA][RB];
#pragma unroll
    for (int r = 0; r < RA; ++r)
#pragma unroll
        for (int c = 0; c < RB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    f32x4 ra[LA::UP], rb[LB::UP];
    const int n_chunks = c_count;                 // this workgroup's chunks of the k range
    const int cps = p.chunks_per_step;
    const int a_off = wm * WTM + RA * li;
    const int b_off = wn * WTN + RB * li;

    // C: the dense matrix, or this task's tile from the tile table (tile-local coordinates)
    float* __restrict__ C = p.c_tiles ? reinterpret_cast<float*>(p.c_tiles[(int64_t)ti * p.n_j + tj]) -
                                            ((int64_t)(ti * p.T) * p.ldc + tj * p.T)
                                      : p.C;
    // The small shape (one 32 x 32 block per wave, one wave per SIMD) asks for its C values now: its
    // products are short, and 16 dependent load -> multiply-add -> store round trips at the end of the
    // kernel, with nothing else on the SIMD to fill them, cost more than the k loop's last chunks.
    constexpr bool C_EARLY = (RA * RB == 1) && (EPI == EPI_AXPBY);
    float c_early[16];
    if constexpr (C_EARLY) {
        const int colb = col0 + wn * WTN + li;
        if (p.beta != 0.f) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = row0 + wm * WTM + 8 * (v >> 2) + 4 * lh + (v & 3);
                c_early[v] = (row < row_end && colb < col_end) ? gload<float>(C + (int64_t)row * p.ldc + colb) : 0.f;
            }
        }
    }

    // one 16-k chunk from LDS stage st
    auto compute = [&](int st) {
        const float* as = As + st * STAGE_A + lh * LDA_S + a_off;
        const float* bs = Bs + st * STAGE_B + lh * LDB_S + b_off;
#pragma unroll
        for (int kp = 0; kp < BK / 2; ++kp) {
            const VA a = *reinterpret_cast<const VA*>(as + (2 * kp) * LDA_S);
            const VB b = *reinterpret_cast<const VB*>(bs + (2 * kp) * LDB_S);
#pragma unroll
            for (int r = 0; r < RA; ++r)
#pragma unroll
                for (int cc = 0; cc < RB; ++cc)
                    acc[r][cc] = __builtin_amdgcn_mfma_f32_32x32x2f32(vget<RA>(a, r), vget<RB>(b, cc),
                                                                      acc[r][cc], 0, 0, 0);
        }
    };

    // The same chunk in pieces, for the loop that carries the first k pair's fragments across the barrier.
    auto read_frag = [&](int st, int kp, VA& a, VB& b) {
        a = *reinterpret_cast<const VA*>(As + st * STAGE_A + (lh + 2 * kp) * LDA_S + a_off);
        b = *reinterpret_cast<const VB*>(Bs + st * STAGE_B + (lh + 2 * kp) * LDB_S + b_off);
    };
    auto mfma_step = [&](const VA& a, const VB& b) {
#pragma unroll
        for (int r = 0; r < RA; ++r)
#pragma unroll
            for (int cc = 0; cc < RB; ++cc)
                acc[r][cc] = __builtin_amdgcn_mfma_f32_32x32x2f32(vget<RA>(a, r), vget<RB>(b, cc), acc[r][cc], 0, 0, 0);
    };
    // k pairs 0 .. BK/2 - 2 of stage st, starting from the fragments of pair 0 in (a, b); on return
    // (a, b) hold the fragments of the last pair, not yet multiplied
    auto compute_head = [&](int st, VA& a, VB& b) {
#pragma unroll
        for (int kp = 0; kp + 1 < BK / 2; ++kp) {
            VA an;
            VB bn;
            read_frag(st, kp + 1, an, bn);
            mfma_step(a, b);
            a = an;
            b = bn;
        }
    };

    int ld_step = 0, ld_within = 0;      // chunk the next issue fetches
    const int bcol = col0 - tj * p.T;    // column inside the task's tile column (tile tables)

    const int a_valid = min(BM, row_end - row0), b_valid = min(BN, col_end - col0);
    if (p.fast_a && p.fast_b && p.fast_k && a_valid >= 4 && b_valid >= 4 && (A_KC || a_valid % 4 == 0) &&
        (B_KC || b_valid % 4 == 0)) {
        // ---- every chunk a full 16 k: unpredicated loads from a running origin plus fixed
        // per-thread offsets (clamped into the tile's valid extent on edge tiles)
        uint32_t offa[LA::UP], offb[LB::UP];
        LA::init_offsets(offa, p.lda, a_valid, tid);
        LB::init_offsets(offb, p.ldb, b_valid, tid);
        const float* a_org = A + (A_KC ? (int64_t)row0 * p.lda : (int64_t)row0);
        const float* b_org = B + (B_KC ? (int64_t)col0 * p.ldb : (int64_t)col0);
        const int64_t a_adv = A_KC ? (int64_t)BK : (int64_t)BK * p.lda;
        const int64_t b_adv = B_KC ? (int64_t)BK : (int64_t)BK * p.ldb;
        if constexpr (EPI == EPI_PARTIAL) {     // dense operands only: the part starts c_begin chunks in
            a_org += (int64_t)c_begin * a_adv;
            b_org += (int64_t)c_begin * b_adv;
        }
        // The origin of the next B chunk changes tile at a k-step boundary when B is a tile table;
        // that (uniform) branch is kept apart from the loads so that loads, MFMAs and LDS traffic
        // of one iteration form a single scheduling region.
        auto next_b_origin = [&]() {
            if (p.b_tiles && ld_within == 0) {
                const float* t = reinterpret_cast<const float*>(p.b_tiles[(int64_t)ld_step * p.n_j + tj]);
                b_org = t + (B_KC ? (int64_t)bcol * p.ldb : (int64_t)bcol);
            }
        };
        // An m/n-contiguous operand of the 256-wide shape goes straight into LDS: a k row of the stage
        // is 256 floats = the 64 x 16 bytes of one direct load, thread tid's unit p of the register
        // path is exactly lane tid % 64 of the load for row tid / 64 + 8 p, so the same offsets serve.
        // A k-contiguous operand has to be transposed on the way and keeps the register path.
        constexpr bool A_DMA = !A_KC && BM == 256 && NT == 512;
        constexpr bool B_DMA = !B_KC && BN == 256 && NT == 512;
        typedef __attribute__((address_space(3))) float lds_float;
        const uint32_t lds_a = (uint32_t)(uintptr_t)((lds_float*)As), lds_b = (uint32_t)(uintptr_t)((lds_float*)Bs);
        const int wave_u = __builtin_amdgcn_readfirstlane(wave);
        // one direct load (unit p) of the chunk that goes to stage st
        auto dma_a = [&](int st, int pp) {
            dma16(lds_a + (uint32_t)((st * STAGE_A + (wave_u + (NT / 64) * pp) * LDA_S) * 4), offa[pp], a_org);
        };
        auto dma_b = [&](int st, int pp) {
            dma16(lds_b + (uint32_t)((st * STAGE_B + (wave_u + (NT / 64) * pp) * LDB_S) * 4), offb[pp], b_org);
        };
        // st: the stage the chunk is headed for (direct loads need it at issue time)
        auto issue = [&](int st) {
            if constexpr (A_DMA) {
#pragma unroll
                for (int pp = 0; pp < LA::UP; ++pp) dma_a(st, pp);
            }
            if constexpr (B_DMA) {
#pragma unroll
                for (int pp = 0; pp < LB::UP; ++pp) dma_b(st, pp);
            }
            if constexpr (!A_DMA) LA::load_fast(ra, offa, a_org);
            a_org += a_adv;
            if constexpr (!B_DMA) LB::load_fast(rb, offb, b_org);
            b_org += b_adv;
            ld_within = (ld_within + 1 == cps) ? 0 : ld_within + 1;
            ld_step += (ld_within == 0);
        };
        auto dma_wait = [&]() {
            if constexpr (A_DMA || B_DMA) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        };
        constexpr int UPA = A_DMA ? 0 : LA::UP, UPB = B_DMA ? 0 : LB::UP;   // registers staged per chunk
        constexpr int N_VMEM = UPA + UPB;                     // global load instructions per chunk (to registers)
        constexpr int NKP = BK / 2 - 1;                         // k pairs multiplied before the barrier
        constexpr int N_LATE = RA * RB;                         // the last k pair, multiplied after the barrier
        // Only the last chunk of the whole product can be ragged here (K % BK != 0): it takes the
        // predicated, zero-filling loads, in an iteration of its own after the steady loop.
        const int n_fast = TAIL ? n_chunks - 1 : n_chunks;
        auto issue_tail_to = [&](f32x4 (&xa)[LA::UP], f32x4 (&xb)[LB::UP]) {
            const int kk = (p.K / BK) * BK, step = (n_chunks - 1) / cps;
            const float* bsrc = B;
            int bm0 = col0, bm1 = col_end, bk0 = kk, bk1 = p.K;
            if (p.b_tiles) {
                bsrc = reinterpret_cast<const float*>(p.b_tiles[(int64_t)step * p.n_j + tj]);
                bm0 = bcol; bm1 = col_end - tj * p.T;
                bk0 = kk - step * p.T; bk1 = p.K - step * p.T;
            }
            LA::load(xa, A, p.lda, row0, row_end, kk, p.K, p.vec_a, tid);
            LB::load(xb, bsrc, p.ldb, bm0, bm1, bk0, bk1, p.vec_b, tid);
        };
        auto issue_tail = [&]() { issue_tail_to(ra, rb); };
        // ---- small macro tile (one MFMA per k pair, one wave per SIMD): two chunks of loads in flight.
        // A chunk's 32 MFMAs last 0.85 us; loads issued in one half of a chunk and stored in the other
        // had a quarter of a microsecond to arrive, less than the memory latency, and with a single
        // wave per SIMD nothing else fills the wait.  Here chunk c + 2 is requested at the top of the
        // iteration that multiplies chunk c and goes into the second of two register sets; it is
        // stored to LDS in the second half of iteration c + 1, one and a half chunk times later.
        // Chunk i lives in register set i % 2 and in LDS stage i % 2.
        constexpr bool DEEP = (RA * RB == 1);
        if constexpr (DEEP) {
            f32x4 ra2[LA::UP], rb2[LB::UP];
            enum { FETCH_FAST = 0, FETCH_TAIL = 1, FETCH_NONE = 2 };
            auto kind_of = [&](int i) { return i >= n_chunks ? FETCH_NONE : (i < n_fast ? FETCH_FAST : FETCH_TAIL); };
            // (a request behind a branch makes the compiler's wait counts assume the path without it, and
            // the stores of the older set then wait for the newer loads as well: the steady loop below
            // requests unconditionally, only the first and last iterations pass `kind` at run time)
            auto fetch = [&](auto set_tag, int kind) {
                constexpr int S = decltype(set_tag)::value;
                if (kind == FETCH_FAST) {
                    next_b_origin();
                    if constexpr (S == 0) { LA::load_fast(ra, offa, a_org); LB::load_fast(rb, offb, b_org); }
                    else { LA::load_fast(ra2, offa, a_org); LB::load_fast(rb2, offb, b_org); }
                    a_org += a_adv;
                    b_org += b_adv;
                    ld_within = (ld_within + 1 == cps) ? 0 : ld_within + 1;
                    ld_step += (ld_within == 0);
                } else if (TAIL && kind == FETCH_TAIL) {
                    if constexpr (S == 0) issue_tail_to(ra, rb);
                    else issue_tail_to(ra2, rb2);
                }
            };
            // Fragments run FD k pairs ahead of the MFMAs: an LDS read takes longer than the one MFMA
            // (64 cycles) that a distance of one pair would give it.  Slot j % FD holds pair j; the
            // number of pairs of a chunk is a multiple of FD, so the slots carry over from chunk to chunk.
            constexpr int FD = 4, NP = BK / 2;
            static_assert(NP % FD == 0 && NP > FD, "fragment ring must divide the chunk");
            float fra[FD], frb[FD];
            auto ring_read = [&](int st, int pair, int slot) { read_frag(st, pair, fra[slot], frb[slot]); };
            // multiplies chunk c (parity P), requests chunk c + 2, stores chunk c + 1
            auto chunk = [&](auto par_tag, auto kind) {     // kind: an int, or an integral_constant
                constexpr int P = decltype(par_tag)::value;
                fetch(par_tag, kind);
                sched_group<0x020, LA::UP + LB::UP>();      // the requests first, not wherever the scheduler has room
                float* a_next = As + (1 - P) * STAGE_A;
                float* b_next = Bs + (1 - P) * STAGE_B;
                constexpr int UPT = LA::UP + LB::UP;
                for_each_index(std::make_integer_sequence<int, NKP>{}, [&](auto kp_tag) {
                    constexpr int KP = decltype(kp_tag)::value;
                    mfma_step(fra[KP % FD], frb[KP % FD]);
                    if constexpr (KP + FD < NP) ring_read(P, KP + FD, KP % FD);
#pragma unroll
                    for (int q = 0; q < UPT; ++q)
                        if (ChunkPlan::pair_of_piece<NKP, UPT>(q) == KP) {
                            if constexpr (P == 0) {
                                if (q < LA::UP) LA::store_one(ra2[q], a_next, tid, q);
                                else LB::store_one(rb2[q - LA::UP], b_next, tid, q - LA::UP);
                            } else {
                                if (q < LA::UP) LA::store_one(ra[q], a_next, tid, q);
                                else LB::store_one(rb[q - LA::UP], b_next, tid, q - LA::UP);
                            }
                        }
                    sched_group<0x008, 1>();
                    sched_group<0x100, (KP + FD < NP ? 2 : 0)>();
                    constexpr int NST = ChunkPlan::stores_of_pair<NKP, LA::UP, LB::UP, LA::STORE_INSTS, LB::STORE_INSTS>(KP);
                    sched_group<0x200, NST>();
                });
                __builtin_amdgcn_sched_barrier(0);
                __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
                // the stage of chunk c + 1 is complete: its first pairs, around the last MFMA of chunk c
#pragma unroll
                for (int j = 0; j + 1 < FD; ++j) ring_read(1 - P, j, j);
                mfma_step(fra[FD - 1], frb[FD - 1]);
                ring_read(1 - P, FD - 1, FD - 1);
                __builtin_amdgcn_sched_group_barrier(0x100, 2 * (FD - 1), 0);
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            if (n_chunks > 0) {
                fetch(std::integral_constant<int, 0>{}, kind_of(0));
                LA::store(ra, As, tid);
                LB::store(rb, Bs, tid);
                fetch(std::integral_constant<int, 1>{}, kind_of(1));
            }
            __syncthreads();
            if (n_chunks > 0) {
#pragma unroll
                for (int j = 0; j < FD; ++j) ring_read(0, j, j);
            }
            int c = 0;
            for (; c + 3 < n_fast; c += 2) {
                chunk(std::integral_constant<int, 0>{}, std::integral_constant<int, FETCH_FAST>{});
                chunk(std::integral_constant<int, 1>{}, std::integral_constant<int, FETCH_FAST>{});
            }
            for (; c + 1 < n_chunks; ++c) {
                if (c & 1) chunk(std::integral_constant<int, 1>{}, kind_of(c + 2));
                else chunk(std::integral_constant<int, 0>{}, kind_of(c + 2));
            }
            if (c < n_chunks) {   // the last chunk: nothing left to request or store
                const int st = c & 1;
                for_each_index(std::make_integer_sequence<int, NP>{}, [&](auto kp_tag) {
                    constexpr int KP = decltype(kp_tag)::value;
                    mfma_step(fra[KP % FD], frb[KP % FD]);
                    if constexpr (KP + FD < NP) ring_read(st, KP + FD, KP % FD);
                });
                __syncthreads();
            }
        } else {
        if (n_chunks > 0) {
            if (!TAIL || n_fast > 0) {
                next_b_origin();
                issue(0);
                if constexpr (!A_DMA) LA::store(ra, As, tid);
                if constexpr (!B_DMA) LB::store(rb, Bs, tid);
                dma_wait();
            } else {
                issue_tail();
                LA::store(ra, As, tid);
                LB::store(rb, Bs, tid);
            }
        }
        __syncthreads();
        VA fa;      // fragments of the first k pair of the chunk about to be multiplied
        VB fb;
        if (n_chunks > 0) read_frag(0, 0, fa, fb);
        // Steady state: nothing in the body is conditional.  The global loads of the next chunk are
        // spread over the first half of this chunk's MFMAs -- the vector-memory unit takes a wave's
        // loads at a limited rate, and a wave that issues them all up front sits in that queue
        // while its MFMAs wait behind them ...
        // The barrier sits before the chunk's last k pair: by then every LDS read of the chunk has been
        // issued, so the stage may be overwritten, and the first fragments of the next chunk are
        // requested right behind the barrier, their latency covered by the last pair's MFMAs (otherwise
        // both waves of a SIMD wait for those fragments together and the MFMA pipe idles).
        int c = 0;
        for (; c + 1 < n_fast; ++c) {
            next_b_origin();
            issue((c + 1) & 1);
            {
                const int st = c & 1;
                float* a_next = As + ((c + 1) & 1) * STAGE_A;
                float* b_next = Bs + ((c + 1) & 1) * STAGE_B;
                for_each_index(std::make_integer_sequence<int, NKP>{}, [&](auto kp_tag) {
                    constexpr int KP = decltype(kp_tag)::value;
                    VA an;
                    VB bn;
                    read_frag(st, KP + 1, an, bn);
                    mfma_step(fa, fb);
                    if constexpr (UPA + UPB > 0) {
#pragma unroll
                        for (int q = 0; q < UPA + UPB; ++q)
                            if (ChunkPlan::pair_of_piece<NKP, (UPA + UPB > 0 ? UPA + UPB : 1)>(q) == KP) {
                                if (q < UPA) LA::store_one(ra[q], a_next, tid, q);
                                else LB::store_one(rb[q - UPA], b_next, tid, q - UPA);
                            }
                    }
                    sched_group<0x100, 2>();
                    constexpr int NLD = ChunkPlan::loads_of_pair<NKP, N_VMEM>(KP);
                    constexpr int NST = (UPA + UPB > 0)
                        ? ChunkPlan::stores_of_pair<NKP, UPA, (UPA + UPB > 0 ? UPB : 1), LA::STORE_INSTS, LB::STORE_INSTS>(KP) : 0;
                    if constexpr (NLD > 0) sched_mix<RA * RB, NLD, 0x020>();
                    else sched_mix<RA * RB, NST, 0x200>();
                    fa = an;
                    fb = bn;
                });
            }
            __builtin_amdgcn_sched_barrier(0);
            dma_wait();
            __syncthreads();
            __builtin_amdgcn_sched_barrier(0);
            VA na;
            VB nb;
            read_frag((c + 1) & 1, 0, na, nb);
            mfma_step(fa, fb);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);         // the two fragment reads first
            __builtin_amdgcn_sched_group_barrier(0x008, N_LATE, 0);
            __builtin_amdgcn_sched_barrier(0);
            fa = na;
            fb = nb;
        }
        if (TAIL && c + 1 < n_chunks) {
            issue_tail();
            compute_head(c & 1, fa, fb);
            LA::store(ra, As + ((c + 1) & 1) * STAGE_A, tid);
            LB::store(rb, Bs + ((c + 1) & 1) * STAGE_B, tid);
            __syncthreads();
            VA na;
            VB nb;
            read_frag((c + 1) & 1, 0, na, nb);
            mfma_step(fa, fb);
            fa = na;
            fb = nb;
            ++c;
        }
        if (c < n_chunks) {
            compute_head(c & 1, fa, fb);
            mfma_step(fa, fb);
            __syncthreads();
        }
        }   // !DEEP
    } else {
        // ---- ragged k-steps, unaligned operands, tiny edge tiles: predicated, zero-filling loaders.
        // Where only the k-steps are ragged, the chunks that are full (all but the last of a step)
        // still take the unpredicated loads.
        const bool full_ok = p.fast_a && p.fast_b && a_valid >= 4 && b_valid >= 4 && (A_KC || a_valid % 4 == 0) &&
                             (B_KC || b_valid % 4 == 0);
        uint32_t offa[LA::UP], offb[LB::UP];
        if (full_ok) {
            LA::init_offsets(offa, p.lda, a_valid, tid);
            LB::init_offsets(offb, p.ldb, b_valid, tid);
        }
        auto issue = [&]() {
            const int kk = ld_step * p.T + ld_within * BK;
            const int klim = min(p.K, (ld_step + 1) * p.T);
            const float* bsrc = B;
            int bm0 = col0, bm1 = col_end, bk0 = kk, bk1 = klim;
            if (p.b_tiles) {
                bsrc = reinterpret_cast<const float*>(p.b_tiles[(int64_t)ld_step * p.n_j + tj]);
                bm0 = bcol; bm1 = col_end - tj * p.T;
                bk0 = kk - ld_step * p.T; bk1 = klim - ld_step * p.T;
            }
            if (full_ok && kk + BK <= klim) {
                LA::load_fast(ra, offa, A + (A_KC ? (int64_t)row0 * p.lda + kk : (int64_t)kk * p.lda + row0));
                LB::load_fast(rb, offb, bsrc + (B_KC ? (int64_t)bm0 * p.ldb + bk0 : (int64_t)bk0 * p.ldb + bm0));
            } else {
                LA::load(ra, A, p.lda, row0, row_end, kk, klim, p.vec_a, tid);
                LB::load(rb, bsrc, p.ldb, bm0, bm1, bk0, bk1, p.vec_b, tid);
            }
            if (++ld_within == cps) { ld_within = 0; ++ld_step; }
        };
        if (n_chunks > 0) {
            issue();
            LA::store(ra, As, tid);
            LB::store(rb, Bs, tid);
        }
        __syncthreads();
        for (int c = 0; c < n_chunks; ++c) {
            const bool more = (c + 1 < n_chunks);
            if (more) issue();
            compute(c & 1);
            if (more) {
                LA::store(ra, As + ((c + 1) & 1) * STAGE_A, tid);
                LB::store(rb, Bs + ((c + 1) & 1) * STAGE_B, tid);
            }
            __syncthreads();
        }
    }

    // -- epilogue.  acc[r][cc][v] is element (row, col) of the wave tile with
    //    row = RA * (8*(v/4) + 4*lh + v%4) + r,  col = RB * li + cc.
    if constexpr (EPI == EPI_PARTIAL) {
        // the raw sum over this segment of the k range: BM x BN floats in its slot of the workspace
        float* __restrict__ W = p.partial + (int64_t)ws_slot * (int64_t)(BM * BN);
#pragma unroll
        for (int r = 0; r < RA; ++r)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                float* dst = W + (wm * WTM + RA * (8 * (v >> 2) + 4 * lh + (v & 3)) + r) * BN + wn * WTN + RB * li;
#pragma unroll
                for (int cc = 0; cc < RB; cc += 4) {
                    if constexpr (RB % 4 == 0) {
                        gstore<f32x4>(dst + cc, f32x4{acc[r][cc][v], acc[r][cc + 1][v], acc[r][cc + 2][v], acc[r][cc + 3][v]});
                    } else {
#pragma unroll
                        for (int e = 0; e < RB; ++e) gstore<float>(dst + e, acc[r][e][v]);
                    }
                }
            }
        return;
    }
    const float* __restrict__ aux = reinterpret_cast<const float*>(p.aux);
    const float alpha = p.alpha, beta = p.beta;
    const int colb = col0 + wn * WTN + RB * li;
    const bool cvec = p.vec_c && (RB == 4) && (colb + 3 < col_end);
    float bv[RB];   // this lane's columns of the bias row
#pragma unroll
    for (int cc = 0; cc < RB; ++cc) bv[cc] = (p.bias && colb + cc < col_end) ? gload<float>(p.bias + colb + cc) : 0.f;
    // Two passes per row block: first every value the epilogue reads (C, or the stored activations, or
    // the velocities), then the arithmetic and the stores.  Written as one pass, each of the 16 rows
    // waits for its own loads before its stores go out and the next row's loads cannot pass those
    // stores (they may alias as far as the compiler knows): 16 memory round trips in a row per block.
#pragma unroll
    for (int r = 0; r < RA; ++r) {
        constexpr bool READS_C = (EPI == EPI_AXPBY && !C_EARLY) || EPI == EPI_MOMENTUM;
        constexpr bool READS_X = EPI == EPI_DACT || EPI == EPI_MOMENTUM;      // aux, or the velocity
        // rows per pass: all 16 of the block, or 4 where two operands are read and registers are short
        constexpr int G = (READS_C && READS_X && RA * RB >= 8) ? 4 : 16;
        const bool need_c = (EPI == EPI_MOMENTUM) || (EPI == EPI_AXPBY && !C_EARLY && beta != 0.f);
#pragma unroll
        for (int g = 0; g < 16; g += G) {
        float cin[READS_C ? G : 1][RB], xin[READS_X ? G : 1][RB];
#pragma unroll
        for (int vv = 0; vv < G; ++vv) {
            const int v = g + vv;
            const int row = row0 + wm * WTM + RA * (8 * (v >> 2) + 4 * lh + (v & 3)) + r;
            const bool live = row < row_end;
            if constexpr (READS_C) {
                const float* src = C + (int64_t)row * p.ldc + colb;
                if (live && need_c && cvec) {
                    const f32x4 q = gload<f32x4>(src);
#pragma unroll
                    for (int cc = 0; cc < RB; ++cc) cin[vv][cc] = q[cc & 3];
                } else {
#pragma unroll
                    for (int cc = 0; cc < RB; ++cc) cin[vv][cc] = (live && need_c && colb + cc < col_end) ? gload<float>(src + cc) : 0.f;
                }
            }
            if constexpr (READS_X) {
                const float* src = (EPI == EPI_DACT) ? aux + (int64_t)row * p.ldaux + colb : p.state + (int64_t)row * p.ldstate + colb;
#pragma unroll
                for (int cc = 0; cc < RB; ++cc) xin[vv][cc] = (live && colb + cc < col_end) ? gload<float>(src + cc) : 0.f;
            }
        }
#pragma unroll
        for (int vv = 0; vv < G; ++vv) {
            const int v = g + vv;
            const int row = row0 + wm * WTM + RA * (8 * (v >> 2) + 4 * lh + (v & 3)) + r;
            if (row >= row_end) continue;
            float o[RB];
#pragma unroll
            for (int cc = 0; cc < RB; ++cc) o[cc] = acc[r][cc][v] + bv[cc];
            float* dst = C + (int64_t)row * p.ldc + colb;
            if (EPI == EPI_AXPBY) {
                if (C_EARLY) {
                    if (beta != 0.f) o[0] = fmaf(alpha, o[0], beta * c_early[v]);
                    else o[0] = alpha * o[0];
                } else if (beta != 0.f) {
#pragma unroll
                    for (int cc = 0; cc < RB; ++cc) o[cc] = fmaf(alpha, o[cc], beta * cin[READS_C ? vv : 0][cc]);
                } else {
#pragma unroll
                    for (int cc = 0; cc < RB; ++cc) o[cc] = alpha * o[cc];
                }
            } else if (EPI == EPI_MOMENTUM) {
                float* st = p.state + (int64_t)row * p.ldstate + colb;
#pragma unroll
                for (int cc = 0; cc < RB; ++cc)
                    if (colb + cc < col_end) {
                        const float vel = fmaf(p.mu, xin[READS_X ? vv : 0][cc], o[cc]);
                        gstore<float>(st + cc, vel);
                        o[cc] = fmaf(alpha, vel, cin[READS_C ? vv : 0][cc]);
                    }
            } else if (EPI == EPI_ACT) {
#pragma unroll
                for (int cc = 0; cc < RB; ++cc) o[cc] = act_apply(p.act, o[cc]);
            } else if (EPI == EPI_DACT) {
#pragma unroll
                for (int cc = 0; cc < RB; ++cc) o[cc] = o[cc] * act_slope(p.act, xin[READS_X ? vv : 0][cc]);
            }
            if (cvec) {
                f32x4 ov;
#pragma unroll
                for (int cc = 0; cc < RB; ++cc) ov[cc & 3] = o[cc];
                gstore<f32x4>(dst, ov);
            } else {
#pragma unroll
                for (int cc = 0; cc < RB; ++cc)
                    if (colb + cc < col_end) gstore<float>(dst + cc, o[cc]);
            }
        }
        }
    }
}

// ---- host-side launcher -------------------------------------------------------------------------
template <int RA, int RB, int WM, int WN, int BK>
struct Cfg {
    static constexpr int BM = WM * 32 * RA, BN = WN * 32 * RB, NT = WM * WN * 64;
    static constexpr size_t LDS = 2 * (size_t)BK * ((BM + PAD) + (BN + PAD)) * sizeof(float);
};

template <int RA, int RB, int WM, int WN, int BK, bool A_KC, bool B_KC, int EPI, bool TAIL, bool LSH = false>
static hipError_t launch_one(const GemmParams& p, int grid, hipStream_t stream)
{
    typedef Cfg<RA, RB, WM, WN, BK> C;
    auto kern = tile_gemm_f32<RA, RB, WM, WN, BK, A_KC, B_KC, EPI, TAIL, LSH>;
    static bool attr_set = false;   // per instantiation; the attribute is per function, idempotent
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS, stream, p);
    return hipGetLastError();
}

template <int RA, int RB, int WM, int WN, int BK, bool STRIPS_ONLY = false>
static hipError_t launch_cfg(GemmParams& p, const GemmDesc& d, hipStream_t stream)
{
    typedef Cfg<RA, RB, WM, WN, BK> C;
    const int64_t T = d.T;
    p.fast_k = (T % BK == 0 || T >= d.K);   // every k chunk is full, except a ragged last one when K % BK != 0
    p.n_i = (int)((d.M + T - 1) / T);
    p.n_j = (int)((d.N + T - 1) / T);
    const int64_t n_k = (d.K + T - 1) / T;
    const int64_t last_m = d.M - (int64_t)(p.n_i - 1) * T;
    const int64_t last_n = d.N - (int64_t)(p.n_j - 1) * T;
    const int64_t full_m = p.n_i > 1 ? T : last_m, full_n = p.n_j > 1 ? T : last_n;
    p.tpm = (int)((full_m + C::BM - 1) / C::BM);
    p.tpn = (int)((full_n + C::BN - 1) / C::BN);
    p.tpm_last = (int)((last_m + C::BM - 1) / C::BM);
    p.tpn_last = (int)((last_n + C::BN - 1) / C::BN);
    p.macro_cols = (p.n_j - 1) * p.tpn + p.tpn_last;
    const int64_t macro_rows = (int64_t)(p.n_i - 1) * p.tpm + p.tpm_last;
    int64_t grid = macro_rows * p.macro_cols;
    if (grid <= 0 || grid > 0x7fffffff) return hipErrorInvalidValue;
    if (d.sk_grid_limit > 0 && d.sk_grid_limit < grid) grid = d.sk_grid_limit;   // the first macro tiles only
    const int64_t full_k = n_k > 1 ? T : d.K;
    p.chunks_per_step = (int)((full_k + BK - 1) / BK);
    const int64_t last_k = d.K - (n_k - 1) * T;
    p.n_chunks = (int)((n_k - 1) * p.chunks_per_step + (last_k + BK - 1) / BK);

    const bool tail = p.fast_k && (d.K % BK != 0);   // ragged last chunk inside the unpredicated loop
    if (d.l_shape) {
        // the two strips beyond (l_row0, l_col0) of a dense NN product, small shape
        if constexpr (RA * RB == 1) {
            if (!d.a_kcontig || d.b_kcontig || d.epilogue != EPI_AXPBY || d.b_tiles || d.c_tiles || d.l_row0 < 0 || d.l_col0 < 0 ||
                d.l_row0 > d.M || d.l_col0 > d.N)
                return hipErrorInvalidValue;
            const int64_t rcols = (d.N - d.l_col0 + C::BN - 1) / C::BN, bcols = (d.l_col0 + C::BN - 1) / C::BN;
            const int64_t n_right = ((d.M + C::BM - 1) / C::BM) * rcols;
            const int64_t n_bottom = ((d.M - d.l_row0 + C::BM - 1) / C::BM) * bcols;
            if (n_right + n_bottom <= 0 || n_right + n_bottom > 0x7fffffff) return hipErrorInvalidValue;
            p.l_split = (int)n_right; p.l_row0 = (int)d.l_row0; p.l_col0 = (int)d.l_col0;
            p.l_rcols = (int)(rcols > 0 ? rcols : 1); p.l_bcols = (int)(bcols > 0 ? bcols : 1);
            return tail ? launch_one<RA, RB, WM, WN, BK, true, false, EPI_AXPBY, true, true>(p, (int)(n_right + n_bottom), stream)
                        : launch_one<RA, RB, WM, WN, BK, true, false, EPI_AXPBY, false, true>(p, (int)(n_right + n_bottom), stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
    if constexpr (STRIPS_ONLY) return hipErrorInvalidValue;
    else {
    if (d.epilogue == EPI_PARTIAL) {
        // segments of full interior tiles of a dense NN product on the unpredicated path (large shape)
        if constexpr (RA == 2 && RB == 4 && WM == 4 && WN == 2) {
            if (!d.a_kcontig || d.b_kcontig || tail || !p.fast_k || !p.fast_a || !p.fast_b || !p.vec_c || d.b_tiles ||
                d.c_tiles || d.sk_n_segments <= 0 || !d.sk_segments || !d.sk_partial || d.M % C::BM || d.N % C::BN || T % C::BM)
                return hipErrorInvalidValue;
            p.segments = d.sk_segments;
            p.partial = d.sk_partial;
            return launch_one<RA, RB, WM, WN, BK, true, false, EPI_PARTIAL, false>(p, d.sk_n_segments, stream);
        } else {
            return hipErrorInvalidValue;
        }
    }
#define TG_LAUNCH(AK, BKC, E)                                                                        \
    return tail ? launch_one<RA, RB, WM, WN, BK, AK, BKC, E, true>(p, (int)grid, stream)              \
                : launch_one<RA, RB, WM, WN, BK, AK, BKC, E, false>(p, (int)grid, stream)
#define TG_EPI(AK, BKC)                                            \
    switch (d.epilogue) {                                          \
        case EPI_AXPBY: TG_LAUNCH(AK, BKC, EPI_AXPBY);             \
        case EPI_ACT: TG_LAUNCH(AK, BKC, EPI_ACT);         \
        case EPI_DACT: TG_LAUNCH(AK, BKC, EPI_DACT);       \
        default: return hipErrorInvalidValue;                      \
    }
    if (d.a_kcontig && !d.b_kcontig) { TG_EPI(true, false) }
    if (!d.a_kcontig && !d.b_kcontig) {
        if (d.epilogue == EPI_MOMENTUM) TG_LAUNCH(false, false, EPI_MOMENTUM);
        TG_EPI(false, false)
    }
    if (d.a_kcontig && d.b_kcontig) { TG_EPI(true, true) }
    return hipErrorInvalidValue;   // (m-contiguous A) x (k-contiguous B) is not used by any pass
    }
#undef TG_EPI
#undef TG_LAUNCH
}

int pick_config_est(const GemmDesc& d, double* est_us_per_k)
{
    if (est_us_per_k) *est_us_per_k = 0.0;
    if (d.config >= 1 && d.config <= 3) return d.config;
    // Large macro tiles are the most efficient per flop; smaller ones spread small products over
    // the 256 CUs.  Pick the shape with the least estimated time.
    auto tiles = [&](int64_t bm, int64_t bn) {
        const int64_t T = d.T;
        const int64_t n_i = (d.M + T - 1) / T, n_j = (d.N + T - 1) / T;
        const int64_t lm = d.M - (n_i - 1) * T, ln = d.N - (n_j - 1) * T;
        const int64_t fm = n_i > 1 ? T : lm, fn = n_j > 1 ? T : ln;
        return ((n_i - 1) * ((fm + bm - 1) / bm) + (lm + bm - 1) / bm) *
               ((n_j - 1) * ((fn + bn - 1) / bn) + (ln + bn - 1) / bn);
    };
    // Cost model, fitted to square NN products of 1536 .. 8192 with T = 512 (times in us per unit of K
    // for the busiest CU; tiles per CU = ceil(tiles / 256)):
    //   256 x 256: one workgroup per CU, 0.230 per tile;
    //   128 x 128: two workgroups share a CU, 0.061 per tile (0.081 for a single tile, 0.067 each for two);
    //   64 x 64:   two per CU, 0.0155 per tile plus 1.2 tiles' worth of ramp and tail.
    // It reproduces the measured order at every size of that sweep (64 x 64 wins up to 3584 and at
    // 4608 / 5120, 256 x 256 at 4096 and from 7168, 128 x 128 at 6144).
    auto per_cu = [&](int64_t n_tiles) { return (double)((n_tiles + 255) / 256); };
    const double t3 = per_cu(tiles(256, 256)), t2 = per_cu(tiles(128, 128)), t1 = per_cu(tiles(64, 64));
    const double c3 = 0.230 * t3;
    const double c2 = t2 <= 1.0 ? 0.081 : t2 <= 2.0 ? 0.134 : 0.061 * t2;
    const double c1 = 0.0155 * (t1 + 1.2);
    if (est_us_per_k) *est_us_per_k = c3 <= c2 && c3 <= c1 ? c3 : (c2 <= c1 ? c2 : c1);
    if (c3 <= c2 && c3 <= c1) return 3;
    return c2 <= c1 ? 2 : 1;
}

int pick_config(const GemmDesc& d) { return pick_config_est(d, nullptr); }

hipError_t launch_tile_gemm_f32(const GemmDesc& d, hipStream_t stream)
{
    if (d.M <= 0 || d.N <= 0 || d.K < 0 || d.T <= 0) return hipErrorInvalidValue;
    if (d.M > 0x7fffffff || d.N > 0x7fffffff || d.K > 0x7fffffff) return hipErrorInvalidValue;
    GemmParams p;
    p.A = d.A; p.B = d.B; p.C = d.C; p.aux = d.aux;
    p.lda = d.lda; p.ldb = d.ldb; p.ldc = d.ldc; p.ldaux = d.ldaux;
    p.M = (int)d.M; p.N = (int)d.N; p.K = (int)d.K;
    // a tile size beyond every dimension means "one task, one k-step"; clamp so that the index
    // arithmetic in the kernel stays inside int
    int64_t T = d.T;
    const int64_t big = (d.M > d.N ? d.M : d.N) > d.K ? (d.M > d.N ? d.M : d.N) : d.K;
    if (T > big) T = big > 0 ? big : 1;
    p.T = (int)T;
    p.alpha = d.alpha; p.beta = d.beta; p.act = d.act;
    p.sr = 0; p.sr_key = 0; p.sr_row0 = 0; p.bias = d.bias; p.vec_bias = false;
    p.state = d.state; p.ldstate = d.ldstate; p.mu = d.mu;
    p.master = nullptr; p.ldmaster = 0;
    if (d.master) return hipErrorInvalidValue;   // fp32 C is its own master copy
    if (d.epilogue == EPI_MOMENTUM && !d.state) return hipErrorInvalidValue;
    p.b_tiles = d.b_tiles; p.c_tiles = d.c_tiles;
    p.segments = nullptr; p.partial = nullptr;
    p.l_split = 0; p.l_row0 = 0; p.l_col0 = 0; p.l_rcols = 1; p.l_bcols = 1;
    const bool t4 = (T % 4 == 0);
    auto al16 = [](const void* q) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0; };
    p.vec_a = t4 && al16(d.A) && (d.lda % 4 == 0);
    p.vec_b = t4 && al16(d.B) && (d.ldb % 4 == 0);
    p.vec_c = t4 && al16(d.C) && (d.ldc % 4 == 0);
    // the unpredicated load path keeps per-thread byte offsets in 32 bits and needs full chunks
    auto off32 = [](int64_t ld) { return 256 * ld * 4 + 4096 < ((int64_t)1 << 31); };
    p.fast_a = p.vec_a && off32(d.lda);
    p.fast_b = p.vec_b && off32(d.ldb);
    GemmDesc dd = d;
    dd.T = (int32_t)T;
    // the strips stream whole rows of A and columns of B from HBM, 64-k stages fetch them in 256-byte pieces
    if (d.l_shape) return (d.K % 64 == 0 && T % 64 == 0) ? launch_cfg<1, 1, 2, 2, 64, true>(p, dd, stream)
                                                         : launch_cfg<1, 1, 2, 2, SMALL_BK>(p, dd, stream);
    switch (pick_config(dd)) {
        case 3: return launch_cfg<2, 4, 4, 2, 32>(p, dd, stream);   // 256 x 256, 512 threads
        case 2: return launch_cfg<2, 2, 2, 2, 32>(p, dd, stream);   // 128 x 128, 256 threads
        // 64 x 64, 256 threads: the shape for products too small to fill the chip with larger tiles, or
        // whose large tiles would leave a last round mostly empty; its k loop keeps two chunks of loads
        // in flight (see the kernel)
        default: return launch_cfg<1, 1, 2, 2, SMALL_BK>(p, dd, stream);
    }
}

}  // namespace tg
