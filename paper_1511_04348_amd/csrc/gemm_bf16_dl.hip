// bf16 -> fp32 tile GEMM for gfx950 (CDNA4) with direct global -> LDS loads: the tile product of
// Algorithm 1 of the paper for operands whose layout allows it (16-byte aligned rows, whole 32-k
// chunks); everything else takes the register-staged kernel of gemm_bf16.hip.
//
// What gfx950 adds and this kernel is built on:
//   * global_load_lds_dwordx4: a wave moves 64 x 16 bytes from global memory straight into 1 KB of
//     LDS (lane l lands at base + 16 l, base in M0).  No staging registers, no LDS store
//     instructions, and the load is asynchronous: four 32-k stages ride in LDS, three of them in
//     flight while the fourth is multiplied.
//   * ds_read_b64_tr_b16: a 16-lane group reads a 4 (k) x 16 (n) patch of 16-bit elements and
//     hands every lane the 4 consecutive k of one n -- the MFMA operand layout straight from a
//     row-major [k][n] tile, so m/n-contiguous operands need no transposition in registers.
//
// LDS layouts (chosen so that every read is bank-conflict free, verified with the LDS conflict
// counter):
//   * k-contiguous operand (row-major A; W in D W^T): rows of 32 k = 64 B = four 16-byte pieces,
//     piece kp of row m stored at slot 4 m + (kp ^ ((m / 4) % 4)); read with ds_read_b128.
//   * m/n-contiguous operand (row-major B; A^T and D in A^T D): bricks of 4 k x 32 mn = 256 B,
//     brick (kb, nb) at (kb * (BMN / 32) + nb) * 256; a half wave reads one whole brick per
//     ds_read_b64_tr_b16.
// Since the lane -> global address map of a direct load is free, both layouts are produced by
// choosing which 16 bytes each lane fetches.
//
// Schedule: 8 waves, wave tile 128 x 64 (4 x 2 MFMA blocks of 32 x 32), two waves per SIMD.  A
// wave alternates between a memory phase (LDS reads of its operands for one chunk, then its share
// of the direct loads three chunks ahead) and an MFMA phase (16 MFMAs); the upper four waves run
// one phase behind the lower four, so that on every SIMD one wave feeds the MFMA pipe while the
// other waits on memory.  Phases are separated by workgroup barriers; before each barrier a wave
// waits until its own share of all but the two youngest chunks has landed.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_bf16_common.h"

namespace tg {
namespace bf {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) char lds_char;

constexpr int DL_BK = 32;          // k per LDS stage
constexpr int DL_STAGES = 4;
constexpr int DL_RA = 4, DL_RB = 2, DL_WM = 2, DL_WN = 4;
constexpr int DL_NW = DL_WM * DL_WN;
constexpr int DL_BM = DL_WM * DL_RA * 32, DL_BN = DL_WN * DL_RB * 32;
constexpr int DL_LDS = DL_STAGES * (DL_BM + DL_BN) * DL_BK * 2;

// One direct load: lane l moves 16 bytes from sbase + voff(l) to LDS byte address lds_addr + 16 l.
// The compiler does not see an LDS write here, so it inserts no waits for it: every consumer
// below is ordered by an explicit vmcnt wait and a barrier.
__device__ inline void dma16(uint32_t lds_addr, uint32_t voff, const void* sbase)
{
    // base and LDS address are the same in every lane; make the compiler keep them in scalar registers
    const uint64_t b = reinterpret_cast<uint64_t>(sbase);
    const uint32_t blo = __builtin_amdgcn_readfirstlane((uint32_t)b), bhi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    sbase = reinterpret_cast<const void*>(((uint64_t)bhi << 32) | blo);
    lds_addr = __builtin_amdgcn_readfirstlane(lds_addr);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :: "s"(lds_addr), "v"(voff), "s"(sbase) : "memory");
}

// Entry `idx` (the same in every lane) of a table of device pointers, through the scalar unit: the
// compiler would use a vector load here (the direct loads above are opaque memory operations to it)
// and wait for it with vmcnt(0), which also drains every direct load in flight.
__device__ inline const void* table_entry(const void* const* table, int64_t idx)
{
    const uint64_t a = reinterpret_cast<uint64_t>(table + idx);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)a), hi = __builtin_amdgcn_readfirstlane((uint32_t)(a >> 32));
    const uint64_t addr = ((uint64_t)hi << 32) | lo;
    uint64_t v;
    asm volatile("s_load_dwordx2 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(addr) : "memory");
    return reinterpret_cast<const void*>(v);
}

// ---- k-contiguous operand: BMN rows of 64 bytes per stage -----------------------------------------
// A 1 KB block is 16 rows x 4 pieces; wave w moves blocks w, w + NW, ...
template <int BMN>
struct DlKC {
    static constexpr int BYTES = BMN * DL_BK * 2;
    static constexpr int PER = BYTES / 1024 / DL_NW;
    static_assert(BYTES % (1024 * DL_NW) == 0, "blocks per wave");
    uint32_t off[PER];     // byte offset of this lane's 16 bytes from the chunk origin (row mn0, k0)
    uint32_t rd[2];        // LDS read offset of the lane for the two 16-k steps of a chunk

    // `valid` (>= 1) of the BMN rows exist: rows beyond them are clamped onto the last valid one, so
    // every address stays inside the matrix; what they load only reaches rows / columns of the
    // product that the epilogue never stores.
    __device__ inline void init(int64_t ld, int valid, int wave, int lane, int wave_row0)
    {
        const int kp = (lane & 3) ^ ((lane >> 4) & 3);     // piece held by LDS slot lane % 4 of this row
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int row = 16 * (wave + DL_NW * i) + (lane >> 2);
            off[i] = (uint32_t)((int64_t)min(row, valid - 1) * ld * 2 + (kp << 4));
        }
        const int li = lane & 31, lh = lane >> 5;
#pragma unroll
        for (int s = 0; s < 2; ++s) rd[s] = (uint32_t)((wave_row0 + li) * 64 + (((2 * s + lh) ^ ((li >> 2) & 3)) << 4));
    }
    // origin: element (mn0, k0) of the chunk
    __device__ inline void issue(uint32_t lds_stage, const uint16_t* origin, int wave) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) dma16(lds_stage + (wave + DL_NW * i) * 1024, off[i], origin);
    }
    // 8 consecutive k (k = 16 s + 8 lh ..) of row wave_row0 + 32 r + li
    __device__ inline bf16x8 read(const lds_char* stage, int s, int r) const
    {
        return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(stage + rd[s] + r * 32 * 64);
    }
    static __device__ inline const uint16_t* chunk_origin(const uint16_t* X, int64_t ld, int mn0, int k0)
    {
        return X + (int64_t)mn0 * ld + k0;
    }
};

// ---- m/n-contiguous operand: 32 k-rows of BMN elements per stage, stored as bricks ---------------
// A 1 KB block is four bricks side by side (4 k-rows x 128 mn); wave w moves blocks w, w + NW, ...
template <int BMN>
struct DlMC {
    static constexpr int NB = BMN / 32;                  // bricks per k-group
    static constexpr int BYTES = BMN * DL_BK * 2;
    static constexpr int PER = BYTES / 1024 / DL_NW;
    static_assert(BYTES % (1024 * DL_NW) == 0 && NB % 4 == 0, "blocks per wave");
    uint32_t off[PER];
    uint32_t rd;

    // `valid` (>= 8, a multiple of 8) of the BMN columns exist: pieces beyond them are clamped onto
    // the last valid eight.
    __device__ inline void init(int64_t ld, int valid, int wave, int lane, int wave_col0)
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int brick = 4 * (wave + DL_NW * i) + (lane >> 4);
            const int kb = brick / NB, nb = brick % NB;
            const int krow = 4 * kb + ((lane & 15) >> 2);
            const int mn = 32 * nb + 8 * (lane & 3);
            off[i] = (uint32_t)(((int64_t)krow * ld + min(mn, valid - 8)) * 2);
        }
        // transposing read: in a 16-lane group lane sl points at k-row sl / 4, columns 4 (sl % 4) ..
        // of the group's 16 columns, and receives the 4 k of column sl; lanes 32.. take the k-group
        // 8 further on
        const int sl = lane & 15, b16 = (lane >> 4) & 1, lh = lane >> 5;
        rd = (uint32_t)((2 * lh * NB + wave_col0 / 32) * 256 + (sl >> 2) * 64 + (16 * b16 + 4 * (sl & 3)) * 2);
    }
    // origin: element (k0, mn0) of the chunk
    __device__ inline void issue(uint32_t lds_stage, const uint16_t* origin, int wave) const
    {
#pragma unroll
        for (int i = 0; i < PER; ++i) dma16(lds_stage + (wave + DL_NW * i) * 1024, off[i], origin);
    }
    // 8 consecutive k (k = 16 s + 8 lh ..) of column wave_col0 + 32 r + li
    __device__ inline bf16x8 read(const lds_char* stage, int s, int r) const
    {
        const lds_char* bp = stage + rd + (4 * s * NB + r) * 256;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)bp);
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(bp + NB * 256));
        const s16x8 w = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        return __builtin_bit_cast(bf16x8, w);
    }
    static __device__ inline const uint16_t* chunk_origin(const uint16_t* X, int64_t ld, int mn0, int k0)
    {
        return X + (int64_t)k0 * ld + mn0;
    }
};

template <int BMN, bool KC> struct PickDl { typedef DlKC<BMN> type; };
template <int BMN> struct PickDl<BMN, false> { typedef DlMC<BMN> type; };

template <bool A_KC, bool B_KC, int EPI, bool OUT_BF16>
__global__ __launch_bounds__(DL_NW * 64) void tile_gemm_bf16_dl(const GemmParams p)
{
    constexpr int RA = DL_RA, RB = DL_RB, WN = DL_WN, BM = DL_BM, BN = DL_BN;
    constexpr int WTM = 32 * RA, WTN = 32 * RB;
    typedef typename PickDl<BM, A_KC>::type LA;
    typedef typename PickDl<BN, B_KC>::type LB;
    constexpr int A_BYTES = LA::BYTES, STAGE = LA::BYTES + LB::BYTES;
    constexpr int PER = LA::PER + LB::PER;     // direct loads per wave per chunk

    extern __shared__ __attribute__((aligned(1024))) char smem[];
    const uint32_t lds0 = (uint32_t)(uintptr_t)((lds_char*)smem);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool late = wave >= DL_NW / 2;       // waves w and w + 4 share a SIMD
    const int wm = wave / WN, wn = wave % WN;

    // the tile coordinates are the same in every lane; kept in scalar registers they make the tile
    // table lookups scalar loads (a vector load there would have to be waited for with vmcnt(0),
    // draining the direct loads in flight)
    // EPI_PARTIAL (the balanced schedule of the in-core product, see gemm_kernel.h): this workgroup's
    // segment of a macro tile's k range comes from a table; its sum goes to a slot of the workspace
    int seg_tile = -1, seg_first = 0, seg_chunks = p.n_chunks, seg_slot = 0;
    if constexpr (EPI == EPI_PARTIAL) {
        const SkSegment sg = p.segments[blockIdx.x];
        seg_tile = __builtin_amdgcn_readfirstlane(sg.tile);
        seg_first = __builtin_amdgcn_readfirstlane(sg.first_chunk);
        seg_chunks = __builtin_amdgcn_readfirstlane(sg.n_chunks);
        seg_slot = __builtin_amdgcn_readfirstlane(sg.slot);
    }
    TileCoord tc = decode_tile<BM, BN>(p, seg_tile);
    tc.ti = __builtin_amdgcn_readfirstlane(tc.ti);
    tc.tj = __builtin_amdgcn_readfirstlane(tc.tj);
    tc.row0 = __builtin_amdgcn_readfirstlane(tc.row0);
    tc.col0 = __builtin_amdgcn_readfirstlane(tc.col0);
    tc.row_end = __builtin_amdgcn_readfirstlane(tc.row_end);
    tc.col_end = __builtin_amdgcn_readfirstlane(tc.col_end);
    const int tj = tc.tj, row0 = tc.row0, col0 = tc.col0;
    const uint16_t* __restrict__ A = reinterpret_cast<const uint16_t*>(p.A);
    const uint16_t* __restrict__ B = reinterpret_cast<const uint16_t*>(p.B);

    LA la;
    LB lb;
    la.init(p.lda, max(min(BM, tc.row_end - row0), A_KC ? 1 : 8), wave, lane, wm * WTM);
    lb.init(p.ldb, max(min(BN, tc.col_end - col0), B_KC ? 1 : 8), wave, lane, wn * WTN);

    f32x16 acc[RA][RB];
#pragma unroll
    for (int r = 0; r < RA; ++r)
#pragma unroll
        for (int c = 0; c < RB; ++c)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[r][c][v] = 0.f;

    const int n_chunks = seg_chunks;
    const int cps = p.chunks_per_step;
    const int bcol = col0 - tj * p.T;          // column inside the task's tile column (tile tables)

    // the chunk the next issue fetches: k-step, chunk within the step, and its origins
    int ld_step = 0, ld_within = 0, ld_chunk = 0;
    const uint16_t* a_org = LA::chunk_origin(A, p.lda, row0, 0);
    const uint16_t* b_org = LB::chunk_origin(B, p.ldb, col0, 0);
    const int64_t a_adv = A_KC ? (int64_t)DL_BK : (int64_t)DL_BK * p.lda;
    const int64_t b_adv = B_KC ? (int64_t)DL_BK : (int64_t)DL_BK * p.ldb;
    if constexpr (EPI == EPI_PARTIAL) {      // dense operands only
        a_org += seg_first * a_adv;
        b_org += seg_first * b_adv;
    }
    auto issue = [&]() {
        if (p.b_tiles && ld_within == 0) {
            const uint16_t* t = reinterpret_cast<const uint16_t*>(table_entry(p.b_tiles, (int64_t)ld_step * p.n_j + tj));
            b_org = LB::chunk_origin(t, p.ldb, bcol, 0);
        }
        const uint32_t st = lds0 + (uint32_t)(ld_chunk & (DL_STAGES - 1)) * STAGE;
        la.issue(st, a_org, wave);
        lb.issue(st + A_BYTES, b_org, wave);
        a_org += a_adv;
        b_org += b_adv;
        ++ld_chunk;
        ld_within = (ld_within + 1 == cps) ? 0 : ld_within + 1;
        ld_step += (ld_within == 0);
    };
    // Phase boundary.  In the steady state a wave has its shares of three chunks outstanding; the
    // oldest must have landed before anyone reads it.  Near the end fewer are outstanding than the
    // constant assumes, so the last boundaries wait for everything.
    // The LDS reads of the phase must have completed as well (lgkmcnt): the stage they came from is
    // overwritten by other waves' direct loads after a later barrier.
    auto boundary = [&](bool drain) {
        if (drain) asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" :: "n"(2 * PER) : "memory");
        __syncthreads();
    };

#pragma unroll
    for (int c = 0; c < DL_STAGES - 1; ++c)
        if (c < n_chunks) issue();
    boundary(n_chunks <= DL_STAGES);
    if (late) boundary(n_chunks <= DL_STAGES);
    for (int c = 0; c < n_chunks; ++c) {
        const bool drain = (c + DL_STAGES >= n_chunks);
        // memory phase: operands of chunk c, then this wave's share of chunk c + 3, whose stage was
        // last read (chunk c - 1) before the barrier this phase started with
        const lds_char* st = (const lds_char*)smem + (c & (DL_STAGES - 1)) * STAGE;
        bf16x8 af[2][RA], bfr[2][RB];
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int r = 0; r < RA; ++r) af[s][r] = la.read(st, s, r);
#pragma unroll
            for (int cc = 0; cc < RB; ++cc) bfr[s][cc] = lb.read(st + A_BYTES, s, cc);
        }
        if (c + DL_STAGES - 1 < n_chunks) issue();
        boundary(drain);
        // MFMA phase
        __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int s = 0; s < 2; ++s)
#pragma unroll
            for (int r = 0; r < RA; ++r)
#pragma unroll
                for (int cc = 0; cc < RB; ++cc)
                    acc[r][cc] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[s][cc], af[s][r], acc[r][cc], 0, 0, 0);   // transposed block
        __builtin_amdgcn_s_setprio(0);
        boundary(drain);
    }
    if (!late) boundary(true);      // every wave passes the same number of barriers

    // every wave has passed its last LDS read and all direct loads have landed: the stages are free, and
    // each wave takes 32 x 68 floats of them for the transposition of its accumulators
    float* area = reinterpret_cast<float*>(smem) + wave * (32 * (32 * RB + 4));
    if constexpr (EPI == EPI_PARTIAL) {
        // the raw sums, as a plain store into a "matrix" of pitch BN whose entry (row0, col0) is the slot's first float
        GemmParams q = p;
        q.C = p.partial + (int64_t)seg_slot * (BM * BN) - ((int64_t)row0 * BN + col0);
        q.ldc = BN;
        q.alpha = 1.f; q.beta = 0.f;
        q.bias = nullptr; q.c_tiles = nullptr; q.master = nullptr; q.sr = 0;
        q.vec_c = true;
        epilogue_rows<RA, RB, EPI_AXPBY, false>(q, tc, acc, row0 + wm * WTM, col0 + wn * WTN, lane, area);
    } else {
        epilogue_rows<RA, RB, EPI, OUT_BF16>(p, tc, acc, row0 + wm * WTM, col0 + wn * WTN, lane, area);
    }
}

template <bool A_KC, bool B_KC, int EPI, bool OB>
static hipError_t launch_dl(const GemmParams& p, int grid, hipStream_t stream)
{
    auto kern = tile_gemm_bf16_dl<A_KC, B_KC, EPI, OB>;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, DL_LDS);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(DL_NW * 64), DL_LDS, stream, p);
    return hipGetLastError();
}

bool bf16_dl_applicable(const GemmDesc& d)
{
    const int64_t T = d.T;      // already clamped to the largest dimension by the caller
    if (d.M <= 0 || d.N <= 0 || T <= 0) return false;
    // every chunk a whole 32 k
    if (d.K % DL_BK != 0 || d.K <= 0 || !(T % DL_BK == 0 || T >= d.K)) return false;
    // 16-byte pieces: aligned bases and pitches; tile tables hold slot addresses aligned by the cache
    auto aligned = [](const void* q, int64_t ld) { return (reinterpret_cast<uintptr_t>(q) & 15) == 0 && ld % 8 == 0; };
    if (!aligned(d.A, d.lda) || !aligned(d.B, d.ldb)) return false;
    // m/n-contiguous operands move in pieces of 8 columns: every tile extent a multiple of 8
    const int64_t n_i = (d.M + T - 1) / T, n_j = (d.N + T - 1) / T;
    const int64_t last_m = d.M - (n_i - 1) * T, last_n = d.N - (n_j - 1) * T;
    if (!d.a_kcontig && (last_m % 8 != 0 || (n_i > 1 && T % 8 != 0))) return false;
    if (!d.b_kcontig && (last_n % 8 != 0 || (n_j > 1 && T % 8 != 0))) return false;
    // per-lane byte offsets are 32-bit
    auto fits = [](int64_t ld, bool kc) { return (kc ? 256 : 32) * ld * 2 + 4096 < ((int64_t)1 << 31); };
    if (!fits(d.lda, d.a_kcontig != 0) || !fits(d.ldb, d.b_kcontig != 0)) return false;
    // layouts and epilogues the kernel is instantiated for
    if (!d.a_kcontig && d.b_kcontig) return false;
    if (d.epilogue != EPI_AXPBY && d.epilogue != EPI_PARTIAL && !d.out_bf16) return false;
    return true;
}

hipError_t launch_tile_gemm_bf16_dl(GemmParams p, const GemmDesc& d, hipStream_t stream)
{
    if (!bf16_dl_applicable(d)) return hipErrorNotSupported;
    int64_t grid = fill_grid(p, d, DL_BM, DL_BN, DL_BK);
    if (grid == 0) return hipErrorInvalidValue;
    if (d.sk_grid_limit > 0 && d.sk_grid_limit < grid) grid = d.sk_grid_limit;     // the first macro tiles only
    if (d.epilogue == EPI_PARTIAL) {
        // segments of whole interior tiles of a dense NN product with a float result
        if (!d.a_kcontig || d.b_kcontig || d.out_bf16 || d.b_tiles || d.c_tiles || d.sk_n_segments <= 0 || !d.sk_segments ||
            !d.sk_partial || d.M % DL_BM || d.N % DL_BN || d.T % DL_BM)
            return hipErrorInvalidValue;
        p.segments = d.sk_segments;
        p.partial = d.sk_partial;
        return launch_dl<true, false, EPI_PARTIAL, false>(p, d.sk_n_segments, stream);
    }

#define TGD_LAUNCH(AK, BKC, E, OB) return launch_dl<AK, BKC, E, OB>(p, (int)grid, stream)
#define TGD_EPI(AK, BKC)                                                            \
    if (d.epilogue == EPI_AXPBY && !d.out_bf16) { TGD_LAUNCH(AK, BKC, EPI_AXPBY, false); }    \
    if (d.epilogue == EPI_AXPBY && d.out_bf16) { TGD_LAUNCH(AK, BKC, EPI_AXPBY, true); }      \
    if (d.epilogue == EPI_ACT && d.out_bf16) { TGD_LAUNCH(AK, BKC, EPI_ACT, true); }  \
    if (d.epilogue == EPI_DACT && d.out_bf16) { TGD_LAUNCH(AK, BKC, EPI_DACT, true); } \
    return hipErrorNotSupported;
    if (d.a_kcontig && !d.b_kcontig) { TGD_EPI(true, false) }
    if (!d.a_kcontig && !d.b_kcontig) {
        if (d.epilogue == EPI_MOMENTUM && d.out_bf16) { TGD_LAUNCH(false, false, EPI_MOMENTUM, true); }
        TGD_EPI(false, false)
    }
    if (d.a_kcontig && d.b_kcontig) { TGD_EPI(true, true) }
    return hipErrorNotSupported;
#undef TGD_EPI
#undef TGD_LAUNCH
}

}  // namespace bf
}  // namespace tg
