// Internal interface between the runtime (engine, MLP passes) and the tile GEMM kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tg {

enum { EPI_AXPBY = 0, EPI_ACT = 1, EPI_DACT = 2, EPI_MOMENTUM = 3, EPI_PARTIAL = 4 };
enum { ACT_SIGMOID = 0, ACT_TANH = 1, ACT_RELU = 2 };   // same values as TGEMM_ACT_* of the C ABI

// A segment of the balanced schedule (launch_gemm_balanced): n_chunks chunks of the k range of
// macro tile `tile` (its number in the launch's task-by-task order) from chunk first_chunk on; the sum
// goes to slot `slot` of the workspace.
struct SkSegment {
    int32_t tile, first_chunk, n_chunks, slot;
};

// What a caller asks for: out = epilogue(op(A) op(B)), tiled by T (section 3.1 of the paper).
//   EPI_AXPBY    C = alpha * (A B) + beta * C       (beta == 0: C is not read)
//   EPI_ACT      C = act(A B)                        act: sigmoid, tanh or max(0, .)
//   EPI_DACT     C = (A B) * act'(z) with act' written in terms of the stored activation aux = act(z)
//                (aux: M x N, leading dimension ldaux): aux (1 - aux), 1 - aux^2, or [aux > 0]
//   EPI_PARTIAL  (launch_gemm_balanced's own use) the raw sum over a part of
//                the k range of one macro tile, stored to a workspace
//   EPI_MOMENTUM S = mu * S + (A B);  C = C + alpha * S   (S: M x N floats, leading dimension ldstate;
//                the update with a velocity matrix; S is dense also when C is a tile table).  Offered for the layout of the
//                dW product (both operands m/n-contiguous).
// a_kcontig: A stored M x K row-major (k contiguous); otherwise stored K x M (m contiguous).
// b_kcontig: B stored N x K row-major (k contiguous); otherwise stored K x N (n contiguous).
struct GemmDesc {
    const void* A;
    const void* B;
    float* C;
    const void* aux;
    int64_t lda, ldb, ldc, ldaux;
    int64_t M, N, K;
    int32_t T;
    int32_t a_kcontig, b_kcontig;
    int32_t epilogue;
    float alpha, beta;
    int32_t config;   // 0 = automatic, 1..3 = small / medium / large macro tile
    int32_t out_bf16; // bf16 kernel only: C (and aux) hold bf16 bit patterns instead of float
    int32_t act;      // ACT_* for EPI_ACT / EPI_DACT
    // Optional row vector (N floats, device) added to every row of A B before the epilogue function:
    // EPI_ACT gives act(A B + 1 bias^T), EPI_AXPBY alpha (A B + 1 bias^T) + beta C.  NULL = none.
    // The bf16 kernels take it with EPI_ACT and with EPI_AXPBY into a float C only.
    const float* bias;
    // bf16 kernel, EPI_AXPBY with out_bf16: round the result stochastically instead of to nearest.
    // Entry (row, col) of this launch draws its 16 random bits from rounding_bits(sr_key,
    // sr_row0 + row, col); sr_row0 places a launch that covers a band of rows inside the whole matrix.
    int32_t sr;
    uint32_t sr_key;
    int64_t sr_row0;
    float* state;     // EPI_MOMENTUM: S
    int64_t ldstate;
    float mu;
    // bf16 kernel, EPI_AXPBY (beta != 0) or EPI_MOMENTUM with out_bf16: an fp32 copy of C (M x N,
    // leading dimension ldmaster).  The old value of C is taken from it instead of from the bf16 C,
    // the fp32 result is stored back into it, and C receives that result rounded to bf16.  The copy is dense also when C is a tile table.
    float* master;
    int64_t ldmaster;
    // Optional tile tables (device arrays of device pointers) for operands that live as separate
    // T x T tiles in cache slots instead of one dense matrix.  Entry [step * n_j + tj] of b_tiles
    // is the B tile of k-step `step` and task column tj; entry [ti * n_j + tj] of c_tiles is the C
    // tile of task (ti, tj).  Inside a tile the pitch is ldb / ldc.  NULL = dense operand.
    const void* const* b_tiles;
    void* const* c_tiles;
    // Set only by launch_gemm_balanced (zero otherwise): launch the first sk_grid_limit macro tiles
    // of the product only; or, with EPI_PARTIAL, one workgroup per entry of the segment table
    // sk_segments (device memory, sk_n_segments entries), which store their sums to sk_partial.
    int32_t sk_grid_limit, sk_n_segments;
    const SkSegment* sk_segments;
    float* sk_partial;
    // fp32, EPI_AXPBY, dense NN operands, small shape: with l_shape set the launch computes only the
    // entries of C in columns >= l_col0 (all rows) and in rows >= l_row0 (columns < l_col0): the two
    // strips that a product leaves beyond a block of whole macro tiles.
    int32_t l_shape;
    int64_t l_row0, l_col0;
};

// Kernel argument block (filled by the launcher).
struct GemmParams {
    const void* A;
    const void* B;
    float* C;
    const void* aux;
    int64_t lda, ldb, ldc, ldaux;
    int M, N, K, T;
    int n_i, n_j;               // task grid
    int tpm, tpn;               // macro tiles per full task, rows / cols
    int tpm_last, tpn_last;     // macro tiles of the last (possibly ragged) task row / col
    int macro_cols;             // macro-tile columns of the whole matrix
    int chunks_per_step;        // BK-chunks in a full k-step
    int n_chunks;               // BK-chunks over all k-steps
    float alpha, beta;
    int act;                    // ACT_* for the activation epilogues
    const float* bias;          // see GemmDesc
    float* state;               // EPI_MOMENTUM
    int64_t ldstate;
    float mu;
    float* master;              // fp32 copy of a bf16 C (see GemmDesc); vec_c then also covers it
    int64_t ldmaster;
    int sr;                     // stochastic rounding of a bf16 result (see GemmDesc)
    uint32_t sr_key;
    uint32_t sr_row0;
    bool vec_a, vec_b, vec_c;   // vector access is legal for this operand
    bool vec_aux;               // bf16 kernels: 8-byte access to aux is legal
    bool vec_bias;              // bf16 kernels: 16-byte access to bias is legal
    bool fast_a, fast_b;        // interior tiles may use the unpredicated, 32-bit-offset load path
    bool fast_k;                // every k chunk is full (fp32 kernel: except a ragged last chunk of the product)
    const void* const* b_tiles; // see GemmDesc
    void* const* c_tiles;
    int l_split, l_row0, l_col0; // strips launch (see the kernel's LSH parameter):
    int l_rcols, l_bcols;        // macro-tile columns of the right strip and of the bottom strip
    const SkSegment* segments;  // EPI_PARTIAL: one entry per workgroup
    float* partial;             // EPI_PARTIAL: workspace, 256 x 256 floats per segment
};

int pick_config(const GemmDesc& d);
// the same choice; *est_us_per_k (optional) receives the cost model's time of the chosen shape in
// microseconds per unit of K
int pick_config_est(const GemmDesc& d, double* est_us_per_k);
hipError_t launch_tile_gemm_f32(const GemmDesc& d, hipStream_t stream);
// C += A B (A row-major M x K, B row-major K x N, C float: the in-core tgemm_run) with the work spread
// evenly over the compute units when the 256 x 256 macro tiles do not come out as whole rounds of
// one tile per unit.  The interior (the multiples of 256 in M and N) runs its whole rounds as usual;
// the tiles of the last, partial round are cut along k into segments -- the (tile, chunk) pairs laid
// end to end and divided into as many equal ranges as there are units -- which run as workgroups of
// their own, longest first, and leave their sums in a workspace; a fix-up kernel then adds each
// tile's segment sums in ascending order of k, and that sum to C.  The remainder strips (fewer than
// 256 rows / columns) run as one launch of small macro tiles on a side stream.
// An element's summation order is still a function of the sizes and the unit count alone.
// Returns hipErrorNotSupported -- having launched nothing -- when the product does not qualify or the
// estimate promises no gain, unless whatever_the_estimate (the caller then uses launch_tile_gemm_f32).  The main work is enqueued
// on `stream`; the strips on `side` behind `fork` (recorded on stream when the segments are
// enqueued), and stream waits for `join` (recorded on side) at the end.  *ws: plan and device workspace
// (128 MiB, allocated at the first qualifying call), kept across calls; released by sk_destroy.
struct SkWorkspace;
void sk_destroy(SkWorkspace* ws);
// With bf16 (A, B bf16 bit patterns, C float) the direct-to-LDS kernel runs the whole rounds and the
// segments; products with strips (M or N no multiple of 256) are declined.
hipError_t launch_gemm_balanced(const GemmDesc& d, bool bf16, SkWorkspace** ws, int n_cus, bool whatever_the_estimate,
                                hipStream_t stream, hipStream_t side, hipEvent_t fork, hipEvent_t join, int* launches);
// A, B are bf16 bit patterns; accumulation is fp32.  With out_bf16 the result is rounded to nearest
// even into bf16 and aux is read as bf16; otherwise C is float (aux unused).
hipError_t launch_tile_gemm_bf16(const GemmDesc& d, hipStream_t stream);
namespace bf {
// whether the direct-to-LDS bf16 kernel takes the product (d.T already clamped to the largest dimension)
bool bf16_dl_applicable(const GemmDesc& d);
}
inline hipError_t launch_tile_gemm(const GemmDesc& d, int dtype_bf16, hipStream_t stream)
{
    return dtype_bf16 ? launch_tile_gemm_bf16(d, stream) : launch_tile_gemm_f32(d, stream);
}

// Counter-based random bits for stochastic rounding.  mix32 is the 32-bit finalizer of MurmurHash3
// (a bijection of the 32-bit integers with good avalanche); all arithmetic is modulo 2^32.
//   step_key(seed, layer, step) = mix32(mix32(mix32(mix32(seed_lo) ^ seed_hi) ^ layer) ^ step)
//   pair_bits(key, row, col)    = mix32(mix32(row + key) + (col / 2) * 0x9E3779B9)
//   rounding_bits(key, row, col) = 16 bits of pair_bits: the low half for even col, the high half for odd col
__host__ __device__ inline uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x85ebca6bu;
    x ^= x >> 13; x *= 0xc2b2ae35u;
    x ^= x >> 16;
    return x;
}
inline uint32_t sr_step_key(uint64_t seed, uint32_t layer, uint32_t step)
{
    return mix32(mix32(mix32(mix32((uint32_t)seed) ^ (uint32_t)(seed >> 32)) ^ layer) ^ step);
}

#ifdef __HIPCC__
// Activation and its slope in terms of the activation's own value (what the backward pass has stored).
__device__ inline float act_apply(int act, float z)
{
    if (act == ACT_RELU) return fmaxf(z, 0.f);
    if (act == ACT_TANH) {
        const float t = __expf(-2.f * fabsf(z));
        return copysignf((1.f - t) / (1.f + t), z);
    }
    return 1.f / (1.f + __expf(-z));
}
__device__ inline float act_slope(int act, float a)
{
    if (act == ACT_RELU) return a > 0.f ? 1.f : 0.f;
    if (act == ACT_TANH) return 1.f - a * a;
    return a * (1.f - a);
}

// Loads / stores through explicitly global (address space 1) pointers.  Operand pointers that come
// out of a tile table are "generic" to the compiler, which would otherwise emit flat memory
// instructions; those count against the LDS wait counter and stall the LDS reads behind every
// outstanding prefetch.
#define TG_GLOBAL __attribute__((address_space(1)))
template <typename V, typename E>
__device__ inline V gload(const E* p)
{
    return *reinterpret_cast<const TG_GLOBAL V*>((const TG_GLOBAL E*)p);
}
template <typename V, typename E>
__device__ inline void gstore(E* p, const V& v)
{
    *reinterpret_cast<TG_GLOBAL V*>((TG_GLOBAL E*)p) = v;
}
#endif

}  // namespace tg
