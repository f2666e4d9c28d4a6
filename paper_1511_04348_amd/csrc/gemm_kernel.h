// Internal interface between the runtime (engine, MLP passes) and the tile GEMM kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tg {

enum { EPI_AXPBY = 0, EPI_SIGMOID = 1, EPI_DSIGMOID = 2 };

// What a caller asks for: out = epilogue(op(A) op(B)), tiled by T (section 3.1 of the paper).
//   EPI_AXPBY    C = alpha * (A B) + beta * C       (beta == 0: C is not read)
//   EPI_SIGMOID  C = sigmoid(A B)
//   EPI_DSIGMOID C = (A B) * aux * (1 - aux)         (aux: M x N, leading dimension ldaux)
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
    // Optional tile tables (device arrays of device pointers) for operands that live as separate
    // T x T tiles in cache slots instead of one dense matrix.  Entry [step * n_j + tj] of b_tiles
    // is the B tile of k-step `step` and task column tj; entry [ti * n_j + tj] of c_tiles is the C
    // tile of task (ti, tj).  Inside a tile the pitch is ldb / ldc.  NULL = dense operand.
    const void* const* b_tiles;
    void* const* c_tiles;
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
    bool vec_a, vec_b, vec_c;   // vector access is legal for this operand
    bool vec_aux;               // bf16 kernels: 8-byte access to aux is legal
    bool fast_a, fast_b;        // interior tiles may use the unpredicated, 32-bit-offset load path
    bool fast_k;                // every k chunk is full (no ragged k-step tails)
    const void* const* b_tiles; // see GemmDesc
    void* const* c_tiles;
};

int pick_config(const GemmDesc& d);
hipError_t launch_tile_gemm_f32(const GemmDesc& d, hipStream_t stream);
// A, B are bf16 bit patterns; accumulation is fp32.  With out_bf16 the result is rounded to nearest
// even into bf16 and aux is read as bf16; otherwise C is float (aux unused).
hipError_t launch_tile_gemm_bf16(const GemmDesc& d, hipStream_t stream);
inline hipError_t launch_tile_gemm(const GemmDesc& d, int dtype_bf16, hipStream_t stream)
{
    return dtype_bf16 ? launch_tile_gemm_bf16(d, stream) : launch_tile_gemm_f32(d, stream);
}

#ifdef __HIPCC__
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
