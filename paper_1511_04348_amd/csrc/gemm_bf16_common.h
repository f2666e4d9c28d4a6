// Pieces shared by the two bf16 tile GEMM kernels (register-staged and direct-to-LDS): the
// workgroup -> macro tile decode, the epilogue, and the grid arithmetic of the launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.h"

namespace tg {
namespace bf {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ inline float bf16_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);   // NaN stays NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Stochastic rounding: the 16 bits below the bf16 cut plus 16 uniform random bits carry into the kept
// half with probability (dropped fraction), so the expected result is the unrounded value; a value
// that bf16 holds exactly never moves.  Infinities and NaNs go the nearest-even way.
__device__ inline uint16_t f32_to_bf16_sr(float f, uint32_t r16)
{
    const uint32_t u = __float_as_uint(f);
    if ((u & 0x7f800000u) == 0x7f800000u) return f32_to_bf16_rne(f);
    return (uint16_t)((u + r16) >> 16);
}
// 32 random bits shared by columns 2 (col / 2) and 2 (col / 2) + 1 of a row (hrow: the row's hash)
__device__ inline uint32_t pair_bits(uint32_t hrow, int col) { return mix32(hrow + (uint32_t)(col >> 1) * 0x9E3779B9u); }

// Which macro tile a workgroup owns.  Workgroups are numbered XCD by XCD (consecutive logical ids
// stay on one XCD and share its L2) and task by task (the T x T task grid is the L2 blocking).
struct TileCoord {
    int ti, tj;             // task (output tile of section 3.1)
    int row0, col0;         // first row / column of the macro tile
    int row_end, col_end;   // end of the task's rows / columns (clamped to the matrix)
};

// macro_tile >= 0: that macro tile (its number in the task-by-task order) instead of the workgroup's own.
template <int BM, int BN>
__device__ inline TileCoord decode_tile(const GemmParams& p, int macro_tile = -1)
{
    int lid = macro_tile;
    if (macro_tile < 0) {
        const int n = gridDim.x, b = blockIdx.x;
        const int q = n >> 3, r = n & 7, xcd = b & 7, local = b >> 3;
        lid = xcd * q + (xcd < r ? xcd : r) + local;
    }
    TileCoord t;
    const int band = p.tpm * p.macro_cols;
    t.ti = lid / band;
    const int in_band = lid - t.ti * band;
    const int h = (t.ti == p.n_i - 1) ? p.tpm_last : p.tpm;
    t.tj = in_band / (h * p.tpn);
    if (t.tj > p.n_j - 1) t.tj = p.n_j - 1;
    const int in_task = in_band - t.tj * h * p.tpn;
    const int wcols = (t.tj == p.n_j - 1) ? p.tpn_last : p.tpn;
    const int si = in_task / wcols, sj = in_task - si * wcols;
    t.row0 = t.ti * p.T + si * BM;
    t.col0 = t.tj * p.T + sj * BN;
    t.row_end = min(p.M, (t.ti + 1) * p.T);
    t.col_end = min(p.N, (t.tj + 1) * p.T);
    return t;
}

typedef float f32x4 __attribute__((ext_vector_type(4)));

// The fp32 result of an update goes back into the master copy of a bf16 C (quad: columns col .. col + 3).
__device__ inline void store_master(const GemmParams& p, const TileCoord& t, int row, int col, const f32x4& o, bool vec)
{
    float* dst = p.master + (int64_t)row * p.ldmaster + col;
    if (vec && col + 3 < t.col_end) {
        gstore<f32x4>(dst, o);
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (col + e < t.col_end) gstore<float>(dst + e, o[e]);
    }
}

// The kernels feed the MFMA with the B fragment as its first and the A fragment as its second
// operand, i.e. they accumulate the transposed 32 x 32 block: a lane then owns one row of C and
// four consecutive columns per register quad,
//    acc[r][cc][v]:  row = 32 r + li,  col = 32 cc + 8 (v / 4) + 4 lh + v % 4     (li = lane % 32, lh = lane / 32),
// which turns the epilogue's traffic into 16-byte (fp32) or 8-byte (bf16) accesses.  Everything the
// epilogue reads for one r is requested before the first value is used.
// wrow0 / wcol0: first row / column of the wave tile in the matrix.
template <int RA, int RB, int EPI, bool OUT_BF16>
__device__ inline void epilogue(const GemmParams& p, const TileCoord& t, const f32x16 (&acc)[RA][RB], int wrow0,
                                int wcol0, int li, int lh)
{
    const float alpha = p.alpha, beta = p.beta;
    // C: the dense matrix, or this task's tile from the tile table (tile-local coordinates)
    const int64_t c_shift = p.c_tiles ? ((int64_t)(t.ti * p.T) * p.ldc + t.tj * p.T) : 0;
    void* c_base = p.c_tiles ? p.c_tiles[(int64_t)t.ti * p.n_j + t.tj] : (void*)p.C;
    float* __restrict__ Cf = reinterpret_cast<float*>(c_base) - c_shift;
    uint16_t* __restrict__ Cb = reinterpret_cast<uint16_t*>(c_base) - c_shift;
    const uint16_t* __restrict__ aux = reinterpret_cast<const uint16_t*>(p.aux);
    // with an fp32 master copy the old value is read from it quad by quad in the second loop
    // (wave tiles of up to 64 x 64 only: the 64 x 128 wave tile has no registers to spare for it, and
    // the launcher sends updates with a master copy to the smaller shape)
    constexpr bool MASTER = OUT_BF16 && RA * RB <= 4 && (EPI == EPI_AXPBY || EPI == EPI_MOMENTUM);
    const bool from_master = MASTER && (EPI == EPI_AXPBY) && p.master != nullptr;
    const bool read_c = (EPI == EPI_AXPBY) && beta != 0.f && !from_master;
    const bool vec_c = p.vec_c, vec_aux = p.vec_aux;
#pragma unroll
    for (int r = 0; r < RA; ++r) {
        const int row = wrow0 + 32 * r + li;
        if (row >= t.row_end) continue;
        const int64_t crow = (int64_t)row * p.ldc;
        f32x4 in[RB][4];     // C (AXPBY) or the activation (DSIGMOID) at this lane's 4 x RB quads
        if (read_c || EPI == EPI_DACT) {
#pragma unroll
            for (int cc = 0; cc < RB; ++cc)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int col = wcol0 + 32 * cc + 8 * g + 4 * lh;
                    f32x4 x = {0.f, 0.f, 0.f, 0.f};
                    if (EPI == EPI_DACT) {
                        const uint16_t* src = aux + (int64_t)row * p.ldaux + col;
                        if (vec_aux && col + 3 < t.col_end) {
                            const u32x2 w = gload<u32x2>(src);
                            x[0] = __uint_as_float(w[0] << 16); x[1] = __uint_as_float(w[0] & 0xffff0000u);
                            x[2] = __uint_as_float(w[1] << 16); x[3] = __uint_as_float(w[1] & 0xffff0000u);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < t.col_end) x[e] = bf16_to_f32(gload<uint16_t>(src + e));
                        }
                    } else if (OUT_BF16) {
                        const uint16_t* src = Cb + crow + col;
                        if (vec_c && col + 3 < t.col_end) {
                            const u32x2 w = gload<u32x2>(src);
                            x[0] = __uint_as_float(w[0] << 16); x[1] = __uint_as_float(w[0] & 0xffff0000u);
                            x[2] = __uint_as_float(w[1] << 16); x[3] = __uint_as_float(w[1] & 0xffff0000u);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < t.col_end) x[e] = bf16_to_f32(gload<uint16_t>(src + e));
                        }
                    } else {
                        const float* src = Cf + crow + col;
                        if (vec_c && col + 3 < t.col_end) {
                            x = gload<f32x4>(src);
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < t.col_end) x[e] = gload<float>(src + e);
                        }
                    }
                    in[cc][g] = x;
                }
        }
#pragma unroll
        for (int cc = 0; cc < RB; ++cc)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int col = wcol0 + 32 * cc + 8 * g + 4 * lh;
                if (col >= t.col_end) continue;
                f32x4 bv = {0.f, 0.f, 0.f, 0.f};   // this quad's columns of the bias row
                if ((EPI == EPI_ACT || (EPI == EPI_AXPBY && !OUT_BF16)) && p.bias) {   // the forward products
                    if (col + 3 < t.col_end && p.vec_bias) {
                        bv = gload<f32x4>(p.bias + col);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < t.col_end) bv[e] = gload<float>(p.bias + col + e);
                    }
                }
                f32x4 old = {0.f, 0.f, 0.f, 0.f};
                if (MASTER && EPI == EPI_AXPBY && from_master) {
                    const float* src = p.master + (int64_t)row * p.ldmaster + col;
                    if (vec_c && col + 3 < t.col_end) {
                        old = gload<f32x4>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < t.col_end) old[e] = gload<float>(src + e);
                    }
                }
                f32x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = acc[r][cc][4 * g + e] + bv[e];
                    if (EPI == EPI_AXPBY) {
                        v = from_master ? fmaf(alpha, v, beta * old[e]) : read_c ? fmaf(alpha, v, beta * in[cc][g][e]) : alpha * v;
                    } else if (EPI == EPI_MOMENTUM) {
                        if (col + e < t.col_end) {   // S = mu S + acc; C = C + alpha S (C read here, entry by entry)
                            float* st = p.state + (int64_t)row * p.ldstate + col + e;
                            const float vel = fmaf(p.mu, gload<float>(st), v);
                            gstore<float>(st, vel);
                            const float c_old = !OUT_BF16 ? gload<float>(Cf + crow + col + e)
                                                : (MASTER && p.master) ? gload<float>(p.master + (int64_t)row * p.ldmaster + col + e)
                                                                       : bf16_to_f32(gload<uint16_t>(Cb + crow + col + e));
                            v = fmaf(alpha, vel, c_old);
                        }
                    } else if (EPI == EPI_ACT) {
                        v = act_apply(p.act, v);
                    } else if (EPI == EPI_DACT) {
                        v = v * act_slope(p.act, in[cc][g][e]);
                    }
                    o[e] = v;
                }
                if (OUT_BF16) {
                    if (MASTER && p.master) store_master(p, t, row, col, o, vec_c);
                    uint16_t b[4];
                    if ((EPI == EPI_AXPBY || EPI == EPI_MOMENTUM) && p.sr) {
                        // col is even when T is (pairs col / 2 and col / 2 + 1); odd tile sizes go column by column
                        const uint32_t hrow = mix32(p.sr_row0 + (uint32_t)row + p.sr_key);
                        const bool even = (col & 1) == 0;
                        const uint32_t b0 = pair_bits(hrow, col), b1 = pair_bits(hrow, col + 2);
                        const uint32_t bm = even ? b0 : pair_bits(hrow, col + 1);
                        const uint32_t be = even ? b1 : pair_bits(hrow, col + 3);
                        b[0] = f32_to_bf16_sr(o[0], even ? b0 & 0xffffu : b0 >> 16);
                        b[1] = f32_to_bf16_sr(o[1], even ? b0 >> 16 : bm & 0xffffu);
                        b[2] = f32_to_bf16_sr(o[2], even ? b1 & 0xffffu : bm >> 16);
                        b[3] = f32_to_bf16_sr(o[3], even ? b1 >> 16 : be & 0xffffu);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) b[e] = f32_to_bf16_rne(o[e]);
                    }
                    uint16_t* dst = Cb + crow + col;
                    if (vec_c && col + 3 < t.col_end) {
                        u32x2 w;
                        w[0] = (uint32_t)b[0] | ((uint32_t)b[1] << 16);
                        w[1] = (uint32_t)b[2] | ((uint32_t)b[3] << 16);
                        gstore<u32x2>(dst, w);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < t.col_end) gstore<uint16_t>(dst + e, b[e]);
                    }
                } else {
                    float* dst = Cf + crow + col;
                    if (vec_c && col + 3 < t.col_end) {
                        gstore<f32x4>(dst, o);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (col + e < t.col_end) gstore<float>(dst + e, o[e]);
                    }
                }
            }
    }
}

// ---- the same epilogue through a transposition in LDS ---------------------------------------------
// In the accumulator layout a wave's global access covers 32 rows with 32 bytes each; every 128-byte
// line of C is touched by four instructions, and a round of workgroups asks for all of C in that
// shape at the same moment.  Here a wave first writes a 32-row block of its accumulators into a
// private LDS area (row pitch 32 RB + 4 floats: conflict free for the 16-byte writes) and reads it back
// row by row: lane l then holds columns 4 (l % LPR) .. + 3 of row l / LPR, so that one instruction
// covers whole rows of the block (256 contiguous bytes each at RB = 2) for C, for the stored
// activations and for the result.  Arithmetic, rounding and random bits per element are those of
// `epilogue` above (tested bit for bit against it).
// One quad = 4 consecutive columns col .. col + 3 of one row; x = the accumulator values.
template <int EPI, bool OUT_BF16>
__device__ inline f32x4 quad_input(const GemmParams& p, const TileCoord& t, const float* Cf, const uint16_t* Cb,
                                   const uint16_t* aux, bool read_c, int row, int col)
{
    f32x4 x = {0.f, 0.f, 0.f, 0.f};
    if (EPI == EPI_DACT) {
        const uint16_t* src = aux + (int64_t)row * p.ldaux + col;
        if (p.vec_aux && col + 3 < t.col_end) {
            const u32x2 w = gload<u32x2>(src);
            x[0] = __uint_as_float(w[0] << 16); x[1] = __uint_as_float(w[0] & 0xffff0000u);
            x[2] = __uint_as_float(w[1] << 16); x[3] = __uint_as_float(w[1] & 0xffff0000u);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < t.col_end) x[e] = bf16_to_f32(gload<uint16_t>(src + e));
        }
    } else if (read_c) {
        const int64_t at = (int64_t)row * p.ldc + col;
        if (OUT_BF16 && p.master) {
            const float* src = p.master + (int64_t)row * p.ldmaster + col;
            if (p.vec_c && col + 3 < t.col_end) {
                x = gload<f32x4>(src);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < t.col_end) x[e] = gload<float>(src + e);
            }
        } else if (OUT_BF16) {
            if (p.vec_c && col + 3 < t.col_end) {
                const u32x2 w = gload<u32x2>(Cb + at);
                x[0] = __uint_as_float(w[0] << 16); x[1] = __uint_as_float(w[0] & 0xffff0000u);
                x[2] = __uint_as_float(w[1] << 16); x[3] = __uint_as_float(w[1] & 0xffff0000u);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < t.col_end) x[e] = bf16_to_f32(gload<uint16_t>(Cb + at + e));
            }
        } else {
            if (p.vec_c && col + 3 < t.col_end) {
                x = gload<f32x4>(Cf + at);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (col + e < t.col_end) x[e] = gload<float>(Cf + at + e);
            }
        }
    }
    return x;
}

template <int EPI, bool OUT_BF16>
__device__ inline void quad_finish(const GemmParams& p, const TileCoord& t, float* Cf, uint16_t* Cb, bool read_c,
                                   int row, int col, const f32x4& a, const f32x4& in)
{
    const float alpha = p.alpha, beta = p.beta;
    const int64_t crow = (int64_t)row * p.ldc;
    f32x4 bv = {0.f, 0.f, 0.f, 0.f};
    if ((EPI == EPI_ACT || (EPI == EPI_AXPBY && !OUT_BF16)) && p.bias) {
        if (col + 3 < t.col_end && p.vec_bias) {
            bv = gload<f32x4>(p.bias + col);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < t.col_end) bv[e] = gload<float>(p.bias + col + e);
        }
    }
    f32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float v = a[e] + bv[e];
        if (EPI == EPI_AXPBY) {
            v = read_c ? fmaf(alpha, v, beta * in[e]) : alpha * v;
        } else if (EPI == EPI_MOMENTUM) {
            if (col + e < t.col_end) {
                float* st = p.state + (int64_t)row * p.ldstate + col + e;
                const float vel = fmaf(p.mu, gload<float>(st), v);
                gstore<float>(st, vel);
                const float c_old = !OUT_BF16 ? gload<float>(Cf + crow + col + e)
                                    : p.master ? gload<float>(p.master + (int64_t)row * p.ldmaster + col + e)
                                               : bf16_to_f32(gload<uint16_t>(Cb + crow + col + e));
                v = fmaf(alpha, vel, c_old);
            }
        } else if (EPI == EPI_ACT) {
            v = act_apply(p.act, v);
        } else if (EPI == EPI_DACT) {
            v = v * act_slope(p.act, in[e]);
        }
        o[e] = v;
    }
    if (OUT_BF16) {
        if ((EPI == EPI_AXPBY || EPI == EPI_MOMENTUM) && p.master)
            store_master(p, t, row, col, o, p.vec_c);
        uint16_t b[4];
        if ((EPI == EPI_AXPBY || EPI == EPI_MOMENTUM) && p.sr) {
            const uint32_t hrow = mix32(p.sr_row0 + (uint32_t)row + p.sr_key);
            const bool even = (col & 1) == 0;
            const uint32_t b0 = pair_bits(hrow, col), b1 = pair_bits(hrow, col + 2);
            const uint32_t bm = even ? b0 : pair_bits(hrow, col + 1);
            const uint32_t be = even ? b1 : pair_bits(hrow, col + 3);
            b[0] = f32_to_bf16_sr(o[0], even ? b0 & 0xffffu : b0 >> 16);
            b[1] = f32_to_bf16_sr(o[1], even ? b0 >> 16 : bm & 0xffffu);
            b[2] = f32_to_bf16_sr(o[2], even ? b1 & 0xffffu : bm >> 16);
            b[3] = f32_to_bf16_sr(o[3], even ? b1 >> 16 : be & 0xffffu);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) b[e] = f32_to_bf16_rne(o[e]);
        }
        uint16_t* dst = Cb + crow + col;
        if (p.vec_c && col + 3 < t.col_end) {
            u32x2 w;
            w[0] = (uint32_t)b[0] | ((uint32_t)b[1] << 16);
            w[1] = (uint32_t)b[2] | ((uint32_t)b[3] << 16);
            gstore<u32x2>(dst, w);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < t.col_end) gstore<uint16_t>(dst + e, b[e]);
        }
    } else {
        float* dst = Cf + crow + col;
        if (p.vec_c && col + 3 < t.col_end) {
            gstore<f32x4>(dst, o);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (col + e < t.col_end) gstore<float>(dst + e, o[e]);
        }
    }
}

// lds: this wave's private area of 32 x (32 RB + 4) floats; every wave of the workgroup must be done
// with whatever the area held before.
template <int RA, int RB, int EPI, bool OUT_BF16>
__device__ inline void epilogue_rows(const GemmParams& p, const TileCoord& t, const f32x16 (&acc)[RA][RB], int wrow0,
                                     int wcol0, int lane, float* lds)
{
    constexpr int PITCH = 32 * RB + 4;
    constexpr int LPR = 8 * RB;            // lanes per row of the block
    constexpr int RPI = 64 / LPR;          // rows per instruction
    constexpr int NI = 32 / RPI;           // instructions per 32-row block
    const int li = lane & 31, lh = lane >> 5;
    const int rl = lane / LPR, cl = 4 * (lane % LPR);
    const int64_t c_shift = p.c_tiles ? ((int64_t)(t.ti * p.T) * p.ldc + t.tj * p.T) : 0;
    void* c_base = p.c_tiles ? p.c_tiles[(int64_t)t.ti * p.n_j + t.tj] : (void*)p.C;
    float* __restrict__ Cf = reinterpret_cast<float*>(c_base) - c_shift;
    uint16_t* __restrict__ Cb = reinterpret_cast<uint16_t*>(c_base) - c_shift;
    const uint16_t* __restrict__ aux = reinterpret_cast<const uint16_t*>(p.aux);
    const bool read_c = (EPI == EPI_AXPBY) && p.beta != 0.f;
    const int col = wcol0 + cl;
#pragma unroll
    for (int r = 0; r < RA; ++r) {
        // what the block needs from memory, requested first
        f32x4 in[NI];
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = wrow0 + 32 * r + RPI * j + rl;
            in[j] = f32x4{0.f, 0.f, 0.f, 0.f};
            if (row < t.row_end && col < t.col_end) in[j] = quad_input<EPI, OUT_BF16>(p, t, Cf, Cb, aux, read_c, row, col);
        }
        // accumulator layout -> LDS: lane (li, lh) owns row li, columns 32 cc + 8 g + 4 lh .. + 3
#pragma unroll
        for (int cc = 0; cc < RB; ++cc)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                f32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[r][cc][4 * g + e];
                *reinterpret_cast<f32x4*>(lds + li * PITCH + 32 * cc + 8 * g + 4 * lh) = v;
            }
        // LDS -> row layout, finish, store (the area belongs to this wave alone; its LDS accesses
        // execute in order)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int row = wrow0 + 32 * r + RPI * j + rl;
            const f32x4 a = *reinterpret_cast<const f32x4*>(lds + (RPI * j + rl) * PITCH + cl);
            if (row < t.row_end && col < t.col_end) quad_finish<EPI, OUT_BF16>(p, t, Cf, Cb, read_c, row, col, a, in[j]);
        }
    }
}

// Fills the task grid, macro-tile and chunk counts of `p` for BM x BN macro tiles and chunks of
// CHUNK_K; returns the grid size (0 if it does not fit a launch).
inline int64_t fill_grid(GemmParams& p, const GemmDesc& d, int BM, int BN, int CHUNK_K)
{
    const int64_t T = d.T;
    p.n_i = (int)((d.M + T - 1) / T);
    p.n_j = (int)((d.N + T - 1) / T);
    const int64_t n_k = (d.K + T - 1) / T;
    const int64_t last_m = d.M - (int64_t)(p.n_i - 1) * T;
    const int64_t last_n = d.N - (int64_t)(p.n_j - 1) * T;
    const int64_t full_m = p.n_i > 1 ? T : last_m, full_n = p.n_j > 1 ? T : last_n;
    p.tpm = (int)((full_m + BM - 1) / BM);
    p.tpn = (int)((full_n + BN - 1) / BN);
    p.tpm_last = (int)((last_m + BM - 1) / BM);
    p.tpn_last = (int)((last_n + BN - 1) / BN);
    p.macro_cols = (p.n_j - 1) * p.tpn + p.tpn_last;
    const int64_t macro_rows = (int64_t)(p.n_i - 1) * p.tpm + p.tpm_last;
    const int64_t grid = macro_rows * p.macro_cols;
    if (grid <= 0 || grid > 0x7fffffff) return 0;
    const int64_t full_k = n_k > 1 ? T : d.K;
    p.chunks_per_step = (int)((full_k + CHUNK_K - 1) / CHUNK_K);
    const int64_t last_k = d.K - (n_k - 1) * T;
    p.n_chunks = (int)((n_k - 1) * p.chunks_per_step + (last_k + CHUNK_K - 1) / CHUNK_K);
    return grid;
}

// The direct-to-LDS kernel (gemm_bf16_dl.hip): 256 x 256 macro tiles.  It needs 16-byte aligned
// operand rows and whole 32-k chunks; the launcher returns hipErrorNotSupported (and launches
// nothing) when bf16_dl_applicable(d) is false.  d.T must already be clamped to the problem.
bool bf16_dl_applicable(const GemmDesc& d);
hipError_t launch_tile_gemm_bf16_dl(GemmParams p, const GemmDesc& d, hipStream_t stream);

}  // namespace bf
}  // namespace tg
