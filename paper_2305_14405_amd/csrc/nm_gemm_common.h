// Declarations shared by the GEMM kernels of this library (device code; included by nm_gemm.hip).
#pragma once

#include <mutex>
#include <type_traits>

#include "nm_device.h"

namespace nm {

constexpr int kGemmThreads = 256;
constexpr int kBK = 64;  // bytes of k per pipeline stage

struct GemmParams {
    int M, N, K;
    const int8_t* A; long lda;
    const int8_t* W; long ldw;
    int inner_count;
    long a_outer, a_inner, w_outer, w_inner, o_outer, o_inner;
    const float* bias;
    const float* alpha_vec;
    float alpha;
    const int8_t* resid;
    float resid_scale;
    int has_table;
    DevTable table;
    float out_inv_scale;
    const float* out_inv_scale_vec;
    int split_cols;
    float inv3[3];
    long ldo;
    int vec_out;
    int q16;       // int8 output rows may be written with 16-byte stores
    int r16;       // int8 residual rows may be read with 16-byte loads (and N % 16 == 0)
    int vec_cols;  // bias / per-column scale vectors may be read with 16-byte loads
    int8_t* out_q;
    float* out_f32;
    int32_t* out_acc;
    uint16_t* dbg_seg;
    int tiles_m, tiles_n;
    int group_m;  // tile kernel: tile rows per group of the XCD-aware tile order
    // LayerNorm-PWL folded into the epilogue (EPI_F32_RESID_LN): y = fma(d * r, gamma, beta) with
    // r = PWL_rsqrt(var + eps); outputs its int8 code and / or fp32 value, row stride N
    const float* ln_gamma;
    const float* ln_beta;
    float ln_eps, ln_inv_scale;
    DevTable ln_table;
    int8_t* ln_out_q;
    float* ln_out_f32;
    // convolution in matrix form (streaming kernel with kConv): row m of A is the output position
    // (b, ho, wo), column k the (tap, channel) pair; A points to the NHWC image tensor
    int cH, cW, cCin, cKw, cStride, cPad, cHo, cWo;
};

// XOR swizzle of the 16-byte chunk index inside a 64-byte LDS row: rows that fall into the same
// bank window get different chunk positions, for both a 128-byte and a 256-byte wide LDS port.
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 2) & 3); }

__device__ __forceinline__ int lds_off(int row, int chunk) { return row * kBK + ((chunk ^ swz(row)) << 4); }


enum { EPI_GENERIC = 0, EPI_Q = 1, EPI_Q_TABLE = 2, EPI_F32_RESID = 3, EPI_ACC = 4, EPI_Q_TABLE_RESID = 5, EPI_F32_RESID_LN = 6, EPI_Q_TABLE2 = 7 };
// EPI_Q_TABLE2: EPI_Q_TABLE for a merged table in its two-level form (one byte per primary cell naming the
// merged segment, one {k, b} per merged segment; tile kernel only).
// EPI_F32_RESID_LN: EPI_F32_RESID followed by LayerNorm-PWL over the row, inside the kernel: the tile
// covers whole rows (tile kernel only).
// EPI_Q_TABLE_RESID: int8 residual, table (no input clamp), int8 output: the last convolution of a
// residual block (sum with the shortcut, ReLU).


template <int BK>
__device__ __forceinline__ int swz_bk(int row)
{
    return BK == 64 ? swz(row) : ((row >> 1) & 7);
}
template <int BK>
__device__ __forceinline__ int lds_off_bk(int row, int chunk)
{
    return row * BK + ((chunk ^ swz_bk<BK>(row)) << 4);
}

}  // namespace nm
