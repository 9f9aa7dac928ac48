// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "nm.h"

namespace nm {

// One PWL table as the kernels see it.  kb[s] = {k, b} of segment s (device memory).
struct DevTable {
    const float2* kb;
    float lo, hi, inv_w;
    int nseg;
    int clamp_input;
    // two-level form of a merged table (NM_TABLE_COMPACT), null / 0 otherwise: cellmap[cell] is
    // the merged segment of a primary cell, ckb[segment] its {k, b}; nkb segments
    const float2* ckb;
    const uint8_t* cellmap;
    int nkb;
    // a table of two segments (without the clamp flag): its two lines and the smallest fp32 value
    // whose segment index is 1, so that a kernel may pick the line with one compare (two_seg != 0)
    int two_seg;
    float k0, b0, k1, b1, tau;
};

struct HostTable {
    nm_table_desc desc;
    float inv_w;
    int n_distinct;
    std::vector<float> k, b;
    size_t blob_offset;  // in float2 units
    // two-level form (NM_TABLE_COMPACT): one {k, b} per merged segment and a byte per primary cell
    std::vector<float> ck, cb;
    std::vector<uint8_t> cellmap;
    size_t cblob_offset = 0;  // float2 units
    size_t map_offset = 0;    // float2 units (the map's bytes start there)
};

int32_t launch_layernorm2(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const DevTable& t, const DevTable& t2, int two,
                          float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* seg, uint16_t* seg2,
                          hipStream_t stream);

}  // namespace nm

struct nm_tables {
    std::vector<nm::HostTable> tables;
    float2* d_blob = nullptr;
    int device = -1;
};

namespace nm {

void set_error(const char* fmt, ...);
int32_t fail(int32_t code, const char* fmt, ...);
int32_t check_hip(hipError_t e, const char* what);

// Validates idx and fills dt.  Returns NM_OK or an error (message set).
// two_level: also hand out the two-level form of a table built with NM_TABLE_COMPACT (only kernels
// that look tables up in two steps ask for it; everything else works on the expanded form).
int32_t get_dev_table(const nm_tables* t, int32_t idx, DevTable* dt, const char* what, bool two_level = false);

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// ---- generic (possibly batched, strided) GEMM launcher used by the public entry points --------
struct GemmArgs {
    int M = 0, N = 0, K = 0;
    const int8_t* A = nullptr; long lda = 0;
    const int8_t* W = nullptr; long ldw = 0;
    int w_is_kn = 0;  // 0: W is [N, K] (K contiguous); 1: W is [K, N] (N contiguous)
    // batching: grid.y = outer_count * inner_count problems
    int outer_count = 1, inner_count = 1;
    long a_outer = 0, a_inner = 0, w_outer = 0, w_inner = 0, o_outer = 0, o_inner = 0;
    const float* bias = nullptr;
    const float* alpha_vec = nullptr;
    float alpha = 1.0f;
    const int8_t* resid = nullptr;
    float resid_scale = 0.0f;
    int has_table = 0;
    DevTable table{};
    float out_inv_scale = 1.0f;
    const float* out_inv_scale_vec = nullptr;
    int split_cols = 0;  // > 0: out scale of column n is inv3[n / split_cols]
    float inv3[3] = {1.0f, 1.0f, 1.0f};
    long ldo = 0;  // row stride of resid and of every output
    int8_t* out_q = nullptr;
    float* out_f32 = nullptr;
    int32_t* out_acc = nullptr;
    uint16_t* dbg_seg = nullptr;
    // LayerNorm-PWL of the fp32 result, folded into the kernel when the shape allows it (else the
    // caller runs the row kernel): gamma / beta [N], rsqrt table, int8 and / or fp32 output [M, N]
    int ln = 0;
    const float* ln_gamma = nullptr;
    const float* ln_beta = nullptr;
    float ln_eps = 0.0f, ln_inv_scale = 1.0f;
    DevTable ln_table{};
    int8_t* ln_out_q = nullptr;
    float* ln_out_f32 = nullptr;
    // conv != 0: A is an NHWC image [B, cH, cW, cCin] and row m = (b, ho, wo) of the matrix is
    // gathered from it (K = kh * cKw * cCin, tap major); M = B * cHo * cWo
    int conv = 0;
    int cH = 0, cW = 0, cCin = 0, cKw = 0, cStride = 1, cPad = 0, cHo = 0, cWo = 0;
};

int32_t launch_gemm(const GemmArgs& g, hipStream_t stream);
// True when launch_gemm would fold the LayerNorm described by g.ln_* into the GEMM kernel.
bool gemm_folds_layernorm(const GemmArgs& g);

int32_t launch_softmax(const void* in, int32_t in_dtype, float alpha, int64_t rows, int32_t cols,
                       const DevTable& t_exp, const DevTable& t_recip, float out_inv_scale,
                       int8_t* out_q, float* out_f32, uint16_t* seg_exp, uint16_t* seg_recip,
                       hipStream_t stream);

int32_t launch_layernorm(const float* in, const float* gamma, const float* beta, float eps,
                         int64_t rows, int32_t cols, const DevTable& t, float out_inv_scale,
                         int8_t* out_q, float* out_f32, uint16_t* seg, hipStream_t stream);

int32_t launch_layernorm2(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const DevTable& t, const DevTable& t2, int two,
                          float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* seg, uint16_t* seg2,
                          hipStream_t stream);

}  // namespace nm
