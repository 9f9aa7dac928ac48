// int8 convolution as a matrix product (paper Section 3.1: the matrix dimensions follow from the
// width, height and channel counts of the convolution), with the fused PWL epilogue of the GEMM,
// and the two pooling operators of a residual CNN.
//
// Three routes, chosen on the host:
//  * 1x1, stride 1, no padding: the NHWC activation tensor already IS the [B*H*W, Cin] matrix;
//  * Cin a multiple of 64 (every convolution of a ResNet-50 body): the streaming GEMM kernel
//    gathers the rows of the patch matrix straight from the image while loading its A operand
//    (no patch matrix in memory);
//  * anything else (the 3-channel stem, odd channel counts): a small kernel writes the patch
//    matrix [B*Ho*Wo, K16] (K rounded up to 16, zero filled) into the caller's workspace and the
//    GEMM runs on it.
#include "nm_device.h"

namespace nm {

constexpr int kConvThreads = 256;

// Patch matrix: row m = (b, ho, wo), column k = (tap i, tap j, channel c), zeros in the padding
// and in the columns K .. K16-1.  One thread writes 16 consecutive columns of one row.
__global__ __launch_bounds__(kConvThreads) void im2col_kernel(
    const int8_t* __restrict__ x, int H, int W, int Cin, int kw, int stride, int pad, int Ho, int Wo,
    int K, int K16, long rows, int8_t* __restrict__ out)
{
    const int chunks = K16 / 16;
    const long total = rows * chunks;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const long m = idx / chunks;
        const int k0 = (int)(idx % chunks) * 16;
        const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho);
        const long b = m / ((long)Wo * Ho);
        unsigned word[4] = {0, 0, 0, 0};
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            const int k = k0 + e;
            int v = 0;
            if (k < K) {
                const int c = k % Cin, tap = k / Cin;
                const int hi = ho * stride - pad + tap / kw, wi = wo * stride - pad + tap % kw;
                if ((unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W)
                    v = x[((b * H + hi) * W + wi) * Cin + c];
            }
            word[e >> 2] |= (unsigned)(v & 0xff) << (8 * (e & 3));
        }
        *reinterpret_cast<v4i*>(out + m * K16 + k0) = v4i{(int)word[0], (int)word[1], (int)word[2], (int)word[3]};
    }
}

// Max pooling on int8 codes (exact, order-free); padding never takes part.  One thread per
// output position and group of four channels (C % 4 == 0) or per single channel.
template <bool kVec>
__global__ __launch_bounds__(kConvThreads) void maxpool_kernel(
    const int8_t* __restrict__ x, int H, int W, int C, int k, int stride, int pad, int Ho, int Wo,
    long total, int8_t* __restrict__ y)
{
    const int cg = kVec ? C / 4 : C;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int c = (int)(idx % cg);
        const long m = idx / cg;
        const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho);
        const long b = m / ((long)Wo * Ho);
        int best[4] = {-128, -128, -128, -128};
        for (int i = 0; i < k; ++i) {
            const int hi = ho * stride - pad + i;
            if ((unsigned)hi >= (unsigned)H) continue;
            for (int j = 0; j < k; ++j) {
                const int wi = wo * stride - pad + j;
                if ((unsigned)wi >= (unsigned)W) continue;
                const long off = ((b * H + hi) * W + wi) * C;
                if (kVec) {
                    const unsigned w = *reinterpret_cast<const unsigned*>(x + off + 4 * c);
#pragma unroll
                    for (int e = 0; e < 4; ++e) best[e] = max(best[e], (int)(int8_t)(w >> (8 * e)));
                } else {
                    best[0] = max(best[0], (int)x[off + c]);
                }
            }
        }
        if (kVec) *reinterpret_cast<unsigned*>(y + m * C + 4 * c) = pack4(best[0], best[1], best[2], best[3]);
        else y[m * C + c] = (int8_t)best[0];
    }
}

// Global average pooling: exact int32 sum over the positions, one fp32 multiply, requantise.
__global__ __launch_bounds__(kConvThreads) void avgpool_kernel(
    const int8_t* __restrict__ x, int B, int HW, int C, float alpha, float out_inv_scale,
    int8_t* __restrict__ out_q, float* __restrict__ out_f32)
{
    const long total = (long)B * C;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int c = (int)(idx % C);
        const long b = idx / C;
        int acc = 0;
        for (int p = 0; p < HW; ++p) acc += (int)x[(b * HW + p) * C + c];
        const float v = (float)acc * alpha;
        if (out_f32) out_f32[idx] = v;
        if (out_q) out_q[idx] = (int8_t)requant(v, out_inv_scale);
    }
}

static int grid_for(long units)
{
    long b = (units + kConvThreads - 1) / kConvThreads;
    if (b > 256L * 32) b = 256L * 32;
    return (int)(b < 1 ? 1 : b);
}

struct ConvPlan {
    int Ho, Wo, K, K16;
    long M;
    int route;  // 0: plain matrix, 1: gathered operand, 2: patch matrix in the workspace
    size_t ws_bytes;
};

static int32_t plan_conv(const nm_conv_desc* d, const char* what, ConvPlan* pl)
{
    if (!d) return fail(NM_ERR_INVALID_ARG, "%s: desc is NULL", what);
    if (d->B < 0 || d->H < 1 || d->W < 1 || d->Cin < 1 || d->Cout < 1 || d->kh < 1 || d->kw < 1 ||
        d->stride < 1 || d->pad < 0)
        return fail(NM_ERR_INVALID_ARG, "%s: bad convolution geometry", what);
    if (d->H + 2 * d->pad < d->kh || d->W + 2 * d->pad < d->kw)
        return fail(NM_ERR_INVALID_ARG, "%s: filter larger than the padded image", what);
    pl->Ho = (d->H + 2 * d->pad - d->kh) / d->stride + 1;
    pl->Wo = (d->W + 2 * d->pad - d->kw) / d->stride + 1;
    const int64_t K = (int64_t)d->kh * d->kw * d->Cin;
    const int64_t M = (int64_t)d->B * pl->Ho * pl->Wo;
    if (K > 65536) return fail(NM_ERR_UNSUPPORTED, "%s: kh*kw*Cin %lld > 65536", what, (long long)K);
    if (M * d->Cout >= (1LL << 31) || M * K >= (1LL << 40) || (int64_t)d->B * d->H * d->W * d->Cin >= (1LL << 40))
        return fail(NM_ERR_UNSUPPORTED, "%s: tensor too large", what);
    if (M >= (1LL << 31)) return fail(NM_ERR_UNSUPPORTED, "%s: more than 2^31 output positions", what);
    pl->K = (int)K;
    pl->K16 = (int)((K + 15) / 16 * 16);
    pl->M = (long)M;
    const bool plain = d->kh == 1 && d->kw == 1 && d->stride == 1 && d->pad == 0;
    const bool gather = d->Cin % 64 == 0 && aligned(d->x, 16) && aligned(d->w, 16);
    pl->route = plain ? 0 : gather ? 1 : 2;
    pl->ws_bytes = pl->route == 2 ? (size_t)M * pl->K16 + (size_t)d->Cout * pl->K16 : 0;
    return NM_OK;
}

// Copies the [Cout, K] filter matrix into rows of K16 bytes (zero tail) for the patch-matrix route.
__global__ __launch_bounds__(kConvThreads) void pad_rows_kernel(const int8_t* __restrict__ w, int rows, int K,
                                                                 int K16, int8_t* __restrict__ out)
{
    const long total = (long)rows * K16;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int k = (int)(idx % K16);
        out[idx] = k < K ? w[(idx / K16) * K + k] : (int8_t)0;
    }
}

}  // namespace nm

using namespace nm;

extern "C" {

int32_t nm_conv2d_workspace(const nm_conv_desc* d, size_t* bytes)
{
    ConvPlan pl;
    int32_t rc = plan_conv(d, "nm_conv2d_workspace", &pl);
    if (rc) return rc;
    if (!bytes) return fail(NM_ERR_INVALID_ARG, "nm_conv2d_workspace: bytes is NULL");
    *bytes = pl.ws_bytes;
    return NM_OK;
}

int32_t nm_conv2d_pwl(const nm_conv_desc* d, void* ws, size_t ws_bytes, void* stream_)
{
    ConvPlan pl;
    int32_t rc = plan_conv(d, "nm_conv2d_pwl", &pl);
    if (rc) return rc;
    if (!d->out_q && !d->out_f32 && !d->dbg_acc) return fail(NM_ERR_INVALID_ARG, "nm_conv2d_pwl: no output");
    GemmArgs g;
    if (d->table_idx >= 0) {
        rc = get_dev_table(d->tables, d->table_idx, &g.table, "nm_conv2d_pwl");
        if (rc) return rc;
        g.has_table = 1;
    }
    if (pl.M == 0) return NM_OK;  // an empty batch may come with NULL pointers
    if (!d->x || !d->w) return fail(NM_ERR_INVALID_ARG, "nm_conv2d_pwl: x or w is NULL");
    hipStream_t stream = (hipStream_t)stream_;
    g.M = (int)pl.M; g.N = d->Cout; g.K = pl.K;
    g.W = d->w; g.ldw = pl.K;
    g.bias = d->bias; g.alpha_vec = d->alpha_vec; g.alpha = d->alpha;
    g.resid = d->resid; g.resid_scale = d->resid_scale;
    g.out_inv_scale = d->out_inv_scale;
    g.ldo = d->Cout;
    g.out_q = d->out_q; g.out_f32 = d->out_f32; g.out_acc = d->dbg_acc;
    if (pl.route == 0) {
        g.A = d->x; g.lda = d->Cin;
    } else if (pl.route == 1) {
        g.A = d->x; g.lda = d->Cin;
        g.conv = 1;
        g.cH = d->H; g.cW = d->W; g.cCin = d->Cin; g.cKw = d->kw; g.cStride = d->stride; g.cPad = d->pad;
        g.cHo = pl.Ho; g.cWo = pl.Wo;
    } else {
        if (!ws) return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace is NULL");
        if (!aligned(ws, 256)) return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace not 256-byte aligned");
        if (ws_bytes < pl.ws_bytes)
            return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace %zu bytes < %zu needed", ws_bytes, pl.ws_bytes);
        int8_t* patches = static_cast<int8_t*>(ws);
        int8_t* wpad = patches + (size_t)pl.M * pl.K16;
        hipLaunchKernelGGL(im2col_kernel, dim3(grid_for(pl.M * (pl.K16 / 16))), dim3(kConvThreads), 0, stream,
                           d->x, d->H, d->W, d->Cin, d->kw, d->stride, d->pad, pl.Ho, pl.Wo, pl.K, pl.K16, pl.M,
                           patches);
        hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for((long)d->Cout * pl.K16)), dim3(kConvThreads), 0, stream,
                           d->w, d->Cout, pl.K, pl.K16, wpad);
        if ((rc = check_hip(hipGetLastError(), "nm_conv2d_pwl patch matrix launch"))) return rc;
        g.A = patches; g.lda = pl.K16;
        g.W = wpad; g.ldw = pl.K16;
        g.K = pl.K16;
    }
    return launch_gemm(g, stream);
}

int32_t nm_maxpool_i8(const int8_t* x, int32_t B, int32_t H, int32_t W, int32_t C, int32_t k,
                      int32_t stride, int32_t pad, int8_t* y, void* stream)
{
    if (B < 0 || H < 1 || W < 1 || C < 1 || k < 1 || stride < 1 || pad < 0 || pad >= k)
        return fail(NM_ERR_INVALID_ARG, "nm_maxpool_i8: bad geometry");
    if (H + 2 * pad < k || W + 2 * pad < k) return fail(NM_ERR_INVALID_ARG, "nm_maxpool_i8: window larger than the padded image");
    const int Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
    const int64_t rows = (int64_t)B * Ho * Wo;
    if (rows * C >= (1LL << 40) || (int64_t)B * H * W * C >= (1LL << 40))
        return fail(NM_ERR_UNSUPPORTED, "nm_maxpool_i8: tensor too large");
    if (rows == 0) return NM_OK;
    if (!x || !y) return fail(NM_ERR_INVALID_ARG, "nm_maxpool_i8: NULL pointer");
    const bool vec = C % 4 == 0 && aligned(x, 4) && aligned(y, 4);
    const long total = rows * (vec ? C / 4 : C);
    if (vec) hipLaunchKernelGGL(maxpool_kernel<true>, dim3(grid_for(total)), dim3(kConvThreads), 0, (hipStream_t)stream,
                                x, H, W, C, k, stride, pad, Ho, Wo, total, y);
    else hipLaunchKernelGGL(maxpool_kernel<false>, dim3(grid_for(total)), dim3(kConvThreads), 0, (hipStream_t)stream,
                            x, H, W, C, k, stride, pad, Ho, Wo, total, y);
    return check_hip(hipGetLastError(), "nm_maxpool_i8 launch");
}

int32_t nm_avgpool_i8(const int8_t* x, int32_t B, int32_t HW, int32_t C, float alpha, float out_inv_scale,
                      int8_t* out_q, float* out_f32, void* stream)
{
    if (B < 0 || HW < 1 || C < 1) return fail(NM_ERR_INVALID_ARG, "nm_avgpool_i8: bad shape");
    if (HW > (1 << 23)) return fail(NM_ERR_UNSUPPORTED, "nm_avgpool_i8: more than 2^23 positions (int32 sum)");
    if (!out_q && !out_f32) return fail(NM_ERR_INVALID_ARG, "nm_avgpool_i8: no output");
    if (B == 0) return NM_OK;
    if (!x) return fail(NM_ERR_INVALID_ARG, "nm_avgpool_i8: x is NULL");
    hipLaunchKernelGGL(avgpool_kernel, dim3(grid_for((long)B * C)), dim3(kConvThreads), 0, (hipStream_t)stream,
                       x, B, HW, C, alpha, out_inv_scale, out_q, out_f32);
    return check_hip(hipGetLastError(), "nm_avgpool_i8 launch");
}

}  // extern "C"
