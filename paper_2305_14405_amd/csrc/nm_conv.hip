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
//    matrix [B*Ho*Wo, K16] (K rounded up to 64, zero filled) into the caller's workspace and the
//    GEMM runs on it.
#include <type_traits>

#include "nm_device.h"

namespace nm {

constexpr int kConvThreads = 256;

// Patch matrix: row m = (b, ho, wo), column k = (tap i, tap j, channel c), zeros in the padding
// and in the columns K .. K16-1 (K16: K rounded up to 64).  One thread writes 16 consecutive
// columns of one row.
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
        // (tap row, tap column, channel) of column k0, then stepped along the 16 columns
        int c = k0 % Cin, tap = k0 / Cin;
        int ti = tap / kw, tj = tap % kw;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            int v = 0;
            if (k0 + e < K) {
                const int hi = ho * stride - pad + ti, wi = wo * stride - pad + tj;
                if ((unsigned)hi < (unsigned)H && (unsigned)wi < (unsigned)W)
                    v = x[((b * H + hi) * W + wi) * Cin + c];
            }
            word[e >> 2] |= (unsigned)(v & 0xff) << (8 * (e & 3));
            if (++c == Cin) { c = 0; if (++tj == kw) { tj = 0; ++ti; } }
        }
        *reinterpret_cast<v4i*>(out + m * K16 + k0) = v4i{(int)word[0], (int)word[1], (int)word[2], (int)word[3]};
    }
}

// Max pooling on int8 codes (exact, order-free); padding never takes part.  One thread per
// output position and 16 channels (C % 16 == 0, 16-byte loads).
__global__ __launch_bounds__(kConvThreads) void maxpool16_kernel(
    const int8_t* __restrict__ x, int H, int W, int C, int k, int stride, int pad, int Ho, int Wo,
    long total, int8_t* __restrict__ y)
{
    const int cg = C / 16;
    for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
        const int c = (int)(idx % cg);
        const long m = idx / cg;
        const int wo = (int)(m % Wo), ho = (int)((m / Wo) % Ho);
        const long b = m / ((long)Wo * Ho);
        int best[16];
#pragma unroll
        for (int e = 0; e < 16; ++e) best[e] = -128;
        for (int i = 0; i < k; ++i) {
            const int hi = ho * stride - pad + i;
            if ((unsigned)hi >= (unsigned)H) continue;
            for (int j = 0; j < k; ++j) {
                const int wi = wo * stride - pad + j;
                if ((unsigned)wi >= (unsigned)W) continue;
                const v4i w4 = *reinterpret_cast<const v4i*>(x + ((b * H + hi) * W + wi) * C + 16 * c);
#pragma unroll
                for (int e = 0; e < 16; ++e) best[e] = max(best[e], (int)(int8_t)((unsigned)w4[e >> 2] >> (8 * (e & 3))));
            }
        }
        v4i o;
#pragma unroll
        for (int q = 0; q < 4; ++q) o[q] = (int)pack4(best[4 * q], best[4 * q + 1], best[4 * q + 2], best[4 * q + 3]);
        *reinterpret_cast<v4i*>(y + m * C + 16 * c) = o;
    }
}

// The same with four channels (C % 4 == 0) or one channel per thread.
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
// kVec (C a multiple of 4, 4-byte aligned tensors): a thread owns four neighbouring channels of an
// image and reads them as one word per position, eight positions in flight; otherwise one channel
// per thread, byte by byte.
template <bool kVec>
__global__ __launch_bounds__(kConvThreads) void avgpool_kernel(
    const int8_t* __restrict__ x, int B, int HW, int C, float alpha, float out_inv_scale,
    int8_t* __restrict__ out_q, float* __restrict__ out_f32)
{
    if (kVec) {
        const int C4 = C / 4;
        const long total = (long)B * C4;
        for (long idx = (long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (long)gridDim.x * blockDim.x) {
            const int c4 = (int)(idx % C4);
            const long b = idx / C4;
            const int8_t* src = x + b * HW * (long)C + 4 * c4;
            int acc[4] = {0, 0, 0, 0};
            int p = 0;
            for (; p + 8 <= HW; p += 8) {
                int w[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) w[u] = *reinterpret_cast<const int*>(src + (long)(p + u) * C);
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc[e] += (int)(int8_t)(w[u] >> (8 * e));
            }
            for (; p < HW; ++p) {
                const int w = *reinterpret_cast<const int*>(src + (long)p * C);
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] += (int)(int8_t)(w >> (8 * e));
            }
            float v[4];
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v[e] = (float)acc[e] * alpha;
                q[e] = requant(v[e], out_inv_scale);
            }
            if (out_f32) *reinterpret_cast<v4f*>(out_f32 + 4 * idx) = v4f{v[0], v[1], v[2], v[3]};
            if (out_q) *reinterpret_cast<unsigned*>(out_q + 4 * idx) = pack4(q[0], q[1], q[2], q[3]);
        }
        return;
    }
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

// ---------------------------------------------------------------------------------------------
// Direct convolution for images with at most four channels (the stem of a CNN: 7x7, stride 2,
// three channels).  A patch matrix would be 50 times the image; instead a workgroup stages the
// part of the image its 16 x 16 output positions need in LDS, one 4-byte pixel per position
// (missing channels and everything outside the image are zero), and the filter as rows of 32
// bytes per filter row (kw <= 8 pixels of 4 bytes, zero filled).  One MFMA k-step is then one
// filter row: the operand bytes of output position (ho, wo) are 32 consecutive LDS bytes starting
// at pixel (ho*stride + i, wo*stride); bytes beyond the kw-th pixel meet zero filter bytes.
// Accumulators and epilogue arithmetic are those of the matrix product (exact integers, the same
// fp32 operations), so the result is bit-identical to the other routes.
// A wavefront owns 4 rows x 16 columns of positions and all (up to 64) output channels.
// ---------------------------------------------------------------------------------------------
struct StemParams {
    const int8_t* x; const int8_t* w;   // w: the packed filter [64][kh][32] (stem_pack_filter_kernel)
    const float* bias; const float* alpha_vec;
    float alpha, out_inv_scale;
    int has_table;
    DevTable table;
    int B, H, W, Cin, Cout, kh, kw, stride, pad, Ho, Wo;
    int prow, pcol, pitch;   // staged image patch: rows, pixels per row, bytes per row
    int8_t* out_q;
};

// Packs the filter [Cout][kh][kw][Cin] into [64][kh][8 pixels of 4 bytes] (zero filled), once per
// call, so that every workgroup of the convolution copies it with wide loads.
__global__ __launch_bounds__(256) void stem_pack_filter_kernel(const int8_t* __restrict__ w, int Cout, int kh,
                                                               int kw, int Cin, int8_t* __restrict__ out)
{
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < 64 * kh * 8; idx += gridDim.x * blockDim.x) {
        const int j = idx % 8, i = (idx / 8) % kh, n = idx / (8 * kh);
        unsigned px = 0;
        if (n < Cout && j < kw) {
            const int8_t* src = w + (((long)n * kh + i) * kw + j) * Cin;
            for (int ch = 0; ch < Cin; ++ch) px |= (unsigned)(uint8_t)src[ch] << (8 * ch);
        }
        *reinterpret_cast<unsigned*>(out + (n * kh + i) * 32 + 4 * j) = px;
    }
}

__global__ __launch_bounds__(256) void stem_conv_kernel(StemParams p)
{
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t* sX = smem;                                   // [prow][pitch]
    int8_t* sW = smem + p.prow * p.pitch;                // [64][kh][32]
    int8_t* sO = sW + 64 * p.kh * 32;                    // [4 wavefronts][64 positions][80]
    float* s_cols = reinterpret_cast<float*>(sO + 4 * 64 * 80);   // scale | bias, 64 each
    float2* s_kb = reinterpret_cast<float2*>(s_cols + 128);

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int tiles_w = (p.Wo + 15) / 16;
    const int ho0 = (blockIdx.x / tiles_w) * 16, wo0 = (blockIdx.x % tiles_w) * 16;
    const long b = blockIdx.y;
    const int hi0 = ho0 * p.stride - p.pad, wi0 = wo0 * p.stride - p.pad;

    if (p.has_table) stage_table(s_kb, p.table);
    if (tid < 64) {
        s_cols[tid] = tid < p.Cout ? (p.alpha_vec ? p.alpha_vec[tid] : p.alpha) : 0.0f;
        s_cols[64 + tid] = (tid < p.Cout && p.bias) ? p.bias[tid] : 0.0f;
    }
    // image patch: one dword per pixel
    for (int idx = tid; idx < p.prow * p.pcol; idx += 256) {
        const int r = idx / p.pcol, c = idx % p.pcol;
        const int hi = hi0 + r, wi = wi0 + c;
        unsigned px = 0;
        if ((unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W) {
            const int8_t* src = p.x + ((b * p.H + hi) * p.W + wi) * p.Cin;
            for (int ch = 0; ch < p.Cin; ++ch) px |= (unsigned)(uint8_t)src[ch] << (8 * ch);
        }
        *reinterpret_cast<unsigned*>(sX + r * p.pitch + 4 * c) = px;
    }
    // zero the slack at the end of every patch row (read by the last positions' 32-byte windows)
    for (int idx = tid; idx < p.prow * ((p.pitch - 4 * p.pcol) / 4); idx += 256) {
        const int per = (p.pitch - 4 * p.pcol) / 4;
        *reinterpret_cast<unsigned*>(sX + (idx / per) * p.pitch + 4 * p.pcol + 4 * (idx % per)) = 0u;
    }
    // filter, already packed as [n][i][8 pixels of 4 bytes]: straight 16-byte copies
    for (int idx = tid; idx < 64 * p.kh * 2; idx += 256)
        *reinterpret_cast<v4i*>(sW + 16 * idx) = *reinterpret_cast<const v4i*>(p.w + 16 * idx);
    __syncthreads();

    // lane (m, half): position m of a 32-position block; block t covers wavefront rows 2t, 2t+1
    const int fr = lane & 31, half = lane >> 5;
    v16i acc[2][2];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[t][j][v] = 0;
    int offA[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        const int pr = wave * 4 + 2 * t + (fr >> 4), pc = fr & 15;   // position inside the 16 x 16 tile
        offA[t] = pr * p.stride * p.pitch + pc * p.stride * 4 + 16 * half;
    }
    for (int i = 0; i < p.kh; ++i) {
        v4i fa[2], fw[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int8_t* a = sX + offA[t] + i * p.pitch;   // 4-byte aligned
            const unsigned* a4 = reinterpret_cast<const unsigned*>(a);
            fa[t] = v4i{(int)a4[0], (int)a4[1], (int)a4[2], (int)a4[3]};
        }
#pragma unroll
        for (int j = 0; j < 2; ++j)
            fw[j] = *reinterpret_cast<const v4i*>(sW + ((32 * j + fr) * p.kh + i) * 32 + 16 * half);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j)
                acc[t][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fa[t], acc[t][j], 0, 0, 0);
    }

    // epilogue: lane (m, half) holds, per group g of four registers, channels 32j + 8g + 4half .. +3
    int8_t* patch = sO + wave * (64 * 80);
    // (twice: a table of two segments, ReLU, is evaluated with a compare instead of index and gather)
    auto finish = [&](auto two_c) {
        constexpr bool kTwoSeg = decltype(two_c)::value;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = 32 * j + 8 * g + 4 * half;
                    const v4f sc = *reinterpret_cast<const v4f*>(s_cols + n);
                    const v4f bi = *reinterpret_cast<const v4f*>(s_cols + 64 + n);
                    int q[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        float v = __builtin_fmaf((float)acc[t][j][4 * g + e], sc[e], bi[e]);
                        if (kTwoSeg) v = pwl_eval_two_segments(v, p.table);
                        else if (p.has_table) { int sg; v = pwl_eval(v, p.table, s_kb, sg); }
                        q[e] = requant(v, p.out_inv_scale);
                    }
                    *reinterpret_cast<unsigned*>(patch + (32 * t + fr) * 80 + n) = pack4(q[0], q[1], q[2], q[3]);
                }
    };
    if (p.has_table && p.table.two_seg) finish(std::true_type{});
    else finish(std::false_type{});
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // 16-byte stores: position rows of Cout bytes are contiguous along wo
    const int chunks = p.Cout / 16;
    for (int c = lane; c < 64 * chunks; c += 64) {
        const int pos = c / chunks, cc = c % chunks;
        const int ho = ho0 + wave * 4 + (pos >> 4), wo = wo0 + (pos & 15);
        if (ho < p.Ho && wo < p.Wo)
            *reinterpret_cast<v4i*>(p.out_q + ((b * p.Ho + ho) * p.Wo + wo) * p.Cout + 16 * cc) =
                *reinterpret_cast<const v4i*>(patch + pos * 80 + 16 * cc);
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
    int route;  // 0: plain matrix, 1: gathered operand, 2: patch matrix in the workspace, 3: direct (few channels)
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
    pl->K16 = (int)((K + 63) / 64 * 64);  // whole 64-byte k-slices: the streaming GEMM runs on the patch matrix
    pl->M = (long)M;
    const bool plain = d->kh == 1 && d->kw == 1 && d->stride == 1 && d->pad == 0;
    const bool gather = d->Cin % 64 == 0 && aligned(d->x, 16) && aligned(d->w, 16) &&
                        (int64_t)d->H * d->W * d->Cin < (1LL << 31);   // 32-bit offsets inside one image
    // direct kernel: few input channels, a filter row fits 32 bytes, int8 output only
    const bool direct = !plain && d->Cin <= 4 && d->kw <= 8 && d->Cout <= 64 && d->Cout % 16 == 0 && d->out_q &&
                        !d->out_f32 && !d->dbg_acc && !d->resid && aligned(d->out_q, 16) &&
                        15 * d->stride + d->kh <= 64 && d->B <= 65535;
    pl->route = plain ? 0 : gather ? 1 : direct ? 3 : 2;
    pl->ws_bytes = pl->route == 2 ? (size_t)M * pl->K16 + (size_t)d->Cout * pl->K16
                 : pl->route == 3 ? (size_t)64 * d->kh * 32 : 0;   // patch matrix + filter rows | packed filter
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
    if (pl.route == 3) {
        if (!ws) return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace is NULL");
        if (!aligned(ws, 256)) return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace not 256-byte aligned");
        if (ws_bytes < pl.ws_bytes)
            return fail(NM_ERR_WORKSPACE, "nm_conv2d_pwl: workspace %zu bytes < %zu needed", ws_bytes, pl.ws_bytes);
        hipLaunchKernelGGL(stem_pack_filter_kernel, dim3((64 * d->kh * 8 + 255) / 256), dim3(256), 0, stream, d->w,
                           d->Cout, d->kh, d->kw, d->Cin, static_cast<int8_t*>(ws));
        StemParams sp{};
        sp.x = d->x; sp.w = static_cast<const int8_t*>(ws); sp.bias = d->bias; sp.alpha_vec = d->alpha_vec; sp.alpha = d->alpha;
        sp.out_inv_scale = d->out_inv_scale; sp.has_table = g.has_table; sp.table = g.table;
        sp.B = d->B; sp.H = d->H; sp.W = d->W; sp.Cin = d->Cin; sp.Cout = d->Cout; sp.kh = d->kh; sp.kw = d->kw;
        sp.stride = d->stride; sp.pad = d->pad; sp.Ho = pl.Ho; sp.Wo = pl.Wo;
        sp.prow = 15 * d->stride + d->kh;
        sp.pcol = 15 * d->stride + d->kw;
        // a position's window is 32 bytes from its first pixel: the last position's reaches 8 pixels
        sp.pitch = ((15 * d->stride + 8) * 4 + 15) / 16 * 16;
        if (sp.pitch < 4 * sp.pcol) sp.pitch = (4 * sp.pcol + 15) / 16 * 16;
        sp.out_q = d->out_q;
        const size_t shmem = (size_t)sp.prow * sp.pitch + 64 * (size_t)d->kh * 32 + 4 * 64 * 80 + 128 * sizeof(float) +
                             (g.has_table ? sizeof(float2) * (size_t)g.table.nseg : 0);
        if (shmem > 64 * 1024) return fail(NM_ERR_UNSUPPORTED, "nm_conv2d_pwl: direct route needs %zu bytes of LDS", shmem);
        const dim3 grid(((pl.Ho + 15) / 16) * ((pl.Wo + 15) / 16), d->B);
        hipLaunchKernelGGL(stem_conv_kernel, grid, dim3(256), shmem, stream, sp);
        return check_hip(hipGetLastError(), "nm_conv2d_pwl direct launch");
    }
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
    if (C % 16 == 0 && aligned(x, 16) && aligned(y, 16)) {
        const long total16 = rows * (C / 16);
        hipLaunchKernelGGL(maxpool16_kernel, dim3(grid_for(total16)), dim3(kConvThreads), 0, (hipStream_t)stream,
                           x, H, W, C, k, stride, pad, Ho, Wo, total16, y);
        return check_hip(hipGetLastError(), "nm_maxpool_i8 launch");
    }
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
    const bool vec = C % 4 == 0 && aligned(x, 4) && (!out_q || aligned(out_q, 4)) && (!out_f32 || aligned(out_f32, 16));
    if (vec)
        hipLaunchKernelGGL(avgpool_kernel<true>, dim3(grid_for((long)B * (C / 4))), dim3(kConvThreads), 0,
                           (hipStream_t)stream, x, B, HW, C, alpha, out_inv_scale, out_q, out_f32);
    else
        hipLaunchKernelGGL(avgpool_kernel<false>, dim3(grid_for((long)B * C)), dim3(kConvThreads), 0,
                           (hipStream_t)stream, x, B, HW, C, alpha, out_inv_scale, out_q, out_f32);
    return check_hip(hipGetLastError(), "nm_avgpool_i8 launch");
}

int32_t nm_cnn_workspace(const nm_cnn_op* ops, int32_t n_ops, size_t* bytes)
{
    if (!ops || n_ops < 1) return fail(NM_ERR_INVALID_ARG, "nm_cnn_workspace: no steps");
    if (!bytes) return fail(NM_ERR_INVALID_ARG, "nm_cnn_workspace: bytes is NULL");
    size_t need = 0;
    for (int32_t i = 0; i < n_ops; ++i) {
        if (ops[i].kind == NM_OP_CONV) {
            size_t b = 0;
            int32_t rc = nm_conv2d_workspace(&ops[i].conv, &b);
            if (rc) return rc;
            if (b > need) need = b;
        } else if (ops[i].kind < NM_OP_CONV || ops[i].kind > NM_OP_GEMM) {
            return fail(NM_ERR_INVALID_ARG, "nm_cnn_workspace: step %d has unknown kind %d", i, ops[i].kind);
        }
    }
    *bytes = need;
    return NM_OK;
}

int32_t nm_cnn_run(const nm_cnn_op* ops, int32_t n_ops, void* ws, size_t ws_bytes, void* stream)
{
    if (!ops || n_ops < 1) return fail(NM_ERR_INVALID_ARG, "nm_cnn_run: no steps");
    for (int32_t i = 0; i < n_ops; ++i) {
        const nm_cnn_op& o = ops[i];
        int32_t rc;
        switch (o.kind) {
        case NM_OP_CONV: rc = nm_conv2d_pwl(&o.conv, ws, ws_bytes, stream); break;
        case NM_OP_MAXPOOL: rc = nm_maxpool_i8(o.x, o.B, o.H, o.W, o.C, o.k, o.stride, o.pad, o.y, stream); break;
        case NM_OP_AVGPOOL: rc = nm_avgpool_i8(o.x, o.B, o.H, o.C, o.alpha, o.out_inv_scale, o.y, o.y_f32, stream); break;
        case NM_OP_GEMM: rc = nm_gemm_pwl(&o.gemm, stream); break;
        default: return fail(NM_ERR_INVALID_ARG, "nm_cnn_run: step %d has unknown kind %d", i, o.kind);
        }
        if (rc) return rc;
    }
    return NM_OK;
}

}  // extern "C"
