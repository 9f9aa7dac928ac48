// Fused attention for gfx950: scores = Q K^T, softmax-PWL, context = P V in one kernel, per
// (batch, head, block of 128 queries).  The int32 scores and the int8 probabilities never leave
// registers (they are written out only when the caller asks for them).
//
// Paper basis: Section 3.1 (attention is a linear operation mapped to matrix products) and
// Section 3.2 (exp and 1/x as PWL tables); the arithmetic is exactly that of the three separate
// entry points (nm_attn_scores, nm_softmax_pwl, nm_attn_context), including the normative order
// of the row sum, so the results are bit-identical to the unfused path.
//
// Layout trick: a wavefront owns 32 queries.  K rows feed the MFMA's row operand and Q rows its
// column operand, so lane (m, h) (m = query, h = lane / 32) ends with the scores of query m for
// the keys 32*blk + 8*g + 4*h + e (blk = key block, g = 0..3, e = 0..3): groups of four
// consecutive keys, which are exactly the 4-element groups of the normative row sum (accumulator
// index 8*blk + 2*g + h).  The butterfly over accumulators is then: in-register adds over blk
// (masks 32, 16, 8), over g (masks 4, 2) and one cross-lane add with lane ^ 32 (mask 1).
// The int8 probabilities are packed in place, four per register, and that register quadruple IS
// the operand of the second product: the contraction index of an integer MFMA may be permuted
// freely as long as both operands use the same permutation, so V^T is written to LDS with the key
// order (blk, h, g, e) that matches the way the probabilities sit in the lanes.
#include <climits>

#include "nm_device.h"

namespace nm {

struct AttnParams {
    const int8_t* qkv;
    int B, S, H, heads;
    float alpha_scores, inv_s_p, alpha_ctx, inv_s_ctx;
    DevTable t_exp, t_recip;
    int8_t* ctx;
    int32_t* scores_out;  // optional [B, heads, S, S]
    int8_t* p_out;        // optional [B, heads, S, S]
};

constexpr int kAttnThreads = 256;
constexpr int kHeadDim = 64;

__device__ __forceinline__ int attn_swz(int row) { return ((row >> 1) & 3) ^ ((row >> 2) & 3); }
__device__ __forceinline__ int attn_koff(int row, int chunk) { return row * 64 + ((chunk ^ attn_swz(row)) << 4); }

// kFull: S == 32 * NB, so no key or query is masked (removes every per-key predicate).
template <int NB, bool kFull>
__global__ __launch_bounds__(kAttnThreads) void attention_pwl_kernel(AttnParams p)
{
    constexpr int SK = NB * 32;   // padded key count
    constexpr int SV = SK + 16;   // row stride of the transposed V image (bank spread)
    __shared__ __attribute__((aligned(16))) int8_t sK[SK * 64];
    __shared__ __attribute__((aligned(16))) int8_t sVt[kHeadDim * SV];
    extern __shared__ float2 s_kb[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 31, h = lane >> 5;
    const int b = blockIdx.y / p.heads, head = blockIdx.y % p.heads;
    const int S = kFull ? 32 * NB : p.S, H = p.H;
    const long ld = 3L * H;
    const int8_t* __restrict__ base = p.qkv + (long)b * S * ld + head * kHeadDim;

    stage_table(s_kb, p.t_exp);
    // K tile -> LDS (rows past S are zero), V tile -> LDS transposed with the key permutation
    for (int idx = tid; idx < SK * 4; idx += kAttnThreads) {
        const int r = idx >> 2, c = idx & 3;
        v4i kv = {0, 0, 0, 0}, vv = {0, 0, 0, 0};
        if (r < S) {
            kv = *reinterpret_cast<const v4i*>(base + (long)r * ld + H + 16 * c);
            vv = *reinterpret_cast<const v4i*>(base + (long)r * ld + 2 * H + 16 * c);
        }
        *reinterpret_cast<v4i*>(&sK[attn_koff(r, c)]) = kv;
        const int pos = (r & ~31) + 16 * ((r >> 2) & 1) + 4 * ((r >> 3) & 3) + (r & 3);
#pragma unroll
        for (int e = 0; e < 16; ++e)
            sVt[(16 * c + e) * SV + pos] = (int8_t)((unsigned)vv[e >> 2] >> (8 * (e & 3)));
    }
    // this lane's query row, straight from global memory into the MFMA operand registers
    const int m = blockIdx.x * 128 + wave * 32 + fr;
    v4i qf[2] = {{0, 0, 0, 0}, {0, 0, 0, 0}};
    if (m < S) {
        qf[0] = *reinterpret_cast<const v4i*>(base + (long)m * ld + 16 * h);
        qf[1] = *reinterpret_cast<const v4i*>(base + (long)m * ld + 32 + 16 * h);
    }
    __syncthreads();

    // ---- scores ---------------------------------------------------------------------------------
    v16i acc[NB];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk) {
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[blk][v] = 0;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const v4i kf = *reinterpret_cast<const v4i*>(&sK[attn_koff(32 * blk + fr, 2 * ks + h)]);
            acc[blk] = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf, qf[ks], acc[blk], 0, 0, 0);
        }
    }
    const long row_ss = ((long)blockIdx.y * S + m) * S;  // offset of this query's row in [B,heads,S,S]
    const bool vec4 = (S & 3) == 0;
    if (p.scores_out && m < S) {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int key = 32 * blk + 8 * g + 4 * h;
                if (vec4 && key < S) {
                    *reinterpret_cast<v4i*>(p.scores_out + row_ss + key) =
                        v4i{acc[blk][4 * g], acc[blk][4 * g + 1], acc[blk][4 * g + 2], acc[blk][4 * g + 3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (key + e < S) p.scores_out[row_ss + key + e] = acc[blk][4 * g + e];
                }
            }
    }

    // ---- softmax-PWL ----------------------------------------------------------------------------
    int mi = INT_MIN;
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int key = 32 * blk + 8 * (v >> 2) + 4 * h + (v & 3);
            if (kFull || key < S) mi = max(mi, acc[blk][v]);
        }
    mi = max(mi, __shfl_xor(mi, 32, 64));

    // exp values replace the scores in place (same registers, float bits)
    float part[NB][4];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            float s = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int key = 32 * blk + 8 * g + 4 * h + e;
                float x = 0.0f;
                if (kFull || key < S) {
                    const float t = (float)(acc[blk][4 * g + e] - mi) * p.alpha_scores;
                    int seg;
                    x = pwl_eval(t, p.t_exp, s_kb, seg);
                    s = s + x;
                }
                acc[blk][4 * g + e] = __float_as_int(x);
            }
            part[blk][g] = s;
        }
    // butterfly over the accumulator index 8*blk + 2*g + h: masks 32, 16, 8 (blk), 4, 2 (g), 1 (h)
#pragma unroll
    for (int mask = NB / 2; mask >= 1; mask >>= 1)
#pragma unroll
        for (int blk = 0; blk < mask; ++blk)
#pragma unroll
            for (int g = 0; g < 4; ++g) part[blk][g] = part[blk][g] + part[blk + mask][g];
    const float s02 = part[0][0] + part[0][2];
    const float s13 = part[0][1] + part[0][3];
    const float sh = s02 + s13;
    const float sum = sh + __shfl_xor(sh, 32, 64);
    int segr;
    const float r = pwl_eval(sum, p.t_recip, p.t_recip.kb, segr);

    unsigned pk[NB][4];
#pragma unroll
    for (int blk = 0; blk < NB; ++blk)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int key = 32 * blk + 8 * g + 4 * h + e;
                q[e] = (kFull || key < S) ? requant(__int_as_float(acc[blk][4 * g + e]) * r, p.inv_s_p) : 0;
            }
            pk[blk][g] = pack4(q[0], q[1], q[2], q[3]);
        }
    if (p.p_out && m < S) {
#pragma unroll
        for (int blk = 0; blk < NB; ++blk)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int key = 32 * blk + 8 * g + 4 * h;
                if (vec4 && key < S) {
                    *reinterpret_cast<unsigned*>(p.p_out + row_ss + key) = pk[blk][g];
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (key + e < S) p.p_out[row_ss + key + e] = (int8_t)(pk[blk][g] >> (8 * e));
                }
            }
    }

    // ---- context --------------------------------------------------------------------------------
    const long orow = ((long)b * S + m) * H + head * kHeadDim;
#pragma unroll
    for (int cb = 0; cb < 2; ++cb) {
        v16i a2;
#pragma unroll
        for (int v = 0; v < 16; ++v) a2[v] = 0;
#pragma unroll
        for (int blk = 0; blk < NB; ++blk) {
            const v4i vf = *reinterpret_cast<const v4i*>(&sVt[(32 * cb + fr) * SV + 32 * blk + 16 * h]);
            const v4i pf = {(int)pk[blk][0], (int)pk[blk][1], (int)pk[blk][2], (int)pk[blk][3]};
            a2 = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, a2, 0, 0, 0);
        }
        if (m < S) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                int q[4];
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    q[e] = requant(__builtin_fmaf((float)a2[4 * g + e], p.alpha_ctx, 0.0f), p.inv_s_ctx);
                *reinterpret_cast<unsigned*>(p.ctx + orow + 32 * cb + 8 * g + 4 * h) = pack4(q[0], q[1], q[2], q[3]);
            }
        }
    }
}

}  // namespace nm

using namespace nm;

extern "C" int32_t nm_attention_pwl(const int8_t* qkv, int32_t B, int32_t S, int32_t H, int32_t heads,
                                    float alpha_scores, const nm_tables* tables, int32_t exp_idx,
                                    int32_t recip_idx, float inv_s_p, float alpha_ctx, float inv_s_ctx,
                                    int8_t* ctx, int32_t* scores_out, int8_t* p_out, void* stream)
{
    if (!qkv || !ctx) return fail(NM_ERR_INVALID_ARG, "nm_attention_pwl: NULL pointer");
    if (B < 1 || S < 1 || H < 1 || heads < 1) return fail(NM_ERR_INVALID_ARG, "nm_attention_pwl: dimensions must be >= 1");
    if (H % heads != 0) return fail(NM_ERR_INVALID_ARG, "nm_attention_pwl: H %d not divisible by heads %d", H, heads);
    AttnParams p{};
    int32_t rc = get_dev_table(tables, exp_idx, &p.t_exp, "nm_attention_pwl(exp)");
    if (rc) return rc;
    rc = get_dev_table(tables, recip_idx, &p.t_recip, "nm_attention_pwl(recip)");
    if (rc) return rc;
    if (H / heads != kHeadDim) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: head size %d (only 64 is fused)", H / heads);
    if (S > 256) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: S %d > 256 (use the three separate calls)", S);
    if ((int64_t)B * heads > 65535) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: B * heads > 65535");
    if ((int64_t)B * S * 3 * H >= (1LL << 31)) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: B*S*3H >= 2^31");
    if (!aligned(qkv, 16) || H % 16 != 0 || !aligned(ctx, 4) || H % 4 != 0 || (scores_out && !aligned(scores_out, 16)) ||
        (p_out && !aligned(p_out, 4)))
        return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: pointers / H not aligned for the fused kernel");
    p.qkv = qkv; p.B = B; p.S = S; p.H = H; p.heads = heads;
    p.alpha_scores = alpha_scores; p.inv_s_p = inv_s_p; p.alpha_ctx = alpha_ctx; p.inv_s_ctx = inv_s_ctx;
    p.ctx = ctx; p.scores_out = scores_out; p.p_out = p_out;
    const dim3 grid((S + 127) / 128, B * heads);
    const size_t shmem = sizeof(float2) * (size_t)p.t_exp.nseg;
    hipStream_t st = (hipStream_t)stream;
#define NM_ATTN_LAUNCH(NBV)                                                                         \
    do {                                                                                            \
        if (S == 32 * NBV) hipLaunchKernelGGL((attention_pwl_kernel<NBV, true>), grid, dim3(kAttnThreads), shmem, st, p); \
        else hipLaunchKernelGGL((attention_pwl_kernel<NBV, false>), grid, dim3(kAttnThreads), shmem, st, p);              \
    } while (0)
    if (S <= 32) NM_ATTN_LAUNCH(1);
    else if (S <= 64) NM_ATTN_LAUNCH(2);
    else if (S <= 128) NM_ATTN_LAUNCH(4);
    else NM_ATTN_LAUNCH(8);
#undef NM_ATTN_LAUNCH
    return check_hip(hipGetLastError(), "nm_attention_pwl launch");
}
