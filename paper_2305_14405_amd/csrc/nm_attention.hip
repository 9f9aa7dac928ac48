// Fused attention for gfx950: scores = Q K^T, softmax-PWL, context = P V in one kernel, per
// (batch, head, block of 64 or 128 queries).  The int32 scores and the int8 probabilities never leave
// registers (they are written out only when the caller asks for them).
//
// Paper basis: Section 3.1 (attention is a linear operation mapped to matrix products) and
// Section 3.2 (exp and 1/x as PWL tables); the arithmetic is exactly that of the three separate
// entry points (nm_attn_scores, nm_softmax_pwl, nm_attn_context), including the normative order
// of the row sum, so the results are bit-identical to the unfused path.
//
// Layout: a wavefront owns 16 queries and uses the 16x16x64 integer MFMA (one instruction covers
// the whole head dimension).  K rows feed the row operand and Q rows the column operand, so lane
// (m, hq) (m = lane % 16 = query, hq = lane / 16) ends with the scores of query m for the keys
// 16*blk + 4*hq + e (blk = key block, e = 0..3): groups of four consecutive keys, which are the
// 4-element groups of the normative row sum (accumulator index (4*blk + hq) % 64).  The butterfly
// over accumulators is then: in-register adds over blk (masks 32, 16, 8, 4) and two cross-lane
// adds (lane ^ 32 for mask 2, lane ^ 16 for mask 1).  Arithmetic dominates this kernel (about 20
// vector instructions per score against 1/16 of an MFMA), so a wavefront of 16 queries costs
// nothing in matrix throughput and gives the scheduler four times more, smaller units to balance
// over the compute units than a 32x32 tiling would.
// The int8 probabilities are packed in place, four per register, and four such registers ARE the
// operand of the second product: the contraction index of an integer MFMA may be permuted freely
// as long as both operands use the same permutation.  V stays row-major in LDS ([key][64 bytes],
// copied like K); its operand fragments (one head column per lane, 16 keys) come out of the
// transposing LDS read of gfx950 (ds_read_b64_tr_b8: within 16 lanes, lane j receives byte j % 8
// of the eight rows addressed by lanes j / 8, j / 8 + 2, ...), with the row addresses chosen so
// that the keys arrive in the order the probabilities have in the lanes.
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
    int ctx_vec16;        // ctx is 16-byte aligned: context rows leave as 16-byte stores
};

// Wavefronts per workgroup: four (64 queries) up to 256 keys, where many small workgroups balance
// best; eight (128 queries) beyond 256 keys, where the K / V staging per workgroup is large and is then
// shared by twice as many queries.
constexpr int attn_waves(int nkb) { return nkb >= 8 ? 8 : 4; }
constexpr int kHeadDim = 64;

// K image: 64-byte rows, the four 16-byte chunks of a row rotated by (row / 4) % 4 so that the 16
// lanes of an operand read (16 consecutive rows, one chunk) cover all banks.
__device__ __forceinline__ int attn_koff(int row, int chunk) { return row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4); }
// V image: the same, with the rotation also depending on (row / 16) % 4, because one transposing
// read touches rows 16 apart.
__device__ __forceinline__ int attn_vswz(int row) { return ((row >> 2) & 3) ^ ((row >> 4) & 3); }
__device__ __forceinline__ int attn_voff(int row, int chunk) { return row * 64 + ((chunk ^ attn_vswz(row)) << 4); }

constexpr int kCtxPatch = 16 * 80;   // per wavefront: 16 context rows of 64 bytes, 80 apart
constexpr size_t attn_lds_bytes(int nkb) { return 2 * (size_t)nkb * 64 * 64 + (size_t)attn_waves(nkb) * kCtxPatch; }

// op(v, value of lane ^ MASK) for MASK 32 or 16 with the half / row swap instructions: swapping a
// register with a copy of itself leaves {lower halves (even rows) twice} in one and {upper halves
// (odd rows) twice} in the other; op is commutative, so op(first, second) is what every lane needs.
template <int MASK, typename Op>
__device__ __forceinline__ int swap_reduce(int v, Op op)
{
    if (MASK == 32) {
        const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
        return op((int)r[0], (int)r[1]);
    }
    const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    return op((int)r[0], (int)r[1]);
}

// NKB: padded key count / 64.  kFull: S == 64 * NKB, so no key or query is masked (removes every
// per-key predicate).
template <int NKB, bool kFull>
__global__ __launch_bounds__(64 * attn_waves(NKB)) __attribute__((amdgpu_waves_per_eu(2))) void attention_pwl_kernel(AttnParams p)
{
    constexpr int kAttnThreads = 64 * attn_waves(NKB);
    constexpr int kQueries = 16 * attn_waves(NKB);   // queries per workgroup
    constexpr int SK = NKB * 64;   // padded key count
    constexpr int NBLK = SK / 16;  // 16-key blocks
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    int8_t* sK = smem;
    int8_t* sV = smem + SK * 64;
    int8_t* sO = smem + 2 * SK * 64;   // context patches
    float2* s_kb = reinterpret_cast<float2*>(smem + attn_lds_bytes(NKB));

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int fr = lane & 15, hq = lane >> 4;
    // Workgroups are dealt to the eight XCDs round-robin by linear id.  Renumber them so that an
    // XCD receives consecutive (head, query block) pairs: the query blocks of a head share its K
    // and V, and neighbouring heads share 128-byte lines (a head's rows are 64-byte halves), so
    // these fetches then meet in one L2 instead of going to memory once per XCD.
    int bx = blockIdx.x, by = blockIdx.y;
    {
        const int total = gridDim.x * gridDim.y;
        if ((total & 7) == 0) {
            const int lin = blockIdx.x + gridDim.x * blockIdx.y;
            const int v = (lin & 7) * (total >> 3) + (lin >> 3);
            bx = v % gridDim.x;
            by = v / gridDim.x;
        }
    }
    const int b = by / p.heads, head = by % p.heads;
    const int S = kFull ? SK : p.S, H = p.H;
    const long ld = 3L * H;
    const int8_t* __restrict__ base = p.qkv + (long)b * S * ld + head * kHeadDim;

    float2* s_kb_recip = s_kb + p.t_exp.nseg;
    stage_table(s_kb, p.t_exp);
    stage_table(s_kb_recip, p.t_recip);
    // K and V tiles -> LDS, row-major.  With every row present the copy is a direct global -> LDS
    // load (16 rows of 64 bytes per wavefront instruction; the chunk rotation is applied to the
    // source address).  Otherwise through registers: K rows past S are zero; V rows past S stay
    // unwritten (they only ever meet zero probabilities).
    if (kFull) {
        const unsigned lds_k = (unsigned)(uintptr_t)sK, lds_v = (unsigned)(uintptr_t)sV;
        for (int blk16 = __builtin_amdgcn_readfirstlane(wave); blk16 < SK / 16; blk16 += kAttnThreads / 64) {
            const int r = 16 * blk16 + (lane >> 2);
            dma16(base + (long)r * ld + H + 16 * ((lane & 3) ^ ((r >> 2) & 3)), lds_k + 1024 * blk16);
            dma16(base + (long)r * ld + 2 * H + 16 * ((lane & 3) ^ attn_vswz(r)), lds_v + 1024 * blk16);
        }
    } else {
        for (int idx = tid; idx < SK * 4; idx += kAttnThreads) {
            const int r = idx >> 2, c = idx & 3;
            v4i kv = {0, 0, 0, 0};
            if (r < S) {
                kv = *reinterpret_cast<const v4i*>(base + (long)r * ld + H + 16 * c);
                *reinterpret_cast<v4i*>(&sV[attn_voff(r, c)]) = *reinterpret_cast<const v4i*>(base + (long)r * ld + 2 * H + 16 * c);
            }
            *reinterpret_cast<v4i*>(&sK[attn_koff(r, c)]) = kv;
        }
    }
    // this lane's query row, straight from global memory into the MFMA operand registers
    const int m = bx * kQueries + wave * 16 + fr;
    v4i qf = {0, 0, 0, 0};
    if (kFull || m < S) qf = *reinterpret_cast<const v4i*>(base + (long)m * ld + 16 * hq);
    if (kFull) wait_vmcnt<0>();   // this wavefront's K loads have landed (the barrier covers the others')
    __syncthreads();

    // ---- scores ---------------------------------------------------------------------------------
    v4i acc[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        const v4i kf = *reinterpret_cast<const v4i*>(&sK[attn_koff(16 * blk + fr, hq)]);
        acc[blk] = __builtin_amdgcn_mfma_i32_16x16x64_i8(kf, qf, v4i{0, 0, 0, 0}, 0, 0, 0);
        // keeps the operand reads of later blocks from piling up in registers
        if ((blk & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
    const long row_ss = ((long)by * S + m) * S;  // offset of this query's row in [B,heads,S,S]
    const bool vec4 = (S & 3) == 0;
    if (p.scores_out && (kFull || m < S)) {
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            const int key = 16 * blk + 4 * hq;
            if (vec4 && (kFull || key < S)) {
                *reinterpret_cast<v4i*>(p.scores_out + row_ss + key) = acc[blk];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (key + e < S) p.scores_out[row_ss + key + e] = acc[blk][e];
            }
        }
    }

    // ---- softmax-PWL ----------------------------------------------------------------------------
    int mi = INT_MIN;
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk)
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (kFull || 16 * blk + 4 * hq + e < S) mi = max(mi, acc[blk][e]);
    mi = swap_reduce<32>(mi, [](int a, int b) { return max(a, b); });
    mi = swap_reduce<16>(mi, [](int a, int b) { return max(a, b); });

    // exp values replace the scores in place (same registers, float bits).  Keys 256.. wrap onto
    // the 64 accumulators of keys 0..255 (accumulator = (key / 4) % 64) and continue their sums.
    constexpr int NP = NBLK < 16 ? NBLK : 16;
    float part[NP];
    const float clo = p.t_exp.clamp_input ? p.t_exp.lo : -__builtin_inff();
    const float chi = p.t_exp.clamp_input ? p.t_exp.hi : __builtin_inff();
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        float s = blk < 16 ? 0.0f : part[blk & 15];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = 0.0f;
            if (kFull || 16 * blk + 4 * hq + e < S) {
                const float t = (float)(acc[blk][e] - mi) * p.alpha_scores;
                x = pwl_eval_bounded(t, clo, chi, p.t_exp, s_kb);
                s = s + x;
            }
            acc[blk][e] = __float_as_int(x);
        }
        part[blk & 15] = s;
        // bounds the number of table look-ups in flight (each holds two registers)
        if (NBLK > 16 && (blk & 3) == 3) __builtin_amdgcn_sched_barrier(0);
    }
    // butterfly over the accumulator index 4*blk + hq: masks 32, 16, 8, 4 (blk), then 2, 1 (hq)
#pragma unroll
    for (int mask = NP / 2; mask >= 1; mask >>= 1)
#pragma unroll
        for (int blk = 0; blk < mask; ++blk) part[blk] = part[blk] + part[blk + mask];
    float sum = part[0];
    const auto addf = [](int a, int b) { return __float_as_int(__int_as_float(a) + __int_as_float(b)); };
    sum = __int_as_float(swap_reduce<32>(__float_as_int(sum), addf));
    sum = __int_as_float(swap_reduce<16>(__float_as_int(sum), addf));
    int segr;
    const float r = pwl_eval(sum, p.t_recip, s_kb_recip, segr);

    unsigned pk[NBLK];
#pragma unroll
    for (int blk = 0; blk < NBLK; ++blk) {
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            q[e] = (kFull || 16 * blk + 4 * hq + e < S) ? requant(__int_as_float(acc[blk][e]) * r, p.inv_s_p) : 0;
        pk[blk] = pack4(q[0], q[1], q[2], q[3]);
    }
    if (p.p_out && (kFull || m < S)) {
#pragma unroll
        for (int blk = 0; blk < NBLK; ++blk) {
            const int key = 16 * blk + 4 * hq;
            if (vec4 && (kFull || key < S)) {
                *reinterpret_cast<unsigned*>(p.p_out + row_ss + key) = pk[blk];
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (key + e < S) p.p_out[row_ss + key + e] = (int8_t)(pk[blk] >> (8 * e));
            }
        }
    }

    // ---- context --------------------------------------------------------------------------------
    // Operand slot s (0..15) of lane group hq must hold key 64*kb + 16*(s/4) + 4*hq + s%4 (where the
    // probabilities sit).  A transposing read delivers eight rows: this lane supplies the address of
    // row (lane % 16) / 2 of its group, shifted by 8 bytes for odd lanes so that lanes 8..15 of the
    // group receive head columns 8..15.
    typedef int v2i_t __attribute__((ext_vector_type(2)));
    const int tr_t = fr >> 1, tr_half = fr & 1;
    int voff[2];   // this lane's row address for the two reads of an operand (kb = 0, cb = 0)
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
        const int sidx = 8 * hh + tr_t;
        const int key = 16 * (sidx >> 2) + 4 * hq + (sidx & 3);
        voff[hh] = key * 64 + 8 * tr_half;   // chunk position added per product: (cb ^ hq ^ (sidx >> 2)) * 16
    }
    v4i a2[4];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) a2[cb] = v4i{0, 0, 0, 0};
#pragma unroll
    for (int kb = 0; kb < NKB; ++kb) {
        const v4i pf = {(int)pk[4 * kb], (int)pk[4 * kb + 1], (int)pk[4 * kb + 2], (int)pk[4 * kb + 3]};
#pragma unroll
        for (int cb = 0; cb < 4; ++cb) {
            v2i_t part[2];
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                const int chunk = cb ^ hq ^ ((8 * hh + tr_t) >> 2);
                part[hh] = __builtin_amdgcn_ds_read_tr8_b64_v2i32(
                    (__attribute__((address_space(3))) v2i_t*)(sV + 4096 * kb + voff[hh] + 16 * chunk));
            }
            const v4i vf = {part[0][0], part[0][1], part[1][0], part[1][1]};
            a2[cb] = __builtin_amdgcn_mfma_i32_16x16x64_i8(vf, pf, a2[cb], 0, 0, 0);
        }
    }
    // lane (m, hq) holds head columns 16*cb + 4*hq + e of query m: through a per-wavefront LDS patch
    // so that every lane stores 16 consecutive bytes
    int8_t* patch = sO + wave * kCtxPatch;
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) {
        int q[4];
#pragma unroll
        for (int e = 0; e < 4; ++e)
            q[e] = requant(__builtin_fmaf((float)a2[cb][e], p.alpha_ctx, 0.0f), p.inv_s_ctx);
        *reinterpret_cast<unsigned*>(patch + fr * 80 + 16 * cb + 4 * hq) = pack4(q[0], q[1], q[2], q[3]);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    {
        const int mq = bx * kQueries + wave * 16 + (lane >> 2), c = lane & 3;
        if (kFull || mq < S) {
            const v4i o = *reinterpret_cast<const v4i*>(patch + (lane >> 2) * 80 + 16 * c);
            int8_t* dst = p.ctx + ((long)b * S + mq) * H + head * kHeadDim + 16 * c;
            if (p.ctx_vec16) {
                *reinterpret_cast<v4i*>(dst) = o;
            } else {
#pragma unroll
                for (int w = 0; w < 4; ++w) *reinterpret_cast<int*>(dst + 4 * w) = o[w];
            }
        }
    }
}

template <int NKB>
static int32_t launch_attention(const AttnParams& p, hipStream_t st)
{
    const size_t shmem = attn_lds_bytes(NKB) + sizeof(float2) * ((size_t)p.t_exp.nseg + (size_t)p.t_recip.nseg);
    static bool configured = false;  // one attribute call per instantiation pair
    if (!configured) {
        int32_t rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_pwl_kernel<NKB, true>),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
                               "hipFuncSetAttribute(attention_pwl_kernel)");
        if (rc) return rc;
        rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(attention_pwl_kernel<NKB, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
                       "hipFuncSetAttribute(attention_pwl_kernel)");
        if (rc) return rc;
        configured = true;
    }
    constexpr int kThreads = 64 * attn_waves(NKB), kQueries = 16 * attn_waves(NKB);
    const dim3 grid((p.S + kQueries - 1) / kQueries, p.B * p.heads);
    if (p.S == 64 * NKB) hipLaunchKernelGGL((attention_pwl_kernel<NKB, true>), grid, dim3(kThreads), shmem, st, p);
    else hipLaunchKernelGGL((attention_pwl_kernel<NKB, false>), grid, dim3(kThreads), shmem, st, p);
    return NM_OK;
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
    if (!(alpha_scores == alpha_scores) || __builtin_isinf(alpha_scores))
        return fail(NM_ERR_INVALID_ARG, "nm_attention_pwl: alpha_scores must be finite");
    if (H % heads != 0) return fail(NM_ERR_INVALID_ARG, "nm_attention_pwl: H %d not divisible by heads %d", H, heads);
    AttnParams p{};
    int32_t rc = get_dev_table(tables, exp_idx, &p.t_exp, "nm_attention_pwl(exp)");
    if (rc) return rc;
    rc = get_dev_table(tables, recip_idx, &p.t_recip, "nm_attention_pwl(recip)");
    if (rc) return rc;
    if (H / heads != kHeadDim) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: head size %d (only 64 is fused)", H / heads);
    if (S > 512) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: S %d > 512 (use the three separate calls)", S);
    if ((int64_t)B * heads > 65535) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: B * heads > 65535");
    if ((int64_t)B * S * 3 * H >= (1LL << 31)) return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: B*S*3H >= 2^31");
    if (!aligned(qkv, 16) || H % 16 != 0 || !aligned(ctx, 4) || H % 4 != 0 || (scores_out && !aligned(scores_out, 16)) ||
        (p_out && !aligned(p_out, 4)))
        return fail(NM_ERR_UNSUPPORTED, "nm_attention_pwl: pointers / H not aligned for the fused kernel");
    p.qkv = qkv; p.B = B; p.S = S; p.H = H; p.heads = heads;
    p.alpha_scores = alpha_scores; p.inv_s_p = inv_s_p; p.alpha_ctx = alpha_ctx; p.inv_s_ctx = inv_s_ctx;
    p.ctx = ctx; p.scores_out = scores_out; p.p_out = p_out;
    p.ctx_vec16 = aligned(ctx, 16) ? 1 : 0;
    hipStream_t st = (hipStream_t)stream;
    if (S <= 64) rc = launch_attention<1>(p, st);
    else if (S <= 128) rc = launch_attention<2>(p, st);
    else if (S <= 256) rc = launch_attention<4>(p, st);
    else rc = launch_attention<8>(p, st);
    if (rc) return rc;
    return check_hip(hipGetLastError(), "nm_attention_pwl launch");
}
