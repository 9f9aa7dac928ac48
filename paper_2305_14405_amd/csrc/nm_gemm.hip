// int8 x int8 -> int32 GEMM on the gfx950 matrix cores with the fused epilogue
// (dequantise, bias, residual, PWL table lookup from LDS, requantise), plus the two attention
// products, which are the same kernel launched over (batch, head) with strided operands.
//
// Paper basis: Section 3.1 (fully connected layers, attention and residual additions are matrix
// multiplications / additions) and Section 3.2 (the nonlinearity after a linear operator is the
// element-wise PWL calculation y = k[s]*x + b[s]).  The paper blocks its matrices for a systolic
// array with a three-level buffer hierarchy; here the blocking is for CDNA4: a workgroup of four or
// eight wavefronts owns a BM x BN tile of the output, the k-loop streams 64- or 128-byte slices of
// both operands through a ring of LDS stages, and each wavefront issues 32x32x32 int8 MFMAs on its
// WM x WN sub-tile with int32 accumulators that never leave registers until the epilogue.
// Two kernels: gemm_stream_kernel (aligned operands, K a multiple of 64: operands go global -> LDS
// directly; also gathers the rows of a convolution's patch matrix on the fly) in several tile
// configurations chosen by launch_gemm, and gemm_pwl_kernel (any shape and alignment, W as [N,K]
// or [K,N], operands through registers).
//
// Operand roles: the MFMA's first operand supplies the rows of its 32x32 result and the second
// the columns.  W rows (output columns n) go first and A rows (output rows m) second, so a lane
// ends up with one output row m and, per group of four accumulator registers, four consecutive
// output columns n: four int8 results pack into one 32-bit store and bias / per-column scales
// are read as four consecutive floats.
//
// Both operands are K-contiguous, which is what the int8 MFMA wants: a lane feeds 16 consecutive
// k of one row.  The same k of A and W always meet in the same (lane group, byte) slot, and int32
// addition is exact, so results do not depend on tiling, on the k order or on any split of K.
#include <cstdlib>
#include <cstring>

#include "nm_gemm_common.h"
#include "nm_gemm_tile.h"

namespace nm {

// A line of zeros in device memory: the source of operand bytes that fall into a convolution's
// padding (the direct global -> LDS loads cannot substitute a value, only an address).
__device__ __attribute__((aligned(256))) int8_t g_zero_line[256];

// Debug switch: NM_GEMM_GENERIC=1 in the environment sends every shape to the generic kernel.
static bool force_generic()
{
    static const bool v = [] { const char* e = getenv("NM_GEMM_GENERIC"); return e && e[0] == '1'; }();
    return v;
}
// Debug switch, read once per process: NM_GEMM_CFG=big|wide|split|small|mid3|mid2|oldbig forces that
// tile configuration wherever its requirements hold (tuning aid; "oldbig" is the streaming kernel's
// 256x192 configuration, which the tile kernel has replaced).
static int forced_cfg()
{
    static const int v = [] {
        const char* e = getenv("NM_GEMM_CFG");
        if (!e) return -1;
        static const char* const names[] = {"big", "wide", "split", "small", "mid3", "mid2", "oldbig"};
        for (int i = 0; i < 7; ++i)
            if (!strcmp(e, names[i])) return i;
        return -1;
    }();
    return v;
}

// 16 bytes of a row-major int8 matrix at (row, k .. k+15); zeros outside [0,nrows) x [0,K).
template <bool kAligned>
__device__ __forceinline__ v4i load_chunk(const int8_t* __restrict__ X, long ld, int row, int nrows,
                                          int k, int K)
{
    v4i v = {0, 0, 0, 0};
    if (row < nrows) {
        const int8_t* p = X + (long)row * ld + k;
        if (kAligned) {
            if (k < K) v = *reinterpret_cast<const v4i*>(p);
        } else {
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                unsigned word = 0;
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    if (k + 4 * w + b < K) word |= (unsigned)(uint8_t)p[4 * w + b] << (8 * b);
                v[w] = (int)word;
            }
        }
    }
    return v;
}

// ---------------------------------------------------------------------------------------------
// Epilogue shared by both kernels.  A lane holds, for one output row m, four consecutive columns
// nb .. nb+3 (one group of four accumulator registers).
// ---------------------------------------------------------------------------------------------
// Epilogue specialisations: the generic one reads every option at run time; the others fix the
// set of outputs and options the encoder layer uses, which removes dead code from the unrolled
// epilogue (it is instantiated once per accumulator group).
struct Epi4 {
    float y[4];
    int q[4];
    int s[4];
};

// Per-column parameters of four consecutive columns, loaded once and reused for every row.
struct Col4 {
    float scale[4], bias[4], inv[4];
};

__device__ __forceinline__ void load4(const float* __restrict__ v, int nb, int N, bool vec, float (&out)[4])
{
    if (vec && nb + 3 < N) {
        const v4f t = *reinterpret_cast<const v4f*>(v + nb);
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = t[e];
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (nb + e < N) out[e] = v[nb + e];
    }
}

template <int kEpi>
__device__ __forceinline__ void load_cols(const GemmParams& p, int nb, Col4& c)
{
    const float alpha = p.alpha, ois = p.out_inv_scale;
#pragma unroll
    for (int e = 0; e < 4; ++e) { c.scale[e] = alpha; c.bias[e] = 0.0f; c.inv[e] = ois; }
    if (kEpi == EPI_ACC) return;
    if (p.bias) load4(p.bias, nb, p.N, p.vec_cols, c.bias);
    if (p.alpha_vec) load4(p.alpha_vec, nb, p.N, p.vec_cols, c.scale);
    if (kEpi == EPI_F32_RESID) return;
    if (kEpi == EPI_GENERIC && p.out_inv_scale_vec) {
        load4(p.out_inv_scale_vec, nb, p.N, p.vec_cols, c.inv);
    } else if (p.split_cols > 0) {
        const float i0 = p.inv3[0], i1 = p.inv3[1], i2 = p.inv3[2];
#pragma unroll
        for (int e = 0; e < 4; ++e) c.inv[e] = nb + e >= 2 * p.split_cols ? i2 : (nb + e >= p.split_cols ? i1 : i0);
    }
}

// Residual codes of four consecutive columns of one row.
__device__ __forceinline__ void load_resid4(const GemmParams& p, long rowoff, int nb, bool vec, int (&r4)[4])
{
    if (vec) {
        const unsigned w = *reinterpret_cast<const unsigned*>(p.resid + rowoff + nb);
#pragma unroll
        for (int e = 0; e < 4; ++e) r4[e] = (int)(int8_t)(w >> (8 * e));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) r4[e] = nb + e < p.N ? (int)p.resid[rowoff + nb + e] : 0;
    }
}

// The arithmetic of the epilogue for four columns of one row (no global memory access).
// kTwoSeg: the table has two segments and is evaluated with a compare (specialised table epilogues)
template <int kEpi, bool kTwoSeg = false>
__device__ __forceinline__ void epi_math(const GemmParams& p, const float2* s_kb, const int (&a4)[4],
                                         const Col4& c, const int (&r4)[4], Epi4& o)
{
    const bool use_resid = kEpi == EPI_GENERIC ? p.resid != nullptr : (kEpi == EPI_F32_RESID || kEpi == EPI_Q_TABLE_RESID);
    const bool use_table = kEpi == EPI_GENERIC ? p.has_table != 0 : (kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID);
    const bool need_q = kEpi == EPI_GENERIC ? p.out_q != nullptr : (kEpi == EPI_Q || kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID);
#pragma unroll
    for (int e = 0; e < 4; ++e) { o.y[e] = 0.0f; o.q[e] = 0; o.s[e] = 0; }
    if (kEpi == EPI_ACC) return;
    const float rs = p.resid_scale;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float v = __builtin_fmaf((float)a4[e], c.scale[e], c.bias[e]);
        if (use_resid) v = __builtin_fmaf((float)r4[e], rs, v);
        if (use_table) {
            if (kTwoSeg) v = pwl_eval_two_segments(v, p.table);
            else if (kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID) v = pwl_eval_noclamp(v, p.table, s_kb, o.s[e]);
            else if (p.table.cellmap) v = pwl_eval_two_level(v, p.table, s_kb, o.s[e]);  // merged table, two steps
            else v = pwl_eval(v, p.table, s_kb, o.s[e]);
        }
        o.y[e] = v;
        if (need_q) o.q[e] = requant(v, c.inv[e]);
    }
}

template <int kEpi>
__device__ __forceinline__ void epi_store(const GemmParams& p, long rowoff, int nb,
                                          const int (&a4)[4], const Epi4& o, bool vec, bool skip_q)
{
    const bool st_q = (kEpi == EPI_GENERIC ? p.out_q != nullptr : (kEpi == EPI_Q || kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID)) && !skip_q;
    const bool st_f = kEpi == EPI_GENERIC ? p.out_f32 != nullptr : kEpi == EPI_F32_RESID;
    const bool st_a = kEpi == EPI_GENERIC ? p.out_acc != nullptr : kEpi == EPI_ACC;
    const bool st_s = kEpi == EPI_GENERIC && p.dbg_seg && p.has_table;
    if (vec) {
        if (st_q) *reinterpret_cast<unsigned*>(p.out_q + rowoff + nb) = pack4(o.q[0], o.q[1], o.q[2], o.q[3]);
        if (st_f) *reinterpret_cast<v4f*>(p.out_f32 + rowoff + nb) = v4f{o.y[0], o.y[1], o.y[2], o.y[3]};
        if (st_a) *reinterpret_cast<v4i*>(p.out_acc + rowoff + nb) = v4i{a4[0], a4[1], a4[2], a4[3]};
        if (st_s)
            *reinterpret_cast<uint2*>(p.dbg_seg + rowoff + nb) =
                make_uint2((unsigned)o.s[0] | ((unsigned)o.s[1] << 16), (unsigned)o.s[2] | ((unsigned)o.s[3] << 16));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (nb + e < p.N) {
                if (st_q) p.out_q[rowoff + nb + e] = (int8_t)o.q[e];
                if (st_f) p.out_f32[rowoff + nb + e] = o.y[e];
                if (st_a) p.out_acc[rowoff + nb + e] = a4[e];
                if (st_s) p.dbg_seg[rowoff + nb + e] = (uint16_t)o.s[e];
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Generic kernel: any shape and alignment, W as [N, K] or [K, N].  Operands go global -> registers
// -> LDS (two stages); out-of-range rows and the k tail are zero-filled.
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int WM, int WN, bool kAligned, bool kWKN>
__global__ __launch_bounds__(kGemmThreads) void gemm_pwl_kernel(GemmParams p)
{
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int WAVES_N = BN / WN;
    static_assert((BM / WM) * (BN / WN) == kGemmThreads / 64, "four wavefronts per workgroup");
    constexpr int LA = BM / 64, LW = BN / 64;  // 16-byte chunks per thread and stage

    __shared__ __attribute__((aligned(16))) int8_t sA[2][BM * kBK];
    __shared__ __attribute__((aligned(16))) int8_t sW[2][BN * kBK];
    extern __shared__ float2 s_kb[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wave_m = (wave / WAVES_N) * WM;
    const int wave_n = (wave % WAVES_N) * WN;

    const int tile_m = blockIdx.x % p.tiles_m;
    const int tile_n = blockIdx.x / p.tiles_m;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int outer = blockIdx.y / p.inner_count;
    const int inner = blockIdx.y % p.inner_count;
    const int8_t* __restrict__ A = p.A + outer * p.a_outer + inner * p.a_inner;
    const int8_t* __restrict__ W = p.W + outer * p.w_outer + inner * p.w_inner;
    const long obase = outer * p.o_outer + inner * p.o_inner;

    if (p.has_table) { if (p.table.cellmap) stage_table_two_level(s_kb, p.table); else stage_table(s_kb, p.table); }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    v4i ra[LA], rw[LW];
    const int ld_row = tid >> 2, ld_chunk = tid & 3;

    auto fetch = [&](int k0) {
#pragma unroll
        for (int i = 0; i < LA; ++i)
            ra[i] = load_chunk<kAligned>(A, p.lda, m0 + ld_row + 64 * i, p.M, k0 + 16 * ld_chunk, p.K);
        if (!kWKN) {
#pragma unroll
            for (int i = 0; i < LW; ++i)
                rw[i] = load_chunk<kAligned>(W, p.ldw, n0 + ld_row + 64 * i, p.N, k0 + 16 * ld_chunk, p.K);
        } else {
            // W is [K, N]: this thread takes k-row kk and 16 consecutive n
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                const int idx = tid + kGemmThreads * i;  // 0 .. 64 * BN/16 - 1
                const int kk = idx / (BN / 16), nc = idx % (BN / 16);
                rw[i] = load_chunk<kAligned>(W, p.ldw, k0 + kk, p.K, n0 + 16 * nc, p.N);
            }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < LA; ++i)
            *reinterpret_cast<v4i*>(&sA[buf][lds_off(ld_row + 64 * i, ld_chunk)]) = ra[i];
        if (!kWKN) {
#pragma unroll
            for (int i = 0; i < LW; ++i)
                *reinterpret_cast<v4i*>(&sW[buf][lds_off(ld_row + 64 * i, ld_chunk)]) = rw[i];
        } else {
#pragma unroll
            for (int i = 0; i < LW; ++i) {
                const int idx = tid + kGemmThreads * i;
                const int kk = idx / (BN / 16), nc = idx % (BN / 16);
#pragma unroll
                for (int b = 0; b < 16; ++b) {
                    const int n = 16 * nc + b;
                    sW[buf][lds_off(n, kk >> 4) + (kk & 15)] = (int8_t)((unsigned)rw[i][b >> 2] >> (8 * (b & 3)));
                }
            }
        }
    };

    const int nk = (p.K + kBK - 1) / kBK;
    fetch(0);
    stash(0);
    __syncthreads();

    const int frag_row = lane & 31, frag_half = lane >> 5;
    for (int kt = 0; kt < nk; ++kt) {
        const int cur = kt & 1;
        if (kt + 1 < nk) fetch((kt + 1) * kBK);
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            v4i fa[TM], fw[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const v4i*>(&sA[cur][lds_off(wave_m + 32 * i + frag_row, 2 * ks + frag_half)]);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fw[j] = *reinterpret_cast<const v4i*>(&sW[cur][lds_off(wave_n + 32 * j + frag_row, 2 * ks + frag_half)]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fa[i], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) stash(cur ^ 1);
        __syncthreads();
    }

#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int nb = n0 + wave_n + 32 * j + 8 * g + 4 * frag_half;
            if (nb >= p.N) continue;
            const bool vec = p.vec_out && nb + 3 < p.N;
            Col4 c;
            load_cols<EPI_GENERIC>(p, nb, c);
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const int m = m0 + wave_m + 32 * i + frag_row;
                if (m >= p.M) continue;
                const long rowoff = obase + (long)m * p.ldo;
                int a4[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) a4[e] = acc[i][j][4 * g + e];
                int r4[4] = {0, 0, 0, 0};
                if (p.resid) load_resid4(p, rowoff, nb, vec, r4);
                Epi4 o;
                epi_math<EPI_GENERIC>(p, s_kb, a4, c, r4, o);
                epi_store<EPI_GENERIC>(p, rowoff, nb, a4, o, vec, false);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Streaming kernel: K a multiple of 64 (of BK), 16-byte aligned rows, W as [N, K].  Operands go global -> LDS directly (global_load_lds_dwordx4: a wavefront
// instruction moves 64 x 16 bytes into 1 KB of consecutive LDS, no registers in between) through
// a ring of kStages stages; a wavefront waits with an explicit vmcnt for the stage it is about to
// use while the loads of the later stages stay in flight.  The LDS image of a stage is
// (BM + BN) rows of BK bytes: 1 KB of consecutive rows per wavefront instruction, with the chunk
// swizzle applied on the global side (with 64-byte rows lane p of an instruction fetches row p/4,
// logical chunk (p%4) ^ swz(row)).  Rows past the matrix edge are clamped to the last row: they only feed
// accumulators that are never stored.
// Workgroups are numbered so that the eight XCDs (workgroup id mod 8) each own a compact block of
// output tiles: the A rows and W rows a block needs fit that XCD's L2.
// int8 output goes through a per-wavefront LDS patch so that rows leave as 16-byte stores.
// ---------------------------------------------------------------------------------------------
// LDS offset of (row, 16-byte chunk) for rows of BK bytes.  BK = 64: four chunks, the swizzle of
// the generic kernel.  BK = 128: eight chunks, 16 consecutive rows spread over all chunk positions
// of two adjacent rows' worth of banks.
// KSPLIT = 2 doubles the wavefronts of a workgroup without shrinking the wavefront tile: two
// wavefronts share each WM x WN sub-tile and take alternate 32-byte k-steps of every k-slice (so
// the LDS read traffic and the operand traffic stay those of the KSPLIT = 1 kernel, while each
// SIMD has two wavefronts whose LDS waits and MFMAs overlap).  After the main loop the two swap
// halves of their int32 partial accumulators through LDS (integer addition is exact in any
// order) and each finishes half of the sub-tile's rows, which also halves the epilogue per
// wavefront.  Used where the grid has fewer workgroups than CUs times two (N = 768 GEMMs).
//
// kConv: the A operand is gathered from an NHWC image (convolution as a matrix product, paper
// Section 3.1).  A k-slice never straddles a filter tap (Cin % BK == 0), so for the slice of tap
// (i, j) and channels c0.. a lane's 16 bytes are x[b, ho*stride - pad + i, wo*stride - pad + j,
// c0 + 16*chunk ..] or, in the padding, 16 bytes of the zero line; only the per-lane source
// address of the direct global -> LDS load changes, the rest of the kernel is the same.
// Wavefronts per SIMD the register allocation should leave room for: as many workgroups per CU as
// the operand ring lets LDS hold (small rings exist so that several workgroups overlap), at most 3.
constexpr int stream_waves_per_simd(int ring_bytes, int waves)
{
    const int wgs = ring_bytes <= 49152 ? 3 : ring_bytes <= 73728 ? 2 : 1;
    const int w = wgs * waves / 4;
    return w < 1 ? 1 : w > 3 ? 3 : w;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int KSPLIT, int BK, int kStages, int kEpi, bool kConv = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N * KSPLIT,
                             stream_waves_per_simd(kStages * (BM + BN) * BK, WAVES_M * WAVES_N * KSPLIT))
void gemm_stream_kernel(GemmParams p)
{
    constexpr int NWT = WAVES_M * WAVES_N;       // wavefront tiles per workgroup
    constexpr int NW = NWT * KSPLIT;             // wavefronts per workgroup
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int TMF = TM / KSPLIT;             // 32-row blocks a wavefront finishes
    constexpr int ROWS = BM + BN;
    constexpr int CPR = BK / 16;                 // 16-byte chunks per LDS row
    constexpr int RPI = 64 / CPR;                // rows moved by one wavefront instruction (1 KB)
    constexpr int NBLK = ROWS / RPI;             // 1 KB blocks per stage
    constexpr int LB = (NBLK + NW - 1) / NW;     // blocks per wavefront (some have LB - 1)
    constexpr int STAGE_BYTES = ROWS * BK;
    constexpr int SW = WN + 16;                  // row stride of the int8 output patch
    constexpr int KS = BK / 32;                  // MFMA k-steps per k-slice
    constexpr int KSW = KS / KSPLIT;             // ... per wavefront
    static_assert(BK == 64 || BK == 128, "k-slice of 64 or 128 bytes");
    static_assert(KSPLIT == 1 || KSPLIT == 2, "one or two wavefronts per sub-tile");
    static_assert(TM % KSPLIT == 0 && KS % KSPLIT == 0, "halves split evenly");
    static_assert(BM % 32 == 0 && BN % 32 == 0 && ROWS % RPI == 0, "tile shape");
    static_assert(WM * SW * NWT <= kStages * STAGE_BYTES, "output patch fits the operand ring");
    static_assert(KSPLIT == 1 || NW * TMF * TN * 4096 <= kStages * STAGE_BYTES, "exchange fits the ring");
    static_assert(kStages >= 2 && kStages <= 4, "ring depth");

    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    float* s_cols = reinterpret_cast<float*>(smem + kStages * STAGE_BYTES);  // scale | bias | inv, BN each
    float2* s_kb = reinterpret_cast<float2*>(s_cols + 3 * BN);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_t = wave % NWT;               // which sub-tile
    const int kg = wave / NWT;                   // which half of the k-steps (0 when KSPLIT == 1)
    const int wave_m = (wave_t / WAVES_N) * WM;
    const int wave_n = (wave_t % WAVES_N) * WN;

    // XCD-aware tile order: ids that share (id mod 8) are renumbered to be consecutive, then
    // consecutive ids fill groups of 8 tile rows column by column
    int id = blockIdx.x;
    const int ntiles = p.tiles_m * p.tiles_n;
    if (ntiles % 8 == 0) id = (id % 8) * (ntiles / 8) + id / 8;
    constexpr int GM = 8;
    const int group = id / (GM * p.tiles_n);
    const int first_m = group * GM;
    const int gm = min(GM, p.tiles_m - first_m);
    const int in_group = id - group * GM * p.tiles_n;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;
    const int outer = blockIdx.y / p.inner_count;
    const int inner = blockIdx.y % p.inner_count;
    const int8_t* __restrict__ A = p.A + outer * p.a_outer + inner * p.a_inner;
    const int8_t* __restrict__ W = p.W + outer * p.w_outer + inner * p.w_inner;
    const long obase = outer * p.o_outer + inner * p.o_inner;

    if (p.has_table) { if (p.table.cellmap) stage_table_two_level(s_kb, p.table); else stage_table(s_kb, p.table); }
    // per-column epilogue parameters of this tile go to LDS now (their latency hides behind the
    // main loop) so that the epilogue itself issues no global loads for them
    if (kEpi != EPI_ACC) {
        for (int t = tid; t < BN; t += 64 * NW) {
            const int n = n0 + t;
            float sc = p.alpha, bi = 0.0f, iv = p.out_inv_scale;
            if (n < p.N) {
                if (p.bias) bi = p.bias[n];
                if (p.alpha_vec) sc = p.alpha_vec[n];
                if (kEpi == EPI_GENERIC && p.out_inv_scale_vec) iv = p.out_inv_scale_vec[n];
                else if (p.split_cols > 0) iv = n >= 2 * p.split_cols ? p.inv3[2] : (n >= p.split_cols ? p.inv3[1] : p.inv3[0]);
            }
            s_cols[t] = sc;
            s_cols[BN + t] = bi;
            s_cols[2 * BN + t] = iv;
        }
    }

    // per-lane source pointers of this wavefront's blocks (k = 0)
    const int8_t* src[LB];
    int conv_h[LB], conv_w[LB];  // kConv, A rows: top-left input coordinate of the lane's output position
    const bool has_last = wave + (LB - 1) * NW < NBLK;  // wave-uniform
#pragma unroll
    for (int b = 0; b < LB; ++b) {
        int blk = wave + b * NW;
        if (blk >= NBLK) blk = wave;  // unused slot
        const int r = blk * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ swz_bk<BK>(r);
        conv_h[b] = 0; conv_w[b] = 0;
        if (r < BM) {
            const int m = min(m0 + r, p.M - 1);
            if (kConv) {
                const int wo = m % p.cWo, t = m / p.cWo;
                const int ho = t % p.cHo, bi = t / p.cHo;
                conv_h[b] = ho * p.cStride - p.cPad;
                conv_w[b] = wo * p.cStride - p.cPad;
                src[b] = A + (long)bi * p.cH * p.cW * p.cCin + 16 * chunk;  // image base + chunk
            } else {
                src[b] = A + (long)m * p.lda + 16 * chunk;
            }
        } else {
            src[b] = W + (long)min(n0 + r - BM, p.N - 1) * p.ldw + 16 * chunk;
        }
    }
    const unsigned lds_base = (unsigned)(uintptr_t)smem;
    // Issue the loads of k-slice kt into ring slot `stage`; with parts > 1 only the blocks b with
    // b % parts == part, so that the issue slots can be spread between the MFMAs of the main loop
    // (a wavefront issues in order: a burst of LB loads would stall its MFMA stream).
    // kConv: slices are issued in increasing kt, so the tap (ti, tj) and the channel offset tc of
    // the slice being issued are kept as running (wave-uniform) counters.
    int ti = 0, tj = 0, tc = 0;
    const int8_t* zero_src = g_zero_line + 16 * (lane % CPR);
    auto issue = [&](int kt, int stage, int part, int parts) {
        const unsigned dst = lds_base + stage * STAGE_BYTES + wave * 1024;
#pragma unroll
        for (int b = 0; b < LB; ++b)
            if (b % parts == part && (b < LB - 1 || has_last)) {
                const int blk = wave + b * NW;
                if (kConv && blk * RPI < BM) {  // wave-uniform: an A block
                    // offsets inside one image fit 32 bits (checked on the host): cheap integer
                    // arithmetic and one select instead of 64-bit multiplies under a branch
                    const int hi = conv_h[b] + ti, wi = conv_w[b] + tj;
                    const bool inside = (unsigned)hi < (unsigned)p.cH && (unsigned)wi < (unsigned)p.cW;
                    const int off = (hi * p.cW + wi) * p.cCin + tc;
                    const int8_t* g = inside ? src[b] + off : zero_src;
                    dma16(g, dst + b * NW * 1024);
                } else {
                    dma16(src[b] + (long)kt * BK, dst + b * NW * 1024);
                }
            }
        if (kConv && part == parts - 1) {  // the slice is complete: advance to the next one
            tc += BK;
            if (tc == p.cCin) { tc = 0; if (++tj == p.cKw) { tj = 0; ++ti; } }
        }
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    // The specialised residual epilogues read the int8 residual rows this wavefront will finish
    // with 16-byte row loads, issued now so that they travel during the main loop; after it they
    // pass through the (then free) LDS patch to the lanes that need them.
    constexpr bool kResid8 = kEpi == EPI_F32_RESID || kEpi == EPI_Q_TABLE_RESID;
    constexpr int RCPR = WN / 16;                 // 16-byte chunks per residual row of the sub-tile
    constexpr int RCH = 32 * TMF * RCPR;          // chunks of the rows this wavefront finishes
    constexpr int RL = (RCH + 63) / 64;
    v4i rpre[RL];
    const bool resid_rows = kResid8 && p.r16;     // uniform
    if (resid_rows) {
#pragma unroll
        for (int t = 0; t < RL; ++t) {
            const int c = lane + 64 * t;
            rpre[t] = v4i{0, 0, 0, 0};
            if (c < RCH) {
                const int mr = m0 + wave_m + 32 * (kg * TMF) + c / RCPR, n = n0 + wave_n + 16 * (c % RCPR);
                if (mr < p.M && n + 15 < p.N)
                    rpre[t] = *reinterpret_cast<const v4i*>(p.resid + obase + (long)mr * p.ldo + n);
            }
        }
    }

    const int nk = p.K / BK;
#pragma unroll
    for (int st = 0; st < kStages - 1; ++st)
        if (st < nk) issue(st, st, 0, 1);

    const int frag_row = lane & 31, frag_half = lane >> 5;
    // LDS offsets of this lane's fragments inside a stage, per k-step this wavefront owns
    int offA[KSW][TM], offW[KSW][TN];
#pragma unroll
    for (int kk = 0; kk < KSW; ++kk) {
        const int ks = KSPLIT == 1 ? kk : kg + KSPLIT * kk;
#pragma unroll
        for (int i = 0; i < TM; ++i) offA[kk][i] = lds_off_bk<BK>(wave_m + 32 * i + frag_row, 2 * ks + frag_half);
#pragma unroll
        for (int j = 0; j < TN; ++j) offW[kk][j] = BM * BK + lds_off_bk<BK>(wave_n + 32 * j + frag_row, 2 * ks + frag_half);
    }
    int stage = 0;
    for (int kt = 0; kt < nk; ++kt) {
        // The loads of stage kt are older than those of the stages issued after it: wait until only
        // the younger ones are in flight.  `young` = number of younger stages already issued.
        const int young = min(kStages - 2, nk - 1 - kt);
        if (young <= 0) wait_vmcnt<0>();
        else if (young == 1) { if (has_last) wait_vmcnt<LB>(); else wait_vmcnt<LB - 1>(); }
        else { if (has_last) wait_vmcnt<2 * LB>(); else wait_vmcnt<2 * (LB - 1)>(); }
        __syncthreads();  // stage kt has landed for every wavefront; stage kt - 1 is free again
        int nxt = stage + kStages - 1;
        if (nxt >= kStages) nxt -= kStages;
        const bool more = kt + kStages - 1 < nk;
        const int8_t* st = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < KSW; ++kk) {
            v4i fa[TM], fw[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const v4i*>(st + offA[kk][i]);
#pragma unroll
            for (int j = 0; j < TN; ++j) fw[j] = *reinterpret_cast<const v4i*>(st + offW[kk][j]);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[j], fa[i], acc[i][j], 0, 0, 0);
            if (more) issue(kt + kStages - 1, nxt, kk, KSW);  // in the shadow of the MFMAs just issued
        }
        stage = stage + 1 == kStages ? 0 : stage + 1;
    }

    // ---- combine the two k-halves (KSPLIT == 2): swap accumulator halves through LDS ----------
    v16i fin[TMF][TN];
    __syncthreads();  // every wavefront is done with the ring
    if (KSPLIT == 2) {
        int* xch = reinterpret_cast<int*>(smem);
        const int mine = (wave_t * 2 + kg) * (TMF * TN * 1024), other = (wave_t * 2 + (1 - kg)) * (TMF * TN * 1024);
#pragma unroll
        for (int i = 0; i < TMF; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)  // give away the row blocks the partner finishes
                    xch[mine + ((i * TN + j) * 16 + v) * 64 + lane] = kg == 0 ? acc[TMF + i][j][v] : acc[i][j][v];
        __syncthreads();
#pragma unroll
        for (int i = 0; i < TMF; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    fin[i][j][v] = (kg == 0 ? acc[i][j][v] : acc[TMF + i][j][v]) + xch[other + ((i * TN + j) * 16 + v) * 64 + lane];
        __syncthreads();  // the exchange area is about to become the output patch
    } else {
#pragma unroll
        for (int i = 0; i < TMF; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j) fin[i][j] = acc[i][j];
    }
    const int row_blk0 = kg * TMF;  // first 32-row block of the sub-tile this wavefront finishes

    // ---- epilogue ------------------------------------------------------------------------------
    const bool patch_q = (kEpi == EPI_GENERIC || kEpi == EPI_Q || kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID) &&
                         p.out_q != nullptr && p.q16;  // uniform: int8 rows leave through LDS
    int8_t* patch = smem + wave_t * (WM * SW);
    // the specialised residual epilogue fetches all of the lane's residual words up front
    unsigned resw[TMF][TN][4];
    if (resid_rows) {
#pragma unroll
        for (int t = 0; t < RL; ++t) {
            const int c = lane + 64 * t;
            if (c < RCH) *reinterpret_cast<v4i*>(patch + (32 * row_blk0 + c / RCPR) * SW + 16 * (c % RCPR)) = rpre[t];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int i = 0; i < TMF; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g)
                    resw[i][j][g] = *reinterpret_cast<const unsigned*>(
                        patch + (32 * (row_blk0 + i) + frag_row) * SW + 32 * j + 8 * g + 4 * frag_half);
        // the patch is reused for the output rows: every lane's reads come first
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    } else if (kEpi == EPI_F32_RESID || kEpi == EPI_Q_TABLE_RESID) {
#pragma unroll
        for (int i = 0; i < TMF; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int m = m0 + wave_m + 32 * (row_blk0 + i) + frag_row;
                    const int nb = n0 + wave_n + 32 * j + 8 * g + 4 * frag_half;
                    resw[i][j][g] = 0;
                    if (m < p.M && nb + 3 < p.N)
                        resw[i][j][g] = *reinterpret_cast<const unsigned*>(p.resid + obase + (long)m * p.ldo + nb);
                }
    }
    // Row blocks outermost: as soon as a block of 32 rows is finished its int8 rows are read back
    // from the patch and stored, so the stores of one block overlap the arithmetic of the next
    // (the patch rows of a block are written and read by the same wavefront: no workgroup barrier).
    // The body exists twice: for a tile that lies wholly inside the output (and vector-aligned
    // outputs) every bounds test is a compile-time constant, which leaves straight-line code whose
    // table look-ups the scheduler can batch; edge tiles take the guarded copy.
    auto finish_rows = [&](auto full_c, auto two_c) {
        constexpr bool kFullTile = decltype(full_c)::value;
        constexpr bool kTwoSeg = decltype(two_c)::value;   // two-segment table: compare instead of gather
#pragma unroll
        for (int i = 0; i < TMF; ++i) {
            const int prow = 32 * (row_blk0 + i) + frag_row;  // row inside the sub-tile
            const int m = m0 + wave_m + prow;
            const long rowoff = obase + (long)m * p.ldo;
#pragma unroll
            for (int j = 0; j < TN; ++j) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int cl = wave_n + 32 * j + 8 * g + 4 * frag_half;  // column inside the tile
                    const int nb = n0 + cl;
                    if (!kFullTile && (nb >= p.N || m >= p.M)) continue;
                    const bool vec = kFullTile || (p.vec_out && nb + 3 < p.N);
                    Col4 c;
                    {
                        const v4f sc = *reinterpret_cast<const v4f*>(s_cols + cl);
                        const v4f bi = *reinterpret_cast<const v4f*>(s_cols + BN + cl);
                        const v4f iv = *reinterpret_cast<const v4f*>(s_cols + 2 * BN + cl);
#pragma unroll
                        for (int e = 0; e < 4; ++e) { c.scale[e] = sc[e]; c.bias[e] = bi[e]; c.inv[e] = iv[e]; }
                    }
                    int a4[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) a4[e] = fin[i][j][4 * g + e];
                    int r4[4] = {0, 0, 0, 0};
                    if (kEpi == EPI_F32_RESID || kEpi == EPI_Q_TABLE_RESID) {
                        if (kFullTile || nb + 3 < p.N) {
#pragma unroll
                            for (int e = 0; e < 4; ++e) r4[e] = (int)(int8_t)(resw[i][j][g] >> (8 * e));
                        } else {
                            load_resid4(p, rowoff, nb, false, r4);
                        }
                    } else if (kEpi == EPI_GENERIC && p.resid) {
                        load_resid4(p, rowoff, nb, vec, r4);
                    }
                    Epi4 o;
                    epi_math<kEpi, kTwoSeg>(p, s_kb, a4, c, r4, o);
                    epi_store<kEpi>(p, rowoff, nb, a4, o, vec, patch_q);
                    if (patch_q)
                        *reinterpret_cast<unsigned*>(patch + prow * SW + 32 * j + 8 * g + 4 * frag_half) =
                            pack4(o.q[0], o.q[1], o.q[2], o.q[3]);
                }
            }
            if (patch_q) {
                // same wavefront wrote these 32 patch rows: order its LDS writes before its reads
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                constexpr int PCPR = WN / 16;  // 16-byte chunks per patch row
                for (int c = lane; c < 32 * PCPR; c += 64) {
                    const int row = 32 * (row_blk0 + i) + c / PCPR, cc = c % PCPR;
                    const int mr = m0 + wave_m + row, n = n0 + wave_n + 16 * cc;
                    if (kFullTile || (mr < p.M && n < p.N)) {
                        const v4i v = *reinterpret_cast<const v4i*>(patch + row * SW + 16 * cc);
                        int8_t* dst = p.out_q + obase + (long)mr * p.ldo + n;
                        if (kFullTile || n + 15 < p.N) {
                            *reinterpret_cast<v4i*>(dst) = v;
                        } else {
                            for (int b = 0; b < 16 && n + b < p.N; ++b)
                                dst[b] = (int8_t)((unsigned)v[b >> 2] >> (8 * (b & 3)));
                        }
                    }
                }
            }
        }
    };
    constexpr bool kTableEpi = kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE_RESID;
    if (m0 + BM <= p.M && n0 + BN <= p.N && p.vec_out) {
        if (kTableEpi && p.table.two_seg) finish_rows(std::true_type{}, std::integral_constant<bool, kTableEpi>{});
        else finish_rows(std::true_type{}, std::false_type{});
    } else {
        finish_rows(std::false_type{}, std::false_type{});
    }
}

template <int BM, int BN, int WM, int WN>
static void launch_cfg(const GemmParams& p, bool al, bool wkn, dim3 grid, size_t shmem, hipStream_t s)
{
    if (al && !wkn) hipLaunchKernelGGL((gemm_pwl_kernel<BM, BN, WM, WN, true, false>), grid, dim3(kGemmThreads), shmem, s, p);
    else if (!al && !wkn) hipLaunchKernelGGL((gemm_pwl_kernel<BM, BN, WM, WN, false, false>), grid, dim3(kGemmThreads), shmem, s, p);
    else if (al && wkn) hipLaunchKernelGGL((gemm_pwl_kernel<BM, BN, WM, WN, true, true>), grid, dim3(kGemmThreads), shmem, s, p);
    else hipLaunchKernelGGL((gemm_pwl_kernel<BM, BN, WM, WN, false, true>), grid, dim3(kGemmThreads), shmem, s, p);
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int KSPLIT, int BK, int kStages, int kEpi, bool kConv = false>
static int32_t launch_stream_epi(GemmParams& p, int batches, size_t table_bytes, hipStream_t s)
{
    auto kern = gemm_stream_kernel<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, kEpi, kConv>;
    const size_t shmem = (size_t)kStages * (BM + BN) * BK + 3 * BN * sizeof(float) + table_bytes;
    static std::once_flag once;  // one attribute call per instantiation
    static int32_t once_rc = NM_OK;
    std::call_once(once, [&] {
        once_rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
                            "hipFuncSetAttribute(gemm_stream_kernel)");
    });
    if (once_rc) return once_rc;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n, batches), dim3(64 * WAVES_M * WAVES_N * KSPLIT), shmem, s, p);
    return NM_OK;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int KSPLIT, int BK, int kStages>
static int32_t launch_stream(GemmParams& p, int epi, int batches, size_t table_bytes, hipStream_t s)
{
    switch (epi) {
    case EPI_Q: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q>(p, batches, table_bytes, s);
    case EPI_Q_TABLE: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q_TABLE>(p, batches, table_bytes, s);
    case EPI_F32_RESID: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_F32_RESID>(p, batches, table_bytes, s);
    case EPI_Q_TABLE_RESID: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q_TABLE_RESID>(p, batches, table_bytes, s);
    case EPI_ACC: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_ACC>(p, batches, table_bytes, s);
    default: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_GENERIC>(p, batches, table_bytes, s);
    }
}

// Convolutions use three epilogues (everything else falls to the generic one).
template <int BM, int BN, int WAVES_M, int WAVES_N, int KSPLIT, int BK, int kStages>
static int32_t launch_stream_conv(GemmParams& p, int epi, size_t table_bytes, hipStream_t s)
{
    switch (epi) {
    case EPI_Q: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q, true>(p, 1, table_bytes, s);
    case EPI_Q_TABLE: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q_TABLE, true>(p, 1, table_bytes, s);
    case EPI_Q_TABLE_RESID: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_Q_TABLE_RESID, true>(p, 1, table_bytes, s);
    default: return launch_stream_epi<BM, BN, WAVES_M, WAVES_N, KSPLIT, BK, kStages, EPI_GENERIC, true>(p, 1, table_bytes, s);
    }
}

// The LayerNorm-folding kernel: workgroups of 64 rows x all N columns (eight wavefronts, each all 64
// rows of N / 8 columns), 64-byte k-slices so that two ring stages of 64 + N rows fit LDS.
bool gemm_folds_layernorm(const GemmArgs& g)
{
    if (force_generic() || g.conv || g.w_is_kn || g.outer_count * g.inner_count != 1) return false;
    if (g.N != 768 && g.N != 1024) return false;
    if (g.K % 64 != 0 || g.K / 64 < 3 || g.alpha_vec || g.has_table || !g.resid || !g.ln_gamma || !g.ln_beta) return false;
    if (!(g.ln_out_q || g.ln_out_f32)) return false;
    const bool al = aligned(g.A, 16) && g.lda % 16 == 0 && aligned(g.W, 16) && g.ldw % 16 == 0 && aligned(g.resid, 16) &&
                    g.ldo == g.N && aligned(g.ln_gamma, 16) && aligned(g.ln_beta, 16) &&
                    (!g.ln_out_q || aligned(g.ln_out_q, 16)) && (!g.ln_out_f32 || aligned(g.ln_out_f32, 16)) &&
                    (!g.bias || aligned(g.bias, 4));
    return al && (int64_t)g.M * g.lda < (1LL << 32) && (int64_t)g.N * g.ldw < (1LL << 32);
}

int32_t launch_gemm(const GemmArgs& g, hipStream_t stream)
{
    if (g.M == 0) return NM_OK;
    if (g.ln) {
        if (!gemm_folds_layernorm(g)) return fail(NM_ERR_UNSUPPORTED, "gemm: this shape does not fold the LayerNorm");
        GemmParams q{};
        q.M = g.M; q.N = g.N; q.K = g.K; q.A = g.A; q.lda = g.lda; q.W = g.W; q.ldw = g.ldw; q.inner_count = 1;
        q.bias = g.bias; q.alpha = g.alpha; q.resid = g.resid; q.resid_scale = g.resid_scale; q.ldo = g.ldo;
        q.ln_gamma = g.ln_gamma; q.ln_beta = g.ln_beta; q.ln_eps = g.ln_eps; q.ln_inv_scale = g.ln_inv_scale;
        q.ln_table = g.ln_table; q.ln_out_q = g.ln_out_q; q.ln_out_f32 = g.ln_out_f32;
        int32_t rc = g.N == 768 ? launch_tile_epi<64, 768, 1, 8, 2, EPI_F32_RESID_LN, 64>(q, 0, stream)
                                : launch_tile_epi<64, 1024, 1, 8, 2, EPI_F32_RESID_LN, 64>(q, 0, stream);
        if (rc) return rc;
        return check_hip(hipGetLastError(), "gemm + LayerNorm launch");
    }
    GemmParams p{};
    p.M = g.M; p.N = g.N; p.K = g.K;
    p.A = g.A; p.lda = g.lda; p.W = g.W; p.ldw = g.ldw;
    p.inner_count = g.inner_count;
    p.a_outer = g.a_outer; p.a_inner = g.a_inner; p.w_outer = g.w_outer; p.w_inner = g.w_inner;
    p.o_outer = g.o_outer; p.o_inner = g.o_inner;
    p.bias = g.bias; p.alpha_vec = g.alpha_vec; p.alpha = g.alpha;
    p.resid = g.resid; p.resid_scale = g.resid_scale;
    p.has_table = g.has_table; p.table = g.table;
    p.out_inv_scale = g.out_inv_scale; p.out_inv_scale_vec = g.out_inv_scale_vec;
    p.split_cols = g.split_cols;
    for (int i = 0; i < 3; ++i) p.inv3[i] = g.inv3[i];
    p.ldo = g.ldo;
    p.cH = g.cH; p.cW = g.cW; p.cCin = g.cCin; p.cKw = g.cKw; p.cStride = g.cStride; p.cPad = g.cPad;
    p.cHo = g.cHo; p.cWo = g.cWo;
    p.out_q = g.out_q; p.out_f32 = g.out_f32; p.out_acc = g.out_acc; p.dbg_seg = g.dbg_seg;
    p.ln_gamma = g.ln_gamma; p.ln_beta = g.ln_beta; p.ln_eps = g.ln_eps; p.ln_inv_scale = g.ln_inv_scale;
    p.ln_table = g.ln_table; p.ln_out_q = g.ln_out_q; p.ln_out_f32 = g.ln_out_f32;

    // 16-byte loads need every row start and every batch offset on a 16-byte boundary
    const bool a_al = aligned(g.A, 16) && g.lda % 16 == 0 && g.a_outer % 16 == 0 && g.a_inner % 16 == 0;
    const bool w_al = aligned(g.W, 16) && g.ldw % 16 == 0 && g.w_outer % 16 == 0 && g.w_inner % 16 == 0;
    const bool al = a_al && w_al && g.K % 16 == 0 && (!g.w_is_kn || g.N % 16 == 0);
    p.vec_out = g.ldo % 4 == 0 && g.o_outer % 4 == 0 && g.o_inner % 4 == 0 &&
                (!g.out_q || aligned(g.out_q, 4)) && (!g.out_f32 || aligned(g.out_f32, 16)) &&
                (!g.out_acc || aligned(g.out_acc, 16)) && (!g.dbg_seg || aligned(g.dbg_seg, 8)) &&
                (!g.resid || aligned(g.resid, 4));
    p.r16 = g.resid && aligned(g.resid, 16) && g.ldo % 16 == 0 && g.o_outer % 16 == 0 && g.o_inner % 16 == 0 && g.N % 16 == 0;
    p.q16 = g.out_q && aligned(g.out_q, 16) && g.ldo % 16 == 0 && g.o_outer % 16 == 0 && g.o_inner % 16 == 0;

    // LDS bytes of the table: {k, b} per segment, or for the two-level form of a merged table one
    // {k, b} per merged segment plus a byte per primary cell
    const size_t table_bytes = !g.has_table ? 0
                             : g.table.cellmap ? 8 * (size_t)g.table.nkb + (((size_t)g.table.nseg + 7) & ~(size_t)7)
                                               : sizeof(float2) * (size_t)g.table.nseg;
    const int batches = g.outer_count * g.inner_count;
    if (batches > 65535) return fail(NM_ERR_UNSUPPORTED, "gemm: more than 65535 batched problems");
    int32_t rc = NM_OK;
    p.vec_cols = (!g.bias || aligned(g.bias, 16)) && (!g.alpha_vec || aligned(g.alpha_vec, 16)) &&
                 (!g.out_inv_scale_vec || aligned(g.out_inv_scale_vec, 16));
    int epi = EPI_GENERIC;
    if (!g.out_inv_scale_vec && !g.dbg_seg && !(g.has_table && g.table.cellmap)) {
        const bool only_q = g.out_q && !g.out_f32 && !g.out_acc;
        // EPI_Q_TABLE is compiled without the input clamp; a table with that flag takes the generic epilogue
        if (only_q && !g.resid) epi = !g.has_table ? EPI_Q : g.table.clamp_input ? EPI_GENERIC : EPI_Q_TABLE;
        else if (g.out_f32 && !g.out_q && !g.out_acc && g.resid && !g.has_table && p.vec_out) epi = EPI_F32_RESID;
        else if (only_q && g.resid && g.has_table && !g.table.clamp_input && p.vec_out) epi = EPI_Q_TABLE_RESID;
        else if (g.out_acc && !g.out_q && !g.out_f32) epi = EPI_ACC;
    }
    // Tile configuration, from same-process timings of every configuration on the shapes of the
    // workloads.  NARROW (256x64) for outputs of at most 64 columns.  Wide outputs (N >= 1536): BIG
    // (256x192, two 128-byte stages, one workgroup per CU) when its tiles fill whole rounds of the
    // 256 CUs to at least 90 %, WIDE (256x128 with 128x64 wavefront tiles, 48 KB ring) when those come six or more to a CU.
    // Otherwise by the number of 128x128 tiles: three or more per CU -> MID2 (two 64-byte stages,
    // 32 KB: four workgroups share a CU and one's epilogue overlaps another's loads); 1.25 to 3 per
    // CU -> MID3 (three stages), or SMALL (64x128, two wavefronts per sub-tile on alternate
    // k-steps, 128-byte slices) for long contractions; fewer -> SPLIT (128x128, same scheme), or
    // SMALL when even those would leave more than a third of the CUs idle.
    const bool k128 = g.K % 128 == 0 && (!g.conv || g.cCin % 128 == 0);  // 128-byte k-slices fetch ~1.5x faster
    const long big_tiles = (long)((g.M + 255) / 256) * ((g.N + 191) / 192) * batches;
    const long mid_tiles = (long)((g.M + 127) / 128) * ((g.N + 127) / 128) * batches;
    const long wide_tiles = (long)((g.M + 255) / 256) * ((g.N + 127) / 128) * batches;
    const bool split_ok = k128 && table_bytes <= 32768;
    // share of CU slots the BIG tiles use over their rounds (one workgroup per CU; a single partly
    // filled round counts as full: there is nothing better to do with the idle CUs)
    const double big_fill = big_tiles <= 256 ? 1.0 : (double)big_tiles / (double)((big_tiles + 255) / 256 * 256);
    enum { CFG_BIG, CFG_WIDE, CFG_SPLIT, CFG_SMALL, CFG_MID3, CFG_MID2, CFG_NARROW } cfg;
    if (g.N <= 64) cfg = CFG_NARROW;
    else if (g.N >= 1536 && g.K > 256 && wide_tiles >= 1536) cfg = CFG_WIDE;
    else if (!g.conv && k128 && g.N >= 1536 && big_tiles >= 192 && big_fill >= 0.9) cfg = CFG_BIG;
    else if (mid_tiles >= 768) cfg = CFG_MID2;
    else if (mid_tiles >= 320) cfg = (split_ok && g.K >= 2048) ? CFG_SMALL : CFG_MID3;
    else if (split_ok) cfg = (mid_tiles < 160 && g.M > 64) ? CFG_SMALL : CFG_SPLIT;
    else cfg = CFG_MID3;
    bool old_big = false;
    if (g.N > 64) {
        const int f = forced_cfg();
        if (f == 6 && !g.conv && k128) { cfg = CFG_BIG; old_big = true; }
        if (f == 0 && !g.conv && k128) cfg = CFG_BIG;
        else if (f == 1) cfg = CFG_WIDE;
        else if (f == 2 && split_ok) cfg = CFG_SPLIT;
        else if (f == 3 && split_ok) cfg = CFG_SMALL;
        else if (f == 4) cfg = CFG_MID3;
        else if (f == 5) cfg = CFG_MID2;
    }
    if (g.conv) {
        // gathered A operand: streaming kernel only (the caller has checked Cin % 64 == 0, 16-byte
        // aligned image and weights); one problem, no batching
        if (!w_al || !aligned(g.A, 16) || g.cCin % 64 != 0 || g.K % (g.cCin * g.cKw) != 0)
            return fail(NM_ERR_UNSUPPORTED, "conv gemm: operands not aligned for the gathered loader");
        if (cfg == CFG_NARROW) rc = launch_stream_conv<256, 64, 4, 1, 1, 64, 2>(p, epi, table_bytes, stream);
        else if (cfg == CFG_WIDE) rc = launch_stream_conv<256, 128, 2, 2, 1, 64, 2>(p, epi, table_bytes, stream);
        else if (cfg == CFG_MID2) rc = launch_stream_conv<128, 128, 2, 2, 1, 64, 2>(p, epi, table_bytes, stream);
        else if (cfg == CFG_SPLIT) rc = launch_stream_conv<128, 128, 2, 2, 2, 128, 3>(p, epi, table_bytes, stream);
        else if (cfg == CFG_SMALL) rc = launch_stream_conv<64, 128, 1, 2, 2, 128, 3>(p, epi, table_bytes, stream);
        else rc = launch_stream_conv<128, 128, 2, 2, 1, 64, 3>(p, epi, table_bytes, stream);
        if (rc) return rc;
        return check_hip(hipGetLastError(), "conv gemm launch");
    }
    const bool stream_ok = al && !g.w_is_kn && g.K % 64 == 0 && !force_generic();
    // the tile kernel: plain matrix products with the encoder layer's epilogues
    // int8 output through a merged table kept in two levels: the tile kernel has an epilogue for it
    // (elsewhere the generic one looks it up)
    const bool two_level_q = g.has_table && g.table.cellmap && !g.table.clamp_input && g.out_q && !g.out_f32 &&
                             !g.out_acc && !g.resid && !g.out_inv_scale_vec && !g.dbg_seg && g.table.nkb <= 256 &&
                             g.table.nseg <= 1024;
    const bool tile_epi = (epi == EPI_Q || epi == EPI_Q_TABLE || two_level_q) ? p.q16 != 0
                        : epi == EPI_F32_RESID ? (p.r16 != 0 && aligned(g.out_f32, 16) && g.ldo % 4 == 0) : false;
    const bool tile_ok = stream_ok && tile_epi && batches == 1 && g.K % 128 == 0 && g.K / 128 >= 3 && !g.alpha_vec &&
                         g.N % 16 == 0 && g.split_cols % 4 == 0 && (int64_t)g.M * g.lda < (1LL << 32) &&
                         (int64_t)g.N * g.ldw < (1LL << 32) && table_bytes <= 40 * 1024;
    // Which tile: the one whose workgroups fill whole rounds of the 256 CUs best, weighted by how much
    // operand traffic per matrix instruction the tile shape costs (weights from timings of the
    // encoder shapes: 256x192 1.0, 256x128 0.92, 128x192 0.85, 128x128 0.75) and by the share of the
    // tiles' area that lies inside the output.
    int tile_cfg = -1;
    if (tile_ok && !old_big && forced_cfg() < 0) {
        static const struct { int bm, bn, stages; double quality; } kTiles[4] = {
            {256, 192, 2, 1.0}, {256, 128, 3, 0.92}, {128, 192, 3, 0.85}, {128, 128, 3, 0.75}};
        double best = 0.0;
        for (int c = 0; c < 4; ++c) {
            if (g.K / 128 < kTiles[c].stages + 1) continue;
            const long tm = (g.M + kTiles[c].bm - 1) / kTiles[c].bm, tn = (g.N + kTiles[c].bn - 1) / kTiles[c].bn;
            const long tiles = tm * tn, slots = (tiles + 255) / 256 * 256;
            const double inside = (double)g.M * g.N / ((double)tiles * kTiles[c].bm * kTiles[c].bn);
            const double score = (double)tiles / (double)slots * inside * kTiles[c].quality;
            if (score > best) { best = score; tile_cfg = c; }
        }
        // small problems stay with the streaming kernel's small tiles
        if ((long)g.M * g.N < 128L * 128 * 96) tile_cfg = -1;
    } else if (tile_ok && !old_big && forced_cfg() == 0 && g.K / 128 >= 3) {
        tile_cfg = 0;
    }
    if (tile_cfg >= 0 && two_level_q) epi = EPI_Q_TABLE2;
    if (tile_cfg == 0) {
        rc = launch_tile<256, 192, 4, 2, 2>(p, epi, table_bytes, stream);
    } else if (tile_cfg == 1) {
        rc = launch_tile<256, 128, 4, 2, 3>(p, epi, table_bytes, stream);
    } else if (tile_cfg == 2) {
        rc = launch_tile<128, 192, 2, 2, 3>(p, epi, table_bytes, stream);
    } else if (tile_cfg == 3) {
        rc = launch_tile<128, 128, 2, 2, 3>(p, epi, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_WIDE) {
        rc = launch_stream<256, 128, 2, 2, 1, 64, 2>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_BIG) {
        rc = launch_stream<256, 192, 4, 2, 1, 128, 2>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_MID2) {
        rc = launch_stream<128, 128, 2, 2, 1, 64, 2>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_SMALL) {
        rc = launch_stream<64, 128, 1, 2, 2, 128, 3>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_SPLIT) {
        rc = launch_stream<128, 128, 2, 2, 2, 128, 3>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && cfg == CFG_MID3) {
        rc = launch_stream<128, 128, 2, 2, 1, 64, 3>(p, epi, batches, table_bytes, stream);
    } else if (stream_ok && g.N > 32 && g.M >= 1024) {
        // narrow outputs with many rows (the 64-channel convolutions of a residual CNN)
        rc = launch_stream<256, 64, 4, 1, 1, 64, 2>(p, epi, batches, table_bytes, stream);
    } else if (g.N <= 64) {
        p.tiles_m = (g.M + 127) / 128; p.tiles_n = (g.N + 63) / 64;
        launch_cfg<128, 64, 32, 64>(p, al, g.w_is_kn, dim3(p.tiles_m * p.tiles_n, batches), table_bytes, stream);
    } else {
        p.tiles_m = (g.M + 127) / 128; p.tiles_n = (g.N + 127) / 128;
        launch_cfg<128, 128, 64, 64>(p, al, g.w_is_kn, dim3(p.tiles_m * p.tiles_n, batches), table_bytes, stream);
    }
    if (rc) return rc;
    return check_hip(hipGetLastError(), "gemm launch");
}

}  // namespace nm

using namespace nm;

extern "C" {

int32_t nm_gemm_pwl(const nm_gemm_desc* d, void* stream)
{
    if (!d) return fail(NM_ERR_INVALID_ARG, "nm_gemm_pwl: desc is NULL");
    if (d->M < 1 || d->N < 1 || d->K < 1) return fail(NM_ERR_INVALID_ARG, "nm_gemm_pwl: M, N, K must be >= 1");
    if (!d->A || !d->W) return fail(NM_ERR_INVALID_ARG, "nm_gemm_pwl: A or W is NULL");
    if (!d->out_q && !d->out_f32 && !d->out_acc) return fail(NM_ERR_INVALID_ARG, "nm_gemm_pwl: no output");
    if (d->K > 65536) return fail(NM_ERR_UNSUPPORTED, "nm_gemm_pwl: K %d > 65536", d->K);
    if ((int64_t)d->M * d->N >= (1LL << 31)) return fail(NM_ERR_UNSUPPORTED, "nm_gemm_pwl: M*N >= 2^31");
    if (d->split_cols < 0 || (d->split_cols > 0 && d->out_inv_scale_vec))
        return fail(NM_ERR_INVALID_ARG, "nm_gemm_pwl: split_cols must be >= 0 and excludes out_inv_scale_vec");
    GemmArgs g;
    g.M = d->M; g.N = d->N; g.K = d->K;
    g.A = d->A; g.lda = d->K; g.W = d->W; g.ldw = d->K;
    g.bias = d->bias; g.alpha_vec = d->alpha_vec; g.alpha = d->alpha;
    g.resid = d->resid; g.resid_scale = d->resid_scale;
    if (d->table_idx >= 0) {
        int32_t rc = get_dev_table(d->tables, d->table_idx, &g.table, "nm_gemm_pwl", true);
        if (rc) return rc;
        g.has_table = 1;
    }
    g.out_inv_scale = d->out_inv_scale; g.out_inv_scale_vec = d->out_inv_scale_vec;
    g.split_cols = d->split_cols;
    for (int i = 0; i < 3; ++i) g.inv3[i] = d->out_inv_scale3[i];
    g.ldo = d->N;
    g.out_q = d->out_q; g.out_f32 = d->out_f32; g.out_acc = d->out_acc; g.dbg_seg = d->dbg_seg;
    return launch_gemm(g, (hipStream_t)stream);
}

static int32_t check_attn(const char* what, const void* a, const void* b, const void* c, int32_t B,
                          int32_t S, int32_t H, int32_t heads)
{
    if (!a || !b || !c) return fail(NM_ERR_INVALID_ARG, "%s: NULL pointer", what);
    if (B < 1 || S < 1 || H < 1 || heads < 1) return fail(NM_ERR_INVALID_ARG, "%s: dimensions must be >= 1", what);
    if (H % heads != 0) return fail(NM_ERR_INVALID_ARG, "%s: H %d not divisible by heads %d", what, H, heads);
    if (S > 4096) return fail(NM_ERR_UNSUPPORTED, "%s: S %d > 4096", what, S);
    if ((int64_t)B * heads > 65535) return fail(NM_ERR_UNSUPPORTED, "%s: B * heads > 65535", what);
    if ((int64_t)B * S * 3 * H >= (1LL << 31)) return fail(NM_ERR_UNSUPPORTED, "%s: B*S*3H >= 2^31", what);
    return NM_OK;
}

int32_t nm_attn_scores(const int8_t* qkv, int32_t B, int32_t S, int32_t H, int32_t heads,
                       int32_t* scores, void* stream)
{
    int32_t rc = check_attn("nm_attn_scores", qkv, qkv, scores, B, S, H, heads);
    if (rc) return rc;
    const int d = H / heads;
    GemmArgs g;
    g.M = S; g.N = S; g.K = d;
    g.A = qkv; g.lda = 3L * H; g.W = qkv + H; g.ldw = 3L * H;
    g.outer_count = B; g.inner_count = heads;
    g.a_outer = (long)S * 3 * H; g.a_inner = d;
    g.w_outer = (long)S * 3 * H; g.w_inner = d;
    g.o_outer = (long)heads * S * S; g.o_inner = (long)S * S;
    g.ldo = S;
    g.out_acc = scores;
    return launch_gemm(g, (hipStream_t)stream);
}

int32_t nm_attn_context(const int8_t* p, const int8_t* qkv, int32_t B, int32_t S, int32_t H,
                        int32_t heads, float alpha, float out_inv_scale, int8_t* ctx, void* stream)
{
    int32_t rc = check_attn("nm_attn_context", p, qkv, ctx, B, S, H, heads);
    if (rc) return rc;
    const int d = H / heads;
    GemmArgs g;
    g.M = S; g.N = d; g.K = S;
    g.A = p; g.lda = S;
    g.W = qkv + 2L * H; g.ldw = 3L * H; g.w_is_kn = 1;  // V is [S, d] per head: k = j runs over rows
    g.outer_count = B; g.inner_count = heads;
    g.a_outer = (long)heads * S * S; g.a_inner = (long)S * S;
    g.w_outer = (long)S * 3 * H; g.w_inner = d;
    g.o_outer = (long)S * H; g.o_inner = d;
    g.ldo = H;
    g.alpha = alpha; g.out_inv_scale = out_inv_scale;
    g.out_q = ctx;
    return launch_gemm(g, (hipStream_t)stream);
}

}  // extern "C"
