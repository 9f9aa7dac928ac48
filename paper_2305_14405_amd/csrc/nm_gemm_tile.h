// The large-tile int8 GEMM kernel (paper Section 3.1: fully connected layers as matrix products;
// Section 3.2: the nonlinearity behind one is the PWL calculation y = k[s]*x + b[s]).
#pragma once

#include "nm_gemm_common.h"

namespace nm {

// ---------------------------------------------------------------------------------------------
// Tile kernel: the large-tile path for the plain matrix products of the encoder layer (aligned
// operands, K a multiple of 128, scalar alpha, int8 output with or without the table, or fp32
// output with the int8 residual).  Same LDS image and MFMA operand roles as the streaming kernel;
// what differs is how the instruction stream is laid out:
//  * the k-loop is software-pipelined by hand and its issue order is pinned with scheduling
//    barriers: one matrix instruction, then at most one LDS fragment read (for the NEXT k-step, into
//    the other of two fragment register sets) and one global -> LDS load in its shadow.  A wavefront
//    therefore never waits for a fragment it has just asked for, and the one barrier per k-slice
//    sits in the middle of a k-step whose fragments are already in registers;
//  * a k-slice's ring slot is refilled right after that barrier (all of its fragments have been
//    read by then), addresses are one scalar base per operand plus a 32-bit lane offset;
//  * first slice, steady state and the last slices are straight-line code around one loop, so the
//    accumulators stay in the same registers throughout;
//  * the per-column vectors and the table are fetched when the kernel starts but written to LDS
//    after the k-loop (nothing in front of the first operand slice waits for them);
//  * the epilogue works on groups of four columns; the table look-up of a group is issued three
//    groups before its result is used, and int8 rows leave through an LDS patch as 16-byte stores.
// Eight wavefronts as 4 x 2 (64 x 96 each) keep two wavefronts on every SIMD: the fp32 epilogue
// issues almost twice as fast that way as with four wavefronts of 128 x 96 (measured: a single
// wavefront cannot issue dependent-free vector instructions back to back at the SIMD's full rate).
// ---------------------------------------------------------------------------------------------
template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int kEpi, int BK = 128>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 1) void gemm_tile_kernel(GemmParams p)
{
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;
    constexpr int TM = WM / 32, TN = WN / 32;
    constexpr int ROWS = BM + BN;
    constexpr int CPR = BK / 16;
    constexpr int RPI = 64 / CPR;
    constexpr int NBLK = ROWS / RPI;         // 1 KB blocks of a k-slice
    constexpr int LB = (NBLK + NW - 1) / NW; // ... per wavefront: when they do not split evenly the last
                                             // ones are fetched twice into spare LDS behind the stage
    constexpr int ABLK = BM / RPI;           // blocks that hold A rows
    constexpr bool kEven = NBLK % NW == 0 && ABLK % NW == 0;
    constexpr int LBA = ABLK / NW;           // A blocks per wavefront (even split)
    constexpr int STAGE_BYTES = LB * NW * 1024;
    constexpr int KS = BK / 32;
    constexpr int NR = TM + TN;              // fragments per k-step
    constexpr int NMF = TM * TN;             // matrix instructions per k-step
    constexpr int HALF = NMF - NR >= 1 ? NMF - NR : 1;  // ... of the last k-step in front of the slice barrier
    constexpr int POST = NMF - HALF;                    // issue slots behind it
    constexpr int RPS = (NR + POST - 1) / POST;         // fragment reads per slot there
    constexpr int RPS2 = (NR + NMF - 1) / NMF;          // ... and in the other k-steps
    constexpr int DPS = (LB + POST + NMF - 1) / (POST + NMF);  // refill loads per slot (those slots and the next k-step's)
    static_assert(ROWS % RPI == 0 && BM % RPI == 0, "whole blocks");
    static_assert(TM >= 2 && TN >= 2 && KS % 2 == 0, "wavefront tile");
    constexpr bool kTable = kEpi == EPI_Q_TABLE || kEpi == EPI_Q_TABLE2;
    static_assert(kEpi == EPI_Q || kTable || kEpi == EPI_F32_RESID || kEpi == EPI_F32_RESID_LN,
                  "epilogues of the tile kernel");
    static_assert(kEpi != EPI_F32_RESID_LN || WAVES_M == 1, "row statistics: a wavefront holds all rows of its columns");
    constexpr bool kResid = kEpi == EPI_F32_RESID || kEpi == EPI_F32_RESID_LN;

    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    float* s_bias = reinterpret_cast<float*>(smem + STAGES * STAGE_BYTES);
    float2* s_kb = reinterpret_cast<float2*>(s_bias + BN);

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = (wave / WAVES_N) * WM;
    const int wave_n = (wave % WAVES_N) * WN;

    // XCD-aware tile order, as in the streaming kernel
    int id = blockIdx.x;
    const int ntiles = p.tiles_m * p.tiles_n;
    if (ntiles % 8 == 0) id = (id % 8) * (ntiles / 8) + id / 8;
    const int GM = p.group_m;
    const int group = id / (GM * p.tiles_n);
    const int first_m = group * GM;
    const int gm = min(GM, p.tiles_m - first_m);
    const int in_group = id - group * GM * p.tiles_n;
    const int tile_m = first_m + in_group % gm;
    const int tile_n = in_group / gm;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    // per-lane byte offsets of this wavefront's blocks (rows past the edge are clamped: they only
    // feed accumulators that are never stored); M * K and N * K fit 32 bits (host)
    unsigned voff[LB];
#pragma unroll
    for (int b = 0; b < LB; ++b) {
        const int blk = wave + b * NW;
        const int r = blk * RPI + lane / CPR;
        const int chunk = (lane % CPR) ^ swz_bk<BK>(r);
        const bool is_a = kEven ? b < LBA : blk < ABLK;  // wave-uniform
        if (is_a) voff[b] = (unsigned)min(m0 + r, p.M - 1) * (unsigned)p.lda + 16u * chunk;
        else voff[b] = (unsigned)min(n0 + r - BM, p.N - 1) * (unsigned)p.ldw + 16u * chunk;
    }
    const unsigned lds_base = (unsigned)(uintptr_t)smem;
    const int8_t* __restrict__ gA = p.A;
    const int8_t* __restrict__ gW = p.W;
    auto issue1 = [&](int kt, int slot, int b) {
        const unsigned dst = lds_base + slot * STAGE_BYTES + (wave + b * NW) * 1024;
        const bool is_a = kEven ? b < LBA : wave + b * NW < ABLK;
        dma16s((is_a ? gA : gW) + (long)kt * BK, voff[b], dst);
    };
    const int nk = p.K / BK;  // >= STAGES + 1 (host)
#pragma unroll
    for (int st = 0; st < STAGES; ++st)
#pragma unroll
        for (int b = 0; b < LB; ++b) issue1(st, st, b);

    // epilogue parameters: fetched now, parked in registers until the k-loop is over
    constexpr int BPT = (BN + 64 * NW - 1) / (64 * NW);
    float bias_reg[BPT];
#pragma unroll
    for (int t = 0; t < BPT; ++t) {
        const int c = tid + t * 64 * NW;
        bias_reg[t] = (p.bias && c < BN && n0 + c < p.N) ? p.bias[n0 + c] : 0.0f;
    }
    constexpr int KPT = 4;  // table entries per thread held in registers (more are staged late)
    float2 kb_reg[KPT];
    if (kEpi == EPI_Q_TABLE) {
#pragma unroll
        for (int t = 0; t < KPT; ++t) {
            const int e = tid + t * 64 * NW;
            kb_reg[t] = e < p.table.nseg ? p.table.kb[e] : make_float2(0.0f, 0.0f);
        }
    }
    // two-level form: at most 256 merged segments and 256 cells (host), i.e. one {k, b} pair and one
    // word of four cell bytes per thread at most
    unsigned map_reg = 0;
    if (kEpi == EPI_Q_TABLE2) {
        kb_reg[0] = tid < p.table.nkb ? p.table.ckb[tid] : make_float2(0.0f, 0.0f);
        if (tid < (p.table.nseg + 3) / 4) map_reg = reinterpret_cast<const unsigned*>(p.table.cellmap)[tid];
    }

    // the int8 residual tile (fp32 epilogue) as 16-byte row pieces
    constexpr int CPRW = BN / 16;
    constexpr int RPT = (BM * CPRW + 64 * NW - 1) / (64 * NW);
    v4i res_reg[RPT];
    if (kResid) {
#pragma unroll
        for (int t = 0; t < RPT; ++t) {
            const int c = tid + t * 64 * NW, row = c / CPRW, cc = c % CPRW;
            const int mr = m0 + row, n = n0 + 16 * cc;
            res_reg[t] = v4i{0, 0, 0, 0};
            if (c < BM * CPRW && mr < p.M && n < p.N) res_reg[t] = *reinterpret_cast<const v4i*>(p.resid + (long)mr * p.ldo + n);
        }
    }

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    const int frag_row = lane & 31, frag_half = lane >> 5;
    int offA[KS], offW[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int ra = wave_m + frag_row, rw = wave_n + frag_row;
        offA[ks] = lds_off_bk<BK>(ra, 2 * ks + frag_half);
        offW[ks] = BM * BK + lds_off_bk<BK>(rw, 2 * ks + frag_half);
    }
    v4i fa[2][TM], fw[2][TN];
    // fragment t of a k-step, in the order the matrix instructions of that k-step need them
    auto ldfrag1 = [&](int buf, int slot, int ks, int t) {
        const int8_t* st = smem + slot * STAGE_BYTES;
        if (t == 0) fw[buf][0] = *reinterpret_cast<const v4i*>(st + offW[ks]);
        else if (t == 1) fa[buf][0] = *reinterpret_cast<const v4i*>(st + offA[ks]);
        else if (t < 1 + TN) fw[buf][t - 1] = *reinterpret_cast<const v4i*>(st + offW[ks] + (t - 1) * 32 * BK);
        else fa[buf][t - TN] = *reinterpret_cast<const v4i*>(st + offA[ks] + (t - TN) * 32 * BK);
    };

    // k-slice 0 has landed (the younger slices of the prologue stay in flight)
    wait_vmcnt<(STAGES - 1) * LB>();
    __syncthreads();
#pragma unroll
    for (int t = 0; t < NR; ++t) ldfrag1(0, 0, 0, t);

    int slot = 0, pslot = 0;
    // One k-slice.  MORE: slice kt + STAGES exists and refills this slice's slot (first blocks);
    // MOREP: the rest of the refill begun during the previous slice; YOUNG: slices younger than
    // kt + 1 in flight when kt + 1 is awaited (-1: there is no slice kt + 1).
    auto slice = [&](auto more_c, auto morep_c, auto young_c, int kt) {
        constexpr bool MORE = decltype(more_c)::value, MOREP = decltype(morep_c)::value;
        constexpr int YOUNG = decltype(young_c)::value;
        const int nslot = slot + 1 == STAGES ? 0 : slot + 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int cur = ks & 1;
#pragma unroll
            for (int t = 0; t < NMF; ++t) {
                const int i = t / TN, j = t % TN;
                if (ks == KS - 1 && t == HALF && YOUNG >= 0) {
                    // every wavefront has read all of slice kt (its last fragments were requested
                    // during the previous k-step); slice kt + 1 has landed for this wavefront
                    wait_vmcnt<(YOUNG > 0 ? YOUNG : 0) * LB>();
                    __syncthreads();
                    __builtin_amdgcn_sched_barrier(0);
                }
                acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[cur][j], fa[cur][i], acc[i][j], 0, 0, 0);
                if (ks < KS - 1) {
#pragma unroll
                    for (int r = t * RPS2; r < (t + 1) * RPS2; ++r)
                        if (r < NR) ldfrag1(cur ^ 1, slot, ks + 1, r);
                    if (MOREP && ks == 0) {
#pragma unroll
                        for (int d = (POST + t) * DPS; d < (POST + t + 1) * DPS; ++d)
                            if (d < LB) issue1(kt - 1 + STAGES, pslot, d);
                    }
                } else if (t >= HALF) {
                    const int u = t - HALF;
                    if (YOUNG >= 0) {
#pragma unroll
                        for (int r = u * RPS; r < (u + 1) * RPS; ++r)
                            if (r < NR) ldfrag1(cur ^ 1, nslot, 0, r);
                    }
                    if (MORE) {
#pragma unroll
                        for (int d = u * DPS; d < (u + 1) * DPS; ++d)
                            if (d < LB) issue1(kt + STAGES, slot, d);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        pslot = slot;
        slot = nslot;
    };
    using T_ = std::true_type;
    using F_ = std::false_type;
    slice(T_{}, F_{}, std::integral_constant<int, STAGES - 2>{}, 0);
    for (int kt = 1; kt < nk - STAGES; ++kt) slice(T_{}, T_{}, std::integral_constant<int, STAGES - 2>{}, kt);
    slice(F_{}, T_{}, std::integral_constant<int, STAGES - 2>{}, nk - STAGES);
    auto tail = [&](auto self, auto r_c) -> void {
        constexpr int R = decltype(r_c)::value;  // slices after this one
        slice(F_{}, F_{}, std::integral_constant<int, R - 1>{}, nk - 1 - R);
        if constexpr (R > 0) self(self, std::integral_constant<int, R - 1>{});
    };
    tail(tail, std::integral_constant<int, STAGES - 2>{});
    __syncthreads();  // every wavefront is done with the ring

#pragma unroll
    for (int t = 0; t < BPT; ++t) {
        const int c = tid + t * 64 * NW;
        if (c < BN) s_bias[c] = bias_reg[t];
    }
    if (kEpi == EPI_Q_TABLE) {
#pragma unroll
        for (int t = 0; t < KPT; ++t) {
            const int e = tid + t * 64 * NW;
            if (e < p.table.nseg) s_kb[e] = kb_reg[t];
        }
        for (int e = tid + KPT * 64 * NW; e < p.table.nseg; e += 64 * NW) s_kb[e] = p.table.kb[e];
    }
    const uint8_t* s_map = reinterpret_cast<const uint8_t*>(s_kb + p.table.nkb);  // cell -> merged segment
    if (kEpi == EPI_Q_TABLE2) {
        if (tid < p.table.nkb) s_kb[tid] = kb_reg[0];
        if (tid < (p.table.nseg + 3) / 4) reinterpret_cast<unsigned*>(s_kb + p.table.nkb)[tid] = map_reg;
    }
    constexpr int RW = BN + 16;  // row stride of the residual image
    int8_t* s_res = smem;        // in the ring, which is free now
    if (kResid) {
#pragma unroll
        for (int t = 0; t < RPT; ++t) {
            const int c = tid + t * 64 * NW, row = c / CPRW, cc = c % CPRW;
            if (c < BM * CPRW) *reinterpret_cast<v4i*>(s_res + row * RW + 16 * cc) = res_reg[t];
        }
    }
    __syncthreads();

    // ---- epilogue -----------------------------------------------------------------------------
    const float alpha = p.alpha;
    const bool full = m0 + BM <= p.M && n0 + BN <= p.N;
    v4f bi[TN][4];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) bi[j][g] = *reinterpret_cast<const v4f*>(s_bias + wave_n + 32 * j + 8 * g + 4 * frag_half);
    constexpr int NG = TM * TN * 4;  // groups of four columns per lane
    if constexpr (kTable || kEpi == EPI_Q) {
        constexpr int SW = WN + 16;
        static_assert(NW * WM * SW <= STAGES * STAGE_BYTES, "patch fits the ring");
        int8_t* patch = smem + wave * (WM * SW);
        // inverse output scale of a group (the QKV projection has one per column third)
        float inv_g[TN][4];
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wave_n + 32 * j + 8 * g + 4 * frag_half;
                inv_g[j][g] = p.split_cols > 0 ? (n >= 2 * p.split_cols ? p.inv3[2] : n >= p.split_cols ? p.inv3[1] : p.inv3[0])
                                               : p.out_inv_scale;
            }
        constexpr int DEPTH = 3;
        float x[DEPTH + 1][4];
        float2 kb[DEPTH + 1][4];
        const float tlo = p.table.lo, tiw = p.table.inv_w, tmax = (float)(p.table.nseg - 1);
        // group index -> (i, j, g), i innermost: consecutive groups use different accumulators
        auto stage_a = [&](int G) {
            const int i = G % TM, jg = G / TM, j = jg / 4, g = jg % 4;
            unsigned cellv[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = __builtin_fmaf((float)acc[i][j][4 * g + e], alpha, bi[j][g][e]);
                x[G % (DEPTH + 1)][e] = v;
                if (kTable) {  // segment of v (subtract, multiply, clamp in float, floor)
                    float u = v - tlo;
                    u = u * tiw;
                    u = __builtin_amdgcn_fmed3f(u, 0.0f, tmax);
                    if (kEpi == EPI_Q_TABLE2) cellv[e] = s_map[(int)u];
                    else kb[G % (DEPTH + 1)][e] = s_kb[(int)u];
                }
            }
            if (kEpi == EPI_Q_TABLE2) {  // second level: the four cell bytes have been requested together
#pragma unroll
                for (int e = 0; e < 4; ++e) kb[G % (DEPTH + 1)][e] = s_kb[cellv[e]];
            }
        };
        auto stage_b = [&](int G) {
            const int i = G % TM, jg = G / TM, j = jg / 4, g = jg % 4;
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float v = x[G % (DEPTH + 1)][e];
                if (kTable) v = __builtin_fmaf(kb[G % (DEPTH + 1)][e].x, v, kb[G % (DEPTH + 1)][e].y);
                q[e] = requant(v, inv_g[j][g]);
            }
            *reinterpret_cast<unsigned*>(patch + (32 * i + frag_row) * SW + 32 * j + 8 * g + 4 * frag_half) =
                pack4(q[0], q[1], q[2], q[3]);
        };
#pragma unroll
        for (int G = 0; G < NG + DEPTH; ++G) {
            if (G < NG) stage_a(G);
            __builtin_amdgcn_sched_barrier(0);
            if (G >= DEPTH) stage_b(G - DEPTH);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the wavefront reads back the rows it wrote: order its LDS writes before its reads
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        constexpr int PCPR = WN / 16;
        constexpr int NCH = WM * PCPR / 64;  // 16-byte chunks per lane
        static_assert(WM * PCPR % 64 == 0, "chunks split evenly");
        v4i rows[NCH];
#pragma unroll
        for (int t = 0; t < NCH; ++t) {
            const int c = lane + 64 * t, row = c / PCPR, cc = c % PCPR;
            rows[t] = *reinterpret_cast<const v4i*>(patch + row * SW + 16 * cc);
        }
#pragma unroll
        for (int t = 0; t < NCH; ++t) {
            const int c = lane + 64 * t, row = c / PCPR, cc = c % PCPR;
            const int mr = m0 + wave_m + row, n = n0 + wave_n + 16 * cc;
            if (full || (mr < p.M && n < p.N)) *reinterpret_cast<v4i*>(p.out_q + (long)mr * p.ldo + n) = rows[t];
        }
    } else if constexpr (kEpi == EPI_F32_RESID) {
        const float rs = p.resid_scale;
#pragma unroll
        for (int G = 0; G < NG; ++G) {
            const int i = G % TM, jg = G / TM, j = jg / 4, g = jg % 4;
            const int row = wave_m + 32 * i + frag_row, cl = wave_n + 32 * j + 8 * g + 4 * frag_half;
            const unsigned rw = *reinterpret_cast<const unsigned*>(s_res + row * RW + cl);
            v4f y;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = __builtin_fmaf((float)acc[i][j][4 * g + e], alpha, bi[j][g][e]);
                y[e] = __builtin_fmaf((float)(int)(int8_t)(rw >> (8 * e)), rs, v);
            }
            const int m = m0 + row, n = n0 + cl;
            if (full || (m < p.M && n < p.N)) *reinterpret_cast<v4f*>(p.out_f32 + (long)m * p.ldo + n) = y;
        }
    } else {
        // ---- fp32 result + residual, then LayerNorm-PWL over the row (the tile covers whole rows:
        // BN == N, n0 == 0, and every wavefront holds all BM rows of its WN columns).  Row sums keep
        // the normative order: column group G (four consecutive columns) belongs to accumulator
        // G % 64, an accumulator adds its groups in increasing G and each group's elements in
        // increasing column, starting from +0; the 64 accumulators of a row are then combined by the
        // butterfly 32, 16, 8, 4, 2, 1.  Groups 64 apart live in different wavefronts, so the
        // accumulators pass through LDS: round s adds the groups G with G / 64 == s.
        static_assert(BM <= 64 && BN % 256 == 0 && WN % 4 == 0, "row block shape");
        constexpr int NS = (BN / 4 + 63) / 64;         // rounds
        float* s_part = reinterpret_cast<float*>(smem + BM * RW);  // [BM][64] accumulators, behind the residual image
        float* s_stat = s_part + BM * 64;                           // [BM] mean, then [BM] scale
        static_assert(BM * RW + (BM * 64 + 2 * BM) * 4 <= STAGES * STAGE_BYTES, "statistics fit the ring");
        const float rs = p.resid_scale;
        const float inv_L = (float)(1.0 / (double)BN);
        // the fp32 values of the lane (they replace the accumulators)
        float xv[TM][TN][16];
#pragma unroll
        for (int G = 0; G < NG; ++G) {
            const int i = G % TM, jg = G / TM, j = jg / 4, g = jg % 4;
            const int row = 32 * i + frag_row, cl = wave_n + 32 * j + 8 * g + 4 * frag_half;
            const unsigned rw = *reinterpret_cast<const unsigned*>(s_res + row * RW + cl);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const float v = __builtin_fmaf((float)acc[i][j][4 * g + e], alpha, bi[j][g][e]);
                xv[i][j][4 * g + e] = __builtin_fmaf((float)(int)(int8_t)(rw >> (8 * e)), rs, v);
            }
        }
        // one pass over the row: SQ == false sums x, SQ == true sums fma(d, d, .)
        auto row_pass = [&](auto sq_c) {
            constexpr bool SQ = decltype(sq_c)::value;
#pragma unroll
            for (int s = 0; s < NS; ++s) {
#pragma unroll
                for (int j = 0; j < TN; ++j)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const int G = (wave_n + 32 * j + 8 * g + 4 * frag_half) >> 2;  // column group in the row
                        if ((G >> 6) != s) continue;                                 // wave-uniform (G and G ^ 1 share a round)
#pragma unroll
                        for (int i = 0; i < TM; ++i) {
                            float* slot = s_part + (32 * i + frag_row) * 64 + (G & 63);
                            float a = s == 0 ? 0.0f : *slot;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                a = SQ ? __builtin_fmaf(xv[i][j][4 * g + e], xv[i][j][4 * g + e], a) : a + xv[i][j][4 * g + e];
                            *slot = a;
                        }
                    }
                __syncthreads();
            }
            // butterfly over the 64 accumulators of each row: lane = accumulator
            for (int row = wave; row < BM; row += NW) {
                float v = s_part[row * 64 + lane];
#pragma unroll
                for (int mask = 32; mask >= 1; mask >>= 1) v = v + __shfl_xor(v, mask, 64);
                if (lane == 0) s_stat[row] = v * inv_L;
            }
            __syncthreads();
        };
        row_pass(std::false_type{});
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const float mu = s_stat[32 * i + frag_row];
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) xv[i][j][v] = xv[i][j][v] - mu;
        }
        __syncthreads();  // every lane has read its means before the variances overwrite them
        row_pass(std::true_type{});
        // scale of a row: r = PWL_rsqrt(var + eps), one look-up per row
        if (tid < BM) {
            int sr;
            const float u = s_stat[tid] + p.ln_eps;
            s_stat[BM + tid] = pwl_eval(u, p.ln_table, p.ln_table.kb, sr);
        }
        __syncthreads();
        // y = fma(d * r, gamma, beta); int8 rows leave through an LDS image as 16-byte stores
        int8_t* s_out = smem;  // [BM][RW], over the residual image (its last reader was the first loop above)
        const float inv = p.ln_inv_scale;
#pragma unroll
        for (int G = 0; G < NG; ++G) {
            const int i = G % TM, jg = G / TM, j = jg / 4, g = jg % 4;
            const int row = 32 * i + frag_row, cl = wave_n + 32 * j + 8 * g + 4 * frag_half;
            const float r = s_stat[BM + row];
            const v4f ga = *reinterpret_cast<const v4f*>(p.ln_gamma + cl);
            const v4f be = *reinterpret_cast<const v4f*>(p.ln_beta + cl);
            v4f y;
            int q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                y[e] = __builtin_fmaf(xv[i][j][4 * g + e] * r, ga[e], be[e]);
                q[e] = requant(y[e], inv);
            }
            if (p.ln_out_q) *reinterpret_cast<unsigned*>(s_out + row * RW + cl) = pack4(q[0], q[1], q[2], q[3]);
            if (p.ln_out_f32 && m0 + row < p.M) *reinterpret_cast<v4f*>(p.ln_out_f32 + (long)(m0 + row) * BN + cl) = y;
        }
        if (p.ln_out_q) {
            __syncthreads();
            for (int c = tid; c < BM * CPRW; c += 64 * NW) {
                const int row = c / CPRW, cc = c % CPRW;
                if (m0 + row < p.M)
                    *reinterpret_cast<v4i*>(p.ln_out_q + (long)(m0 + row) * BN + 16 * cc) =
                        *reinterpret_cast<const v4i*>(s_out + row * RW + 16 * cc);
            }
        }
    }
}

// Tile rows per group of the tile order.  Workgroup i runs on XCD i % 8, and the kernel hands XCD x the
// x-th eighth of the tile sequence, which walks groups of group_m tile rows column by column.  An
// eighth of r x c tiles reads r * BM rows of A and c * BN rows of W through that XCD's L2: pick the
// r (a divisor of the eighth, with whole columns: tiles_n % c == 0) that makes this sum smallest.
static inline int xcd_group_rows(int tiles_m, int tiles_n, int BM, int BN)
{
    const int ntiles = tiles_m * tiles_n;
    if (ntiles % 8 != 0) return 8;
    const int share = ntiles / 8;
    int best = 8;
    long best_cost = -1;
    for (int r = 1; r <= tiles_m && r <= share; ++r) {
        if (share % r != 0 || tiles_m % r != 0) continue;
        const int c = share / r;
        if (c > tiles_n || tiles_n % c != 0) continue;
        const long cost = (long)r * BM + (long)c * BN;
        if (best_cost < 0 || cost < best_cost) best_cost = cost, best = r;
    }
    return best;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int kEpi, int BK = 128>
static int32_t launch_tile_epi(GemmParams& p, size_t table_bytes, hipStream_t s)
{
    auto kern = gemm_tile_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, kEpi, BK>;
    constexpr int NW = WAVES_M * WAVES_N, NBLK = (BM + BN) * BK / 1024;
    const size_t shmem = (size_t)STAGES * ((NBLK + NW - 1) / NW * NW) * 1024 + BN * sizeof(float) + table_bytes;
    static std::once_flag once;  // one attribute call per instantiation
    static int32_t once_rc = NM_OK;
    std::call_once(once, [&] {
        once_rc = check_hip(hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024),
                            "hipFuncSetAttribute(gemm_tile_kernel)");
    });
    if (once_rc) return once_rc;
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    p.group_m = xcd_group_rows(p.tiles_m, p.tiles_n, BM, BN);
    hipLaunchKernelGGL(kern, dim3(p.tiles_m * p.tiles_n), dim3(64 * WAVES_M * WAVES_N), shmem, s, p);
    return NM_OK;
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES>
static int32_t launch_tile(GemmParams& p, int epi, size_t table_bytes, hipStream_t s)
{
    switch (epi) {
    case EPI_Q: return launch_tile_epi<BM, BN, WAVES_M, WAVES_N, STAGES, EPI_Q>(p, table_bytes, s);
    case EPI_Q_TABLE: return launch_tile_epi<BM, BN, WAVES_M, WAVES_N, STAGES, EPI_Q_TABLE>(p, table_bytes, s);
    case EPI_Q_TABLE2: return launch_tile_epi<BM, BN, WAVES_M, WAVES_N, STAGES, EPI_Q_TABLE2>(p, table_bytes, s);
    default: return launch_tile_epi<BM, BN, WAVES_M, WAVES_N, STAGES, EPI_F32_RESID>(p, table_bytes, s);
    }
}

}  // namespace nm
