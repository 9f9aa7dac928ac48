// Row-wise and element-wise PWL kernels for gfx950: stand-alone PWL, softmax-PWL, LayerNorm-PWL.
//
// These kernels are bound by HBM bandwidth (5 bytes per element: a 4-byte input, a 1-byte code),
// so their design is about memory access: each lane owns groups of four consecutive elements
// (one 16-byte load, one packed 4-byte int8 store), a row is held entirely in registers between
// its reductions (read once, written once), sub-wavefront rows share a wavefront so short rows
// still issue full-width memory instructions, and the {k, b} table of the per-element function
// sits in LDS.
//
// Row sums use the library's normative order: element j goes to accumulator (j / 4) % 64, each
// accumulator adds in increasing j from +0, and the partial sums are combined by a butterfly with
// partner masks 32, 16, 8, 4, 2, 1.  A row of at most 4*G elements (G a power of two below 64)
// only has G non-zero accumulators; adding the +0 of an empty accumulator changes nothing, so a
// butterfly over the G lanes that own the row gives the same bits.
#include "nm_device.h"

namespace nm {

constexpr int kRowThreads = 256;
constexpr int kApplyGroupsPerTrip = 8;  // pwl_apply: 16-byte groups a lane loads per trip

// One butterfly step: op(v, value of lane ^ MASK), without going through LDS.  Masks 1 and 2 are
// quad permutes, 4 and 8 compositions of the row mirrors (lane ^ 7 ^ 3, lane ^ 15 ^ 7), 16 and 32
// the gfx950 row / half swaps: swapping a register with a copy of itself leaves {even rows twice}
// in one and {odd rows twice} in the other (halves likewise), and op is commutative, so
// op(first, second) is op(v, partner) in every lane.
template <int MASK, typename Op>
__device__ __forceinline__ int butterfly_step(int v, Op op)
{
    if (MASK == 1) return op(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xf, 0xf, false));
    if (MASK == 2) return op(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xf, 0xf, false));
    if (MASK == 4) {
        const int t = __builtin_amdgcn_update_dpp(0, v, 0x141, 0xf, 0xf, false);   // lane ^ 7
        return op(v, __builtin_amdgcn_update_dpp(0, t, 0x1B, 0xf, 0xf, false));     // ... ^ 3
    }
    if (MASK == 8) {
        const int t = __builtin_amdgcn_update_dpp(0, v, 0x140, 0xf, 0xf, false);   // lane ^ 15
        return op(v, __builtin_amdgcn_update_dpp(0, t, 0x141, 0xf, 0xf, false));    // ... ^ 7
    }
    if (MASK == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
        return op((int)r[0], (int)r[1]);
    }
    const auto r = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return op((int)r[0], (int)r[1]);
}

struct AddF32 {
    __device__ __forceinline__ int operator()(int a, int b) const { return __float_as_int(__int_as_float(a) + __int_as_float(b)); }
};
struct MaxF32 {
    __device__ __forceinline__ int operator()(int a, int b) const { return __float_as_int(__builtin_fmaxf(__int_as_float(a), __int_as_float(b))); }
};
struct MaxI32 {
    __device__ __forceinline__ int operator()(int a, int b) const { return max(a, b); }
};

// Butterfly over the G lanes that own a row, partner masks G/2 ... 1 in that order.
template <int G, typename Op>
__device__ __forceinline__ int group_reduce(int v, Op op)
{
    if (G > 32) v = butterfly_step<32>(v, op);
    if (G > 16) v = butterfly_step<16>(v, op);
    if (G > 8) v = butterfly_step<8>(v, op);
    if (G > 4) v = butterfly_step<4>(v, op);
    if (G > 2) v = butterfly_step<2>(v, op);
    if (G > 1) v = butterfly_step<1>(v, op);
    return v;
}

template <int G>
__device__ __forceinline__ float group_sum(float v)
{
    return __int_as_float(group_reduce<G>(__float_as_int(v), AddF32{}));
}

// ------------------------------------------------------------------------------------------
// Stand-alone element-wise PWL (the non-fused element-wise path).
// ------------------------------------------------------------------------------------------
// kTwo: the table is in its two-level form (merged segments + cell map).  kLean: fp32 input and int8
// output only (the streaming case: no run-time tests of optional outputs inside the loop).
template <bool kVec, bool kTwo = false, bool kLean = false>
__global__ __launch_bounds__(kRowThreads) void pwl_apply_kernel(
    const void* __restrict__ in, int in_is_i32, float alpha, long n, DevTable t,
    float out_inv_scale, int8_t* __restrict__ out_q, float* __restrict__ out_f32,
    uint16_t* __restrict__ dbg_seg, int streams)
{
    extern __shared__ float2 s_kb[];
    // uniform tables sit in LDS as two arrays, k[] then b[]: consecutive segments then fall into
    // consecutive banks (64 of them before two meet) instead of bank pairs (32), which halves the
    // conflicts of the data-dependent look-up
    float* s_k = reinterpret_cast<float*>(s_kb);
    float* s_b = s_k + t.nseg;
    if (kTwo) {
        stage_table_two_level(s_kb, t);
    } else {
        for (int i = threadIdx.x; i < t.nseg; i += blockDim.x) {
            const float2 e = t.kb[i];
            s_k[i] = e.x;
            s_b[i] = e.y;
        }
    }
    __syncthreads();
    auto lookup = [&](float x, int& seg) {
        if (kTwo) return pwl_eval_two_level(x, t, s_kb, seg);
        const float xc = __builtin_amdgcn_fmed3f(x, t.lo, t.hi);
        x = t.clamp_input ? xc : x;
        seg = seg_index(x, t.lo, t.inv_w, t.nseg);
        return __builtin_fmaf(s_k[seg], x, s_b[seg]);
    };
    const long nthreads = (long)gridDim.x * blockDim.x;
    const long tid = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (kVec) {
        const long ngroups = n / 4;
        // one group of four elements: load, scale, PWL, requantise, store
        auto load_group = [&](long gidx, float (&x)[4]) {
            if (!kLean && in_is_i32) {
                const v4i* ptr = reinterpret_cast<const v4i*>(in) + gidx;
                v4i a = streams ? __builtin_nontemporal_load(ptr) : *ptr;  // block-uniform choice
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = (float)a[e] * alpha;
            } else {
                const v4f* ptr = reinterpret_cast<const v4f*>(in) + gidx;
                v4f a = streams ? __builtin_nontemporal_load(ptr) : *ptr;
#pragma unroll
                for (int e = 0; e < 4; ++e) x[e] = a[e] * alpha;
            }
        };
        auto finish_group = [&](long gidx, const float (&x)[4]) {
            float y[4];
            int s[4], q[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                y[e] = lookup(x[e], s[e]);
                q[e] = requant(y[e], out_inv_scale);
            }
            if (!kLean && out_f32) reinterpret_cast<v4f*>(out_f32)[gidx] = v4f{y[0], y[1], y[2], y[3]};
            if (kLean || out_q) reinterpret_cast<unsigned*>(out_q)[gidx] = pack4(q[0], q[1], q[2], q[3]);
            if (!kLean && dbg_seg)
                reinterpret_cast<uint2*>(dbg_seg)[gidx] =
                    make_uint2((unsigned)s[0] | ((unsigned)s[1] << 16),
                               (unsigned)s[2] | ((unsigned)s[3] << 16));
        };
        // kApplyGroupsPerTrip groups per trip: their loads are issued together (more bytes in flight
        // per lane); a block's groups are neighbours (32 KB contiguous per block and trip) and the grid
        // moves through the buffer as one front.  Groups a whole grid apart (the same lane's loads
        // 16 MB from each other) measured 7 % slower.
        constexpr int kUnroll = kApplyGroupsPerTrip;
        const long per_block = (long)blockDim.x * kUnroll;
        long base = (long)blockIdx.x * per_block;
        for (; base + per_block <= ngroups; base += per_block * gridDim.x) {
            float x[kUnroll][4];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) load_group(base + u * (long)blockDim.x + threadIdx.x, x[u]);
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) finish_group(base + u * (long)blockDim.x + threadIdx.x, x[u]);
        }
        // the (at most one) partly filled span of this block
        for (long gidx = base + threadIdx.x; gidx < ngroups && gidx < base + per_block; gidx += blockDim.x) {
            float x[4];
            load_group(gidx, x);
            finish_group(gidx, x);
        }
    }
    // scalar path: everything when !kVec, the (< 4 element) tail otherwise
    const long first = kVec ? (n / 4) * 4 : 0;
    for (long i = first + tid; i < n; i += nthreads) {
        float x = in_is_i32 ? (float)reinterpret_cast<const int*>(in)[i] * alpha
                            : reinterpret_cast<const float*>(in)[i] * alpha;
        int s;
        float y = lookup(x, s);
        if (out_f32) out_f32[i] = y;
        if (out_q) out_q[i] = (int8_t)requant(y, out_inv_scale);
        if (dbg_seg) dbg_seg[i] = (uint16_t)s;
    }
}

// ------------------------------------------------------------------------------------------
// Softmax-PWL.  G lanes own a row (G = 64 for rows longer than 128 elements); a lane owns the
// 4-element groups g, g + G, ... (C of them).
// ------------------------------------------------------------------------------------------
// kFull: cols == 4 * G * C (every lane's groups are inside the row; implies kVec).  Rows past
// the end are then computed on a copy of the last row and only their stores are masked, so the
// whole body is straight-line code: no per-element predicates, and the table look-ups of a row
// are issued together instead of one per basic block.
// kU (kFull only): rows a lane group handles per trip; their loads are all issued before the first
// row is computed (more bytes in flight per lane; a block then covers kU * kRowsPerBlock consecutive
// rows per trip).  kStream: loads marked non-temporal, for inputs too large to be cache-resident.
template <int G, int C, bool kI32, bool kVec, bool kFull, int kU = 1, bool kStream = false>
__global__ __launch_bounds__(kRowThreads) void softmax_pwl_kernel(
    const void* __restrict__ in, float alpha, long rows, int cols, DevTable t_exp, DevTable t_recip,
    float out_inv_scale, int8_t* __restrict__ out_q, float* __restrict__ out_f32,
    uint16_t* __restrict__ seg_exp, uint16_t* __restrict__ seg_recip)
{
    // both tables in LDS (the per-row reciprocal look-up would otherwise add one more global-memory
    // round trip to every row's dependency chain)
    extern __shared__ float2 s_kb[];
    float2* s_kb_recip = s_kb + t_exp.nseg;
    stage_table(s_kb, t_exp);
    stage_table(s_kb_recip, t_recip);
    __syncthreads();
    constexpr int kRowsPerWave = 64 / G;
    constexpr int kRowsPerBlock = kRowsPerWave * (kRowThreads / 64);
    const int lane = threadIdx.x & 63;
    const int g = lane % G;
    const int sub = (threadIdx.x >> 6) * kRowsPerWave + lane / G;
    const float clo = t_exp.clamp_input ? t_exp.lo : -__builtin_inff();
    const float chi = t_exp.clamp_input ? t_exp.hi : __builtin_inff();

    static_assert(kU == 1 || kFull, "several rows per trip: full rows only");
    for (long row00 = (long)blockIdx.x * (kRowsPerBlock * kU); row00 < rows;
         row00 += (long)gridDim.x * (kRowsPerBlock * kU)) {
      v4i raw[kU][C];
      if (kFull) {
#pragma unroll
        for (int ur = 0; ur < kU; ++ur) {
            const long r = row00 + ur * kRowsPerBlock + sub;
            const int* src = reinterpret_cast<const int*>(in) + (r < rows ? r : rows - 1) * (long)cols;
#pragma unroll
            for (int c = 0; c < C; ++c) {
                const v4i* ptr = reinterpret_cast<const v4i*>(src + 4 * (g + G * c));
                raw[ur][c] = kStream ? __builtin_nontemporal_load(ptr) : *ptr;
            }
        }
      }
#pragma unroll
      for (int ur = 0; ur < kU; ++ur) {
        const long row0 = row00 + ur * kRowsPerBlock;
        if (ur > 0 && row0 >= rows) break;  // block-uniform
        const long row = row0 + sub;
        const bool live = row < rows;
        const long base = (kFull && !live ? rows - 1 : row) * (long)cols;
        float e[C][4];
        bool ok[C][4];
        int ai[C][4];
        // ---- load + row maximum -------------------------------------------------------------
        int mi = INT_MIN;
        float mf = -INFINITY;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int j0 = 4 * (g + G * c);
#pragma unroll
            for (int q = 0; q < 4; ++q) ok[c][q] = kFull || (live && (j0 + q) < cols);
            if (kFull) {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    if (kI32) ai[c][q] = raw[ur][c][q];
                    else e[c][q] = __int_as_float(raw[ur][c][q]);
                }
            } else if (kVec) {
                if (ok[c][0]) {  // cols % 4 == 0: a group is all in or all out
                    if (kI32) {
                        v4i a = *reinterpret_cast<const v4i*>(reinterpret_cast<const int*>(in) + base + j0);
#pragma unroll
                        for (int q = 0; q < 4; ++q) ai[c][q] = a[q];
                    } else {
                        v4f a = *reinterpret_cast<const v4f*>(reinterpret_cast<const float*>(in) + base + j0);
#pragma unroll
                        for (int q = 0; q < 4; ++q) e[c][q] = a[q];
                    }
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[c][q]) {
                        if (kI32) ai[c][q] = reinterpret_cast<const int*>(in)[base + j0 + q];
                        else e[c][q] = reinterpret_cast<const float*>(in)[base + j0 + q];
                    }
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (ok[c][q]) {
                    if (kI32) mi = max(mi, ai[c][q]);
                    else mf = __builtin_fmaxf(mf, e[c][q]);
                }
        }
        if (kI32) mi = group_reduce<G>(mi, MaxI32{});
        else mf = __int_as_float(group_reduce<G>(__float_as_int(mf), MaxF32{}));
        // ---- exp + canonical sum ------------------------------------------------------------
        float part = 0.0f;
        int se[C][4];
#pragma unroll
        for (int c = 0; c < C; ++c) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (ok[c][q]) {
                    float tt = kI32 ? (float)(ai[c][q] - mi) * alpha : (e[c][q] - mf) * alpha;
                    // int32 scores times a finite alpha cannot be NaN: the clamp flag folds into the bounds
                    e[c][q] = kI32 ? pwl_eval_bounded(tt, clo, chi, t_exp, s_kb, se[c][q])
                                   : pwl_eval(tt, t_exp, s_kb, se[c][q]);
                    part = part + e[c][q];
                } else {
                    e[c][q] = 0.0f;
                    se[c][q] = 0;
                }
            }
        }
        const float S = group_sum<G>(part);
        int sr;
        const float r = pwl_eval(S, t_recip, s_kb_recip, sr);
        if (seg_recip && live && g == 0) seg_recip[row] = (uint16_t)sr;
        // ---- scale + store -------------------------------------------------------------------
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int j0 = 4 * (g + G * c);
            float p[4];
            int qv[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                p[q] = e[c][q] * r;
                qv[q] = requant(p[q], out_inv_scale);
            }
            if (kVec) {
                if (kFull ? live : ok[c][0]) {
                    if (out_f32) *reinterpret_cast<v4f*>(out_f32 + base + j0) = v4f{p[0], p[1], p[2], p[3]};
                    if (out_q) *reinterpret_cast<unsigned*>(out_q + base + j0) = pack4(qv[0], qv[1], qv[2], qv[3]);
                    if (seg_exp)
                        *reinterpret_cast<uint2*>(seg_exp + base + j0) =
                            make_uint2((unsigned)se[c][0] | ((unsigned)se[c][1] << 16),
                                       (unsigned)se[c][2] | ((unsigned)se[c][3] << 16));
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[c][q]) {
                        if (out_f32) out_f32[base + j0 + q] = p[q];
                        if (out_q) out_q[base + j0 + q] = (int8_t)qv[q];
                        if (seg_exp) seg_exp[base + j0 + q] = (uint16_t)se[c][q];
                    }
            }
        }
      }
    }
}

// ------------------------------------------------------------------------------------------
// LayerNorm-PWL.  Same ownership as softmax.
// ------------------------------------------------------------------------------------------
template <int G, int C, bool kVec, bool kFull>
__global__ __launch_bounds__(kRowThreads) void layernorm_pwl_kernel(
    const float* __restrict__ in, const float* __restrict__ gamma, const float* __restrict__ beta,
    float eps, float inv_L, long rows, int cols, DevTable t, DevTable t2, int two_tables,
    float out_inv_scale, int8_t* __restrict__ out_q, float* __restrict__ out_f32,
    uint16_t* __restrict__ seg, uint16_t* __restrict__ seg2)
{
    constexpr int kRowsPerWave = 64 / G;
    constexpr int kRowsPerBlock = kRowsPerWave * (kRowThreads / 64);
    const int lane = threadIdx.x & 63;
    const int g = lane % G;
    const int sub = (threadIdx.x >> 6) * kRowsPerWave + lane / G;
    // The rsqrt table goes to LDS while the first row is on its way from memory (staged after the
    // row's loads are issued; every thread of a block makes the same number of trips, so the
    // barrier inside the first trip is reached by all): the look-up then costs an LDS access
    // instead of a second global-memory round trip in each row's dependency chain.
    extern __shared__ float2 s_kb[];
    bool staged = false;

    for (long row0 = (long)blockIdx.x * kRowsPerBlock; row0 < rows;
         row0 += (long)gridDim.x * kRowsPerBlock) {
        const long row = row0 + sub;
        const bool live = row < rows;
        const long base = (kFull && !live ? rows - 1 : row) * (long)cols;
        float x[C][4];
        bool ok[C][4];
        float part = 0.0f;
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int j0 = 4 * (g + G * c);
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                ok[c][q] = kFull || (live && (j0 + q) < cols);
                x[c][q] = 0.0f;
            }
            if (kVec) {
                if (ok[c][0]) {
                    v4f a = *reinterpret_cast<const v4f*>(in + base + j0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) x[c][q] = a[q];
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[c][q]) x[c][q] = in[base + j0 + q];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (ok[c][q]) part = part + x[c][q];
        }
        if (!staged) {
            stage_table(s_kb, t);
            if (two_tables) stage_table(s_kb + t.nseg, t2);
            __syncthreads();
            staged = true;
        }
        const float mu = group_sum<G>(part) * inv_L;
        float part2 = 0.0f;
#pragma unroll
        for (int c = 0; c < C; ++c)
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (ok[c][q]) {
                    x[c][q] = x[c][q] - mu;
                    part2 = __builtin_fmaf(x[c][q], x[c][q], part2);
                }
        const float var = group_sum<G>(part2) * inv_L;
        const float u = var + eps;
        int sr;
        float r = pwl_eval(u, t, s_kb, sr);   // rsqrt table, or the sqrt table of the two-table form
        if (seg && live && g == 0) seg[row] = (uint16_t)sr;
        if (two_tables) {                      // ... followed by the reciprocal table
            int sr2;
            r = pwl_eval(r, t2, s_kb + t.nseg, sr2);
            if (seg2 && live && g == 0) seg2[row] = (uint16_t)sr2;
        }
#pragma unroll
        for (int c = 0; c < C; ++c) {
            const int j0 = 4 * (g + G * c);
            float y[4];
            int qv[4];
            if (kVec) {
                if (kFull ? live : ok[c][0]) {
                    v4f ga = *reinterpret_cast<const v4f*>(gamma + j0);
                    v4f be = *reinterpret_cast<const v4f*>(beta + j0);
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        y[q] = __builtin_fmaf(x[c][q] * r, ga[q], be[q]);
                        qv[q] = requant(y[q], out_inv_scale);
                    }
                    if (out_f32) *reinterpret_cast<v4f*>(out_f32 + base + j0) = v4f{y[0], y[1], y[2], y[3]};
                    if (out_q) *reinterpret_cast<unsigned*>(out_q + base + j0) = pack4(qv[0], qv[1], qv[2], qv[3]);
                }
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (ok[c][q]) {
                        float yy = __builtin_fmaf(x[c][q] * r, gamma[j0 + q], beta[j0 + q]);
                        if (out_f32) out_f32[base + j0 + q] = yy;
                        if (out_q) out_q[base + j0 + q] = (int8_t)requant(yy, out_inv_scale);
                    }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Host launchers
// ------------------------------------------------------------------------------------------

static int blocks_for(long units, int per_block, long cap_override = 0)
{
    long b = (units + per_block - 1) / per_block;
    const long cap = cap_override ? cap_override : 256L * 16;  // 256 compute units, several resident blocks each
    if (b > cap) b = cap;
    if (b < 1) b = 1;
    return (int)b;
}

// Inputs beyond what the 256 MB last-level cache can hold take the streaming variant of the softmax
// kernel (several rows per trip, non-temporal loads: +5 points of HBM peak on buffers that are not
// cache-resident, -13 on ones that are); smaller ones were probably just written by the previous
// kernel and are read through the caches.  (The same variant of LayerNorm measured no gain.)
static bool streaming_input(long bytes) { return bytes >= (192L << 20); }

// rows per trip of the streaming variants: about eight 16-byte loads in flight per lane
constexpr int rows_per_trip(int C) { return C >= 8 ? 1 : C >= 3 ? 2 : C == 2 ? 4 : 8; }

// Pick (G, C) so that G * 4 * C >= cols: G lanes per row, C groups per lane.
struct RowShape { int G, C; };
static RowShape row_shape(int cols)
{
    int groups = (cols + 3) / 4;
    int G = 1;
    while (G < 64 && G < groups) G *= 2;
    int C = (groups + G - 1) / G;
    static const int allowed[] = {1, 2, 3, 4, 6, 8, 12, 16};
    for (int a : allowed)
        if (a >= C) return {G, a};
    return {G, -1};
}

template <bool kI32, bool kVec>
static bool launch_softmax_t(RowShape rs, dim3 grid_hint, size_t shmem, hipStream_t stream,
                             const void* in, float alpha, long rows, int cols, const DevTable& te,
                             const DevTable& tr, float ois, int8_t* oq, float* of, uint16_t* se,
                             uint16_t* sr)
{
    (void)grid_hint;
    const bool streams = streaming_input(rows * (long)cols * 4);
#define NM_SM_CASE(GG, CC)                                                                          \
    if (rs.G == GG && rs.C == CC) {                                                                 \
        constexpr int rpb = (64 / GG) * (kRowThreads / 64);                                         \
        constexpr int ku = kVec ? rows_per_trip(CC) : 1;                                            \
        if (kVec && cols == 4 * GG * CC && streams)                                                 \
            hipLaunchKernelGGL((softmax_pwl_kernel<GG, CC, kI32, kVec, kVec, ku, kVec>),            \
                               dim3(blocks_for(rows, rpb * ku)), dim3(kRowThreads), shmem, stream,  \
                               in, alpha, rows, cols, te, tr, ois, oq, of, se, sr);                 \
        else if (kVec && cols == 4 * GG * CC)                                                       \
            hipLaunchKernelGGL((softmax_pwl_kernel<GG, CC, kI32, kVec, kVec>),                      \
                               dim3(blocks_for(rows, rpb)), dim3(kRowThreads), shmem, stream, in,   \
                               alpha, rows, cols, te, tr, ois, oq, of, se, sr);                     \
        else                                                                                        \
            hipLaunchKernelGGL((softmax_pwl_kernel<GG, CC, kI32, kVec, false>),                     \
                               dim3(blocks_for(rows, rpb)), dim3(kRowThreads), shmem, stream, in,   \
                               alpha, rows, cols, te, tr, ois, oq, of, se, sr);                     \
        return true;                                                                                \
    }
    NM_SM_CASE(1, 1) NM_SM_CASE(2, 1) NM_SM_CASE(4, 1) NM_SM_CASE(8, 1) NM_SM_CASE(16, 1)
    NM_SM_CASE(32, 1) NM_SM_CASE(64, 1) NM_SM_CASE(64, 2) NM_SM_CASE(64, 3) NM_SM_CASE(64, 4)
    NM_SM_CASE(64, 6) NM_SM_CASE(64, 8) NM_SM_CASE(64, 12) NM_SM_CASE(64, 16)
#undef NM_SM_CASE
    return false;
}

int32_t launch_softmax(const void* in, int32_t in_dtype, float alpha, int64_t rows, int32_t cols,
                       const DevTable& t_exp, const DevTable& t_recip, float out_inv_scale,
                       int8_t* out_q, float* out_f32, uint16_t* seg_exp, uint16_t* seg_recip,
                       hipStream_t stream)
{
    if (rows == 0) return NM_OK;
    RowShape rs = row_shape(cols);
    if (rs.C < 0) return fail(NM_ERR_UNSUPPORTED, "softmax: cols %d not supported", cols);
    const bool vec = cols % 4 == 0 && aligned(in, 16) && (!out_f32 || aligned(out_f32, 16)) &&
                     (!out_q || aligned(out_q, 4)) && (!seg_exp || aligned(seg_exp, 8));
    const size_t shmem = sizeof(float2) * ((size_t)t_exp.nseg + (size_t)t_recip.nseg);
    bool ok;
    const bool i32 = in_dtype == NM_DT_I32;
    if (i32 && vec) ok = launch_softmax_t<true, true>(rs, dim3(), shmem, stream, in, alpha, rows, cols, t_exp, t_recip, out_inv_scale, out_q, out_f32, seg_exp, seg_recip);
    else if (i32) ok = launch_softmax_t<true, false>(rs, dim3(), shmem, stream, in, alpha, rows, cols, t_exp, t_recip, out_inv_scale, out_q, out_f32, seg_exp, seg_recip);
    else if (vec) ok = launch_softmax_t<false, true>(rs, dim3(), shmem, stream, in, alpha, rows, cols, t_exp, t_recip, out_inv_scale, out_q, out_f32, seg_exp, seg_recip);
    else ok = launch_softmax_t<false, false>(rs, dim3(), shmem, stream, in, alpha, rows, cols, t_exp, t_recip, out_inv_scale, out_q, out_f32, seg_exp, seg_recip);
    if (!ok) return fail(NM_ERR_UNSUPPORTED, "softmax: no kernel for cols %d", cols);
    return check_hip(hipGetLastError(), "softmax launch");
}

template <bool kVec>
static bool launch_layernorm_t(RowShape rs, hipStream_t stream, const float* in, const float* gamma,
                               const float* beta, float eps, float inv_L, long rows, int cols,
                               const DevTable& t, const DevTable& t2, int two, float ois, int8_t* oq, float* of,
                               uint16_t* seg, uint16_t* seg2)
{
    const size_t shmem = sizeof(float2) * ((size_t)t.nseg + (two ? (size_t)t2.nseg : 0));
#define NM_LN_CASE(GG, CC)                                                                          \
    if (rs.G == GG && rs.C == CC) {                                                                 \
        constexpr int rpb = (64 / GG) * (kRowThreads / 64);                                         \
        if (kVec && cols == 4 * GG * CC)                                                            \
            hipLaunchKernelGGL((layernorm_pwl_kernel<GG, CC, kVec, kVec>), dim3(blocks_for(rows, rpb)), \
                               dim3(kRowThreads), shmem, stream, in, gamma,                         \
                               beta, eps, inv_L, rows, cols, t, t2, two, ois, oq, of, seg, seg2);   \
        else                                                                                        \
            hipLaunchKernelGGL((layernorm_pwl_kernel<GG, CC, kVec, false>), dim3(blocks_for(rows, rpb)), \
                               dim3(kRowThreads), shmem, stream, in, gamma,                         \
                               beta, eps, inv_L, rows, cols, t, t2, two, ois, oq, of, seg, seg2);   \
        return true;                                                                                \
    }
    NM_LN_CASE(1, 1) NM_LN_CASE(2, 1) NM_LN_CASE(4, 1) NM_LN_CASE(8, 1) NM_LN_CASE(16, 1)
    NM_LN_CASE(32, 1) NM_LN_CASE(64, 1) NM_LN_CASE(64, 2) NM_LN_CASE(64, 3) NM_LN_CASE(64, 4)
    NM_LN_CASE(64, 6) NM_LN_CASE(64, 8) NM_LN_CASE(64, 12) NM_LN_CASE(64, 16)
#undef NM_LN_CASE
    return false;
}

int32_t launch_layernorm(const float* in, const float* gamma, const float* beta, float eps,
                         int64_t rows, int32_t cols, const DevTable& t, float out_inv_scale,
                         int8_t* out_q, float* out_f32, uint16_t* seg, hipStream_t stream)
{
    return launch_layernorm2(in, gamma, beta, eps, rows, cols, t, t, 0, out_inv_scale, out_q, out_f32, seg,
                             nullptr, stream);
}

int32_t launch_layernorm2(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const DevTable& t, const DevTable& t2, int two,
                          float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* seg, uint16_t* seg2,
                          hipStream_t stream)
{
    if (rows == 0) return NM_OK;
    RowShape rs = row_shape(cols);
    if (rs.C < 0) return fail(NM_ERR_UNSUPPORTED, "layernorm: cols %d not supported", cols);
    const float inv_L = (float)(1.0 / (double)cols);
    const bool vec = cols % 4 == 0 && aligned(in, 16) && aligned(gamma, 16) && aligned(beta, 16) &&
                     (!out_f32 || aligned(out_f32, 16)) && (!out_q || aligned(out_q, 4));
    bool ok = vec ? launch_layernorm_t<true>(rs, stream, in, gamma, beta, eps, inv_L, rows, cols, t, t2, two, out_inv_scale, out_q, out_f32, seg, seg2)
                  : launch_layernorm_t<false>(rs, stream, in, gamma, beta, eps, inv_L, rows, cols, t, t2, two, out_inv_scale, out_q, out_f32, seg, seg2);
    if (!ok) return fail(NM_ERR_UNSUPPORTED, "layernorm: no kernel for cols %d", cols);
    return check_hip(hipGetLastError(), "layernorm launch");
}

}  // namespace nm

using namespace nm;

extern "C" {

int32_t nm_pwl_apply(const void* in, int32_t in_dtype, float alpha, int64_t n,
                     const nm_tables* tables, int32_t idx, float out_inv_scale, int8_t* out_q,
                     float* out_f32, uint16_t* dbg_seg, void* stream)
{
    if (in_dtype != NM_DT_I32 && in_dtype != NM_DT_F32)
        return fail(NM_ERR_INVALID_ARG, "nm_pwl_apply: bad in_dtype %d", in_dtype);
    if (n < 0) return fail(NM_ERR_INVALID_ARG, "nm_pwl_apply: n < 0");
    DevTable t;
    int32_t rc = get_dev_table(tables, idx, &t, "nm_pwl_apply", true);
    if (rc) return rc;
    if (n == 0) return NM_OK;  // an empty buffer may be a NULL pointer
    if (!in) return fail(NM_ERR_INVALID_ARG, "nm_pwl_apply: in is NULL");
    if (!out_q && !out_f32 && !dbg_seg) return fail(NM_ERR_INVALID_ARG, "nm_pwl_apply: no output");
    const bool vec = aligned(in, 16) && (!out_f32 || aligned(out_f32, 16)) &&
                     (!out_q || aligned(out_q, 4)) && (!dbg_seg || aligned(dbg_seg, 8));
    const bool two = t.cellmap != nullptr;  // two-level form: merged segments + one byte per cell
    const size_t shmem = two ? 8 * (size_t)t.nkb + (((size_t)t.nseg + 7) & ~(size_t)7) : sizeof(float2) * (size_t)t.nseg;
    // vector path: one 32 KB span per block up to 2^20 blocks (one span per block measured 3 % faster
    // at 2^26 elements than 4096 blocks looping over two spans each)
    const int blocks = vec ? blocks_for((n + 3) / 4, kRowThreads * kApplyGroupsPerTrip, 1L << 20)
                           : blocks_for(n, kRowThreads);
    auto launch = [&](auto kern) {
        hipLaunchKernelGGL(kern, dim3(blocks), dim3(kRowThreads), shmem, (hipStream_t)stream, in,
                           in_dtype == NM_DT_I32, alpha, (long)n, t, out_inv_scale, out_q, out_f32, dbg_seg,
                           (int)streaming_input((long)n * 4));
    };
    const bool lean = vec && !two && in_dtype == NM_DT_F32 && out_q && !out_f32 && !dbg_seg;
    if (lean) launch(pwl_apply_kernel<true, false, true>);
    else if (vec && two) launch(pwl_apply_kernel<true, true>);
    else if (vec) launch(pwl_apply_kernel<true, false>);
    else if (two) launch(pwl_apply_kernel<false, true>);
    else launch(pwl_apply_kernel<false, false>);
    return check_hip(hipGetLastError(), "nm_pwl_apply launch");
}

int32_t nm_softmax_pwl(const void* in, int32_t in_dtype, float alpha, int64_t rows, int32_t cols,
                       const nm_tables* tables, int32_t exp_idx, int32_t recip_idx,
                       float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg_exp,
                       uint16_t* dbg_seg_recip, void* stream)
{
    if (in_dtype != NM_DT_I32 && in_dtype != NM_DT_F32)
        return fail(NM_ERR_INVALID_ARG, "nm_softmax_pwl: bad in_dtype %d", in_dtype);
    if (rows < 0 || cols < 1) return fail(NM_ERR_INVALID_ARG, "nm_softmax_pwl: bad shape");
    if (!(alpha == alpha) || __builtin_isinf(alpha)) return fail(NM_ERR_INVALID_ARG, "nm_softmax_pwl: alpha must be finite");
    if (cols > 4096) return fail(NM_ERR_UNSUPPORTED, "nm_softmax_pwl: cols %d > 4096", cols);
    if (rows > (1LL << 40) / cols) return fail(NM_ERR_UNSUPPORTED, "nm_softmax_pwl: too many elements");
    DevTable te, tr;
    int32_t rc = get_dev_table(tables, exp_idx, &te, "nm_softmax_pwl(exp)");
    if (rc) return rc;
    rc = get_dev_table(tables, recip_idx, &tr, "nm_softmax_pwl(recip)");
    if (rc) return rc;
    if (rows == 0) return NM_OK;  // an empty matrix may be a NULL pointer
    if (!in) return fail(NM_ERR_INVALID_ARG, "nm_softmax_pwl: in is NULL");
    if (!out_q && !out_f32) return fail(NM_ERR_INVALID_ARG, "nm_softmax_pwl: no output");
    return launch_softmax(in, in_dtype, alpha, rows, cols, te, tr, out_inv_scale, out_q, out_f32,
                          dbg_seg_exp, dbg_seg_recip, (hipStream_t)stream);
}

int32_t nm_layernorm_pwl(const float* in, const float* gamma, const float* beta, float eps,
                         int64_t rows, int32_t cols, const nm_tables* tables, int32_t rsqrt_idx,
                         float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg,
                         void* stream)
{
    if (rows < 0 || cols < 1) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl: bad shape");
    if (cols > 4096) return fail(NM_ERR_UNSUPPORTED, "nm_layernorm_pwl: cols %d > 4096", cols);
    if (!gamma || !beta) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl: gamma or beta is NULL");
    DevTable t;
    int32_t rc = get_dev_table(tables, rsqrt_idx, &t, "nm_layernorm_pwl");
    if (rc) return rc;
    if (rows == 0) return NM_OK;  // an empty matrix may be a NULL pointer
    if (!in) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl: in is NULL");
    if (!out_q && !out_f32) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl: no output");
    return launch_layernorm(in, gamma, beta, eps, rows, cols, t, out_inv_scale, out_q, out_f32,
                            dbg_seg, (hipStream_t)stream);
}

int32_t nm_layernorm_pwl2(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const nm_tables* tables, int32_t sqrt_idx,
                          int32_t recip_idx, float out_inv_scale, int8_t* out_q, float* out_f32,
                          uint16_t* dbg_seg_sqrt, uint16_t* dbg_seg_recip, void* stream)
{
    if (rows < 0 || cols < 1) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl2: bad shape");
    if (cols > 4096) return fail(NM_ERR_UNSUPPORTED, "nm_layernorm_pwl2: cols %d > 4096", cols);
    if (!gamma || !beta) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl2: gamma or beta is NULL");
    DevTable t, t2;
    int32_t rc = get_dev_table(tables, sqrt_idx, &t, "nm_layernorm_pwl2(sqrt)");
    if (rc) return rc;
    if ((rc = get_dev_table(tables, recip_idx, &t2, "nm_layernorm_pwl2(recip)"))) return rc;
    if (rows == 0) return NM_OK;
    if (!in) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl2: in is NULL");
    if (!out_q && !out_f32) return fail(NM_ERR_INVALID_ARG, "nm_layernorm_pwl2: no output");
    return launch_layernorm2(in, gamma, beta, eps, rows, cols, t, t2, 1, out_inv_scale, out_q, out_f32,
                             dbg_seg_sqrt, dbg_seg_recip, (hipStream_t)stream);
}

}  // extern "C"
