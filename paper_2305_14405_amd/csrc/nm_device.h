// Device-side PWL primitives (gfx950).  Compiled with -ffp-contract=off: every fused multiply-add
// is an explicit __builtin_fmaf, everything else is a separately rounded fp32 operation.
#pragma once

#include <hip/hip_runtime.h>

#include "nm_internal.h"

namespace nm {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));

// Segment of x (paper Section 3.2: uniform segments, inputs outside the range use the edge
// segments): one subtract, one multiply, clamp in float, floor.  After the clamp u >= 0, so the
// float -> int conversion (which truncates) IS the floor.  The clamp is one median-of-three; for a
// NaN it returns the smaller bound, 0, as fmin(fmax(NaN, 0), nseg - 1) does.
__device__ __forceinline__ int seg_index(float x, float lo, float inv_w, int nseg)
{
    float u = x - lo;
    u = u * inv_w;
    u = __builtin_amdgcn_fmed3f(u, 0.0f, (float)(nseg - 1));
    return (int)u;
}

// y = k[s]*x + b[s] (one fma).  kb may point to LDS or to global memory.
__device__ __forceinline__ float pwl_eval(float x, const DevTable& t, const float2* kb, int& seg)
{
    // one median-of-three plus a select (a branch here would split the caller's unrolled loops
    // into small blocks and serialise their LDS gathers); NaN: med3 returns the smallest non-NaN
    // operand, lo, as fmin(fmax(NaN, lo), hi) does
    const float xc = __builtin_amdgcn_fmed3f(x, t.lo, t.hi);
    x = t.clamp_input ? xc : x;
    seg = seg_index(x, t.lo, t.inv_w, t.nseg);
    float2 e = kb[seg];
    return __builtin_fmaf(e.x, x, e.y);
}

// The same for a value that cannot be NaN (an int32 accumulator times finite multipliers): the
// clamp flag is folded into the bounds (clo, chi = lo, hi with the flag, -inf, +inf without), so no
// select is needed; identical results for every non-NaN x.
__device__ __forceinline__ float pwl_eval_bounded(float x, float clo, float chi, const DevTable& t,
                                                  const float2* kb, int& seg)
{
    x = __builtin_amdgcn_fmed3f(x, clo, chi);
    seg = seg_index(x, t.lo, t.inv_w, t.nseg);
    const float2 e = kb[seg];
    return __builtin_fmaf(e.x, x, e.y);
}
__device__ __forceinline__ float pwl_eval_bounded(float x, float clo, float chi, const DevTable& t,
                                                  const float2* kb)
{
    int seg;
    return pwl_eval_bounded(x, clo, chi, t, kb, seg);
}

// Without the clamp flag.
__device__ __forceinline__ float pwl_eval_noclamp(float x, const DevTable& t, const float2* kb, int& seg)
{
    seg = seg_index(x, t.lo, t.inv_w, t.nseg);
    const float2 e = kb[seg];
    return __builtin_fmaf(e.x, x, e.y);
}

// A table of two segments (no clamp flag): both lines, and a compare against the smallest value of
// segment 1 (found on the host with the index arithmetic itself) instead of index, gather and one
// line.  The same value as pwl_eval_noclamp for every x, NaN and infinities included.
__device__ __forceinline__ float pwl_eval_two_segments(float x, const DevTable& t)
{
    const float y0 = __builtin_fmaf(t.k0, x, t.b0), y1 = __builtin_fmaf(t.k1, x, t.b1);
    return x >= t.tau ? y1 : y0;
}

// Symmetric int8 code: round-to-nearest-even of v * inv_scale, saturated to [-127, 127].
// Returns a word whose LOW BYTE is the code (the other bytes are not meaningful): saturate first
// (the bounds are integers and rounding is monotone, so clamp and round commute), then add
// 1.5 * 2^23: at that magnitude one ulp is 1, so the fp32 addition itself rounds to the nearest
// integer, ties to even, and the low mantissa bits are the two's-complement integer.  A NaN
// saturates to -127 (the median-of-three returns the smaller bound).
__device__ __forceinline__ int requant(float v, float inv_scale)
{
    float r = __builtin_amdgcn_fmed3f(v * inv_scale, -127.0f, 127.0f);
    return __float_as_int(r + 12582912.0f);
}

// Packs the low bytes of four words into one (a in byte 0).
__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d)
{
    const unsigned lo = __builtin_amdgcn_perm((unsigned)b, (unsigned)a, 0x0c0c0400u);  // a0 b0 0 0
    const unsigned hi = __builtin_amdgcn_perm((unsigned)d, (unsigned)c, 0x04000c0cu);  // 0 0 c0 d0
    return lo | hi;
}

// Copy a table's {k, b} pairs into LDS (all threads of the block take part; the caller
// synchronises before the first lookup).
__device__ __forceinline__ void stage_table(float2* dst, const DevTable& t)
{
    for (int i = threadIdx.x; i < t.nseg; i += blockDim.x) dst[i] = t.kb[i];
}

// Two-level form of a merged table (paper Algorithm 2: neighbouring primary segments with nearly
// equal slope share one line): nkb {k, b} pairs, then one byte per primary cell naming its merged
// segment.  LDS bytes: 8 * nkb + nseg (instead of 8 * nseg).
__device__ __forceinline__ size_t two_level_bytes(const DevTable& t) { return 8 * (size_t)t.nkb + (((size_t)t.nseg + 7) & ~(size_t)7); }
__device__ __forceinline__ void stage_table_two_level(float2* dst, const DevTable& t)
{
    for (int i = threadIdx.x; i < t.nkb; i += blockDim.x) dst[i] = t.ckb[i];
    uint8_t* map = reinterpret_cast<uint8_t*>(dst + t.nkb);
    for (int i = threadIdx.x; i < t.nseg; i += blockDim.x) map[i] = t.cellmap[i];
}

// Look-up in two steps: the primary cell of x exactly as for a uniform table (`cell` is what the
// debug outputs report), then that cell's merged segment.
__device__ __forceinline__ float pwl_eval_two_level(float x, const DevTable& t, const float2* staged, int& cell)
{
    const float xc = __builtin_amdgcn_fmed3f(x, t.lo, t.hi);
    x = t.clamp_input ? xc : x;
    cell = seg_index(x, t.lo, t.inv_w, t.nseg);
    const uint8_t* map = reinterpret_cast<const uint8_t*>(staged + t.nkb);
    const float2 e = staged[map[cell]];
    return __builtin_fmaf(e.x, x, e.y);
}

// Direct global -> LDS load: every lane supplies its own global address of 16 bytes; the wavefront's
// 1 KB lands contiguously at lds_addr (wave-uniform), lane i at lds_addr + 16*i.  Asynchronous:
// completion is tracked by the vector-memory counter (wait_vmcnt), not by the LDS counter.
// The LDS address travels in M0, which is an operand of the statement (the register allocator
// knows it is written here); one wait state separates the M0 write from its use.
__device__ __forceinline__ void dma16(const void* gptr, unsigned lds_addr)
{
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "{m0}"(lds_addr) : "memory");
}

// The same with a wave-uniform base pointer and a 32-bit per-lane byte offset (the k-loop then
// advances one scalar pointer instead of one 64-bit address per lane and load).
__device__ __forceinline__ void dma16s(const void* sbase, unsigned voff, unsigned lds_addr)
{
    asm volatile("s_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(voff), "s"(sbase), "{m0}"(lds_addr) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

}  // namespace nm
