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
// float -> int conversion (which truncates) IS the floor.
__device__ __forceinline__ int seg_index(float x, float lo, float inv_w, int nseg)
{
    float u = x - lo;
    u = u * inv_w;
    u = __builtin_fminf(__builtin_fmaxf(u, 0.0f), (float)(nseg - 1));
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

// Symmetric int8 code: round-to-nearest-even of v * inv_scale, saturated to [-127, 127].
__device__ __forceinline__ int requant(float v, float inv_scale)
{
    float r = __builtin_rintf(v * inv_scale);
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d)
{
    return (unsigned)(a & 0xff) | ((unsigned)(b & 0xff) << 8) | ((unsigned)(c & 0xff) << 16) |
           ((unsigned)(d & 0xff) << 24);
}

// Copy a table's {k, b} pairs into LDS (all threads of the block take part; the caller
// synchronises before the first lookup).
__device__ __forceinline__ void stage_table(float2* dst, const DevTable& t)
{
    for (int i = threadIdx.x; i < t.nseg; i += blockDim.x) dst[i] = t.kb[i];
}

}  // namespace nm
