/*
 * nm_oracle.c -- CPU oracle for the NeuralMatrix int8 + piecewise-linear (PWL) encoder path.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, obviously-correct restatement of what
 * the GPU library must compute.  Only the tests, the smoke check and the cpu_baseline leg of the
 * benchmark may call it.  It shares no code, header, table or constant with the GPU library and
 * must never be imported by the product path.
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC nm_oracle.c -o libnm_oracle.so -lm
 * (contraction is OFF: every fused multiply-add below is an explicit fmaf()).
 *
 * What follows the paper, and where:
 *   - PWL tables: Section 3.2 "Post-Training Approximation" (fixed-length segments, one line per
 *     segment through the function values at the two segment ends, so neighbouring lines meet;
 *     inputs outside the range use the first / last segment's line) and the first step of
 *     Algorithm 3 (k_i, b_i of the chord).
 *   - Vertical bias correction: Algorithm 3 and Section 3.2 "Vertical Bias Correction"
 *     (shift b_i by the difference between the segment mean of f and the segment mean of the
 *     chord).
 *   - Horizontal size optimisation: Algorithm 2 and Section 3.2 "Horizontal Size Optimization".
 *   - Run-time PWL evaluation: Section 3 overview (operations that are, or have been made,
 *     piecewise linear are evaluated by one common PWL calculation): find the segment of each
 *     element, gather that segment's k and b, evaluate y = k*x + b element-wise.
 *   - Linear operations as matrix multiply/add: Section 3.1.
 * The paper does not say how softmax and LayerNorm are decomposed, how tensors are quantised to
 * INT8, or in which order sums are taken.  The readings used here are listed next to each
 * function; they are the normative definition for the GPU library as well.
 *
 * Precision: integer work is exact.  Floating-point work is IEEE binary32 with round-to-nearest-
 * even, in exactly the operation order written here, because fp32 values decide integers (segment
 * indices, int8 codes) and both sides must take those decisions in the same precision.  The
 * "exact" functions at the end use binary64 and the true nonlinear functions; they provide the
 * calibration ranges (Section 3.2 step 1: obtain the input range by running the model) and the
 * accuracy reference.
 *
 * Pins (tests/test_oracle_*.py): table end-point interpolation, analytic chord error bound,
 * affine functions reproduced exactly, ReLU exact, brute-force segment search over all int8
 * inputs, integer GEMM against an int64 library matmul, rounding ties, hand-derived summation-
 * order cases, softmax shift invariance / constant rows / distance to true softmax, LayerNorm
 * constant rows / distance to a library layer norm, mean preservation and the 5/6 MSE asymptote of
 * Algorithm 3, the worked GELU merge example of Algorithm 2, exact-mode layer against a library
 * fp64 transformer layer.  Parity unpinned: the aggregate percentages the paper reports for
 * Algorithms 2 and 3 (their ranges and hyper-parameters are not given).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define NMO_OK 0
#define NMO_ERR_ARG (-1)
#define NMO_ERR_ALLOC (-3)

enum { NMO_F_GELU = 0, NMO_F_EXP = 1, NMO_F_RECIP = 2, NMO_F_RSQRT = 3, NMO_F_RELU = 4,
       NMO_F_SQRT = 5, NMO_F_IDENTITY = 6 };
enum { NMO_FLAG_CLAMP_INPUT = 1, NMO_FLAG_BIAS_CORRECT = 2 };
enum { NMO_DT_I32 = 0, NMO_DT_F32 = 1 };

typedef double (*nmo_fn)(double);

/* One uniform PWL table.  k and b point at nseg floats each. */
typedef struct {
    float lo;
    float hi;
    float inv_w; /* (float)(nseg / (hi - lo)), the division done in binary64 */
    int32_t nseg;
    int32_t flags;
    const float* k;
    const float* b;
} nmo_table;

/* ------------------------------------------------------------------------------------------- */
/* The nonlinear functions and their antiderivatives, binary64.                                 */
/* ------------------------------------------------------------------------------------------- */

static double std_normal_cdf(double x) { return 0.5 * (1.0 + erf(x / sqrt(2.0))); }
static double std_normal_pdf(double x) { return exp(-0.5 * x * x) / sqrt(2.0 * acos(-1.0)); }

/* GELU(x) = x * Phi(x) (the erf form; the paper only names the function). */
static double f_gelu(double x) { return x * std_normal_cdf(x); }
static double f_exp(double x) { return exp(x); }
static double f_recip(double x) { return 1.0 / x; }
static double f_rsqrt(double x) { return 1.0 / sqrt(x); }
static double f_relu(double x) { return x > 0.0 ? x : 0.0; }
static double f_sqrt(double x) { return sqrt(x); }
static double f_identity(double x) { return x; }

/* Antiderivatives, used only for the segment mean of Algorithm 3. */
static double F_gelu(double x)
{
    return 0.5 * ((x * x - 1.0) * std_normal_cdf(x) + x * std_normal_pdf(x));
}
static double F_exp(double x) { return exp(x); }
static double F_recip(double x) { return log(x); }
static double F_rsqrt(double x) { return 2.0 * sqrt(x); }
static double F_relu(double x) { return x > 0.0 ? 0.5 * x * x : 0.0; }
static double F_sqrt(double x) { return (2.0 / 3.0) * x * sqrt(x); }
static double F_identity(double x) { return 0.5 * x * x; }

static nmo_fn fn_of(int func)
{
    switch (func) {
    case NMO_F_GELU: return f_gelu;
    case NMO_F_EXP: return f_exp;
    case NMO_F_RECIP: return f_recip;
    case NMO_F_RSQRT: return f_rsqrt;
    case NMO_F_RELU: return f_relu;
    case NMO_F_SQRT: return f_sqrt;
    case NMO_F_IDENTITY: return f_identity;
    default: return NULL;
    }
}
static nmo_fn antiderivative_of(int func)
{
    switch (func) {
    case NMO_F_GELU: return F_gelu;
    case NMO_F_EXP: return F_exp;
    case NMO_F_RECIP: return F_recip;
    case NMO_F_RSQRT: return F_rsqrt;
    case NMO_F_RELU: return F_relu;
    case NMO_F_SQRT: return F_sqrt;
    case NMO_F_IDENTITY: return F_identity;
    default: return NULL;
    }
}

/* Evaluate one of the built-in functions (for tests and accuracy reports). */
double nmo_eval_fn(int func, double x)
{
    nmo_fn f = fn_of(func);
    return f ? f(x) : NAN;
}

/* ------------------------------------------------------------------------------------------- */
/* Algorithm 3: chord of f over [x0, x1], optionally shifted by the expectation bias.           */
/* ------------------------------------------------------------------------------------------- */

/*
 * k = (f(x1) - f(x0)) / (x1 - x0),  b = f(x0) - k*x0.
 * dE = mean of f over the segment - (f(x0) + f(x1)) / 2   (the chord's mean is the average of
 * its end values).  Reading of the condition: the algorithm box applies the shift when
 * dE <= E_th while the text applies it when the difference exceeds the threshold; the text's
 * intent is followed: shift when |dE| > e_th (e_th = 0 shifts always).
 * F is an antiderivative of f; with F == NULL no correction is made.
 */
static void chord_segment(nmo_fn f, nmo_fn F, double x0, double x1, int correct, double e_th,
                          double* k, double* b)
{
    double f0 = f(x0), f1 = f(x1);
    double kk = (f1 - f0) / (x1 - x0);
    double bb = f0 - kk * x0;
    if (correct && F) {
        double dE = (F(x1) - F(x0)) / (x1 - x0) - 0.5 * (f0 + f1);
        if (fabs(dE) > e_th) bb += dE;
    }
    *k = kk;
    *b = bb;
}

/*
 * Uniform table (Section 3.2, Post-Training Approximation): nseg segments of equal length
 * w = (hi - lo) / nseg, break points x_i = lo + i*w, all in binary64; the results are rounded
 * once to binary32.
 */
int nmo_table_build_fn(nmo_fn f, nmo_fn F, float lo, float hi, int32_t nseg, int32_t flags,
                       double e_th, float* k, float* b, float* inv_w)
{
    if (!f || !k || !b || !inv_w || nseg < 1 || !(hi > lo)) return NMO_ERR_ARG;
    double L = (double)lo, R = (double)hi;
    double w = (R - L) / (double)nseg;
    for (int32_t i = 0; i < nseg; ++i) {
        double x0 = L + (double)i * w;
        double x1 = L + (double)(i + 1) * w;
        double kk, bb;
        chord_segment(f, F, x0, x1, (flags & NMO_FLAG_BIAS_CORRECT) != 0, e_th, &kk, &bb);
        k[i] = (float)kk;
        b[i] = (float)bb;
    }
    *inv_w = (float)((double)nseg / (R - L));
    return NMO_OK;
}

int nmo_table_build(int32_t func, float lo, float hi, int32_t nseg, int32_t flags, double e_th,
                    float* k, float* b, float* inv_w)
{
    return nmo_table_build_fn(fn_of(func), antiderivative_of(func), lo, hi, nseg, flags, e_th, k,
                              b, inv_w);
}

/* ------------------------------------------------------------------------------------------- */
/* Algorithm 2: horizontal size optimisation.                                                   */
/* ------------------------------------------------------------------------------------------- */

/*
 * Walk the primary segments of length dlx from r_min.  `kept` is the slope of the primary segment
 * at the last start point that was recorded.  A primary segment whose slope differs from `kept`
 * by more than dk_th starts a new merged segment.  Reading of the box's index bookkeeping: the
 * cursor is a running position, separate from the stored points; (r_max - r_min) / dlx must be a
 * whole number so that no evaluation falls outside the range.  Returns the number of start points
 * written to xs (r_min first); xs must hold nprimary doubles.
 */
int32_t nmo_size_optimize(nmo_fn f, double r_min, double r_max, double dlx, double dk_th,
                          double* xs, int32_t cap)
{
    if (!f || !xs || cap < 1 || !(dlx > 0.0) || !(r_max > r_min)) return NMO_ERR_ARG;
    double nd = (r_max - r_min) / dlx;
    int32_t nprimary = (int32_t)llround(nd);
    if (nprimary < 1 || fabs(nd - (double)nprimary) > 1e-9 * nd) return NMO_ERR_ARG;
    int32_t n = 0;
    xs[n++] = r_min;
    double kept = (f(r_min + dlx) - f(r_min)) / dlx;
    for (int32_t j = 1; j < nprimary; ++j) {
        double x = r_min + (double)j * dlx;
        double kj = (f(r_min + (double)(j + 1) * dlx) - f(x)) / dlx;
        if (fabs(kj - kept) <= dk_th) continue; /* merge with the running segment */
        if (n >= cap) return NMO_ERR_ARG;
        xs[n++] = x;
        kept = kj;
    }
    return n;
}

int32_t nmo_size_optimize_builtin(int32_t func, double r_min, double r_max, double dlx,
                                  double dk_th, double* xs, int32_t cap)
{
    return nmo_size_optimize(fn_of(func), r_min, r_max, dlx, dk_th, xs, cap);
}

/*
 * Chords (Algorithm 3) over the merged segments [xs[i], xs[i+1]) with xs[n] = r_max, expanded
 * onto the uniform primary grid of nprimary cells so that the uniform segment search below can
 * evaluate it: every primary cell inside a merged segment carries that segment's k and b.
 */
int nmo_table_build_merged(int32_t func, float lo, float hi, int32_t nprimary, double dk_th,
                           int32_t flags, double e_th, float* k, float* b, float* inv_w,
                           int32_t* n_merged)
{
    nmo_fn f = fn_of(func), F = antiderivative_of(func);
    if (!f || !k || !b || !inv_w || nprimary < 1 || !(hi > lo)) return NMO_ERR_ARG;
    double L = (double)lo, R = (double)hi;
    double w = (R - L) / (double)nprimary;
    double* xs = (double*)malloc(sizeof(double) * (size_t)(nprimary + 1));
    if (!xs) return NMO_ERR_ALLOC;
    int32_t n = nmo_size_optimize(f, L, R, w, dk_th, xs, nprimary);
    if (n < 1) { free(xs); return NMO_ERR_ARG; }
    xs[n] = R;
    int32_t cell = 0;
    for (int32_t i = 0; i < n; ++i) {
        double kk, bb;
        chord_segment(f, F, xs[i], xs[i + 1], (flags & NMO_FLAG_BIAS_CORRECT) != 0, e_th, &kk, &bb);
        /* cells whose left edge lies in [xs[i], xs[i+1]) */
        while (cell < nprimary && L + ((double)cell + 0.5) * w < xs[i + 1]) {
            k[cell] = (float)kk;
            b[cell] = (float)bb;
            ++cell;
        }
    }
    *inv_w = (float)((double)nprimary / (R - L));
    if (n_merged) *n_merged = n;
    free(xs);
    return NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* Run-time PWL: segment index, evaluation, requantisation.                                     */
/* ------------------------------------------------------------------------------------------- */

/*
 * Segment of x ("quantising x"): u = (x - lo) * inv_w with one fp32 subtract and one fp32
 * multiply, clamped IN FLOAT to [0, nseg-1], then floor.  A break point belongs to the segment on
 * its right; x >= hi lands in the last segment and x < lo (and NaN) in the first, which is the
 * paper's rule that out-of-range inputs share the parameters of the edge segments.
 */
static inline int32_t segidx(float x, const nmo_table* t)
{
    float u = x - t->lo;
    u = u * t->inv_w;
    u = fminf(fmaxf(u, 0.0f), (float)(t->nseg - 1));
    return (int32_t)floorf(u);
}

/* y = k[s]*x + b[s] as one fused multiply-add.  With CLAMP_INPUT x is first clamped to [lo,hi]. */
static inline float pwl_eval(float x, const nmo_table* t, int32_t* seg_out)
{
    if (t->flags & NMO_FLAG_CLAMP_INPUT) x = fminf(fmaxf(x, t->lo), t->hi);
    int32_t s = segidx(x, t);
    if (seg_out) *seg_out = s;
    return fmaf(t->k[s], x, t->b[s]);
}

/* Symmetric int8 code: round-to-nearest-even of v*inv_scale, saturated to [-127, 127]. */
static inline int8_t requant(float v, float inv_scale)
{
    float r = rintf(v * inv_scale);
    r = fminf(fmaxf(r, -127.0f), 127.0f);
    return (int8_t)r;
}

int32_t nmo_segidx(float x, const nmo_table* t) { return segidx(x, t); }
float nmo_pwl_eval(float x, const nmo_table* t) { return pwl_eval(x, t, NULL); }
int8_t nmo_requant(float v, float inv_scale) { return requant(v, inv_scale); }

/*
 * Stand-alone element-wise PWL over a flat buffer.  int32 input is first converted to fp32 and
 * multiplied by alpha; fp32 input is multiplied by alpha as well (alpha = 1 leaves it unchanged).
 */
int nmo_pwl_apply(const void* in, int32_t in_dtype, float alpha, int64_t n, const nmo_table* t,
                  float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg)
{
    if (!in || !t || n < 0) return NMO_ERR_ARG;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        float x = (in_dtype == NMO_DT_I32) ? (float)((const int32_t*)in)[i] * alpha
                                           : ((const float*)in)[i] * alpha;
        int32_t s;
        float y = pwl_eval(x, t, &s);
        if (out_f32) out_f32[i] = y;
        if (out_q) out_q[i] = requant(y, out_inv_scale);
        if (dbg_seg) dbg_seg[i] = (uint16_t)s;
    }
    return NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* A merged table in its own form (Algorithm 2's output), evaluated directly.                   */
/* ------------------------------------------------------------------------------------------- */

/*
 * Algorithm 2 returns start points, all of them multiples of the primary length dLx from r_min;
 * merged segment i covers [x_i, x_{i+1}) and has one line (Algorithm 3).  Here the start points are
 * kept as primary-cell numbers (x_i = lo + start_cell[i] * dLx, start_cell[0] = 0, increasing).
 */
typedef struct {
    float lo, hi;
    float inv_w;            /* (float)(nprimary / (hi - lo)) */
    int32_t nprimary;       /* primary cells of length dLx */
    int32_t flags;          /* NMO_FLAG_CLAMP_INPUT */
    int32_t nseg;           /* merged segments */
    const int32_t* start_cell; /* [nseg] */
    const float* k;         /* [nseg] */
    const float* b;         /* [nseg] */
} nmo_merged_table;

/* Start cells and one chord per merged segment (no expansion onto the primary grid). */
int nmo_table_build_merged_direct(int32_t func, float lo, float hi, int32_t nprimary, double dk_th,
                                  int32_t flags, double e_th, int32_t* start_cell, float* k, float* b,
                                  float* inv_w, int32_t* n_merged)
{
    nmo_fn f = fn_of(func), F = antiderivative_of(func);
    if (!f || !start_cell || !k || !b || !inv_w || !n_merged || nprimary < 1 || !(hi > lo)) return NMO_ERR_ARG;
    double L = (double)lo, R = (double)hi;
    double w = (R - L) / (double)nprimary;
    double* xs = (double*)malloc(sizeof(double) * (size_t)(nprimary + 1));
    if (!xs) return NMO_ERR_ALLOC;
    int32_t n = nmo_size_optimize(f, L, R, w, dk_th, xs, nprimary);
    if (n < 1) { free(xs); return NMO_ERR_ARG; }
    xs[n] = R;
    for (int32_t i = 0; i < n; ++i) {
        double kk, bb;
        chord_segment(f, F, xs[i], xs[i + 1], (flags & NMO_FLAG_BIAS_CORRECT) != 0, e_th, &kk, &bb);
        k[i] = (float)kk;
        b[i] = (float)bb;
        start_cell[i] = (int32_t)llround((xs[i] - L) / w);
    }
    *inv_w = (float)((double)nprimary / (R - L));
    *n_merged = n;
    free(xs);
    return NMO_OK;
}

/*
 * Evaluation: x is quantised to its primary cell exactly as for a uniform table (one subtract, one
 * multiply, clamp in float, floor: inputs outside the range fall into the edge cells and so share
 * the edge segments' parameters), then the merged segment is the one whose start point is the last
 * at or below that cell (binary search over the start points), then y = fma(k, x, b).
 */
int nmo_pwl_apply_merged(const void* in, int32_t in_dtype, float alpha, int64_t n,
                         const nmo_merged_table* t, float out_inv_scale, int8_t* out_q, float* out_f32,
                         uint16_t* dbg_seg, uint16_t* dbg_cell)
{
    if (!in || !t || n < 0 || t->nseg < 1 || t->start_cell[0] != 0) return NMO_ERR_ARG;
    for (int64_t i = 0; i < n; ++i) {
        float x = (in_dtype == NMO_DT_I32) ? (float)((const int32_t*)in)[i] * alpha
                                           : ((const float*)in)[i] * alpha;
        if (t->flags & NMO_FLAG_CLAMP_INPUT) x = fminf(fmaxf(x, t->lo), t->hi);
        float u = x - t->lo;
        u = u * t->inv_w;
        u = fminf(fmaxf(u, 0.0f), (float)(t->nprimary - 1));
        int32_t cell = (int32_t)floorf(u);
        int32_t lo_i = 0, hi_i = t->nseg - 1;      /* last start point <= cell */
        while (lo_i < hi_i) {
            int32_t mid = (lo_i + hi_i + 1) / 2;
            if (t->start_cell[mid] <= cell) lo_i = mid; else hi_i = mid - 1;
        }
        float y = fmaf(t->k[lo_i], x, t->b[lo_i]);
        if (out_f32) out_f32[i] = y;
        if (out_q) out_q[i] = requant(y, out_inv_scale);
        if (dbg_seg) dbg_seg[i] = (uint16_t)lo_i;
        if (dbg_cell) dbg_cell[i] = (uint16_t)cell;
    }
    return NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* Canonical row reduction.                                                                     */
/* ------------------------------------------------------------------------------------------- */

/*
 * The order of a row sum decides fp32 bits, and those decide segment indices, so ONE order is
 * normative (the paper is silent on it).  A row is dealt to 64 accumulators in groups of four
 * consecutive elements: element j belongs to accumulator (j / 4) % 64.  Each accumulator starts
 * at +0 and adds its elements in increasing j.  The 64 partial sums are then combined by a
 * butterfly: for mask = 32, 16, 8, 4, 2, 1 every accumulator a becomes v[a] + v[a xor mask].
 * Addition commutes, so all 64 end with the same value.
 * sq != 0 accumulates x*x with a fused multiply-add instead of x.
 */
static float canonical_sum(const float* x, int32_t n, int sq)
{
    float v[64];
    for (int a = 0; a < 64; ++a) v[a] = 0.0f;
    for (int32_t j = 0; j < n; ++j) {
        int a = (j / 4) % 64;
        v[a] = sq ? fmaf(x[j], x[j], v[a]) : v[a] + x[j];
    }
    for (int mask = 32; mask >= 1; mask >>= 1) {
        float w[64];
        for (int a = 0; a < 64; ++a) w[a] = v[a] + v[a ^ mask];
        for (int a = 0; a < 64; ++a) v[a] = w[a];
    }
    return v[0];
}

float nmo_canonical_sum(const float* x, int32_t n) { return canonical_sum(x, n, 0); }
float nmo_canonical_sumsq(const float* x, int32_t n) { return canonical_sum(x, n, 1); }

/* ------------------------------------------------------------------------------------------- */
/* Softmax with PWL exp and PWL reciprocal.                                                     */
/* ------------------------------------------------------------------------------------------- */

/*
 * Per row (reading; the paper lists e^x and 1/x among its functions but not the decomposition):
 *   m   = max_j in_j                      (integer max for int32 input)
 *   t_j = (float)(in_j - m) * alpha       (the subtraction is exact for int32 input)
 *   e_j = PWL_exp(t_j)
 *   S   = canonical_sum(e)
 *   r   = PWL_recip(S)
 *   p_j = e_j * r
 * Outputs: p (fp32), its int8 code, the exp segment of every element, the recip segment per row.
 */
int nmo_softmax_pwl(const void* in, int32_t in_dtype, float alpha, int64_t rows, int32_t cols,
                    const nmo_table* t_exp, const nmo_table* t_recip, float out_inv_scale,
                    int8_t* out_q, float* out_f32, uint16_t* dbg_seg_exp, uint16_t* dbg_seg_recip)
{
    if (!in || !t_exp || !t_recip || rows < 0 || cols < 1) return NMO_ERR_ARG;
    int err = 0;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float* e = (float*)malloc(sizeof(float) * (size_t)cols);
        if (!e) { err = 1; continue; }
        size_t base = (size_t)r * (size_t)cols;
        if (in_dtype == NMO_DT_I32) {
            const int32_t* a = (const int32_t*)in + base;
            int32_t m = a[0];
            for (int32_t j = 1; j < cols; ++j) if (a[j] > m) m = a[j];
            for (int32_t j = 0; j < cols; ++j) {
                float t = (float)(a[j] - m) * alpha;
                int32_t s;
                e[j] = pwl_eval(t, t_exp, &s);
                if (dbg_seg_exp) dbg_seg_exp[base + j] = (uint16_t)s;
            }
        } else {
            const float* a = (const float*)in + base;
            float m = a[0];
            for (int32_t j = 1; j < cols; ++j) m = fmaxf(m, a[j]);
            for (int32_t j = 0; j < cols; ++j) {
                float t = (a[j] - m) * alpha;
                int32_t s;
                e[j] = pwl_eval(t, t_exp, &s);
                if (dbg_seg_exp) dbg_seg_exp[base + j] = (uint16_t)s;
            }
        }
        float S = canonical_sum(e, cols, 0);
        int32_t sr;
        float rcp = pwl_eval(S, t_recip, &sr);
        if (dbg_seg_recip) dbg_seg_recip[r] = (uint16_t)sr;
        for (int32_t j = 0; j < cols; ++j) {
            float p = e[j] * rcp;
            if (out_f32) out_f32[base + j] = p;
            if (out_q) out_q[base + j] = requant(p, out_inv_scale);
        }
        free(e);
    }
    return err ? NMO_ERR_ALLOC : NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* LayerNorm with PWL reciprocal square root.                                                   */
/* ------------------------------------------------------------------------------------------- */

/*
 * Per row of length L (reading; the paper lists sqrt and 1/x, the build's workload definition
 * uses one rsqrt table):
 *   mu  = canonical_sum(x) * inv_L                inv_L = (float)(1.0 / L)
 *   d_j = x_j - mu
 *   var = canonical_sum of d_j*d_j (fused multiply-add accumulation) * inv_L
 *   u   = var + eps
 *   r   = PWL_rsqrt(u)
 *   y_j = fmaf(d_j * r, gamma_j, beta_j)
 */
static int layernorm_core(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const nmo_table* t_rsqrt, const nmo_table* t_recip,
                          float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg,
                          uint16_t* dbg_seg2)
{
    if (!in || !gamma || !beta || !t_rsqrt || rows < 0 || cols < 1) return NMO_ERR_ARG;
    const float inv_L = (float)(1.0 / (double)cols);
    int err = 0;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        float* d = (float*)malloc(sizeof(float) * (size_t)cols);
        if (!d) { err = 1; continue; }
        size_t base = (size_t)r * (size_t)cols;
        const float* x = in + base;
        float mu = canonical_sum(x, cols, 0) * inv_L;
        for (int32_t j = 0; j < cols; ++j) d[j] = x[j] - mu;
        float var = canonical_sum(d, cols, 1) * inv_L;
        float u = var + eps;
        int32_t s;
        float rs = pwl_eval(u, t_rsqrt, &s);   /* rsqrt table, or sqrt table when t_recip is given */
        if (dbg_seg) dbg_seg[r] = (uint16_t)s;
        if (t_recip) {
            int32_t s2;
            rs = pwl_eval(rs, t_recip, &s2);
            if (dbg_seg2) dbg_seg2[r] = (uint16_t)s2;
        }
        for (int32_t j = 0; j < cols; ++j) {
            float y = fmaf(d[j] * rs, gamma[j], beta[j]);
            if (out_f32) out_f32[base + j] = y;
            if (out_q) out_q[base + j] = requant(y, out_inv_scale);
        }
        free(d);
    }
    return err ? NMO_ERR_ALLOC : NMO_OK;
}

int nmo_layernorm_pwl(const float* in, const float* gamma, const float* beta, float eps,
                      int64_t rows, int32_t cols, const nmo_table* t_rsqrt, float out_inv_scale,
                      int8_t* out_q, float* out_f32, uint16_t* dbg_seg)
{
    return layernorm_core(in, gamma, beta, eps, rows, cols, t_rsqrt, NULL, out_inv_scale, out_q, out_f32,
                          dbg_seg, NULL);
}

/*
 * The variant with the two functions the paper's list names (square root and reciprocal) instead of
 * one rsqrt table: sd = PWL_sqrt(var + eps); r = PWL_recip(sd); everything else as above.
 */
int nmo_layernorm_pwl2(const float* in, const float* gamma, const float* beta, float eps,
                       int64_t rows, int32_t cols, const nmo_table* t_sqrt, const nmo_table* t_recip,
                       float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg_sqrt,
                       uint16_t* dbg_seg_recip)
{
    if (!t_recip) return NMO_ERR_ARG;
    return layernorm_core(in, gamma, beta, eps, rows, cols, t_sqrt, t_recip, out_inv_scale, out_q, out_f32,
                          dbg_seg_sqrt, dbg_seg_recip);
}

/* ------------------------------------------------------------------------------------------- */
/* int8 GEMM with the fused dequantise / bias / residual / PWL / requantise epilogue.           */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t M, N, K;
    const int8_t* A;             /* [M, K], K contiguous */
    const int8_t* W;             /* [N, K], K contiguous (a fully connected layer's weight) */
    const float* bias;           /* [N] or NULL */
    const float* alpha_vec;      /* [N] per-column dequantisation scale, or NULL -> alpha */
    float alpha;
    const int8_t* resid;         /* [M, N] int8 residual or NULL */
    float resid_scale;
    const nmo_table* table;      /* NULL -> no nonlinearity */
    float out_inv_scale;
    const float* out_inv_scale_vec; /* [N] per-column or NULL -> out_inv_scale */
    int8_t* out_q;               /* any of the outputs may be NULL */
    float* out_f32;
    int32_t* out_acc;
    uint16_t* dbg_seg;
} nmo_gemm;

/*
 * acc[m,n] = sum_k A[m,k] * W[n,k]            exact in int32 (Section 3.1: a fully connected
 *                                              layer is a matrix multiplication)
 * v = fmaf((float)acc, alpha_n, bias_n)        int -> float conversion rounds to nearest even
 * v = fmaf((float)resid[m,n], resid_scale, v)  if a residual is given (matrix addition)
 * v = PWL(v)                                   if a table is given
 * outputs: v, requant(v), acc, segment index
 */
int nmo_gemm_pwl(const nmo_gemm* g)
{
    if (!g || !g->A || !g->W || g->M < 0 || g->N < 1 || g->K < 1) return NMO_ERR_ARG;
    const int32_t M = g->M, N = g->N, K = g->K;
#pragma omp parallel for schedule(static)
    for (int32_t m = 0; m < M; ++m) {
        const int8_t* a = g->A + (size_t)m * K;
        for (int32_t n = 0; n < N; ++n) {
            const int8_t* w = g->W + (size_t)n * K;
            int32_t acc = 0;
            for (int32_t k = 0; k < K; ++k) acc += (int32_t)a[k] * (int32_t)w[k];
            size_t o = (size_t)m * N + n;
            if (g->out_acc) g->out_acc[o] = acc;
            float scale = g->alpha_vec ? g->alpha_vec[n] : g->alpha;
            float v = fmaf((float)acc, scale, g->bias ? g->bias[n] : 0.0f);
            if (g->resid) v = fmaf((float)g->resid[o], g->resid_scale, v);
            if (g->table) {
                int32_t s;
                v = pwl_eval(v, g->table, &s);
                if (g->dbg_seg) g->dbg_seg[o] = (uint16_t)s;
            }
            if (g->out_f32) g->out_f32[o] = v;
            if (g->out_q)
                g->out_q[o] = requant(v, g->out_inv_scale_vec ? g->out_inv_scale_vec[n]
                                                              : g->out_inv_scale);
        }
    }
    return NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* int8 convolution (NHWC) with the same fused epilogue, and the two pooling operators of a    */
/* residual CNN.                                                                                */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t B, H, W, Cin;        /* input  x: int8 [B, H, W, Cin] (channels contiguous) */
    int32_t Cout, kh, kw;        /* weight w: int8 [Cout, kh, kw, Cin] */
    int32_t stride, pad;         /* same in both directions; padding is the zero code */
    const int8_t* x;
    const int8_t* w;
    const float* bias;           /* [Cout] or NULL */
    const float* alpha_vec;      /* [Cout] per-channel scale (a folded batch normalisation), or NULL -> alpha */
    float alpha;
    const int8_t* resid;         /* [B, Ho, Wo, Cout] int8 residual or NULL */
    float resid_scale;
    const nmo_table* table;      /* NULL -> no nonlinearity */
    float out_inv_scale;
    int8_t* out_q;               /* [B, Ho, Wo, Cout]; any output may be NULL */
    float* out_f32;
    int32_t* out_acc;
} nmo_conv;

/*
 * Section 3.1: a convolution is a linear operation whose matrix form has one row per output
 * position and one column per output channel; written here as its direct definition,
 *   acc[b,ho,wo,n] = sum_{i<kh, j<kw, c<Cin} x[b, ho*stride - pad + i, wo*stride - pad + j, c] * w[n,i,j,c]
 * (positions outside the image contribute nothing), exact in int32, followed by the epilogue of
 * the matrix product: v = fmaf((float)acc, alpha_n, bias_n); residual; PWL; requantise.
 * Ho = (H + 2 pad - kh) / stride + 1, Wo likewise.
 */
int nmo_conv2d_pwl(const nmo_conv* g)
{
    if (!g || !g->x || !g->w || g->B < 0 || g->H < 1 || g->W < 1 || g->Cin < 1 || g->Cout < 1 ||
        g->kh < 1 || g->kw < 1 || g->stride < 1 || g->pad < 0)
        return NMO_ERR_ARG;
    if (g->H + 2 * g->pad < g->kh || g->W + 2 * g->pad < g->kw) return NMO_ERR_ARG;
    const int32_t Ho = (g->H + 2 * g->pad - g->kh) / g->stride + 1;
    const int32_t Wo = (g->W + 2 * g->pad - g->kw) / g->stride + 1;
    const int64_t rows = (int64_t)g->B * Ho * Wo;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const int32_t wo = (int32_t)(r % Wo), ho = (int32_t)((r / Wo) % Ho), b = (int32_t)(r / ((int64_t)Wo * Ho));
        for (int32_t n = 0; n < g->Cout; ++n) {
            int32_t acc = 0;
            for (int32_t i = 0; i < g->kh; ++i) {
                const int32_t hi = ho * g->stride - g->pad + i;
                if (hi < 0 || hi >= g->H) continue;
                for (int32_t j = 0; j < g->kw; ++j) {
                    const int32_t wi = wo * g->stride - g->pad + j;
                    if (wi < 0 || wi >= g->W) continue;
                    const int8_t* xp = g->x + (((size_t)b * g->H + hi) * g->W + wi) * g->Cin;
                    const int8_t* wp = g->w + (((size_t)n * g->kh + i) * g->kw + j) * g->Cin;
                    for (int32_t c = 0; c < g->Cin; ++c) acc += (int32_t)xp[c] * (int32_t)wp[c];
                }
            }
            const size_t o = (size_t)r * g->Cout + n;
            if (g->out_acc) g->out_acc[o] = acc;
            float v = fmaf((float)acc, g->alpha_vec ? g->alpha_vec[n] : g->alpha, g->bias ? g->bias[n] : 0.0f);
            if (g->resid) v = fmaf((float)g->resid[o], g->resid_scale, v);
            if (g->table) {
                int32_t s;
                v = pwl_eval(v, g->table, &s);
            }
            if (g->out_f32) g->out_f32[o] = v;
            if (g->out_q) g->out_q[o] = requant(v, g->out_inv_scale);
        }
    }
    return NMO_OK;
}

/*
 * Max pooling over k x k windows (stride, zero-free padding: positions outside the image are
 * left out of the maximum).  The paper does not discuss pooling; the maximum of int8 codes that
 * share one scale is exact and order-free, so it is taken directly on the codes.
 * x: int8 [B, H, W, C] -> y: int8 [B, Ho, Wo, C].
 */
int nmo_maxpool_i8(const int8_t* x, int32_t B, int32_t H, int32_t W, int32_t C, int32_t k,
                   int32_t stride, int32_t pad, int8_t* y)
{
    if (!x || !y || B < 0 || H < 1 || W < 1 || C < 1 || k < 1 || stride < 1 || pad < 0 || pad >= k)
        return NMO_ERR_ARG;
    const int32_t Ho = (H + 2 * pad - k) / stride + 1, Wo = (W + 2 * pad - k) / stride + 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < (int64_t)B * Ho * Wo; ++r) {
        const int32_t wo = (int32_t)(r % Wo), ho = (int32_t)((r / Wo) % Ho), b = (int32_t)(r / ((int64_t)Wo * Ho));
        for (int32_t c = 0; c < C; ++c) {
            int32_t best = -128;
            for (int32_t i = 0; i < k; ++i)
                for (int32_t j = 0; j < k; ++j) {
                    const int32_t hi = ho * stride - pad + i, wi = wo * stride - pad + j;
                    if (hi < 0 || hi >= H || wi < 0 || wi >= W) continue;
                    const int32_t v = x[(((size_t)b * H + hi) * W + wi) * C + c];
                    if (v > best) best = v;
                }
            y[(size_t)r * C + c] = (int8_t)best;
        }
    }
    return NMO_OK;
}

/*
 * Global average pooling, a linear operation (Section 3.1: a product with a constant matrix):
 * acc[b,c] = sum over the H*W positions of x[b,.,.,c] (exact in int32),
 * v = (float)acc * alpha with alpha = (float)(s_x / (H*W)) supplied by the caller, requantised.
 * x: int8 [B, HW, C] -> out_q int8 [B, C], out_f32 fp32 [B, C] (either may be NULL).
 */
int nmo_avgpool_i8(const int8_t* x, int32_t B, int32_t HW, int32_t C, float alpha,
                   float out_inv_scale, int8_t* out_q, float* out_f32)
{
    if (!x || B < 0 || HW < 1 || C < 1) return NMO_ERR_ARG;
    for (int32_t b = 0; b < B; ++b)
        for (int32_t c = 0; c < C; ++c) {
            int32_t acc = 0;
            for (int32_t p = 0; p < HW; ++p) acc += x[((size_t)b * HW + p) * C + c];
            const float v = (float)acc * alpha;
            if (out_f32) out_f32[(size_t)b * C + c] = v;
            if (out_q) out_q[(size_t)b * C + c] = requant(v, out_inv_scale);
        }
    return NMO_OK;
}

/* ------------------------------------------------------------------------------------------- */
/* One post-LayerNorm transformer encoder layer (BERT ordering), no mask, no dropout.           */
/* ------------------------------------------------------------------------------------------- */

typedef struct {
    int32_t B, S, H, heads, F;
    const int8_t* Wqkv; const float* bqkv; /* [3H, H] rows: Wq, Wk, Wv; [3H] */
    const int8_t* Wo;   const float* bo;   /* [H, H], [H] */
    const int8_t* W1;   const float* b1;   /* [F, H], [F] */
    const int8_t* W2;   const float* b2;   /* [H, F], [H] */
    const float* gamma1; const float* beta1; /* [H] */
    const float* gamma2; const float* beta2; /* [H] */
    float eps1, eps2;
    /* fp32 multipliers, already formed by the caller from the tensors' scales */
    float alpha_qkv;            /* s_x * s_wqkv */
    float inv_s_q, inv_s_k, inv_s_v;
    float alpha_scores;         /* s_q * s_k / sqrt(d) */
    float inv_s_p;
    float alpha_ctx;            /* s_p * s_v */
    float inv_s_ctx;
    float alpha_o;              /* s_ctx * s_wo */
    float resid1_scale;         /* s_x */
    float inv_s_ln1;
    float alpha_1;              /* s_ln1 * s_w1 */
    float inv_s_ffn1;
    float alpha_2;              /* s_ffn1 * s_w2 */
    float resid2_scale;         /* s_ln1 */
    float inv_s_out;
    const nmo_table* t_gelu;
    const nmo_table* t_exp;
    const nmo_table* t_recip;
    const nmo_table* t_rsqrt;
} nmo_layer;

/* Optional copies of every intermediate tensor (any pointer may be NULL). */
typedef struct {
    int8_t* qkv;      /* [M, 3H]  columns: Q | K | V, head t at columns t*d .. t*d+d-1 of each */
    int32_t* scores;  /* [B, heads, S, S] */
    int8_t* p;        /* [B, heads, S, S] */
    int8_t* ctx;      /* [M, H] */
    float* attn;      /* [M, H]  out-projection + bias + residual */
    int8_t* ln1;      /* [M, H] */
    int8_t* ffn1;     /* [M, F] */
    float* ffn2;      /* [M, H]  FFN2 + bias + residual */
} nmo_taps;

#define TAKE(ptr, type, count) \
    type* ptr = (type*)malloc(sizeof(type) * (size_t)(count)); \
    if (!ptr) rc = NMO_ERR_ALLOC

/*
 * x: int8 [M, H] with M = B*S.  y_q: int8 [M, H] (NULL allowed), y_f32: fp32 [M, H] (NULL
 * allowed).  Steps (all linear operations are integer matrix products, Section 3.1; all
 * nonlinear operators are PWL tables, Section 3.2):
 *   1 QKV projection, requantised per third with its own scale
 *   2 scores = Q K^T per (batch, head), int32
 *   3 softmax-PWL over each score row
 *   4 context = P V per (batch, head), requantised
 *   5 output projection + bias + residual(x)            -> fp32
 *   6 LayerNorm-PWL                                      -> int8
 *   7 FFN1 + bias, GELU-PWL, requantised
 *   8 FFN2 + bias + residual(LN1 output)                -> fp32
 *   9 LayerNorm-PWL                                      -> int8 (+ fp32)
 */
int nmo_encoder_layer(const nmo_layer* L, const int8_t* x, int8_t* y_q, float* y_f32,
                      const nmo_taps* taps)
{
    if (!L || !x || L->B < 1 || L->S < 1 || L->H < 1 || L->heads < 1 || L->F < 1 ||
        L->H % L->heads != 0)
        return NMO_ERR_ARG;
    const int32_t B = L->B, S = L->S, H = L->H, nh = L->heads, F = L->F, d = H / nh;
    const int32_t M = B * S;
    int rc = NMO_OK;
    TAKE(qkv, int8_t, (size_t)M * 3 * H);
    TAKE(scores, int32_t, (size_t)B * nh * S * S);
    TAKE(p, int8_t, (size_t)B * nh * S * S);
    TAKE(ctx, int8_t, (size_t)M * H);
    TAKE(attn, float, (size_t)M * H);
    TAKE(ln1, int8_t, (size_t)M * H);
    TAKE(ffn1, int8_t, (size_t)M * F);
    TAKE(ffn2, float, (size_t)M * H);
    TAKE(oscale, float, (size_t)3 * H);
    if (rc != NMO_OK) goto done;

    /* 1 */
    for (int32_t n = 0; n < 3 * H; ++n)
        oscale[n] = n < H ? L->inv_s_q : (n < 2 * H ? L->inv_s_k : L->inv_s_v);
    {
        nmo_gemm g;
        memset(&g, 0, sizeof g);
        g.M = M; g.N = 3 * H; g.K = H; g.A = x; g.W = L->Wqkv; g.bias = L->bqkv;
        g.alpha = L->alpha_qkv; g.out_inv_scale_vec = oscale; g.out_q = qkv;
        rc = nmo_gemm_pwl(&g);
        if (rc != NMO_OK) goto done;
    }
    /* 2: scores[b,t,i,j] = sum_c Q[b,i,t,c] * K[b,j,t,c] */
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t b = 0; b < B; ++b)
        for (int32_t t = 0; t < nh; ++t)
            for (int32_t i = 0; i < S; ++i)
                for (int32_t j = 0; j < S; ++j) {
                    const int8_t* q = qkv + ((size_t)(b * S + i) * 3 * H) + t * d;
                    const int8_t* kk = qkv + ((size_t)(b * S + j) * 3 * H) + H + t * d;
                    int32_t acc = 0;
                    for (int32_t c = 0; c < d; ++c) acc += (int32_t)q[c] * (int32_t)kk[c];
                    scores[(((size_t)b * nh + t) * S + i) * S + j] = acc;
                }
    /* 3 */
    rc = nmo_softmax_pwl(scores, NMO_DT_I32, L->alpha_scores, (int64_t)B * nh * S, S, L->t_exp,
                         L->t_recip, L->inv_s_p, p, NULL, NULL, NULL);
    if (rc != NMO_OK) goto done;
    /* 4: ctx[b,i,t,c] = requant( (sum_j P[b,t,i,j] * V[b,j,t,c]) * alpha_ctx ) */
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t b = 0; b < B; ++b)
        for (int32_t t = 0; t < nh; ++t)
            for (int32_t i = 0; i < S; ++i)
                for (int32_t c = 0; c < d; ++c) {
                    const int8_t* pr = p + (((size_t)b * nh + t) * S + i) * S;
                    int32_t acc = 0;
                    for (int32_t j = 0; j < S; ++j)
                        acc += (int32_t)pr[j] *
                               (int32_t)qkv[((size_t)(b * S + j) * 3 * H) + 2 * H + t * d + c];
                    float v = fmaf((float)acc, L->alpha_ctx, 0.0f);
                    ctx[(size_t)(b * S + i) * H + t * d + c] = requant(v, L->inv_s_ctx);
                }
    /* 5 */
    {
        nmo_gemm g;
        memset(&g, 0, sizeof g);
        g.M = M; g.N = H; g.K = H; g.A = ctx; g.W = L->Wo; g.bias = L->bo; g.alpha = L->alpha_o;
        g.resid = x; g.resid_scale = L->resid1_scale; g.out_f32 = attn;
        rc = nmo_gemm_pwl(&g);
        if (rc != NMO_OK) goto done;
    }
    /* 6 */
    rc = nmo_layernorm_pwl(attn, L->gamma1, L->beta1, L->eps1, M, H, L->t_rsqrt, L->inv_s_ln1, ln1,
                           NULL, NULL);
    if (rc != NMO_OK) goto done;
    /* 7 */
    {
        nmo_gemm g;
        memset(&g, 0, sizeof g);
        g.M = M; g.N = F; g.K = H; g.A = ln1; g.W = L->W1; g.bias = L->b1; g.alpha = L->alpha_1;
        g.table = L->t_gelu; g.out_inv_scale = L->inv_s_ffn1; g.out_q = ffn1;
        rc = nmo_gemm_pwl(&g);
        if (rc != NMO_OK) goto done;
    }
    /* 8 */
    {
        nmo_gemm g;
        memset(&g, 0, sizeof g);
        g.M = M; g.N = H; g.K = F; g.A = ffn1; g.W = L->W2; g.bias = L->b2; g.alpha = L->alpha_2;
        g.resid = ln1; g.resid_scale = L->resid2_scale; g.out_f32 = ffn2;
        rc = nmo_gemm_pwl(&g);
        if (rc != NMO_OK) goto done;
    }
    /* 9 */
    rc = nmo_layernorm_pwl(ffn2, L->gamma2, L->beta2, L->eps2, M, H, L->t_rsqrt, L->inv_s_out, y_q,
                           y_f32, NULL);
    if (rc != NMO_OK) goto done;

    if (taps) {
        if (taps->qkv) memcpy(taps->qkv, qkv, (size_t)M * 3 * H);
        if (taps->scores) memcpy(taps->scores, scores, sizeof(int32_t) * (size_t)B * nh * S * S);
        if (taps->p) memcpy(taps->p, p, (size_t)B * nh * S * S);
        if (taps->ctx) memcpy(taps->ctx, ctx, (size_t)M * H);
        if (taps->attn) memcpy(taps->attn, attn, sizeof(float) * (size_t)M * H);
        if (taps->ln1) memcpy(taps->ln1, ln1, (size_t)M * H);
        if (taps->ffn1) memcpy(taps->ffn1, ffn1, (size_t)M * F);
        if (taps->ffn2) memcpy(taps->ffn2, ffn2, sizeof(float) * (size_t)M * H);
    }
done:
    free(qkv); free(scores); free(p); free(ctx); free(attn); free(ln1); free(ffn1); free(ffn2);
    free(oscale);
    return rc;
}

/* ------------------------------------------------------------------------------------------- */
/* Exact-function, binary64 version of the same layer.                                          */
/* ------------------------------------------------------------------------------------------- */

static double q8(double v, double inv_scale)
{
    double r = rint(v * inv_scale);
    if (r < -127.0) r = -127.0;
    if (r > 127.0) r = 127.0;
    return r;
}

/*
 * The same network with the true GELU / exp / division / square root in binary64 and plain
 * left-to-right sums.  Weights and the input are the same int8 tensors.
 * quantise = 0: activations are never rounded; absmax[0..8] receives the largest magnitude of
 *   x, Q, K, V, P, ctx, LN1 output, FFN1 output (after GELU), layer output, in real units.  This
 *   is the calibration run (Section 3.2 step 1) that yields static activation scales, and
 *   absmax[9..12] the observed ranges of the inputs to GELU (min, max), and the largest softmax
 *   denominator and LayerNorm variance + eps, from which table ranges can be chosen.
 * quantise = 1: every activation is rounded to its int8 grid exactly where the PWL layer does,
 *   using the layer's inverse scales; y is then the reference the PWL layer's output is compared
 *   with to report the approximation error.
 * y: [M, H] binary64, real units.
 */
int nmo_encoder_layer_exact(const nmo_layer* L, const int8_t* x, int32_t quantise, double* y,
                            double* absmax)
{
    if (!L || !x || !y || L->H % L->heads != 0) return NMO_ERR_ARG;
    const int32_t B = L->B, S = L->S, H = L->H, nh = L->heads, F = L->F, d = H / nh;
    const int32_t M = B * S;
    int rc = NMO_OK;
    /* am[9] holds max(-v) while running so that one max-reduction serves every entry */
    double am[13];
    for (int i = 0; i < 13; ++i) am[i] = 0.0;
    am[9] = -INFINITY; am[10] = -INFINITY;
    TAKE(qkv, double, (size_t)M * 3 * H);
    TAKE(ctx, double, (size_t)M * H);
    TAKE(ln1, double, (size_t)M * H);
    TAKE(ffn1, double, (size_t)M * F);
    TAKE(pre, double, (size_t)M * H);
    if (rc != NMO_OK) goto done;
    const double s_x = (double)L->resid1_scale;
    for (size_t i = 0; i < (size_t)M * H; ++i) am[0] = fmax(am[0], fabs((double)x[i] * s_x));

    /* QKV: real value = acc * alpha_qkv + bias; kept in code units (value * inverse scale) */
#pragma omp parallel for schedule(static) reduction(max : am[:13])
    for (int32_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < 3 * H; ++n) {
            int64_t acc = 0;
            for (int32_t k = 0; k < H; ++k)
                acc += (int64_t)x[(size_t)m * H + k] * (int64_t)L->Wqkv[(size_t)n * H + k];
            double v = (double)acc * (double)L->alpha_qkv + (L->bqkv ? (double)L->bqkv[n] : 0.0);
            int which = n / H;
            am[1 + which] = fmax(am[1 + which], fabs(v));
            double inv = which == 0 ? L->inv_s_q : (which == 1 ? L->inv_s_k : L->inv_s_v);
            qkv[(size_t)m * 3 * H + n] = quantise ? q8(v, inv) : v * inv;
        }
    /* attention, in code units so that alpha_scores / alpha_ctx apply unchanged */
#pragma omp parallel for collapse(2) schedule(static) reduction(max : am[:13])
    for (int32_t b = 0; b < B; ++b)
        for (int32_t t = 0; t < nh; ++t) {
            double* e = (double*)malloc(sizeof(double) * (size_t)S);
            if (!e) { rc = NMO_ERR_ALLOC; continue; }
            for (int32_t i = 0; i < S; ++i) {
                double mx = -INFINITY;
                for (int32_t j = 0; j < S; ++j) {
                    double acc = 0.0;
                    for (int32_t c = 0; c < d; ++c)
                        acc += qkv[(size_t)(b * S + i) * 3 * H + t * d + c] *
                               qkv[(size_t)(b * S + j) * 3 * H + H + t * d + c];
                    e[j] = acc * (double)L->alpha_scores;
                    if (e[j] > mx) mx = e[j];
                }
                double sum = 0.0;
                for (int32_t j = 0; j < S; ++j) { e[j] = exp(e[j] - mx); sum += e[j]; }
                am[11] = fmax(am[11], sum);
                for (int32_t j = 0; j < S; ++j) {
                    double pj = e[j] / sum;
                    am[4] = fmax(am[4], fabs(pj));
                    e[j] = quantise ? q8(pj, L->inv_s_p) : pj * (double)L->inv_s_p;
                }
                for (int32_t c = 0; c < d; ++c) {
                    double acc = 0.0;
                    for (int32_t j = 0; j < S; ++j)
                        acc += e[j] * qkv[(size_t)(b * S + j) * 3 * H + 2 * H + t * d + c];
                    double v = acc * (double)L->alpha_ctx;
                    am[5] = fmax(am[5], fabs(v));
                    ctx[(size_t)(b * S + i) * H + t * d + c] =
                        quantise ? q8(v, L->inv_s_ctx) : v * (double)L->inv_s_ctx;
                }
            }
            free(e);
        }
    if (rc != NMO_OK) goto done;
    /* out-projection + bias + residual(x), LayerNorm 1 */
#pragma omp parallel for schedule(static) reduction(max : am[:13])
    for (int32_t m = 0; m < M; ++m) {
        double* row = pre + (size_t)m * H;
        for (int32_t n = 0; n < H; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < H; ++k)
                acc += ctx[(size_t)m * H + k] * (double)L->Wo[(size_t)n * H + k];
            row[n] = acc * (double)L->alpha_o + (L->bo ? (double)L->bo[n] : 0.0) +
                     (double)x[(size_t)m * H + n] * s_x;
        }
        double mu = 0.0, var = 0.0;
        for (int32_t n = 0; n < H; ++n) mu += row[n];
        mu /= H;
        for (int32_t n = 0; n < H; ++n) { double dd = row[n] - mu; var += dd * dd; }
        var /= H;
        am[12] = fmax(am[12], var + (double)L->eps1);
        double rs = 1.0 / sqrt(var + (double)L->eps1);
        for (int32_t n = 0; n < H; ++n) {
            double v = (row[n] - mu) * rs * (double)L->gamma1[n] + (double)L->beta1[n];
            am[6] = fmax(am[6], fabs(v));
            ln1[(size_t)m * H + n] = quantise ? q8(v, L->inv_s_ln1) : v * (double)L->inv_s_ln1;
        }
    }
    /* FFN1 + bias, GELU */
#pragma omp parallel for schedule(static) reduction(max : am[:13])
    for (int32_t m = 0; m < M; ++m)
        for (int32_t n = 0; n < F; ++n) {
            double acc = 0.0;
            for (int32_t k = 0; k < H; ++k)
                acc += ln1[(size_t)m * H + k] * (double)L->W1[(size_t)n * H + k];
            double v = acc * (double)L->alpha_1 + (L->b1 ? (double)L->b1[n] : 0.0);
            am[9] = fmax(am[9], -v);
            am[10] = fmax(am[10], v);
            double g = f_gelu(v);
            am[7] = fmax(am[7], fabs(g));
            ffn1[(size_t)m * F + n] = quantise ? q8(g, L->inv_s_ffn1) : g * (double)L->inv_s_ffn1;
        }
    /* FFN2 + bias + residual(LN1 output), LayerNorm 2 */
    {
        const double s_ln1 = (double)L->resid2_scale;
#pragma omp parallel for schedule(static) reduction(max : am[:13])
        for (int32_t m = 0; m < M; ++m) {
            double* row = pre + (size_t)m * H;
            for (int32_t n = 0; n < H; ++n) {
                double acc = 0.0;
                for (int32_t k = 0; k < F; ++k)
                    acc += ffn1[(size_t)m * F + k] * (double)L->W2[(size_t)n * F + k];
                row[n] = acc * (double)L->alpha_2 + (L->b2 ? (double)L->b2[n] : 0.0) +
                         ln1[(size_t)m * H + n] * s_ln1;
            }
            double mu = 0.0, var = 0.0;
            for (int32_t n = 0; n < H; ++n) mu += row[n];
            mu /= H;
            for (int32_t n = 0; n < H; ++n) { double dd = row[n] - mu; var += dd * dd; }
            var /= H;
            am[12] = fmax(am[12], var + (double)L->eps2);
            double rs = 1.0 / sqrt(var + (double)L->eps2);
            for (int32_t n = 0; n < H; ++n) {
                double v = (row[n] - mu) * rs * (double)L->gamma2[n] + (double)L->beta2[n];
                am[8] = fmax(am[8], fabs(v));
                y[(size_t)m * H + n] = quantise ? q8(v, L->inv_s_out) / (double)L->inv_s_out : v;
            }
        }
    }
    am[9] = -am[9];
    if (absmax) memcpy(absmax, am, sizeof am);
done:
    free(qkv); free(ctx); free(ln1); free(ffn1); free(pre);
    return rc;
}
