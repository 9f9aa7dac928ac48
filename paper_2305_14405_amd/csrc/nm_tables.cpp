// Host side of the library: error reporting and PWL table construction / upload.
//
// Table construction follows the paper's Section 3.2: the input range is cut into segments of
// fixed length, each fitted by the line through the function values at its two ends (Algorithm 3,
// first step), which makes neighbouring lines meet; optionally the intercept is shifted by the
// expectation bias (rest of Algorithm 3) and neighbouring primary segments of similar slope are
// merged first (Algorithm 2).  Everything is computed in binary64 and rounded once to binary32.
#include <cmath>
#include <cstring>
#include <limits>
#include <new>

#include "nm_internal.h"

namespace nm {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
}

int32_t fail(int32_t code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int32_t check_hip(hipError_t e, const char* what)
{
    if (e == hipSuccess) return NM_OK;
    return fail(NM_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

// The smallest fp32 x whose segment index in a two-segment table is 1, i.e. for which the kernels'
// index arithmetic, u = (x - lo) * inv_w in fp32 (one subtract, one multiply), gives u >= 1.  Both
// operations round monotonically and inv_w > 0, so the set is an upper interval of the floats and
// bisection over their order finds its first element (+inf if there is none).  x >= tau then decides
// exactly what the index computation decides, for every x (a NaN compares false: segment 0, as there).
static float two_segment_threshold(float lo, float inv_w)
{
    auto in_upper = [&](float x) {
        volatile float u = x - lo;
        u = u * inv_w;
        return u >= 1.0f;
    };
    // floats in increasing order <-> unsigned keys in increasing order
    auto to_float = [](uint32_t key) {
        const uint32_t bits = (key & 0x80000000u) ? key ^ 0x80000000u : ~key;
        float f;
        std::memcpy(&f, &bits, sizeof f);
        return f;
    };
    auto to_key = [](float f) {
        uint32_t bits;
        std::memcpy(&bits, &f, sizeof bits);
        return (bits & 0x80000000u) ? ~bits : bits ^ 0x80000000u;
    };
    const float big = std::numeric_limits<float>::max();
    if (!in_upper(big)) return std::numeric_limits<float>::infinity();
    if (in_upper(-big)) return -big;
    uint32_t a = to_key(-big), b = to_key(big);   // in_upper(a) false, in_upper(b) true
    while (b - a > 1) {
        const uint32_t mid = a + (b - a) / 2;
        if (in_upper(to_float(mid))) b = mid; else a = mid;
    }
    return to_float(b);
}

int32_t get_dev_table(const nm_tables* t, int32_t idx, DevTable* dt, const char* what, bool two_level)
{
    if (!t) return fail(NM_ERR_INVALID_ARG, "%s: tables is NULL", what);
    if (idx < 0 || idx >= (int32_t)t->tables.size())
        return fail(NM_ERR_INVALID_ARG, "%s: table index %d out of range [0, %zu)", what, idx,
                    t->tables.size());
    const HostTable& h = t->tables[idx];
    dt->kb = t->d_blob + h.blob_offset;
    dt->lo = h.desc.lo;
    dt->hi = h.desc.hi;
    dt->inv_w = h.inv_w;
    dt->nseg = h.desc.nseg;
    dt->clamp_input = (h.desc.flags & NM_TABLE_CLAMP_INPUT) ? 1 : 0;
    dt->ckb = nullptr; dt->cellmap = nullptr; dt->nkb = 0;
    dt->two_seg = 0; dt->k0 = dt->b0 = dt->k1 = dt->b1 = dt->tau = 0.0f;
    if (h.desc.nseg == 2 && !dt->clamp_input) {
        dt->two_seg = 1;
        dt->k0 = h.k[0]; dt->b0 = h.b[0]; dt->k1 = h.k[1]; dt->b1 = h.b[1];
        dt->tau = two_segment_threshold(h.desc.lo, h.inv_w);
    }
    if (two_level && !h.cellmap.empty()) {
        dt->ckb = t->d_blob + h.cblob_offset;
        dt->cellmap = reinterpret_cast<const uint8_t*>(t->d_blob + h.map_offset);
        dt->nkb = (int)h.ck.size();
    }
    return NM_OK;
}

// ---- the functions and their primitives ------------------------------------------------------

static const double kSqrt2 = 1.4142135623730951;
static const double kInvSqrt2Pi = 0.3989422804014327;

static double normal_cdf(double x) { return 0.5 * std::erfc(-x / kSqrt2); }
static double normal_pdf(double x) { return kInvSqrt2Pi * std::exp(-0.5 * x * x); }

static bool eval_f(int func, double x, double* y)
{
    switch (func) {
    case NM_FUNC_GELU: *y = x * normal_cdf(x); return true;
    case NM_FUNC_EXP: *y = std::exp(x); return true;
    case NM_FUNC_RECIP: *y = 1.0 / x; return true;
    case NM_FUNC_RSQRT: *y = 1.0 / std::sqrt(x); return true;
    case NM_FUNC_RELU: *y = x > 0.0 ? x : 0.0; return true;
    case NM_FUNC_SQRT: *y = std::sqrt(x); return true;
    case NM_FUNC_IDENTITY: *y = x; return true;
    default: return false;
    }
}

// Integral of f from a to c (closed forms).
static double integral_f(int func, double a, double c)
{
    auto P = [func](double x) -> double {
        switch (func) {
        case NM_FUNC_GELU: return 0.5 * ((x * x - 1.0) * normal_cdf(x) + x * normal_pdf(x));
        case NM_FUNC_EXP: return std::exp(x);
        case NM_FUNC_RECIP: return std::log(x);
        case NM_FUNC_RSQRT: return 2.0 * std::sqrt(x);
        case NM_FUNC_RELU: return x > 0.0 ? 0.5 * x * x : 0.0;
        case NM_FUNC_SQRT: return x * std::sqrt(x) * (2.0 / 3.0);
        default: return 0.5 * x * x;  // identity
        }
    };
    return P(c) - P(a);
}

struct Line { double k, b; };

// Algorithm 3 for one segment [a, c].
static Line fit_segment(int func, double a, double c, bool correct, double e_th)
{
    double fa = 0, fc = 0;
    eval_f(func, a, &fa);
    eval_f(func, c, &fc);
    Line ln;
    ln.k = (fc - fa) / (c - a);
    ln.b = fa - ln.k * a;
    if (correct) {
        // mean of f over the segment minus the mean of the chord
        double shift = integral_f(func, a, c) / (c - a) - 0.5 * (fa + fc);
        if (std::fabs(shift) > e_th) ln.b += shift;
    }
    return ln;
}

static int32_t validate_desc(const nm_table_desc* d, bool need_func)
{
    if (!d) return fail(NM_ERR_INVALID_ARG, "table descriptor is NULL");
    if (!(d->hi > d->lo) || !std::isfinite(d->lo) || !std::isfinite(d->hi))
        return fail(NM_ERR_INVALID_ARG, "table range needs finite lo < hi");
    if (d->nseg < 1) return fail(NM_ERR_INVALID_ARG, "table needs nseg >= 1 (got %d)", d->nseg);
    if (d->nseg > NM_MAX_SEGMENTS)
        return fail(NM_ERR_UNSUPPORTED, "nseg %d exceeds NM_MAX_SEGMENTS %d", d->nseg,
                    NM_MAX_SEGMENTS);
    if (need_func) {
        // thresholds of Algorithm 3 / Algorithm 2: finite and not negative
        if ((d->flags & NM_TABLE_BIAS_CORRECT) && !(d->e_th >= 0.0f && std::isfinite(d->e_th)))
            return fail(NM_ERR_INVALID_ARG, "e_th must be finite and >= 0");
        if ((d->flags & NM_TABLE_MERGE) && !(d->dk_th >= 0.0f && std::isfinite(d->dk_th)))
            return fail(NM_ERR_INVALID_ARG, "dk_th must be finite and >= 0");
        double y;
        if (!eval_f(d->func, 1.0, &y))
            return fail(NM_ERR_INVALID_ARG, "unknown function id %d", d->func);
        if ((d->func == NM_FUNC_RECIP || d->func == NM_FUNC_RSQRT) && !(d->lo > 0.0f))
            return fail(NM_ERR_INVALID_ARG, "1/x and 1/sqrt(x) tables need lo > 0");
        if (d->func == NM_FUNC_SQRT && d->lo < 0.0f)
            return fail(NM_ERR_INVALID_ARG, "sqrt table needs lo >= 0");
    }
    return NM_OK;
}

static int32_t build_host(const nm_table_desc* d, float* k, float* b, float* inv_w, int32_t* n_distinct)
{
    const int n = d->nseg;
    const double lo = (double)d->lo, hi = (double)d->hi;
    const double w = (hi - lo) / (double)n;
    const bool correct = (d->flags & NM_TABLE_BIAS_CORRECT) != 0;
    int distinct = 0;
    if (!(d->flags & NM_TABLE_MERGE)) {
        for (int i = 0; i < n; ++i) {
            Line ln = fit_segment(d->func, lo + (double)i * w, lo + (double)(i + 1) * w, correct,
                                  (double)d->e_th);
            k[i] = (float)ln.k;
            b[i] = (float)ln.b;
        }
        distinct = n;
    } else {
        // Algorithm 2 over the n primary cells: a cell whose slope differs from the slope at the
        // last kept start point by more than dk_th opens a new merged segment.
        auto cell_slope = [&](int i) {
            double f0 = 0, f1 = 0;
            eval_f(d->func, lo + (double)i * w, &f0);
            eval_f(d->func, lo + (double)(i + 1) * w, &f1);
            return (f1 - f0) / w;
        };
        int start = 0;
        double kept = cell_slope(0);
        auto close_segment = [&](int first, int last_excl) {
            double a = lo + (double)first * w;
            double c = last_excl == n ? hi : lo + (double)last_excl * w;
            Line ln = fit_segment(d->func, a, c, correct, (double)d->e_th);
            for (int i = first; i < last_excl; ++i) {
                k[i] = (float)ln.k;
                b[i] = (float)ln.b;
            }
            ++distinct;
        };
        for (int i = 1; i < n; ++i) {
            double ki = cell_slope(i);
            if (std::fabs(ki - kept) <= (double)d->dk_th) continue;
            close_segment(start, i);
            start = i;
            kept = ki;
        }
        close_segment(start, n);
    }
    *inv_w = (float)((double)n / (hi - lo));
    if (n_distinct) *n_distinct = distinct;
    return NM_OK;
}

// The two-level form of a table whose neighbouring cells share parameters (Algorithm 2 merges
// them): runs of bit-identical {k, b} become one segment each.  At most 256 segments (the map holds
// one byte per cell).
static int32_t make_compact(HostTable& h)
{
    h.ck.clear(); h.cb.clear(); h.cellmap.assign(h.k.size(), 0);
    for (size_t i = 0; i < h.k.size(); ++i) {
        const bool same = i > 0 && std::memcmp(&h.k[i], &h.k[i - 1], sizeof(float)) == 0 &&
                          std::memcmp(&h.b[i], &h.b[i - 1], sizeof(float)) == 0;
        if (!same) {
            if (h.ck.size() == 256)
                return fail(NM_ERR_UNSUPPORTED, "NM_TABLE_COMPACT: more than 256 merged segments");
            h.ck.push_back(h.k[i]);
            h.cb.push_back(h.b[i]);
        }
        h.cellmap[i] = (uint8_t)(h.ck.size() - 1);
    }
    return NM_OK;
}

static int32_t upload(nm_tables* t, hipStream_t stream)
{
    size_t total = 0;
    for (auto& h : t->tables) {
        h.blob_offset = total;
        total += ((size_t)h.desc.nseg + 15) / 16 * 16;  // 128-byte aligned tables
        if (!h.cellmap.empty()) {
            h.cblob_offset = total;
            total += (h.ck.size() + 15) / 16 * 16;
            h.map_offset = total;
            total += (h.cellmap.size() + 127) / 128 * 16;  // bytes, rounded up to 128, in float2 units
        }
    }
    std::vector<float2> blob(total, make_float2(0.f, 0.f));
    for (auto& h : t->tables) {
        for (int i = 0; i < h.desc.nseg; ++i) blob[h.blob_offset + i] = make_float2(h.k[i], h.b[i]);
        for (size_t i = 0; i < h.ck.size(); ++i) blob[h.cblob_offset + i] = make_float2(h.ck[i], h.cb[i]);
        if (!h.cellmap.empty())
            std::memcpy(reinterpret_cast<uint8_t*>(blob.data() + h.map_offset), h.cellmap.data(), h.cellmap.size());
    }
    int32_t rc = check_hip(hipGetDevice(&t->device), "hipGetDevice");
    if (rc) return rc;
    rc = check_hip(hipMalloc((void**)&t->d_blob, total * sizeof(float2)), "hipMalloc(tables)");
    if (rc) { t->d_blob = nullptr; return rc == NM_ERR_HIP ? NM_ERR_ALLOC : rc; }
    rc = check_hip(hipMemcpyAsync(t->d_blob, blob.data(), total * sizeof(float2),
                                  hipMemcpyHostToDevice, stream), "hipMemcpyAsync(tables)");
    if (rc) return rc;
    // the staging vector dies at return: wait for the copy
    return check_hip(hipStreamSynchronize(stream), "hipStreamSynchronize(tables)");
}

}  // namespace nm

using namespace nm;

extern "C" {

const char* nm_last_error(void) { return g_err; }

int32_t nm_version(void) { return 1000; }

int32_t nm_table_build_host(const nm_table_desc* desc, float* k, float* b, float* inv_w,
                            int32_t* n_distinct)
{
    int32_t rc = validate_desc(desc, true);
    if (rc) return rc;
    if (!k || !b || !inv_w) return fail(NM_ERR_INVALID_ARG, "nm_table_build_host: NULL output");
    return build_host(desc, k, b, inv_w, n_distinct);
}

static int32_t make_tables(const nm_table_desc* descs, int32_t n, const float* const* k,
                           const float* const* b, void* stream, nm_tables** out, const char* what)
{
    if (!descs || !out) return fail(NM_ERR_INVALID_ARG, "%s: NULL argument", what);
    *out = nullptr;
    if (n < 1 || n > NM_MAX_TABLES)
        return fail(NM_ERR_INVALID_ARG, "%s: table count %d outside [1, %d]", what, n, NM_MAX_TABLES);
    const bool from_arrays = k != nullptr || b != nullptr;
    if (from_arrays && (!k || !b)) return fail(NM_ERR_INVALID_ARG, "%s: k or b is NULL", what);
    for (int i = 0; i < n; ++i) {
        int32_t rc = validate_desc(&descs[i], !from_arrays);
        if (rc) return rc;
        if (from_arrays && (!k[i] || !b[i]))
            return fail(NM_ERR_INVALID_ARG, "%s: k[%d] or b[%d] is NULL", what, i, i);
    }
    nm_tables* t = new (std::nothrow) nm_tables;
    if (!t) return fail(NM_ERR_ALLOC, "%s: out of host memory", what);
    t->tables.resize(n);
    for (int i = 0; i < n; ++i) {
        HostTable& h = t->tables[i];
        h.desc = descs[i];
        h.k.resize(descs[i].nseg);
        h.b.resize(descs[i].nseg);
        if (from_arrays) {
            std::memcpy(h.k.data(), k[i], sizeof(float) * descs[i].nseg);
            std::memcpy(h.b.data(), b[i], sizeof(float) * descs[i].nseg);
            h.inv_w = (float)((double)descs[i].nseg / ((double)descs[i].hi - (double)descs[i].lo));
            h.n_distinct = descs[i].nseg;
        } else {
            build_host(&descs[i], h.k.data(), h.b.data(), &h.inv_w, &h.n_distinct);
        }
        if (descs[i].flags & NM_TABLE_COMPACT) {
            int32_t rc = make_compact(h);
            if (rc) { delete t; return rc; }
        }
    }
    int32_t rc = upload(t, (hipStream_t)stream);
    if (rc) {
        nm_tables_destroy(t);
        return rc;
    }
    *out = t;
    return NM_OK;
}

int32_t nm_build_tables(const nm_table_desc* descs, int32_t n, void* stream, nm_tables** out)
{
    return make_tables(descs, n, nullptr, nullptr, stream, out, "nm_build_tables");
}

int32_t nm_tables_from_arrays(const nm_table_desc* descs, int32_t n, const float* const* k,
                              const float* const* b, void* stream, nm_tables** out)
{
    if (!k || !b) return fail(NM_ERR_INVALID_ARG, "nm_tables_from_arrays: k or b is NULL");
    return make_tables(descs, n, k, b, stream, out, "nm_tables_from_arrays");
}

int32_t nm_tables_count(const nm_tables* t) { return t ? (int32_t)t->tables.size() : 0; }

int32_t nm_tables_get(const nm_tables* t, int32_t idx, nm_table_desc* desc, float* k_host,
                      float* b_host, float* inv_w)
{
    if (!t) return fail(NM_ERR_INVALID_ARG, "nm_tables_get: tables is NULL");
    if (idx < 0 || idx >= (int32_t)t->tables.size())
        return fail(NM_ERR_INVALID_ARG, "nm_tables_get: index %d out of range", idx);
    const HostTable& h = t->tables[idx];
    if (desc) *desc = h.desc;
    if (k_host) std::memcpy(k_host, h.k.data(), sizeof(float) * h.k.size());
    if (b_host) std::memcpy(b_host, h.b.data(), sizeof(float) * h.b.size());
    if (inv_w) *inv_w = h.inv_w;
    return NM_OK;
}

int32_t nm_tables_get_compact(const nm_tables* t, int32_t idx, int32_t* n_segments, uint8_t* cell_to_segment,
                              float* k_host, float* b_host)
{
    if (!t) return fail(NM_ERR_INVALID_ARG, "nm_tables_get_compact: tables is NULL");
    if (idx < 0 || idx >= (int32_t)t->tables.size())
        return fail(NM_ERR_INVALID_ARG, "nm_tables_get_compact: index %d out of range", idx);
    const HostTable& h = t->tables[idx];
    if (h.cellmap.empty()) return fail(NM_ERR_INVALID_ARG, "nm_tables_get_compact: table %d was not built with NM_TABLE_COMPACT", idx);
    if (n_segments) *n_segments = (int32_t)h.ck.size();
    if (cell_to_segment) std::memcpy(cell_to_segment, h.cellmap.data(), h.cellmap.size());
    if (k_host) std::memcpy(k_host, h.ck.data(), sizeof(float) * h.ck.size());
    if (b_host) std::memcpy(b_host, h.cb.data(), sizeof(float) * h.cb.size());
    return NM_OK;
}

void nm_tables_destroy(nm_tables* t)
{
    if (!t) return;
    if (t->d_blob) (void)hipFree(t->d_blob);
    delete t;
}

}  // extern "C"
