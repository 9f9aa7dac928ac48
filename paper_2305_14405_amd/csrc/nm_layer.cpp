// nm_encoder_layer: one post-LayerNorm transformer encoder layer as a fixed sequence of kernel
// launches on one stream (paper Section 3: linear operators as matrix products, nonlinear
// operators as PWL tables).  Host code only: it validates, carves the workspace and queues the
// nine steps; nothing is allocated and the host never waits for the GPU.
#include <cmath>
#include <cstdlib>
#include <mutex>

#include "nm_internal.h"

namespace nm {

// Debug switch: NM_ATTN_UNFUSED=1 keeps attention on the three separate kernels.
static bool unfused_attention()
{
    static const bool v = [] { const char* e = getenv("NM_ATTN_UNFUSED"); return e && e[0] == '1'; }();
    return v;
}

static size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct LayerPlan {
    size_t off_qkv, off_scores, off_p, off_ctx, off_attn, off_ln1, off_ffn1, off_ffn2, total;
};

static bool fused_attention_shape(const nm_layer_desc* d)
{
    return d->H / d->heads == 64 && d->S <= 512 && d->H % 16 == 0 && !unfused_attention();
}

static LayerPlan plan_layer(const nm_layer_desc* d)
{
    const size_t M = (size_t)d->B * d->S, H = d->H, F = d->F;
    const size_t SS = (size_t)d->B * d->heads * d->S * d->S;
    LayerPlan p{};
    size_t o = 0;
    auto take = [&o](size_t bytes) { size_t at = o; o = round_up(o + bytes, 256); return at; };
    p.off_qkv = take(M * 3 * H);
    // the score and probability tensors exist only on the three-kernel attention path (the fused
    // kernel keeps them in registers; every workspace tensor is 256-byte aligned, so whether it
    // runs depends on the shape alone)
    const bool fused = fused_attention_shape(d);
    p.off_scores = take(fused ? 0 : SS * sizeof(int32_t));
    p.off_p = take(fused ? 0 : SS);
    p.off_ctx = take(M * H);
    p.off_attn = take(M * H * sizeof(float));
    p.off_ln1 = take(M * H);
    p.off_ffn1 = take(M * F);
    p.off_ffn2 = take(M * H * sizeof(float));
    p.total = o;
    return p;
}

static int32_t validate_layer(const nm_layer_desc* d, const char* what, bool numbers = false)
{
    if (!d) return fail(NM_ERR_INVALID_ARG, "%s: desc is NULL", what);
    if (d->B < 1 || d->S < 1 || d->H < 1 || d->heads < 1 || d->F < 1)
        return fail(NM_ERR_INVALID_ARG, "%s: dimensions must be >= 1", what);
    if (d->H % d->heads != 0)
        return fail(NM_ERR_INVALID_ARG, "%s: H %d not divisible by heads %d", what, d->H, d->heads);
    if (d->S > 4096 || d->H > 4096)
        return fail(NM_ERR_UNSUPPORTED, "%s: S and H must be <= 4096 (row kernels)", what);
    if (d->F > 65536) return fail(NM_ERR_UNSUPPORTED, "%s: F > 65536", what);
    if ((int64_t)d->B * d->heads > 65535) return fail(NM_ERR_UNSUPPORTED, "%s: B * heads > 65535", what);
    const int64_t M = (int64_t)d->B * d->S;
    if (M * 3 * d->H >= (1LL << 31) || M * d->F >= (1LL << 31))
        return fail(NM_ERR_UNSUPPORTED, "%s: B*S*max(3H, F) >= 2^31", what);
    if (!numbers) return NM_OK;  // a workspace query has dimensions only
    // every multiplier must be finite (a NaN or infinity would reach the table look-ups, whose
    // kernels assume finite inputs); the score scale is a positive number by its definition
    const float mult[] = {d->alpha_qkv, d->inv_s_q, d->inv_s_k, d->inv_s_v, d->alpha_scores, d->inv_s_p,
                          d->alpha_ctx, d->inv_s_ctx, d->alpha_o, d->resid1_scale, d->inv_s_ln1, d->alpha_1,
                          d->inv_s_ffn1, d->alpha_2, d->resid2_scale, d->inv_s_out, d->eps1, d->eps2};
    for (float v : mult)
        if (!std::isfinite(v)) return fail(NM_ERR_INVALID_ARG, "%s: a scale / multiplier is not finite", what);
    if (!(d->alpha_scores > 0.0f)) return fail(NM_ERR_INVALID_ARG, "%s: alpha_scores must be > 0", what);
    return NM_OK;
}

// ---- scratch of the entry point that allocates nothing --------------------------------------
// One array per GPU, in the library's own device image (zero-initialised storage, so it adds
// nothing to the file).  Host code never uses the array's name as an address: the device address is
// looked up once per device and cached.
constexpr size_t kStaticScratchBytes = (size_t)NM_NOALLOC_MAX_WORKSPACE;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's copy of `scratch`.
static int32_t static_scratch(void** out)
{
    int dev = -1;
    int32_t rc = check_hip(hipGetDevice(&dev), "hipGetDevice");
    if (rc) return rc;
    if (dev < 0 || dev >= kMaxDevices) return fail(NM_ERR_UNSUPPORTED, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        rc = check_hip(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)), "hipGetSymbolAddress(scratch)");
        if (rc) return rc;
        if (!ptr) return fail(NM_ERR_HIP, "hipGetSymbolAddress(scratch) returned NULL");
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return NM_OK;
}

}  // namespace nm

using namespace nm;

extern "C" {

int32_t nm_encoder_layer_workspace(const nm_layer_desc* desc, size_t* bytes)
{
    int32_t rc = validate_layer(desc, "nm_encoder_layer_workspace");
    if (rc) return rc;
    if (!bytes) return fail(NM_ERR_INVALID_ARG, "nm_encoder_layer_workspace: bytes is NULL");
    *bytes = plan_layer(desc).total;
    return NM_OK;
}

int32_t nm_encoder_layer(const nm_layer_desc* d, const int8_t* x, int8_t* y_q, float* y_f32,
                         void* ws, size_t ws_bytes, const nm_layer_taps* taps, void* stream_)
{
    int32_t rc = validate_layer(d, "nm_encoder_layer", true);
    if (rc) return rc;
    if (!x) return fail(NM_ERR_INVALID_ARG, "nm_encoder_layer: x is NULL");
    if (!y_q && !y_f32) return fail(NM_ERR_INVALID_ARG, "nm_encoder_layer: no output");
    if (!d->Wqkv || !d->Wo || !d->W1 || !d->W2 || !d->gamma1 || !d->beta1 || !d->gamma2 || !d->beta2)
        return fail(NM_ERR_INVALID_ARG, "nm_encoder_layer: NULL weight or LayerNorm vector");
    DevTable t_gelu, t_exp, t_recip, t_rsqrt;
    // the GELU table in its two-level form where it has one (FFN1's epilogue looks it up that way);
    // the row kernels and the attention kernel read the expanded form of theirs
    if ((rc = get_dev_table(d->tables, d->gelu_idx, &t_gelu, "nm_encoder_layer(gelu)", true))) return rc;
    if ((rc = get_dev_table(d->tables, d->exp_idx, &t_exp, "nm_encoder_layer(exp)"))) return rc;
    if ((rc = get_dev_table(d->tables, d->recip_idx, &t_recip, "nm_encoder_layer(recip)"))) return rc;
    if ((rc = get_dev_table(d->tables, d->rsqrt_idx, &t_rsqrt, "nm_encoder_layer(rsqrt)"))) return rc;
    const LayerPlan plan = plan_layer(d);
    if (!ws) return fail(NM_ERR_WORKSPACE, "nm_encoder_layer: workspace is NULL");
    if (!aligned(ws, 256)) return fail(NM_ERR_WORKSPACE, "nm_encoder_layer: workspace not 256-byte aligned");
    if (ws_bytes < plan.total)
        return fail(NM_ERR_WORKSPACE, "nm_encoder_layer: workspace %zu bytes < %zu needed", ws_bytes, plan.total);

    hipStream_t stream = (hipStream_t)stream_;
    char* w = static_cast<char*>(ws);
    const int B = d->B, S = d->S, H = d->H, nh = d->heads, F = d->F;
    const int M = B * S;
    auto pick = [&](void* tap, size_t off) -> void* { return tap ? tap : (void*)(w + off); };
    int8_t* qkv = (int8_t*)pick(taps ? taps->qkv : nullptr, plan.off_qkv);
    int32_t* scores = (int32_t*)pick(taps ? taps->scores : nullptr, plan.off_scores);
    int8_t* pm = (int8_t*)pick(taps ? taps->p : nullptr, plan.off_p);
    int8_t* ctx = (int8_t*)pick(taps ? taps->ctx : nullptr, plan.off_ctx);
    float* attn = (float*)pick(taps ? taps->attn : nullptr, plan.off_attn);
    int8_t* ln1 = (int8_t*)pick(taps ? taps->ln1 : nullptr, plan.off_ln1);
    int8_t* ffn1 = (int8_t*)pick(taps ? taps->ffn1 : nullptr, plan.off_ffn1);
    float* ffn2 = (float*)pick(taps ? taps->ffn2 : nullptr, plan.off_ffn2);

    // 1: QKV projection, three output scales by column third
    {
        GemmArgs g;
        g.M = M; g.N = 3 * H; g.K = H;
        g.A = x; g.lda = H; g.W = d->Wqkv; g.ldw = H;
        g.bias = d->bqkv; g.alpha = d->alpha_qkv;
        g.split_cols = H; g.inv3[0] = d->inv_s_q; g.inv3[1] = d->inv_s_k; g.inv3[2] = d->inv_s_v;
        g.ldo = 3L * H; g.out_q = qkv;
        if ((rc = launch_gemm(g, stream))) return rc;
    }
    // 2-4: attention.  One fused kernel when the shape allows it (the scores and probabilities then
    // stay in registers; the taps, if given, still receive them), else three kernels.
    // taps supplied by the caller replace workspace tensors and may be less aligned: the fused
    // kernel then still runs if they are aligned enough, else the three-kernel path needs the
    // caller's score / probability taps as storage (the workspace has none for a fused shape)
    bool fused = fused_attention_shape(d);
    if (fused && !(aligned(qkv, 16) && aligned(ctx, 4) && (!(taps && taps->scores) || aligned(taps->scores, 16)))) {
        if (!(taps && taps->scores && taps->p))
            return fail(NM_ERR_UNSUPPORTED, "nm_encoder_layer: qkv / ctx / scores taps must be 16-byte aligned");
        fused = false;
    }
    if (fused) {
        if ((rc = nm_attention_pwl(qkv, B, S, H, nh, d->alpha_scores, d->tables, d->exp_idx, d->recip_idx,
                                   d->inv_s_p, d->alpha_ctx, d->inv_s_ctx, ctx, taps ? taps->scores : nullptr,
                                   taps ? taps->p : nullptr, stream)))
            return rc;
    } else {
        if ((rc = nm_attn_scores(qkv, B, S, H, nh, scores, stream))) return rc;
        if ((rc = launch_softmax(scores, NM_DT_I32, d->alpha_scores, (int64_t)B * nh * S, S, t_exp, t_recip,
                                 d->inv_s_p, pm, nullptr, nullptr, nullptr, stream)))
            return rc;
        if ((rc = nm_attn_context(pm, qkv, B, S, H, nh, d->alpha_ctx, d->inv_s_ctx, ctx, stream))) return rc;
    }
    // 5: output projection + bias + residual(x) -> fp32;  6: LayerNorm-PWL -> int8.  One kernel when
    // the caller asks for it and the shape allows (the fp32 tensor then never reaches memory, so not
    // when its tap is wanted), else two.
    const bool want_fold = (d->flags & NM_LAYER_FOLD_LAYERNORM) && !(d->flags & NM_LAYER_NO_FOLD_LAYERNORM);
    {
        GemmArgs g;
        g.M = M; g.N = H; g.K = H;
        g.A = ctx; g.lda = H; g.W = d->Wo; g.ldw = H;
        g.bias = d->bo; g.alpha = d->alpha_o;
        g.resid = x; g.resid_scale = d->resid1_scale;
        g.ldo = H; g.out_f32 = attn;
        g.ln_gamma = d->gamma1; g.ln_beta = d->beta1; g.ln_eps = d->eps1; g.ln_inv_scale = d->inv_s_ln1;
        g.ln_table = t_rsqrt; g.ln_out_q = ln1;
        if (want_fold && !(taps && taps->attn) && gemm_folds_layernorm(g)) {
            g.ln = 1;
            if ((rc = launch_gemm(g, stream))) return rc;
        } else {
            if ((rc = launch_gemm(g, stream))) return rc;
            if ((rc = launch_layernorm(attn, d->gamma1, d->beta1, d->eps1, M, H, t_rsqrt, d->inv_s_ln1, ln1,
                                       nullptr, nullptr, stream)))
                return rc;
        }
    }
    // 7: FFN1 + bias, GELU-PWL in the epilogue -> int8
    {
        GemmArgs g;
        g.M = M; g.N = F; g.K = H;
        g.A = ln1; g.lda = H; g.W = d->W1; g.ldw = H;
        g.bias = d->b1; g.alpha = d->alpha_1;
        g.has_table = 1; g.table = t_gelu;
        g.out_inv_scale = d->inv_s_ffn1;
        g.ldo = F; g.out_q = ffn1;
        if ((rc = launch_gemm(g, stream))) return rc;
    }
    // 8: FFN2 + bias + residual(LN1 output) -> fp32;  9: LayerNorm-PWL -> layer output (one kernel or two, as above)
    {
        GemmArgs g;
        g.M = M; g.N = H; g.K = F;
        g.A = ffn1; g.lda = F; g.W = d->W2; g.ldw = F;
        g.bias = d->b2; g.alpha = d->alpha_2;
        g.resid = ln1; g.resid_scale = d->resid2_scale;
        g.ldo = H; g.out_f32 = ffn2;
        g.ln_gamma = d->gamma2; g.ln_beta = d->beta2; g.ln_eps = d->eps2; g.ln_inv_scale = d->inv_s_out;
        g.ln_table = t_rsqrt; g.ln_out_q = y_q; g.ln_out_f32 = y_f32;
        if (want_fold && !(taps && taps->ffn2) && gemm_folds_layernorm(g)) {
            g.ln = 1;
            return launch_gemm(g, stream);
        }
        if ((rc = launch_gemm(g, stream))) return rc;
    }
    return launch_layernorm(ffn2, d->gamma2, d->beta2, d->eps2, M, H, t_rsqrt, d->inv_s_out, y_q, y_f32,
                            nullptr, stream);
}

int32_t nm_encoder_layer_noalloc(const nm_layer_desc* d, const int8_t* x, int8_t* y_q, float* y_f32, void* stream)
{
    int32_t rc = validate_layer(d, "nm_encoder_layer_noalloc");  // dimensions; nm_encoder_layer checks the rest
    if (rc) return rc;
    const size_t need = plan_layer(d).total;
    if (need > kStaticScratchBytes)
        return fail(NM_ERR_WORKSPACE,
                    "nm_encoder_layer_noalloc: this shape needs %zu bytes of scratch, the built-in buffer holds %zu "
                    "(use nm_encoder_layer with a workspace of your own)", need, kStaticScratchBytes);
    void* ws = nullptr;
    if ((rc = static_scratch(&ws))) return rc;
    return nm_encoder_layer(d, x, y_q, y_f32, ws, kStaticScratchBytes, nullptr, stream);
}

// ---- stack of layers -------------------------------------------------------------------------

static int32_t validate_stack(const nm_layer_desc* descs, int32_t n_layers, const char* what, size_t* layer_ws)
{
    if (!descs) return fail(NM_ERR_INVALID_ARG, "%s: descs is NULL", what);
    if (n_layers < 1) return fail(NM_ERR_INVALID_ARG, "%s: n_layers %d < 1", what, n_layers);
    size_t need = 0;
    for (int32_t l = 0; l < n_layers; ++l) {
        int32_t rc = validate_layer(&descs[l], what);
        if (rc) return rc;
        if (descs[l].B != descs[0].B || descs[l].S != descs[0].S || descs[l].H != descs[0].H)
            return fail(NM_ERR_INVALID_ARG, "%s: layer %d has another B, S or H than layer 0", what, l);
        const size_t t = plan_layer(&descs[l]).total;
        if (t > need) need = t;
    }
    *layer_ws = need;
    return NM_OK;
}

int32_t nm_encoder_stack_workspace(const nm_layer_desc* descs, int32_t n_layers, size_t* bytes)
{
    size_t layer_ws = 0;
    int32_t rc = validate_stack(descs, n_layers, "nm_encoder_stack_workspace", &layer_ws);
    if (rc) return rc;
    if (!bytes) return fail(NM_ERR_INVALID_ARG, "nm_encoder_stack_workspace: bytes is NULL");
    const size_t act = round_up((size_t)descs[0].B * descs[0].S * descs[0].H, 256);
    *bytes = layer_ws + 2 * act;
    return NM_OK;
}

int32_t nm_encoder_stack(const nm_layer_desc* descs, int32_t n_layers, const int8_t* x, int8_t* y_q,
                         float* y_f32, void* ws, size_t ws_bytes, void* stream)
{
    size_t layer_ws = 0;
    int32_t rc = validate_stack(descs, n_layers, "nm_encoder_stack", &layer_ws);
    if (rc) return rc;
    if (!x) return fail(NM_ERR_INVALID_ARG, "nm_encoder_stack: x is NULL");
    if (!y_q && !y_f32) return fail(NM_ERR_INVALID_ARG, "nm_encoder_stack: no output");
    const size_t act = round_up((size_t)descs[0].B * descs[0].S * descs[0].H, 256);
    if (!ws) return fail(NM_ERR_WORKSPACE, "nm_encoder_stack: workspace is NULL");
    if (!aligned(ws, 256)) return fail(NM_ERR_WORKSPACE, "nm_encoder_stack: workspace not 256-byte aligned");
    if (ws_bytes < layer_ws + 2 * act)
        return fail(NM_ERR_WORKSPACE, "nm_encoder_stack: workspace %zu bytes < %zu needed", ws_bytes, layer_ws + 2 * act);
    // two activation buffers in front of the per-layer workspace; layer l writes buffer l % 2
    char* w = static_cast<char*>(ws);
    int8_t* act_buf[2] = {reinterpret_cast<int8_t*>(w), reinterpret_cast<int8_t*>(w + act)};
    void* lws = w + 2 * act;
    const int8_t* in = x;
    for (int32_t l = 0; l < n_layers; ++l) {
        const bool last = l == n_layers - 1;
        int8_t* out = last ? y_q : act_buf[l & 1];
        if ((rc = nm_encoder_layer(&descs[l], in, out, last ? y_f32 : nullptr, lws, ws_bytes - 2 * act, nullptr, stream)))
            return rc;
        in = out;
    }
    return NM_OK;
}

}  // extern "C"
