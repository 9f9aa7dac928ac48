/*
 * Sanitizer run of the CPU oracle (test infrastructure): every entry point is called on small,
 * ragged inputs held in heap buffers of exactly the documented size, so that AddressSanitizer sees
 * any access outside them and UndefinedBehaviorSanitizer any overflow, bad shift or misaligned
 * access.  Built and run by tests/test_sanitizers.py with -fsanitize=address,undefined.
 */
#include "../../oracle/nm_oracle.c"

#include <stdio.h>

static uint32_t g_state = 12345u;
static uint32_t rnd(void) { g_state = g_state * 1664525u + 1013904223u; return g_state >> 8; }
static void fill_i8(int8_t* p, size_t n, int amp) { for (size_t i = 0; i < n; ++i) p[i] = (int8_t)((int)(rnd() % (2 * amp + 1)) - amp); }
static void fill_f32(float* p, size_t n, float lo, float hi) { for (size_t i = 0; i < n; ++i) p[i] = lo + (hi - lo) * (float)(rnd() % 10001) / 10000.0f; }
#define NEW(T, n) ((T*)malloc(sizeof(T) * (size_t)((n) > 0 ? (n) : 1)))
#define CHECK(x) do { int rc_ = (x); if (rc_ != NMO_OK) { printf("FAILED %s -> %d (line %d)\n", #x, rc_, __LINE__); return 1; } } while (0)

static int make_table(int func, float lo, float hi, int nseg, int flags, nmo_table* t)
{
    float* k = NEW(float, nseg); float* b = NEW(float, nseg); float iw = 0;
    int rc = nmo_table_build(func, lo, hi, nseg, flags, 0.0, k, b, &iw);
    t->lo = lo; t->hi = hi; t->inv_w = iw; t->nseg = nseg; t->flags = flags & 1; t->k = k; t->b = b;
    return rc;
}
static void free_table(nmo_table* t) { free((void*)t->k); free((void*)t->b); }

int main(void)
{
    /* tables: every function, odd segment counts, Algorithm 3 and Algorithm 2 */
    static const float range[7][2] = {{-8, 8}, {-16, 0}, {1, 64}, {1e-3f, 64}, {-8, 8}, {0.25f, 64}, {-3, 5}};
    for (int f = 0; f < 7; ++f)
        for (int nseg = 1; nseg <= 67; nseg += 11)
            for (int flags = 0; flags <= 2; flags += 2) {
                nmo_table t;
                CHECK(make_table(f, range[f][0], range[f][1], nseg, flags, &t));
                free_table(&t);
                float* k = NEW(float, nseg); float* b = NEW(float, nseg); float iw; int32_t nm = 0;
                CHECK(nmo_table_build_merged(f, range[f][0], range[f][1], nseg, 0.02, flags, 0.0, k, b, &iw, &nm));
                if (nm < 1 || nm > nseg) { printf("FAILED merged count\n"); return 1; }
                free(k); free(b);
            }
    {   /* a merged table in its own form, evaluated directly */
        const int np_ = 37;
        int32_t* st = NEW(int32_t, np_); float* k = NEW(float, np_); float* b = NEW(float, np_); float iw; int32_t nm = 0;
        CHECK(nmo_table_build_merged_direct(0, -8, 8, np_, 0.03, 2, 0.0, st, k, b, &iw, &nm));
        nmo_merged_table mt = {-8, 8, iw, np_, 1, nm, st, k, b};
        const int n = 301;
        float* x = NEW(float, n); fill_f32(x, n, -12, 12); x[0] = NAN; x[1] = INFINITY; x[2] = -INFINITY;
        float* y = NEW(float, n); int8_t* q = NEW(int8_t, n); uint16_t* s1 = NEW(uint16_t, n); uint16_t* s2 = NEW(uint16_t, n);
        CHECK(nmo_pwl_apply_merged(x, NMO_DT_F32, 1.0f, n, &mt, 9.0f, q, y, s1, s2));
        free(st); free(k); free(b); free(x); free(y); free(q); free(s1); free(s2);
    }
    double* xs = NEW(double, 17);
    if (nmo_size_optimize_builtin(0, -4.0, 4.0, 0.5, 0.1, xs, 16) < 1) { printf("FAILED size_optimize\n"); return 1; }
    free(xs);

    nmo_table gelu, ex, rc, rs, sq;
    CHECK(make_table(0, -8, 8, 37, 0, &gelu)); CHECK(make_table(1, -16, 0, 64, 1, &ex));
    CHECK(make_table(2, 1, 64, 33, 0, &rc)); CHECK(make_table(3, 1e-3f, 64, 29, 0, &rs)); CHECK(make_table(5, 0.25f, 64, 31, 0, &sq));

    /* element-wise PWL: fp32 and int32 inputs, every output */
    for (int n = 0; n <= 131; n += 131) {
        float* x = NEW(float, n); fill_f32(x, (size_t)n, -12, 12);
        if (n > 3) { x[0] = NAN; x[1] = INFINITY; x[2] = -INFINITY; }
        int32_t* xi = NEW(int32_t, n); for (int i = 0; i < n; ++i) xi[i] = (int32_t)(rnd() % 80001) - 40000;
        float* y = NEW(float, n); int8_t* q = NEW(int8_t, n); uint16_t* s = NEW(uint16_t, n);
        CHECK(nmo_pwl_apply(x, NMO_DT_F32, 1.0f, n, &gelu, 9.0f, q, y, s));
        CHECK(nmo_pwl_apply(xi, NMO_DT_I32, 2e-4f, n, &ex, 100.0f, q, y, s));
        free(x); free(xi); free(y); free(q); free(s);
    }
    /* row kernels: ragged column counts around the groups of four and the 64 accumulators */
    static const int cols_list[] = {1, 3, 4, 5, 63, 64, 65, 255, 257, 700};
    for (unsigned c = 0; c < sizeof cols_list / sizeof cols_list[0]; ++c) {
        const int rows = 3, cols = cols_list[c];
        int32_t* a = NEW(int32_t, rows * cols); for (int i = 0; i < rows * cols; ++i) a[i] = (int32_t)(rnd() % 6001) - 3000;
        float* xf = NEW(float, rows * cols); fill_f32(xf, (size_t)rows * cols, -3, 3);
        float* g = NEW(float, cols); float* be = NEW(float, cols); fill_f32(g, (size_t)cols, 0.9f, 1.1f); fill_f32(be, (size_t)cols, -0.1f, 0.1f);
        float* y = NEW(float, rows * cols); int8_t* q = NEW(int8_t, rows * cols);
        uint16_t* se = NEW(uint16_t, rows * cols); uint16_t* sr = NEW(uint16_t, rows); uint16_t* sr2 = NEW(uint16_t, rows);
        CHECK(nmo_softmax_pwl(a, NMO_DT_I32, 3e-3f, rows, cols, &ex, &rc, 127.0f, q, y, se, sr));
        CHECK(nmo_softmax_pwl(xf, NMO_DT_F32, 1.0f, rows, cols, &ex, &rc, 127.0f, q, y, se, sr));
        CHECK(nmo_layernorm_pwl(xf, g, be, 1e-5f, rows, cols, &rs, 20.0f, q, y, sr));
        CHECK(nmo_layernorm_pwl2(xf, g, be, 1e-5f, rows, cols, &sq, &rc, 20.0f, q, y, sr, sr2));
        (void)nmo_canonical_sum(xf, cols); (void)nmo_canonical_sumsq(xf, cols);
        free(a); free(xf); free(g); free(be); free(y); free(q); free(se); free(sr); free(sr2);
    }
    /* GEMM with every option, shapes off every grid; extreme operands near the int32 range */
    {
        const int M = 7, N = 5, K = 131;
        int8_t* A = NEW(int8_t, M * K); int8_t* W = NEW(int8_t, N * K); int8_t* R = NEW(int8_t, M * N);
        fill_i8(A, (size_t)M * K, 127); fill_i8(W, (size_t)N * K, 127); fill_i8(R, (size_t)M * N, 127);
        float* bias = NEW(float, N); float* av = NEW(float, N); float* ov = NEW(float, N);
        fill_f32(bias, N, -1, 1); fill_f32(av, N, 1e-4f, 2e-4f); fill_f32(ov, N, 5, 50);
        int8_t* q = NEW(int8_t, M * N); float* y = NEW(float, M * N); int32_t* acc = NEW(int32_t, M * N); uint16_t* seg = NEW(uint16_t, M * N);
        nmo_gemm g; memset(&g, 0, sizeof g);
        g.M = M; g.N = N; g.K = K; g.A = A; g.W = W; g.bias = bias; g.alpha_vec = av; g.resid = R; g.resid_scale = 0.01f;
        g.table = &gelu; g.out_inv_scale_vec = ov; g.out_q = q; g.out_f32 = y; g.out_acc = acc; g.dbg_seg = seg;
        CHECK(nmo_gemm_pwl(&g));
        const int K2 = 65536; int8_t* A2 = NEW(int8_t, K2); int8_t* W2 = NEW(int8_t, K2);
        memset(A2, 127, K2); memset(W2, -127, K2);
        memset(&g, 0, sizeof g); g.M = 1; g.N = 1; g.K = K2; g.A = A2; g.W = W2; g.alpha = 1e-9f; g.out_acc = acc; g.out_f32 = y;
        CHECK(nmo_gemm_pwl(&g));
        if (acc[0] != -65536 * 16129) { printf("FAILED extreme accumulator\n"); return 1; }
        free(A); free(W); free(R); free(bias); free(av); free(ov); free(q); free(y); free(acc); free(seg); free(A2); free(W2);
    }
    /* convolution and pooling: padding, stride, odd channel counts */
    {
        nmo_table relu; CHECK(make_table(4, -8, 8, 2, 0, &relu));
        const int B = 2, H = 7, Wd = 5, Cin = 3, Cout = 5, kh = 3, kw = 3, stride = 2, pad = 1;
        const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (Wd + 2 * pad - kw) / stride + 1;
        int8_t* x = NEW(int8_t, B * H * Wd * Cin); int8_t* w = NEW(int8_t, Cout * kh * kw * Cin); int8_t* r = NEW(int8_t, B * Ho * Wo * Cout);
        fill_i8(x, (size_t)B * H * Wd * Cin, 127); fill_i8(w, (size_t)Cout * kh * kw * Cin, 127); fill_i8(r, (size_t)B * Ho * Wo * Cout, 100);
        float* bias = NEW(float, Cout); float* av = NEW(float, Cout); fill_f32(bias, Cout, -1, 1); fill_f32(av, Cout, 1e-3f, 2e-3f);
        int8_t* q = NEW(int8_t, B * Ho * Wo * Cout); float* y = NEW(float, B * Ho * Wo * Cout); int32_t* acc = NEW(int32_t, B * Ho * Wo * Cout);
        nmo_conv c; memset(&c, 0, sizeof c);
        c.B = B; c.H = H; c.W = Wd; c.Cin = Cin; c.Cout = Cout; c.kh = kh; c.kw = kw; c.stride = stride; c.pad = pad;
        c.x = x; c.w = w; c.bias = bias; c.alpha_vec = av; c.resid = r; c.resid_scale = 0.02f; c.table = &relu; c.out_inv_scale = 30.0f;
        c.out_q = q; c.out_f32 = y; c.out_acc = acc;
        CHECK(nmo_conv2d_pwl(&c));
        const int Hp = (H + 2 - 3) / 2 + 1, Wp = (Wd + 2 - 3) / 2 + 1;
        int8_t* mp = NEW(int8_t, B * Hp * Wp * Cin);
        CHECK(nmo_maxpool_i8(x, B, H, Wd, Cin, 3, 2, 1, mp));
        int8_t* aq = NEW(int8_t, B * Cin); float* af = NEW(float, B * Cin);
        CHECK(nmo_avgpool_i8(x, B, H * Wd, Cin, 0.01f, 10.0f, aq, af));
        free(x); free(w); free(r); free(bias); free(av); free(q); free(y); free(acc); free(mp); free(aq); free(af); free_table(&relu);
    }
    /* one ragged encoder layer, quantised and exact mode, with every tap */
    {
        const int B = 2, S = 10, H = 24, heads = 3, F = 40, M = B * S;
        nmo_layer L; memset(&L, 0, sizeof L);
        L.B = B; L.S = S; L.H = H; L.heads = heads; L.F = F;
        int8_t* Wqkv = NEW(int8_t, 3 * H * H); int8_t* Wo = NEW(int8_t, H * H); int8_t* W1 = NEW(int8_t, F * H); int8_t* W2 = NEW(int8_t, H * F);
        fill_i8(Wqkv, (size_t)3 * H * H, 127); fill_i8(Wo, (size_t)H * H, 127); fill_i8(W1, (size_t)F * H, 127); fill_i8(W2, (size_t)H * F, 127);
        float* bqkv = NEW(float, 3 * H); float* bo = NEW(float, H); float* b1 = NEW(float, F); float* b2 = NEW(float, H);
        float* g1 = NEW(float, H); float* be1 = NEW(float, H); float* g2 = NEW(float, H); float* be2 = NEW(float, H);
        fill_f32(bqkv, 3 * H, -.1f, .1f); fill_f32(bo, H, -.1f, .1f); fill_f32(b1, F, -.1f, .1f); fill_f32(b2, H, -.1f, .1f);
        fill_f32(g1, H, .9f, 1.1f); fill_f32(be1, H, -.1f, .1f); fill_f32(g2, H, .9f, 1.1f); fill_f32(be2, H, -.1f, .1f);
        L.Wqkv = Wqkv; L.bqkv = bqkv; L.Wo = Wo; L.bo = bo; L.W1 = W1; L.b1 = b1; L.W2 = W2; L.b2 = b2;
        L.gamma1 = g1; L.beta1 = be1; L.gamma2 = g2; L.beta2 = be2; L.eps1 = L.eps2 = 1e-5f;
        L.alpha_qkv = 2e-4f; L.inv_s_q = L.inv_s_k = L.inv_s_v = 40.0f; L.alpha_scores = 1e-4f; L.inv_s_p = 127.0f;
        L.alpha_ctx = 2e-4f; L.inv_s_ctx = 50.0f; L.alpha_o = 1e-4f; L.resid1_scale = 0.02f; L.inv_s_ln1 = 30.0f;
        L.alpha_1 = 2e-4f; L.inv_s_ffn1 = 40.0f; L.alpha_2 = 1e-4f; L.resid2_scale = 0.03f; L.inv_s_out = 30.0f;
        L.t_gelu = &gelu; L.t_exp = &ex; L.t_recip = &rc; L.t_rsqrt = &rs;
        int8_t* x = NEW(int8_t, M * H); fill_i8(x, (size_t)M * H, 127);
        int8_t* yq = NEW(int8_t, M * H); float* yf = NEW(float, M * H);
        nmo_taps T; memset(&T, 0, sizeof T);
        T.qkv = NEW(int8_t, M * 3 * H); T.scores = NEW(int32_t, B * heads * S * S); T.p = NEW(int8_t, B * heads * S * S);
        T.ctx = NEW(int8_t, M * H); T.attn = NEW(float, M * H); T.ln1 = NEW(int8_t, M * H); T.ffn1 = NEW(int8_t, M * F); T.ffn2 = NEW(float, M * H);
        CHECK(nmo_encoder_layer(&L, x, yq, yf, &T));
        CHECK(nmo_encoder_layer(&L, x, yq, NULL, NULL));
        double* ye = NEW(double, M * H); double am[13];
        CHECK(nmo_encoder_layer_exact(&L, x, 1, ye, am));
        CHECK(nmo_encoder_layer_exact(&L, x, 0, ye, am));
        free(Wqkv); free(Wo); free(W1); free(W2); free(bqkv); free(bo); free(b1); free(b2); free(g1); free(be1); free(g2); free(be2);
        free(x); free(yq); free(yf); free(T.qkv); free(T.scores); free(T.p); free(T.ctx); free(T.attn); free(T.ln1); free(T.ffn1); free(T.ffn2); free(ye);
    }
    free_table(&gelu); free_table(&ex); free_table(&rc); free_table(&rs); free_table(&sq);
    printf("SANITIZE_OK\n");
    return 0;
}
