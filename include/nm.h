/*
 * nm.h -- C ABI of the MI355X (gfx950) NeuralMatrix inference library.
 *
 * The library computes transformer encoder layers (and residual CNNs, as convolutions in matrix
 * form) with linear matrix operations only (paper, Section 3): every linear operator is an
 * int8 x int8 -> int32 matrix product (Section 3.1) and
 * every nonlinear operator (GELU, the exponential and the reciprocal of softmax, the reciprocal
 * square root of LayerNorm) is a piecewise-linear table y = k[s]*x + b[s] whose segment s is found
 * by quantising x (Section 3.2, Post-Training Approximation; Algorithm 3 for k, b; Algorithm 2
 * for merged segments).
 *
 * Conventions
 *   - Plain C.  Every function returns an nm_status (0 = NM_OK, negative = error) unless stated.
 *     After an error nm_last_error() returns a thread-local description.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     memory.  The library allocates only nm_tables objects.  Compute entry points are
 *     asynchronous on the given stream (a hipStream_t passed as void*, NULL = default stream),
 *     allocate nothing and never synchronise with the host.
 *   - Arguments are validated before the first HIP call; validation failures leave the GPU
 *     untouched (and work on a machine without a GPU).
 *   - Matrices are row-major.  Activations are [rows, cols]; weights are [N, K] with K contiguous
 *     (the layout of a fully connected layer's weight, and the one the int8 matrix cores want for
 *     both operands).  Attention tensors are [B, S, heads, d] viewed as [B*S, H]; a head is a
 *     column slice, nothing is transposed in memory by the caller.
 *   - Floating-point work is IEEE binary32, round-to-nearest-even, in one normative operation
 *     order, so that segment indices and int8 codes are reproducible bit for bit:
 *       segment:   u = (x - lo) * inv_w  (one subtract, one multiply), clamped in float to
 *                  [0, nseg-1], floor.  A break point belongs to the segment on its right;
 *                  x >= hi uses the last segment, x < lo and NaN the first (inputs outside the
 *                  range share the edge segments' parameters).
 *       PWL:       y = fma(k[s], x, b[s])
 *       int8 code: q = clamp(rint(v * inv_scale), -127, 127)
 *       row sum:   element j goes to accumulator (j / 4) % 64; each accumulator adds its elements
 *                  in increasing j starting from +0; the 64 partial sums are combined by a
 *                  butterfly with partner masks 32, 16, 8, 4, 2, 1.
 */
#ifndef NM_H
#define NM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    NM_OK = 0,
    NM_ERR_INVALID_ARG = -1, /* null pointer, non-positive dimension, hi <= lo, nseg < 1, ... */
    NM_ERR_UNSUPPORTED = -2, /* a shape the kernels do not cover (limits are stated per call) */
    NM_ERR_ALLOC = -3,
    NM_ERR_HIP = -4,         /* a HIP runtime call failed; see nm_last_error() */
    NM_ERR_WORKSPACE = -5    /* workspace too small or misaligned */
} nm_status;

/* Nonlinear functions a table can be built for (the paper's four: e^x, sqrt x, 1/x, GELU, plus
 * the reciprocal square root LayerNorm uses here, ReLU which is already piecewise linear, and the
 * identity). */
enum { NM_FUNC_GELU = 0, NM_FUNC_EXP = 1, NM_FUNC_RECIP = 2, NM_FUNC_RSQRT = 3, NM_FUNC_RELU = 4,
       NM_FUNC_SQRT = 5, NM_FUNC_IDENTITY = 6 };

enum {
    NM_TABLE_CLAMP_INPUT = 1,  /* clamp x to [lo, hi] before evaluation instead of extrapolating */
    NM_TABLE_BIAS_CORRECT = 2, /* Algorithm 3: shift b by the expectation bias when |dE| > e_th */
    NM_TABLE_MERGE = 4,        /* Algorithm 2: merge neighbouring primary segments whose slope
                                  stays within dk_th of the slope at the last kept start point;
                                  nseg is then the number of primary cells */
    NM_TABLE_COMPACT = 8       /* keep a merged table in two levels as well: one {k, b} per merged
                                  segment plus one byte per primary cell naming its segment (at most
                                  256 segments), so that a kernel holds n_segments * 8 + nseg bytes of
                                  it instead of nseg * 8.  nm_pwl_apply, nm_gemm_pwl and the FFN1
                                  product of nm_encoder_layer / nm_encoder_stack look such a table up
                                  in two steps (cell of x, segment of the cell); the other entry
                                  points use its expanded form.  Results are identical either way;
                                  reported segment indices are always primary cell indices */
};

enum { NM_DT_I32 = 0, NM_DT_F32 = 1 };

#define NM_MAX_SEGMENTS 4096 /* per table */
#define NM_MAX_TABLES 16     /* per nm_tables object */

typedef struct {
    int32_t func;  /* NM_FUNC_* */
    float lo;      /* range of the approximated input; hi > lo */
    float hi;
    int32_t nseg;  /* number of uniform segments (cells), 1 .. NM_MAX_SEGMENTS */
    int32_t flags; /* NM_TABLE_* */
    float e_th;    /* Algorithm 3 threshold (0 = always correct) */
    float dk_th;   /* Algorithm 2 slope threshold (used with NM_TABLE_MERGE) */
} nm_table_desc;

typedef struct nm_tables nm_tables; /* opaque: host copy + device blob of up to 16 tables */

/* Thread-local text of the last error on this thread ("" if none). Never NULL. */
const char* nm_last_error(void);

/* Library version, major * 1000 + minor. */
int32_t nm_version(void);

/*
 * Host-only table construction (Section 3.2: fixed-length segments, each fitted by the line
 * through the function values at its two ends, so neighbouring lines meet; Algorithm 3 step 1;
 * with NM_TABLE_BIAS_CORRECT the rest of Algorithm 3; with NM_TABLE_MERGE Algorithm 2 first and
 * the chords are taken over the merged segments, expanded back onto the nseg primary cells).
 * All arithmetic in binary64, results rounded once to binary32.
 * k, b: host arrays of desc->nseg floats (written).  inv_w: host, receives (float)(nseg/(hi-lo)).
 * n_distinct (may be NULL): number of distinct (k, b) pairs = segments after merging.
 * Never touches the GPU.
 */
int32_t nm_table_build_host(const nm_table_desc* desc, float* k, float* b, float* inv_w,
                            int32_t* n_distinct);

/*
 * Build n tables on the host (as nm_table_build_host) and upload them as one device blob on
 * `stream`.  descs: host array of n descriptors, 1 <= n <= NM_MAX_TABLES.  *out receives a new
 * object owned by the caller (nm_tables_destroy).  This is an offline call: it waits for the
 * upload on `stream` before it returns, so the tables may be used from any stream afterwards.
 */
int32_t nm_build_tables(const nm_table_desc* descs, int32_t n, void* stream, nm_tables** out);

/*
 * Same, but k and b come from the caller: k[i], b[i] are host arrays of descs[i].nseg floats.
 * descs[i].func / e_th / dk_th are ignored, lo / hi / nseg / NM_TABLE_CLAMP_INPUT /
 * NM_TABLE_COMPACT are used (the two-level form is derived from runs of equal {k, b}).
 */
int32_t nm_tables_from_arrays(const nm_table_desc* descs, int32_t n, const float* const* k,
                              const float* const* b, void* stream, nm_tables** out);

/* Number of tables in the object (0 for NULL). */
int32_t nm_tables_count(const nm_tables* t);

/*
 * Read table idx back from the host copy.  Any of desc, k_host, b_host, inv_w may be NULL.
 * k_host, b_host: host arrays of nseg floats.
 */
int32_t nm_tables_get(const nm_tables* t, int32_t idx, nm_table_desc* desc, float* k_host,
                      float* b_host, float* inv_w);

/*
 * The two-level form of table idx (built with NM_TABLE_COMPACT): number of merged segments, the
 * segment of every primary cell (host array of nseg bytes), and the segments' parameters (host
 * arrays of *n_segments floats; query the count first).  Any output may be NULL.
 */
int32_t nm_tables_get_compact(const nm_tables* t, int32_t idx, int32_t* n_segments, uint8_t* cell_to_segment,
                              float* k_host, float* b_host);

/* Frees the host copy and the device blob.  NULL is allowed.  The caller must make sure no kernel
 * that uses the tables is still running. */
void nm_tables_destroy(nm_tables* t);

/* ---------------------------------------------------------------------------------------------
 * nm_gemm_pwl: int8 GEMM with the fused epilogue (Section 3.1: a fully connected layer is a
 * matrix multiplication, a residual connection a matrix addition; Section 3.2 for the table).
 *
 *   acc[m,n] = sum_k A[m,k] * W[n,k]                      exact, int32
 *   v = fma((float)acc, alpha_n, bias_n)                   alpha_n = alpha_vec ? alpha_vec[n] : alpha
 *   v = fma((float)resid[m,n], resid_scale, v)             if resid
 *   v = PWL_table(v)                                       if table_idx >= 0
 *   out_f32[m,n] = v;  out_q[m,n] = int8 code of v with out_inv_scale_n;  out_acc[m,n] = acc;
 *   dbg_seg[m,n] = segment index of v (only written when a table is given)
 *
 * All pointers are device pointers; A [M,K], W [N,K], resid / outputs [M,N], all contiguous.
 * bias, alpha_vec, out_inv_scale_vec: [N] or NULL.  Any output may be NULL (at least one is
 * required).  Limits: 1 <= M, N, K; K <= 65536 (so |acc| <= K * 127^2 < 2^31); M*N < 2^31.
 * Shapes whose K is a multiple of 16 with 16-byte aligned A and W take the fast loader; any
 * other shape is computed by a slower loader with identical results.
 * Debug switches (environment, read once per process; results never change, only the kernel that
 * computes them): NM_GEMM_GENERIC=1 sends every shape to the generic kernel; NM_GEMM_CFG=
 * big|wide|split|small|mid3|mid2|oldbig forces a tile configuration where its requirements hold;
 * NM_ATTN_UNFUSED=1 keeps nm_encoder_layer's attention on the three separate kernels.
 * --------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t M, N, K;
    const int8_t* A;
    const int8_t* W;
    const float* bias;
    const float* alpha_vec;
    float alpha;
    const int8_t* resid;
    float resid_scale;
    const nm_tables* tables;
    int32_t table_idx; /* -1 = no nonlinearity */
    float out_inv_scale;
    const float* out_inv_scale_vec;
    int8_t* out_q;
    float* out_f32;
    int32_t* out_acc;
    uint16_t* dbg_seg;
    /* split_cols > 0: the int8 code of column n uses out_inv_scale3[min(n / split_cols, 2)] instead of
     * out_inv_scale (a fused Q | K | V projection has one output scale per third); out_inv_scale_vec
     * must then be NULL.  0: not used. */
    int32_t split_cols;
    float out_inv_scale3[3];
} nm_gemm_desc;

int32_t nm_gemm_pwl(const nm_gemm_desc* desc, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_softmax_pwl: row softmax with PWL exponential and PWL reciprocal (the paper lists e^x and
 * 1/x among the functions it approximates; the decomposition is this library's):
 *   m = max_j in_j;  t_j = (float)(in_j - m) * alpha;  e_j = PWL_exp(t_j);
 *   S = canonical row sum of e;  r = PWL_recip(S);  p_j = e_j * r.
 * in: device [rows, cols] int32 (NM_DT_I32; the subtraction is then exact) or fp32 (NM_DT_F32).
 * Outputs (device, any may be NULL, at least one of out_q / out_f32 required): out_q int8 codes
 * of p with out_inv_scale, out_f32 p, dbg_seg_exp [rows, cols] exp segment of every element,
 * dbg_seg_recip [rows] reciprocal segment of every row.
 * Limits: 1 <= cols <= 4096, rows >= 0, rows * cols < 2^40; alpha finite (NM_ERR_INVALID_ARG).
 * --------------------------------------------------------------------------------------------- */
int32_t nm_softmax_pwl(const void* in, int32_t in_dtype, float alpha, int64_t rows, int32_t cols,
                       const nm_tables* tables, int32_t exp_idx, int32_t recip_idx,
                       float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg_exp,
                       uint16_t* dbg_seg_recip, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_layernorm_pwl: row LayerNorm with a PWL reciprocal square root:
 *   mu = rowsum(x) * inv_L;  d_j = x_j - mu;  var = rowsum_fma(d_j * d_j) * inv_L;
 *   r = PWL_rsqrt(var + eps);  y_j = fma(d_j * r, gamma_j, beta_j);   inv_L = (float)(1.0 / cols)
 * in: device fp32 [rows, cols]; gamma, beta: device fp32 [cols].
 * Outputs (device, any may be NULL, at least one of out_q / out_f32 required): out_q int8 codes of
 * y with out_inv_scale, out_f32 y, dbg_seg [rows] the rsqrt segment of every row.
 * Limits: 1 <= cols <= 4096, rows >= 0.
 * --------------------------------------------------------------------------------------------- */
int32_t nm_layernorm_pwl(const float* in, const float* gamma, const float* beta, float eps,
                         int64_t rows, int32_t cols, const nm_tables* tables, int32_t rsqrt_idx,
                         float out_inv_scale, int8_t* out_q, float* out_f32, uint16_t* dbg_seg,
                         void* stream);

/*
 * nm_layernorm_pwl2: the same with the two functions the paper's list names instead of one rsqrt
 * table: sd = PWL_sqrt(var + eps); r = PWL_recip(sd).  dbg_seg_sqrt / dbg_seg_recip: [rows].
 */
int32_t nm_layernorm_pwl2(const float* in, const float* gamma, const float* beta, float eps,
                          int64_t rows, int32_t cols, const nm_tables* tables, int32_t sqrt_idx,
                          int32_t recip_idx, float out_inv_scale, int8_t* out_q, float* out_f32,
                          uint16_t* dbg_seg_sqrt, uint16_t* dbg_seg_recip, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_pwl_apply: the stand-alone element-wise PWL calculation over a flat buffer (Section 3: an
 * operator that is piecewise linear is evaluated by finding each element's segment, gathering k
 * and b, and one multiply-add):  x = (float)in_i * alpha;  y = PWL(x).
 * in: device int32 or fp32 [n].  Outputs (device, any may be NULL, at least one required):
 * out_q int8, out_f32, dbg_seg uint16.  n >= 0.
 * --------------------------------------------------------------------------------------------- */
int32_t nm_pwl_apply(const void* in, int32_t in_dtype, float alpha, int64_t n,
                     const nm_tables* tables, int32_t idx, float out_inv_scale, int8_t* out_q,
                     float* out_f32, uint16_t* dbg_seg, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Attention products (Section 3.1: attention is a linear operation mapped to matrix products).
 * qkv: device int8 [B*S, 3H]: columns [0,H) queries, [H,2H) keys, [2H,3H) values; head t owns
 * columns t*d .. t*d+d-1 of each third, d = H / heads.
 *   nm_attn_scores :  scores[b,t,i,j] = sum_c Q[b,i,t,c] * K[b,j,t,c]       int32 [B,heads,S,S]
 *   nm_attn_context:  acc = sum_j P[b,t,i,j] * V[b,j,t,c];  v = fma((float)acc, alpha, 0);
 *                     ctx[b,i,t*d+c] = int8 code of v with out_inv_scale      int8 [B*S, H]
 * p: device int8 [B,heads,S,S].  Limits: H % heads == 0, S <= 4096.
 * --------------------------------------------------------------------------------------------- */
int32_t nm_attn_scores(const int8_t* qkv, int32_t B, int32_t S, int32_t H, int32_t heads,
                       int32_t* scores, void* stream);
int32_t nm_attn_context(const int8_t* p, const int8_t* qkv, int32_t B, int32_t S, int32_t H,
                        int32_t heads, float alpha, float out_inv_scale, int8_t* ctx,
                        void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_attention_pwl: the three attention steps in one kernel (scores, softmax-PWL, context), with
 * results bit-identical to nm_attn_scores -> nm_softmax_pwl -> nm_attn_context; the int32 scores
 * and the int8 probabilities stay in registers.  scores_out / p_out (device, [B,heads,S,S]) may be
 * NULL; when given they receive the intermediate tensors.
 * Limits: head size H / heads == 64, S <= 512, qkv 16-byte aligned, H % 16 == 0; other shapes
 * return NM_ERR_UNSUPPORTED and the caller uses the three separate calls.  alpha_scores must be
 * finite (NM_ERR_INVALID_ARG otherwise).
 * --------------------------------------------------------------------------------------------- */
int32_t nm_attention_pwl(const int8_t* qkv, int32_t B, int32_t S, int32_t H, int32_t heads,
                         float alpha_scores, const nm_tables* tables, int32_t exp_idx,
                         int32_t recip_idx, float inv_s_p, float alpha_ctx, float inv_s_ctx,
                         int8_t* ctx, int32_t* scores_out, int8_t* p_out, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_encoder_layer: one post-LayerNorm (BERT ordering) encoder layer, no mask, no dropout:
 *   1 QKV projection (+bias), each third requantised with its own scale
 *   2 scores = Q K^T per (batch, head)                        int32
 *   3 softmax-PWL over each score row                          int8
 *   4 context = P V per (batch, head), requantised             int8
 *   5 output projection + bias + residual(x)                   fp32
 *   6 LayerNorm-PWL                                            int8
 *   7 FFN1 + bias, GELU-PWL in the GEMM epilogue               int8
 *   8 FFN2 + bias + residual(LN1 output)                       fp32
 *   9 LayerNorm-PWL                                            int8 (+ fp32)
 * All weight / vector pointers are device pointers.  The float multipliers are formed by the
 * caller from the tensors' quantisation scales (s_*) and passed as binary32 numbers.
 * --------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t B, S, H, heads, F;
    const int8_t* Wqkv; const float* bqkv; /* [3H, H] rows Wq | Wk | Wv; [3H] */
    const int8_t* Wo;   const float* bo;   /* [H, H]; [H] */
    const int8_t* W1;   const float* b1;   /* [F, H]; [F] */
    const int8_t* W2;   const float* b2;   /* [H, F]; [H] */
    const float* gamma1; const float* beta1; /* [H] */
    const float* gamma2; const float* beta2; /* [H] */
    float eps1, eps2;
    float alpha_qkv;              /* s_x * s_wqkv */
    float inv_s_q, inv_s_k, inv_s_v;
    float alpha_scores;           /* s_q * s_k / sqrt(d) */
    float inv_s_p;
    float alpha_ctx;              /* s_p * s_v */
    float inv_s_ctx;
    float alpha_o;                /* s_ctx * s_wo */
    float resid1_scale;           /* s_x */
    float inv_s_ln1;
    float alpha_1;                /* s_ln1 * s_w1 */
    float inv_s_ffn1;
    float alpha_2;                /* s_ffn1 * s_w2 */
    float resid2_scale;           /* s_ln1 */
    float inv_s_out;
    const nm_tables* tables;
    int32_t gelu_idx, exp_idx, recip_idx, rsqrt_idx;
    int32_t flags;                /* NM_LAYER_* (0: the library chooses) */
} nm_layer_desc;

/* Steps 5+6 and 8+9 as one kernel each (the LayerNorm runs in the epilogue of the matrix product,
 * on workgroups that own whole rows; the fp32 tensor between them never reaches memory).  Needs
 * H = 768 or 1024 and aligned operands; where that does not hold, or taps of the fp32 tensors are
 * asked for, the two-kernel path runs.  Results are identical either way. */
enum { NM_LAYER_FOLD_LAYERNORM = 1, NM_LAYER_NO_FOLD_LAYERNORM = 2 };

/* Optional device buffers that receive the intermediate tensors (any may be NULL; a non-NULL
 * buffer is used as that tensor's storage, so it costs nothing extra). */
typedef struct {
    int8_t* qkv;     /* [B*S, 3H] */
    int32_t* scores; /* [B, heads, S, S] */
    int8_t* p;       /* [B, heads, S, S] */
    int8_t* ctx;     /* [B*S, H] */
    float* attn;     /* [B*S, H] */
    int8_t* ln1;     /* [B*S, H] */
    int8_t* ffn1;    /* [B*S, F] */
    float* ffn2;     /* [B*S, H] */
} nm_layer_taps;

/* Bytes of device workspace nm_encoder_layer needs for this shape (host computation only). */
int32_t nm_encoder_layer_workspace(const nm_layer_desc* desc, size_t* bytes);

/*
 * x: device int8 [B*S, H].  y_q: device int8 [B*S, H] or NULL.  y_f32: device fp32 [B*S, H] or
 * NULL (at least one required).  ws: device workspace of at least the queried size, 256-byte
 * aligned; its contents are scratch.  taps may be NULL.
 * Limits: those of the calls above; H % heads == 0.
 */
int32_t nm_encoder_layer(const nm_layer_desc* desc, const int8_t* x, int8_t* y_q, float* y_f32,
                         void* ws, size_t ws_bytes, const nm_layer_taps* taps, void* stream);

/*
 * nm_encoder_layer_noalloc: nm_encoder_layer for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation): the workspace is
 * a buffer of NM_NOALLOC_MAX_WORKSPACE bytes built into the library's device image (each GPU the
 * library runs on holds one until the process ends), so the caller passes inputs and outputs only.
 * Same results as nm_encoder_layer, no taps.  Calls nothing that allocates or frees.
 * Returns NM_ERR_WORKSPACE (message says how much is needed) when nm_encoder_layer_workspace of
 * the shape exceeds NM_NOALLOC_MAX_WORKSPACE: B32 S128 H768 F3072 fits, B16 S512 H768 does not.
 * Every call on a GPU uses that GPU's one buffer, whose contents are scratch and survive from call
 * to call (nothing in it needs to start at zero): two calls that overlap in time on the same GPU,
 * from different streams or threads, race.  Calls on one stream are ordered and safe.
 */
#define NM_NOALLOC_MAX_WORKSPACE (64u << 20)
int32_t nm_encoder_layer_noalloc(const nm_layer_desc* desc, const int8_t* x, int8_t* y_q, float* y_f32,
                                 void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_encoder_stack: n_layers encoder layers back to back on one stream (the paper's Section 4
 * models are stacks of identical layers: 12 for BERT-base, 24 for BERT-large).  Layer l reads the
 * int8 output of layer l-1, so descs[l].resid1_scale / alpha_qkv must be formed from layer l-1's
 * output scale (the caller's job, as for every other multiplier).  All layers share B, S and H;
 * F and the tables may differ per layer.
 * descs: HOST array of n_layers descriptors (read during the call only).  x, y_q, y_f32 as for
 * nm_encoder_layer (y_f32 is the last layer's fp32 output).  If only y_f32 is given and
 * n_layers > 1 the intermediate layers still produce int8.  The workspace holds two activation
 * buffers plus the largest per-layer workspace; query it first.  Nothing is allocated and the
 * host does not wait for the GPU.
 * --------------------------------------------------------------------------------------------- */
int32_t nm_encoder_stack_workspace(const nm_layer_desc* descs, int32_t n_layers, size_t* bytes);
int32_t nm_encoder_stack(const nm_layer_desc* descs, int32_t n_layers, const int8_t* x, int8_t* y_q,
                         float* y_f32, void* ws, size_t ws_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_conv2d_pwl: int8 convolution in its matrix form (paper Section 3.1: a convolution becomes a
 * matrix product whose dimensions follow from the width, height and channel counts) with the
 * epilogue of nm_gemm_pwl:
 *   acc[b,ho,wo,n] = sum_{i,j,c} x[b, ho*stride - pad + i, wo*stride - pad + j, c] * w[n,i,j,c]
 *                    (exact int32; positions outside the image contribute nothing)
 *   v = fma((float)acc, alpha_n, bias_n);  v = fma((float)resid, resid_scale, v) if resid;
 *   v = PWL(v) if table_idx >= 0 (ReLU is the exact two-segment table);  outputs v and its int8 code.
 * Ho = (H + 2*pad - kh) / stride + 1, Wo likewise.
 * x: device int8 [B, H, W, Cin] (channels contiguous).  w: device int8 [Cout, kh, kw, Cin].
 * bias, alpha_vec: device fp32 [Cout] or NULL (alpha_vec NULL -> alpha; a folded batch
 * normalisation is a per-channel alpha_vec and bias).  resid: device int8 [B, Ho, Wo, Cout] or
 * NULL.  Outputs (device, any may be NULL, at least one required): out_q int8, out_f32, dbg_acc
 * int32, each [B, Ho, Wo, Cout].
 * Workspace: needed only when Cin is not a multiple of 64 (or x / w are not 16-byte aligned) and
 * the convolution is not 1x1 / stride 1 / no padding (a patch matrix, or for images of at most
 * four channels a few KB for the repacked filter); query nm_conv2d_workspace (0 otherwise; ws may
 * then be NULL).  256-byte aligned, contents are scratch.  Nothing is allocated, the host
 * does not wait.  Limits: kh*kw*Cin <= 65536, B*Ho*Wo < 2^31, B*Ho*Wo*Cout < 2^31.
 * --------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t B, H, W, Cin, Cout, kh, kw, stride, pad;
    const int8_t* x;
    const int8_t* w;
    const float* bias;
    const float* alpha_vec;
    float alpha;
    const int8_t* resid;
    float resid_scale;
    const nm_tables* tables;
    int32_t table_idx; /* -1: no table */
    float out_inv_scale;
    int8_t* out_q;
    float* out_f32;
    int32_t* dbg_acc;
} nm_conv_desc;

int32_t nm_conv2d_workspace(const nm_conv_desc* desc, size_t* bytes);
int32_t nm_conv2d_pwl(const nm_conv_desc* desc, void* ws, size_t ws_bytes, void* stream);

/*
 * nm_maxpool_i8: k x k max pooling on int8 codes that share one scale (exact; the paper does not
 * discuss pooling).  Positions outside the image never take part.  x: device int8 [B, H, W, C];
 * y: device int8 [B, Ho, Wo, C] with Ho = (H + 2*pad - k) / stride + 1.  Requires pad < k.
 */
int32_t nm_maxpool_i8(const int8_t* x, int32_t B, int32_t H, int32_t W, int32_t C, int32_t k,
                      int32_t stride, int32_t pad, int8_t* y, void* stream);

/*
 * nm_avgpool_i8: global average pooling as the linear operation it is (Section 3.1):
 * acc[b,c] = sum over the HW positions (exact int32), v = (float)acc * alpha with alpha =
 * s_x / HW formed by the caller, out_f32 = v, out_q = its int8 code.  x: device int8 [B, HW, C].
 */
int32_t nm_avgpool_i8(const int8_t* x, int32_t B, int32_t HW, int32_t C, float alpha, float out_inv_scale,
                      int8_t* out_q, float* out_f32, void* stream);

/* ---------------------------------------------------------------------------------------------
 * nm_cnn_run: a list of convolution / pooling / matrix-product steps queued back to back on one
 * stream (a whole residual CNN in one call; the steps are the entry points above, so results are
 * identical to calling them one by one).  ops: HOST array, read during the call only; every tensor
 * pointer inside is a device pointer owned by the caller, who also wires each step's input to an
 * earlier step's output.  ws: one workspace shared by all steps (query nm_cnn_workspace: the
 * largest any step needs).  Stops at the first failing step and returns its status.
 * --------------------------------------------------------------------------------------------- */
enum { NM_OP_CONV = 0, NM_OP_MAXPOOL = 1, NM_OP_AVGPOOL = 2, NM_OP_GEMM = 3 };

typedef struct {
    int32_t kind;                 /* NM_OP_* */
    nm_conv_desc conv;            /* NM_OP_CONV */
    nm_gemm_desc gemm;            /* NM_OP_GEMM */
    /* NM_OP_MAXPOOL: x [B,H,W,C] -> y, window k, stride, pad.  NM_OP_AVGPOOL: x [B,HW,C] (H = HW,
     * W unused), alpha, out_inv_scale -> y (int8) and / or y_f32. */
    const int8_t* x;
    int8_t* y;
    float* y_f32;
    int32_t B, H, W, C, k, stride, pad;
    float alpha, out_inv_scale;
} nm_cnn_op;

int32_t nm_cnn_workspace(const nm_cnn_op* ops, int32_t n_ops, size_t* bytes);
int32_t nm_cnn_run(const nm_cnn_op* ops, int32_t n_ops, void* ws, size_t ws_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* NM_H */
