/*
 * sp_oracle.c -- CPU oracle for the K-student forward of Student Parallelism.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * HIP path is checked against.  It shares no code with the HIP path and must
 * never be reached from a product code path: only the test-suite, the smoke
 * check and the benchmark's cpu_baseline leg may build, load or call it.
 *
 * What is computed (paper: Section 3.1, Eq. 1; Section 3.2, Algorithm 2 lines
 * 5-6; Section 3.3): every student is an independent shallow BERT-like encoder
 * (token + position embedding, LayerNorm, N post-LN transformer layers), its
 * first-token state is pooled (dense + tanh) and classified; the ensemble
 * output for a sample is the sum, taken in training order, of the first
 * k_active students' outputs (dropping students from the tail is the paper's
 * adaptive student pruning).  Every sample is processed on its own, over
 * exactly its own tokens (no padding positions take part in attention).
 *
 * Arithmetic type: `real` is double by default and float when compiled with
 * -DSPO_REAL_FLOAT.  Both builds export the same symbols with double-typed
 * interfaces; conversion happens at the interface only.
 *
 * Parity pins (tests marked "not gpu"): LayerNorm, softmax, GELU, attention,
 * the encoder layer and the whole forward are pinned against closed forms,
 * brute force, and library routines (torch.nn.functional, torch.nn
 * .TransformerEncoderLayer, transformers.BertForSequenceClassification).
 * Agreement with the paper's accuracy and latency tables is PARITY UNPINNED:
 * it needs datasets and trained weights that do not exist here.
 *
 * Weight blob (float32, host), per student m = 0..K-1, in this order:
 *   tok_emb[V][H] pos_emb[P][H] emb_ln_g[H] emb_ln_b[H]
 *   per layer l = 0..Ly-1:
 *     Wq[H][H] bq[H] Wk[H][H] bk[H] Wv[H][H] bv[H] Wo[H][H] bo[H]
 *     ln1_g[H] ln1_b[H] W1[H][F] b1[F] W2[F][H] b2[H] ln2_g[H] ln2_b[H]
 *   Wp[H][H] bp[H] Wc[H][C] bc[C]
 * Every matrix is [in][out] row-major: y[o] = b[o] + sum_i x[i] * W[i][o].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef SPO_REAL_FLOAT
typedef float real;
#define R_SQRT sqrtf
#define R_EXP expf
#define R_ERF erff
#define R_TANH tanhf
#else
typedef double real;
#define R_SQRT sqrt
#define R_EXP exp
#define R_ERF erf
#define R_TANH tanh
#endif

typedef struct {
    int32_t K, layers, hidden, heads, ffn, vocab, max_pos, classes;
    double ln_eps;
} spo_config;

/* ---- blob geometry ------------------------------------------------------ */

static size_t layer_floats(const spo_config* c)
{
    size_t H = (size_t)c->hidden, F = (size_t)c->ffn;
    return 4 * (H * H + H) + 2 * H + (H * F + F) + (F * H + H) + 2 * H;
}

static size_t student_floats(const spo_config* c)
{
    size_t H = (size_t)c->hidden;
    return (size_t)c->vocab * H + (size_t)c->max_pos * H + 2 * H
         + (size_t)c->layers * layer_floats(c)
         + H * H + H + H * (size_t)c->classes + (size_t)c->classes;
}

/* number of float32 values in a blob for this configuration */
size_t spo_blob_floats(const spo_config* c) { return (size_t)c->K * student_floats(c); }

int spo_real_bytes(void) { return (int)sizeof(real); }

/* ---- a0: packing (integer, exact) --------------------------------------- */

/* cu[i] = sum of lengths[0..i-1]; cu has batch+1 entries.  Returns 0, or -1
 * when a length is < 1 (a sample without its first token has no pooled
 * state) or the total overflows int32. */
int spo_pack(const int32_t* lengths, int32_t batch, int32_t* cu)
{
    int64_t acc = 0;
    cu[0] = 0;
    for (int32_t i = 0; i < batch; ++i) {
        if (lengths[i] < 1) return -1;
        acc += lengths[i];
        if (acc > INT32_MAX) return -1;
        cu[i + 1] = (int32_t)acc;
    }
    return 0;
}

/* ---- elementary pieces --------------------------------------------------- */

/* LayerNorm over one row of n values: biased variance, eps inside the root. */
static void layernorm_row(const real* u, const float* g, const float* b, int n, real eps, real* out)
{
    real mean = 0;
    for (int c = 0; c < n; ++c) mean += u[c];
    mean /= (real)n;
    real var = 0;
    for (int c = 0; c < n; ++c) { real dlt = u[c] - mean; var += dlt * dlt; }
    var /= (real)n;
    real inv = (real)1 / R_SQRT(var + eps);
    for (int c = 0; c < n; ++c) out[c] = (real)g[c] * ((u[c] - mean) * inv) + (real)b[c];
}

/* GELU, exact erf form. */
static real gelu(real u) { return (real)0.5 * u * ((real)1 + R_ERF(u * (real)0.70710678118654752440)); }

/* softmax of one row in place: subtract the row maximum, exponentiate, divide. */
static void softmax_row(real* s, int n)
{
    real mx = s[0];
    for (int j = 1; j < n; ++j) if (s[j] > mx) mx = s[j];
    real sum = 0;
    for (int j = 0; j < n; ++j) { s[j] = R_EXP(s[j] - mx); sum += s[j]; }
    for (int j = 0; j < n; ++j) s[j] = s[j] / sum;
}

/* y[L][out] = x[L][in] . W[in][out] + b ; each y element sums i ascending. */
static void linear(const real* x, int L, int in, int out, const float* W, const float* b, real* y)
{
    for (int t = 0; t < L; ++t) {
        real* yr = y + (size_t)t * out;
        for (int o = 0; o < out; ++o) yr[o] = (real)b[o];
        for (int i = 0; i < in; ++i) {
            real xi = x[(size_t)t * in + i];
            const float* wr = W + (size_t)i * out;
            for (int o = 0; o < out; ++o) yr[o] += xi * (real)wr[o];
        }
    }
}

/* Multi-head attention over ONE sequence of L tokens.  q, k, v, o are
 * [L][A*d]; head h owns columns h*d .. h*d+d-1.  Scores are scaled by
 * 1/sqrt(d); every query attends to all L keys of its own sequence and to
 * nothing else.  probs (optional) receives [A][L][L]. */
static void attention(const real* q, const real* k, const real* v, int L, int A, int d, real* o, real* probs)
{
    int H = A * d;
    real scale = (real)1 / R_SQRT((real)d);
    real* s = (real*)malloc(sizeof(real) * (size_t)L);
    for (int h = 0; h < A; ++h) {
        for (int i = 0; i < L; ++i) {
            for (int j = 0; j < L; ++j) {
                real acc = 0;
                for (int e = 0; e < d; ++e)
                    acc += q[(size_t)i * H + h * d + e] * k[(size_t)j * H + h * d + e];
                s[j] = acc * scale;
            }
            softmax_row(s, L);
            if (probs) memcpy(probs + ((size_t)h * L + i) * L, s, sizeof(real) * (size_t)L);
            for (int e = 0; e < d; ++e) {
                real acc = 0;
                for (int j = 0; j < L; ++j) acc += s[j] * v[(size_t)j * H + h * d + e];
                o[(size_t)i * H + h * d + e] = acc;
            }
        }
    }
    free(s);
}

/* pointers into one layer's slice of the blob */
typedef struct {
    const float *Wq, *bq, *Wk, *bk, *Wv, *bv, *Wo, *bo, *ln1g, *ln1b, *W1, *b1, *W2, *b2, *ln2g, *ln2b;
} layer_w;

static const float* carve_layer(const float* p, int H, int F, layer_w* w)
{
    size_t HH = (size_t)H * H, HF = (size_t)H * F;
    w->Wq = p; p += HH; w->bq = p; p += H;
    w->Wk = p; p += HH; w->bk = p; p += H;
    w->Wv = p; p += HH; w->bv = p; p += H;
    w->Wo = p; p += HH; w->bo = p; p += H;
    w->ln1g = p; p += H; w->ln1b = p; p += H;
    w->W1 = p; p += HF; w->b1 = p; p += F;
    w->W2 = p; p += HF; w->b2 = p; p += H;
    w->ln2g = p; p += H; w->ln2b = p; p += H;
    return p;
}

/* optional per-layer taps, each may be NULL: qkv [L][3H], att [L][H],
 * x1 [L][H], g [L][F], x2 [L][H] */
typedef struct { double *qkv, *att, *x1, *g, *x2; } layer_taps;

static void put_tap(double* dst, const real* src, size_t n) { if (dst) for (size_t i = 0; i < n; ++i) dst[i] = (double)src[i]; }

/* One post-LN transformer encoder layer on one sequence, in place on x[L][H]:
 *   a  = MHA(x Wq + bq, x Wk + bk, x Wv + bv)
 *   x1 = LN(x + a Wo + bo)
 *   x  = LN(x1 + gelu(x1 W1 + b1) W2 + b2)                                   */
static void encoder_layer(real* x, int L, int H, int A, int F, const layer_w* w, real eps, const layer_taps* tp)
{
    size_t LH = (size_t)L * H;
    real* q = (real*)malloc(sizeof(real) * LH);
    real* k = (real*)malloc(sizeof(real) * LH);
    real* v = (real*)malloc(sizeof(real) * LH);
    real* a = (real*)malloc(sizeof(real) * LH);
    real* y = (real*)malloc(sizeof(real) * LH);
    real* x1 = (real*)malloc(sizeof(real) * LH);
    real* g = (real*)malloc(sizeof(real) * (size_t)L * F);

    linear(x, L, H, H, w->Wq, w->bq, q);
    linear(x, L, H, H, w->Wk, w->bk, k);
    linear(x, L, H, H, w->Wv, w->bv, v);
    if (tp && tp->qkv)
        for (int t = 0; t < L; ++t) {
            put_tap(tp->qkv + (size_t)t * 3 * H, q + (size_t)t * H, H);
            put_tap(tp->qkv + (size_t)t * 3 * H + H, k + (size_t)t * H, H);
            put_tap(tp->qkv + (size_t)t * 3 * H + 2 * H, v + (size_t)t * H, H);
        }
    attention(q, k, v, L, A, H / A, a, NULL);
    if (tp) put_tap(tp->att, a, LH);

    linear(a, L, H, H, w->Wo, w->bo, y);
    for (size_t i = 0; i < LH; ++i) y[i] += x[i];
    for (int t = 0; t < L; ++t) layernorm_row(y + (size_t)t * H, w->ln1g, w->ln1b, H, eps, x1 + (size_t)t * H);
    if (tp) put_tap(tp->x1, x1, LH);

    linear(x1, L, H, F, w->W1, w->b1, g);
    for (size_t i = 0; i < (size_t)L * F; ++i) g[i] = gelu(g[i]);
    if (tp) put_tap(tp->g, g, (size_t)L * F);
    linear(g, L, F, H, w->W2, w->b2, y);
    for (size_t i = 0; i < LH; ++i) y[i] += x1[i];
    for (int t = 0; t < L; ++t) layernorm_row(y + (size_t)t * H, w->ln2g, w->ln2b, H, eps, x + (size_t)t * H);
    if (tp) put_tap(tp->x2, x, LH);

    free(q); free(k); free(v); free(a); free(y); free(x1); free(g);
}

/* Student m on one sequence: returns z[C] (its classifier output) and, when
 * asked, the pooled vector p[H] and the taps (x0 [L][H]; per layer l the
 * buffers at taps[l]). */
static void student_sequence(const spo_config* c, const float* sw, const int32_t* ids, int L,
                             real* z, real* pooled_out, double* x0_tap, const layer_taps* taps)
{
    int H = c->hidden, F = c->ffn, C = c->classes;
    const float* tok = sw;
    const float* pos = tok + (size_t)c->vocab * H;
    const float* eg = pos + (size_t)c->max_pos * H;
    const float* eb = eg + H;
    const float* p = eb + H;
    real eps = (real)c->ln_eps;

    real* x = (real*)malloc(sizeof(real) * (size_t)L * H);
    real* u = (real*)malloc(sizeof(real) * (size_t)H);
    for (int i = 0; i < L; ++i) {
        const float* te = tok + (size_t)ids[i] * H;
        const float* pe = pos + (size_t)i * H;       /* position of a token = its index inside its own sequence */
        for (int e = 0; e < H; ++e) u[e] = (real)te[e] + (real)pe[e];
        layernorm_row(u, eg, eb, H, eps, x + (size_t)i * H);
    }
    put_tap(x0_tap, x, (size_t)L * H);

    for (int l = 0; l < c->layers; ++l) {
        layer_w w;
        p = carve_layer(p, H, F, &w);
        encoder_layer(x, L, H, c->heads, F, &w, eps, taps ? &taps[l] : NULL);
    }
    const float* Wp = p; const float* bp = Wp + (size_t)H * H;
    const float* Wc = bp + H; const float* bc = Wc + (size_t)H * C;

    /* pooled = tanh(first-token state . Wp + bp); z = pooled . Wc + bc */
    real* pl = (real*)malloc(sizeof(real) * (size_t)H);
    linear(x, 1, H, H, Wp, bp, pl);
    for (int e = 0; e < H; ++e) pl[e] = R_TANH(pl[e]);
    if (pooled_out) memcpy(pooled_out, pl, sizeof(real) * (size_t)H);
    linear(pl, 1, H, C, Wc, bc, z);
    free(pl); free(u); free(x);
}

static int check_inputs(const spo_config* c, const int32_t* ids, const int32_t* cu, int32_t B, int32_t k_active)
{
    if (!c || !ids || !cu || B < 1) return -1;
    if (k_active < 1 || k_active > c->K) return -2;
    if (c->hidden % c->heads) return -3;
    if (cu[0] != 0) return -4;
    for (int32_t b = 0; b < B; ++b) {
        int32_t L = cu[b + 1] - cu[b];
        if (L < 1 || L > c->max_pos) return -4;
    }
    for (int32_t t = 0; t < cu[B]; ++t) if (ids[t] < 0 || ids[t] >= c->vocab) return -5;
    return 0;
}

/* The whole forward.  logits[B][C] = sum over m = 0..k_active-1 (ascending)
 * of student m's output for that sequence.  z_all (optional) receives the
 * separate terms as [k_active][B][C]; pooled_all (optional) the pooled
 * vectors as [k_active][B][H].  Returns 0 or a negative argument error. */
int spo_forward(const spo_config* c, const float* blob, const int32_t* ids, const int32_t* cu,
                int32_t B, int32_t k_active, double* logits, double* z_all, double* pooled_all)
{
    int rc = check_inputs(c, ids, cu, B, k_active);
    if (rc) return rc;
    int C = c->classes, H = c->hidden;
    size_t sf = student_floats(c);
    real* z = (real*)malloc(sizeof(real) * (size_t)k_active * B * C);
    real* pl = pooled_all ? (real*)malloc(sizeof(real) * (size_t)k_active * B * H) : NULL;

    #pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int32_t m = 0; m < k_active; ++m)
        for (int32_t b = 0; b < B; ++b)
            student_sequence(c, blob + (size_t)m * sf, ids + cu[b], cu[b + 1] - cu[b],
                             z + ((size_t)m * B + b) * C, pl ? pl + ((size_t)m * B + b) * H : NULL, NULL, NULL);

    for (int32_t b = 0; b < B; ++b)
        for (int cc = 0; cc < C; ++cc) {
            real acc = 0;
            for (int32_t m = 0; m < k_active; ++m) acc += z[((size_t)m * B + b) * C + cc];
            logits[(size_t)b * C + cc] = (double)acc;
        }
    if (z_all) for (size_t i = 0; i < (size_t)k_active * B * C; ++i) z_all[i] = (double)z[i];
    if (pooled_all) for (size_t i = 0; i < (size_t)k_active * B * H; ++i) pooled_all[i] = (double)pl[i];
    free(z); free(pl);
    return 0;
}

/* Intermediate activations of student m on sequence b, for kernel-by-kernel
 * comparison.  x0 [L][H]; qkv [Ly][L][3H]; att, x1, x2 [Ly][L][H]; g [Ly][L][F];
 * z [C].  Any output pointer may be NULL. */
int spo_forward_taps(const spo_config* c, const float* blob, const int32_t* ids, const int32_t* cu,
                     int32_t B, int32_t m, int32_t b, double* x0, double* qkv, double* att,
                     double* x1, double* g, double* x2, double* z_out)
{
    int rc = check_inputs(c, ids, cu, B, 1);
    if (rc) return rc;
    if (m < 0 || m >= c->K || b < 0 || b >= B) return -2;
    int L = cu[b + 1] - cu[b], H = c->hidden, F = c->ffn;
    layer_taps* tp = (layer_taps*)calloc((size_t)c->layers, sizeof(layer_taps));
    for (int l = 0; l < c->layers; ++l) {
        tp[l].qkv = qkv ? qkv + (size_t)l * L * 3 * H : NULL;
        tp[l].att = att ? att + (size_t)l * L * H : NULL;
        tp[l].x1 = x1 ? x1 + (size_t)l * L * H : NULL;
        tp[l].g = g ? g + (size_t)l * L * F : NULL;
        tp[l].x2 = x2 ? x2 + (size_t)l * L * H : NULL;
    }
    real* z = (real*)malloc(sizeof(real) * (size_t)c->classes);
    student_sequence(c, blob + (size_t)m * student_floats(c), ids + cu[b], L, z, NULL, x0, tp);
    if (z_out) for (int i = 0; i < c->classes; ++i) z_out[i] = (double)z[i];
    free(z); free(tp);
    return 0;
}

/* ---- double-typed doors to the elementary pieces (for the pins) ---------- */

void spo_layernorm(const double* u, const float* g, const float* b, int n, double eps, double* out)
{
    real* ur = (real*)malloc(sizeof(real) * (size_t)n);
    real* orr = (real*)malloc(sizeof(real) * (size_t)n);
    for (int i = 0; i < n; ++i) ur[i] = (real)u[i];
    layernorm_row(ur, g, b, n, (real)eps, orr);
    for (int i = 0; i < n; ++i) out[i] = (double)orr[i];
    free(ur); free(orr);
}

double spo_gelu(double u) { return (double)gelu((real)u); }

void spo_softmax(double* s, int n)
{
    real* r = (real*)malloc(sizeof(real) * (size_t)n);
    for (int i = 0; i < n; ++i) r[i] = (real)s[i];
    softmax_row(r, n);
    for (int i = 0; i < n; ++i) s[i] = (double)r[i];
    free(r);
}

void spo_linear(const double* x, int L, int in, int out, const float* W, const float* b, double* y)
{
    real* xr = (real*)malloc(sizeof(real) * (size_t)L * in);
    real* yr = (real*)malloc(sizeof(real) * (size_t)L * out);
    for (size_t i = 0; i < (size_t)L * in; ++i) xr[i] = (real)x[i];
    linear(xr, L, in, out, W, b, yr);
    for (size_t i = 0; i < (size_t)L * out; ++i) y[i] = (double)yr[i];
    free(xr); free(yr);
}

/* q, k, v, o: [L][A*d]; probs (optional): [A][L][L] */
void spo_attention(const double* q, const double* k, const double* v, int L, int A, int d, double* o, double* probs)
{
    size_t n = (size_t)L * A * d, np = (size_t)A * L * L;
    real* qr = (real*)malloc(sizeof(real) * n); real* kr = (real*)malloc(sizeof(real) * n);
    real* vr = (real*)malloc(sizeof(real) * n); real* orr = (real*)malloc(sizeof(real) * n);
    real* pr = probs ? (real*)malloc(sizeof(real) * np) : NULL;
    for (size_t i = 0; i < n; ++i) { qr[i] = (real)q[i]; kr[i] = (real)k[i]; vr[i] = (real)v[i]; }
    attention(qr, kr, vr, L, A, d, orr, pr);
    for (size_t i = 0; i < n; ++i) o[i] = (double)orr[i];
    if (probs) for (size_t i = 0; i < np; ++i) probs[i] = (double)pr[i];
    free(qr); free(kr); free(vr); free(orr); free(pr);
}

/* one encoder layer on one sequence; lw points at the layer's slice of a blob
 * (Wq .. ln2_b, layout above); x [L][H] in, out [L][H]. */
void spo_encoder_layer(const double* x, int L, int H, int A, int F, const float* lw, double eps, double* out)
{
    layer_w w;
    carve_layer(lw, H, F, &w);
    real* xr = (real*)malloc(sizeof(real) * (size_t)L * H);
    for (size_t i = 0; i < (size_t)L * H; ++i) xr[i] = (real)x[i];
    encoder_layer(xr, L, H, A, F, &w, (real)eps, NULL);
    for (size_t i = 0; i < (size_t)L * H; ++i) out[i] = (double)xr[i];
    free(xr);
}
