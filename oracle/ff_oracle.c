/*
 * CPU oracle for one Llama-style decoder step (TEST INFRASTRUCTURE, not a product path).
 *
 * This is the plain definition of what the whole-model decode kernel computes: the six matrix
 * operations per layer of the paper's sublayer table (Section 2.1: QKV projection, QK^T, PV,
 * attention output projection, GLU in/gate projection, GLU output projection) with pre-RMSNorm,
 * RoPE, grouped-query attention and SwiGLU, followed by the final norm and LM head.  The fused
 * kernel re-associates these sums (split-KV attention with an online-softmax merge, Section 4.2)
 * but reaches exactly this result up to rounding order, so nothing here is blocked, fused or
 * split: every sum is a plain loop.
 *
 * Arithmetic: every activation and accumulator is fp64.  Parameters are the stored values widened
 * exactly (bf16, or dequantised int8/int4 codes).  The only rounding is where the model itself
 * stores a value: keys and values go into the cache as bf16 (round-to-nearest-even), and the
 * current token attends to its own *stored* key/value.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may load this library.
 * It shares no code with the HIP path.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define FFO_W_BF16 0
#define FFO_W_INT8 1
#define FFO_W_INT4 2
#define FFO_GROUP 128

/* ---------- scalar formats ---------- */

double ffo_bf16_to_f64(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* IEEE binary16 -> double, written out from the format definition */
double ffo_f16_to_f64(uint16_t h) {
    int sign = (h >> 15) & 1, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 0) v = ldexp((double)m, -24);
    else if (e == 31) v = m ? NAN : INFINITY;
    else v = ldexp((double)(m + 1024), e - 25);
    return sign ? -v : v;
}

/* double -> bf16, one rounding, round-to-nearest-even (finite inputs) */
uint16_t ffo_f64_to_bf16(double x) {
    if (x == 0.0 || !isfinite(x)) {
        float f = (float)x;
        uint32_t u;
        memcpy(&u, &f, 4);
        return (uint16_t)(u >> 16);
    }
    int e;
    double m = frexp(fabs(x), &e);         /* |x| = m * 2^e, m in [0.5, 1) */
    int q = e - 8;                         /* bf16 has 8 significant bits: ulp = 2^(e-8) */
    if (q < -133) q = -133;                /* subnormal range: smallest step 2^-133 */
    double t = ldexp(fabs(x), -q);
    double r = nearbyint(t);               /* default rounding mode: ties to even */
    (void)m;
    float f = (float)ldexp(r, q);          /* exactly representable in fp32 */
    if (x < 0) f = -f;
    uint32_t u;
    memcpy(&u, &f, 4);
    return (uint16_t)(u >> 16);
}

/* ---------- weight-only quantisation formats ---------- */

/* int8 per-output-channel: w[n][k] = q[n][k] * s[n] */
double ffo_dequant_int8(int8_t q, uint16_t s_f16) { return (double)q * ffo_f16_to_f64(s_f16); }

/* int4 group-128 along K: w[n][k] = (code - z[n][k/128]) * s[n][k/128]; two codes per byte,
 * low nibble holds the even k. */
double ffo_dequant_int4(const uint8_t *row_packed, int k, uint16_t s_f16, uint16_t z_f16) {
    uint8_t b = row_packed[k >> 1];
    int code = (k & 1) ? (b >> 4) : (b & 15);
    return ((double)code - ffo_f16_to_f64(z_f16)) * ffo_f16_to_f64(s_f16);
}

typedef struct {
    int32_t wdtype; /* FFO_W_* */
    int32_t n, k;   /* rows (outputs), columns (inputs); row-major [n][k] */
    const void *w;
    const uint16_t *s; /* fp16 scales: [n] (int8) or [n][k/128] (int4) */
    const uint16_t *z; /* fp16 zeros [n][k/128] (int4) */
} ffo_mat;

double ffo_mat_at(const ffo_mat *m, int r, int c) {
    if (m->wdtype == FFO_W_BF16) return ffo_bf16_to_f64(((const uint16_t *)m->w)[(size_t)r * m->k + c]);
    if (m->wdtype == FFO_W_INT8)
        return ffo_dequant_int8(((const int8_t *)m->w)[(size_t)r * m->k + c], m->s[r]);
    int g = m->k / FFO_GROUP;
    return ffo_dequant_int4((const uint8_t *)m->w + (size_t)r * (m->k / 2), c, m->s[(size_t)r * g + c / FFO_GROUP],
                            m->z[(size_t)r * g + c / FFO_GROUP]);
}

/* dequantised matrix as fp32 (the products are exact in fp32), for bit-exact comparison */
void ffo_dequant_matrix(const ffo_mat *m, float *out) {
    for (int r = 0; r < m->n; r++)
        for (int c = 0; c < m->k; c++) out[(size_t)r * m->k + c] = (float)ffo_mat_at(m, r, c);
}

/* y = W x */
void ffo_matvec(const ffo_mat *m, const double *x, double *y) {
#pragma omp parallel for schedule(static)
    for (int r = 0; r < m->n; r++) {
        double acc = 0.0;
        for (int c = 0; c < m->k; c++) acc += ffo_mat_at(m, r, c) * x[c];
        y[r] = acc;
    }
}

/* ---------- pointwise pieces ---------- */

/* RMSNorm with a gain: y_i = x_i / sqrt(mean(x^2) + eps) * g_i */
void ffo_rmsnorm(const double *x, const uint16_t *gain_bf16, int d, double eps, double *y) {
    double ss = 0.0;
    for (int i = 0; i < d; i++) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / d + eps);
    for (int i = 0; i < d; i++) y[i] = x[i] * r * ffo_bf16_to_f64(gain_bf16[i]);
}

/* Rotary embedding of one head vector at position pos, rotate-half pairing: element i is
 * paired with i + hd/2 and the pair is rotated by pos * theta^(-2i/hd) radians. */
void ffo_rope(double *v, int hd, int pos, double theta) {
    int half = hd / 2;
    for (int i = 0; i < half; i++) {
        double ang = (double)pos * pow(theta, -2.0 * i / hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

double ffo_silu(double z) { return z / (1.0 + exp(-z)); }

/* Core attention for ONE query head over n_keys cached rows: softmax(alpha * q K^T) V with the
 * full score row materialised.  K and V are bf16 rows with a row stride (in elements).  If probs
 * is non-NULL the softmax row is written there. */
void ffo_attention_head(const double *q, const uint16_t *K, const uint16_t *V, int n_keys, int hd,
                        size_t row_stride, double alpha, double *o, double *probs) {
    double *s = (double *)malloc(sizeof(double) * (size_t)(n_keys > 0 ? n_keys : 1));
    double mx = -INFINITY;
    for (int i = 0; i < n_keys; i++) {
        double acc = 0.0;
        for (int e = 0; e < hd; e++) acc += q[e] * ffo_bf16_to_f64(K[i * row_stride + e]);
        s[i] = alpha * acc;
        if (s[i] > mx) mx = s[i];
    }
    double den = 0.0;
    for (int i = 0; i < n_keys; i++) {
        s[i] = exp(s[i] - mx);
        den += s[i];
    }
    for (int e = 0; e < hd; e++) o[e] = 0.0;
    for (int i = 0; i < n_keys; i++) {
        double p = s[i] / den;
        if (probs) probs[i] = p;
        for (int e = 0; e < hd; e++) o[e] += p * ffo_bf16_to_f64(V[i * row_stride + e]);
    }
    free(s);
}

/* ---------- the decoder ---------- */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    double rms_eps, rope_theta;
} ffo_config;

typedef struct {
    const uint16_t *attn_norm, *ffn_norm; /* bf16 [d_model] */
    ffo_mat wq, wk, wv, wo, w_gate, w_up, w_down;
} ffo_layer;

typedef struct {
    const uint16_t *embed;      /* bf16 [vocab][d_model] */
    const uint16_t *final_norm; /* bf16 [d_model] */
    ffo_mat lm_head;
} ffo_head;

/* One layer for one sequence.  x (fp64 [d_model]) is updated in place.  Kc/Vc are this layer's
 * cache for this sequence, bf16 [max_ctx][n_kv_heads][head_dim]; rows 0..pos-1 are valid on entry
 * and row pos is written here.  The current token attends to rows 0..pos inclusive. */
void ffo_layer_step(const ffo_config *c, const ffo_layer *L, double *x, uint16_t *Kc, uint16_t *Vc, int pos) {
    int d = c->d_model, hd = c->head_dim, Hq = c->n_q_heads, Hkv = c->n_kv_heads, F = c->d_ffn;
    int G = Hq / Hkv;
    size_t row = (size_t)Hkv * hd;
    double *n = malloc(sizeof(double) * d), *q = malloc(sizeof(double) * Hq * hd);
    double *k = malloc(sizeof(double) * row), *v = malloc(sizeof(double) * row);
    double *o = malloc(sizeof(double) * Hq * hd), *a = malloc(sizeof(double) * d);
    double *g = malloc(sizeof(double) * F), *u = malloc(sizeof(double) * F);

    ffo_rmsnorm(x, L->attn_norm, d, c->rms_eps, n);
    ffo_matvec(&L->wq, n, q);
    ffo_matvec(&L->wk, n, k);
    ffo_matvec(&L->wv, n, v);
    for (int h = 0; h < Hq; h++) ffo_rope(q + h * hd, hd, pos, c->rope_theta);
    for (int j = 0; j < Hkv; j++) ffo_rope(k + j * hd, hd, pos, c->rope_theta);
    for (size_t i = 0; i < row; i++) {
        Kc[(size_t)pos * row + i] = ffo_f64_to_bf16(k[i]);
        Vc[(size_t)pos * row + i] = ffo_f64_to_bf16(v[i]);
    }
    double alpha = 1.0 / sqrt((double)hd);
#pragma omp parallel for schedule(static)
    for (int h = 0; h < Hq; h++) {
        int j = h / G;
        ffo_attention_head(q + h * hd, Kc + j * hd, Vc + j * hd, pos + 1, hd, row, alpha, o + h * hd, NULL);
    }
    ffo_matvec(&L->wo, o, a);
    for (int i = 0; i < d; i++) x[i] += a[i];

    ffo_rmsnorm(x, L->ffn_norm, d, c->rms_eps, n);
    ffo_matvec(&L->w_gate, n, g);
    ffo_matvec(&L->w_up, n, u);
    for (int i = 0; i < F; i++) g[i] = ffo_silu(g[i]) * u[i];
    ffo_matvec(&L->w_down, g, a);
    for (int i = 0; i < d; i++) x[i] += a[i];

    free(n); free(q); free(k); free(v); free(o); free(a); free(g); free(u);
}

void ffo_embed(const ffo_config *c, const ffo_head *H, int token, double *x) {
    for (int i = 0; i < c->d_model; i++) x[i] = ffo_bf16_to_f64(H->embed[(size_t)token * c->d_model + i]);
}

void ffo_logits(const ffo_config *c, const ffo_head *H, const double *x, double *logits) {
    double *n = malloc(sizeof(double) * c->d_model);
    ffo_rmsnorm(x, H->final_norm, c->d_model, c->rms_eps, n);
    ffo_matvec(&H->lm_head, n, logits);
    free(n);
}

/* Whole step for a batch of independent sequences.  kv holds, for layer l and sequence b,
 * K at kv + ((l*batch + b)*2 + 0)*max_ctx*row and V at (...*2 + 1)*..., bf16. */
void ffo_decode_step(const ffo_config *c, const ffo_layer *layers, const ffo_head *H, const int32_t *tokens,
                     const int32_t *positions, int batch, uint16_t *kv, int max_ctx, double *logits) {
    size_t row = (size_t)c->n_kv_heads * c->head_dim;
    size_t plane = (size_t)max_ctx * row;
    double *x = malloc(sizeof(double) * c->d_model);
    for (int b = 0; b < batch; b++) {
        ffo_embed(c, H, tokens[b], x);
        for (int l = 0; l < c->n_layers; l++) {
            uint16_t *Kc = kv + ((size_t)(l * batch + b) * 2) * plane;
            ffo_layer_step(c, &layers[l], x, Kc, Kc + plane, positions[b]);
        }
        ffo_logits(c, H, x, logits + (size_t)b * c->vocab);
    }
    free(x);
}

int ffo_sizeof_layer(void) { return (int)sizeof(ffo_layer); }
int ffo_sizeof_mat(void) { return (int)sizeof(ffo_mat); }
