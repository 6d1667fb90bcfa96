/* CPU oracle: transformer forward with a KV cache, in double precision.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU library is checked
 * against; nothing in the product path may call it.  It shares no code with the HIP sources.
 *
 * What it computes.  The paper (Sec. II-A, Eq. 1-3; Alg. 1 Stage B; Sec. III-C) fixes the speculative
 * loop but only *names* the network ("LLaMA-2 family").  The forward pass below is therefore the textbook
 * pre-norm LLaMA block -- RMSNorm, rotary position embedding on q and k (rotate-half pairing), causal
 * soft-max attention with grouped KV heads, SwiGLU feed-forward, residual adds, final RMSNorm and an
 * untied output projection -- written operation by operation with no blocking or fusion.  The draft model
 * of Alg. 1 ("remove the layers in the prune set", Stage A last line; Sec. III-C "architecture-compatible
 * ... KV reuse") is this same forward with a per-layer skip mask: a skipped sub-layer leaves the residual
 * stream untouched and writes no KV entry.
 *
 * Precision.  Weight matrices and KV-cache entries are *stored* in the model's storage type (float32, or
 * bfloat16 with round-to-nearest-even); every other quantity, and every accumulation, is double.  Sums run
 * in ascending index order.
 *
 * Parity pins (tests/test_oracle_*.py): an independent PyTorch-CPU LLaMA forward on the tiny config;
 * cached forward == full recompute; row i of a multi-row forward == one-row decode of the same prefix;
 * RoPE norm/relative-position invariants; RMSNorm unit RMS; soft-max closed forms.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, max_seq;
    int32_t dtype; /* 0 = float32, 1 = bfloat16 : storage of weight matrices and of the KV cache */
    double rms_eps, rope_theta;
} orc_config;

enum { W_ATTN_NORM, W_Q, W_K, W_V, W_O, W_FFN_NORM, W_GATE, W_UP, W_DOWN, W_PER_LAYER };

typedef struct {
    orc_config c;
    const void *tok_emb, *lm_head;
    const float *final_norm;
    const void **lw;      /* [L][W_PER_LAYER] borrowed host pointers */
    float *kc, *vc;       /* [L][max_seq][H_kv*hd], values already rounded to the storage type */
} orc_model;

/* ---- storage-type helpers ---------------------------------------------------------------------------- */
static inline double load_w(const void *w, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float *)w)[i];
    uint32_t u = (uint32_t)((const uint16_t *)w)[i] << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* value as it reads back after being written to a cache of the storage type */
float orc_round_storage(double v, int dtype) {
    float f = (float)v;
    if (dtype == 0) return f;
    uint32_t u;
    memcpy(&u, &f, 4);
    u = (u + 0x7FFFu + ((u >> 16) & 1u)) & 0xFFFF0000u; /* bf16 round-to-nearest-even */
    memcpy(&f, &u, 4);
    return f;
}

/* ---- primitives (exported so tests can pin each one) -------------------------------------------------- */

/* out = h * g / sqrt(mean(h^2) + eps) */
void orc_rmsnorm(const double *h, const float *g, int d, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += h[i] * h[i];
    double r = 1.0 / sqrt(ss / (double)d + eps);
    for (int i = 0; i < d; ++i) out[i] = h[i] * r * (double)g[i];
}

/* Y[m][n] = sum_k W[n][k] * X[m][k];  W row-major [N][Kd] in storage type, X,Y double row-major */
void orc_matmul(const void *W, int dtype, int N, int Kd, const double *X, int M, double *Y) {
    /* X transposed once so the m-loop is contiguous; each Y[m][n] is still a plain ascending-k sum */
    double *XT = (double *)malloc(sizeof(double) * (size_t)Kd * (size_t)M);
    for (int m = 0; m < M; ++m)
        for (int k = 0; k < Kd; ++k) XT[(size_t)k * M + m] = X[(size_t)m * Kd + k];
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)Kd);
        double *acc = (double *)malloc(sizeof(double) * (size_t)M);
#pragma omp for schedule(static)
        for (int n = 0; n < N; ++n) {
            for (int k = 0; k < Kd; ++k) wrow[k] = load_w(W, dtype, (size_t)n * Kd + k);
            for (int m = 0; m < M; ++m) acc[m] = 0.0;
            for (int k = 0; k < Kd; ++k) {
                const double w = wrow[k];
                const double *xt = XT + (size_t)k * M;
                for (int m = 0; m < M; ++m) acc[m] += w * xt[m];
            }
            for (int m = 0; m < M; ++m) Y[(size_t)m * N + n] = acc[m];
        }
        free(wrow);
        free(acc);
    }
    free(XT);
}

/* rotary embedding of one head vector at position pos: pairs (i, i + hd/2), angle = pos * theta^(-2i/hd) */
void orc_rope(double *v, int hd, int pos, double theta) {
    int half = hd / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)hd);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

/* one query head over cache positions 0..n_pos-1 of one KV head.
 * kc, vc point at position 0 of that KV head; consecutive positions are `stride` floats apart. */
void orc_attend(const double *q, const float *kc, const float *vc, int n_pos, int hd, size_t stride, double *out) {
    double *p = (double *)malloc(sizeof(double) * (size_t)n_pos);
    double scale = 1.0 / sqrt((double)hd), mx = -INFINITY, den = 0.0;
    for (int j = 0; j < n_pos; ++j) {
        double s = 0.0;
        for (int i = 0; i < hd; ++i) s += q[i] * (double)kc[(size_t)j * stride + i];
        p[j] = s * scale;
        if (p[j] > mx) mx = p[j];
    }
    for (int j = 0; j < n_pos; ++j) {
        p[j] = exp(p[j] - mx);
        den += p[j];
    }
    for (int i = 0; i < hd; ++i) out[i] = 0.0;
    for (int j = 0; j < n_pos; ++j) {
        double w = p[j] / den;
        for (int i = 0; i < hd; ++i) out[i] += w * (double)vc[(size_t)j * stride + i];
    }
    free(p);
}

double orc_silu(double z) { return z / (1.0 + exp(-z)); }

/* ---- model ------------------------------------------------------------------------------------------- */

/* wtable: [tok_emb, final_norm, lm_head, then per layer the W_PER_LAYER tensors in enum order].
 * Matrices are row-major [out_features][in_features] in the storage type; norm gains are float32. */
orc_model *orc_create(const orc_config *c, const void *const *wtable) {
    if (!c || !wtable) return NULL;
    if (c->n_layers < 1 || c->d_model < 1 || c->n_heads < 1 || c->n_kv_heads < 1 || c->head_dim < 2 ||
        (c->head_dim & 1) || c->d_ffn < 1 || c->vocab < 1 || c->max_seq < 1 || (c->dtype != 0 && c->dtype != 1) ||
        c->n_heads % c->n_kv_heads != 0)
        return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->c = *c;
    m->tok_emb = wtable[0];
    m->final_norm = (const float *)wtable[1];
    m->lm_head = wtable[2];
    size_t nl = (size_t)c->n_layers * W_PER_LAYER;
    m->lw = (const void **)malloc(sizeof(void *) * nl);
    for (size_t i = 0; i < nl; ++i) m->lw[i] = wtable[3 + i];
    size_t kvn = (size_t)c->n_layers * c->max_seq * c->n_kv_heads * c->head_dim;
    m->kc = (float *)calloc(kvn, sizeof(float));
    m->vc = (float *)calloc(kvn, sizeof(float));
    if (!m->kc || !m->vc) {
        free(m->kc); free(m->vc); free(m->lw); free(m);
        return NULL;
    }
    return m;
}

void orc_destroy(orc_model *m) {
    if (!m) return;
    free(m->kc); free(m->vc); free(m->lw); free(m);
}

float *orc_kcache(orc_model *m) { return m->kc; }
float *orc_vcache(orc_model *m) { return m->vc; }

/* Forward of M rows: tokens[m] sits at position pos0+m; row m attends to cache positions 0..pos0+m.
 * skip: NULL (full model) or uint8[L] with bit0 = skip attention sub-layer, bit1 = skip FFN sub-layer.
 * Writes K/V at pos0..pos0+M-1 for every layer whose attention sub-layer runs.
 * logits: rows logits_from..M-1 are written to logits[(m-logits_from)*V + v].
 * hidden (optional, may be NULL): final residual stream [M][d] before the last norm.
 * Returns 0, or -1 on bad arguments. */
int orc_forward(orc_model *mdl, const int32_t *tokens, int M, int pos0, const uint8_t *skip, int logits_from,
                double *logits, double *hidden) {
    if (!mdl || !tokens || M < 1 || pos0 < 0 || pos0 + M > mdl->c.max_seq || logits_from < 0 || logits_from > M)
        return -1;
    const orc_config *c = &mdl->c;
    const int d = c->d_model, H = c->n_heads, Hk = c->n_kv_heads, hd = c->head_dim, F = c->d_ffn, V = c->vocab;
    const int dq = H * hd, dkv = Hk * hd, grp = H / Hk, dt = c->dtype;
    for (int m = 0; m < M; ++m)
        if (tokens[m] < 0 || tokens[m] >= V) return -1;

    double *h = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *xn = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)M * dq);
    double *k = (double *)malloc(sizeof(double) * (size_t)M * dkv);
    double *v = (double *)malloc(sizeof(double) * (size_t)M * dkv);
    double *att = (double *)malloc(sizeof(double) * (size_t)M * dq);
    double *proj = (double *)malloc(sizeof(double) * (size_t)M * d);
    double *g = (double *)malloc(sizeof(double) * (size_t)M * F);
    double *u = (double *)malloc(sizeof(double) * (size_t)M * F);

    for (int m = 0; m < M; ++m)
        for (int i = 0; i < d; ++i) h[(size_t)m * d + i] = load_w(mdl->tok_emb, dt, (size_t)tokens[m] * d + i);

    for (int l = 0; l < c->n_layers; ++l) {
        const void **w = mdl->lw + (size_t)l * W_PER_LAYER;
        const int sk = skip ? skip[l] : 0;
        if (!(sk & 1)) { /* attention sub-layer: h += W_o * Attn(RoPE(W_q x), RoPE(W_k x), W_v x) */
            for (int m = 0; m < M; ++m)
                orc_rmsnorm(h + (size_t)m * d, (const float *)w[W_ATTN_NORM], d, c->rms_eps, xn + (size_t)m * d);
            orc_matmul(w[W_Q], dt, dq, d, xn, M, q);
            orc_matmul(w[W_K], dt, dkv, d, xn, M, k);
            orc_matmul(w[W_V], dt, dkv, d, xn, M, v);
            float *kcl = mdl->kc + (size_t)l * c->max_seq * dkv;
            float *vcl = mdl->vc + (size_t)l * c->max_seq * dkv;
            for (int m = 0; m < M; ++m) {
                int pos = pos0 + m;
                for (int hh = 0; hh < H; ++hh) orc_rope(q + (size_t)m * dq + (size_t)hh * hd, hd, pos, c->rope_theta);
                for (int hh = 0; hh < Hk; ++hh) orc_rope(k + (size_t)m * dkv + (size_t)hh * hd, hd, pos, c->rope_theta);
                for (int i = 0; i < dkv; ++i) {
                    kcl[(size_t)pos * dkv + i] = orc_round_storage(k[(size_t)m * dkv + i], dt);
                    vcl[(size_t)pos * dkv + i] = orc_round_storage(v[(size_t)m * dkv + i], dt);
                }
            }
#pragma omp parallel for collapse(2) schedule(dynamic)
            for (int m = 0; m < M; ++m)
                for (int hh = 0; hh < H; ++hh) {
                    int kvh = hh / grp;
                    orc_attend(q + (size_t)m * dq + (size_t)hh * hd, kcl + (size_t)kvh * hd, vcl + (size_t)kvh * hd,
                               pos0 + m + 1, hd, (size_t)dkv, att + (size_t)m * dq + (size_t)hh * hd);
                }
            orc_matmul(w[W_O], dt, d, dq, att, M, proj);
            for (size_t i = 0; i < (size_t)M * d; ++i) h[i] += proj[i];
        }
        if (!(sk & 2)) { /* feed-forward sub-layer: h += W_down * (silu(W_gate x) * (W_up x)) */
            for (int m = 0; m < M; ++m)
                orc_rmsnorm(h + (size_t)m * d, (const float *)w[W_FFN_NORM], d, c->rms_eps, xn + (size_t)m * d);
            orc_matmul(w[W_GATE], dt, F, d, xn, M, g);
            orc_matmul(w[W_UP], dt, F, d, xn, M, u);
            for (size_t i = 0; i < (size_t)M * F; ++i) g[i] = orc_silu(g[i]) * u[i];
            orc_matmul(w[W_DOWN], dt, d, F, g, M, proj);
            for (size_t i = 0; i < (size_t)M * d; ++i) h[i] += proj[i];
        }
    }
    if (hidden) memcpy(hidden, h, sizeof(double) * (size_t)M * d);
    int nrows = M - logits_from;
    if (nrows > 0 && logits) {
        for (int m = logits_from; m < M; ++m)
            orc_rmsnorm(h + (size_t)m * d, mdl->final_norm, d, c->rms_eps, xn + (size_t)(m - logits_from) * d);
        orc_matmul(mdl->lm_head, dt, V, d, xn, nrows, logits);
    }
    free(h); free(xn); free(q); free(k); free(v); free(att); free(proj); free(g); free(u);
    return 0;
}
