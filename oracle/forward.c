/*
 * CPU oracle: layer-masked forward pass of a LLaMA-style decoder with a KV cache.
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain definition that the
 * HIP path is checked against. Nothing on the product path may call it, and it
 * shares no code, header, table or helper with the HIP sources.
 *
 * What it computes (paper Sec. 3.1 and Sec. 4.2): the model M has
 * L = 2*n_blocks sublayers (attention and MLP counted separately); a mask
 * z in {0,1}^L marks the sublayers the draft model M(z) skips (z=1: the
 * sublayer is the identity on the residual stream). The full model is z = 0.
 * A KV cache is kept (App. C.1, experimental setup).
 *
 * Arithmetic: everything is double precision. The only roundings are the ones
 * that are part of the data the two sides exchange: weights arrive already in
 * their storage type (fp32 or bf16), keys and values are rounded to the
 * cache's storage type when they are written, and logits are rounded to fp32
 * when they are returned (the token decision is taken on fp32 logits).
 *
 * Layout: every matrix is row-major [out_features][in_features].
 * Mask layout: mask[2b] = skip attention of block b, mask[2b+1] = skip its MLP.
 * RoPE: rotate-half pairing (i, i + head_dim/2), angle pos * base^(-2i/head_dim).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_blocks, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab, max_seq;
    double rope_base, rms_eps;
    int32_t weight_dtype; /* 0 = fp32, 1 = bf16 (bit patterns in uint16) */
    int32_t kv_dtype;     /* 0 = fp32, 1 = bf16 */
} orc_cfg;

typedef struct {
    orc_cfg cfg;
    const void *embed, *lm_head;
    const float *final_norm;
    const float **attn_norm, **mlp_norm;
    const void **wq, **wk, **wv, **wo, **wg, **wu, **wd;
    /* caches hold values already rounded to kv_dtype: [n_blocks][max_seq][n_kv_heads*head_dim] */
    float *kcache, *vcache;
} orc_model;

static double bf16_bits_to_double(uint16_t b) {
    uint32_t u = ((uint32_t)b) << 16;
    float f;
    memcpy(&f, &u, 4);
    return (double)f;
}

/* round-to-nearest-even of a double to bf16, returned as float */
static float round_to_bf16(double x) {
    float f = (float)x; /* first to fp32, the precision a cache writer holds the value in */
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return f; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return f;
}

static double weight_at(const void *w, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float *)w)[i];
    return bf16_bits_to_double(((const uint16_t *)w)[i]);
}

/* Y[r][o] = sum_k W[o][k] * X[r][k]   for r < n, o < N */
static void matmul_rows(const void *W, int dtype, int N, int K, const double *X, int n, double *Y) {
#pragma omp parallel
    {
        double *wrow = (double *)malloc(sizeof(double) * (size_t)K);
#pragma omp for schedule(static)
        for (int o = 0; o < N; ++o) {
            for (int k = 0; k < K; ++k) wrow[k] = weight_at(W, dtype, (size_t)o * K + k);
            for (int r = 0; r < n; ++r) {
                const double *x = X + (size_t)r * K;
                double acc = 0.0;
#pragma omp simd reduction(+ : acc)
                for (int k = 0; k < K; ++k) acc += wrow[k] * x[k];
                Y[(size_t)r * N + o] = acc;
            }
        }
        free(wrow);
    }
}

/* out = x * rsqrt(mean(x^2) + eps) * gain */
static void rmsnorm(const double *x, const float *gain, int d, double eps, double *out) {
    double ss = 0.0;
    for (int i = 0; i < d; ++i) ss += x[i] * x[i];
    double r = 1.0 / sqrt(ss / (double)d + eps);
    for (int i = 0; i < d; ++i) out[i] = x[i] * r * (double)gain[i];
}

static void rope(double *v, int head_dim, int pos, double base) {
    int half = head_dim / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(base, -2.0 * (double)i / (double)head_dim);
        double c = cos(ang), s = sin(ang);
        double a = v[i], b = v[i + half];
        v[i] = a * c - b * s;
        v[i + half] = b * c + a * s;
    }
}

orc_model *orc_create(const orc_cfg *cfg, const void *embed, const void *lm_head, const float *final_norm,
                      const float **attn_norm, const void **wq, const void **wk, const void **wv,
                      const void **wo, const float **mlp_norm, const void **wg, const void **wu,
                      const void **wd) {
    orc_model *m = (orc_model *)calloc(1, sizeof(orc_model));
    m->cfg = *cfg;
    m->embed = embed;
    m->lm_head = lm_head;
    m->final_norm = final_norm;
    int nb = cfg->n_blocks;
#define COPYP(field, type)                                         \
    m->field = (type *)malloc(sizeof(type) * (size_t)(nb ? nb : 1)); \
    for (int b = 0; b < nb; ++b) m->field[b] = field[b];
    COPYP(attn_norm, const float *)
    COPYP(mlp_norm, const float *)
    COPYP(wq, const void *)
    COPYP(wk, const void *)
    COPYP(wv, const void *)
    COPYP(wo, const void *)
    COPYP(wg, const void *)
    COPYP(wu, const void *)
    COPYP(wd, const void *)
#undef COPYP
    size_t n = (size_t)(nb ? nb : 1) * cfg->max_seq * cfg->n_kv_heads * cfg->head_dim;
    m->kcache = (float *)calloc(n, sizeof(float));
    m->vcache = (float *)calloc(n, sizeof(float));
    return m;
}

void orc_destroy(orc_model *m) {
    if (!m) return;
    free(m->attn_norm); free(m->mlp_norm);
    free(m->wq); free(m->wk); free(m->wv); free(m->wo);
    free(m->wg); free(m->wu); free(m->wd);
    free(m->kcache); free(m->vcache);
    free(m);
}

/*
 * Forward n rows: row r carries token tokens[r] at position start + r.
 * mask: 2*n_blocks bytes (NULL = full model). Retained attention sublayers
 * write their keys/values at positions start..start+n-1 of the cache and row r
 * attends to positions 0..start+r.
 * logits_out: [n - logits_from][vocab] fp32 for rows r >= logits_from (NULL: skip the head).
 * hidden_out: [n][d_model] fp32, the final-RMSNorm output of each row (NULL: skip).
 * Returns 0, or -1 on a range error.
 */
int orc_forward(orc_model *m, const int32_t *tokens, int n, int start, const uint8_t *mask,
                int logits_from, float *logits_out, float *hidden_out) {
    const orc_cfg *c = &m->cfg;
    const int d = c->d_model, H = c->n_heads, Hkv = c->n_kv_heads, hd = c->head_dim, F = c->d_ffn;
    const int qd = H * hd, kvd = Hkv * hd, group = H / Hkv;
    if (n <= 0 || start < 0 || start + n > c->max_seq) return -1;
    for (int r = 0; r < n; ++r)
        if (tokens[r] < 0 || tokens[r] >= c->vocab) return -1;

    double *h = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *nrm = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)n * qd);
    double *kk = (double *)malloc(sizeof(double) * (size_t)n * kvd);
    double *vv = (double *)malloc(sizeof(double) * (size_t)n * kvd);
    double *att = (double *)malloc(sizeof(double) * (size_t)n * qd);
    double *proj = (double *)malloc(sizeof(double) * (size_t)n * d);
    double *g = (double *)malloc(sizeof(double) * (size_t)n * F);
    double *u = (double *)malloc(sizeof(double) * (size_t)n * F);

    for (int r = 0; r < n; ++r)
        for (int i = 0; i < d; ++i) h[(size_t)r * d + i] = weight_at(m->embed, c->weight_dtype, (size_t)tokens[r] * d + i);

    for (int b = 0; b < c->n_blocks; ++b) {
        if (!(mask && mask[2 * b])) {
            /* attention sublayer */
            for (int r = 0; r < n; ++r) rmsnorm(h + (size_t)r * d, m->attn_norm[b], d, c->rms_eps, nrm + (size_t)r * d);
            matmul_rows(m->wq[b], c->weight_dtype, qd, d, nrm, n, q);
            matmul_rows(m->wk[b], c->weight_dtype, kvd, d, nrm, n, kk);
            matmul_rows(m->wv[b], c->weight_dtype, kvd, d, nrm, n, vv);
            float *kc = m->kcache + (size_t)b * c->max_seq * kvd;
            float *vc = m->vcache + (size_t)b * c->max_seq * kvd;
            for (int r = 0; r < n; ++r) {
                int pos = start + r;
                for (int hh = 0; hh < H; ++hh) rope(q + (size_t)r * qd + hh * hd, hd, pos, c->rope_base);
                for (int hh = 0; hh < Hkv; ++hh) rope(kk + (size_t)r * kvd + hh * hd, hd, pos, c->rope_base);
                for (int i = 0; i < kvd; ++i) {
                    double kx = kk[(size_t)r * kvd + i], vx = vv[(size_t)r * kvd + i];
                    kc[(size_t)pos * kvd + i] = c->kv_dtype ? round_to_bf16(kx) : (float)kx;
                    vc[(size_t)pos * kvd + i] = c->kv_dtype ? round_to_bf16(vx) : (float)vx;
                }
            }
            const double scale = 1.0 / sqrt((double)hd);
#pragma omp parallel for collapse(2) schedule(static)
            for (int r = 0; r < n; ++r) {
                for (int hh = 0; hh < H; ++hh) {
                    int len = start + r + 1;
                    int kvh = hh / group;
                    const double *qv = q + (size_t)r * qd + hh * hd;
                    double *s = (double *)malloc(sizeof(double) * (size_t)len);
                    double mx = -INFINITY;
                    for (int t = 0; t < len; ++t) {
                        const float *kt = kc + (size_t)t * kvd + kvh * hd;
                        double acc = 0.0;
                        for (int i = 0; i < hd; ++i) acc += qv[i] * (double)kt[i];
                        s[t] = acc * scale;
                        if (s[t] > mx) mx = s[t];
                    }
                    double den = 0.0;
                    for (int t = 0; t < len; ++t) { s[t] = exp(s[t] - mx); den += s[t]; }
                    double *o = att + (size_t)r * qd + hh * hd;
                    for (int i = 0; i < hd; ++i) o[i] = 0.0;
                    for (int t = 0; t < len; ++t) {
                        const float *vt = vc + (size_t)t * kvd + kvh * hd;
                        double p = s[t] / den;
                        for (int i = 0; i < hd; ++i) o[i] += p * (double)vt[i];
                    }
                    free(s);
                }
            }
            matmul_rows(m->wo[b], c->weight_dtype, d, qd, att, n, proj);
            for (size_t i = 0; i < (size_t)n * d; ++i) h[i] += proj[i];
        }
        if (!(mask && mask[2 * b + 1])) {
            /* MLP sublayer: h += Wd (silu(Wg x) * (Wu x)) */
            for (int r = 0; r < n; ++r) rmsnorm(h + (size_t)r * d, m->mlp_norm[b], d, c->rms_eps, nrm + (size_t)r * d);
            matmul_rows(m->wg[b], c->weight_dtype, F, d, nrm, n, g);
            matmul_rows(m->wu[b], c->weight_dtype, F, d, nrm, n, u);
            for (size_t i = 0; i < (size_t)n * F; ++i) {
                double a = g[i];
                u[i] = (a / (1.0 + exp(-a))) * u[i];
            }
            matmul_rows(m->wd[b], c->weight_dtype, d, F, u, n, proj);
            for (size_t i = 0; i < (size_t)n * d; ++i) h[i] += proj[i];
        }
    }

    for (int r = 0; r < n; ++r) rmsnorm(h + (size_t)r * d, m->final_norm, d, c->rms_eps, nrm + (size_t)r * d);
    if (hidden_out)
        for (size_t i = 0; i < (size_t)n * d; ++i) hidden_out[i] = (float)nrm[i];
    if (logits_out && logits_from < n) {
        int nl = n - logits_from;
        double *lg = (double *)malloc(sizeof(double) * (size_t)nl * c->vocab);
        matmul_rows(m->lm_head, c->weight_dtype, c->vocab, d, nrm + (size_t)logits_from * d, nl, lg);
        for (size_t i = 0; i < (size_t)nl * c->vocab; ++i) logits_out[i] = (float)lg[i];
        free(lg);
    }
    free(h); free(nrm); free(q); free(kk); free(vv); free(att); free(proj); free(g); free(u);
    return 0;
}

/* raw cache access for tests: copies the cached key/value row of one block and position */
int orc_read_kv(const orc_model *m, int block, int pos, float *k_out, float *v_out) {
    const orc_cfg *c = &m->cfg;
    if (block < 0 || block >= c->n_blocks || pos < 0 || pos >= c->max_seq) return -1;
    size_t kvd = (size_t)c->n_kv_heads * c->head_dim;
    size_t off = ((size_t)block * c->max_seq + pos) * kvd;
    memcpy(k_out, m->kcache + off, kvd * sizeof(float));
    memcpy(v_out, m->vcache + off, kvd * sizeof(float));
    return 0;
}
