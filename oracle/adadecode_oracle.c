/*
 * CPU oracle for the AdaDecode hot path -- TEST INFRASTRUCTURE ONLY (see adadecode_oracle.h).
 *
 * Each function names the passage of the paper (arxiv 2506.03700) it follows.  The decoder itself is
 * "the LM" of Algorithm 1 (its first line and the "update KV cache at layer l" step); the paper does
 * not spell it out, so it is the standard Llama block: RMSNorm, rotary position embedding applied to
 * the two halves of each head, grouped-query causal attention, SwiGLU feed-forward.
 */
#include "adadecode_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

struct orc_model {
    orc_config cfg;
    orc_layer_weights *layers;
    orc_top_weights top;
};

struct orc_kv {
    const orc_model *model;
    int32_t max_pos;
    int32_t *len;       /* [n_layers] */
    double **k, **v;    /* [n_layers] -> [max_pos][n_kv_heads*head_dim] */
};

/* ---- reading stored weights ---------------------------------------------------------------------- */

static inline double bf16_value(uint16_t bits) {
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)bits << 16;
    return (double)c.f;
}

/* IEEE half precision (1 sign, 5 exponent, 10 fraction bits) widened exactly */
static inline double f16_value(uint16_t bits) {
    const int sign = bits >> 15, e = (bits >> 10) & 31, f = bits & 1023;
    double v;
    if (e == 0) v = ldexp((double)f, -24);                     /* zero and subnormals: f * 2^-24 */
    else if (e == 31) v = f ? NAN : INFINITY;
    else v = ldexp((double)(1024 + f), e - 25);                /* (1 + f/1024) * 2^(e-15) */
    return sign ? -v : v;
}

/* The same values from a table indexed by the 16 bits (filled once from f16_value, which stays the definition): the
 * two ldexp calls per element made fp16 models twenty times slower to check than bf16 ones. */
static double f16_table[65536];
static int f16_table_ready = 0;
static void f16_table_init(void) {
#pragma omp critical(orc_f16_table)
    {
        if (!f16_table_ready) {
            for (uint32_t b = 0; b < 65536u; ++b) f16_table[b] = f16_value((uint16_t)b);
            f16_table_ready = 1;
        }
    }
}

static inline double weight_at(const void *w, int32_t wdtype, size_t i) {
    if (wdtype == ORC_F32) return (double)((const float *)w)[i];
    return wdtype == ORC_BF16 ? bf16_value(((const uint16_t *)w)[i]) : f16_value(((const uint16_t *)w)[i]);
}

/* A value as a bf16 cache stores it: to fp32, then round-to-nearest-even to 8 significand bits. */
static inline double round_to_bf16(double x) {
    union { uint32_t u; float f; } c;
    c.f = (float)x;
    c.u += 0x7FFFu + ((c.u >> 16) & 1u);
    c.u &= 0xFFFF0000u;
    return (double)c.f;
}

/* A value as an fp16 cache stores it: to fp32, then round-to-nearest-even to half precision (11 significand
 * bits above 2^-14, multiples of 2^-24 below; finite inputs far below the half-precision maximum). */
static inline double round_to_f16(double x) {
    const float f = (float)x;
    const double a = fabs((double)f);
    if (a == 0.0) return (double)f;
    int e;
    (void)frexp(a, &e);                                         /* a = frac * 2^e, frac in [0.5, 1) */
    const int q = (e - 1 < -14 ? -14 : e - 1) - 10;             /* exponent of the last kept bit */
    const double r = ldexp(nearbyint(ldexp(a, -q)), q);         /* nearbyint: ties to even (default mode) */
    return f < 0 ? -r : r;
}

/* sum_i w[off+i] * x[i] */
static double dot_w(const void *w, int32_t wdtype, size_t off, const double *x, int32_t n) {
    double acc = 0.0;
    if (wdtype == ORC_F32) {
        const float *p = (const float *)w + off;
#pragma omp simd reduction(+ : acc)
        for (int32_t i = 0; i < n; ++i) acc += (double)p[i] * x[i];
    } else if (wdtype == ORC_BF16) {
        const uint16_t *p = (const uint16_t *)w + off;
#pragma omp simd reduction(+ : acc)
        for (int32_t i = 0; i < n; ++i) acc += bf16_value(p[i]) * x[i];
    } else {
        const uint16_t *p = (const uint16_t *)w + off;
        if (!f16_table_ready) f16_table_init();
#pragma omp simd reduction(+ : acc)
        for (int32_t i = 0; i < n; ++i) acc += f16_table[p[i]] * x[i];
    }
    return acc;
}

/* out[r][i] = sum_k W[i][k] x[r][k]   (W is [n_out][n_in]) */
static void linear(const void *W, int32_t wdtype, int32_t n_out, int32_t n_in, const double *x, int32_t m,
                   double *out) {
#pragma omp parallel for schedule(static)
    for (int32_t i = 0; i < n_out; ++i)
        for (int32_t r = 0; r < m; ++r)
            out[(size_t)r * n_out + i] = dot_w(W, wdtype, (size_t)i * n_in, x + (size_t)r * n_in, n_in);
}

/* ---- building blocks ------------------------------------------------------------------------------ */

/* RMSNorm: out_i = x_i * w_i / sqrt(mean_j x_j^2 + eps). */
void orc_rmsnorm(const double *x, const void *w, int32_t wdtype, int32_t n, double eps, double *out) {
    double ss = 0.0;
    for (int32_t i = 0; i < n; ++i) ss += x[i] * x[i];
    const double scale = 1.0 / sqrt(ss / (double)n + eps);
    for (int32_t i = 0; i < n; ++i) out[i] = x[i] * scale * weight_at(w, wdtype, (size_t)i);
}

/* Rotary embedding of one head vector at position pos: element i is paired with element i + dh/2 and
 * the pair is rotated by the angle pos * base^(-2i/dh). */
void orc_rope(double *vec, int32_t head_dim, int32_t pos, double base) {
    const int32_t half = head_dim / 2;
    for (int32_t i = 0; i < half; ++i) {
        const double theta = (double)pos * pow(base, -2.0 * (double)i / (double)head_dim);
        const double c = cos(theta), s = sin(theta);
        const double a = vec[i], b = vec[i + half];
        vec[i] = a * c - b * s;
        vec[i + half] = a * s + b * c;
    }
}

/* Greedy form of Eq. 1: the sampled token is the argmax (lowest index among equals) and the quantity
 * compared with gamma is its softmax probability, 1 / sum_t exp(z_t - z_max).  The margin is the gap
 * between the largest and the second largest logit (0 for an exact tie). */
void orc_confidence(const double *z, int32_t n, int32_t *token, double *conf, double *margin) {
    int32_t best = 0;
    for (int32_t t = 1; t < n; ++t)
        if (z[t] > z[best]) best = t;
    double second = -INFINITY, denom = 0.0;
    for (int32_t t = 0; t < n; ++t) {
        if (t != best && z[t] > second) second = z[t];
        denom += exp(z[t] - z[best]);
    }
    *token = best;
    *conf = 1.0 / denom;
    if (margin) *margin = (n > 1) ? z[best] - second : INFINITY;
}

/* ---- sampling (Sec. 2.2) ---------------------------------------------------------------------------- */

/* softmax(z / temperature): the distribution a token is sampled from when decoding is not greedy */
void orc_softmax_t(const double *z, int32_t n, double temperature, double *p) {
    double zmax = z[0];
    for (int32_t j = 1; j < n; ++j)
        if (z[j] > zmax) zmax = z[j];
    double sum = 0.0;
    for (int32_t j = 0; j < n; ++j) {
        p[j] = exp((z[j] - zmax) / temperature);
        sum += p[j];
    }
    for (int32_t j = 0; j < n; ++j) p[j] /= sum;
}

/* Inversion sampling: token j owns the interval [c_{j-1}, c_j) of the cumulative weights, and the draw
 * u * c_{n-1} falls into exactly one interval of positive length. */
int32_t orc_sample_cdf(const double *w, int32_t n, double u, double *margin) {
    double total = 0.0;
    for (int32_t j = 0; j < n; ++j) total += w[j];
    const double target = u * total;
    double c = 0.0;
    int32_t last_pos = 0;
    for (int32_t j = 0; j < n; ++j) {
        const double lo = c;
        c += w[j];
        if (w[j] > 0.0) last_pos = j;
        if (c > target) {
            if (margin) *margin = fmin(target - lo, c - target) / total;
            return j;
        }
    }
    if (margin) *margin = 0.0;
    return last_pos;
}

/* Eq. 2: the drafted token t survives with probability min(1, p(t) / q(t)); a rejected token is replaced by a
 * draw from the normalised positive part of p - q. */
int orc_accept_or_resample(const double *p, const double *q, int32_t n, int32_t t, double u_accept, double u_resample,
                           int32_t *replacement, double *ratio, double *margin) {
    const double r = (q[t] > 0.0) ? p[t] / q[t] : (p[t] > 0.0 ? INFINITY : 0.0);
    if (ratio) *ratio = r;
    double mg = (r >= 1.0) ? 1.0 : fabs(u_accept - r);
    const int accepted = u_accept < fmin(1.0, r);
    if (!accepted) {
        double *res = (double *)malloc(sizeof(double) * (size_t)n);
        double mass = 0.0;
        for (int32_t j = 0; j < n; ++j) {
            res[j] = (p[j] > q[j]) ? p[j] - q[j] : 0.0;
            mass += res[j];
        }
        double ms;
        *replacement = orc_sample_cdf(mass > 0.0 ? res : p, n, u_resample, &ms);
        if (ms < mg) mg = ms;
        free(res);
    }
    if (margin) *margin = mg;
    return accepted;
}

/* ---- model and cache objects ---------------------------------------------------------------------- */

orc_model *orc_model_new(const orc_config *cfg, const orc_layer_weights *layers, const orc_top_weights *top) {
    if (!cfg || !layers || !top) return NULL;
    if (cfg->n_layers < 1 || cfg->n_kv_heads < 1 || cfg->n_q_heads % cfg->n_kv_heads != 0 ||
        cfg->head_dim % 2 != 0 || cfg->n_exit < 0 || cfg->n_exit > ORC_MAX_EXIT)
        return NULL;
    orc_model *m = (orc_model *)calloc(1, sizeof *m);
    f16_table_init();
    m->cfg = *cfg;
    m->layers = (orc_layer_weights *)malloc(sizeof(orc_layer_weights) * (size_t)cfg->n_layers);
    memcpy(m->layers, layers, sizeof(orc_layer_weights) * (size_t)cfg->n_layers);
    m->top = *top;
    return m;
}

void orc_model_free(orc_model *m) {
    if (!m) return;
    free(m->layers);
    free(m);
}

orc_kv *orc_kv_new(const orc_model *model, int32_t max_pos) {
    const orc_config *c = &model->cfg;
    orc_kv *kv = (orc_kv *)calloc(1, sizeof *kv);
    kv->model = model;
    kv->max_pos = max_pos;
    kv->len = (int32_t *)calloc((size_t)c->n_layers, sizeof(int32_t));
    kv->k = (double **)calloc((size_t)c->n_layers, sizeof(double *));
    kv->v = (double **)calloc((size_t)c->n_layers, sizeof(double *));
    const size_t row = (size_t)c->n_kv_heads * c->head_dim;
    for (int32_t l = 0; l < c->n_layers; ++l) {
        kv->k[l] = (double *)calloc((size_t)max_pos * row, sizeof(double));
        kv->v[l] = (double *)calloc((size_t)max_pos * row, sizeof(double));
    }
    return kv;
}

void orc_kv_free(orc_kv *kv) {
    if (!kv) return;
    for (int32_t l = 0; l < kv->model->cfg.n_layers; ++l) {
        free(kv->k[l]);
        free(kv->v[l]);
    }
    free(kv->k);
    free(kv->v);
    free(kv->len);
    free(kv);
}

int32_t orc_kv_len(const orc_kv *kv, int32_t layer) { return kv->len[layer - 1]; }
void orc_kv_set_len(orc_kv *kv, int32_t layer, int32_t len) { kv->len[layer - 1] = len; }

/* Sec. 2.2: on a rejection the cache entries of every later token are removed, at every layer. */
void orc_kv_truncate(orc_kv *kv, int32_t new_len) {
    for (int32_t l = 0; l < kv->model->cfg.n_layers; ++l)
        if (kv->len[l] > new_len) kv->len[l] = new_len;
}

void orc_kv_write(orc_kv *kv, int32_t layer, int32_t pos0, int32_t n, const float *k, const float *v) {
    const size_t row = (size_t)kv->model->cfg.n_kv_heads * kv->model->cfg.head_dim;
    for (size_t i = 0; i < (size_t)n * row; ++i) {
        kv->k[layer - 1][(size_t)pos0 * row + i] = (double)k[i];
        kv->v[layer - 1][(size_t)pos0 * row + i] = (double)v[i];
    }
}

void orc_kv_read(const orc_kv *kv, int32_t layer, int32_t pos0, int32_t n, double *k, double *v) {
    const size_t row = (size_t)kv->model->cfg.n_kv_heads * kv->model->cfg.head_dim;
    memcpy(k, kv->k[layer - 1] + (size_t)pos0 * row, (size_t)n * row * sizeof(double));
    memcpy(v, kv->v[layer - 1] + (size_t)pos0 * row, (size_t)n * row * sizeof(double));
}

/* ---- the decoder layer ---------------------------------------------------------------------------- */

void orc_embed(const orc_model *model, const int32_t *tokens, int32_t m, double *hidden) {
    const int32_t d = model->cfg.d_model;
    for (int32_t r = 0; r < m; ++r)
        for (int32_t i = 0; i < d; ++i)
            hidden[(size_t)r * d + i] = weight_at(model->top.embed, model->cfg.wdtype, (size_t)tokens[r] * d + i);
}

/* Algorithm 1, the layer-update step (one layer over all rows pending at it, their K/V joining its cache): the rows are
 * the pending tokens of this layer, at consecutive positions that continue the layer's cache.  Row r
 * attends to every cached position 0..pos[r], which includes the rows before it in the same call. */
int orc_layer_step(const orc_model *model, orc_kv *kv, int32_t layer, double *hidden, const int32_t *pos,
                   int32_t m) {
    const orc_config *c = &model->cfg;
    if (layer < 1 || layer > c->n_layers || m < 1) return -1;
    if (pos[0] != kv->len[layer - 1]) return -2;
    for (int32_t r = 1; r < m; ++r)
        if (pos[r] != pos[0] + r) return -2;
    if (pos[m - 1] >= kv->max_pos) return -3;

    const orc_layer_weights *w = &model->layers[layer - 1];
    const int32_t d = c->d_model, dh = c->head_dim, hq = c->n_q_heads, hkv = c->n_kv_heads, f = c->d_ffn;
    const int32_t dq = hq * dh, dkv = hkv * dh, group = hq / hkv, dt = c->wdtype;
    double *K = kv->k[layer - 1], *V = kv->v[layer - 1];

    double *a = (double *)malloc(sizeof(double) * (size_t)m * d);
    double *q = (double *)malloc(sizeof(double) * (size_t)m * dq);
    double *kk = (double *)malloc(sizeof(double) * (size_t)m * dkv);
    double *vv = (double *)malloc(sizeof(double) * (size_t)m * dkv);
    double *o = (double *)malloc(sizeof(double) * (size_t)m * dq);
    double *t = (double *)malloc(sizeof(double) * (size_t)m * d);
    double *g = (double *)malloc(sizeof(double) * (size_t)m * f);
    double *u = (double *)malloc(sizeof(double) * (size_t)m * f);

    /* attention sub-block: a = RMSNorm(x); q,k,v = Wq a, Wk a, Wv a; rotate q and k; store k,v */
    for (int32_t r = 0; r < m; ++r) orc_rmsnorm(hidden + (size_t)r * d, w->attn_norm, dt, d, c->rms_eps, a + (size_t)r * d);
    linear(w->wq, dt, dq, d, a, m, q);
    linear(w->wk, dt, dkv, d, a, m, kk);
    linear(w->wv, dt, dkv, d, a, m, vv);
    for (int32_t r = 0; r < m; ++r) {
        for (int32_t h = 0; h < hq; ++h) orc_rope(q + (size_t)r * dq + (size_t)h * dh, dh, pos[r], c->rope_base);
        for (int32_t h = 0; h < hkv; ++h) orc_rope(kk + (size_t)r * dkv + (size_t)h * dh, dh, pos[r], c->rope_base);
        if (c->kv_dtype == ORC_BF16)   /* the cache's storage format: quantise what is stored */
            for (int32_t e = 0; e < dkv; ++e) {
                kk[(size_t)r * dkv + e] = round_to_bf16(kk[(size_t)r * dkv + e]);
                vv[(size_t)r * dkv + e] = round_to_bf16(vv[(size_t)r * dkv + e]);
            }
        else if (c->kv_dtype == ORC_F16)
            for (int32_t e = 0; e < dkv; ++e) {
                kk[(size_t)r * dkv + e] = round_to_f16(kk[(size_t)r * dkv + e]);
                vv[(size_t)r * dkv + e] = round_to_f16(vv[(size_t)r * dkv + e]);
            }
        memcpy(K + (size_t)pos[r] * dkv, kk + (size_t)r * dkv, sizeof(double) * (size_t)dkv);
        memcpy(V + (size_t)pos[r] * dkv, vv + (size_t)r * dkv, sizeof(double) * (size_t)dkv);
    }
    /* o_h = sum_j softmax_j(q_h . K[j][g] / sqrt(dh)) V[j][g],  j = 0..pos[r],  g = h / (Hq/Hkv) */
    const double inv_sqrt_dh = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2) schedule(static)
    for (int32_t r = 0; r < m; ++r) {
        for (int32_t h = 0; h < hq; ++h) {
            const int32_t gk = h / group, n_ctx = pos[r] + 1;
            const double *qh = q + (size_t)r * dq + (size_t)h * dh;
            double *s = (double *)malloc(sizeof(double) * (size_t)n_ctx);
            double smax = -INFINITY;
            for (int32_t j = 0; j < n_ctx; ++j) {
                const double *kj = K + (size_t)j * dkv + (size_t)gk * dh;
                double acc = 0.0;
                for (int32_t e = 0; e < dh; ++e) acc += qh[e] * kj[e];
                s[j] = acc * inv_sqrt_dh;
                if (s[j] > smax) smax = s[j];
            }
            double denom = 0.0;
            for (int32_t j = 0; j < n_ctx; ++j) {
                s[j] = exp(s[j] - smax);
                denom += s[j];
            }
            double *oh = o + (size_t)r * dq + (size_t)h * dh;
            for (int32_t e = 0; e < dh; ++e) oh[e] = 0.0;
            for (int32_t j = 0; j < n_ctx; ++j) {
                const double p = s[j] / denom;
                const double *vj = V + (size_t)j * dkv + (size_t)gk * dh;
                for (int32_t e = 0; e < dh; ++e) oh[e] += p * vj[e];
            }
            free(s);
        }
    }
    /* x' = x + Wo o */
    linear(w->wo, dt, d, dq, o, m, t);
    for (size_t i = 0; i < (size_t)m * d; ++i) hidden[i] += t[i];
    /* feed-forward sub-block: b = RMSNorm(x'); y = x' + Wd (silu(Wg b) * (Wu b)) */
    for (int32_t r = 0; r < m; ++r) orc_rmsnorm(hidden + (size_t)r * d, w->ffn_norm, dt, d, c->rms_eps, a + (size_t)r * d);
    linear(w->w_gate, dt, f, d, a, m, g);
    linear(w->w_up, dt, f, d, a, m, u);
    for (size_t i = 0; i < (size_t)m * f; ++i) g[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
    linear(w->w_down, dt, d, f, g, m, t);
    for (size_t i = 0; i < (size_t)m * d; ++i) hidden[i] += t[i];

    kv->len[layer - 1] += m;
    free(a); free(q); free(kk); free(vv); free(o); free(t); free(g); free(u);
    return 0;
}

/* ---- exit head and verification ------------------------------------------------------------------- */

/* Sec. 2.1: p(t | h) = softmax(E h) with E = E* T (T = identity when no transform is given).  The
 * hidden state first goes through the model's final RMSNorm, which the exit heads share with the
 * final head in this build's workloads. */
static void head_logits(const orc_model *model, int32_t head_index, const double *h, double *z) {
    const orc_config *c = &model->cfg;
    const int32_t d = c->d_model;
    double *n = (double *)malloc(sizeof(double) * (size_t)d);
    orc_rmsnorm(h, model->top.final_norm, c->wdtype, d, c->rms_eps, n);
    if (head_index >= 0 && model->top.exit_T[head_index]) {
        double *tn = (double *)malloc(sizeof(double) * (size_t)d);
        linear(model->top.exit_T[head_index], c->wdtype, d, d, n, 1, tn);
        free(n);
        n = tn;
    }
    linear(model->top.lm_head, c->wdtype, c->vocab, d, n, 1, z);
    free(n);
}

void orc_head(const orc_model *model, int32_t head_index, const double *h, int32_t *token, double *conf,
              double *margin, double *logits_out) {
    const int32_t V = model->cfg.vocab;
    double *z = logits_out ? logits_out : (double *)malloc(sizeof(double) * (size_t)V);
    head_logits(model, head_index, h, z);
    orc_confidence(z, V, token, conf, margin);
    if (!logits_out) free(z);
}

/* Eq. 2 at temperature 0.  The draft distribution is one-hot on the drafted token t, so the acceptance
 * probability min(1, p*(t)/1) is taken as "t is the final layer's greedy choice", and the replacement
 * drawn from Normalize(max(0, p* - p_draft)) at temperature 0 is argmax p*.  Row j's final-layer argmax
 * is compared with the token drafted for the next position; the first mismatch ends the accepted run. */
void orc_verify(const orc_model *model, const double *hidden, const int32_t *draft, int32_t m, int32_t *n_accept,
                int32_t *next_token, int32_t *row_argmax, double *row_margin) {
    const int32_t d = model->cfg.d_model;
    int32_t acc = m - 1, nxt = -1;
    for (int32_t j = 0; j < m; ++j) {
        int32_t tok;
        double conf, margin;
        orc_head(model, -1, hidden + (size_t)j * d, &tok, &conf, &margin, NULL);
        if (row_argmax) row_argmax[j] = tok;
        if (row_margin) row_margin[j] = margin;
        if (nxt < 0 && (j == m - 1 || tok != draft[j])) {
            acc = j;
            nxt = tok;
        }
    }
    *n_accept = acc;
    *next_token = nxt;
}

/* ---- generation ----------------------------------------------------------------------------------- */

/* Algorithm 1's initialisation of the cache from the prompt: the rows of positions first .. n-1 go through every
 * layer, a chunk of rows at a time (the cache holds the rows before `first` already).  If last_h is given it
 * receives the final-layer hidden state of the last row. */
static int prefill(const orc_model *model, orc_kv *kv, const int32_t *tokens, int32_t first, int32_t n, double *last_h) {
    const orc_config *c = &model->cfg;
    const int32_t chunk = 64, d = c->d_model;
    double *h = (double *)malloc(sizeof(double) * (size_t)chunk * d);
    int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)chunk);
    int rc = 0;
    for (int32_t s = first; s < n && rc == 0; s += chunk) {
        const int32_t m = (n - s < chunk) ? n - s : chunk;
        orc_embed(model, tokens + s, m, h);
        for (int32_t r = 0; r < m; ++r) pos[r] = s + r;
        for (int32_t l = 1; l <= c->n_layers && rc == 0; ++l) rc = orc_layer_step(model, kv, l, h, pos, m);
        if (rc == 0 && last_h && s + m == n) memcpy(last_h, h + (size_t)(m - 1) * d, sizeof(double) * (size_t)d);
    }
    free(h);
    free(pos);
    return rc;
}

/* Standard autoregressive greedy decoding: the result AdaDecode must reproduce (Sec. 4.2). */
int orc_generate_greedy(const orc_model *model, orc_kv *kv, const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                        int32_t eos_id, int32_t *out_tokens, int32_t *n_out, double *margins) {
    const orc_config *c = &model->cfg;
    double *h = (double *)malloc(sizeof(double) * (size_t)c->d_model);
    orc_kv_truncate(kv, 0);
    int rc = prefill(model, kv, prompt, 0, n_prompt, h);
    int32_t n = 0, pos = n_prompt;
    while (rc == 0 && n < max_new) {
        int32_t tok;
        double conf, margin;
        orc_head(model, -1, h, &tok, &conf, &margin, NULL);
        out_tokens[n] = tok;
        if (margins) margins[n] = margin;
        ++n;
        if (tok == eos_id || n == max_new) break;
        orc_embed(model, &tok, 1, h);
        for (int32_t l = 1; l <= c->n_layers && rc == 0; ++l) rc = orc_layer_step(model, kv, l, h, &pos, 1);
        ++pos;
    }
    *n_out = n;
    free(h);
    return rc;
}

static void emit(orc_event *events, int64_t max_events, int64_t *n_events, orc_event ev) {
    if (events && *n_events < max_events) events[*n_events] = ev;
    ++*n_events;
}

static int32_t exit_head_index(const orc_config *c, int32_t layer) {
    for (int32_t i = 0; i < c->n_exit; ++i)
        if (c->exit_layers[i] == layer) return i;
    return -1;
}

/*
 * Algorithm 1 (adaptive layer parallelism), greedy decoding or, with temperature > 0, sampled decoding.
 *
 * State, in the listing's notation.  The open tokens (the early predictions since the last verification,
 * oldest first, then the current token t_i) keep their position, id and hidden row in slots; P[l] is the
 * pending list of layer l.  The loop follows the listing step by step: t_i joins P[l], layer l runs over the
 * whole list at once, the head of that layer may predict t_{i+1} early, in which case t_i joins every deeper
 * list and the next token starts; at the last layer the tokens of P[L] are verified and the list is emptied.
 *
 * Readings of points the pseudo-code leaves open:
 *  - a token leaves a layer's pending list once the layer has processed it (the listing only empties
 *    the last layer's list, but Fig. 2 (left) shows each token going through each layer once);
 *  - the exit test is made only at layers that carry a head, which are all below the last layer; the
 *    last layer always verifies;
 *  - the cache is initialised from the prompt without its last token, which becomes the first current
 *    token (so the first generated token is produced by the loop itself);
 *  - the confidence is the softmax probability at temperature 1 of the greedy token, compared with
 *    gamma strictly (Eq. 1; Sec. 4.4: gamma = 1 never exits, gamma = 0 always does);
 *  - at most max_pending early predictions may be unverified (App. D, "maximum number of early
 *    predictions"): when the cap is reached the current token runs to the last layer;
 *  - with a token budget instead of an EOS stop, a token that would be the last one is not drafted:
 *    it runs to the last layer, so that every returned token is verified; an early prediction equal to
 *    the EOS id is not taken either;
 *  - sampled decoding (temperature > 0): the head's token is drawn from softmax(z / temperature) and the
 *    probability compared with gamma is that token's (Eq. 1); the head's whole distribution is kept until
 *    the verification, which walks the drafts in order with Eq. 2, replaces the first rejected one by a
 *    draw from the residual distribution, and, if none is rejected, draws the next token from the final
 *    distribution of the newest row.  Every draw is an input (gp->uniforms), one column per use, so that a
 *    position that samples at several heads uses a fresh draw at each.
 */
int orc_generate_ada(const orc_model *model, orc_kv *kv, const int32_t *prompt, int32_t n_prompt,
                     const orc_gen_params *gp, int32_t *out_tokens, int32_t *n_out, orc_stats *stats,
                     orc_event *events, int64_t max_events, int64_t *n_events_out) {
    const orc_config *c = &model->cfg;
    const int32_t L = c->n_layers, d = c->d_model;
    if (n_prompt < 1 || gp->max_new < 1 || gp->max_pending < 0) return -1;
    const int32_t cap_rows = gp->max_pending + 1;
    const int sampled = gp->temperature > 0.0;
    if (sampled && (!gp->uniforms || cap_rows > 9)) return -1;

    /* the open tokens (early predictions that still owe deeper layers, oldest first, then the current token t_i):
     * position, token id, hidden row; a token is named by its slot in these arrays */
    int32_t *row_pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap_rows);
    int32_t *row_tok = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap_rows);
    /* P[l], 1 <= l <= L: the per-layer pending lists of Algorithm 1 (the tokens layer l still has to run), as slots in arrival order;
     * nP[l] of them, stored at P + l * cap_rows */
    int32_t *P = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap_rows * (size_t)(L + 1));
    int32_t *nP = (int32_t *)calloc((size_t)(L + 1), sizeof(int32_t));
    int32_t *row_arg = (int32_t *)malloc(sizeof(int32_t) * (size_t)cap_rows);
    double *row_margin = (double *)malloc(sizeof(double) * (size_t)cap_rows);
    double *row_h = (double *)malloc(sizeof(double) * (size_t)cap_rows * d);
    const int32_t V = c->vocab, ucols = c->n_exit + 3;
    /* sampled runs keep the draft distribution of every open row's successor, and work on one final distribution */
    double *row_q = sampled ? (double *)malloc(sizeof(double) * (size_t)cap_rows * V) : NULL;
    double *zbuf = sampled ? (double *)malloc(sizeof(double) * (size_t)V) : NULL;
    double *pbuf = sampled ? (double *)malloc(sizeof(double) * (size_t)V) : NULL;
    orc_stats st;
    memset(&st, 0, sizeof st);
    int64_t n_events = 0;

    /* the cache starts from the prompt without its last token; the rows of the first keep_cache positions may be taken
     * over from an earlier run on a prompt that began with the same tokens (a row depends on the tokens up to its
     * position only), the rest is computed */
    const int32_t keep = gp->keep_cache;
    if (keep < 0 || keep > n_prompt - 1) return -1;
    for (int32_t l = 1; l <= L; ++l)
        if (orc_kv_len(kv, l) < keep) return -1;
    orc_kv_truncate(kv, keep);
    int rc = prefill(model, kv, prompt, keep, n_prompt - 1, NULL);
    int32_t cur = prompt[n_prompt - 1], pos = n_prompt - 1;
    int32_t n_rows = 0, n_y = 0, n_verified = 0, done = 0;

    while (rc == 0 && !done) {
        /* the current token t_i takes the next slot */
        const int32_t ti = n_rows;
        row_pos[ti] = pos;
        row_tok[ti] = cur;
        orc_embed(model, &cur, 1, row_h + (size_t)ti * d);
        ++n_rows;
        const int exits_ok = (n_rows - 1 < gp->max_pending) && (n_y + 1 < gp->max_new);

        for (int32_t l = 1; l <= L && rc == 0; ++l) {
            /* P[l] <- P[l] (+) t_i */
            int32_t *Pl = P + (size_t)l * cap_rows;
            Pl[nP[l]++] = ti;
            /* layer l runs once over every token of P[l] together; their K/V entries join the layer's cache.  Tokens
             * enter the lists in order and leave them together, so P[l] is a run of neighbouring slots that ends with
             * t_i, at consecutive positions that continue the layer's cache (checked: anything else would mean a token
             * skipped a layer) */
            const int32_t m = nP[l], first = Pl[0];
            for (int32_t k = 0; k < m; ++k)
                if (Pl[k] != first + k) rc = -4;
            if (Pl[m - 1] != ti) rc = -4;
            if (rc != 0) break;
            rc = orc_layer_step(model, kv, l, row_h + (size_t)first * d, row_pos + first, m);
            if (rc != 0) break;
            /* a token has passed layer l once it has been processed there: it leaves P[l] (Fig. 2, left).  P[L] is kept
             * until the verification below has looked at its tokens */
            if (l < L) nP[l] = 0;
            ++st.layer_steps;
            st.layer_step_rows += m;
            if (m <= 8) ++st.steps_by_m[m];
            emit(events, max_events, &n_events, (orc_event){ORC_EV_LAYER_STEP, l, row_pos[first], m, 0, 0, 0.0, 0.0});

            int32_t hi = (l < L) ? exit_head_index(c, l) : -1;
            if (hi >= 0 && gp->head_mask != 0 && !((gp->head_mask >> hi) & 1)) hi = -1;   /* head switched off */
            if (hi >= 0 && exits_ok && (!gp->forced_exit || gp->forced_exit[pos] == l)) {
                /* Eq. 1 on the newest row only: the older rows already have a drafted successor */
                int32_t tok;
                double conf, margin;
                if (!sampled) {
                    orc_head(model, hi, row_h + (size_t)(n_rows - 1) * d, &tok, &conf, &margin, NULL);
                } else {
                    double *q = row_q + (size_t)(n_rows - 1) * V;
                    head_logits(model, hi, row_h + (size_t)(n_rows - 1) * d, zbuf);
                    orc_softmax_t(zbuf, V, gp->temperature, q);
                    tok = orc_sample_cdf(q, V, (double)gp->uniforms[(size_t)pos * ucols + hi], &margin);
                    conf = q[tok];
                }
                ++st.head_evals;
                int fire = gp->forced_exit ? 1 : (conf > gp->gamma);
                if (gp->scripted_draft && gp->scripted_draft[pos] >= 0) tok = gp->scripted_draft[pos];
                if (tok == gp->eos_id) fire = 0;
                emit(events, max_events, &n_events, (orc_event){ORC_EV_HEAD, l, pos, 1, tok, fire, conf, margin});
                if (fire) {
                    /* early prediction: y <- y (+) t_{i+1}; P[l'] <- P[l'] (+) t_i for all deeper layers l' (they are
                     * owed to t_i and run together with later tokens); start the next token at once */
                    out_tokens[n_y++] = tok;
                    ++st.early_preds;
                    for (int32_t l2 = l + 1; l2 <= L; ++l2) P[(size_t)l2 * cap_rows + nP[l2]++] = ti;
                    cur = tok;
                    ++pos;
                    break;
                }
            }
            if (l == L) {
                /* the final layer is reached: P[L] holds every open token, each now complete at every layer; verify
                 * them in order, then empty P[L] */
                int32_t n_accept, next;
                const int32_t n_draft = n_rows - 1;
                if (nP[L] != n_rows || Pl[0] != 0) { rc = -4; break; }
                for (int32_t l2 = 1; l2 < L; ++l2)
                    if (nP[l2] != 0) rc = -4;
                if (rc != 0) break;
                nP[L] = 0;
                if (gp->no_verify) {
                    /* ablation: the drafts stand unchecked; the newest row's final head gives the next token */
                    const int32_t r = n_rows - 1;
                    double conf = 0.0, margin = 0.0;
                    if (!sampled) {
                        orc_head(model, -1, row_h + (size_t)r * d, &next, &conf, &margin, NULL);
                    } else {
                        head_logits(model, -1, row_h + (size_t)r * d, zbuf);
                        orc_softmax_t(zbuf, V, gp->temperature, pbuf);
                        next = orc_sample_cdf(pbuf, V, (double)gp->uniforms[(size_t)row_pos[r] * ucols + c->n_exit], &margin);
                    }
                    n_accept = n_draft;
                    ++st.verifies;
                    emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY, L, row_pos[0], n_rows, next, n_accept, 0.0, 0.0});
                    for (int32_t q = 0; q < n_rows; ++q)
                        emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY_ROW, L, row_pos[q], 1, q == r ? next : -1, -1, 0.0, q == r ? margin : INFINITY});
                } else if (!sampled) {
                    orc_verify(model, row_h, row_tok + 1, n_rows, &n_accept, &next, row_arg, row_margin);
                    ++st.verifies;
                    emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY, L, row_pos[0], n_rows, next, n_accept, 0.0, 0.0});
                    for (int32_t r = 0; r < n_rows; ++r) {
                        const int32_t cmp = (r < n_rows - 1 && r <= n_accept) ? (row_arg[r] == row_tok[r + 1]) : -1;
                        emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY_ROW, L, row_pos[r], 1, row_arg[r], cmp, 0.0, row_margin[r]});
                    }
                } else {
                    /* Eq. 2, draft by draft in position order, against the final distribution of the row before it */
                    double ratio[8 + 1] = {0}, mg[8 + 1] = {0};
                    int32_t flag[8 + 1];
                    n_accept = n_draft;
                    next = -1;
                    for (int32_t r = 0; r < n_rows; ++r) flag[r] = -1;
                    for (int32_t r = 0; r < n_draft && next < 0; ++r) {
                        const float *u = gp->uniforms + (size_t)row_pos[r] * ucols;
                        head_logits(model, -1, row_h + (size_t)r * d, zbuf);
                        orc_softmax_t(zbuf, V, gp->temperature, pbuf);
                        int32_t repl = -1;
                        flag[r] = orc_accept_or_resample(pbuf, row_q + (size_t)r * V, V, row_tok[r + 1], (double)u[c->n_exit + 1],
                                                         (double)u[c->n_exit + 2], &repl, &ratio[r], &mg[r]);
                        if (!flag[r]) {
                            n_accept = r;
                            next = repl;
                        }
                    }
                    if (next < 0) {
                        /* nothing rejected: the newest row's final distribution gives the next token */
                        const int32_t r = n_rows - 1;
                        head_logits(model, -1, row_h + (size_t)r * d, zbuf);
                        orc_softmax_t(zbuf, V, gp->temperature, pbuf);
                        next = orc_sample_cdf(pbuf, V, (double)gp->uniforms[(size_t)row_pos[r] * ucols + c->n_exit], &mg[r]);
                    }
                    ++st.verifies;
                    emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY, L, row_pos[0], n_rows, next, n_accept, 0.0, 0.0});
                    for (int32_t r = 0; r < n_rows; ++r) {
                        const int32_t tk = (r == n_accept) ? next : (r < n_accept ? row_tok[r + 1] : -1);
                        emit(events, max_events, &n_events, (orc_event){ORC_EV_VERIFY_ROW, L, row_pos[r], 1, tk, flag[r], ratio[r], mg[r]});
                    }
                }
                if (n_accept < n_draft) {
                    ++st.rejections;
                    st.rolled_back += n_draft - n_accept - 1;
                }
                /* keep the accepted drafts, replace what follows by the final layer's token, and drop
                 * the cache entries of every position after the last accepted row */
                n_y = n_y - n_draft + n_accept;
                out_tokens[n_y++] = next;
                n_verified = n_y;
                pos = row_pos[n_accept] + 1;
                orc_kv_truncate(kv, pos);
                cur = next;
                n_rows = 0;
                if (n_verified >= gp->max_new || next == gp->eos_id) done = 1;
            }
        }
    }
    st.tokens = n_verified;
    *n_out = n_verified;
    if (stats) *stats = st;
    if (n_events_out) *n_events_out = n_events;
    free(row_pos); free(row_tok); free(P); free(nP); free(row_arg); free(row_margin); free(row_h);
    free(row_q); free(zbuf); free(pbuf);
    return rc;
}

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the row loops may use from now on (no effect on any result: rows are independent). */
void orc_set_num_threads(int n) {
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}
