/* Driver for the AddressSanitizer + UndefinedBehaviorSanitizer build of the CPU oracle (host code only): walks
 * every entry point of oracle/adadecode_oracle.c on a small random model, in all three storage types, with the
 * edge cases that stress its indexing (ragged calls, caches filled to the last position, rollbacks, forced
 * schedules, scripted wrong drafts, sampled decoding, the ablation switches).  The checks of the results are in
 * the Python tests; this program only has to run clean under the sanitizers.  Exit status 0 = ran through. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/adadecode_oracle.h"

static uint64_t rng_state = 88172645463325252ull;
static double uniform(void) {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (double)(rng_state >> 11) / 9007199254740992.0;
}
static float gauss(void) { return (float)(sqrt(-2.0 * log(uniform() + 1e-300)) * cos(6.283185307179586 * uniform())); }

static uint16_t to_bf16(float x) { uint32_t u; memcpy(&u, &x, 4); u += 0x7FFFu + ((u >> 16) & 1u); return (uint16_t)(u >> 16); }
/* fp32 -> IEEE half bits for test data: round to nearest even in the normal range, tiny values to zero, large to the largest finite */
static uint16_t to_f16(float x) {
    uint32_t u;
    memcpy(&u, &x, 4);
    const uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    const int32_t e = (int32_t)((u >> 23) & 0xFF) - 127 + 15;
    uint32_t man = u & 0x7FFFFFu;
    if (e <= 0) return sign;
    if (e >= 31) return (uint16_t)(sign | 0x7BFFu);
    uint32_t h = ((uint32_t)e << 10) | (man >> 13);
    const uint32_t rest = man & 0x1FFFu;
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) ++h;
    if (h >= 0x7C00u) h = 0x7BFFu;
    return (uint16_t)(sign | h);
}

static void *tensor(size_t n, float std, float mean, int dtype) {
    size_t es = dtype == ORC_F32 ? 4 : 2;
    char *p = (char *)malloc(n * es);
    if (!p) exit(3);
    for (size_t i = 0; i < n; ++i) {
        float v = mean + std * gauss();
        if (dtype == ORC_F32) ((float *)p)[i] = v;
        else ((uint16_t *)p)[i] = dtype == ORC_BF16 ? to_bf16(v) : to_f16(v);
    }
    return p;
}

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "driver check failed: %s (line %d)\n", #c, __LINE__); exit(2); } } while (0)

static void run(int dtype, int gqa) {
    orc_config c;
    memset(&c, 0, sizeof c);
    c.n_layers = 5; c.d_model = 96; c.n_q_heads = 6; c.n_kv_heads = gqa ? 2 : 6; c.head_dim = 32; c.d_ffn = 136; c.vocab = 203;
    c.rope_base = 10000.0; c.rms_eps = 1e-5; c.wdtype = dtype; c.kv_dtype = dtype;
    c.n_exit = 2; c.exit_layers[0] = 2; c.exit_layers[1] = 4;
    const int d = c.d_model, dq = c.n_q_heads * c.head_dim, dkv = c.n_kv_heads * c.head_dim, f = c.d_ffn, V = c.vocab;
    orc_layer_weights lw[5];
    void *keep[64];
    int nk = 0;
    for (int l = 0; l < c.n_layers; ++l) {
        lw[l].attn_norm = keep[nk++] = tensor(d, 0.1f, 1.0f, dtype);
        lw[l].wq = keep[nk++] = tensor((size_t)dq * d, 0.05f, 0.f, dtype);
        lw[l].wk = keep[nk++] = tensor((size_t)dkv * d, 0.05f, 0.f, dtype);
        lw[l].wv = keep[nk++] = tensor((size_t)dkv * d, 0.05f, 0.f, dtype);
        lw[l].wo = keep[nk++] = tensor((size_t)d * dq, 0.01f, 0.f, dtype);
        lw[l].ffn_norm = keep[nk++] = tensor(d, 0.1f, 1.0f, dtype);
        lw[l].w_gate = keep[nk++] = tensor((size_t)f * d, 0.05f, 0.f, dtype);
        lw[l].w_up = keep[nk++] = tensor((size_t)f * d, 0.05f, 0.f, dtype);
        lw[l].w_down = keep[nk++] = tensor((size_t)d * f, 0.01f, 0.f, dtype);
    }
    orc_top_weights top;
    memset(&top, 0, sizeof top);
    top.embed = keep[nk++] = tensor((size_t)V * d, 0.3f, 0.f, dtype);
    top.final_norm = keep[nk++] = tensor(d, 0.1f, 1.0f, dtype);
    top.lm_head = keep[nk++] = tensor((size_t)V * d, 0.3f, 0.f, dtype);
    top.exit_T[0] = keep[nk++] = tensor((size_t)d * d, 0.05f, 0.f, dtype);     /* head 0 with a transform, head 1 without */
    orc_model *m = orc_model_new(&c, lw, &top);
    CHECK(m);
    const int max_pos = 48;
    orc_kv *kv = orc_kv_new(m, max_pos);
    CHECK(kv);

    /* ragged layer steps up to the cache's last position, heads, verification, cache access */
    int32_t toks[48], pos[8];
    for (int i = 0; i < 48; ++i) toks[i] = (int32_t)(uniform() * V);
    double *h = (double *)malloc(sizeof(double) * 8 * d), *z = (double *)malloc(sizeof(double) * V);
    int start = 0;
    const int sizes[] = {1, 8, 3, 7, 2, 8, 5, 6, 8};
    for (int s = 0; s < 9 && start < max_pos; ++s) {
        int n = sizes[s];
        if (start + n > max_pos) n = max_pos - start;
        for (int i = 0; i < n; ++i) pos[i] = start + i;
        orc_embed(m, toks + start, n, h);
        for (int l = 1; l <= c.n_layers; ++l) CHECK(orc_layer_step(m, kv, l, h, pos, n) == 0);
        int32_t tok, nacc, next, arg[8], draft[8] = {1, 2, 3, 4, 5, 6, 7, 8};
        double conf, margin, mar[8];
        for (int hi = -1; hi < c.n_exit; ++hi) orc_head(m, hi, h + (size_t)(n - 1) * d, &tok, &conf, &margin, z);
        CHECK(conf > 0.0 && conf <= 1.0);
        orc_verify(m, h, draft, n, &nacc, &next, arg, mar);
        CHECK(nacc >= 0 && nacc < n);
        start += n;
    }
    CHECK(start == max_pos);
    CHECK(orc_layer_step(m, kv, 1, h, pos, 1) != 0);                 /* the cache is full: refused, nothing written */
    double *kk = (double *)malloc(sizeof(double) * max_pos * dkv), *vv = (double *)malloc(sizeof(double) * max_pos * dkv);
    float *kf = (float *)malloc(sizeof(float) * max_pos * dkv);
    for (int l = 1; l <= c.n_layers; ++l) {
        CHECK(orc_kv_len(kv, l) == max_pos);
        orc_kv_read(kv, l, 0, max_pos, kk, vv);
        for (int i = 0; i < max_pos * dkv; ++i) kf[i] = (float)kk[i];
        orc_kv_write(kv, l, 0, max_pos, kf, kf);
    }
    orc_kv_truncate(kv, 17);
    orc_kv_set_len(kv, 2, 9);
    CHECK(orc_kv_len(kv, 1) == 17 && orc_kv_len(kv, 2) == 9);

    /* generation: greedy, Algorithm 1 over thresholds and caps, forced schedules with scripted drafts, end-of-sequence,
     * sampled decoding, the ablation switches */
    int32_t prompt[9], out[64], n_out;
    for (int i = 0; i < 9; ++i) prompt[i] = (int32_t)(uniform() * V);
    double margins[64];
    CHECK(orc_generate_greedy(m, kv, prompt, 9, 30, -1, out, &n_out, margins) == 0 && n_out == 30);
    const int32_t eos = out[7];
    uint8_t forced[48];
    int32_t script[48];
    float *u = (float *)malloc(sizeof(float) * max_pos * (c.n_exit + 3));
    for (int i = 0; i < max_pos; ++i) {
        const double r = uniform();
        forced[i] = r < 0.3 ? 2 : (r < 0.6 ? 4 : 0);
        script[i] = (i % 5 == 0) ? (int32_t)(uniform() * V) : -1;
    }
    for (int i = 0; i < max_pos * (c.n_exit + 3); ++i) u[i] = (float)(uniform() * 0.999);
    orc_event *ev = (orc_event *)malloc(sizeof(orc_event) * 4096);
    const double gammas[] = {0.0, 0.02, 0.5, 1.0};
    for (int gi = 0; gi < 4; ++gi)
        for (int cap = 0; cap <= 7; cap += (cap == 0 ? 1 : 3))
            for (int variant = 0; variant < 6; ++variant) {
                orc_gen_params gp;
                memset(&gp, 0, sizeof gp);
                gp.gamma = gammas[gi]; gp.max_pending = cap; gp.max_new = 30; gp.eos_id = -1;
                if (variant == 1) { gp.forced_exit = forced; gp.scripted_draft = script; }
                if (variant == 2) gp.eos_id = eos;
                if (variant == 3) { gp.temperature = 0.7; gp.uniforms = u; }
                if (variant == 4) { gp.head_mask = 2; gp.no_verify = 1; }
                if (variant == 5) { gp.temperature = 0.05; gp.uniforms = u; gp.forced_exit = forced; gp.scripted_draft = script; gp.head_mask = 1; }
                orc_stats st;
                int64_t nev = 0;
                /* a small event buffer on purpose: the count goes on, the writes must stop */
                CHECK(orc_generate_ada(m, kv, prompt, 9, &gp, out, &n_out, &st, ev, variant == 0 ? 16 : 4096, &nev) == 0);
                CHECK(n_out >= 1 && n_out <= 30 && st.tokens == n_out && nev > 0);
            }
    /* the building blocks of the sampled form */
    double *p = (double *)malloc(sizeof(double) * V), *q = (double *)malloc(sizeof(double) * V);
    for (int i = 0; i < V; ++i) z[i] = gauss();
    orc_softmax_t(z, V, 0.3, p);
    for (int i = 0; i < V; ++i) z[i] = gauss();
    orc_softmax_t(z, V, 1.5, q);
    for (int k = 0; k < 50; ++k) {
        double mg, ratio;
        int32_t repl;
        const int32_t t = orc_sample_cdf(q, V, uniform() * 0.999, &mg);
        CHECK(t >= 0 && t < V);
        (void)orc_accept_or_resample(p, q, V, t, uniform() * 0.999, uniform() * 0.999, &repl, &ratio, &mg);
    }
    (void)orc_accept_or_resample(p, p, V, 3, 0.999, 0.5, &(int32_t){0}, &(double){0}, &(double){0});   /* zero residual */
    double vec[32];
    for (int i = 0; i < 32; ++i) vec[i] = gauss();
    orc_rope(vec, 32, 47, 10000.0);
    orc_rmsnorm(vec, top.final_norm, dtype, 32, 1e-5, vec);
    orc_set_num_threads(orc_num_threads());

    free(p); free(q); free(ev); free(u); free(kk); free(vv); free(kf); free(h); free(z);
    orc_kv_free(kv);
    orc_model_free(m);
    for (int i = 0; i < nk; ++i) free(keep[i]);
}

int main(void) {
    for (int dtype = ORC_F32; dtype <= ORC_F16; ++dtype)
        for (int gqa = 0; gqa < 2; ++gqa) run(dtype, gqa);
    printf("oracle driver: ran through\n");
    return 0;
}
