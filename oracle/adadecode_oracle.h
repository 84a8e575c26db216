/*
 * CPU oracle for the AdaDecode hot path (arxiv 2506.03700) -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision implementation of what the GPU library computes: the Llama-style
 * decoder layer step over m ragged rows, the exit head (Sec. 2.1; Eq. 1), the verification of early
 * predictions (Sec. 2.2; Eq. 2, at temperature 0 and in its general form with sampled tokens), plain greedy
 * decoding, and Algorithm 1.
 * It shares no code with the HIP path and must never be linked into, imported by or called from the
 * product: only tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * Arithmetic: every value is a double; weights are read as stored (fp32, or bf16 / fp16 bit patterns widened
 * exactly) and never rounded again.  The one storage format that is part of a workload's definition, a 16-bit
 * KV cache, is modelled as such: entries are quantised to its type when they are stored (kv_dtype), and every
 * later read sees the stored value.  Dot products may be summed in any order (the compiler is allowed
 * to vectorise them); nothing else is reordered, blocked or fused.
 *
 * Pins (tests/test_oracle_*.py): whole-sequence causal forward written with library matmul/softmax,
 * closed forms for RMSNorm / RoPE / softmax confidence, AdaDecode == greedy by brute force, deferred
 * KV == sequential KV, the worked example of Fig. 2 (left), gamma = 0 and gamma = 1 (Sec. 4.4); for the
 * sampled form: inversion sampling against a library cumulative sum / search, the output law of
 * draft-accept-resample against its closed form (exactly the final distribution when every draft is taken),
 * and the low-temperature limit against greedy decoding.
 * Parity unpinned: natural exit and rejection *rates* on random-init models (the paper's 5-6 % are
 * for trained heads on real data); they are reported, not checked.
 */
#ifndef ADADECODE_ORACLE_H
#define ADADECODE_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F16 = 2 };   /* fp32, bf16 bit patterns, IEEE half precision */
enum { ORC_MAX_EXIT = 8 };

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    double  rope_base, rms_eps;
    int32_t wdtype;                       /* ORC_F32, ORC_BF16 or ORC_F16: storage of every weight tensor */
    int32_t n_exit;
    int32_t exit_layers[ORC_MAX_EXIT];    /* 1-based, ascending, each < n_layers */
    int32_t kv_dtype;                     /* storage format of the KV cache: ORC_F32 keeps the computed values,
                                             ORC_BF16 / ORC_F16 round every stored K (after the rotary embedding) and
                                             V entry to that type, round-to-nearest-even, as a 16-bit cache does;
                                             attention then reads the stored values */
} orc_config;

/* All matrices are [out_features, in_features] row-major. */
typedef struct { const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down; } orc_layer_weights;
typedef struct { const void *embed, *final_norm, *lm_head; const void *exit_T[ORC_MAX_EXIT]; /* NULL = identity */ } orc_top_weights;

typedef struct orc_model orc_model;
typedef struct orc_kv orc_kv;

/* The model keeps the pointers; the caller keeps the buffers alive. */
orc_model *orc_model_new(const orc_config *, const orc_layer_weights *layers, const orc_top_weights *);
void       orc_model_free(orc_model *);
orc_kv    *orc_kv_new(const orc_model *, int32_t max_pos);
void       orc_kv_free(orc_kv *);
int32_t    orc_kv_len(const orc_kv *, int32_t layer /*1-based*/);
void       orc_kv_set_len(orc_kv *, int32_t layer, int32_t len);
void       orc_kv_truncate(orc_kv *, int32_t new_len);                 /* every layer: len = min(len, new_len) */
/* copy n positions starting at pos0; k and v are [n][n_kv_heads*head_dim] */
void       orc_kv_write(orc_kv *, int32_t layer, int32_t pos0, int32_t n, const float *k, const float *v);
void       orc_kv_read(const orc_kv *, int32_t layer, int32_t pos0, int32_t n, double *k, double *v);

/* --- building blocks, exported so that tests can pin each one ------------------------------------ */
void orc_rmsnorm(const double *x, const void *w, int32_t wdtype, int32_t n, double eps, double *out);
void orc_rope(double *vec, int32_t head_dim, int32_t pos, double base);     /* one head vector, in place */
/* logits z[V] -> lowest-index argmax, max-softmax confidence, top-2 logit margin */
void orc_confidence(const double *z, int32_t n, int32_t *token, double *conf, double *margin);

void orc_embed(const orc_model *, const int32_t *tokens, int32_t m, double *hidden /*[m][d]*/);
/* One decoder layer over m rows at consecutive positions pos[0..m), pos[0] == kv_len(layer).
 * Returns 0, or -1 (bad layer / m), -2 (positions not consecutive or not at the cache end), -3 (beyond max_pos). */
int  orc_layer_step(const orc_model *, orc_kv *, int32_t layer, double *hidden /*[m][d] in place*/,
                    const int32_t *pos, int32_t m);
/* Head on one row. head_index: -1 = final head (no T); i >= 0 = exit head i (uses exit_T[i] if given).
 * logits_out may be NULL. */
void orc_head(const orc_model *, int32_t head_index, const double *h, int32_t *token, double *conf,
              double *margin, double *logits_out);
/* Verification at temperature 0 of m rows of final-layer hidden states against m-1 drafted tokens. */
void orc_verify(const orc_model *, const double *hidden /*[m][d]*/, const int32_t *draft /*[m-1]*/, int32_t m,
                int32_t *n_accept, int32_t *next_token, int32_t *row_argmax /*[m] or NULL*/,
                double *row_margin /*[m] or NULL*/);

/* --- sampling (Sec. 2.2: the token of Eq. 1 may be sampled; Eq. 2 in its general form) -------------------
 * Random numbers are inputs: every draw is a uniform u in [0, 1) handed in by the caller. */
/* p = softmax(z / temperature), temperature > 0 */
void    orc_softmax_t(const double *z, int32_t n, double temperature, double *p);
/* Inversion of the cumulative distribution in index order over weights w >= 0 (not necessarily normalised):
 * returns the first j whose cumulative weight exceeds u * sum(w); if rounding leaves none, the last j with
 * w[j] > 0.  margin (may be NULL): distance from u * sum(w) to the nearer end of j's interval, as a
 * fraction of sum(w): how far u is from producing a neighbouring token. */
int32_t orc_sample_cdf(const double *w, int32_t n, double u, double *margin);
/* Eq. 2 for one token t drafted from q and checked against p: accepted (returns 1) iff
 * u_accept < min(1, p[t] / q[t]); otherwise returns 0 and *replacement is drawn with u_resample from
 * Normalize(max(0, p - q)) (from p itself if that residual is identically zero).  *ratio = p[t] / q[t].
 * *margin (may be NULL): min of |u_accept - ratio| (1 if ratio >= 1) and, after a rejection, the replacement
 * draw's orc_sample_cdf margin. */
int     orc_accept_or_resample(const double *p, const double *q, int32_t n, int32_t t, double u_accept,
                               double u_resample, int32_t *replacement, double *ratio, double *margin);

/* --- generation ------------------------------------------------------------------------------------ */
enum { ORC_EV_LAYER_STEP = 1, ORC_EV_HEAD = 2, ORC_EV_VERIFY = 3, ORC_EV_VERIFY_ROW = 4 };
typedef struct {
    int32_t kind;
    int32_t layer;      /* LAYER_STEP, HEAD */
    int32_t pos;        /* LAYER_STEP: first position; HEAD / VERIFY_ROW: the row's position; VERIFY: first row's position */
    int32_t m;          /* LAYER_STEP / VERIFY: rows */
    int32_t token;      /* HEAD: argmax (sampled runs: the sampled token); VERIFY: next token; VERIFY_ROW: argmax
                           (sampled runs: the draft checked on that row, the next token on row n_accept, else -1) */
    int32_t flag;       /* HEAD: 1 = exit taken; VERIFY: n_accept; VERIFY_ROW: 1 = row was compared and matched
                           (accepted), 0 = mismatched (rejected), -1 = not compared */
    double  conf;       /* HEAD: the token's probability; VERIFY_ROW of a sampled run: the ratio of Eq. 2 (0 if not compared) */
    double  margin;     /* HEAD / VERIFY_ROW: top-2 logit margin; sampled runs: how far the row's uniform draws were
                           from changing its decisions (see orc_sample_cdf, orc_accept_or_resample) */
} orc_event;

typedef struct {
    double  gamma;
    int32_t max_pending;            /* cap on unverified early predictions */
    int32_t max_new;
    int32_t eos_id;                 /* -1: none */
    const uint8_t *forced_exit;     /* NULL, or [max_pos]: 0 = full depth, else the exit layer forced for that position */
    const int32_t *scripted_draft;  /* NULL, or [max_pos]: if >= 0, the token drafted when position pos exits early
                                       (replaces the head's argmax; lets a test force a rejection) */
    double temperature;             /* 0: greedy (Eq. 1 and Eq. 2 at temperature 0).  > 0: tokens are sampled from
                                       softmax(z / temperature) and verified with the general Eq. 2 */
    const float *uniforms;          /* sampled runs: [max_pos][n_exit + 3] draws in [0, 1).  For the row at position
                                       pos: column i < n_exit samples its successor at exit head i; column n_exit
                                       samples its successor at the final layer; column n_exit + 1 decides the
                                       acceptance of the token drafted after it; column n_exit + 2 draws that
                                       token's replacement after a rejection */
    /* ablation switches (Table 3 of the paper, in shape only) */
    int32_t head_mask;              /* 0: every exit head may fire; else bit i enables exit head i (one bit set =
                                       the fixed-layer variant with a single head) */
    int32_t no_verify;              /* 1: no verification -- every early prediction is kept as emitted, and the last
                                       layer only produces the next token from the newest row (the output may then
                                       differ from plain decoding) */
    int32_t keep_cache;             /* 0, or the number of leading prompt positions (at most n_prompt - 1) whose rows the
                                       cache already holds at every layer from an earlier run on a prompt with the same
                                       leading tokens: they are kept instead of being computed again (a time saver for
                                       tests that restart a run from a longer prompt; the result is the same) */
} orc_gen_params;

typedef struct {
    int64_t tokens, layer_steps, layer_step_rows, head_evals, verifies, early_preds, rejections, rolled_back;
    int64_t steps_by_m[9];
} orc_stats;

/* Plain greedy decoding.  margins may be NULL; else [max_new] top-2 logit margin of each emitted token. */
int orc_generate_greedy(const orc_model *, orc_kv *, const int32_t *prompt, int32_t n_prompt, int32_t max_new,
                        int32_t eos_id, int32_t *out_tokens, int32_t *n_out, double *margins);
/* Algorithm 1.  events may be NULL; at most max_events are written, *n_events counts all of them. */
int orc_generate_ada(const orc_model *, orc_kv *, const int32_t *prompt, int32_t n_prompt, const orc_gen_params *,
                     int32_t *out_tokens, int32_t *n_out, orc_stats *, orc_event *events, int64_t max_events,
                     int64_t *n_events);

int orc_num_threads(void);
void orc_set_num_threads(int n);   /* timing aid: threads used by the row loops; results do not depend on it */

#ifdef __cplusplus
}
#endif
#endif
