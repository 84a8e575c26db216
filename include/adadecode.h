/*
 * adadecode.h -- C ABI of the MI355X (gfx950) implementation of AdaDecode's hot path
 * (arxiv 2506.03700, the AdaDecode paper).
 *
 * The library runs, on one GPU and at batch 1, the three operations Algorithm 1 is made of, plus the
 * loop itself:
 *   ad_layer_step   Algorithm 1's layer-update step: one decoder layer over all rows pending at that layer, whose
 *                   K/V entries join the layer's cache (ad_layer_steps: a range of consecutive layers over the same rows)
 *   ad_exit_head    Eq. 1 at temperature 0: greedy token of an intermediate-layer head and its probability
 *   ad_verify       Eq. 2 at temperature 0: accept the early predictions that equal the final layer's
 *                   greedy tokens, replace the first that does not
 *   ad_generate     Algorithm 1 (prefill, layer loop with early exits, deferred layers, verification,
 *                   rollback) driven by the three calls above
 *
 * Conventions
 *   - Layers are 1-based; positions are 0-based; all matrices are [out_features, in_features] row-major.
 *   - "dev" pointers are device memory the caller allocated (for instance through PyTorch) and owns; the
 *     library never allocates or frees device memory.  "host" pointers are ordinary host memory, read or
 *     written before the call returns.  "pinned host or dev" pointers are written by a kernel: valid
 *     after the stream has been synchronised.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream).
 *   - Every call returns an ad_status; nothing is thrown or aborted.  ad_last_error() gives the text of
 *     the last failure on the calling thread.  A call that fails leaves the cache lengths unchanged.
 *   - One call at a time per ad_model: calls share the model's scratch area, so calls on the same model
 *     must be issued on one stream (or otherwise ordered); different models are independent.
 */
#ifndef ADADECODE_H
#define ADADECODE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ad_model ad_model;   /* opaque: configuration, packed weights, scratch */
typedef struct ad_kv ad_kv;         /* opaque: per-layer KV cache with per-layer lengths */

typedef enum {
    AD_OK = 0,
    AD_EINVAL = 1,   /* null pointer, bad configuration */
    AD_ERANGE = 2,   /* m outside [1, m_max], layer out of range, position beyond max_pos */
    AD_ESTATE = 3,   /* positions not consecutive or not at the layer's cache end; head on a layer without one */
    AD_EDEVICE = 4,  /* HIP error (text in ad_last_error) */
    AD_ENOMEM = 5    /* workspace / storage too small */
} ad_status;

typedef enum { AD_F32 = 0, AD_BF16 = 1, AD_F16 = 2 } ad_dtype;

enum { AD_MAX_EXIT = 8, AD_M_MAX = 8 };

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;   /* d_model % 16 == 0 and <= 8192 (fp32: 5120),
                                                                                   head_dim 64 or 128, d_ffn % 8 == 0 */
    float   rope_base, rms_eps;
    int32_t dtype;                       /* ad_dtype: storage of the weights passed in and of the KV cache.  AD_F16 is
                                            IEEE half precision, the precision the paper's models run in (Sec. 4.2);
                                            hidden states are fp32 at the boundary for every dtype */
    int32_t n_exit;                      /* number of exit heads */
    int32_t exit_layers[AD_MAX_EXIT];    /* 1-based, ascending, each < n_layers (Sec. 2.1: heads at chosen layers) */
    int32_t m_max;                       /* largest number of rows per call, 1..AD_M_MAX */
} ad_config;

/* One decoder layer.  Norm vectors have d_model elements; all tensors are of cfg.dtype. */
typedef struct {
    const void *attn_norm, *wq, *wk, *wv, *wo, *ffn_norm, *w_gate, *w_up, *w_down;   /* dev */
} ad_layer_weights;

/* embed [vocab, d], final_norm [d], lm_head [vocab, d] (may alias embed).  exit_T is NULL, or an array
 * of n_exit dev pointers, each NULL (identity) or a [d, d] transform T: the exit head is then
 * E = E* T, the lightweight head of Sec. 2.1, applied after the shared final norm. */
typedef struct {
    const void *embed, *final_norm, *lm_head;   /* dev */
    const void *const *exit_T;                  /* host array of dev pointers, or NULL */
} ad_top_weights;

/* Bytes of device workspace ad_model_create needs (0 if the configuration is invalid).  It holds the
 * library's own streaming layout of every weight matrix plus scratch. */
size_t    ad_workspace_bytes(const ad_config *);

/* Re-lays the weights out into `workspace` (dev, 256-byte aligned, ad_workspace_bytes() bytes, zero-filled
 * or not) on `stream` and returns a handle.  After the stream has been synchronised the caller may free
 * the original weight buffers; `workspace` must stay alive until ad_model_destroy. */
ad_status ad_model_create(const ad_config *, const ad_layer_weights *layers /*host [n_layers]*/,
                          const ad_top_weights *, void *workspace, size_t workspace_bytes, void *stream,
                          ad_model **out);
ad_status ad_model_destroy(ad_model *);

/* KV cache.  Storage layout (caller-visible, so that tests and benchmarks can fill or read it), with
 * stride = max_pos rounded up to a multiple of 64 and elements of cfg.dtype:
 *   per layer: K [kv head][position 0..stride)[head_dim]   (keys after rotary embedding)
 *        then  V [kv head][head_dim][position 0..stride)   (transposed: positions are contiguous)
 * Entries at positions >= the layer's length are dead, not zeroed. */
size_t    ad_kv_bytes(const ad_config *, int32_t max_pos);
/* Also fills the cache's rotary table on `stream` and synchronises it. */
ad_status ad_kv_create(const ad_model *, void *kv_storage /*dev*/, size_t kv_storage_bytes, int32_t max_pos, void *stream,
                       ad_kv **out);
ad_status ad_kv_destroy(ad_kv *);
ad_status ad_kv_len(const ad_kv *, int32_t layer, int32_t *len);
ad_status ad_kv_set_len(ad_kv *, int32_t layer, int32_t len);   /* declare a prefilled cache (benchmarks) */
/* Rollback after a rejected early prediction (Sec. 2.2): every layer's length becomes min(len, new_len). */
ad_status ad_kv_truncate(ad_kv *, int32_t new_len);

/* hidden[r] = embedding row of tokens[r].  tokens: host [m]; hidden: dev [m, d] fp32. */
ad_status ad_embed(const ad_model *, const int32_t *tokens, int32_t m, void *hidden, void *stream);

/* One decoder layer over the m pending rows of that layer (Algorithm 1, the layer-update step; Sec. 2.2).  hidden: dev [m, d] fp32, updated in place.  pos: host [m], consecutive, and
 * pos[0] must equal the layer's current cache length; the rows' K/V are appended and the length grows
 * by m.  Row r attends to positions 0..pos[r]. */
ad_status ad_layer_step(const ad_model *, ad_kv *, int32_t layer, void *hidden, const int32_t *pos, int32_t m,
                        void *stream);

/* The same rows through layers first_layer .. first_layer + n_layers - 1 one after the other: the stretch of
 * Algorithm 1's layer loop between two points where the set of pending rows can change (an exit head, or the layer at
 * which earlier tokens' deferred rows join).  Computes what n_layers calls of ad_layer_step with the same hidden, pos
 * and m compute (so pos[0] must equal the cache length of every layer in the range); results may differ from those
 * calls in the last bits, because inside a range a layer hands its output to the next layer's QKV projection already
 * normalised and packed.  In AD_LAYER_FUSED mode the whole range is one kernel launch.  Errors as ad_layer_step; a
 * range that leaves 1..n_layers is AD_ERANGE. */
ad_status ad_layer_steps(const ad_model *, ad_kv *, int32_t first_layer, int32_t n_layers, void *hidden, const int32_t *pos,
                         int32_t m, void *stream);

/* How ad_layer_step and ad_layer_steps run.  AD_LAYER_KERNELS (the default): one kernel per phase (QKV, attention, fold, Wo,
 * gate/up, down).  AD_LAYER_FUSED (bf16 models with d_model <= 5120 only): one persistent kernel with one workgroup per compute unit
 * and grid barriers between the phases; it needs the device to itself while it runs (no other kernel of this
 * process may occupy compute units at the same time, or a barrier wait can time out).  A time-out is noticed by
 * the next call on the model, which returns AD_EDEVICE and puts the barrier back in order: the layer-step call
 * that timed out had already returned AD_OK and advanced the cache lengths of its layers by m, and the rows it
 * appended are invalid, so the caller must take the cache back to its length before that call (ad_kv_truncate or
 * ad_kv_set_len) before going on.  Both modes compute the same function; results may differ in the last bits. */
enum { AD_LAYER_KERNELS = 0, AD_LAYER_FUSED = 1 };
ad_status ad_set_layer_mode(ad_model *, int32_t mode);

/* Eq. 1 at temperature 0 for the exit head at `layer` (which must be one of exit_layers; layer ==
 * n_layers selects the final head): token = argmax_t z_t (lowest id among equals), conf = softmax
 * probability of that token, with z = E* T norm(hidden_row).  hidden_row: dev [d] fp32.
 * token, conf: pinned host or dev. */
ad_status ad_exit_head(const ad_model *, int32_t layer, const void *hidden_row, int32_t *token, float *conf,
                       void *stream);

/* Eq. 2 at temperature 0 over the m rows of the last layer's pending list.  hidden: dev [m, d] fp32,
 * outputs of layer L, in position order; draft: host [m-1], draft[j] = the token early-predicted after
 * row j (i.e. row j+1's token).  With a_j = final-head argmax of row j: n_accept = the first j with
 * a_j != draft[j] (or m-1 if none), next_token = a_{n_accept}.  n_accept, next_token: pinned host or dev.
 * row_argmax: NULL, or pinned host or dev [m]. */
ad_status ad_verify(const ad_model *, const void *hidden, const int32_t *draft, int32_t m, int32_t *n_accept,
                    int32_t *next_token, int32_t *row_argmax, void *stream);

/* ad_verify for callers that cannot allocate device memory and have no workspace to lend at that point: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same result.  The
 * per-workgroup partials of the vocabulary pass (the only scratch this call needs beyond the model's weights) are
 * kept in a static device array inside the library (512 KiB per GPU, room for 4096 workgroups x 8 rows; a device
 * whose vocabulary pass would use more workgroups gets AD_ERANGE) instead of the model's workspace, and the call
 * performs no allocation of any kind: no hipMalloc / hipFree, no event creation (its launches are not sampled by
 * ad_profile_start).  All models on one GPU share that array and it keeps the last call's contents (every slot
 * that is read has been rewritten by the same call, nothing needs clearing): calls that overlap on one GPU race,
 * so issue them on one stream or order them otherwise. */
ad_status ad_verify_static(const ad_model *, const void *hidden, const int32_t *draft, int32_t m, int32_t *n_accept,
                           int32_t *next_token, int32_t *row_argmax, void *stream);

/* The logits the head at `layer` assigns to m rows (the distributions that sampled decoding draws from and
 * verifies against; also used by tests).  logits: dev [m, vocab] fp32. */
ad_status ad_head_logits(const ad_model *, int32_t layer, const void *hidden, int32_t m, void *logits, void *stream);

/* ---- sampled decoding (Sec. 2.2: the token of Eq. 1 may be drawn with any sampling strategy; Eq. 2 in its
 * general form).  Random numbers are inputs: every draw is a uniform u in [0, 1) supplied by the caller and
 * turned into a token by inversion of the cumulative distribution in token-id order (the first id whose
 * cumulative probability exceeds u).  temperature > 0 scales the logits: p = softmax(z / temperature).
 *
 * ad_sample_logits: token ~ softmax(logits / temperature) with the draw u; prob = that token's probability
 * (the quantity Eq. 1 compares with gamma).  logits: dev [vocab] fp32.  token, prob: pinned host or dev. */
ad_status ad_sample_logits(const ad_model *, const void *logits, float temperature, float u, int32_t *token, float *prob,
                           void *stream);

/* Eq. 2 over the m rows of the last layer's pending list.  final_logits: dev [m, vocab] fp32, the final head's
 * logits of the rows in position order (p* = softmax(. / temperature)); draft_logits: dev [m-1, vocab] fp32,
 * row k = the logits that draft[k] (the token predicted early after row k) was drawn from; draft, u_accept,
 * u_resample: host [m-1]; all draws in [0, 1).  In order k = 0, 1, ...: draft[k] is accepted iff
 * u_accept[k] < min(1, p*_k(draft[k]) / p_draft_k(draft[k])); the first rejected draft ends the run:
 * n_accept = k and next_token is drawn with u_resample[k] from Normalize(max(0, p*_k - p_draft_k)) (from p*_k if
 * that residual is identically zero).  If every draft is accepted, n_accept = m-1 and next_token is drawn from
 * p*_{m-1} with u_final.  ratio: NULL, or [m-1]: the probability ratio of each draft that was checked, 0 for
 * the rest.  n_accept, next_token, ratio: pinned host or dev.  Uses the model's scratch: calls on one model
 * must be stream-ordered. */
ad_status ad_verify_sampled(const ad_model *, const void *final_logits, const void *draft_logits, const int32_t *draft,
                            int32_t m, float temperature, const float *u_accept, const float *u_resample, float u_final,
                            int32_t *n_accept, int32_t *next_token, float *ratio, void *stream);

/* ---- Algorithm 1 --------------------------------------------------------------------------------- */
typedef struct {
    float   gamma;               /* early-prediction threshold of Eq. 1 (strict >) */
    int32_t max_pending;         /* cap on unverified early predictions (App. D), 0..m_max-1 */
    int32_t max_new;             /* number of tokens to generate (all returned tokens are verified) */
    int32_t eos_id;              /* -1: none */
    const uint8_t *forced_exit;  /* host; NULL, or [max_pos]: 0 = full depth, else the exit layer forced for the
                                    token at that absolute position (confidence ignored) */
    const int32_t *scripted_draft; /* host; NULL, or [max_pos]: if >= 0, replaces the head's token when the
                                    token at that position exits early (failure injection for tests) */
    float   temperature;         /* 0: greedy decoding (Eq. 1 and Eq. 2 at temperature 0).  > 0: sampled decoding:
                                    tokens are drawn from softmax(z / temperature), the probability compared with
                                    gamma is the drawn token's, and verification is ad_verify_sampled's */
    const float *uniforms;       /* host; sampled decoding only: [max_pos][n_exit + 3] draws in [0, 1).  Row = the
                                    absolute position of a token; column i < n_exit draws its successor at exit
                                    head i, column n_exit draws its successor at the final layer, column
                                    n_exit + 1 decides the acceptance of the token drafted after it, column
                                    n_exit + 2 draws that token's replacement after a rejection */
    /* ablation switches (the variants of Table 3, in shape only) */
    int32_t head_mask;           /* 0: every exit head may fire; else bit i enables exit head i (a single bit = the
                                    fixed-layer variant with one head) */
    int32_t no_verify;           /* 1: early predictions are kept unchecked; the last layer only produces the next
                                    token from the newest row (the output may then differ from plain decoding) */
    int32_t no_issue_ahead;      /* 0: behind the kernels of a head evaluation the library already issues the first
                                    kernel of what the schedule expects to do next (the QKV projection of the next
                                    layer step, or the next token's embedding and its first QKV projection), so the
                                    GPU has work while the host waits for the outcome and decides; work issued for
                                    an outcome that did not occur is dropped.  1: nothing is issued before the
                                    outcome is known.  Tokens, statistics and events are the same either way. */
} ad_gen_params;

typedef struct {
    int64_t tokens, layer_steps, layer_step_rows, head_evals, verifies, early_preds, rejections, rolled_back;
    int64_t steps_by_m[AD_M_MAX + 1];
    int64_t bytes_algorithmic;   /* weight + KV bytes the steps above must move */
} ad_stats;

enum { AD_EV_LAYER_STEP = 1, AD_EV_HEAD = 2, AD_EV_VERIFY = 3, AD_EV_VERIFY_ROW = 4 };
/* Decision trace, one record per scheduler action (same meaning of the fields for every kind:
 * LAYER_STEP: layer, pos = first row's position, m.  HEAD: layer, pos, token, flag = exit taken, conf.
 * VERIFY: pos = first row's position, m, token = next token, flag = n_accept.
 * VERIFY_ROW: pos, token = final-head argmax, flag = 1 matched / 0 mismatched / -1 not compared.
 * Sampled decoding: HEAD: token = the drawn token, conf = its probability.  VERIFY_ROW: flag = 1 accepted /
 * 0 rejected / -1 not checked, conf = the ratio of Eq. 2 (0 if not checked), token = the accepted draft, on row
 * n_accept the next token, -1 on later rows.) */
typedef struct { int32_t kind, layer, pos, m, token, flag; float conf; float reserved; } ad_event;

/* Runs Algorithm 1 from an empty cache: prompt (host [n_prompt]) -> out_tokens (host [max_new]).
 * events: NULL, or host [max_events]; *n_events counts every event even beyond max_events.
 * The host thread takes every exit decision: after each head evaluation it polls a word in pinned memory that the
 * head's last kernel sets (falling back to a stream synchronisation if the word does not appear), so the call
 * occupies one host core while it runs.  When it returns, on success or with an error, nothing it enqueued is still
 * running on the stream.  Calls on one model must not overlap (they share the model's workspace and result words). */
ad_status ad_generate(const ad_model *, ad_kv *, const int32_t *prompt, int32_t n_prompt, const ad_gen_params *,
                      int32_t *out_tokens, int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events,
                      int64_t *n_events, void *stream);

/* ---- measurement ------------------------------------------------------------------------------------
 * Samples one of the library's two big kernels: AD_PROF_GEMM, the weight-streaming GEMM kernel (the vocabulary
 * pass of Eq. 1 / Eq. 2, and every projection of the layer step in AD_LAYER_KERNELS mode), or AD_PROF_LAYER,
 * the fused layer-step kernel (AD_LAYER_FUSED mode).  Every `period`-th launch of that kind is bracketed by a
 * pair of events on the launch stream.  ad_profile_stop synchronises, and reports the number of launches
 * seen, the number sampled, the summed duration of the sampled launches and the bytes those launches had to
 * move (GEMM: rows x inputs x element size of the matrix; layer step: its weights, the KV rows read and the KV
 * rows written -- the algorithmic figures), and the same byte count over all launches.  At most max_samples
 * launches are sampled (bounded event pool, 1..65536). */
enum { AD_PROF_GEMM = 0, AD_PROF_LAYER = 1 };
ad_status ad_profile_start(ad_model *, int32_t kind, int32_t period, int32_t max_samples);
ad_status ad_profile_stop(ad_model *, int64_t *n_launches, int64_t *n_samples, double *sampled_ms, int64_t *sampled_bytes,
                          int64_t *total_bytes);

/* Phase trace of the fused layer-step kernel: while `ticks` (dev, [n_workgroups][n_stamps] int64) is set, every
 * fused launch overwrites it with each workgroup's wall-clock ticks (100 MHz) at the kernel's start, before and
 * after each of its five grid barriers, and at its end.  ticks == NULL stops it.  The two counts are returned
 * through the pointers (either may be NULL); bytes is the size of the buffer. */
ad_status ad_layer_trace(ad_model *, void *ticks, size_t bytes, int32_t *n_workgroups, int32_t *n_stamps);

/* Measurement aid, no part of the method: kernels that only read the bytes one layer step has to read (layer
 * `layer`'s packed weights and 2 * n_kv_heads * head_dim * ctx cache elements of that layer) and drop them, on the
 * same grid as the layer step's kernels.  AD_PROBE_ONE_KERNEL: one launch reads all of it: the time the machine
 * needs for the bytes alone.  AD_PROBE_PER_PHASE: five launches queued behind each other, one per phase of the
 * layer step that reads from memory (QKV weights; cache rows; Wo; gate/up; down weights), each reading that phase's
 * bytes: the same bytes with the phases' dependence kept (a kernel boundary between them), nothing else.  The
 * caller times the calls (events on `stream`).  ctx in 0..max_pos. */
enum { AD_PROBE_ONE_KERNEL = 0, AD_PROBE_PER_PHASE = 1 };
ad_status ad_probe_stream(const ad_model *, const ad_kv *, int32_t layer, int32_t ctx, int32_t mode, void *stream);

const char *ad_last_error(void);   /* thread-local, never NULL */
const char *ad_version(void);

#ifdef __cplusplus
}
#endif
#endif
