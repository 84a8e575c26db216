// Host scheduler of Algorithm 1 (adaptive layer parallelism): which rows go through which layer when,
// when an early prediction is taken, and what a verification keeps.  It talks to the model only through
// the Backend interface, so the same code drives the GPU kernels and, in CPU tests, a scripted stand-in.
#pragma once
#include <stdint.h>
#include <vector>

#include "../../include/adadecode.h"

namespace ad {

// What the schedule does right after the head evaluation it is about to ask for, if that evaluation turns out as
// the schedule expects:
//   AHEAD_LAYER: rows [row0, row0 + m) go on through layer `layer` (no early prediction is taken);
//   AHEAD_TOKEN: the token the evaluation produces is embedded into row `row0` and passes layer 1 alone (m = 1):
//                an early prediction is taken, or the evaluation is the verification.
// A backend may issue the part of that work that changes no state the other outcome needs (the embedding into a
// free row, the QKV projection into its workspace) behind the head's kernels, so that it runs while the host
// still waits for the outcome and decides; when the next calls ask for exactly that work it is not issued again,
// otherwise it is dropped.  Results are the same either way.
enum { AHEAD_NONE = 0, AHEAD_LAYER = 1, AHEAD_TOKEN = 2 };
struct Ahead { int32_t kind, layer, row0, m; };

struct Backend {
    virtual ~Backend() {}
    // hint for the next exit_head / verify call only
    virtual void expect(const Ahead &) {}
    // Full-depth pass over prompt tokens [0, n): "KV cache <- LM(x)".
    virtual int prefill(const int32_t *tokens, int32_t n) = 0;
    // hidden row `row` <- embedding of token
    virtual int embed(int32_t token, int32_t row) = 0;
    // layer `layer` over hidden rows [row0, row0 + m) at positions pos0 .. pos0 + m - 1
    virtual int layer_step(int32_t layer, int32_t row0, int32_t m, int32_t pos0) = 0;
    // the same rows through layers first_layer .. first_layer + count - 1, one after the other
    virtual int layer_steps(int32_t first_layer, int32_t count, int32_t row0, int32_t m, int32_t pos0) {
        for (int32_t l = first_layer; l < first_layer + count; ++l) {
            const int rc = layer_step(l, row0, m, pos0);
            if (rc != AD_OK) return rc;
        }
        return AD_OK;
    }
    // Eq. 1 at temperature 0 on one row; the result must be final when the call returns
    virtual int exit_head(int32_t layer, int32_t row, int32_t pos, int32_t *token, float *conf) = 0;
    // Eq. 2 at temperature 0 on rows [0, m)
    virtual int verify(int32_t m, int32_t pos0, const int32_t *draft, int32_t *n_accept, int32_t *next, int32_t *row_argmax) = 0;
    // Sampled decoding (temperature > 0).  Eq. 1 with the token drawn from softmax(z / temperature) by the uniform
    // draw u; prob is that token's probability.  The backend keeps the row's distribution for verify_sampled.
    virtual int sample_head(int32_t, int32_t, int32_t, float, float, int32_t *, float *) { return AD_ESTATE; }
    // Eq. 2 over rows [0, m): draft[k] was drawn at row k; u_accept[k], u_resample[k] belong to it; u_final draws
    // the next token if nothing is rejected.  ratio[k]: p*(t) / p_draft(t) of the drafts that were checked, else 0.
    virtual int verify_sampled(int32_t, int32_t, const int32_t *, float, const float *, const float *, float, int32_t *, int32_t *,
                               float *) { return AD_ESTATE; }
    virtual int truncate(int32_t new_len) = 0;
};

struct SchedConfig {
    int32_t n_layers;
    int32_t n_exit;
    int32_t exit_layers[AD_MAX_EXIT];
    int32_t m_max;
};

// Returns an ad_status.  out_tokens must hold max_new entries.
int run_algorithm1(Backend &be, const SchedConfig &cfg, const ad_gen_params &gp, const int32_t *prompt, int32_t n_prompt,
                   int32_t *out_tokens, int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events,
                   int64_t *n_events);

}  // namespace ad
