// CPU-only test hook for the host scheduler: runs Algorithm 1 over a scripted backend whose "model" is a
// table of head outputs per position, so that every scheduling path (exit, cap, budget flush, rejection,
// rollback) can be driven from a test without a GPU.  Built into libad_sched_test.so, never into the
// product library.
#include <string.h>

#include <vector>

#include "ad_sched.h"

namespace {

// the calls of Backend::layer_steps of the last run: (first layer, layers, first row, rows, first position)
std::vector<int32_t> g_stretches;

// the hints of Backend::expect of the last run: (kind, layer, first row, rows, 1 if the calls that followed the
// head evaluation asked for exactly the hinted work, else 0)
std::vector<int32_t> g_hints;

struct Scripted : ad::Backend {
    ad::Ahead hint{ad::AHEAD_NONE, 0, 0, 0}, watch{ad::AHEAD_NONE, 0, 0, 0};
    bool watch_embedded = false;
    void expect(const ad::Ahead &a) override { hint = a; }
    void head_called() { watch = hint; hint.kind = ad::AHEAD_NONE; watch_embedded = false; }
    void settle(bool hit) {
        const int32_t rec[5] = {watch.kind, watch.layer, watch.row0, watch.m, hit ? 1 : 0};
        g_hints.insert(g_hints.end(), rec, rec + 5);
        watch.kind = ad::AHEAD_NONE;
    }

    int32_t n_layers, n_exit, max_pos;
    const int32_t *exit_layers;
    // table mode: head_tok/head_conf are [max_pos][n_exit] and final_tok is [max_pos], indexed by position.
    // sequence mode: the k-th exit_head call returns head_tok[k], head_conf[k]; the verify calls consume
    // final_tok in order, one entry per row (for replaying a recorded run, where a position can be visited
    // again with a different token after a rollback).
    int32_t seq_mode, n_head, n_final;
    int32_t head_cursor = 0, final_cursor = 0;
    const int32_t *head_tok;
    const float *head_conf;
    const int32_t *final_tok;
    int32_t len[256];
    int32_t row_pos[AD_M_MAX];
    int fail_code = 0;

    int prefill(const int32_t *, int32_t n) override {
        for (int l = 0; l < n_layers; ++l) len[l] = n;
        return AD_OK;
    }
    int embed(int32_t, int32_t row) override {
        if (watch.kind == ad::AHEAD_TOKEN && !watch_embedded && row == watch.row0) watch_embedded = true;
        else if (watch.kind != ad::AHEAD_NONE) settle(false);
        return AD_OK;
    }
    int layer_step(int32_t layer, int32_t row0, int32_t m, int32_t pos0) override {
        if (layer < 1 || layer > n_layers || m < 1 || row0 + m > AD_M_MAX) return AD_ERANGE;
        if (pos0 != len[layer - 1]) return AD_ESTATE;                 // must continue the layer's cache
        if (layer > 1 && len[layer - 1] + m > len[layer - 2]) return AD_ESTATE;   // a layer never overtakes the one below
        if (pos0 + m > max_pos) return AD_ERANGE;
        for (int i = 0; i < m; ++i) row_pos[row0 + i] = pos0 + i;
        len[layer - 1] += m;
        return AD_OK;
    }
    int layer_steps(int32_t first_layer, int32_t count, int32_t row0, int32_t m, int32_t pos0) override {
        const int32_t rec[5] = {first_layer, count, row0, m, pos0};
        g_stretches.insert(g_stretches.end(), rec, rec + 5);
        if (watch.kind != ad::AHEAD_NONE)
            settle(first_layer == watch.layer && row0 == watch.row0 && m == watch.m && (watch.kind == ad::AHEAD_LAYER || watch_embedded));
        return ad::Backend::layer_steps(first_layer, count, row0, m, pos0);
    }
    int exit_head(int32_t layer, int32_t row, int32_t pos, int32_t *token, float *conf) override {
        head_called();
        if (layer == n_layers && !seq_mode) {
            // the final head on one row (a run without verification asks for it): the scripted final token
            if (row_pos[row] != pos || len[n_layers - 1] != pos + 1) return AD_ESTATE;
            *token = final_tok[pos];
            *conf = 1.0f;
            return AD_OK;
        }
        int slot = -1;
        for (int i = 0; i < n_exit; ++i)
            if (exit_layers[i] == layer) slot = i;
        if (slot < 0 || row_pos[row] != pos) return AD_ESTATE;
        if (seq_mode) {
            if (head_cursor >= n_head) return AD_ERANGE;
            *token = head_tok[head_cursor];
            *conf = head_conf[head_cursor++];
            return AD_OK;
        }
        *token = head_tok[(size_t)pos * n_exit + slot];
        *conf = head_conf[(size_t)pos * n_exit + slot];
        return AD_OK;
    }
    int verify(int32_t m, int32_t pos0, const int32_t *draft, int32_t *n_accept, int32_t *next, int32_t *row_argmax) override {
        head_called();
        for (int l = 1; l < n_layers; ++l)
            if (len[l] != len[0]) return AD_ESTATE;                   // every layer must have caught up
        if (len[0] != pos0 + m) return AD_ESTATE;
        int acc = m - 1;
        if (seq_mode && final_cursor + m > n_final) return AD_ERANGE;
        for (int j = 0; j < m; ++j) row_argmax[j] = seq_mode ? final_tok[final_cursor + j] : final_tok[pos0 + j];
        if (seq_mode) final_cursor += m;
        for (int j = 0; j < m - 1; ++j)
            if (row_argmax[j] != draft[j]) { acc = j; break; }
        *n_accept = acc;
        *next = row_argmax[acc];
        return AD_OK;
    }
    // Sampled decoding over the same tables: the "drawn" token and its probability are the scripted head outputs
    // (the draw is ignored); draft k is accepted iff u_accept[k] < accept_below; the replacement after a rejection
    // and the next token after a clean run are the scripted final tokens.
    float accept_below = 0.5f;
    float last_u_head = -1.0f, last_u_final = -1.0f, last_u_accept0 = -1.0f, last_u_resample0 = -1.0f;
    int sample_head(int32_t layer, int32_t row, int32_t pos, float, float u, int32_t *token, float *prob) override {
        last_u_head = u;
        return exit_head(layer, row, pos, token, prob);
    }
    int verify_sampled(int32_t m, int32_t pos0, const int32_t *, float, const float *u_accept, const float *u_resample, float u_final,
                       int32_t *n_accept, int32_t *next, float *ratio) override {
        for (int l = 1; l < n_layers; ++l)
            if (len[l] != len[0]) return AD_ESTATE;
        if (len[0] != pos0 + m) return AD_ESTATE;
        if (seq_mode) return AD_ESTATE;
        last_u_final = u_final;
        if (m > 1) { last_u_accept0 = u_accept[0]; last_u_resample0 = u_resample[0]; }
        int acc = m - 1;
        for (int j = 0; j < m - 1; ++j) {
            ratio[j] = accept_below;
            if (!(u_accept[j] < accept_below)) { acc = j; break; }
        }
        *n_accept = acc;
        *next = final_tok[pos0 + acc];
        return AD_OK;
    }
    int truncate(int32_t new_len) override {
        for (int l = 0; l < n_layers; ++l)
            if (len[l] > new_len) len[l] = new_len;
        return AD_OK;
    }
};

}  // namespace

extern "C" int ad_sched_test_run(int32_t n_layers, int32_t n_exit, const int32_t *exit_layers, int32_t m_max, int32_t max_pos,
                                 int32_t seq_mode, int32_t n_head, int32_t n_final,
                                 const int32_t *head_tok, const float *head_conf, const int32_t *final_tok,
                                 const ad_gen_params *gp, const int32_t *prompt, int32_t n_prompt, int32_t *out_tokens,
                                 int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events, int64_t *n_events,
                                 float *last_draws /* NULL, or [4]: the head, final, first-acceptance and first-replacement
                                                      draws the backend saw last in a sampled run */) {
    if (n_layers < 1 || n_layers > 256 || n_exit < 0 || n_exit > AD_MAX_EXIT) return AD_EINVAL;
    g_stretches.clear();
    g_hints.clear();
    Scripted be;
    be.n_layers = n_layers; be.n_exit = n_exit; be.max_pos = max_pos; be.exit_layers = exit_layers;
    be.head_tok = head_tok; be.head_conf = head_conf; be.final_tok = final_tok;
    be.seq_mode = seq_mode; be.n_head = n_head; be.n_final = n_final;
    memset(be.len, 0, sizeof be.len);
    ad::SchedConfig sc;
    memset(&sc, 0, sizeof sc);
    sc.n_layers = n_layers; sc.n_exit = n_exit; sc.m_max = m_max;
    for (int i = 0; i < n_exit; ++i) sc.exit_layers[i] = exit_layers[i];
    const int rc = ad::run_algorithm1(be, sc, *gp, prompt, n_prompt, out_tokens, n_out, stats, events, max_events, n_events);
    if (be.watch.kind != ad::AHEAD_NONE) be.settle(false);      // hinted work that the end of the run left unasked
    if (last_draws) {
        last_draws[0] = be.last_u_head; last_draws[1] = be.last_u_final; last_draws[2] = be.last_u_accept0; last_draws[3] = be.last_u_resample0;
    }
    return rc;
}

// The stretches of layers the scheduler handed to the backend in the last ad_sched_test_run of this process:
// copies up to max_records records of 5 int32 (first layer, layers, first row, rows, first position) and returns
// how many there were.
extern "C" int64_t ad_sched_test_stretches(int32_t *out, int64_t max_records) {
    const int64_t n = (int64_t)(g_stretches.size() / 5);
    for (int64_t i = 0; i < n && i < max_records; ++i)
        for (int k = 0; k < 5; ++k) out[i * 5 + k] = g_stretches[(size_t)i * 5 + k];
    return n;
}

// The hints the scheduler gave before the head evaluations of the last run, in order: records of 5 int32 (kind,
// layer, first row, rows, 1 if the calls after the evaluation asked for exactly that work).
extern "C" int64_t ad_sched_test_hints(int32_t *out, int64_t max_records) {
    const int64_t n = (int64_t)(g_hints.size() / 5);
    for (int64_t i = 0; i < n && i < max_records; ++i)
        for (int k = 0; k < 5; ++k) out[i * 5 + k] = g_hints[(size_t)i * 5 + k];
    return n;
}
