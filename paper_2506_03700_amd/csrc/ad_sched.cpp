// Algorithm 1 of arxiv 2506.03700 as a host-side schedule over a Backend (see ad_sched.h).
//
// Bookkeeping.  Between two verifications the scheduler holds the "open" tokens: the early-predicted
// tokens that still owe their deeper layers, oldest first, followed by the current token.  Token k of
// that list has been through depth[k] layers.  A token leaves the layer loop only at a head layer and
// the next token starts again at layer 1, so when the current token reaches layer l every open token
// has depth >= l-1, and those with depth == l-1 form the tail of the list: that tail is the pending
// list P[l] of the paper, a run of consecutive positions that continues layer l's cache.
//
// Points the listing leaves open, and what is done here:
//  * a token is removed from P[l] once layer l has processed it (Fig. 2, left: each token passes each
//    layer once);
//  * the exit test happens only at layers that carry a head (all below the last layer); the last layer
//    always verifies;
//  * the prompt is prefilled without its last token, which becomes the first current token;
//  * the threshold test is strict (Eq. 1), on the greedy token's softmax probability;
//  * at most max_pending early predictions stay unverified (App. D); at the cap the current token runs to
//    the last layer;
//  * generation stops after max_new verified tokens: a token that would be the last is not drafted, and
//    an early prediction equal to eos_id is not taken, so EOS is only ever emitted by the last layer;
//  * sampled decoding (temperature > 0): the head's token is drawn from its distribution and the probability
//    compared with gamma is that token's; the verification applies Eq. 2 in its general form.  The uniform
//    draws come from the caller's table, one row per position and one column per use (exit head i, final
//    layer, acceptance, replacement), so that a position that samples at several heads uses fresh draws;
//  * before a greedy head evaluation the backend is told what follows under the expected outcome (Backend::expect),
//    so that it can issue the start of that work before the outcome is known; the schedule itself, and every
//    result, is the same with and without it;
//  * ablation switches: head_mask switches exit heads off (one bit left = the fixed-layer variant); no_verify keeps
//    every early prediction unchecked and lets the last layer produce only the next token from the newest row.
#include "ad_sched.h"

#include <string.h>

namespace ad {

namespace {

struct Trace {
    ad_event *ev;
    int64_t cap, n;
    void add(int32_t kind, int32_t layer, int32_t pos, int32_t m, int32_t token, int32_t flag, float conf) {
        if (ev && n < cap) ev[n] = ad_event{kind, layer, pos, m, token, flag, conf, 0.0f};
        ++n;
    }
};

int head_slot(const SchedConfig &c, int32_t layer) {
    for (int32_t i = 0; i < c.n_exit; ++i)
        if (c.exit_layers[i] == layer) return i;
    return -1;
}

}  // namespace

int run_algorithm1(Backend &be, const SchedConfig &cfg, const ad_gen_params &gp, const int32_t *prompt, int32_t n_prompt,
                   int32_t *out_tokens, int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events,
                   int64_t *n_events) {
    if (!prompt || !out_tokens || !n_out || n_prompt < 1 || gp.max_new < 1) return AD_EINVAL;
    if (gp.max_pending < 0 || gp.max_pending + 1 > cfg.m_max) return AD_ERANGE;
    const int32_t L = cfg.n_layers;
    const bool sampled = gp.temperature > 0.0f;
    if (sampled && !gp.uniforms) return AD_EINVAL;
    const int32_t ucols = cfg.n_exit + 3;
    ad_stats st;
    memset(&st, 0, sizeof st);
    Trace tr{events, max_events, 0};

    int rc = be.truncate(0);
    if (rc == AD_OK && n_prompt > 1) rc = be.prefill(prompt, n_prompt - 1);
    if (rc != AD_OK) return rc;

    // open tokens
    int32_t open_pos[AD_M_MAX], open_tok[AD_M_MAX], open_depth[AD_M_MAX], row_arg[AD_M_MAX];
    int32_t n_open = 0;
    int32_t cur = prompt[n_prompt - 1], pos = n_prompt - 1;
    int32_t n_emitted = 0;      // tokens in out_tokens, verified or not
    bool finished = false;
    const bool issue_ahead = !gp.no_issue_ahead && !sampled && !gp.no_verify;
    bool last_take[AD_MAX_EXIT] = {};

    while (!finished) {
        open_pos[n_open] = pos;
        open_tok[n_open] = cur;
        open_depth[n_open] = 0;
        if ((rc = be.embed(cur, n_open)) != AD_OK) return rc;
        ++n_open;
        const bool may_exit = (n_open - 1 < gp.max_pending) && (n_emitted + 1 < gp.max_new);
        bool exited = false;

        // an exit head is evaluated after layer ll
        auto head_due = [&](int32_t ll) {
            const int32_t sl = head_slot(cfg, ll);
            const bool on = sl >= 0 && (gp.head_mask == 0 || ((gp.head_mask >> sl) & 1));
            return ll < L && may_exit && on && (!gp.forced_exit || gp.forced_exit[pos] == ll);
        };
        for (int32_t l = 1; l <= L && !exited; ++l) {
            int32_t first = n_open - 1;
            while (first > 0 && open_depth[first - 1] == l - 1) --first;
            const int32_t m = n_open - first;
            // the same rows go through the following layers too, up to the layer after which a head is evaluated or the
            // deferred rows of an earlier token join: the backend gets that stretch of layers as one call
            const int32_t l0 = l;
            while (l < L && !head_due(l) && !(first > 0 && open_depth[first - 1] == l)) ++l;
            if ((rc = be.layer_steps(l0, l - l0 + 1, first, m, open_pos[first])) != AD_OK) return rc;
            for (int32_t k = first; k < n_open; ++k) open_depth[k] = l;
            for (int32_t ll = l0; ll <= l; ++ll) {
                ++st.layer_steps;
                st.layer_step_rows += m;
                ++st.steps_by_m[m];
                tr.add(AD_EV_LAYER_STEP, ll, open_pos[first], m, 0, 0, 0.0f);
            }

            const int32_t slot = head_slot(cfg, l);
            if (head_due(l)) {
                int32_t tok = -1;
                float conf = 0.0f;
                if (sampled) {
                    rc = be.sample_head(l, n_open - 1, pos, gp.temperature, gp.uniforms[(size_t)pos * ucols + slot], &tok, &conf);
                } else {
                    if (issue_ahead) {
                        // expected outcome: the forced one, else what this head decided last time
                        if (gp.forced_exit || last_take[slot]) {
                            be.expect(Ahead{AHEAD_TOKEN, 1, n_open, 1});
                        } else {
                            int32_t f2 = n_open - 1;       // the rows of layer l + 1: those at depth l
                            while (f2 > 0 && open_depth[f2 - 1] == l) --f2;
                            be.expect(Ahead{AHEAD_LAYER, l + 1, f2, n_open - f2});
                        }
                    }
                    rc = be.exit_head(l, n_open - 1, pos, &tok, &conf);
                }
                if (rc != AD_OK) return rc;
                ++st.head_evals;
                bool take = gp.forced_exit ? true : (conf > gp.gamma);
                if (gp.scripted_draft && gp.scripted_draft[pos] >= 0) tok = gp.scripted_draft[pos];
                if (tok == gp.eos_id) take = false;
                last_take[slot] = take;
                tr.add(AD_EV_HEAD, l, pos, 1, tok, take ? 1 : 0, conf);
                if (take) {
                    out_tokens[n_emitted++] = tok;
                    ++st.early_preds;
                    cur = tok;
                    ++pos;
                    exited = true;
                }
            }
        }
        if (exited) continue;

        // the current token reached the last layer: every open token is complete, verify the drafts
        int32_t n_accept = 0, next = -1;
        const int32_t n_draft = n_open - 1;
        if (gp.no_verify) {
            // ablation: the drafts stand; the final head on the newest row gives the next token
            float conf = 0.0f;
            if (sampled)
                rc = be.sample_head(L, n_open - 1, pos, gp.temperature, gp.uniforms[(size_t)pos * ucols + cfg.n_exit], &next, &conf);
            else
                rc = be.exit_head(L, n_open - 1, pos, &next, &conf);
            if (rc != AD_OK) return rc;
            n_accept = n_draft;
            ++st.verifies;
            tr.add(AD_EV_VERIFY, L, open_pos[0], n_open, next, n_accept, 0.0f);
            for (int32_t k = 0; k < n_open; ++k) tr.add(AD_EV_VERIFY_ROW, L, open_pos[k], 1, k == n_open - 1 ? next : -1, -1, 0.0f);
        } else if (!sampled) {
            // whatever the verification keeps, its next token starts in row 0 (unless it is certainly the last one)
            if (issue_ahead && n_emitted - n_draft + 1 < gp.max_new) be.expect(Ahead{AHEAD_TOKEN, 1, 0, 1});
            if ((rc = be.verify(n_open, open_pos[0], open_tok + 1, &n_accept, &next, row_arg)) != AD_OK) return rc;
            ++st.verifies;
            tr.add(AD_EV_VERIFY, L, open_pos[0], n_open, next, n_accept, 0.0f);
            for (int32_t k = 0; k < n_open; ++k) {
                const int32_t cmp = (k < n_draft && k <= n_accept) ? (row_arg[k] == open_tok[k + 1] ? 1 : 0) : -1;
                tr.add(AD_EV_VERIFY_ROW, L, open_pos[k], 1, row_arg[k], cmp, 0.0f);
            }
        } else {
            float u_acc[AD_M_MAX], u_res[AD_M_MAX], ratio[AD_M_MAX];
            for (int32_t k = 0; k < n_draft; ++k) {
                u_acc[k] = gp.uniforms[(size_t)open_pos[k] * ucols + cfg.n_exit + 1];
                u_res[k] = gp.uniforms[(size_t)open_pos[k] * ucols + cfg.n_exit + 2];
                ratio[k] = 0.0f;
            }
            const float u_final = gp.uniforms[(size_t)open_pos[n_open - 1] * ucols + cfg.n_exit];
            if ((rc = be.verify_sampled(n_open, open_pos[0], open_tok + 1, gp.temperature, u_acc, u_res, u_final, &n_accept, &next, ratio)) != AD_OK)
                return rc;
            ++st.verifies;
            tr.add(AD_EV_VERIFY, L, open_pos[0], n_open, next, n_accept, 0.0f);
            for (int32_t k = 0; k < n_open; ++k) {
                const bool checked = k < n_draft && k <= n_accept;
                const int32_t tok = (k == n_accept) ? next : (k < n_accept ? open_tok[k + 1] : -1);
                tr.add(AD_EV_VERIFY_ROW, L, open_pos[k], 1, tok, checked ? (k < n_accept ? 1 : 0) : -1, checked ? ratio[k] : 0.0f);
            }
        }
        if (n_accept < n_draft) {
            ++st.rejections;
            st.rolled_back += n_draft - n_accept - 1;
        }
        n_emitted = n_emitted - n_draft + n_accept;
        out_tokens[n_emitted++] = next;
        pos = open_pos[n_accept] + 1;
        if ((rc = be.truncate(pos)) != AD_OK) return rc;
        cur = next;
        n_open = 0;
        if (n_emitted >= gp.max_new || next == gp.eos_id) finished = true;
    }
    st.tokens = n_emitted;
    *n_out = n_emitted;
    if (stats) {
        const int64_t keep = stats->bytes_algorithmic;   // filled in by the caller's backend
        *stats = st;
        stats->bytes_algorithmic = keep;
    }
    if (n_events) *n_events = tr.n;
    return AD_OK;
}

}  // namespace ad
