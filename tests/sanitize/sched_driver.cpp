// Driver for the AddressSanitizer + UndefinedBehaviorSanitizer build of the host scheduler (ad_sched.cpp) over the
// scripted backend of ad_sched_testhook.cpp: Algorithm 1 with random head tables over many layer counts, head
// placements, caps, thresholds, forced schedules, scripted drafts, end-of-sequence tokens, sampled decoding and
// the ablation switches, with event buffers smaller than the run.  The results are checked by the Python tests;
// this program only has to run clean under the sanitizers.  Exit status 0 = ran through.
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <vector>

#include "../../include/adadecode.h"

extern "C" int ad_sched_test_run(int32_t n_layers, int32_t n_exit, const int32_t *exit_layers, int32_t m_max, int32_t max_pos,
                                 int32_t seq_mode, int32_t n_head, int32_t n_final, const int32_t *head_tok, const float *head_conf,
                                 const int32_t *final_tok, const ad_gen_params *gp, const int32_t *prompt, int32_t n_prompt,
                                 int32_t *out_tokens, int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events,
                                 int64_t *n_events, float *last_draws);
extern "C" int64_t ad_sched_test_stretches(int32_t *out, int64_t max_records);

static uint64_t s = 0x9E3779B97F4A7C15ull;
static double uniform() { s ^= s << 13; s ^= s >> 7; s ^= s << 17; return (double)(s >> 11) / 9007199254740992.0; }

#define CHECK(c) do { if (!(c)) { fprintf(stderr, "driver check failed: %s (line %d)\n", #c, __LINE__); exit(2); } } while (0)

int main() {
    int runs = 0;
    for (int n_layers : {1, 2, 4, 7, 32})
        for (int n_exit = 0; n_exit <= 3 && n_exit < n_layers; ++n_exit)
            for (int m_max : {1, 3, 8})
                for (int variant = 0; variant < 7; ++variant) {
                    int32_t exits[AD_MAX_EXIT] = {0};
                    for (int i = 0; i < n_exit; ++i) exits[i] = 1 + (i * (n_layers - 1)) / n_exit;     // ascending, < n_layers
                    const int max_new = 40, n_prompt = 1 + (int)(uniform() * 6), max_pos = n_prompt + max_new + 1;
                    const int vocab = 11;                                   // small: drafts are often right by chance
                    std::vector<int32_t> head_tok((size_t)max_pos * (n_exit ? n_exit : 1)), final_tok(max_pos), prompt(n_prompt), script(max_pos, -1);
                    std::vector<float> head_conf(head_tok.size()), u((size_t)max_pos * (n_exit + 3));
                    std::vector<uint8_t> forced(max_pos, 0);
                    for (auto &t : final_tok) t = (int32_t)(uniform() * vocab);
                    for (size_t i = 0; i < head_tok.size(); ++i) {
                        head_tok[i] = uniform() < 0.6 ? final_tok[i / (n_exit ? n_exit : 1)] : (int32_t)(uniform() * vocab);
                        head_conf[i] = (float)uniform();
                    }
                    for (auto &t : prompt) t = (int32_t)(uniform() * vocab);
                    for (auto &x : u) x = (float)(uniform() * 0.999);
                    for (int i = 0; i < max_pos; ++i) {
                        if (n_exit && uniform() < 0.6) forced[i] = (uint8_t)exits[(int)(uniform() * n_exit)];
                        if (uniform() < 0.2) script[i] = (int32_t)(uniform() * vocab);
                    }
                    ad_gen_params gp;
                    memset(&gp, 0, sizeof gp);
                    gp.gamma = (float)uniform(); gp.max_pending = m_max - 1; gp.max_new = max_new; gp.eos_id = -1;
                    if (variant == 1 || variant == 5) { gp.forced_exit = forced.data(); gp.scripted_draft = script.data(); }
                    if (variant == 2) gp.eos_id = 3;
                    if (variant == 3 || variant == 5) { gp.temperature = 0.5f; gp.uniforms = u.data(); }
                    if (variant == 4) { gp.head_mask = 1; gp.no_verify = 1; }
                    if (variant == 6) gp.max_pending = 0;
                    std::vector<int32_t> out(max_new + AD_M_MAX);
                    std::vector<ad_event> ev(variant == 0 ? 5 : 8192);
                    int32_t n_out = 0;
                    int64_t n_ev = 0;
                    ad_stats st;
                    float draws[4];
                    const int rc = ad_sched_test_run(n_layers, n_exit, exits, m_max, max_pos, 0, (int32_t)head_tok.size(), max_pos,
                                                     head_tok.data(), head_conf.data(), final_tok.data(), &gp, prompt.data(), n_prompt,
                                                     out.data(), &n_out, &st, ev.data(), (int64_t)ev.size(), &n_ev, draws);
                    CHECK(rc == AD_OK);
                    CHECK(n_out >= 1 && n_out <= max_new && st.tokens == n_out && n_ev > 0);
                    std::vector<int32_t> rec(5 * 16);
                    CHECK(ad_sched_test_stretches(rec.data(), 16) > 0);
                    ++runs;
                }
    // argument errors come back as status codes
    ad_gen_params gp;
    memset(&gp, 0, sizeof gp);
    gp.max_new = 4; gp.max_pending = 9;
    int32_t one = 1, n_out = 0, out[16];
    float c = 0.5f;
    ad_stats st;
    int64_t n_ev;
    int32_t ex[1] = {1};
    CHECK(ad_sched_test_run(2, 1, ex, 4, 8, 0, 8, 8, out, &c, out, &gp, &one, 1, out, &n_out, &st, nullptr, 0, &n_ev, nullptr) == AD_ERANGE);
    printf("scheduler driver: %d runs through\n", runs);
    return 0;
}
