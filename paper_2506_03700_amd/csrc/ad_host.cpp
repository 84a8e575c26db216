// C ABI of the library (include/adadecode.h): model and cache objects, argument checks, and the launch
// sequences of the layer step (Algorithm 1's "update KV cache at layer l"), the exit head (Eq. 1) and the
// verification (Eq. 2).  All arithmetic is in the kernels (ad_kernels.hip); this file only lays out
// memory and enqueues work.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <new>
#include <vector>

#include "../../include/adadecode.h"
#include "ad_internal.h"
#include "ad_sched.h"

using namespace ad;

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

int hip_fail(int hip_code, const char *what) {
    return fail(AD_EDEVICE, "%s: %s", what, hip_error_text(hip_code));
}

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

struct LayerPacked {
    char *wqkv, *wo, *wgu, *wd, *attn_norm, *ffn_norm;
};

struct Layout {
    // sizes
    size_t elem;
    int planes;
    int d, dq, dkv, nqkv, f, dh, V;
    int kt_d, kt_q, kt_f;
    size_t sz_wqkv, sz_wo, sz_wgu, sz_wd, sz_norm, sz_embed, sz_head, sz_T;
    // offsets
    std::vector<size_t> layer_off;   // start of each layer's block
    size_t off_embed, off_final_norm, off_head, off_T[AD_MAX_EXIT];
    size_t off_scratch, scratch_bytes;
    size_t total;
};

// The public dtype codes and the kernels' element kinds are the same numbers.
static_assert(AD_F32 == kElemF32 && AD_BF16 == kElemBF16 && AD_F16 == kElemF16, "dtype codes");
static inline int elem_kind(const ad_config &c) { return c.dtype; }

bool config_ok(const ad_config *c, const char **why) {
    *why = "";
    if (!c) { *why = "null config"; return false; }
    if (c->n_layers < 1 || c->d_model < 16 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->d_ffn < 8 || c->vocab < 1) { *why = "non-positive dimension"; return false; }
    if (c->d_model % 16) { *why = "d_model must be a multiple of 16"; return false; }
    if (c->d_ffn % 8) { *why = "d_ffn must be a multiple of 8"; return false; }
    if (c->head_dim != 64 && c->head_dim != 128) { *why = "head_dim must be 64 or 128"; return false; }
    if (c->n_q_heads % c->n_kv_heads) { *why = "n_q_heads must be a multiple of n_kv_heads"; return false; }
    if (c->dtype != AD_F32 && c->dtype != AD_BF16 && c->dtype != AD_F16) { *why = "unknown dtype"; return false; }
    if (c->m_max < 1 || c->m_max > AD_M_MAX) { *why = "m_max must be in 1..8"; return false; }
    if (c->n_exit < 0 || c->n_exit > AD_MAX_EXIT) { *why = "n_exit out of range"; return false; }
    for (int i = 0; i < c->n_exit; ++i) {
        if (c->exit_layers[i] < 1 || c->exit_layers[i] >= c->n_layers) { *why = "exit layer must be in 1..n_layers-1"; return false; }
        if (i && c->exit_layers[i] <= c->exit_layers[i - 1]) { *why = "exit layers must ascend"; return false; }
    }
    if (!(c->rope_base > 0.f) || !(c->rms_eps >= 0.f)) { *why = "bad rope_base / rms_eps"; return false; }
    if (c->d_model > gemm_max_stationary_k(c->dtype == AD_F32 ? 3 : 1)) { *why = "d_model above 8192 (fp32 models: 5120) is not supported"; return false; }
    {
        // the kernels address a packed matrix with a 32-bit byte offset
        const int planes = c->dtype == AD_F32 ? 3 : 1;
        const int64_t d = c->d_model, dq = (int64_t)c->n_q_heads * c->head_dim, dkv = (int64_t)c->n_kv_heads * c->head_dim;
        const size_t lim = (size_t)1 << 32;
        if (packed_bytes(c->vocab, d, planes) >= lim || packed_bytes(2 * (int64_t)c->d_ffn, d, planes) >= lim ||
            packed_bytes(d, c->d_ffn, planes) >= lim || packed_bytes(dq + 2 * dkv, d, planes) >= lim || packed_bytes(d, dq, planes) >= lim) {
            *why = "a weight matrix would take 4 GiB or more in the library's layout (vocab x d_model, 2 d_ffn x d_model, ...)";
            return false;
        }
    }
    return true;
}

void make_layout(const ad_config &c, Layout &L) {
    L.elem = c.dtype == AD_F32 ? 4 : 2;
    L.planes = c.dtype == AD_F32 ? 3 : 1;
    L.d = c.d_model; L.dh = c.head_dim; L.dq = c.n_q_heads * c.head_dim; L.dkv = c.n_kv_heads * c.head_dim;
    L.nqkv = L.dq + 2 * L.dkv; L.f = c.d_ffn; L.V = c.vocab;
    L.kt_d = (L.d + 31) / 32; L.kt_q = (L.dq + 31) / 32; L.kt_f = (L.f + 31) / 32;
    L.sz_wqkv = packed_bytes(L.nqkv, L.d, L.planes);
    L.sz_wo = packed_bytes(L.d, L.dq, L.planes);
    L.sz_wgu = packed_bytes(2 * (int64_t)L.f, L.d, L.planes);
    L.sz_wd = packed_bytes(L.d, L.f, L.planes);
    L.sz_norm = align_up(L.d * L.elem);
    L.sz_embed = align_up((size_t)L.V * L.d * L.elem);
    L.sz_head = packed_bytes(L.V, L.d, L.planes);
    L.sz_T = packed_bytes(L.d, L.d, L.planes);
    size_t off = 0;
    L.layer_off.resize(c.n_layers);
    for (int l = 0; l < c.n_layers; ++l) {
        L.layer_off[l] = off;
        off += L.sz_wqkv + L.sz_wo + L.sz_wgu + L.sz_wd + 2 * L.sz_norm;
    }
    L.off_embed = off; off += L.sz_embed;
    L.off_final_norm = off; off += L.sz_norm;
    L.off_head = off; off += L.sz_head;
    for (int i = 0; i < AD_MAX_EXIT; ++i) { L.off_T[i] = off; if (i < c.n_exit) off += L.sz_T; }
    L.off_scratch = off;
    size_t s = 0;
    s += align_up(act_packed_bytes(L.d));                      // B1 (exit-head transform output)
    s += align_up(act_packed_bytes(L.dq));                     // Bo (attention output)
    s += align_up(act_packed_bytes(L.f));                      // Bg (SwiGLU output)
    s += align_up(act_packed_bytes(L.d));                      // Bx (x' * ffn norm weight, packed by the Wo epilogue)
    s += align_up((size_t)(L.d / 16) * 8 * 4);                 // per-tile sums of squares of x'
    s += align_up(act_packed_bytes(L.d));                      // Bq (y * next layer's attention norm weight, packed by the down epilogue)
    s += align_up((size_t)(L.d / 16) * 8 * 4);                 // per-tile sums of squares of y
    s += align_up((size_t)8 * L.nqkv * 4);                     // qkv
    s += 2 * align_up((size_t)8 * L.d * 4);                    // x1, rows
    s += align_up((size_t)4096 * 8 * 4 * 4);                   // head partials (up to 4096 workgroups)
    s += align_up((size_t)kBarrierWords * 4);                  // grid-barrier counters of the fused layer step
    s += align_up((size_t)64 * 4);                             // sampled verification: (max, sum) per row
    s += 2 * align_up((size_t)AD_M_MAX * L.V * 4);             // sampled decoding: draft and final logits of the open rows
    L.scratch_bytes = s;
    L.total = off + s;
}

}  // namespace

struct Profile {
    bool on = false;
    int32_t kind = AD_PROF_GEMM;
    int32_t period = 1, max_samples = 0;
    int64_t launches = 0, total_bytes = 0;
    std::vector<void *> start, stop;
    std::vector<int64_t> bytes;
};

struct ad_model {
    mutable Profile prof;
    ad_config cfg;
    Layout lay;
    char *ws;
    int n_wg;
    std::vector<LayerPacked> layers;
    char *embed, *final_norm, *head, *T[AD_MAX_EXIT];
    // scratch
    char *B1, *Bo, *Bg, *Bx, *Bq;
    float *ssq, *ssq_q;
    float *qkv, *x1, *rows, *head_part;
    float *samp_stats, *draft_logits, *final_logits;   // sampled decoding
    // pinned host results for ad_generate
    int32_t *pin;         // [0..8) tok, [8] n_accept, [9] next, [16..24) row argmax, [28] the head's done word
    mutable int32_t done_seq = 0;   // last value asked for in the done word (unique per head evaluation of this model)
    float *pin_conf;      // [8]
    // fused layer step: mode, barrier counters (device), barriers completed so far, abort word (pinned host)
    int32_t layer_mode;
    unsigned *bar_ctr;
    mutable unsigned bar_round;
    unsigned *bar_abort;
    long long *layer_trace;   // device buffer for the fused kernel's phase timestamps, or null
};

struct ad_kv {
    const ad_model *model;
    char *storage;
    size_t layer_bytes, half_bytes;
    float *rope;          // [stride][dh/2][2]
    int32_t stride;       // max_pos rounded up to 64: positions per (head, dim) row of V, rows per head of K
    float *part;
    int32_t max_pos;
    std::vector<int32_t> len;
};

extern "C" {

const char *ad_last_error(void) { return g_err; }
const char *ad_version(void) { return "adadecode-gfx950 0.1"; }

size_t ad_workspace_bytes(const ad_config *cfg) {
    const char *why;
    if (!config_ok(cfg, &why)) { fail(AD_EINVAL, "%s", why); return 0; }
    Layout L;
    make_layout(*cfg, L);
    return L.total;
}

ad_status ad_model_create(const ad_config *cfg, const ad_layer_weights *layers, const ad_top_weights *top, void *workspace,
                          size_t workspace_bytes, void *stream, ad_model **out) {
    const char *why;
    if (!config_ok(cfg, &why)) return (ad_status)fail(AD_EINVAL, "ad_model_create: %s", why);
    if (!layers || !top || !workspace || !out) return (ad_status)fail(AD_EINVAL, "ad_model_create: null argument");
    if (((uintptr_t)workspace & 255u) != 0) return (ad_status)fail(AD_EINVAL, "ad_model_create: workspace must be 256-byte aligned");
    if (!top->embed || !top->final_norm || !top->lm_head) return (ad_status)fail(AD_EINVAL, "ad_model_create: null top weight");
    for (int l = 0; l < cfg->n_layers; ++l) {
        const ad_layer_weights &w = layers[l];
        if (!w.attn_norm || !w.wq || !w.wk || !w.wv || !w.wo || !w.ffn_norm || !w.w_gate || !w.w_up || !w.w_down)
            return (ad_status)fail(AD_EINVAL, "ad_model_create: null weight in layer %d", l + 1);
    }
    ad_model *m = new (std::nothrow) ad_model();
    if (!m) return (ad_status)fail(AD_ENOMEM, "ad_model_create: out of host memory");
    m->cfg = *cfg;
    make_layout(*cfg, m->lay);
    const Layout &L = m->lay;
    if (workspace_bytes < L.total) {
        delete m;
        return (ad_status)fail(AD_ENOMEM, "ad_model_create: workspace has %zu bytes, %zu needed", workspace_bytes, L.total);
    }
    int n_cu = 0, rc = device_info(&n_cu);
    if (rc) { delete m; return (ad_status)hip_fail(rc, "device query"); }
    m->n_wg = n_cu;
    m->ws = (char *)workspace;
    const int ek = elem_kind(*cfg);
    const size_t tile_kb = (size_t)L.planes * 1024u;

#define AD_TRY(expr, what) do { int rc_ = (expr); if (rc_) { delete m; return (ad_status)hip_fail(rc_, what); } } while (0)
    AD_TRY(launch_zero(m->ws + L.off_scratch, L.scratch_bytes, stream), "zero scratch");
    m->layers.resize(cfg->n_layers);
    for (int l = 0; l < cfg->n_layers; ++l) {
        char *p = m->ws + L.layer_off[l];
        LayerPacked &lp = m->layers[l];
        lp.wqkv = p; p += L.sz_wqkv;
        lp.wo = p; p += L.sz_wo;
        lp.wgu = p; p += L.sz_wgu;
        lp.wd = p; p += L.sz_wd;
        lp.attn_norm = p; p += L.sz_norm;
        lp.ffn_norm = p;
        const ad_layer_weights &w = layers[l];
        // q, k, v share one packed matrix: q rows first, then k, then v
        AD_TRY(launch_pack_weights(w.wq, nullptr, ek, L.dq, L.d, 0, lp.wqkv, stream), "pack wq");
        AD_TRY(launch_pack_weights(w.wk, nullptr, ek, L.dkv, L.d, 0, lp.wqkv + (size_t)(L.dq / 16) * L.kt_d * tile_kb, stream), "pack wk");
        AD_TRY(launch_pack_weights(w.wv, nullptr, ek, L.dkv, L.d, 0, lp.wqkv + (size_t)((L.dq + L.dkv) / 16) * L.kt_d * tile_kb, stream), "pack wv");
        AD_TRY(launch_pack_weights(w.wo, nullptr, ek, L.d, L.dq, 0, lp.wo, stream), "pack wo");
        AD_TRY(launch_pack_weights(w.w_gate, w.w_up, ek, L.f, L.d, 1, lp.wgu, stream), "pack gate/up");
        AD_TRY(launch_pack_weights(w.w_down, nullptr, ek, L.d, L.f, 0, lp.wd, stream), "pack down");
        AD_TRY(launch_zero(lp.attn_norm, 2 * L.sz_norm, stream), "zero norms");
        AD_TRY(launch_copy(w.attn_norm, lp.attn_norm, align_up(L.d * L.elem, 16), stream), "copy attn_norm");
        AD_TRY(launch_copy(w.ffn_norm, lp.ffn_norm, align_up(L.d * L.elem, 16), stream), "copy ffn_norm");
    }
    m->embed = m->ws + L.off_embed;
    m->final_norm = m->ws + L.off_final_norm;
    m->head = m->ws + L.off_head;
    AD_TRY(launch_copy(top->embed, m->embed, align_up((size_t)L.V * L.d * L.elem, 16), stream), "copy embed");
    AD_TRY(launch_copy(top->final_norm, m->final_norm, align_up(L.d * L.elem, 16), stream), "copy final_norm");
    AD_TRY(launch_pack_weights(top->lm_head, nullptr, ek, L.V, L.d, 0, m->head, stream), "pack lm_head");
    for (int i = 0; i < AD_MAX_EXIT; ++i) {
        m->T[i] = nullptr;
        if (i < cfg->n_exit && top->exit_T && top->exit_T[i]) {
            m->T[i] = m->ws + L.off_T[i];
            AD_TRY(launch_pack_weights(top->exit_T[i], nullptr, ek, L.d, L.d, 0, m->T[i], stream), "pack exit transform");
        }
    }
    char *s = m->ws + L.off_scratch;
    auto take = [&](size_t bytes) { char *p = s; s += align_up(bytes); return p; };
    m->B1 = take(act_packed_bytes(L.d));
    m->Bo = take(act_packed_bytes(L.dq));
    m->Bg = take(act_packed_bytes(L.f));
    m->Bx = take(act_packed_bytes(L.d));
    m->ssq = (float *)take((size_t)(L.d / 16) * 8 * 4);
    m->Bq = take(act_packed_bytes(L.d));
    m->ssq_q = (float *)take((size_t)(L.d / 16) * 8 * 4);
    m->qkv = (float *)take((size_t)8 * L.nqkv * 4);
    m->x1 = (float *)take((size_t)8 * L.d * 4);
    m->rows = (float *)take((size_t)8 * L.d * 4);
    m->head_part = (float *)take((size_t)4096 * 8 * 4 * 4);
    m->bar_ctr = (unsigned *)take((size_t)kBarrierWords * 4);     // zeroed with the rest of the scratch above
    m->bar_round = 0;
    m->samp_stats = (float *)take((size_t)64 * 4);
    m->draft_logits = (float *)take((size_t)AD_M_MAX * L.V * 4);
    m->final_logits = (float *)take((size_t)AD_M_MAX * L.V * 4);
    m->pin = (int32_t *)pinned_alloc(4096);
    if (!m->pin) { delete m; return (ad_status)fail(AD_ENOMEM, "ad_model_create: pinned allocation failed"); }
    m->pin_conf = (float *)(m->pin + 32);
    m->bar_abort = (unsigned *)(m->pin + 64);
    *m->bar_abort = 0;
    m->layer_mode = AD_LAYER_KERNELS;
    m->layer_trace = nullptr;
    {   // set-up for ad_verify_static on this device: the address of the library's static scratch
        float *part = nullptr;
        AD_TRY(static_head_scratch(&part), "address of the static scratch");
    }
    AD_TRY(stream_sync(stream), "model creation");
#undef AD_TRY
    *out = m;
    return AD_OK;
}

ad_status ad_model_destroy(ad_model *m) {
    if (!m) return AD_OK;
    for (void *e : m->prof.start) event_destroy(e);
    for (void *e : m->prof.stop) event_destroy(e);
    pinned_free(m->pin);
    delete m;
    return AD_OK;
}

// ---- KV cache --------------------------------------------------------------------------------------

static size_t rope_table_bytes(const ad_config &c, int32_t max_pos) {
    const size_t stride = ((size_t)max_pos + 63) / 64 * 64;
    return align_up(stride * (c.head_dim / 2) * 2 * 4);
}

static size_t attn_part_bytes(const ad_config &c, int32_t max_pos) {
    const int C = attn_chunk(elem_kind(c), c.head_dim);
    const size_t S = (size_t)(max_pos + C - 1) / C + 1;
    return align_up((size_t)c.n_q_heads * 8 * S * (c.head_dim + 2) * 4);
}

size_t ad_kv_bytes(const ad_config *cfg, int32_t max_pos) {
    const char *why;
    if (!config_ok(cfg, &why) || max_pos < 1) { fail(AD_EINVAL, "ad_kv_bytes: %s", max_pos < 1 ? "max_pos < 1" : why); return 0; }
    const size_t elem = cfg->dtype == AD_F32 ? 4 : 2;
    const size_t stride = ((size_t)max_pos + 63) / 64 * 64;
    const size_t cache = (size_t)cfg->n_layers * 2 * cfg->n_kv_heads * stride * cfg->head_dim * elem;
    return align_up(cache) + attn_part_bytes(*cfg, max_pos) + rope_table_bytes(*cfg, max_pos);
}

ad_status ad_kv_create(const ad_model *model, void *kv_storage, size_t kv_storage_bytes, int32_t max_pos, void *stream, ad_kv **out) {
    if (!model || !kv_storage || !out || max_pos < 1) return (ad_status)fail(AD_EINVAL, "ad_kv_create: bad argument");
    if (((uintptr_t)kv_storage & 255u) != 0) return (ad_status)fail(AD_EINVAL, "ad_kv_create: storage must be 256-byte aligned");
    const size_t need = ad_kv_bytes(&model->cfg, max_pos);
    if (kv_storage_bytes < need) return (ad_status)fail(AD_ENOMEM, "ad_kv_create: storage has %zu bytes, %zu needed", kv_storage_bytes, need);
    ad_kv *kv = new (std::nothrow) ad_kv();
    if (!kv) return (ad_status)fail(AD_ENOMEM, "ad_kv_create: out of host memory");
    const ad_config &c = model->cfg;
    const size_t elem = c.dtype == AD_F32 ? 4 : 2;
    kv->model = model;
    kv->storage = (char *)kv_storage;
    kv->stride = (max_pos + 63) / 64 * 64;
    kv->half_bytes = (size_t)c.n_kv_heads * (size_t)kv->stride * c.head_dim * elem;
    kv->layer_bytes = 2 * kv->half_bytes;
    kv->part = (float *)(kv->storage + align_up((size_t)c.n_layers * kv->layer_bytes));
    kv->rope = (float *)((char *)kv->part + attn_part_bytes(c, max_pos));
    kv->max_pos = max_pos;
    kv->len.assign(c.n_layers, 0);
    // rotary table for every position of this cache; frequencies base^(-2i/dh) in double
    RopeArgs ra;
    ra.table = kv->rope; ra.n_pos = kv->stride; ra.half = c.head_dim / 2;
    for (int i = 0; i < ra.half; ++i) ra.inv_freq[i] = pow((double)c.rope_base, -2.0 * (double)i / (double)c.head_dim);
    int rc = launch_rope_table(ra, stream);
    if (!rc) rc = stream_sync(stream);
    if (rc) { delete kv; return (ad_status)hip_fail(rc, "ad_kv_create: rotary table"); }
    *out = kv;
    return AD_OK;
}

ad_status ad_kv_destroy(ad_kv *kv) { delete kv; return AD_OK; }

ad_status ad_kv_len(const ad_kv *kv, int32_t layer, int32_t *len) {
    if (!kv || !len) return (ad_status)fail(AD_EINVAL, "ad_kv_len: null argument");
    if (layer < 1 || layer > (int32_t)kv->len.size()) return (ad_status)fail(AD_ERANGE, "ad_kv_len: layer %d out of range", layer);
    *len = kv->len[layer - 1];
    return AD_OK;
}

ad_status ad_kv_set_len(ad_kv *kv, int32_t layer, int32_t len) {
    if (!kv) return (ad_status)fail(AD_EINVAL, "ad_kv_set_len: null argument");
    if (layer < 1 || layer > (int32_t)kv->len.size()) return (ad_status)fail(AD_ERANGE, "ad_kv_set_len: layer %d out of range", layer);
    if (len < 0 || len > kv->max_pos) return (ad_status)fail(AD_ERANGE, "ad_kv_set_len: length %d outside 0..%d", len, kv->max_pos);
    kv->len[layer - 1] = len;
    return AD_OK;
}

ad_status ad_kv_truncate(ad_kv *kv, int32_t new_len) {
    if (!kv) return (ad_status)fail(AD_EINVAL, "ad_kv_truncate: null argument");
    if (new_len < 0) return (ad_status)fail(AD_ERANGE, "ad_kv_truncate: negative length");
    for (auto &l : kv->len)
        if (l > new_len) l = new_len;
    return AD_OK;
}

// ---- steps -----------------------------------------------------------------------------------------

// Counts a launch of the profiled kind; returns true if it is to be sampled (the start event is then recorded and
// the caller records p.stop.back() after the launch).
static bool profile_begin(Profile &p, int32_t kind, int64_t bytes, void *stream) {
    if (!p.on || p.kind != kind) return false;
    const bool sample = (p.launches % p.period == 0) && (int32_t)p.bytes.size() < p.max_samples;
    ++p.launches;
    p.total_bytes += bytes;
    if (!sample) return false;
    void *a = event_create(), *b = event_create();
    if (!a || !b) { event_destroy(a); event_destroy(b); return false; }
    p.start.push_back(a); p.stop.push_back(b); p.bytes.push_back(bytes);
    (void)event_record(a, stream);
    return true;
}

// Launches the weight-streaming kernel; when profiling is on, every period-th launch is timed with events.
static int gemm(const ad_model *m, const GemmArgs &g, int64_t rows, int64_t cols, const LaunchCtx &ctx) {
    Profile &p = m->prof;
    const int64_t bytes = rows * cols * (int64_t)m->lay.elem;
    const bool sample = profile_begin(p, AD_PROF_GEMM, bytes, ctx.stream);
    const int rc = launch_gemm(g, m->lay.planes, ctx);
    if (sample) (void)event_record(p.stop.back(), ctx.stream);
    return rc;
}

ad_status ad_embed(const ad_model *m, const int32_t *tokens, int32_t n, void *hidden, void *stream) {
    if (!m || !tokens || !hidden) return (ad_status)fail(AD_EINVAL, "ad_embed: null argument");
    if (n < 1 || n > m->cfg.m_max) return (ad_status)fail(AD_ERANGE, "ad_embed: m = %d outside 1..%d", n, m->cfg.m_max);
    EmbedArgs a;
    memset(&a, 0, sizeof a);
    a.table = m->embed; a.elem = elem_kind(m->cfg); a.d = m->cfg.d_model; a.m = n; a.out = (float *)hidden;
    for (int i = 0; i < n; ++i) {
        if (tokens[i] < 0 || tokens[i] >= m->cfg.vocab) return (ad_status)fail(AD_ERANGE, "ad_embed: token %d outside the vocabulary", tokens[i]);
        a.tok[i] = tokens[i];
    }
    int rc = launch_embed(a, stream);
    return rc ? (ad_status)hip_fail(rc, "ad_embed") : AD_OK;
}

// One row's embedding, the token id read by the kernel from *token_src (written by an earlier kernel on the stream).
static int embed_from(const ad_model *m, const int32_t *token_src, void *hidden, void *stream) {
    EmbedArgs a;
    memset(&a, 0, sizeof a);
    a.table = m->embed; a.elem = elem_kind(m->cfg); a.d = m->cfg.d_model; a.m = 1; a.out = (float *)hidden;
    a.tok_src = token_src; a.vocab = m->cfg.vocab;
    const int rc = launch_embed(a, stream);
    return rc ? hip_fail(rc, "embedding issued ahead") : AD_OK;
}

// The fused layer step's grid barrier gave up in an earlier launch (it never should: the grid is co-resident):
// report it once, and put the counters back in order for later calls.
static int fused_health(const ad_model *m, void *stream) {
    if (*(volatile unsigned *)m->bar_abort == 0) return AD_OK;
    int rc = stream_sync(stream);
    if (!rc) rc = launch_zero(m->bar_ctr, (size_t)kBarrierWords * 4, stream);
    if (!rc) rc = stream_sync(stream);
    *(volatile unsigned *)m->bar_abort = 0;
    m->bar_round = 0;
    if (rc) return hip_fail(rc, "fused layer step: resetting the grid barrier");
    return fail(AD_EDEVICE, "fused layer step: a grid barrier timed out in an earlier call; its result and the KV cache rows it appended are "
                            "invalid (take the cache back to its length before that call)");
}

static int64_t layer_step_bytes(const ad_config &c, int32_t ctx, int32_t m) {
    const int64_t s = c.dtype == AD_F32 ? 4 : 2;
    const int64_t dq = (int64_t)c.n_q_heads * c.head_dim, dkv = (int64_t)c.n_kv_heads * c.head_dim, d = c.d_model, f = c.d_ffn;
    const int64_t w = ((dq + 2 * dkv) * d + d * dq + 3 * d * f) * s;
    return w + 2 * dkv * s * ((int64_t)ctx + m) + 2 * dkv * s * m;
}

// Step 1 of a layer: q, k, v = W (RMSNorm(x)).  The norm is fused into the GEMM (B operand built from x in its
// prologue, or taken packed, with the sums of squares, from the previous layer's last step).
static void qkv_args(const ad_model *m, int32_t ly, const void *hidden, int32_t n, bool from_prev, GemmArgs &gq) {
    const ad_config &c = m->cfg;
    const Layout &L = m->lay;
    const LayerPacked &lp = m->layers[ly - 1];
    const int ek = elem_kind(c);
    memset(&gq, 0, sizeof gq);
    gq.elem = ek;
    gq.W = lp.wqkv; gq.NT = L.nqkv / 16; gq.KT = L.kt_d; gq.N = L.nqkv; gq.K = L.d; gq.m = n; gq.mode = GEMM_STATIONARY;
    gq.inv_dim = 1.0f / (float)L.d; gq.eps = c.rms_eps;
    if (from_prev) { gq.B = m->Bq; gq.ssq_in = m->ssq_q; gq.ssq_tiles = L.d / 16; }
    else { gq.x = (const float *)hidden; gq.ldx = L.d; gq.norm_w = lp.attn_norm; gq.norm_elem = ek; }
    gq.epi = EPI_STORE; gq.out = m->qkv; gq.ld = L.nqkv;
}

// Step 1 of layer `layer` over n rows, issued on its own ahead of the rest of the step (which layer_steps then runs
// with first_qkv_issued set, provided nothing else used the q/k/v workspace in between).  Separate-kernel mode only.
static int qkv_ahead(const ad_model *m, int32_t layer, const void *hidden, int32_t n, void *stream) {
    GemmArgs gq;
    qkv_args(m, layer, hidden, n, false, gq);
    const int rc = gemm(m, gq, m->lay.nqkv, m->lay.d, LaunchCtx{stream, m->n_wg});
    return rc ? hip_fail(rc, "layer step: qkv issued ahead") : AD_OK;
}

// Layers layer .. layer + count - 1 over the same rows.  The fused mode runs them in one launch (the layers' weights
// and caches are laid out at a constant distance from one layer to the next); otherwise one layer at a time.
static int layer_steps(const ad_model *m, ad_kv *kv, int32_t layer, int32_t count, void *hidden, const int32_t *pos, int32_t n,
                       void *stream, const char *who, bool first_qkv_issued = false) {
    if (!m || !kv || !hidden || !pos) return fail(AD_EINVAL, "%s: null argument", who);
    if (kv->model != m) return fail(AD_EINVAL, "%s: cache belongs to another model", who);
    const ad_config &c = m->cfg;
    if (count < 1 || layer < 1 || layer > c.n_layers - (count - 1))
        return fail(AD_ERANGE, "%s: layers %d..%d outside 1..%d", who, layer, layer + count - 1, c.n_layers);
    if (n < 1 || n > c.m_max) return fail(AD_ERANGE, "%s: m = %d outside 1..%d", who, n, c.m_max);
    for (int i = 1; i < n; ++i)
        if (pos[i] != pos[0] + i) return fail(AD_ESTATE, "%s: positions are not consecutive", who);
    for (int32_t l = layer; l < layer + count; ++l)
        if (pos[0] != kv->len[l - 1]) return fail(AD_ESTATE, "%s: pos[0] = %d but layer %d's cache ends at %d", who, pos[0], l, kv->len[l - 1]);
    if (pos[0] < 0 || pos[n - 1] >= kv->max_pos) return fail(AD_ERANGE, "%s: position %d beyond max_pos %d", who, pos[n - 1], kv->max_pos);
    const Layout &L = m->lay;
    const LaunchCtx ctx{stream, m->n_wg};
    const int ek = elem_kind(c);
    const bool fused = m->layer_mode == AD_LAYER_FUSED;
    int rc;
    // The arguments of layer ly's five steps.  from_prev: the layer before it ran in this same call and its down
    // projection left this layer's QKV input behind (see step 5); feeds_next: this layer's down projection does
    // that for the layer after it.
    GemmArgs gq, go, gg, gd;
    AttnArgs a;
    auto build = [&](int32_t ly, bool from_prev, bool feeds_next) {
        const LayerPacked &lp = m->layers[ly - 1];
        // 1. q, k, v = W (RMSNorm(x))
        qkv_args(m, ly, hidden, n, from_prev, gq);
        // 2. rotary embedding, KV append, attention (partials + combine)
        memset(&a, 0, sizeof a);
        a.qkv = m->qkv; a.ld = L.nqkv; a.rope = kv->rope + (size_t)pos[0] * (L.dh / 2) * 2;
        a.Kc = kv->storage + (size_t)(ly - 1) * kv->layer_bytes; a.Vc = (char *)a.Kc + kv->half_bytes;
        a.stride = kv->stride; a.pos0 = pos[0]; a.m = n; a.Hq = c.n_q_heads; a.Hkv = c.n_kv_heads; a.dh = L.dh;
        a.C = attn_chunk(ek, L.dh);
        a.S = pos[0] > 0 ? (pos[0] + a.C - 1) / a.C : 1;
        a.part = kv->part; a.Bo = m->Bo; a.Bo_KT = L.kt_q; a.scale = 1.0f / sqrtf((float)L.dh); a.kv_elem = ek;
        attn_finish(a);
        // 3. x' = x + Wo o
        memset(&go, 0, sizeof go);
        go.elem = ek;
        go.W = lp.wo; go.B = m->Bo; go.NT = L.d / 16; go.KT = L.kt_q; go.N = L.d; go.K = L.dq; go.m = n; go.mode = GEMM_STREAMED;
        go.epi = EPI_RESID; go.resid = (const float *)hidden; go.out = m->x1; go.ld = L.d;
        // ... and the Wo epilogue already prepares the gate/up GEMM's input: x' * ffn norm weight packed, sum(x'^2) per tile
        go.Bnext = m->Bx; go.Bnext_KT = L.kt_d; go.next_norm_w = lp.ffn_norm; go.next_norm_elem = ek; go.ssq_out = m->ssq;
        // 4. g = silu(Wg b) * (Wu b), b = RMSNorm(x') fused as in step 1
        memset(&gg, 0, sizeof gg);
        gg.elem = ek;
        gg.W = lp.wgu; gg.NT = (2 * L.f) / 16; gg.KT = L.kt_d; gg.N = 2 * L.f; gg.K = L.d; gg.m = n; gg.mode = GEMM_STATIONARY;
        gg.B = m->Bx; gg.ssq_in = m->ssq; gg.ssq_tiles = go.NT; gg.inv_dim = 1.0f / (float)L.d; gg.eps = c.rms_eps;
        gg.epi = EPI_SWIGLU; gg.Bnext = m->Bg; gg.Bnext_KT = L.kt_f;
        // 5. y = x' + Wd g
        memset(&gd, 0, sizeof gd);
        gd.elem = ek;
        gd.W = lp.wd; gd.B = m->Bg; gd.NT = L.d / 16; gd.KT = L.kt_f; gd.N = L.d; gd.K = L.f; gd.m = n; gd.mode = GEMM_STREAMED;
        gd.epi = EPI_RESID; gd.resid = m->x1; gd.out = (float *)hidden; gd.ld = L.d;
        // ... and, like step 3 for step 4, prepares the next layer's QKV input: y * its attention norm weight packed, sum(y^2) per tile
        if (feeds_next) {
            gd.Bnext = m->Bq; gd.Bnext_KT = L.kt_d; gd.next_norm_w = m->layers[ly].attn_norm; gd.next_norm_elem = ek; gd.ssq_out = m->ssq_q;
        }
    };

    if (!fused) {
        // one kernel per phase, layer after layer
        for (int32_t ly = layer; ly < layer + count; ++ly) {
            build(ly, ly > layer, ly + 1 < layer + count);
            if (!(first_qkv_issued && ly == layer) && (rc = gemm(m, gq, L.nqkv, L.d, ctx))) return hip_fail(rc, "layer step: qkv");
            if ((rc = launch_attn(a, ctx))) return hip_fail(rc, "layer step: attention");
            if ((rc = gemm(m, go, L.d, L.dq, ctx))) return hip_fail(rc, "layer step: wo");
            if ((rc = gemm(m, gg, 2 * (int64_t)L.f, L.d, ctx))) return hip_fail(rc, "layer step: gate/up");
            if ((rc = gemm(m, gd, L.d, L.f, ctx))) return hip_fail(rc, "layer step: down");
        }
    } else {
        // the whole stretch in one persistent kernel
        if (first_qkv_issued) return fail(AD_ESTATE, "%s: the fused layer step runs its own QKV projection", who);
        const LayerPacked &lp = m->layers[layer - 1];
        if ((rc = fused_health(m, stream))) return rc;
        // the stretch's first layer as it runs when it is also the last (nothing handed on), then the two variants
        // that differ for the layers that follow / are followed by another
        FusedArgs f;
        build(layer, false, false);
        f.qkv = gq; f.wo = go; f.gu = gg; f.down_last = gd; f.attn = a;
        build(layer, true, count > 1);
        f.qkv_next = gq; f.down = gd;
        f.n_layers = count;
        f.w_stride = count > 1 ? (long long)(m->layers[layer].wqkv - lp.wqkv) : 0;
        f.kv_stride = (long long)kv->layer_bytes;
        for (int32_t l = layer; l < layer + count - 1; ++l) {   // layers l and l + 1 (1-based): records at one distance
            const LayerPacked &p0 = m->layers[l - 1], &p1 = m->layers[l];
            if (p1.wqkv - p0.wqkv != f.w_stride || p1.wo - p0.wo != f.w_stride || p1.wgu - p0.wgu != f.w_stride || p1.wd - p0.wd != f.w_stride ||
                p1.attn_norm - p0.attn_norm != f.w_stride || p1.ffn_norm - p0.ffn_norm != f.w_stride)
                return fail(AD_ESTATE, "%s: layer weights are not laid out at a constant distance", who);
        }
        f.nwg_qkv = fused_phase_workgroups(gq.NT, m->n_wg);
        f.nwg_wo = fused_phase_workgroups(go.NT, m->n_wg);
        f.nwg_gu = fused_phase_workgroups(gg.NT, m->n_wg);
        f.nwg_down = fused_phase_workgroups(gd.NT, m->n_wg);
        f.ctr = m->bar_ctr; f.round0 = m->bar_round; f.abort_flag = m->bar_abort; f.trace = m->layer_trace;
        const bool sample = profile_begin(m->prof, AD_PROF_LAYER, count * layer_step_bytes(c, pos[0], n), stream);
        rc = launch_layer_fused(f, ctx);
        if (sample) (void)event_record(m->prof.stop.back(), stream);
        if (rc) return hip_fail(rc, "layer step: fused kernel");
        m->bar_round += fused_barriers(count);
    }
    for (int32_t l = layer; l < layer + count; ++l) kv->len[l - 1] += n;
    return AD_OK;
}

ad_status ad_layer_step(const ad_model *m, ad_kv *kv, int32_t layer, void *hidden, const int32_t *pos, int32_t n, void *stream) {
    return (ad_status)layer_steps(m, kv, layer, 1, hidden, pos, n, stream, "ad_layer_step");
}

ad_status ad_layer_steps(const ad_model *m, ad_kv *kv, int32_t first_layer, int32_t n_layers, void *hidden, const int32_t *pos, int32_t n,
                         void *stream) {
    return (ad_status)layer_steps(m, kv, first_layer, n_layers, hidden, pos, n, stream, "ad_layer_steps");
}

// Head at `layer` over n rows; shared by ad_exit_head, ad_verify, ad_verify_static and ad_head_logits.
// head_part: where the vocabulary pass keeps its per-workgroup partials (null: the model's workspace).
// profiled: the launches take part in ad_profile_start's sampling (which creates events).
static int run_head(const ad_model *m, int32_t layer, const void *hidden, int32_t n, GemmArgs &g, void *stream, const char *who,
                    float *head_part = nullptr, bool profiled = true) {
    const ad_config &c = m->cfg;
    int slot = -1;
    if (layer != c.n_layers) {
        for (int i = 0; i < c.n_exit; ++i)
            if (c.exit_layers[i] == layer) slot = i;
        if (slot < 0) return fail(AD_ESTATE, "%s: layer %d has no exit head", who, layer);
    }
    const Layout &L = m->lay;
    const LaunchCtx ctx{stream, m->n_wg};
    const int ek = elem_kind(c);
    int rc;
    g.elem = ek;
    g.W = m->head; g.NT = (L.V + 15) / 16; g.KT = L.kt_d; g.N = L.V; g.K = L.d; g.m = n; g.mode = GEMM_STATIONARY;
    g.epi = EPI_HEAD; g.head_part = head_part ? head_part : m->head_part;
    auto gemm = [&](const ad_model *mm, const GemmArgs &ga, int64_t rows, int64_t cols, const LaunchCtx &c) {
        return profiled ? ::gemm(mm, ga, rows, cols, c) : launch_gemm(ga, mm->lay.planes, c);
    };
    if (slot >= 0 && m->T[slot]) {
        // lightweight head of Sec. 2.1: E = E* T, applied as E* (T norm(h))
        GemmArgs t;
        memset(&t, 0, sizeof t);
        t.elem = ek;
        t.W = m->T[slot]; t.NT = L.d / 16; t.KT = L.kt_d; t.N = L.d; t.K = L.d; t.m = n; t.mode = GEMM_STATIONARY;
        t.x = (const float *)hidden; t.ldx = L.d; t.norm_w = m->final_norm; t.norm_elem = ek; t.inv_dim = 1.0f / (float)L.d; t.eps = c.rms_eps;
        t.epi = EPI_PACK; t.Bnext = m->B1; t.Bnext_KT = L.kt_d;
        if ((rc = gemm(m, t, L.d, L.d, ctx))) return hip_fail(rc, who);
        g.B = m->B1;
    } else {
        g.x = (const float *)hidden; g.ldx = L.d; g.norm_w = m->final_norm; g.norm_elem = ek; g.inv_dim = 1.0f / (float)L.d; g.eps = c.rms_eps;
    }
    if ((rc = gemm(m, g, L.V, L.d, ctx))) return hip_fail(rc, who);
    return AD_OK;
}

// done_flag / done_seq: see GemmArgs (null: none)
static int exit_head(const ad_model *m, int32_t layer, const void *hidden_row, int32_t *token, float *conf, void *stream,
                     int32_t *done_flag, int32_t done_seq) {
    if (!m || !hidden_row || !token || !conf) return fail(AD_EINVAL, "ad_exit_head: null argument");
    if (layer < 1 || layer > m->cfg.n_layers) return fail(AD_ERANGE, "ad_exit_head: layer %d outside 1..%d", layer, m->cfg.n_layers);
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.tok_out = token; g.conf_out = conf; g.done_flag = done_flag; g.done_seq = done_seq;
    return run_head(m, layer, hidden_row, 1, g, stream, "ad_exit_head");
}

ad_status ad_exit_head(const ad_model *m, int32_t layer, const void *hidden_row, int32_t *token, float *conf, void *stream) {
    return (ad_status)exit_head(m, layer, hidden_row, token, conf, stream, nullptr, 0);
}

static int verify(const ad_model *m, const void *hidden, const int32_t *draft, int32_t n, int32_t *n_accept, int32_t *next_token,
                  int32_t *row_argmax, void *stream, int32_t *done_flag, int32_t done_seq) {
    if (!m || !hidden || !n_accept || !next_token || (n > 1 && !draft)) return fail(AD_EINVAL, "ad_verify: null argument");
    if (n < 1 || n > m->cfg.m_max) return fail(AD_ERANGE, "ad_verify: m = %d outside 1..%d", n, m->cfg.m_max);
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.verify = 1; g.n_accept_out = n_accept; g.next_out = next_token; g.tok_out = row_argmax;
    g.done_flag = done_flag; g.done_seq = done_seq;
    for (int i = 0; i + 1 < n; ++i) g.draft[i] = draft[i];
    return run_head(m, m->cfg.n_layers, hidden, n, g, stream, "ad_verify");
}

ad_status ad_verify(const ad_model *m, const void *hidden, const int32_t *draft, int32_t n, int32_t *n_accept, int32_t *next_token,
                    int32_t *row_argmax, void *stream) {
    return (ad_status)verify(m, hidden, draft, n, n_accept, next_token, row_argmax, stream, nullptr, 0);
}

ad_status ad_verify_static(const ad_model *m, const void *hidden, const int32_t *draft, int32_t n, int32_t *n_accept, int32_t *next_token,
                           int32_t *row_argmax, void *stream) {
    if (!m || !hidden || !n_accept || !next_token || (n > 1 && !draft)) return (ad_status)fail(AD_EINVAL, "ad_verify_static: null argument");
    if (n < 1 || n > m->cfg.m_max) return (ad_status)fail(AD_ERANGE, "ad_verify_static: m = %d outside 1..%d", n, m->cfg.m_max);
    const int parts = head_grid((m->lay.V + 15) / 16, m->n_wg);
    if (parts > kStaticHeadParts)
        return (ad_status)fail(AD_ERANGE, "ad_verify_static: the vocabulary pass would run on %d workgroups, the static scratch holds the partials of %d",
                               parts, kStaticHeadParts);
    float *part = nullptr;
    const int rc = static_head_scratch(&part);
    if (rc) return (ad_status)hip_fail(rc, "ad_verify_static: address of the static scratch");
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.verify = 1; g.n_accept_out = n_accept; g.next_out = next_token; g.tok_out = row_argmax;
    for (int i = 0; i + 1 < n; ++i) g.draft[i] = draft[i];
    return (ad_status)run_head(m, m->cfg.n_layers, hidden, n, g, stream, "ad_verify_static", part, false);
}

ad_status ad_head_logits(const ad_model *m, int32_t layer, const void *hidden, int32_t n, void *logits, void *stream) {
    if (!m || !hidden || !logits) return (ad_status)fail(AD_EINVAL, "ad_head_logits: null argument");
    if (layer < 1 || layer > m->cfg.n_layers) return (ad_status)fail(AD_ERANGE, "ad_head_logits: layer %d outside 1..%d", layer, m->cfg.n_layers);
    if (n < 1 || n > m->cfg.m_max) return (ad_status)fail(AD_ERANGE, "ad_head_logits: m = %d outside 1..%d", n, m->cfg.m_max);
    GemmArgs g;
    memset(&g, 0, sizeof g);
    g.logits = (float *)logits;
    return (ad_status)run_head(m, layer, hidden, n, g, stream, "ad_head_logits");
}

ad_status ad_sample_logits(const ad_model *m, const void *logits, float temperature, float u, int32_t *token, float *prob, void *stream) {
    if (!m || !logits || !token || !prob) return (ad_status)fail(AD_EINVAL, "ad_sample_logits: null argument");
    if (!(temperature > 0.f) || !(u >= 0.f && u < 1.f)) return (ad_status)fail(AD_ERANGE, "ad_sample_logits: temperature must be > 0 and u in [0, 1)");
    SampleArgs a;
    a.z = (const float *)logits; a.V = m->cfg.vocab; a.inv_t = 1.0f / temperature; a.u = u; a.tok_out = token; a.prob_out = prob;
    const int rc = launch_sample_row(a, stream);
    return rc ? (ad_status)hip_fail(rc, "ad_sample_logits") : AD_OK;
}

ad_status ad_verify_sampled(const ad_model *m, const void *final_logits, const void *draft_logits, const int32_t *draft, int32_t n,
                            float temperature, const float *u_accept, const float *u_resample, float u_final, int32_t *n_accept,
                            int32_t *next_token, float *ratio, void *stream) {
    if (!m || !final_logits || !n_accept || !next_token || (n > 1 && (!draft || !draft_logits || !u_accept || !u_resample)))
        return (ad_status)fail(AD_EINVAL, "ad_verify_sampled: null argument");
    if (n < 1 || n > m->cfg.m_max) return (ad_status)fail(AD_ERANGE, "ad_verify_sampled: m = %d outside 1..%d", n, m->cfg.m_max);
    if (!(temperature > 0.f) || !(u_final >= 0.f && u_final < 1.f)) return (ad_status)fail(AD_ERANGE, "ad_verify_sampled: temperature must be > 0 and draws in [0, 1)");
    VerifySampledArgs a;
    memset(&a, 0, sizeof a);
    a.zf = (const float *)final_logits; a.zq = (const float *)draft_logits; a.V = m->cfg.vocab; a.m = n; a.inv_t = 1.0f / temperature;
    for (int i = 0; i + 1 < n; ++i) {
        if (draft[i] < 0 || draft[i] >= m->cfg.vocab) return (ad_status)fail(AD_ERANGE, "ad_verify_sampled: draft token outside the vocabulary");
        if (!(u_accept[i] >= 0.f && u_accept[i] < 1.f) || !(u_resample[i] >= 0.f && u_resample[i] < 1.f))
            return (ad_status)fail(AD_ERANGE, "ad_verify_sampled: draws must be in [0, 1)");
        a.draft[i] = draft[i]; a.u_accept[i] = u_accept[i]; a.u_resample[i] = u_resample[i];
    }
    a.u_final = u_final; a.stats = m->samp_stats; a.n_accept_out = n_accept; a.next_out = next_token; a.ratio_out = ratio;
    const int rc = launch_verify_sampled(a, stream);
    return rc ? (ad_status)hip_fail(rc, "ad_verify_sampled") : AD_OK;
}

// ---- measurement -------------------------------------------------------------------------------------

static void profile_clear(Profile &p) {
    for (void *e : p.start) event_destroy(e);
    for (void *e : p.stop) event_destroy(e);
    p.start.clear(); p.stop.clear(); p.bytes.clear();
    p.launches = 0; p.total_bytes = 0; p.on = false;
}

ad_status ad_set_layer_mode(ad_model *m, int32_t mode) {
    if (!m) return (ad_status)fail(AD_EINVAL, "ad_set_layer_mode: null model");
    if (mode != AD_LAYER_KERNELS && mode != AD_LAYER_FUSED) return (ad_status)fail(AD_EINVAL, "ad_set_layer_mode: unknown mode %d", mode);
    if (mode == AD_LAYER_FUSED && (m->cfg.dtype != AD_BF16 || m->cfg.d_model > 5120))
        return (ad_status)fail(AD_ESTATE, "ad_set_layer_mode: the fused layer step needs a bf16 model with d_model <= 5120");
    m->layer_mode = mode;
    return AD_OK;
}

ad_status ad_probe_stream(const ad_model *m, const ad_kv *kv, int32_t layer, int32_t ctx, int32_t mode, void *stream) {
    if (!m || !kv) return (ad_status)fail(AD_EINVAL, "ad_probe_stream: null argument");
    if (kv->model != m) return (ad_status)fail(AD_EINVAL, "ad_probe_stream: cache belongs to another model");
    if (layer < 1 || layer > m->cfg.n_layers) return (ad_status)fail(AD_ERANGE, "ad_probe_stream: layer %d outside 1..%d", layer, m->cfg.n_layers);
    if (ctx < 0 || ctx > kv->max_pos) return (ad_status)fail(AD_ERANGE, "ad_probe_stream: ctx %d outside 0..%d", ctx, kv->max_pos);
    if (mode != AD_PROBE_ONE_KERNEL && mode != AD_PROBE_PER_PHASE) return (ad_status)fail(AD_EINVAL, "ad_probe_stream: unknown mode %d", mode);
    const Layout &L = m->lay;
    const LayerPacked &lp = m->layers[layer - 1];
    const char *cache = (const char *)kv->storage + (size_t)(layer - 1) * kv->layer_bytes;
    // as many bytes of the layer's cache as ctx positions of K and V hold (the cache is position-major per head;
    // the probe reads the same number of bytes from the start of the layer's block)
    size_t kv_bytes = 2 * (size_t)m->cfg.n_kv_heads * m->cfg.head_dim * (m->cfg.dtype == AD_F32 ? 4 : 2) * (size_t)ctx;
    kv_bytes = (kv_bytes < kv->layer_bytes ? kv_bytes : kv->layer_bytes) & ~(size_t)15;
    unsigned *sink = m->bar_ctr + 24;       // a word of the model's scratch that nothing reads; the probe never writes it
    int rc;
    if (mode == AD_PROBE_ONE_KERNEL) {
        // the four matrices of a layer are adjacent in the packed model
        rc = launch_probe_stream(lp.wqkv, L.sz_wqkv + L.sz_wo + L.sz_wgu + L.sz_wd, cache, kv_bytes, sink, m->n_wg, stream);
    } else {
        rc = launch_probe_stream(lp.wqkv, L.sz_wqkv, nullptr, 0, sink, m->n_wg, stream);
        if (!rc && kv_bytes) rc = launch_probe_stream(cache, kv_bytes, nullptr, 0, sink, m->n_wg, stream);
        if (!rc) rc = launch_probe_stream(lp.wo, L.sz_wo, nullptr, 0, sink, m->n_wg, stream);
        if (!rc) rc = launch_probe_stream(lp.wgu, L.sz_wgu, nullptr, 0, sink, m->n_wg, stream);
        if (!rc) rc = launch_probe_stream(lp.wd, L.sz_wd, nullptr, 0, sink, m->n_wg, stream);
    }
    return rc ? (ad_status)hip_fail(rc, "ad_probe_stream") : AD_OK;
}

ad_status ad_layer_trace(ad_model *m, void *ticks, size_t bytes, int32_t *n_workgroups, int32_t *n_stamps) {
    if (!m) return (ad_status)fail(AD_EINVAL, "ad_layer_trace: null model");
    if (n_workgroups) *n_workgroups = m->n_wg;
    if (n_stamps) *n_stamps = kFusedTraceStamps;
    if (ticks && bytes < (size_t)m->n_wg * kFusedTraceStamps * 8) return (ad_status)fail(AD_ENOMEM, "ad_layer_trace: buffer too small");
    m->layer_trace = (long long *)ticks;
    return AD_OK;
}

ad_status ad_profile_start(ad_model *m, int32_t kind, int32_t period, int32_t max_samples) {
    if (!m) return (ad_status)fail(AD_EINVAL, "ad_profile_start: null model");
    if (kind != AD_PROF_GEMM && kind != AD_PROF_LAYER) return (ad_status)fail(AD_EINVAL, "ad_profile_start: unknown kind %d", kind);
    if (period < 1 || max_samples < 1 || max_samples > 65536) return (ad_status)fail(AD_ERANGE, "ad_profile_start: period >= 1 and 1 <= max_samples <= 65536");
    profile_clear(m->prof);
    m->prof.kind = kind;
    m->prof.period = period;
    m->prof.max_samples = max_samples;
    m->prof.on = true;
    return AD_OK;
}

ad_status ad_profile_stop(ad_model *m, int64_t *n_launches, int64_t *n_samples, double *sampled_ms, int64_t *sampled_bytes,
                          int64_t *total_bytes) {
    if (!m || !n_launches || !n_samples || !sampled_ms || !sampled_bytes || !total_bytes) return (ad_status)fail(AD_EINVAL, "ad_profile_stop: null argument");
    Profile &p = m->prof;
    if (!p.on) return (ad_status)fail(AD_ESTATE, "ad_profile_stop: profiling is not on");
    double ms = 0.0;
    int64_t bytes = 0, n = 0;
    for (size_t i = 0; i < p.start.size(); ++i) {
        float t = 0.f;
        // waits for the stop event, so every sampled launch has finished when this loop ends
        int rc = stream_sync_event(p.stop[i]);
        if (!rc) rc = event_elapsed_ms(p.start[i], p.stop[i], &t);
        if (rc) { profile_clear(p); return (ad_status)hip_fail(rc, "ad_profile_stop"); }
        ms += t; bytes += p.bytes[i]; ++n;
    }
    *n_launches = p.launches; *n_samples = n; *sampled_ms = ms; *sampled_bytes = bytes; *total_bytes = p.total_bytes;
    profile_clear(p);
    return AD_OK;
}

// ---- Algorithm 1 over the GPU steps ------------------------------------------------------------------

namespace {

struct GpuBackend : Backend {
    const ad_model *m;
    ad_kv *kv;
    void *stream;
    int64_t bytes = 0;
    bool in_prefill = false;   // the prompt pass is not part of the decode-step byte count
    int32_t pos_buf[AD_M_MAX];

    float *row(int32_t r) const { return m->rows + (size_t)r * m->cfg.d_model; }

    // The decision after a head evaluation is taken on the host (Algorithm 1's branch on the confidence, the
    // verification's accept count), so the GPU idles from the head's last kernel until the next launch arrives.
    // Waiting for the stream to drain adds the runtime's completion path to that gap; instead the head's second
    // kernel publishes a sequence number in pinned memory after its results, and this thread polls that word.
    // If it does not appear within kPollMs (a failed launch, a device error), the ordinary wait takes over
    // and reports what happened.
    static constexpr int kPollMs = 200;
    int32_t *done_flag() const { return m->pin + 28; }
    int32_t next_seq() const {
        if (++m->done_seq == 0) ++m->done_seq;     // 0 is the word's initial value
        return m->done_seq;
    }
    int wait_done(const char *what) {
        const volatile int32_t *flag = done_flag();
        const int32_t want = m->done_seq;
        const auto t0 = std::chrono::steady_clock::now();
        for (unsigned spins = 1; *flag != want; ++spins) {
            __builtin_ia32_pause();
            if ((spins & 4095) == 0 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(kPollMs)) break;
        }
        std::atomic_thread_fence(std::memory_order_acquire);
        if (*flag == want && ++polled < kSyncEvery) return AD_OK;
        // now and then, and whenever the word did not appear, drain the stream: the runtime releases what it keeps
        // per launch, and errors of earlier launches surface here
        polled = 0;
        const int rc = stream_sync(stream);
        if (rc) return hip_fail(rc, what);
        if (*flag != want) return fail(AD_EDEVICE, "%s: the head finished without publishing its result", what);
        return AD_OK;
    }
    static constexpr int kSyncEvery = 256;
    int polled = 0;

    int layer_step(int32_t layer, int32_t row0, int32_t n, int32_t pos0) override { return layer_steps(layer, 1, row0, n, pos0); }
    int layer_steps(int32_t first_layer, int32_t count, int32_t row0, int32_t n, int32_t pos0) override {
        for (int i = 0; i < n; ++i) pos_buf[i] = pos0 + i;
        if (!in_prefill) bytes += count * layer_step_bytes(m->cfg, pos0, n);
        // the step's QKV projection may already be on the stream
        const bool qkv_there = issued.kind != AHEAD_NONE && issued.layer == first_layer && issued.row0 == row0 && issued.m == n &&
                               (issued.kind == AHEAD_LAYER || embed_taken) && m->layer_mode == AD_LAYER_KERNELS;
        issued.kind = AHEAD_NONE;
        return ::layer_steps(m, kv, first_layer, count, row(row0), pos_buf, n, stream, "ad_layer_steps", qkv_there);
    }
    int prefill(const int32_t *tokens, int32_t n) override {
        const int32_t chunk = m->cfg.m_max;
        in_prefill = true;
        int rc = AD_OK;
        for (int32_t s = 0; s < n && rc == AD_OK; s += chunk) {
            const int32_t k = (n - s < chunk) ? n - s : chunk;
            rc = ad_embed(m, tokens + s, k, row(0), stream);
            if (rc == AD_OK) rc = layer_steps(1, m->cfg.n_layers, 0, k, s);
        }
        in_prefill = false;
        return rc;
    }
    // ---- work issued ahead of a head's outcome (see Backend::expect) ----
    Ahead hint{AHEAD_NONE, 0, 0, 0};      // for the next head evaluation
    Ahead issued{AHEAD_NONE, 0, 0, 0};    // what is in flight or done, not yet taken over by the schedule
    const int32_t *issued_tok = nullptr;  // AHEAD_TOKEN: the pinned word the embedding kernel read its token from
    bool embed_taken = false;             // AHEAD_TOKEN: the schedule has asked for exactly that embedding

    void expect(const Ahead &a) override { hint = a; }
    // Behind the head's kernels: the embedding of the token they produce (tok_src, pinned) if that is what comes
    // next, and the QKV projection of the step that follows.  Only in separate-kernel mode: the fused layer
    // kernel has no entry behind its QKV phase.
    int issue_ahead(const int32_t *tok_src) {
        const Ahead h = hint;
        hint.kind = issued.kind = AHEAD_NONE;
        if (h.kind == AHEAD_NONE || m->layer_mode != AD_LAYER_KERNELS) return AD_OK;
        if (h.layer < 1 || h.layer > m->cfg.n_layers || h.row0 < 0 || h.m < 1 || h.row0 + h.m > m->cfg.m_max) return AD_OK;
        int rc = AD_OK;
        if (h.kind == AHEAD_TOKEN) rc = embed_from(m, tok_src, row(h.row0), stream);
        if (rc == AD_OK) rc = qkv_ahead(m, h.layer, row(h.row0), h.m, stream);
        if (rc != AD_OK) return rc;
        issued = h; issued_tok = tok_src; embed_taken = false;
        return AD_OK;
    }

    int embed(int32_t token, int32_t r) override {
        if (issued.kind == AHEAD_TOKEN && !embed_taken && issued.row0 == r && *(const volatile int32_t *)issued_tok == token) {
            embed_taken = true;           // the row already holds this token's embedding
            return AD_OK;
        }
        issued.kind = AHEAD_NONE;
        return ad_embed(m, &token, 1, row(r), stream);
    }
    int exit_head(int32_t layer, int32_t r, int32_t, int32_t *token, float *conf) override {
        int rc = ::exit_head(m, layer, row(r), m->pin, m->pin_conf, stream, done_flag(), next_seq());
        if (rc == AD_OK) rc = issue_ahead(m->pin);
        if (rc != AD_OK) return rc;
        if ((rc = wait_done("ad_generate: exit head"))) return rc;
        if ((rc = fused_health(m, stream))) return rc;
        *token = m->pin[0];
        *conf = m->pin_conf[0];
        const int64_t s = m->cfg.dtype == AD_F32 ? 4 : 2;
        bytes += (int64_t)m->cfg.vocab * m->cfg.d_model * s;
        return AD_OK;
    }
    int verify(int32_t n, int32_t, const int32_t *draft, int32_t *n_accept, int32_t *next, int32_t *row_argmax) override {
        int rc = ::verify(m, row(0), draft, n, m->pin + 8, m->pin + 9, m->pin + 16, stream, done_flag(), next_seq());
        if (rc == AD_OK) rc = issue_ahead(m->pin + 9);
        if (rc != AD_OK) return rc;
        if ((rc = wait_done("ad_generate: verify"))) return rc;
        if ((rc = fused_health(m, stream))) return rc;
        *n_accept = m->pin[8];
        *next = m->pin[9];
        for (int i = 0; i < n; ++i) row_argmax[i] = m->pin[16 + i];
        const int64_t s = m->cfg.dtype == AD_F32 ? 4 : 2;
        bytes += (int64_t)m->cfg.vocab * m->cfg.d_model * s;
        return AD_OK;
    }
    // Eq. 1 with a sampled token: the head's logits stay in the draft slot of this row until the verification
    int sample_head(int32_t layer, int32_t r, int32_t, float temperature, float u, int32_t *token, float *prob) override {
        float *z = m->draft_logits + (size_t)r * m->cfg.vocab;
        hint.kind = issued.kind = AHEAD_NONE;
        int rc = ad_head_logits(m, layer, row(r), 1, z, stream);
        if (rc == AD_OK) rc = ad_sample_logits(m, z, temperature, u, m->pin, m->pin_conf, stream);
        if (rc != AD_OK) return rc;
        if ((rc = stream_sync(stream))) return hip_fail(rc, "ad_generate: sampled head");
        if ((rc = fused_health(m, stream))) return rc;
        *token = m->pin[0];
        *prob = m->pin_conf[0];
        const int64_t s = m->cfg.dtype == AD_F32 ? 4 : 2;
        bytes += (int64_t)m->cfg.vocab * m->cfg.d_model * s;
        return AD_OK;
    }
    int verify_sampled(int32_t n, int32_t, const int32_t *draft, float temperature, const float *u_accept, const float *u_resample,
                       float u_final, int32_t *n_accept, int32_t *next, float *ratio) override {
        hint.kind = issued.kind = AHEAD_NONE;
        int rc = ad_head_logits(m, m->cfg.n_layers, row(0), n, m->final_logits, stream);
        if (rc == AD_OK)
            rc = ad_verify_sampled(m, m->final_logits, m->draft_logits, draft, n, temperature, u_accept, u_resample, u_final, m->pin + 8,
                                   m->pin + 9, m->pin_conf + 8, stream);
        if (rc != AD_OK) return rc;
        if ((rc = stream_sync(stream))) return hip_fail(rc, "ad_generate: sampled verify");
        if ((rc = fused_health(m, stream))) return rc;
        *n_accept = m->pin[8];
        *next = m->pin[9];
        for (int i = 0; i + 1 < n; ++i) ratio[i] = m->pin_conf[8 + i];
        const int64_t s = m->cfg.dtype == AD_F32 ? 4 : 2;
        bytes += (int64_t)m->cfg.vocab * m->cfg.d_model * s;
        return AD_OK;
    }
    int truncate(int32_t new_len) override { return ad_kv_truncate(kv, new_len); }
};

}  // namespace

ad_status ad_generate(const ad_model *m, ad_kv *kv, const int32_t *prompt, int32_t n_prompt, const ad_gen_params *gp,
                      int32_t *out_tokens, int32_t *n_out, ad_stats *stats, ad_event *events, int64_t max_events,
                      int64_t *n_events, void *stream) {
    if (!m || !kv || !prompt || !gp || !out_tokens || !n_out) return (ad_status)fail(AD_EINVAL, "ad_generate: null argument");
    if (kv->model != m) return (ad_status)fail(AD_EINVAL, "ad_generate: cache belongs to another model");
    if (n_prompt < 1 || gp->max_new < 1) return (ad_status)fail(AD_EINVAL, "ad_generate: empty prompt or max_new < 1");
    if (gp->max_pending < 0 || gp->max_pending + 1 > m->cfg.m_max)
        return (ad_status)fail(AD_ERANGE, "ad_generate: max_pending %d outside 0..%d", gp->max_pending, m->cfg.m_max - 1);
    if (gp->temperature < 0.f || (gp->temperature > 0.f && !gp->uniforms))
        return (ad_status)fail(AD_EINVAL, "ad_generate: sampled decoding needs temperature > 0 and the table of uniform draws");
    if ((int64_t)n_prompt + gp->max_new > kv->max_pos)
        return (ad_status)fail(AD_ERANGE, "ad_generate: prompt + max_new = %lld exceeds max_pos %d", (long long)n_prompt + gp->max_new, kv->max_pos);
    for (int i = 0; i < n_prompt; ++i)
        if (prompt[i] < 0 || prompt[i] >= m->cfg.vocab) return (ad_status)fail(AD_ERANGE, "ad_generate: prompt token outside the vocabulary");
    SchedConfig sc;
    sc.n_layers = m->cfg.n_layers; sc.n_exit = m->cfg.n_exit; sc.m_max = m->cfg.m_max;
    for (int i = 0; i < AD_MAX_EXIT; ++i) sc.exit_layers[i] = m->cfg.exit_layers[i];
    GpuBackend be;
    be.m = m; be.kv = kv; be.stream = stream;
    int rc = run_algorithm1(be, sc, *gp, prompt, n_prompt, out_tokens, n_out, stats, events, max_events, n_events);
    if (stats) stats->bytes_algorithmic = be.bytes;
    // nothing the call enqueued (work issued ahead of an outcome included) is still running when it returns
    if (rc != AD_OK) (void)stream_sync(stream);
    if (rc == AD_OK && (rc = stream_sync(stream))) return (ad_status)hip_fail(rc, "ad_generate");
    if (rc == AD_OK) rc = fused_health(m, stream);
    return (ad_status)rc;
}

}  // extern "C"
