// Internal interface between the host side of the library (C ABI, model and cache objects, scheduler)
// and its gfx950 kernels.  Not installed; the public interface is include/adadecode.h.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace ad {

enum : int { kElemF32 = 0, kElemBF16 = 1, kElemF16 = 2 };   // host-side names of ElemKind (ad_device.h)

// ---- packed operand layouts ---------------------------------------------------------------------------
// Weight matrix W [N, K] -> tiles of 16 output rows x 32 inputs.  Tile (rt, ks) is stored as P planes of
// 64 lanes x 8 bf16 (1 KiB per plane): lane l holds W[rt*16 + (l & 15)][ks*32 + (l >> 4)*8 .. +8), which
// is the A operand of one 16x16x32 bf16 MFMA, so that a wavefront loads a whole tile plane with one
// 128-bit load per lane from 1 KiB of contiguous memory.  Tiles are ordered [rt][ks][plane].
// 16-bit weights (bf16 or fp16) have one plane; fp32 weights are split exactly into three bf16 planes (W = p0 + p1 + p2).
// Rows >= N and inputs >= K are zero.
//
// Activation block [m <= 8 tokens, K]: the MFMA's B operand has 16 columns; columns 0..7 are the tokens' bf16
// "hi" parts and columns 8..15 their "lo" parts (x = hi + lo to 16 mantissa bits), so one MFMA yields both
// partial products and the activations keep near-fp32 precision.  Lane l of the operand of k-step ks holds
// column (l & 15) and inputs ks*32 + (l >> 4)*8 .. +8.  In memory the block is ordered
// [token][k-step][hi, lo][lane group l >> 4][8 inputs]: the 128 bytes a token contributes to a k-step are one
// cache line, and a call with m tokens touches m lines per k-step (KT * 1 KiB for a full block).
constexpr int kTileRows = 16;
constexpr int kTileK = 32;
constexpr int kThreads = 1024;   // one workgroup per CU, 16 wavefronts
constexpr int kWaves = kThreads / 64;

inline size_t packed_bytes(int64_t N, int64_t K, int planes) {
    const int64_t nt = (N + kTileRows - 1) / kTileRows, kt = (K + kTileK - 1) / kTileK;
    return (size_t)(nt * kt * planes) * 1024u;
}
inline size_t act_packed_bytes(int64_t K) { return (size_t)((K + kTileK - 1) / kTileK) * 1024u; }

enum EpiKind : int { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2, EPI_HEAD = 3, EPI_PACK = 4 };
enum GemmMode : int { GEMM_STREAMED = 0, GEMM_STATIONARY = 1 };

struct GemmArgs {
    // what a kernel needs before it can issue its first loads comes first (one line of the argument block)
    const void *W;        // packed weights
    // activations: either fp32 rows x [m][ldx] (stationary mode; multiplied by norm_w and, in the epilogue, by
    // rsqrt(mean(x^2) + eps) when norm_w is given), or a packed block B
    const float *x;
    const void *B;
    const void *norm_w;
    int NT, KT;           // row tiles, k-steps
    int K;                // valid inputs
    int m;                // tokens
    int tq, tr;           // row tiles per workgroup: workgroup w of the GEMM's n takes tq tiles, the first tr of them one more
                          // (set by the launchers for the grid they choose)
    int ldx;
    int N;                // valid output rows (EPI_SWIGLU: rows of the interleaved gate/up matrix = 2F)
    // ---- end of the first line ----
    int mode;             // GemmMode
    int elem;             // ElemKind of the weights: fp32 (three bf16 planes), bf16, or fp16 (fp16 MFMA, fp16 hi/lo activations)
    int norm_elem;        // ElemKind of norm_w
    float inv_dim, eps;
    int epi;
    // EPI_STORE: out[t*ld + n] = scale_t * acc
    // EPI_RESID: out[t*ld + n] = resid[t*ld + n] + acc
    // EPI_SWIGLU: tile rows 0..7 gate, 8..15 up of features tile*8 .. +8; packs silu(gate)*up into Bnext
    // EPI_PACK: packs scale_t * acc into Bnext (used for the exit-head transform T)
    // EPI_HEAD: per-token argmax / log-sum-exp over all rows; partials per workgroup, folded by a second kernel
    float *out;
    const float *resid;
    int ld;
    void *Bnext;          // packed activations written by the epilogue
    int Bnext_KT;         // k-steps of that block (the K of the GEMM that will read it, in units of 32)
    // EPI_RESID in streamed mode, optional (Bnext non-null): the epilogue also prepares the next GEMM's input, which is
    // RMSNorm(out): it packs out * next_norm_w into Bnext and writes the sum of squares of its 16 outputs per token
    // to ssq_out[tile][token].  The consumer (stationary mode, B = that block, ssq_in = those partials, ssq_tiles
    // of them) only has to load its operand registers and add the partials up for the 1/rms factor.
    const void *next_norm_w;
    int next_norm_elem;
    float *ssq_out;
    const float *ssq_in;
    int ssq_tiles;
    // head
    float *head_part;     // [nwg][8][4] (max, sumexp, argmax as int bits, unused)
    int n_parts;          // workgroups that wrote head_part (set by the launcher)
    float *logits;        // null or [m][N]
    int32_t *tok_out;     // [m] (or null)
    float *conf_out;      // [m] (or null)
    int32_t *n_accept_out, *next_out;   // verify outputs or null
    int32_t draft[8];
    int verify;
    // optional: host-visible word that the head's second kernel sets to done_seq, at system scope, after its results
    // are written; a host thread that polls it learns the outcome without waiting for the stream to drain
    int32_t *done_flag;
    int32_t done_seq;
};

static_assert(offsetof(GemmArgs, mode) == 64, "GemmArgs: the first line holds the fields needed first");
// the launchers' partition of a GEMM's NT row tiles over n workgroups
inline void set_tile_partition(GemmArgs &g, int n) { g.tq = g.NT / n; g.tr = g.NT % n; }

struct RopeArgs {
    float *table;         // [n_pos][half][2] (cos, sin)
    int n_pos, half;
    double inv_freq[64];  // base^(-2i/dh)
};

struct AttnArgs {
    const float *qkv;     // [m][ld]: q heads, then k heads, then v heads
    int ld;
    const float *rope;    // [m][dh/2][2]: rows pos0 .. pos0+m-1 of the cache's rotary table
    void *Kc, *Vc;        // this layer's cache: K [Hkv][stride][dh], V [Hkv][dh][stride]
    int stride;           // positions per cache row block (max_pos rounded up to 64)
    int pos0, m, Hq, Hkv, dh;
    int C, S;             // chunk (positions per work item), splits
    float *part;          // [Hkv][S][R][dh+2]
    void *Bo;             // packed attention output for the Wo GEMM
    int Bo_KT;            // k-steps of that block (n_q_heads * head_dim / 32)
    float scale;
    int kv_elem;          // ElemKind of the cache (and of the 16-bit operands of the MFMA kernel)
    // derived by attn_finish() from the fields above, so that the kernels need no integer division on their way to the
    // first load: query heads per kv head, query rows per kv head, and the multipliers of div_small() for S, G and R
    int G, R;
    unsigned mul_S, mul_G, mul_R;
};
// x / d == (x * div_multiplier(d)) >> 32 for 0 <= x < 65536 and 1 < d < 65536 (the error of the rounded-up reciprocal,
// x / 2^32, stays below the 1 / d that separates x / d from the next integer); d == 1, whose multiplier would be
// 2^32, is encoded as 0
inline unsigned div_multiplier(int d) { return d <= 1 ? 0u : (unsigned)((0x100000000ull + (unsigned long long)d - 1) / (unsigned long long)d); }
inline void attn_finish(AttnArgs &a) {
    a.G = a.Hq / a.Hkv;
    a.R = a.G * a.m;
    a.mul_S = div_multiplier(a.S);
    a.mul_G = div_multiplier(a.G);
    a.mul_R = div_multiplier(a.R);
}

// n_layers consecutive decoder-layer steps over the same rows as a single persistent kernel (bf16 models): the four
// GEMMs and the attention phase of the first of these layers with their usual arguments, the distance in bytes from
// one layer's weights (and norm weights) and cache to the next layer's, the number of workgroups that own row tiles in
// each GEMM, and the grid barrier.  qkv reads the caller's rows (first layer); qkv_next reads what the down projection
// of the layer before left packed (`down`: a layer that is followed by another; down_last: the last one).
struct FusedArgs {
    GemmArgs qkv, qkv_next, wo, gu, down, down_last;
    AttnArgs attn;
    int n_layers;
    long long w_stride, kv_stride;
    int nwg_qkv, nwg_wo, nwg_gu, nwg_down;
    unsigned *ctr;          // barrier counters: kBarrierWords zero-initialised words, owned by the model
    unsigned round0;        // barriers completed by earlier launches on these counters
    unsigned *abort_flag;   // pinned host word, set when a barrier wait timed out
    long long *trace;       // null, or [workgroups][kFusedTraceStamps] wall-clock ticks (100 MHz) at the phase boundaries
};
constexpr int kFusedTraceStamps = 12;      // of the launch's last layer: start, before and after each of its 5 barriers, end
constexpr int kBarrierWords = 32 * 9;      // one 128-byte line for the global counter and for each of 8 groups
inline unsigned fused_barriers(int n_layers) { return 6u * (unsigned)n_layers - 1u; }   // barriers per launch

struct EmbedArgs {
    const void *table; int elem; int d; int m; int32_t tok[8]; float *out;
    // null, or where the kernel reads the m token ids instead of tok[] (device-visible memory that an earlier kernel
    // on the stream wrote); ids outside [0, vocab) are clamped
    const int32_t *tok_src; int vocab;
};

// Sampled decoding (Sec. 2.2).  inv_t = 1 / temperature; u, u_accept, u_resample, u_final are uniform draws in [0, 1).
struct SampleArgs {
    const float *z;         // dev [V] logits
    int V;
    float inv_t, u;
    int32_t *tok_out;       // pinned host or dev
    float *prob_out;        // pinned host or dev: probability of the drawn token
};
struct VerifySampledArgs {
    const float *zf;        // dev [m][V]: final-layer logits of the m rows
    const float *zq;        // dev [m - 1][V]: logits each draft was drawn from (row k: the draft that follows row k)
    int V, m;
    float inv_t;
    int32_t draft[8];
    float u_accept[8], u_resample[8], u_final;
    float *stats;           // dev scratch [2 * (2m - 1)]: (max, sum of exp) per row
    int32_t *n_accept_out, *next_out;   // pinned host or dev
    float *ratio_out;       // null, or pinned host or dev [m - 1]: p*(t) / p_draft(t) of the drafts that were checked, else 0
};

struct LaunchCtx { void *stream; int n_wg; };

// All launchers return 0 or a hipError_t value.
// mode 0: W [N, K] -> packed.  mode 1: gate (src) and up (src2), each [N, K], interleaved 8 rows at a time.
int launch_pack_weights(const void *src, const void *src2, int src_elem, int64_t N, int64_t K, int mode, void *dst,
                        void *stream);
// reads the two ranges (bytes, multiples of 16) on n_wg workgroups and drops the data; sink: any device word
int launch_probe_stream(const void *p0, size_t bytes0, const void *p1, size_t bytes1, unsigned *sink, int n_wg, void *stream);
int launch_copy(const void *src, void *dst, size_t bytes, void *stream);
int launch_zero(void *dst, size_t bytes, void *stream);
int launch_embed(const EmbedArgs &, void *stream);
int launch_rope_table(const RopeArgs &, void *stream);
int gemm_max_stationary_k(int planes);   // largest d_model the stationary GEMM variants cover
int launch_gemm(const GemmArgs &, int planes, const LaunchCtx &);   // EPI_HEAD: also launches the vocabulary combine
int head_grid(int n_tiles, int n_wg);                               // workgroups launch_gemm uses for n_tiles row tiles
// The library's own static device array for the vocabulary pass's per-workgroup partials (room for kStaticHeadParts
// workgroups): its address on the current device, resolved on first use per device.  Allocates nothing.
constexpr int kStaticHeadParts = 4096;
int static_head_scratch(float **ptr);
int launch_attn(const AttnArgs &, const LaunchCtx &);
int launch_sample_row(const SampleArgs &, void *stream);
int launch_verify_sampled(const VerifySampledArgs &, void *stream);
int launch_layer_fused(const FusedArgs &, const LaunchCtx &);   // n_wg must not exceed the number of compute units
int fused_phase_workgroups(int n_tiles, int n_wg);               // workgroups that own row tiles of a GEMM phase
int attn_chunk(int kv_elem, int dh);   // cached positions per attention work item
int device_info(int *n_cu);
const char *hip_error_text(int code);
int stream_sync(void *stream);
void *event_create();
void event_destroy(void *ev);
int event_record(void *ev, void *stream);
int event_elapsed_ms(void *start, void *stop, float *ms);
int stream_sync_event(void *ev);
void *pinned_alloc(size_t bytes);
void pinned_free(void *);

}  // namespace ad
