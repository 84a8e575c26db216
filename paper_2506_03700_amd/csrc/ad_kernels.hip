// gfx950 kernels of the AdaDecode hot path: weight re-layout, activation packing, the weight-streaming
// skinny GEMM with its fused epilogues (QKV store, residual + next-norm packing, SwiGLU, vocabulary
// argmax / log-sum-exp), split-context GQA attention with KV append, and the embedding gather.
//
// Algorithm 1's layer step is one pass of:  pack -> GEMM(QKV) -> attention -> GEMM(Wo) -> GEMM(gate/up)
// -> GEMM(down); the exit head (Eq. 1) and the verification (Eq. 2) are pack -> GEMM(E*) with the
// EPI_HEAD epilogue.  Every phase is written as a device function over (workgroup index, workgroup
// count) so that it can run as a kernel of its own or as a stage of a longer kernel.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_internal.h"

namespace ad {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// ---------------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void split_hi_lo(float x, uint16_t &hi, uint16_t &lo) {
    hi = f32_to_bf16_bits(x);
    lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
}

__device__ __forceinline__ float load_w(const void *p, int is_bf16, size_t i) {
    return is_bf16 ? bf16_bits_to_f32(((const uint16_t *)p)[i]) : ((const float *)p)[i];
}

// index (in bf16 elements) of input k of column col in a packed activation block
__device__ __forceinline__ size_t act_index(int k, int col) {
    return ((size_t)((k >> 5) * 4 + ((k & 31) >> 3)) * 16 + col) * 8 + (k & 7);
}

__device__ __forceinline__ void store_act(uint16_t *B, int k, int t, float v) {
    uint16_t hi, lo;
    split_hi_lo(v, hi, lo);
    B[act_index(k, t)] = hi;
    B[act_index(k, 8 + t)] = lo;
}

// ---------------------------------------------------------------------------------------------------
// weight re-layout (runs once, at model creation)
// ---------------------------------------------------------------------------------------------------
// One thread per (tile, lane).  mode 0: dst row r = src row r.  mode 1 (gate/up interleave): tile rt holds
// gate rows rt*8..+8 in tile rows 0..7 and up rows rt*8..+8 in tile rows 8..15.
__global__ void k_pack_weights(const void *src, const void *src2, int is_bf16, int64_t N, int64_t K, int64_t NT,
                               int64_t KT, int mode, uint16_t *dst) {
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= NT * KT * 64) return;
    const int lane = (int)(gid & 63);
    const int64_t tile = gid >> 6, rt = tile / KT, ks = tile % KT;
    const int i = lane & 15, g = lane >> 4;
    const void *s = src;
    int64_t row;
    if (mode == 0) {
        row = rt * 16 + i;
    } else {
        row = rt * 8 + (i & 7);
        if (i >= 8) s = src2;
    }
    const int planes = is_bf16 ? 1 : 3;
    uint16_t *d = dst + (size_t)tile * planes * 512 + (size_t)lane * 8;
    for (int e = 0; e < 8; ++e) {
        const int64_t k = ks * 32 + g * 8 + e;
        const bool ok = row < N && k < K;
        if (is_bf16) {
            d[e] = ok ? ((const uint16_t *)s)[row * K + k] : (uint16_t)0;
        } else {
            const float w = ok ? ((const float *)s)[row * K + k] : 0.0f;
            const uint16_t p0 = f32_to_bf16_bits(w);
            const float r1 = w - bf16_bits_to_f32(p0);
            const uint16_t p1 = f32_to_bf16_bits(r1);
            const float r2 = r1 - bf16_bits_to_f32(p1);
            d[e] = p0;
            d[512 + e] = p1;
            d[1024 + e] = f32_to_bf16_bits(r2);
        }
    }
}

__global__ void k_copy16(const u32x4 *src, u32x4 *dst, size_t n16) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

__global__ void k_zero16(u32x4 *dst, size_t n16) {
    const u32x4 z = {0, 0, 0, 0};
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = z;
}

__global__ void k_embed(EmbedArgs a) {
    for (int idx = blockIdx.x * blockDim.x + threadIdx.x; idx < a.m * a.d; idx += gridDim.x * blockDim.x) {
        const int r = idx / a.d, c = idx % a.d;
        a.out[idx] = load_w(a.table, a.is_bf16, (size_t)a.tok[r] * a.d + c);
    }
}

// ---------------------------------------------------------------------------------------------------
// phase: pack activations (first phase of a layer step / of a head evaluation)
// ---------------------------------------------------------------------------------------------------
// B = hi/lo split of x * norm_w (the RMSNorm's 1/rms factor is applied in the consuming GEMM's epilogue,
// since it is a per-token scalar and commutes with the matrix product); ssq[c][t] = sum of x^2 over the
// 16 inputs of chunk c.  Also fills the rotary table for the call's positions.
__device__ void pack_phase(const PackArgs &a, int wg, int nwg) {
    const int gtid = wg * blockDim.x + threadIdx.x, gsize = nwg * blockDim.x;
    const int chunks = a.d / 16;
    for (int idx = gtid; idx < chunks * a.m; idx += gsize) {
        const int t = idx / chunks, c = idx % chunks;
        const float *x = a.x + (size_t)t * a.d + c * 16;
        float s = 0.0f;
        uint16_t hi[16], lo[16];
        for (int e = 0; e < 16; ++e) {
            const float v = x[e];
            s += v * v;
            split_hi_lo(v * load_w(a.norm_w, a.norm_is_bf16, (size_t)c * 16 + e), hi[e], lo[e]);
        }
        uint16_t *B = (uint16_t *)a.B;
        for (int e = 0; e < 16; ++e) {
            B[act_index(c * 16 + e, t)] = hi[e];
            B[act_index(c * 16 + e, 8 + t)] = lo[e];
        }
        a.ssq[c * 8 + t] = s;
    }
    if (a.rope) {
        const int half = a.head_dim / 2;
        for (int idx = gtid; idx < a.m * half; idx += gsize) {
            const int t = idx / half, i = idx % half;
            // the angle is formed in double so that large positions keep their phase
            const double ang = (double)(a.pos0 + t) * a.inv_freq[i];
            a.rope[idx * 2] = (float)cos(ang);
            a.rope[idx * 2 + 1] = (float)sin(ang);
        }
    }
}

__global__ void __launch_bounds__(256) k_pack(PackArgs a) { pack_phase(a, blockIdx.x, gridDim.x); }

// ---------------------------------------------------------------------------------------------------
// phase: weight-streaming skinny GEMM   out[t][n] = sum_k W[n][k] * act[t][k],  m <= 8 tokens
// ---------------------------------------------------------------------------------------------------
// Work split.  Workgroup wg owns the contiguous block of row tiles [NT*wg/nwg, NT*(wg+1)/nwg), processed in
// rounds of at most kMaxTilesPerRound tiles.  Within a round the (tile, k-step) pairs are linearised with
// the k-step fastest -- which is also the order of the packed weights in memory -- and cut into kWaves
// equal contiguous ranges, one per wavefront: every wavefront streams one contiguous piece of HBM with
// 128-bit loads, U tile planes in flight at a time.  A range may cross tile boundaries; each (wavefront,
// tile) partial accumulator goes to an LDS slot and the slots of a tile are summed in wavefront order
// (fixed order: results are reproducible), then the epilogue runs on the reduced 16 x m block.
struct GemmLds {
    float slots[(kWaves + kMaxTilesPerRound) * 256];   // [slot][col 0..15][row 0..15]
    float red[kMaxTilesPerRound * 128];                // [tile][token 0..7][row 0..15]
    float scale[8];
    float run_max[8], run_sum[8];
    int run_idx[8];
    int flag;
};

template <int NPL, int U>
__device__ __forceinline__ void wave_stream(const bf16x8 *__restrict__ W, const bf16x8 *__restrict__ B, int KT, int xa, int xb,
                                            int m, float *slots, int wave, int lane) {
    int tile = xa / KT, ks = xa % KT;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    const bool bact = (lane & 7) < m;
    const bf16x8 *pa = W + (size_t)xa * NPL * 64 + lane;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    for (int x = xa; x < xb; x += U) {
        const int n = (xb - x < U) ? xb - x : U;
        bf16x8 a[U][NPL], b[U];
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (j < n) {
#pragma unroll
                for (int p = 0; p < NPL; ++p) a[j][p] = __builtin_nontemporal_load(pa + (j * NPL + p) * 64);
                int kk = ks + j;
                while (kk >= KT) kk -= KT;
                b[j] = bact ? B[kk * 64 + lane] : zero;
            }
        }
#pragma unroll
        for (int j = 0; j < U; ++j) {
            if (j < n) {
#pragma unroll
                for (int p = 0; p < NPL; ++p) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][p], b[j], acc, 0, 0, 0);
                if (++ks == KT) {
                    *(f32x4 *)(slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
                    acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                    ks = 0;
                    ++tile;
                }
            }
        }
        pa += (size_t)n * NPL * 64;
    }
    if (ks != 0) *(f32x4 *)(slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
}

__device__ __forceinline__ int range_start(int tot, int w) { return (int)(((long)tot * w) / kWaves); }

// merge (max, sumexp, argmax) pairs; lower index wins ties
__device__ __forceinline__ void lse_merge(float &M, float &S, int &I, float m2, float s2, int i2) {
    if (m2 > M || (m2 == M && i2 < I)) I = i2;
    const float nm = fmaxf(M, m2);
    if (nm == -INFINITY) { M = nm; S = 0.f; return; }
    S = S * __expf(M - nm) + s2 * __expf(m2 - nm);
    M = nm;
}

template <int NPL, int U>
__device__ void gemm_phase(const GemmArgs &g, int wg, int nwg, GemmLds &L) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = (int)(((long)g.NT * wg) / nwg), t1 = (int)(((long)g.NT * (wg + 1)) / nwg);
    if (g.epi == EPI_HEAD && tid < 8) {
        L.run_max[tid] = -INFINITY;
        L.run_sum[tid] = 0.f;
        L.run_idx[tid] = 0x7fffffff;
    }
    bool have_scale = false;
    for (int ta = t0; ta < t1; ta += kMaxTilesPerRound) {
        const int tb = (t1 < ta + kMaxTilesPerRound) ? t1 : ta + kMaxTilesPerRound, nt = tb - ta;
        const int tot = nt * g.KT;
        const int xa = range_start(tot, wave), xb = range_start(tot, wave + 1);
        wave_stream<NPL, U>((const bf16x8 *)g.W + (size_t)ta * g.KT * NPL * 64, (const bf16x8 *)g.B, g.KT, xa, xb, g.m,
                            L.slots, wave, lane);
        if (!have_scale) {
            // per-token RMSNorm factor from the producer's partial sums of squares (fixed summation order)
            if (wave < g.m) {
                float s = 1.0f;
                if (g.ssq) {
                    s = 0.f;
                    for (int i = lane; i < g.n_ssq; i += 64) s += g.ssq[i * 8 + wave];
                    for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
                    s = 1.0f / sqrtf(s * g.inv_dim + g.eps);
                }
                if (lane == 0) L.scale[wave] = s;
            }
            have_scale = true;
        }
        __syncthreads();
        // reduce the slots of each tile in wavefront order
        for (int idx = tid; idx < nt * 128; idx += kThreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15;
            float v = 0.f;
            if (t < g.m) {
                const int x0 = T * g.KT, x1 = x0 + g.KT - 1;
                int w0 = (int)(((long)x0 * kWaves) / tot), w1 = (int)(((long)x1 * kWaves) / tot);
                while (w0 + 1 < kWaves && range_start(tot, w0 + 1) <= x0) ++w0;
                while (range_start(tot, w0) > x0) --w0;
                while (w1 + 1 < kWaves && range_start(tot, w1 + 1) <= x1) ++w1;
                while (range_start(tot, w1) > x1) --w1;
                for (int w = w0; w <= w1; ++w) {
                    if (range_start(tot, w) == range_start(tot, w + 1)) continue;   // wavefront had no work
                    const float *s = L.slots + (w + T) * 256;
                    v += s[t * 16 + i] + s[(t + 8) * 16 + i];
                }
            }
            L.red[idx] = v;
        }
        __syncthreads();
        // epilogue
        if (g.epi == EPI_STORE) {
            for (int idx = tid; idx < nt * 128; idx += kThreads) {
                const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                if (t < g.m && n < g.N) g.out[(size_t)t * g.ld + n] = L.scale[t] * L.red[idx];
            }
        } else if (g.epi == EPI_RESID) {
            for (int idx = tid; idx < nt * 128; idx += kThreads) {
                const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                float y = 0.f;
                if (t < g.m && n < g.N) {
                    y = g.resid[(size_t)t * g.ld + n] + L.scale[t] * L.red[idx];
                    g.out[(size_t)t * g.ld + n] = y;
                    if (g.Bnext) store_act((uint16_t *)g.Bnext, n, t, y * load_w(g.norm_w, g.norm_is_bf16, (size_t)n));
                }
                float s = y * y;
                for (int off = 8; off > 0; off >>= 1) s += __shfl_xor(s, off);
                if (i == 0 && g.ssq_next) g.ssq_next[(size_t)(ta + T) * 8 + t] = s;
            }
        } else if (g.epi == EPI_SWIGLU) {
            for (int idx = tid; idx < nt * 128; idx += kThreads) {
                const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, f = (ta + T) * 8 + i;
                if (t < g.m && i < 8 && f * 2 < g.N) {
                    const float gate = L.scale[t] * L.red[idx], up = L.scale[t] * L.red[idx + 8];
                    store_act((uint16_t *)g.Bnext, f, t, gate / (1.0f + __expf(-gate)) * up);
                }
            }
        } else if (g.epi == EPI_PACK) {
            for (int idx = tid; idx < nt * 128; idx += kThreads) {
                const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                if (t < g.m && n < g.N) store_act((uint16_t *)g.Bnext, n, t, L.scale[t] * L.red[idx]);
            }
        } else {  // EPI_HEAD: running (max, sum of exp, argmax) per token over this workgroup's rows
            if (g.logits) {
                for (int idx = tid; idx < nt * 128; idx += kThreads) {
                    const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                    if (t < g.m && n < g.N) g.logits[(size_t)t * g.N + n] = L.scale[t] * L.red[idx];
                }
            }
            if (wave < g.m) {
                const int t = wave;
                float M = -INFINITY, S = 0.f;
                int I = 0x7fffffff;
                for (int j = lane; j < nt * 16; j += 64) {
                    const int n = (ta + (j >> 4)) * 16 + (j & 15);
                    if (n < g.N) lse_merge(M, S, I, L.scale[t] * L.red[(j >> 4) * 128 + t * 16 + (j & 15)], 1.0f, n);
                }
                for (int off = 32; off > 0; off >>= 1) {
                    const float m2 = __shfl_xor(M, off), s2 = __shfl_xor(S, off);
                    const int i2 = __shfl_xor(I, off);
                    lse_merge(M, S, I, m2, s2, i2);
                }
                if (lane == 0) {
                    float rm = L.run_max[t], rsum = L.run_sum[t];
                    int ri = L.run_idx[t];
                    lse_merge(rm, rsum, ri, M, S, I);
                    L.run_max[t] = rm;
                    L.run_sum[t] = rsum;
                    L.run_idx[t] = ri;
                }
            }
        }
        __syncthreads();
    }
    if (g.epi != EPI_HEAD) return;

    // Vocabulary-wide combine: every workgroup publishes its per-token partial; the workgroup that arrives
    // last folds all partials in workgroup order (fixed order, lowest token id wins ties) and writes the result.
    if (tid < g.m) {
        float *p = g.head_part + ((size_t)wg * 8 + tid) * 4;
        p[0] = L.run_max[tid];
        p[1] = L.run_sum[tid];
        p[2] = __int_as_float(L.run_idx[tid]);
    }
    __threadfence();
    __syncthreads();
    if (tid == 0) {
        const unsigned old = __hip_atomic_fetch_add(g.head_counter, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
        L.flag = (old + 1u == (unsigned)nwg);
        if (L.flag) __hip_atomic_store(g.head_counter, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (!L.flag) return;
    __threadfence();
    if (wave < g.m) {
        const int t = wave;
        float M = -INFINITY, S = 0.f;
        int I = 0x7fffffff;
        for (int w = lane; w < nwg; w += 64) {
            const float *p = g.head_part + ((size_t)w * 8 + t) * 4;
            const float pm = __builtin_nontemporal_load(p), ps = __builtin_nontemporal_load(p + 1);
            const int pi = __float_as_int(__builtin_nontemporal_load(p + 2));
            lse_merge(M, S, I, pm, ps, pi);
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float m2 = __shfl_xor(M, off), s2 = __shfl_xor(S, off);
            const int i2 = __shfl_xor(I, off);
            lse_merge(M, S, I, m2, s2, i2);
        }
        if (lane == 0) {
            L.run_idx[t] = I;
            L.run_sum[t] = S;
            if (g.tok_out) g.tok_out[t] = I;
            if (g.conf_out) g.conf_out[t] = 1.0f / S;   // exp(max - logsumexp)
        }
    }
    __syncthreads();
    if (g.verify && tid == 0) {
        // Eq. 2 at temperature 0: the first row whose final-layer token differs from the token drafted
        // after it ends the accepted run and supplies the replacement.
        int acc = g.m - 1;
        for (int j = 0; j < g.m - 1; ++j)
            if (L.run_idx[j] != g.draft[j]) { acc = j; break; }
        *g.n_accept_out = acc;
        *g.next_out = L.run_idx[acc];
    }
}

template <int NPL, int U>
__global__ void __launch_bounds__(kThreads) k_gemm(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    gemm_phase<NPL, U>(g, blockIdx.x, gridDim.x, *reinterpret_cast<GemmLds *>(lds_raw));
}

// ---------------------------------------------------------------------------------------------------
// phase: rotary embedding + KV append + split-context grouped-query attention
// ---------------------------------------------------------------------------------------------------
// Work item (kv head g, split s): the cache positions [s*C, min((s+1)*C, pos0)) of that head, and for the
// last split also the call's m new rows (rotated, rounded to the cache type, appended to the cache, and
// attended to under the causal mask).  All G*m query rows of the group share the K/V tile staged in LDS.
// Each item writes an unnormalised partial (max, sum, o[dh]) per query row; the workgroup that finishes a
// head's last item combines the head's partials in split order and packs the result for the Wo GEMM.
template <typename KVT>
__device__ __forceinline__ float kv_to_f32(KVT v);
template <>
__device__ __forceinline__ float kv_to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float kv_to_f32<uint16_t>(uint16_t v) { return bf16_bits_to_f32(v); }
template <typename KVT>
__device__ __forceinline__ KVT f32_to_kv(float v);
template <>
__device__ __forceinline__ float f32_to_kv<float>(float v) { return v; }
template <>
__device__ __forceinline__ uint16_t f32_to_kv<uint16_t>(float v) { return f32_to_bf16_bits(v); }

constexpr int kAttnMaxRows = 32;    // G*m query rows per kv head (more are processed in passes)
// keys per work item: a chunk of cached positions plus up to 8 new rows; sized so that the K and V tiles fit LDS
constexpr int attn_max_keys(size_t kv_elem, int dh) { return (kv_elem * dh <= 256) ? 136 : 72; }

template <typename KVT, int DH>
__device__ void attn_phase(const AttnArgs &a, int wg, int nwg, char *lds_raw) {
    constexpr int KPAD = 16 / sizeof(KVT);            // row padding (elements) against LDS bank conflicts
    constexpr int KROW = DH + KPAD;
    constexpr int kAttnMaxKeys = attn_max_keys(sizeof(KVT), DH);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = a.Hq / a.Hkv, R = G * a.m;
    float *qs = (float *)lds_raw;                                  // [kAttnMaxRows][DH]
    float *sc = qs + kAttnMaxRows * DH;                            // [kAttnMaxRows][kAttnMaxKeys]
    float *st = sc + kAttnMaxRows * kAttnMaxKeys;                  // [kAttnMaxRows][2]
    int *flag = (int *)(st + kAttnMaxRows * 2);
    KVT *Ks = (KVT *)(flag + 4);                                   // [kAttnMaxKeys][KROW]
    KVT *Vs = Ks + kAttnMaxKeys * KROW;
    const int half = DH / 2;
    const int n_items = a.Hkv * a.S;
    const size_t part_row = DH + 2;

    for (int item = wg; item < n_items; item += nwg) {
        const int g = item / a.S, s = item % a.S;
        const int c0 = s * a.C, c1 = (c0 + a.C < a.pos0) ? c0 + a.C : a.pos0;
        const int nc = (c1 > c0) ? c1 - c0 : 0;
        const bool last = (s == a.S - 1);
        const int nk = nc + (last ? a.m : 0);
        KVT *Kg = (KVT *)a.Kc + (size_t)g * a.max_pos * DH, *Vg = (KVT *)a.Vc + (size_t)g * a.max_pos * DH;
        // stage the cached chunk (contiguous in memory) with 128-bit loads
        constexpr int VEC = 16 / sizeof(KVT);
        for (int idx = tid; idx < nc * (DH / VEC); idx += kThreads) {
            const int j = idx / (DH / VEC), c = idx % (DH / VEC);
            *(u32x4 *)(Ks + j * KROW + c * VEC) = *(const u32x4 *)(Kg + (size_t)(c0 + j) * DH + c * VEC);
            *(u32x4 *)(Vs + j * KROW + c * VEC) = *(const u32x4 *)(Vg + (size_t)(c0 + j) * DH + c * VEC);
        }
        // the call's own rows: rotate k, round to the cache type, append, and stage
        if (last) {
            for (int idx = tid; idx < a.m * half; idx += kThreads) {
                const int t = idx / half, i = idx % half;
                const float *kp = a.qkv + (size_t)t * a.ld + (size_t)a.Hq * DH + (size_t)g * DH;
                const float *vp = kp + (size_t)a.Hkv * DH;
                const float c = a.rope[(t * half + i) * 2], sn = a.rope[(t * half + i) * 2 + 1];
                const float x = kp[i], y = kp[i + half];
                const KVT k0 = f32_to_kv<KVT>(x * c - y * sn), k1 = f32_to_kv<KVT>(x * sn + y * c);
                const KVT v0 = f32_to_kv<KVT>(vp[i]), v1 = f32_to_kv<KVT>(vp[i + half]);
                Ks[(nc + t) * KROW + i] = k0;
                Ks[(nc + t) * KROW + i + half] = k1;
                Vs[(nc + t) * KROW + i] = v0;
                Vs[(nc + t) * KROW + i + half] = v1;
                const size_t o = (size_t)(a.pos0 + t) * DH;
                Kg[o + i] = k0;
                Kg[o + i + half] = k1;
                Vg[o + i] = v0;
                Vg[o + i + half] = v1;
            }
        }
        for (int r0 = 0; r0 < R; r0 += kAttnMaxRows) {
            const int nr = (R - r0 < kAttnMaxRows) ? R - r0 : kAttnMaxRows;
            // rotated, pre-scaled queries
            for (int idx = tid; idx < nr * half; idx += kThreads) {
                const int rr = idx / half, i = idx % half, r = r0 + rr, t = r / G, hq = g * G + r % G;
                const float *qp = a.qkv + (size_t)t * a.ld + (size_t)hq * DH;
                const float c = a.rope[(t * half + i) * 2], sn = a.rope[(t * half + i) * 2 + 1];
                const float x = qp[i], y = qp[i + half];
                qs[rr * DH + i] = (x * c - y * sn) * a.scale;
                qs[rr * DH + i + half] = (x * sn + y * c) * a.scale;
            }
            __syncthreads();
            // scores
            for (int p = tid; p < nr * nk; p += kThreads) {
                const int rr = p / nk, j = p % nk, t = (r0 + rr) / G;
                float acc = 0.f;
                const KVT *kr = Ks + j * KROW;
                const float *qr = qs + rr * DH;
#pragma unroll 2
                for (int e = 0; e < DH; e += VEC) {
                    const u32x4 kw = *(const u32x4 *)(kr + e);
                    if constexpr (sizeof(KVT) == 2) {
                        const f32x4 q0 = *(const f32x4 *)(qr + e), q1 = *(const f32x4 *)(qr + e + 4);
                        acc += q0[0] * __uint_as_float(kw[0] << 16) + q0[1] * __uint_as_float(kw[0] & 0xffff0000u) +
                               q0[2] * __uint_as_float(kw[1] << 16) + q0[3] * __uint_as_float(kw[1] & 0xffff0000u) +
                               q1[0] * __uint_as_float(kw[2] << 16) + q1[1] * __uint_as_float(kw[2] & 0xffff0000u) +
                               q1[2] * __uint_as_float(kw[3] << 16) + q1[3] * __uint_as_float(kw[3] & 0xffff0000u);
                    } else {
                        const f32x4 q0 = *(const f32x4 *)(qr + e);
                        acc += q0[0] * __uint_as_float(kw[0]) + q0[1] * __uint_as_float(kw[1]) +
                               q0[2] * __uint_as_float(kw[2]) + q0[3] * __uint_as_float(kw[3]);
                    }
                }
                if (j >= nc && j - nc > t) acc = -INFINITY;     // causal mask among the call's own rows
                sc[rr * kAttnMaxKeys + j] = acc;
            }
            __syncthreads();
            // per-row max and sum of exponentials (one wavefront per row)
            for (int rr = wave; rr < nr; rr += kWaves) {
                float mx = -INFINITY;
                for (int j = lane; j < nk; j += 64) mx = fmaxf(mx, sc[rr * kAttnMaxKeys + j]);
                for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
                float sum = 0.f;
                for (int j = lane; j < nk; j += 64) {
                    const float sv = sc[rr * kAttnMaxKeys + j];
                    const float pv = (sv == -INFINITY) ? 0.f : __expf(sv - mx);
                    sc[rr * kAttnMaxKeys + j] = pv;
                    sum += pv;
                }
                for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0) {
                    st[rr * 2] = mx;
                    st[rr * 2 + 1] = sum;
                }
            }
            __syncthreads();
            // o = P V
            for (int idx = tid; idx < nr * DH; idx += kThreads) {
                const int rr = idx / DH, e = idx % DH;
                float acc = 0.f;
                for (int j = 0; j < nk; ++j) acc += sc[rr * kAttnMaxKeys + j] * kv_to_f32<KVT>(Vs[j * KROW + e]);
                float *pr = a.part + (((size_t)g * a.S + s) * R + (r0 + rr)) * part_row;
                pr[e] = acc;
                if (e == 0) {
                    pr[DH] = st[rr * 2];
                    pr[DH + 1] = st[rr * 2 + 1];
                }
            }
            __syncthreads();
        }
        // publish; the last item of this head to finish combines
        __threadfence();
        __syncthreads();
        if (tid == 0) {
            const unsigned old = __hip_atomic_fetch_add(a.counters + g, 1u, __ATOMIC_ACQ_REL, __HIP_MEMORY_SCOPE_AGENT);
            flag[0] = (old + 1u == (unsigned)a.S);
            if (flag[0]) __hip_atomic_store(a.counters + g, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (flag[0]) {
            __threadfence();
            for (int idx = tid; idx < R * DH; idx += kThreads) {
                const int r = idx / DH, e = idx % DH, t = r / G, hq = g * G + r % G;
                float M = -INFINITY;
                for (int ss = 0; ss < a.S; ++ss)
                    M = fmaxf(M, __builtin_nontemporal_load(a.part + (((size_t)g * a.S + ss) * R + r) * part_row + DH));
                float den = 0.f, num = 0.f;
                for (int ss = 0; ss < a.S; ++ss) {
                    const float *pr = a.part + (((size_t)g * a.S + ss) * R + r) * part_row;
                    const float pm = __builtin_nontemporal_load(pr + DH);
                    const float w = (pm == -INFINITY) ? 0.f : __expf(pm - M);
                    den += w * __builtin_nontemporal_load(pr + DH + 1);
                    num += w * __builtin_nontemporal_load(pr + e);
                }
                store_act((uint16_t *)a.Bo, hq * DH + e, t, num / den);
            }
        }
        __syncthreads();
    }
}

constexpr size_t attn_lds_bytes(size_t kv_elem, int dh) {
    return (size_t)kAttnMaxRows * dh * 4 + (size_t)kAttnMaxRows * attn_max_keys(kv_elem, dh) * 4 + kAttnMaxRows * 2 * 4 + 16 +
           2 * (size_t)attn_max_keys(kv_elem, dh) * (dh + 16 / kv_elem) * kv_elem;
}
int attn_chunk(int kv_is_bf16, int dh) { return attn_max_keys(kv_is_bf16 ? 2 : 4, dh) - 8; }

template <typename KVT, int DH>
__global__ void __launch_bounds__(kThreads) k_attn(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    attn_phase<KVT, DH>(a, blockIdx.x, gridDim.x, lds_raw);
}

// ---------------------------------------------------------------------------------------------------
// host-side launchers
// ---------------------------------------------------------------------------------------------------
static inline hipStream_t S(void *s) { return (hipStream_t)s; }

int launch_pack_weights(const void *src, const void *src2, int src_is_bf16, int64_t N, int64_t K, int mode, void *dst,
                        void *stream) {
    const int64_t rows = (mode == 0) ? N : 2 * N;
    const int64_t NT = (rows + 15) / 16, KT = (K + 31) / 32;
    const int64_t threads = NT * KT * 64;
    hipLaunchKernelGGL(k_pack_weights, dim3((unsigned)((threads + 255) / 256)), dim3(256), 0, S(stream), src, src2, src_is_bf16,
                       N, K, NT, KT, mode, (uint16_t *)dst);
    return (int)hipGetLastError();
}

int launch_copy(const void *src, void *dst, size_t bytes, void *stream) {
    hipLaunchKernelGGL(k_copy16, dim3(2048), dim3(256), 0, S(stream), (const u32x4 *)src, (u32x4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}

int launch_zero(void *dst, size_t bytes, void *stream) {
    hipLaunchKernelGGL(k_zero16, dim3(1024), dim3(256), 0, S(stream), (u32x4 *)dst, bytes / 16);
    return (int)hipGetLastError();
}

int launch_embed(const EmbedArgs &a, void *stream) {
    hipLaunchKernelGGL(k_embed, dim3(32), dim3(256), 0, S(stream), a);
    return (int)hipGetLastError();
}

int launch_pack(const PackArgs &a, const LaunchCtx &c) {
    const int work = (a.d / 16) * a.m;
    int grid = (work + 255) / 256;
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL(k_pack, dim3(grid), dim3(256), 0, S(c.stream), a);
    return (int)hipGetLastError();
}

int launch_gemm(const GemmArgs &g, int planes, const LaunchCtx &c) {
    int grid = c.n_wg < g.NT ? c.n_wg : g.NT;
    if (grid < 1) grid = 1;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm<1, 8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(GemmLds));
        if (e == hipSuccess)
            e = hipFuncSetAttribute((const void *)k_gemm<3, 2>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(GemmLds));
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    if (planes == 1)
        hipLaunchKernelGGL((k_gemm<1, 8>), dim3(grid), dim3(kThreads), sizeof(GemmLds), S(c.stream), g);
    else
        hipLaunchKernelGGL((k_gemm<3, 2>), dim3(grid), dim3(kThreads), sizeof(GemmLds), S(c.stream), g);
    return (int)hipGetLastError();
}

template <typename KVT, int DH>
static int launch_attn_t(const AttnArgs &a, const LaunchCtx &c) {
    const size_t lds = attn_lds_bytes(sizeof(KVT), DH);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn<KVT, DH>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    int grid = a.Hkv * a.S;
    if (grid > c.n_wg) grid = c.n_wg;
    hipLaunchKernelGGL((k_attn<KVT, DH>), dim3(grid), dim3(kThreads), lds, S(c.stream), a);
    return (int)hipGetLastError();
}

int launch_attn(const AttnArgs &a, const LaunchCtx &c) {
    if (a.kv_is_bf16) {
        if (a.dh == 128) return launch_attn_t<uint16_t, 128>(a, c);
        if (a.dh == 64) return launch_attn_t<uint16_t, 64>(a, c);
    } else {
        if (a.dh == 128) return launch_attn_t<float, 128>(a, c);
        if (a.dh == 64) return launch_attn_t<float, 64>(a, c);
    }
    return (int)hipErrorInvalidValue;
}

int device_info(int *n_cu) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    hipDeviceProp_t p;
    e = hipGetDeviceProperties(&p, dev);
    if (e != hipSuccess) return (int)e;
    *n_cu = p.multiProcessorCount;
    return 0;
}

const char *hip_error_text(int code) { return hipGetErrorString((hipError_t)code); }
int stream_sync(void *stream) { return (int)hipStreamSynchronize(S(stream)); }
void *event_create() {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return (void *)e;
}
void event_destroy(void *ev) { if (ev) (void)hipEventDestroy((hipEvent_t)ev); }
int event_record(void *ev, void *stream) { return (int)hipEventRecord((hipEvent_t)ev, S(stream)); }
int event_elapsed_ms(void *start, void *stop, float *ms) { return (int)hipEventElapsedTime(ms, (hipEvent_t)start, (hipEvent_t)stop); }
int stream_sync_event(void *ev) { return (int)hipEventSynchronize((hipEvent_t)ev); }
void *pinned_alloc(size_t bytes) {
    void *p = nullptr;
    if (hipHostMalloc(&p, bytes, hipHostMallocDefault) != hipSuccess) return nullptr;
    return p;
}
void pinned_free(void *p) { if (p) (void)hipHostFree(p); }

}  // namespace ad
