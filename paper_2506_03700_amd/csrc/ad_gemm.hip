// The weight-streaming skinny GEMM   out[t][n] = sum_k W[n][k] * act[t][k]   for m <= 8 tokens, with the
// epilogues of the layer step and of the vocabulary pass fused in.  Every projection of the decoder layer
// (QKV, attention output, gate/up, down) and the LM head of Eq. 1 / Eq. 2 run through this kernel.
//
// The contraction is bound by reading W once from HBM (about m flop per byte), so the kernel is organised
// around the weight stream: W is stored as 1 KiB MFMA A-operand tiles (see ad_internal.h), a workgroup owns
// a contiguous block of row tiles, and each of its 16 wavefronts streams contiguous pieces with 128-bit
// loads, two batches in flight.  The MFMA (16x16x32 bf16) is only the cheapest way to multiply a tile by
// the 2m hi/lo activation columns; it is idle most of the time.
//
// Two ways of feeding the activations (the B operand):
//  * stationary (QKV, gate/up, exit-head transform, LM head: several row tiles per workgroup, K = d):
//    wavefront w owns a fixed K slice for all the workgroup's tiles and keeps its slice of B in registers.
//    B is built in the prologue straight from the fp32 activations: x * norm_w split into bf16 hi/lo
//    (the RMSNorm's 1/rms is a per-token scalar, applied in the epilogue), together with the slice's sum
//    of squares; or it is loaded from a packed block an earlier epilogue wrote.
//  * streamed (attention output, down: one or two row tiles per workgroup, K up to d_ffn): the (tile,
//    k-step) pairs of the workgroup are cut into 16 contiguous ranges and B tiles are loaded next to the
//    A tiles from the packed block the previous kernel wrote (L2 hits).
// Partial accumulators meet in LDS and are summed in wavefront order (fixed order: reproducible).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_device.h"
#include "ad_internal.h"

namespace ad {

constexpr int kTilesPerRound = 8;       // stationary mode: row tiles reduced together
constexpr int kKsMax = 10;              // stationary mode: most k-steps per wavefront (K <= 16 * 10 * 32 = 5120)

struct GemmLds {
    // stationary: [tile 0..8)[wave][token 0..8)[row 0..16)      streamed: [slot][col 0..16)[row 0..16)
    float slots[kTilesPerRound * kWaves * 8 * 16];
    float red[kTilesPerRound * 128];    // [tile][token][row]
    float ssq_part[kWaves * 8];
    float scale[8];
    float run_max[8], run_sum[8];
    int run_idx[8];
};

__device__ __forceinline__ int part_start(int tot, int w) { return (int)(((long)tot * w) / kWaves); }

// merge (max, sumexp, argmax) pairs; the lower index wins ties
__device__ __forceinline__ void lse_merge(float &M, float &S, int &I, float m2, float s2, int i2) {
    if (m2 > M || (m2 == M && i2 < I)) I = i2;
    const float nm = fmaxf(M, m2);
    if (nm == -INFINITY) { M = nm; S = 0.f; return; }
    S = S * __expf(M - nm) + s2 * __expf(m2 - nm);
    M = nm;
}

// ---- epilogue on a reduced round: L.red[T*128 + t*16 + i] holds row (ta+T)*16+i of token t -------------
__device__ __forceinline__ void epilogue(const GemmArgs &g, GemmLds &L, int ta, int nt, int tid, int lane, int wave) {
    if (g.epi == EPI_STORE) {
        for (int idx = tid; idx < nt * 128; idx += kThreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) g.out[(size_t)t * g.ld + n] = L.scale[t] * L.red[idx];
        }
    } else if (g.epi == EPI_RESID) {
        for (int idx = tid; idx < nt * 128; idx += kThreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) g.out[(size_t)t * g.ld + n] = g.resid[(size_t)t * g.ld + n] + L.scale[t] * L.red[idx];
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
}

// ---- stationary mode -------------------------------------------------------------------------------------
template <int NPL, int KSW>
__device__ __forceinline__ void load_tile_slice(bf16x8 (&a)[KSW][NPL], const bf16x8 *p, int nks) {
    if (nks == KSW) {   // the common case: straight-line loads
#pragma unroll
        for (int j = 0; j < KSW; ++j)
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = __builtin_nontemporal_load(p + (size_t)(j * NPL + q) * 64);
    } else {
#pragma unroll
        for (int j = 0; j < KSW; ++j)
            if (j < nks) {
#pragma unroll
                for (int q = 0; q < NPL; ++q) a[j][q] = __builtin_nontemporal_load(p + (size_t)(j * NPL + q) * 64);
            }
    }
}

template <int NPL, int KSW>
__device__ __forceinline__ void mma_tile_slice(const bf16x8 (&a)[KSW][NPL], const bf16x8 (&b)[KSW], int nks, float *slot,
                                               int lane, int m) {
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    if (nks == KSW) {
#pragma unroll
        for (int j = 0; j < KSW; ++j)
#pragma unroll
            for (int q = 0; q < NPL; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][q], b[j], acc, 0, 0, 0);
    } else {
#pragma unroll
        for (int j = 0; j < KSW; ++j)
            if (j < nks) {
#pragma unroll
                for (int q = 0; q < NPL; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][q], b[j], acc, 0, 0, 0);
            }
    }
    // columns n and n+8 hold the hi and lo partial products of token n
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] += __shfl_xor(acc[c], 8);
    const int n = lane & 15;
    if (n < m) *(f32x4 *)(slot + n * 16 + (lane >> 4) * 4) = acc;
}

// KSW: most k-steps a wavefront owns (its B slice and one weight-tile slice take 4*KSW registers each).
// DB: keep the next tile's slice in flight while the current one is multiplied (needs a second buffer).
template <int NPL, int KSW, bool DB>
__device__ void gemm_stationary(const GemmArgs &g, int wg, int nwg, GemmLds &L) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4, t_lane = n & 7;
    const int t0 = (int)(((long)g.NT * wg) / nwg), t1 = (int)(((long)g.NT * (wg + 1)) / nwg);
    const int ks0 = part_start(g.KT, wave), nks = part_start(g.KT, wave + 1) - ks0;
    if (g.epi == EPI_HEAD && tid < 8) {
        L.run_max[tid] = -INFINITY;
        L.run_sum[tid] = 0.f;
        L.run_idx[tid] = 0x7fffffff;
    }
    // first weight tile goes in flight before anything else
    bf16x8 a0[KSW][NPL], a1[DB ? KSW : 1][NPL], b[KSW];
    const bf16x8 *wp = (const bf16x8 *)g.W + ((size_t)t0 * g.KT + ks0) * NPL * 64 + lane;
    const size_t tstride = (size_t)g.KT * NPL * 64;
    if (t0 < t1) load_tile_slice<NPL, KSW>(a0, wp, nks);

    // B slice of this wavefront
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    float ssq = 0.f;
    if (g.x) {
#pragma unroll
        for (int j = 0; j < KSW; ++j) {
            b[j] = zero;
            const int k = (ks0 + j) * 32 + gq * 8;
            if (j < nks && t_lane < g.m && k < g.K) {
                const float *xp = g.x + (size_t)t_lane * g.ldx + k;
                const f32x4 x0 = *(const f32x4 *)xp, x1 = *(const f32x4 *)(xp + 4);
                float w[8];
                load_w8(g.norm_w, g.norm_is_bf16, (size_t)k, w);
                union { bf16x8 v; uint16_t u[8]; } cv;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float xv = e < 4 ? x0[e] : x1[e - 4];
                    ssq += xv * xv;
                    uint16_t hi, lo;
                    split_hi_lo(xv * w[e], hi, lo);
                    cv.u[e] = (n < 8) ? hi : lo;
                }
                b[j] = cv.v;
            }
        }
        // sum of squares of this K slice, per token (lanes n < 8 of the four lane groups)
        ssq += __shfl_xor(ssq, 16);
        ssq += __shfl_xor(ssq, 32);
        if (lane < 8) L.ssq_part[wave * 8 + lane] = ssq;
    } else {
#pragma unroll
        for (int j = 0; j < KSW; ++j) b[j] = (j < nks && t_lane < g.m) ? ((const bf16x8 *)g.B)[(size_t)(ks0 + j) * 64 + lane] : zero;
    }
    __syncthreads();
    if (tid < 8) {
        float s = 1.0f;
        if (g.x && g.norm_w) {
            s = 0.f;
            for (int w = 0; w < kWaves; ++w) s += L.ssq_part[w * 8 + tid];
            s = 1.0f / sqrtf(s * g.inv_dim + g.eps);
        }
        L.scale[tid] = s;
    }

    auto finish_round = [&](int done) {
        // tiles [ta, done) of this round are in the slots: sum them over the wavefronts, then the epilogue
        const int ta = t0 + ((done - t0 - 1) / kTilesPerRound) * kTilesPerRound, nt = done - ta;
        __syncthreads();
        for (int idx = tid; idx < nt * 128; idx += kThreads) {
            const int T = idx >> 7, tt = (idx >> 4) & 7, i = idx & 15;
            float v = 0.f;
            if (tt < g.m) {
                const float *s = L.slots + (size_t)T * kWaves * 128 + tt * 16 + i;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) v += s[w * 128];
            }
            L.red[idx] = v;
        }
        __syncthreads();
        epilogue(g, L, ta, nt, tid, lane, wave);
        __syncthreads();
    };
    if constexpr (DB) {
        for (int t = t0; t < t1; t += 2) {
            // tile t is in a0 (already in flight); tile t+1 goes into a1, then tile t+2 into a0
            const int T0 = (t - t0) % kTilesPerRound;
            if (t + 1 < t1) load_tile_slice<NPL, KSW>(a1, wp + tstride, nks);
            mma_tile_slice<NPL, KSW>(a0, b, nks, L.slots + ((size_t)T0 * kWaves + wave) * 128, lane, g.m);
            if (t + 2 < t1) load_tile_slice<NPL, KSW>(a0, wp + 2 * tstride, nks);
            bool round_end = (t + 1 == t1);
            if (!round_end) {
                mma_tile_slice<NPL, KSW>(a1, b, nks, L.slots + ((size_t)(T0 + 1) * kWaves + wave) * 128, lane, g.m);
                round_end = (T0 + 1 == kTilesPerRound - 1) || (t + 2 >= t1);
            }
            wp += 2 * tstride;
            if (round_end) finish_round((t + 2 < t1) ? t + 2 : t1);
        }
    } else {
        for (int t = t0; t < t1; ++t) {
            const int T0 = (t - t0) % kTilesPerRound;
            mma_tile_slice<NPL, KSW>(a0, b, nks, L.slots + ((size_t)T0 * kWaves + wave) * 128, lane, g.m);
            wp += tstride;
            if (t + 1 < t1) load_tile_slice<NPL, KSW>(a0, wp, nks);
            if (T0 == kTilesPerRound - 1 || t + 1 == t1) finish_round(t + 1);
        }
    }
    if (g.epi == EPI_HEAD && tid < g.m) {
        float *p = g.head_part + ((size_t)wg * 8 + tid) * 4;
        p[0] = L.run_max[tid];
        p[1] = L.run_sum[tid];
        p[2] = __int_as_float(L.run_idx[tid]);
    }
}

// ---- streamed mode -----------------------------------------------------------------------------------------
template <int NPL, int U>
__device__ void gemm_streamed(const GemmArgs &g, int wg, int nwg, GemmLds &L) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t0 = (int)(((long)g.NT * wg) / nwg), t1 = (int)(((long)g.NT * (wg + 1)) / nwg);
    if (tid < 8) L.scale[tid] = 1.0f;
    const bool bact = (lane & 7) < g.m;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const bf16x8 *B = (const bf16x8 *)g.B;
    const int KT = g.KT;
    for (int ta = t0; ta < t1; ta += 8) {
        const int tb = (t1 < ta + 8) ? t1 : ta + 8, nt = tb - ta;
        const int tot = nt * KT;
        const int xa = part_start(tot, wave), xb = part_start(tot, wave + 1);
        // the wavefront's contiguous range of (tile, k-step) pairs, U at a time, two batches in flight
        int tile = xa / KT, ks = xa % KT;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        const bf16x8 *pa = (const bf16x8 *)g.W + ((size_t)ta * KT + xa) * NPL * 64 + lane;
        bf16x8 a0[U][NPL], b0[U], a1[U][NPL], b1[U];
        auto load = [&](bf16x8 (&a)[U][NPL], bf16x8 (&b)[U], const bf16x8 *p, int x, int ks_at) {
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (x + j < xb) {
#pragma unroll
                    for (int q = 0; q < NPL; ++q) a[j][q] = __builtin_nontemporal_load(p + (size_t)(j * NPL + q) * 64);
                    int kk = ks_at + j;
                    while (kk >= KT) kk -= KT;
                    b[j] = bact ? B[(size_t)kk * 64 + lane] : zero;
                }
        };
        auto mma = [&](const bf16x8 (&a)[U][NPL], const bf16x8 (&b)[U], int x) {
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (x + j < xb) {
#pragma unroll
                    for (int q = 0; q < NPL; ++q) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][q], b[j], acc, 0, 0, 0);
                    if (++ks == KT) {
                        *(f32x4 *)(L.slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
                        acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                        ks = 0;
                        ++tile;
                    }
                }
        };
        if (xa < xb) load(a0, b0, pa, xa, ks);
        for (int x = xa; x < xb; x += 2 * U) {
            int ks_next = ks + U;
            while (ks_next >= KT) ks_next -= KT;
            if (x + U < xb) load(a1, b1, pa + (size_t)U * NPL * 64, x + U, ks_next);
            mma(a0, b0, x);
            int ks_next2 = ks + U;     // ks has advanced by the first batch
            while (ks_next2 >= KT) ks_next2 -= KT;
            if (x + 2 * U < xb) load(a0, b0, pa + (size_t)2 * U * NPL * 64, x + 2 * U, ks_next2);
            if (x + U < xb) mma(a1, b1, x + U);
            pa += (size_t)2 * U * NPL * 64;
        }
        if (ks != 0) *(f32x4 *)(L.slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
        __syncthreads();
        // sum the slots of each tile in wavefront order
        for (int idx = tid; idx < nt * 128; idx += kThreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15;
            float v = 0.f;
            if (t < g.m) {
                const int x0 = T * KT, x1 = x0 + KT - 1;
                int w0 = (int)(((long)x0 * kWaves) / tot), w1 = (int)(((long)x1 * kWaves) / tot);
                while (w0 + 1 < kWaves && part_start(tot, w0 + 1) <= x0) ++w0;
                while (part_start(tot, w0) > x0) --w0;
                while (w1 + 1 < kWaves && part_start(tot, w1 + 1) <= x1) ++w1;
                while (part_start(tot, w1) > x1) --w1;
                for (int w = w0; w <= w1; ++w) {
                    if (part_start(tot, w) == part_start(tot, w + 1)) continue;   // wavefront had no work
                    const float *s = L.slots + (w + T) * 256;
                    v += s[t * 16 + i] + s[(t + 8) * 16 + i];
                }
            }
            L.red[idx] = v;
        }
        __syncthreads();
        epilogue(g, L, ta, nt, tid, lane, wave);
        __syncthreads();
    }
}

enum { GEMM_STATIONARY_8 = 1, GEMM_STATIONARY_WIDE = 2 };   // kernel variants of the stationary mode

template <int NPL, int MODE>
__global__ void __launch_bounds__(kThreads) k_gemm(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    GemmLds &L = *reinterpret_cast<GemmLds *>(lds_raw);
    if constexpr (MODE == GEMM_STATIONARY_8)
        gemm_stationary<NPL, 8, true>(g, blockIdx.x, gridDim.x, L);
    else if constexpr (MODE == GEMM_STATIONARY_WIDE)
        gemm_stationary<NPL, (NPL == 1 ? kKsMax : 4), false>(g, blockIdx.x, gridDim.x, L);
    else
        gemm_streamed<NPL, (NPL == 1 ? 4 : 2)>(g, blockIdx.x, gridDim.x, L);
}

// Second pass of the vocabulary reduction: fold the per-workgroup (max, sum of exp, argmax) partials in
// workgroup order (fixed order; the lowest token id wins ties), one wavefront per token, then apply the
// verification rule of Eq. 2 at temperature 0 if asked.
__global__ void __launch_bounds__(512) k_head_combine(GemmArgs g) {
    __shared__ int idx_sh[8];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (wave < g.m) {
        const int t = wave;
        float M = -INFINITY, S = 0.f;
        int I = 0x7fffffff;
        for (int w = lane; w < g.n_parts; w += 64) {
            const float *p = g.head_part + ((size_t)w * 8 + t) * 4;
            lse_merge(M, S, I, p[0], p[1], __float_as_int(p[2]));
        }
        for (int off = 32; off > 0; off >>= 1) {
            const float m2 = __shfl_xor(M, off), s2 = __shfl_xor(S, off);
            const int i2 = __shfl_xor(I, off);
            lse_merge(M, S, I, m2, s2, i2);
        }
        if (lane == 0) {
            idx_sh[t] = I;
            if (g.tok_out) g.tok_out[t] = I;
            if (g.conf_out) g.conf_out[t] = 1.0f / S;   // exp(max - logsumexp)
        }
    }
    __syncthreads();
    if (g.verify && threadIdx.x == 0) {
        // the first row whose final-layer token differs from the token drafted after it ends the accepted
        // run and supplies the replacement
        int acc = g.m - 1;
        for (int j = 0; j < g.m - 1; ++j)
            if (idx_sh[j] != g.draft[j]) { acc = j; break; }
        *g.n_accept_out = acc;
        *g.next_out = idx_sh[acc];
    }
}

template <int NPL, int MODE>
static int launch_one(const GemmArgs &g, int grid, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm<NPL, MODE>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(GemmLds));
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_gemm<NPL, MODE>), dim3(grid), dim3(kThreads), sizeof(GemmLds), s, g);
    return (int)hipGetLastError();
}

int launch_gemm(const GemmArgs &g, int planes, const LaunchCtx &c) {
    int grid = c.n_wg < g.NT ? c.n_wg : g.NT;
    if (grid < 1) grid = 1;
    hipStream_t s = (hipStream_t)c.stream;
    int rc;
    if (g.mode == GEMM_STATIONARY) {
        // k-steps per wavefront: up to 8 runs double-buffered; bf16 up to 10 and fp32 up to 4 single-buffered
        const int ksw = (g.KT + kWaves - 1) / kWaves;
        if (planes == 1) {
            if (ksw <= 8) rc = launch_one<1, GEMM_STATIONARY_8>(g, grid, s);
            else if (ksw <= kKsMax) rc = launch_one<1, GEMM_STATIONARY_WIDE>(g, grid, s);
            else return (int)hipErrorInvalidValue;
        } else {
            if (ksw <= 4) rc = launch_one<3, GEMM_STATIONARY_WIDE>(g, grid, s);
            else return (int)hipErrorInvalidValue;
        }
    } else {
        rc = planes == 1 ? launch_one<1, GEMM_STREAMED>(g, grid, s) : launch_one<3, GEMM_STREAMED>(g, grid, s);
    }
    if (rc) return rc;
    if (g.epi == EPI_HEAD) {
        GemmArgs h = g;
        h.n_parts = grid;
        hipLaunchKernelGGL(k_head_combine, dim3(1), dim3(512), 0, s, h);
        rc = (int)hipGetLastError();
    }
    return rc;
}

int gemm_max_stationary_k(int planes) { return (planes == 1 ? kKsMax : 4) * kWaves * 32; }

}  // namespace ad
