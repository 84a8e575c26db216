// The weight-streaming skinny GEMM   out[t][n] = sum_k W[n][k] * act[t][k]   for m <= 8 tokens, with the
// epilogues of the layer step and of the vocabulary pass fused in.  Every projection of the decoder layer
// (QKV, attention output, gate/up, down) and the LM head of Eq. 1 / Eq. 2 run through this kernel.
//
// The contraction is bound by reading W once from HBM (about m flop per byte), so the kernel is organised
// around the weight stream: W is stored as 1 KiB MFMA A-operand tiles (see ad_internal.h), a workgroup owns
// a contiguous block of row tiles, and each of its wavefronts streams contiguous pieces with 128-bit
// loads, two batches in flight.  The MFMA (16x16x32 bf16) is only the cheapest way to multiply a tile by
// the 2m hi/lo activation columns; it is idle most of the time.
//
// Two ways of feeding the activations (the B operand):
//  * stationary (QKV, gate/up, exit-head transform, LM head: several row tiles per workgroup, K = d):
//    8 wavefronts per workgroup; wavefront w owns a fixed K slice for all the workgroup's tiles and keeps its
//    slice of B in registers.
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
constexpr int kStatWaves = 8;           // stationary mode: wavefronts per workgroup (512 threads, up to 256 registers each)
constexpr int kStatThreads = kStatWaves * 64;
constexpr int kKsMax = 20;              // stationary mode: most k-steps per wavefront (K <= 8 * 20 * 32 = 5120)

struct GemmLds {
    // stationary: [tile 0..8)[wave][token 0..8)[row 0..16)      streamed: [slot][col 0..16)[row 0..16)
    float slots[kTilesPerRound * kWaves * 8 * 16];
    float red[kTilesPerRound * 128];    // [tile][token][row]
    float ssq_part[kWaves * 8];
    float scale[8];
    float run_max[8], run_sum[8];
    int run_idx[8];
};

__device__ __forceinline__ int part_start(int tot, int w, int nw = kWaves) { return (int)(((long)tot * w) / nw); }

// merge (max, sumexp, argmax) pairs; the lower index wins ties
__device__ __forceinline__ void lse_merge(float &M, float &S, int &I, float m2, float s2, int i2) {
    if (m2 > M || (m2 == M && i2 < I)) I = i2;
    const float nm = fmaxf(M, m2);
    if (nm == -INFINITY) { M = nm; S = 0.f; return; }
    S = S * __expf(M - nm) + s2 * __expf(m2 - nm);
    M = nm;
}

// ---- epilogue on a reduced round: L.red[T*128 + t*16 + i] holds row (ta+T)*16+i of token t -------------
__device__ __forceinline__ void epilogue(const GemmArgs &g, GemmLds &L, int ta, int nt, int tid, int lane, int wave, int nthreads) {
    if (g.epi == EPI_STORE) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) g.out[(size_t)t * g.ld + n] = L.scale[t] * L.red[idx];
        }
    } else if (g.epi == EPI_RESID) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) g.out[(size_t)t * g.ld + n] = g.resid[(size_t)t * g.ld + n] + L.scale[t] * L.red[idx];
        }
    } else if (g.epi == EPI_SWIGLU) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, f = (ta + T) * 8 + i;
            if (t < g.m && i < 8 && f * 2 < g.N) {
                const float gate = L.scale[t] * L.red[idx], up = L.scale[t] * L.red[idx + 8];
                store_act((uint16_t *)g.Bnext, f, t, gate / (1.0f + __expf(-gate)) * up);
            }
        }
    } else if (g.epi == EPI_PACK) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) store_act((uint16_t *)g.Bnext, n, t, L.scale[t] * L.red[idx]);
        }
    } else {  // EPI_HEAD: running (max, sum of exp, argmax) per token over this workgroup's rows
        if (g.logits) {
            for (int idx = tid; idx < nt * 128; idx += nthreads) {
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
// The wavefront's weight stream is a sequence of chunks of CH k-steps: its K slice of tile t0, of tile t0+1, ...
// (a slice of nks k-steps is NCH = ceil(nks / CH) chunks).  Two chunk buffers alternate, so one chunk is in
// flight while the other is multiplied.
template <int NPL, int CH>
__device__ __forceinline__ void load_chunk(bf16x8 (&a)[CH][NPL], const bf16x8 *p, int n) {
    if (n == CH) {   // the common case: straight-line loads
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = __builtin_nontemporal_load(p + (size_t)(j * NPL + q) * 64);
    } else {
#pragma unroll
        for (int j = 0; j < CH; ++j)
            if (j < n) {
#pragma unroll
                for (int q = 0; q < NPL; ++q) a[j][q] = __builtin_nontemporal_load(p + (size_t)(j * NPL + q) * 64);
            }
    }
}

// one fp32 activation slice -> bf16 hi (lanes n < 8) or lo (lanes n >= 8) B operand registers
__device__ __forceinline__ bf16x8 make_b(const f32x4 &x0, const f32x4 &x1, const float (&w)[8], bool lo_lane, float &ssq) {
    union { bf16x8 v; uint16_t u[8]; } cv;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const float xv = e < 4 ? x0[e] : x1[e - 4];
        ssq += xv * xv;
        uint16_t hi, lo;
        split_hi_lo(xv * w[e], hi, lo);
        cv.u[e] = lo_lane ? lo : hi;
    }
    return cv.v;
}

template <int NPL, int CH>
__device__ void gemm_stationary(const GemmArgs &g, int wg, int nwg, GemmLds &L) {
    constexpr int NCHMAX = (kKsMax + CH - 1) / CH, KSB = NCHMAX * CH;   // B registers cover whole chunks
    constexpr int kWaves = kStatWaves, kThreads = kStatThreads;         // this mode's workgroup shape
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4, t_lane = n & 7;
    const int t0 = (int)(((long)g.NT * wg) / nwg), t1 = (int)(((long)g.NT * (wg + 1)) / nwg);
    const int ks0 = part_start(g.KT, wave, kWaves), nks = part_start(g.KT, wave + 1, kWaves) - ks0;
    const int nch = (nks + CH - 1) / CH;                 // chunks per tile (0 if this wavefront has no K slice)
    const int total = (t1 - t0) * nch;                   // chunks in this wavefront's stream
    if (g.epi == EPI_HEAD && tid < 8) {
        L.run_max[tid] = -INFINITY;
        L.run_sum[tid] = 0.f;
        L.run_idx[tid] = 0x7fffffff;
    }
    bf16x8 a0[CH][NPL], a1[CH][NPL], b[KSB];
    const bf16x8 *wbase = (const bf16x8 *)g.W + ((size_t)t0 * g.KT + ks0) * NPL * 64 + lane;
    const size_t tstride = (size_t)g.KT * NPL * 64;
    auto chunk_ptr = [&](int c) { return wbase + (size_t)(c / nch) * tstride + (size_t)(c % nch) * CH * NPL * 64; };
    auto chunk_len = [&](int c) { const int r = nks - (c % nch) * CH; return r < CH ? r : CH; };
    // the first two weight chunks go in flight before anything else
    if (total > 0) load_chunk<NPL, CH>(a0, chunk_ptr(0), chunk_len(0));
    if (total > 1) load_chunk<NPL, CH>(a1, chunk_ptr(1), chunk_len(1));

    // B slice of this wavefront.  Its K slice is read in passes of 8 k-steps = 256 inputs: lane l takes inputs
    // 4l .. 4l+3 of every token (one coalesced 128-bit load per token and pass, all issued up front), multiplies
    // by the norm weights, splits into bf16 hi/lo and writes them, in B-operand order, into a wavefront-private
    // strip of LDS from which each lane then reads its operand registers.  The strip aliases the reduction slots,
    // which are not in use yet.
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const bool lane_on = t_lane < g.m;
    constexpr int NPASS = KSB / 8;
    // 16-byte units of the strip are permuted (unit u -> u ^ ((u >> 4) & 15)) so that the 8-byte writes of a
    // wavefront, which all go to the same operand column, spread over the LDS banks
    uint16_t *strip16 = reinterpret_cast<uint16_t *>(L.slots) + (size_t)wave * 8 * 512;
    const bf16x8 *strip = reinterpret_cast<const bf16x8 *>(strip16);
    auto sw = [](int u) { return u ^ ((u >> 4) & 15); };
    if (g.x) {
        f32x4 xr[NPASS][8], wr[NPASS];
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int k = (ks0 + p * 8) * 32 + lane * 4;
            const int kc = (k > g.K - 4) ? g.K - 4 : k;              // clamped address, masked result
            if (p * 8 < nks) {
                float w8[8];
                load_w8(g.norm_w, g.norm_is_bf16, (size_t)(kc & ~7), w8);
                const int o = kc & 4;
                wr[p] = (f32x4){w8[o], w8[o + 1], w8[o + 2], w8[o + 3]};
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < g.m) xr[p][t] = *(const f32x4 *)(g.x + (size_t)t * g.ldx + kc);
            }
        }
        float ssq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            const int jn = (nks - p * 8 < 8) ? nks - p * 8 : 8;       // k-steps of this pass (<= 0: none)
            if (jn > 0) {
                const int k = (ks0 + p * 8) * 32 + lane * 4;
                const bool k_on = (lane >> 3) < jn && k < g.K;
                // position of inputs 4l..4l+3 in the operand: k-step l/8, lane group (l%8)/2, elements (l%2)*4..+3
                const int u0 = (lane >> 3) * 64 + ((lane & 7) >> 1) * 16;     // unit of column 0
#pragma unroll
                for (int t = 0; t < 8; ++t)
                    if (t < g.m) {
                        union { uint16_t u[4]; uint64_t v; } hi, lo;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const float xv = k_on ? xr[p][t][e] : 0.f;
                            ssq[t] += xv * xv;
                            split_hi_lo(xv * wr[p][e], hi.u[e], lo.u[e]);
                        }
                        *(uint64_t *)(strip16 + sw(u0 + t) * 8 + (lane & 1) * 4) = hi.v;
                        *(uint64_t *)(strip16 + sw(u0 + 8 + t) * 8 + (lane & 1) * 4) = lo.v;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) b[p * 8 + jj] = (lane_on && jj < jn) ? strip[sw(jj * 64 + lane)] : zero;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int jj = 0; jj < 8; ++jj) b[p * 8 + jj] = zero;
            }
        }
        // sum of squares of this K slice, per token, over the 64 lanes (fixed butterfly order)
#pragma unroll
        for (int t = 0; t < 8; ++t)
            if (t < g.m) {
                float v = ssq[t];
                for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
                if (lane == 0) L.ssq_part[wave * 8 + t] = v;
            }
    } else {
#pragma unroll
        for (int j = 0; j < KSB; ++j) {
            int ks = ks0 + j;
            if (ks > g.KT - 1) ks = g.KT - 1;
            const bf16x8 v = ((const bf16x8 *)g.B)[(size_t)ks * 64 + lane];
            b[j] = (lane_on && j < nks) ? v : zero;
        }
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
        epilogue(g, L, ta, nt, tid, lane, wave, kThreads);
        __syncthreads();
    };

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // multiply chunk c (held in `a`) into the tile accumulator; at the end of a tile publish it to the slots
    auto mma_chunk = [&](const bf16x8 (&a)[CH][NPL], int c) {
        const int cc = c % nch, len = chunk_len(c);
#pragma unroll
        for (int q = 0; q < NCHMAX; ++q) {      // q == cc selects the B registers of this chunk statically
            if (q == cc) {
#pragma unroll
                for (int j = 0; j < CH; ++j)
                    if (j < len) {
#pragma unroll
                        for (int pl = 0; pl < NPL; ++pl) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[j][pl], b[q * CH + j], acc, 0, 0, 0);
                    }
            }
        }
        if (cc == nch - 1) {
            // columns n and n+8 hold the hi and lo partial products of token n
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[e] = add_lane_xor8(acc[e]);
            const int T = (c / nch) % kTilesPerRound;
            if (n < g.m) *(f32x4 *)(L.slots + ((size_t)T * kWaves + wave) * 128 + n * 16 + gq * 4) = acc;
            acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
    };
    if (nch == 0) {
        // no K slice (more wavefronts than k-steps): contribute zeros and keep the barriers aligned
        for (int t = t0; t < t1; ++t) {
            const int T = (t - t0) % kTilesPerRound;
            if (n < g.m) *(f32x4 *)(L.slots + ((size_t)T * kWaves + wave) * 128 + n * 16 + gq * 4) = acc;
            if (T == kTilesPerRound - 1 || t + 1 == t1) finish_round(t + 1);
        }
    } else {
        auto tile_done = [&](int c) {
            // a round ends when the tile that chunk c completes is the last of its round or of the workgroup
            if (c % nch == nch - 1) {
                const int t = t0 + c / nch;
                if ((t - t0) % kTilesPerRound == kTilesPerRound - 1 || t + 1 == t1) finish_round(t + 1);
            }
        };
        for (int c = 0; c < total; c += 2) {
            // chunks c and c+1 are in a0 and a1 (in flight or landed); refill each buffer as soon as it is consumed
            mma_chunk(a0, c);
            if (c + 2 < total) load_chunk<NPL, CH>(a0, chunk_ptr(c + 2), chunk_len(c + 2));
            tile_done(c);
            if (c + 1 < total) {
                mma_chunk(a1, c + 1);
                if (c + 3 < total) load_chunk<NPL, CH>(a1, chunk_ptr(c + 3), chunk_len(c + 3));
                tile_done(c + 1);
            }
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
        epilogue(g, L, ta, nt, tid, lane, wave, kThreads);
        __syncthreads();
    }
}

template <int NPL, int MODE>
__global__ void __launch_bounds__(MODE == GEMM_STATIONARY ? kStatThreads : kThreads) k_gemm(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    GemmLds &L = *reinterpret_cast<GemmLds *>(lds_raw);
    if constexpr (MODE == GEMM_STATIONARY)
        gemm_stationary<NPL, (NPL == 1 ? 8 : 2)>(g, blockIdx.x, gridDim.x, L);
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
    hipLaunchKernelGGL((k_gemm<NPL, MODE>), dim3(grid), dim3(MODE == GEMM_STATIONARY ? kStatThreads : kThreads), sizeof(GemmLds), s, g);
    return (int)hipGetLastError();
}

int launch_gemm(const GemmArgs &g, int planes, const LaunchCtx &c) {
    // equal numbers of row tiles per workgroup: with per = ceil(NT / n_wg) tiles each, ceil(NT / per) workgroups
    const int per = (g.NT + c.n_wg - 1) / c.n_wg;
    int grid = (g.NT + per - 1) / (per < 1 ? 1 : per);
    if (grid < 1) grid = 1;
    hipStream_t s = (hipStream_t)c.stream;
    int rc;
    if (g.mode == GEMM_STATIONARY) {
        if ((g.KT + kStatWaves - 1) / kStatWaves > kKsMax || g.K < 8) return (int)hipErrorInvalidValue;
        rc = planes == 1 ? launch_one<1, GEMM_STATIONARY>(g, grid, s) : launch_one<3, GEMM_STATIONARY>(g, grid, s);
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

int gemm_max_stationary_k(int) { return kKsMax * kStatWaves * 32; }

}  // namespace ad
