// Device side of the weight-streaming skinny GEMM   out[t][n] = sum_k W[n][k] * act[t][k]   for m <= 8 tokens,
// with the epilogues of the layer step and of the vocabulary pass fused in.  Included by the stand-alone GEMM
// kernel (ad_gemm.hip) and by the fused layer-step kernel (ad_layer_fused.hip).
//
// The contraction is bound by reading W once from HBM (about m flop per byte), so the code is organised
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
//    k-step) pairs of the workgroup are cut into contiguous ranges, one per wavefront, and B tiles are loaded
//    next to the A tiles from the packed block the previous step wrote (L2 hits).
// Partial accumulators meet in LDS and are summed in wavefront order (fixed order: reproducible).
//
// Each mode is split into a *stream* object, which can put the first weight batches in flight before anything
// that depends on the activations exists (the fused kernel does so before a grid barrier), and the function
// that consumes it.  The `Io` policy says how data exchanged between workgroups is read and written: plain
// loads and stores when a kernel boundary orders producer and consumer, agent-scope atomics when both run
// inside one kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_device.h"
#include "ad_internal.h"

namespace ad {

constexpr int kTilesPerRound = 8;       // row tiles reduced together
constexpr int kStatWaves = 8;           // stationary mode: wavefronts per workgroup (512 threads, up to 256 registers each)
constexpr int kStatThreads = kStatWaves * 64;
constexpr int kKsMax = 20;              // stationary mode, fp32 weights and the fused layer kernel: most k-steps per
                                        // wavefront (K <= 8 * 20 * 32 = 5120)
constexpr int kKsMaxWide = 32;          // stationary mode, 16-bit weights: K <= 8 * 32 * 32 = 8192

struct GemmLds {
    // stationary: [tile 0..8)[wave][token 0..8)[row 0..16)      streamed: [slot][col 0..16)[row 0..16)
    float slots[kTilesPerRound * kWaves * 8 * 16];
    float red[kTilesPerRound * 128];    // [tile][token][row]
    float ssq_part[kWaves * 8];
    float scale[8];
    float run_max[8], run_sum[8];
    int run_idx[8];
};

// ---- how data shared between workgroups is accessed ------------------------------------------------------
struct IoPlain {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ f32x2 ld2(const float *p) { return *(const f32x2 *)p; }
    static __device__ __forceinline__ f32x4 ld4(const float *p) { return *(const f32x4 *)p; }
    static __device__ __forceinline__ bf16x8 ldb(const bf16x8 *p) { return *p; }
    static __device__ __forceinline__ void st(float *p, float v) { *p = v; }
    static __device__ __forceinline__ void st2(float *p, f32x2 v) { *(f32x2 *)p = v; }
    static __device__ __forceinline__ void st16(uint16_t *p, uint16_t v) { *p = v; }
};
// Relaxed agent-scope atomics: stores go through to memory and loads do not use a stale copy in another
// XCD's L2, so a grid barrier built from the same kind of atomics is enough to order them (the storing
// wavefront waits for its stores to complete before it arrives at the barrier).
struct IoAgent {
    static __device__ __forceinline__ float ld(const float *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    static __device__ __forceinline__ f32x2 ld2(const float *p) {
        union { uint64_t u; f32x2 v; } c;
        c.u = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c.v;
    }
    static __device__ __forceinline__ f32x4 ld4(const float *p) {
        union { uint64_t u[2]; f32x4 v; } c;
        c.u[0] = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        c.u[1] = __hip_atomic_load((const uint64_t *)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c.v;
    }
    static __device__ __forceinline__ bf16x8 ldb(const bf16x8 *p) {
        union { uint64_t u[2]; bf16x8 v; } c;
        c.u[0] = __hip_atomic_load((const uint64_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        c.u[1] = __hip_atomic_load((const uint64_t *)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return c.v;
    }
    static __device__ __forceinline__ void st(float *p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
    static __device__ __forceinline__ void st2(float *p, f32x2 v) {
        union { uint64_t u; f32x2 v; } c;
        c.v = v;
        __hip_atomic_store((uint64_t *)p, c.u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    static __device__ __forceinline__ void st16(uint16_t *p, uint16_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
};

// Stores as IoAgent; loads are ordinary (served by this XCD's L2, shared by its workgroups).  For data that
// every workgroup reads: the consumer must have invalidated its caches (an agent-scope acquire fence) after the
// grid barrier that follows the producer's stores.
struct IoAcquired : IoAgent {
    static __device__ __forceinline__ float ld(const float *p) { return *p; }
    static __device__ __forceinline__ f32x2 ld2(const float *p) { return *(const f32x2 *)p; }
    static __device__ __forceinline__ f32x4 ld4(const float *p) { return *(const f32x4 *)p; }
    static __device__ __forceinline__ bf16x8 ldb(const bf16x8 *p) { return *p; }
};

template <class Io, bool F16>
__device__ __forceinline__ void store_act_io(uint16_t *B, int KT, int k, int t, float v) {
    uint16_t hi, lo;
    split_hi_lo<F16>(v, hi, lo);
    Io::st16(B + act_index(k, t, KT), hi);
    Io::st16(B + act_index(k, 8 + t, KT), lo);
}

struct NoTail {
    __device__ __forceinline__ void operator()() const {}
};

__device__ __forceinline__ int part_start(int tot, int w, int nw) { return (int)(((long)tot * w) / nw); }

// merge (max, sumexp, argmax) pairs; the lower index wins ties
__device__ __forceinline__ void lse_merge(float &M, float &S, int &I, float m2, float s2, int i2) {
    if (m2 > M || (m2 == M && i2 < I)) I = i2;
    const float nm = fmaxf(M, m2);
    if (nm == -INFINITY) { M = nm; S = 0.f; return; }
    S = S * __expf(M - nm) + s2 * __expf(m2 - nm);
    M = nm;
}

// ---- epilogue on a reduced round: L.red[T*128 + t*16 + i] holds row (ta+T)*16+i of token t -------------
// EPI: the epilogue kind when it is known at compile time, or -1 to take g.epi.
template <class Io, int EPI, bool F16>
__device__ __forceinline__ void epilogue(const GemmArgs &g, GemmLds &L, int ta, int nt, int tid, int lane, int wave, int nthreads) {
    const int epi = EPI >= 0 ? EPI : g.epi;
    if (epi == EPI_STORE) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) Io::st(g.out + (size_t)t * g.ld + n, L.scale[t] * L.red[idx]);
        }
    } else if (epi == EPI_RESID) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) Io::st(g.out + (size_t)t * g.ld + n, Io::ld(g.resid + (size_t)t * g.ld + n) + L.scale[t] * L.red[idx]);
        }
    } else if (epi == EPI_SWIGLU) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, f = (ta + T) * 8 + i;
            if (t < g.m && i < 8 && f * 2 < g.N) {
                const float gate = L.scale[t] * L.red[idx], up = L.scale[t] * L.red[idx + 8];
                store_act_io<Io, F16>((uint16_t *)g.Bnext, g.Bnext_KT, f, t, gate / (1.0f + __expf(-gate)) * up);
            }
        }
    } else if (epi == EPI_PACK) {
        for (int idx = tid; idx < nt * 128; idx += nthreads) {
            const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
            if (t < g.m && n < g.N) store_act_io<Io, F16>((uint16_t *)g.Bnext, g.Bnext_KT, n, t, L.scale[t] * L.red[idx]);
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
// Weights are addressed as a uniform base pointer plus a 32-bit byte offset (a configuration with a packed
// matrix of 4 GiB or more is refused when the model is created), which costs one address register per load instead of two.  `unit` counts 16 bytes.
__device__ __forceinline__ bf16x8 load_tile(const bf16x8 *W, unsigned unit) {
    return __builtin_nontemporal_load((const bf16x8 *)((const char *)W + (unit << 4)));
}

template <int NPL, int CH>
__device__ __forceinline__ void load_chunk(bf16x8 (&a)[CH][NPL], const bf16x8 *W, unsigned p, int n) {
    if (n == CH) {   // the common case: straight-line loads
#pragma unroll
        for (int j = 0; j < CH; ++j)
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = load_tile(W, p + (unsigned)(j * NPL + q) * 64u);
    } else {
        // a short chunk: entries past the end repeat its last k-step (same cache lines; their products are skipped),
        // so that the buffer is still filled by straight-line loads into fixed registers
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int jj = j < n ? j : n - 1;
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = load_tile(W, p + (unsigned)(jj * NPL + q) * 64u);
        }
    }
}

// This wavefront's share of workgroup wg's weights (row tiles [t0, t1), k-steps [ks0, ks0 + nks)) and its two
// chunk buffers.
template <int NPL, int CH>
struct StatStream {
    bf16x8 a0[CH][NPL], a1[CH][NPL];
    const bf16x8 *W;
    unsigned wbase, tstride;       // 16-byte units
    int t0, t1, ks0, nks, nch, total;

    __device__ __forceinline__ void init(const GemmArgs &g, int wg, int nwg, long long w_off = 0) {
        const int tid_ = thread_index(), lane = tid_ & 63, wave = tid_ >> 6;
        t0 = wg * g.tq + (wg < g.tr ? wg : g.tr);
        t1 = t0 + g.tq + (wg < g.tr ? 1 : 0);
        if (wg >= nwg) t0 = t1 = 0;                // not one of this GEMM's workgroups
        ks0 = part_start(g.KT, wave, kStatWaves);
        nks = part_start(g.KT, wave + 1, kStatWaves) - ks0;
        nch = (nks + CH - 1) / CH;                 // chunks per tile (0 if this wavefront has no K slice)
        total = (t1 - t0) * nch;                   // chunks in this wavefront's stream
        W = (const bf16x8 *)((const char *)g.W + w_off);
        wbase = (unsigned)(((size_t)t0 * g.KT + ks0) * NPL * 64 + lane);
        tstride = (unsigned)g.KT * NPL * 64u;
    }
    __device__ __forceinline__ unsigned chunk_ptr(int c) const { return wbase + (unsigned)(c / nch) * tstride + (unsigned)(c % nch) * (CH * NPL * 64u); }
    __device__ __forceinline__ int chunk_len(int c) const { const int r = nks - (c % nch) * CH; return r < CH ? r : CH; }
    // The first two weight chunks go in flight.  The loads are unconditional (a wavefront with fewer chunks reads
    // the start of the matrix instead, and nothing is done with it): code after this call then knows how many loads
    // are outstanding, and can wait for an earlier load without waiting for these.
    __device__ __forceinline__ void prefetch() {
        // the address arithmetic of these loads stays here (behind an opaque copy of the base offset) instead of
        // being hoisted to where the caller's own stream needs the registers
        asm volatile("" : "+v"(wbase));
        const unsigned lane = (unsigned)thread_index() & 63;
        const unsigned p0 = total > 0 ? chunk_ptr(0) : lane, p1 = total > 1 ? chunk_ptr(1) : lane;
        const int n0 = total > 0 ? chunk_len(0) : 1, n1 = total > 1 ? chunk_len(1) : 1;
        load_chunk_clamped(a0, p0, n0);
        load_chunk_clamped(a1, p1, n1);
    }
    __device__ __forceinline__ void load_chunk_clamped(bf16x8 (&a)[CH][NPL], unsigned p, int n) {
#pragma unroll
        for (int j = 0; j < CH; ++j) {
            const int jj = j < n ? j : n - 1;
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = load_tile(W, p + (unsigned)(jj * NPL + q) * 64u);
        }
    }
};

// `tail` runs once, after the workgroup's last MFMA and before its last reduction and epilogue.
// PREFETCHED: S.prefetch() has been called already (a phase whose weights went in flight while the workgroup
// waited for its inputs).  Otherwise the function calls it itself, right after it has issued the loads of its
// activations: a wavefront's loads return in order, so activations requested behind 16 KiB of weights would arrive
// after them, and the B operand, without which no weight can be consumed, would be late by the whole prefetch.
// All loads of the prologue are unconditional (rows, k-steps and tiles past the end are clamped to the last valid
// one, which costs no extra cache lines, and masked afterwards), so that their number is known at compile time and
// the waits for the activations do not also wait for the weights behind them.
// NCHMAX: most chunks per tile and wavefront this instance covers (the B slice takes NCHMAX * CH registers x 4).
// F16: the weights and the 16-bit halves of the activations are fp16 (else bf16).
template <int NPL, int CH, int NCHMAX, class Io, int EPI, bool F16, bool PREFETCHED, class Tail>
__device__ __forceinline__ void gemm_stationary(const GemmArgs &g, StatStream<NPL, CH> &S, GemmLds &L, Tail tail, long long w_off = 0) {
    constexpr int KSB = NCHMAX * CH;   // B registers cover whole chunks
    constexpr int kWaves = kStatWaves, kThreads = kStatThreads;         // this mode's workgroup shape
    const int tid = thread_index(), lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4, t_lane = n & 7;
    const int t0 = S.t0, t1 = S.t1, ks0 = S.ks0, nks = S.nks, nch = S.nch, total = S.total;
    const int epi = EPI >= 0 ? EPI : g.epi;
    if (epi == EPI_HEAD && tid < 8) {
        L.run_max[tid] = -INFINITY;
        L.run_sum[tid] = 0.f;
        L.run_idx[tid] = 0x7fffffff;
    }
    bf16x8 b[KSB];

    // B slice of this wavefront.  Its K slice is read in passes of 8 k-steps = 256 inputs: lane l takes inputs
    // 4l .. 4l+3 of every token (one coalesced 128-bit load per token and pass), multiplies
    // by the norm weights, splits into bf16 hi/lo and writes them, in B-operand order, into a wavefront-private
    // strip of LDS from which each lane then reads its operand registers.  The strip aliases the reduction slots,
    // which are not in use yet.
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const bool lane_on = t_lane < g.m;
    constexpr int NPASS = (KSB + 7) / 8;
    // 16-byte units of the strip are permuted (unit u -> u ^ ((u >> 4) & 15)) so that the 8-byte writes of a
    // wavefront, which all go to the same operand column, spread over the LDS banks
    uint16_t *strip16 = reinterpret_cast<uint16_t *>(L.slots) + (size_t)wave * 8 * 512;
    const bf16x8 *strip = reinterpret_cast<const bf16x8 *>(strip16);
    auto sw = [](int u) { return u ^ ((u >> 4) & 15); };
    if (g.x) {
        // two passes' worth of loads are in flight: those of pass p + 1 are issued before pass p is converted
        f32x4 xr[2][8];
        u32x4 wraw[2];
        const bool w16 = g.norm_elem != ELEM_F32;
        const char *wsrc = g.norm_w ? (const char *)g.norm_w + w_off : (const char *)g.x;     // without a norm vector: any valid address
        auto load_pass = [&](f32x4 (&xp)[8], u32x4 &wp, int p) {
            const int k = (ks0 + p * 8) * 32 + lane * 4;
            const int kc = (k > g.K - 4) ? g.K - 4 : k;              // clamped address, masked result
            // the lane's four norm weights: 16-bit kinds load the aligned group of eight that holds them
            wp = *(const u32x4 *)(wsrc + (w16 ? (size_t)(kc & ~7) * 2 : (size_t)kc * 4));
#pragma unroll
            for (int t = 0; t < 8; ++t) xp[t] = Io::ld4(g.x + (size_t)(t < g.m ? t : g.m - 1) * g.ldx + kc);
        };
        auto norm4 = [&](const u32x4 &raw, int p) -> f32x4 {
            if (!g.norm_w) return (f32x4){1.f, 1.f, 1.f, 1.f};
            if (g.norm_elem == ELEM_F32) return (f32x4){__uint_as_float(raw[0]), __uint_as_float(raw[1]), __uint_as_float(raw[2]), __uint_as_float(raw[3])};
            const int k = (ks0 + p * 8) * 32 + lane * 4;
            const int kc = (k > g.K - 4) ? g.K - 4 : k;
            const unsigned lo = (kc & 4) ? raw[2] : raw[0], hi = (kc & 4) ? raw[3] : raw[1];
            if (g.norm_elem == ELEM_BF16)
                return (f32x4){__uint_as_float(lo << 16), __uint_as_float(lo & 0xffff0000u), __uint_as_float(hi << 16), __uint_as_float(hi & 0xffff0000u)};
            return (f32x4){f16_bits_to_f32((uint16_t)(lo & 0xffffu)), f16_bits_to_f32((uint16_t)(lo >> 16)),
                           f16_bits_to_f32((uint16_t)(hi & 0xffffu)), f16_bits_to_f32((uint16_t)(hi >> 16))};
        };
        load_pass(xr[0], wraw[0], 0);
        if (NPASS > 1) load_pass(xr[1], wraw[1], 1);
        if (!PREFETCHED) S.prefetch();
        float ssq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            if (p > 0 && p + 1 < NPASS) load_pass(xr[(p + 1) & 1], wraw[(p + 1) & 1], p + 1);
            const f32x4 (&xp)[8] = xr[p & 1];
            const f32x4 wp = norm4(wraw[p & 1], p);
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
                            const float xv = k_on ? xp[t][e] : 0.f;
                            ssq[t] += xv * xv;
                            split_hi_lo<F16>(xv * wp[e], hi.u[e], lo.u[e]);
                        }
                        *(uint64_t *)(strip16 + sw(u0 + t) * 8 + (lane & 1) * 4) = hi.v;
                        *(uint64_t *)(strip16 + sw(u0 + 8 + t) * 8 + (lane & 1) * 4) = lo.v;
                    }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    if (p * 8 + jj < KSB) b[p * 8 + jj] = (lane_on && jj < jn) ? strip[sw(jj * 64 + lane)] : zero;
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
            } else {
#pragma unroll
                for (int jj = 0; jj < 8; ++jj)
                    if (p * 8 + jj < KSB) b[p * 8 + jj] = zero;
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
        // B was packed by an earlier epilogue.  The lanes of tokens past the call's load token 0's unit (the same cache
        // lines) and k-steps past the slice repeat its last one; both are zeroed below.
        const int src_lane = lane_on ? lane : (lane & ~7);
        const int ks_last = nks > 0 ? ks0 + nks - 1 : (ks0 < g.KT ? ks0 : g.KT - 1);
#pragma unroll
        for (int j = 0; j < KSB; ++j) b[j] = Io::ldb((const bf16x8 *)g.B + act_operand_index(j < nks ? ks0 + j : ks_last, src_lane, g.KT));
        // the producer left per-tile sums of squares: wavefront t adds up token t's, in tile order per lane and
        // then across the lanes (fixed order).  The first 512 tiles' loads are issued before the weights'.
        const int t = wave;
        float sq[8];
        const float *sq_src = g.ssq_in ? g.ssq_in : (const float *)g.B;      // without partial sums: any valid address
        const int sq_last = g.ssq_in ? g.ssq_tiles - 1 : 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int tile = lane + 64 * i;
            sq[i] = Io::ld(sq_src + (size_t)(tile < sq_last ? tile : sq_last) * 8 + t);
        }
        if (!PREFETCHED) S.prefetch();
#pragma unroll
        for (int j = 0; j < KSB; ++j)
            if (!(lane_on && j < nks)) b[j] = zero;
        if (g.ssq_in) {
            float v = 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i)
                if (t < g.m && lane + 64 * i < g.ssq_tiles) v += sq[i];
            if (t < g.m)
                for (int i = lane + 512; i < g.ssq_tiles; i += 64) v += Io::ld(g.ssq_in + (size_t)i * 8 + t);
            for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
            if (lane == 0) L.ssq_part[t] = v;
        }
    }
    // The per-token factor 1 / rms is only needed by the epilogue: it is formed from the wavefronts' partial sums at the
    // first reduction (after that reduction's barrier, which also orders the partial sums), not here on the way to the
    // first product.  Only a B operand built through the strips needs a barrier now: the strips alias the slots.
    if (g.x) __syncthreads();
    bool scale_set = false;

    auto finish_round = [&](int done) {
        // tiles [ta, done) of this round are in the slots: sum them over the wavefronts, then the epilogue
        const int ta = t0 + ((done - t0 - 1) / kTilesPerRound) * kTilesPerRound, nt = done - ta;
        __syncthreads();
        if (!scale_set) {
            scale_set = true;
            if (tid < 8) {
                float s = 1.0f;
                if (g.x && g.norm_w) {
                    s = 0.f;
                    for (int w = 0; w < kWaves; ++w) s += L.ssq_part[w * 8 + tid];
                    s = 1.0f / sqrtf(s * g.inv_dim + g.eps);
                } else if (!g.x && g.ssq_in) {
                    s = 1.0f / sqrtf(L.ssq_part[tid] * g.inv_dim + g.eps);
                }
                L.scale[tid] = s;
            }
        }
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
        epilogue<Io, EPI, F16>(g, L, ta, nt, tid, lane, wave, kThreads);
        __syncthreads();
    };

    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    // multiply chunk c (held in `a`) into the tile accumulator; at the end of a tile publish it to the slots
    auto mma_chunk = [&](const bf16x8 (&a)[CH][NPL], int c) {
        const int cc = c % nch, len = S.chunk_len(c);
#pragma unroll
        for (int q = 0; q < NCHMAX; ++q) {      // q == cc selects the B registers of this chunk statically
            if (q == cc) {
#pragma unroll
                for (int j = 0; j < CH; ++j)
                    if (j < len) {
#pragma unroll
                        for (int pl = 0; pl < NPL; ++pl) acc = mma16<F16>(a[j][pl], b[q * CH + j], acc);
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
            if (T == kTilesPerRound - 1 && t + 1 < t1) finish_round(t + 1);
        }
    } else {
        auto tile_done = [&](int c) {
            // a round ends when the tile that chunk c completes is the last of its round (the workgroup's last
            // round is finished after the loop)
            if (c % nch == nch - 1) {
                const int t = t0 + c / nch;
                if ((t - t0) % kTilesPerRound == kTilesPerRound - 1 && t + 1 < t1) finish_round(t + 1);
            }
        };
        // chunks c and c+1 are in a0 and a1 (in flight or landed); each buffer is refilled as soon as it is consumed.
        // While four chunks remain the refills are unconditional, so that the number of loads behind a chunk is
        // known where it is multiplied and only its own loads are waited for (with a refill under a condition the
        // wait has to allow for its absence, and then also covers the refill just issued: one chunk in flight, not two).
        int c = 0;
#pragma nounroll
        for (; c + 4 <= total; c += 2) {
            mma_chunk(S.a0, c);
            load_chunk<NPL, CH>(S.a0, S.W, S.chunk_ptr(c + 2), S.chunk_len(c + 2));
            tile_done(c);
            mma_chunk(S.a1, c + 1);
            load_chunk<NPL, CH>(S.a1, S.W, S.chunk_ptr(c + 3), S.chunk_len(c + 3));
            tile_done(c + 1);
        }
#pragma nounroll
        for (; c < total; c += 2) {
            mma_chunk(S.a0, c);
            if (c + 2 < total) load_chunk<NPL, CH>(S.a0, S.W, S.chunk_ptr(c + 2), S.chunk_len(c + 2));
            tile_done(c);
            if (c + 1 < total) {
                mma_chunk(S.a1, c + 1);
                if (c + 3 < total) load_chunk<NPL, CH>(S.a1, S.W, S.chunk_ptr(c + 3), S.chunk_len(c + 3));
                tile_done(c + 1);
            }
        }
    }
    // the weight stream has ended: the tail runs here, with the chunk buffers and the B slice dead
    __builtin_amdgcn_sched_barrier(0);      // keep the tail's loads out of the stream's register live ranges
    tail();
    __builtin_amdgcn_sched_barrier(0);
    if (t1 > t0) finish_round(t1);
    if (epi == EPI_HEAD && tid < g.m) {
        float *p = g.head_part + ((size_t)blockIdx.x * 8 + tid) * 4;
        p[0] = L.run_max[tid];
        p[1] = L.run_sum[tid];
        p[2] = __int_as_float(L.run_idx[tid]);
    }
}

// ---- streamed mode -----------------------------------------------------------------------------------------
// NW wavefronts; the workgroup's tiles are taken in rounds of up to 8, and inside a round wavefront w streams
// the contiguous range [xa, xb) of the round's (tile, k-step) pairs, U pairs per batch, two batches in flight.
template <int NPL, int U, int NW>
struct StreamStream {
    bf16x8 a0[U][NPL], a1[U][NPL];
    int t0, t1;
    bool primed;

    __device__ __forceinline__ void init(const GemmArgs &g, int wg, int nwg) {
        t0 = wg * g.tq + (wg < g.tr ? wg : g.tr);
        t1 = t0 + g.tq + (wg < g.tr ? 1 : 0);
        if (wg >= nwg) t0 = t1 = 0;                // not one of this GEMM's workgroups
        primed = false;
    }
    // Batch [x, x + U) of (tile, k-step) pairs of a round whose first pair sits at unit offset `base`: entries past
    // `x_ok` (the wavefront's last pair, or any valid pair of the round if it has none) repeat that pair -- the same
    // cache lines, products skipped -- so that every call issues exactly U * NPL loads into fixed registers and the
    // code around it can wait for an earlier batch without waiting for this one.
    static __device__ __forceinline__ void load_a(bf16x8 (&a)[U][NPL], const bf16x8 *W, unsigned base, int x, int x_ok) {
#pragma unroll
        for (int j = 0; j < U; ++j) {
            const int xx = x + j < x_ok ? x + j : x_ok;
#pragma unroll
            for (int q = 0; q < NPL; ++q) a[j][q] = load_tile(W, base + (unsigned)(xx * NPL + q) * 64u);
        }
    }
    static __device__ __forceinline__ int valid_pair(int xa, int xb, int tot) { return xb > xa ? xb - 1 : (xa < tot ? xa : tot - 1); }
    // the A tiles of the first two batches of the first round go in flight
    __device__ __forceinline__ void prefetch(const GemmArgs &g, long long w_off = 0) {
        const int tid_ = thread_index(), lane = tid_ & 63, wave = tid_ >> 6;
        if (t0 < t1) {
            const int tb = (t1 < t0 + 8) ? t1 : t0 + 8, tot = (tb - t0) * g.KT;
            const int xa = part_start(tot, wave, NW), xb = part_start(tot, wave + 1, NW);
            unsigned base = (unsigned)((size_t)t0 * g.KT * NPL * 64 + lane);
            asm volatile("" : "+v"(base));     // keep the address arithmetic of these loads here (see StatStream)
            const int x_ok = valid_pair(xa, xb, tot);
            const bf16x8 *W = (const bf16x8 *)((const char *)g.W + w_off);
            load_a(a0, W, base, xa, x_ok);
            load_a(a1, W, base, xa + U, x_ok);
        }
        primed = true;
    }
};

// ONE_ROUND: the caller guarantees at most 8 row tiles per workgroup (then there is no loop over rounds, and the
// tail runs with the stream's buffers dead).
template <int NPL, int U, int NW, class Io, int EPI, bool ONE_ROUND, bool F16, class Tail>
__device__ __forceinline__ void gemm_streamed(const GemmArgs &g, StreamStream<NPL, U, NW> &S, GemmLds &L, Tail tail, long long w_off = 0) {
    constexpr int NTHREADS = NW * 64;
    constexpr int RP = (kTilesPerRound * 128 + NTHREADS - 1) / NTHREADS;   // residual entries per thread and round
    const int tid = thread_index(), lane = tid & 63, wave = tid >> 6;
    const int t0 = S.t0, t1 = S.t1;
    const int epi = EPI >= 0 ? EPI : g.epi;
    if (tid < 8) L.scale[tid] = 1.0f;
    const bool bact = (lane & 7) < g.m;
    const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
    const bf16x8 *B = (const bf16x8 *)g.B;
    const int KT = g.KT;
    for (int ta = t0; ta < t1; ta += (ONE_ROUND ? (1 << 30) : 8)) {
        const int tb = (t1 < ta + 8) ? t1 : ta + 8, nt = tb - ta;
        const int tot = nt * KT;
        const int xa = part_start(tot, wave, NW), xb = part_start(tot, wave + 1, NW);
        int tile = xa / KT, ks = xa % KT;
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        const bf16x8 *W = (const bf16x8 *)((const char *)g.W + w_off);
        const unsigned base = (unsigned)((size_t)ta * KT * NPL * 64 + lane);
        const int x_ok = StreamStream<NPL, U, NW>::valid_pair(xa, xb, tot);
        bf16x8 b0[U], b1[U];
        // the B operands of batch [x, x + U), whose first pair is k-step ks_at of its tile: every call issues exactly U
        // loads (entries past the range read unit 0 of the block and are never multiplied; lanes of tokens past the
        // call's read token 0's unit and are zeroed where the operand is used -- not here, where overwriting the
        // register would have to wait for the load)
        const int src_lane = bact ? lane : (lane & ~7);
        auto load_b = [&](bf16x8 (&b)[U], int x, int ks_at) {
#pragma unroll
            for (int j = 0; j < U; ++j) {
                int kk = ks_at + j;
                if (KT >= U) kk -= (kk >= KT) ? KT : 0;
                else kk %= KT;
                const bool on = x + j < xb;
                b[j] = Io::ldb(B + (on ? act_operand_index(kk, src_lane, KT) : 0));
            }
        };
        auto mma = [&](const bf16x8 (&a)[U][NPL], const bf16x8 (&b)[U], int x) {
#pragma unroll
            for (int j = 0; j < U; ++j)
                if (x + j < xb) {
                    const bf16x8 bb = bact ? b[j] : zero;
#pragma unroll
                    for (int q = 0; q < NPL; ++q) acc = mma16<F16>(a[j][q], bb, acc);
                    if (++ks == KT) {
                        *(f32x4 *)(L.slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
                        acc = (f32x4){0.f, 0.f, 0.f, 0.f};
                        ks = 0;
                        ++tile;
                    }
                }
        };
        // residual values of this thread's output entries (and the next GEMM's norm weights for them), ahead of the stream
        float rpre[RP], npre[RP];
        if (epi == EPI_RESID) {
#pragma unroll
            for (int j = 0; j < RP; ++j) {
                const int idx = tid + j * NTHREADS, T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                const bool on = idx < nt * 128 && t < g.m && n < g.N;
                rpre[j] = on ? Io::ld(g.resid + (size_t)t * g.ld + n) : 0.f;
                npre[j] = (on && g.Bnext) ? load_w((const char *)g.next_norm_w + w_off, g.next_norm_elem, (size_t)n) : 0.f;
            }
        }
        // Two batches are in flight while a third is multiplied: a0/b0 hold batch x, a1/b1 batch x + U.  While four
        // whole batches remain, every load of the loop is in range and unconditional, so each multiplication waits for
        // its own operands only; the last batches take their loads under conditions (no duplicate traffic at the end).
        const bool primed = S.primed && ta == t0;     // the A tiles of batches 0 and 1 are in flight already
        auto wrap = [&](int k) { if (KT >= U) return k - (k >= KT ? KT : 0); return k % KT; };
        int ks_b = ks;                                  // k-step of the first pair of the batch whose B operands load next
        if (!primed) {
            S.load_a(S.a0, W, base, xa, x_ok);
            S.load_a(S.a1, W, base, xa + U, x_ok);
        }
        load_b(b0, xa, ks_b);
        ks_b = wrap(ks_b + U);
        load_b(b1, xa + U, ks_b);
        ks_b = wrap(ks_b + U);
        int x = xa;
#pragma nounroll
        for (; x + 4 * U <= xb; x += 2 * U) {
            mma(S.a0, b0, x);
            S.load_a(S.a0, W, base, x + 2 * U, x_ok);
            load_b(b0, x + 2 * U, ks_b);
            ks_b = wrap(ks_b + U);
            mma(S.a1, b1, x + U);
            S.load_a(S.a1, W, base, x + 3 * U, x_ok);
            load_b(b1, x + 3 * U, ks_b);
            ks_b = wrap(ks_b + U);
        }
#pragma nounroll
        for (; x < xb; x += 2 * U) {
            mma(S.a0, b0, x);
            if (x + 2 * U < xb) {
                S.load_a(S.a0, W, base, x + 2 * U, x_ok);
                load_b(b0, x + 2 * U, ks_b);
                ks_b = wrap(ks_b + U);
            }
            mma(S.a1, b1, x + U);
            if (x + 3 * U < xb) {
                S.load_a(S.a1, W, base, x + 3 * U, x_ok);
                load_b(b1, x + 3 * U, ks_b);
                ks_b = wrap(ks_b + U);
            }
        }
        if (ks != 0) *(f32x4 *)(L.slots + (wave + tile) * 256 + (lane & 15) * 16 + (lane >> 4) * 4) = acc;
        __builtin_amdgcn_sched_barrier(0);  // keep the tail's loads out of the stream's register live ranges
        if (tb == t1) tail();
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
        // The sum of a tile's slots, in wavefront order: wavefronts w0 .. w1 hold pairs of tile T (pairs [T * KT, T * KT + KT)
        // of the round; wavefront w holds pairs [tot * w / NW, tot * (w + 1) / NW)), those without pairs are skipped.
        auto tile_sum = [&](int T, int t, int i) {
            const int x0 = T * KT, x1 = x0 + KT - 1;
            int w0 = 0, w1 = NW - 1;
            while (w0 + 1 < NW && part_start(tot, w0 + 1, NW) <= x0) ++w0;
            while (w1 > 0 && part_start(tot, w1, NW) > x1) --w1;
            float v = 0.f;
            for (int w = w0; w <= w1; ++w) {
                if (part_start(tot, w, NW) == part_start(tot, w + 1, NW)) continue;   // wavefront had no work
                const float *s = L.slots + (w + T) * 256;
                v += s[t * 16 + i] + s[(t + 8) * 16 + i];
            }
            return v;
        };
        if (epi == EPI_RESID) {
            // each thread sums its own output entries and finishes them
#pragma unroll
            for (int j = 0; j < RP; ++j) {
                const int idx = tid + j * NTHREADS, T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15, n = (ta + T) * 16 + i;
                const bool on = idx < nt * 128 && t < g.m && n < g.N;
                const float y = on ? rpre[j] + tile_sum(T, t, i) : 0.f;
                if (on) Io::st(g.out + (size_t)t * g.ld + n, y);
                if (g.Bnext) {
                    // input of the next GEMM: y * norm weight, packed; and this tile's share of sum(y^2) per token
                    // (the 16 outputs of a (tile, token) pair sit in 16 neighbouring lanes)
                    if (on) store_act_io<Io, F16>((uint16_t *)g.Bnext, g.Bnext_KT, n, t, y * npre[j]);
                    float q = y * y;
                    q += __shfl_xor(q, 8);
                    q += __shfl_xor(q, 4);
                    q += __shfl_xor(q, 2);
                    q += __shfl_xor(q, 1);
                    if (i == 0 && idx < nt * 128 && t < g.m) Io::st(g.ssq_out + (size_t)(ta + T) * 8 + t, q);
                }
            }
        } else {
            for (int idx = tid; idx < nt * 128; idx += NTHREADS) {
                const int T = idx >> 7, t = (idx >> 4) & 7, i = idx & 15;
                L.red[idx] = t < g.m ? tile_sum(T, t, i) : 0.f;
            }
            __syncthreads();
            epilogue<Io, EPI, F16>(g, L, ta, nt, tid, lane, wave, NTHREADS);
        }
        __syncthreads();
        if (ONE_ROUND) break;     // (said here as well, so that the body is not compiled as a loop)
    }
    if (t1 == t0) tail();
}

}  // namespace ad
