// Device side of the attention phase for a bf16 KV cache: work items of the split-context MFMA attention and
// the fold of the splits.  Included by the stand-alone attention kernels (ad_attention.hip) and by the fused
// layer-step kernel (ad_layer_fused.hip); the `Io` policy (ad_gemm_device.h) says how data exchanged between
// workgroups -- q/k/v rows in, partials out and in, packed output -- is accessed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_device.h"
#include "ad_gemm_device.h"
#include "ad_internal.h"

namespace ad {

// ---------------------------------------------------------------------------------------------------
// bf16 cache: MFMA kernel.  4 wavefronts per item, each takes one block of 32 cached positions.
// ---------------------------------------------------------------------------------------------------
// Scores  S^T[key][row] = K[key][:] . q[row][:]  : A operand = K rows straight from the cache (lane (i, gq)
// holds 8 consecutive dims of one key), B operand = the rotated, pre-scaled queries split into bf16 hi/lo
// columns (rows of a block of 8 query rows in columns 0..7, their lo parts in columns 8..15).  The 16 rows
// of the two score tiles are assigned to keys so that lane group gq ends up with 8 consecutive keys of
// its column, which is exactly the B operand layout of the second product
//   O^T[dim][row] = V^T[dim][key] . P^T[key][row]
// whose A operand is a 128-bit load from the transposed V cache.  P is split hi/lo over the column pair
// as well, so both products carry about 16 mantissa bits of the activations.
constexpr int kAttnWaves = 4;            // key blocks of an item that are processed at once
constexpr int kAttnRowsPerPass = 32;
constexpr int kAttnSlots = 5;   // 4 cached blocks + the call's own rows

// RP: query rows per pass (a multiple of 8; more rows take more passes)
template <int DH, int RP = kAttnRowsPerPass>
struct AttnMfmaLds {
    bf16x8 qb[(RP / 8) * (DH / 32) * 64];                // [row block][k-step][lane]
    uint16_t knew[8 * DH];                               // the call's own K rows, cache type: [row][dim]
    uint16_t vnewT[DH * 8];                              // the call's own V rows, transposed: [dim][row]
    float part[kAttnSlots * RP * (DH + 4)];              // rows padded to 16 bytes for 128-bit LDS stores
};

// Work items wg, wg + nwg, ... of the attention phase.  NTHREADS is 256 (4 wavefronts: wavefront w takes key
// block w and all row blocks) or 512 (8 wavefronts: wavefronts w and w + 4 both take key block w and share its
// row blocks of 8 query rows between them).
// The wavefront's cached block of an item: K rows and V columns as MFMA A operands.
template <int DH>
struct AttnKv {
    bf16x8 k[2][DH / 32], v[DH / 16];
};

// Loads wavefront (tid >> 6) & 3's block of 32 cached positions of work item `item` (nothing if the block is
// empty or the wavefront has no query rows).  Does not depend on the queries, so it can be issued early.
template <int DH, int NTHREADS>
__device__ __forceinline__ void attn_load_kv(const AttnArgs &a, int item, AttnKv<DH> &kv, long long kv_off = 0) {
    constexpr int KS = DH / 32, DT = DH / 16;
    const int tid = thread_index(), lane = tid & 63, wave = (tid >> 6) & 3, rh = tid >> 8;
    const int n = lane & 15, gq = lane >> 4;
    if (item >= a.Hkv * a.S) return;
    const int g = div_small(item, a.mul_S), s = item - g * a.S;
    const int c0 = s * a.C, c1 = (c0 + a.C < a.pos0) ? c0 + a.C : a.pos0;
    const int nbc = (c1 > c0) ? (c1 - c0 + 31) / 32 : 0;
    const int R = a.R;
    if (wave >= nbc || R <= rh * 8) return;
    const uint16_t *Kg = (const uint16_t *)((const char *)a.Kc + kv_off) + (size_t)g * a.stride * DH;
    const uint16_t *Vg = (const uint16_t *)((const char *)a.Vc + kv_off) + (size_t)g * DH * a.stride;
    const int kb0 = c0 + wave * 32;
#pragma unroll
    for (int aa = 0; aa < 2; ++aa) {
        int key = kb0 + 8 * (n >> 2) + 4 * aa + (n & 3);
        if (key > a.pos0 - 1) key = a.pos0 - 1;     // dead positions are masked at use; stay in live memory
#pragma unroll
        for (int j = 0; j < KS; ++j) kv.k[aa][j] = *(const bf16x8 *)(Kg + (size_t)key * DH + j * 32 + gq * 8);
    }
#pragma unroll
    for (int dt = 0; dt < DT; ++dt) kv.v[dt] = *(const bf16x8 *)(Vg + (size_t)(dt * 16 + n) * a.stride + kb0 + gq * 8);
}

// `kv`: register block for the cached K/V; if `preloaded`, it already holds (or has in flight) the block of the
// first item, wg.
// F16: the cache, and the 16-bit halves of the queries and probabilities, are fp16 (else bf16).
template <int DH, int NTHREADS, class Io, bool F16, int RP = kAttnRowsPerPass>
__device__ __forceinline__ void attn_mfma_items(const AttnArgs &a, AttnMfmaLds<DH, RP> &L, int wg, int nwg, AttnKv<DH> &kv, bool preloaded,
                                                long long kv_off = 0) {
    constexpr int KS = DH / 32, DT = DH / 16, half = DH / 2, PR = DH + 2, PL = DH + 4;
    constexpr int NRH = NTHREADS / 256;      // wavefronts per key block
    const int tid = thread_index(), lane = tid & 63, wave = (tid >> 6) & 3, rh = tid >> 8;
    const int n = lane & 15, gq = lane >> 4;
    const int G = a.G, R = a.R;
    const int n_items = a.Hkv * a.S;
    uint16_t *qb16 = (uint16_t *)L.qb;

    for (int item = wg; item < n_items; item += nwg) {
        const int g = div_small(item, a.mul_S), s = item - g * a.S;
        const int c0 = s * a.C, c1 = (c0 + a.C < a.pos0) ? c0 + a.C : a.pos0;
        const int nc = (c1 > c0) ? c1 - c0 : 0;
        const bool last = (s == a.S - 1);
        const int nbc = (nc + 31) / 32;
        uint16_t *Kg = (uint16_t *)((char *)a.Kc + kv_off) + (size_t)g * a.stride * DH;
        uint16_t *Vg = (uint16_t *)((char *)a.Vc + kv_off) + (size_t)g * DH * a.stride;

        if (last) {
            // the call's own rows: rotate k, round to bf16, append to the cache, keep a copy in LDS
            for (int idx = tid; idx < a.m * half; idx += NTHREADS) {
                const int t = idx / half, i = idx % half;
                const float *kp = a.qkv + (size_t)t * a.ld + (size_t)a.Hq * DH + (size_t)g * DH;
                const float *vp = kp + (size_t)a.Hkv * DH;
                const float c = a.rope[(t * half + i) * 2], sn = a.rope[(t * half + i) * 2 + 1];
                const float x = Io::ld(kp + i), y = Io::ld(kp + i + half);
                const uint16_t k0 = f32_to_16<F16>(x * c - y * sn), k1 = f32_to_16<F16>(x * sn + y * c);
                const uint16_t v0 = f32_to_16<F16>(Io::ld(vp + i)), v1 = f32_to_16<F16>(Io::ld(vp + i + half));
                L.knew[t * DH + i] = k0;
                L.knew[t * DH + i + half] = k1;
                L.vnewT[i * 8 + t] = v0;
                L.vnewT[(i + half) * 8 + t] = v1;
                const size_t p = (size_t)(a.pos0 + t);
                Kg[p * DH + i] = k0;
                Kg[p * DH + i + half] = k1;
                Vg[(size_t)i * a.stride + p] = v0;
                Vg[(size_t)(i + half) * a.stride + p] = v1;
            }
        }
        const int kb0 = c0 + wave * 32;           // first cached position of this wavefront's block
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        const bool has_rows = R > rh * 8;         // this wavefront has a row block in the first pass at least
        for (int r0 = 0; r0 < R; r0 += RP) {
            const int nr = (R - r0 < RP) ? R - r0 : RP;
            const int nblk = (nr + 7) / 8;
            // this wavefront's cached block goes in flight first: it does not depend on the queries (a later pass
            // over more rows loads it again, from L2: the registers are reused for the call's own rows below)
            if (!(preloaded && item == wg && r0 == 0)) attn_load_kv<DH, NTHREADS>(a, item, kv, kv_off);
            // queries: rotate, scale, split hi/lo, store in B-operand order.  Each thread first issues the loads of
            // all its elements (at most 8 for 32 rows of 128 dims), then does the arithmetic.
            constexpr int QIT = (RP * half + NTHREADS - 1) / NTHREADS;
            float qx[QIT], qy[QIT], qc[QIT], qs_[QIT];
#pragma unroll
            for (int it = 0; it < QIT; ++it) {
                const int idx = tid + it * NTHREADS, rr = idx / half, i = idx % half, r = r0 + rr;
                qx[it] = qy[it] = qc[it] = qs_[it] = 0.f;
                if (idx < nblk * 8 * half && rr < nr) {
                    const int t = div_small(r, a.mul_G), hq = g * G + (r - t * G);
                    const float *qp = a.qkv + (size_t)t * a.ld + (size_t)hq * DH;
                    qx[it] = Io::ld(qp + i);
                    qy[it] = Io::ld(qp + i + half);
                    qc[it] = a.rope[(t * half + i) * 2];
                    qs_[it] = a.rope[(t * half + i) * 2 + 1];
                }
            }
#pragma unroll
            for (int it = 0; it < QIT; ++it) {
                const int idx = tid + it * NTHREADS, rr = idx / half, i = idx % half;
                if (idx < nblk * 8 * half) {
                    const float q0 = (qx[it] * qc[it] - qy[it] * qs_[it]) * a.scale;
                    const float q1 = (qx[it] * qs_[it] + qy[it] * qc[it]) * a.scale;
                    const int b = rr >> 3, col = rr & 7;
                    uint16_t hi, lo;
                    int d = i;
                    split_hi_lo<F16>(q0, hi, lo);
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col) * 8 + (d & 7)] = hi;
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col + 8) * 8 + (d & 7)] = lo;
                    d = i + half;
                    split_hi_lo<F16>(q1, hi, lo);
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col) * 8 + (d & 7)] = hi;
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col + 8) * 8 + (d & 7)] = lo;
                }
            }
            __syncthreads();

            // this wavefront's key blocks: one cached block (row blocks rh, rh + NRH, ...), and, in the item that
            // holds the end of the cache, the call's own rows: row block b of those goes to wavefront NW - 1 - b, so
            // that the wavefronts with the least cached work (none at all while m <= 2) take them in parallel
            constexpr int NW = NTHREADS / 64;
            const int wave8 = tid >> 6;
            for (int pass = 0; pass < 2; ++pass) {
                const bool is_new = (pass == 1);
                if (!is_new && (!has_rows || rh >= nblk || wave >= nbc)) continue;
                if (is_new && !(last && NW - 1 - wave8 < nblk)) continue;
                const int slot = is_new ? 4 : wave;
                const int b_first = is_new ? NW - 1 - wave8 : rh, b_step = is_new ? nblk : NRH;
                bf16x8 (&kreg)[2][KS] = kv.k;
                bf16x8 (&vreg)[DT] = kv.v;
                if (!is_new) {
                    if (kb0 + 32 > a.pos0) {      // ragged end of the cache: dead positions contribute nothing
#pragma unroll
                        for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (kb0 + gq * 8 + e >= a.pos0) vreg[dt][e] = 0;
                        }
                    }
                } else {
#pragma unroll
                    for (int aa = 0; aa < 2; ++aa) {
                        const int key = 8 * (n >> 2) + 4 * aa + (n & 3);
#pragma unroll
                        for (int j = 0; j < KS; ++j)
                            kreg[aa][j] = (key < a.m) ? *(const bf16x8 *)(L.knew + key * DH + j * 32 + gq * 8) : zero;
                    }
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        // keys gq * 8 .. + 7 of dimension dt * 16 + n: only the first lane group has live keys
                        bf16x8 cv = (gq == 0) ? *(const bf16x8 *)(L.vnewT + (dt * 16 + n) * 8) : zero;
#pragma unroll
                        for (int e = 0; e < 8; ++e)
                            if (e >= a.m) cv[e] = 0;
                        vreg[dt] = cv;
                    }
                }
                // Half precision has a narrow exponent range: probabilities below 2^-14 of their block's maximum would
                // be subnormal.  They enter the MFMA scaled by 2^10 (exact), and the products are scaled back.
                constexpr float kPScale = F16 ? 1024.0f : 1.0f;
                for (int b = b_first; b < nblk; b += b_step) {
                    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < KS; ++j) {
                        const bf16x8 q = L.qb[(b * KS + j) * 64 + lane];
                        s0 = mma16<F16>(kreg[0][j], q, s0);
                        s1 = mma16<F16>(kreg[1][j], q, s1);
                    }
                    // lane (n, gq) now holds, for query row b*8 + (n & 7), the keys gq*8 + 0..3 (s0) and
                    // gq*8 + 4..7 (s1) of the block: hi part in columns 0..7, lo part in columns 8..15
                    float sc[8];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        sc[c] = add_lane_xor8(s0[c]);
                        sc[4 + c] = add_lane_xor8(s1[c]);
                    }
                    const int rr = b * 8 + (n & 7), t_row = div_small(r0 + rr, a.mul_G);
                    float mx = -INFINITY;
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        const int key = gq * 8 + c;
                        const bool vis = is_new ? (key < a.m && key <= t_row) : (kb0 + key < a.pos0);
                        if (!vis) sc[c] = -INFINITY;
                        mx = fmaxf(mx, sc[c]);
                    }
                    mx = fmaxf(mx, __shfl_xor(mx, 16));
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    float sum = 0.f;
                    union { bf16x8 v; uint16_t u[8]; } pb;
#pragma unroll
                    for (int c = 0; c < 8; ++c) {
                        const float p = (sc[c] == -INFINITY) ? 0.f : __expf(sc[c] - mx);
                        sum += p;
                        uint16_t hi, lo;
                        split_hi_lo<F16>(p * kPScale, hi, lo);
                        pb.u[c] = (n < 8) ? hi : lo;
                    }
                    sum += __shfl_xor(sum, 16);
                    sum += __shfl_xor(sum, 32);
                    float *prow = L.part + ((size_t)slot * RP + rr) * PL;
                    f32x4 o[DT];
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
                        o[dt] = mma16<F16>(vreg[dt], pb.v, o[dt]);
                    }
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) o[dt][c] = add_lane_xor8(o[dt][c]) * (1.0f / kPScale);
                        if (n < 8 && rr < nr) *(f32x4 *)(prow + dt * 16 + gq * 4) = o[dt];
                    }
                    if (n < 8 && gq == 0 && rr < nr) {
                        prow[DH] = mx;
                        prow[DH + 1] = sum;
                    }
                }
            }
            __syncthreads();
            // fold this item's (up to 5) block partials in block order and publish one partial per row: a thread takes two
            // neighbouring dimensions of a row (DH / 2 threads, whole wavefronts, per row), derives the blocks' weights
            // exp(max_p - M) itself from their (max, sum) pairs (the same LDS words for the whole wavefront), and stores
            // eight bytes
            for (int idx = tid; idx < nr * half; idx += NTHREADS) {
                const int rr = idx / half, e = (idx % half) * 2;
                float mp[kAttnSlots], M = -INFINITY;
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    const bool on = p < 4 ? p < nbc : last;
                    mp[p] = on ? L.part[((size_t)p * RP + rr) * PL + DH] : -INFINITY;
                    M = fmaxf(M, mp[p]);
                }
                // (all slots are read, so that the reads go out together; what a slot without data holds is dropped)
                float sm[kAttnSlots];
                f32x2 v[kAttnSlots];
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    sm[p] = L.part[((size_t)p * RP + rr) * PL + DH + 1];
                    v[p] = *(const f32x2 *)(L.part + ((size_t)p * RP + rr) * PL + e);
                }
                float den = 0.f;
                f32x2 num = {0.f, 0.f};
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    const float w = (mp[p] == -INFINITY) ? 0.f : __expf(mp[p] - M);
                    const bool on = w != 0.f;
                    den += on ? w * sm[p] : 0.f;
                    num[0] += on ? w * v[p][0] : 0.f;
                    num[1] += on ? w * v[p][1] : 0.f;
                }
                float *out = a.part + (((size_t)g * a.S + s) * R + (r0 + rr)) * PR;
                Io::st2(out + e, num);
                if (e == 0) Io::st2(out + DH, (f32x2){M, den});
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// fold the splits of every query row, in split order, and pack the result for the Wo GEMM
// ---------------------------------------------------------------------------------------------------
// One wavefront per query row: the splits' (max, sum) pairs give the weights exp(max_s - M), then the lanes
// accumulate the weighted partial outputs in split order, two dimensions per lane, 32 splits' rows in flight at a
// time (at most 64 splits, i.e. one round trip to memory, for contexts up to 8192).
template <class Io, bool F16>
__device__ __forceinline__ void attn_combine_row(const AttnArgs &a, int row /* 0 .. Hkv * R */) {
    constexpr int NB = 32;                             // splits whose rows are in flight together
    const int DH = a.dh, PR = DH + 2, S = a.S;
    const int G = a.G, R = a.R;
    const int lane = thread_index() & 63;
    const int g = div_small(row, a.mul_R), r = row - g * R, t = div_small(r, a.mul_G), hq = g * G + (r - t * G);
    const float *base = a.part + ((size_t)g * S * R + r) * PR;
    const size_t sstride = (size_t)R * PR;
    const int e = 2 * lane;                            // this lane's two dimensions
    const bool e_on = e < DH;
    // batch [s0 + s1, s0 + s1 + NB) of partial rows, one 8-byte load per split and lane; splits past the end
    // repeat the last one (weight 0)
    auto load_batch = [&](f32x2 (&v)[NB], int first, int end) {
#pragma unroll
        for (int k = 0; k < NB; ++k) {
            const int ss = (first + k < end) ? first + k : end - 1;
            v[k] = e_on ? Io::ld2(base + (size_t)ss * sstride + e) : (f32x2){0.f, 0.f};
        }
    };
    // the maxima of the groups of 64 splits after the first (contexts beyond 64 splits only)
    float M = -INFINITY;
    for (int s = 64 + lane; s < S; s += 64) M = fmaxf(M, Io::ld(base + s * sstride + DH));
    float den = 0.f, o0 = 0.f, o1 = 0.f;
    for (int s0 = 0; s0 < S; s0 += 64) {
        const int ns = (S - s0 < 64) ? S - s0 : 64, sl = s0 + lane;
        // (max, sum) of split s0 + lane, and the first batch of rows: all loads are issued before any is used
        float pm = -INFINITY, ps = 0.f;
        if (sl < S) {
            pm = Io::ld(base + sl * sstride + DH);
            ps = Io::ld(base + sl * sstride + DH + 1);
        }
        f32x2 v[NB];
        load_batch(v, s0, s0 + ns);
        if (s0 == 0) {
            M = fmaxf(M, pm);
            for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
        }
        const float w = (pm == -INFINITY) ? 0.f : __expf(pm - M);
        float wl = w * ps;
        for (int off = 32; off > 0; off >>= 1) wl += __shfl_xor(wl, off);
        den += wl;
        for (int s1 = 0; s1 < ns; s1 += NB) {
            if (s1 > 0) load_batch(v, s0 + s1, s0 + ns);
#pragma unroll
            for (int k = 0; k < NB; ++k) {
                const float ws = (s1 + k < ns) ? __shfl(w, s1 + k) : 0.f;
                o0 += ws * v[k][0];
                o1 += ws * v[k][1];
            }
        }
    }
    if (e_on) {
        store_act_io<Io, F16>((uint16_t *)a.Bo, a.Bo_KT, hq * DH + e, t, o0 / den);
        store_act_io<Io, F16>((uint16_t *)a.Bo, a.Bo_KT, hq * DH + e + 1, t, o1 / den);
    }
}

}  // namespace ad
