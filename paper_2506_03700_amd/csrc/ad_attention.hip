// Attention phase of the layer step: rotary embedding of q and k, KV append, and grouped-query causal
// attention of the call's m rows over the layer's cache, split over the context.
//
// Cache layout of one layer (elements of the cache type, stride = max_pos rounded up to 64):
//   K [kv head][position 0..stride)[head_dim]   (rotated keys, one 2*dh- or 4*dh-byte row per position)
//   V [kv head][head_dim][position 0..stride)   (transposed, so that 8 consecutive positions of one
//                                                dimension are one 128-bit load: the MFMA operand of P.V)
//
// Work item (kv head g, split s): cache positions [s*C, min((s+1)*C, pos0)) of head g; the last split also
// takes the call's own m rows (rotated, rounded to the cache type, appended to the cache, attended to under
// the causal mask).  All G*m query rows of the group are processed against each K/V element while it is in
// registers or LDS, so the cache is read once.  An item writes one unnormalised partial (o[dh], max, sum)
// per query row; a second, small kernel folds the partials of each row in split order (fixed order:
// results are reproducible) and packs the result as the activation block of the Wo GEMM.  There is no
// fence or atomic inside either kernel: the kernel boundary orders them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_device.h"
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
constexpr int kAttnThreads = 256;
constexpr int kAttnWaves = 4;
constexpr int kAttnRowsPerPass = 32;
constexpr int kAttnSlots = 5;   // 4 cached blocks + the call's own rows

template <int DH>
struct AttnMfmaLds {
    bf16x8 qb[4 * (DH / 32) * 64];                       // [row block][k-step][lane]
    uint16_t knew[8 * DH], vnew[8 * DH];                  // the call's own rows, cache type
    float part[kAttnSlots * kAttnRowsPerPass * (DH + 4)];   // rows padded to 16 bytes for 128-bit LDS stores
};

template <int DH>
__global__ void __launch_bounds__(kAttnThreads) k_attn_mfma(AttnArgs a) {
    constexpr int KS = DH / 32, DT = DH / 16, half = DH / 2, PR = DH + 2, PL = DH + 4;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    AttnMfmaLds<DH> &L = *reinterpret_cast<AttnMfmaLds<DH> *>(lds_raw);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = lane & 15, gq = lane >> 4;
    const int G = a.Hq / a.Hkv, R = G * a.m;
    const int n_items = a.Hkv * a.S;
    uint16_t *qb16 = (uint16_t *)L.qb;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int g = item / a.S, s = item % a.S;
        const int c0 = s * a.C, c1 = (c0 + a.C < a.pos0) ? c0 + a.C : a.pos0;
        const int nc = (c1 > c0) ? c1 - c0 : 0;
        const bool last = (s == a.S - 1);
        const int nbc = (nc + 31) / 32;
        uint16_t *Kg = (uint16_t *)a.Kc + (size_t)g * a.stride * DH;
        uint16_t *Vg = (uint16_t *)a.Vc + (size_t)g * DH * a.stride;

        if (last) {
            // the call's own rows: rotate k, round to bf16, append to the cache, keep a copy in LDS
            for (int idx = tid; idx < a.m * half; idx += kAttnThreads) {
                const int t = idx / half, i = idx % half;
                const float *kp = a.qkv + (size_t)t * a.ld + (size_t)a.Hq * DH + (size_t)g * DH;
                const float *vp = kp + (size_t)a.Hkv * DH;
                const float c = a.rope[(t * half + i) * 2], sn = a.rope[(t * half + i) * 2 + 1];
                const float x = kp[i], y = kp[i + half];
                const uint16_t k0 = f32_to_bf16_bits(x * c - y * sn), k1 = f32_to_bf16_bits(x * sn + y * c);
                const uint16_t v0 = f32_to_bf16_bits(vp[i]), v1 = f32_to_bf16_bits(vp[i + half]);
                L.knew[t * DH + i] = k0;
                L.knew[t * DH + i + half] = k1;
                L.vnew[t * DH + i] = v0;
                L.vnew[t * DH + i + half] = v1;
                const size_t p = (size_t)(a.pos0 + t);
                Kg[p * DH + i] = k0;
                Kg[p * DH + i + half] = k1;
                Vg[(size_t)i * a.stride + p] = v0;
                Vg[(size_t)(i + half) * a.stride + p] = v1;
            }
        }
        // this wavefront's cached block goes in flight first: it does not depend on the queries
        const int kb0 = c0 + wave * 32;           // first cached position of the block
        const bf16x8 zero = {0, 0, 0, 0, 0, 0, 0, 0};
        bf16x8 kc[2][KS], vc[DT];
        if (wave < nbc) {
#pragma unroll
            for (int aa = 0; aa < 2; ++aa) {
                int key = kb0 + 8 * (n >> 2) + 4 * aa + (n & 3);
                if (key > a.pos0 - 1) key = a.pos0 - 1;     // dead positions are masked below; stay in live memory
#pragma unroll
                for (int j = 0; j < KS; ++j) kc[aa][j] = *(const bf16x8 *)(Kg + (size_t)key * DH + j * 32 + gq * 8);
            }
#pragma unroll
            for (int dt = 0; dt < DT; ++dt) vc[dt] = *(const bf16x8 *)(Vg + (size_t)(dt * 16 + n) * a.stride + kb0 + gq * 8);
        }
        for (int r0 = 0; r0 < R; r0 += kAttnRowsPerPass) {
            const int nr = (R - r0 < kAttnRowsPerPass) ? R - r0 : kAttnRowsPerPass;
            const int nblk = (nr + 7) / 8;
            // queries: rotate, scale, split hi/lo, store in B-operand order.  Each thread first issues the loads of
            // all its elements (at most 8 for 32 rows of 128 dims), then does the arithmetic.
            constexpr int QIT = (kAttnRowsPerPass * half + kAttnThreads - 1) / kAttnThreads;
            float qx[QIT], qy[QIT], qc[QIT], qs_[QIT];
#pragma unroll
            for (int it = 0; it < QIT; ++it) {
                const int idx = tid + it * kAttnThreads, rr = idx / half, i = idx % half, r = r0 + rr;
                qx[it] = qy[it] = qc[it] = qs_[it] = 0.f;
                if (idx < nblk * 8 * half && rr < nr) {
                    const int t = r / G, hq = g * G + r % G;
                    const float *qp = a.qkv + (size_t)t * a.ld + (size_t)hq * DH;
                    qx[it] = qp[i];
                    qy[it] = qp[i + half];
                    qc[it] = a.rope[(t * half + i) * 2];
                    qs_[it] = a.rope[(t * half + i) * 2 + 1];
                }
            }
#pragma unroll
            for (int it = 0; it < QIT; ++it) {
                const int idx = tid + it * kAttnThreads, rr = idx / half, i = idx % half;
                if (idx < nblk * 8 * half) {
                    const float q0 = (qx[it] * qc[it] - qy[it] * qs_[it]) * a.scale;
                    const float q1 = (qx[it] * qs_[it] + qy[it] * qc[it]) * a.scale;
                    const int b = rr >> 3, col = rr & 7;
                    uint16_t hi, lo;
                    int d = i;
                    split_hi_lo(q0, hi, lo);
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col) * 8 + (d & 7)] = hi;
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col + 8) * 8 + (d & 7)] = lo;
                    d = i + half;
                    split_hi_lo(q1, hi, lo);
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col) * 8 + (d & 7)] = hi;
                    qb16[(((b * KS + (d >> 5)) * 64) + ((d & 31) >> 3) * 16 + col + 8) * 8 + (d & 7)] = lo;
                }
            }
            __syncthreads();

            // this wavefront's key blocks: one cached block, and (one wavefront only) the call's own rows
            const int w_new = nbc % kAttnWaves;
            for (int pass = 0; pass < 2; ++pass) {
                const bool is_new = (pass == 1);
                if (!is_new && wave >= nbc) continue;
                if (is_new && !(last && wave == w_new)) continue;
                const int slot = is_new ? 4 : wave;
                bf16x8 kreg[2][KS], vreg[DT];
                if (!is_new) {
#pragma unroll
                    for (int aa = 0; aa < 2; ++aa)
#pragma unroll
                        for (int j = 0; j < KS; ++j) kreg[aa][j] = kc[aa][j];
                    const bool ragged = kb0 + 32 > a.pos0;
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        bf16x8 v = vc[dt];
                        if (ragged) {
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (kb0 + gq * 8 + e >= a.pos0) v[e] = 0;
                        }
                        vreg[dt] = v;
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
                        union { bf16x8 v; uint16_t u[8]; } cv;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int key = gq * 8 + e;
                            cv.u[e] = (key < a.m) ? L.vnew[key * DH + dt * 16 + n] : (uint16_t)0;
                        }
                        vreg[dt] = cv.v;
                    }
                }
                for (int b = 0; b < nblk; ++b) {
                    f32x4 s0 = {0.f, 0.f, 0.f, 0.f}, s1 = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int j = 0; j < KS; ++j) {
                        const bf16x8 q = L.qb[(b * KS + j) * 64 + lane];
                        s0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[0][j], q, s0, 0, 0, 0);
                        s1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kreg[1][j], q, s1, 0, 0, 0);
                    }
                    // lane (n, gq) now holds, for query row b*8 + (n & 7), the keys gq*8 + 0..3 (s0) and
                    // gq*8 + 4..7 (s1) of the block: hi part in columns 0..7, lo part in columns 8..15
                    float sc[8];
#pragma unroll
                    for (int c = 0; c < 4; ++c) {
                        sc[c] = add_lane_xor8(s0[c]);
                        sc[4 + c] = add_lane_xor8(s1[c]);
                    }
                    const int rr = b * 8 + (n & 7), t_row = (r0 + rr) / G;
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
                        split_hi_lo(p, hi, lo);
                        pb.u[c] = (n < 8) ? hi : lo;
                    }
                    sum += __shfl_xor(sum, 16);
                    sum += __shfl_xor(sum, 32);
                    float *prow = L.part + ((size_t)slot * kAttnRowsPerPass + rr) * PL;
                    f32x4 o[DT];
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
                        o[dt] = (f32x4){0.f, 0.f, 0.f, 0.f};
                        o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vreg[dt], pb.v, o[dt], 0, 0, 0);
                    }
#pragma unroll
                    for (int dt = 0; dt < DT; ++dt) {
#pragma unroll
                        for (int c = 0; c < 4; ++c) o[dt][c] = add_lane_xor8(o[dt][c]);
                        if (n < 8 && rr < nr) *(f32x4 *)(prow + dt * 16 + gq * 4) = o[dt];
                    }
                    if (n < 8 && gq == 0 && rr < nr) {
                        prow[DH] = mx;
                        prow[DH + 1] = sum;
                    }
                }
            }
            __syncthreads();
            // fold this item's (up to 5) block partials in block order and publish one partial per row:
            // first the weights exp(max_p - M) of each row's blocks, then the weighted sums, all loads up front
            float *wts = reinterpret_cast<float *>(L.qb);       // [row][8]: weights of the 5 slots, M, sum (queries are done)
            if (tid < nr) {
                float mp[kAttnSlots], M = -INFINITY;
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    const bool on = p < 4 ? p < nbc : last;
                    mp[p] = on ? L.part[((size_t)p * kAttnRowsPerPass + tid) * PL + DH] : -INFINITY;
                    M = fmaxf(M, mp[p]);
                }
                float den = 0.f;
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    const float w = (mp[p] == -INFINITY) ? 0.f : __expf(mp[p] - M);
                    wts[tid * 8 + p] = w;
                    if (w != 0.f) den += w * L.part[((size_t)p * kAttnRowsPerPass + tid) * PL + DH + 1];
                }
                wts[tid * 8 + 5] = M;
                wts[tid * 8 + 6] = den;
            }
            __syncthreads();
            for (int idx = tid; idx < nr * DH; idx += kAttnThreads) {
                const int rr = idx / DH, e = idx % DH;
                float v[kAttnSlots], w[kAttnSlots];
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p) {
                    w[p] = wts[rr * 8 + p];
                    v[p] = L.part[((size_t)p * kAttnRowsPerPass + rr) * PL + e];    // slots without data have weight 0
                }
                float num = 0.f;
#pragma unroll
                for (int p = 0; p < kAttnSlots; ++p)
                    if (w[p] != 0.f) num += w[p] * v[p];
                float *out = a.part + (((size_t)g * a.S + s) * R + (r0 + rr)) * PR;
                out[e] = num;
                if (e == 0) {
                    out[DH] = wts[rr * 8 + 5];
                    out[DH + 1] = wts[rr * 8 + 6];
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// any cache type: plain vector-ALU kernel (used for fp32 caches, where the model is small)
// ---------------------------------------------------------------------------------------------------
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

constexpr int kValuThreads = 1024;
constexpr int kValuMaxRows = 32;
// keys per work item: a chunk of cached positions plus up to 8 new rows; sized so that the K and V tiles fit LDS
constexpr int valu_max_keys(size_t kv_elem, int dh) { return (kv_elem * dh <= 256) ? 136 : 72; }

template <typename KVT, int DH>
__global__ void __launch_bounds__(kValuThreads) k_attn_valu(AttnArgs a) {
    constexpr int KROW = DH + 16 / sizeof(KVT);       // padded row against LDS bank conflicts
    constexpr int MAXK = valu_max_keys(sizeof(KVT), DH);
    constexpr int half = DH / 2;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int G = a.Hq / a.Hkv, R = G * a.m;
    float *qs = (float *)lds_raw;                   // [kValuMaxRows][DH]
    float *sc = qs + kValuMaxRows * DH;             // [kValuMaxRows][MAXK]
    float *st = sc + kValuMaxRows * MAXK;           // [kValuMaxRows][2]
    KVT *Ks = (KVT *)(st + kValuMaxRows * 2 + 4);   // [MAXK][KROW]
    KVT *Vs = Ks + MAXK * KROW;
    const int n_items = a.Hkv * a.S;
    const size_t PR = DH + 2;

    for (int item = blockIdx.x; item < n_items; item += gridDim.x) {
        const int g = item / a.S, s = item % a.S;
        const int c0 = s * a.C, c1 = (c0 + a.C < a.pos0) ? c0 + a.C : a.pos0;
        const int nc = (c1 > c0) ? c1 - c0 : 0;
        const bool last = (s == a.S - 1);
        const int nk = nc + (last ? a.m : 0);
        KVT *Kg = (KVT *)a.Kc + (size_t)g * a.stride * DH, *Vg = (KVT *)a.Vc + (size_t)g * DH * a.stride;
        for (int idx = tid; idx < nc * DH; idx += kValuThreads) {
            const int j = idx / DH, e = idx % DH;
            Ks[j * KROW + e] = Kg[(size_t)(c0 + j) * DH + e];
        }
        for (int idx = tid; idx < nc * DH; idx += kValuThreads) {
            const int e = idx / nc, j = idx % nc;
            Vs[j * KROW + e] = Vg[(size_t)e * a.stride + c0 + j];
        }
        if (last) {
            for (int idx = tid; idx < a.m * half; idx += kValuThreads) {
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
                const size_t p = (size_t)(a.pos0 + t);
                Kg[p * DH + i] = k0;
                Kg[p * DH + i + half] = k1;
                Vg[(size_t)i * a.stride + p] = v0;
                Vg[(size_t)(i + half) * a.stride + p] = v1;
            }
        }
        for (int r0 = 0; r0 < R; r0 += kValuMaxRows) {
            const int nr = (R - r0 < kValuMaxRows) ? R - r0 : kValuMaxRows;
            for (int idx = tid; idx < nr * half; idx += kValuThreads) {
                const int rr = idx / half, i = idx % half, r = r0 + rr, t = r / G, hq = g * G + r % G;
                const float *qp = a.qkv + (size_t)t * a.ld + (size_t)hq * DH;
                const float c = a.rope[(t * half + i) * 2], sn = a.rope[(t * half + i) * 2 + 1];
                const float x = qp[i], y = qp[i + half];
                qs[rr * DH + i] = (x * c - y * sn) * a.scale;
                qs[rr * DH + i + half] = (x * sn + y * c) * a.scale;
            }
            __syncthreads();
            for (int p = tid; p < nr * nk; p += kValuThreads) {
                const int rr = p / nk, j = p % nk, t = (r0 + rr) / G;
                float acc = 0.f;
                const KVT *kr = Ks + j * KROW;
                const float *qr = qs + rr * DH;
#pragma unroll 8
                for (int e = 0; e < DH; ++e) acc += qr[e] * kv_to_f32<KVT>(kr[e]);
                if (j >= nc && j - nc > t) acc = -INFINITY;     // causal mask among the call's own rows
                sc[rr * MAXK + j] = acc;
            }
            __syncthreads();
            for (int rr = wave; rr < nr; rr += kValuThreads / 64) {
                float mx = -INFINITY;
                for (int j = lane; j < nk; j += 64) mx = fmaxf(mx, sc[rr * MAXK + j]);
                for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
                float sum = 0.f;
                for (int j = lane; j < nk; j += 64) {
                    const float sv = sc[rr * MAXK + j];
                    const float pv = (sv == -INFINITY) ? 0.f : __expf(sv - mx);
                    sc[rr * MAXK + j] = pv;
                    sum += pv;
                }
                for (int off = 32; off > 0; off >>= 1) sum += __shfl_xor(sum, off);
                if (lane == 0) {
                    st[rr * 2] = mx;
                    st[rr * 2 + 1] = sum;
                }
            }
            __syncthreads();
            for (int idx = tid; idx < nr * DH; idx += kValuThreads) {
                const int rr = idx / DH, e = idx % DH;
                float acc = 0.f;
                for (int j = 0; j < nk; ++j) acc += sc[rr * MAXK + j] * kv_to_f32<KVT>(Vs[j * KROW + e]);
                float *pr = a.part + (((size_t)g * a.S + s) * R + (r0 + rr)) * PR;
                pr[e] = acc;
                if (e == 0) {
                    pr[DH] = st[rr * 2];
                    pr[DH + 1] = st[rr * 2 + 1];
                }
            }
            __syncthreads();
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// fold the splits of every query row, in split order, and pack the result for the Wo GEMM
// ---------------------------------------------------------------------------------------------------
// One wavefront per query row: the splits' (max, sum) pairs give the weights exp(max_s - M), then the lanes
// accumulate the weighted partial outputs, two or one dimension per lane, 8 splits' rows in flight at a time.
__global__ void __launch_bounds__(256) k_attn_combine(AttnArgs a) {
    const int DH = a.dh, PR = DH + 2;
    const int G = a.Hq / a.Hkv, R = G * a.m;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = blockIdx.x * 4 + wave;           // 0 .. Hkv * R
    if (row >= a.Hkv * R) return;
    const int g = row / R, r = row % R, t = r / G, hq = g * G + r % G;
    const float *base = a.part + ((size_t)g * a.S * R + r) * PR;
    const size_t sstride = (size_t)R * PR;
    float M = -INFINITY;
    for (int s = lane; s < a.S; s += 64) M = fmaxf(M, base[s * sstride + DH]);
    for (int off = 32; off > 0; off >>= 1) M = fmaxf(M, __shfl_xor(M, off));
    float den = 0.f, o0 = 0.f, o1 = 0.f;
    const int e0 = lane, e1 = lane + 64;
    for (int s0 = 0; s0 < a.S; s0 += 64) {
        // weights of up to 64 splits, one per lane
        const int sl = s0 + lane;
        float w = 0.f, wl = 0.f;
        if (sl < a.S) {
            const float pm = base[sl * sstride + DH];
            w = (pm == -INFINITY) ? 0.f : __expf(pm - M);
            wl = w * base[sl * sstride + DH + 1];
        }
        for (int off = 32; off > 0; off >>= 1) wl += __shfl_xor(wl, off);
        den += wl;
        const int ns = (a.S - s0 < 64) ? a.S - s0 : 64;
        for (int s1 = 0; s1 < ns; s1 += 8) {
            float v0[8], v1[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int ss = (s1 + k < ns) ? s1 + k : ns - 1;
                const float *pr = base + (size_t)(s0 + ss) * sstride;
                v0[k] = pr[e0];
                v1[k] = (e1 < DH) ? pr[e1] : 0.f;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float ws = (s1 + k < ns) ? __shfl(w, s1 + k) : 0.f;
                o0 += ws * v0[k];
                o1 += ws * v1[k];
            }
        }
    }
    if (e0 < DH) store_act((uint16_t *)a.Bo, hq * DH + e0, t, o0 / den);
    if (e1 < DH) store_act((uint16_t *)a.Bo, hq * DH + e1, t, o1 / den);
}

// ---------------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------------
constexpr size_t valu_lds_bytes(size_t kv_elem, int dh) {
    return (size_t)kValuMaxRows * dh * 4 + (size_t)kValuMaxRows * valu_max_keys(kv_elem, dh) * 4 + kValuMaxRows * 2 * 4 + 16 +
           2 * (size_t)valu_max_keys(kv_elem, dh) * (dh + 16 / kv_elem) * kv_elem;
}

int attn_chunk(int kv_is_bf16, int dh) { return kv_is_bf16 ? 128 : valu_max_keys(4, dh) - 8; }

template <typename KVT, int DH>
static int launch_valu(const AttnArgs &a, const LaunchCtx &c) {
    const size_t lds = valu_lds_bytes(sizeof(KVT), DH);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_valu<KVT, DH>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    int grid = a.Hkv * a.S;
    if (grid > 4 * c.n_wg) grid = 4 * c.n_wg;
    hipLaunchKernelGGL((k_attn_valu<KVT, DH>), dim3(grid), dim3(kValuThreads), lds, (hipStream_t)c.stream, a);
    return (int)hipGetLastError();
}

template <int DH>
static int launch_mfma(const AttnArgs &a, const LaunchCtx &c) {
    const size_t lds = sizeof(AttnMfmaLds<DH>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_mfma<DH>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    int grid = a.Hkv * a.S;
    if (grid > 8 * c.n_wg) grid = 8 * c.n_wg;
    hipLaunchKernelGGL((k_attn_mfma<DH>), dim3(grid), dim3(kAttnThreads), lds, (hipStream_t)c.stream, a);
    return (int)hipGetLastError();
}

int launch_attn(const AttnArgs &a, const LaunchCtx &c) {
    int rc;
    if (a.kv_is_bf16) {
        if (a.dh == 128) rc = launch_mfma<128>(a, c);
        else if (a.dh == 64) rc = launch_mfma<64>(a, c);
        else return (int)hipErrorInvalidValue;
    } else {
        if (a.dh == 128) rc = launch_valu<float, 128>(a, c);
        else if (a.dh == 64) rc = launch_valu<float, 64>(a, c);
        else return (int)hipErrorInvalidValue;
    }
    if (rc) return rc;
    const int rows = a.Hq * a.m;
    hipLaunchKernelGGL(k_attn_combine, dim3((rows + 3) / 4), dim3(256), 0, (hipStream_t)c.stream, a);
    return (int)hipGetLastError();
}

}  // namespace ad
