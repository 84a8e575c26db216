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

#include "ad_attention_device.h"
#include "ad_device.h"
#include "ad_internal.h"

namespace ad {

// ---------------------------------------------------------------------------------------------------
// bf16 cache: MFMA kernel (device code in ad_attention_device.h), 8 wavefronts per work item: two per block of
// 32 cached positions, which share the blocks of 8 query rows between them
// ---------------------------------------------------------------------------------------------------
constexpr int kAttnThreads = 512;

// NT, RP: 512 threads and 32 query rows per pass; or, for calls with at most 16 query rows per kv head and more work
// items than compute units, 256 threads (one wavefront per block of 32 positions) and 8 rows per pass, whose
// registers and 30 KB of LDS let workgroups share a compute unit, so that one item's loads overlap another's
// arithmetic (an item is a chain of dependent steps; with one workgroup per compute unit, items run one after the
// other).  Measured on the 8B shape at context 6000 (376 items): faster up to 16 rows, slower from 24 rows on.
template <int DH, bool F16, int NT, int RP>
__global__ void __launch_bounds__(NT, NT == 256 ? 2 : 1) k_attn_mfma(AttnArgs a) {
    warm_kernel_args<sizeof(AttnArgs)>();
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    AttnKv<DH> kv;
    attn_mfma_items<DH, NT, IoPlain, F16, RP>(a, *reinterpret_cast<AttnMfmaLds<DH, RP> *>(lds_raw), blockIdx.x, gridDim.x, kv, false);
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
__global__ void __launch_bounds__(256) k_attn_combine(AttnArgs a) {
    warm_kernel_args<sizeof(AttnArgs)>();
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row < a.Hq * a.m) {
        if (a.kv_elem == ELEM_F16) attn_combine_row<IoPlain, true>(a, row);
        else attn_combine_row<IoPlain, false>(a, row);
    }
}

// ---------------------------------------------------------------------------------------------------
// launchers
// ---------------------------------------------------------------------------------------------------
constexpr size_t valu_lds_bytes(size_t kv_elem, int dh) {
    return (size_t)kValuMaxRows * dh * 4 + (size_t)kValuMaxRows * valu_max_keys(kv_elem, dh) * 4 + kValuMaxRows * 2 * 4 + 16 +
           2 * (size_t)valu_max_keys(kv_elem, dh) * (dh + 16 / kv_elem) * kv_elem;
}

int attn_chunk(int kv_elem, int dh) { return kv_elem != kElemF32 ? 128 : valu_max_keys(4, dh) - 8; }

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

template <int DH, bool F16, int NT, int RP>
static int launch_mfma_as(const AttnArgs &a, const LaunchCtx &c) {
    const size_t lds = sizeof(AttnMfmaLds<DH, RP>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_attn_mfma<DH, F16, NT, RP>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    int grid = a.Hkv * a.S;
    if (grid > 8 * c.n_wg) grid = 8 * c.n_wg;
    hipLaunchKernelGGL((k_attn_mfma<DH, F16, NT, RP>), dim3(grid), dim3(NT), lds, (hipStream_t)c.stream, a);
    return (int)hipGetLastError();
}

template <int DH, bool F16>
static int launch_mfma(const AttnArgs &a, const LaunchCtx &c) {
    const int rows = (a.Hq / a.Hkv) * a.m;
    if (rows <= 16 && a.Hkv * a.S > c.n_wg) return launch_mfma_as<DH, F16, 256, 8>(a, c);
    return launch_mfma_as<DH, F16, kAttnThreads, kAttnRowsPerPass>(a, c);
}

int launch_attn(const AttnArgs &a, const LaunchCtx &c) {
    int rc;
    if (a.kv_elem == kElemBF16) {
        if (a.dh == 128) rc = launch_mfma<128, false>(a, c);
        else if (a.dh == 64) rc = launch_mfma<64, false>(a, c);
        else return (int)hipErrorInvalidValue;
    } else if (a.kv_elem == kElemF16) {
        if (a.dh == 128) rc = launch_mfma<128, true>(a, c);
        else if (a.dh == 64) rc = launch_mfma<64, true>(a, c);
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
