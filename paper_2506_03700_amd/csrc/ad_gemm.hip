// Stand-alone launches of the weight-streaming skinny GEMM (device code in ad_gemm_device.h): every projection
// of the decoder layer when the layer step runs as separate kernels, the exit-head transform, and the LM head
// of Eq. 1 / Eq. 2 with its vocabulary reduction.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <string.h>

#include <mutex>

#include "ad_device.h"
#include "ad_gemm_device.h"
#include "ad_internal.h"

namespace ad {

// NCHMAX (stationary mode): chunks of k-steps per tile and wavefront that the B registers cover.  Chunks have 8
// k-steps for 16-bit weights, except in the widest instance (NCHMAX 8), whose 32 B registers leave room for
// chunks of 4 only; fp32 weights (three planes per k-step) have chunks of 2.
template <int NPL, int MODE, int NCHMAX, bool F16>
__global__ void __launch_bounds__(MODE == GEMM_STATIONARY ? kStatThreads : kThreads) k_gemm(GemmArgs g) {
    warm_kernel_args<sizeof(GemmArgs)>();
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    GemmLds &L = *reinterpret_cast<GemmLds *>(lds_raw);
    if constexpr (MODE == GEMM_STATIONARY) {
        constexpr int CH = NPL == 1 ? (NCHMAX > 3 ? 4 : 8) : 2;
        StatStream<NPL, CH> S;
        S.init(g, blockIdx.x, 0x7fffffff);       // every workgroup of this launch has tiles (the grid size is an argument fetch away)
        gemm_stationary<NPL, CH, NCHMAX, IoPlain, -1, F16, false>(g, S, L, NoTail());
    } else {
        constexpr int U = NPL == 1 ? 4 : 2;
        StreamStream<NPL, U, kWaves> S;
        S.init(g, blockIdx.x, 0x7fffffff);
        S.prefetch(g);
        gemm_streamed<NPL, U, kWaves, IoPlain, -1, false, F16>(g, S, L, NoTail());
    }
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
    if (g.done_flag && threadIdx.x == 0) {
        // the other wavefronts' results were written before the barrier above: this release covers them too
        __hip_atomic_store(g.done_flag, g.done_seq, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
    }
}

template <int NPL, int MODE, int NCHMAX, bool F16 = false>
static int launch_one(const GemmArgs &g, int grid, hipStream_t s) {
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_gemm<NPL, MODE, NCHMAX, F16>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)sizeof(GemmLds));
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    GemmArgs ga = g;
    set_tile_partition(ga, grid);
    hipLaunchKernelGGL((k_gemm<NPL, MODE, NCHMAX, F16>), dim3(grid), dim3(MODE == GEMM_STATIONARY ? kStatThreads : kThreads), sizeof(GemmLds), s, ga);
    return (int)hipGetLastError();
}

// 16-bit weights: the instance whose B registers cover the wavefront's K slice (d_model <= 4096, <= 6144, <= 8192)
template <bool F16>
static int stationary16(const GemmArgs &g, int nks, int grid, hipStream_t s) {
    if (nks <= 16) return launch_one<1, GEMM_STATIONARY, 2, F16>(g, grid, s);
    if (nks <= 24) return launch_one<1, GEMM_STATIONARY, 3, F16>(g, grid, s);
    return launch_one<1, GEMM_STATIONARY, kKsMaxWide / 4, F16>(g, grid, s);
}

int launch_gemm(const GemmArgs &g, int planes, const LaunchCtx &c) {
    // equal numbers of row tiles per workgroup: with per = ceil(NT / n_wg) tiles each, ceil(NT / per) workgroups
    const int grid = head_grid(g.NT, c.n_wg);
    hipStream_t s = (hipStream_t)c.stream;
    const bool f16 = g.elem == kElemF16;
    if ((planes == 1) != (g.elem != kElemF32)) return (int)hipErrorInvalidValue;     // fp32 weights are three bf16 planes
    int rc;
    if (g.mode == GEMM_STATIONARY) {
        const int nks = (g.KT + kStatWaves - 1) / kStatWaves;     // most k-steps of a wavefront
        if (nks > (planes == 1 ? kKsMaxWide : kKsMax) || g.K < 8) return (int)hipErrorInvalidValue;
        if (planes != 1) rc = launch_one<3, GEMM_STATIONARY, kKsMax / 2>(g, grid, s);
        else if (f16) rc = stationary16<true>(g, nks, grid, s);
        else rc = stationary16<false>(g, nks, grid, s);
    } else {
        if (planes != 1) rc = launch_one<3, GEMM_STREAMED, 0>(g, grid, s);
        else rc = f16 ? launch_one<1, GEMM_STREAMED, 0, true>(g, grid, s) : launch_one<1, GEMM_STREAMED, 0>(g, grid, s);
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

// ---- scratch for callers that cannot allocate --------------------------------------------------------------
// The vocabulary pass leaves one (max, sum of exp, argmax) partial per workgroup and token, which its second kernel
// folds.  Normally they live in the model's workspace; the allocation-free entry point keeps them in this
// file-scope array instead: kStaticHeadParts workgroups x 8 tokens x 4 floats = 512 KiB, held by every GPU the
// library runs on until the process ends.  In host code the array's name is only a stand-in for the symbol: its
// device address is asked for once per device (with that device current) and kept.
static __device__ __align__(256) float scratch[(size_t)kStaticHeadParts * 8 * 4];

int static_head_scratch(float **ptr) {
    constexpr int kMaxDevices = 64;
    static float *addr[kMaxDevices];
    static bool have[kMaxDevices];
    static std::mutex mu;
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return (int)e;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(mu);
    if (!have[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return (int)e;
        if (!p) return (int)hipErrorInvalidSymbol;
        addr[dev] = (float *)p;
        have[dev] = true;
    }
    *ptr = addr[dev];
    return 0;
}

int head_grid(int n_tiles, int n_wg) {
    const int per = (n_tiles + n_wg - 1) / n_wg;
    const int grid = (n_tiles + per - 1) / (per < 1 ? 1 : per);
    return grid < 1 ? 1 : grid;
}

int gemm_max_stationary_k(int planes) { return (planes == 1 ? kKsMaxWide : kKsMax) * kStatWaves * 32; }

}  // namespace ad
