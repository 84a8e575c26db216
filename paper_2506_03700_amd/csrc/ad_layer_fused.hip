// The whole decoder-layer step ("update the KV cache at layer l" of Algorithm 1, for m <= 8 ragged rows) as ONE
// persistent kernel for bf16 models: one workgroup of 8 wavefronts per compute unit runs the six phases
//   QKV projection (RMSNorm fused) | attention items | fold of the splits | Wo + residual |
//   gate/up (RMSNorm fused) + SwiGLU | down + residual
// separated by five grid barriers.  A launch runs a stretch of consecutive layers over the same rows, with a sixth
// barrier from each layer to the next.  Compared with one kernel per phase this removes the launch gaps and lets
// every workgroup put the first weight batches of the next phase (or of the next layer's first phase) in flight
// *while* it waits at the barrier (weights do not depend on the previous phase), so the HBM stream hardly stops at
// a phase boundary.
//
// Data handed from one phase to the next (q/k/v rows, attention partials, packed activations, x') is written
// and read with relaxed agent-scope atomics (see IoAgent): the stores go through to memory, a wavefront waits
// for its stores to complete before it arrives at the barrier, and the loads do not use a stale line of another
// XCD's L2.  The barrier itself is two levels of relaxed agent-scope counters (eight groups, then one global
// counter); no cache write-back is issued anywhere (every exchanged value is stored write-through).  Where the
// next phase reads a large block that all workgroups share (the packed B operands, x') with ordinary loads, the
// barrier ends with one agent-scope acquire fence issued by thread 0 of each workgroup: it invalidates that compute
// unit's L1 and the non-local lines of its XCD's L2, which is all an ordinary load can have stale; one thread is
// enough because the invalidate acts on the caches, not on the issuing wavefront, and the workgroup's other
// wavefronts are held at the workgroup barrier that follows it.  Weights and the cached K/V rows were written by
// earlier kernels and are read with ordinary loads.
//
// Every wait is bounded: a workgroup that waits longer than kBarrierTimeoutTicks sets the host-visible abort
// flag and the whole grid leaves the kernel (the host then reports an error and resets the counters).  The
// grid must be co-resident, which holds because it has one workgroup per compute unit and layer steps of a
// model are stream-ordered.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "ad_attention_device.h"
#include "ad_device.h"
#include "ad_gemm_device.h"
#include "ad_internal.h"

namespace ad {

constexpr int kFusedThreads = 512;
constexpr long long kBarrierTimeoutTicks = 20000000;   // 0.2 s of the 100 MHz wall clock

struct GridBarrier {
    unsigned *ctr;         // [0]: global counter; [16]: "a workgroup gave up"; [32 * (1 + g)]: counter of group g
    unsigned round;        // barriers completed, over all launches (wraps; only differences are used)
    unsigned *abort_flag;  // host-visible
    int *ok;               // in LDS

    // Returns false (to every thread of the workgroup) if the wait timed out or another workgroup gave up.
    // acquire: also invalidate this compute unit's L1 and this XCD's stale L2 lines, so that ordinary loads after
    // the barrier see what other workgroups stored (write-through) before it.
    // pre: issues the next phase's first weight loads.  It runs after the workgroup has counted itself in (issuing
    // loads to a region nobody has touched yet can stall a wavefront for microseconds, which must not delay the
    // other workgroups) and while wavefront 0 waits for the grid; wavefront 0 issues its own share after the wait,
    // because its polling loads would queue behind them.
    template <class Pre>
    __device__ __forceinline__ bool sync(bool acquire, Pre pre) {
        __builtin_amdgcn_s_waitcnt(0);     // this wavefront's stores have completed
        __syncthreads();
        ++round;
        const int tid = thread_index();
        if (tid >= 64) pre();
        if (tid == 0) {
            const unsigned nwg = gridDim.x, g = blockIdx.x & 7, n_groups = nwg < 8 ? nwg : 8, per = (nwg - g + 7) >> 3;
            const unsigned old = __hip_atomic_fetch_add(ctr + 32 * (1 + g), 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (old + 1 == round * per) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const long long t0 = wall_clock64();
            unsigned spins = 0;
            while ((int)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - round * n_groups) < 0) {
                __builtin_amdgcn_s_sleep(1);
                if ((++spins & 63) == 0 &&
                    (wall_clock64() - t0 > kBarrierTimeoutTicks || __hip_atomic_load(ctr + 16, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0)) {
                    __hip_atomic_store(ctr + 16, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    __hip_atomic_store(abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_SYSTEM);
                    *ok = 0;
                    break;
                }
            }
            if (acquire) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        __syncthreads();
        if (tid < 64) pre();
        return *ok != 0;
    }
};

template <int DH>
union FusedLds {
    GemmLds gemm;
    AttnMfmaLds<DH> attn;
};

// NCHMAX: see gemm_stationary (2 covers d_model <= 4096, 3 covers d_model <= 5120)
template <int DH, int NCHMAX>
__global__ void __launch_bounds__(kFusedThreads) k_layer_fused(FusedArgs f0) {
    warm_kernel_args<sizeof(FusedArgs)>();
    constexpr int CH = 8, U = 8, NW = kFusedThreads / 64;
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    FusedLds<DH> &L = *reinterpret_cast<FusedLds<DH> *>(lds_raw);
    __shared__ int bar_ok;
    const int wg = blockIdx.x, nwg = gridDim.x;
    if (threadIdx.x == 0) bar_ok = 1;
    GridBarrier bar{f0.ctr, f0.round0, f0.abort_flag, &bar_ok};
    // optional trace: wall-clock ticks of this workgroup at the start, and before and after every barrier
    int n_stamp = 0;
    auto stamp = [&]() {
        if (f0.trace && threadIdx.x == 0) f0.trace[(size_t)wg * kFusedTraceStamps + n_stamp] = wall_clock64();
        ++n_stamp;
    };

    StatStream<1, CH> s_qkv;   // the only weight stream that is in flight from one layer to the next
    // the layer's weights, norm weights and cache: those of the first layer moved on by these many bytes
    long long w_off = 0, kv_off = 0;
    s_qkv.init(f0.qkv, wg, f0.nwg_qkv);
    // The arguments are read through a pointer to the argument block that is renewed in every turn of the layer loop:
    // each phase then fetches the fields it needs where it needs them, as in straight-line code (fetched once ahead
    // of the loop, the few hundred words would have to be kept in registers across all phases).
    typedef const __attribute__((address_space(4))) FusedArgs *ArgBlock;
    ArgBlock fp = (ArgBlock)__builtin_amdgcn_kernarg_segment_ptr();   // f0 is the only argument: it starts the block

    for (int l = 0;; ++l) {
        asm volatile("" : "+s"(fp));
        const FusedArgs &f = *(const FusedArgs *)fp;
        StatStream<1, CH> s_gu;
        StreamStream<1, U, NW> s_wo, s_down;
        n_stamp = 0;
        stamp();
        // ---- 1. q, k, v = W (RMSNorm(x)) -----------------------------------------------------------------
        AttnKv<DH> kv;
        auto pre_attn = [&]() { attn_load_kv<DH, kFusedThreads>(f.attn, wg, kv, kv_off); };   // the cached K/V block of the first item
        if (wg < f.nwg_qkv) {
            // first layer: x was written before the launch and is requested ahead of the weights; later layers: the
            // weights went in flight at the barrier that made x visible
            if (l == 0) gemm_stationary<1, CH, NCHMAX, IoAcquired, EPI_STORE, false, false>(f.qkv, s_qkv, L.gemm, NoTail(), w_off);
            else gemm_stationary<1, CH, NCHMAX, IoAcquired, EPI_STORE, false, true>(f.qkv_next, s_qkv, L.gemm, NoTail(), w_off);
        }
        stamp();
        forget(kv.k);
        forget(kv.v);
        if (!bar.sync(false, pre_attn)) return;
        stamp();

        // ---- 2. rotary embedding, KV append, attention partials ----------------------------------------------
        attn_mfma_items<DH, kFusedThreads, IoAgent, false>(f.attn, L.attn, wg, nwg, kv, true, kv_off);
        stamp();
        if (!bar.sync(false, NoTail())) return;
        stamp();

        // ---- 3. fold the splits of each query row (one wavefront per row), packed for Wo -----------------------
        for (int row = (thread_index() >> 6) * nwg + wg; row < f.attn.Hq * f.attn.m; row += NW * nwg) attn_combine_row<IoAgent, false>(f.attn, row);
        s_wo.init(f.wo, wg, f.nwg_wo);
        auto pre_wo = [&]() { s_wo.prefetch(f.wo, w_off); };
        stamp();
        forget(s_wo.a0);
        forget(s_wo.a1);
        if (!bar.sync(true, pre_wo)) return;
        stamp();

        // ---- 4. x' = x + Wo o ----------------------------------------------------------------------------------
        s_gu.init(f.gu, wg, f.nwg_gu, w_off);
        auto pre_gu = [&]() { s_gu.prefetch(); };
        if (wg < f.nwg_wo) gemm_streamed<1, U, NW, IoAcquired, EPI_RESID, true, false>(f.wo, s_wo, L.gemm, NoTail(), w_off);
        stamp();
        forget(s_gu.a0);
        forget(s_gu.a1);
        if (!bar.sync(true, pre_gu)) return;
        stamp();

        // ---- 5. g = silu(Wg b) * (Wu b), b = RMSNorm(x') ---------------------------------------------------------
        s_down.init(f.down_last, wg, f.nwg_down);
        auto pre_down = [&]() { s_down.prefetch(f.down_last, w_off); };
        if (wg < f.nwg_gu) gemm_stationary<1, CH, NCHMAX, IoAcquired, EPI_SWIGLU, false, true>(f.gu, s_gu, L.gemm, NoTail(), w_off);
        stamp();
        forget(s_down.a0);
        forget(s_down.a1);
        if (!bar.sync(true, pre_down)) return;
        stamp();

        // ---- 6. y = x' + Wd g --------------------------------------------------------------------------------------
        // (a layer that is followed by another also leaves that layer's QKV input behind, packed)
        const bool more = l + 1 < f.n_layers;
        if (wg < f.nwg_down) gemm_streamed<1, U, NW, IoAcquired, EPI_RESID, true, false>(more ? f.down : f.down_last, s_down, L.gemm, NoTail(), w_off);
        stamp();
        if (!more) break;

        // ---- next layer: same rows, the next layer's weights and cache ------------------------------------------------
        w_off += f.w_stride;
        kv_off += f.kv_stride;
        // (a stream object of its own: filled under conditions, s_qkv itself would have to keep its old registers
        // alive through all phases)
        StatStream<1, CH> s_next;
        s_next.init(f.qkv, wg, f.nwg_qkv, w_off);
        auto pre_qkv = [&]() { s_next.prefetch(); };
        forget(s_next.a0);
        forget(s_next.a1);
        if (!bar.sync(true, pre_qkv)) return;
        s_qkv = s_next;
    }
}

template <int DH, int NCHMAX>
static int launch_fused_dh(const FusedArgs &f, const LaunchCtx &c) {
    const size_t lds = sizeof(FusedLds<DH>);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k_layer_fused<DH, NCHMAX>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        attr_set = true;
    }
    hipLaunchKernelGGL((k_layer_fused<DH, NCHMAX>), dim3(c.n_wg), dim3(kFusedThreads), lds, (hipStream_t)c.stream, f);
    return (int)hipGetLastError();
}

int fused_phase_workgroups(int n_tiles, int n_wg) {
    const int per = (n_tiles + n_wg - 1) / n_wg;
    return per < 1 ? 1 : (n_tiles + per - 1) / per;
}

int launch_layer_fused(const FusedArgs &f_in, const LaunchCtx &c) {
    FusedArgs f = f_in;
    set_tile_partition(f.qkv, f.nwg_qkv);
    set_tile_partition(f.qkv_next, f.nwg_qkv);
    set_tile_partition(f.down_last, f.nwg_down);
    set_tile_partition(f.wo, f.nwg_wo);
    set_tile_partition(f.gu, f.nwg_gu);
    set_tile_partition(f.down, f.nwg_down);
    if (f.qkv.mode != GEMM_STATIONARY || f.gu.mode != GEMM_STATIONARY) return (int)hipErrorInvalidValue;
    // the streamed phases run a single round of at most 8 row tiles per workgroup
    if (f.wo.NT > 8 * f.nwg_wo || f.down.NT > 8 * f.nwg_down) return (int)hipErrorInvalidValue;
    if ((f.qkv.KT + kStatWaves - 1) / kStatWaves > kKsMax || f.qkv.K < 8) return (int)hipErrorInvalidValue;
    if (f.attn.kv_elem != kElemBF16 || f.qkv.elem != kElemBF16 || c.n_wg < 1 || f.n_layers < 1) return (int)hipErrorInvalidValue;
    const bool small = (f.qkv.KT + kStatWaves - 1) / kStatWaves <= 16;
    if (f.attn.dh == 128) return small ? launch_fused_dh<128, 2>(f, c) : launch_fused_dh<128, 3>(f, c);
    if (f.attn.dh == 64) return small ? launch_fused_dh<64, 2>(f, c) : launch_fused_dh<64, 3>(f, c);
    return (int)hipErrorInvalidValue;
}

}  // namespace ad
