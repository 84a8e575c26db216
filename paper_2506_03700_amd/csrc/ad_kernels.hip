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

#include "ad_device.h"
#include "ad_internal.h"

namespace ad {

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
    const int groups = a.d / 8;       // one thread per (token, 8 consecutive inputs): two 128-bit stores
    const int work = groups * a.m;
    const int rounds = (work + gsize - 1) / gsize;
    for (int it = 0; it < rounds; ++it) {
        const int idx = gtid + it * gsize;
        float s = 0.0f;
        if (idx < work) {
            const int t = idx / groups, c = idx % groups;
            const f32x4 x0 = *(const f32x4 *)(a.x + (size_t)t * a.d + c * 8), x1 = *(const f32x4 *)(a.x + (size_t)t * a.d + c * 8 + 4);
            union { u32x4 v; uint16_t u[8]; } hi, lo;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = e < 4 ? x0[e] : x1[e - 4];
                s += v * v;
                split_hi_lo(v * load_w(a.norm_w, a.norm_is_bf16, (size_t)c * 8 + e), hi.u[e], lo.u[e]);
            }
            uint16_t *B = (uint16_t *)a.B;
            *(u32x4 *)(B + act_index(c * 8, t)) = hi.v;
            *(u32x4 *)(B + act_index(c * 8, 8 + t)) = lo.v;
        }
        // ssq is kept per 16 inputs (the row-tile granularity of the GEMM epilogues): pairs of lanes
        const float s2 = s + __shfl_xor(s, 1);
        if (idx < work && (idx % groups) % 2 == 0) a.ssq[((idx % groups) / 2) * 8 + idx / groups] = s2;
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

    // every workgroup publishes its per-token partial; k_head_combine folds them
    if (tid < g.m) {
        float *p = g.head_part + ((size_t)wg * 8 + tid) * 4;
        p[0] = L.run_max[tid];
        p[1] = L.run_sum[tid];
        p[2] = __int_as_float(L.run_idx[tid]);
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
}

template <int NPL, int U>
__global__ void __launch_bounds__(kThreads) k_gemm(GemmArgs g) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    gemm_phase<NPL, U>(g, blockIdx.x, gridDim.x, *reinterpret_cast<GemmLds *>(lds_raw));
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
    const int work = (a.d / 8) * a.m;
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
    if (g.epi == EPI_HEAD) {
        GemmArgs h = g;
        h.n_parts = grid;
        hipLaunchKernelGGL(k_head_combine, dim3(1), dim3(512), 0, S(c.stream), h);
    }
    return (int)hipGetLastError();
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
