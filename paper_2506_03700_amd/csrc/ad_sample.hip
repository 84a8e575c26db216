// Sampled decoding (Sec. 2.2 of arxiv 2506.03700): the token of Eq. 1 drawn from softmax(z / T), and the
// verification of Eq. 2 in its general form -- a drafted token t survives with probability
// min(1, p*(t) / p_draft(t)); the first rejected draft is replaced by a draw from
// Normalize(max(0, p* - p_draft)); if none is rejected the next token is drawn from the newest row's p*.
//
// Every draw is a uniform number u in [0, 1) handed in by the caller and turned into a token by inversion of
// the cumulative distribution in token-id order: the first id whose cumulative weight exceeds u * (total
// weight).  The vocabulary rows are small (V * 4 bytes, read from L2), so one workgroup of 1024 threads per
// row is enough: thread t owns the contiguous ids [t * seg, (t + 1) * seg), adds their weights up in id order,
// a fixed-order scan over the threads gives each thread the cumulative weight before its segment, and the
// thread whose segment contains the target walks it.  Everything is deterministic (no float atomics).
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "ad_internal.h"

namespace ad {

namespace {

constexpr int kSampleThreads = 1024;
constexpr int kSampleWaves = kSampleThreads / 64;

struct SampleLds {
    float wave_val[kSampleWaves];
    float bcast[4];
    int best;
    int last_pos;
};

// max over the workgroup, returned to every thread
__device__ __forceinline__ float block_max(float v, SampleLds &L) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) L.wave_val[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = L.wave_val[0];
#pragma unroll
    for (int w = 1; w < kSampleWaves; ++w) r = fmaxf(r, L.wave_val[w]);
    return r;
}

// Exclusive prefix of `local` over the threads in thread order (fixed association: butterfly-free scan inside a
// wavefront, then the wavefront totals in order); *total receives the sum over the workgroup.
__device__ __forceinline__ float block_exclusive_scan(float local, SampleLds &L, float *total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float incl = local;
    for (int off = 1; off < 64; off <<= 1) {
        const float up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    __syncthreads();
    if (lane == 63) L.wave_val[wave] = incl;
    __syncthreads();
    float before = 0.f, all = 0.f;
#pragma unroll
    for (int w = 0; w < kSampleWaves; ++w) {
        if (w < wave) before += L.wave_val[w];
        all += L.wave_val[w];
    }
    *total = all;
    return before + (incl - local);
}

// (max z, sum exp((z - max) * inv_t)) of one row, to every thread
__device__ __forceinline__ void row_stats(const float *z, int V, float inv_t, SampleLds &L, float *mx, float *sum) {
    float m = -INFINITY;
    for (int j = threadIdx.x; j < V; j += kSampleThreads) m = fmaxf(m, z[j]);
    m = block_max(m, L);
    float s = 0.f;
    for (int j = threadIdx.x; j < V; j += kSampleThreads) s += expf((z[j] - m) * inv_t);
    float total;
    (void)block_exclusive_scan(s, L, &total);
    *mx = m;
    *sum = total;
}

// Inversion draw over weights w(j) >= 0, j in [0, V).  Returns (to every thread) the token, its weight and the
// total weight.  A total of zero returns token -1.
template <class W>
__device__ __forceinline__ int sample_inverse(W w, int V, float u, SampleLds &L, float *w_tok, float *total_out) {
    const int seg = (V + kSampleThreads - 1) / kSampleThreads;
    const int j0 = min(V, (int)threadIdx.x * seg), j1 = min(V, j0 + seg);
    float local = 0.f;
    int last = -1;
    for (int j = j0; j < j1; ++j) {
        const float x = w(j);
        local += x;
        if (x > 0.f) last = j;
    }
    float total;
    const float before = block_exclusive_scan(local, L, &total);
    if (threadIdx.x == 0) {
        L.best = 0x7fffffff;
        L.last_pos = -1;
    }
    __syncthreads();
    const float target = u * total;
    // the first id of this segment that has weight and whose cumulative weight exceeds the target, if any; the
    // lowest over all threads wins (threads past the target report their first id of positive weight)
    if (before + local > target || before > target) {
        float c = before;
        for (int j = j0; j < j1; ++j) {
            const float x = w(j);
            c += x;
            if (c > target && x > 0.f) {
                atomicMin(&L.best, j);
                break;
            }
        }
    }
    if (last >= 0) atomicMax(&L.last_pos, last);
    __syncthreads();
    // rounding can leave no id above the target (u * total == total): the last id of positive weight
    const int tok = (L.best != 0x7fffffff) ? L.best : L.last_pos;
    if (tok >= j0 && tok < j1) L.bcast[0] = w(tok);
    __syncthreads();
    *w_tok = tok >= 0 ? L.bcast[0] : 0.f;
    *total_out = total;
    return tok;
}

struct SoftmaxWeight {
    const float *z; float mx, inv_t;
    __device__ __forceinline__ float operator()(int j) const { return expf((z[j] - mx) * inv_t); }
};

// max(0, p*(j) - p_draft(j)) up to a common factor, from the log-probabilities a = log p*(j), b = log p_draft(j):
// exp(a - c) * (1 - exp(b - a)) where a > b, with c = the largest such a.  Working relative to c keeps the weights
// in range when every token on which p* exceeds p_draft has a probability far below the smallest fp32 number
// (a dominant token that both distributions agree on leaves exactly that), and 1 - exp(b - a) through expm1 keeps
// the difference of two nearly equal probabilities accurate.
struct ResidualWeight {
    const float *zf, *zq; float mf, lsf, mq, lsq, inv_t, c;
    __device__ __forceinline__ float log_p(int j) const { return (zf[j] - mf) * inv_t - lsf; }
    __device__ __forceinline__ float log_q(int j) const { return (zq[j] - mq) * inv_t - lsq; }
    __device__ __forceinline__ float operator()(int j) const {
        const float a = log_p(j), b = log_q(j);
        return a > b ? expf(a - c) * -expm1f(b - a) : 0.f;
    }
};

__global__ void __launch_bounds__(kSampleThreads) k_sample_row(SampleArgs a) {
    __shared__ SampleLds L;
    float mx, sum;
    row_stats(a.z, a.V, a.inv_t, L, &mx, &sum);
    float w_tok, total;
    const int tok = sample_inverse(SoftmaxWeight{a.z, mx, a.inv_t}, a.V, a.u, L, &w_tok, &total);
    if (threadIdx.x == 0) {
        *a.tok_out = tok;
        *a.prob_out = w_tok / total;
    }
}

// One workgroup per row: rows [0, m) are the final logits, rows [m, 2m - 1) the draft logits.
__global__ void __launch_bounds__(kSampleThreads) k_row_stats(VerifySampledArgs a) {
    __shared__ SampleLds L;
    const int r = blockIdx.x;
    const float *z = r < a.m ? a.zf + (size_t)r * a.V : a.zq + (size_t)(r - a.m) * a.V;
    float mx, sum;
    row_stats(z, a.V, a.inv_t, L, &mx, &sum);
    if (threadIdx.x == 0) {
        a.stats[2 * r] = mx;
        a.stats[2 * r + 1] = sum;
    }
}

__global__ void __launch_bounds__(kSampleThreads) k_verify_sampled(VerifySampledArgs a) {
    __shared__ SampleLds L;
    __shared__ int s_nacc, s_rejected;
    const int n_draft = a.m - 1;
    if (threadIdx.x == 0) {
        int nacc = n_draft, rejected = 0;
        for (int k = 0; k < n_draft; ++k) {
            float ratio = 0.f;
            if (!rejected) {
                const int t = a.draft[k];
                // p*(t) / p_draft(t) through the logarithms, so that two tiny probabilities still have a ratio
                const float lp = (a.zf[(size_t)k * a.V + t] - a.stats[2 * k]) * a.inv_t - logf(a.stats[2 * k + 1]);
                const float lq = (a.zq[(size_t)k * a.V + t] - a.stats[2 * (a.m + k)]) * a.inv_t - logf(a.stats[2 * (a.m + k) + 1]);
                ratio = expf(lp - lq);
                if (!(a.u_accept[k] < fminf(1.0f, ratio))) {
                    rejected = 1;
                    nacc = k;
                }
            }
            if (a.ratio_out) a.ratio_out[k] = ratio;
        }
        s_nacc = nacc;
        s_rejected = rejected;
    }
    __syncthreads();
    const int r = s_nacc;
    const float *zf = a.zf + (size_t)r * a.V;
    const float mf = a.stats[2 * r], sf = a.stats[2 * r + 1];
    int tok = -1;
    float w_tok, total;
    if (s_rejected) {
        const float *zq = a.zq + (size_t)r * a.V;
        ResidualWeight w{zf, zq, mf, logf(sf), a.stats[2 * (a.m + r)], logf(a.stats[2 * (a.m + r) + 1]), a.inv_t, 0.f};
        float c = -INFINITY;
        for (int j = threadIdx.x; j < a.V; j += kSampleThreads) {
            const float la = w.log_p(j);
            if (la > w.log_q(j)) c = fmaxf(c, la);
        }
        w.c = block_max(c, L);
        if (w.c != -INFINITY) tok = sample_inverse(w, a.V, a.u_resample[r], L, &w_tok, &total);
        __syncthreads();
    }
    if (tok < 0)       // nothing rejected (or a residual that is identically zero): draw from the row's final distribution
        tok = sample_inverse(SoftmaxWeight{zf, mf, a.inv_t}, a.V, s_rejected ? a.u_resample[r] : a.u_final, L, &w_tok, &total);
    if (threadIdx.x == 0) {
        *a.n_accept_out = r;
        *a.next_out = tok;
    }
}

}  // namespace

int launch_sample_row(const SampleArgs &a, void *stream) {
    if (a.V < 1 || !(a.inv_t > 0.f)) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(k_sample_row, dim3(1), dim3(kSampleThreads), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

int launch_verify_sampled(const VerifySampledArgs &a, void *stream) {
    if (a.V < 1 || a.m < 1 || a.m > 8 || !(a.inv_t > 0.f)) return (int)hipErrorInvalidValue;
    for (int k = 0; k + 1 < a.m; ++k)
        if (a.draft[k] < 0 || a.draft[k] >= a.V) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(k_row_stats, dim3(2 * a.m - 1), dim3(kSampleThreads), 0, (hipStream_t)stream, a);
    int rc = (int)hipGetLastError();
    if (rc) return rc;
    hipLaunchKernelGGL(k_verify_sampled, dim3(1), dim3(kSampleThreads), 0, (hipStream_t)stream, a);
    return (int)hipGetLastError();
}

}  // namespace ad
