// Device-side helpers shared by the library's kernels: vector types, bf16 conversion, and the index
// function of the packed activation layout (see ad_internal.h).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ad {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;   // also carries 8 fp16 values (see mma16)
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

// ---------------------------------------------------------------------------------------------------
// small helpers
// ---------------------------------------------------------------------------------------------------
__device__ __forceinline__ float bf16_bits_to_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }

// round-to-nearest-even fp32 -> bf16 bits (finite inputs)
__device__ __forceinline__ uint16_t f32_to_bf16_bits(float x) {
    uint32_t u = __float_as_uint(x);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// IEEE half precision <-> fp32 (the conversion instruction rounds to nearest even)
__device__ __forceinline__ float f16_bits_to_f32(uint16_t b) { return (float)__builtin_bit_cast(_Float16, b); }
__device__ __forceinline__ uint16_t f32_to_f16_bits(float x) { return __builtin_bit_cast(uint16_t, (_Float16)x); }

// Kernel arguments are fetched with scalar loads that the compiler places where each field is first used; every
// 64-byte line of the argument block that is touched for the first time costs a trip to memory, and those trips
// come one after the other on the path to the kernel's first useful load.  Reading one word of every line of the
// block at the kernel's entry (and waiting for them together) overlaps them all: later argument loads hit in the
// scalar cache.  BYTES: the size of the kernel's explicit arguments; nothing beyond them is read.
// threadIdx.x as a value the compiler computes afresh at every call.  The phases of a kernel that loops over layers
// derive their lane-dependent addresses from it: derived from threadIdx.x itself they would all count as loop
// invariants, be computed ahead of the loop and be kept in registers (spilled, there are hundreds) through every phase.
__device__ __forceinline__ int thread_index() {
    int t = (int)threadIdx.x;
    asm volatile("" : "+v"(t));
    return t;
}

// Declares the registers of an array to hold nothing that is still needed (no instruction is emitted).  Inside a
// loop, an array that is only filled under a condition would otherwise carry its contents of the previous turn
// all the way round the loop.
template <class T, int A>
__device__ __forceinline__ void forget(T (&r)[A]) {
#pragma unroll
    for (int i = 0; i < A; ++i) asm volatile("" : "=v"(r[i]));
}
template <class T, int A, int B>
__device__ __forceinline__ void forget(T (&r)[A][B]) {
#pragma unroll
    for (int i = 0; i < A; ++i) forget(r[i]);
}

template <int BYTES>
__device__ __forceinline__ void warm_kernel_args() {
    typedef const __attribute__((address_space(4))) uint32_t *kptr;
    kptr p = (kptr)__builtin_amdgcn_kernarg_segment_ptr();
    constexpr int LINES = (BYTES + 63) / 64;
    uint32_t v[LINES];
#pragma unroll
    for (int i = 0; i < LINES; ++i) v[i] = p[i * 16 < BYTES / 4 ? i * 16 : BYTES / 4 - 1];
#pragma unroll
    for (int i = 0; i < LINES; ++i) asm volatile("" ::"s"(v[i]));
}

// Element kinds of stored tensors (weights, norm vectors, embedding table, KV cache).  16-bit activations use
// the same type as the weights they meet in an MFMA: bf16 for fp32 and bf16 models, fp16 for fp16 models.
enum ElemKind : int { ELEM_F32 = 0, ELEM_BF16 = 1, ELEM_F16 = 2 };

// x = hi + lo with hi, lo in the 16-bit type (F16: half precision, else bf16)
template <bool F16>
__device__ __forceinline__ void split_hi_lo(float x, uint16_t &hi, uint16_t &lo) {
    if constexpr (F16) {
        hi = f32_to_f16_bits(x);
        lo = f32_to_f16_bits(x - f16_bits_to_f32(hi));
    } else {
        hi = f32_to_bf16_bits(x);
        lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
    }
}

template <bool F16>
__device__ __forceinline__ uint16_t f32_to_16(float x) { return F16 ? f32_to_f16_bits(x) : f32_to_bf16_bits(x); }

// D += A (16 rows x 32) * B (32 x 16 columns), 16-bit operands of the model's type, fp32 accumulation
template <bool F16>
__device__ __forceinline__ f32x4 mma16(const bf16x8 &a, const bf16x8 &b, const f32x4 &c) {
    if constexpr (F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ float load_w(const void *p, int elem, size_t i) {
    if (elem == ELEM_F32) return ((const float *)p)[i];
    const uint16_t b = ((const uint16_t *)p)[i];
    return elem == ELEM_BF16 ? bf16_bits_to_f32(b) : f16_bits_to_f32(b);
}

// eight consecutive weights starting at element k (k a multiple of 8); a null vector means all ones
__device__ __forceinline__ void load_w8(const void *p, int elem, size_t k, float (&w)[8]) {
    if (!p) {
#pragma unroll
        for (int e = 0; e < 8; ++e) w[e] = 1.0f;
    } else if (elem == ELEM_BF16) {
        const u32x4 v = *(const u32x4 *)((const uint16_t *)p + k);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w[2 * e] = __uint_as_float(v[e] << 16);
            w[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
        }
    } else if (elem == ELEM_F16) {
        const u32x4 v = *(const u32x4 *)((const uint16_t *)p + k);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w[2 * e] = f16_bits_to_f32((uint16_t)(v[e] & 0xffffu));
            w[2 * e + 1] = f16_bits_to_f32((uint16_t)(v[e] >> 16));
        }
    } else {
        const f32x4 v0 = *(const f32x4 *)((const float *)p + k), v1 = *(const f32x4 *)((const float *)p + k + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            w[e] = v0[e];
            w[4 + e] = v1[e];
        }
    }
}

// v + (v of the lane 8 places away within its group of 16 lanes): the hi and lo columns of an MFMA result.
// A DPP row rotation by 8, so it costs one VALU instruction and no LDS traffic.
__device__ __forceinline__ float add_lane_xor8(float v) {
    const int o = __builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x128 /* row_ror:8 */, 0xf, 0xf, false);
    return v + __int_as_float(o);
}

// x / d for small non-negative x and d, with the multiplier the host derived from d (div_multiplier in ad_internal.h)
// (a multiplier of 0 stands for d == 1)
__device__ __forceinline__ int div_small(int x, unsigned mul) { return mul ? (int)__umulhi((unsigned)x, mul) : x; }

// index (in bf16 elements) of input k of column col (token col & 7, hi/lo part col >> 3) in a packed activation
// block of KT k-steps (see ad_internal.h)
__device__ __forceinline__ size_t act_index(int k, int col, int KT) {
    return ((((size_t)(col & 7) * KT + (k >> 5)) * 2 + (col >> 3)) * 4 + ((k & 31) >> 3)) * 8 + (k & 7);
}

// index (in 16-byte units) of the MFMA B operand register of lane `lane` for k-step ks of such a block
__device__ __forceinline__ size_t act_operand_index(int ks, int lane, int KT) {
    const int n = lane & 15;
    return (((size_t)(n & 7) * KT + ks) * 2 + (n >> 3)) * 4 + (lane >> 4);
}

}  // namespace ad
