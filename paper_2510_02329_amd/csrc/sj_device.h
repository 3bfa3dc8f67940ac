// Device-side building blocks: storage types, 16-byte MFMA operand fragments, wave helpers.
//
// All matrix work uses the 16x16 MFMA shapes of CDNA4 with one common operand convention:
// for a tile product D[16x16] += A[16 x KSTEP] * B[16 x KSTEP]^T, lane l = 16*g + r holds the
// 16 bytes A[r][g*KF .. g*KF+KF) (and likewise for B), KF = elements per 16 bytes, KSTEP = 4*KF.
// After the product lane l holds D[4g+i][r] in accumulator element i (i = 0..3).
//   bf16: KF = 8, one v_mfma_f32_16x16x32_bf16 per fragment pair.
//   fp32: KF = 4, four v_mfma_f32_16x16x4_f32 (element i of both fragments feeds product i), so
//         the contraction covers the same 16 k-values in a different order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sj {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint16_t bf16_t;   // storage: bf16 bit pattern

union Frag {
    u32x4 u;
    f32x4 f;
    bf16x8 h;
    uint16_t s[8];
};

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);      // round to nearest even (finite inputs)
    return (bf16_t)(u >> 16);
}

template <typename T> struct Traits;

template <> struct Traits<float> {
    static constexpr int KF = 4;
    static constexpr int KSTEP = 16;
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.f[i], b.f[i], c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
    // packs 4*KF/4.. probabilities of one lane into a B fragment: fp32 takes 4 values
    static __device__ __forceinline__ void pack(Frag& f, int j, float v) { f.f[j] = v; }
};

template <> struct Traits<bf16_t> {
    static constexpr int KF = 8;
    static constexpr int KSTEP = 32;
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.h, b.h, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void pack(Frag& f, int j, float v) { f.s[j] = f32_to_bf16(v); }
};

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// Sum over a 256-thread block; every thread gets the result.  Fixed order -> deterministic.
__device__ __forceinline__ float block_sum_256(float v, float* lds4) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds4[w] = v;
    __syncthreads();
    return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}
__device__ __forceinline__ double block_sum_256(double v, double* lds4) {
    v = wave_sum(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds4[w] = v;
    __syncthreads();
    return (lds4[0] + lds4[1]) + (lds4[2] + lds4[3]);
}

}  // namespace sj
