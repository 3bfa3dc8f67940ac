// Device-side building blocks: storage types, 16-byte MFMA operand fragments, wave helpers.
//
// All matrix work uses the 16x16 MFMA shapes of CDNA4 with one common operand convention:
// for a tile product D[16x16] += A[16 x KSTEP] * B[16 x KSTEP]^T, lane l = 16*g + r holds the
// 16 bytes A[r][g*KF .. g*KF+KF) (and likewise for B), KF = elements per 16 bytes, KSTEP = 4*KF.
// After the product lane l holds D[4g+i][r] in accumulator element i (i = 0..3).
//   bf16: KF = 8, one v_mfma_f32_16x16x32_bf16 per fragment pair.
//   fp32: KF = 4, four v_mfma_f32_16x16x4_f32 (element i of both fragments feeds product i), so
//         the contraction covers the same 16 k-values in a different order.
//
// Activations (the few-row operand) are fp32 values.  In bf16 mode they are written as three bf16
// planes (hi = bf16(x), mid = bf16(x - hi), lo = x - hi - mid, together all 24 significant bits)
// and a kernel multiplies the first SPL of them by the same weight fragment, accumulating in fp32:
// SPL = 1 is plain bf16 rounding (2^-9), SPL = 2 carries 16 bits (2^-18), SPL = 3 is exact.
// Only the weights and the cache are bf16.  Rounding every GEMM input to bf16 leaves the logits
// of a 32-layer decoder outside the parity bar against an fp64 reference; two planes are well
// inside it.  The weight stream from HBM - the bound of this path - is unchanged; the matrix cores
// have the headroom for the extra products.
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
// round to nearest even: the hardware conversion of gfx950 (v_cvt_pk_bf16_f32)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    const __bf16 b = (__bf16)f;
    return __builtin_bit_cast(bf16_t, b);
}

template <typename T> struct Traits;

template <> struct Traits<float> {
    static constexpr int KF = 4;
    static constexpr int KSTEP = 16;
    static constexpr int NS = 1;          // activation planes: fp32 operands are exact
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& c) {
#pragma unroll
        for (int i = 0; i < 4; ++i) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a.f[i], b.f[i], c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const float* p) { return *p; }
    static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
    // packs 4*KF/4.. probabilities of one lane into a B fragment: fp32 takes 4 values
    static __device__ __forceinline__ void pack(Frag& f, int j, float v) { f.f[j] = v; }
    template <int SPL> static __device__ __forceinline__ void pack_split(Frag* f, int j, float v) { f[0].f[j] = v; }
    static __device__ __forceinline__ void store_split(float* p, size_t, float v) { *p = v; }
    // four neighbouring values (p 16-byte aligned)
    static __device__ __forceinline__ void store_split4(float* p, size_t, const float (&v)[4]) {
        *reinterpret_cast<float4*>(p) = float4{v[0], v[1], v[2], v[3]};
    }
};

template <> struct Traits<bf16_t> {
    static constexpr int KF = 8;
    static constexpr int KSTEP = 32;
    static constexpr int NS = 3;          // fp32 activations are carried as three bf16 planes
    static __device__ __forceinline__ void mma(const Frag& a, const Frag& b, f32x4& c) {
        c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a.h, b.h, c, 0, 0, 0);
    }
    static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
    static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
    static __device__ __forceinline__ void pack(Frag& f, int j, float v) { f.s[j] = f32_to_bf16(v); }
    // v = hi + mid + lo exactly: each part takes the next 8 significant bits of the fp32 value
    template <int SPL> static __device__ __forceinline__ void pack_split(Frag* f, int j, float v) {
        const bf16_t h = f32_to_bf16(v);
        f[0].s[j] = h;
        if constexpr (SPL >= 2) {
            const float r1 = v - bf16_to_f32(h);
            const bf16_t m = f32_to_bf16(r1);
            f[1].s[j] = m;
            if constexpr (SPL >= 3) f[2].s[j] = f32_to_bf16(r1 - bf16_to_f32(m));
        }
    }
    static __device__ __forceinline__ void store_split(bf16_t* p, size_t plane, float v) {
        const bf16_t h = f32_to_bf16(v);
        const float r1 = v - bf16_to_f32(h);
        const bf16_t m = f32_to_bf16(r1);
        p[0] = h;
        p[plane] = m;
        p[2 * plane] = f32_to_bf16(r1 - bf16_to_f32(m));
    }
    // four neighbouring values (p 8-byte aligned): one 8-byte store per plane
    static __device__ __forceinline__ void store_split4(bf16_t* p, size_t plane, const float (&v)[4]) {
        bf16_t h[4], m[4], l[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            h[i] = f32_to_bf16(v[i]);
            const float r1 = v[i] - bf16_to_f32(h[i]);
            m[i] = f32_to_bf16(r1);
            l[i] = f32_to_bf16(r1 - bf16_to_f32(m[i]));
        }
        auto pack = [](const bf16_t (&x)[4]) { return uint2{(uint32_t)x[0] | ((uint32_t)x[1] << 16), (uint32_t)x[2] | ((uint32_t)x[3] << 16)}; };
        *reinterpret_cast<uint2*>(p) = pack(h);
        *reinterpret_cast<uint2*>(p + plane) = pack(m);
        *reinterpret_cast<uint2*>(p + 2 * plane) = pack(l);
    }
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

// ---- coherent accessors (agent scope: write-through / cache-bypassing single accesses) ----------
__device__ __forceinline__ void st_coh(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(unsigned* p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(unsigned long long* p, unsigned long long v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_coh(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_coh(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// Element offset of operand element (row, k) inside one plane.  tks == 0: row-major with leading dimension ld.
// tks > 0 (= K / KSTEP): the plane is stored in blocks of one MFMA fragment, [row tile][k-step][16 rows][KSTEP
// elements]: the 1 KB that the many-row GEMM moves into LDS with one load instruction is consecutive memory (lane
// 16 g + r of that load reads the 16 bytes at row r, element g * KF of the block), where a row-major fragment
// touches 16 cache lines and uses half of each; a producer still writes a row's KSTEP elements contiguously.
template <typename T>
__device__ __forceinline__ size_t opnd_off(int row, int k, int ld, int tks) {
    constexpr int KSTEP = Traits<T>::KSTEP;
    if (tks == 0) return (size_t)row * ld + k;
    return (((size_t)(row >> 4) * tks + k / KSTEP) * 16 + (row & 15)) * KSTEP + (k % KSTEP);
}

// Workgroup barrier that waits for this wave's LDS traffic only.  __syncthreads() also waits for every
// outstanding global load (its fence drains the vector-memory counter), which would empty a prefetch
// pipeline at each barrier; kernels that keep loads in flight across barriers order LDS themselves: data
// written by direct global->LDS loads is covered by an explicit vmcnt wait of the loading wave.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ void wait_vm0() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// immediate of s_waitcnt vmcnt(n) with the other counters left alone (vmcnt sits in bits 3:0 and 15:14)
constexpr int vmcnt_imm(int n) { return (n & 15) | ((n >> 4) << 14) | (7 << 4) | (15 << 8); }

}  // namespace sj
