// Few-row weight-streaming GEMM with the weights delivered through an LDS ring by loader waves:
// Y[R][N] = X[R][K] * W[N][K]^T, R <= 16, W in the re-tiled layout (paper: the projections of the target
// forward, Eq. 2 / Eq. 4).  Same arguments, grid meaning (x: groups of NT n-tiles, y: K-slices) and
// epilogues as gemm_skinny_kernel; it is a candidate launch shape that the start-up measurement may pick.
//
// Why a second kernel: in the register-ring kernel a wave alternates between requesting and consuming, and
// its requests are bounded by its registers.  Here two LOADER waves do nothing but issue direct
// global->LDS loads with the streaming cache policy, a ring of NSA stages of 8 KB ahead of the consumers
// (measured on this part: 7.2 TB/s sustained against 6.1 TB/s with the default policy and 7.0 TB/s for a
// plain read kernel), and eight COMPUTE waves read one 1 KB fragment each per stage.
//
// Stage = one n-tile x 8 consecutive k-steps = 8 KB of consecutive memory (the re-tiled layout keeps a
// tile's k-steps contiguous).  Compute wave w multiplies fragment w of every stage, i.e. k-steps
// ks0 + 8 kb + w of the slice: the waves interleave K, so the workgroup pulls one contiguous stream per
// tile, and a wave's operand fragment changes only every NT stages.  One LDS-only barrier per stage keeps
// loaders and consumers in lock step.  The 8 waves' accumulators meet in LDS (the ring's memory, free by
// then) and are added in wave order: deterministic.
//
// PACK (two operand planes, at most 8 rows): MFMA row r < 8 of the B operand carries plane 0 of row r,
// row r + 8 plane 1 of the same row, so ONE product per weight fragment yields both planes' contributions
// in output columns r and r + 8, which the reduction adds (hi first).  Without PACK one product per plane.
#pragma once
#include "sj_kernels.h"

namespace sj {

constexpr int RING_CW = 8;         // compute waves = fragments (k-steps) per stage
constexpr int RING_LW = 2;         // loader waves
constexpr int RING_THREADS = (RING_CW + RING_LW) * 64;

// the loader's last NSA - 1 iterations: iteration I may leave NSA - 3 - I stages of its loads in flight
template <int I, int NSA, int PER>
__device__ __forceinline__ void ring_tail_waits() {
    if constexpr (I < NSA - 1) {
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSA - 3 - I > 0 ? NSA - 3 - I : 0) * PER));
        lds_barrier();
        ring_tail_waits<I + 1, NSA, PER>();
    }
}

template <typename T, int NT, int EPI, int SPL, bool PACK, int NSA>
__global__ __launch_bounds__(RING_THREADS) void gemm_ring_kernel(GemmArgs a) {
    static_assert(!PACK || SPL == 2, "packing is for two planes");
    static_assert(NSA >= 3 && (NSA & (NSA - 1)) == 0, "ring depth: a power of two");
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    constexpr int PER = RING_CW / RING_LW;             // fragments per loader wave and stage
    constexpr int LDS_STAGES = NSA > NT ? NSA : NT;    // the reduction needs NT x 8 KB
    static_assert((NSA - 1) * PER < 64, "the load counter holds 63");
    __shared__ u32x4 ring[LDS_STAGES][RING_CW][64];
    const int lane = threadIdx.x & 63, w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int r = lane & 15, g = lane >> 4;
    const int KS = a.K / KSTEP;
    const int nt0 = blockIdx.x * NT;
    // K-slices of whole stages (the host launches this kernel only when KS / gridDim.y is a multiple of 8)
    const int nkb = KS / RING_CW / (int)gridDim.y;
    const int ks0 = blockIdx.y * nkb * RING_CW;
    const int nstages = nkb * NT;                      // >= NSA (host-checked)

    if (w >= RING_CW) {
        // ---------------- loader waves: stage s = (k-block s / NT, tile s % NT) -> buffer s % NSA ----------------
        const int lw = w - RING_CW;
        const char* src = reinterpret_cast<const char*>(a.Wt) + (((size_t)nt0 * KS + ks0 + lw * PER) * 64 + lane) * 16;
        const size_t tile_step = (size_t)KS * 1024;                   // next tile, same k-block
        const size_t kb_step = (size_t)RING_CW * 1024 - (size_t)(NT - 1) * tile_step;   // first tile of the next k-block
        int t = 0, buf = 0;
        auto issue = [&]() {
            u32x4* dst = &ring[buf][lw * PER][0];
#pragma unroll
            for (int j = 0; j < PER; ++j)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src + j * 1024),
                                                 (__attribute__((address_space(3))) void*)(dst + j * 64), 16, 0, 2);
            buf = (buf + 1) & (NSA - 1);
            if (++t == NT) { t = 0; src += kb_step; } else src += tile_step;
        };
#pragma unroll
        for (int s = 0; s < NSA - 1; ++s) issue();
        __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSA - 2) * PER));       // stage 0 has landed
        lds_barrier();
        // iteration s: buffer (s - 1) % NSA was read before the barrier that ended iteration s - 1
        for (int s = 0; s + NSA - 1 < nstages; ++s) {
            issue();
            __builtin_amdgcn_s_waitcnt(vmcnt_imm((NSA - 2) * PER));   // stage s + 1 has landed
            lds_barrier();
        }
        // everything is requested: the last NSA - 1 iterations only wait, for one stage less each
        ring_tail_waits<0, NSA, PER>();
        __syncthreads();                               // the reduction's barrier (every wave of the workgroup arrives)
        return;
    }

    // ---------------- compute waves ----------------
    constexpr int NB = PACK ? 1 : SPL;                 // operand fragments (products) per weight fragment
    const T* Xr[NB];
    if constexpr (PACK) {
        const int row = r & 7;
        Xr[0] = reinterpret_cast<const T*>(a.X) + (size_t)(r >> 3) * a.xplane + (size_t)(row < a.R ? row : 0) * a.ldx +
                (size_t)(ks0 + w) * KSTEP + g * KF;
    } else {
#pragma unroll
        for (int sp = 0; sp < NB; ++sp)
            Xr[sp] = reinterpret_cast<const T*>(a.X) + (size_t)sp * a.xplane + (size_t)(r < a.R ? r : 0) * a.ldx +
                     (size_t)(ks0 + w) * KSTEP + g * KF;
    }
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    Frag fb[NB], fbn[NB];
    auto load_b = [&](Frag (&f)[NB], int kb) {
#pragma unroll
        for (int sp = 0; sp < NB; ++sp) f[sp].u = *reinterpret_cast<const u32x4*>(Xr[sp] + (size_t)kb * (RING_CW * KSTEP));
    };
    load_b(fb, 0);
    lds_barrier();                                     // stage 0 is in LDS
    int buf = 0;
    for (int kb = 0; kb < nkb; ++kb) {
        load_b(fbn, min(kb + 1, nkb - 1));             // always issued: no load under a branch
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            Frag fa;
            fa.u = ring[buf][w][lane];
#pragma unroll
            for (int sp = 0; sp < NB; ++sp) Traits<T>::mma(fa, fb[sp], acc[t]);
            buf = (buf + 1) & (NSA - 1);
            lds_barrier();                             // this buffer is free; the next stage has landed
        }
#pragma unroll
        for (int sp = 0; sp < NB; ++sp) fb[sp] = fbn[sp];
    }

    // every stage has been read (last barrier above): the ring's memory now holds the 8 waves' accumulators,
    // red[w][t][row * 16 + n] with D[n = 4g + i][row = r] in lane 16g + r
    float* red = reinterpret_cast<float*>(&ring[0][0][0]);
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) red[(w * NT + t) * 256 + r * 16 + 4 * g + i] = acc[t][i];
    __syncthreads();
    if constexpr (EPI != EPI_LOGITS && NT <= RING_CW) {
        // One wave per tile, four neighbouring columns of a row per lane (lane l: row l / 4, columns 4 (l % 4) ..):
        // 16-byte LDS reads and 8- or 16-byte stores, seven waves at work instead of four threads' worth of scalar
        // reads per tile (the scalar form below took 2.9 us of the 39 us gate/up launch).  Same sums in the same order.
        if (w >= NT) return;
        const int t = w, row = lane >> 2, n0 = (lane & 3) * 4;
        auto sum_at = [&](int pos) {
            f32x4 sum = *reinterpret_cast<const f32x4*>(red + t * 256 + pos);
#pragma unroll
            for (int ww = 1; ww < RING_CW; ++ww) sum += *reinterpret_cast<const f32x4*>(red + (ww * NT + t) * 256 + pos);
            return sum;
        };
        f32x4 v = sum_at(lane * 4);
        if constexpr (PACK) v += sum_at(((lane + 32) & 63) * 4);   // the second plane's products sit 8 rows further on
        if constexpr (EPI == EPI_PARTIAL) {
            if (row < a.R)
                *reinterpret_cast<f32x4*>(a.out + ((size_t)blockIdx.y * a.slice_rows + row) * a.N + (size_t)(nt0 + t) * 16 + n0) = v;
        } else {
            // tile column n < 8 is gate of FFN column 8 * tile + n, column n + 8 its up projection: two lanes further on
            f32x4 up;
#pragma unroll
            for (int i = 0; i < 4; ++i) up[i] = __shfl_down(v[i], 2, 64);
            if (row < a.R && n0 < 8) {
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) y[i] = v[i] / (1.0f + expf(-v[i])) * up[i];
                Traits<T>::store_split4(reinterpret_cast<T*>(a.act) + (size_t)row * (a.N / 2) + (size_t)(nt0 + t) * 8 + n0, a.actplane, y);
            }
        }
        return;
    }
    if (threadIdx.x >= 256) return;
    const int tid = threadIdx.x, er = tid >> 4, en = tid & 15;
    float v[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        float sum = red[t * 256 + tid];
#pragma unroll
        for (int ww = 1; ww < RING_CW; ++ww) sum += red[(ww * NT + t) * 256 + tid];
        if constexpr (PACK) {
            // the second plane's products sit 8 rows further on (threads of rows >= 8 read in-bounds values they never store)
            const int o = (tid + 128) & 255;
            float lo = red[t * 256 + o];
#pragma unroll
            for (int ww = 1; ww < RING_CW; ++ww) lo += red[(ww * NT + t) * 256 + o];
            sum += lo;
        }
        v[t] = sum;
    }
    few_epilogue<T, NT, EPI>(a, v, er, en, nt0);
}

}  // namespace sj
