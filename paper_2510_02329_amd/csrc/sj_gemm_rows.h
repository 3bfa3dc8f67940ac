// Weight-streaming GEMM for more than one row tile (batched verification: R = batch * (gamma + 1)
// rows, up to 144 per launch): Y[R][N] = X[R][K] * W[N][K]^T with W in the re-tiled layout.
// Paper reference: the projections of the target forward, Eq. 2 / Eq. 4.
//
// With many rows the few-row kernel's scheme (every wave fetches its own operand fragments) turns the
// operand into the dominant traffic.  Here a workgroup is 4 waves that share ONE K-slice and own two
// n-tiles each: the operand fragments of a stage (KB k-steps, all row tiles, all planes) are staged
// once per workgroup in LDS in MFMA fragment order and read by all waves, while every wave streams
// its own weight tiles through registers.  Each weight byte is read once per launch; the row tiles
// live in the accumulators (2 x 9 tiles x 4 registers).  An operand fragment read from LDS feeds two
// products (one per n-tile of the wave): at 16 cycles per product and 128 bytes per cycle of LDS
// that is the ratio at which the LDS stops being the bound.  72 KB of LDS per workgroup lets two
// workgroups share a CU.  No cross-wave reduction is needed, so the epilogue runs straight from the
// accumulators.  Split-K across workgroups (gridDim.y slices, partials summed by the consumer in
// slice order) keeps the short projections on all CUs.
//
// MFMA convention as in the few-row kernel: A = weight fragment (rows = n), B = operand fragment
// (rows = m), lane 16g + r then holds D[n = 4g + i][m = r].
#pragma once
#include "sj_kernels.h"

namespace sj {

constexpr int ROWS_MT = 9;         // row tiles per launch (144 rows)
constexpr int ROWS_WAVES = 4;      // waves per workgroup
constexpr int ROWS_NTW = 2;        // n-tiles per wave
constexpr int ROWS_NT = ROWS_WAVES * ROWS_NTW;   // n-tiles per workgroup

template <typename T, int SPL> constexpr int rows_kb() { return 2; }   // k-steps per stage

template <typename T, int EPI, int SPL>
__global__ __launch_bounds__(ROWS_WAVES * 64) void gemm_rows_kernel(GemmArgs a, int mt) {
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    constexpr int KB = rows_kb<T, SPL>();
    constexpr int NTHR = ROWS_WAVES * 64;
    constexpr int XR = (SPL * ROWS_MT * 16 * KB * 4 + NTHR - 1) / NTHR;    // staged 16-byte granules per thread
    __shared__ u32x4 Bs[2][SPL][ROWS_MT][KB][64];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int KS = a.K / KSTEP, ntiles = a.N / 16;
    const int nt0 = (blockIdx.x * ROWS_WAVES + w) * ROWS_NTW;   // this wave's tiles nt0, nt0 + 1
    const bool live0 = nt0 < ntiles, live1 = nt0 + 1 < ntiles;  // a trailing workgroup may own fewer tiles
    const int ks0 = (int)((long long)blockIdx.y * KS / gridDim.y), ks1 = (int)((long long)(blockIdx.y + 1) * KS / gridDim.y);
    const int nks = ks1 - ks0, nstage = (nks + KB - 1) / KB;
    const u32x4* Wt0 = reinterpret_cast<const u32x4*>(a.Wt) + ((size_t)(live0 ? nt0 : 0) * KS + ks0) * 64 + lane;
    const u32x4* Wt1 = reinterpret_cast<const u32x4*>(a.Wt) + ((size_t)(live1 ? nt0 + 1 : 0) * KS + ks0) * 64 + lane;
    const int rows = mt * 16;
    const int ngran = SPL * rows * KB * 4;             // granules of one stage

    f32x4 acc[ROWS_NTW][ROWS_MT];
#pragma unroll
    for (int t = 0; t < ROWS_NTW; ++t)
#pragma unroll
        for (int m = 0; m < ROWS_MT; ++m) acc[t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

    // stage s covers k-steps [s*KB, s*KB + KB) of the slice; indices past the slice are clamped to its
    // last k-step (loaded again, multiplied never), so all loads are branch-free
    Frag wq[4][KB][ROWS_NTW];    // weight stages in flight: the one being multiplied + 3 ahead
    u32x4 xq[XR];
    // a thread stages the same granules (plane, row, k-step of the stage, 16-byte column) every stage:
    // source offset without the stage's k offset, k-step inside the stage, LDS slot (-1: none)
    size_t xsrc[XR];
    int xkb[XR], xdst[XR];
#pragma unroll
    for (int i = 0; i < XR; ++i) {
        const int raw = i * NTHR + tid, idx = min(raw, ngran - 1);
        const int gq = idx & 3, kb = (idx >> 2) % KB, row = (idx / (4 * KB)) % rows, sp = idx / (4 * KB * rows);
        xsrc[i] = sp * a.xplane + (size_t)(row < a.R ? row : 0) * a.ldx + (size_t)ks0 * KSTEP + gq * KF;
        xkb[i] = kb;
        xdst[i] = (raw < ngran) ? (((sp * ROWS_MT + (row >> 4)) * KB + kb) * 64 + gq * 16 + (row & 15)) : -1;
    }
    auto load_w = [&](int buf, int s) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            const size_t k = (size_t)min(s * KB + kb, nks - 1) * 64;
            wq[buf][kb][0].u = __builtin_nontemporal_load(Wt0 + k);
            wq[buf][kb][1].u = __builtin_nontemporal_load(Wt1 + k);
        }
    };
    auto load_x = [&](int s) {
#pragma unroll
        for (int i = 0; i < XR; ++i)
            xq[i] = *reinterpret_cast<const u32x4*>(reinterpret_cast<const T*>(a.X) + xsrc[i] + (size_t)min(s * KB + xkb[i], nks - 1) * KSTEP);
    };
    auto store_x = [&](int buf) {
        u32x4* dst = &Bs[buf][0][0][0][0];
#pragma unroll
        for (int i = 0; i < XR; ++i)
            if (xdst[i] >= 0) dst[xdst[i]] = xq[i];
    };
    auto compute = [&](int buf, int wb, int s) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            if (s * KB + kb < nks) {
#pragma unroll
                for (int m = 0; m < ROWS_MT; ++m) {
                    if (m < mt) {
#pragma unroll
                        for (int sp = 0; sp < SPL; ++sp) {
                            Frag b;
                            b.u = Bs[buf][sp][m][kb][lane];
                            Traits<T>::mma(wq[wb][kb][0], b, acc[0][m]);
                            Traits<T>::mma(wq[wb][kb][1], b, acc[1][m]);
                        }
                    }
                }
            }
        }
    };

    // Weights run 3 stages ahead of the products (a stage is consumed in well under the latency of HBM),
    // the staged operand one stage ahead (it comes from L2).  All loads are issued unconditionally with
    // clamped stage indices; only the products of padding iterations are skipped.
    if (nstage > 0) {
        load_x(0);
        load_w(0, 0);
        load_w(1, min(1, nstage - 1));
        load_w(2, min(2, nstage - 1));
        store_x(0);
        __syncthreads();
        for (int s = 0; s < nstage; s += 4) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int st = s + j;
                // operand first: loads return in order, so waiting for it must not mean waiting for the
                // weights requested in the same iteration
                load_x(min(st + 1, nstage - 1));
                load_w((j + 3) & 3, min(st + 3, nstage - 1));
                if (st < nstage) compute(j & 1, j, st);
                store_x((j + 1) & 1);
                __syncthreads();
            }
        }
    }

    // ---- epilogue from the accumulators: lane holds columns nt*16 + 4g .. +3 of row m*16 + r
#pragma unroll
    for (int t = 0; t < ROWS_NTW; ++t) {
        const int nt = nt0 + t;
        if (nt >= ntiles) continue;                        // wave-uniform
#pragma unroll
        for (int m = 0; m < ROWS_MT; ++m) {
            if (m >= mt) continue;                         // wave-uniform
            const int row = m * 16 + r;
            const bool valid = row < a.R;
            const f32x4 v = acc[t][m];
            if constexpr (EPI == EPI_PARTIAL) {
                if (valid)
                    *reinterpret_cast<f32x4*>(a.out + ((size_t)blockIdx.y * a.slice_rows + row) * a.N + (size_t)nt * 16 + 4 * g) = v;
            } else if constexpr (EPI == EPI_SWIGLU) {
                // tile rows 0-7 are gate of FFN columns 8*nt .. 8*nt+7, rows 8-15 their up projections:
                // the up value of this lane's gate sits two lane groups further
                float y[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float up = __shfl_down(v[i], 32, 64);
                    const float gate = v[i];
                    y[i] = gate / (1.0f + expf(-gate)) * up;
                }
                if (valid && g < 2)
                    Traits<T>::store_split4(reinterpret_cast<T*>(a.act) + (size_t)row * (a.N / 2) + (size_t)nt * 8 + 4 * g, a.actplane, y);
            } else {
                // logits + this tile's softmax partial of the row (max, sum exp((l - max)/T), lowest arg-max)
                float mx = v[0];
                int arg = nt * 16 + 4 * g;
#pragma unroll
                for (int i = 1; i < 4; ++i)
                    if (v[i] > mx) { mx = v[i]; arg = nt * 16 + 4 * g + i; }
#pragma unroll
                for (int o = 16; o < 64; o <<= 1) {
                    const float omx = __shfl_xor(mx, o, 64);
                    const int oarg = __shfl_xor(arg, o, 64);
                    if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
                }
                float se = 0.f;
                if (a.inv_temp > 0.f) {
#pragma unroll
                    for (int i = 0; i < 4; ++i) se += expf((v[i] - mx) * a.inv_temp);
                    se += __shfl_xor(se, 16, 64);
                    se += __shfl_xor(se, 32, 64);
                }
                if (valid) {
                    *reinterpret_cast<f32x4*>(a.out + (size_t)row * a.N + (size_t)nt * 16 + 4 * g) = v;
                    if (g == 0) a.stats[(size_t)row * ntiles + nt] = float4{mx, se, __int_as_float(arg), 0.f};
                }
            }
        }
    }
}

}  // namespace sj

namespace sj {

// ---------------------------------------------------------------------------------------------
// Second arrangement of the same product, built on two observations from the kernel above:
//  * a wave's loads return in order, so a wave that requests weights (HBM, ~2 us) and operand
//    (L2, < 1 us) can never consume the operand before the weights requested ahead of it arrive -
//    mixing the two streams in one wave ties the short latency to the long one;
//  * a barrier per two k-steps keeps all waves in lock step with the slowest weight load.
// Here the two streams belong to different waves.  Two LOADER waves move the workgroup's weight tiles
// (8 n-tiles x 4 k-steps = 32 KB per stage) straight from global memory into a ring of 4 LDS
// buffers, three stages ahead: up to 96 KB per CU in flight, no registers, and they alone wait for
// HBM (two waves because one wave can have at most 63 loads outstanding).  Four COMPUTE waves share
// those tiles and split the ROWS: wave w owns row tiles w, w + 4, w + 8, reads their operand
// fragments straight into a private register ring (3 k-steps ahead) and keeps 3 x 8 accumulator
// tiles.  One workgroup barrier per 4 k-steps; a weight fragment read from LDS feeds up to 6
// products, so LDS reads are a third of the MFMA time.
constexpr int R2_CW = 4;           // compute waves
constexpr int R2_LW = 2;           // loader waves (each moves half of the n-tiles)
constexpr int R2_NT = 8;           // n-tiles per workgroup
constexpr int R2_KB = 4;           // k-steps per stage
constexpr int R2_NB = 4;           // LDS stage buffers
constexpr int R2_MTW = 3;          // row tiles per compute wave
constexpr int R2_RING = 4;         // operand ring (k-steps)

template <typename T, int EPI, int SPL>
__global__ __launch_bounds__((R2_CW + R2_LW) * 64) void gemm_rows2_kernel(GemmArgs a, int mt) {
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    __shared__ u32x4 Ws[R2_NB][R2_KB][R2_NT][64];      // 4 x 32 KB
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int KS = a.K / KSTEP, ntiles = a.N / 16;
    const int nt0 = blockIdx.x * R2_NT;
    const int ks0 = (int)((long long)blockIdx.y * KS / gridDim.y), ks1 = (int)((long long)(blockIdx.y + 1) * KS / gridDim.y);
    const int nks = ks1 - ks0, nstage = (nks + R2_KB - 1) / R2_KB;
    if (nstage <= 0) return;                           // uniform for the workgroup

    if (w >= R2_CW) {
        // ---------------- loader waves: stage s -> buffer s % 4, up to three stages ahead -----------------
        // tiles past the end of N (last workgroup) and k-steps past the slice re-read valid ones
        const int half = w - R2_CW;                    // this wave moves tiles half*4 .. half*4 + 3
        const char* Wbase = reinterpret_cast<const char*>(a.Wt) + (size_t)lane * 16;
        auto issue = [&](int s) {
            u32x4* dst = &Ws[s % R2_NB][0][0][0];
#pragma unroll
            for (int kb = 0; kb < R2_KB; ++kb) {
                const size_t k = (size_t)(ks0 + min(s * R2_KB + kb, nks - 1));
#pragma unroll
                for (int tt = 0; tt < R2_NT / R2_LW; ++tt) {
                    const int t = half * (R2_NT / R2_LW) + tt;
                    const size_t tile = (size_t)min(nt0 + t, ntiles - 1);
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(Wbase + (tile * KS + k) * 1024),
                                                     (__attribute__((address_space(3))) void*)(dst + (kb * R2_NT + t) * 64), 16, 0, 0);
                }
            }
        };
        // every stage is 16 loads of this wave; stages are always issued (clamped), so the number of
        // loads outstanding behind the stage that has to be complete is known: 2 stages = 32 loads
        // (a stage index past the end re-reads the last stage into its own buffer: same bytes)
        issue(0);
        issue(min(1, nstage - 1));
        issue(min(2, nstage - 1));
        asm volatile("s_waitcnt vmcnt(32)" ::: "memory");          // stage 0 has landed
        __syncthreads();
        for (int s = 0; s < nstage; ++s) {
            // buffer (s + 3) % 4 = (s - 1) % 4 was released by the barrier that ended iteration s - 1
            issue(min(s + 3, nstage - 1));
            asm volatile("s_waitcnt vmcnt(32)" ::: "memory");      // stage s + 1 has landed
            __syncthreads();
        }
        wait_vm0();
        return;
    }

    // ---------------- compute waves ----------------
    // row tiles of this wave and their operand rows (rows past R re-read row 0; never stored)
    const T* Xr[R2_MTW];
#pragma unroll
    for (int i = 0; i < R2_MTW; ++i) {
        const int row = (w + R2_CW * i) * 16 + r;
        Xr[i] = reinterpret_cast<const T*>(a.X) + (size_t)(row < a.R ? row : 0) * a.ldx + (size_t)ks0 * KSTEP + g * KF;
    }
    const int my_tiles = (mt > w) ? (mt - w + R2_CW - 1) / R2_CW : 0;     // row tiles w, w+4, .. below mt

    f32x4 acc[R2_MTW][R2_NT];
#pragma unroll
    for (int i = 0; i < R2_MTW; ++i)
#pragma unroll
        for (int t = 0; t < R2_NT; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    Frag bq[R2_RING][R2_MTW][SPL];
    auto load_b = [&](int slot, int kk) {
        const size_t k = (size_t)min(kk, nks - 1) * KSTEP;
#pragma unroll
        for (int i = 0; i < R2_MTW; ++i)
#pragma unroll
            for (int sp = 0; sp < SPL; ++sp) bq[slot][i][sp].u = *reinterpret_cast<const u32x4*>(Xr[i] + sp * a.xplane + k);
    };
#pragma unroll
    for (int j = 0; j < R2_RING - 1; ++j) load_b(j, j);
    __syncthreads();                                   // stage 0 is in LDS
    for (int s = 0; s < nstage; ++s) {
        const u32x4* Wb = &Ws[s % R2_NB][0][0][0];
#pragma unroll
        for (int kb = 0; kb < R2_KB; ++kb) {
            const int kk = s * R2_KB + kb;
            load_b((kb + R2_RING - 1) % R2_RING, kk + R2_RING - 1);
            if (kk < nks) {
                Frag wf[R2_NT];
#pragma unroll
                for (int t = 0; t < R2_NT; ++t) wf[t].u = Wb[(kb * R2_NT + t) * 64 + lane];
#pragma unroll
                for (int i = 0; i < R2_MTW; ++i) {
                    if (i < my_tiles) {
#pragma unroll
                        for (int sp = 0; sp < SPL; ++sp)
#pragma unroll
                            for (int t = 0; t < R2_NT; ++t) Traits<T>::mma(wf[t], bq[kb % R2_RING][i][sp], acc[i][t]);
                    }
                }
            }
        }
        __syncthreads();                               // everyone is done with this buffer; the next one has landed
    }

    // ---- epilogue from the accumulators: lane holds columns nt*16 + 4g .. +3 of row m*16 + r
#pragma unroll
    for (int i = 0; i < R2_MTW; ++i) {
        if (i >= my_tiles) continue;                       // wave-uniform
        const int row = (w + R2_CW * i) * 16 + r;
        const bool valid = row < a.R;
#pragma unroll
        for (int t = 0; t < R2_NT; ++t) {
            const int nt = nt0 + t;
            if (nt >= ntiles) continue;                    // uniform
            const f32x4 v = acc[i][t];
            if constexpr (EPI == EPI_PARTIAL) {
                if (valid)
                    *reinterpret_cast<f32x4*>(a.out + ((size_t)blockIdx.y * a.slice_rows + row) * a.N + (size_t)nt * 16 + 4 * g) = v;
            } else if constexpr (EPI == EPI_SWIGLU) {
                // tile rows 0-7 are gate of FFN columns 8*nt .. 8*nt+7, rows 8-15 their up projections:
                // the up value of this lane's gate sits two lane groups further
                float y[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float up = __shfl_down(v[e], 32, 64);
                    const float gate = v[e];
                    y[e] = gate / (1.0f + expf(-gate)) * up;
                }
                if (valid && g < 2)
                    Traits<T>::store_split4(reinterpret_cast<T*>(a.act) + (size_t)row * (a.N / 2) + (size_t)nt * 8 + 4 * g, a.actplane, y);
            } else {
                // logits + this tile's softmax partial of the row (max, sum exp((l - max)/T), lowest arg-max)
                float mx = v[0];
                int arg = nt * 16 + 4 * g;
#pragma unroll
                for (int e = 1; e < 4; ++e)
                    if (v[e] > mx) { mx = v[e]; arg = nt * 16 + 4 * g + e; }
#pragma unroll
                for (int o = 16; o < 64; o <<= 1) {
                    const float omx = __shfl_xor(mx, o, 64);
                    const int oarg = __shfl_xor(arg, o, 64);
                    if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
                }
                float se = 0.f;
                if (a.inv_temp > 0.f) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) se += expf((v[e] - mx) * a.inv_temp);
                    se += __shfl_xor(se, 16, 64);
                    se += __shfl_xor(se, 32, 64);
                }
                if (valid) {
                    *reinterpret_cast<f32x4*>(a.out + (size_t)row * a.N + (size_t)nt * 16 + 4 * g) = v;
                    if (g == 0) a.stats[(size_t)row * ntiles + nt] = float4{mx, se, __int_as_float(arg), 0.f};
                }
            }
        }
    }
}

}  // namespace sj
