// Weight-streaming GEMM for more than one row tile (batched verification: R = batch * (gamma + 1)
// rows, up to 144 per launch): Y[R][N] = X[R][K] * W[N][K]^T with W in the re-tiled layout.
// Paper reference: the projections of the target forward, Eq. 2 / Eq. 4.
//
// With many rows the few-row kernel's scheme (every wave fetches the operand fragments of all rows
// for its own K-slice) makes the operand the dominant traffic, and every weight byte should still be
// read once.  Two measured facts shaped this kernel:
//  * a wave's loads return in order, so a wave that requests weights (HBM, ~2 us) and operand
//    (L2, < 1 us) can never consume the operand before the weights requested ahead of it arrive -
//    mixing the two streams in one wave ties the short latency to the long one;
//  * a workgroup barrier every two k-steps keeps all waves in lock step with the slowest weight load.
// So the two streams belong to different waves.  Two LOADER waves move the workgroup's weight tiles
// (8 n-tiles x 4 k-steps = 32 KB per stage) straight from global memory into a ring of 4 LDS
// buffers, three stages ahead: up to 96 KB per CU in flight, no registers, and they alone wait for
// HBM (two waves because one wave can have at most 63 loads outstanding).  Four COMPUTE waves share
// those tiles and split the ROWS: wave w owns row tiles w, w + 4, w + 8, reads their operand
// fragments straight into a private register ring (3 k-steps ahead) and keeps 3 x 8 accumulator
// tiles.  One workgroup barrier per 4 k-steps; a weight fragment read from LDS feeds up to 6
// products, so LDS reads are a third of the MFMA time.  No cross-wave reduction is needed: the
// epilogue runs straight from the accumulators.  Split-K across workgroups (gridDim.y slices,
// partials summed by the consumer in slice order) keeps the short projections on all CUs.
//
// MFMA convention as in the few-row kernel: A = weight fragment (rows = n), B = operand fragment
// (rows = m), lane 16g + r then holds D[n = 4g + i][m = r].
#pragma once
#include <type_traits>

#include "sj_kernels.h"

namespace sj {

constexpr int ROWS_MT = 9;         // row tiles per launch (144 rows)
constexpr int R2_CW = 4;           // compute waves
constexpr int R2_LW = 2;           // loader waves (each moves half of the n-tiles)
constexpr int R2_NT = 8;           // n-tiles per workgroup
constexpr int R2_KB = 4;           // k-steps per stage
constexpr int R2_NB = 4;           // LDS stage buffers
constexpr int R2_MTW = 3;          // row tiles per compute wave (4 waves x 3 >= 9 row tiles)
constexpr int R2_RING = 4;         // operand ring (k-steps) = k-steps per stage

// Epilogue of the many-row kernels for ONE accumulator tile (row tile m, n-tile nt): the lane holds columns
// nt*16 + 4g .. +3 of row m*16 + r.  Uniform per wave; rows >= R take part in the shuffles and store nothing.
template <typename T, int EPI>
__device__ __forceinline__ void rows_epilogue_tile(const GemmArgs& a, const f32x4& v, int m, int nt, int ntiles, int r, int g) {
    const int row = m * 16 + r;
    const bool valid = row < a.R;
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
            Traits<T>::store_split4(reinterpret_cast<T*>(a.act) + opnd_off<T>(row, nt * 8 + 4 * g, a.N / 2, a.act_tks), a.actplane, y);
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

// The same over a wave's tiles: wave w owns row tiles w, w + 4, w + 8.
template <typename T, int EPI, int NT = R2_NT>
__device__ __forceinline__ void rows_epilogue(const GemmArgs& a, const f32x4 (&acc)[R2_MTW][NT], int w, int my_tiles, int nt0,
                                              int ntiles, int r, int g) {
#pragma unroll
    for (int i = 0; i < R2_MTW; ++i) {
        if (i >= my_tiles) continue;                       // wave-uniform
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            if (nt0 + t >= ntiles) continue;               // uniform
            rows_epilogue_tile<T, EPI>(a, acc[i][t], w + R2_CW * i, nt0 + t, ntiles, r, g);
        }
    }
}

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
        lds_barrier();
        for (int s = 0; s < nstage; ++s) {
            // buffer (s + 3) % 4 = (s - 1) % 4 was released by the barrier that ended iteration s - 1
            issue(min(s + 3, nstage - 1));
            asm volatile("s_waitcnt vmcnt(32)" ::: "memory");      // stage s + 1 has landed
            lds_barrier();
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
    lds_barrier();                                   // stage 0 is in LDS
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
        lds_barrier();                               // everyone is done with this buffer; the next one has landed
    }

    rows_epilogue<T, EPI>(a, acc, w, my_tiles, nt0, ntiles, r, g);
}

// ---------------------------------------------------------------------------------------------
// Same product with the OPERAND delivered through LDS as well (one or two operand planes).
// Measured on the kernel above: with the compute waves' own operand loads taken out it runs at
// max(weight stream, MFMA), with them near the sum, and a row-major operand fragment touches 16 cache
// lines of which it uses half.  Here the compute waves issue no global loads at all: loader waves
// fetch the operand fragments of all row tiles next to the weight tiles of the same k-step, from
// planes that the producing kernels wrote as fragments (opnd_off: 1 KB of consecutive memory each;
// row-major planes are still accepted).  A stage is ONE k-step; a wave's loads come back in the order
// it issued them, so weights (HBM: 8 stages of 8 KB) and operand (an L2 hit: 5 stages of
// 9 x SPL KB) are fetched by different loader waves with rings of their own; one barrier per k-step;
// the compute waves read the fragments of step s + 1 from LDS while they multiply step s.  An
// operand fragment in LDS has the layout the lanes read it in (lane l: 16 bytes at l * 16), which is
// also how a direct global->LDS load of 16 bytes per lane deposits it.
constexpr int R4_NSW = 8;          // weight stages (k-steps) in LDS: HBM latency to cover
constexpr int R4_NSX = 5;          // operand stages: an L2 hit away
constexpr int R4_LW = 4;           // loader waves: two for the weights, two for the operand

// NT = n-tiles per workgroup: 8, or 7 where that makes the number of workgroups a multiple of the CU count
// (gate/up projection of the 8B shape: 1792 n-tiles = 256 x 7).
// Several row groups in ONE launch (a.rgroups > 1): the weights should come from HBM once for all of them, so the
// workgroups that share an n-tile group must run at the same time on compute units that share a cache.  Workgroups
// are handed to the 8 XCDs (each with an L2 of its own) round robin by index, so workgroup i works for XCD i % 8;
// within an XCD consecutive workgroups take the row groups of one n-tile group, then the next n-tile group: the first
// of them pulls a weight tile from HBM, the others find it in their L2 a moment later.
//
// EIGHT compute waves with an even split of the 9 x NT accumulator tiles: wave w = (a = w % 4, b = w / 4) owns row tiles
// a and a + 4 for the n-tiles of half b, and n-tile w of row tile 8: 9 tiles each for NT = 8 (8 / 8 / 8 / 8 / 7 / 7 / 7 / 6
// for NT = 7), 36 accumulator registers, two compute waves per SIMD.  An earlier form with four compute waves (row tiles
// w, w + 4, w + 8: one wave with three) measured the same on two-plane operands, where the L2 traffic of the operand sets
// the pace, and 12 % slower on the one-plane LM head of the verify-head workload (909 -> 799 us).
constexpr int R8_CW = 8;

// RT = row tiles of a row group: 9 (144 rows), or 18 with a single operand plane (288 rows: the same 18 operand
// fragments per k-step in LDS, half as many workgroups re-reading every weight tile through L2).  A wave owns RT / 4
// whole row tiles for its half of the n-tiles and n-tile w of each of the RT % 4 tiles left over.
template <typename T, int EPI, int SPL, int NT = R2_NT, int RT = ROWS_MT>
__global__ __launch_bounds__((R8_CW + R4_LW) * 64) void gemm_rows8_kernel(GemmArgs a, int mt) {
    static_assert(SPL <= 2, "three operand planes do not fit");
    static_assert(NT == 7 || NT == 8, "n-tile halves are 4 + 4 or 4 + 3");
    static_assert(RT * SPL <= 2 * ROWS_MT, "the operand stages in LDS hold 18 fragments");
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    constexpr int NX = RT * SPL;                       // operand fragments per stage
    constexpr int NFULL = RT / 4, NREM = RT % 4;       // whole row tiles per wave; tiles shared out by n-tile
    __shared__ u32x4 Wst[R4_NSW][NT][64];
    __shared__ u32x4 Xst[R4_NSX][NX][64];
    const int tid = threadIdx.x, lane = tid & 63, w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, g = lane >> 4;
    const int KS = a.K / KSTEP, ntiles = a.N / 16;
    int bx = blockIdx.x;
    if (a.rgroups > 1) {
        const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
        const int rg = j % a.rgroups;
        bx = (j / a.rgroups) * 8 + xcd;
        if (bx * NT >= ntiles) return;                 // padding of the grid to whole XCD rounds (uniform)
        const int row0 = rg * (RT * 16), nr = min(RT * 16, a.R - row0);
        a.X = reinterpret_cast<const char*>(a.X) + (size_t)row0 * a.ldx * sizeof(T);
        if (EPI == EPI_SWIGLU) a.act = reinterpret_cast<char*>(a.act) + (size_t)row0 * (a.N / 2) * sizeof(T);
        else a.out += (size_t)row0 * a.N;
        if (EPI == EPI_LOGITS) a.stats += (size_t)row0 * ntiles;
        a.R = nr;
        mt = (nr + 15) / 16;
    }
    const int nt0 = bx * NT;
    const int ks0 = (int)((long long)blockIdx.y * KS / gridDim.y), ks1 = (int)((long long)(blockIdx.y + 1) * KS / gridDim.y);
    const int nks = ks1 - ks0;
    if (nks <= 0) return;                              // uniform for the workgroup

    if (w >= R8_CW) {
        // ---------------- loader waves ----------------
        // A wave's loads come back in the order it issued them, so the weights (HBM, deep ring) and the operand (L2, shallow
        // ring) are fetched by different waves.  Stage = k-step of the slice (clamped: a stage past the end re-reads the last
        // one into its own buffer).  The compute waves read stage s + 1 while they multiply stage s, so stage s + 2 has to be
        // in LDS when iteration s ends: NS - 3 stages of a loader wave's loads may still be in flight.
        const int lw = w - R8_CW;
        auto run = [&](auto nl_tag, auto ns_tag, auto aux_tag, auto make_src, auto dst_of) {
            constexpr int NL = decltype(nl_tag)::value, NS = decltype(ns_tag)::value, AUX = decltype(aux_tag)::value;
            const char* src[NL];
            size_t step[NL];
#pragma unroll
            for (int j = 0; j < NL; ++j) make_src(j, src[j], step[j]);
            auto issue = [&](int s) {
                const size_t k = (size_t)min(s, nks - 1);
#pragma unroll
                for (int j = 0; j < NL; ++j)
                    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(src[j] + k * step[j]),
                                                     (__attribute__((address_space(3))) void*)dst_of(s % NS, j), 16, 0, AUX);
            };
            constexpr int BEHIND = (NS - 3) * NL;
            static_assert((NS - 1) * NL < 64, "the load counter holds 63");
#pragma unroll
            for (int s = 0; s < NS - 1; ++s) issue(s);
            __builtin_amdgcn_s_waitcnt(vmcnt_imm(BEHIND));            // stages 0 and 1 have landed
            lds_barrier();
            for (int s = 0; s < nks; ++s) {
                issue(s + NS - 1);
                __builtin_amdgcn_s_waitcnt(vmcnt_imm(BEHIND));        // stage s + 2 has landed
                lds_barrier();
            }
            wait_vm0();
        };
        if (lw < 2) {
            auto make_src = [&](int j, const char*& sp, size_t& st) {
                const size_t tile = (size_t)min(nt0 + min(lw + 2 * j, NT - 1), ntiles - 1);
                sp = reinterpret_cast<const char*>(a.Wt) + ((tile * KS + ks0) * 64 + lane) * 16;
                st = 1024;
            };
            auto dst_of = [&](int buf, int j) { return &Wst[buf][min(lw + 2 * j, NT - 1)][0]; };
            if (a.rgroups > 1)
                run(std::integral_constant<int, (NT + 1) / 2>{}, std::integral_constant<int, R4_NSW>{}, std::integral_constant<int, 0>{}, make_src, dst_of);
            else
                run(std::integral_constant<int, (NT + 1) / 2>{}, std::integral_constant<int, R4_NSW>{}, std::integral_constant<int, 2>{}, make_src, dst_of);
        } else {
            const int x = lw - 2;
            auto make_src = [&](int j, const char*& sp, size_t& st) {
                const int it = min(x + 2 * j, NX - 1);
                const int m = it / SPL, p = it % SPL;
                const T* plane = reinterpret_cast<const T*>(a.X) + (size_t)p * a.xplane;
                if (a.x_tks) {
                    const size_t mt_ok = m * 16 < a.R ? m : 0;
                    sp = reinterpret_cast<const char*>(plane + ((mt_ok * a.x_tks + ks0) * 16 + r) * KSTEP + g * KF);
                    st = (size_t)16 * KSTEP * sizeof(T);
                } else {
                    const int row = m * 16 + r;
                    sp = reinterpret_cast<const char*>(plane + (size_t)(row < a.R ? row : 0) * a.ldx + (size_t)ks0 * KSTEP + g * KF);
                    st = (size_t)KSTEP * sizeof(T);
                }
            };
            auto dst_of = [&](int buf, int j) { return &Xst[buf][min(x + 2 * j, NX - 1)][0]; };
            run(std::integral_constant<int, (NX + 1) / 2>{}, std::integral_constant<int, R4_NSX>{}, std::integral_constant<int, 0>{}, make_src, dst_of);
        }
        return;
    }

    // ---------------- compute waves ----------------
    const int ra = w & 3, nb = w >> 2;                 // row tiles ra, ra + 4; n-tiles of half nb; n-tile w of row tile 8
    constexpr int NH = 4;                              // n-tiles of half 0 (half 1 has NT - 4)
    const int t0 = nb * NH, nh = nb == 0 ? NH : NT - NH;
    f32x4 acc[NFULL][NH], acc8[NREM];
#pragma unroll
    for (int i = 0; i < NFULL; ++i)
#pragma unroll
        for (int t = 0; t < NH; ++t) acc[i][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int j = 0; j < NREM; ++j) acc8[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    struct Frags { Frag wf[NH]; Frag w8; Frag bq[NFULL + NREM][SPL]; };
    Frags fA, fB;
    auto fetch = [&](Frags& f, int s) {
        const u32x4* Xs = &Xst[s % R4_NSX][0][0];
        const u32x4* Ws = &Wst[s % R4_NSW][0][0];
#pragma unroll
        for (int sp = 0; sp < SPL; ++sp) {
#pragma unroll
            for (int i = 0; i < NFULL; ++i) f.bq[i][sp].u = Xs[((ra + 4 * i) * SPL + sp) * 64 + lane];
#pragma unroll
            for (int j = 0; j < NREM; ++j) f.bq[NFULL + j][sp].u = Xs[((4 * NFULL + j) * SPL + sp) * 64 + lane];
        }
#pragma unroll
        for (int t = 0; t < NH; ++t) f.wf[t].u = Ws[min(t0 + t, NT - 1) * 64 + lane];
        f.w8.u = Ws[min(w, NT - 1) * 64 + lane];
    };
    // No predicate in the k-step: a tile that does not exist (row tiles past the rows re-read tile 0, n-tiles past the
    // workgroup's are clamped) is multiplied into an accumulator that the epilogue never stores.
    auto multiply = [&](const Frags& f) {
#pragma unroll
        for (int sp = 0; sp < SPL; ++sp) {
#pragma unroll
            for (int t = 0; t < NH; ++t)
#pragma unroll
                for (int i = 0; i < NFULL; ++i) Traits<T>::mma(f.wf[t], f.bq[i][sp], acc[i][t]);
#pragma unroll
            for (int j = 0; j < NREM; ++j) Traits<T>::mma(f.w8, f.bq[NFULL + j][sp], acc8[j]);
        }
    };
    lds_barrier();                                     // stages 0 and 1 are in LDS
    fetch(fA, 0);
    for (int s = 0; s < nks; s += 2) {
        fetch(fB, s + 1);
        multiply(fA);
        lds_barrier();                                 // stage s + 2 has landed
        if (s + 1 < nks) {                             // uniform
            fetch(fA, s + 2);
            multiply(fB);
            lds_barrier();                             // stage s + 3 has landed
        }
    }
#pragma unroll
    for (int t = 0; t < NH; ++t) {
        if (t >= nh || nt0 + t0 + t >= ntiles) continue;   // uniform
#pragma unroll
        for (int i = 0; i < NFULL; ++i)
            if (ra + 4 * i < mt) rows_epilogue_tile<T, EPI>(a, acc[i][t], ra + 4 * i, nt0 + t0 + t, ntiles, r, g);
    }
    if (w < NT && nt0 + w < ntiles) {
#pragma unroll
        for (int j = 0; j < NREM; ++j)
            if (4 * NFULL + j < mt) rows_epilogue_tile<T, EPI>(a, acc8[j], 4 * NFULL + j, nt0 + w, ntiles, r, g);
    }
}

}  // namespace sj
