// Persistent whole-forward kernel for small row counts (R = batch * (gamma + 1) <= 8, bf16).
//
// At batch 1 a decoder layer streams 436 MB of weights in ~60 us, split over five dependent stages
// (QKV, attention, O, gate/up, down).  Launched as separate kernels every stage pays a drain and a
// ramp of the memory pipeline.  Here ONE cooperative grid (one workgroup of 8 waves per CU) walks
// all stages of all layers (Eq. 2 / Eq. 4 of the paper: the target forward over the draft block):
//   * stages are separated by a flag-based grid barrier (every workgroup publishes an epoch flag,
//     workgroup 0 collects them and releases one "go" word; about 2 us, no read-modify-write);
//   * every wave owns a register ring of weight tiles; after it has arrived at a barrier it already
//     issues the loads of its first tiles of the NEXT stage (weights do not depend on activations),
//     so HBM keeps streaming while the barrier resolves;
//   * data exchanged between workgroups (activations, partial sums of squares) is written with
//     agent-scope write-through stores and read after an agent-scope acquire at the barrier - no
//     L2 write-back fences.
// Matrix products: D[16 weight rows][16] += W tile (A operand, 1 KB contiguous) x packed
// activation tile (B operand).  With R <= 8 the 16 B-operand rows carry BOTH bf16 planes of the
// fp32 activation: row r is hi = bf16(x_r), row r + 8 is lo = bf16(x_r - hi); the two halves of D
// are added in the epilogue.  One MFMA per weight tile, 16 significant bits of activation.
// RMSNorm is split around the product: the producer of the residual writes x * gain as packed
// planes plus per-tile sums of squares; the consumer scales its outputs by 1/rms of the row.
#pragma once
#include "sj_kernels.h"
#include <cstddef>

namespace sj {

constexpr int MEGA_SW = 8;                        // streaming waves: weight ring + MFMA (+ attention)
constexpr int MEGA_THREADS = (MEGA_SW + 1) * 64;  // plus one service wave: barriers, operand staging, epilogues
constexpr int MEGA_D = 16;                        // ring depth (1 KB weight tiles per streaming wave)
constexpr int MEGA_DD = 8;                        // ring depth of the down projection (weights + operand rings)
constexpr int MEGA_MAXR = 8;
constexpr int MEGA_BIG = 128 * 1024;              // LDS bytes of the staged operand / attention scratch
constexpr unsigned MEGA_SPIN_LIMIT = 400000u;

struct MegaBar {
    unsigned go;
    unsigned abort;
    unsigned pad[30];
    unsigned flag[1024 * 32];         // one flag per workgroup, 128 bytes apart
};

struct MegaLayer {
    const u32x4* wqkv;
    const u32x4* wo;
    const u32x4* wgu;                 // 8 gate rows + 8 up rows per tile
    const u32x4* wd;
    const bf16_t* attn_gain;
    const bf16_t* ffn_gain;
};

struct MegaArgs {
    const MegaLayer* layers;          // device array [NL]
    const u32x4* lm_head;
    const bf16_t* final_gain;
    const bf16_t* embed;
    int32_t NL;
    ModelDims md;
    const StepParams* sp;
    KvView<bf16_t> kv;
    float* x;                         // [R][d] residual stream
    float* qkv;                       // [R][Nqkv]
    bf16_t* Bx;                       // packed operand of QKV / gate-up / LM head: [d/32][64][8]
    bf16_t* Battn;                    // packed operand of the O projection: [Hq*hd/32][64][8]
    bf16_t* Bact;                     // packed operand of the down projection: [F/32][64][8]
    float* ssq;                       // [R][d/16] sums of squares of the residual, one per 16 columns
    float* hn32;                      // [R][d] final hidden state after the last RMSNorm
    float* row_scale;                 // [R] 1/rms of the final hidden state
    float* logits;                    // [R][V]
    float4* stats;                    // [R][V/16]
    float* cs;                        // rotary table [R][hd/2][2]
    MegaBar* bar;
    unsigned epoch0;                  // barrier epochs of this launch start above this value
    unsigned long long* prof;         // optional: timestamps (100 MHz) of workgroup 0 at every stage boundary
    double log_base;
};

// element offset inside a packed operand: row16 in 0..15 (0-7 hi plane of rows 0-7, 8-15 lo plane)
__device__ __forceinline__ size_t packed_off(int row16, int k) {
    return ((size_t)(k >> 5) * 64 + (size_t)((k & 31) >> 3) * 16 + row16) * 8 + (k & 7);
}
// Every lane of a 16-lane row group holds the value of column k0 + n (n = lane % 16, k0 a multiple of
// 16) of row r: the hi / lo bf16 planes of 8 neighbouring columns are gathered into 16 bytes and
// written by the lanes with n % 8 == 0 as two 8-byte write-through stores per plane.
__device__ __forceinline__ void store_packed_row16(bf16_t* B, int r, int k, int n, float v, bool valid) {
    const bf16_t h = f32_to_bf16(v);
    const bf16_t l = f32_to_bf16(v - bf16_to_f32(h));
    unsigned h32 = (unsigned)h | ((unsigned)(__shfl_down((int)h, 1, 64) & 0xffff) << 16);
    unsigned l32 = (unsigned)l | ((unsigned)(__shfl_down((int)l, 1, 64) & 0xffff) << 16);
    unsigned long long h64 = (unsigned long long)h32 | ((unsigned long long)(unsigned)__shfl_down((int)h32, 2, 64) << 32);
    unsigned long long l64 = (unsigned long long)l32 | ((unsigned long long)(unsigned)__shfl_down((int)l32, 2, 64) << 32);
    const unsigned long long h64b = __shfl_down(h64, 4, 64), l64b = __shfl_down(l64, 4, 64);
    if (valid && (n & 7) == 0) {
        unsigned long long* ph = reinterpret_cast<unsigned long long*>(B + packed_off(r, k));
        unsigned long long* pl = reinterpret_cast<unsigned long long*>(B + packed_off(r + 8, k));
        st_coh(ph, h64); st_coh(ph + 1, h64b);
        st_coh(pl, l64); st_coh(pl + 1, l64b);
    }
}

struct AttnShared {
    bf16_t q[2][16][128];             // rotated queries of one head, hi / lo planes, row = block row j
    bf16_t knew[32][128];             // rotated keys of the block's own rows, as the cache stores them
    bf16_t vnewT[128][32];            // values of the block's own rows, transposed
    float o[MEGA_SW][16][128];        // per-wave unnormalised outputs
    float2 ml[MEGA_SW][16];           // per-wave running max and sum
};

struct MegaShared {
    float inv_rms[MEGA_MAXR];
    int ok;
    int pad[7];
    float red[2][MEGA_SW][256];       // per-wave accumulator tiles, double-buffered by item parity
    __attribute__((aligned(1024))) unsigned char big[MEGA_BIG];   // staged B operand (k-step tiles of 1 KB) or attention scratch
};
static_assert(sizeof(AttnShared) <= MEGA_BIG, "attention scratch must fit the staging area");

// ---- grid barrier, run by the service wave alone --------------------------------------------------
struct GridSync {
    MegaBar* bar;
    unsigned epoch;
    // Publishes this workgroup's flag once the wave's own stores have completed, waits for the release
    // word (workgroup 0 collects all flags), then drops stale cache lines.  false = timed out / aborted.
    __device__ __forceinline__ bool sync() {
        const int lane = threadIdx.x & 63;
        wait_vm0();
        ++epoch;
        if (lane == 0) st_coh(&bar->flag[blockIdx.x * 32], epoch);
        int ok = 1;
        if (blockIdx.x == 0) {
            for (unsigned w = lane; w < gridDim.x; w += 64) {
                unsigned spins = 0;
                while (ld_coh(&bar->flag[w * 32]) < epoch) {
                    if (++spins > MEGA_SPIN_LIMIT || ld_coh(&bar->abort)) { ok = 0; break; }
                }
            }
            ok = __all(ok);
            if (lane == 0) { if (!ok) st_coh(&bar->abort, 1u); st_coh(&bar->go, epoch); }
        }
        if (lane == 0) {
            unsigned spins = 0;
            while (ld_coh(&bar->go) < epoch) {
                if (++spins > MEGA_SPIN_LIMIT || ld_coh(&bar->abort)) { ok = 0; break; }
            }
            if (ld_coh(&bar->abort)) ok = 0;
            if (!ok) st_coh(&bar->abort, 1u);
        }
        ok = __shfl(ok, 0, 64);
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");     // L1 / L2 lines written by other workgroups are stale
        return ok != 0;
    }
};

// ---- weight ring ---------------------------------------------------------------------------------
// A stage streams, per streaming wave, KW consecutive k-steps of each of the workgroup's tiles
// (tile = blockIdx.x + item * gridDim.x).  prefetch() fills the ring with the first D weight tiles.
struct Stream {
    const char* W;        // tiled weights of the stage
    int ntiles, KS, KW;   // tiles in the matrix, k-steps per tile, k-steps per wave and tile
    int ks0;              // first k-step of this wave
    int n_items;          // tiles this workgroup owns
    __device__ __forceinline__ void init(const u32x4* w, int nt, int ks) {
        W = reinterpret_cast<const char*>(w); ntiles = nt; KS = ks; KW = ks / MEGA_SW;
        ks0 = (__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) % MEGA_SW) * KW;
        n_items = ((int)blockIdx.x < nt) ? (nt - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    }
    // wave-uniform byte address of the 1 KB tile (item, k-step kk of this wave's slice)
    __device__ __forceinline__ const char* tile_base(int item, int kk) const {
        return W + (((size_t)(blockIdx.x + (size_t)item * gridDim.x)) * KS + ks0 + kk) * 1024;
    }
};

// 16 bytes per lane from a wave-uniform base: scalar base + 32-bit lane offset addressing
__device__ __forceinline__ u32x4 ld_tile_nt(const char* base, unsigned voff) {
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(base + voff));
}
__device__ __forceinline__ u32x4 ld_tile(const char* base, unsigned voff) {
    return *reinterpret_cast<const u32x4*>(base + voff);
}

template <int D>
__device__ __forceinline__ void prefetch(const Stream& s, Frag (&rw)[MEGA_D]) {
    if (s.n_items > 0) {
        const char* p = s.tile_base(0, 0);
        const unsigned voff = (threadIdx.x & 63) * 16;
#pragma unroll
        for (int i = 0; i < D; ++i) rw[i].u = ld_tile_nt(p + i * 1024, voff);
    }
}

// Streaming-wave side of one GEMM stage.  Requires KW % D == 0.  BLDS: the packed operand has been
// staged into sm.big by the service wave (k-step kk at byte kk * 1024); otherwise it is read from
// global memory through a second ring.  Returns false if the step was aborted.
template <int D, bool BLDS>
__device__ __forceinline__ bool stream_stage(const Stream& s, const bf16_t* __restrict__ Bp, Frag (&rw)[MEGA_D],
                                             Frag (&rb)[MEGA_D], MegaShared& sm) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const unsigned voff = lane * 16;
    lds_barrier();                                        // operand staged, 1/rms ready, caches acquired
    if (!sm.ok) return false;
    const char* B = reinterpret_cast<const char*>(Bp) + (size_t)s.ks0 * 1024;
    const unsigned char* Bl = sm.big + (size_t)s.ks0 * 1024 + voff;
    if (!BLDS && s.n_items > 0) {
#pragma unroll
        for (int i = 0; i < D; ++i) rb[i].u = ld_tile(B + i * 1024, voff);
    }
    const int groups = s.KW / D;
    for (int item = 0; item < s.n_items; ++item) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int kg = 0; kg < groups; ++kg) {
            int nitem = item, nkg = kg + 1;
            if (nkg == groups) { nkg = 0; ++nitem; }
            const unsigned char* bl = Bl + (size_t)(kg * D) * 1024;
            if (nitem < s.n_items) {
                const char* wn = s.tile_base(nitem, nkg * D);
                const char* bn = B + (size_t)(nkg * D) * 1024;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    Frag fb;
                    if (BLDS) fb.u = *reinterpret_cast<const u32x4*>(bl + i * 1024); else fb = rb[i];
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rw[i].h, fb.h, acc, 0, 0, 0);
                    rw[i].u = ld_tile_nt(wn + i * 1024, voff);
                    if (!BLDS) rb[i].u = ld_tile(bn + i * 1024, voff);
                }
            } else {
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    Frag fb;
                    if (BLDS) fb.u = *reinterpret_cast<const u32x4*>(bl + i * 1024); else fb = rb[i];
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rw[i].h, fb.h, acc, 0, 0, 0);
                }
            }
        }
        // D[n = 4g+i][col = lane%16]  ->  red[.][w][col*16 + n]
        float* red = sm.red[item & 1][w];
        const int c = lane & 15, g = lane >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) red[c * 16 + 4 * g + i] = acc[i];
        lds_barrier();                                    // the service wave may reduce this item now
    }
    return true;
}

// Service-wave side: after the operand is staged, reduce every item's partial tiles and run the
// stage's epilogue.  epi(tile, r, n, v, valid, half) is called twice per item (half 0: rows 0-3,
// half 1: rows 4-7) with r = row, n = weight row inside the tile (all 64 lanes take part).
template <typename Epi>
__device__ __forceinline__ void service_stage(int n_items, int R, MegaShared& sm, Epi epi) {
    const int lane = threadIdx.x & 63;
    lds_barrier();
    for (int item = 0; item < n_items; ++item) {
        lds_barrier();
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int e = lane + 64 * half, r = e >> 4, n = e & 15;
            float v = 0.f;
#pragma unroll
            for (int ww = 0; ww < MEGA_SW; ++ww) v += sm.red[item & 1][ww][e] + sm.red[item & 1][ww][e + 128];
            epi((int)(blockIdx.x + item * gridDim.x), r, n, v, r < R, half);
        }
    }
}

// operand tiles global -> LDS (1 KB per k-step), issued back to back by the service wave
__device__ __forceinline__ void stage_operand(const bf16_t* __restrict__ Bp, int KS, MegaShared& sm) {
    const char* g = reinterpret_cast<const char*>(Bp) + (threadIdx.x & 63) * 16;
    for (int t = 0; t < KS; ++t)
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(g + (size_t)t * 1024),
                                         (__attribute__((address_space(3))) void*)(sm.big + (size_t)t * 1024), 16, 0, 0);
}

// 1/rms of every row from the per-tile sums of squares (service wave; nt tiles of 16 columns)
__device__ __forceinline__ void compute_inv_rms(const float* __restrict__ ssq, int nt, int R, int d, float eps, MegaShared& sm) {
    const int lane = threadIdx.x & 63;
    float v[MEGA_MAXR];
#pragma unroll
    for (int r = 0; r < MEGA_MAXR; ++r) {
        v[r] = 0.f;
        if (r < R) for (int t = lane; t < nt; t += 64) v[r] += ssq[(size_t)r * nt + t];
    }
#pragma unroll
    for (int r = 0; r < MEGA_MAXR; ++r) {
        const float tot = wave_sum(v[r]);
        if (lane == 0 && r < R) sm.inv_rms[r] = 1.0f / sqrtf(tot / (float)d + eps);
    }
}

// ---- attention of one (sequence, query head) by the 8 streaming waves of one workgroup -------------
// The rps block rows of the head are one MFMA query tile.  Cached keys 0..L-1 are read from the cache in
// steps of 32, wave w taking steps w, w+8, ...; the block's own keys (positions L..L+rps-1) are rotated
// here, kept in LDS in the cache's storage format and handled as one more step, so that no workgroup
// has to wait for another one's cache append.  The workgroup of a kv head's first query head also
// writes the new K / V rows to the cache.  The service wave only takes part in the barriers.
__device__ __noinline__ void attention_wg(const MegaArgs& a, size_t layer_off, int item, AttnShared& as) {
    constexpr int HD = 128, KSTEP = 32, KF = 8, KK = HD / KSTEP, HT = HD / 16;
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int rps = sp->rps;
    const int bi = item / md.Hq, qh = item % md.Hq, kvh = qh / md.G;
    const bool writer = (qh % md.G) == 0;
    const int b = sp->seq_base + bi;
    const int L = a.kv.len[b], cap = a.kv.cap[b];
    const int Nq = md.Hq * HD, Nk = md.Hkv * HD, Nqkv = Nq + 2 * Nk;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 15, g = lane >> 4;
    constexpr int NT = MEGA_SW * 64;
    bf16_t* Kb = a.kv.K + layer_off + a.kv.seq_off[b] + (size_t)kvh * cap * HD;
    bf16_t* Vb = a.kv.V + layer_off + a.kv.seq_off[b] + (size_t)kvh * HD * cap;

    auto astamp = [&](int i) { if (a.prof && blockIdx.x == 0 && tid == 0) a.prof[3000 + i] = wall_clock64(); };
    astamp(0);
    // zero the padding of the LDS operands (q, knew, vnewT are contiguous: 24 KB)
    for (int p = tid; p < (int)((sizeof(as.q) + sizeof(as.knew) + sizeof(as.vnewT)) / 4); p += NT)
        reinterpret_cast<uint32_t*>(&as.q[0][0][0])[p] = 0u;
    lds_barrier();
    const int half = HD / 2;
    // rotary pairs of q (work items 0 .. rps*64-1) and k (rps*64 .. 2*rps*64-1), then the values
    for (int p = tid; p < 2 * rps * half + rps * HD; p += NT) {
        if (p < 2 * rps * half) {
            const int i = p % half, j = (p / half) % rps, isk = p / (half * rps);
            const int row = bi * rps + j;
            const float c = a.cs[((size_t)row * half + i) * 2], s = a.cs[((size_t)row * half + i) * 2 + 1];
            const int col = isk ? Nq + kvh * HD + i : qh * HD + i;
            const float lo = a.qkv[(size_t)row * Nqkv + col], hi = a.qkv[(size_t)row * Nqkv + col + half];
            const float olo = lo * c - hi * s, ohi = hi * c + lo * s;
            const bf16_t h0 = f32_to_bf16(olo), h1 = f32_to_bf16(ohi);
            if (!isk) {
                as.q[0][j][i] = h0; as.q[0][j][i + half] = h1;
                as.q[1][j][i] = f32_to_bf16(olo - bf16_to_f32(h0));
                as.q[1][j][i + half] = f32_to_bf16(ohi - bf16_to_f32(h1));
            } else {
                as.knew[j][i] = h0; as.knew[j][i + half] = h1;
                if (writer && L + j < cap) {
                    bf16_t* k = Kb + (size_t)(L + j) * HD;
                    k[i] = h0; k[i + half] = h1;
                }
            }
        } else {
            const int e = p - 2 * rps * half, j = e / HD, dcol = e % HD;
            const bf16_t v = f32_to_bf16(a.qkv[(size_t)(bi * rps + j) * Nqkv + Nq + Nk + kvh * HD + dcol]);
            as.vnewT[dcol][j] = v;
            if (writer && L + j < cap) Vb[(size_t)dcol * cap + L + j] = v;
        }
    }
    astamp(1);
    lds_barrier();
    astamp(2);

    f32x4 o[HT];
    float m_run = -INFINITY, l_run = 0.f;
#pragma unroll
    for (int ht = 0; ht < HT; ++ht) o[ht] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nsteps = (L + KSTEP - 1) / KSTEP;                  // steps over the cached keys
    // one step: K rows (two S^T tiles), V^T rows, online softmax, PV.  `limit` = last visible key index
    // relative to key0 semantics below; cached steps see keys < L, the block step sees jj <= j.
    auto step = [&](const Frag (&kf)[2][KK], const Frag (&vf)[HT], int key0, int limit) {
        f32x4 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl) {
                    Frag qf;
                    qf.u = *reinterpret_cast<const u32x4*>(&as.q[pl][r][kk * KSTEP + g * KF]);
                    s[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[t][kk].h, qf.h, s[t], 0, 0, 0);
                }
        }
        Frag pf[2];
        float mx = -INFINITY;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int key = key0 + KF * g + 4 * t + i;
                const float v = (key <= limit) ? s[t][i] * md.scale : -INFINITY;
                s[t][i] = v;
                mx = fmaxf(mx, v);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        const float m_new = fmaxf(m_run, mx);
        const bool dead = (m_new == -INFINITY);
        const float alpha = dead ? 1.f : expf(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = dead ? 0.f : expf(s[t][i] - m_new);
                psum += p;
                Traits<bf16_t>::pack_split<2>(pf, 4 * t + i, p);
            }
        l_run = l_run * alpha + psum;
        m_run = m_new;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) {
            o[ht] *= alpha;
#pragma unroll
            for (int pl = 0; pl < 2; ++pl) o[ht] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[ht].h, pf[pl].h, o[ht], 0, 0, 0);
        }
    };
    for (int st = w; st < nsteps; st += MEGA_SW) {
        const int key0 = st * KSTEP;
        Frag kf[2][KK], vf[HT];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int krow = key0 + KF * (r >> 2) + 4 * t + (r & 3);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = *reinterpret_cast<const u32x4*>(Kb + (size_t)krow * HD + kk * KSTEP + g * KF);
        }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) vf[ht].u = *reinterpret_cast<const u32x4*>(Vb + (size_t)(ht * 16 + r) * cap + key0 + g * KF);
        step(kf, vf, key0, (r < rps) ? L - 1 : -1);
    }
    astamp(3);
    if (w == nsteps % MEGA_SW) {
        // the block's own keys: key index jj = 0..31 (rows >= rps are zero padding), row j sees jj <= j
        Frag kf[2][KK], vf[HT];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int krow = KF * (r >> 2) + 4 * t + (r & 3);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kf[t][kk].u = *reinterpret_cast<const u32x4*>(&as.knew[krow][kk * KSTEP + g * KF]);
        }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) vf[ht].u = *reinterpret_cast<const u32x4*>(&as.vnewT[ht * 16 + r][g * KF]);
        step(kf, vf, 0, (r < rps) ? r : -1);
    }
    {
        float l = l_run;
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        if (g == 0) as.ml[w][r] = float2{m_run, l};
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int i = 0; i < 4; ++i) as.o[w][r][ht * 16 + 4 * g + i] = o[ht][i];
    }
    astamp(4);
    lds_barrier();
    astamp(5);
    // merge the waves (fixed order) and write this head's columns of the O-projection operand; each
    // 16-lane group holds 16 neighbouring columns of one row
    for (int e = tid; e < rps * HD; e += NT) {
        const int j = e / HD, dcol = e % HD;
        float mx = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < MEGA_SW; ++ww) mx = fmaxf(mx, as.ml[ww][j].x);
        float den = 0.f, num = 0.f;
#pragma unroll
        for (int ww = 0; ww < MEGA_SW; ++ww) {
            const float2 ml = as.ml[ww][j];
            const float wgt = (ml.x == -INFINITY) ? 0.f : expf(ml.x - mx);
            den += wgt * ml.y;
            if (wgt != 0.f) num += wgt * as.o[ww][j][dcol];
        }
        const bool valid = j < rps;
        store_packed_row16(a.Battn, valid ? bi * rps + j : 0, qh * HD + dcol, dcol & 15, valid ? num / den : 0.f, valid);
    }
    astamp(6);
    wait_vm0();
    astamp(7);
}

// ---- the kernel -----------------------------------------------------------------------------------
__global__ __launch_bounds__(MEGA_THREADS) void mega_forward_kernel(MegaArgs a) {
    extern __shared__ __align__(1024) unsigned char smem_raw[];
    MegaShared& sm = *reinterpret_cast<MegaShared*>(smem_raw);
    AttnShared& as = *reinterpret_cast<AttnShared*>(sm.big);
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int R = sp->nseq * sp->rps;
    const int d = md.d, tid = threadIdx.x, lane = tid & 63;
    const int Nq = md.Hq * md.hd, Nk = md.Hkv * md.hd, Nqkv = Nq + 2 * Nk;
    const int ntx = d / 16, ntv = md.V / 16;
    const bool service = tid >= MEGA_SW * 64;
    const int n_attn = sp->nseq * md.Hq;                  // one workgroup per (sequence, query head)
    const bool has_attn = (int)blockIdx.x < n_attn;
    const int KWd = md.F / 32 / MEGA_SW;                  // k-steps per wave of the down projection

    if (tid == 0) sm.ok = 1;
    __syncthreads();

    if (service) {
        // =============================== service wave =============================================
        GridSync gs{a.bar, a.epoch0};
        int prof_i = 0;
        auto stamp = [&]() { if (a.prof && blockIdx.x == 0 && lane == 0) a.prof[prof_i] = wall_clock64(); ++prof_i; };
        auto items_of = [&](int nt) { return ((int)blockIdx.x < nt) ? (nt - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0; };
        auto leave = [&]() { sm.ok = 0; };
        stamp();
        // stage 0: embedding rows -> residual, packed operand of the first QKV, sums of squares, rotary table
        {
            const bf16_t* gain = a.layers[0].attn_gain;
            for (int tile = blockIdx.x; tile < ntx; tile += gridDim.x) {
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int e = lane + 64 * half, r = e >> 4, n = e & 15, col = tile * 16 + n;
                    float v = 0.f;
                    const bool valid = r < R;
                    if (valid) {
                        const int bi = r / sp->rps, j = r % sp->rps, b = sp->seq_base + bi;
                        int tok = (sp->tok_mode == 1) ? sp->prefill_tokens[j]
                                                      : (j == 0 ? a.kv.pending[b] : sp->draft_tokens[bi * sp->gamma + (j - 1)]);
                        tok = min(max(tok, 0), md.V - 1);
                        v = bf16_to_f32(a.embed[(size_t)tok * d + col]);
                        st_coh(&a.x[(size_t)r * d + col], v);
                    }
                    store_packed_row16(a.Bx, r & 7, col, n, v * bf16_to_f32(gain[col]), valid);
                    float ss = v * v;
#pragma unroll
                    for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
                    if (valid && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
                }
            }
            if ((int)blockIdx.x < R) {
                const int r = blockIdx.x, bi = r / sp->rps, j = r % sp->rps, b = sp->seq_base + bi;
                const int pos = a.kv.len[b] + j, half = md.hd >> 1;
                for (int i = lane; i < half; i += 64) {
                    const double inv_freq = exp(-2.0 * (double)i / (double)md.hd * a.log_base);
                    double s, c;
                    sincos((double)pos * inv_freq, &s, &c);
                    st_coh(&a.cs[((size_t)r * half + i) * 2], (float)c);
                    st_coh(&a.cs[((size_t)r * half + i) * 2 + 1], (float)s);
                }
            }
        }
        stamp();
        if (!gs.sync()) { leave(); return; }
        stamp();
        for (int l = 0; l < a.NL; ++l) {
            const MegaLayer& Lw = a.layers[l];
            // ---- QKV projection: qkv = (x * gain) W^T / rms
            stage_operand(a.Bx, d / 32, sm);
            compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
            wait_vm0();
            service_stage(items_of(Nqkv / 16), R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
                if (valid) st_coh(&a.qkv[(size_t)r * Nqkv + tile * 16 + n], v * sm.inv_rms[r]);
            });
            stamp();
            if (!gs.sync()) { leave(); return; }
            stamp();
            // ---- attention: the streaming waves of the first nseq * Hq workgroups
            if (has_attn) {
                for (int item = blockIdx.x; item < n_attn; item += gridDim.x) {
                    // release + the three barriers inside the attention + its end
                    lds_barrier(); lds_barrier(); lds_barrier(); lds_barrier(); lds_barrier();
                }
            }
            stamp();
            if (!gs.sync()) { leave(); return; }
            stamp();
            // ---- O projection + residual; operand and sums of squares for the FFN norm
            stage_operand(a.Battn, Nq / 32, sm);
            float xpre[2];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int e = lane + 64 * half, r = e >> 4, n = e & 15;
                xpre[half] = (r < R && (int)blockIdx.x < ntx) ? ld_coh(&a.x[(size_t)r * d + blockIdx.x * 16 + n]) : 0.f;
            }
            wait_vm0();
            service_stage(items_of(ntx), R, sm, [&](int tile, int r, int n, float v, bool valid, int half) {
                const int col = tile * 16 + n;
                float xn = 0.f;
                if (valid) {
                    const float xo = (tile == (int)blockIdx.x) ? xpre[half] : ld_coh(&a.x[(size_t)r * d + col]);
                    xn = xo + v;
                    st_coh(&a.x[(size_t)r * d + col], xn);
                }
                store_packed_row16(a.Bx, r & 7, col, n, xn * bf16_to_f32(Lw.ffn_gain[col]), valid);
                float ss = xn * xn;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
                if (valid && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
            });
            stamp();
            if (!gs.sync()) { leave(); return; }
            stamp();
            // ---- gate / up projection + SwiGLU -> operand of the down projection
            stage_operand(a.Bx, d / 32, sm);
            compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
            wait_vm0();
            service_stage(items_of(2 * md.F / 16), R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
                const float up = __shfl_down(v, 8, 64);
                const float sc = sm.inv_rms[r & 7];
                const float gate = v * sc, u = up * sc;
                // lanes n < 8 hold 8 neighbouring FFN columns: replicate them so that the 16-lane packer sees
                // columns 8*tile .. 8*tile+7 in lanes 0-7 (lanes 8-15 carry padding that is not stored)
                const float act = gate / (1.0f + expf(-gate)) * u;
                const bf16_t h = f32_to_bf16(act), lo = f32_to_bf16(act - bf16_to_f32(h));
                unsigned h32 = (unsigned)h | ((unsigned)(__shfl_down((int)h, 1, 64) & 0xffff) << 16);
                unsigned l32 = (unsigned)lo | ((unsigned)(__shfl_down((int)lo, 1, 64) & 0xffff) << 16);
                unsigned long long h64 = (unsigned long long)h32 | ((unsigned long long)(unsigned)__shfl_down((int)h32, 2, 64) << 32);
                unsigned long long l64 = (unsigned long long)l32 | ((unsigned long long)(unsigned)__shfl_down((int)l32, 2, 64) << 32);
                const unsigned long long h64b = __shfl_down(h64, 4, 64), l64b = __shfl_down(l64, 4, 64);
                if (valid && n == 0) {
                    unsigned long long* ph = reinterpret_cast<unsigned long long*>(a.Bact + packed_off(r, tile * 8));
                    unsigned long long* pl = reinterpret_cast<unsigned long long*>(a.Bact + packed_off(r + 8, tile * 8));
                    st_coh(ph, h64); st_coh(ph + 1, h64b);
                    st_coh(pl, l64); st_coh(pl + 1, l64b);
                }
            });
            stamp();
            if (!gs.sync()) { leave(); return; }
            stamp();
            // ---- down projection + residual; operand and sums of squares for the next norm
            const bool last = (l + 1 == a.NL);
            const bf16_t* ngain = last ? a.final_gain : a.layers[l + 1].attn_gain;
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int e = lane + 64 * half, r = e >> 4, n = e & 15;
                xpre[half] = (r < R && (int)blockIdx.x < ntx) ? ld_coh(&a.x[(size_t)r * d + blockIdx.x * 16 + n]) : 0.f;
            }
            wait_vm0();
            service_stage(items_of(ntx), R, sm, [&](int tile, int r, int n, float v, bool valid, int half) {
                const int col = tile * 16 + n;
                float xn = 0.f;
                if (valid) {
                    const float xo = (tile == (int)blockIdx.x) ? xpre[half] : ld_coh(&a.x[(size_t)r * d + col]);
                    xn = xo + v;
                    st_coh(&a.x[(size_t)r * d + col], xn);
                }
                const float y = xn * bf16_to_f32(ngain[col]);
                store_packed_row16(a.Bx, r & 7, col, n, y, valid);
                if (last && valid) a.hn32[(size_t)r * d + col] = y;
                float ss = xn * xn;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
                if (valid && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
            });
            stamp();
            if (!gs.sync()) { leave(); return; }
            stamp();
        }
        // ---- LM head: logits and per-tile softmax partials (Eq. 2's p, merged by the tail kernels)
        stage_operand(a.Bx, d / 32, sm);
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        wait_vm0();
        if (blockIdx.x == 0 && lane < R) a.row_scale[lane] = sm.inv_rms[lane];
        // this wave stored the final hidden state as x * gain in its own down-projection epilogue: apply
        // 1/rms so that the judge (Eq. 5) and the debug read-out see the normed state
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int e = lane + 64 * half, r = e >> 4, n = e & 15;
            if (r < R)
                for (int tile = blockIdx.x; tile < ntx; tile += gridDim.x) a.hn32[(size_t)r * d + tile * 16 + n] *= sm.inv_rms[r];
        }
        service_stage(items_of(ntv), R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
            const float logit = v * sm.inv_rms[r & 7];
            float mx = logit;
            int arg = tile * 16 + n;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) {
                const float omx = __shfl_xor(mx, o, 64);
                const int oarg = __shfl_xor(arg, o, 64);
                if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
            }
            float se = 0.f;
            if (md.inv_temp > 0.f) {
                se = expf((logit - mx) * md.inv_temp);
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) se += __shfl_xor(se, o, 64);
            }
            if (valid) {
                a.logits[(size_t)r * md.V + tile * 16 + n] = logit;
                if (n == 0) a.stats[(size_t)r * ntv + tile] = float4{mx, se, __int_as_float(arg), 0.f};
            }
        });
        stamp();
        return;
    }

    // ================================= streaming waves ============================================
    Frag rw[MEGA_D], rb[MEGA_D];
    Stream st;
    (void)KWd;
    st.init(a.layers[0].wqkv, Nqkv / 16, d / 32);
    prefetch<MEGA_D>(st, rw);
    for (int l = 0; l < a.NL; ++l) {
        const MegaLayer& Lw = a.layers[l];
        if (!stream_stage<MEGA_D, true>(st, a.Bx, rw, rb, sm)) return;
        st.init(Lw.wo, ntx, Nq / 32);
        if (has_attn) {
            // the ring is filled after the attention so that it is not live across it
            for (int item = blockIdx.x; item < n_attn; item += gridDim.x) {
                lds_barrier();                               // released by the service wave: qkv is complete
                if (!sm.ok) return;
                attention_wg(a, (size_t)l * a.kv.layer_stride, item, as);
                lds_barrier();
            }
        }
        prefetch<MEGA_D>(st, rw);
        if (!stream_stage<MEGA_D, true>(st, a.Battn, rw, rb, sm)) return;
        st.init(Lw.wgu, 2 * md.F / 16, d / 32);
        prefetch<MEGA_D>(st, rw);
        if (!stream_stage<MEGA_D, true>(st, a.Bx, rw, rb, sm)) return;
        st.init(Lw.wd, ntx, md.F / 32);
        prefetch<MEGA_DD>(st, rw);
        if (!stream_stage<MEGA_DD, false>(st, a.Bact, rw, rb, sm)) return;
        if (l + 1 == a.NL) st.init(a.lm_head, ntv, d / 32);
        else st.init(a.layers[l + 1].wqkv, Nqkv / 16, d / 32);
        prefetch<MEGA_D>(st, rw);
    }
    stream_stage<MEGA_D, true>(st, a.Bx, rw, rb, sm);
}

}  // namespace sj
