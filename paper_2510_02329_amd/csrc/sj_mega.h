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

constexpr int MEGA_THREADS = 512;
constexpr int MEGA_WAVES = 8;
constexpr int MEGA_D = 16;            // ring depth (weight tiles of 1 KB per wave)
constexpr int MEGA_MAXR = 8;
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
    float* hn32;                      // [R][d] final hidden state times final gain, NOT yet divided by rms
    float* row_scale;                 // [R] 1/rms of the final hidden state
    float* logits;                    // [R][V]
    float4* stats;                    // [R][V/16]
    float* cs;                        // rotary table [R][hd/2][2]
    MegaBar* bar;
    unsigned epoch0;                  // barrier epochs of this launch start above this value
    unsigned long long* prof;         // optional: timestamps (100 MHz) of workgroup 0 at every stage boundary
    double log_base;
};

// ---- coherent accessors (agent scope: write-through / cache-bypassing single accesses) ----------
__device__ __forceinline__ void st_coh(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(bf16_t* p, bf16_t v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void st_coh(unsigned* p, unsigned v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ unsigned ld_coh(const unsigned* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float ld_coh(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }

// workgroup barrier that waits for LDS traffic only: outstanding global loads (the weight ring)
// stay in flight across it
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// element offset inside a packed operand: row16 in 0..15 (0-7 hi plane of rows 0-7, 8-15 lo plane)
__device__ __forceinline__ size_t packed_off(int row16, int k) {
    return ((size_t)(k >> 5) * 64 + (size_t)((k & 31) >> 3) * 16 + row16) * 8 + (k & 7);
}
__device__ __forceinline__ void store_packed(bf16_t* B, int r, int k, float v) {
    const bf16_t h = f32_to_bf16(v);
    st_coh(B + packed_off(r, k), h);
    st_coh(B + packed_off(r + 8, k), f32_to_bf16(v - bf16_to_f32(h)));
}

struct MegaShared {
    float inv_rms[MEGA_MAXR];
    float part[4][MEGA_MAXR];
    int ok;
    int pad[3];
    float red[2][MEGA_WAVES][256];    // per-wave accumulator tiles, double-buffered by item parity;
                                      // the attention stage reuses the memory from here on
};

struct GridSync {
    MegaBar* bar;
    unsigned epoch;
    // all waves: finish this workgroup's stores, then publish the flag
    __device__ __forceinline__ void arrive() {
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)\n\ts_barrier" ::: "memory");
        ++epoch;
        if (threadIdx.x == 0) st_coh(&bar->flag[blockIdx.x * 32], epoch);
    }
    // returns false if the barrier timed out or another workgroup gave up: the caller must leave
    __device__ __forceinline__ bool wait(MegaShared& sm) {
        if (blockIdx.x == 0) {
            bool fine = true;
            for (unsigned w = threadIdx.x; w < gridDim.x; w += MEGA_THREADS) {
                unsigned spins = 0;
                while (ld_coh(&bar->flag[w * 32]) < epoch) {
                    if (++spins > MEGA_SPIN_LIMIT || ld_coh(&bar->abort)) { fine = false; break; }
                }
            }
            if (!fine) st_coh(&bar->abort, 1u);
            lds_barrier();
            if (threadIdx.x == 0) st_coh(&bar->go, epoch);
        }
        if (threadIdx.x == 0) {
            unsigned spins = 0;
            int ok = 1;
            while (ld_coh(&bar->go) < epoch) {
                if (++spins > MEGA_SPIN_LIMIT || ld_coh(&bar->abort)) { ok = 0; break; }
            }
            if (ld_coh(&bar->abort)) ok = 0;
            if (!ok) st_coh(&bar->abort, 1u);
            sm.ok = ok;
        }
        lds_barrier();
        const bool ok = sm.ok != 0;
        // every wave drops stale L1 / L2 lines before it reads what other workgroups wrote
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        lds_barrier();
        return ok;
    }
};

// ---- weight ring ---------------------------------------------------------------------------------
// A stage streams, per wave, KW consecutive k-steps of each of the workgroup's tiles
// (tile = blockIdx.x + item * gridDim.x).  prefetch() fills the ring with the first D weight tiles.
struct Stream {
    const char* W;        // tiled weights of the stage
    int ntiles, KS, KW;   // tiles in the matrix, k-steps per tile, k-steps per wave and tile
    int ks0;              // first k-step of this wave
    int n_items;          // tiles this workgroup owns
    __device__ __forceinline__ void init(const u32x4* w, int nt, int ks) {
        W = reinterpret_cast<const char*>(w); ntiles = nt; KS = ks; KW = ks / MEGA_WAVES;
        ks0 = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)) * KW;
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

// Runs one GEMM stage.  Requires KW % D == 0.  epi(tile, r, n, v, valid) is called by threads 0..255
// for every tile: r = row, n = weight row inside the tile, v = hi + lo halves summed over the waves.
template <int D, typename Epi>
__device__ __forceinline__ void gemm_stage(const Stream& s, const bf16_t* __restrict__ Bp, int R, Frag (&rw)[MEGA_D],
                                           Frag (&rb)[MEGA_D], MegaShared& sm, Epi epi) {
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const unsigned voff = lane * 16;
    const char* B = reinterpret_cast<const char*>(Bp) + (size_t)s.ks0 * 1024;
    if (s.n_items > 0) {
#pragma unroll
        for (int i = 0; i < D; ++i) rb[i].u = ld_tile(B + i * 1024, voff);
    }
    const int groups = s.KW / D;
    for (int item = 0; item < s.n_items; ++item) {
        f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
        for (int kg = 0; kg < groups; ++kg) {
            int nitem = item, nkg = kg + 1;
            if (nkg == groups) { nkg = 0; ++nitem; }
            if (nitem < s.n_items) {
                const char* wn = s.tile_base(nitem, nkg * D);
                const char* bn = B + (size_t)(nkg * D) * 1024;
#pragma unroll
                for (int i = 0; i < D; ++i) {
                    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rw[i].h, rb[i].h, acc, 0, 0, 0);
                    rw[i].u = ld_tile_nt(wn + i * 1024, voff);
                    rb[i].u = ld_tile(bn + i * 1024, voff);
                }
            } else {
#pragma unroll
                for (int i = 0; i < D; ++i) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(rw[i].h, rb[i].h, acc, 0, 0, 0);
            }
        }
        // D[n = 4g+i][col = lane%16]  ->  red[.][w][col*16 + n]
        float* red = sm.red[item & 1][w];
        const int c = lane & 15, g = lane >> 4;
#pragma unroll
        for (int i = 0; i < 4; ++i) red[c * 16 + 4 * g + i] = acc[i];
        lds_barrier();
        const int tid = threadIdx.x;
        if (tid < 256) {
            const int r = tid >> 4, n = tid & 15;
            float v = 0.f;
            if (r < MEGA_MAXR) {
#pragma unroll
                for (int ww = 0; ww < MEGA_WAVES; ++ww) v += sm.red[item & 1][ww][tid] + sm.red[item & 1][ww][tid + 128];
            }
            epi((int)(blockIdx.x + item * gridDim.x), r, n, v, r < R);
        }
    }
}

// 1/rms of every row from the per-tile sums of squares (nt tiles of 16 columns)
__device__ __forceinline__ void compute_inv_rms(const float* __restrict__ ssq, int nt, int R, int d, float eps, MegaShared& sm) {
    const int tid = threadIdx.x;
    if (tid < 256) {
        for (int r = 0; r < R; ++r) {
            float v = 0.f;
            for (int t = tid; t < nt; t += 256) v += ssq[(size_t)r * nt + t];
            v = wave_sum(v);
            if ((tid & 63) == 0) sm.part[tid >> 6][r] = v;
        }
    }
    lds_barrier();
    if (tid < R) sm.inv_rms[tid] = 1.0f / sqrtf(((sm.part[0][tid] + sm.part[1][tid]) + (sm.part[2][tid] + sm.part[3][tid])) / (float)d + eps);
    lds_barrier();
}

// ---- attention of one (sequence, kv head) by one workgroup ---------------------------------------
// LDS: Q planes [2][32][128] bf16, per-wave partial outputs [8][32][128] fp32 and (max, sum) [8][32].
struct AttnShared {
    bf16_t q[2][32][128];
    float o[MEGA_WAVES][32][128];
    float2 ml[MEGA_WAVES][32];
};

__device__ __forceinline__ void attention_wg(const MegaArgs& a, size_t layer_off, int item, AttnShared& as) {
    constexpr int HD = 128, KSTEP = 32, KF = 8, KK = HD / KSTEP, HT = HD / 16, MQ = 2;
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int rps = sp->rps;
    const int bi = item / md.Hkv, kvh = item % md.Hkv;
    const int b = sp->seq_base + bi;
    const int L = a.kv.len[b], cap = a.kv.cap[b];
    const int M = md.G * rps;
    const int Nq = md.Hq * HD, Nk = md.Hkv * HD, Nqkv = Nq + 2 * Nk;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6, r = lane & 15, g = lane >> 4;
    bf16_t* Kb = a.kv.K + layer_off + a.kv.seq_off[b] + (size_t)kvh * cap * HD;
    bf16_t* Vb = a.kv.V + layer_off + a.kv.seq_off[b] + (size_t)kvh * HD * cap;

    // rotary on q (G heads) and k (this kv head) of every block row; q -> LDS planes, k / v -> cache
    for (int p = tid; p < 2 * 32 * 128 / 2; p += MEGA_THREADS) reinterpret_cast<uint32_t*>(&as.q[0][0][0])[p] = 0u;
    __syncthreads();
    const int half = HD / 2;
    for (int p = tid; p < (md.G + 1) * rps * half; p += MEGA_THREADS) {
        const int i = p % half, j = (p / half) % rps, hh = p / (half * rps);
        const int row = bi * rps + j;
        const float c = a.cs[((size_t)row * half + i) * 2], s = a.cs[((size_t)row * half + i) * 2 + 1];
        const int col = (hh < md.G) ? (kvh * md.G + hh) * HD + i : Nq + kvh * HD + i;
        const float lo = a.qkv[(size_t)row * Nqkv + col], hi = a.qkv[(size_t)row * Nqkv + col + half];
        const float olo = lo * c - hi * s, ohi = hi * c + lo * s;
        if (hh < md.G) {
            const int m = hh * rps + j;
            const bf16_t h0 = f32_to_bf16(olo), h1 = f32_to_bf16(ohi);
            as.q[0][m][i] = h0; as.q[0][m][i + half] = h1;
            as.q[1][m][i] = f32_to_bf16(olo - bf16_to_f32(h0));
            as.q[1][m][i + half] = f32_to_bf16(ohi - bf16_to_f32(h1));
        } else if (L + j < cap) {
            bf16_t* k = Kb + (size_t)(L + j) * HD;
            k[i] = f32_to_bf16(olo);
            k[i + half] = f32_to_bf16(ohi);
        }
    }
    for (int e = tid; e < rps * HD; e += MEGA_THREADS) {
        const int j = e / HD, dcol = e % HD;
        if (L + j < cap) Vb[(size_t)dcol * cap + L + j] = f32_to_bf16(a.qkv[(size_t)(bi * rps + j) * Nqkv + Nq + Nk + kvh * HD + dcol]);
    }
    __syncthreads();      // stores of the new rows are complete and visible to this workgroup's loads

    // keys: steps of 32, wave w takes steps w, w+8, ...
    const int kv_end = min(L + rps, cap);
    f32x4 o[HT][MQ];
    float m_run[MQ], l_run[MQ];
    int limit[MQ];
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        m_run[mq] = -INFINITY; l_run[mq] = 0.f;
        const int m = mq * 16 + r;
        limit[mq] = (m < M) ? L + (m % rps) : -1;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) o[ht][mq] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    for (int key0 = w * KSTEP; key0 < kv_end; key0 += MEGA_WAVES * KSTEP) {
        f32x4 s[2][MQ];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int mq = 0; mq < MQ; ++mq) s[t][mq] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int krow = key0 + KF * (r >> 2) + 4 * t + (r & 3);
            Frag kf[KK];
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) kf[kk].u = *reinterpret_cast<const u32x4*>(Kb + (size_t)krow * HD + kk * KSTEP + g * KF);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                for (int mq = 0; mq < MQ; ++mq)
#pragma unroll
                    for (int pl = 0; pl < 2; ++pl) {
                        Frag qf;
                        qf.u = *reinterpret_cast<const u32x4*>(&as.q[pl][mq * 16 + r][kk * KSTEP + g * KF]);
                        s[t][mq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kf[kk].h, qf.h, s[t][mq], 0, 0, 0);
                    }
        }
        Frag vf[HT];
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) vf[ht].u = *reinterpret_cast<const u32x4*>(Vb + (size_t)(ht * 16 + r) * cap + key0 + g * KF);
        Frag pf[MQ][2];
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int key = key0 + KF * g + 4 * t + i;
                    const float v = (key <= limit[mq]) ? s[t][mq][i] * md.scale : -INFINITY;
                    s[t][mq][i] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[mq], mx);
            const bool dead = (m_new == -INFINITY);
            const float alpha = dead ? 1.f : expf(m_run[mq] - m_new);
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = dead ? 0.f : expf(s[t][mq][i] - m_new);
                    psum += p;
                    Traits<bf16_t>::pack_split<2>(pf[mq], 4 * t + i, p);
                }
            l_run[mq] = l_run[mq] * alpha + psum;
            m_run[mq] = m_new;
#pragma unroll
            for (int ht = 0; ht < HT; ++ht) o[ht][mq] *= alpha;
        }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int mq = 0; mq < MQ; ++mq)
#pragma unroll
                for (int pl = 0; pl < 2; ++pl) o[ht][mq] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vf[ht].h, pf[mq][pl].h, o[ht][mq], 0, 0, 0);
    }
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        float l = l_run[mq];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        const int m = mq * 16 + r;
        if (g == 0) as.ml[w][m] = float2{m_run[mq], l};
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
#pragma unroll
            for (int i = 0; i < 4; ++i) as.o[w][m][ht * 16 + 4 * g + i] = o[ht][mq][i];
    }
    __syncthreads();
    // merge the 8 waves (fixed order) and write the O-projection operand
    for (int e = tid; e < M * HD; e += MEGA_THREADS) {
        const int m = e / HD, dcol = e % HD;
        float mx = -INFINITY;
#pragma unroll
        for (int ww = 0; ww < MEGA_WAVES; ++ww) mx = fmaxf(mx, as.ml[ww][m].x);
        float den = 0.f, num = 0.f;
#pragma unroll
        for (int ww = 0; ww < MEGA_WAVES; ++ww) {
            const float2 ml = as.ml[ww][m];
            const float wgt = (ml.x == -INFINITY) ? 0.f : expf(ml.x - mx);
            den += wgt * ml.y;
            if (wgt != 0.f) num += wgt * as.o[ww][m][dcol];
        }
        const int gi = m / rps, j = m % rps;
        store_packed(a.Battn, bi * rps + j, (kvh * md.G + gi) * HD + dcol, num / den);
    }
}

// ---- the kernel -----------------------------------------------------------------------------------
__global__ __launch_bounds__(MEGA_THREADS) void mega_forward_kernel(MegaArgs a) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    MegaShared& sm = *reinterpret_cast<MegaShared*>(smem_raw);
    AttnShared& as = *reinterpret_cast<AttnShared*>(smem_raw + offsetof(MegaShared, red));
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int R = sp->nseq * sp->rps;
    const int d = md.d, tid = threadIdx.x;
    const int Nq = md.Hq * md.hd, Nk = md.Hkv * md.hd, Nqkv = Nq + 2 * Nk;
    const int ntx = d / 16;
    const bool lead = (blockIdx.x == 0) || (tid < 64);     // these poll the barrier: they prefetch after it
    GridSync gs{a.bar, a.epoch0};
    Frag rw[MEGA_D], rb[MEGA_D];
    Stream st;
    int prof_i = 0;
    auto stamp = [&]() { if (a.prof && blockIdx.x == 0 && tid == 0) a.prof[prof_i] = wall_clock64(); ++prof_i; };
    stamp();

    // stage 0: embedding rows -> residual, packed operand of the first QKV, sums of squares, rotary table
    {
        const bf16_t* gain = a.layers[0].attn_gain;
        for (int tile = blockIdx.x; tile < ntx; tile += gridDim.x) {
            if (tid < 256) {
                const int r = tid >> 4, n = tid & 15, col = tile * 16 + n;
                float v = 0.f;
                if (r < R) {
                    const int bi = r / sp->rps, j = r % sp->rps, b = sp->seq_base + bi;
                    int tok = (sp->tok_mode == 1) ? sp->prefill_tokens[j]
                                                  : (j == 0 ? a.kv.pending[b] : sp->draft_tokens[bi * sp->gamma + (j - 1)]);
                    tok = min(max(tok, 0), md.V - 1);
                    v = bf16_to_f32(a.embed[(size_t)tok * d + col]);
                    st_coh(&a.x[(size_t)r * d + col], v);
                    store_packed(a.Bx, r, col, v * bf16_to_f32(gain[col]));
                }
                float ss = v * v;
#pragma unroll
                for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
                if (r < R && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
            }
        }
        if ((int)blockIdx.x < R) {
            const int r = blockIdx.x, bi = r / sp->rps, j = r % sp->rps, b = sp->seq_base + bi;
            const int pos = a.kv.len[b] + j, half = md.hd >> 1;
            for (int i = tid; i < half; i += MEGA_THREADS) {
                const double inv_freq = exp(-2.0 * (double)i / (double)md.hd * a.log_base);
                double s, c;
                sincos((double)pos * inv_freq, &s, &c);
                st_coh(&a.cs[((size_t)r * half + i) * 2], (float)c);
                st_coh(&a.cs[((size_t)r * half + i) * 2 + 1], (float)s);
            }
        }
    }
    st.init(a.layers[0].wqkv, Nqkv / 16, d / 32);
    stamp(); gs.arrive();
    if (!lead) prefetch<MEGA_D>(st, rw);
    if (!gs.wait(sm)) return;
    if (lead) prefetch<MEGA_D>(st, rw);
    stamp();

    for (int l = 0; l < a.NL; ++l) {
        const MegaLayer& Lw = a.layers[l];
        // ---- QKV projection: qkv = (x * gain) W^T / rms
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        gemm_stage<MEGA_D>(st, a.Bx, R, rw, rb, sm, [&](int tile, int r, int n, float v, bool valid) {
            if (valid) st_coh(&a.qkv[(size_t)r * Nqkv + tile * 16 + n], v * sm.inv_rms[r]);
        });
        st.init(Lw.wo, d / 16, Nq / 32);
        stamp(); gs.arrive();
        // ---- attention (+ rotary, cache append) by the first nseq * Hkv workgroups.  The two kinds of
        // workgroup take separate paths so that the weight ring is not live across the attention code.
        const int n_attn = sp->nseq * md.Hkv;
        if ((int)blockIdx.x < n_attn) {
            if (!gs.wait(sm)) return; stamp();
            for (int item = blockIdx.x; item < n_attn; item += gridDim.x)
                attention_wg(a, (size_t)l * a.kv.layer_stride, item, as);
            stamp(); gs.arrive();
            if (!lead) prefetch<MEGA_D>(st, rw);
            if (!gs.wait(sm)) return; stamp();
            if (lead) prefetch<MEGA_D>(st, rw);
        } else {
            if (!lead) prefetch<MEGA_D>(st, rw);
            if (!gs.wait(sm)) return; stamp();
            if (lead) prefetch<MEGA_D>(st, rw);
            stamp(); gs.arrive();
            if (!gs.wait(sm)) return; stamp();
        }
        // ---- O projection + residual; operand and sums of squares for the FFN norm
        gemm_stage<MEGA_D>(st, a.Battn, R, rw, rb, sm, [&](int tile, int r, int n, float v, bool valid) {
            const int col = tile * 16 + n;
            float xn = 0.f;
            if (valid) {
                xn = ld_coh(&a.x[(size_t)r * d + col]) + v;
                st_coh(&a.x[(size_t)r * d + col], xn);
                store_packed(a.Bx, r, col, xn * bf16_to_f32(Lw.ffn_gain[col]));
            }
            float ss = xn * xn;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
            if (valid && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
        });
        st.init(Lw.wgu, 2 * md.F / 16, d / 32);
        stamp(); gs.arrive();
        if (!lead) prefetch<MEGA_D>(st, rw);
        if (!gs.wait(sm)) return; stamp();
        if (lead) prefetch<MEGA_D>(st, rw);
        // ---- gate / up projection + SwiGLU -> operand of the down projection
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        gemm_stage<MEGA_D>(st, a.Bx, R, rw, rb, sm, [&](int tile, int r, int n, float v, bool valid) {
            const float up = __shfl_down(v, 8, 64);
            if (valid && n < 8) {
                const float gate = v * sm.inv_rms[r], u = up * sm.inv_rms[r];
                store_packed(a.Bact, r, tile * 8 + n, gate / (1.0f + expf(-gate)) * u);
            }
        });
        st.init(Lw.wd, d / 16, md.F / 32);
        stamp(); gs.arrive();
        if (!lead) prefetch<MEGA_D / 2>(st, rw);
        if (!gs.wait(sm)) return; stamp();
        if (lead) prefetch<MEGA_D / 2>(st, rw);
        // ---- down projection + residual; operand and sums of squares for the next norm
        const bool last = (l + 1 == a.NL);
        const bf16_t* ngain = last ? a.final_gain : a.layers[l + 1].attn_gain;
        gemm_stage<MEGA_D / 2>(st, a.Bact, R, rw, rb, sm, [&](int tile, int r, int n, float v, bool valid) {
            const int col = tile * 16 + n;
            float xn = 0.f;
            if (valid) {
                xn = ld_coh(&a.x[(size_t)r * d + col]) + v;
                st_coh(&a.x[(size_t)r * d + col], xn);
                const float y = xn * bf16_to_f32(ngain[col]);
                store_packed(a.Bx, r, col, y);
                if (last) a.hn32[(size_t)r * d + col] = y;
            }
            float ss = xn * xn;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
            if (valid && n == 0) st_coh(&a.ssq[(size_t)r * ntx + tile], ss);
        });
        if (last) st.init(a.lm_head, md.V / 16, d / 32);
        else st.init(a.layers[l + 1].wqkv, Nqkv / 16, d / 32);
        stamp(); gs.arrive();
        if (!lead) prefetch<MEGA_D>(st, rw);
        if (!gs.wait(sm)) return; stamp();
        if (lead) prefetch<MEGA_D>(st, rw);
    }
    // ---- LM head: logits and per-tile softmax partials (Eq. 2's p, merged by the tail kernels)
    compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
    if (blockIdx.x == 0 && tid < R) a.row_scale[tid] = sm.inv_rms[tid];
    // the final hidden state was stored as x * gain by this workgroup's own down-projection epilogue:
    // apply 1/rms so that the judge (Eq. 5) and the debug read-out see the normed state
    if (tid < 16 * R) {
        const int r = tid >> 4, n = tid & 15;
        for (int tile = blockIdx.x; tile < ntx; tile += gridDim.x) a.hn32[(size_t)r * d + tile * 16 + n] *= sm.inv_rms[r];
    }
    const int ntv = md.V / 16;
    gemm_stage<MEGA_D>(st, a.Bx, R, rw, rb, sm, [&](int tile, int r, int n, float v, bool valid) {
        const float logit = v * sm.inv_rms[r < MEGA_MAXR ? r : 0];
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
}

}  // namespace sj
