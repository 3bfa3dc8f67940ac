// Rotary + cache append + multi-query causal decode attention of one layer in ONE launch
// (paper Eq. 2: the target model scores the gamma + 1 rows of a block against the cached context).
//
// Workgroup = 4 waves = one (key range, kv head, group of query tiles, sequence).  The M = G*rps query
// rows that share a kv head are the MFMA "columns":
//   S^T[key][m]  = K[key][:] . Q[m][:]           (A = K rows,   B = Q rows)
//   O^T[hd][m]  += V^T[hd][keys] . P^T[keys][m]  (A = V^T rows, B = the S^T accumulators, re-packed)
// The key order inside a 4*KF-key step is permuted (S tile t, A row a <-> key KF*(a/4) + 4t + a%4)
// so that a lane's S^T accumulators are exactly its B-operand elements of the second product:
// no LDS transpose, no cross-lane traffic except the running-max reduction over the 4 lane groups.
//
// The step is bound by dependent memory round trips, not by bytes, so the kernel is organised around
// having few of them:
//  * round trip 1 - everything that does not depend on anything computed here is requested at once,
//    without branches: the wave's first K / V step from the cache, its share of the QKV split-K
//    partials for the query fragments, and the partials of the block's own K / V rows;
//  * the waves rotate their share of the query rows and exchange the MFMA fragments through LDS;
//    the workgroup that owns the end of the context also builds the block's own K / V rows (rotary
//    on K, rounding to the storage type), keeps them in LDS as one more key step - query row j sees
//    new rows 0..j - and appends them to the cache (the q-group-0 workgroup writes);
//  * the 4 waves' results are merged through LDS, each wave merging a quarter of the head tiles in
//    wave order; with one key range per (sequence, kv head, q group) that is the result;
//  * otherwise each workgroup publishes its partial with write-through stores and draws a ticket
//    (round trips 2, 3); the workgroup that draws the last ticket reads the ranges back (round trip 4)
//    and merges them in range order (fixed order -> bit-reproducible), then writes the O-projection
//    operand planes.
// A row whose position would fall outside the sequence's capacity writes nothing to the cache (the
// host refuses such calls before launching).
#pragma once
#include "sj_kernels.h"

namespace sj {

#ifdef SJ_ATTN_PROF
__device__ unsigned long long attn_prof[4096 * 16];
#define ATTN_STAMP(k) do { if ((threadIdx.x & 63) == 0) attn_prof[((((blockIdx.z * gridDim.y + blockIdx.y) * gridDim.x + blockIdx.x) & 1023) * 4 + (threadIdx.x >> 6)) * 16 + (k)] = wall_clock64(); } while (0)
#else
#define ATTN_STAMP(k) do { } while (0)
#endif

// m / d for 0 <= m < 2^20, 0 < d: reciprocal estimate + one correction step either way
__device__ __forceinline__ int small_div(int m, int d) {
    int q = (int)((float)m * __frcp_rn((float)d));
    q -= (q * d > m);
    q += ((q + 1) * d <= m);
    return q;
}

template <typename T, int HD, int MQ, int SPL>
struct AttnSmem {
    static constexpr int HT = HD / 16, KK = HD / Traits<T>::KSTEP;
    union {
        struct {
            T knew[64][HD];                 // the block's own K rows (rotated, storage-rounded), zero-padded
            T vnewT[HD][64];                // the block's own V rows, transposed
            u32x4 q[MQ][KK][SPL][64];       // query fragments in lane order
        } in;
        struct {
            f32x4 o[4][4 * MQ][64];         // the 4 waves' accumulators of 4 head tiles, in lane order
            float m[4][MQ][64];
            float l[4][MQ][64];
        } mg;
    };
    int last;
};

// floats per published partial of one workgroup
template <int HD, int MQ> constexpr int attn_partial_floats() { return (HD / 16 * MQ * 4 + 2 * MQ) * 64; }

template <typename T, int HD, int MQ, int SPL, int PB = 4>
__global__ __launch_bounds__(256) void attn_fused_kernel(const StepParams* __restrict__ sp, ModelDims md,
                                                         const float* __restrict__ part, int nparts, int R,
                                                         const float* __restrict__ cs, KvView<T> kv, int layer,
                                                         int wave_keys, int nchunk_max, float* __restrict__ opart,
                                                         unsigned* __restrict__ tickets, T* __restrict__ attn_out,
                                                         size_t aplane, int otks) {
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    constexpr int NS = KF / 4;       // S^T tiles per step of KSTEP keys
    static_assert(SPL <= Traits<T>::NS, "more planes than the storage type has");
    constexpr int KK = HD / KSTEP;   // contraction steps over the head dimension
    constexpr int HT = HD / 16, HALF = HD / 2, NSLOT = HT * MQ * 4;
    constexpr int NG = MQ * KK / 2;  // query fragment groups: (q tile, pair of head-dim steps kk, kk + KK/2)
    constexpr int HPW = HT / 4;      // head tiles per wave in the merges: wave w takes tiles w, w + 4, ..
    // PB = split-K partials of the QKV product fetched per batch of independent loads.  With at most two partials a
    // batch of four only repeats loads: they fill the wave's load queue ahead of the K / V requests (64 entries; query
    // fragments + own rows + one key step came to 72) and cost 1.2 us of the 14.5 us launch at batch 1.
    __shared__ AttnSmem<T, HD, MQ, SPL> sm;

    const int chunk = blockIdx.x, kvh = blockIdx.y % md.Hkv, qg = blockIdx.y / md.Hkv, bi = blockIdx.z;
    const int qgroups = gridDim.y / md.Hkv;
    const int b = sp->seq_base + bi;
    const int rps = sp->rps;
    const int M = md.G * rps;
    const int L = kv.len[b], cap = kv.cap[b];
    const int wg_keys = 4 * wave_keys;
    const int nch = max(1, (L + wg_keys - 1) / wg_keys);   // key ranges of the cached context
    if (chunk >= nch) return;
    const bool tail = (chunk == nch - 1);                  // this workgroup also takes the block's own rows
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, r = lane & 15, g = lane >> 4;
    const int Nq = md.Hq * HD, Nk = md.Hkv * HD, N = Nq + 2 * Nk;
    T* Kb = kv.K + (size_t)layer * kv.layer_stride + kv.seq_off[b] + (size_t)kvh * cap * HD;
    T* Vb = kv.V + (size_t)layer * kv.layer_stride + kv.seq_off[b] + (size_t)kvh * HD * cap;
    ATTN_STAMP(0);

    // ---------------- round trip 1: all independent loads, branch-free (indices clamped) --------------
    const int key_lo = chunk * wg_keys + wave * wave_keys;
    const int key_hi = min(key_lo + wave_keys, L);
    // two register sets of one key step each: the next step is requested before the current one is used
    Frag kf[2][NS][KK], vf[2][HT];
    auto load_keys = [&](int set, int key0) {
#pragma unroll
        for (int t = 0; t < NS; ++t) {
            const int krow = key0 + KF * (r >> 2) + 4 * t + (r & 3);
#pragma unroll
            for (int kk = 0; kk < KK; ++kk)
                kf[set][t][kk].u = *reinterpret_cast<const u32x4*>(Kb + (size_t)krow * HD + kk * KSTEP + g * KF);
        }
#pragma unroll
        for (int ht = 0; ht < HT; ++ht)
            vf[set][ht].u = *reinterpret_cast<const u32x4*>(Vb + (size_t)(ht * 16 + r) * cap + key0 + g * KF);
    };
    load_keys(0, min(key_lo, cap - KSTEP));            // capacities are multiples of 64: always inside

    // query fragment group gq = (q tile mq, head-dim step kk): 4 split-K partials per batch of loads
    float4 qa[PB][KF / 4], qc[PB][KF / 4];
    auto q_row = [&](int gq, int& row, int& head, bool& valid) {
        const int mq = gq / (KK / 2);
        const int m = (qg * MQ + mq) * 16 + r;
        valid = m < M;                                 // padding rows read row 0 (valid memory), masked later
        const int gi = valid ? small_div(m, rps) : 0, j = valid ? m - gi * rps : 0;
        row = bi * rps + j;
        head = kvh * md.G + gi;
    };
    auto q_issue = [&](int gq, int s0) {
        int row, head; bool valid;
        q_row(gq, row, head, valid);
        const int i0 = (gq % (KK / 2)) * KSTEP + g * KF;
        const int off0 = row * N + head * HD + i0;     // the partials hold fewer than 2^31 elements
#pragma unroll
        for (int u = 0; u < PB; ++u) {
            const float* pl = part + (off0 + min(s0 + u, nparts - 1) * R * N);
#pragma unroll
            for (int e = 0; e < KF / 4; ++e) {
                qa[u][e] = *reinterpret_cast<const float4*>(pl + 4 * e);
                qc[u][e] = *reinterpret_cast<const float4*>(pl + HALF + 4 * e);
            }
        }
    };
    q_issue(min(wave, NG - 1), 0);

    // the block's own rows: work item = (row j, K or V, column pair (i, i + HALF)), NB items per thread
    // and batch (one batch covers 8 rows of head dimension 128), 4 split-K partials of both columns each
    constexpr int NB = 4;
    const int nr_total = rps * HD;
    float nlo[NB][PB], nhi[NB][PB], ncs[NB][2];
    auto nr_item = [&](int it, int& j, int& i, bool& isv) {
        j = it / HD;
        const int w = it % HD;
        i = w % HALF;
        isv = w >= HALF;
    };
    auto nr_issue = [&](int base, int s0) {
#pragma unroll
        for (int u = 0; u < NB; ++u) {
            int j, i; bool isv;
            nr_item(min(base + u * 256 + tid, nr_total - 1), j, i, isv);
            const int row = bi * rps + j, col = (isv ? Nq + Nk : Nq) + kvh * HD + i;
            const int off0 = row * N + col;
#pragma unroll
            for (int v = 0; v < PB; ++v) {
                const float* pl = part + (off0 + min(s0 + v, nparts - 1) * R * N);
                nlo[u][v] = pl[0];
                nhi[u][v] = pl[HALF];
            }
            ncs[u][0] = cs[(row * HALF + i) * 2];
            ncs[u][1] = cs[(row * HALF + i) * 2 + 1];
        }
    };
    nr_issue(0, 0);
    ATTN_STAMP(1);

    // ---------------- query fragments: rotate this wave's groups, exchange through LDS ----------------
    for (int gq = wave; gq < NG; gq += 4) {
        float lo[KF], hi[KF];
#pragma unroll
        for (int e = 0; e < KF; ++e) { lo[e] = 0.f; hi[e] = 0.f; }
        for (int s0 = 0; s0 < nparts; s0 += PB) {
            if (gq != wave || s0 != 0) q_issue(gq, s0);
#pragma unroll
            for (int u = 0; u < PB; ++u) {
                const float wgt = (s0 + u < nparts) ? 1.f : 0.f;
#pragma unroll
                for (int e = 0; e < KF / 4; ++e) {
                    lo[4 * e] += wgt * qa[u][e].x; lo[4 * e + 1] += wgt * qa[u][e].y; lo[4 * e + 2] += wgt * qa[u][e].z; lo[4 * e + 3] += wgt * qa[u][e].w;
                    hi[4 * e] += wgt * qc[u][e].x; hi[4 * e + 1] += wgt * qc[u][e].y; hi[4 * e + 2] += wgt * qc[u][e].z; hi[4 * e + 3] += wgt * qc[u][e].w;
                }
            }
        }
        int row, head; bool valid;
        q_row(gq, row, head, valid);
        const int mq = gq / (KK / 2), kk = gq % (KK / 2), i0 = kk * KSTEP + g * KF;
        const float* csr = cs + (row * HALF + i0) * 2;
        Frag f0[SPL], f1[SPL];
#pragma unroll
        for (int e = 0; e < KF; ++e) {
            const float c = csr[2 * e], s = csr[2 * e + 1];
            Traits<T>::template pack_split<SPL>(f0, e, lo[e] * c - hi[e] * s);
            Traits<T>::template pack_split<SPL>(f1, e, hi[e] * c + lo[e] * s);
        }
#pragma unroll
        for (int pl = 0; pl < SPL; ++pl) {
            sm.in.q[mq][kk][pl][lane] = f0[pl].u;
            sm.in.q[mq][kk + KK / 2][pl][lane] = f1[pl].u;
        }
    }
    ATTN_STAMP(2);

    // ---------------- the block's own K / V rows (tail workgroup): LDS, and the cache if q group 0 ----
    if (tail) {
        const bool writer = (qg == 0);
        const int rpad = (rps + KSTEP - 1) / KSTEP * KSTEP;
        for (int base = 0; base < nr_total; base += NB * 256) {
            float lo[NB], hi[NB];
#pragma unroll
            for (int u = 0; u < NB; ++u) { lo[u] = 0.f; hi[u] = 0.f; }
            for (int s0 = 0; s0 < nparts; s0 += PB) {
                if (base != 0 || s0 != 0) nr_issue(base, s0);
#pragma unroll
                for (int u = 0; u < NB; ++u)
#pragma unroll
                    for (int v = 0; v < PB; ++v) {
                        const float wgt = (s0 + v < nparts) ? 1.f : 0.f;
                        lo[u] += wgt * nlo[u][v];
                        hi[u] += wgt * nhi[u][v];
                    }
            }
#pragma unroll
            for (int u = 0; u < NB; ++u) {
                const int it = base + u * 256 + tid;
                if (it < nr_total) {
                    int j, i; bool isv;
                    nr_item(it, j, i, isv);
                    const float c = isv ? 1.f : ncs[u][0], s = isv ? 0.f : ncs[u][1];
                    const float olo = lo[u] * c - hi[u] * s, ohi = hi[u] * c + lo[u] * s;
                    const bool in_cap = writer && L + j < cap;
                    if (!isv) {
                        Traits<T>::store(&sm.in.knew[j][i], olo);
                        Traits<T>::store(&sm.in.knew[j][i + HALF], ohi);
                        if (in_cap) {
                            Kb[(size_t)(L + j) * HD + i] = sm.in.knew[j][i];
                            Kb[(size_t)(L + j) * HD + i + HALF] = sm.in.knew[j][i + HALF];
                        }
                    } else {
                        Traits<T>::store(&sm.in.vnewT[i][j], olo);
                        Traits<T>::store(&sm.in.vnewT[i + HALF][j], ohi);
                        if (in_cap) {
                            Vb[(size_t)i * cap + L + j] = sm.in.vnewT[i][j];
                            Vb[(size_t)(i + HALF) * cap + L + j] = sm.in.vnewT[i + HALF][j];
                        }
                    }
                }
            }
        }
        for (int e = tid; e < (rpad - rps) * HD; e += 256) {     // padding rows of the last key step
            const int j = rps + e / HD, dcol = e % HD;
            Traits<T>::store(&sm.in.knew[j][dcol], 0.f);
            Traits<T>::store(&sm.in.vnewT[dcol][j], 0.f);
        }
    }
    __syncthreads();
    ATTN_STAMP(3);

    Frag qf[MQ][KK][SPL];
    bool rowvalid[MQ];
    int jrow[MQ], girow[MQ];
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        const int m = (qg * MQ + mq) * 16 + r;
        rowvalid[mq] = m < M;
        girow[mq] = rowvalid[mq] ? small_div(m, rps) : 0;
        jrow[mq] = rowvalid[mq] ? m - girow[mq] * rps : 0;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk)
#pragma unroll
            for (int pl = 0; pl < SPL; ++pl) qf[mq][kk][pl].u = sm.in.q[mq][kk][pl][lane];
    }

    f32x4 o[HT][MQ];
    float m_run[MQ], l_run[MQ];
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        m_run[mq] = -INFINITY;
        l_run[mq] = 0.f;
#pragma unroll
        for (int ht = 0; ht < HT; ++ht) o[ht][mq] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // one step of KSTEP keys held in kf / vf; visible(mq, kidx) says whether query row mq of this lane
    // sees the key with in-step index kidx = KF*g + 4t + i
    auto consume = [&](int set, auto visible) {
        f32x4 s[NS][MQ];
#pragma unroll
        for (int t = 0; t < NS; ++t)
#pragma unroll
            for (int mq = 0; mq < MQ; ++mq) {
                s[t][mq] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
#pragma unroll
                    for (int pl = 0; pl < SPL; ++pl) Traits<T>::mma(kf[set][t][kk], qf[mq][kk][pl], s[t][mq]);
            }
        Frag pf[MQ][SPL];
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            float mx = -INFINITY;
#pragma unroll
            for (int t = 0; t < NS; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = visible(mq, KF * g + 4 * t + i) ? s[t][mq][i] * md.scale : -INFINITY;
                    s[t][mq][i] = v;
                    mx = fmaxf(mx, v);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[mq], mx);
            const bool dead = (m_new == -INFINITY);
            const float alpha = dead ? 1.f : __expf(m_run[mq] - m_new);
            float psum = 0.f;
#pragma unroll
            for (int t = 0; t < NS; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float p = dead ? 0.f : __expf(s[t][mq][i] - m_new);
                    psum += p;
                    Traits<T>::template pack_split<SPL>(pf[mq], 4 * t + i, p);
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
                for (int pl = 0; pl < SPL; ++pl) Traits<T>::mma(vf[set][ht], pf[mq][pl], o[ht][mq]);
    };

    // ---------------- cached keys of this wave ----------------
    // one step of the cache from register set `set`; columns of V past the context hold whatever the
    // cache had: zero them so that 0 * value stays 0
    auto cached_step = [&](int set, int key0) {
        if (key0 + KSTEP > L) {
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
#pragma unroll
                for (int e = 0; e < KF; ++e)
                    if (key0 + g * KF + e >= L) {
                        if constexpr (sizeof(T) == 2) vf[set][ht].s[e] = 0; else vf[set][ht].f[e] = 0.f;
                    }
        }
        consume(set, [&](int mq, int kidx) { return rowvalid[mq] && key0 + kidx < L; });
    };
    {
        int key0 = key_lo;                             // set 0 holds this step
        while (key0 + KSTEP < key_hi) {                // at least two steps left: no branch around the loads
            load_keys(1, key0 + KSTEP);
            cached_step(0, key0);
            load_keys(0, min(key0 + 2 * KSTEP, cap - KSTEP));   // may lie past this wave's range: in bounds, unused then
            cached_step(1, key0 + KSTEP);
            key0 += 2 * KSTEP;
        }
        if (key0 < key_hi) cached_step(0, key0);
    }
    ATTN_STAMP(4);
    // ---------------- the block's own rows: row j of the block sees new rows 0..j ----------------
    if (tail && wave == 3) {
        const int rpad = (rps + KSTEP - 1) / KSTEP * KSTEP;
        for (int j0 = 0; j0 < rpad; j0 += KSTEP) {
#pragma unroll
            for (int t = 0; t < NS; ++t) {
                const int krow = j0 + KF * (r >> 2) + 4 * t + (r & 3);
#pragma unroll
                for (int kk = 0; kk < KK; ++kk)
                    kf[0][t][kk].u = *reinterpret_cast<const u32x4*>(&sm.in.knew[krow][kk * KSTEP + g * KF]);
            }
#pragma unroll
            for (int ht = 0; ht < HT; ++ht)
                vf[0][ht].u = *reinterpret_cast<const u32x4*>(&sm.in.vnewT[ht * 16 + r][j0 + g * KF]);
            consume(0, [&](int mq, int kidx) { return rowvalid[mq] && j0 + kidx <= jrow[mq]; });
        }
    }
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        float l = l_run[mq];
        l += __shfl_xor(l, 16, 64);
        l += __shfl_xor(l, 32, 64);
        l_run[mq] = l;
    }
    ATTN_STAMP(5);

    // ---------------- merge of the 4 waves through LDS, 4 head tiles per round: wave w merges tile 4h + w ----
    __syncthreads();                    // the input area is dead from here on (same LDS as the merge area)
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) { sm.mg.m[wave][mq][lane] = m_run[mq]; sm.mg.l[wave][mq][lane] = l_run[mq]; }
    float mw[MQ], lw[MQ];               // merged running max and sum of the workgroup
    f32x4 ow[HPW][MQ];                  // merged accumulators of head tiles wave + 4*hh
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh) {
        if (hh > 0) __syncthreads();    // everyone has read the previous round
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int mq = 0; mq < MQ; ++mq) sm.mg.o[wave][j * MQ + mq][lane] = o[4 * hh + j][mq];
        __syncthreads();
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            float mv[4], f[4];
            float mn = -INFINITY;
#pragma unroll
            for (int w = 0; w < 4; ++w) { mv[w] = sm.mg.m[w][mq][lane]; mn = fmaxf(mn, mv[w]); }
            float l = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                f[w] = (mv[w] == -INFINITY) ? 0.f : __expf(mv[w] - mn);
                l += f[w] * sm.mg.l[w][mq][lane];
            }
            mw[mq] = mn;
            lw[mq] = l;
            f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int w = 0; w < 4; ++w) acc += sm.mg.o[w][wave * MQ + mq][lane] * f[w];
            ow[hh][mq] = acc;
        }
    }
    ATTN_STAMP(6);

    auto write_out = [&](int mq, int ht, const float (&v)[4]) {
        if (rowvalid[mq]) {
            const int row = bi * rps + jrow[mq];
            Traits<T>::store_split4(attn_out + opnd_off<T>(row, (kvh * md.G + girow[mq]) * HD + ht * 16 + 4 * g, md.Hq * HD, otks), aplane, v);
        }
    };

    if (nch == 1) {
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            const float inv = 1.f / lw[mq];
#pragma unroll
            for (int hh = 0; hh < HPW; ++hh) {
                const float v[4] = {ow[hh][mq][0] * inv, ow[hh][mq][1] * inv, ow[hh][mq][2] * inv, ow[hh][mq][3] * inv};
                write_out(mq, wave + 4 * hh, v);
            }
        }
        return;
    }

    // ---------------- several key ranges: publish, draw a ticket, the last one merges ----------------
    constexpr int PF = attn_partial_floats<HD, MQ>();
    const size_t group = ((size_t)bi * md.Hkv + kvh) * qgroups + qg;
    float* mine = opart + (group * nchunk_max + chunk) * PF;
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq)
#pragma unroll
            for (int i = 0; i < 4; ++i) st_coh(mine + (((wave + 4 * hh) * MQ + mq) * 4 + i) * 64 + lane, ow[hh][mq][i]);
    if (wave == 0) {
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            st_coh(mine + (NSLOT + mq) * 64 + lane, mw[mq]);
            st_coh(mine + (NSLOT + MQ + mq) * 64 + lane, lw[mq]);
        }
    }
    ATTN_STAMP(7);
    wait_vm0();                         // this wave's write-through stores are acknowledged ..
    __syncthreads();                    // .. and so are the other waves', before the ticket is drawn
    if (tid == 0) {
        const unsigned t = __hip_atomic_fetch_add(&tickets[group], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        sm.last = (t == (unsigned)(nch - 1));
    }
    ATTN_STAMP(8);
    __syncthreads();
    ATTN_STAMP(9);
    if (!sm.last) return;

    // ranges in order, CB per batch of independent loads, running maximum carried across batches
    const float* base = opart + group * nchunk_max * PF;
    constexpr int CB = (MQ <= 2) ? 8 : (MQ == 3 ? 4 : 2);
    float mx[MQ], den[MQ], num[HPW][MQ][4];
#pragma unroll
    for (int mq = 0; mq < MQ; ++mq) {
        mx[mq] = -INFINITY;
        den[mq] = 0.f;
#pragma unroll
        for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
            for (int i = 0; i < 4; ++i) num[hh][mq][i] = 0.f;
    }
    for (int c0 = 0; c0 < nch; c0 += CB) {
        float mv[CB][MQ], lv[CB][MQ], ov[CB][HPW][MQ][4];
#pragma unroll
        for (int u = 0; u < CB; ++u) {
            const float* pc = base + (size_t)min(c0 + u, nch - 1) * PF;
#pragma unroll
            for (int mq = 0; mq < MQ; ++mq) {
                mv[u][mq] = ld_coh(pc + (NSLOT + mq) * 64 + lane);
                lv[u][mq] = ld_coh(pc + (NSLOT + MQ + mq) * 64 + lane);
#pragma unroll
                for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
                    for (int i = 0; i < 4; ++i) ov[u][hh][mq][i] = ld_coh(pc + (((wave + 4 * hh) * MQ + mq) * 4 + i) * 64 + lane);
            }
        }
        if (c0 == 0) ATTN_STAMP(10);
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            float bm = mx[mq];
#pragma unroll
            for (int u = 0; u < CB; ++u) bm = fmaxf(bm, (c0 + u < nch) ? mv[u][mq] : -INFINITY);
            const float resc = (mx[mq] == -INFINITY) ? 0.f : __expf(mx[mq] - bm);
            mx[mq] = bm;
            den[mq] *= resc;
#pragma unroll
            for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
                for (int i = 0; i < 4; ++i) num[hh][mq][i] *= resc;
#pragma unroll
            for (int u = 0; u < CB; ++u) {
                const float f = (c0 + u < nch && mv[u][mq] != -INFINITY) ? __expf(mv[u][mq] - bm) : 0.f;
                den[mq] += f * lv[u][mq];
#pragma unroll
                for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
                    for (int i = 0; i < 4; ++i) num[hh][mq][i] += f * ov[u][hh][mq][i];
            }
        }
    }
    ATTN_STAMP(11);
#pragma unroll
    for (int hh = 0; hh < HPW; ++hh)
#pragma unroll
        for (int mq = 0; mq < MQ; ++mq) {
            const float inv = 1.f / den[mq];
            const float v[4] = {num[hh][mq][0] * inv, num[hh][mq][1] * inv, num[hh][mq][2] * inv, num[hh][mq][3] * inv};
            write_out(mq, wave + 4 * hh, v);
        }
    ATTN_STAMP(12);
    if (tid == 0) st_coh(&tickets[group], 0u);   // ready for the next launch
}

}  // namespace sj
