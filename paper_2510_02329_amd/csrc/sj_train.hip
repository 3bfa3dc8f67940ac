// Training of the judge verifier on the device (paper Sec. 3.4 "Verifier Training" and appendix
// "Training Logistic Regressor"): L2-regularised logistic regression on (hidden state, label) pairs
// for every C of a grid, model selection by validation ROC-AUC, thresholds with the best F1 and the
// best recall.
//
//   f(w, b) = 1/2 |w|^2 + C sum_i log(1 + exp(-t_i (w.h_i + b))),  t_i = 2 y_i - 1   (bias unpenalised)
//
// f is strictly convex, so any solver reaches the same optimum; this one is a truncated Newton
// method: conjugate gradients on the Newton system, every gradient and every Hessian-vector product
// being ONE pass over the feature matrix (the only large object: n x d floats, HBM-bound):
//   per row i:  z_i = h_i . x + x_b;   c_i = sigmoid(z_i) - y_i   (gradient at x)
//                                   or c_i = D_i z_i,  D_i = s_i (1 - s_i)   (Hessian times x)
//   out += c_i h_i,  out_b += c_i
// A workgroup holds four rows in registers at a time (the next four are requested before the current
// ones are used); the dot products are reduced across it and the same registers feed the update of
// the accumulators - the matrix is read once per pass.  All arithmetic is fp64 on the
// fp32 features (the pass stays HBM-bound: 2 fp64 FMAs per 4 bytes).  Sums are taken in a fixed order
// (rows of a workgroup, lanes, waves, workgroups), so a run is bit-reproducible.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <vector>

#include "../../include/sj.h"

__attribute__((visibility("hidden"))) int sj_set_error(int code, const char* msg);   // defined next to sj_last_error

namespace {

int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    return sj_set_error(code, buf);
}

#define HIPCHK(expr)                                                                              \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail(SJ_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
    } while (0)
#define LAUNCHCHK(name)                                                                          \
    do {                                                                                         \
        hipError_t e_ = hipGetLastError();                                                       \
        if (e_ != hipSuccess) return fail(SJ_EHIP, "launch of %s failed: %s", name, hipGetErrorString(e_)); \
    } while (0)

constexpr int PASS_WG = 256;        // workgroups of a pass: one per compute unit
constexpr int PASS_WAVES = 4;
enum { PASS_GRAD = 0, PASS_HESS = 1, PASS_SCORE = 2 };

struct PassArgs {
    const float* H;        // [n][d]
    const int32_t* y;      // [n] labels (gradient pass)
    double* D;             // [n] s (1 - s): written by the gradient pass, read by the Hessian pass
    const double* x;       // [d + 1] point (gradient) or direction (Hessian); entry d = bias
    double* partial;       // [PASS_WG][d + 2]: sum c h, sum c, sum of losses
    double* z_out;         // [n] (score pass)
    long long n;
    int d;
};

// Workgroup barrier that waits for this wave's LDS traffic only: __syncthreads() would also wait for the
// next rows' loads, which are meant to stay in flight across the barriers of the current rows.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// One pass over the matrix.  A workgroup of four waves takes four rows (two when d > 4096) at a time; wave w owns the
// columns [w * NJW * 256, (w + 1) * NJW * 256): lane l holds elements 4l .. 4l + 3 of each of its NJW
// 256-column pieces, so every load instruction of a wave covers 1 KB of consecutive memory, and its
// slice of x and of the accumulator stays in registers.  Per group of rows: partial dot products of
// the four rows -> LDS -> wave w finishes row w (sigmoid / loss / D) -> LDS -> every wave updates its
// columns with the four coefficients.  The next group's loads are issued before the current group is
// used.  Columns at or past d are loaded from a clamped address and meet x = 0; their accumulators
// are never stored.
template <int NJW, int MODE>
__global__ __launch_bounds__(256) void lr_pass_kernel(PassArgs a) {
    constexpr int RB = NJW > 4 ? 2 : 4;                  // rows per group (wide rows: fewer, to stay in registers)
    __shared__ double part[2][PASS_WAVES][RB];           // [parity][column owner][row]
    __shared__ double coef[2][RB];
    __shared__ double tail[PASS_WAVES][2];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;

    int off[NJW];
    double xr[NJW][4], acc[NJW][4];
#pragma unroll
    for (int j = 0; j < NJW; ++j) {
        const int e = (w * NJW + j) * 256 + lane * 4;
        off[j] = min(e, a.d - 4);
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            xr[j][k] = e + k < a.d ? a.x[e + k] : 0.0;
            acc[j][k] = 0.0;
        }
    }
    const double xb = a.x[a.d];
    double accb = 0.0, loss = 0.0;

    const long long ngroups = (a.n + RB - 1) / RB;
    float4 bufA[RB][NJW], bufB[RB][NJW];
    double auxA = 0.0, auxB = 0.0;                       // of row w of the group (label or D)
    auto load = [&](float4 (&buf)[RB][NJW], double& aux, long long grp) {
        const long long g = grp < ngroups ? grp : ngroups - 1;   // groups past the end re-read the last (not used)
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const long long i = g * RB + rb;
            const float* row = a.H + (i < a.n ? i : a.n - 1) * a.d;
#pragma unroll
            for (int j = 0; j < NJW; ++j) buf[rb][j] = *reinterpret_cast<const float4*>(row + off[j]);
        }
        const int wr = w < RB ? w : RB - 1;
        const long long iw = g * RB + wr < a.n ? g * RB + wr : a.n - 1;
        if constexpr (MODE == PASS_GRAD) aux = (double)a.y[iw];
        if constexpr (MODE == PASS_HESS) aux = a.D[iw];
    };
    auto process = [&](const float4 (&buf)[RB][NJW], double aux, long long grp, int par) {
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            double dot = 0.0;
#pragma unroll
            for (int j = 0; j < NJW; ++j)
                dot += (double)buf[rb][j].x * xr[j][0] + (double)buf[rb][j].y * xr[j][1] + (double)buf[rb][j].z * xr[j][2] +
                       (double)buf[rb][j].w * xr[j][3];
            dot = wave_sum(dot);
            if (lane == 0) part[par][w][rb] = dot;
        }
        lds_barrier();
        if (w < RB) {   // wave w finishes row w of the group (wave-uniform)
            const long long i = grp * RB + w;
            const double z = part[par][0][w] + part[par][1][w] + part[par][2][w] + part[par][3][w] + xb;
            double c = 0.0;
            if (i < a.n) {                               // wave-uniform
                if constexpr (MODE == PASS_GRAD) {
                    const double s = 1.0 / (1.0 + exp(-z));
                    c = s - aux;
                    const double m = aux > 0.5 ? -z : z; // -t z
                    loss += fmax(m, 0.0) + log1p(exp(-fabs(m)));
                    if (lane == 0) a.D[i] = s * (1.0 - s);
                } else if constexpr (MODE == PASS_HESS) {
                    c = aux * z;
                } else {
                    if (lane == 0) a.z_out[i] = z;
                }
            }
            accb += c;
            if (lane == 0) coef[par][w] = c;
        }
        if constexpr (MODE == PASS_SCORE) return;
        lds_barrier();
#pragma unroll
        for (int rb = 0; rb < RB; ++rb) {
            const double c = coef[par][rb];
#pragma unroll
            for (int j = 0; j < NJW; ++j) {
                acc[j][0] += c * (double)buf[rb][j].x;
                acc[j][1] += c * (double)buf[rb][j].y;
                acc[j][2] += c * (double)buf[rb][j].z;
                acc[j][3] += c * (double)buf[rb][j].w;
            }
        }
    };

    // groups blockIdx.x, + gridDim.x, ...: the loop is uniform for the workgroup (barriers inside).  A slot
    // of `part` / `coef` is written again two groups later, after a barrier every wave passes only once
    // all reads of the earlier group are done.
    const long long G = gridDim.x;
    load(bufA, auxA, blockIdx.x);
    for (long long grp = blockIdx.x; grp < ngroups; grp += 2 * G) {
        load(bufB, auxB, grp + G);
        process(bufA, auxA, grp, 0);
        load(bufA, auxA, grp + 2 * G);
        if (grp + G < ngroups) process(bufB, auxB, grp + G, 1);
    }
    if constexpr (MODE == PASS_SCORE) return;

    double* out = a.partial + (size_t)blockIdx.x * (a.d + 2);
#pragma unroll
    for (int j = 0; j < NJW; ++j) {
        const int e = (w * NJW + j) * 256 + lane * 4;
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (e + k < a.d) out[e + k] = acc[j][k];
    }
    if (lane == 0) { tail[w][0] = accb; tail[w][1] = loss; }
    __syncthreads();
    if (tid == 0) {
        double sb = 0.0, sl = 0.0;
        for (int ww = 0; ww < PASS_WAVES; ++ww) { sb += tail[ww][0]; sl += tail[ww][1]; }
        out[a.d] = sb;
        out[a.d + 1] = sl;
    }
}

// raw[e] = sum over workgroups of partial[g][e]  (e <= d + 1), in a fixed order: thread (slice q, column c)
// adds workgroups 16 q .. 16 q + 15 in order, the 16 slice sums are then added in slice order.
__global__ __launch_bounds__(1024) void lr_reduce_kernel(const double* __restrict__ partial, int d, double* __restrict__ raw) {
    static_assert(PASS_WG == 256, "16 slices of 16 workgroups");
    __shared__ double sl[16][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int e = blockIdx.x * 64 + c;
    const int ec = e < d + 2 ? e : d + 1;
    double v[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = partial[(size_t)(q * 16 + i) * (d + 2) + ec];
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += v[i];
    sl[q][c] = s;
    __syncthreads();
    if (q == 0 && e < d + 2) {
        double t = 0.0;
#pragma unroll
        for (int i = 0; i < 16; ++i) t += sl[i][c];
        raw[e] = t;
    }
}

// ---- vector kernels of the solver: one workgroup of 1024 threads over the d + 1 unknowns -------------
struct Status {
    double f, gmax, gg, rr, pq, gs, pad0, pad1;
};

__device__ __forceinline__ double block_sum_1024(double v, double* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t += red[i];
    return t;
}
__device__ __forceinline__ double block_max_1024(double v, double* red) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmax(v, __shfl_xor(v, o, 64));
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    double t = 0.0;
#pragma unroll
    for (int i = 0; i < 16; ++i) t = fmax(t, red[i]);
    return t;
}

// g = (x_w, 0) + C raw;  f = 1/2 |x_w|^2 + C * loss;  gmax = max |g|;  gg = g.g
__global__ __launch_bounds__(1024) void grad_finish_kernel(int d, double C, const double* __restrict__ x,
                                                           const double* __restrict__ raw, double* __restrict__ g,
                                                           Status* __restrict__ st) {
    __shared__ double red[16];
    double ww = 0.0, gg = 0.0, gm = 0.0;
    for (int e = threadIdx.x; e <= d; e += 1024) {
        const double xe = e < d ? x[e] : 0.0;
        const double ge = xe + C * raw[e];
        g[e] = ge;
        ww += xe * xe;
        gg += ge * ge;
        gm = fmax(gm, fabs(ge));
    }
    ww = block_sum_1024(ww, red);
    gg = block_sum_1024(gg, red);
    gm = block_max_1024(gm, red);
    if (threadIdx.x == 0) { st->f = 0.5 * ww + C * raw[d + 1]; st->gmax = gm; st->gg = gg; }
}

// conjugate gradients on  Hess s = -g:  s = 0, r = -g, p = r
__global__ __launch_bounds__(1024) void cg_init_kernel(int d, const double* __restrict__ g, double* __restrict__ s,
                                                       double* __restrict__ r, double* __restrict__ p, Status* __restrict__ st) {
    for (int e = threadIdx.x; e <= d; e += 1024) { s[e] = 0.0; r[e] = -g[e]; p[e] = -g[e]; }
    if (threadIdx.x == 0) st->rr = st->gg;
}

// q = (p_w, 0) + C raw  (Hessian times p);  alpha = rr / p.q;  s += alpha p;  r -= alpha q;
// beta = r.r / rr;  p = r + beta p
__global__ __launch_bounds__(1024) void cg_step_kernel(int d, double C, const double* __restrict__ raw, double* __restrict__ s,
                                                       double* __restrict__ r, double* __restrict__ p, Status* __restrict__ st) {
    __shared__ double red[16];
    double pq = 0.0;
    for (int e = threadIdx.x; e <= d; e += 1024) {
        const double pe = p[e];
        pq += pe * ((e < d ? pe : 0.0) + C * raw[e]);
    }
    pq = block_sum_1024(pq, red);
    const double rr = st->rr;
    const double alpha = pq > 0.0 ? rr / pq : 0.0;
    double rn = 0.0;
    for (int e = threadIdx.x; e <= d; e += 1024) {
        const double pe = p[e];
        const double qe = (e < d ? pe : 0.0) + C * raw[e];
        s[e] += alpha * pe;
        const double re = r[e] - alpha * qe;
        r[e] = re;
        rn += re * re;
    }
    rn = block_sum_1024(rn, red);
    const double beta = rr > 0.0 ? rn / rr : 0.0;
    for (int e = threadIdx.x; e <= d; e += 1024) p[e] = r[e] + beta * p[e];
    __syncthreads();                                       // everyone has read st->rr
    if (threadIdx.x == 0) { st->rr = rn; st->pq = pq; }
}

// xt = x + alpha s;  gs = g.s
__global__ __launch_bounds__(1024) void trial_kernel(int d, double alpha, const double* __restrict__ x, const double* __restrict__ s,
                                                     const double* __restrict__ g, double* __restrict__ xt, Status* __restrict__ st) {
    __shared__ double red[16];
    double gs = 0.0;
    for (int e = threadIdx.x; e <= d; e += 1024) {
        xt[e] = x[e] + alpha * s[e];
        gs += g[e] * s[e];
    }
    gs = block_sum_1024(gs, red);
    if (threadIdx.x == 0) st->gs = gs;
}

// ---- validation: ROC-AUC by its pair definition, F1 of every candidate threshold --------------------
// Candidate i < n is theta = score_i, candidate n is theta = 0.  For each candidate:
//   tp = #{acceptable j: score_j > theta},  fp = #{unacceptable j: score_j > theta};
// for an acceptable sample i also  below2 = 2 #{unacceptable j: score_j < score_i} + #{... == score_i}.
__global__ __launch_bounds__(256) void val_scores_kernel(long long n, const double* __restrict__ z, double* __restrict__ score) {
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    if (i < n) score[i] = 1.0 / (1.0 + exp(-z[i]));
}

__global__ __launch_bounds__(256) void val_count_kernel(long long n, const double* __restrict__ score, const int32_t* __restrict__ y,
                                                        int want_f1, int32_t* __restrict__ tp, int32_t* __restrict__ fp,
                                                        long long* __restrict__ below2) {
    __shared__ double ss[256];
    __shared__ int32_t ys[256];
    const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
    const double si = i < n ? score[i] : 0.0;              // candidate n: theta = 0
    const bool pos_i = i < n && y[i] != 0;
    int ctp = 0, cfp = 0;
    long long b2 = 0;
    // blockIdx.y takes every gridDim.y-th tile of j; the counts are integers, so the order of the atomic
    // additions does not matter
    for (long long j0 = (long long)blockIdx.y * 256; j0 < n; j0 += 256LL * gridDim.y) {
        __syncthreads();
        const long long j = j0 + threadIdx.x;
        ss[threadIdx.x] = j < n ? score[j] : -1.0;         // scores are in [0, 1]: -1 never counts
        ys[threadIdx.x] = j < n ? y[j] : -1;
        __syncthreads();
        const int m = (int)((n - j0) < 256 ? (n - j0) : 256);
        for (int k = 0; k < m; ++k) {
            const double sj = ss[k];
            const bool pj = ys[k] != 0;
            if (want_f1) { ctp += (pj && sj > si); cfp += (!pj && sj > si); }
            if (!pj) b2 += (sj < si) ? 2 : (sj == si ? 1 : 0);
        }
    }
    if (i <= n && want_f1) { atomicAdd(&tp[i], ctp); atomicAdd(&fp[i], cfp); }
    if (i < n && pos_i) atomicAdd(reinterpret_cast<unsigned long long*>(&below2[i]), (unsigned long long)b2);
}

struct ValResult {
    unsigned long long auc2;      // 2 * (pairs ordered correctly) + ties
    long long n_pos, n_neg;
    double f1, theta_f1, theta_recall;
};

__global__ __launch_bounds__(1024) void val_select_kernel(long long n, const double* __restrict__ score, const int32_t* __restrict__ y,
                                                          int want_f1, const int32_t* __restrict__ tp, const int32_t* __restrict__ fp,
                                                          const long long* __restrict__ below2, ValResult* __restrict__ out) {
    __shared__ unsigned long long s_auc[1024];
    __shared__ long long s_pos[1024];
    __shared__ double s_f1[1024], s_th[1024], s_neg[1024];
    unsigned long long auc2 = 0;
    long long npos = 0;
    double negmax = 0.0;
    for (long long i = threadIdx.x; i < n; i += 1024) {
        auc2 += (unsigned long long)below2[i];
        npos += y[i] != 0;
        if (y[i] == 0) negmax = fmax(negmax, score[i]);
    }
    s_auc[threadIdx.x] = auc2; s_pos[threadIdx.x] = npos; s_neg[threadIdx.x] = negmax;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) {
            s_auc[threadIdx.x] += s_auc[threadIdx.x + o];
            s_pos[threadIdx.x] += s_pos[threadIdx.x + o];
            s_neg[threadIdx.x] = fmax(s_neg[threadIdx.x], s_neg[threadIdx.x + o]);
        }
        __syncthreads();
    }
    const long long total_pos = s_pos[0];
    // best F1, the smallest threshold among equals: F1 = 2 tp / (2 tp + fp + fn), fn = n_pos - tp
    double bf = -1.0, bt = 0.0;
    if (want_f1)
        for (long long i = threadIdx.x; i <= n; i += 1024) {
            const double t = (double)tp[i];
            const double f1 = tp[i] == 0 ? 0.0 : 2.0 * t / (2.0 * t + (double)fp[i] + (double)(total_pos - tp[i]));
            const double th = i < n ? score[i] : 0.0;
            if (f1 > bf || (f1 == bf && th < bt)) { bf = f1; bt = th; }
        }
    s_f1[threadIdx.x] = bf; s_th[threadIdx.x] = bt;
    __syncthreads();
    for (int o = 512; o > 0; o >>= 1) {
        if (threadIdx.x < o) {
            const double f1 = s_f1[threadIdx.x + o], th = s_th[threadIdx.x + o];
            if (f1 > s_f1[threadIdx.x] || (f1 == s_f1[threadIdx.x] && th < s_th[threadIdx.x])) { s_f1[threadIdx.x] = f1; s_th[threadIdx.x] = th; }
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        out->auc2 = s_auc[0];
        out->n_pos = total_pos;
        out->n_neg = n - total_pos;
        out->f1 = s_f1[0];
        out->theta_f1 = s_th[0];
        out->theta_recall = s_neg[0];
    }
}

// ---- host side -----------------------------------------------------------------------------------------
struct Work {
    std::vector<void*> allocs;
    ~Work() { for (void* p : allocs) (void)hipFree(p); }
    template <typename T> int get(T*& p, size_t count) {
        void* q = nullptr;
        hipError_t e = hipMalloc(&q, count * sizeof(T));
        if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? SJ_ENOMEM : SJ_EHIP, "hipMalloc(%zu) failed: %s", count * sizeof(T), hipGetErrorString(e));
        allocs.push_back(q);
        p = static_cast<T*>(q);
        return SJ_OK;
    }
};

template <int MODE>
int launch_pass(int d, const PassArgs& a, hipStream_t st) {
    const int nj = (d + 1023) / 1024;                   // 256-column pieces per wave
#define SJ_PASS(NJ)                                                                                   \
    if (nj <= NJ) {                                                                                   \
        lr_pass_kernel<NJ, MODE><<<PASS_WG, 256, 0, st>>>(a);                                         \
        LAUNCHCHK("lr_pass");                                                                         \
        return SJ_OK;                                                                                 \
    }
    SJ_PASS(1) SJ_PASS(2) SJ_PASS(3) SJ_PASS(4) SJ_PASS(6) SJ_PASS(8)
#undef SJ_PASS
    return fail(SJ_EINVAL, "d = %d above 8192 is not supported", d);
}

struct Solver {
    hipStream_t st;
    int d;
    long long n;
    const float* H;
    const int32_t* y;
    double *D, *partial, *raw, *x, *xt, *g, *gt, *s, *r, *p;
    Status* status;
    Status host;

    int read_status() {
        HIPCHK(hipMemcpyAsync(&host, status, sizeof(Status), hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        return SJ_OK;
    }
    int reduce() {
        lr_reduce_kernel<<<(d + 2 + 63) / 64, 1024, 0, st>>>(partial, d, raw);
        LAUNCHCHK("lr_reduce");
        return SJ_OK;
    }
    // f, g at `at`; fills D
    int gradient(double C, const double* at, double* gout) {
        PassArgs a{H, y, D, at, partial, nullptr, n, d};
        int rc;
        if ((rc = launch_pass<PASS_GRAD>(d, a, st))) return rc;
        if ((rc = reduce())) return rc;
        grad_finish_kernel<<<1, 1024, 0, st>>>(d, C, at, raw, gout, status);
        LAUNCHCHK("grad_finish");
        return SJ_OK;
    }
    int hess_pass(const double* dir) {
        PassArgs a{H, nullptr, D, dir, partial, nullptr, n, d};
        int rc;
        if ((rc = launch_pass<PASS_HESS>(d, a, st))) return rc;
        return reduce();
    }

    // Truncated Newton from x = 0.  Stops when max |g| <= tol * max(1, C n).
    int fit(double C, int* iters_out, int* converged) {
        int rc;
        HIPCHK(hipMemsetAsync(x, 0, (size_t)(d + 1) * sizeof(double), st));
        if ((rc = gradient(C, x, g))) return rc;
        if ((rc = read_status())) return rc;
        const double tol = 1e-11 * fmax(1.0, C * (double)n);
        double g0 = sqrt(host.gg);
        *converged = 0;
        int it = 0, passes = 0;
        for (; it < 100; ++it) {
            if (host.gmax <= tol) { *converged = 1; break; }
            const double f = host.f, gnorm = sqrt(host.gg);
            // inexact Newton: the system is solved to a tolerance that tightens with the gradient
            const double eta = fmin(0.1, sqrt(gnorm / fmax(g0, 1e-300)));
            cg_init_kernel<<<1, 1024, 0, st>>>(d, g, s, r, p, status);
            LAUNCHCHK("cg_init");
            for (int k = 0; k < 4 * (d + 1) + 50; ++k) {
                if ((rc = hess_pass(p))) return rc;
                cg_step_kernel<<<1, 1024, 0, st>>>(d, C, raw, s, r, p, status);
                LAUNCHCHK("cg_step");
                if ((rc = read_status())) return rc;
                ++passes;
                if (sqrt(host.rr) <= eta * gnorm || host.pq <= 0.0) break;
            }
            double alpha = 1.0;
            bool moved = false;
            for (int ls = 0; ls < 40; ++ls) {
                trial_kernel<<<1, 1024, 0, st>>>(d, alpha, x, s, g, xt, status);
                LAUNCHCHK("trial");
                if ((rc = gradient(C, xt, gt))) return rc;
                if ((rc = read_status())) return rc;
                ++passes;
                // near the optimum the decrease is below the rounding of f: take the step
                if (host.f <= f + 1e-4 * alpha * host.gs || fabs(host.gs) <= 1e-9 * fabs(f)) { moved = true; break; }
                alpha *= 0.5;
            }
            if (!moved) break;                               // no descent within rounding: the point is kept
            std::swap(x, xt);
            std::swap(g, gt);                                // status already describes the new point
        }
        if (iters_out) *iters_out = passes;
        return SJ_OK;
    }
};

}  // namespace

extern "C" int sj_judge_train(const float* H_train, const int32_t* y_train, int64_t n_train, const float* H_val,
                              const int32_t* y_val, int64_t n_val, int32_t d, const double* C_grid, int32_t n_C,
                              double* w_all, double* auc, int32_t* passes, int32_t* best_index, double* w_best,
                              double* theta_f1, double* theta_recall, void* stream) {
    if (!H_train || !y_train || !H_val || !y_val || !C_grid || !auc || !best_index || !w_best || !theta_f1 || !theta_recall)
        return fail(SJ_EINVAL, "null argument");
    if (n_train < 2 || n_val < 2 || n_C < 1) return fail(SJ_EINVAL, "need at least two samples per set and one C");
    if (n_val > (1 << 24)) return fail(SJ_EINVAL, "validation set above 2^24 samples is not supported");
    if (d < 4 || d % 4 || d > 8192) return fail(SJ_EINVAL, "d must be a multiple of 4 in 4 .. 8192");
    if (((uintptr_t)H_train | (uintptr_t)H_val) & 15) return fail(SJ_EINVAL, "feature matrices must be 16-byte aligned");
    for (int c = 0; c < n_C; ++c)
        if (!(C_grid[c] > 0.0) || !std::isfinite(C_grid[c])) return fail(SJ_EINVAL, "C[%d] must be positive and finite", c);
    hipStream_t st = (hipStream_t)stream;

    // labels: 0 / 1, both classes in both sets (the optimum does not exist otherwise)
    std::vector<int32_t> lab((size_t)(n_train > n_val ? n_train : n_val));
    for (int pass = 0; pass < 2; ++pass) {
        const int64_t n = pass ? n_val : n_train;
        HIPCHK(hipMemcpyAsync(lab.data(), pass ? y_val : y_train, (size_t)n * 4, hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        int64_t ones = 0;
        for (int64_t i = 0; i < n; ++i) {
            if (lab[i] != 0 && lab[i] != 1) return fail(SJ_EINVAL, "label %lld of the %s set is %d (must be 0 or 1)", (long long)i, pass ? "validation" : "training", lab[i]);
            ones += lab[i];
        }
        if (ones == 0 || ones == n) return fail(SJ_EINVAL, "the %s set holds one class only", pass ? "validation" : "training");
    }

    Work wk;
    Solver sv{};
    sv.st = st; sv.d = d; sv.n = n_train; sv.H = H_train; sv.y = y_train;
    int rc;
    const size_t nv = (size_t)d + 2;
    if ((rc = wk.get(sv.D, (size_t)n_train))) return rc;
    if ((rc = wk.get(sv.partial, (size_t)PASS_WG * nv))) return rc;
    if ((rc = wk.get(sv.raw, nv)) || (rc = wk.get(sv.x, nv)) || (rc = wk.get(sv.xt, nv)) || (rc = wk.get(sv.g, nv)) ||
        (rc = wk.get(sv.gt, nv)) || (rc = wk.get(sv.s, nv)) || (rc = wk.get(sv.r, nv)) || (rc = wk.get(sv.p, nv)))
        return rc;
    if ((rc = wk.get(sv.status, 1))) return rc;
    double *zval, *score, *xbest;
    int32_t *tp, *fp;
    long long* below2;
    ValResult* vres;
    if ((rc = wk.get(zval, (size_t)n_val)) || (rc = wk.get(score, (size_t)n_val)) || (rc = wk.get(xbest, nv)) ||
        (rc = wk.get(tp, (size_t)n_val + 1)) || (rc = wk.get(fp, (size_t)n_val + 1)) || (rc = wk.get(below2, (size_t)n_val)) ||
        (rc = wk.get(vres, 1)))
        return rc;

    auto validate = [&](const double* xdev, int want_f1, ValResult* host_res) -> int {
        PassArgs a{H_val, nullptr, nullptr, xdev, nullptr, zval, (long long)n_val, d};
        int rc2;
        if ((rc2 = launch_pass<PASS_SCORE>(d, a, st))) return rc2;
        val_scores_kernel<<<(unsigned)((n_val + 255) / 256), 256, 0, st>>>(n_val, zval, score);
        LAUNCHCHK("val_scores");
        HIPCHK(hipMemsetAsync(tp, 0, (size_t)(n_val + 1) * 4, st));
        HIPCHK(hipMemsetAsync(fp, 0, (size_t)(n_val + 1) * 4, st));
        HIPCHK(hipMemsetAsync(below2, 0, (size_t)n_val * 8, st));
        const unsigned xb = (unsigned)((n_val + 1 + 255) / 256);
        const unsigned yb = xb >= 1024 ? 1 : (1024 + xb - 1) / xb;       // about 1024 workgroups in all
        val_count_kernel<<<dim3(xb, yb), 256, 0, st>>>(n_val, score, y_val, want_f1, tp, fp, below2);
        LAUNCHCHK("val_count");
        val_select_kernel<<<1, 1024, 0, st>>>(n_val, score, y_val, want_f1, tp, fp, below2, vres);
        LAUNCHCHK("val_select");
        HIPCHK(hipMemcpyAsync(host_res, vres, sizeof(ValResult), hipMemcpyDeviceToHost, st));
        HIPCHK(hipStreamSynchronize(st));
        return SJ_OK;
    };

    int best = -1;
    unsigned long long best_auc2 = 0;
    for (int c = 0; c < n_C; ++c) {
        int np = 0, conv = 0;
        if ((rc = sv.fit(C_grid[c], &np, &conv))) return rc;
        if (!conv) return fail(SJ_EHIP, "the solver did not converge for C[%d] = %g", c, C_grid[c]);
        if (passes) passes[c] = np;
        if (w_all) {
            HIPCHK(hipMemcpyAsync(w_all + (size_t)c * (d + 1), sv.x, (size_t)(d + 1) * sizeof(double), hipMemcpyDeviceToHost, st));
            HIPCHK(hipStreamSynchronize(st));
        }
        ValResult vr{};
        if ((rc = validate(sv.x, 0, &vr))) return rc;
        auc[c] = (double)vr.auc2 / (2.0 * (double)vr.n_pos * (double)vr.n_neg);
        if (best < 0 || vr.auc2 > best_auc2) {               // equal AUC keeps the earlier C
            best = c;
            best_auc2 = vr.auc2;
            HIPCHK(hipMemcpyAsync(xbest, sv.x, (size_t)(d + 1) * sizeof(double), hipMemcpyDeviceToDevice, st));
        }
    }
    ValResult vr{};
    if ((rc = validate(xbest, 1, &vr))) return rc;
    HIPCHK(hipMemcpyAsync(w_best, xbest, (size_t)(d + 1) * sizeof(double), hipMemcpyDeviceToHost, st));
    HIPCHK(hipStreamSynchronize(st));
    *best_index = best;
    *theta_f1 = vr.theta_f1;
    *theta_recall = vr.theta_recall;
    return SJ_OK;
}
