// HIP kernels of the verification step.  Each kernel cites the part of the method it carries out
// (paper "Method": Eq. 2 / Eq. 4 target forward, Eq. 3 ratio test, Eq. 5 judge, Sec. 3.1 scan and
// extra token, Sec. 2.2 residual resampling).  Workgroups are 256 threads unless noted.
#pragma once
#include "sj_types.h"

namespace sj {

// ---------------------------------------------------------------------------------------------
// Weight re-tiling (model load).  Row-major W[N][K] -> tiles [N/16][K/KSTEP][64 lanes][16 bytes]
// in MFMA A-operand order, so that one wave-wide 16-byte load reads 1 KB of contiguous memory.
// interleave = 1 (stacked [gate; up] source, N = 2F): destination tile t holds gate rows
// 8t..8t+7 in its rows 0-7 and up rows 8t..8t+7 in its rows 8-15, so every tile carries both
// projections of 8 FFN columns and SwiGLU can be applied inside the tile's own epilogue.
template <typename T>
__global__ void retile_kernel(const T* __restrict__ src, T* __restrict__ dst, int N, int K, int interleave) {
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    const int KS = K / KSTEP;
    const size_t total = (size_t)(N / 16) * KS * 64;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int lane = (int)(idx & 63);
        const size_t tile = idx >> 6;
        const int ks = (int)(tile % KS);
        const int nt = (int)(tile / KS);
        const int r = lane & 15, g = lane >> 4;
        const int srow = interleave ? ((r >> 3) * (N / 2) + nt * 8 + (r & 7)) : nt * 16 + r;
        const u32x4* s = reinterpret_cast<const u32x4*>(src + (size_t)srow * K + ks * KSTEP + g * KF);
        reinterpret_cast<u32x4*>(dst)[idx] = *s;
    }
}

// K/V upload of one (seq, layer): host layout [Hkv][len][hd] -> K [Hkv][cap][hd], V [Hkv][hd][cap].
template <typename T>
__global__ void kv_scatter_kernel(const T* __restrict__ ksrc, const T* __restrict__ vsrc, T* __restrict__ K,
                                  T* __restrict__ V, int Hkv, int len, int cap, int hd) {
    const size_t total = (size_t)Hkv * len * hd;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int dcol = (int)(idx % hd);
        const int pos = (int)((idx / hd) % len);
        const int h = (int)(idx / ((size_t)hd * len));
        K[((size_t)h * cap + pos) * hd + dcol] = ksrc[idx];
        V[((size_t)h * hd + dcol) * cap + pos] = vsrc[idx];
    }
}

template <typename T>
__global__ void kv_gather_kernel(T* __restrict__ kdst, T* __restrict__ vdst, const T* __restrict__ K,
                                 const T* __restrict__ V, int Hkv, int pos0, int n, int cap, int hd) {
    const size_t total = (size_t)Hkv * n * hd;
    for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total;
         idx += (size_t)gridDim.x * blockDim.x) {
        const int dcol = (int)(idx % hd);
        const int pos = pos0 + (int)((idx / hd) % n);
        const int h = (int)(idx / ((size_t)hd * n));
        kdst[idx] = K[((size_t)h * cap + pos) * hd + dcol];
        vdst[idx] = V[((size_t)h * hd + dcol) * cap + pos];
    }
}

// Caller-supplied hidden states [R][d] (storage dtype) -> operand plane 0 in the layout the LM-head kernel
// reads (opnd_off), and their fp32 copy for the judge.  One thread per 4 consecutive columns.
template <typename T>
__global__ __launch_bounds__(256) void hidden_in_kernel(const T* __restrict__ src, T* __restrict__ xn, float* __restrict__ hn32,
                                                        int R, int d, int tks) {
    const size_t n4 = (size_t)R * d / 4;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += (size_t)gridDim.x * blockDim.x) {
        const int row = (int)(i / (d / 4)), k = (int)(i % (d / 4)) * 4;
        T* out = xn + opnd_off<T>(row, k, d, tks);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const T v = src[(size_t)row * d + k + e];
            out[e] = v;
            hn32[(size_t)row * d + k + e] = Traits<T>::load(&v);
        }
    }
}

__global__ void set_params_kernel(StepParams p, StepParams* dst) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = p;
}

__global__ void set_state_kernel(int32_t* len, int32_t* pending, int seq, int l, int p) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { len[seq] = l; pending[seq] = p; }
}

// ---------------------------------------------------------------------------------------------
// Step start (Eq. 2 input): one workgroup per query row.  Resolves the row's token and position,
// gathers its embedding into the fp32 residual stream and writes the row's rotary cos/sin table
// (angle = pos * base^(-2i/hd), evaluated in double so the table is correctly rounded fp32).
template <typename T>
__global__ __launch_bounds__(256) void step_begin_kernel(const StepParams* __restrict__ sp, ModelDims md,
                                                         const T* __restrict__ embed, const int32_t* __restrict__ len,
                                                         const int32_t* __restrict__ pending, float* __restrict__ x,
                                                         float* __restrict__ cs, int32_t* __restrict__ row_tok,
                                                         double log_base) {
    const int r = blockIdx.x;
    const int rps = sp->rps;
    const int bi = r / rps, j = r % rps;
    const int b = sp->seq_base + bi;
    int tok;
    if (sp->tok_mode == 1) tok = sp->prefill_tokens[j];
    else if (sp->tok_mode == 2) tok = sp->draft_tokens[bi * rps + j];
    else tok = (j == 0) ? pending[b] : sp->draft_tokens[bi * sp->gamma + (j - 1)];
    tok = min(max(tok, 0), md.V - 1);
    const int pos = len[b] + j;
    if (threadIdx.x == 0) row_tok[r] = tok;
    const T* e = embed + (size_t)tok * md.d;
    for (int c = threadIdx.x; c < md.d; c += 256) x[(size_t)r * md.d + c] = Traits<T>::load(e + c);
    const int half = md.hd >> 1;
    for (int i = threadIdx.x; i < half; i += 256) {
        const double inv_freq = exp(-2.0 * (double)i / (double)md.hd * log_base);
        double s, c;
        sincos((double)pos * inv_freq, &s, &c);
        cs[((size_t)r * half + i) * 2 + 0] = (float)c;
        cs[((size_t)r * half + i) * 2 + 1] = (float)s;
    }
}

// ---------------------------------------------------------------------------------------------
// Residual add + RMSNorm.  x[r] += sum_s part[s][r] (fixed order), then
// xn[r] = x[r] * gain / sqrt(mean(x[r]^2) + eps) as the next GEMM's operand (three planes in bf16),
// optionally also in fp32 (final hidden state for the judge, Eq. 4).
template <typename T, int PB = 8>
__global__ __launch_bounds__(1024) void add_rmsnorm_kernel(int R, int d, float eps, float* __restrict__ x,
                                                           const float* __restrict__ part, int nparts,
                                                           const T* __restrict__ gain, T* __restrict__ xn,
                                                           size_t xplane, float* __restrict__ xn32, int tks) {
    // one workgroup of 1024 threads per row, 4 columns per thread and pass; all loads of a pass are
    // independent.  Rows wider than 16384 columns are not supported (host-checked).
    constexpr int MAXP = 4;
    __shared__ float red[16];
    const int r = blockIdx.x;
    float* xr = x + (size_t)r * d;
    f32x4 v[MAXP];
    float ss = 0.f;
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int c = (p * 1024 + threadIdx.x) * 4;
        v[p] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (c < d) {
            v[p] = *reinterpret_cast<const f32x4*>(xr + c);
            // partials in batches of PB independent loads (index clamped, surplus ignored), added in order
            for (int s0 = 0; s0 < nparts; s0 += PB) {
                f32x4 t[PB];
#pragma unroll
                for (int u = 0; u < PB; ++u)
                    t[u] = *reinterpret_cast<const f32x4*>(part + ((size_t)min(s0 + u, nparts - 1) * R + r) * d + c);
#pragma unroll
                for (int u = 0; u < PB; ++u)
                    if (s0 + u < nparts) v[p] += t[u];
            }
            if (nparts) *reinterpret_cast<f32x4*>(xr + c) = v[p];
            ss += v[p][0] * v[p][0] + v[p][1] * v[p][1] + v[p][2] * v[p][2] + v[p][3] * v[p][3];
        }
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) tot += red[w];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int p = 0; p < MAXP; ++p) {
        const int c = (p * 1024 + threadIdx.x) * 4;
        if (c < d) {
            float y[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) y[i] = v[p][i] * inv * Traits<T>::load(gain + c + i);
            Traits<T>::store_split4(xn + opnd_off<T>(r, c, d, tks), xplane, y);
            if (xn32) *reinterpret_cast<f32x4*>(xn32 + (size_t)r * d + c) = f32x4{y[0], y[1], y[2], y[3]};
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Weight-streaming skinny GEMM: Y[R][N] = X[R][K] * W[N][K]^T with W in the re-tiled layout.
// Every byte of W is read exactly once; X (a few rows) is re-read from cache.
// Workgroup (bx, by): n-tiles [bx*NT, bx*NT+NT), K-slice by of gridDim.y; its 4 waves split that
// slice again and are summed through LDS in wave order (deterministic).
enum { EPI_PARTIAL = 0, EPI_SWIGLU = 1, EPI_LOGITS = 2 };

struct GemmArgs {
    const void* Wt;     // tiled weights
    const void* X;      // [SPL planes][MT*16][ldx] storage dtype, rows >= R are padding
    size_t xplane;      // elements between consecutive planes of X
    size_t actplane;    // same for act
    int32_t ldx, K, N, R;
    int32_t slice_rows; // EPI_PARTIAL: rows between consecutive K-slices of out (>= R)
    float* out;         // EPI_PARTIAL: [gridDim.y][slice_rows][N] fp32;  EPI_LOGITS: [R][N] fp32
    void* act;          // EPI_SWIGLU: [MT*16][N/2] storage dtype = silu(gate) * up
    float4* stats;      // EPI_LOGITS: [R][gridDim.x] (max, sum exp((l-max)/T), argmax as float bits, 0)
    float inv_temp;     // 1/T, 0 when T = 0
    int32_t x_tks;      // 0: X planes are row-major; else K / KSTEP: fragment-tiled planes (opnd_off)
    int32_t act_tks;    // same for act (its K is N/2)
    int32_t rgroups;    // many-row kernel: row groups of one launch (0 or 1: the launch is one group of R rows); with
                        // more, R is the total row count and every workgroup derives its group's rows and pointers
};

// Epilogue of the few-row kernels for one (row, column en of every tile) position: v[t] is the finished sum of tile
// nt0 + t.  Every thread of the first 256 of the workgroup calls it (16 consecutive lanes share a row; rows >= R
// take part in the shuffles and store nothing).
template <typename T, int NT, int EPI>
__device__ __forceinline__ void few_epilogue(const GemmArgs& a, const float (&v)[NT], int row, int en, int nt0) {
    if constexpr (EPI == EPI_PARTIAL) {
        if (row < a.R) {
#pragma unroll
            for (int t = 0; t < NT; ++t)
                a.out[((size_t)blockIdx.y * a.slice_rows + row) * a.N + (size_t)(nt0 + t) * 16 + en] = v[t];
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        // tile column en < 8 is gate of FFN column 8*tile + en, column en + 8 its up projection
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const float up = __shfl_down(v[t], 8, 64);
            if (row < a.R && en < 8) {
                const float gate = v[t];
                const float y = gate / (1.0f + expf(-gate)) * up;
                Traits<T>::store_split(reinterpret_cast<T*>(a.act) + (size_t)row * (a.N / 2) + (size_t)(nt0 + t) * 8 + en,
                                       a.actplane, y);
            }
        }
    } else {
        // logits + this workgroup's softmax partial for the row (16 lanes share a row)
        float mx = v[0];
        int arg = nt0 * 16 + en;
#pragma unroll
        for (int t = 1; t < NT; ++t)
            if (v[t] > mx) { mx = v[t]; arg = (nt0 + t) * 16 + en; }
#pragma unroll
        for (int o = 1; o < 16; o <<= 1) {
            const float omx = __shfl_xor(mx, o, 64);
            const int oarg = __shfl_xor(arg, o, 64);
            if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
        }
        float se = 0.f;
        if (a.inv_temp > 0.f) {
#pragma unroll
            for (int t = 0; t < NT; ++t) se += expf((v[t] - mx) * a.inv_temp);
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) se += __shfl_xor(se, o, 64);
        }
        if (row < a.R) {
#pragma unroll
            for (int t = 0; t < NT; ++t) a.out[(size_t)row * a.N + (size_t)(nt0 + t) * 16 + en] = v[t];
            if (en == 0) a.stats[(size_t)row * gridDim.x + blockIdx.x] = float4{mx, se, __int_as_float(arg), 0.f};
        }
    }
}

#ifdef SJ_GEMM_PROF
__device__ unsigned long long gemm_prof[8192 * 8];
#define GEMM_STAMP(k) do { if ((threadIdx.x & 63) == 0) gemm_prof[(((blockIdx.y * gridDim.x + blockIdx.x) * WAVES + (threadIdx.x >> 6)) & 8191) * 8 + (k)] = wall_clock64(); } while (0)
#else
#define GEMM_STAMP(k) do { } while (0)
#endif

template <typename T, int NT, int MT, int EPI, int SPL, int WAVES, int D = 2>
__global__ __launch_bounds__(WAVES * 64) void gemm_skinny_kernel(GemmArgs a) {
    constexpr int KF = Traits<T>::KF, KSTEP = Traits<T>::KSTEP;
    __shared__ float red[WAVES][NT * MT][256];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int r = lane & 15, g = lane >> 4;
    const int KS = a.K / KSTEP;
    const int nt0 = blockIdx.x * NT;
    const int parts = gridDim.y * WAVES, part = blockIdx.y * WAVES + w;
    const int ks0 = (int)((long long)part * KS / parts), ks1 = (int)((long long)(part + 1) * KS / parts);
    const u32x4* Wt = reinterpret_cast<const u32x4*>(a.Wt) + ((size_t)nt0 * KS + ks0) * 64 + lane;
    // padding rows (>= R) feed columns of D that are never stored: let them re-read row 0 instead of
    // touching more cache lines
    const T* Xr[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = m * 16 + r;
        Xr[m] = reinterpret_cast<const T*>(a.X) + (size_t)(row < a.R ? row : 0) * a.ldx + (size_t)ks0 * KSTEP + g * KF;
    }

    f32x4 acc[NT][MT];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int m = 0; m < MT; ++m) acc[t][m] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Ring of D single-k-step register buffers.  The load of step i + D - 1 is always issued (index
    // clamped to the last step) before step i is consumed, so the loop body is branch-free around the
    // loads - a load under a branch makes the compiler wait for everything outstanding - and the wave
    // keeps D - 1 k-steps of weight tiles in flight, waited for one step at a time.
    Frag fa[D][NT], fb[D][MT][SPL];
    auto load = [&](int buf, int ks) {
#pragma unroll
        for (int t = 0; t < NT; ++t) fa[buf][t].u = __builtin_nontemporal_load(Wt + ((size_t)t * KS + ks) * 64);
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int sp = 0; sp < SPL; ++sp)
                fb[buf][m][sp].u = *reinterpret_cast<const u32x4*>(Xr[m] + sp * a.xplane + (size_t)ks * KSTEP);
    };
    auto compute = [&](int buf) {
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int sp = 0; sp < SPL; ++sp) Traits<T>::mma(fa[buf][t], fb[buf][m][sp], acc[t][m]);
    };
    const int nks = ks1 - ks0;
    GEMM_STAMP(0);
    if (nks > 0) {
#pragma unroll
        for (int j = 0; j < D - 1; ++j) load(j, min(j, nks - 1));
        GEMM_STAMP(1);
        for (int c = 0; c < nks; c += D) {
#pragma unroll
            for (int j = 0; j < D; ++j) {
                load((j + D - 1) % D, min(c + j + D - 1, nks - 1));
                if (c + j < nks) compute(j);
            }
        }
    }

    GEMM_STAMP(2);
    // D[n = 4g+i][row = r]  ->  red[w][tile][row*16 + n]
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[w][t * MT + m][r * 16 + 4 * g + i] = acc[t][m][i];
    __syncthreads();

    GEMM_STAMP(3);
    // the first 256 threads own one (row, column) position of every tile; partial sums are added in
    // wave order
    if (threadIdx.x >= 256) return;
    const int tid = threadIdx.x;
    const int er = tid >> 4, en = tid & 15;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int row = m * 16 + er;
        float v[NT];
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float sum = red[0][t * MT + m][tid];
#pragma unroll
            for (int ww = 1; ww < WAVES; ++ww) sum += red[ww][t * MT + m][tid];
            v[t] = sum;
        }
        few_epilogue<T, NT, EPI>(a, v, row, en, nt0);
    }
}

// ---------------------------------------------------------------------------------------------
// Vocabulary softmax statistics of each row from the LM-head workgroups' partials:
// row max, Z = sum exp((l - max)/T), lowest-index arg-max.  One workgroup per row.
__device__ __forceinline__ void softmax_merge_row(int r, const float4* __restrict__ stats, int nblk, float inv_temp,
                                                  float4* __restrict__ rowstat) {
    __shared__ float smx[4];
    __shared__ int sarg[4];
    __shared__ float red[4];
    const float4* s = stats + (size_t)r * nblk;
    float mx = -INFINITY;
    int arg = 0x7fffffff;
    for (int i = threadIdx.x; i < nblk; i += 256) {
        const float4 v = s[i];
        const int a = __float_as_int(v.z);
        if (v.x > mx || (v.x == mx && a < arg)) { mx = v.x; arg = a; }
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const float omx = __shfl_xor(mx, o, 64);
        const int oarg = __shfl_xor(arg, o, 64);
        if (omx > mx || (omx == mx && oarg < arg)) { mx = omx; arg = oarg; }
    }
    if ((threadIdx.x & 63) == 0) { smx[threadIdx.x >> 6] = mx; sarg[threadIdx.x >> 6] = arg; }
    __syncthreads();
    mx = smx[0]; arg = sarg[0];
    for (int w = 1; w < 4; ++w)
        if (smx[w] > mx || (smx[w] == mx && sarg[w] < arg)) { mx = smx[w]; arg = sarg[w]; }
    float z = 0.f;
    if (inv_temp > 0.f)
        for (int i = threadIdx.x; i < nblk; i += 256) {
            const float4 v = s[i];
            z += v.y * expf((v.x - mx) * inv_temp);
        }
    z = block_sum_256(z, red);
    if (threadIdx.x == 0) rowstat[r] = float4{mx, z, __int_as_float(arg), 0.f};
}

__global__ __launch_bounds__(256) void softmax_merge_kernel(const float4* __restrict__ stats, int nblk, float inv_temp,
                                                            float4* __restrict__ rowstat) {
    softmax_merge_row(blockIdx.x, stats, nblk, inv_temp, rowstat);
}

// ---------------------------------------------------------------------------------------------
// Judge verifier (Eq. 5): score = sigmoid(w . h + b) on the final, normed hidden state of the row
// whose input is the draft token.  One workgroup per (sequence, draft position); entry j scores
// d_{j+1}, i.e. block row j + 1.
// In the top-k mode (the relaxed baseline of Sec. 4.1) the workgroup also ranks d_{j+1} in the target's
// row j: the number of vocabulary entries with a larger logit, or an equal one at a lower index.
template <typename T>
__device__ __forceinline__ void judge_token(int blk, const StepParams* __restrict__ sp, int d,
                                            const float* __restrict__ hn32, const float* __restrict__ row_scale,
                                            const T* __restrict__ w, const T* __restrict__ bias,
                                            float* __restrict__ scores, int V, const float* __restrict__ logits,
                                            int32_t* __restrict__ ranks) {
    __shared__ float red[4];
    const int gamma = sp->gamma;
    const int bi = blk / gamma, j = blk % gamma;
    const int row = bi * (gamma + 1) + j + 1;
    if (sp->mode == 3) {                                   // uniform for the launch
        const float* l = logits + (size_t)(row - 1) * V;
        const int tok = min(max(sp->draft_tokens[bi * gamma + j], 0), V - 1);
        const float ref = l[tok];
        int cnt = 0;
        for (int c = threadIdx.x * 4; c < V; c += 1024) {  // V is a multiple of 128
            const float4 v = *reinterpret_cast<const float4*>(l + c);
            cnt += (v.x > ref || (v.x == ref && c < tok)) + (v.y > ref || (v.y == ref && c + 1 < tok)) +
                   (v.z > ref || (v.z == ref && c + 2 < tok)) + (v.w > ref || (v.w == ref && c + 3 < tok));
        }
        const float total = block_sum_256((float)cnt, red);   // exact: counts stay below 2^24
        if (threadIdx.x == 0) ranks[blk] = (int)total;
        __syncthreads();
    }
    const float* h = hn32 + (size_t)row * d;
    float acc = 0.f;
    for (int c = threadIdx.x; c < d; c += 256) acc += h[c] * Traits<T>::load(w + c);
    acc = block_sum_256(acc, red);
    if (threadIdx.x == 0) {
        // row_scale: the hidden state was stored without its 1/rms factor (applied here)
        const float z = acc * (row_scale ? row_scale[row] : 1.0f) + Traits<T>::load(bias);
        scores[blk] = 1.0f / (1.0f + expf(-z));
    }
}

template <typename T>
__global__ __launch_bounds__(256) void judge_kernel(const StepParams* __restrict__ sp, int d,
                                                    const float* __restrict__ hn32, const float* __restrict__ row_scale,
                                                    const T* __restrict__ w, const T* __restrict__ bias,
                                                    float* __restrict__ scores, int V, const float* __restrict__ logits,
                                                    int32_t* __restrict__ ranks) {
    judge_token<T>(blockIdx.x, sp, d, hn32, row_scale, w, bias, scores, V, logits, ranks);
}

// The two of them in one launch (they do not depend on each other: the judge reads hidden states, and in the top-k
// mode raw logits): workgroups [0, R) merge the softmax statistics of a row, the others score one draft token each.
template <typename T>
__global__ __launch_bounds__(256) void merge_judge_kernel(int R, const float4* __restrict__ stats, int nblk, float inv_temp,
                                                          float4* __restrict__ rowstat, const StepParams* __restrict__ sp, int d,
                                                          const float* __restrict__ hn32, const T* __restrict__ w,
                                                          const T* __restrict__ bias, float* __restrict__ scores, int V,
                                                          const float* __restrict__ logits, int32_t* __restrict__ ranks) {
    if ((int)blockIdx.x < R) softmax_merge_row(blockIdx.x, stats, nblk, inv_temp, rowstat);
    else judge_token<T>(blockIdx.x - R, sp, d, hn32, nullptr, w, bias, scores, V, logits, ranks);
}

// ---------------------------------------------------------------------------------------------
// Ratio test (Eq. 3), OR with the judge (Sec. 3.2), first-rejection scan (Sec. 3.1): one wave per
// sequence, lane j handles draft d_{j+1}:  accept iff u*q(d) < p(d)  with p(d) read from block row j,
// or score > theta.  accepted_len = number of leading accepted lanes (ballot + count trailing ones).
// One wave, lane j; returns accepted_len to every lane; `write` says whether this wave stores the results.
__device__ __forceinline__ int accept_scan_seq(int bi, int j, bool write, const StepParams* __restrict__ sp, int V, float inv_temp,
                                               const float* __restrict__ logits, const float4* __restrict__ rowstat,
                                               const float* __restrict__ scores, float* __restrict__ p_at_d,
                                               int32_t* __restrict__ bits, int32_t* __restrict__ nacc,
                                               const int32_t* __restrict__ ranks) {
    const int gamma = sp->gamma;
    bool ok = false;
    if (j < gamma) {
        const int row = bi * (gamma + 1) + j;
        int tok = sp->draft_tokens[bi * gamma + j];
        tok = min(max(tok, 0), V - 1);
        const float4 st = rowstat[row];
        float p;
        if (inv_temp > 0.f) p = expf((logits[(size_t)row * V + tok] - st.x) * inv_temp) / st.y;
        else p = (tok == __float_as_int(st.z)) ? 1.f : 0.f;
        const float q = sp->draft_probs[((size_t)bi * gamma + j) * V + tok];
        const float u = sp->uniforms[bi * (gamma + 1) + j];
        const bool a = (u * q < p);
        const bool jd = scores[bi * gamma + j] > sp->theta;
        const bool tk = (sp->mode == 3) && ranks[bi * gamma + j] < sp->topk;
        ok = (sp->mode == 1) ? a : (sp->mode == 2) ? jd : (sp->mode == 3) ? tk : (a || jd);
        if (write) {
            p_at_d[bi * gamma + j] = p;
            bits[bi * gamma + j] = (a ? 1 : 0) | (jd ? 2 : 0) | (tk ? 4 : 0);
        }
    }
    const unsigned long long mask = __ballot(ok);
    const int n = __builtin_ctzll(~mask);          // lanes >= gamma vote false, so n <= gamma
    if (write && j == 0) {
        nacc[bi] = n;
        sp->accepted_len[bi] = n;
    }
    return n;
}

__global__ __launch_bounds__(64) void accept_scan_kernel(const StepParams* __restrict__ sp, int V, float inv_temp,
                                                         const float* __restrict__ logits,
                                                         const float4* __restrict__ rowstat,
                                                         const float* __restrict__ scores,
                                                         float* __restrict__ p_at_d, int32_t* __restrict__ bits,
                                                         int32_t* __restrict__ nacc, const int32_t* __restrict__ ranks) {
    accept_scan_seq(blockIdx.x, threadIdx.x, true, sp, V, inv_temp, logits, rowstat, scores, p_at_d, bits, nacc, ranks);
}

// ---------------------------------------------------------------------------------------------
// Extra token (Sec. 3.1 bonus / Sec. 2.2 residual), inverse CDF in vocabulary order with one
// uniform.  Weights are formed in double from the fp32 logits so that the draw is reproducible
// from those logits to ~1e-15:  e_k = exp((l_k - max)/T),  Z = sum e_k,
//   all accepted:  w_k = e_k          else:  w_k = max(0, e_k - Z * q_k)   (q = draft law of the
// first rejected token);  if sum w = 0 fall back to w = e.
// Element k belongs to slab k / slab_len; slab s is owned by thread s % 256 of workgroup s / 256.
//   pass 1 (resample_e):    per-slab sums of e               -> epart
//   pass 2 (resample_w):    Z from epart, per-slab sums of w -> wpart
//   pass 3 (resample_pick): scan the slab sums, walk the hit slab, commit the sequence state.
struct ResampleArgs {
    int32_t V, nslab, slab_len;   // nslab = 256 * gridDim.x of passes 1, 2
    float inv_temp;
    const float* logits;
    const float4* rowstat;
    const int32_t* nacc;
    double* epart;    // [nseq][nslab]
    double* wpart;    // [nseq][nslab]
};

__device__ __forceinline__ double e_of(float logit, float mx, float inv_temp) {
    return exp(((double)logit - (double)mx) * (double)inv_temp);
}

// pass 1 of the draw for the row after `n` accepted tokens
__device__ __forceinline__ void resample_e_slab(const StepParams* __restrict__ sp, const ResampleArgs& a, int n) {
    const int bi = blockIdx.y, slab = blockIdx.x * 256 + threadIdx.x;
    const int gamma = sp->gamma;
    const int row = bi * (gamma + 1) + n;
    const float mx = a.rowstat[row].x;
    const float* l = a.logits + (size_t)row * a.V;
    const int k0 = slab * a.slab_len, k1 = min(a.V, k0 + a.slab_len);
    double s = 0.0;
    if (((a.slab_len | a.V) & 3) == 0) {               // 16-byte loads; same summation order
        for (int k = k0; k < k1; k += 4) {
            const float4 v = *reinterpret_cast<const float4*>(l + k);
            s += e_of(v.x, mx, a.inv_temp);
            s += e_of(v.y, mx, a.inv_temp);
            s += e_of(v.z, mx, a.inv_temp);
            s += e_of(v.w, mx, a.inv_temp);
        }
    } else {
        for (int k = k0; k < k1; ++k) s += e_of(l[k], mx, a.inv_temp);
    }
    a.epart[(size_t)bi * a.nslab + slab] = s;
}

__global__ __launch_bounds__(256) void resample_e_kernel(const StepParams* __restrict__ sp, ResampleArgs a) {
    resample_e_slab(sp, a, a.nacc[blockIdx.y]);
}

// Scan and pass 1 in one launch: pass 1 only needs accepted_len to know its row, and the scan is a handful of loads,
// so the first wave of EVERY workgroup repeats it for the workgroup's sequence (same inputs, same arithmetic, same
// result) and the workgroups with blockIdx.x == 0 store it.
__global__ __launch_bounds__(256) void scan_resample_e_kernel(const StepParams* __restrict__ sp, ResampleArgs a,
                                                              const float* __restrict__ scores, float* __restrict__ p_at_d,
                                                              int32_t* __restrict__ bits, int32_t* __restrict__ nacc,
                                                              const int32_t* __restrict__ ranks) {
    __shared__ int n_sh;
    if (threadIdx.x < 64) {
        const int n = accept_scan_seq(blockIdx.y, threadIdx.x, blockIdx.x == 0, sp, a.V, a.inv_temp, a.logits, a.rowstat, scores,
                                      p_at_d, bits, nacc, ranks);
        if (threadIdx.x == 0) n_sh = n;
    }
    __syncthreads();
    resample_e_slab(sp, a, n_sh);
}

// sum of n slab sums by a 256-thread block: 8 independent loads per thread and batch (index clamped,
// surplus ignored), fixed order
__device__ __forceinline__ double total_of(const double* part, int n, double* lds4) {
    double s = 0.0;
    for (int i0 = threadIdx.x; i0 < n; i0 += 256 * 8) {
        double t[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) t[u] = part[min(i0 + 256 * u, n - 1)];
#pragma unroll
        for (int u = 0; u < 8; ++u) s += (i0 + 256 * u < n) ? t[u] : 0.0;
    }
    return block_sum_256(s, lds4);
}

__global__ __launch_bounds__(256) void resample_w_kernel(const StepParams* __restrict__ sp, ResampleArgs a) {
    __shared__ double red[4];
    const int bi = blockIdx.y, slab = blockIdx.x * 256 + threadIdx.x;
    const int gamma = sp->gamma;
    const int n = a.nacc[bi];
    const double Z = total_of(a.epart + (size_t)bi * a.nslab, a.nslab, red);
    const int row = bi * (gamma + 1) + n;
    const float mx = a.rowstat[row].x;
    const float* l = a.logits + (size_t)row * a.V;
    const int k0 = slab * a.slab_len, k1 = min(a.V, k0 + a.slab_len);
    double s = 0.0;
    if (n < gamma) {
        const float* q = sp->draft_probs + ((size_t)bi * gamma + n) * a.V;
        if (((a.slab_len | a.V) & 3) == 0 && (reinterpret_cast<uintptr_t>(q) & 15) == 0) {   // 16-byte loads; same order
            for (int k = k0; k < k1; k += 4) {
                const float4 v = *reinterpret_cast<const float4*>(l + k);
                const float4 u = *reinterpret_cast<const float4*>(q + k);
                s += fmax(0.0, e_of(v.x, mx, a.inv_temp) - Z * (double)u.x);
                s += fmax(0.0, e_of(v.y, mx, a.inv_temp) - Z * (double)u.y);
                s += fmax(0.0, e_of(v.z, mx, a.inv_temp) - Z * (double)u.z);
                s += fmax(0.0, e_of(v.w, mx, a.inv_temp) - Z * (double)u.w);
            }
        } else {
            for (int k = k0; k < k1; ++k) s += fmax(0.0, e_of(l[k], mx, a.inv_temp) - Z * (double)q[k]);
        }
    }
    a.wpart[(size_t)bi * a.nslab + slab] = s;
}

__global__ __launch_bounds__(256) void resample_pick_kernel(const StepParams* __restrict__ sp, ResampleArgs a,
                                                            int32_t* __restrict__ len, int32_t* __restrict__ pending) {
    __shared__ double red[4];
    __shared__ double wave_tot[4];
    constexpr int PICK_LDS = 8192;               // slab sums staged in LDS (64 KB)
    __shared__ double before_of[257];
    __shared__ double slab_w[256];
    __shared__ double part_lds[PICK_LDS];
    __shared__ int hit_slab;
    __shared__ double hit_before;
    const int bi = blockIdx.x;
    const int b = sp->seq_base + bi;
    const int gamma = sp->gamma;
    const int n = a.nacc[bi];
    const int row = bi * (gamma + 1) + n;
    const float4 st = a.rowstat[row];
    int next = -1;
    if (!(a.inv_temp > 0.f)) {
        next = __float_as_int(st.z);                 // one-hot target: residual and bonus are the arg-max
    } else {
        const double* ep = a.epart + (size_t)bi * a.nslab;
        const double* wp = a.wpart + (size_t)bi * a.nslab;
        const double Z = total_of(ep, a.nslab, red);
        double W = (n < gamma) ? total_of(wp, a.nslab, red) : 0.0;
        const bool use_e = (n == gamma) || !(W > 0.0);
        const double* part = use_e ? ep : wp;
        if (use_e) W = Z;
        const double target = (double)sp->uniforms[bi * (gamma + 1) + gamma] * W;
        // exclusive scan of the slab sums in slab order: thread t owns slabs [t*per, t*per+per).  The sums
        // are staged in LDS with coalesced loads first when they fit (a thread's own range is strided
        // in memory: reading it directly is `per` dependent round trips)
        const int per = a.nslab / 256;
        const bool in_lds = a.nslab <= PICK_LDS;
        if (in_lds) {
            for (int i0 = threadIdx.x; i0 < a.nslab; i0 += 256 * 8) {
                double t[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t[u] = part[min(i0 + 256 * u, a.nslab - 1)];
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (i0 + 256 * u < a.nslab) part_lds[i0 + 256 * u] = t[u];
            }
            __syncthreads();
        }
        auto slab_sum = [&](int i) { return in_lds ? part_lds[i] : part[i]; };
        double mine = 0.0;
        for (int i = 0; i < per; ++i) mine += slab_sum(threadIdx.x * per + i);
        double incl = mine;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            const double t = __shfl_up(incl, o, 64);
            if ((int)(threadIdx.x & 63) >= o) incl += t;
        }
        if ((threadIdx.x & 63) == 63) wave_tot[threadIdx.x >> 6] = incl;
        if (threadIdx.x == 0) { hit_slab = 0x7fffffff; hit_before = 0.0; before_of[256] = INFINITY; }
        __syncthreads();
        double before = incl - mine;
        for (int w = 0; w < (int)(threadIdx.x >> 6); ++w) before += wave_tot[w];
        before_of[threadIdx.x] = before;
        __syncthreads();
        // owner: the thread whose range of the cumulative sum holds the target (lowest wins a tie)
        if (before <= target && target < before_of[threadIdx.x + 1] && mine > 0.0) atomicMin(&hit_slab, (int)threadIdx.x);
        __syncthreads();
        const int owner = hit_slab;
        __syncthreads();
        if ((int)threadIdx.x == owner) {
            double c = before;
            int hs = -1, last_pos = -1;
            double hb = 0.0, last_before = 0.0;
            for (int i = 0; i < per; ++i) {
                const double v = slab_sum(threadIdx.x * per + i);
                if (v > 0.0) { last_pos = threadIdx.x * per + i; last_before = c; }
                if (c + v > target) { hs = threadIdx.x * per + i; hb = c; break; }
                c += v;
            }
            if (hs < 0) { hs = last_pos; hb = last_before; }
            hit_slab = hs;
            hit_before = hb;
        }
        __syncthreads();
        const float mx = st.x;
        const float* l = a.logits + (size_t)row * a.V;
        const float* q = (n < gamma) ? sp->draft_probs + ((size_t)bi * gamma + n) * a.V : nullptr;
        auto weight = [&](int k) {
            const double e = e_of(l[k], mx, a.inv_temp);
            return use_e ? e : fmax(0.0, e - Z * (double)q[k]);
        };
        // the weights of the slab that holds the target, one per thread (slabs of up to 256 entries),
        // then scanned in vocabulary order by one thread
        const bool have_slab = (owner != 0x7fffffff && hit_slab >= 0);
        const int hk0 = have_slab ? hit_slab * a.slab_len : 0, hk1 = have_slab ? min(a.V, hk0 + a.slab_len) : 0;
        const bool staged = have_slab && a.slab_len <= 256;
        if (staged && hk0 + (int)threadIdx.x < hk1) slab_w[threadIdx.x] = weight(hk0 + threadIdx.x);
        __syncthreads();
        if (threadIdx.x == 0) {
            if (have_slab) {
                double c = hit_before;
                int last_pos = -1;
                for (int k = hk0; k < hk1; ++k) {
                    const double v = staged ? slab_w[k - hk0] : weight(k);
                    if (v > 0.0) last_pos = k;
                    c += v;
                    if (c > target) { next = k; break; }
                }
                if (next < 0) next = last_pos;
            }
            if (next < 0) {            // rounding at the very top of the CDF: last token with weight
                for (int k = a.V - 1; k >= 0; --k)
                    if (weight(k) > 0.0) { next = k; break; }
                if (next < 0) next = __float_as_int(st.z);
            }
        }
    }
    if (threadIdx.x == 0) {
        sp->next_token[bi] = next;
        len[b] += 1 + n;           // commit: rows beyond the new length are dead
        pending[b] = next;
    }
}

// Draft proposal (Eq. 1), output of one single-row decode: the row's next-token law q = softmax(l / T)
// as fp32 probabilities into column j of draft_probs [nseq][gamma][V], and the token just drawn from it
// (the sequence's new pending token) into draft_tokens [nseq][gamma].  T = 0: one-hot at the arg-max.
__global__ __launch_bounds__(256) void draft_emit_kernel(int V, float inv_temp, const float* __restrict__ logits,
                                                         const float4* __restrict__ rowstat,
                                                         const int32_t* __restrict__ pending, int seq_base, int gamma, int j,
                                                         int32_t* __restrict__ draft_tokens, float* __restrict__ draft_probs) {
    const int bi = blockIdx.y;
    const float4 st = rowstat[bi];
    const float* l = logits + (size_t)bi * V;
    float* q = draft_probs + ((size_t)bi * gamma + j) * V;
    const float invz = 1.0f / st.y;
    const int arg = __float_as_int(st.z);
    for (int k = blockIdx.x * 256 + threadIdx.x; k < V; k += gridDim.x * 256)
        q[k] = (inv_temp > 0.f) ? expf((l[k] - st.x) * inv_temp) * invz : (k == arg ? 1.f : 0.f);
    if (blockIdx.x == 0 && threadIdx.x == 0) draft_tokens[bi * gamma + j] = pending[seq_base + bi];
}

// Teacher-forced scoring (Sec. 3.3, the terms of Eq. 7): log-probability of a given next token under every
// row's distribution, logp[r] = (l[r][t] - max) / T - log Z from the row's softmax statistics; T = 0: 0 for
// the arg-max, -inf otherwise.  Optionally copies the normed hidden state of row `hrow` of every sequence
// (the judge's feature of the token fed there, Eq. 4).
__global__ __launch_bounds__(256) void score_gather_kernel(int nseq, int rps, int V, int d, float inv_temp,
                                                           const float* __restrict__ logits, const float4* __restrict__ rowstat,
                                                           const int32_t* __restrict__ targets, float* __restrict__ logp,
                                                           const float* __restrict__ hn32, int hrow, float* __restrict__ hidden_out) {
    const int R = nseq * rps;
    for (int r = blockIdx.x * 256 + threadIdx.x; r < R; r += gridDim.x * 256) {
        const int t = min(max(targets[r], 0), V - 1);
        const float4 st = rowstat[r];
        logp[r] = (inv_temp > 0.f) ? (logits[(size_t)r * V + t] - st.x) * inv_temp - logf(st.y)
                                   : (t == __float_as_int(st.z) ? 0.f : -INFINITY);
    }
    if (hidden_out)
        for (int i = blockIdx.x * 256 + threadIdx.x; i < nseq * d; i += gridDim.x * 256)
            hidden_out[i] = hn32[((size_t)(i / d) * rps + hrow) * d + i % d];
}

// the cache rows of this call are kept: advance every sequence's length by rps
__global__ void advance_len_kernel(const StepParams* __restrict__ sp, int32_t* __restrict__ len) {
    const int bi = blockIdx.x * blockDim.x + threadIdx.x;
    if (bi < sp->nseq) len[sp->seq_base + bi] += sp->rps;
}

// Prefill bookkeeping: advance the length by the chunk; after the last chunk the pending token is the
// arg-max continuation of the last prompt token.
__global__ void prefill_commit_kernel(const StepParams* __restrict__ sp, const float4* __restrict__ rowstat,
                                      int32_t* __restrict__ len, int32_t* __restrict__ pending, int last) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        const int b = sp->seq_base;
        len[b] += sp->rps;
        if (last) pending[b] = __float_as_int(rowstat[sp->rps - 1].z);
    }
}

}  // namespace sj
