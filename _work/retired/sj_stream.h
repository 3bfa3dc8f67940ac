// The stages of the persistent forward kernel as separate launches (small row counts, bf16).
//
// Same building blocks as sj_mega.h - one workgroup per CU, 8 streaming waves with a register ring of
// weight tiles, one service wave that stages the packed two-plane operand into LDS and runs the
// epilogue, RMSNorm split around the product - but every stage is its own kernel and the stages are
// chained by a captured launch graph instead of device-side grid barriers.  Measured on the 8B-shaped
// single-sequence workload it is faster than the persistent kernel (nothing spins on the device) but
// slower than the default many-small-workgroups kernels, whose finer grain balances the CUs better
// for the short projections; it is kept as an opt-in variant.  Paper reference: the target forward
// of Eq. 2 / Eq. 4.
#pragma once
#include "sj_mega.h"

namespace sj {

enum { SEPI_QKV = 0, SEPI_RESID = 1, SEPI_SWIGLU = 2, SEPI_LOGITS = 3 };

struct StreamStage {
    const u32x4* W;          // tiled weights
    int32_t ntiles, KS;      // n-tiles of 16 rows, k-steps of 32
    const bf16_t* B;         // packed operand [KS][64][8]
    const bf16_t* gain_next; // SEPI_RESID: gain of the norm that follows the residual add
    int32_t last;            // SEPI_RESID: this is the last layer's down projection (also writes hn32)
};

// stage 0: embedding rows -> residual, packed operand of the first QKV, sums of squares, rotary table.
// One wave per 16-column tile; workgroups 0..R-1 also fill their row of the rotary table.
__global__ __launch_bounds__(64) void stream_embed_kernel(MegaArgs a) {
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int R = sp->nseq * sp->rps, d = md.d, ntx = d / 16, lane = threadIdx.x;
    const bf16_t* gain = a.layers[0].attn_gain;
    const int tile = blockIdx.x;
    if (tile < ntx) {
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
                a.x[(size_t)r * d + col] = v;
            }
            store_packed_row16(a.Bx, r & 7, col, n, v * bf16_to_f32(gain[col]), valid);
            float ss = v * v;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
            if (valid && n == 0) a.ssq[(size_t)r * ntx + tile] = ss;
        }
    }
    if ((int)blockIdx.x < R) {
        const int r = blockIdx.x, bi = r / sp->rps, j = r % sp->rps, b = sp->seq_base + bi;
        const int pos = a.kv.len[b] + j, half = md.hd >> 1;
        for (int i = lane; i < half; i += 64) {
            const double inv_freq = exp(-2.0 * (double)i / (double)md.hd * a.log_base);
            double s, c;
            sincos((double)pos * inv_freq, &s, &c);
            a.cs[((size_t)r * half + i) * 2] = (float)c;
            a.cs[((size_t)r * half + i) * 2 + 1] = (float)s;
        }
    }
}

// rotary + cache append + attention of one (sequence, query head) per workgroup (8 waves)
__global__ __launch_bounds__(MEGA_SW * 64) void stream_attn_kernel(MegaArgs a, size_t layer_off) {
    extern __shared__ __align__(1024) unsigned char smem_raw[];
    AttnShared& as = *reinterpret_cast<AttnShared*>(smem_raw);
    attention_wg(a, layer_off, blockIdx.x, as);
}

// one projection: D = ring depth, BLDS = operand staged to LDS (K <= 4096) or read through a second ring
template <int EPI, int D, bool BLDS>
__global__ __launch_bounds__(MEGA_THREADS) void stream_gemm_kernel(MegaArgs a, StreamStage s) {
    extern __shared__ __align__(1024) unsigned char smem_raw[];
    MegaShared& sm = *reinterpret_cast<MegaShared*>(smem_raw);
    const ModelDims& md = a.md;
    const StepParams* sp = a.sp;
    const int R = sp->nseq * sp->rps;
    const int d = md.d, tid = threadIdx.x, lane = tid & 63;
    const int ntx = d / 16;
    if (tid == 0) sm.ok = 1;
    __syncthreads();
    if (tid < MEGA_SW * 64) {
        Frag rw[MEGA_D], rb[MEGA_D];
        Stream st;
        st.init(s.W, s.ntiles, s.KS);
        prefetch<D>(st, rw);
        stream_stage<D, BLDS>(st, s.B, rw, rb, sm);
        return;
    }
    // ---- service wave
    const int n_items = ((int)blockIdx.x < s.ntiles) ? (s.ntiles - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x : 0;
    if (BLDS) stage_operand(s.B, s.KS, sm);
    if constexpr (EPI == SEPI_QKV) {
        const int Nqkv = s.ntiles * 16;
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        wait_vm0();
        service_stage(n_items, R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
            if (valid) a.qkv[(size_t)r * Nqkv + tile * 16 + n] = v * sm.inv_rms[r];
        });
    } else if constexpr (EPI == SEPI_RESID) {
        float xpre[2];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int e = lane + 64 * half, r = e >> 4, n = e & 15;
            xpre[half] = (r < R && (int)blockIdx.x < ntx) ? a.x[(size_t)r * d + blockIdx.x * 16 + n] : 0.f;
        }
        wait_vm0();
        service_stage(n_items, R, sm, [&](int tile, int r, int n, float v, bool valid, int half) {
            const int col = tile * 16 + n;
            float xn = 0.f;
            if (valid) {
                const float xo = (tile == (int)blockIdx.x) ? xpre[half] : a.x[(size_t)r * d + col];
                xn = xo + v;
                a.x[(size_t)r * d + col] = xn;
            }
            const float y = xn * bf16_to_f32(s.gain_next[col]);
            store_packed_row16(a.Bx, r & 7, col, n, y, valid);
            if (s.last && valid) a.hn32[(size_t)r * d + col] = y;
            float ss = xn * xn;
#pragma unroll
            for (int o = 1; o < 16; o <<= 1) ss += __shfl_xor(ss, o, 64);
            if (valid && n == 0) a.ssq[(size_t)r * ntx + tile] = ss;
        });
    } else if constexpr (EPI == SEPI_SWIGLU) {
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        wait_vm0();
        service_stage(n_items, R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
            const float up = __shfl_down(v, 8, 64);
            const float sc = sm.inv_rms[r & 7];
            const float gate = v * sc, u = up * sc;
            const float act = gate / (1.0f + expf(-gate)) * u;
            // lanes n = 0..7 hold FFN columns 8*tile .. 8*tile+7: gather their two planes into 16 bytes each
            const bf16_t h = f32_to_bf16(act), lo = f32_to_bf16(act - bf16_to_f32(h));
            unsigned h32 = (unsigned)h | ((unsigned)(__shfl_down((int)h, 1, 64) & 0xffff) << 16);
            unsigned l32 = (unsigned)lo | ((unsigned)(__shfl_down((int)lo, 1, 64) & 0xffff) << 16);
            unsigned long long h64 = (unsigned long long)h32 | ((unsigned long long)(unsigned)__shfl_down((int)h32, 2, 64) << 32);
            unsigned long long l64 = (unsigned long long)l32 | ((unsigned long long)(unsigned)__shfl_down((int)l32, 2, 64) << 32);
            const unsigned long long h64b = __shfl_down(h64, 4, 64), l64b = __shfl_down(l64, 4, 64);
            if (valid && n == 0) {
                unsigned long long* ph = reinterpret_cast<unsigned long long*>(a.Bact + packed_off(r, tile * 8));
                unsigned long long* pl = reinterpret_cast<unsigned long long*>(a.Bact + packed_off(r + 8, tile * 8));
                ph[0] = h64; ph[1] = h64b;
                pl[0] = l64; pl[1] = l64b;
            }
        });
    } else {
        const int ntv = s.ntiles;
        compute_inv_rms(a.ssq, ntx, R, d, md.eps, sm);
        wait_vm0();
        if (blockIdx.x == 0 && lane < R) a.row_scale[lane] = sm.inv_rms[lane];
        // the final hidden state was stored as x * gain: apply 1/rms so that the judge (Eq. 5) and the
        // debug read-out see the normed state
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int e = lane + 64 * half, r = e >> 4, n = e & 15;
            if (r < R)
                for (int tile = blockIdx.x; tile < ntx; tile += gridDim.x) a.hn32[(size_t)r * d + tile * 16 + n] *= sm.inv_rms[r];
        }
        service_stage(n_items, R, sm, [&](int tile, int r, int n, float v, bool valid, int) {
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
    }
}

}  // namespace sj
