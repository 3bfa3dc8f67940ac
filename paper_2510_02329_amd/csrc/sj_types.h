// Plain structs shared by the kernels and the host code: per-call parameters, model dimensions, cache view.
#pragma once
#include "sj_device.h"

namespace sj {

// Per-call parameters, kept in device memory so that a captured launch graph can be replayed with
// new caller pointers: only this struct is rewritten between replays.
struct StepParams {
    int32_t nseq;        // sequences processed by this call
    int32_t seq_base;    // first sequence index (prefill of one sequence: its index)
    int32_t rps;         // query rows per sequence (verify: gamma + 1; prefill: chunk length)
    int32_t gamma;       // draft length (verify only)
    int32_t tok_mode;    // 0: row 0 = pending token, rows 1.. = draft tokens; 1: rows = prefill tokens;
                         // 2: every row's token is given: draft_tokens [nseq, rps]
    int32_t mode;        // SJ_MODE_*
    float theta;         // judge threshold
    int32_t topk;        // k of the top-k mode
    const int32_t* draft_tokens;   // [nseq, gamma]
    const float* draft_probs;      // [nseq, gamma, V]
    const float* uniforms;         // [nseq, gamma + 1]
    int32_t* accepted_len;         // [nseq]
    int32_t* next_token;           // [nseq]
    const int32_t* prefill_tokens; // [rps] (tok_mode 1)
};

struct ModelDims {
    int32_t d, Hq, Hkv, hd, F, V, G;   // G = Hq / Hkv
    float eps, inv_temp, temperature, scale;   // scale = 1/sqrt(hd)
};

// KV cache view.  K of (layer, seq): [Hkv][cap][hd]; V is stored transposed: [Hkv][hd][cap], so that
// both MFMA operands of attention are 16-byte contiguous loads.  seq_off[b] = element offset of
// sequence b inside one layer; layer_stride = elements per layer.
template <typename T> struct KvView {
    T* K;
    T* V;
    const int64_t* seq_off;
    const int32_t* cap;
    int32_t* len;
    int32_t* pending;
    int64_t layer_stride;
};

}  // namespace sj
