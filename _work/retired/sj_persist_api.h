// Host-side interface of the persistent whole-forward kernel (sj_persist.hip): the argument block the
// library fills and the two calls it makes.  The kernel itself is described in sj_persist.hip.
#pragma once
#include "sj_types.h"

namespace sj {

constexpr int PERSIST_MAXR = 8;          // query rows of the whole batch: both bf16 planes share one MFMA operand tile
constexpr int PERSIST_WGS = 256;         // one workgroup per compute unit; the work split below assumes exactly this many

// Device-wide barrier state.  Every workgroup publishes its epoch in PERSIST_REPL replicas of a dense flag array
// (1 KB per replica, replicas far apart in memory) and polls the whole of ONE replica with a single 1 KB read: one
// memory round trip from the last arrival to the release, and the 256 pollers are spread over the replicas.
constexpr int PERSIST_REPL = 8;
struct PersistBar {
    unsigned abort;                      // set when a bounded wait ran out: every later wait falls through
    unsigned pad[63];
    struct Replica {
        unsigned flag[PERSIST_WGS];
        unsigned pad[4096 - PERSIST_WGS];
    } rep[PERSIST_REPL];
};

struct PersistLayer {
    const u32x4* wqkv;
    const u32x4* wo;
    const u32x4* wgu;                    // 8 gate rows + 8 up rows per tile
    const u32x4* wd;
    const bf16_t* attn_gain;
    const bf16_t* ffn_gain;
};

// How one weight matrix is split over the 256 workgroups: every workgroup owns `nt` neighbouring n-tiles and
// one of `ksplit` K-slices; its 8 compute waves split that slice again (kw k-steps each).
struct PersistSplit {
    int32_t nt, ksplit, kw;
};

struct PersistArgs {
    const PersistLayer* layers;          // device array [NL]
    const u32x4* lm_head;
    const bf16_t* final_gain;
    const bf16_t* embed;
    int32_t NL;
    ModelDims md;
    const StepParams* sp;
    KvView<bf16_t> kv;
    // Everything one phase writes and another workgroup reads later in the same launch lives in a slot of its own
    // (per layer, per producer) that is written once per launch: a line that was never read before its data was
    // complete cannot be stale in any cache, so consumers use ordinary cached loads and no cache invalidation.
    float* x;                            // [R][d] residual stream (read and written by the same workgroup only)
    float* qkv;                          // [NL] slots of [2][8][Nqkv]: K-slice partials of the QKV projection
    bf16_t* Bx;                          // [2 NL + 1] slots of [d/32][64][8]: packed operand of QKV (slot 2l), gate/up
                                         // (slot 2l + 1) and the LM head (slot 2 NL)
    bf16_t* Battn;                       // [NL] slots of [Hq*hd/32][64][8]: packed operand of the O projection
    bf16_t* Bact;                        // [NL] slots of [F/32][64][8]: packed operand of the down projection
    float* ssq;                          // [2 NL + 1] slots of [8][d/16]: sums of squares of the residual per 16 columns
    bf16_t* knew;                        // [NL][nseq][Hkv] slots of [8][hd]: the block's own K rows as stored in the cache
    bf16_t* vnewT;                       // [NL][nseq][Hkv] slots of [hd][8]: the block's own V rows, transposed
    float* hn32;                         // [R][d] final hidden state after the last RMSNorm
    float* logits;                       // [R][V]
    float4* stats;                       // [R][V/16]
    float* cs;                           // rotary table [R][hd/2][2]
    float* apart;                        // attention partials [tasks][PERSIST_APART floats]
    int32_t chunk_keys;                  // cached keys per attention task (a multiple of 32)
    int32_t nch_max;                     // key chunks per (sequence, kv head, query tile), the block's own rows included
    PersistBar* bar;
    unsigned epoch0;                     // barrier epochs of this launch start above this value
    PersistSplit s_qkv, s_o, s_gu, s_d;  // s_gu.ksplit = s_o.ksplit = s_d.ksplit = 1
    double log_base;
    unsigned long long* prof;            // optional: timestamps (100 MHz) of workgroup 0, wave 0 at phase boundaries
};

constexpr int PERSIST_APART = (128 / 16 * 4 + 2) * 64;   // floats per attention task: 8 head tiles + max + sum, lane order

// grid barriers one launch passes (the host advances epoch0 by this)
inline unsigned persist_barriers(int n_layers) { return 1u + 6u * (unsigned)n_layers; }

// Whether the (nt, ksplit, kw) splits are ones the kernel is instantiated for; fills them in.
bool persist_plan(const ModelDims& md, int n_layers, PersistArgs* a);
size_t persist_lds_bytes();
// Enqueues the forward (embedding .. LM head with per-tile softmax statistics) on `st`; hipSuccess or the launch error.
hipError_t persist_launch(const PersistArgs& a, hipStream_t st);

}  // namespace sj
