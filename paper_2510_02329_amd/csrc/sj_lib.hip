// Host side of the C ABI declared in include/sj.h: argument checking, memory ownership, weight
// upload / re-tiling, and the kernel sequence of one verification step.
#include "../../include/sj.h"
#include "sj_kernels.h"
#include "sj_attn.h"
#include "sj_gemm_rows.h"
#include "sj_gemm_ring.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <memory>
#include <mutex>
#include <string>
#include <type_traits>
#include <vector>

using namespace sj;

// ------------------------------------------------------------------------------------------------
// errors

static thread_local std::string g_err;

static int fail(int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
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

// ------------------------------------------------------------------------------------------------
// objects

struct LayerW {
    void *attn_norm = nullptr, *wqkv = nullptr, *wo = nullptr, *ffn_norm = nullptr, *wgu = nullptr, *wd = nullptr;
};

struct GemmPlan;
struct TunedPlans;

struct sj_model {
    sj_config cfg{};
    ModelDims md{};
    size_t esz = 0;
    void *embed = nullptr, *final_norm = nullptr, *lm_head = nullptr, *judge_w = nullptr, *judge_b = nullptr;
    std::vector<LayerW> layers;
    std::vector<void*> allocs;
    int64_t weight_bytes = 0;
    int device = 0;
    unsigned temp_gen = 0;                     // bumped by sj_set_temperature: captured launch graphs carry the old value
    // launch shapes measured for this model, keyed by (rows, operand planes): a second cache object on the same
    // model reuses them, so two objects of one process run the same kernels (bit-identical results)
    mutable std::mutex tuned_mu;
    mutable std::map<std::pair<int, int>, std::shared_ptr<TunedPlans>> tuned;
};

// Up to two row tiles (32 rows) the few-row kernel (every wave fetches its own operand fragments) is the faster
// one (gate/up of the 70B shape at 24 rows: 179 us against 262 us); from three on the loader-wave kernels.
constexpr int FEW_ROWS = 32;

// Shape of a split-K projection launch: NT n-tiles and `waves` waves per workgroup, `split` K-slices
// across workgroups (summed by the consumer), `depth` k-steps in the few-row kernel's load ring.  The chip has
// 256 CUs and these kernels are a single wave of workgroups long, so a launch whose workgroup count is not a
// multiple of 256 leaves CUs idle for its whole duration: plan_partial takes, among the first tile groupings
// the kernel is instantiated for, the one that wastes the fewest workgroup slots, every wave keeping at least
// 8 k-steps; tune_plans then measures that choice against the other shapes on the model's own weights.
// waves == RING_WAVES selects the LDS-ring kernel (8 compute + 2 loader waves); `depth` is then its ring depth in
// stages (4 or 8).
struct GemmPlan { int nt = 4, waves = 4, split = 1, depth = 2; };
constexpr int RING_WAVES = RING_CW + RING_LW;
constexpr int RING_ROWS = 16;                  // one MFMA row tile
constexpr int RING_PACK_ROWS = 8;              // both operand planes in one product
struct TunedPlans { GemmPlan qkv, o, d, gu, lm; };

struct sj_kv {
    const sj_model* m = nullptr;
    int batch = 0, max_rows = 0, rpad = 0, mpad = 0;
    std::vector<int32_t> cap, len_upper;
    std::vector<int64_t> seq_off;
    int64_t layer_stride = 0;
    void *K = nullptr, *V = nullptr;
    int64_t* seq_off_dev = nullptr;
    int32_t *cap_dev = nullptr, *len_dev = nullptr, *pending_dev = nullptr;
    // workspace
    StepParams* sp_dev = nullptr;
    float *x = nullptr, *hn32 = nullptr, *part = nullptr, *opart = nullptr, *cs = nullptr, *logits = nullptr;
    float *scores = nullptr, *p_at_d = nullptr;
    int32_t* ranks = nullptr;        // [R] rank of every draft token in its target row (top-k mode)
    int topk = 2;
    void *xn = nullptr, *attn_out = nullptr, *act = nullptr;
    unsigned* tickets = nullptr;
    float4 *stats = nullptr, *rowstat = nullptr;
    int32_t *row_tok = nullptr, *bits = nullptr, *nacc = nullptr, *prefill_tok = nullptr, *draft_tok = nullptr;
    double *epart = nullptr, *wpart = nullptr;
    int chunk_keys = 64, nchunk_max = 1, nslab = 0, slab_len = 0;
    GemmPlan plan_qkv[2], plan_o[2], plan_d[2];   // [0]: few-row kernel (at most 32 rows), [1]: more
    GemmPlan plan_gu;                             // gate / up projection with few rows (no K-slices)
    GemmPlan plan_lm{8, 4, 1, 2};                 // LM head with few rows: nt in {4, 8}, waves in {4, 8}
    int lm_nt = 2;
    int mode = SJ_MODE_TWO_STAGE;
    int planes = 2;            // bf16 planes of the activation operand (fp32 storage: always 1)
    int32_t* pinned_state = nullptr;      // [2*batch] staging of sj_kv_rewind
    hipEvent_t rewind_done = nullptr;
    bool rewind_pending = false;
    // optional timing of one kernel class (eager launches only)
    // captured launch graphs of the full step, keyed by (gamma, planes)
    std::map<int, hipGraphExec_t> graphs;
    unsigned graph_gen = 0;               // temp_gen of the model the graphs were captured with
    hipStream_t cap_stream = nullptr;
    bool use_graph = true;
    int timing_class = 0;
    std::vector<hipEvent_t> tev;          // start/stop pairs
    size_t tev_used = 0;
    int last_gamma = 0, last_rows = 0;
    std::vector<void*> allocs;
};

static size_t esz_of(int dtype) { return dtype == SJ_DTYPE_FP32 ? 4 : 2; }

template <typename P> static int dev_alloc(std::vector<void*>& owner, P** p, size_t bytes, bool zero = true) {
    void* q = nullptr;
    if (bytes == 0) bytes = 256;
    hipError_t e = hipMalloc(&q, bytes);
    if (e != hipSuccess) return fail(e == hipErrorOutOfMemory ? SJ_ENOMEM : SJ_EHIP, "hipMalloc(%zu) failed: %s", bytes,
                                     hipGetErrorString(e));
    owner.push_back(q);
    if (zero) HIPCHK(hipMemset(q, 0, bytes));
    *p = reinterpret_cast<P*>(q);
    return SJ_OK;
}

static void free_all(std::vector<void*>& v) {
    for (void* p : v) (void)hipFree(p);
    v.clear();
}

// ------------------------------------------------------------------------------------------------
// model load

static int check_config(const sj_config* c) {
    if (!c) return fail(SJ_EINVAL, "config is null");
    if (c->dtype != SJ_DTYPE_FP32 && c->dtype != SJ_DTYPE_BF16) return fail(SJ_EINVAL, "dtype must be 0 (fp32) or 1 (bf16)");
    if (c->n_layers < 0 || c->d_model <= 0 || c->vocab <= 0) return fail(SJ_EINVAL, "non-positive model dimension");
    if (c->d_model % 64 || c->vocab % 128) return fail(SJ_EINVAL, "d_model must be a multiple of 64 and vocab of 128");
    if (c->d_model > 16384) return fail(SJ_EINVAL, "d_model above 16384 is not supported");
    if (c->max_gamma < 1 || c->max_gamma > 63) return fail(SJ_EINVAL, "max_gamma must be in 1..63");
    if (!(c->temperature >= 0.f)) return fail(SJ_EINVAL, "temperature must be >= 0");
    if (c->n_layers > 0) {
        if (c->n_q_heads <= 0 || c->n_kv_heads <= 0 || c->d_ffn <= 0) return fail(SJ_EINVAL, "non-positive model dimension");
        if (c->head_dim != 64 && c->head_dim != 128) return fail(SJ_EINVAL, "head_dim must be 64 or 128");
        if (c->n_q_heads % c->n_kv_heads) return fail(SJ_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
        if (c->d_ffn % 64) return fail(SJ_EINVAL, "d_ffn must be a multiple of 64");
        if (!(c->rope_base > 1.f) || !(c->rms_eps >= 0.f)) return fail(SJ_EINVAL, "bad rope_base / rms_eps");
    }
    return SJ_OK;
}

namespace {
struct Loader {
    sj_model* m;
    sj_tensor_fn fn;
    void* user;
    void* host = nullptr;      // pinned staging
    void* dev = nullptr;       // device staging (source of the re-tile)
    size_t cap = 0;

    int fetch(int id, int layer, size_t off_bytes, size_t bytes) {
        if (off_bytes + bytes > cap) return fail(SJ_EINVAL, "internal: staging too small");
        if (fn(user, id, layer, (char*)host + off_bytes, bytes) != 0)
            return fail(SJ_ECALLBACK, "tensor provider failed for tensor %d layer %d", id, layer);
        return SJ_OK;
    }
    int plain(int id, int layer, size_t elems, void** out) {       // vectors, embedding: kept row-major
        const size_t bytes = elems * m->esz;
        int rc = fetch(id, layer, 0, bytes);
        if (rc) return rc;
        rc = dev_alloc(m->allocs, out, bytes, false);
        if (rc) return rc;
        HIPCHK(hipMemcpy(*out, host, bytes, hipMemcpyHostToDevice));
        return SJ_OK;
    }
    // one or more [n_i, K] matrices stacked along N, re-tiled into one device matrix
    int tiled(const int* ids, const int* ns, int count, int layer, int K, int interleave, void** out) {
        size_t off = 0;
        int N = 0;
        for (int i = 0; i < count; ++i) {
            const size_t bytes = (size_t)ns[i] * K * m->esz;
            int rc = fetch(ids[i], layer, off, bytes);
            if (rc) return rc;
            off += bytes;
            N += ns[i];
        }
        HIPCHK(hipMemcpy(dev, host, off, hipMemcpyHostToDevice));
        int rc = dev_alloc(m->allocs, out, off, false);
        if (rc) return rc;
        const int blocks = 4096;
        if (m->cfg.dtype == SJ_DTYPE_FP32)
            retile_kernel<float><<<blocks, 256>>>((const float*)dev, (float*)*out, N, K, interleave);
        else
            retile_kernel<bf16_t><<<blocks, 256>>>((const bf16_t*)dev, (bf16_t*)*out, N, K, interleave);
        LAUNCHCHK("retile");
        HIPCHK(hipDeviceSynchronize());
        m->weight_bytes += (int64_t)off;
        return SJ_OK;
    }
};
}  // namespace

extern "C" int sj_model_load(const sj_config* cfg, sj_tensor_fn provider, void* user, sj_model** out) {
    int rc = check_config(cfg);
    if (rc) return rc;
    if (!provider || !out) return fail(SJ_EINVAL, "provider / out is null");
    sj_model* m = new (std::nothrow) sj_model();
    if (!m) return fail(SJ_ENOMEM, "host allocation failed");
    m->cfg = *cfg;
    m->esz = esz_of(cfg->dtype);
    const int d = cfg->d_model, hd = cfg->head_dim, V = cfg->vocab, F = cfg->d_ffn;
    const int Nq = cfg->n_q_heads * hd, Nk = cfg->n_kv_heads * hd;
    ModelDims& md = m->md;
    md.d = d; md.Hq = cfg->n_q_heads; md.Hkv = cfg->n_kv_heads; md.hd = hd; md.F = F; md.V = V;
    md.G = cfg->n_layers > 0 ? cfg->n_q_heads / cfg->n_kv_heads : 1;
    md.eps = cfg->rms_eps;
    md.temperature = cfg->temperature;
    md.inv_temp = cfg->temperature > 0.f ? 1.0f / cfg->temperature : 0.f;
    md.scale = cfg->n_layers > 0 ? (float)(1.0 / std::sqrt((double)hd)) : 1.f;

    Loader ld{m, provider, user};
    size_t need = (size_t)V * d;
    if (cfg->n_layers > 0) need = std::max({need, (size_t)(Nq + 2 * Nk) * d, (size_t)2 * F * d});
    ld.cap = need * m->esz;
    auto cleanup = [&](int code) {
        if (ld.host) (void)hipHostFree(ld.host);
        if (ld.dev) (void)hipFree(ld.dev);
        if (code) { free_all(m->allocs); delete m; }
        return code;
    };
    if (hipGetDevice(&m->device) != hipSuccess) return cleanup(fail(SJ_EHIP, "no HIP device available"));
    {
        hipError_t e = hipHostMalloc(&ld.host, ld.cap, hipHostMallocDefault);
        if (e != hipSuccess) { ld.host = nullptr; return cleanup(fail(SJ_EHIP, "hipHostMalloc(%zu) failed: %s", ld.cap, hipGetErrorString(e))); }
        e = hipMalloc(&ld.dev, ld.cap);
        if (e != hipSuccess) { ld.dev = nullptr; return cleanup(fail(SJ_ENOMEM, "hipMalloc(%zu) failed: %s", ld.cap, hipGetErrorString(e))); }
    }
    m->layers.resize(cfg->n_layers);
    if (cfg->n_layers > 0) {
        if ((rc = ld.plain(SJ_T_EMBED, -1, (size_t)V * d, &m->embed))) return cleanup(rc);
        if ((rc = ld.plain(SJ_T_FINAL_NORM, -1, d, &m->final_norm))) return cleanup(rc);
    }
    for (int l = 0; l < cfg->n_layers; ++l) {
        LayerW& L = m->layers[l];
        if ((rc = ld.plain(SJ_T_ATTN_NORM, l, d, &L.attn_norm))) return cleanup(rc);
        if ((rc = ld.plain(SJ_T_FFN_NORM, l, d, &L.ffn_norm))) return cleanup(rc);
        const int qkv_ids[3] = {SJ_T_WQ, SJ_T_WK, SJ_T_WV}, qkv_ns[3] = {Nq, Nk, Nk};
        if ((rc = ld.tiled(qkv_ids, qkv_ns, 3, l, d, 0, &L.wqkv))) return cleanup(rc);
        const int o_id = SJ_T_WO, o_n = d;
        if ((rc = ld.tiled(&o_id, &o_n, 1, l, Nq, 0, &L.wo))) return cleanup(rc);
        const int gu_ids[2] = {SJ_T_W_GATE, SJ_T_W_UP}, gu_ns[2] = {F, F};
        if ((rc = ld.tiled(gu_ids, gu_ns, 2, l, d, 1, &L.wgu))) return cleanup(rc);
        const int d_id = SJ_T_W_DOWN, d_n = d;
        if ((rc = ld.tiled(&d_id, &d_n, 1, l, F, 0, &L.wd))) return cleanup(rc);
    }
    const int lm_id = SJ_T_LM_HEAD, lm_n = V;
    if ((rc = ld.tiled(&lm_id, &lm_n, 1, -1, d, 0, &m->lm_head))) return cleanup(rc);
    if ((rc = ld.plain(SJ_T_JUDGE_W, -1, d, &m->judge_w))) return cleanup(rc);
    if ((rc = ld.plain(SJ_T_JUDGE_B, -1, 1, &m->judge_b))) return cleanup(rc);
    cleanup(0);
    *out = m;
    return SJ_OK;
}

extern "C" int sj_model_free(sj_model* m) {
    if (!m) return fail(SJ_EINVAL, "model is null");
    free_all(m->allocs);
    delete m;
    return SJ_OK;
}

extern "C" int64_t sj_model_weight_bytes(const sj_model* m) { return m ? m->weight_bytes : 0; }

extern "C" int sj_set_temperature(sj_model* m, float temperature) {
    if (!m) return fail(SJ_EINVAL, "model is null");
    if (!(temperature >= 0.f)) return fail(SJ_EINVAL, "temperature must be >= 0");
    HIPCHK(hipDeviceSynchronize());                            // no step in flight still reads the old value
    m->cfg.temperature = temperature;
    m->md.temperature = temperature;
    m->md.inv_temp = temperature > 0.f ? 1.0f / temperature : 0.f;
    ++m->temp_gen;
    return SJ_OK;
}

// ------------------------------------------------------------------------------------------------
// kv / workspace

// Can the LDS-ring kernel run this product in this launch shape?  bf16 with one or two operand planes, one row tile,
// whole groups of n-tiles, K-slices of whole 8-k-step stages, and at least `depth` stages per workgroup.
static bool ring_fits(const GemmPlan& p, int ntiles, int ksteps, int rows, int planes, bool bf16) {
    if (p.waves != RING_WAVES || !bf16 || planes > 2 || rows > RING_ROWS) return false;
    if (p.nt < 1 || p.split < 1 || ntiles % p.nt || ksteps % (RING_CW * p.split)) return false;
    const int nstages = ksteps / RING_CW / p.split * p.nt;
    return (p.depth == 4 || p.depth == 8) && nstages >= p.depth;
}

// Rule shape of a split-K projection on the LDS-ring kernel (rows <= 8, two planes: the measured case), or waves = 0
// when no shape fits.  Fewest idle workgroup slots first (256 CUs, one round); among those at least two n-tiles per
// workgroup (with one, the operand is as much traffic as the weights) and two K-slices, else four, else one, else
// eight (measured on 4096 x 4096, 4096 x 14336 and 6144 x 4096: the middle of the range wins, and fewer slices are
// less work for the kernel that adds them).
static GemmPlan ring_rule_partial(int ntiles, int ksteps) {
    static const int nts[] = {2, 3, 4, 8, 1}, splits[] = {2, 4, 1, 8};
    GemmPlan best;
    best.waves = 0;
    double best_waste = 1e30;
    for (int split : splits)
        for (int nt : nts) {
            GemmPlan p;
            p.nt = nt; p.waves = RING_WAVES; p.split = split;
            const int nstages = (ksteps / RING_CW / split) * nt;
            p.depth = nstages >= 16 ? 8 : 4;
            if (!ring_fits(p, ntiles, ksteps, 1, 2, true)) continue;
            const int wgs = ntiles / nt * split;
            const double waste = (double)((wgs + 255) / 256 * 256) / wgs + (nt == 1 ? 0.25 : 0.0);
            if (waste < best_waste - 1e-9) { best = p; best_waste = waste; }
        }
    return best;
}

static GemmPlan plan_partial(int ntiles, int ksteps, bool one_row_tile) {
    static const int cand[3][2] = {{4, 4}, {3, 8}, {6, 4}};
    GemmPlan best;
    if (!one_row_tile) {
        // loader-wave kernel: 8 n-tiles per workgroup, one workgroup per CU; as many K-slices (at most 8, of at
        // least 8 k-steps each) as fit one round of the chip - a second, partly filled round costs a whole one
        const int groups = (ntiles + 7) / 8;
        best.nt = 8; best.waves = 8;
        best.split = std::max(1, std::min({8, 256 / std::max(groups, 1), ksteps / 8}));
        return best;
    }
    double best_waste = 1e30;
    for (const auto& c : cand) {
        if (ntiles % c[0]) continue;
        int split = 1;
        while (split < 8 && ksteps / (c[1] * split * 2) >= 8) split *= 2;
        const int wgs = ntiles / c[0] * split;
        const double waste = (double)((wgs + 255) / 256 * 256) / wgs;
        if (waste < best_waste - 1e-9) { best.nt = c[0]; best.waves = c[1]; best.split = split; best_waste = waste; }
    }
    // short K-slices (at most 8 k-steps per wave): a deeper register ring puts the whole slice in flight
    best.depth = (best.nt == 4 && best.waves == 4 && ksteps / (best.split * 4) <= 8) ? 4 : 2;
    return best;
}

static int tune_plans(sj_kv* kv, int rows);

// the launch shapes the rule gives (before any measurement)
static void rule_plans(sj_kv* kv) {
    const sj_config& c = kv->m->cfg;
    const int d = c.d_model, hd = c.head_dim, Nq = c.n_q_heads * hd, Nk = c.n_kv_heads * hd, F = c.d_ffn;
    const int kstep = (c.dtype == SJ_DTYPE_FP32) ? 16 : 32;
    for (int i = 0; i < 2; ++i) {
        kv->plan_qkv[i] = plan_partial((Nq + 2 * Nk) / 16, d / kstep, i == 0);
        kv->plan_o[i] = plan_partial(d / 16, Nq / kstep, i == 0);
        kv->plan_d[i] = plan_partial(d / 16, F / kstep, i == 0);
    }
    kv->plan_gu = GemmPlan{};
    kv->plan_gu.nt = (2 * F / 16) % 7 == 0 ? 7 : 8;       // whole rounds of workgroups where 7 tiles give them
    kv->plan_gu.waves = 8; kv->plan_gu.split = 1; kv->plan_gu.depth = 2;
    kv->plan_lm = GemmPlan{8, 4, 1, 2};
    // at most 8 rows with two bf16 planes: the LDS-ring kernel where a shape of it fits (3 - 8 % faster on the
    // 8B-shaped projections at 6 rows; the start-up measurement may still prefer another shape)
    // (SJ_RING_ROWS = 0..16 moves the row limit of this rule; from 9 rows on, and with one plane, the kernel takes one
    // product per plane and measures equal to the register-ring kernel)
    int ring_rows = RING_PACK_ROWS;
    if (const char* e = std::getenv("SJ_RING_ROWS")) ring_rows = std::min(std::max(std::atoi(e), 0), RING_ROWS);
    if (c.dtype == SJ_DTYPE_BF16 && kv->planes <= 2 && kv->max_rows <= ring_rows) {
        const GemmPlan rq = ring_rule_partial((Nq + 2 * Nk) / 16, d / kstep), ro = ring_rule_partial(d / 16, Nq / kstep),
                       rd = ring_rule_partial(d / 16, F / kstep);
        if (rq.waves) kv->plan_qkv[0] = rq;
        if (ro.waves) kv->plan_o[0] = ro;
        if (rd.waves) kv->plan_d[0] = rd;
        GemmPlan g = kv->plan_gu;
        g.waves = RING_WAVES; g.depth = 8;
        if (ring_fits(g, 2 * F / 16, d / kstep, 1, 2, true)) kv->plan_gu = g;
        GemmPlan l{8, RING_WAVES, 1, 4};
        if (ring_fits(l, c.vocab / 16, d / kstep, 1, 2, true)) kv->plan_lm = l;
    }
}

extern "C" int sj_kv_create(const sj_model* m, int32_t batch, const int32_t* capacity, sj_kv** out) {
    if (!m || !out) return fail(SJ_EINVAL, "model / out is null");
    if (batch < 1 || batch > 4096) return fail(SJ_EINVAL, "batch must be in 1..4096");
    const sj_config& c = m->cfg;
    if (c.n_layers > 0 && !capacity) return fail(SJ_EINVAL, "capacity is null");
    sj_kv* kv = new (std::nothrow) sj_kv();
    if (!kv) return fail(SJ_ENOMEM, "host allocation failed");
    kv->m = m;
    kv->batch = batch;
    if (const char* e = std::getenv("SJ_NO_GRAPH")) kv->use_graph = !(e[0] == '1');
    kv->cap.assign(batch, 64);
    kv->len_upper.assign(batch, 0);
    kv->seq_off.assign(batch, 0);
    int64_t off = 0;
    int cap_max = 64;
    for (int b = 0; b < batch; ++b) {
        int cp = 64;
        if (c.n_layers > 0) {
            if (capacity[b] < 1 || capacity[b] > (1 << 24)) { delete kv; return fail(SJ_EINVAL, "capacity[%d] out of range", b); }
            cp = (capacity[b] + 63) / 64 * 64;
        }
        kv->cap[b] = cp;
        kv->seq_off[b] = off;
        off += (int64_t)cp * c.n_kv_heads * c.head_dim;
        cap_max = std::max(cap_max, cp);
    }
    kv->layer_stride = off;
    const int R = batch * (c.max_gamma + 1);
    kv->max_rows = R;
    kv->rpad = (R + 15) / 16 * 16;
    const int d = c.d_model, V = c.vocab;
    auto& A = kv->allocs;
    int rc = SJ_OK;
    auto bail = [&](int code) { free_all(kv->allocs); delete kv; return code; };
#define ALLOC(ptr, bytes) if ((rc = dev_alloc(A, &(ptr), (bytes)))) return bail(rc)
    ALLOC(kv->seq_off_dev, sizeof(int64_t) * batch);
    ALLOC(kv->cap_dev, sizeof(int32_t) * batch);
    ALLOC(kv->len_dev, sizeof(int32_t) * 2 * batch);           // lengths, then pending tokens: one copy rewinds both
    kv->pending_dev = kv->len_dev + batch;
    ALLOC(kv->sp_dev, sizeof(StepParams));
    ALLOC(kv->xn, (size_t)3 * kv->rpad * d * m->esz);          // up to three operand planes
    ALLOC(kv->hn32, (size_t)R * d * 4);
    ALLOC(kv->row_tok, (size_t)R * 4);
    ALLOC(kv->logits, (size_t)R * V * 4);
    kv->lm_nt = 2;
    ALLOC(kv->stats, (size_t)R * (V / 16) * sizeof(float4));
    ALLOC(kv->rowstat, (size_t)R * sizeof(float4));
    ALLOC(kv->scores, (size_t)R * 4);
    ALLOC(kv->ranks, (size_t)R * 4);
    ALLOC(kv->p_at_d, (size_t)R * 4);
    ALLOC(kv->bits, (size_t)R * 4);
    ALLOC(kv->nacc, (size_t)batch * 4);
    ALLOC(kv->draft_tok, (size_t)batch * 4);
    // resampling slabs: about 16 vocabulary entries per thread
    {
        int blocks = std::max(1, (V / 16 + 255) / 256);
        kv->nslab = blocks * 256;
        kv->slab_len = (V + kv->nslab - 1) / kv->nslab;
    }
    ALLOC(kv->epart, (size_t)batch * kv->nslab * 8);
    ALLOC(kv->wpart, (size_t)batch * kv->nslab * 8);
    if (c.n_layers > 0) {
        const int hd = c.head_dim, Nq = c.n_q_heads * hd, Nk = c.n_kv_heads * hd, F = c.d_ffn;
        const int G = c.n_q_heads / c.n_kv_heads;
        size_t part_elems = 0;
        rule_plans(kv);
        for (int i = 0; i < 2; ++i)
            part_elems = std::max({part_elems, (size_t)kv->plan_qkv[i].split * R * (Nq + 2 * Nk),
                                   (size_t)kv->plan_o[i].split * R * d, (size_t)kv->plan_d[i].split * R * d});
        // room for any few-row plan the start-up measurement may pick (at most 8 K-slices of at most 32 rows)
        part_elems = std::max(part_elems, (size_t)8 * std::min(R, FEW_ROWS) * std::max(Nq + 2 * Nk, d));
        kv->mpad = (G * (c.max_gamma + 1) + 63) / 64 * 64;   // whole groups of 4 MFMA tiles
        // key ranges of attention: one wave takes chunk_keys keys (at least one 32-key step, more when the
        // total context would otherwise need more than 1024 waves: every range costs a partial
        // result and a share of the final merge), a workgroup 4 waves' worth
        {
            const int64_t total_keys = off / ((int64_t)c.n_kv_heads * hd);
            int ck = 32;
            while (ck < 1024 && total_keys * c.n_kv_heads / ck > 1024) ck *= 2;
            if (const char* e = std::getenv("SJ_ATTN_CK")) { const int v = std::atoi(e); if (v >= 32 && v <= 4096 && (v & (v - 1)) == 0) ck = v; }
            kv->chunk_keys = ck;
            kv->nchunk_max = (cap_max + 4 * ck - 1) / (4 * ck);
        }
        ALLOC(kv->K, (size_t)kv->layer_stride * c.n_layers * m->esz);
        ALLOC(kv->V, (size_t)kv->layer_stride * c.n_layers * m->esz);
        ALLOC(kv->x, (size_t)R * d * 4);
        if (part_elems >= ((size_t)1 << 31)) return bail(fail(SJ_EINVAL, "batch * (max_gamma + 1) rows need a projection workspace beyond 2^31 elements"));
        ALLOC(kv->part, part_elems * 4);
        // per (sequence, kv head, key range): mpad rows of hd accumulators + (max, sum) in lane order
        ALLOC(kv->opart, (size_t)batch * c.n_kv_heads * kv->nchunk_max * kv->mpad * (hd + 8) * 4);
        ALLOC(kv->tickets, (size_t)batch * c.n_kv_heads * (kv->mpad / 16) * 4);
        ALLOC(kv->attn_out, (size_t)3 * kv->rpad * Nq * m->esz);
        ALLOC(kv->act, (size_t)3 * kv->rpad * F * m->esz);
        ALLOC(kv->cs, (size_t)R * hd * 4);
        ALLOC(kv->prefill_tok, (size_t)R * 4);
    }
#undef ALLOC
    if (hipMemcpy(kv->seq_off_dev, kv->seq_off.data(), sizeof(int64_t) * batch, hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(kv->cap_dev, kv->cap.data(), sizeof(int32_t) * batch, hipMemcpyHostToDevice) != hipSuccess)
        return bail(fail(SJ_EHIP, "hipMemcpy of cache geometry failed"));
    if (c.n_layers > 0) {
        const char* e = std::getenv("SJ_TUNE");
        if (!(e && e[0] == '0') && (rc = tune_plans(kv, std::min(R, FEW_ROWS)))) return bail(rc);
    }
    *out = kv;
    return SJ_OK;
}

extern "C" int sj_kv_free(sj_kv* kv) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    (void)hipDeviceSynchronize();
    if (kv->pinned_state) (void)hipHostFree(kv->pinned_state);
    if (kv->rewind_done) (void)hipEventDestroy(kv->rewind_done);
    for (hipEvent_t e : kv->tev) (void)hipEventDestroy(e);
    for (auto& g : kv->graphs) (void)hipGraphExecDestroy(g.second);
    if (kv->cap_stream) (void)hipStreamDestroy(kv->cap_stream);
    free_all(kv->allocs);
    delete kv;
    return SJ_OK;
}

extern "C" int sj_set_mode(sj_kv* kv, int32_t mode) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (mode < 0 || mode > 3) return fail(SJ_EINVAL, "mode must be 0, 1, 2 or 3");
    kv->mode = mode;
    return SJ_OK;
}

extern "C" int sj_set_topk(sj_kv* kv, int32_t k) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (k < 1) return fail(SJ_EINVAL, "k must be at least 1");
    kv->topk = k;
    return SJ_OK;
}

extern "C" int sj_kv_rewind(sj_kv* kv, const int32_t* len_host, const int32_t* pending_host, void* stream) {
    if (!kv || !len_host || !pending_host) return fail(SJ_EINVAL, "null argument");
    for (int b = 0; b < kv->batch; ++b) {
        if (len_host[b] < 0 || len_host[b] > kv->cap[b]) return fail(SJ_ECAPACITY, "len[%d] = %d outside capacity %d", b, len_host[b], kv->cap[b]);
        if (pending_host[b] < 0 || pending_host[b] >= kv->m->cfg.vocab) return fail(SJ_EINVAL, "pending[%d] out of range", b);
    }
    hipStream_t st = (hipStream_t)stream;
    if (!kv->pinned_state) {
        HIPCHK(hipHostMalloc((void**)&kv->pinned_state, sizeof(int32_t) * 2 * kv->batch, hipHostMallocDefault));
        HIPCHK(hipEventCreateWithFlags(&kv->rewind_done, hipEventDisableTiming));
    }
    if (kv->rewind_pending) HIPCHK(hipEventSynchronize(kv->rewind_done));   // staging still being read
    std::memcpy(kv->pinned_state, len_host, sizeof(int32_t) * kv->batch);
    std::memcpy(kv->pinned_state + kv->batch, pending_host, sizeof(int32_t) * kv->batch);
    HIPCHK(hipMemcpyAsync(kv->len_dev, kv->pinned_state, sizeof(int32_t) * 2 * kv->batch, hipMemcpyHostToDevice, st));
    HIPCHK(hipEventRecord(kv->rewind_done, st));
    kv->rewind_pending = true;
    for (int b = 0; b < kv->batch; ++b) kv->len_upper[b] = len_host[b];
    return SJ_OK;
}

extern "C" int sj_set_kernel_timing(sj_kv* kv, int32_t kernel_class) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (kernel_class < 0 || kernel_class > 4) return fail(SJ_EINVAL, "kernel_class must be 0..4");
    kv->timing_class = kernel_class;
    kv->tev_used = 0;
    return SJ_OK;
}

extern "C" int sj_kernel_class_shape(const sj_kv* kv, int32_t kernel_class, int32_t rows, char* buf, int32_t buf_len) {
    if (!kv || !buf || buf_len < 1) return fail(SJ_EINVAL, "kv / buf is null");
    if (kernel_class < 1 || kernel_class > 5) return fail(SJ_EINVAL, "kernel_class must be in 1..5");
    if (rows < 1) return fail(SJ_EINVAL, "rows must be positive");
    if (rows > FEW_ROWS) {
        const GemmPlan* p = kernel_class == 1 ? &kv->plan_qkv[1] : kernel_class == 2 ? &kv->plan_o[1] : kernel_class == 4 ? &kv->plan_d[1] : nullptr;
        snprintf(buf, (size_t)buf_len, "gemm_rows%s: row groups of 144 in one launch, 8 or 7 n-tiles per workgroup, %d K-slice(s)",
                 kv->planes == 3 ? "2" : "8", p ? p->split : 1);
        return SJ_OK;
    }
    const GemmPlan& p = kernel_class == 1 ? kv->plan_qkv[0] : kernel_class == 2 ? kv->plan_o[0] : kernel_class == 3 ? kv->plan_gu
                        : kernel_class == 4 ? kv->plan_d[0] : kv->plan_lm;
    const bool ring = p.waves == RING_WAVES && rows <= RING_ROWS && kv->planes <= 2 && kv->m->cfg.dtype == SJ_DTYPE_BF16;
    if (ring)
        snprintf(buf, (size_t)buf_len, "gemm_ring: %d n-tiles per workgroup, 8 compute + 2 loader waves, %d K-slice(s), LDS ring of %d stages",
                 p.nt, p.split, p.depth);
    else if (p.waves == RING_WAVES)
        snprintf(buf, (size_t)buf_len, "gemm_skinny: rule shape (the LDS-ring plan does not take %d rows)", rows);
    else
        snprintf(buf, (size_t)buf_len, "gemm_skinny: %d n-tiles x %d waves per workgroup, %d K-slice(s), register ring of %d", p.nt, p.waves,
                 p.split, p.depth);
    return SJ_OK;
}

extern "C" int sj_get_kernel_timing(sj_kv* kv, double* total_ms, int64_t* launches) {
    if (!kv || !total_ms || !launches) return fail(SJ_EINVAL, "null argument");
    HIPCHK(hipDeviceSynchronize());
    double tot = 0.0;
    for (size_t i = 0; i + 1 < kv->tev_used; i += 2) {
        float ms = 0.f;
        HIPCHK(hipEventElapsedTime(&ms, kv->tev[i], kv->tev[i + 1]));
        tot += ms;
    }
    *total_ms = tot;
    *launches = (int64_t)(kv->tev_used / 2);
    kv->tev_used = 0;
    return SJ_OK;
}

// records an event on the stream if kernel class `cls` is being timed; pairs are (start, stop)
static int time_mark(sj_kv* kv, int cls, hipStream_t st) {
    if (kv->timing_class != cls) return SJ_OK;
    if (kv->tev_used == kv->tev.size()) {
        if (kv->tev.size() >= (1u << 16)) return SJ_OK;         // enough samples; stop recording
        hipEvent_t e;
        HIPCHK(hipEventCreate(&e));
        kv->tev.push_back(e);
    }
    HIPCHK(hipEventRecord(kv->tev[kv->tev_used++], st));
    return SJ_OK;
}

extern "C" int sj_set_operand_planes(sj_kv* kv, int32_t planes) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (planes < 1 || planes > 3) return fail(SJ_EINVAL, "planes must be 1, 2 or 3");
    if (planes == kv->planes) return SJ_OK;
    kv->planes = planes;
    // the launch shapes were chosen for the previous plane count (some exist for one or two planes only): back to
    // the rule's shapes, then the measured ones for this count (taken from the model's record when there is one)
    if (kv->m->cfg.n_layers > 0 && kv->m->cfg.dtype == SJ_DTYPE_BF16) {
        HIPCHK(hipDeviceSynchronize());
        rule_plans(kv);
        const char* e = std::getenv("SJ_TUNE");
        if (!(e && e[0] == '0')) {
            const int rc = tune_plans(kv, std::min(kv->max_rows, FEW_ROWS));
            if (rc) return rc;
        }
    }
    return SJ_OK;
}

static int check_seq_layer(const sj_kv* kv, int seq, int layer) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (kv->m->cfg.n_layers == 0) return fail(SJ_EINVAL, "head-only model has no cache");
    if (seq < 0 || seq >= kv->batch) return fail(SJ_EINVAL, "seq %d out of range", seq);
    if (layer < 0 || layer >= kv->m->cfg.n_layers) return fail(SJ_EINVAL, "layer %d out of range", layer);
    return SJ_OK;
}

extern "C" int sj_kv_set_layer(sj_kv* kv, int32_t seq, int32_t layer, const void* k_host, const void* v_host, int32_t len) {
    int rc = check_seq_layer(kv, seq, layer);
    if (rc) return rc;
    if (!k_host || !v_host) return fail(SJ_EINVAL, "k_host / v_host is null");
    if (len < 0 || len > kv->cap[seq]) return fail(SJ_ECAPACITY, "len %d exceeds capacity %d", len, kv->cap[seq]);
    if (len == 0) return SJ_OK;
    const sj_config& c = kv->m->cfg;
    const size_t esz = kv->m->esz, bytes = (size_t)c.n_kv_heads * len * c.head_dim * esz;
    void *ks = nullptr, *vs = nullptr;
    HIPCHK(hipMalloc(&ks, bytes));
    if (hipMalloc(&vs, bytes) != hipSuccess) { (void)hipFree(ks); return fail(SJ_ENOMEM, "hipMalloc failed"); }
    hipError_t e1 = hipMemcpy(ks, k_host, bytes, hipMemcpyHostToDevice);
    hipError_t e2 = hipMemcpy(vs, v_host, bytes, hipMemcpyHostToDevice);
    if (e1 == hipSuccess && e2 == hipSuccess) {
        const size_t off = (size_t)layer * kv->layer_stride + kv->seq_off[seq];
        if (c.dtype == SJ_DTYPE_FP32)
            kv_scatter_kernel<float><<<1024, 256>>>((const float*)ks, (const float*)vs, (float*)kv->K + off,
                                                     (float*)kv->V + off, c.n_kv_heads, len, kv->cap[seq], c.head_dim);
        else
            kv_scatter_kernel<bf16_t><<<1024, 256>>>((const bf16_t*)ks, (const bf16_t*)vs, (bf16_t*)kv->K + off,
                                                      (bf16_t*)kv->V + off, c.n_kv_heads, len, kv->cap[seq], c.head_dim);
        e1 = hipGetLastError();
        e2 = hipDeviceSynchronize();
    }
    (void)hipFree(ks);
    (void)hipFree(vs);
    if (e1 != hipSuccess || e2 != hipSuccess)
        return fail(SJ_EHIP, "cache upload failed: %s", hipGetErrorString(e1 != hipSuccess ? e1 : e2));
    return SJ_OK;
}

extern "C" int sj_kv_set_state(sj_kv* kv, int32_t seq, int32_t len, int32_t pending_token) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    if (seq < 0 || seq >= kv->batch) return fail(SJ_EINVAL, "seq %d out of range", seq);
    if (len < 0 || len > kv->cap[seq]) return fail(SJ_ECAPACITY, "len %d exceeds capacity %d", len, kv->cap[seq]);
    if (pending_token < 0 || pending_token >= kv->m->cfg.vocab) return fail(SJ_EINVAL, "pending token out of range");
    HIPCHK(hipDeviceSynchronize());
    set_state_kernel<<<1, 1>>>(kv->len_dev, kv->pending_dev, seq, len, pending_token);
    LAUNCHCHK("set_state");
    HIPCHK(hipDeviceSynchronize());
    kv->len_upper[seq] = len;
    return SJ_OK;
}

extern "C" int sj_kv_set(sj_kv* kv, int32_t seq, const void* k_host, const void* v_host, int32_t len, int32_t pending_token) {
    int rc = check_seq_layer(kv, seq, 0);
    if (rc) return rc;
    if (len < 0 || len > kv->cap[seq]) return fail(SJ_ECAPACITY, "len %d exceeds capacity %d", len, kv->cap[seq]);
    if (pending_token < 0 || pending_token >= kv->m->cfg.vocab) return fail(SJ_EINVAL, "pending token out of range");
    if (len > 0 && (!k_host || !v_host)) return fail(SJ_EINVAL, "k_host / v_host is null");
    const sj_config& c = kv->m->cfg;
    const size_t per_layer = (size_t)c.n_kv_heads * len * c.head_dim * kv->m->esz;
    for (int l = 0; l < c.n_layers && len > 0; ++l)
        if ((rc = sj_kv_set_layer(kv, seq, l, (const char*)k_host + l * per_layer, (const char*)v_host + l * per_layer, len)))
            return rc;
    return sj_kv_set_state(kv, seq, len, pending_token);
}

extern "C" int sj_kv_read(const sj_kv* kv, int32_t seq, int32_t layer, int32_t pos0, int32_t n, void* k_host, void* v_host) {
    int rc = check_seq_layer(kv, seq, layer);
    if (rc) return rc;
    if (!k_host || !v_host) return fail(SJ_EINVAL, "k_host / v_host is null");
    if (pos0 < 0 || n < 1 || pos0 + n > kv->cap[seq]) return fail(SJ_EINVAL, "rows %d..%d outside capacity %d", pos0, pos0 + n, kv->cap[seq]);
    const sj_config& c = kv->m->cfg;
    const size_t esz = kv->m->esz, bytes = (size_t)c.n_kv_heads * n * c.head_dim * esz;
    void *ks = nullptr, *vs = nullptr;
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMalloc(&ks, bytes));
    if (hipMalloc(&vs, bytes) != hipSuccess) { (void)hipFree(ks); return fail(SJ_ENOMEM, "hipMalloc failed"); }
    const size_t off = (size_t)layer * kv->layer_stride + kv->seq_off[seq];
    if (c.dtype == SJ_DTYPE_FP32)
        kv_gather_kernel<float><<<256, 256>>>((float*)ks, (float*)vs, (const float*)kv->K + off, (const float*)kv->V + off,
                                               c.n_kv_heads, pos0, n, kv->cap[seq], c.head_dim);
    else
        kv_gather_kernel<bf16_t><<<256, 256>>>((bf16_t*)ks, (bf16_t*)vs, (const bf16_t*)kv->K + off, (const bf16_t*)kv->V + off,
                                                c.n_kv_heads, pos0, n, kv->cap[seq], c.head_dim);
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpy(k_host, ks, bytes, hipMemcpyDeviceToHost);
    if (e == hipSuccess) e = hipMemcpy(v_host, vs, bytes, hipMemcpyDeviceToHost);
    (void)hipFree(ks);
    (void)hipFree(vs);
    if (e != hipSuccess) return fail(SJ_EHIP, "cache read failed: %s", hipGetErrorString(e));
    return SJ_OK;
}

static int refresh_lengths(sj_kv* kv) {
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMemcpy(kv->len_upper.data(), kv->len_dev, sizeof(int32_t) * kv->batch, hipMemcpyDeviceToHost));
    return SJ_OK;
}

extern "C" int sj_kv_state(const sj_kv* kv, int32_t* len_host, int32_t* pending_host) {
    if (!kv) return fail(SJ_EINVAL, "kv is null");
    HIPCHK(hipDeviceSynchronize());
    if (len_host) HIPCHK(hipMemcpy(len_host, kv->len_dev, sizeof(int32_t) * kv->batch, hipMemcpyDeviceToHost));
    if (pending_host) HIPCHK(hipMemcpy(pending_host, kv->pending_dev, sizeof(int32_t) * kv->batch, hipMemcpyDeviceToHost));
    return SJ_OK;
}

// ------------------------------------------------------------------------------------------------
// kernel sequence


// Few rows (at most 32 = two MFMA row tiles): Y = X W^T with the few-row kernel.  X has SPL planes `xplane`
// elements apart; act (EPI_SWIGLU) planes are `actplane` apart.  NT n-tiles per workgroup (N/16 must be a
// multiple of NT), WAVES waves split the K-slice, D = depth of the register ring.
template <typename T, int NT, int EPI, int SPL, int WAVES, int D = 2>
static int gemm(hipStream_t st, const void* Wt, const void* X, size_t xplane, int ldx, int K, int N, int rows, int split,
                float* out, void* act, size_t actplane, float4* stats, float inv_temp) {
    if (rows > FEW_ROWS) return fail(SJ_EINVAL, "internal: few-row kernel called with %d rows", rows);
    const int ngroups = N / 16 / NT;
    GemmArgs a{};
    a.Wt = Wt; a.X = X; a.xplane = xplane; a.actplane = actplane;
    a.ldx = ldx; a.K = K; a.N = N; a.R = rows; a.slice_rows = rows;
    a.inv_temp = inv_temp;
    a.out = out; a.stats = stats; a.act = act;
    if (rows <= 16) gemm_skinny_kernel<T, NT, 1, EPI, SPL, WAVES, D><<<dim3(ngroups, split), WAVES * 64, 0, st>>>(a);
    else gemm_skinny_kernel<T, NT, 2, EPI, SPL, WAVES, D><<<dim3(ngroups, split), WAVES * 64, 0, st>>>(a);
    LAUNCHCHK("gemm_skinny");
    return SJ_OK;
}

// The same product on the LDS-ring kernel (bf16, at most two planes, at most 16 rows; ring_fits has been checked).
template <typename T, int NT, int EPI, int SPL, int NSA>
static int gemm_ring(hipStream_t st, const void* Wt, const void* X, size_t xplane, int ldx, int K, int N, int rows, int split,
                     float* out, void* act, size_t actplane, float4* stats, float inv_temp) {
    GemmArgs a{};
    a.Wt = Wt; a.X = X; a.xplane = xplane; a.actplane = actplane;
    a.ldx = ldx; a.K = K; a.N = N; a.R = rows; a.slice_rows = rows;
    a.inv_temp = inv_temp;
    a.out = out; a.stats = stats; a.act = act;
    const dim3 grid(N / 16 / NT, split);
    if (SPL == 2 && rows <= RING_PACK_ROWS) gemm_ring_kernel<T, NT, EPI, 2, true, NSA><<<grid, RING_THREADS, 0, st>>>(a);
    else gemm_ring_kernel<T, NT, EPI, SPL, false, NSA><<<grid, RING_THREADS, 0, st>>>(a);
    LAUNCHCHK("gemm_ring");
    return SJ_OK;
}

// The few-row split-K projection in the launch shape of a plan.  Shapes beyond the first four exist for the
// default two-plane / one-plane operands only (they are what the start-up measurement may pick).
template <typename T, int SPL>
static int few_partial(const GemmPlan& p, hipStream_t st, const void* W, const void* X, size_t xplane, int ldx, int K, int N,
                       int rows, float* out) {
    if (p.waves == RING_WAVES) {
        if constexpr (std::is_same<T, bf16_t>::value && SPL <= 2) {
            if (ring_fits(p, N / 16, K / Traits<T>::KSTEP, rows, SPL, true)) {
#define SJ_RING(NT, NSA)                                                                                            \
    if (p.nt == NT && p.depth == NSA)                                                                               \
        return gemm_ring<T, NT, EPI_PARTIAL, SPL, NSA>(st, W, X, xplane, ldx, K, N, rows, p.split, out, nullptr, 0, nullptr, 0.f);
                SJ_RING(1, 8) SJ_RING(2, 8) SJ_RING(3, 8) SJ_RING(4, 8) SJ_RING(8, 8)
                SJ_RING(1, 4) SJ_RING(2, 4) SJ_RING(3, 4) SJ_RING(4, 4)
#undef SJ_RING
            }
        }
        // more rows than the kernel takes, or a shape that is not instantiated: the register-ring kernel's rule shape
        return few_partial<T, SPL>(plan_partial(N / 16, K / Traits<T>::KSTEP, true), st, W, X, xplane, ldx, K, N, rows, out);
    }
#define SJ_SHAPE(NT, WV, D)                                                                                         \
    if (p.nt == NT && p.waves == WV && p.depth == D)                                                                \
        return gemm<T, NT, EPI_PARTIAL, SPL, WV, D>(st, W, X, xplane, ldx, K, N, rows, p.split, out, nullptr, 0, nullptr, 0.f);
    SJ_SHAPE(4, 4, 2) SJ_SHAPE(4, 4, 4) SJ_SHAPE(3, 8, 2) SJ_SHAPE(6, 4, 2)
    if constexpr (SPL <= 2) {
        SJ_SHAPE(5, 4, 2) SJ_SHAPE(8, 8, 2) SJ_SHAPE(4, 8, 2) SJ_SHAPE(8, 4, 2) SJ_SHAPE(3, 4, 4)
        SJ_SHAPE(2, 4, 4) SJ_SHAPE(2, 4, 2) SJ_SHAPE(2, 8, 2)
    }
#undef SJ_SHAPE
    // a shape that is not instantiated for this plane count: the rule's shape always is
    const GemmPlan q = plan_partial(N / 16, K / Traits<T>::KSTEP, true);
    if (q.nt != p.nt || q.waves != p.waves || q.depth != p.depth) return few_partial<T, SPL>(q, st, W, X, xplane, ldx, K, N, rows, out);
    return fail(SJ_EINVAL, "internal: no few-row kernel for %d tiles x %d waves, ring %d", p.nt, p.waves, p.depth);
}

// The few-row gate / up projection (SwiGLU epilogue, no K-slices) in the launch shape of a plan.
template <typename T, int SPL>
static int few_swiglu(const GemmPlan& p, hipStream_t st, const void* W, const void* X, size_t xplane, int K, int N2, int rows,
                      void* act, size_t actplane) {
    if (p.waves == RING_WAVES) {
        if constexpr (std::is_same<T, bf16_t>::value && SPL <= 2) {
            if (ring_fits(p, N2 / 16, K / Traits<T>::KSTEP, rows, SPL, true)) {
#define SJ_RING(NT, NSA)                                                                                            \
    if (p.nt == NT && p.depth == NSA)                                                                               \
        return gemm_ring<T, NT, EPI_SWIGLU, SPL, NSA>(st, W, X, xplane, K, K, N2, rows, 1, nullptr, act, actplane, nullptr, 0.f);
                SJ_RING(7, 8) SJ_RING(8, 8) SJ_RING(4, 8) SJ_RING(2, 8) SJ_RING(7, 4) SJ_RING(8, 4) SJ_RING(4, 4)
#undef SJ_RING
            }
        }
        GemmPlan q;
        q.nt = (N2 / 16) % 7 == 0 ? 7 : 8; q.waves = 8; q.split = 1; q.depth = 2;
        return few_swiglu<T, SPL>(q, st, W, X, xplane, K, N2, rows, act, actplane);
    }
#define SJ_SHAPE(NT, WV, D)                                                                                         \
    if (p.nt == NT && p.waves == WV && p.depth == D)                                                                \
        return gemm<T, NT, EPI_SWIGLU, SPL, WV, D>(st, W, X, xplane, K, K, N2, rows, 1, nullptr, act, actplane, nullptr, 0.f);
    SJ_SHAPE(7, 8, 2) SJ_SHAPE(8, 8, 2)
    if constexpr (SPL <= 2) {
        SJ_SHAPE(4, 8, 2) SJ_SHAPE(4, 4, 2) SJ_SHAPE(2, 8, 2) SJ_SHAPE(2, 4, 2) SJ_SHAPE(1, 8, 2)
        SJ_SHAPE(7, 8, 3) SJ_SHAPE(7, 8, 4) SJ_SHAPE(8, 8, 4)
    }
#undef SJ_SHAPE
    GemmPlan q;
    q.nt = (N2 / 16) % 7 == 0 ? 7 : 8; q.waves = 8; q.split = 1; q.depth = 2;
    if (q.nt != p.nt || q.waves != p.waves || q.depth != p.depth) return few_swiglu<T, SPL>(q, st, W, X, xplane, K, N2, rows, act, actplane);
    return fail(SJ_EINVAL, "internal: no few-row gate/up kernel for %d tiles x %d waves", p.nt, p.waves);
}

// The few-row LM head (logits + per-workgroup softmax statistics: V / 16 / nt entries per row) in the launch shape of a plan.
template <typename T, int SPL>
static int few_logits(const GemmPlan& p, hipStream_t st, const void* W, const void* X, size_t xplane, int K, int V, int rows,
                      float* logits, float4* stats, float inv_temp) {
    if (p.waves == RING_WAVES) {
        if constexpr (std::is_same<T, bf16_t>::value && SPL <= 2) {
            if (ring_fits(p, V / 16, K / Traits<T>::KSTEP, rows, SPL, true)) {
#define SJ_RING(NT, NSA)                                                                                            \
    if (p.nt == NT && p.depth == NSA)                                                                               \
        return gemm_ring<T, NT, EPI_LOGITS, SPL, NSA>(st, W, X, xplane, K, K, V, rows, 1, logits, nullptr, 0, stats, inv_temp);
                SJ_RING(8, 4) SJ_RING(8, 8) SJ_RING(4, 8)
#undef SJ_RING
            }
        }
        // the statistics are laid out for p.nt tiles per workgroup: only a kernel with the same count may stand in
        if (p.nt == 8) return few_logits<T, SPL>(GemmPlan{8, 4, 1, 2}, st, W, X, xplane, K, V, rows, logits, stats, inv_temp);
        if (p.nt == 4) {
            if constexpr (SPL <= 2) return few_logits<T, SPL>(GemmPlan{4, 8, 1, 2}, st, W, X, xplane, K, V, rows, logits, stats, inv_temp);
        }
        return fail(SJ_EINVAL, "internal: no few-row LM-head kernel for %d tiles per workgroup", p.nt);
    }
#define SJ_SHAPE(NT, WV)                                                                                            \
    if (p.nt == NT && p.waves == WV)                                                                                \
        return gemm<T, NT, EPI_LOGITS, SPL, WV>(st, W, X, xplane, K, K, V, rows, 1, logits, nullptr, 0, stats, inv_temp);
    SJ_SHAPE(8, 4)
    if constexpr (SPL <= 2) { SJ_SHAPE(8, 8) SJ_SHAPE(4, 8) SJ_SHAPE(4, 4) }
#undef SJ_SHAPE
    if (p.nt != 8 || p.waves != 4) return few_logits<T, SPL>(GemmPlan{8, 4, 1, 2}, st, W, X, xplane, K, V, rows, logits, stats, inv_temp);
    return fail(SJ_EINVAL, "internal: no few-row LM-head kernel for %d tiles x %d waves", p.nt, p.waves);
}

// Picks between the rule's plan and measured candidates.  time_plan(plan, us) times one plan.  The first timings of
// a process run on a GPU that is still raising its clocks, so the rule's plan is timed (and discarded) first; the
// fastest candidate then has to beat the rule's plan by 5 % in two alternating confirmation rounds before it
// replaces it - a choice made on one noisy sample would differ from run to run, and the measurement does not see
// what more K-slices cost the kernel that sums them.
template <typename TimeFn>
static int pick_plan(GemmPlan& plan, const std::vector<GemmPlan>& candidates, TimeFn time_plan) {
    int rc;
    double us = 0.0, best_us = 1e30;
    if ((rc = time_plan(plan, us)) || (rc = time_plan(plan, us))) return rc;       // warm-up
    GemmPlan best = plan;
    bool found = false;
    for (const GemmPlan& p : candidates) {
        if (p.nt == plan.nt && p.waves == plan.waves && p.split == plan.split && p.depth == plan.depth) continue;
        if ((rc = time_plan(p, us))) return rc;
        if (us < best_us) { best_us = us; best = p; found = true; }
    }
    if (!found) return SJ_OK;
    double base_sum = 0.0, cand_sum = 0.0;
    for (int round = 0; round < 2; ++round) {
        if ((rc = time_plan(plan, us))) return rc;
        base_sum += us;
        if ((rc = time_plan(best, us))) return rc;
        cand_sum += us;
    }
    if (cand_sum < 0.95 * base_sum) plan = best;
    return SJ_OK;
}

// Launch shapes of the three split-K projections for few rows, chosen by measurement when the cache object is
// created: which of (n-tiles, waves, K-slices, ring depth) streams a given weight matrix fastest depends on its
// shape and on the number of row tiles in ways the workgroup-count rule of plan_partial does not capture (70B-shaped
// QKV with two row tiles: 50 us with the rule's shape, 35 us with the best one).  Every candidate runs over up to 16
// layers' weights back to back (distinct layers, so nothing is served from cache); the rule's plan stays unless a
// candidate is at least 5 % faster (pick_plan).  SJ_TUNE=0 keeps the rule's plans (launch shapes then never differ between runs).
template <typename T, int SPL>
static int tune_one(sj_kv* kv, GemmPlan& plan, void* LayerW::*which, const void* X, int K, int N, int rows,
                    hipEvent_t e0, hipEvent_t e1) {
    const sj_model* m = kv->m;
    const int ksteps = K / Traits<T>::KSTEP, ntiles = N / 16;
    const int nl = std::min(m->cfg.n_layers, 16);
    const size_t xplane = (size_t)kv->rpad * K;
    auto time_plan = [&](const GemmPlan& p, double& us) -> int {
        float ms = 0.f;
        for (int rep = 0; rep < 2; ++rep) {                 // the first repetition warms up
            HIPCHK(hipEventRecord(e0, nullptr));
            for (int l = 0; l < nl; ++l) {
                const int rc = few_partial<T, SPL>(p, nullptr, m->layers[l].*which, X, xplane, K, K, N, rows, kv->part);
                if (rc) return rc;
            }
            HIPCHK(hipEventRecord(e1, nullptr));
            HIPCHK(hipEventSynchronize(e1));
            HIPCHK(hipEventElapsedTime(&ms, e0, e1));
        }
        us = (double)ms * 1e3 / nl;
        return SJ_OK;
    };
    static const int shapes[][3] = {{4, 4, 2}, {4, 4, 4}, {3, 8, 2}, {6, 4, 2}, {5, 4, 2}, {8, 8, 2}, {4, 8, 2}, {8, 4, 2}, {3, 4, 4},
                                    {2, 4, 4}, {2, 4, 2}, {2, 8, 2}};
    std::vector<GemmPlan> cands;
    for (int i = 0; i < (int)(sizeof(shapes) / sizeof(shapes[0])); ++i) {
        if (SPL > 2 && i >= 4) break;
        const int nt = shapes[i][0], wv = shapes[i][1], dp = shapes[i][2];
        if (ntiles % nt) continue;
        for (int split = 1; split <= 8; split *= 2) {
            const int kpw = ksteps / (wv * split);          // k-steps of a wave
            const long long wgs = (long long)ntiles / nt * split;
            if (kpw < 4 || (dp == 4 && kpw > 8) || wgs < 128 || wgs > 4096) continue;
            GemmPlan p;
            p.nt = nt; p.waves = wv; p.split = split; p.depth = dp;
            cands.push_back(p);
        }
    }
    // the LDS-ring kernel's shapes
    for (int nt : {1, 2, 3, 4, 8})
        for (int split = 1; split <= 8; split *= 2)
            for (int depth : {8, 4}) {
                GemmPlan p;
                p.nt = nt; p.waves = RING_WAVES; p.split = split; p.depth = depth;
                if (!ring_fits(p, ntiles, ksteps, rows, SPL, std::is_same<T, bf16_t>::value)) continue;
                const long long wgs = (long long)ntiles / nt * split;
                if (wgs < 128 || wgs > 4096) continue;
                cands.push_back(p);
            }
    return pick_plan(plan, cands, time_plan);
}

template <typename T, int SPL>
static int tune_gate_up(sj_kv* kv, int rows, hipEvent_t e0, hipEvent_t e1) {
    const sj_model* m = kv->m;
    const int d = m->cfg.d_model, F = m->cfg.d_ffn, ntiles = 2 * F / 16;
    const int nl = std::min(m->cfg.n_layers, 16);
    auto time_plan = [&](const GemmPlan& p, double& us) -> int {
        float ms = 0.f;
        for (int rep = 0; rep < 2; ++rep) {                 // the first repetition warms up
            HIPCHK(hipEventRecord(e0, nullptr));
            for (int l = 0; l < nl; ++l) {
                const int rc = few_swiglu<T, SPL>(p, nullptr, m->layers[l].wgu, kv->xn, (size_t)kv->rpad * d, d, 2 * F, rows, kv->act,
                                                  (size_t)kv->rpad * F);
                if (rc) return rc;
            }
            HIPCHK(hipEventRecord(e1, nullptr));
            HIPCHK(hipEventSynchronize(e1));
            HIPCHK(hipEventElapsedTime(&ms, e0, e1));
        }
        us = (double)ms * 1e3 / nl;
        return SJ_OK;
    };
    static const int shapes[][3] = {{7, 8, 2}, {8, 8, 2}, {4, 8, 2}, {4, 4, 2}, {2, 8, 2}, {2, 4, 2}, {1, 8, 2}, {7, 8, 3}, {7, 8, 4}, {8, 8, 4}};
    std::vector<GemmPlan> cands;
    for (int i = 0; i < (int)(sizeof(shapes) / sizeof(shapes[0])); ++i) {
        if (SPL > 2 && i >= 2) break;
        const int nt = shapes[i][0], wv = shapes[i][1];
        if (ntiles % nt || (d / Traits<T>::KSTEP) / wv < 4 || ntiles / nt < 128) continue;
        GemmPlan p;
        p.nt = nt; p.waves = wv; p.split = 1; p.depth = shapes[i][2];
        cands.push_back(p);
    }
    for (int nt : {7, 8, 4, 2})
        for (int depth : {8, 4}) {
            GemmPlan p;
            p.nt = nt; p.waves = RING_WAVES; p.split = 1; p.depth = depth;
            if (nt == 2 && depth == 4) continue;                 // not instantiated
            if (!ring_fits(p, ntiles, d / Traits<T>::KSTEP, rows, SPL, std::is_same<T, bf16_t>::value) || ntiles / nt < 128) continue;
            cands.push_back(p);
        }
    return pick_plan(kv->plan_gu, cands, time_plan);
}

template <typename T, int SPL>
static int tune_lm_head(sj_kv* kv, int rows, hipEvent_t e0, hipEvent_t e1) {
    const sj_model* m = kv->m;
    const int d = m->cfg.d_model, V = m->cfg.vocab;
    auto time_plan = [&](const GemmPlan& p, double& us) -> int {
        float ms = 0.f;
        for (int rep = 0; rep < 2; ++rep) {                 // the first repetition warms up
            HIPCHK(hipEventRecord(e0, nullptr));
            for (int l = 0; l < 3; ++l) {
                const int rc = few_logits<T, SPL>(p, nullptr, m->lm_head, kv->xn, (size_t)kv->rpad * d, d, V, rows, kv->logits, kv->stats,
                                                  m->md.inv_temp);
                if (rc) return rc;
            }
            HIPCHK(hipEventRecord(e1, nullptr));
            HIPCHK(hipEventSynchronize(e1));
            HIPCHK(hipEventElapsedTime(&ms, e0, e1));
        }
        us = (double)ms * 1e3 / 3;
        return SJ_OK;
    };
    static const int shapes[][2] = {{8, 4}, {8, 8}, {4, 8}, {4, 4}};
    std::vector<GemmPlan> cands;
    for (int i = 0; i < (int)(sizeof(shapes) / sizeof(shapes[0])); ++i) {
        if (SPL > 2) break;
        const int nt = shapes[i][0], wv = shapes[i][1];
        if ((V / 16) % nt || (d / Traits<T>::KSTEP) / wv < 4) continue;
        GemmPlan p;
        p.nt = nt; p.waves = wv; p.split = 1; p.depth = 2;
        cands.push_back(p);
    }
    static const int ring_shapes[][2] = {{8, 4}, {8, 8}, {4, 8}};
    for (const auto& rs : ring_shapes) {
        GemmPlan p;
        p.nt = rs[0]; p.waves = RING_WAVES; p.split = 1; p.depth = rs[1];
        if (ring_fits(p, V / 16, d / Traits<T>::KSTEP, rows, SPL, std::is_same<T, bf16_t>::value)) cands.push_back(p);
    }
    return pick_plan(kv->plan_lm, cands, time_plan);
}

static int tune_plans(sj_kv* kv, int rows) {
    const sj_model* m = kv->m;
    const sj_config& c = m->cfg;
    const int d = c.d_model, Nq = c.n_q_heads * c.head_dim, Nk = c.n_kv_heads * c.head_dim, F = c.d_ffn;
    const std::pair<int, int> key(rows, c.dtype == SJ_DTYPE_FP32 ? 1 : kv->planes);
    {
        std::lock_guard<std::mutex> lock(m->tuned_mu);
        auto it = m->tuned.find(key);
        if (it != m->tuned.end()) {                          // measured before on this model: same shapes again
            const TunedPlans& t = *it->second;
            kv->plan_qkv[0] = t.qkv; kv->plan_o[0] = t.o; kv->plan_d[0] = t.d; kv->plan_gu = t.gu; kv->plan_lm = t.lm;
            return SJ_OK;
        }
    }
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIPCHK(hipEventCreate(&e0));
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(SJ_EHIP, "hipEventCreate failed"); }
    int rc = SJ_OK;
#define SJ_TUNE3(T, SPL)                                                                                          \
    do {                                                                                                          \
        if (!rc) rc = tune_one<T, SPL>(kv, kv->plan_qkv[0], &LayerW::wqkv, kv->xn, d, Nq + 2 * Nk, rows, e0, e1);  \
        if (!rc) rc = tune_one<T, SPL>(kv, kv->plan_o[0], &LayerW::wo, kv->attn_out, Nq, d, rows, e0, e1);         \
        if (!rc) rc = tune_one<T, SPL>(kv, kv->plan_d[0], &LayerW::wd, kv->act, F, d, rows, e0, e1);               \
        if (!rc) rc = tune_gate_up<T, SPL>(kv, rows, e0, e1);                                                     \
        if (!rc) rc = tune_lm_head<T, SPL>(kv, rows, e0, e1);                                                     \
    } while (0)
    if (c.dtype == SJ_DTYPE_FP32) SJ_TUNE3(float, 1);
    else if (kv->planes == 1) SJ_TUNE3(bf16_t, 1);
    else if (kv->planes == 3) SJ_TUNE3(bf16_t, 3);
    else SJ_TUNE3(bf16_t, 2);
#undef SJ_TUNE3
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (!rc) {
        auto t = std::make_shared<TunedPlans>();
        t->qkv = kv->plan_qkv[0]; t->o = kv->plan_o[0]; t->d = kv->plan_d[0]; t->gu = kv->plan_gu; t->lm = kv->plan_lm;
        std::lock_guard<std::mutex> lock(m->tuned_mu);
        m->tuned.emplace(key, t);
    }
    if (const char* e = std::getenv("SJ_TUNE_LOG")) {
        if (e[0] == '1') {
            auto show = [](const char* name, const GemmPlan& p) {
                fprintf(stderr, "[sj] %-8s %d n-tiles x %d waves, %d K-slice(s), ring %d\n", name, p.nt, p.waves, p.split, p.depth);
            };
            fprintf(stderr, "[sj] launch shapes for %d rows, d_model %d:\n", rows, d);
            show("QKV", kv->plan_qkv[0]); show("O", kv->plan_o[0]); show("gate/up", kv->plan_gu); show("down", kv->plan_d[0]);
            show("LM head", kv->plan_lm);
        }
    }
    return rc;
}

// More rows: groups of at most 144 rows (9 MFMA row tiles) through the loader-wave kernel; the statistics
// of EPI_LOGITS are per n-tile there ([rows][N/16]).
template <typename T, int EPI, int SPL>
static int gemm_rows(hipStream_t st, const void* Wt, const void* X, size_t xplane, int ldx, int K, int N, int rows, int split,
                     float* out, void* act, size_t actplane, float4* stats, float inv_temp, bool tiled) {
    const int ntiles = N / 16;
    // fragment-tiled operand planes: a group of 144 rows starts row0 * K elements into the plane in either layout
    if (tiled && ldx != K) return fail(SJ_EINVAL, "a tiled operand has no padding between rows");
    // a single operand plane: row groups of 288 (the 18 operand fragments of a k-step fill the same LDS stages)
    constexpr int RT = (SPL == 1) ? 2 * ROWS_MT : ROWS_MT;
    const int group_rows = RT * 16;
    auto args_of = [&](int row0, int nr) {
        GemmArgs a{};
        a.Wt = Wt;
        a.X = (const char*)X + (size_t)row0 * ldx * sizeof(T);
        a.xplane = xplane; a.actplane = actplane;
        a.ldx = ldx; a.K = K; a.N = N;
        a.R = nr; a.slice_rows = rows;
        a.inv_temp = inv_temp;
        a.x_tks = tiled ? K / Traits<T>::KSTEP : 0;
        a.act_tks = tiled ? (N / 2) / Traits<T>::KSTEP : 0;
        if (EPI == EPI_PARTIAL) a.out = out + (size_t)row0 * N;            // [split][rows][N]
        else if (EPI == EPI_LOGITS) { a.out = out + (size_t)row0 * N; a.stats = stats + (size_t)row0 * ntiles; }
        else a.act = (char*)act + (size_t)row0 * (N / 2) * sizeof(T);
        return a;
    };
    if constexpr (SPL <= 2) {
        // one launch for all row groups: the workgroups of an n-tile group run side by side on one XCD, so the
        // weights are fetched from HBM once for all rows (gemm_rows8_kernel).  7 n-tiles per workgroup where that
        // fills whole rounds of the chip and 8 do not (gate/up of the 8B shape: 256 workgroups instead of 224), from
        // 8 row tiles on (below that the lighter weight stream per CU loses)
        const int rgroups = (rows + group_rows - 1) / group_rows;
        const int mt = (std::min(rows, group_rows) + 15) / 16;
        GemmArgs a = args_of(0, rgroups > 1 ? rows : std::min(rows, group_rows));
        a.rgroups = rgroups;
        const bool seven = EPI == EPI_SWIGLU && mt >= 8 && ntiles % 7 == 0 && (ntiles / 7) % 256 == 0 && ((ntiles + 7) / 8) % 256 != 0;
        const int per = seven ? 7 : R2_NT, ngroups = (ntiles + per - 1) / per;
        const int gx = rgroups > 1 ? (ngroups + 7) / 8 * 8 * rgroups : ngroups;
        const dim3 grid(gx, EPI == EPI_PARTIAL ? split : 1);
        if (seven) gemm_rows8_kernel<T, EPI, SPL, 7, RT><<<grid, (R8_CW + R4_LW) * 64, 0, st>>>(a, mt);
        else gemm_rows8_kernel<T, EPI, SPL, R2_NT, RT><<<grid, (R8_CW + R4_LW) * 64, 0, st>>>(a, mt);
        LAUNCHCHK("gemm_rows");
    } else {
        for (int row0 = 0; row0 < rows; row0 += group_rows) {
            const int nr = std::min(group_rows, rows - row0);
            const GemmArgs a = args_of(row0, nr);
            const dim3 grid((ntiles + R2_NT - 1) / R2_NT, EPI == EPI_PARTIAL ? split : 1);
            gemm_rows2_kernel<T, EPI, SPL><<<grid, (R2_CW + R2_LW) * 64, 0, st>>>(a, (nr + 15) / 16);
            LAUNCHCHK("gemm_rows");
        }
    }
    return SJ_OK;
}

template <typename T, int SPL>
struct Runner {
    const sj_model* m;
    sj_kv* kv;
    hipStream_t st;
    int nseq, rps, R;

    KvView<T> view() const {
        KvView<T> v;
        v.K = (T*)kv->K; v.V = (T*)kv->V; v.seq_off = kv->seq_off_dev; v.cap = kv->cap_dev;
        v.len = kv->len_dev; v.pending = kv->pending_dev; v.layer_stride = kv->layer_stride;
        return v;
    }
    size_t plane(int ld) const { return (size_t)kv->rpad * ld; }
    // Operand planes are written as MFMA fragments when the many-row kernel that reads operands through LDS
    // consumes them (more than FEW_ROWS rows, at most two planes); row-major otherwise.
    bool tiled() const { return R > FEW_ROWS && SPL <= 2; }
    int tks(int K) const { return tiled() ? K / Traits<T>::KSTEP : 0; }
    // the same for a single exact plane (hidden states handed in by the caller), whatever SPL is
    int tks1(int K) const { return R > FEW_ROWS ? K / Traits<T>::KSTEP : 0; }
    int partial_gemm(const void* W, const void* X, int ldx, int K, int N, const GemmPlan (&pl)[2]) {
        if (R > FEW_ROWS) return gemm_rows<T, EPI_PARTIAL, SPL>(st, W, X, plane(ldx), ldx, K, N, R, pl[1].split, kv->part, nullptr, 0, nullptr, 0.f, tiled());
        return few_partial<T, SPL>(pl[0], st, W, X, plane(ldx), ldx, K, N, R, kv->part);
    }
    int nparts(const GemmPlan (&pl)[2]) const { return pl[R <= FEW_ROWS ? 0 : 1].split; }
    // gate / up projection with the SwiGLU epilogue: 7 n-tiles per workgroup when that gives a whole
    // number of workgroups per CU (2F/16 = 1792 tiles -> 256 workgroups), else 8
    int gate_up(const void* W) {
        const ModelDims& md = m->md;
        if (R > FEW_ROWS) return gemm_rows<T, EPI_SWIGLU, SPL>(st, W, kv->xn, plane(md.d), md.d, md.d, 2 * md.F, R, 1, nullptr, kv->act, plane(md.F), nullptr, 0.f, tiled());
        return few_swiglu<T, SPL>(kv->plan_gu, st, W, kv->xn, plane(md.d), md.d, 2 * md.F, R, kv->act, plane(md.F));
    }

    // rotary + cache append + attention of one layer from the QKV partials in kv->part
    int attention(int layer) {
        const ModelDims& md = m->md;
        const int M = md.G * rps;
        const int mtiles = (M + 15) / 16;
        // one query tile per workgroup while the launch stays small (shortest dependent chain per wave;
        // K / V are then read once per tile), up to 4 tiles per workgroup for large batches
        const bool small = (long long)nseq * md.Hkv * kv->nchunk_max * mtiles <= 512;
        const int mq = small ? 1 : std::min(mtiles, 4);
        const int qgroups = (mtiles + mq - 1) / mq;
        dim3 grid(kv->nchunk_max, md.Hkv * qgroups, nseq);
        const bool pb2 = nparts(kv->plan_qkv) <= 2;        // at most two QKV partials: fetch them two at a time
#define ATTN_PB(HD, MQ, PB)                                                                                            \
    attn_fused_kernel<T, HD, MQ, SPL, PB><<<grid, 256, 0, st>>>(kv->sp_dev, md, kv->part, nparts(kv->plan_qkv), R, kv->cs, view(), \
                                                                layer, kv->chunk_keys, kv->nchunk_max, kv->opart, kv->tickets,  \
                                                                (T*)kv->attn_out, plane(md.Hq * md.hd), tks(md.Hq * md.hd))
#define ATTN(HD, MQ)                                                                                                   \
    do { if (pb2) ATTN_PB(HD, MQ, 2); else ATTN_PB(HD, MQ, 4); } while (0)
        if (md.hd == 128) {
            switch (mq) { case 1: ATTN(128, 1); break; case 2: ATTN(128, 2); break; case 3: ATTN(128, 3); break; default: ATTN(128, 4); }
        } else {
            switch (mq) { case 1: ATTN(64, 1); break; case 2: ATTN(64, 2); break; case 3: ATTN(64, 3); break; default: ATTN(64, 4); }
        }
#undef ATTN
#undef ATTN_PB
        LAUNCHCHK("attn_fused");
        return SJ_OK;
    }

    // residual add of `parts` pending split-K partials + RMSNorm into the operand planes (batches of loads as wide as
    // the partials there are: an eight-wide clamped batch for two partials repeats six loads)
    void norm(int parts, const void* gain, float* xn32) {
        const int d = m->md.d;
        if (parts <= 2)
            add_rmsnorm_kernel<T, 2><<<R, 1024, 0, st>>>(R, d, m->md.eps, kv->x, kv->part, parts, (const T*)gain, (T*)kv->xn, plane(d), xn32, tks(d));
        else if (parts <= 4)
            add_rmsnorm_kernel<T, 4><<<R, 1024, 0, st>>>(R, d, m->md.eps, kv->x, kv->part, parts, (const T*)gain, (T*)kv->xn, plane(d), xn32, tks(d));
        else
            add_rmsnorm_kernel<T, 8><<<R, 1024, 0, st>>>(R, d, m->md.eps, kv->x, kv->part, parts, (const T*)gain, (T*)kv->xn, plane(d), xn32, tks(d));
    }

    // decoder layers (Eq. 2 / Eq. 4): leaves the last down-projection partials pending in kv->part
    int layers() {
        const ModelDims& md = m->md;
        const sj_config& c = m->cfg;
        const int d = md.d, Nq = md.Hq * md.hd, Nk = md.Hkv * md.hd, Nqkv = Nq + 2 * Nk;
        step_begin_kernel<T><<<R, 256, 0, st>>>(kv->sp_dev, md, (const T*)m->embed, kv->len_dev, kv->pending_dev, kv->x,
                                                 kv->cs, kv->row_tok, std::log((double)c.rope_base));
        LAUNCHCHK("step_begin");
        int pending_parts = 0;
        int rc;
        for (int l = 0; l < c.n_layers; ++l) {
            const LayerW& L = m->layers[l];
            norm(pending_parts, L.attn_norm, nullptr);
            LAUNCHCHK("add_rmsnorm");
            if ((rc = time_mark(kv, 1, st))) return rc;
            if ((rc = partial_gemm(L.wqkv, kv->xn, d, d, Nqkv, kv->plan_qkv))) return rc;
            if ((rc = time_mark(kv, 1, st))) return rc;
            if ((rc = attention(l))) return rc;
            if ((rc = time_mark(kv, 2, st))) return rc;
            if ((rc = partial_gemm(L.wo, kv->attn_out, Nq, Nq, d, kv->plan_o))) return rc;
            if ((rc = time_mark(kv, 2, st))) return rc;
            norm(nparts(kv->plan_o), L.ffn_norm, nullptr);
            LAUNCHCHK("add_rmsnorm");
            if ((rc = time_mark(kv, 3, st))) return rc;
            if ((rc = gate_up(L.wgu))) return rc;
            if ((rc = time_mark(kv, 3, st))) return rc;
            if ((rc = time_mark(kv, 4, st))) return rc;
            if ((rc = partial_gemm(L.wd, kv->act, md.F, md.F, d, kv->plan_d))) return rc;
            if ((rc = time_mark(kv, 4, st))) return rc;
            pending_parts = nparts(kv->plan_d);
        }
        norm(pending_parts, m->final_norm, kv->hn32);
        LAUNCHCHK("add_rmsnorm");
        return SJ_OK;
    }

    // LM head -> logits + softmax statistics of every row (Eq. 2's p, kept as (max, Z, arg-max)).
    // Hidden states handed in by the caller are already in the storage dtype: one plane suffices then.
    int lm_gemm(bool exact_operand, int& nblk) {
        const ModelDims& md = m->md;
        int rc;
        if (R > FEW_ROWS) {
            rc = exact_operand
                ? gemm_rows<T, EPI_LOGITS, 1>(st, m->lm_head, kv->xn, plane(md.d), md.d, md.d, md.V, R, 1, kv->logits, nullptr, 0, kv->stats, md.inv_temp, true)
                : gemm_rows<T, EPI_LOGITS, SPL>(st, m->lm_head, kv->xn, plane(md.d), md.d, md.d, md.V, R, 1, kv->logits, nullptr, 0, kv->stats, md.inv_temp, tiled());
            nblk = md.V / 16;
        } else {
            rc = exact_operand
                ? few_logits<T, 1>(kv->plan_lm, st, m->lm_head, kv->xn, plane(md.d), md.d, md.V, R, kv->logits, kv->stats, md.inv_temp)
                : few_logits<T, SPL>(kv->plan_lm, st, m->lm_head, kv->xn, plane(md.d), md.d, md.V, R, kv->logits, kv->stats, md.inv_temp);
            nblk = md.V / 16 / kv->plan_lm.nt;
        }
        return rc;
    }
    // judge_gamma > 0: the judge scores of the gamma draft tokens per sequence (Eq. 5) are computed by the same launch
    // that merges the softmax statistics (tail() is then told that they exist)
    int lm_head(bool exact_operand, int judge_gamma = 0) {
        int nblk = 0;
        const int rc = lm_gemm(exact_operand, nblk);
        if (rc) return rc;
        const ModelDims& md = m->md;
        if (judge_gamma > 0) {
            merge_judge_kernel<T><<<R + nseq * judge_gamma, 256, 0, st>>>(R, kv->stats, nblk, md.inv_temp, kv->rowstat, kv->sp_dev, md.d, kv->hn32,
                                                                          (const T*)m->judge_w, (const T*)m->judge_b, kv->scores, md.V,
                                                                          kv->logits, kv->ranks);
            LAUNCHCHK("merge_judge");
        } else {
            softmax_merge_kernel<<<R, 256, 0, st>>>(kv->stats, nblk, md.inv_temp, kv->rowstat);
            LAUNCHCHK("softmax_merge");
        }
        return SJ_OK;
    }

    // Eq. 3, Eq. 5, scan, extra token, state commit
    int tail(int gamma, bool judged) {
        const ModelDims& md = m->md;
        if (gamma > 0 && !judged) {                        // gamma = 0: a plain decode step (draft proposal)
            judge_kernel<T><<<nseq * gamma, 256, 0, st>>>(kv->sp_dev, md.d, kv->hn32, nullptr, (const T*)m->judge_w, (const T*)m->judge_b, kv->scores,
                                                             md.V, kv->logits, kv->ranks);
            LAUNCHCHK("judge");
        }
        ResampleArgs ra{};
        ra.V = md.V; ra.nslab = kv->nslab; ra.slab_len = kv->slab_len; ra.inv_temp = md.inv_temp;
        ra.logits = kv->logits; ra.rowstat = kv->rowstat; ra.nacc = kv->nacc; ra.epart = kv->epart; ra.wpart = kv->wpart;
        if (md.inv_temp > 0.f) {
            dim3 g(kv->nslab / 256, nseq);
            scan_resample_e_kernel<<<g, 256, 0, st>>>(kv->sp_dev, ra, kv->scores, kv->p_at_d, kv->bits, kv->nacc, kv->ranks);
            LAUNCHCHK("scan_resample_e");
            if (gamma > 0) {                               // gamma = 0: always the bonus draw from the row itself, no residual
                resample_w_kernel<<<g, 256, 0, st>>>(kv->sp_dev, ra);
                LAUNCHCHK("resample_w");
            }
        } else {
            accept_scan_kernel<<<nseq, 64, 0, st>>>(kv->sp_dev, md.V, md.inv_temp, kv->logits, kv->rowstat, kv->scores, kv->p_at_d,
                                                     kv->bits, kv->nacc, kv->ranks);
            LAUNCHCHK("accept_scan");
        }
        resample_pick_kernel<<<nseq, 256, 0, st>>>(kv->sp_dev, ra, kv->len_dev, kv->pending_dev);
        LAUNCHCHK("resample_pick");
        return SJ_OK;
    }
};

static int set_params(sj_kv* kv, hipStream_t st, const StepParams& p) {
    set_params_kernel<<<1, 1, 0, st>>>(p, kv->sp_dev);
    LAUNCHCHK("set_params");
    return SJ_OK;
}

template <typename T, int SPL>
static int enqueue_step(sj_model* m, sj_kv* kv, int gamma, hipStream_t st, bool head_only, const void* hidden) {
    int rc;
    Runner<T, SPL> run{m, kv, st, kv->batch, gamma + 1, kv->batch * (gamma + 1)};
    if (head_only) {
        hidden_in_kernel<T><<<1024, 256, 0, st>>>((const T*)hidden, (T*)kv->xn, kv->hn32, run.R, m->md.d, run.tks1(m->md.d));
        LAUNCHCHK("hidden_in");
    } else {
        if ((rc = run.layers())) return rc;
    }
    if ((rc = run.lm_head(head_only, gamma))) return rc;
    return run.tail(gamma, gamma > 0);
}

// The full step is ~200 dependent launches of a few microseconds each: it is captured once per
// (gamma, planes) into a launch graph and replayed; only the per-call parameter block, written by a
// tiny kernel in front of the replay, changes between calls.
template <typename T, int SPL>
static int verify_step_impl(sj_model* m, sj_kv* kv, int gamma, const StepParams& p, hipStream_t st, bool head_only,
                            const void* hidden) {
    int rc;
    const bool graph = kv->use_graph && !head_only && kv->timing_class == 0;
    if (!graph) {
        if ((rc = set_params(kv, st, p))) return rc;
        return enqueue_step<T, SPL>(m, kv, gamma, st, head_only, hidden);
    }
    if (kv->graph_gen != m->temp_gen) {                        // the temperature changed: the graphs hold the old one
        for (auto& g : kv->graphs) (void)hipGraphExecDestroy(g.second);
        kv->graphs.clear();
        kv->graph_gen = m->temp_gen;
    }
    const int key = gamma * 4 + SPL;
    auto it = kv->graphs.find(key);
    if (it == kv->graphs.end()) {
        if (!kv->cap_stream) HIPCHK(hipStreamCreateWithFlags(&kv->cap_stream, hipStreamNonBlocking));
        HIPCHK(hipStreamBeginCapture(kv->cap_stream, hipStreamCaptureModeRelaxed));
        rc = enqueue_step<T, SPL>(m, kv, gamma, kv->cap_stream, false, nullptr);
        hipGraph_t g = nullptr;
        hipError_t e = hipStreamEndCapture(kv->cap_stream, &g);
        if (rc) { if (g) (void)hipGraphDestroy(g); return rc; }
        if (e != hipSuccess) return fail(SJ_EHIP, "hipStreamEndCapture failed: %s", hipGetErrorString(e));
        hipGraphExec_t ex = nullptr;
        e = hipGraphInstantiate(&ex, g, nullptr, nullptr, 0);
        (void)hipGraphDestroy(g);
        if (e != hipSuccess) return fail(SJ_EHIP, "hipGraphInstantiate failed: %s", hipGetErrorString(e));
        it = kv->graphs.emplace(key, ex).first;
    }
    if ((rc = set_params(kv, st, p))) return rc;
    HIPCHK(hipGraphLaunch(it->second, st));
    return SJ_OK;
}

static int dispatch_step(sj_model* m, sj_kv* kv, int gamma, const StepParams& p, hipStream_t st, bool head_only,
                         const void* hidden) {
    if (m->cfg.dtype == SJ_DTYPE_FP32) return verify_step_impl<float, 1>(m, kv, gamma, p, st, head_only, hidden);
    switch (kv->planes) {
        case 1: return verify_step_impl<bf16_t, 1>(m, kv, gamma, p, st, head_only, hidden);
        case 3: return verify_step_impl<bf16_t, 3>(m, kv, gamma, p, st, head_only, hidden);
        default: return verify_step_impl<bf16_t, 2>(m, kv, gamma, p, st, head_only, hidden);
    }
}

template <typename T, int SPL>
static int time_kernel_impl(sj_model* m, sj_kv* kv, int cls, int launches, int gamma, hipStream_t st, double* total_ms) {
    Runner<T, SPL> run{m, kv, st, kv->batch, gamma + 1, kv->batch * (gamma + 1)};
    const ModelDims& md = m->md;
    const int d = md.d, Nq = md.Hq * md.hd, Nk = md.Hkv * md.hd;
    hipEvent_t e0, e1;
    HIPCHK(hipEventCreate(&e0));
    HIPCHK(hipEventCreate(&e1));
    int rc = SJ_OK;
    HIPCHK(hipEventRecord(e0, st));
    for (int i = 0; i < launches && !rc; ++i) {
        if (cls == 5) {                                          // LM head (1 GB at the paper's vocabulary: no reuse either)
            int nblk = 0;
            rc = run.lm_gemm(m->cfg.n_layers == 0, nblk);
            continue;
        }
        const LayerW& L = m->layers[i % m->cfg.n_layers];        // a different layer each time: no cache reuse
        switch (cls) {
            case 1: rc = run.partial_gemm(L.wqkv, kv->xn, d, d, Nq + 2 * Nk, kv->plan_qkv); break;
            case 2: rc = run.partial_gemm(L.wo, kv->attn_out, Nq, Nq, d, kv->plan_o); break;
            case 3: rc = run.gate_up(L.wgu); break;
            default: rc = run.partial_gemm(L.wd, kv->act, md.F, md.F, d, kv->plan_d); break;
        }
    }
    hipError_t e = hipEventRecord(e1, st);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    if (e != hipSuccess) return fail(SJ_EHIP, "kernel timing failed: %s", hipGetErrorString(e));
    *total_ms = ms;
    return SJ_OK;
}

extern "C" int sj_time_kernel_class(sj_model* m, sj_kv* kv, int32_t kernel_class, int32_t launches, void* stream, double* total_ms) {
    if (!m || !kv || !total_ms) return fail(SJ_EINVAL, "null argument");
    if (kv->m != m) return fail(SJ_EINVAL, "kv was created for a different model");
    if (kernel_class < 1 || kernel_class > 5 || launches < 1) return fail(SJ_EINVAL, "kernel_class must be 1..5, launches >= 1");
    if (kernel_class != 5 && m->cfg.n_layers == 0) return fail(SJ_EINVAL, "a head-only model has only the LM head (class 5)");
    if (kv->last_gamma < 1) return fail(SJ_EINVAL, "run a verification step first (the operands of the last step are reused)");
    hipStream_t st = (hipStream_t)stream;
    if (m->cfg.dtype == SJ_DTYPE_FP32) return time_kernel_impl<float, 1>(m, kv, kernel_class, launches, kv->last_gamma, st, total_ms);
    if (kv->planes == 1) return time_kernel_impl<bf16_t, 1>(m, kv, kernel_class, launches, kv->last_gamma, st, total_ms);
    if (kv->planes == 3) return time_kernel_impl<bf16_t, 3>(m, kv, kernel_class, launches, kv->last_gamma, st, total_ms);
    return time_kernel_impl<bf16_t, 2>(m, kv, kernel_class, launches, kv->last_gamma, st, total_ms);
}

static int check_step_args(sj_model* m, sj_kv* kv, int gamma, const void* a, const void* b, const void* c, const void* d,
                           const void* e) {
    if (!m || !kv) return fail(SJ_EINVAL, "model / kv is null");
    if (kv->m != m) return fail(SJ_EINVAL, "kv was created for a different model");
    if (gamma < 1 || gamma > m->cfg.max_gamma) return fail(SJ_EINVAL, "gamma %d outside 1..%d", gamma, m->cfg.max_gamma);
    if (!a || !b || !c || !d || !e) return fail(SJ_EINVAL, "null device pointer argument");
    return SJ_OK;
}

extern "C" int sj_verify_step(sj_model* m, sj_kv* kv, int32_t gamma, const int32_t* draft_tokens, const float* draft_probs,
                              const float* uniforms, float judge_threshold, int32_t* accepted_len, int32_t* next_token,
                              void* stream) {
    int rc = check_step_args(m, kv, gamma, draft_tokens, draft_probs, uniforms, accepted_len, next_token);
    if (rc) return rc;
    if (m->cfg.n_layers == 0) return fail(SJ_EINVAL, "head-only model: use sj_verify_head");
    if (!(judge_threshold == judge_threshold)) return fail(SJ_EINVAL, "judge_threshold is NaN");
    // capacity: the host keeps an upper bound of every length; refresh it only when the bound trips
    bool tight = true;
    for (int b = 0; b < kv->batch; ++b) tight = tight && (kv->len_upper[b] + gamma + 1 <= kv->cap[b]);
    if (!tight) {
        if ((rc = refresh_lengths(kv))) return rc;
        for (int b = 0; b < kv->batch; ++b)
            if (kv->len_upper[b] + gamma + 1 > kv->cap[b])
                return fail(SJ_ECAPACITY, "sequence %d: len %d + gamma + 1 exceeds capacity %d", b, kv->len_upper[b], kv->cap[b]);
    }
    StepParams p{};
    p.nseq = kv->batch; p.seq_base = 0; p.rps = gamma + 1; p.gamma = gamma; p.tok_mode = 0; p.mode = kv->mode; p.topk = kv->topk;
    p.theta = judge_threshold;
    p.draft_tokens = draft_tokens; p.draft_probs = draft_probs; p.uniforms = uniforms;
    p.accepted_len = accepted_len; p.next_token = next_token;
    hipStream_t st = (hipStream_t)stream;
    rc = dispatch_step(m, kv, gamma, p, st, false, nullptr);
    if (rc) return rc;
    for (int b = 0; b < kv->batch; ++b) kv->len_upper[b] += gamma + 1;
    kv->last_gamma = gamma;
    kv->last_rows = kv->batch * (gamma + 1);
    return SJ_OK;
}

// Layers only (no LM head, no decisions) over one row per sequence, then the rows are kept.
template <typename T, int SPL>
static int feed_pending_impl(sj_model* m, sj_kv* kv, hipStream_t st) {
    Runner<T, SPL> run{m, kv, st, kv->batch, 1, kv->batch};
    int rc = run.layers();
    if (rc) return rc;
    advance_len_kernel<<<(kv->batch + 63) / 64, 64, 0, st>>>(kv->sp_dev, kv->len_dev);
    LAUNCHCHK("advance_len");
    return SJ_OK;
}

extern "C" int sj_draft_block(sj_model* m, sj_kv* kv, int32_t gamma, const float* uniforms, int32_t feed_last,
                              int32_t* draft_tokens, float* draft_probs, void* stream) {
    if (!m || !kv) return fail(SJ_EINVAL, "model / kv is null");
    if (kv->m != m) return fail(SJ_EINVAL, "kv was created for a different model");
    if (gamma < 1 || gamma > 63) return fail(SJ_EINVAL, "gamma %d outside 1..63", gamma);
    if (!uniforms || !draft_tokens || !draft_probs) return fail(SJ_EINVAL, "null device pointer argument");
    if (m->cfg.n_layers == 0) return fail(SJ_EINVAL, "head-only model has no decode loop");
    const int need = gamma + (feed_last ? 1 : 0);
    int rc = refresh_lengths(kv);
    if (rc) return rc;
    for (int b = 0; b < kv->batch; ++b)
        if (kv->len_upper[b] + need > kv->cap[b])
            return fail(SJ_ECAPACITY, "sequence %d: len %d + %d rows exceeds capacity %d", b, kv->len_upper[b], need, kv->cap[b]);
    hipStream_t st = (hipStream_t)stream;
    const int V = m->cfg.vocab;
    for (int j = 0; j < gamma; ++j) {
        // one decode step = a verification step without draft tokens: the "all accepted" token is drawn from
        // the row's distribution with the step's uniform and becomes the pending token; length += 1
        StepParams p{};
        p.nseq = kv->batch; p.seq_base = 0; p.rps = 1; p.gamma = 0; p.tok_mode = 0; p.mode = kv->mode; p.topk = kv->topk;
        p.theta = 0.5f;
        p.draft_tokens = nullptr; p.draft_probs = nullptr; p.uniforms = uniforms + (size_t)j * kv->batch;
        p.accepted_len = kv->nacc; p.next_token = kv->draft_tok;   // scratch: the token is read back from the state
        if ((rc = dispatch_step(m, kv, 0, p, st, false, nullptr))) return rc;
        draft_emit_kernel<<<dim3(std::min(64, (V + 255) / 256), kv->batch), 256, 0, st>>>(V, m->md.inv_temp, kv->logits, kv->rowstat,
                                                                                          kv->pending_dev, 0, gamma, j, draft_tokens, draft_probs);
        LAUNCHCHK("draft_emit");
    }
    if (feed_last) {
        StepParams p{};
        p.nseq = kv->batch; p.seq_base = 0; p.rps = 1; p.gamma = 0; p.tok_mode = 0; p.mode = kv->mode; p.topk = kv->topk;
        if ((rc = set_params(kv, st, p))) return rc;
        if (m->cfg.dtype == SJ_DTYPE_FP32) rc = feed_pending_impl<float, 1>(m, kv, st);
        else if (kv->planes == 1) rc = feed_pending_impl<bf16_t, 1>(m, kv, st);
        else if (kv->planes == 3) rc = feed_pending_impl<bf16_t, 3>(m, kv, st);
        else rc = feed_pending_impl<bf16_t, 2>(m, kv, st);
        if (rc) return rc;
    }
    for (int b = 0; b < kv->batch; ++b) kv->len_upper[b] += need;
    kv->last_gamma = 0;
    kv->last_rows = kv->batch;
    return SJ_OK;
}

// forward + LM head over given tokens, then the gather of the targets' log-probabilities
template <typename T, int SPL>
static int score_impl(sj_model* m, sj_kv* kv, int n, const int32_t* targets, float* logprob, int hrow, float* hidden_out,
                      hipStream_t st) {
    Runner<T, SPL> run{m, kv, st, kv->batch, n, kv->batch * n};
    int rc;
    if ((rc = run.layers())) return rc;
    if ((rc = run.lm_head(false))) return rc;
    const int R = kv->batch * n, work = std::max(R, hidden_out ? kv->batch * m->md.d : 0);
    score_gather_kernel<<<std::min(256, (work + 255) / 256), 256, 0, st>>>(kv->batch, n, m->md.V, m->md.d, m->md.inv_temp, kv->logits,
                                                                       kv->rowstat, targets, logprob, kv->hn32, hrow, hidden_out);
    LAUNCHCHK("score_gather");
    return SJ_OK;
}

extern "C" int sj_score_block(sj_model* m, sj_kv* kv, int32_t n, const int32_t* input_tokens, const int32_t* target_tokens,
                              float* logprob, int32_t hidden_row, float* hidden_out, void* stream) {
    if (!m || !kv) return fail(SJ_EINVAL, "model / kv is null");
    if (kv->m != m) return fail(SJ_EINVAL, "kv was created for a different model");
    if (m->cfg.n_layers == 0) return fail(SJ_EINVAL, "head-only model has no forward");
    if (n < 1 || n > m->cfg.max_gamma + 1) return fail(SJ_EINVAL, "n %d outside 1..max_gamma + 1 = %d", n, m->cfg.max_gamma + 1);
    if (!input_tokens || !target_tokens || !logprob) return fail(SJ_EINVAL, "null device pointer argument");
    if (hidden_out && (hidden_row < 0 || hidden_row >= n)) return fail(SJ_EINVAL, "hidden_row %d outside the block", hidden_row);
    int rc = refresh_lengths(kv);
    if (rc) return rc;
    for (int b = 0; b < kv->batch; ++b)
        if (kv->len_upper[b] + n > kv->cap[b])
            return fail(SJ_ECAPACITY, "sequence %d: len %d + %d rows exceeds capacity %d", b, kv->len_upper[b], n, kv->cap[b]);
    hipStream_t st = (hipStream_t)stream;
    StepParams p{};
    p.nseq = kv->batch; p.seq_base = 0; p.rps = n; p.gamma = n - 1; p.tok_mode = 2; p.mode = kv->mode; p.topk = kv->topk;
    p.draft_tokens = input_tokens;
    if ((rc = set_params(kv, st, p))) return rc;
    if (m->cfg.dtype == SJ_DTYPE_FP32) rc = score_impl<float, 1>(m, kv, n, target_tokens, logprob, hidden_row, hidden_out, st);
    else if (kv->planes == 1) rc = score_impl<bf16_t, 1>(m, kv, n, target_tokens, logprob, hidden_row, hidden_out, st);
    else if (kv->planes == 3) rc = score_impl<bf16_t, 3>(m, kv, n, target_tokens, logprob, hidden_row, hidden_out, st);
    else rc = score_impl<bf16_t, 2>(m, kv, n, target_tokens, logprob, hidden_row, hidden_out, st);
    if (rc) return rc;
    kv->last_gamma = 0;
    kv->last_rows = kv->batch * n;
    return SJ_OK;
}

extern "C" int sj_verify_head(sj_model* m, sj_kv* kv, int32_t gamma, const void* hidden, const int32_t* draft_tokens,
                              const float* draft_probs, const float* uniforms, float judge_threshold, int32_t* accepted_len,
                              int32_t* next_token, void* stream) {
    int rc = check_step_args(m, kv, gamma, draft_tokens, draft_probs, uniforms, accepted_len, next_token);
    if (rc) return rc;
    if (!hidden) return fail(SJ_EINVAL, "hidden is null");
    if (!(judge_threshold == judge_threshold)) return fail(SJ_EINVAL, "judge_threshold is NaN");
    StepParams p{};
    p.nseq = kv->batch; p.seq_base = 0; p.rps = gamma + 1; p.gamma = gamma; p.tok_mode = 0; p.mode = kv->mode; p.topk = kv->topk;
    p.theta = judge_threshold;
    p.draft_tokens = draft_tokens; p.draft_probs = draft_probs; p.uniforms = uniforms;
    p.accepted_len = accepted_len; p.next_token = next_token;
    hipStream_t st = (hipStream_t)stream;
    rc = dispatch_step(m, kv, gamma, p, st, true, hidden);
    if (rc) return rc;
    kv->last_gamma = gamma;
    kv->last_rows = kv->batch * (gamma + 1);
    return SJ_OK;
}

// ------------------------------------------------------------------------------------------------
// sj_verify_head for callers that cannot allocate: the workspace lives in a static device array.

constexpr size_t SJ_STATIC_BYTES = SJ_STATIC_WORKSPACE_BYTES;  // per GPU, held until the process ends
static __device__ __align__(256) unsigned char scratch[SJ_STATIC_BYTES];

// The array's device address: looked up once per device with that device current (every GPU holds its own copy).
static int static_scratch_base(unsigned char** out) {
    constexpr int MAXDEV = 64;
    static unsigned char* base[MAXDEV] = {};
    static std::mutex mu;
    int dev = 0;
    HIPCHK(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAXDEV) return fail(SJ_EINVAL, "device index %d not supported by the static workspace", dev);
    std::lock_guard<std::mutex> lock(mu);
    if (!base[dev]) {
        void* p = nullptr;
        HIPCHK(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SJ_EHIP, "hipGetSymbolAddress returned a null address");
        base[dev] = (unsigned char*)p;
    }
    *out = base[dev];
    return SJ_OK;
}

__global__ void fill_i32_kernel(int32_t* p, int n, int32_t v) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) p[i] = v;
}

extern "C" int sj_verify_head_static(sj_model* m, int32_t batch, int32_t gamma, const void* hidden, const int32_t* draft_tokens,
                                     const float* draft_probs, const float* uniforms, float judge_threshold,
                                     int32_t* accepted_len, int32_t* next_token, void* stream) {
    if (!m) return fail(SJ_EINVAL, "model is null");
    if (batch < 1) return fail(SJ_EINVAL, "batch must be positive");
    if (gamma < 1 || gamma > m->cfg.max_gamma) return fail(SJ_EINVAL, "gamma %d outside 1..%d", gamma, m->cfg.max_gamma);
    if (!hidden || !draft_tokens || !draft_probs || !uniforms || !accepted_len || !next_token)
        return fail(SJ_EINVAL, "null device pointer argument");
    if (!(judge_threshold == judge_threshold)) return fail(SJ_EINVAL, "judge_threshold is NaN");
    const int64_t R = (int64_t)batch * (gamma + 1);
    const int d = m->cfg.d_model, V = m->cfg.vocab;
    if (R > SJ_STATIC_MAX_ROWS) return fail(SJ_EINVAL, "batch * (gamma + 1) = %lld rows exceed the static workspace's %d", (long long)R, SJ_STATIC_MAX_ROWS);
    unsigned char* base = nullptr;
    int rc = static_scratch_base(&base);
    if (rc) return rc;
    // carve the workspace (256-byte aligned pieces); a shape that does not fit is refused
    sj_kv kv;
    kv.m = m;
    kv.batch = batch;
    kv.max_rows = (int)R;
    kv.rpad = ((int)R + 15) / 16 * 16;
    kv.use_graph = false;
    kv.nslab = std::max(1, (V / 16 + 255) / 256) * 256;
    kv.slab_len = (V + kv.nslab - 1) / kv.nslab;
    size_t off = 0;
    bool fits = true;
    auto take = [&](size_t bytes) -> void* {
        const size_t at = off;
        off = (off + bytes + 255) / 256 * 256;
        if (off > SJ_STATIC_BYTES) { fits = false; return (void*)base; }
        return (void*)(base + at);
    };
    kv.sp_dev = (StepParams*)take(sizeof(StepParams));
    kv.len_dev = (int32_t*)take(sizeof(int32_t) * 2 * batch);
    kv.pending_dev = kv.len_dev + batch;
    kv.xn = take((size_t)kv.rpad * d * m->esz);                // hidden states are in the storage type: one plane
    kv.hn32 = (float*)take((size_t)R * d * 4);
    kv.logits = (float*)take((size_t)R * V * 4);
    kv.stats = (float4*)take((size_t)R * (V / 16) * sizeof(float4));
    kv.rowstat = (float4*)take((size_t)R * sizeof(float4));
    kv.scores = (float*)take((size_t)R * 4);
    kv.ranks = (int32_t*)take((size_t)R * 4);
    kv.p_at_d = (float*)take((size_t)R * 4);
    kv.bits = (int32_t*)take((size_t)R * 4);
    kv.nacc = (int32_t*)take((size_t)batch * 4);
    kv.epart = (double*)take((size_t)batch * kv.nslab * 8);
    kv.wpart = (double*)take((size_t)batch * kv.nslab * 8);
    if (!fits)
        return fail(SJ_EINVAL, "%lld rows of vocabulary %d, width %d need more than the %zu bytes of the static workspace", (long long)R, V, d,
                    SJ_STATIC_BYTES);
    hipStream_t st = (hipStream_t)stream;
    // the resampling step adds to a length word: it starts at zero on every call (the array keeps the last call's contents)
    fill_i32_kernel<<<1, 256, 0, st>>>(kv.len_dev, 2 * batch, 0);
    LAUNCHCHK("fill_i32");
    StepParams p{};
    p.nseq = batch; p.seq_base = 0; p.rps = gamma + 1; p.gamma = gamma; p.tok_mode = 0; p.mode = SJ_MODE_TWO_STAGE; p.topk = 2;
    p.theta = judge_threshold;
    p.draft_tokens = draft_tokens; p.draft_probs = draft_probs; p.uniforms = uniforms;
    p.accepted_len = accepted_len; p.next_token = next_token;
    return dispatch_step(m, &kv, gamma, p, st, true, hidden);
}

template <typename T, int SPL>
static int prefill_impl(sj_model* m, sj_kv* kv, int seq, const int32_t* tokens, int n, hipStream_t st) {
    const int chunk_max = std::min(kv->max_rows, m->cfg.max_gamma + 1);
    for (int t0 = 0; t0 < n; t0 += chunk_max) {
        const int cn = std::min(chunk_max, n - t0);
        const bool last = (t0 + cn == n);
        HIPCHK(hipMemcpyAsync(kv->prefill_tok, tokens + t0, sizeof(int32_t) * cn, hipMemcpyHostToDevice, st));
        StepParams p{};
        p.nseq = 1; p.seq_base = seq; p.rps = cn; p.gamma = cn - 1; p.tok_mode = 1; p.prefill_tokens = kv->prefill_tok;
        int rc = set_params(kv, st, p);
        if (rc) return rc;
        Runner<T, SPL> run{m, kv, st, 1, cn, cn};
        if ((rc = run.layers())) return rc;
        if (last && (rc = run.lm_head(false))) return rc;
        prefill_commit_kernel<<<1, 1, 0, st>>>(kv->sp_dev, kv->rowstat, kv->len_dev, kv->pending_dev, last ? 1 : 0);
        LAUNCHCHK("prefill_commit");
        HIPCHK(hipStreamSynchronize(st));     // the pageable token copy of the next chunk must not race
    }
    return SJ_OK;
}

extern "C" int sj_prefill(sj_model* m, sj_kv* kv, int32_t seq, const int32_t* tokens_host, int32_t n, void* stream) {
    if (!m || !kv || !tokens_host) return fail(SJ_EINVAL, "null argument");
    if (kv->m != m) return fail(SJ_EINVAL, "kv was created for a different model");
    if (m->cfg.n_layers == 0) return fail(SJ_EINVAL, "head-only model has no cache");
    if (seq < 0 || seq >= kv->batch) return fail(SJ_EINVAL, "seq %d out of range", seq);
    if (n < 1) return fail(SJ_EINVAL, "n must be positive");
    for (int i = 0; i < n; ++i)
        if (tokens_host[i] < 0 || tokens_host[i] >= m->cfg.vocab) return fail(SJ_EINVAL, "token %d out of range", i);
    int rc = refresh_lengths(kv);
    if (rc) return rc;
    if (kv->len_upper[seq] + n > kv->cap[seq]) return fail(SJ_ECAPACITY, "prefill of %d tokens exceeds capacity", n);
    hipStream_t st = (hipStream_t)stream;
    if (m->cfg.dtype == SJ_DTYPE_FP32) rc = prefill_impl<float, 1>(m, kv, seq, tokens_host, n, st);
    else if (kv->planes == 1) rc = prefill_impl<bf16_t, 1>(m, kv, seq, tokens_host, n, st);
    else if (kv->planes == 3) rc = prefill_impl<bf16_t, 3>(m, kv, seq, tokens_host, n, st);
    else rc = prefill_impl<bf16_t, 2>(m, kv, seq, tokens_host, n, st);
    if (rc) return rc;
    kv->len_upper[seq] += n;
    kv->last_gamma = 0;
    kv->last_rows = std::min(n, std::min(kv->max_rows, m->cfg.max_gamma + 1));
    return SJ_OK;
}

extern "C" int sj_debug_fetch(const sj_kv* kv, int32_t what, void* dst_host, size_t nbytes) {
    if (!kv || !dst_host) return fail(SJ_EINVAL, "null argument");
    const int R = kv->last_rows, gamma = kv->last_gamma;
    if (R <= 0) return fail(SJ_EINVAL, "no step has run yet");
    const void* src = nullptr;
    size_t want = 0;
    switch (what) {
        case SJ_DBG_LOGITS: src = kv->logits; want = (size_t)R * kv->m->cfg.vocab * 4; break;
        case SJ_DBG_HIDDEN: src = kv->hn32; want = (size_t)R * kv->m->cfg.d_model * 4; break;
        case SJ_DBG_JUDGE_SCORES: src = kv->scores; want = (size_t)kv->batch * gamma * 4; break;
        case SJ_DBG_P_AT_DRAFT: src = kv->p_at_d; want = (size_t)kv->batch * gamma * 4; break;
        case SJ_DBG_ACCEPT_BITS: src = kv->bits; want = (size_t)kv->batch * gamma * 4; break;
        default: return fail(SJ_EINVAL, "unknown debug item %d", what);
    }
    if (want == 0) return fail(SJ_EINVAL, "item not produced by the last call");
    if (nbytes != want) return fail(SJ_EINVAL, "nbytes %zu != expected %zu", nbytes, want);
    HIPCHK(hipDeviceSynchronize());
    HIPCHK(hipMemcpy(dst_host, src, want, hipMemcpyDeviceToHost));
    return SJ_OK;
}

// the library's other translation units report their errors through this
__attribute__((visibility("hidden"))) int sj_set_error(int code, const char* msg) {
    g_err = msg;
    return code;
}

extern "C" const char* sj_last_error(void) { return g_err.c_str(); }
extern "C" const char* sj_version(void) { return "sj-verify 0.1 (gfx950)"; }
