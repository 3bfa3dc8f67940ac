/*
 * sj.h - C ABI of the draft-block verification step of judge-assisted speculative decoding
 * on one AMD MI355X (gfx950).
 *
 * One call, sj_verify_step, performs for every sequence of a batch what the paper's Method
 * section describes as one verification cycle: the target model reads the pending token and
 * the gamma draft tokens against its KV cache (Eq. 2 / Eq. 4), the draft tokens are tested by
 * the probability-ratio rule (Eq. 3) and by the judge verifier on the target's hidden states
 * (Eq. 5), a token is kept if either test approves it (Sec. 3.2, App. D.2), tokens are accepted
 * until the first rejection (Sec. 3.1), and one more token is emitted from the last
 * distribution or from the residual distribution of modified rejection sampling (Sec. 2.2).
 *
 * Conventions
 *   - Plain C.  No call throws or aborts.  Every function returns SJ_OK (0) or a negative
 *     SJ_E* code; sj_last_error() gives a thread-local message for the last failure.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device memory on the
 *     current device, owned by the caller, and must stay valid until the stream has run.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls that take
 *     a stream are asynchronous on it; their outputs are valid once the stream is synchronised.
 *   - The library owns sj_model / sj_kv and all workspace; it allocates at load / create time
 *     (plus a one-time launch-graph build on the first step of a given gamma), never per step.
 *   - On an argument error no sequence state is modified.
 *   - Storage dtype (sj_config.dtype) applies to weights and the KV cache: 0 = fp32,
 *     1 = bf16 (bit pattern in uint16).  Host tensors handed over are in that dtype.
 *   - Sequences of a batch are independent.
 */
#ifndef SJ_H
#define SJ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SJ_OK         0
#define SJ_EINVAL    -1   /* null pointer, bad shape, gamma / token / index out of range        */
#define SJ_ECAPACITY -2   /* len + gamma + 1 would exceed a sequence's KV capacity              */
#define SJ_EHIP      -3   /* a HIP runtime call failed (message carries hipGetErrorString)      */
#define SJ_ENOMEM    -4   /* host or device allocation failed                                   */
#define SJ_ECALLBACK -5   /* the tensor provider returned non-zero                              */

#define SJ_DTYPE_FP32 0
#define SJ_DTYPE_BF16 1

/* Tensor ids the provider is asked for.  Matrices are [out_features, in_features] row-major
 * (the layout y = x W^T reads), vectors are contiguous.  layer = -1 for model-level tensors. */
enum sj_tensor_id {
    SJ_T_EMBED = 0,      /* [vocab, d_model]                                   */
    SJ_T_ATTN_NORM = 1,  /* [d_model]            RMSNorm gain before attention */
    SJ_T_WQ = 2,         /* [n_q_heads*head_dim, d_model]                      */
    SJ_T_WK = 3,         /* [n_kv_heads*head_dim, d_model]                     */
    SJ_T_WV = 4,         /* [n_kv_heads*head_dim, d_model]                     */
    SJ_T_WO = 5,         /* [d_model, n_q_heads*head_dim]                      */
    SJ_T_FFN_NORM = 6,   /* [d_model]            RMSNorm gain before the FFN   */
    SJ_T_W_GATE = 7,     /* [d_ffn, d_model]                                   */
    SJ_T_W_UP = 8,       /* [d_ffn, d_model]                                   */
    SJ_T_W_DOWN = 9,     /* [d_model, d_ffn]                                   */
    SJ_T_FINAL_NORM = 10,/* [d_model]                                          */
    SJ_T_LM_HEAD = 11,   /* [vocab, d_model]                                   */
    SJ_T_JUDGE_W = 12,   /* [d_model]            judge verifier weights        */
    SJ_T_JUDGE_B = 13    /* [1]                  judge verifier intercept      */
};

/* Model geometry (Llama-3 family decoder, the target models of Sec. 4.1).  n_layers = 0 gives
 * a head-only model (LM head + judge) usable with sj_verify_head only. */
typedef struct sj_config {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab;
    int32_t dtype;          /* SJ_DTYPE_*                                                      */
    float   rope_base;      /* rotary base; pairs (i, i + head_dim/2), angle pos*base^(-2i/hd) */
    float   rms_eps;        /* inside the square root                                          */
    float   temperature;    /* target softmax temperature; 0 = one-hot at the lowest arg-max   */
    int32_t max_gamma;      /* largest draft length any step will use (1..63)                  */
} sj_config;

typedef struct sj_model sj_model;   /* opaque: device-resident, re-tiled weights               */
typedef struct sj_kv sj_kv;         /* opaque: KV cache, per-sequence state, step workspace    */

/* Fills dst (host, nbytes = element count * dtype size) with one tensor.  Return 0 on success.
 * Called once per tensor, one tensor at a time, so the model never has to sit in host memory. */
typedef int (*sj_tensor_fn)(void* user, int32_t tensor_id, int32_t layer, void* dst_host, size_t nbytes);

/* Uploads and re-tiles the target model's weights (needed by Eq. 2 / Eq. 4 / Eq. 5).
 * Requirements: d_model and d_ffn multiples of 64, vocab a multiple of 128, d_model <= 16384;
 * n_q_heads a multiple of n_kv_heads; head_dim in {64, 128}.  Synchronous.  *out is set only on
 * success. */
int sj_model_load(const sj_config* cfg, sj_tensor_fn provider, void* user, sj_model** out);
int sj_model_free(sj_model* m);

/* Creates the per-batch state: a KV cache with `capacity[b]` positions for sequence b (rounded
 * up to a multiple of 64 internally), lengths 0, pending tokens 0, and the step workspace for
 * batch * (max_gamma + 1) query rows.  capacity is a host array of `batch` entries (ignored
 * and may be NULL for a head-only model).  Synchronous.  For a model with layers the call also
 * measures, on the device's default stream and on the model's own weights, which launch shape of
 * each projection kernel is fastest for this row count (some tens of milliseconds; the workspace
 * is used as scratch); the environment variable SJ_TUNE=0 keeps the built-in rule instead, which
 * makes the launch shapes - and with them the summation order of the split-K projections - the
 * same in every run. */
int sj_kv_create(const sj_model* m, int32_t batch, const int32_t* capacity, sj_kv** out);
int sj_kv_free(sj_kv* kv);

/* Overwrites sequence `seq`'s cache with `len` positions given on the host as
 * k_host, v_host = [n_layers][n_kv_heads][len][head_dim] in the storage dtype, and sets its
 * pending token (the last emitted token, not yet cached; row 0 of the next block).
 * Stands in for a real prefill where one is too expensive.  Synchronous. */
int sj_kv_set(sj_kv* kv, int32_t seq, const void* k_host, const void* v_host, int32_t len,
              int32_t pending_token);

/* Same for a single layer: k_host, v_host = [n_kv_heads][len][head_dim].  Lets a large cache be
 * produced layer by layer.  Length / pending token take effect through sj_kv_set_state. */
int sj_kv_set_layer(sj_kv* kv, int32_t seq, int32_t layer, const void* k_host, const void* v_host,
                    int32_t len);
int sj_kv_set_state(sj_kv* kv, int32_t seq, int32_t len, int32_t pending_token);

/* Reads back cache rows pos0 .. pos0+n-1 of one (sequence, layer) into host arrays
 * [n_kv_heads][n][head_dim] (storage dtype).  Rows at or beyond the current length are the
 * dead rows of the last block.  Synchronous. */
int sj_kv_read(const sj_kv* kv, int32_t seq, int32_t layer, int32_t pos0, int32_t n,
               void* k_host, void* v_host);

/* Current lengths / pending tokens, host arrays of `batch` int32 (either may be NULL).  Synchronous. */
int sj_kv_state(const sj_kv* kv, int32_t* len_host, int32_t* pending_host);

/* Runs the target over n prompt tokens (host array) of sequence seq, appends their K/V, advances
 * the length by n and sets the pending token to the arg-max continuation of the last prompt
 * token.  Uses the same kernels as the verification forward.  Synchronises `stream`. */
int sj_prefill(sj_model* m, sj_kv* kv, int32_t seq, const int32_t* tokens_host, int32_t n, void* stream);

/* One verification cycle for every sequence of the batch (Sec. 3.1 - 3.2).
 *   draft_tokens  device int32 [batch, gamma]        d_{t+1..t+gamma}                (Eq. 1)
 *   draft_probs   device float [batch, gamma, vocab] the draft distribution each d was drawn from
 *   uniforms      device float [batch, gamma+1]      in [0,1): entry j tests d_{j+1} (Eq. 3),
 *                                                    the last one draws the emitted token
 *   judge_threshold  theta of Eq. 5; >= 1 disables the judge, < 0 accepts every token
 *   accepted_len  device int32 [batch]  out: n in [0, gamma]
 *   next_token    device int32 [batch]  out: the extra token (bonus if n == gamma, else resampled)
 * Effects: K/V of the gamma+1 block rows are written at positions len..len+gamma; then
 * len += 1 + n and pending = next_token (rows beyond the new len are dead and get overwritten).
 * Errors: SJ_EINVAL (null, gamma outside 1..max_gamma), SJ_ECAPACITY.  Token ids are not read
 * on the host; a draft token outside [0, vocab) is clamped into range on the device. */
int sj_verify_step(sj_model* m, sj_kv* kv, int32_t gamma, const int32_t* draft_tokens,
                   const float* draft_probs, const float* uniforms, float judge_threshold,
                   int32_t* accepted_len, int32_t* next_token, void* stream);

/* Draft proposal (Sec. 2.2, Eq. 1): gamma sequential single-token decodes of a DRAFT model m for every
 * sequence of the batch, producing exactly what sj_verify_step of the target consumes.  Step j feeds
 * the sequence's pending token at position len, appends its K/V, forms q_j = softmax(logits / T) of that
 * row, draws d_{j+1} from q_j by inverse CDF in vocabulary order with uniforms[j][b] (the rule of the
 * extra token of sj_verify_step), makes it the pending token and advances len by 1.
 *   uniforms      device float [gamma, batch]        in [0,1), step-major
 *   feed_last     non-zero: after the last draw the layers (no LM head) also run on d_gamma, so the cache
 *                 holds a row for every drafted token and any accepted length can be kept by length alone
 *   draft_tokens  device int32 [batch, gamma]        out
 *   draft_probs   device float [batch, gamma, vocab] out, fp32 probabilities (one-hot at T = 0)
 * Effects: len += gamma (+1 with feed_last), pending = d_gamma.  After the target's verification accepted n
 * tokens and emitted e, the caller sets the draft cache to len0 + 1 + n, pending e (sj_kv_set_state /
 * sj_kv_rewind): rows beyond the new length are dead.  m is any model with the target's vocabulary.
 * Errors: SJ_EINVAL (null, gamma outside 1..63, head-only model), SJ_ECAPACITY. */
int sj_draft_block(sj_model* m, sj_kv* kv, int32_t gamma, const float* uniforms, int32_t feed_last,
                   int32_t* draft_tokens, float* draft_probs, void* stream);

/* Teacher-forced scoring of a block (Sec. 3.3 "Computing Semantic Preservation Score", Eq. 6 - 7: every term of
 * the score is the log-probability of a known next token after a known prefix).  For every sequence the n
 * given tokens are fed at positions len .. len+n-1 on top of the cache, and
 *   logprob[b][j] = log softmax(logits of row j / T)[target_tokens[b][j]].
 * With inputs [y_{i-1}, x, y_{i+1}, .., y_{i+N-1}] and targets [x, y_{i+1}, .., y_{i+N}] (x = y_i, then x = z_i)
 * the score is  s(y, z_i) = sum_j logprob_z[j] - sum_j logprob_y[j]  (two calls on the same cache).
 *   input_tokens, target_tokens  device int32 [batch, n], 1 <= n <= max_gamma + 1 (out-of-range ids are clamped)
 *   logprob      device float [batch, n] out
 *   hidden_out   device float [batch, d_model] out or NULL: the normed final hidden state of block row
 *                hidden_row (the judge's feature h_z of the token fed in that row, Eq. 4)
 * The cache state (len, pending) is NOT changed: the rows written at len.. are dead.  Launches eagerly.
 * Errors: SJ_EINVAL, SJ_ECAPACITY. */
int sj_score_block(sj_model* m, sj_kv* kv, int32_t n, const int32_t* input_tokens, const int32_t* target_tokens,
                   float* logprob, int32_t hidden_row, float* hidden_out, void* stream);

/* The verification tail alone (LM head, softmax, Eq. 3, Eq. 5, scan, resampling) on given final
 * hidden states: hidden = device [batch*(gamma+1), d_model] in the storage dtype, already
 * RMS-normed, row b*(gamma+1)+j = block row j of sequence b.  No cache is read or written; kv
 * supplies the workspace (it may come from a head-only model). */
int sj_verify_head(sj_model* m, sj_kv* kv, int32_t gamma, const void* hidden,
                   const int32_t* draft_tokens, const float* draft_probs, const float* uniforms,
                   float judge_threshold, int32_t* accepted_len, int32_t* next_token, void* stream);

/* sj_verify_head for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same inputs, outputs and arithmetic as sj_verify_head in the default
 * two-stage mode, but no sj_kv: the workspace is a static device array of SJ_STATIC_WORKSPACE_BYTES that every
 * GPU the library runs on holds until the process ends.  The call allocates nothing (no hipMalloc / hipFree, no
 * allocating library routine) and launches its kernels on `stream`; outputs are valid once the stream is
 * synchronised.  Limits: batch * (gamma + 1) <= SJ_STATIC_MAX_ROWS, and the rows' logits, softmax partials and
 * resampling sums must fit the array (16 rows of a 128256-entry vocabulary at d_model 4096 do); anything larger
 * is refused with SJ_EINVAL before any launch.  All calls on one GPU share the array, which keeps the previous
 * call's contents: calls that overlap on one GPU (different streams or threads) race - serialise them. */
#define SJ_STATIC_MAX_ROWS 32
#define SJ_STATIC_WORKSPACE_BYTES (16u << 20)
int sj_verify_head_static(sj_model* m, int32_t batch, int32_t gamma, const void* hidden,
                          const int32_t* draft_tokens, const float* draft_probs, const float* uniforms,
                          float judge_threshold, int32_t* accepted_len, int32_t* next_token, void* stream);

/* Training of the judge verifier (Sec. 3.4 "Verifier Training", appendix "Training Logistic Regressor"):
 * for every C of the grid, the L2-regularised logistic regression
 *     min over (w, b) of  1/2 |w|^2 + C * sum_i log(1 + exp(-(2 y_i - 1) (w . h_i + b)))      (bias unpenalised)
 * on the training pairs (h_i, y_i); the model with the best ROC-AUC on the validation pairs is kept (equal AUC:
 * the earlier C), and two thresholds for Eq. 5 are chosen on its validation scores sigmoid(w . h + b):
 *   theta_f1      best F1 of the rule "acceptable when score > theta" over theta in {0} and every validation
 *                 score (equal F1: the smallest theta)                                  - the "-F" setting
 *   theta_recall  the largest score of an unacceptable validation sample: the most permissive threshold that
 *                 still rejects all of them                                             - the "-R" setting
 * The paper's grid is 10 logarithmically spaced values from 1e-3 to 1e2.
 *   H_train [n_train, d], H_val [n_val, d]   DEVICE, fp32, row-major, 16-byte aligned (the feature rows
 *                                            sj_score_block / sj_debug_fetch return); d a multiple of 4, <= 8192
 *   y_train [n_train], y_val [n_val]         DEVICE, int32, 1 = acceptable, 0 = not; both classes in each set
 *   C_grid [n_C]                             HOST, positive
 *   w_all [n_C, d + 1] (may be NULL)         HOST out: (w, b) of every C
 *   auc [n_C]                                HOST out: validation ROC-AUC of every C
 *   passes [n_C] (may be NULL)               HOST out: passes over H_train the solver made
 *   best_index, w_best [d + 1], theta_f1, theta_recall   HOST out: the kept model (w, then b) and its thresholds
 * Everything is computed on the device in fp64 (features read as fp32); the call allocates its workspace
 * (about 8 (n_train + 3 n_val) + 2 MB * (d / 1024) bytes), synchronises `stream` and frees it before returning.
 * Errors: SJ_EINVAL (null / misaligned pointer, sizes, a label other than 0 / 1, a set with one class only,
 * non-positive C), SJ_ENOMEM, SJ_EHIP (also when the solver fails to converge). */
int sj_judge_train(const float* H_train, const int32_t* y_train, int64_t n_train, const float* H_val,
                   const int32_t* y_val, int64_t n_val, int32_t d, const double* C_grid, int32_t n_C,
                   double* w_all, double* auc, int32_t* passes, int32_t* best_index, double* w_best,
                   double* theta_f1, double* theta_recall, void* stream);

/* Verifier variants of the paper's ablations and baselines, applied by the following steps:
 *   SJ_MODE_TWO_STAGE (default)  either test approves          (App. D.2)
 *   SJ_MODE_ALIGNMENT            Eq. 3 only (standard speculative decoding)
 *   SJ_MODE_JUDGE                Eq. 5 only
 *   SJ_MODE_TOPK                 the relaxed baseline of Sec. 4.1: d_j is kept when fewer than k entries of
 *                                the target's row precede it (larger logit, or equal logit at a lower
 *                                index); k = 2 (the paper's setting) unless sj_set_topk changes it.
 * In every mode the extra token after a rejection comes from the residual rule of Sec. 2.2.
 * Errors: SJ_EINVAL for a null handle, an unknown mode or k < 1. */
#define SJ_MODE_TWO_STAGE 0
#define SJ_MODE_ALIGNMENT 1
#define SJ_MODE_JUDGE     2
#define SJ_MODE_TOPK      3
int sj_set_mode(sj_kv* kv, int32_t mode);
int sj_set_topk(sj_kv* kv, int32_t k);

/* Sets every sequence's length and pending token from host arrays of `batch` entries, asynchronously
 * on `stream` (a benchmark or a caller rolling back uses it to replay a step from the same state).
 * Cache contents are not touched: rows below the new length must already hold valid K/V. */
int sj_kv_rewind(sj_kv* kv, const int32_t* len_host, const int32_t* pending_host, void* stream);

/* Measurement aid.  kernel_class != 0 makes the following sj_verify_step calls bracket every launch
 * of that class with HIP events on the step's stream: 1 = QKV projection, 2 = O projection,
 * 3 = gate/up projection + SwiGLU, 4 = down projection (timed steps are launched kernel by kernel, not as
 * a captured graph).  sj_get_kernel_timing synchronises, returns the summed duration and launch count since the
 * last call, and clears them.  0 switches it off. */
int sj_set_kernel_timing(sj_kv* kv, int32_t kernel_class);
/* Launches the projection kernel of class 1..4, or 5 = the LM-head product with its softmax partials,
 * `launches` times back to back on `stream`, cycling through
 * the layers' weights (so nothing is re-read from cache) with the operands left by the last step, and
 * returns the elapsed time between two HIP events around the whole series.  Synchronises `stream`. */
int sj_time_kernel_class(sj_model* m, sj_kv* kv, int32_t kernel_class, int32_t launches, void* stream, double* total_ms);
int sj_get_kernel_timing(sj_kv* kv, double* total_ms, int64_t* launches);
/* Writes into buf (host, buf_len bytes, always terminated) the name and launch shape of the kernel that a step of
 * `rows` = batch * (gamma + 1) rows on this cache object uses for kernel class 1..5 (as above): the shape comes from
 * the rule or from the start-up measurement, so a report of a timing can say what was timed. */
int sj_kernel_class_shape(const sj_kv* kv, int32_t kernel_class, int32_t rows, char* buf, int32_t buf_len);

/* bf16 models only: how many bf16 planes carry the fp32 activations (the few-row operand of every
 * matrix product) into the matrix cores.  1 = activations rounded to bf16 at each product
 * (relative 2^-9), 2 = hi + lo planes (2^-18, the default), 3 = exact fp32.  Weights and cache are
 * bf16 in every case and the bytes streamed from HBM do not change.  Ignored for fp32 models. */
int sj_set_operand_planes(sj_kv* kv, int32_t planes);

/* Intermediate results of the last step, copied to the host (synchronous; for parity tests).
 *   SJ_DBG_LOGITS       float [rows, vocab]     rows = batch*(gamma+1)
 *   SJ_DBG_HIDDEN       float [rows, d_model]   final hidden states after the last RMSNorm
 *   SJ_DBG_JUDGE_SCORES float [batch, gamma]    sigmoid scores, entry j for d_{j+1}
 *   SJ_DBG_P_AT_DRAFT   float [batch, gamma]    p(d_{j+1}) under the target
 *   SJ_DBG_ACCEPT_BITS  int32 [batch, gamma]    bit0 = Eq. 3 accepted, bit1 = judge accepted,
 *                                               bit2 = top-k accepted (top-k mode only)
 * nbytes must equal the size above for the gamma of the last step. */
#define SJ_DBG_LOGITS       0
#define SJ_DBG_HIDDEN       1
#define SJ_DBG_JUDGE_SCORES 2
#define SJ_DBG_P_AT_DRAFT   3
#define SJ_DBG_ACCEPT_BITS  4
int sj_debug_fetch(const sj_kv* kv, int32_t what, void* dst_host, size_t nbytes);

/* Temperature T of the target distribution p = softmax(l / T) of Eq. 2 (0 = one-hot at the lowest-index arg-max, the
 * setting of the paper's experiments, Sec. 4.1), replacing sj_config.temperature from the next call on for every cache
 * object of the model.  Synchronises the device.  Errors: SJ_EINVAL (null, negative or NaN). */
int sj_set_temperature(sj_model* m, float temperature);

/* Bytes of weights one step streams from HBM (all projections + LM head), for roofline math. */
int64_t sj_model_weight_bytes(const sj_model* m);

const char* sj_last_error(void);
const char* sj_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SJ_H */
