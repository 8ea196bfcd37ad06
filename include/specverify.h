/*
 * specverify - the verify pass of speculative sampling with KV caching on one MI355X (gfx950).
 *
 * C ABI of the GPU library.  Every pointer marked "dev" is device memory owned by the caller
 * (for instance a PyTorch allocation); everything marked "host" is host memory.  The library
 * never frees caller memory.  `stream` is a hipStream_t passed as void* (NULL = the null
 * stream); all work of a call is enqueued on it and, unless a call says otherwise, nothing
 * synchronises with the host.  Handles are not thread-safe: one stream per handle at a time.
 * Hot-path calls (ss_verify_forward, ss_draft_step, ss_softmax, ss_top_p_filter, ss_top_k_filter,
 * ss_speculative_accept*, ss_greedy_accept, ss_kv_cache_rollback, ss_kv_cache_truncate) allocate
 * nothing and never wait for the device: the entry points without a handle take a caller-owned
 * device workspace (ss_workspace_bytes, ss_workspace_init), the others use what their model
 * allocated when it was created.
 *
 * Return value of every call: SS_OK (0) or a negative code.  Arguments are validated on the
 * host before anything is launched, so SS_EINVAL / SS_ECAPACITY never leave partial device
 * state behind.  ss_last_error() returns a message for the calling thread's last failure.
 * Values that only the device sees (token ids) are clamped into range by the kernels and the
 * event is recorded in a device status word: of the model (ss_device_status) for calls that take
 * one, of the workspace (ss_workspace_status) for the others.
 *
 * Method references are to the paper's sections: Section 3 (autoregressive vs speculative
 * sampling, the K-rows-for-the-price-of-one premise, recovery of the target distribution),
 * Sections 2/4.2 (KV caching), Section 4.3 (draft proposes, target accepts or rejects),
 * Section 4.4 (two caches of different size; the target cache goes stale and is rolled back).
 */
#ifndef SPECVERIFY_H
#define SPECVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SS_OK 0
#define SS_EINVAL (-1)    /* NULL pointer, bad shape, unsupported size */
#define SS_ECAPACITY (-2) /* KV cache or workspace too small for the request */
#define SS_EHIP (-3)      /* a HIP runtime call failed; see ss_last_error() */
#define SS_EABORTED (-4)  /* a bounded wait inside the persistent verify kernel gave up; the call's results are invalid */

#define SS_DTYPE_F32 0
#define SS_DTYPE_BF16 1

#define SS_QUANT_NONE 0
#define SS_QUANT_INT8 1
#define SS_QUANT_INT4_G128 2

#define SS_MAX_ROWS_PER_SEQ 16 /* M = K + 1 query rows per sequence in one call */

typedef void *ss_stream; /* hipStream_t */

/* Decoder shape (Llama style: RMSNorm, rotary embedding with split-half pairing, MHA, SwiGLU,
 * no biases, untied LM head).  head_dim must be a multiple of 32, d_model and d_ff multiples of
 * 8 (bf16) or 4 (f32).  dtype is the storage type of weights and of the KV cache. */
typedef struct {
    int32_t n_layers, d_model, n_heads, head_dim, d_ff, vocab;
    float rope_base, rms_eps;
    int32_t dtype;    /* SS_DTYPE_F32 | SS_DTYPE_BF16 */
    int32_t max_rows; /* largest batch * M any call on this model will pass */
    int32_t max_pos;  /* rotary table length: positions 0..max_pos-1 */
    int32_t weight_quant; /* SS_QUANT_NONE: matrices in the storage type.  Otherwise the four matrices of every
                           * layer and the LM head are quantised weight-only (the quantised model that Sections 2
                           * and 3 assume; the paper fixes no precision, these are this library's two readings):
                           * SS_QUANT_INT8: int8, one fp32 scale per output row (ss_quantize_rows_int8); d_model,
                           *   n_heads*head_dim and d_ff multiples of 16;
                           * SS_QUANT_INT4_G128: int4, two entries per byte, one fp32 scale per group of 128 entries
                           *   along K (ss_quantize_rows_int4); those three sizes multiples of 128.
                           * Both need dtype bf16.  The embedding, the gains and the KV cache keep the storage type;
                           * such a model runs with one launch per phase (the persistent kernel streams
                           * storage-type matrices only). */
} ss_model_cfg;

/* One layer's weights, dev pointers, row-major [out_features][in_features] in the storage type:
 *   wqkv [3*H*hd][d]  rows 0..H*hd-1 = W_q, then W_k, then W_v
 *   wo   [d][H*hd]
 *   wgu  [2*F][d]     rows 0..F-1 = W_gate, rows F..2F-1 = W_up
 *   wd   [d][F]
 *   g1, g2 [d] fp32   RMSNorm gains before attention / before the FFN */
typedef struct {
    const void *wqkv, *wo, *wgu, *wd;
    const float *g1, *g2;
    const float *sqkv, *so, *sgu, *sd; /* quantised models only: dev fp32 scales of the four matrices above, which are
                                        * then int8 [rows][K] or packed int4 [rows][K/2] of the same shapes.
                                        * INT8: one per row ([3*H*hd], [d], [2*F], [d]); INT4_G128: group-major
                                        * [K/128][rows].  Else ignored. */
} ss_layer_weights;

typedef struct {
    const void *embed;              /* dev [vocab][d], storage type */
    const ss_layer_weights *layers; /* host array [n_layers] of dev pointers */
    const float *gf;                /* dev [d] fp32 final RMSNorm gain */
    const void *lm_head;            /* dev [vocab][d], storage type (quantised models: int8 [vocab][d] / int4 [vocab][d/2]) */
    const float *s_head;            /* quantised models only: dev fp32 scales of lm_head, [vocab] / [d/128][vocab] */
} ss_weights;

typedef struct ss_model ss_model;
typedef struct ss_kv_cache ss_kv_cache;

const char *ss_last_error(void);

/* Releases everything the library still holds on every device: all live models and caches are destroyed
 * (their handles become invalid; a later ss_model_destroy / ss_kv_cache_free on them is a no-op).  Meant to be
 * called once before the process ends, while the HIP runtime is still up (a Python binding registers it with
 * atexit), so that no device memory is released from static destructors or interpreter teardown. */
int ss_shutdown(void);

/* For callers that must prove their decode loop allocates nothing: while `on` is non-zero every path of the
 * library that would allocate device memory (ss_model_create, ss_kv_cache_alloc / ss_kv_cache_create) fails with
 * SS_EHIP instead.  The hot-path calls are unaffected: they never allocate.  Switching it on also completes, on the
 * current device, the one-off set-up that ss_speculative_accept_noalloc would otherwise do in its first call there
 * (its built-in scratch array receives its device address), so that call does no set-up work afterwards. */
int ss_freeze_allocations(int32_t on);

/* Reads and clears the device status word of `model` (synchronises `stream`).
 * bit 0: a token id outside [0, vocab) reached a kernel and was clamped.
 * bit 1: a device-wide barrier of the persistent verify kernel gave up waiting (its spin is bounded);
 *        the results of that call are invalid and the barrier state has been reset. */
int ss_device_status(ss_model *model, ss_stream stream, int32_t *status_host);

/* ---- measurement ----------------------------------------------------------------------------
 * With profiling on, every kernel launch of the forward path on `model` is bracketed by a HIP
 * event pair recorded on the call's stream.  ss_profile_read waits for the recorded events, adds
 * the elapsed times up per kernel class and clears the record.  Classes (n_classes >= 9):
 * 0 RMSNorm, 1 QKV GEMM (+rotary, +cache append), 2 attention (+merge), 3 O-projection GEMM,
 * 4 gate/up GEMM (+SwiGLU), 5 down-projection GEMM, 6 LM-head GEMM, 7 other, 8 the persistent
 * verify kernel (with ss_model_set_persistent(model, 1) the whole forward of a small call is one launch of it).
 * total_ms_host / launches_host: host arrays [n_classes].  Event recording perturbs the pass a
 * little, so timed throughput runs keep it off. */
int ss_profile_enable(ss_model *model, int32_t on);
int ss_profile_read(ss_model *model, int32_t n_classes, double *total_ms_host, int64_t *launches_host);

/* Weight-only int8 of a matrix w_dev [rows][K] held in storage type `dtype` (the reading taken of the
 * quantised model Sections 2 and 3 assume; the precision is not fixed there): per row n,
 * scale_dev[n] = fl32(max_k |w[n][k]| / 127) (1 for an all-zero row) and q_dev[n][k] = the nearest
 * integer, ties to even, of fl32(w[n][k] / scale_dev[n]), in [-127, 127].  The row then stands for the
 * real numbers scale[n] * q[n][k].  q_dev: dev int8 [rows][K]; scale_dev: dev fp32 [rows]; both the
 * caller's.  Enqueued on `stream`, no host synchronisation.  rows, K >= 1. */
int ss_quantize_rows_int8(const void *w_dev, int32_t dtype, int64_t rows, int64_t K, int8_t *q_dev, float *scale_dev,
                          ss_stream stream);

/* Weight-only int4 with group scales of the same matrix: along K, groups of 128 consecutive entries of a row share
 * scale = fl32(max |w| / 7) over the group (1 for an all-zero group); q = the nearest integer, ties to even, of
 * fl32(w / scale), in [-7, 7].  q_dev: dev uint8 [rows][K/2], byte b of a row = entry 2b in the low and entry 2b+1
 * in the high four bits (two's complement); scale_dev: dev fp32 [K/128][rows] (group-major).  K a multiple of 128. */
int ss_quantize_rows_int4(const void *w_dev, int32_t dtype, int64_t rows, int64_t K, uint8_t *q_dev, float *scale_dev,
                          ss_stream stream);

/* Read-stream probe of the device the caller has made current: a plain kernel that reads
 * buf_dev[0, bytes) once per launch with wide independent loads and keeps nothing.  One untimed
 * launch, then `iters` launches timed with a HIP event pair on `stream`; *gbps_host receives
 * bytes * iters / elapsed in GB/s (synchronises `stream`).  It gives the HBM read rate a kernel
 * with no dependencies reaches on this device, the practical ceiling the verify pass (a weight
 * stream: Section 2 describes decoding as bound by memory bandwidth) is judged against next to the
 * nominal figure.
 * buf_dev: dev, 16-byte aligned, bytes a multiple of 16 and >= 1 MiB, contents arbitrary, never
 * written; take it larger than the last-level cache or the figure is a cache rate.
 * sink_dev: dev, one uint32 the kernel may write.  iters in [1, 10000]. */
int ss_probe_read_bandwidth(const void *buf_dev, size_t bytes, int32_t iters, uint32_t *sink_dev, double *gbps_host,
                            ss_stream stream);

/* ---- model -------------------------------------------------------------------------------
 * Creates a handle over caller-owned weights (which must outlive it) and allocates the
 * model's activation workspace and rotary table on the current device (the only allocations
 * the forward path ever makes).  A draft that reuses the target's first layers is simply a
 * second model whose pointers alias the target's. */
int ss_model_create(const ss_model_cfg *cfg, const ss_weights *weights, ss_model **out);
int ss_model_destroy(ss_model *model);

/* Selects how the forward path of `model` is launched.  0 (default): one kernel per phase (RMSNorm, QKV
 * GEMM, attention, O projection, gate/up GEMM, down projection ...) for every call.  1: calls whose rows
 * (batch * M) fit the kernel's LDS activation slab (9 rows for bf16 models, 16 for fp32) run as ONE
 * persistent kernel (one workgroup per compute unit, phases ordered by device-wide barriers or by
 * self-validating activations, RMSNorm folded into the GEMMs, weight loads of the next phase in flight
 * across each phase boundary); larger calls still use one kernel per phase.  Measured on the 7B-, 13B- and
 * 3B-shaped models the per-phase path is ahead at every row count from 1 to 9 (by 28 - 39 % on the 7B shape,
 * 35 - 50 % on the other two), which is why the simpler one is the default.  Both paths
 * produce results within the same tolerance of the method; SS_EINVAL if `on` is set and the persistent
 * kernel is not available on this device (it needs every workgroup co-resident, and matrices in the
 * storage type). */
int ss_model_set_persistent(ss_model *model, int32_t on);

/* Tuning and test knobs of the persistent kernel (no effect on the per-phase path).
 * workgroups: size of the grid (every workgroup must be resident at once); 0 = default (one per compute unit), at most that.
 * data_sync: 1 (default): between GEMM phases the consumers validate the activation data itself
 * (elements not yet written carry a reserved bit pattern) instead of waiting at a device-wide
 * barrier; used for a launch only when every workgroup owns part of every GEMM phase (grid <=
 * d_model, d_ff, vocab and 3*n_heads*head_dim/16), otherwise, and with 0, every phase boundary is a
 * barrier.  Results are identical bit for bit in both modes.  SS_EINVAL on a NULL model, a negative or
 * too large grid, or when the persistent kernel is not available. */
int ss_model_set_persistent_options(ss_model *model, int32_t workgroups, int32_t data_sync);

/* Every wait inside the persistent kernel is bounded: after `polls` unsuccessful looks at what it waits
 * for (default 2^20, about a second), a workgroup raises the kernel's abort flag and leaves; every other
 * workgroup leaves at its next wait, the call's results are invalid, and ss_device_status reports bit 1
 * and resets the synchronisation state, after which the model works again.  A small limit makes a call
 * fail fast (and is how the failure path is tested: the kernel still ends normally).  polls >= 1. */
int ss_model_set_wait_limit(ss_model *model, uint32_t polls);

/* Development aid, not part of the method: while buf_dev (dev, `entries` 64-bit words, zero-filled by the caller)
 * is set and entries >= 5 * phases * workgroups of a launch, every workgroup of the persistent kernel records
 * the device clock at five points of each phase (start, prologue done, first activation slab in LDS, last
 * round done, end) at buf[(5 * phase + point) * workgroups + workgroup].  NULL switches it off. */
int ss_model_set_timeline(ss_model *model, unsigned long long *buf_dev, size_t entries);

/* ---- KV cache (Sections 2, 4.2: keys and values of past tokens are kept instead of recomputed;
 *      Section 4.4: the caches of the two models have different sizes and the target's goes stale) ----
 * A contiguous, page-free cache for `batch` sequences of up to `max_seq` positions in the model's
 * storage type.  The keys and values live in ONE caller-owned device buffer of
 * ss_kv_cache_bytes(model, batch, max_seq) bytes (16-byte aligned); the library owns only the handle
 * and a device array len[batch] of current lengths (all 0 after creation).
 * Layout of the buffer: all keys, then all values; per layer l, sequence b, head h (S = max_seq rounded
 * up to 64):
 *   K[l][b][h][S][hd]           keys, already rotated, one row per position
 *   V[l][b][h][S/64][hd][64]    values, transposed inside blocks of 64 positions
 * ss_kv_cache_create clears the buffer (enqueued on `stream`; this call is off the hot path): the
 * attention kernel multiplies the value entries of masked positions inside a sequence's last block of
 * 64 by weights that are exactly zero, so those entries must hold finite numbers.  From then on only
 * this library writes the buffer.  The buffer must outlive the handle; the library never frees it.
 * A model with fewer layers but the same heads and storage type may be run on such a cache: it uses
 * the leading layers (an early-exit draft sharing the target's cache, Section 4.4).
 * ss_kv_cache_alloc is the same with a buffer the library allocates (and frees in ss_kv_cache_free). */
size_t ss_kv_cache_bytes(const ss_model *model, int32_t batch, int32_t max_seq);
int ss_kv_cache_create(const ss_model *model, int32_t batch, int32_t max_seq, void *buf_dev, size_t buf_bytes,
                       ss_stream stream, ss_kv_cache **out);
int ss_kv_cache_alloc(const ss_model *model, int32_t batch, int32_t max_seq, ss_kv_cache **out);
int ss_kv_cache_free(ss_kv_cache *kv);

/* kv_cache_append: raw append for one sequence and one layer of n_rows rows of already-rotated
 * keys and of values, dev [n_rows][H*hd] in the storage type, at positions pos0..pos0+n_rows-1.
 * Lengths do not move; call ss_kv_cache_set_len once all layers are written.  Used to build an
 * existing context; ss_verify_forward / ss_draft_step append their own rows. */
int ss_kv_cache_append(ss_kv_cache *kv, int32_t layer, int32_t seq, int32_t pos0, const void *k_dev,
                       const void *v_dev, int32_t n_rows, ss_stream stream);

/* Sets every sequence's length from a host array [batch] (0 <= len <= max_seq); may raise a length (after
 * raw appends) as well as lower it.  Synchronises `stream` (the host array is read asynchronously): for
 * building contexts, not for the decode loop.  Rows past a length are dead and get overwritten by later
 * appends: truncation moves no data (Section 4.4). */
int ss_kv_cache_set_len(ss_kv_cache *kv, const int32_t *len_host, ss_stream stream);
/* Truncation from a DEVICE array (Section 4.4: the stale tail of a cache is dropped by moving its length):
 * len[b] = min(len[b], max(new_len_dev[b], 0)) for every sequence, enqueued on `stream`, no host
 * synchronisation.  A value above the current length leaves it unchanged and sets bit 2 of the status word
 * status_dev points to (dev int32, may be NULL).  new_len_host (host int32 [batch], may be NULL) lets the
 * library tighten the host-side upper bound it keeps for its capacity checks. */
int ss_kv_cache_truncate(ss_kv_cache *kv, const int32_t *new_len_dev, const int32_t *new_len_host, int32_t *status_dev,
                         ss_stream stream);
/* Copies the device lengths to a host array [batch]; synchronises `stream`. */
int ss_kv_cache_get_len(ss_kv_cache *kv, int32_t *len_host, ss_stream stream);

/* Roll-back after the rejection step, entirely on the device: a verify call appended M rows per
 * sequence, of which only the first n_accepted[b] + 1 (the last committed token and the accepted
 * draft tokens) stay:  len[b] -= M - 1 - n_accepted[b].  n_accepted_dev is dev int32 [batch]
 * with 0 <= n_accepted[b] <= M - 1 (values outside are clamped).  The library keeps a host-side upper
 * bound of every length for its capacity checks; n_accepted_host (host int32 [batch], may be NULL)
 * lets it keep that bound exact, otherwise the bound stays at the unrolled length until the next
 * ss_kv_cache_get_len / ss_kv_cache_set_len. */
int ss_kv_cache_rollback(ss_kv_cache *kv, const int32_t *n_accepted_dev, const int32_t *n_accepted_host,
                         int32_t M, ss_stream stream);

/* ---- target verify pass (Section 3: K draft tokens + 1 bonus row in one pass) ---------------
 * tokens_dev int32 [batch][M] = [last committed token, d_1..d_K] per sequence, 1 <= M <= 16.
 * Runs the decoder over the batch*M rows at positions len[b]..len[b]+M-1, appends their keys
 * and values to the cache (len[b] += M) and writes logits_dev fp32 [batch][M][vocab].
 * Also serves prefill in chunks of <= 16 rows. logits_dev may be NULL (cache fill only). */
int ss_verify_forward(ss_model *model, ss_kv_cache *kv, const int32_t *tokens_dev, int32_t batch,
                      int32_t M, float *logits_dev, ss_stream stream);

/* The decoder layers of the same pass alone (Section 3: the target scores all rows of a call together;
 * Sections 2, 4.2: against the cache) over given hidden rows h_dev fp32 [batch*M][d], updated in place:
 * everything ss_verify_forward does between the embedding and the final norm, cache append included.
 * The entry point of the one-layer workload. */
int ss_decoder_layers_forward(ss_model *model, ss_kv_cache *kv, float *h_dev, int32_t batch, int32_t M,
                              ss_stream stream);

/* ---- draft step (Section 4.3: the draft model proposes one token per call) ------------------
 * tokens_dev int32 [batch][m], m in {1..16} (m = 2 is the catch-up after a fully accepted step).
 * Runs `draft` over the rows, takes the last row's logits of each sequence, and
 *   temperature > 0 : q = softmax(logits / temperature) written to q_rows_dev + b*ldq (fp32
 *                     [vocab]); token ~ q by the integer inverse CDF with uniform u_dev[b]
 *   temperature == 0: token = argmax (lowest index on ties); q_rows_dev and u_dev may be NULL.
 * top_p < 1 (temperature > 0 only): q is restricted to its top-p nucleus and renormalised before
 * the token is drawn (see ss_top_p_filter), and that filtered row is what q_rows_dev receives;
 * top_p >= 1: no filtering; top_p <= 0: SS_EINVAL.
 * top_k >= 1 (temperature > 0 only): q is first restricted to its top_k most probable tokens (see
 * ss_top_k_filter), top-p then works on that row; top_k == 0 or >= vocab: no filtering; < 0: SS_EINVAL.
 * token_out_dev int32 [batch].  Calling it on the target model is an autoregressive decode step. */
int ss_draft_step(ss_model *draft, ss_kv_cache *draft_kv, const int32_t *tokens_dev, int32_t batch,
                  int32_t m, float temperature, float top_p, int32_t top_k, const float *u_dev, float *q_rows_dev,
                  int64_t ldq, int32_t *token_out_dev, ss_stream stream);

/* ---- top-p ("nucleus") selection (Section 3 names sampling from the top-p set beside argmax) --------
 * Every row of probs_dev fp32 [rows][vocab] is restricted to its most probable tokens whose
 * probabilities add up to at least top_p, and renormalised.  The paper gives no arithmetic; this is
 * the rule, chosen so that any implementation keeps the same set:
 *   w_v = min(trunc(p_v * 2^32), 2^32 - 1); S = sum_v w_v (S = 0: the row is returned unchanged);
 *   P24 = nearest integer to top_p * 2^24 (ties to even), clamped to [1, 2^24];
 *   target = ceil(P24 * S / 2^24), at least 1;
 *   kept = the shortest prefix, in the order (w descending, index ascending), whose weights add
 *          up to >= target; S' = their sum; Z' = fl32(S') * 2^-32;
 *   out_v = fl32(p_v / Z') for kept v, 0 otherwise.
 * Filtering the target's and the draft's rows alike and then applying the rejection step emits the
 * filtered target distribution.  out_dev may be probs_dev (in place).  top_p >= 1 copies the rows
 * unchanged; top_p <= 0 is SS_EINVAL. */
int ss_top_p_filter(const float *probs_dev, int32_t rows, int32_t vocab, float top_p, float *out_dev,
                    ss_stream stream);

/* ---- top-k selection (Section 3 lists top-k with top-p among the usual selection rules) ------------
 * Every row of probs_dev fp32 [rows][vocab] is restricted to its top_k most probable tokens and
 * renormalised, in the arithmetic of ss_top_p_filter: weights w_v as there; kept = the first top_k tokens
 * in the order (w descending, index ascending); S' = the sum of their weights (S' = 0: the row is
 * returned unchanged); Z' = fl32(S') * 2^-32; out_v = fl32(p_v / Z') for kept v, 0 otherwise.
 * Where both rules are in force (ss_draft_step, ss_speculative_step) top-k is applied first.
 * out_dev may be probs_dev.  top_k >= vocab copies the rows unchanged; top_k < 1 is SS_EINVAL. */
int ss_top_k_filter(const float *probs_dev, int32_t rows, int32_t vocab, int32_t top_k, float *out_dev,
                    ss_stream stream);

/* ---- device workspace of the entry points that take no handle ---------------------------------
 * ss_softmax, ss_speculative_accept, ss_speculative_accept_logits and ss_greedy_accept keep their
 * intermediate results (row statistics, per-segment partial sums, arrival counters, a status word) in a
 * caller-owned device buffer, so that none of them allocates or waits for the device.
 * ss_workspace_bytes(rows, vocab): size that serves any of these calls touching at most `rows` rows of
 * `vocab` logits or probabilities in total (softmax: rows; accept: batch * (2K + 1); greedy: batch * (K + 1)).
 * ss_workspace_init: clears the buffer (enqueued on `stream`); call it once after allocating.  After that
 * the buffer must only be passed to this library, to one call at a time (calls on different streams
 * need different workspaces); every call leaves it ready for the next.  A call whose need exceeds
 * ws_bytes returns SS_ECAPACITY before anything is launched.
 * ss_workspace_status reads and clears the workspace's status word (synchronises `stream`):
 * bit 0: a draft token id outside [0, vocab) reached the rejection step and was treated as rejected. */
size_t ss_workspace_bytes(int64_t rows, int32_t vocab);
int ss_workspace_init(void *ws_dev, size_t ws_bytes, ss_stream stream);
int ss_workspace_status(void *ws_dev, size_t ws_bytes, ss_stream stream, int32_t *status_host);

/* ---- softmax (the per-position distributions p and q of Section 3 that the rejection step compares;
 *      per-row statistics by wavefront reductions over the vocabulary) ----------------------------
 * probs_dev[r][v] = exp(logits[r][v]/T - max_r) / sum_v exp(...), fp32 [rows][vocab], evaluated with the
 * hardware base-2 exponential and one reciprocal per row (relative error a few 1e-6).  Every entry
 * point of the library that turns logits into probabilities produces these same bits.
 * ws_dev / ws_bytes: workspace, at least ss_workspace_bytes(rows, vocab). */
int ss_softmax(const float *logits_dev, int32_t rows, int32_t vocab, float temperature, float *probs_dev,
               void *ws_dev, size_t ws_bytes, ss_stream stream);

/* ---- modified rejection step (Sections 3, 4.3) -----------------------------------------------
 * p_dev fp32 [batch][K+1][vocab] target probabilities, q_dev fp32 [batch][K][vocab] draft
 * probabilities, draft_tokens_dev int32 [batch][K], uniforms_dev fp32 [batch][K+1] (multiples of
 * 2^-24 in [0,1)).  For i = 0..K-1 in order, draft token d_i is accepted iff
 *     p_i(d_i) >= q_i(d_i)  or  fl32(u_i * q_i(d_i)) < p_i(d_i)         (probability min(1, p/q))
 * stopping at the first rejection; n_accepted[b] = a.  Then with u = uniforms[b][K]:
 *     a < K : next ~ norm(max(0, p_a - q_a));  a = K : next ~ p_K
 * by an integer inverse CDF: w_v = trunc(r_v * 2^32), S = sum w_v, threshold = (u*2^24 * S) >> 24,
 * token = smallest v whose inclusive prefix sum exceeds the threshold.  If the residual weights
 * are all 0 the target row itself is sampled; if those are all 0 too, its argmax.  The result is
 * a pure function of the input bits.  K may be 0.  n_accepted_dev, next_token_dev: int32 [batch].
 * ws_dev / ws_bytes: workspace, at least ss_workspace_bytes(batch * (2K + 1), vocab). */
int ss_speculative_accept(const float *p_dev, const float *q_dev, const int32_t *draft_tokens_dev,
                          const float *uniforms_dev, int32_t batch, int32_t K, int32_t vocab,
                          int32_t *n_accepted_dev, int32_t *next_token_dev, void *ws_dev, size_t ws_bytes,
                          ss_stream stream);

/* ss_speculative_accept for callers that cannot provide or allocate a workspace (code under HIP graph capture, tight
 * serving loops, harnesses that forbid allocation): the same kernels, with their scratch (per-segment weight sums,
 * status word) in a 64 KiB device array built into the library.  Allocates nothing, frees nothing, never waits for
 * the device.  Limit: 256 + 8 * batch * segments bytes must fit the array, where segments <= 16 is the number of
 * vocabulary segments per sequence the kernels use (batch * segments < 1024 + batch, and segments = 1 from batch
 * 1024 on): any batch up to 8160 at any vocabulary; beyond the limit SS_ECAPACITY, before anything is launched.  Every call on a device shares that
 * device's array: calls that overlap in time on one device (different streams) race; consecutive calls need no
 * clearing in between.  status_dev (dev int32, may be NULL): receives bit 0 when a draft token id outside
 * [0, vocab) was treated as rejected (NULL: the flag goes to a word of the array that no call reads).
 * Results are bit-identical to ss_speculative_accept. */
int ss_speculative_accept_noalloc(const float *p_dev, const float *q_dev, const int32_t *draft_tokens_dev,
                                  const float *uniforms_dev, int32_t batch, int32_t K, int32_t vocab,
                                  int32_t *n_accepted_dev, int32_t *next_token_dev, int32_t *status_dev, ss_stream stream);

/* Same step straight from logits: p = softmax(p_logits/T), q = softmax(q_logits/T) are never
 * materialised (one read of the logits for the row statistics, then a re-read of the one or two
 * rows the sampling needs; when the logits are large and no output below is asked for, rows behind
 * a sequence's first rejection, which the method never uses, are not read at all).  Returns exactly
 * what ss_speculative_accept returns on the
 * probabilities ss_softmax would produce.  p_out_dev / q_out_dev, if not NULL, receive those
 * probabilities ([batch][K+1][vocab] / [batch][K][vocab]).  temperature > 0.  No top-p here: a caller
 * that filters (ss_top_p_filter) materialises the probabilities and uses ss_speculative_accept.
 * ws_dev / ws_bytes: workspace, at least ss_workspace_bytes(batch * (2K + 1), vocab). */
int ss_speculative_accept_logits(const float *p_logits_dev, const float *q_logits_dev, float temperature,
                                 const int32_t *draft_tokens_dev, const float *uniforms_dev,
                                 int32_t batch, int32_t K, int32_t vocab, int32_t *n_accepted_dev,
                                 int32_t *next_token_dev, float *p_out_dev, float *q_out_dev,
                                 void *ws_dev, size_t ws_bytes, ss_stream stream);

/* Greedy mode (Section 3 names argmax as the deterministic selection rule; with one-hot p and q the
 * rejection rule of Sections 3 / 4.3 reduces to this): a draft token is accepted iff it equals the argmax
 * of its target row; next = argmax of the first mismatching row, or of the bonus row.  Ties go to the
 * lowest index (the paper does not say; any fixed rule keeps greedy speculative decoding equal to greedy
 * autoregressive decoding, i.e. speculation does not change what is generated, as Section 3 requires).
 * p_logits_dev fp32 [batch][K+1][vocab].  ws_dev / ws_bytes: workspace, at least
 * ss_workspace_bytes(batch * (K + 1), vocab). */
int ss_greedy_accept(const float *p_logits_dev, const int32_t *draft_tokens_dev, int32_t batch, int32_t K,
                     int32_t vocab, int32_t *n_accepted_dev, int32_t *next_token_dev, void *ws_dev, size_t ws_bytes,
                     ss_stream stream);

/* ---- one whole speculative step for a single sequence (Sections 3, 4.3, 4.4) -----------------
 * The calls above, issued back to back without returning to the caller, so that a decode loop
 * pays one library call and one host synchronisation per step:
 *   K x ss_draft_step on (draft, draft_kv): call 0 feeds feed_dev[0 .. *n_feed) (one token, or two
 *     after a step that accepted all K), call i > 0 feeds the token call i-1 produced; the draft's
 *     probability rows go to q_rows_dev [K][vocab] (temperature > 0);
 *   ss_verify_forward on (target, target_kv) over verify_tokens_dev [K+1] = [last committed token,
 *     d_1 .. d_K] -> logits_dev [K+1][vocab];
 *   temperature > 0: ss_softmax -> p_dev [K+1][vocab] (top_k >= 1: then ss_top_k_filter, top_p < 1: then
 *     ss_top_p_filter, in place, as the draft's calls did to their rows), then ss_speculative_accept with
 *     u_accept_dev [K+1]; temperature == 0: ss_greedy_accept (p_dev, q_rows_dev, u_*_dev unused);
 *   both caches rolled back to their committed length.
 * Outputs: result_dev int32 [2] = (n_accepted a, next token y); out_host int32 [K+2] = (a, y, d_1 ..
 * d_K) after a stream synchronisation; feed_dev / *n_feed are rewritten for the next step ([y], or
 * [d_K, y] when a == K: the draft cache is then one row short).
 * draft_kv == target_kv selects the shared-cache scheme for a draft made of the target's leading
 * layers (any model may run on the leading layers of a deeper cache with the same heads and storage
 * type): the draft's K calls append to the target's cache, the length is set back by K before the
 * verify pass rewrites those positions for every layer, and the feed is always one token.
 * All *_dev buffers are the caller's device memory; 1 <= K <= 15; both caches hold one sequence.
 * The step's softmax and rejection kernels use the target model's own workspace (allocated with the model).
 * Errors as in the calls it is made of; shapes and the room both caches need for the whole step
 * (draft: *n_feed + K - 1 rows, target: K + 1) are checked before the first of them runs, so a
 * refused step leaves both caches as they were.  SS_EABORTED: a bounded wait of the persistent kernel
 * gave up in one of the step's forward passes (the flag travels to the host with the step's result); the
 * synchronisation state of both models has been reset, both cache lengths have been put back to the
 * host-tracked values from before the step, *n_feed and feed_dev are unchanged, the outputs are invalid. */
int ss_speculative_step(ss_model *target, ss_kv_cache *target_kv, ss_model *draft, ss_kv_cache *draft_kv,
                        int32_t K, float temperature, float top_p, int32_t top_k, int32_t *feed_dev, int32_t *n_feed,
                        const float *u_draft_dev, const float *u_accept_dev, int32_t *verify_tokens_dev,
                        float *q_rows_dev, float *logits_dev, float *p_dev, int32_t *result_dev,
                        int32_t *out_host, ss_stream stream);

/* ---- one speculative step for a batch of sequences (Sections 3, 4.3, 4.4; every sequence accepts its own
 * number of tokens, so the cache lengths grow ragged) -------------------------------------------
 * The same calls as ss_speculative_step, each over `batch` sequences at once, with two caches of `batch`
 * sequences.  To keep every call rectangular the draft cache is kept one position shorter than in the
 * single-sequence step: with n_b committed tokens of sequence b the target cache holds n_b - 1 positions, the
 * draft cache n_b - 2, and feed_dev int32 [batch][2] holds every sequence's last two committed tokens (a prompt
 * has at least two; prefill the target with all but the last token, the draft with all but the last two).  The
 * first draft call feeds both tokens of every sequence (two rows each), the others one; after the rejection
 * step both caches keep a_b + 1 of the K + 1 positions they gained, and feed_dev is rewritten.  The price of
 * the rectangle is one draft row per sequence and step that the single-sequence step computes only after a
 * fully accepted step; the tokens are the same.
 * u_draft_dev fp32 [K][batch] (call-major), u_accept_dev fp32 [batch][K+1]; draft_tokens_dev int32
 * [2][K][batch] scratch; verify_tokens_dev int32 [batch][K+1]; q_rows_dev fp32 [batch][K][vocab]; logits_dev
 * and p_dev fp32 [batch][K+1][vocab]; result_dev int32 [2][batch] = (n_accepted, next token);
 * out_host int32 [batch][K+2] = (a_b, y_b, d_1 .. d_K) after a stream synchronisation.  temperature, top_p,
 * top_k as in ss_speculative_step.  The target model must have been created with max_rows >= batch * (K + 1),
 * the draft with max_rows >= 2 * batch.  Errors as in ss_speculative_step; SS_EABORTED restores both caches'
 * lengths, the feed is then stale (rebuild it from the caller's token history). */
int ss_speculative_step_batched(ss_model *target, ss_kv_cache *target_kv, ss_model *draft, ss_kv_cache *draft_kv,
                                int32_t batch, int32_t K, float temperature, float top_p, int32_t top_k,
                                int32_t *feed_dev, const float *u_draft_dev, const float *u_accept_dev,
                                int32_t *draft_tokens_dev, int32_t *verify_tokens_dev, float *q_rows_dev,
                                float *logits_dev, float *p_dev, int32_t *result_dev, int32_t *out_host,
                                ss_stream stream);

#ifdef __cplusplus
}
#endif
#endif /* SPECVERIFY_H */
