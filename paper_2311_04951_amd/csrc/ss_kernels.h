// Host-side declarations of the kernel launchers (defined in the .hip files) and the argument
// structs they take.  Everything here is plain data; the C ABI in include/specverify.h sits on top.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace ss {

enum Epilogue : int {
    EPI_STORE = 0,  // out[m][n] = acc
    EPI_RESID = 1,  // out[m][n] = resid[m][n] + acc
    EPI_SWIGLU = 2, // z[m][n] = silu(gate) * up, written as activation planes
    EPI_QKV = 3     // rotary embedding on q, k; q -> activation planes, k, v -> KV cache
};

// Skinny GEMM  out[R][N] = act[R][K] . W[N][K]^T  for a handful of rows R (weights streamed once).
struct GemmArgs {
    const void *W; // [N][K] storage type, row-major
    int N, K;
    const void *act; // activation planes [planes][R16][ld_act]
    size_t act_plane;
    int ld_act;
    int R; // valid rows
    // EPI_STORE / EPI_RESID
    float *out;
    const float *resid;
    int ldo;
    // EPI_SWIGLU (N = F; up rows start at W row F) and EPI_QKV (q rows): activation planes written
    void *act_out;
    size_t act_out_plane;
    int ld_act_out;
    // EPI_QKV
    int H, hd, M, S, max_pos;
    const int32_t *len;  // [batch] lengths before this call's append
    const float2 *rope;  // [max_pos][hd/2] (cos, sin)
    void *kcache, *vcache; // this layer's K and V
    // launches of more than 16 rows only: device workspace for split-K partial tiles (NULL: never split)
    float *splitk_ws;
    size_t splitk_ws_bytes;
    int ksplit, kslabs; // set by the launcher: K splits, K slabs per split
    int splitk_rows;    // set by the launcher: partials are plain rows [split][R][N] (EPI_RESID), not accumulator tiles
    // EPI_RESID, optional: the RMSNorm that follows the projection (gain over the N output columns; planes
    // [planes][R16][norm_ld]).  A launcher that can fold it into its last launch does and returns true.
    const float *norm_gain;
    void *norm_act;
    size_t norm_act_plane;
    int norm_ld;
    float norm_eps;
    // ... a launcher of at most 16 rows defers it instead (returns 2): the planes receive h * gain without the row
    // scale, and nsq_out[row * nsq_ld + tile] the sum of squares of the 16 columns of each output tile.  The GEMM that
    // consumes such planes gets act_nsq / act_nsq_tiles / act_nsq_ld (and norm_eps) and multiplies its sums by
    // 1 / sqrt(sum over the tiles / K + eps) of the row: the norm is linear in the row scale.
    float *nsq_out;
    int nsq_ld;
    const float *act_nsq;
    int act_nsq_tiles, act_nsq_ld;
    // weight-only int8: W is int8 [N][K] and output column n is scaled by wscale[n] (NULL: W is in the storage type).
    // bf16 activation planes only; K a multiple of 16.
    const float *wscale;
    int wbits; // with wscale: 8 = int8, one scale per output column; 4 = int4, two entries per byte, scales [K/128][columns] (at most 16 rows, K % 128 == 0)
};
// 0: no norm written; 1: the RMSNorm asked for through norm_gain has been written as well; 2: written in the deferred
// form (planes without the row scale + per-tile sums of squares in nsq_out)
int launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st);
constexpr int NSQ_MAX_TILES = 320; // most 16-column tiles of a deferred norm (d_model <= 5120); a multiple of 16

struct AttnArgs {
    const void *q; // activation planes [planes][R16][ldq], rotated queries
    size_t q_plane;
    int ldq;
    const void *kcache, *vcache; // this layer
    const int32_t *len;          // [batch] lengths before this call's append
    int B, M, H, hd, S, R;
    int nsplit, chunk;  // positions per split (multiple of 64)
    float *part_o;      // [nsplit][R][H][hd] unnormalised
    float *part_m;      // [nsplit][R][H] running max (log2 domain)
    float *part_l;      // [nsplit][R][H] sum of weights
    void *act_out;      // merged, normalised output as activation planes [planes][R16][ld_out]
    size_t act_out_plane;
    int ld_out;
    float scale_log2e;
};
void launch_attention(int dtype, const AttnArgs &a, hipStream_t st);

void launch_embed(int dtype, const void *embed, const int32_t *tokens, int R, int d, int vocab, float *h,
                  int32_t *status, hipStream_t st);
void launch_rmsnorm_pack(int dtype, const float *h, const float *gain, int R, int d, float eps, void *act,
                         size_t act_plane, int ld_act, hipStream_t st);
// second pass of a split-K residual projection: h[r][:] += sum over splits (in split order) of parts[z][r][:], then,
// with a gain, the RMSNorm of the new row exactly as launch_rmsnorm_pack computes it
void launch_splitk_resid_norm(int dtype, float *h, const float *parts, int ksplit, const float *gain, int R, int d,
                              float eps, void *act, size_t act_plane, int ld_act, hipStream_t st);
// gathers the last row of every sequence: rows b*M + M-1 -> compact rows b (norm + pack)
void launch_rmsnorm_pack_rows(int dtype, const float *h, const float *gain, int nrows, int row0, int row_stride,
                              int d, float eps, void *act, size_t act_plane, int ld_act, hipStream_t st);
// row-wise int8 quantisation of W [rows][K] (storage type): scale = max|w| / 127 (1 for a zero row), q = rint(w / scale)
void launch_quantize_rows_int8(int dtype, const void *W, long long rows, long long K, int8_t *q, float *scale, hipStream_t st);
// int4 with group scales: q [rows][K/2] (entry 2b low, 2b+1 high nibble of byte b), scale [K/128][rows]; K % 128 == 0
void launch_quantize_rows_int4(int dtype, const void *W, long long rows, long long K, uint8_t *q, float *scale, hipStream_t st);
void launch_read_probe(const void *buf, size_t bytes, uint32_t *sink, hipStream_t st);
void launch_len_add(int32_t *len, int batch, int delta, hipStream_t st);
void launch_len_rollback(int32_t *len, const int32_t *n_accepted, int batch, int M, hipStream_t st);
// batched speculative step: verify rows [batch][K+1] and draft tokens [batch][K] from feed [batch][2] and call-major draft tokens [K][batch]
void launch_step_pack_tokens(const int32_t *feed, const int32_t *dtok, int batch, int K, int32_t *vt, int32_t *dbk, hipStream_t st);
// ... and the next feed [batch][2] = [verify row n_accepted[b], next[b]]
void launch_step_next_feed(const int32_t *vt, const int32_t *n_accepted, const int32_t *next, int batch, int K, int32_t *feed, hipStream_t st);
// len[b] = min(len[b], max(new_len[b], 0)); a value above the current length sets bit 2 of *status (may be NULL)
void launch_len_truncate(int32_t *len, const int32_t *new_len, int batch, int32_t *status, hipStream_t st);
// fills n 32-bit words with `value` (a kernel, so that it may be recorded into a graph)
void launch_fill_u32(uint32_t *p, size_t n, uint32_t value, hipStream_t st);
void launch_kv_append(int dtype, void *kc, void *vc, const void *k, const void *v, int seq, int pos0, int n_rows,
                      int H, int hd, int S, hipStream_t st);

// softmax / accept
// Row statistics.  A row longer than one segment is reduced by several workgroups: cnt = one arrival
// counter per row (zero before the launch, left zero), part = row_stats_partial_bytes(rows, V) bytes of
// device memory (rows = rows_a + rows_b); neither is touched when row_stats_segments(V) == 1.
int row_stats_segments(int V);
size_t row_stats_partial_bytes(int rows, int V);
void launch_row_stats(const float *logits, int rows, int V, float inv_t, float2 *stats, unsigned *cnt, float2 *part, hipStream_t st);
void launch_row_stats2(const float *logits_a, int rows_a, float2 *stats_a, const float *logits_b, int rows_b, float2 *stats_b,
                       int V, float inv_t, unsigned *cnt, float2 *part, hipStream_t st);
void launch_softmax_write(const float *logits, int rows, int V, float inv_t, const float2 *stats, float *probs,
                          int64_t probs_ld, hipStream_t st);
struct AcceptArgs {
    const float *p, *q;          // probabilities, or logits when from_logits
    const float2 *p_stats, *q_stats; // (max, Z) per row when from_logits
    int from_logits;
    float inv_t;
    const int32_t *draft;
    const float *u;
    int B, K, V;
    int32_t *n_accepted, *next_token;
    int32_t *status;
};
// row statistics of the logits entry in stages that skip the positions behind a sequence's first rejection
// (a.p / a.q are logits, a.p_stats / a.q_stats the arrays written)
void launch_row_stats_staged(const AcceptArgs &a, float2 *p_stats, float2 *q_stats, unsigned *cnt, float2 *part, hipStream_t st);
// partial: device workspace of accept_workspace_bytes(B, V) bytes (per-segment weight sums)
size_t accept_workspace_bytes(int B, int V);
void launch_accept(const AcceptArgs &a, unsigned long long *partial, hipStream_t st);
void launch_greedy_accept(const float *p_logits, const int32_t *draft, int B, int K, int V, int32_t *row_argmax,
                          int32_t *n_accepted, int32_t *next_token, hipStream_t st);
// token ~ row by the integer inverse CDF (rows are probabilities), or argmax when greedy
// rows of probabilities -> the rows restricted to their top-p nucleus and renormalised (P24 = top_p on a 2^-24 grid); out may alias probs
void launch_top_p_filter(const float *probs, long long ld_in, int rows, int V, unsigned P24, float *out, long long ld_out, hipStream_t st);
// rows of probabilities -> the rows restricted to their k heaviest tokens (ties: lowest index first) and renormalised; 1 <= k < V; out may alias probs
void launch_top_k_filter(const float *probs, long long ld_in, int rows, int V, int k, float *out, long long ld_out, hipStream_t st);
void launch_sample_rows(const float *probs, int64_t ld, int B, int V, const float *u, int32_t *token_out,
                        hipStream_t st);
void launch_argmax_rows(const float *logits, int64_t ld, int B, int V, int32_t *token_out, hipStream_t st);

} // namespace ss
