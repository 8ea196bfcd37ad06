// Per-row softmax statistics and the modified rejection step of speculative sampling
// (Sections 3 and 4.3: the target accepts or rejects the draft's tokens so that the target
// distribution is recovered).
//
//   accept d_i  <=>  p_i(d_i) >= q_i(d_i)  or  fl32(u_i * q_i(d_i)) < p_i(d_i)      (prob. min(1, p/q))
//   on the first rejection: next ~ norm(max(0, p - q));  nothing rejected: next ~ p_{K+1}
//
// Sampling is an integer inverse CDF so that a parallel reduction and a sequential loop pick the same
// token: w_v = trunc(r_v * 2^32) (uint64), S = sum w_v, threshold = (u*2^24 * S) >> 24, token = the
// smallest v whose inclusive prefix exceeds the threshold.  Integer sums are associative, so the
// wavefront reductions below cannot change the answer.
//
// Row statistics (max, Z) use one pass over the vocabulary (online softmax) with wavefront shuffles;
// probabilities are defined by one fixed instruction sequence (prob_from_logit) so that the fused
// logits path and the materialised softmax produce identical bits.
#include "ss_device.h"
#include "ss_kernels.h"
#include <algorithm>

namespace ss {

__device__ __forceinline__ float scaled_logit(float l, float inv_t) { return __fmul_rn(l, inv_t); }
// exp through the hardware's base-2 exponential (one rounded multiply, then v_exp_f32: about 2e-6 relative
// error at x = -30, far inside the tolerance on probabilities; the library routine costs five times the
// instructions and made these kernels ALU-bound)
__device__ __forceinline__ float fast_exp(float x) { return __builtin_amdgcn_exp2f(__fmul_rn(x, 1.4426950408889634f)); }
__device__ __forceinline__ float inv_norm(float Z) { return __fdiv_rn(1.0f, Z); }
// softmax probability of a logit given the row's (max, 1/Z): one fixed instruction sequence
__device__ __forceinline__ float prob_from_logit(float l, float inv_t, float mx, float invZ) {
    return __fmul_rn(fast_exp(__fsub_rn(scaled_logit(l, inv_t), mx)), invZ);
}

// ------------------------------------------------------------------ row statistics

__device__ __forceinline__ void online_add(float &m, float &s, float x) {
    if (x > m) {
        s = s * fast_exp(m - x) + 1.0f;
        m = x;
    } else {
        s += fast_exp(x - m);
    }
}
__device__ __forceinline__ void online_merge(float &m, float &s, float m2, float s2) {
    const float mm = fmaxf(m, m2);
    s = s * fast_exp(m - mm) + s2 * fast_exp(m2 - mm);
    m = mm;
}

// one workgroup per row: stats[row] = (max_v x_v, sum_v exp(x_v - max)), x = logit * inv_t.
// Each thread keeps STATS_UNROLL independent 16-byte loads in flight per step (the row is streamed once
// and the kernel is bound by memory latency otherwise) and folds the step into its running (max, sum)
// with one rescale.
constexpr int STATS_UNROLL = 8;
// A row is cut into segments of STATS_SEG logits (a function of the vocabulary size alone, so every
// entry point computes a row's statistics with the same operations in the same order): one workgroup per
// segment, and the workgroup that finishes a row's last segment merges the segments in index order.
constexpr int STATS_SEG = 16384;
// (max_v x_v, sum_v exp(x_v - max)) of x[0 .. V) by a workgroup of 256 threads; valid in thread 0
__device__ __forceinline__ float2 segment_stats(const float *x, int V, float inv_t, bool vec) {
    float m = -INFINITY, s = 0.f;
    if (vec) {
        const f32x4 *x4 = reinterpret_cast<const f32x4 *>(x);
        const int n4 = V / 4;
        for (int i0 = threadIdx.x; i0 < n4; i0 += 256 * STATS_UNROLL) {
            f32x4 t[STATS_UNROLL];
#pragma unroll
            for (int j = 0; j < STATS_UNROLL; ++j) {
                const int i = i0 + 256 * j;
                t[j] = i < n4 ? __builtin_nontemporal_load(x4 + i) : f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
            }
            float mx = -INFINITY;
#pragma unroll
            for (int j = 0; j < STATS_UNROLL; ++j)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    t[j][e] = scaled_logit(t[j][e], inv_t);
                    mx = fmaxf(mx, t[j][e]);
                }
            if (mx == -INFINITY) continue;
            if (mx > m) {
                s *= fast_exp(m - mx);
                m = mx;
            }
            float add = 0.f;
#pragma unroll
            for (int j = 0; j < STATS_UNROLL; ++j) add += (fast_exp(t[j][0] - m) + fast_exp(t[j][1] - m)) + (fast_exp(t[j][2] - m) + fast_exp(t[j][3] - m));
            s += add;
        }
    } else {
        for (int i = threadIdx.x; i < V; i += 256) online_add(m, s, scaled_logit(x[i], inv_t));
    }
    if (m == -INFINITY) s = 0.f; // a thread that saw nothing: exp(-inf - -inf) must not appear
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float m2 = __shfl_xor(m, o), s2 = __shfl_xor(s, o);
        if (m2 != -INFINITY) {
            if (m == -INFINITY) {
                m = m2;
                s = s2;
            } else {
                online_merge(m, s, m2, s2);
            }
        }
    }
    __shared__ float sm[4], ss_[4];
    if ((threadIdx.x & 63) == 0) {
        sm[threadIdx.x >> 6] = m;
        ss_[threadIdx.x >> 6] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float M = sm[0], S = ss_[0];
        for (int w = 1; w < 4; ++w)
            if (sm[w] != -INFINITY) {
                if (M == -INFINITY) {
                    M = sm[w];
                    S = ss_[w];
                } else {
                    online_merge(M, S, sm[w], ss_[w]);
                }
            }
        return make_float2(M, S);
    }
    return make_float2(0.f, 0.f);
}
// Statistics of segment `seg` of row x[0 .. V) and, by the workgroup that completes the row, of the row.
// cnt: the row's arrival counter (zero between launches); part: the row's nseg partial results.  Both are
// exchanged with agent-coherent accesses (the workgroups of a row run on different XCDs).
__device__ __forceinline__ void row_stats_segmented(const float *x, int V, float inv_t, int seg, int nseg, float2 *out, unsigned *cnt,
                                                    float2 *part) {
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(x) & 15) == 0);
    const int lo = seg * STATS_SEG;
    const float2 r = segment_stats(x + lo, min(STATS_SEG, V - lo), inv_t, vec);
    if (threadIdx.x != 0) return;
    if (nseg == 1) {
        *out = r;
        return;
    }
    __hip_atomic_store(reinterpret_cast<unsigned long long *>(part + seg), __builtin_bit_cast(unsigned long long, r), __ATOMIC_RELAXED,
                       __HIP_MEMORY_SCOPE_AGENT);
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): the partial result is at the memory side before the arrival is counted
    if (__hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != (unsigned)(nseg - 1)) return;
    float M = -INFINITY, S = 0.f;
    for (int sgi = 0; sgi < nseg; ++sgi) {
        const float2 ps = __builtin_bit_cast(float2, ld_coh64(part + sgi));
        if (ps.x != -INFINITY) {
            if (M == -INFINITY) {
                M = ps.x;
                S = ps.y;
            } else {
                online_merge(M, S, ps.x, ps.y);
            }
        }
    }
    *out = make_float2(M, S);
    __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
int row_stats_segments(int V) { return std::max(1, (V + STATS_SEG - 1) / STATS_SEG); }
size_t row_stats_partial_bytes(int rows, int V) {
    const int nseg = row_stats_segments(V);
    return nseg == 1 ? 0 : sizeof(float2) * (size_t)rows * nseg;
}

// Two row sets in one launch (the target's and the draft's logits): rows [0, rows_a) are set a.  grid (segments, rows).
__global__ __launch_bounds__(256) void row_stats_kernel(const float *logits_a, int rows_a, float2 *stats_a, const float *logits_b,
                                                        float2 *stats_b, int V, float inv_t, unsigned *cnt, float2 *part) {
    const int id = blockIdx.y, nseg = gridDim.x;
    const bool first = id < rows_a;
    const int row = first ? id : id - rows_a;
    row_stats_segmented((first ? logits_a : logits_b) + (size_t)row * V, V, inv_t, blockIdx.x, nseg, (first ? stats_a : stats_b) + row,
                        cnt + id, part + (size_t)id * nseg);
}

// cnt: one arrival counter per row, zero before the launch (the kernel leaves them zero); part:
// row_stats_partial_bytes(rows, V) bytes.  Neither is touched when the vocabulary fits one segment.
void launch_row_stats(const float *logits, int rows, int V, float inv_t, float2 *stats, unsigned *cnt, float2 *part, hipStream_t st) {
    if (rows <= 0) return;
    hipLaunchKernelGGL(row_stats_kernel, dim3(row_stats_segments(V), rows), dim3(256), 0, st, logits, rows, stats, nullptr, nullptr, V, inv_t,
                       cnt, part);
}
void launch_row_stats2(const float *logits_a, int rows_a, float2 *stats_a, const float *logits_b, int rows_b, float2 *stats_b,
                       int V, float inv_t, unsigned *cnt, float2 *part, hipStream_t st) {
    if (rows_a + rows_b <= 0) return;
    hipLaunchKernelGGL(row_stats_kernel, dim3(row_stats_segments(V), rows_a + rows_b), dim3(256), 0, st, logits_a, rows_a, stats_a, logits_b,
                       stats_b, V, inv_t, cnt, part);
}

__global__ __launch_bounds__(256) void softmax_write_kernel(const float *logits, int V, float inv_t, const float2 *stats,
                                                            float *probs, int64_t ld) {
    const int row = blockIdx.y;
    const float2 st = stats[row];
    const float invZ = inv_norm(st.y);
    const size_t base = (size_t)row * V, obase = (size_t)row * ld;
    for (int v = blockIdx.x * 256 + threadIdx.x; v < V; v += gridDim.x * 256)
        probs[obase + v] = prob_from_logit(logits[base + v], inv_t, st.x, invZ);
}

void launch_softmax_write(const float *logits, int rows, int V, float inv_t, const float2 *stats, float *probs,
                          int64_t probs_ld, hipStream_t st) {
    if (rows <= 0) return;
    int gx = (V + 256 * 8 - 1) / (256 * 8);
    hipLaunchKernelGGL(softmax_write_kernel, dim3(gx, rows), dim3(256), 0, st, logits, V, inv_t, stats, probs, probs_ld);
}

// ------------------------------------------------------------------ a row of probabilities

struct RowSrc {
    const float *row;
    int from_logits;
    float inv_t, mx, invZ; // invZ = inv_norm(Z)
    __device__ __forceinline__ float conv(float x) const { return from_logits ? prob_from_logit(x, inv_t, mx, invZ) : x; }
    __device__ __forceinline__ float at(int v) const { return conv(row[v]); }
    // probabilities of v..v+3 (0 beyond V); v is a multiple of 4
    __device__ __forceinline__ void load4(int v, int V, bool vec, float (&out)[4]) const {
        if (vec && v + 3 < V) {
            const float4 t = *reinterpret_cast<const float4 *>(row + v);
            out[0] = conv(t.x);
            out[1] = conv(t.y);
            out[2] = conv(t.z);
            out[3] = conv(t.w);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) out[e] = (v + e < V) ? conv(row[v + e]) : 0.f;
        }
    }
};

__device__ __forceinline__ unsigned long long fx_weight(float r) {
    return r > 0.f ? (unsigned long long)(r * 4294967296.0f) : 0ull;
}

template <bool RESID>
__device__ __forceinline__ void weights4(const RowSrc &P, const RowSrc &Q, int v, int V, bool vec,
                                         unsigned long long (&w)[4]) {
    float p[4];
    P.load4(v, V, vec, p);
    if (RESID) {
        float q[4];
        Q.load4(v, V, vec, q);
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = fx_weight(fmaxf(__fsub_rn(p[e], q[e]), 0.f));
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = fx_weight(p[e]);
    }
}

__device__ __forceinline__ unsigned long long shfl_xor_u64(unsigned long long x, int o) {
    const unsigned lo = __shfl_xor((unsigned)x, o), hi = __shfl_xor((unsigned)(x >> 32), o);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long shfl_up_u64(unsigned long long x, int o) {
    const unsigned lo = __shfl_up((unsigned)x, o), hi = __shfl_up((unsigned)(x >> 32), o);
    return ((unsigned long long)hi << 32) | lo;
}
__device__ __forceinline__ unsigned long long shfl_u64(unsigned long long x, int src) {
    const unsigned lo = __shfl((unsigned)x, src), hi = __shfl((unsigned)(x >> 32), src);
    return ((unsigned long long)hi << 32) | lo;
}

// threshold of the inverse CDF: floor(u * 2^24) * S >> 24 with a 128-bit product (u is a multiple of 2^-24)
__device__ __forceinline__ unsigned long long inv_cdf_threshold(float u, unsigned long long S) {
    const unsigned long long mant = (unsigned long long)(u * 16777216.0f);
    return (__umul64hi(mant, S) << 40) | ((mant * S) >> 24);
}

constexpr int SAMPLE_THREADS = 1024, SAMPLE_WAVES = SAMPLE_THREADS / 64;

// Integer inverse CDF over the range [r0, r1) of one row (r0 a multiple of 4) by a 1024-thread
// workgroup.  Wave w owns a contiguous segment of the range; pass A sums every segment, pass B rescans
// the one segment that holds the threshold.  have_T: the threshold T (relative to the weight in front
// of r0, known to fall inside the range) is given; otherwise it is derived from u and the range's
// total, and -1 is returned when that total is 0.  Returns the token to every thread.
template <bool RESID>
__device__ int block_inv_cdf(const RowSrc &P, const RowSrc &Q, int V, int r0, int r1, bool have_T, unsigned long long T,
                             float u, unsigned long long *sm_wave, int *sm_tok) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bool vec = (V % 4 == 0) && ((reinterpret_cast<uintptr_t>(P.row) & 15) == 0) &&
                     (!RESID || (reinterpret_cast<uintptr_t>(Q.row) & 15) == 0);
    int seg = (r1 - r0 + SAMPLE_WAVES - 1) / SAMPLE_WAVES;
    seg = (seg + 255) & ~255;
    const int v_begin = min(r0 + wave * seg, r1), v_end = min(v_begin + seg, r1);

    unsigned long long sum = 0;
    for (int v = v_begin + 4 * lane; v < v_end; v += 256) {
        unsigned long long w[4];
        weights4<RESID>(P, Q, v, V, vec, w);
        sum += (w[0] + w[1]) + (w[2] + w[3]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += shfl_xor_u64(sum, o);
    __syncthreads(); // protects sm_wave / sm_tok against a previous call in the same kernel
    if (lane == 0) sm_wave[wave] = sum;
    if (threadIdx.x == 0) *sm_tok = -1;
    __syncthreads();
    if (!have_T) {
        unsigned long long S = 0;
        for (int w = 0; w < SAMPLE_WAVES; ++w) S += sm_wave[w];
        if (S == 0) return -1;
        T = inv_cdf_threshold(u, S);
    }
    unsigned long long C = 0; // weight of the segments before mine
    for (int w = 0; w < wave; ++w) C += sm_wave[w];
    if (C <= T && T < C + sm_wave[wave]) { // wave-uniform: exactly one wave rescans its segment
        for (int v0 = v_begin; v0 < v_end; v0 += 256) {
            const int v = v0 + 4 * lane;
            unsigned long long w[4] = {0, 0, 0, 0};
            if (v < v_end) weights4<RESID>(P, Q, v, V, vec, w);
            const unsigned long long mine = (w[0] + w[1]) + (w[2] + w[3]);
            unsigned long long incl = mine;
#pragma unroll
            for (int o = 1; o < 64; o <<= 1) {
                const unsigned long long t = shfl_up_u64(incl, o);
                if (lane >= o) incl += t;
            }
            const unsigned long long total = shfl_u64(incl, 63);
            if (C + total > T) {
                unsigned long long run = C + incl - mine;
                if (run <= T && T < run + mine) {
                    int tok = v;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        run += w[e];
                        if (run > T) {
                            tok = v + e;
                            break;
                        }
                    }
                    *sm_tok = tok;
                }
                break;
            }
            C += total;
        }
    }
    __syncthreads();
    return *sm_tok;
}

// (value, index) argmax of one row by the workgroup, lowest index on ties
__device__ int block_argmax(const RowSrc &P, int V, float *sm_val, int *sm_idx) {
    float best = -INFINITY;
    int bi = 0x7fffffff;
    for (int v = threadIdx.x; v < V; v += blockDim.x) {
        const float x = P.at(v);
        if (x > best || bi == 0x7fffffff) {
            best = x;
            bi = v;
        }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        const float b2 = __shfl_xor(best, o);
        const int i2 = __shfl_xor(bi, o);
        if (b2 > best || (b2 == best && i2 < bi)) {
            best = b2;
            bi = i2;
        }
    }
    const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) {
        sm_val[wave] = best;
        sm_idx[wave] = bi;
    }
    __syncthreads();
    best = sm_val[0];
    bi = sm_idx[0];
    for (int w = 1; w < nw; ++w)
        if (sm_val[w] > best || (sm_val[w] == best && sm_idx[w] < bi)) {
            best = sm_val[w];
            bi = sm_idx[w];
        }
    return bi;
}

// ------------------------------------------------------------------ the rejection step

__device__ __forceinline__ RowSrc make_row(const float *base, const float2 *stats, size_t row, int V, int from_logits,
                                           float inv_t) {
    RowSrc r;
    r.row = base + row * (size_t)V;
    r.from_logits = from_logits;
    r.inv_t = inv_t;
    r.mx = 0.f;
    r.invZ = 1.f;
    if (from_logits) {
        const float2 s = stats[row];
        r.mx = s.x;
        r.invZ = inv_norm(s.y);
    }
    return r;
}

// Leading accepted draft tokens of sequence b among its first `upto` positions, by the first `upto`
// threads of a workgroup (one gather of p_i(d_i), q_i(d_i) per thread, all in flight together); every
// thread gets the count.  Only the row statistics of positions up to the first rejection need to exist:
// whatever a later position computes from missing statistics cannot lower the minimum.
__device__ int block_accept_count(const AcceptArgs &a, int b, int upto, int *sm_rej) {
    if (threadIdx.x == 0) *sm_rej = upto;
    __syncthreads();
    if ((int)threadIdx.x < upto) {
        const int i = threadIdx.x;
        const int d = a.draft[b * a.K + i];
        bool acc = false;
        if (d < 0 || d >= a.V) { // cannot be validated on the host: flagged, treated as rejected
            atomicOr(a.status, 1);
        } else {
            const RowSrc P = make_row(a.p, a.p_stats, (size_t)b * (a.K + 1) + i, a.V, a.from_logits, a.inv_t);
            const RowSrc Q = make_row(a.q, a.q_stats, (size_t)b * a.K + i, a.V, a.from_logits, a.inv_t);
            const float pi = P.at(d), qi = Q.at(d);
            acc = (pi >= qi) || (__fmul_rn(a.u[b * (a.K + 1) + i], qi) < pi);
        }
        if (!acc) atomicMin(sm_rej, i);
    }
    __syncthreads();
    return *sm_rej;
}

// Row statistics in stages (logits entry).  Positions behind the first rejection of a sequence are never
// looked at by the method, so their rows need not be read: stage j covers positions [lo, hi) of every
// sequence (target rows lo .. hi-1, draft rows lo .. min(hi, K)-1) and, for lo > 0, a workgroup first counts
// the accepted tokens among positions < lo (their statistics exist if they are needed, see
// block_accept_count) and leaves when a rejection has already happened.  grid (rows of the stage, B).
__global__ __launch_bounds__(256) void row_stats_stage_kernel(AcceptArgs a, float2 *p_stats, float2 *q_stats, int lo, int hi, int nseg,
                                                              unsigned *cnt, float2 *part) {
    __shared__ int sm_rej;
    const int b = blockIdx.z, np = hi - lo;
    const bool target = (int)blockIdx.y < np;
    const int i = lo + (target ? blockIdx.y : blockIdx.y - np);
    if (lo > 0 && block_accept_count(a, b, lo, &sm_rej) < lo) return; // uniform over the workgroup
    const int row = target ? b * (a.K + 1) + i : b * a.K + i;
    const int id = target ? row : a.B * (a.K + 1) + row;
    row_stats_segmented((target ? a.p : a.q) + (size_t)row * a.V, a.V, a.inv_t, blockIdx.x, nseg, (target ? p_stats : q_stats) + row,
                        cnt + id, part + (size_t)id * nseg);
}

// stages of 2, 3, then all remaining positions (K + 1 target rows, K draft rows per sequence); cnt and part
// as for launch_row_stats with B * (2K + 1) rows
void launch_row_stats_staged(const AcceptArgs &a, float2 *p_stats, float2 *q_stats, unsigned *cnt, float2 *part, hipStream_t st) {
    if (a.B <= 0) return;
    const int nseg = row_stats_segments(a.V);
    int lo = 0;
    for (int stage = 0; lo <= a.K; ++stage) {
        int hi = std::min(lo + 2 + stage, a.K + 1);
        if (stage == 2 || a.K + 1 - hi < 2) hi = a.K + 1; // third stage, or a remainder not worth a launch
        const int np = hi - lo, nq = std::min(hi, a.K) - lo;
        hipLaunchKernelGGL(row_stats_stage_kernel, dim3(nseg, np + nq, a.B), dim3(256), 0, st, a, p_stats, q_stats, lo, hi, nseg, cnt, part);
        lo = hi;
    }
}

constexpr int PART_THREADS = 256, PART_UNROLL = 4;

// grid (nseg, B): the accepted count of sequence b, and the total weight of segment blockIdx.x of the
// row the next token is drawn from (residual at the first rejection, else the bonus row).  The
// vocabulary is cut into nseg segments so that a few sequences still fill the chip; integer partial
// sums make the split invisible in the result.
__global__ __launch_bounds__(PART_THREADS) void accept_partial_kernel(AcceptArgs a, int seg_len, unsigned long long *partial) {
    __shared__ int sm_rej;
    __shared__ unsigned long long sm_part[PART_THREADS / 64];
    const int b = blockIdx.y, seg = blockIdx.x, nseg = gridDim.x;
    const int n = block_accept_count(a, b, a.K, &sm_rej);
    if (seg == 0 && threadIdx.x == 0) a.n_accepted[b] = n;
    const RowSrc P = make_row(a.p, a.p_stats, (size_t)b * (a.K + 1) + n, a.V, a.from_logits, a.inv_t);
    const bool resid = n < a.K;
    const RowSrc Q = resid ? make_row(a.q, a.q_stats, (size_t)b * a.K + n, a.V, a.from_logits, a.inv_t) : P;
    const bool vec = (a.V % 4 == 0) && ((reinterpret_cast<uintptr_t>(P.row) & 15) == 0) && ((reinterpret_cast<uintptr_t>(Q.row) & 15) == 0);
    const int r0 = min(seg * seg_len, a.V), r1 = min(r0 + seg_len, a.V);
    unsigned long long sum = 0;
    for (int v0 = r0 + 4 * threadIdx.x; v0 < r1; v0 += 4 * PART_THREADS * PART_UNROLL) {
        unsigned long long w[PART_UNROLL][4];
#pragma unroll
        for (int j = 0; j < PART_UNROLL; ++j) {
            const int v = v0 + 4 * PART_THREADS * j;
            if (v < r1) {
                if (resid) weights4<true>(P, Q, v, a.V, vec, w[j]);
                else weights4<false>(P, P, v, a.V, vec, w[j]);
            } else {
                w[j][0] = w[j][1] = w[j][2] = w[j][3] = 0;
            }
        }
#pragma unroll
        for (int j = 0; j < PART_UNROLL; ++j) sum += (w[j][0] + w[j][1]) + (w[j][2] + w[j][3]);
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) sum += shfl_xor_u64(sum, o);
    if ((threadIdx.x & 63) == 0) sm_part[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned long long t = 0;
        for (int w = 0; w < PART_THREADS / 64; ++w) t += sm_part[w];
        partial[(size_t)b * nseg + seg] = t;
    }
}

// one workgroup per sequence: locate the segment that holds the threshold and rescan it.  All residual
// weights zero (possible only through rounding): sample from p with the same uniform; all of those
// zero too: argmax.
__global__ __launch_bounds__(SAMPLE_THREADS) void accept_finish_kernel(AcceptArgs a, int seg_len, int nseg, const unsigned long long *partial) {
    __shared__ unsigned long long sm_wave[SAMPLE_WAVES];
    __shared__ int sm_tok;
    __shared__ float sm_val[SAMPLE_WAVES];
    __shared__ int sm_idx[SAMPLE_WAVES];
    const int b = blockIdx.x;
    const int n = a.n_accepted[b];
    const float u = a.u[b * (a.K + 1) + a.K];
    const RowSrc P = make_row(a.p, a.p_stats, (size_t)b * (a.K + 1) + n, a.V, a.from_logits, a.inv_t);
    const bool resid = n < a.K;
    const RowSrc Q = resid ? make_row(a.q, a.q_stats, (size_t)b * a.K + n, a.V, a.from_logits, a.inv_t) : P;
    unsigned long long S = 0;
    for (int sgi = 0; sgi < nseg; ++sgi) S += partial[(size_t)b * nseg + sgi];
    int tok = -1;
    if (S != 0) {
        const unsigned long long T = inv_cdf_threshold(u, S);
        unsigned long long C = 0;
        int sgi = 0;
        for (; sgi < nseg - 1; ++sgi) { // the segment with C <= T < C + partial
            const unsigned long long ps = partial[(size_t)b * nseg + sgi];
            if (T < C + ps) break;
            C += ps;
        }
        const int r0 = min(sgi * seg_len, a.V), r1 = min(r0 + seg_len, a.V);
        tok = resid ? block_inv_cdf<true>(P, Q, a.V, r0, r1, true, T - C, u, sm_wave, &sm_tok)
                    : block_inv_cdf<false>(P, P, a.V, r0, r1, true, T - C, u, sm_wave, &sm_tok);
    } else if (resid) {
        tok = block_inv_cdf<false>(P, P, a.V, 0, a.V, false, 0, u, sm_wave, &sm_tok);
    }
    if (tok < 0) tok = block_argmax(P, a.V, sm_val, sm_idx);
    if (threadIdx.x == 0) a.next_token[b] = tok;
}

// segments per sequence: enough workgroups to fill the chip, at least 8192 vocabulary entries each
static int accept_segments(int B, int V, int &seg_len) {
    int nseg = std::max(1, std::min(std::min(16, V / 8192), (1024 + B - 1) / std::max(B, 1)));
    seg_len = (V + nseg - 1) / nseg;
    seg_len = (seg_len + 1023) & ~1023; // multiple of the 4-wide loads of a whole workgroup
    nseg = (V + seg_len - 1) / seg_len;
    return std::max(nseg, 1);
}

size_t accept_workspace_bytes(int B, int V) {
    int seg_len;
    return sizeof(unsigned long long) * (size_t)B * accept_segments(B, V, seg_len);
}

void launch_accept(const AcceptArgs &a, unsigned long long *partial, hipStream_t st) {
    if (a.B <= 0) return;
    int seg_len;
    const int nseg = accept_segments(a.B, a.V, seg_len);
    hipLaunchKernelGGL(accept_partial_kernel, dim3(nseg, a.B), dim3(PART_THREADS), 0, st, a, seg_len, partial);
    hipLaunchKernelGGL(accept_finish_kernel, dim3(a.B), dim3(SAMPLE_THREADS), 0, st, a, seg_len, nseg, partial);
}

// ------------------------------------------------------------------ top-p filter
//
// Top-p ("nucleus") selection of probability rows (Section 3 names it beside argmax; the arithmetic is fixed
// in the header of the C ABI): 32-bit integer weights, kept set = shortest prefix in (weight descending, index
// ascending) order whose weights reach the target, renormalised by one fp32 division per element.  One
// workgroup per row finds the threshold weight by a three-digit radix selection (11 + 11 + 10 bits) over
// histograms of weight sums in LDS: all sums are integers, so the result does not depend on the order in
// which threads add.  Four reads of the row (three digits, one write pass; L2-resident), a fifth only when
// equal weights straddle the boundary.
constexpr int TP_THREADS = 1024, TP_WAVES = TP_THREADS / 64, TP_BINS = 2048, TP_UNROLL = 8;

__device__ __forceinline__ uint32_t fx_weight32(float r) {
    const unsigned long long w = fx_weight(r);
    return w > 0xffffffffull ? 0xffffffffu : (uint32_t)w;
}

// Workgroup-wide exclusive prefix sum of one value per thread in thread order; also returns the total.
__device__ __forceinline__ unsigned long long block_excl_scan(unsigned long long mine, unsigned long long *sm_wave, unsigned long long &total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned long long incl = mine;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long t = shfl_up_u64(incl, o);
        if (lane >= o) incl += t;
    }
    __syncthreads(); // sm_wave may still be read from a previous call
    if (lane == 63) sm_wave[wave] = incl;
    __syncthreads();
    unsigned long long before = 0;
    total = 0;
#pragma unroll
    for (int w = 0; w < TP_WAVES; ++w) {
        const unsigned long long x = sm_wave[w];
        if (w < wave) before += x;
        total += x;
    }
    return before + incl - mine;
}

// BY_COUNT = false: top-p, the histograms hold sums of weights and the selection looks for the weight at which the running
// sum reaches ceil(P24 * S / 2^24).  BY_COUNT = true: top-k (`P24` carries k, 1 <= k < V), the histograms hold counts (tokens
// without a weight count too: they are the tail of the order) and the selection looks for the weight of the k-th token;
// the kept weight is then summed in one more pass over the row.
template <bool BY_COUNT>
__global__ __launch_bounds__(TP_THREADS) void top_p_filter_kernel(const float *probs, long long ld_in, int V, unsigned P24, float *out, long long ld_out) {
    __shared__ unsigned long long hist[TP_BINS];
    __shared__ unsigned long long sm_wave[TP_WAVES];
    __shared__ unsigned long long sm_above, sm_binw;
    __shared__ int sm_bin, sm_cut;
    const float *p = probs + (size_t)blockIdx.x * (size_t)ld_in;
    float *o = out + (size_t)blockIdx.x * (size_t)ld_out;
    const int t = threadIdx.x;

    uint32_t prefix = 0;          // the digits of the threshold weight chosen so far
    unsigned long long need = 0;  // what the keys inside the chosen range still have to contribute
    unsigned long long S = 0, tie_weight = 0, target = 0;
    const int shifts[3] = {21, 10, 0}, nbits[3] = {11, 11, 10};
#pragma unroll
    for (int pass = 0; pass < 3; ++pass) {
        const int sh = shifts[pass], nb = nbits[pass];
        for (int b = t; b < TP_BINS; b += TP_THREADS) hist[b] = 0;
        __syncthreads();
        // A thread adds up runs of elements that fall into one bin before it touches the histogram: in the first
        // digit the weights of a whole vocabulary usually share their leading zeros (one bin), and per-element
        // atomics on one address would serialise.
        uint32_t run_bin = 0xffffffffu;
        unsigned long long run_sum = 0;
        for (int v0 = 0; v0 < V; v0 += TP_UNROLL * TP_THREADS) {
            float x[TP_UNROLL]; // the loads of a batch go out together
#pragma unroll
            for (int e = 0; e < TP_UNROLL; ++e) {
                const int v = v0 + e * TP_THREADS + t;
                x[e] = v < V ? p[v] : 0.f;
            }
#pragma unroll
            for (int e = 0; e < TP_UNROLL; ++e) {
                const uint32_t w = fx_weight32(x[e]);
                // keys inside the range chosen so far (pass 0: every key with a weight)
                if ((BY_COUNT ? v0 + e * TP_THREADS + t < V : w != 0) && (pass == 0 || (w >> (sh + nb)) == prefix)) {
                    const uint32_t bin = (w >> sh) & ((1u << nb) - 1);
                    if (bin != run_bin) {
                        if (run_bin != 0xffffffffu) atomicAdd(&hist[run_bin], run_sum);
                        run_bin = bin;
                        run_sum = 0;
                    }
                    run_sum += BY_COUNT ? 1u : w;
                }
            }
        }
        if (run_bin != 0xffffffffu) atomicAdd(&hist[run_bin], run_sum);
        __syncthreads();
        // thread t owns bins 2047 - 2t and 2046 - 2t, so thread order is descending weight order
        const unsigned long long a = hist[TP_BINS - 1 - 2 * t], b = hist[TP_BINS - 2 - 2 * t];
        unsigned long long total;
        const unsigned long long above = block_excl_scan(a + b, sm_wave, total);
        if (BY_COUNT && pass == 0) {
            need = P24; // the k-th token of the order
            target = need;
        }
        if (!BY_COUNT && pass == 0) {
            S = total;
            if (S == 0) { // nothing has a weight: the row is returned as it is
                for (int v = t; v < V; v += TP_THREADS) o[v] = p[v];
                return;
            }
            // target = ceil(P24 * S / 2^24) from the 128-bit product, at least 1
            const unsigned long long lo = (unsigned long long)P24 * S, hi = __umul64hi((unsigned long long)P24, S);
            const unsigned long long lo2 = lo + 16777215ull, hi2 = hi + (lo2 < lo ? 1ull : 0ull);
            need = (hi2 << 40) | (lo2 >> 24);
            if (need < 1) need = 1;
            target = need;
        }
        if (above < need && need <= above + a) {
            sm_bin = TP_BINS - 1 - 2 * t;
            sm_above = above;
            sm_binw = a;
        } else if (above + a < need && need <= above + a + b) {
            sm_bin = TP_BINS - 2 - 2 * t;
            sm_above = above + a;
            sm_binw = b;
        }
        __syncthreads();
        prefix = (prefix << nb) | (uint32_t)sm_bin;
        need -= sm_above;
        tie_weight = sm_binw;
        __syncthreads(); // everyone has read the choice before the next pass overwrites it
    }
    // prefix = threshold weight tau (>= 1); need = what tokens of weight tau must contribute; tie_weight = their total
    const unsigned long long tau = prefix;
    // (top-k: counts already; tau may be 0 there, when k reaches into the tokens without a weight)
    const unsigned long long n_ties = BY_COUNT ? tie_weight : tie_weight / tau, n_keep = BY_COUNT ? need : (need + tau - 1) / tau;
    int cut = V; // ties are kept up to and including this index
    if (n_keep < n_ties) {
        // the n_keep-th token of weight tau in index order: contiguous chunks per thread, counts scanned over threads
        const int chunk = (V + TP_THREADS - 1) / TP_THREADS;
        const int v0 = min(t * chunk, V), v1 = min(v0 + chunk, V);
        unsigned long long cnt = 0;
        for (int v = v0; v < v1; ++v) cnt += fx_weight32(p[v]) == prefix;
        unsigned long long total;
        const unsigned long long before = block_excl_scan(cnt, sm_wave, total);
        if (before < n_keep && n_keep <= before + cnt) {
            unsigned long long seen = before;
            for (int v = v0; v < v1; ++v)
                if (fx_weight32(p[v]) == prefix && ++seen == n_keep) {
                    sm_cut = v;
                    break;
                }
        }
        __syncthreads();
        cut = sm_cut;
    }
    // weight of the kept set: everything above tau (target - need) plus the kept tokens of weight tau
    unsigned long long kept = target - need + n_keep * tau;
    if (BY_COUNT) { // the weight above tau is not known from counts: one more pass over the row
        unsigned long long mine = 0;
        for (int v = t; v < V; v += TP_THREADS) {
            const uint32_t w = fx_weight32(p[v]);
            mine += w > prefix ? w : 0u;
        }
        unsigned long long total;
        block_excl_scan(mine, sm_wave, total);
        kept = total + n_keep * tau;
        if (kept == 0) { // nothing kept has a weight (then nothing has): the row is returned as it is
            for (int v = t; v < V; v += TP_THREADS) o[v] = p[v];
            return;
        }
    }
    const float Z = __fmul_rn(__ull2float_rn(kept), 2.3283064365386963e-10f);
    for (int v0 = 0; v0 < V; v0 += TP_UNROLL * TP_THREADS) {
        float x[TP_UNROLL];
#pragma unroll
        for (int e = 0; e < TP_UNROLL; ++e) {
            const int v = v0 + e * TP_THREADS + t;
            x[e] = v < V ? p[v] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < TP_UNROLL; ++e) {
            const int v = v0 + e * TP_THREADS + t;
            const uint32_t w = fx_weight32(x[e]);
            if (v < V) o[v] = (w > prefix || (w == prefix && v <= cut)) ? __fdiv_rn(x[e], Z) : 0.f;
        }
    }
}
void launch_top_p_filter(const float *probs, long long ld_in, int rows, int V, unsigned P24, float *out, long long ld_out, hipStream_t st) {
    if (rows <= 0) return;
    hipLaunchKernelGGL(top_p_filter_kernel<false>, dim3(rows), dim3(TP_THREADS), 0, st, probs, ld_in, V, P24, out, ld_out);
}
void launch_top_k_filter(const float *probs, long long ld_in, int rows, int V, int k, float *out, long long ld_out, hipStream_t st) {
    if (rows <= 0) return;
    hipLaunchKernelGGL(top_p_filter_kernel<true>, dim3(rows), dim3(TP_THREADS), 0, st, probs, ld_in, V, (unsigned)k, out, ld_out);
}

// ------------------------------------------------------------------ sampling / argmax of plain rows

__global__ __launch_bounds__(SAMPLE_THREADS) void sample_rows_kernel(const float *probs, int64_t ld, int V, const float *u,
                                                                     int32_t *token_out) {
    __shared__ unsigned long long sm_wave[SAMPLE_WAVES];
    __shared__ int sm_tok;
    __shared__ float sm_val[SAMPLE_WAVES];
    __shared__ int sm_idx[SAMPLE_WAVES];
    const int b = blockIdx.x;
    RowSrc P;
    P.row = probs + (size_t)b * ld;
    P.from_logits = 0;
    P.inv_t = 1.f;
    P.mx = 0.f;
    P.invZ = 1.f;
    int tok = block_inv_cdf<false>(P, P, V, 0, V, false, 0, u[b], sm_wave, &sm_tok);
    if (tok < 0) tok = block_argmax(P, V, sm_val, sm_idx);
    if (threadIdx.x == 0) token_out[b] = tok;
}
void launch_sample_rows(const float *probs, int64_t ld, int B, int V, const float *u, int32_t *token_out,
                        hipStream_t st) {
    if (B <= 0) return;
    hipLaunchKernelGGL(sample_rows_kernel, dim3(B), dim3(SAMPLE_THREADS), 0, st, probs, ld, V, u, token_out);
}

__global__ __launch_bounds__(SAMPLE_THREADS) void argmax_rows_kernel(const float *x, int64_t ld, int V, int32_t *out) {
    __shared__ float sm_val[SAMPLE_WAVES];
    __shared__ int sm_idx[SAMPLE_WAVES];
    RowSrc P;
    P.row = x + (size_t)blockIdx.x * ld;
    P.from_logits = 0;
    P.inv_t = 1.f;
    P.mx = 0.f;
    P.invZ = 1.f;
    const int t = block_argmax(P, V, sm_val, sm_idx);
    if (threadIdx.x == 0) out[blockIdx.x] = t;
}
void launch_argmax_rows(const float *logits, int64_t ld, int B, int V, int32_t *token_out, hipStream_t st) {
    if (B <= 0) return;
    hipLaunchKernelGGL(argmax_rows_kernel, dim3(B), dim3(SAMPLE_THREADS), 0, st, logits, ld, V, token_out);
}

// greedy: accept while the draft token is the target row's argmax; next = argmax at the first mismatch
__global__ void greedy_scan_kernel(const int32_t *row_argmax, const int32_t *draft, int B, int K, int32_t *n_accepted,
                                   int32_t *next_token) {
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int n = 0;
    while (n < K && draft[b * K + n] == row_argmax[b * (K + 1) + n]) ++n;
    n_accepted[b] = n;
    next_token[b] = row_argmax[b * (K + 1) + n];
}
void launch_greedy_accept(const float *p_logits, const int32_t *draft, int B, int K, int V, int32_t *row_argmax,
                          int32_t *n_accepted, int32_t *next_token, hipStream_t st) {
    if (B <= 0) return;
    launch_argmax_rows(p_logits, V, B * (K + 1), V, row_argmax, st);
    hipLaunchKernelGGL(greedy_scan_kernel, dim3((B + 63) / 64), dim3(64), 0, st, row_argmax, draft, B, K, n_accepted, next_token);
}

} // namespace ss
