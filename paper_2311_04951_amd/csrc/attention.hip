// Multi-query-row causal decode attention against the contiguous KV cache ("attention" in Section 3's
// cost breakdown; the cache is the one of Sections 2 and 4.2).
//
// For sequence b, head h, the M = K+1 new rows (row i at absolute position L_b + i) attend cache
// positions 0..L_b + i; the rows' own keys/values were appended before this kernel runs, so everything
// is read back from the cache.  The KV range is split over workgroups (grid.x) and, inside a
// workgroup, over 4 wavefronts; every key/value tile is read from HBM exactly once and serves all M
// rows: the M query rows are the 16-wide B operand of the MFMAs (held in registers), keys and
// (block-transposed) values are the streamed A operand, 16 bytes per lane.
//
//   S^T[pos][m]  = sum_e K[pos][e] * Q[m][e]        (keys as A, queries as B)
//   O^T[e][m]   += sum_pos V^T[e][pos] * P[m][pos]  (transposed values as A, softmax weights as B)
//
// The row order of a key tile is permuted so that the score registers a lane receives are exactly
// the 8 (bf16) or 4 (f32) consecutive positions it must supply as the B operand of the P.V product:
// tile t, row i  <->  position p0 + (i/4)*E + 4t + (i%4).
// Online softmax in the log2 domain per wave; waves, then splits, are merged by log-sum-exp in a
// fixed order.  The second kernel merges the splits, normalises and writes the result as the
// activation planes the O projection consumes.
#include "ss_device.h"
#include "ss_kernels.h"

namespace ss {

constexpr float NEG_BIG = -1.0e30f;

template <typename T, int HD>
__global__ __launch_bounds__(256) void attn_partial_kernel(AttnArgs a) {
    constexpr int E = Traits<T>::E, KB = 4 * E, TPB = E / 4, NKC = HD / KB, NDT = HD / 16, NW = 4;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int split = blockIdx.x, h = blockIdx.y, b = blockIdx.z;
    const int L = a.len[b];
    const int ntot = L + a.M;
    const int p_begin = split * a.chunk;
    const int p_end = min(p_begin + a.chunk, ntot);

    // queries of this sequence as the B operand: lane (c, g) holds row b*M + c
    ActPlanes<T> qp{const_cast<T *>(reinterpret_cast<const T *>(a.q)), a.q_plane, a.ldq};
    const int qrow = min(b * a.M + c, a.R - 1);
    Act<T> q[NKC];
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) q[kc] = load_act(qp, (size_t)qrow * a.ldq + h * HD + kc * KB + g * E);

    const T *Kb = reinterpret_cast<const T *>(a.kcache) + ((size_t)b * a.H + h) * a.S * HD;
    const T *Vb = reinterpret_cast<const T *>(a.vcache) + ((size_t)b * a.H + h) * a.S * HD;

    const bool row_ok = c < a.M;
    const int row_limit = L + c; // last position row c may attend
    float m_run = NEG_BIG, l_run = 0.f;
    f32x4 o[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    for (int p0 = p_begin + wave * KB; p0 < p_end; p0 += NW * KB) {
        f32x4 s[TPB];
#pragma unroll
        for (int t = 0; t < TPB; ++t) {
            s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
            const int pos_i = p0 + (c >> 2) * E + 4 * t + (c & 3);
            const T *krow = Kb + (size_t)pos_i * HD + g * E;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) s[t] = mma(s[t], ld16_stream(krow + kc * KB), q[kc]);
        }
        // lane (c = row, g) holds the scores of positions p0 + g*E + e, e = 4t + v
        float pv[E];
        float bm = NEG_BIG;
#pragma unroll
        for (int t = 0; t < TPB; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int pos = p0 + g * E + 4 * t + v;
                const bool valid = row_ok && pos <= row_limit;
                const float x = valid ? s[t][v] * a.scale_log2e : NEG_BIG;
                pv[4 * t + v] = x;
                bm = fmaxf(bm, x);
            }
        bm = fmaxf(bm, __shfl_xor(bm, 16));
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const float m_new = fmaxf(m_run, bm);
        const float alpha = exp2f(m_run - m_new);
        l_run *= alpha;
#pragma unroll
        for (int e = 0; e < E; ++e) {
            const float p = (pv[e] > 0.5f * NEG_BIG) ? exp2f(pv[e] - m_new) : 0.f;
            l_run += p;
            pv[e] = p;
        }
        m_run = m_new;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[dt] *= alpha;
        const Act<T> P = pack_act(pv, T{});
        const T *vrow = Vb + ((size_t)(p0 >> 6) * HD + c) * 64 + (p0 & 63) + g * E;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[dt] = mma(o[dt], ld16_stream(vrow + (size_t)dt * 16 * 64), P);
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // merge the four waves (fixed order) and write this split's partial
    __shared__ float sm_m[NW][16], sm_l[NW][16];
    __shared__ float sm_o[NW][NDT][4][64];
    if (g == 0) {
        sm_m[wave][c] = m_run;
        sm_l[wave][c] = l_run;
    }
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt)
#pragma unroll
        for (int v = 0; v < 4; ++v) sm_o[wave][dt][v][lane] = o[dt][v];
    __syncthreads();
    float mstar = sm_m[0][c];
#pragma unroll
    for (int w = 1; w < NW; ++w) mstar = fmaxf(mstar, sm_m[w][c]);
    float wt[NW];
#pragma unroll
    for (int w = 0; w < NW; ++w) wt[w] = exp2f(sm_m[w][c] - mstar);
    if (!row_ok) return;
    const int row = b * a.M + c;
    const size_t pidx = ((size_t)split * a.R + row) * a.H + h;
    if (wave == 0 && g == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += sm_l[w][c] * wt[w];
        a.part_m[pidx] = mstar;
        a.part_l[pidx] = l;
    }
    for (int dt = wave; dt < NDT; dt += NW) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += sm_o[w][dt][v][lane] * wt[w];
            a.part_o[pidx * HD + dt * 16 + 4 * g + v] = acc;
        }
    }
}

// merge over splits, normalise, write activation planes: grid (R, H), block HD
template <typename T>
__global__ void attn_merge_kernel(AttnArgs a) {
    const int row = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
    float mstar = NEG_BIG;
    for (int s = 0; s < a.nsplit; ++s) mstar = fmaxf(mstar, a.part_m[((size_t)s * a.R + row) * a.H + h]);
    float l = 0.f, acc = 0.f;
    for (int s = 0; s < a.nsplit; ++s) {
        const size_t pidx = ((size_t)s * a.R + row) * a.H + h;
        const float w = exp2f(a.part_m[pidx] - mstar);
        l += a.part_l[pidx] * w;
        acc += a.part_o[pidx * a.hd + e] * w;
    }
    ActPlanes<T> out{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_out};
    store_act(out, (size_t)row * a.ld_out + h * a.hd + e, acc / l);
}

template <typename T> static void launch_attention_t(const AttnArgs &a, hipStream_t st) {
    dim3 grid(a.nsplit, a.H, a.B);
    if (a.hd == 128) hipLaunchKernelGGL((attn_partial_kernel<T, 128>), grid, dim3(256), 0, st, a);
    else if (a.hd == 64) hipLaunchKernelGGL((attn_partial_kernel<T, 64>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((attn_partial_kernel<T, 32>), grid, dim3(256), 0, st, a);
    hipLaunchKernelGGL((attn_merge_kernel<T>), dim3(a.R, a.H), dim3(a.hd), 0, st, a);
}

void launch_attention(int dtype, const AttnArgs &a, hipStream_t st) {
    if (dtype) launch_attention_t<bf16_t>(a, st);
    else launch_attention_t<float>(a, st);
}

} // namespace ss
