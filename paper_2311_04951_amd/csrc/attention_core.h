// Core of the multi-query-row decode attention: one (sequence, head, KV split) unit per call.
// Shared by the stand-alone attention kernel and the persistent verify kernel.
#pragma once
#include "ss_device.h"
#include "ss_kernels.h"

namespace ss {

constexpr float NEG_BIG = -1.0e30f;

// LDS needed by attn_unit
template <int HD, int NW> struct AttnSmem {
    float m[NW][16], l[NW][16];
    float o[NW][HD / 16][4][64];
};

// One (sequence b, head h, KV split) unit by a workgroup of NW wavefronts; L = cached length of
// sequence b before this pass.  Writes the split's unnormalised partial (part_o, part_m, part_l).  Every thread of the workgroup must call it.
// COH: queries are read and partials written with agent-coherent accesses (persistent kernel).
// DIRECT: there is a single split, so the normalised result goes straight to the activation planes.
template <typename T, int HD, int NW, bool COH = false, bool DIRECT = false>
__device__ __forceinline__ void attn_unit(const AttnArgs &a, int split, int h, int b, int L, AttnSmem<HD, NW> &sm) {
    constexpr int E = Traits<T>::E, KB = 4 * E, TPB = E / 4, NKC = HD / KB, NDT = HD / 16;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int ntot = L + a.M;
    const int p_begin = split * a.chunk;
    const int p_end = min(p_begin + a.chunk, ntot);

    // queries of this sequence as the B operand: lane (c, g) holds row b*M + c
    ActPlanes<T> qp{const_cast<T *>(reinterpret_cast<const T *>(a.q)), a.q_plane, a.ldq};
    const int qrow = min(b * a.M + c, a.R - 1);
    Act<T> q[NKC];
#pragma unroll
    for (int kc = 0; kc < NKC; ++kc) {
        const size_t qo = (size_t)qrow * a.ldq + h * HD + kc * KB + g * E;
        q[kc] = COH ? load_act_coh(qp, qo) : load_act(qp, qo);
    }

    const T *Kb = reinterpret_cast<const T *>(a.kcache) + ((size_t)b * a.H + h) * a.S * HD;
    const T *Vb = reinterpret_cast<const T *>(a.vcache) + ((size_t)b * a.H + h) * a.S * HD;

    const bool row_ok = c < a.M;
    const int row_limit = L + c; // last position row c may attend
    float m_run = NEG_BIG, l_run = 0.f;
    f32x4 o[NDT];
#pragma unroll
    for (int dt = 0; dt < NDT; ++dt) o[dt] = f32x4{0.f, 0.f, 0.f, 0.f};

    // One step covers KB positions.  The key and value chunks of a step do not depend on anything
    // computed here, so the next step's chunks are requested before the current step's arithmetic:
    // a wave pays one memory round trip for its whole KV range instead of two per step.  Plain loads, not
    // non-temporal ones: a load instruction covers half of each line it touches (16 rows x 64 bytes), and the
    // other half, which the next instruction (keys) or the neighbouring wave (values) asks for, should hit
    // (8 % faster at 4096 cached positions, and 20 % fewer bytes fetched).
    struct Tile {
        u32x4 k[TPB][NKC];
        u32x4 v[NDT];
    };
    auto load_tile = [&](int p0, Tile &t) {
#pragma unroll
        for (int tt = 0; tt < TPB; ++tt) {
            const int pos_i = p0 + (c >> 2) * E + 4 * tt + (c & 3);
            const T *krow = Kb + (size_t)pos_i * HD + g * E;
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) t.k[tt][kc] = ld16_global(krow + kc * KB);
        }
        const T *vrow = Vb + ((size_t)(p0 >> 6) * HD + c) * 64 + (p0 & 63) + g * E;
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) t.v[dt] = ld16_global(vrow + (size_t)dt * 16 * 64);
    };
    Tile cur, nxt;
    const int p_first = p_begin + wave * KB;
    if (p_first < p_end) load_tile(p_first, cur);
    for (int p0 = p_first; p0 < p_end; p0 += NW * KB) {
        const bool more = p0 + NW * KB < p_end;
        if (more) load_tile(p0 + NW * KB, nxt);
        f32x4 s[TPB];
#pragma unroll
        for (int t = 0; t < TPB; ++t) {
            s[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kc = 0; kc < NKC; ++kc) s[t] = mma(s[t], cur.k[t][kc], q[kc]);
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
#pragma unroll
        for (int dt = 0; dt < NDT; ++dt) o[dt] = mma(o[dt], cur.v[dt], P);
        if (more) cur = nxt;
    }
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // merge the waves (fixed order) and write this split's partial
    auto &sm_m = sm.m;
    auto &sm_l = sm.l;
    auto &sm_o = sm.o;
    __syncthreads(); // the previous unit's readers are done with the buffers
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
    if (DIRECT) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += sm_l[w][c] * wt[w];
        ActPlanes<T> out{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_out};
        for (int dt = wave; dt < NDT; dt += NW) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                float acc = 0.f;
#pragma unroll
                for (int w = 0; w < NW; ++w) acc += sm_o[w][dt][v][lane] * wt[w];
                const size_t o = (size_t)row * a.ld_out + h * HD + dt * 16 + 4 * g + v;
                if (COH) store_act_coh(out, o, acc / l);
                else store_act(out, o, acc / l);
            }
        }
        return;
    }
    const size_t pidx = ((size_t)split * a.R + row) * a.H + h;
    if (wave == 0 && g == 0) {
        float l = 0.f;
#pragma unroll
        for (int w = 0; w < NW; ++w) l += sm_l[w][c] * wt[w];
        if (COH) {
            st_coh(&a.part_m[pidx], mstar);
            st_coh(&a.part_l[pidx], l);
        } else {
            a.part_m[pidx] = mstar;
            a.part_l[pidx] = l;
        }
    }
    for (int dt = wave; dt < NDT; dt += NW) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float acc = 0.f;
#pragma unroll
            for (int w = 0; w < NW; ++w) acc += sm_o[w][dt][v][lane] * wt[w];
            if (COH) st_coh(&a.part_o[pidx * HD + dt * 16 + 4 * g + v], acc);
            else a.part_o[pidx * HD + dt * 16 + 4 * g + v] = acc;
        }
    }
}


constexpr int ATTN_MAX_SPLITS = 16;

// merged, normalised output of one (row, head) from the splits' partials, element e
// (all loads are issued before the first use so that they overlap)
template <bool COH = false>
__device__ __forceinline__ float attn_merge_elem(const AttnArgs &a, int row, int h, int e) {
    auto rd = [](const float *p) { return COH ? ld_coh(p) : *p; };
    float pm[ATTN_MAX_SPLITS], plv[ATTN_MAX_SPLITS], po[ATTN_MAX_SPLITS];
#pragma unroll
    for (int s = 0; s < ATTN_MAX_SPLITS; ++s) {
        const size_t pidx = ((size_t)s * a.R + row) * a.H + h;
        const bool on = s < a.nsplit;
        pm[s] = on ? rd(&a.part_m[pidx]) : NEG_BIG;
        plv[s] = on ? rd(&a.part_l[pidx]) : 0.f;
        po[s] = on ? rd(&a.part_o[pidx * a.hd + e]) : 0.f;
    }
    float mstar = NEG_BIG;
#pragma unroll
    for (int s = 0; s < ATTN_MAX_SPLITS; ++s) mstar = fmaxf(mstar, pm[s]);
    float l = 0.f, acc = 0.f;
#pragma unroll
    for (int s = 0; s < ATTN_MAX_SPLITS; ++s) {
        const float w = exp2f(pm[s] - mstar);
        l += plv[s] * w;
        acc += po[s] * w;
    }
    return acc / l;
}

} // namespace ss
