// Weight-streaming skinny GEMM for the "linear layers" of the verify pass (Section 3: K+1 rows are
// evaluated together, and the pass is bound by reading the weights once).
//
//   out[m][n] = sum_k act[m][k] * W[n][k],   W row-major [N][K]; the R rows form row tiles of 16, and a
//   workgroup multiplies every weight chunk it streams with up to RT row tiles (weights are read once for
//   up to 16*RT rows).
//
// One workgroup (16 wavefronts) owns 16 output columns (or a pair of 16-column tiles for the fused
// epilogues).  Each lane streams 16-byte chunks of 16 weight rows straight from HBM into registers -
// weights are used exactly once, so they never pass through LDS - and feeds them to MFMA as the A
// operand; the activation rows are the B operand, read as packed planes through L1/L2.  The
// waves interleave over K in 128-byte steps per row, their partial tiles are summed in a fixed
// order through LDS (deterministic), and wave 0 applies the epilogue:
//   STORE   plain fp32 store (LM head)
//   RESID   h += ...            (O projection, down projection)
//   SWIGLU  silu(gate) * up     (gate tile + up tile in one workgroup) -> activation planes
//   QKV     rotary embedding of q and k (pairs j, j + hd/2 sit in the two tiles), q -> activation
//           planes, k and v -> KV cache at positions len[b] + i
#include "ss_device.h"
#include "ss_kernels.h"

namespace ss {

// Sum of the waves' partial tiles of row tile rt (fixed order) and the epilogue, by one wave.
template <typename T, int EPI, int NW>
__device__ __forceinline__ void tile_epilogue(const GemmArgs &a, const float (&red)[NW][(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1][4][64],
                                              const int (&n0)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1], int rt) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    float r[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float sum = red[0][t][v][lane];
#pragma unroll 4
            for (int w2 = 1; w2 < NW; ++w2) sum += red[w2][t][v][lane];
            r[t][v] = sum;
        }

    // lane (c, g) holds row m = rt*16 + c, columns n0 + 4g + v
    const int m = rt * 16 + c;
    if (m >= a.R) return;

    if constexpr (EPI == EPI_STORE || EPI == EPI_RESID) {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = n0[0] + 4 * g + v;
            if (n < a.N) {
                const size_t o = (size_t)m * a.ldo + n;
                a.out[o] = (EPI == EPI_RESID) ? a.resid[o] + r[0][v] : r[0][v];
            }
        }
    } else if constexpr (EPI == EPI_SWIGLU) {
        ActPlanes<T> z{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_act_out};
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = n0[0] + 4 * g + v;
            if (n < a.N) {
                const float gt = r[0][v], up = r[1][v];
                const float s = gt / (1.0f + expf(-gt));
                store_act(z, (size_t)m * a.ld_act_out + n, s * up);
            }
        }
    } else { // EPI_QKV
        const int d_all = a.H * a.hd;
        const int region = n0[0] / d_all; // 0 q, 1 k, 2 v
        const int within = n0[0] - region * d_all;
        const int h = within / a.hd;
        const int j0 = within - h * a.hd + 4 * g; // column inside the head (first half)
        const int b = m / a.M, i = m - b * a.M;
        int pos = a.len[b] + i;
        if (pos > a.max_pos - 1) pos = a.max_pos - 1; // host validation keeps these from happening
        if (pos > a.S - 1) pos = a.S - 1;
        float x0[4], x1[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            x0[v] = r[0][v];
            x1[v] = r[1][v];
        }
        if (region < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float2 cs = a.rope[(size_t)pos * (a.hd / 2) + j0 + v];
                const float p0 = x0[v] * cs.x - x1[v] * cs.y;
                const float p1 = x0[v] * cs.y + x1[v] * cs.x;
                x0[v] = p0;
                x1[v] = p1;
            }
        }
        if (region == 0) {
            ActPlanes<T> q{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_act_out};
            const size_t o = (size_t)m * a.ld_act_out + h * a.hd + j0;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                store_act(q, o + v, x0[v]);
                store_act(q, o + a.hd / 2 + v, x1[v]);
            }
        } else if (region == 1) {
            T *kc = reinterpret_cast<T *>(a.kcache) + (((size_t)b * a.H + h) * a.S + pos) * a.hd + j0;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                kc[v] = to_storage<T>(x0[v]);
                kc[a.hd / 2 + v] = to_storage<T>(x1[v]);
            }
        } else {
            // values are kept transposed inside blocks of 64 positions: [pos/64][hd][64]
            T *vc = reinterpret_cast<T *>(a.vcache) + ((size_t)b * a.H + h) * a.S * a.hd +
                    ((size_t)(pos >> 6) * a.hd) * 64 + (pos & 63);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                vc[(size_t)(j0 + v) * 64] = to_storage<T>(x0[v]);
                vc[(size_t)(j0 + a.hd / 2 + v) * 64] = to_storage<T>(x1[v]);
            }
        }
    }
}

// NW = wavefronts per workgroup (interleaved over K), U = 128-byte steps in flight per wave,
// RT = row tiles (of 16 rows) per workgroup: blockIdx.y covers row tiles [blockIdx.y*RT, +RT)
template <typename T, int EPI, int NW, int U, int RT>
__global__ __launch_bounds__(NW * 64) void gemm_kernel(GemmArgs a) {
    constexpr int E = Traits<T>::E, KB = 4 * E;
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int rt0 = blockIdx.y * RT;
    const int K = a.K;

    int n0[NT];
    if constexpr (EPI == EPI_QKV) {
        const int per_head = a.hd / 32;
        const int hh = blockIdx.x / per_head; // head index over [q heads | k heads | v heads]
        n0[0] = hh * a.hd + (blockIdx.x % per_head) * 16;
        n0[1] = n0[0] + a.hd / 2;
    } else if constexpr (EPI == EPI_SWIGLU) {
        n0[0] = blockIdx.x * 16;
        n0[1] = a.N + n0[0];
    } else {
        n0[0] = blockIdx.x * 16;
    }
    const int nrows_w = (EPI == EPI_SWIGLU) ? 2 * a.N : a.N;

    const T *W = reinterpret_cast<const T *>(a.W);
    const T *wrow[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int n = n0[t] + c;
        if (n > nrows_w - 1) n = nrows_w - 1; // ragged last tile: load a valid row, masked at the store
        wrow[t] = W + (size_t)n * K + g * E;
    }
    ActPlanes<T> act{const_cast<T *>(reinterpret_cast<const T *>(a.act)), a.act_plane, a.ld_act};
    size_t aoff[RT];
    bool row_live[RT]; // rows past R contribute nothing: skip their loads
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        aoff[r] = (size_t)((rt0 + r) * 16 + c) * a.ld_act + g * E;
        row_live[r] = (rt0 + r) * 16 + c < a.R;
    }

    f32x4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Each wave takes 128-byte steps (two k-blocks) of every row, interleaved with the other waves,
    // U steps per iteration so that 2*U*NT weight loads are in flight per lane before the first MFMA.
    const int nkb = (K + KB - 1) / KB;
    for (int kp = wave; 2 * kp < nkb; kp += U * NW) {
        u32x4 w[U][NT][2];
        Act<T> av[U][2][RT];
#pragma unroll
        for (int s = 0; s < U; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int k = (2 * (kp + s * NW) + j) * KB;
                const bool ok = k + g * E < K; // K is a multiple of E
#pragma unroll
                for (int t = 0; t < NT; ++t) w[s][t][j] = ok ? ld16_stream(wrow[t] + k) : zero16();
#pragma unroll
                for (int r = 0; r < RT; ++r) av[s][j][r] = (ok && row_live[r]) ? load_act(act, aoff[r] + k) : zero_act<T>();
            }
#pragma unroll
        for (int s = 0; s < U; ++s)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[r][t] = mma(acc[r][t], w[s][t][j], av[s][j][r]);
    }

    // fixed-order sum of the waves' partial tiles, one row tile at a time; wave 0 applies the epilogue
    __shared__ float red[NW][NT][4][64];
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        if (r > 0) __syncthreads(); // wave 0 has read the previous row tile's partials
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) red[wave][t][v][lane] = acc[r][t][v];
        __syncthreads();
        if (wave == 0) tile_epilogue<T, EPI, NW>(a, red, n0, rt0 + r);
    }
}

template <typename T, int EPI> static void launch_gemm_t(const GemmArgs &a, hipStream_t st) {
    int tiles;
    if (EPI == EPI_QKV) tiles = 3 * a.H * (a.hd / 32);
    else tiles = (a.N + 15) / 16;
    const int row_tiles = (a.R + 15) / 16;
    if (row_tiles <= 1) { // the verify pass proper: 16 waves, two steps in flight
        hipLaunchKernelGGL((gemm_kernel<T, EPI, 16, 2, 1>), dim3(tiles, 1), dim3(16 * 64), 0, st, a);
    } else if (row_tiles <= 3) { // larger batches and prefill chunks: the weights are streamed once for all row tiles
        hipLaunchKernelGGL((gemm_kernel<T, EPI, 8, 1, 3>), dim3(tiles, 1), dim3(8 * 64), 0, st, a);
    } else {
        hipLaunchKernelGGL((gemm_kernel<T, EPI, 8, 1, 5>), dim3(tiles, (row_tiles + 4) / 5), dim3(8 * 64), 0, st, a);
    }
}

void launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st) {
#define SS_CASE(EP)                                                  \
    case EP:                                                         \
        if (dtype) launch_gemm_t<bf16_t, EP>(a, st);                 \
        else launch_gemm_t<float, EP>(a, st);                        \
        break;
    switch (epi) {
        SS_CASE(EPI_STORE)
        SS_CASE(EPI_RESID)
        SS_CASE(EPI_SWIGLU)
        SS_CASE(EPI_QKV)
    }
#undef SS_CASE
}

} // namespace ss
