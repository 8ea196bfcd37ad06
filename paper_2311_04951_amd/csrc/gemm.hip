// Weight-streaming skinny GEMM for the "linear layers" of the verify pass (Section 3: K+1 rows are
// evaluated together, and the pass is bound by reading the weights once).
//
//   out[m][n] = sum_k act[m][k] * W[n][k],   W row-major [N][K]; the R rows form row tiles of 16, and a
//   workgroup multiplies every weight chunk it streams with up to RT row tiles (weights are read once for
//   up to 16*RT rows).
//
// One workgroup (8 wavefronts for at most 16 rows) owns 16 output columns (or a pair of 16-column tiles for the fused
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
#include <type_traits>
#include "ss_device.h"
#include "ss_kernels.h"

namespace ss {

// What an epilogue reads besides the sums (the residual, the sequence's length and the rotary factors): a kernel whose
// K loop takes many memory round trips asks for them in front of it, so that the epilogue does not add two more.
struct EpiPre {
    float resid[4];
    float2 rope[4];
    int pos;
    float gain[4]; // deferred norm, producer: the next norm's gains of the lane's four columns
};
// Deferred norm, consumer: a lane's quarter of its activation row's per-tile sums of squares (lane group g holds tiles
// [g * T/4, (g + 1) * T/4) of row c), requested ahead of the K loop like the rest ...
constexpr int NSQ4 = NSQ_MAX_TILES / 16;
__device__ __forceinline__ void nsq_prefetch(const GemmArgs &a, int rt, float4 (&nsq)[NSQ4]) {
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int m = min(rt * 16 + c, a.R - 1);
    const float4 *p = reinterpret_cast<const float4 *>(a.act_nsq + (size_t)m * a.act_nsq_ld + g * (a.act_nsq_tiles / 4));
    const int n4 = a.act_nsq_tiles / 16;
#pragma unroll
    for (int i = 0; i < NSQ4; ++i) nsq[i] = p[min(i, n4 - 1)]; // (surplus slots repeat the last one and are not added)
}
// ... and 1 / rms of the row from them: fixed order inside a lane, then over the four lane groups
__device__ __forceinline__ float deferred_row_scale(const GemmArgs &a, const float4 (&nsq)[NSQ_MAX_TILES / 16]) {
    const int n4 = a.act_nsq_tiles / 16;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NSQ_MAX_TILES / 16; ++i) s += i < n4 ? (nsq[i].x + nsq[i].y) + (nsq[i].z + nsq[i].w) : 0.f;
    const float s1 = __shfl_xor(s, 16);
    const float lo = (threadIdx.x & 16) ? s1 : s, hi = (threadIdx.x & 16) ? s : s1; // (g even, g odd) of the pair, in that order
    const float pair = lo + hi;
    const float p2 = __shfl_xor(pair, 32);
    const float tot = (threadIdx.x & 32) ? p2 + pair : pair + p2;                   // (groups 0,1) + (groups 2,3)
    return 1.0f / sqrtf(tot / (float)a.K + a.norm_eps);
}
template <typename T, int EPI>
__device__ __forceinline__ void epi_prefetch(const GemmArgs &a, const int (&n0)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1], int rt, EpiPre &pre) {
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int m = min(rt * 16 + c, a.R - 1); // a row past the end asks for the last row's operands and never uses them
    if constexpr (EPI == EPI_RESID) {
#pragma unroll
        for (int v = 0; v < 4; ++v) pre.resid[v] = a.resid[(size_t)m * a.ldo + min(n0[0] + 4 * g + v, a.N - 1)];
        if (a.nsq_out) {
#pragma unroll
            for (int v = 0; v < 4; ++v) pre.gain[v] = a.norm_gain[min(n0[0] + 4 * g + v, a.N - 1)];
        }
    } else if constexpr (EPI == EPI_QKV) {
        const int d_all = a.H * a.hd;
        const int region = n0[0] / d_all;
        const int within = n0[0] - region * d_all;
        const int j0 = within - (within / a.hd) * a.hd + 4 * g;
        const int b = m / a.M, i = m - b * a.M;
        int pos = a.len[b] + i;
        if (pos > a.max_pos - 1) pos = a.max_pos - 1;
        if (pos > a.S - 1) pos = a.S - 1;
        pre.pos = pos;
        if (region < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) pre.rope[v] = a.rope[(size_t)pos * (a.hd / 2) + j0 + v];
        }
    }
}

// Epilogue of one output tile by one wave: lane (c, g) holds r[t][v] = the value of row m = rt*16 + c,
// column n0[t] + 4g + v.  pre: operands fetched ahead by epi_prefetch for this tile and row tile (NULL: read here).
template <typename T, int EPI>
__device__ __forceinline__ void apply_epilogue(const GemmArgs &a, const float (&r)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1][4],
                                               const int (&n0)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1], int rt, const EpiPre *pre = nullptr) {
    const int lane = threadIdx.x & 63, c = lane & 15, g = lane >> 4;
    const int m = rt * 16 + c;
    if (m >= a.R) return;

    if constexpr (EPI == EPI_STORE || EPI == EPI_RESID) {
        float hn[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int n = n0[0] + 4 * g + v;
            hn[v] = 0.f;
            if (n < a.N) {
                const size_t o = (size_t)m * a.ldo + n;
                hn[v] = (EPI == EPI_RESID) ? (pre ? pre->resid[v] : a.resid[o]) + r[0][v] : r[0][v];
                a.out[o] = hn[v];
            }
        }
        if (EPI == EPI_RESID && a.nsq_out && pre) { // deferred norm: h * gain as planes, the tile's sum of squares per row
            ActPlanes<T> np{reinterpret_cast<T *>(a.norm_act), a.norm_act_plane, a.norm_ld};
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int n = n0[0] + 4 * g + v;
                if (n < a.N) store_act(np, (size_t)m * a.norm_ld + n, hn[v] * pre->gain[v]);
            }
            float sq = (hn[0] * hn[0] + hn[1] * hn[1]) + (hn[2] * hn[2] + hn[3] * hn[3]);
            const float s1 = __shfl_xor(sq, 16);
            const float lo = (lane & 16) ? s1 : sq, hi = (lane & 16) ? sq : s1;
            const float pair = lo + hi;
            const float p2 = __shfl_xor(pair, 32);
            const float tot = (lane & 32) ? p2 + pair : pair + p2;
            if (g == 0) a.nsq_out[(size_t)m * a.nsq_ld + n0[0] / 16] = tot;
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
        int pos;
        if (pre) {
            pos = pre->pos;
        } else {
            pos = a.len[b] + i;
            if (pos > a.max_pos - 1) pos = a.max_pos - 1; // host validation keeps these from happening
            if (pos > a.S - 1) pos = a.S - 1;
        }
        float x0[4], x1[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            x0[v] = r[0][v];
            x1[v] = r[1][v];
        }
        if (region < 2) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const float2 cs = pre ? pre->rope[v] : a.rope[(size_t)pos * (a.hd / 2) + j0 + v];
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

// The K steps of a workgroup in rotated order: step i of nst becomes (i + rot) mod nst; steps past the end stay there
// (they are masked).  The offset depends on the workgroup alone, so a tile's sum is always formed in the same order.
__device__ __forceinline__ int k_rotation(int nst) { return (int)((blockIdx.x * 13u) % (unsigned)nst); }
__device__ __forceinline__ int rotated(int i, int rot, int nst) {
    if (i >= nst) return i;
    i += rot;
    return i >= nst ? i - nst : i;
}

// Activations of the kernels for at most 16 rows, through a wave-private piece of LDS.  A step of a wave is UPS units
// of 16 bytes of K for every row and plane: PL * R * UPS pieces.  Loaded per lane into MFMA operand layout that is
// 2 * PL * UPS / 8 load instructions with R / 16 of their lanes active; instead ceil(PL * R * UPS / 64) full-width
// load-to-LDS instructions bring them (lane l of instruction i brings piece 64 i + l; the pieces land in lane order,
// 16 bytes each) and the operands are read back from LDS.  Piece (plane * R + row) * UPS + (unit xor row) holds unit
// `unit` of the row, so that the 16 rows a wave reads together fall into different banks.  Lanes of rows that do not
// exist read a slot that holds zeros.  Measured on the 7B-shaped layer: 5-row pass 3.62 -> 3.37 ms, 1 row 3.29 -> 3.18.
template <typename T, int UPS, int RCAP = 16> struct ActStage { // RCAP: most rows (5, 8 or 16)
    static constexpr int PL = Traits<T>::PLANES, EPU = 16 / (int)sizeof(T);
    static constexpr int NDMA = (PL * RCAP * UPS + 63) / 64; // instructions that bring a step at RCAP rows
    static constexpr int SLOTS = NDMA * 64;                   // ... and the slots they fill
    static constexpr int BYTES = (SLOTS + 1) * 16; // LDS of one step of one wave (the last slot holds zeros)
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    const T *src[NDMA]; // the row (and plane) of this lane's piece of instruction i
    int ucol[NDMA];     // ... and its first K element inside the step
    int rows, npiece, kmax;

    // row0: first row of the tile; K: reduction length (a multiple of EPU)
    __device__ __forceinline__ void init(const GemmArgs &a, int row0, int K, int lane) {
        rows = min(a.R - row0, RCAP);
        npiece = PL * rows * UPS;
        kmax = K - EPU;
#pragma unroll
        for (int i = 0; i < NDMA; ++i) {
            const int p = min(i * 64 + lane, npiece - 1); // surplus lanes repeat the last piece into slots nobody reads
            const int plane = p / (rows * UPS), rem = p - plane * rows * UPS, row = rem / UPS, pos = rem % UPS;
            src[i] = reinterpret_cast<const T *>(a.act) + (size_t)plane * a.act_plane + (size_t)(row0 + row) * a.ld_act;
            ucol[i] = (pos ^ (row & (UPS - 1))) * EPU;
        }
    }
    __device__ __forceinline__ static void clear(unsigned char *region, int lane) {
        if (lane == 0) *reinterpret_cast<u32x4 *>(region + SLOTS * 16) = zero16();
    }
    // asks for the step that starts at K element k0 (columns past the end are clamped to the row's last unit: the
    // weights there are zero, so any finite value does)
    __device__ __forceinline__ void request(unsigned char *region, int k0) const {
#pragma unroll
        for (int i = 0; i < NDMA; ++i)
            if (i * 64 < npiece) __builtin_amdgcn_global_load_lds((gptr)(src[i] + min(k0 + ucol[i], kmax)), (lptr)(region + i * 1024), 16, 0, 0);
    }
    // byte offset in a step's region of row c's unit `unit` of plane pl
    __device__ __forceinline__ int operand_offset(int c, int unit, int pl) const {
        return c < rows ? ((pl * rows + c) * UPS + (unit ^ (c & (UPS - 1)))) * 16 : SLOTS * 16;
    }
};
// cache policy of the weight loads (the non-temporal bit of a load-to-LDS instruction): a weight line is used once,
// the activation lines by every workgroup.  Measured on the 7B-shaped bf16 pass: 3.04 -> 2.85 ms at 5 rows,
// 2.97 -> 2.75 at 1 row (int8 -3.6 %, int4 -2.5 %); the scope bits on top of it change nothing.
constexpr int WEIGHT_STREAM = 2;
// every load of the wave has landed (in registers or in LDS); the compiler may not move LDS reads above
__device__ __forceinline__ void act_stage_wait() {
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)
    asm volatile("" ::: "memory");
}

// Sum of the waves' partial tiles of row tile rt (fixed order) and the epilogue, by one wave.
template <typename T, int EPI, int NW>
__device__ __forceinline__ void tile_epilogue(const GemmArgs &a, const float (&red)[NW][(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1][4][64],
                                              const int (&n0)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1], int rt, const EpiPre *pre = nullptr,
                                              float rs = 1.0f) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63;
    float r[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float sum = red[0][t][v][lane];
#pragma unroll 4
            for (int w2 = 1; w2 < NW; ++w2) sum += red[w2][t][v][lane];
            r[t][v] = sum * rs; // rs: the row scale of a deferred norm (1 otherwise: exact)
        }
    apply_epilogue<T, EPI>(a, r, n0, rt, pre);
}

// The kernel for at most 16 rows: NW = wavefronts per workgroup (interleaved over K), U = 128-byte steps in flight per
// wave, RCAP = most rows (8 or 16: sizes the LDS); blockIdx.x = column tile (pair), blockIdx.y = row tile.
// The weights go through LDS like the activations: loaded straight into MFMA operand layout, a load instruction takes
// 64 bytes of each of 16 weight rows (four lanes per row), i.e. half a cache line per row; a load-to-LDS instruction
// whose lane l brings unit l & 7 of row l >> 3 takes whole 128-byte lines of 8 rows, and two of them bring a step's
// 16 x 128 bytes, which the lanes then read from LDS as operands (same xor placement as the activations).  Measured
// on the 7B-shaped layer: 5-row pass 3.28 -> 3.05 ms, 1 row 3.09 -> 2.99 (requests of whole lines are what counts:
// timing-only variants with a tile-major weight order gained 6 % with a contiguous kilobyte per instruction and
// nothing with half lines).
template <typename T, int EPI, int NW, int U, int RCAP>
__global__ __launch_bounds__(NW * 64) void gemm_kernel(GemmArgs a) {
    constexpr int E = Traits<T>::E, KB = 4 * E, EPU = 16 / (int)sizeof(T);
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int rt = blockIdx.y;
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

    // this lane's pieces of a weight step: instruction i brings rows 8i .. 8i + 7 of the tile, lane l unit
    // (l & 7) xor (row & 7) of row 8i + (l >> 3), into slot 64 i + l = row * 8 + (l & 7)
    const T *W = reinterpret_cast<const T *>(a.W);
    const T *wsrc[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i) wsrc[t][i] = W + (size_t)min(n0[t] + 8 * i + (lane >> 3), nrows_w - 1) * K; // ragged last tile: a valid row, masked at the store
    const int wucol = ((lane & 7) ^ (lane >> 3)) * EPU;
    const int kmax = K - EPU;

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr bool PRE = EPI != EPI_STORE; // the epilogue's own operands, asked for ahead of the K loop
    EpiPre pre;
    if (PRE && wave == 0) epi_prefetch<T, EPI>(a, n0, rt, pre);
    // the row scale of a deferred norm on the activations (1 otherwise), worked out by the epilogue's wave up front
    float rs = 1.0f;
    if (a.act_nsq && wave == 0) {
        float4 nsq[NSQ4];
        nsq_prefetch(a, rt, nsq);
        rs = deferred_row_scale(a, nsq);
    }

    // Each wave takes 128-byte steps (two k-blocks) of every row, interleaved with the other waves, U steps per
    // iteration: all their loads are in flight before the first MFMA.
    // Every workgroup starts at another place of K and wraps around (k_rotation): with all of them walking K in step,
    // the loads of a moment differ by multiples of the row stride and meet in the same memory channels, and all ask
    // for the same activation lines (measured on the 7B-shaped layer: 6 % of the 5-row pass, QKV 33.3 -> 29.7 us).
    const int nkb = (K + KB - 1) / KB;
    const int nst = (nkb + 1) / 2;
    const int rot = k_rotation(nst);
    const bool ragged = (K % (2 * KB)) != 0; // the last step ends inside its 128 bytes
    typedef ActStage<T, 8, RCAP> Stage;
    constexpr int WBYTES = NT * 2048;
    __shared__ __align__(16) unsigned char lds[NW][U][WBYTES + Stage::BYTES];
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    Stage stage;
    stage.init(a, rt * 16, K, lane);
    int rdw[2], rda[2][Stage::PL];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        rdw[j] = (c * 8 + ((4 * j + g) ^ (c & 7))) * 16;
#pragma unroll
        for (int pl = 0; pl < Stage::PL; ++pl) rda[j][pl] = WBYTES + stage.operand_offset(c, 4 * j + g, pl);
    }
#pragma unroll
    for (int s = 0; s < U; ++s) Stage::clear(lds[wave][s] + WBYTES, lane);
    for (int kp = wave; kp < nst; kp += U * NW) {
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (kp + s * NW < nst) { // (the same for the whole wave)
                const int k0 = 2 * rotated(kp + s * NW, rot, nst) * KB;
                const int kw = min(k0 + wucol, kmax); // past a ragged end: the row's last unit, zeroed after the read
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        __builtin_amdgcn_global_load_lds((gptr)(wsrc[t][i] + kw), (lptr)(lds[wave][s] + t * 2048 + i * 1024), 16, 0, WEIGHT_STREAM);
                stage.request(lds[wave][s] + WBYTES, k0);
            }
        }
        act_stage_wait();
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (kp + s * NW < nst) {
                const int st = rotated(kp + s * NW, rot, nst);
                u32x4 w[NT][2];
                Act<T> av[2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
#pragma unroll
                    for (int t = 0; t < NT; ++t) w[t][j] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + t * 2048 + rdw[j]);
#pragma unroll
                    for (int pl = 0; pl < Stage::PL; ++pl) av[j].p[pl] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + rda[j][pl]);
                }
                if (ragged && st == nst - 1) {
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        if ((2 * st + j) * KB + g * E >= K) {
#pragma unroll
                            for (int t = 0; t < NT; ++t) w[t][j] = zero16();
                        }
                }
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int t = 0; t < NT; ++t) acc[t] = mma(acc[t], w[t][j], av[j]);
            }
        }
        asm volatile("" ::: "memory"); // the reads stay above the next requests
    }

    // fixed-order sum of the waves' partial tiles; wave 0 applies the epilogue
    __shared__ float red[NW][NT][4][64];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][t][v][lane] = acc[t][v];
    __syncthreads();
    if (wave == 0) tile_epilogue<T, EPI, NW>(a, red, n0, rt, PRE ? &pre : nullptr, rs);
}

// ---- weight-only int8 matrices (the quantised model Sections 2 and 3 assume; one fp32 scale per output row)
//
// Same decomposition as gemm_kernel for at most 16 rows, a step being 128 entries of K (a 128-byte line of a weight
// row).  A lane's 16-byte unit holds 16 consecutive K entries of its weight row, i.e. two MFMA k-blocks: lane (c, g)
// supplies k = 128*step + 64*h + 16*g + 8*j .. +7 to block (h, j), and reads the activations of exactly those k.  An
// int8 value is exact in bf16, the sum runs in fp32, and the row scale multiplies the finished sum, so the only
// roundings are those of the sum.
__device__ __forceinline__ uint32_t w8_pair_to_bf16x2(uint32_t x, int first_byte) {
    const float f0 = (float)((int)(x << (24 - 8 * first_byte)) >> 24); // sign-extended bytes
    const float f1 = (float)((int)(x << (16 - 8 * first_byte)) >> 24);
    return (f2u(f0) >> 16) | (f2u(f1) & 0xffff0000u); // |q| <= 127: the low 16 bits of the fp32 are zero
}
__device__ __forceinline__ u32x4 w8_to_bf16x8(uint32_t a, uint32_t b) {
    return u32x4{w8_pair_to_bf16x2(a, 0), w8_pair_to_bf16x2(a, 2), w8_pair_to_bf16x2(b, 0), w8_pair_to_bf16x2(b, 2)};
}

template <int EPI, int NW, int U, int RCAP>
__global__ __launch_bounds__(NW * 64) void gemm_w8_kernel(GemmArgs a) {
    typedef bf16_t T;
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int K = a.K;

    int n0[NT];
    if constexpr (EPI == EPI_QKV) {
        const int per_head = a.hd / 32;
        const int hh = blockIdx.x / per_head;
        n0[0] = hh * a.hd + (blockIdx.x % per_head) * 16;
        n0[1] = n0[0] + a.hd / 2;
    } else if constexpr (EPI == EPI_SWIGLU) {
        n0[0] = blockIdx.x * 16;
        n0[1] = a.N + n0[0];
    } else {
        n0[0] = blockIdx.x * 16;
    }
    const int nrows_w = (EPI == EPI_SWIGLU) ? 2 * a.N : a.N;

    // a step is 128 entries of K, a whole 128-byte line of every weight row; as in gemm_kernel the tile's 16 x 128 bytes
    // come through LDS by two load-to-LDS instructions (lane l: unit (l & 7) xor (row & 7) of row 8i + (l >> 3))
    const int8_t *W = reinterpret_cast<const int8_t *>(a.W);
    const int8_t *wsrc[NT][2];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int i = 0; i < 2; ++i) wsrc[t][i] = W + (size_t)min(n0[t] + 8 * i + (lane >> 3), nrows_w - 1) * K; // ragged last tile: a valid row, masked at the store
    const int wucol = ((lane & 7) ^ (lane >> 3)) * 16;
    const int kmax = K - 16; // K is a multiple of 16

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr bool PRE = EPI != EPI_STORE; // the epilogue's own operands, asked for ahead of the K loop
    EpiPre pre;
    if (PRE && wave == 0) epi_prefetch<T, EPI>(a, n0, 0, pre);
    // the row scale of a deferred norm on the activations (1 otherwise), worked out by the epilogue's wave up front
    float rs = 1.0f;
    if (a.act_nsq && wave == 0) {
        float4 nsq[NSQ4];
        nsq_prefetch(a, 0, nsq);
        rs = deferred_row_scale(a, nsq);
    }

    const int nsteps = (K + 127) / 128;
    const int rot = k_rotation(nsteps); // (see gemm_kernel)
    const bool ragged = (K % 128) != 0;
    // lane (c, g) reads units g and 4 + g of its weight row: entries 64h + 16g .. + 15, i.e. two k-blocks (j = 0, 1) of 8
    // entries each, whose activations are unit 8h + 2g + j of the row's 16
    typedef ActStage<T, 16, RCAP> Stage;
    constexpr int WBYTES = NT * 2048;
    __shared__ __align__(16) unsigned char lds[NW][U][WBYTES + Stage::BYTES];
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    Stage stage;
    stage.init(a, 0, K, lane);
    int rdw[2], rda[2][2][Stage::PL];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        rdw[h] = (c * 8 + ((4 * h + g) ^ (c & 7))) * 16;
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int pl = 0; pl < Stage::PL; ++pl) rda[h][j][pl] = WBYTES + stage.operand_offset(c, 8 * h + 2 * g + j, pl);
    }
#pragma unroll
    for (int s = 0; s < U; ++s) Stage::clear(lds[wave][s] + WBYTES, lane);
    for (int ks = wave; ks < nsteps; ks += U * NW) {
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (ks + s * NW < nsteps) { // (the same for the whole wave)
                const int k0 = rotated(ks + s * NW, rot, nsteps) * 128;
                const int kw = min(k0 + wucol, kmax); // past a ragged end: the row's last unit, zeroed after the read
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        __builtin_amdgcn_global_load_lds((gptr)(wsrc[t][i] + kw), (lptr)(lds[wave][s] + t * 2048 + i * 1024), 16, 0, WEIGHT_STREAM);
                stage.request(lds[wave][s] + WBYTES, k0);
            }
        }
        act_stage_wait();
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (ks + s * NW < nsteps) {
                const int k0 = rotated(ks + s * NW, rot, nsteps) * 128;
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    u32x4 w[NT];
                    Act<T> av[2];
#pragma unroll
                    for (int t = 0; t < NT; ++t) w[t] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + t * 2048 + rdw[h]);
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int pl = 0; pl < Stage::PL; ++pl) av[j].p[pl] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + rda[h][j][pl]);
                    if (ragged && k0 + 64 * h + 16 * g >= K) {
#pragma unroll
                        for (int t = 0; t < NT; ++t) w[t] = zero16();
                    }
#pragma unroll
                    for (int j = 0; j < 2; ++j)
#pragma unroll
                        for (int t = 0; t < NT; ++t) acc[t] = mma(acc[t], w8_to_bf16x8(w[t][2 * j], w[t][2 * j + 1]), av[j]);
                }
            }
        }
        asm volatile("" ::: "memory"); // the reads stay above the next requests
    }

    // fixed-order sum of the waves' partial tiles; wave 0 scales the columns and applies the epilogue
    __shared__ float red[NW][NT][4][64];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][t][v][lane] = acc[t][v];
    __syncthreads();
    if (wave != 0) return;
    float r[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float sum = red[0][t][v][lane];
#pragma unroll 4
            for (int w2 = 1; w2 < NW; ++w2) sum += red[w2][t][v][lane];
            r[t][v] = sum * a.wscale[min(n0[t] + 4 * g + v, nrows_w - 1)] * rs;
        }
    apply_epilogue<T, EPI>(a, r, n0, 0, PRE ? &pre : nullptr);
}

// ---- weight-only int4 matrices with one scale per group of 128 K entries (the coarser reading of the same
// quantised model).  A lane's 16-byte unit holds 32 consecutive K entries of its weight row, i.e. four MFMA
// k-blocks (dword j = entries 8j..8j+7, entry e in bits 4e..4e+3, two's complement).  A step is a 128-byte line of
// every weight row = 256 entries of K = two scale groups, the lane's two units being one of each: a group accumulates
// into a fresh tile and the tile is added to the running sum times the group's scales of the lane's four output
// columns (scales are stored group-major, scale[group][column]).  K is a multiple of 128.
__device__ __forceinline__ u32x4 w4_to_bf16x8(uint32_t x) {
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float f0 = (float)((int)(x << (28 - 8 * i)) >> 28); // sign-extended nibbles 2i and 2i + 1
        const float f1 = (float)((int)(x << (24 - 8 * i)) >> 28);
        r[i] = (f2u(f0) >> 16) | (f2u(f1) & 0xffff0000u); // |q| <= 7: exact in bf16
    }
    return u32x4{r[0], r[1], r[2], r[3]};
}

// The same eight entries as bf16 values q + 136 (0x4300 | (q + 8): 128 + n is exact in bf16 for n < 128), without a
// conversion instruction: flip the sign bits (two's complement -> q + 8), split the even and the odd nibbles into bytes,
// and let four byte permutes place a pair of them into the low mantissa bits of 0x4300 4300.  About half the vector
// instructions of w4_to_bf16x8, which bound the kernel for at most 16 rows (its gate/up launch took longer than the
// int8 one for half the bytes); the caller takes 136 * (sum of the activations of the k-block) off the product.
// Measured on the 7B-shaped model: 5-row int4 pass -9 %.
__device__ __forceinline__ u32x4 w4_to_bf16x8_plus136(uint32_t x) {
    x ^= 0x88888888u;
    const uint32_t even = x & 0x0F0F0F0Fu, odd = (x >> 4) & 0x0F0F0F0Fu; // byte i: entry 2i / entry 2i + 1
    uint32_t r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) // bytes [even.i, 0, odd.i, 0] (selector bytes 0-3: second operand, 4-7: first, 0x0c: zero)
        r[i] = __builtin_amdgcn_perm(odd, even, 0x0c000c00u | ((4u + i) << 16) | (uint32_t)i) | 0x43004300u;
    return u32x4{r[0], r[1], r[2], r[3]};
}
constexpr float W4_BIAS = 136.0f;

template <int EPI, int NW, int U, int RCAP>
__global__ __launch_bounds__(NW * 64) void gemm_w4_kernel(GemmArgs a) {
    typedef bf16_t T;
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int K = a.K;

    int n0[NT];
    if constexpr (EPI == EPI_QKV) {
        const int per_head = a.hd / 32;
        const int hh = blockIdx.x / per_head;
        n0[0] = hh * a.hd + (blockIdx.x % per_head) * 16;
        n0[1] = n0[0] + a.hd / 2;
    } else if constexpr (EPI == EPI_SWIGLU) {
        n0[0] = blockIdx.x * 16;
        n0[1] = a.N + n0[0];
    } else {
        n0[0] = blockIdx.x * 16;
    }
    const int nrows_w = (EPI == EPI_SWIGLU) ? 2 * a.N : a.N;

    // the tile's 16 x 128 bytes of a step come through LDS by two load-to-LDS instructions, as in gemm_kernel
    // (lane l: unit (l & 7) xor (row & 7) of row 8i + (l >> 3))
    const unsigned char *W = reinterpret_cast<const unsigned char *>(a.W);
    const unsigned char *wsrc[NT][2];
    int ncol[NT][4]; // the lane's four output columns (weight rows 4g + v of the tile), clamped into the matrix
#pragma unroll
    for (int t = 0; t < NT; ++t) {
#pragma unroll
        for (int i = 0; i < 2; ++i) wsrc[t][i] = W + (size_t)min(n0[t] + 8 * i + (lane >> 3), nrows_w - 1) * (K / 2); // ragged last tile: a valid row, masked at the store
#pragma unroll
        for (int v = 0; v < 4; ++v) ncol[t][v] = min(n0[t] + 4 * g + v, nrows_w - 1);
    }
    const int wucol = ((lane & 7) ^ (lane >> 3)) * 16; // bytes
    const int bmax = K / 2 - 16;
    // calls of more than 16 rows: one workgroup per (column tile, row tile); every row tile streams the (quarter-size)
    // weights again
    const int rt = blockIdx.y;

    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr bool PRE = EPI != EPI_STORE; // the epilogue's own operands, asked for ahead of the K loop
    EpiPre pre;
    if (PRE && wave == 0) epi_prefetch<T, EPI>(a, n0, rt, pre);
    // the row scale of a deferred norm on the activations (1 otherwise), worked out by the epilogue's wave up front
    float rs = 1.0f;
    if (a.act_nsq && wave == 0) {
        float4 nsq[NSQ4];
        nsq_prefetch(a, rt, nsq);
        rs = deferred_row_scale(a, nsq);
    }

    // lane (c, g) reads units g and 4 + g of its weight row: unit 4h + g is entries 128h + 32g .. + 31 of the step, all in
    // scale group h, i.e. four k-blocks (j = 0..3) of 8 entries whose activations are unit 16h + 4g + j of the row's 32
    const int ngroups = K / 128;
    const int nsteps = (ngroups + 1) / 2; // two scale groups (a 128-byte line of a weight row) per step
    const int rot = k_rotation(nsteps);   // (see gemm_kernel)
    typedef ActStage<T, 32, RCAP> Stage;
    constexpr int WBYTES = NT * 2048;
    __shared__ __align__(16) unsigned char lds[NW][U][WBYTES + Stage::BYTES];
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    Stage stage;
    stage.init(a, rt * 16, K, lane);
    int rdw[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) rdw[h] = (c * 8 + ((4 * h + g) ^ (c & 7))) * 16;
#pragma unroll
    for (int s = 0; s < U; ++s) Stage::clear(lds[wave][s] + WBYTES, lane);
    for (int ks = wave; ks < nsteps; ks += U * NW) {
        float sc[U][2][NT][4];
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (ks + s * NW < nsteps) { // (the same for the whole wave)
                const int st = rotated(ks + s * NW, rot, nsteps);
                const int kw = min(st * 128 + wucol, bmax); // past the end (a last step of one group): a valid unit, not used
#pragma unroll
                for (int t = 0; t < NT; ++t) {
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        __builtin_amdgcn_global_load_lds((gptr)(wsrc[t][i] + kw), (lptr)(lds[wave][s] + t * 2048 + i * 1024), 16, 0, WEIGHT_STREAM);
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int v = 0; v < 4; ++v) sc[s][h][t][v] = a.wscale[(size_t)min(2 * st + h, ngroups - 1) * nrows_w + ncol[t][v]];
                }
                stage.request(lds[wave][s] + WBYTES, st * 256);
            }
        }
        act_stage_wait();
#pragma unroll
        for (int s = 0; s < U; ++s) {
            if (ks + s * NW < nsteps) {
                const int st = rotated(ks + s * NW, rot, nsteps);
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (2 * st + h < ngroups) { // (the same for the whole wave)
                        u32x4 w[NT];
                        Act<T> av[4];
#pragma unroll
                        for (int t = 0; t < NT; ++t) w[t] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + t * 2048 + rdw[h]);
#pragma unroll
                        for (int j = 0; j < 4; ++j)
#pragma unroll
                            for (int pl = 0; pl < Stage::PL; ++pl)
                                av[j].p[pl] = *reinterpret_cast<const u32x4 *>(lds[wave][s] + WBYTES + stage.operand_offset(c, 16 * h + 4 * g + j, pl));
                        // the group's activation sums per row (an all-ones weight tile: every output column gets the sum)
                        f32x4 asum = f32x4{0.f, 0.f, 0.f, 0.f};
                        const u32x4 ones = u32x4{0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
#pragma unroll
                        for (int j = 0; j < 4; ++j) asum = mma(asum, ones, av[j]);
#pragma unroll
                        for (int t = 0; t < NT; ++t) {
                            f32x4 part = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                            for (int j = 0; j < 4; ++j) part = mma(part, w4_to_bf16x8_plus136(w[t][j]), av[j]);
#pragma unroll
                            for (int v = 0; v < 4; ++v) acc[t][v] += sc[s][h][t][v] * (part[v] - W4_BIAS * asum[v]);
                        }
                    }
                }
            }
        }
        asm volatile("" ::: "memory"); // the reads stay above the next requests
    }

    // fixed-order sum of the waves' partial tiles; wave 0 applies the epilogue
    __shared__ float red[NW][NT][4][64];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) red[wave][t][v][lane] = acc[t][v];
    __syncthreads();
    if (wave != 0) return;
    tile_epilogue<T, EPI, NW>(a, red, n0, rt, PRE ? &pre : nullptr, rs);
}

// More than 16 rows (larger batches, prefill): the waves of a workgroup split the output columns instead
// of K, so that all of them walk K together and share the activation rows through LDS - with R rows
// the activations a wave needs are R*4/32 times its weight bytes, too much to fetch per wave from L2.
//   * wave w owns the 16 (or, fused epilogues, 2 x 16) weight rows of tile blockIdx.x*NW + w and the
//     complete K sum of its outputs: no reduction across waves;
//   * K is walked in slabs of 256 bytes per row.  The slab of all RT*16 rows goes from memory straight
//     into LDS (global_load_lds, no registers), two steps ahead of its use, into one of three buffers;
//     a 1 KB load instruction carries four rows, and the 16-byte units of a row are stored at position
//     (unit ^ row) so that the 16 rows a wave reads together hit different banks without padding;
//   * three weight slabs per wave in registers (one being multiplied, two in flight).
// Every step issues the same number of memory instructions (addresses are clamped into the operands; weights
// past K are zeroed after the load, so whatever finite activation sits there contributes nothing): the
// waits on "the loads issued two steps ago" are exact counts.
constexpr int WIDE_SLAB_BYTES = 256; // bytes of K per row, plane and slab

// acc0 / acc1 += one weight chunk x one activation k-block, into two independent accumulators
__device__ __forceinline__ void mma_split(f32x4 &acc0, f32x4 &acc1, u32x4 w, const Act<bf16_t> &b, int) {
    const bf16x8 av = __builtin_bit_cast(bf16x8, w);
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[0]), acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[1]), acc1, 0, 0, 0);
}
__device__ __forceinline__ void mma_split(f32x4 &acc0, f32x4 &acc1, u32x4 w, const Act<float> &b, int kb) {
    if (kb & 1) acc1 = mma(acc1, w, b);
    else acc0 = mma(acc0, w, b);
}

__device__ __forceinline__ void wide_barrier() { // workgroup barrier that orders LDS traffic only (no vmcnt(0))
    __builtin_amdgcn_s_waitcnt(0xC07F);
    __builtin_amdgcn_s_barrier();
}
template <int N> __device__ __forceinline__ void wait_vmcnt_at_most() { // s_waitcnt vmcnt(N), N < 64
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// columns of wave tile `tile`: n0[t] = first column of its t-th 16-column output tile; returns the number of wave tiles
template <int EPI>
__device__ __forceinline__ int wide_tile_cols(const GemmArgs &a, int tile, int (&n0)[(EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1]) {
    int ntiles;
    if constexpr (EPI == EPI_QKV) {
        const int per_head = a.hd / 32;
        ntiles = 3 * a.H * per_head;
        const int tl = min(tile, ntiles - 1);
        const int hh = tl / per_head; // head index over [q heads | k heads | v heads]
        n0[0] = hh * a.hd + (tl % per_head) * 16;
        n0[1] = n0[0] + a.hd / 2;
    } else if constexpr (EPI == EPI_SWIGLU) {
        ntiles = (a.N + 15) / 16;
        n0[0] = min(tile, ntiles - 1) * 16;
        n0[1] = a.N + n0[0];
    } else {
        ntiles = (a.N + 15) / 16;
        n0[0] = min(tile, ntiles - 1) * 16;
    }
    return ntiles;
}
// split-K partial tiles: [split][wave tile][row tile][t][v][lane] fp32, i.e. the accumulator layout of a wave
__device__ __forceinline__ size_t splitk_index(int z, int ntiles, int tile, int row_tiles, int rt, int NT, int t, int v, int lane) {
    return (((((size_t)z * ntiles + tile) * row_tiles + rt) * NT + t) * 4 + v) * 64 + lane;
}

// QB = 4: the matrix is int4 with one scale per 128 K entries and output column (bf16 planes, K a multiple of 128, a
// multiple of 4 weight rows).  A slab is exactly one scale group and a lane's single 16-byte load holds 32 K entries =
// its four k-blocks (dword j = entries 32g + 8j .., activations in LDS unit 4g + j): a step multiplies into fresh tiles
// and adds them, times the group's scales of the lane's four columns (one 16-byte load, requested with the weights), to
// the running sums - the arithmetic of gemm_w4_kernel.
// QB = 8 (W8): the matrix is int8 with row scales (bf16 activation planes only).  A lane's 16-byte load then holds 16 K entries,
// two MFMA k-blocks: per slab and tile two loads instead of four, and quarter q = 2h + j of the slab multiplies bytes
// 8j..8j+7 of load h with the activations of k = 64h + 16g + 8j .., which sit in LDS unit 8h + 2g + j of the row.
template <typename T, int EPI, int NW, int RT, int QB = 0>
__global__ __launch_bounds__(NW * 64) void gemm_wide_kernel(GemmArgs a) {
    constexpr bool W8 = QB == 8, W4 = QB == 4;
    static_assert(QB == 0 || Traits<T>::E == 8, "quantised matrices go with bf16 activation planes");
    constexpr int E = Traits<T>::E, KB = 4 * E, PL = Traits<T>::PLANES;
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    constexpr int WIDE_KS = WIDE_SLAB_BYTES / (int)sizeof(T); // elements of K per slab
    constexpr int KBS = WIDE_KS / KB;                         // k-blocks per slab (4)
    constexpr int EPU = 16 / (int)sizeof(T);                  // elements per 16-byte unit
    constexpr int ROWS = RT * 16;
    constexpr int BUF = PL * ROWS * WIDE_SLAB_BYTES;          // bytes of one slab buffer
    constexpr int GROUPS = PL * ROWS / 4;                     // 1 KB load instructions per slab (4 rows each)
    constexpr int DPW = (GROUPS + NW - 1) / NW;               // ... per wave
    constexpr int WLD = W4 ? 1 : (W8 ? KBS / 2 : KBS);        // weight loads per tile and step
    constexpr int WN = NT * WLD + (W4 ? NT : 0);              // weight (and int4 scale) loads per wave and step
    constexpr int WE = W4 ? 32 : (W8 ? 16 : E);               // K entries per weight load
    __shared__ __align__(16) unsigned char slab0[BUF], slab1[BUF], slab2[BUF];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane & 15, g = lane >> 4;
    const int rt0 = blockIdx.y * RT;
    const int K = a.K;
    const int tile = blockIdx.x * NW + wave;

    int n0[NT];
    const int ntiles = wide_tile_cols<EPI>(a, tile, n0);
    const bool tile_live = tile < ntiles; // a dead wave still helps with the slab copies and barriers
    const int nrows_w = (EPI == EPI_SWIGLU) ? 2 * a.N : a.N;

    constexpr size_t WB2 = W4 ? 1 : (W8 ? 2 : 2 * sizeof(T)); // twice the bytes of a matrix entry (an int4 entry is half a byte)
    const char *W = reinterpret_cast<const char *>(a.W);
    const char *wrow[NT]; // byte pointers: this lane's row at its lane group's offset
    const float *srow[NT]; // int4: the scales of the lane's four output columns in group 0
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        int n = n0[t] + c;
        if (n > nrows_w - 1) n = nrows_w - 1; // ragged last tile: load a valid row, masked at the store
        wrow[t] = W + ((size_t)n * K + g * WE) * WB2 / 2;
        srow[t] = W4 ? a.wscale + min(n0[t] + 4 * g, nrows_w - 4) : nullptr; // (nrows_w % 4 == 0: either all four columns exist or none)
    }
    const T *act = reinterpret_cast<const T *>(a.act);
    // split-K (a.ksplit > 1): workgroup z multiplies K slabs [s_lo, s_hi) only and leaves raw partial tiles
    const int nslab_all = (K + WIDE_KS - 1) / WIDE_KS;
    const int s_lo = a.ksplit > 1 ? blockIdx.z * a.kslabs : 0;
    const int s_hi = a.ksplit > 1 ? min(s_lo + a.kslabs, nslab_all) : nslab_all;
    const int nslab = s_hi - s_lo;
    // the workgroup's slabs in rotated order (see gemm_kernel: workgroups that walk K in step meet in the same memory
    // channels and activation lines); a request past the end repeats the last slab of the rotated order
    const int rot = k_rotation(nslab);
    auto slab_at = [&](int sl) { return s_lo + rotated(min(sl, nslab - 1), rot, nslab); };
    const int k_end = min(K, s_hi * WIDE_KS);

    // slab s -> LDS: this wave's DPW instructions; lane l brings row (l / 16) of its 4-row group, LDS unit l % 16
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    const int r4 = lane >> 4, q = lane & 15;
    auto slab_dma = [&](int sl, unsigned char *buf) {
        const int k0 = slab_at(sl) * WIDE_KS; // past the end: any valid slab (never multiplied)
#pragma unroll
        for (int i = 0; i < DPW; ++i) {
            const int grp = min(wave * DPW + i, GROUPS - 1); // a surplus instruction repeats the last group
            const int pr = 4 * grp + r4, pl = pr / ROWS, row = pr % ROWS;
            const int k = min(k0 + (q ^ (row & 15)) * EPU, a.ld_act - EPU);
            const T *src = act + pl * a.act_plane + (size_t)min(rt0 * 16 + row, a.R - 1) * a.ld_act + k;
            __builtin_amdgcn_global_load_lds((gptr)src, (lptr)(buf + grp * 1024), 16, 0, 0);
        }
        asm volatile("" ::: "memory");
    };
    auto w_load = [&](int sl, u32x4 (&w)[NT][WLD], u32x4 (&sc)[W4 ? NT : 1]) {
        const int k0 = slab_at(sl) * WIDE_KS; // past the end: the last slab again (a cache hit; never multiplied)
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int kb = 0; kb < WLD; ++kb) {
                const int k = k0 + kb * 4 * WE;
                w[t][kb] = ld16_global(wrow[t] + (size_t)min(k, K - (g + 1) * WE) * WB2 / 2); // zeroed past K when it is used
            }
        if constexpr (W4) {
#pragma unroll
            for (int t = 0; t < NT; ++t) sc[t] = ld16_global(srow[t] + (size_t)(k0 / WIDE_KS) * nrows_w);
        }
        asm volatile("" ::: "memory");
    };

    // two accumulator sets per output tile (bf16: hi and lo plane; f32: alternate k-blocks) so that
    // consecutive MFMAs never wait on each other
    f32x4 acc[2][RT][NT];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int t = 0; t < NT; ++t) acc[h][r][t] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Activation slabs are requested two steps ahead (three LDS buffers), and so are the weight slabs (three
    // register sets; deeper weight rings were measured and are slower).  A step issues [slab sl+2 -> LDS,
    // weights sl+2 -> registers]; buffers and register sets are compile-time choices, so the loop below is
    // unrolled over three steps and the last one or two steps of a slab count that is not a multiple of
    // three are written out after it (no idle step: the projections with K split four ways have 8 steps).
    u32x4 wring[3][NT][WLD];
    u32x4 sring[3][W4 ? NT : 1]; // int4: the slab's scales (four floats per tile), travelling with its weights
    slab_dma(0, slab0);
    w_load(0, wring[0], sring[0]);
    slab_dma(1, slab1);
    w_load(1, wring[1], sring[1]);
    auto step = [&](int sl, const unsigned char *cur, unsigned char *fill, u32x4 (&wcur)[NT][WLD], u32x4 (&wfill)[NT][WLD],
                    u32x4 (&scur)[W4 ? NT : 1], u32x4 (&sfill)[W4 ? NT : 1]) {
        // this wave's part of slab sl and its weight slab sl have landed: the only younger loads are
        // those of the previous step (slab sl+1, weights sl+1)
        wait_vmcnt_at_most<DPW + WN>();
        wide_barrier(); // everybody's part has landed, and everybody is done reading `fill` (slab sl - 1)
        slab_dma(sl + 2, fill);
        w_load(sl + 2, wfill, sfill);
        const unsigned char *base = cur + (size_t)c * WIDE_SLAB_BYTES;
        // the LDS reads of k-block kb+1 are issued before the MFMAs of k-block kb (the scheduling
        // barriers keep the compiler from sinking them next to their uses, which serialises every
        // MFMA behind an LDS round trip)
        auto read_av = [&](int kb, Act<T> (&av)[RT]) {
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int pl = 0; pl < PL; ++pl)
                    av[r].p[pl] = *reinterpret_cast<const u32x4 *>(base + (size_t)(pl * ROWS + r * 16) * WIDE_SLAB_BYTES +
                                                                   (((W4 ? 4 * g + kb : (W8 ? 8 * (kb >> 1) + 2 * g + (kb & 1) : kb * 4 + g)) ^ c) * 16));
            __builtin_amdgcn_sched_barrier(0);
        };
        Act<T> av[2][RT];
        read_av(0, av[0]);
        if constexpr (W4) {
            f32x4 part[RT][NT]; // this scale group's sums
#pragma unroll
            for (int r = 0; r < RT; ++r)
#pragma unroll
                for (int t = 0; t < NT; ++t) part[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb) {
                if (kb + 1 < KBS) read_av(kb + 1, av[(kb + 1) & 1]);
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    const u32x4 wm = w4_to_bf16x8(wcur[t][0][kb]); // a slab of a K that is a multiple of 128 lies inside K
#pragma unroll
                    for (int r = 0; r < RT; ++r) part[r][t] = mma(part[r][t], wm, av[kb & 1][r]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
#pragma unroll
            for (int t = 0; t < NT; ++t)
#pragma unroll
                for (int r = 0; r < RT; ++r)
#pragma unroll
                    for (int v = 0; v < 4; ++v) acc[0][r][t][v] += u2f(scur[t][v]) * part[r][t][v];
        } else {
#pragma unroll
            for (int kb = 0; kb < KBS; ++kb) {
                if (kb + 1 < KBS) read_av(kb + 1, av[(kb + 1) & 1]);
                const bool in_k = slab_at(sl) * WIDE_KS + (W8 ? (kb >> 1) * 64 + g * 16 : kb * KB + g * E) < k_end;
#pragma unroll
                for (int t = 0; t < NT; ++t) {
                    u32x4 wm;
                    if constexpr (W8) wm = in_k ? w8_to_bf16x8(wcur[t][kb >> 1][2 * (kb & 1)], wcur[t][kb >> 1][2 * (kb & 1) + 1]) : zero16();
                    else wm = in_k ? wcur[t][kb] : zero16();
#pragma unroll
                    for (int r = 0; r < RT; ++r) mma_split(acc[0][r][t], acc[1][r][t], wm, av[kb & 1][r], kb);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    int s0 = 0;
    for (; s0 + 3 <= nslab; s0 += 3) {
        step(s0, slab0, slab2, wring[0], wring[2], sring[0], sring[2]);
        step(s0 + 1, slab1, slab0, wring[1], wring[0], sring[1], sring[0]);
        step(s0 + 2, slab2, slab1, wring[2], wring[1], sring[2], sring[1]);
    }
    if (s0 < nslab) step(s0, slab0, slab2, wring[0], wring[2], sring[0], sring[2]);
    if (s0 + 1 < nslab) step(s0 + 1, slab1, slab0, wring[1], wring[0], sring[1], sring[0]);
    wait_vmcnt_at_most<0>(); // nothing may still be landing in LDS when the workgroup ends
    if (!tile_live) return;
    const int row_tiles = (a.R + 15) / 16;
#pragma unroll
    for (int r = 0; r < RT; ++r) {
        float out[NT][4];
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                out[t][v] = acc[0][r][t][v] + acc[1][r][t][v];
                if constexpr (W8) out[t][v] *= a.wscale[min(n0[t] + 4 * g + v, nrows_w - 1)]; // linear: also right for split-K partials
            }
        if (a.ksplit > 1) {
            if (EPI == EPI_RESID && a.splitk_rows) { // plain rows [split][R][N]: the launch that follows works row by row
                const int row = (rt0 + r) * 16 + c;
                if (row < a.R)
                    *reinterpret_cast<float4 *>(a.splitk_ws + ((size_t)blockIdx.z * a.R + row) * a.N + n0[0] + 4 * g) =
                        make_float4(out[0][0], out[0][1], out[0][2], out[0][3]);
            } else if (rt0 + r < row_tiles) {
#pragma unroll
                for (int t = 0; t < NT; ++t)
#pragma unroll
                    for (int v = 0; v < 4; ++v) a.splitk_ws[splitk_index(blockIdx.z, ntiles, tile, row_tiles, rt0 + r, NT, t, v, lane)] = out[t][v];
            }
        } else {
            apply_epilogue<T, EPI>(a, out, n0, rt0 + r);
        }
    }
}

// Second pass of a split-K launch: one wave per (wave tile, row tile) sums the splits' partial tiles in
// split order and runs the epilogue.  grid (wave tiles, row tiles).
template <typename T, int EPI>
__global__ __launch_bounds__(64) void gemm_splitk_finish_kernel(GemmArgs a) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    const int lane = threadIdx.x, tile = blockIdx.x, rt = blockIdx.y, row_tiles = gridDim.y;
    int n0[NT];
    const int ntiles = wide_tile_cols<EPI>(a, tile, n0);
    float out[NT][4];
#pragma unroll
    for (int t = 0; t < NT; ++t)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            float s = 0.f;
            for (int z = 0; z < a.ksplit; ++z) s += a.splitk_ws[splitk_index(z, ntiles, tile, row_tiles, rt, NT, t, v, lane)];
            out[t][v] = s;
        }
    apply_epilogue<T, EPI>(a, out, n0, rt);
}

// Matrices with few column tiles would leave most of the chip idle (one workgroup per compute unit fits:
// 64 workgroups for a 4096-column projection).  K is then split over up to 4 workgroups whose partial
// tiles a second small launch sums in a fixed order; the split count is the largest that still fits the
// chip in one round, so the extra traffic (partials written and read once) stays a fraction of the weights.
// A residual projection (whole 16-column tiles, dense output rows) leaves its partials as plain rows, and the
// second launch is the RMSNorm kernel with the sum over the splits in front: it completes h and, when the caller
// named the norm that follows, writes that too (returns true then).
template <typename T, int EPI, int NW, int RT, int QB = 0> static int launch_wide(const GemmArgs &a0, int tiles, int row_tiles, hipStream_t st) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    constexpr int WIDE_KS = WIDE_SLAB_BYTES / (int)sizeof(T);
    GemmArgs a = a0;
    const int gx = (tiles + NW - 1) / NW, gy = (row_tiles + RT - 1) / RT;
    const int nslab = (a.K + WIDE_KS - 1) / WIDE_KS;
    int ks = std::min(std::min(256 / std::max(gx * gy, 1), 4), nslab);
    a.ksplit = 1;
    a.kslabs = nslab;
    if (ks > 1 && a.splitk_ws) {
        const int per = (nslab + ks - 1) / ks;
        ks = (nslab + per - 1) / per; // no empty split
        const size_t need = sizeof(float) * (size_t)ks * tiles * row_tiles * NT * 256;
        if (ks > 1 && need <= a.splitk_ws_bytes) {
            a.ksplit = ks;
            a.kslabs = per;
        }
    }
    a.splitk_rows = EPI == EPI_RESID && a.ksplit > 1 && a.ksplit <= 4 && a.N % 16 == 0 && a.ldo == a.N && a.out == a.resid;
    hipLaunchKernelGGL((gemm_wide_kernel<T, EPI, NW, RT, QB>), dim3(gx, gy, a.ksplit), dim3(NW * 64), 0, st, a);
    if (a.splitk_rows) {
        launch_splitk_resid_norm(std::is_same<T, bf16_t>::value ? 1 : 0, a.out, a.splitk_ws, a.ksplit, a.norm_gain, a.R, a.N, a.norm_eps,
                                 a.norm_act, a.norm_act_plane, a.norm_ld, st);
        return a.norm_gain != nullptr ? 1 : 0;
    }
    if (a.ksplit > 1) hipLaunchKernelGGL((gemm_splitk_finish_kernel<T, EPI>), dim3(tiles, row_tiles), dim3(64), 0, st, a);
    return 0;
}

template <typename T, int EPI, int QB> static int launch_wide_any(const GemmArgs &a, int tiles, int row_tiles, hipStream_t st);

template <typename T, int EPI, int NW, int U> static void launch_narrow(const GemmArgs &a, int tiles, hipStream_t st) {
    if (a.R <= 8) hipLaunchKernelGGL((gemm_kernel<T, EPI, NW, U, 8>), dim3(tiles, 1), dim3(NW * 64), 0, st, a);
    else hipLaunchKernelGGL((gemm_kernel<T, EPI, NW, U, 16>), dim3(tiles, 1), dim3(NW * 64), 0, st, a);
}

template <typename T, int EPI> static int launch_gemm_t(const GemmArgs &a, hipStream_t st) {
    int tiles;
    if (EPI == EPI_QKV) tiles = 3 * a.H * (a.hd / 32);
    else tiles = (a.N + 15) / 16;
    const int row_tiles = (a.R + 15) / 16;
    if (row_tiles <= 1) { // the verify pass proper: the waves of a workgroup split K, two steps in flight each
        // fused epilogues (688 gate/up pairs, 384 rotary pairs at the 7B shape: several workgroups per compute unit anyway)
        // run 2 (gate/up) and 4 (QKV) waves per workgroup, the projections with 256 tiles 8: measured over
        // (2 | 3 | 4 | 5 | 6 | 8 | 16 waves) x (1 - 5 steps in flight) per kind of epilogue on the 7B-shaped layer
        if (EPI == EPI_QKV) launch_narrow<T, EPI, 4, 2>(a, tiles, st);
        else if (EPI == EPI_SWIGLU) launch_narrow<T, EPI, 2, 2>(a, tiles, st);
        else launch_narrow<T, EPI, 8, 2>(a, tiles, st);
        return (EPI == EPI_RESID && a.nsq_out) ? 2 : 0;
    }
    return launch_wide_any<T, EPI, 0>(a, tiles, row_tiles, st);
}

template <typename T, int EPI, int QB> static int launch_wide_any(const GemmArgs &a, int tiles, int row_tiles, hipStream_t st) {
    // larger batches and prefill chunks: waves split the columns; fewer waves per workgroup when the
    // matrix has few tiles, so that the launch still covers the chip
    constexpr bool FUSED = EPI == EPI_SWIGLU || EPI == EPI_QKV; // two weight tiles per wave: more registers
    const bool small = tiles < 8 * 128;
    if (row_tiles <= 2) {
        if (small) return launch_wide<T, EPI, 4, 2, QB>(a, tiles, row_tiles, st);
        return launch_wide<T, EPI, 8, 2, QB>(a, tiles, row_tiles, st);
    } else if (row_tiles <= 3) {
        if (small) return launch_wide<T, EPI, 4, 3, QB>(a, tiles, row_tiles, st);
        return launch_wide<T, EPI, 8, 3, QB>(a, tiles, row_tiles, st);
    } else {
        // one workgroup per compute unit fits: 3 waves per workgroup when that fills more of a 256-unit chip
        // in whole rounds than 4 (688 gate/up tiles: 230 workgroups instead of 172; 384 QKV tiles: 128, split in two)
        auto fill = [&](int nw) {
            const int wgs = (tiles + nw - 1) / nw * ((row_tiles + 4) / 5);
            const int ks = std::max(1, std::min(256 / std::max(wgs, 1), 4));
            return (double)(wgs * ks) / (double)((wgs * ks + 255) / 256 * 256);
        };
        if ((small || FUSED) && fill(3) > fill(4) + 0.1) return launch_wide<T, EPI, 3, 5, QB>(a, tiles, row_tiles, st);
        if (small || FUSED) return launch_wide<T, EPI, 4, 5, QB>(a, tiles, row_tiles, st);
        return launch_wide<T, EPI, 8, 5, QB>(a, tiles, row_tiles, st);
    }
}

// (a shape whose LDS does not fit at this row count runs with 8 waves and one step in flight)
template <int EPI, int NW, int U> static void launch_w8(const GemmArgs &a, int tiles, hipStream_t st) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    constexpr int red = NW * NT * 4 * 64 * 4;
    constexpr bool fit8 = NW * U * (NT * 2048 + ActStage<bf16_t, 16, 8>::BYTES) + red <= 160 * 1024;
    constexpr bool fit16 = NW * U * (NT * 2048 + ActStage<bf16_t, 16, 16>::BYTES) + red <= 160 * 1024;
    if (a.R <= 8) {
        if constexpr (fit8) hipLaunchKernelGGL((gemm_w8_kernel<EPI, NW, U, 8>), dim3(tiles, 1), dim3(NW * 64), 0, st, a);
        else hipLaunchKernelGGL((gemm_w8_kernel<EPI, 8, 1, 8>), dim3(tiles, 1), dim3(8 * 64), 0, st, a);
    } else {
        if constexpr (fit16) hipLaunchKernelGGL((gemm_w8_kernel<EPI, NW, U, 16>), dim3(tiles, 1), dim3(NW * 64), 0, st, a);
        else hipLaunchKernelGGL((gemm_w8_kernel<EPI, 8, 1, 16>), dim3(tiles, 1), dim3(8 * 64), 0, st, a);
    }
}

// 8 waves per workgroup for the projections with few tiles, 4 for the fused epilogues; one or two steps in flight per
// wave (measured per kind of epilogue on the 7B-shaped layer among (2 | 3 | 4 | 5 | 6 | 7 | 8 | 16 waves) x (1..3 steps))
template <int EPI> static int launch_gemm_w8(const GemmArgs &a, hipStream_t st) {
    const int tiles = EPI == EPI_QKV ? 3 * a.H * (a.hd / 32) : (a.N + 15) / 16;
    const int row_tiles = (a.R + 15) / 16;
    if (row_tiles > 1) return launch_wide_any<bf16_t, EPI, 8>(a, tiles, row_tiles, st);
    if (EPI == EPI_QKV) launch_w8<EPI, 4, 2>(a, tiles, st);
    else if (EPI == EPI_SWIGLU) launch_w8<EPI, 4, 1>(a, tiles, st);
    else if (EPI == EPI_RESID) launch_w8<EPI, 8, 2>(a, tiles, st);
    else launch_w8<EPI, 8, 1>(a, tiles, st);
    return (EPI == EPI_RESID && a.nsq_out) ? 2 : 0;
}

// One step in flight; 8 waves for the residual projections, 4 for the fused epilogues and the LM head: measured best of
// (2 | 3 | 4 | 5 | 6 | 8 waves) x (1 | 2 | 3 steps) on the 7B-shaped layer
// (a shape whose LDS does not fit at this row count runs with 4 waves and one step in flight)
template <int EPI, int NW, int U> static void launch_w4(const GemmArgs &a, int tiles, int row_tiles, hipStream_t st) {
    constexpr int NT = (EPI == EPI_SWIGLU || EPI == EPI_QKV) ? 2 : 1;
    constexpr int red = NW * NT * 4 * 64 * 4;
    constexpr bool fit5 = NW * U * (NT * 2048 + ActStage<bf16_t, 32, 5>::BYTES) + red <= 160 * 1024;
    constexpr bool fit8 = NW * U * (NT * 2048 + ActStage<bf16_t, 32, 8>::BYTES) + red <= 160 * 1024;
    constexpr bool fit16 = NW * U * (NT * 2048 + ActStage<bf16_t, 32, 16>::BYTES) + red <= 160 * 1024;
    if (a.R <= 5) { // the K + 1 = 5 rows of the usual verify pass: the smaller staging area lets a compute unit hold a workgroup more
        if constexpr (fit5) hipLaunchKernelGGL((gemm_w4_kernel<EPI, NW, U, 5>), dim3(tiles, row_tiles), dim3(NW * 64), 0, st, a);
        else hipLaunchKernelGGL((gemm_w4_kernel<EPI, 4, 1, 5>), dim3(tiles, row_tiles), dim3(4 * 64), 0, st, a);
    } else if (a.R <= 8) {
        if constexpr (fit8) hipLaunchKernelGGL((gemm_w4_kernel<EPI, NW, U, 8>), dim3(tiles, row_tiles), dim3(NW * 64), 0, st, a);
        else hipLaunchKernelGGL((gemm_w4_kernel<EPI, 4, 1, 8>), dim3(tiles, row_tiles), dim3(4 * 64), 0, st, a);
    } else {
        if constexpr (fit16) hipLaunchKernelGGL((gemm_w4_kernel<EPI, NW, U, 16>), dim3(tiles, row_tiles), dim3(NW * 64), 0, st, a);
        else hipLaunchKernelGGL((gemm_w4_kernel<EPI, 4, 1, 16>), dim3(tiles, row_tiles), dim3(4 * 64), 0, st, a);
    }
}

template <int EPI> static int launch_gemm_w4(const GemmArgs &a, hipStream_t st) {
    const int tiles = EPI == EPI_QKV ? 3 * a.H * (a.hd / 32) : (a.N + 15) / 16;
    const int row_tiles = (a.R + 15) / 16;
    const int nrows_w = EPI == EPI_SWIGLU ? 2 * a.N : a.N;
    // more than 16 rows: the wide kernel (it reads a lane's four scales as one 16-byte load); otherwise, or with a
    // row count that is not a multiple of 4, one workgroup per (column tile, row tile)
    if (row_tiles > 1 && nrows_w % 4 == 0 && (reinterpret_cast<uintptr_t>(a.wscale) & 15) == 0) return launch_wide_any<bf16_t, EPI, 4>(a, tiles, row_tiles, st);
    if (EPI == EPI_RESID) launch_w4<EPI, 8, 1>(a, tiles, row_tiles, st);
    else launch_w4<EPI, 4, 1>(a, tiles, row_tiles, st);
    return (EPI == EPI_RESID && a.nsq_out && row_tiles == 1) ? 2 : 0;
}

int launch_gemm(int dtype, int epi, const GemmArgs &a, hipStream_t st) {
    if (a.wscale && a.wbits == 4) { // int4 weights: the caller has checked bf16 planes and K % 128 == 0
        switch (epi) {
        case EPI_STORE: return launch_gemm_w4<EPI_STORE>(a, st);
        case EPI_RESID: return launch_gemm_w4<EPI_RESID>(a, st);
        case EPI_SWIGLU: return launch_gemm_w4<EPI_SWIGLU>(a, st);
        case EPI_QKV: return launch_gemm_w4<EPI_QKV>(a, st);
        }
        return 0;
    }
    if (a.wscale) { // int8 weights: the caller has checked bf16 planes and K % 16 == 0
        switch (epi) {
        case EPI_STORE: return launch_gemm_w8<EPI_STORE>(a, st);
        case EPI_RESID: return launch_gemm_w8<EPI_RESID>(a, st);
        case EPI_SWIGLU: return launch_gemm_w8<EPI_SWIGLU>(a, st);
        case EPI_QKV: return launch_gemm_w8<EPI_QKV>(a, st);
        }
        return 0;
    }
#define SS_CASE(EP)                                                  \
    case EP:                                                         \
        return dtype ? launch_gemm_t<bf16_t, EP>(a, st) : launch_gemm_t<float, EP>(a, st);
    switch (epi) {
        SS_CASE(EPI_STORE)
        SS_CASE(EPI_RESID)
        SS_CASE(EPI_SWIGLU)
        SS_CASE(EPI_QKV)
    }
#undef SS_CASE
    return 0;
}

} // namespace ss
