// The verify pass as ONE persistent kernel (Section 3: the pass is bound by streaming the weights, so
// the design goal is that the HBM stream stops as rarely and as briefly as possible).
//
// One workgroup of 4 wavefronts per compute unit (512 registers per lane) stays resident for the whole
// pass and walks a list of phases: [embedding] then per layer [QKV, attention, O projection, gate/up,
// down projection], then [LM head] and [cache-length update].  Everything one workgroup writes for
// another to read inside the kernel (hidden rows, packed activations, norm partials, new cache rows,
// attention partials) moves through agent-coherent accesses, which are performed at the memory side of
// the per-XCD L2 caches, so no phase boundary carries a cache write-back / invalidate.  Two ways of
// ordering consumers behind producers are used:
//  * flags: a device-wide barrier (each workgroup waits for its store acknowledgements, publishes an
//    epoch in its own slot and polls the slots it depends on: no atomics on a shared counter).  Used
//    in front of the first layer, in front of attention (an attention unit polls only the owners of
//    its head's Q, K, V tiles) and at the end;
//  * data: between GEMM phases the activations validate themselves.  Every element a phase will write
//    is reset beforehand to a reserved bit pattern, the consumer loads its LDS slab without waiting
//    for anybody and loads again whatever still shows the pattern (see slab_unset, slab_retry and
//    clear_outputs).  This removes three dependent trips through the memory fabric (acknowledgement,
//    flag, poll) from every such boundary.
// All waits are bounded and raise an abort flag that makes every workgroup leave.
//
// Every workgroup owns a fixed, byte-balanced share of each weight matrix (a contiguous range of
// output rows / of gate-up or rotary pairs), so the sequence of 16-byte weight chunks a wavefront
// consumes in a phase is static.  It is consumed through a ring of register slots of one "chunk" each
// (8 loads = 8 KB per wavefront): a step multiplies out of its slot and refills it with the chunk RING
// ahead.  The loops that do this contain no other global memory operation and every refill issues the
// same number of loads, pinned in program order, which is what lets the compiler wait for exactly one
// slot (s_waitcnt vmcnt(N)) while the others stay in flight.  The ring is refilled with the first
// chunks of the next phase at each phase boundary (behind the loads of the activation slab, which is
// needed first), so those loads fly while the boundary's dependencies resolve.
//
// GEMM tiles are 16 weight rows (MFMA A operand) x all K; the waves interleave over K in 128-byte
// steps and their partial 16x16 tiles are summed in a fixed order through LDS; the reduced tiles wait
// in an LDS stash and their epilogues (and global stores) run outside the chunk loops.  Paired
// epilogues put the two rows of a pair (gate/up, or rotary j and j + hd/2) 8 rows apart in the same
// tile, so one thread finds both values of a pair in the same stashed tile.  RMSNorm is folded into the GEMMs: the producer packs
// h * gain and publishes per-workgroup partial sums of squares, the consumer multiplies its outputs by
// the row scale.  The hidden rows a phase multiplies with (B operand) are copied once per phase (per
// 8 KB, or in the second instance of the kernel 12 KB, of K per row) into LDS, all loads of the copy in flight together.
#include "attention_core.h"
#include "ss_mega.h"
#include <algorithm>
#include <type_traits>

namespace ss {

constexpr int MNW = MEGA_THREADS / 64; // wavefronts per workgroup
constexpr int CH = 4;                  // 128-byte steps per chunk per wave (8 loads = 8 KB per wave)
// Chunks per LDS activation slab: a template parameter SCK of the kernel, chosen per launch.  4 (8 KB of K per hidden row)
// always fits the rows the kernel takes; 6 (12 KB) is taken when the host finds that it saves slab trips for the model's
// shapes (mega_wants_large_slab) and the rows are few enough for LDS (<= 6 rows of a bf16 model): with d_model = 5120 a
// weight row then fits one slab and a phase stops reloading the slab for every tile.  Every unit of a slab row is
// requested whether K reaches it or not, so the larger slab costs half as many loads again where K is short: for the 7B
// shape (K = 4096 in three of four phases) it is 1 % slower, for the 13B shape 24 - 30 % faster.
constexpr int SCK_SMALL = 4, SCK_LARGE = 6;
constexpr int RING = 2;                // chunks in flight per wave
constexpr int CHUNK_ROW_BYTES = CH * MNW * 128; // bytes of a weight row one chunk covers (all waves)

struct Range {
    int u0, u1, ntiles;
};

__device__ __forceinline__ bool is_gemm(int kind) { return kind == PH_QKV || kind == PH_RESID || kind == PH_SWIGLU || kind == PH_HEAD; }

// the share of phase ph owned by workgroup wg: units are tiles (QKV), pairs (SWIGLU) or rows
__device__ __forceinline__ Range phase_range(const MegaPhase &ph, int wg, int G) {
    const int units = ph.kind == PH_QKV ? ph.N / 16 : ph.N;
    Range r; // wg * units < 2^31 for every shape the host accepts
    r.u0 = (int)((unsigned)wg * (unsigned)units / (unsigned)G);
    r.u1 = (int)((unsigned)(wg + 1) * (unsigned)units / (unsigned)G);
    const int per = ph.kind == PH_QKV ? 1 : (ph.kind == PH_SWIGLU ? 8 : 16);
    r.ntiles = (r.u1 - r.u0 + per - 1) / per;
    return r;
}

// weight row that A-row i (0..15) of tile `tile` stands for
__device__ __forceinline__ int a_row(int kind, int N, const Range &r, int hd, int tile, int i, bool &live) {
    if (kind == PH_QKV) {
        const int t = r.u0 + tile, tph = hd / 16;
        const int hh = t / tph, j0 = (t - hh * tph) * 8;
        live = true;
        return hh * hd + j0 + (i < 8 ? i : hd / 2 + i - 8);
    }
    if (kind == PH_SWIGLU) {
        const int pair = r.u0 + tile * 8 + (i & 7);
        live = pair < r.u1;
        return i < 8 ? pair : N + pair;
    }
    const int row = r.u0 + tile * 16 + i;
    live = row < r.u1;
    return row;
}

template <typename T> __device__ __forceinline__ int chunks_per_tile(int K) {
    const int row_bytes = K * (int)sizeof(T);
    return (row_bytes + CHUNK_ROW_BYTES - 1) / CHUNK_ROW_BYTES;
}

// Position in a workgroup's static chunk sequence.  Everything a step needs rides along (phase
// fields, the tile's per-lane row pointer), so stepping costs no division and no descriptor reload.
struct Cursor {
    bool active; // positions of this workgroup remain in the current phase
    int tile, ck, nck;
    int idx;    // position index inside the phase, padding included
    bool dummy; // a padding position: no data, no math
    Range r;
    int kind, N, kbytes; // phase kind, rows/pairs, bytes per weight row
    const char *W;
    const char *wp; // this lane's pointer into its weight row of the current tile (+ its wave / lane-group offset)
    bool live;      // the lane's A-row exists
};

template <typename T> __device__ __forceinline__ void cursor_tile(Cursor &c, int hd) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, cc = lane & 15, g = lane >> 4;
    const int row = a_row(c.kind, c.N, c.r, hd, c.tile, cc, c.live);
    c.wp = c.W + (size_t)row * c.kbytes + wave * 128 + g * 16;
}

// Position the cursor at this workgroup's first chunk of phase ph (inactive: no share, or not a GEMM).
template <typename T> __device__ __forceinline__ void cursor_begin(Cursor &c, const MegaPhase &ph, int hd, int wg, int G) {
    c.active = false;
    c.dummy = false;
    c.live = false;
    c.tile = 0;
    c.ck = 0;
    c.idx = 0;
    c.nck = 1;
    c.kind = ph.kind;
    c.N = ph.N;
    c.kbytes = 0;
    c.W = nullptr;
    c.wp = nullptr;
    c.r = Range{0, 0, 0};
    if (!is_gemm(ph.kind)) return;
    c.r = phase_range(ph, wg, G);
    if (c.r.ntiles <= 0) return;
    c.active = true;
    c.kbytes = ph.K * (int)sizeof(T);
    c.W = reinterpret_cast<const char *>(ph.W);
    c.nck = chunks_per_tile<T>(ph.K);
    cursor_tile<T>(c, hd);
}

// Advance to the next position of the phase.  Positions are real chunks or padding: a "slab group"
// (the chunks that share one LDS activation slab: the workgroup's whole share when K fits one slab, else
// SCK chunks of a tile) is padded to a multiple of RING positions, so that rounds of RING steps
// never straddle a slab reload or the end of the phase.  While `dummy` is set, (tile, ck, wp) already
// describe the next real chunk.  Touches no memory.
template <typename T, int SCK> __device__ __forceinline__ void cursor_next(Cursor &c, int hd) {
    ++c.idx;
    if (!c.dummy) {
        const bool multi = c.nck > SCK;
        bool group_end;
        if (++c.ck == c.nck) {
            c.ck = 0;
            ++c.tile;
            group_end = multi || c.tile == c.r.ntiles;
            if (c.tile < c.r.ntiles) cursor_tile<T>(c, hd);
        } else {
            group_end = multi && c.ck % SCK == 0;
        }
        if (!group_end) return;
        if (c.idx % RING != 0) {
            c.dummy = true;
            return;
        }
    } else {
        if (c.idx % RING != 0) return;
        c.dummy = false;
    }
    if (c.tile >= c.r.ntiles) c.active = false;
}

// Issue the 2*CH weight loads of chunk c for this lane.  Every call issues exactly 2*CH loads, whatever
// the chunk is (real, padding, dead row, K tail): positions without data read a small zero-filled
// buffer instead.  A fixed number of loads per step is what lets the compiler wait for one ring slot
// with an exact vmcnt(N) and leave the younger slots in flight; a conditional load would force vmcnt(0).
__device__ __forceinline__ void issue_chunk(const Cursor &c, bool valid, const char *zeros, u32x4 (&wbuf)[2 * CH]) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, g = lane >> 4;
    const bool real = valid && c.active && !c.dummy && c.live;
    const char *base = c.wp + (size_t)c.ck * CHUNK_ROW_BYTES;
    const int kb0 = c.ck * CHUNK_ROW_BYTES + wave * 128 + g * 16;
#pragma unroll
    for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int off = i * (MNW * 128) + j * 64;
            const char *a = (real && kb0 + off < c.kbytes) ? base + off : zeros;
            wbuf[2 * i + j] = ld16_global(a);
        }
}

__host__ __device__ constexpr int slab_row_bytes(int sck) { return sck * CH * MNW * 128; } // the K range one slab covers, per hidden row
__host__ __device__ constexpr int slab_pitch(int sck) { return slab_row_bytes(sck) + 48; }    // padded against LDS bank conflicts between rows

// LDS: [ union: activation slab | attention merge area ][ red ][ small ]
constexpr int STASH_TILES = 6; // reduced tiles kept in LDS until the epilogue flush

struct MegaSmemTail {
    float red[2][MNW][4][64]; // partial tiles, double-buffered
    float stash[STASH_TILES][4][64]; // reduced tiles: [slot][accumulator register v][lane]
    int stash_tile[STASH_TILES];     // tile index of each slot
    float scale[16];          // row scales of the current phase
    float sq[MNW][16];        // per wave partial row sums of squares
    float blk[MNW];
    int len[16];              // cached lengths of the sequences before this pass (read once at kernel start)
    int flag;
    int ok;                   // cleared by a wave whose bounded wait for input data ran out
};

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every outstanding
// global load (vmcnt(0)), which would drain the weight ring at each tile; this one waits for the LDS
// queue alone, so prefetched weight loads stay in flight across it.
// (s_waitcnt immediates, gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt_hi[15:14].)
__device__ __forceinline__ void lds_barrier() {
    __builtin_amdgcn_s_waitcnt(0xC07F); // lgkmcnt(0), vmcnt and expcnt untouched
    __builtin_amdgcn_s_barrier();
}


struct MegaSmem {
    unsigned char *u; // slab / attention area
    MegaSmemTail *t;
};

// Device-wide barrier without cache maintenance, in two parts so that weight loads can be put in
// flight between them.  (1) stores_done(): every wave waits until its own stores are acknowledged
// (vmcnt(0): on this ISA loads and stores share the counter, so this also drains the wave's loads).
// (2) grid_arrive(): workgroup barrier, then the epoch is published.  (3) grid_wait(): wave 0 polls all
// slots, workgroup barrier.  Waves other than wave 0 touch no memory in (3), so loads they issue
// between (2) and (3) stay in flight across the whole device-wide barrier.  false = aborted (bounded spin ran out, or another
// workgroup aborted).
__device__ __forceinline__ void stores_done() { __builtin_amdgcn_s_waitcnt(0x0F70); } // vmcnt(0)

__device__ __forceinline__ void grid_arrive(const MegaCall &P, unsigned epoch, MegaSmem &sm) {
    lds_barrier(); // every wave of the workgroup has passed stores_done()
    if (threadIdx.x == 0) __hip_atomic_store(&P.arrive[blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool grid_wait(const MegaCall &P, unsigned epoch, int lo, int hi, MegaSmem &sm) { // slots lo .. hi-1
    if (threadIdx.x < 64) {
        bool ok = true;
        unsigned spins = 0;
        for (;;) {
            bool all = true;
            for (int i = lo + (int)threadIdx.x; i < hi; i += 64) {
                const unsigned v = __hip_atomic_load(&P.arrive[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((int)(v - epoch) < 0) all = false;
            }
            if (__all(all)) break;
            if (++spins > P.spin_limit || __hip_atomic_load(P.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                ok = false;
                break;
            }
        }
        if (threadIdx.x == 0) {
            sm.t->flag = ok ? 1 : 0;
            if (!ok) __hip_atomic_store(P.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    lds_barrier();
    return sm.t->flag != 0;
}

// The attention unit (sequence b, head h) only reads what the QKV phase wrote for head h: its query
// rows, and the new key and value rows of that head.  Its workgroup therefore waits for the owners of
// those QKV tiles only (they publish the same epoch slots), not for the slowest workgroup of the chip;
// workgroups without a unit do not wait at this boundary at all.
__device__ __forceinline__ bool grid_wait_qkv_of_head(const MegaCall &P, unsigned epoch, int h, int G, MegaSmem &sm) {
    if (threadIdx.x < 64) {
        const int tph = P.hd / 16, units = 3 * P.H * tph; // QKV tiles per head and region, and in total
        bool ok = true;
        unsigned spins = 0;
        for (;;) {
            bool all = true;
            for (int region = 0; region < 3; ++region) {
                const int t_lo = (region * P.H + h) * tph, t_hi = t_lo + tph - 1;
                // owner of tile t under the static split u0(wg) = floor(wg * units / G)
                const int w_lo = (int)(((long long)(t_lo + 1) * G - 1) / units), w_hi = (int)(((long long)(t_hi + 1) * G - 1) / units);
                for (int i = w_lo + (int)threadIdx.x; i <= w_hi; i += 64) {
                    const unsigned v = __hip_atomic_load(&P.arrive[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    if ((int)(v - epoch) < 0) all = false;
                }
            }
            if (__all(all)) break;
            if (++spins > P.spin_limit || __hip_atomic_load(P.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                ok = false;
                break;
            }
        }
        if (threadIdx.x == 0) {
            sm.t->flag = ok ? 1 : 0;
            if (!ok) __hip_atomic_store(P.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    lds_barrier();
    return sm.t->flag != 0;
}

// ---------------------------------------------------------------- non-GEMM phases

template <typename T> __device__ __forceinline__ ActPlanes<T> act_planes(const MegaCall &P, int i);

// Embedding phase: every workgroup takes a slice of the columns of all hidden rows (the way the residual
// phases own columns), so the gather is one short step for the whole chip and each workgroup has its own
// partial sums of squares to publish.  Thread t works on hidden row t & 15 and columns (t >> 4) + 16 j of
// the slice; returns this thread's share of its row's sum of squares.
template <typename T>
__device__ __forceinline__ float do_embed(const MegaCall &P, const MegaPhase &ph, int wg, int G) {
    const ActPlanes<T> act = act_planes<T>(P, ACT_A);
    const int c0 = (int)((long long)wg * P.d / G), c1 = (int)((long long)(wg + 1) * P.d / G);
    const int r = threadIdx.x & 15;
    float ss = 0.f;
    if (r >= P.R) return ss;
    const T *src = nullptr;
    if (P.tokens) {
        int tok = P.tokens[r];
        if (tok < 0 || tok >= P.V) {
            atomicOr(P.status, 1);
            tok = tok < 0 ? 0 : P.V - 1;
        }
        src = reinterpret_cast<const T *>(P.embed) + (size_t)tok * P.d;
    }
    for (int e = c0 + (int)(threadIdx.x >> 4); e < c1; e += MEGA_THREADS / 16) {
        float x;
        if (src) {
            x = to_f32(src[e]);
            st_coh(&P.h[(size_t)r * P.d + e], x);
        } else {
            x = ld_coh(&P.h[(size_t)r * P.d + e]);
        }
        store_act_coh(act, (size_t)r * act.ld + e, ph.gain ? x * ldf_global(ph.gain + e) : x);
        ss += x * x;
    }
    return ss;
}

template <typename T, int HD>
__device__ __forceinline__ void do_attn_hd(const MegaCall &P, const MegaPhase &ph, int wg, int G, MegaSmem &sm) {
    AttnArgs a;
    const ActDesc dq = P.act_q, dout = P.act_o;
    a.q = dq.base;
    a.q_plane = dq.plane;
    a.ldq = dq.ld;
    const size_t esz = sizeof(T);
    a.kcache = (char *)P.kc + P.layer_elems * ph.layer * esz;
    a.vcache = (char *)P.vc + P.layer_elems * ph.layer * esz;
    a.len = P.len;
    a.B = P.B; a.M = P.M; a.H = P.H; a.hd = HD; a.S = P.S; a.R = P.R;
    a.nsplit = P.nsplit; a.chunk = P.chunk;
    a.part_o = P.part_o; a.part_m = P.part_m; a.part_l = P.part_l;
    a.act_out = dout.base; a.act_out_plane = dout.plane; a.ld_out = dout.ld;
    a.scale_log2e = P.scale_log2e;
    AttnSmem<HD, MNW> &asm_ = *reinterpret_cast<AttnSmem<HD, MNW> *>(sm.u);
    ActPlanes<T> out{reinterpret_cast<T *>(a.act_out), a.act_out_plane, a.ld_out};
    const int units = P.B * P.H * P.nsplit;
    for (int u = wg; u < units; u += G) {
        const int split = u % P.nsplit, bh = u / P.nsplit;
        const int h = bh % P.H, b = bh / P.H;
        if (P.nsplit == 1) { // one split: no partials, no merge
            attn_unit<T, HD, MNW, true, true>(a, 0, h, b, sm.t->len[b], asm_);
            continue;
        }
        attn_unit<T, HD, MNW, true>(a, split, h, b, sm.t->len[b], asm_);
        // the split that arrives last merges all splits of (b, h); partials travel through
        // coherent accesses, so completing the stores (release at workgroup scope) is all it takes
        bool merge = true;
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        __syncthreads();
        if (P.nsplit > 1) {
            if (threadIdx.x == 0) {
                const unsigned old = __hip_atomic_fetch_add(&P.attn_cnt[bh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sm.t->flag = old == (unsigned)(P.nsplit - 1);
            }
            __syncthreads();
            merge = sm.t->flag != 0;
        }
        if (merge) {
            for (int idx = threadIdx.x; idx < P.M * HD; idx += MEGA_THREADS) {
                const int c = idx / HD, e = idx - c * HD, row = b * P.M + c;
                store_act_coh(out, (size_t)row * a.ld_out + h * HD + e, attn_merge_elem<true>(a, row, h, e));
            }
            if (P.nsplit > 1 && threadIdx.x == 0) __hip_atomic_store(&P.attn_cnt[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
    }
}

template <typename T>
__device__ __forceinline__ void do_attn(const MegaCall &P, const MegaPhase &ph, int wg, int G, MegaSmem &sm) {
    if (P.hd == 128) do_attn_hd<T, 128>(P, ph, wg, G, sm);
    else if (P.hd == 64) do_attn_hd<T, 64>(P, ph, wg, G, sm);
    else do_attn_hd<T, 32>(P, ph, wg, G, sm);
}

// The activation planes a phase reads or writes (selects between named fields, see MegaCall).
__device__ __forceinline__ ActDesc act_desc(const MegaCall &P, int i) {
    // values first, selects second: a conditional expression between two members is an lvalue, i.e. a
    // run-time address into the argument, which is exactly what has to be avoided
    const ActDesc a = P.act_a, q = P.act_q, o = P.act_o, z = P.act_z, a1 = P.act_a1;
    ActDesc r = a1;
    if (i == ACT_A) r = a;
    if (i == ACT_Q) r = q;
    if (i == ACT_O) r = o;
    if (i == ACT_Z) r = z;
    return r;
}
template <typename T> __device__ __forceinline__ ActPlanes<T> act_planes(const MegaCall &P, int i) {
    const ActDesc a = act_desc(P, i);
    return ActPlanes<T>{reinterpret_cast<T *>(a.base), a.plane, a.ld};
}
// the norm partials that go with hidden rows packed into ACT_A (set 0) or ACT_A1 (set 1)
__device__ __forceinline__ float *nsq_set(const MegaCall &P, int act, int G) { return P.nsq + (act == ACT_A1 ? (size_t)16 * G : 0); }

// Row scales 1/sqrt(mean(h^2) + eps) from the producers' partial sums, in two halves so that the loads
// can share a memory round trip with other loads: 32 threads per row, rows beyond P.R are not needed.
struct ScaleLoads {
    float t[2][8];
};
__device__ __forceinline__ bool scale_slot(const MegaCall &P, int G, int half, int q, int &row, int &i) { // false: no such partial
    row = (threadIdx.x >> 5) + half * (MEGA_THREADS / 32);
    i = (threadIdx.x & 31) + 32 * q;
    return row < P.R && i < G;
}
// every thread issues all 16 loads (a fixed number of loads keeps the waits on them exact); slots
// without a partial read a valid address and are ignored when used
__device__ __forceinline__ void scales_issue(const MegaCall &P, const float *nsq, int G, bool only_unset, ScaleLoads &sl) {
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int row, i;
            const bool valid = scale_slot(P, G, half, q, row, i);
            const float *src = &nsq[(size_t)min(row, P.R - 1) * G + min(i, G - 1)];
            if (!only_unset) sl.t[half][q] = ld_coh(src);
            else if (valid && f2u(sl.t[half][q]) == 0xffffffffu) sl.t[half][q] = ld_coh(src);
        }
}
__device__ __forceinline__ void scales_finish(const MegaCall &P, const float *nsq, int G, const ScaleLoads &sl, MegaSmem &sm) {
    const int j = threadIdx.x & 31;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int row = (threadIdx.x >> 5) + half * (MEGA_THREADS / 32);
        float s = 0.f;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int r2, i;
            s += scale_slot(P, G, half, q, r2, i) ? sl.t[half][q] : 0.f;
        }
        if (row < P.R)
            for (int i = 256 + j; i < G; i += 32) s += ld_coh(&nsq[(size_t)row * G + i]); // grids beyond 256 workgroups (flag barriers only)
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) s += __shfl_xor(s, o);
        if (j == 0 && row < 16) sm.t->scale[row] = row < P.R ? 1.0f / sqrtf(s / (float)P.d + P.eps) : 0.f;
    }
}
static_assert(MEGA_THREADS / 32 * 2 >= 16, "two halves of the scale loads cover 16 rows");

// Copy the hidden rows of K slab `slab` of the phase's B operand into LDS (zero beyond K), in two steps:
// slab_issue() puts every load in flight (with_scales: also the loads of the phase's row scales), so the
// whole copy costs one memory round trip, and slab_finish() writes the data to LDS.  Other loads may
// be issued between the two: loads return in order, so the slab does not wait for them.
//
// Self-validating data.  Between a producer's stores and a consumer's loads the usual protocol costs
// three dependent trips through the memory fabric (store acknowledgement, flag, poll) before the slab
// can even be requested.  In data-sync mode a producer just stores, and the consumer loads the slab
// and looks at it: every element of an activation buffer (and every norm partial) is reset, well
// before it is written, to a bit pattern no computed value has (all ones: a NaN with a full payload;
// bf16_rne and the fp32 arithmetic produce other NaNs at most), so a unit that still shows the pattern
// has not arrived and is simply loaded again (bounded).  Each element is validated on its own, so no
// ordering between different stores is assumed.  The resets ride on causality, see clear_outputs().
__host__ __device__ constexpr int slab_units(int sck) { return slab_row_bytes(sck) / 16 / MEGA_THREADS; } // 16-byte units per thread and slab row
template <int NPR, int SCK> struct SlabLoads { // NPR: (plane, row) pairs per batch
    u32x4 v[NPR][slab_units(SCK)]; // [(plane, row) pair][unit]
    ScaleLoads sl;
};
static_assert(slab_row_bytes(SCK_SMALL) % (16 * MEGA_THREADS) == 0 && slab_row_bytes(SCK_LARGE) % (16 * MEGA_THREADS) == 0, "whole units per thread");

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));
// running maximum that ends at all ones iff some element seen was the "not written yet" pattern
template <typename T> __device__ __forceinline__ uint32_t unset_acc(uint32_t m, uint32_t w);
template <> __device__ __forceinline__ uint32_t unset_acc<bf16_t>(uint32_t m, uint32_t w) {
    return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2, m), __builtin_bit_cast(u16x2, w)));
}
template <> __device__ __forceinline__ uint32_t unset_acc<float>(uint32_t m, uint32_t w) { return m > w ? m : w; }
template <typename T> __device__ __forceinline__ bool unset_seen(uint32_t m);
template <> __device__ __forceinline__ bool unset_seen<bf16_t>(uint32_t m) { return (m & 0xffffu) == 0xffffu || (m >> 16) == 0xffffu; }
template <> __device__ __forceinline__ bool unset_seen<float>(uint32_t m) { return m == 0xffffffffu; }
template <typename T> __device__ __forceinline__ bool unit_unset(const u32x4 &v) {
    return unset_seen<T>(unset_acc<T>(unset_acc<T>(v[0], v[1]), unset_acc<T>(v[2], v[3])));
}
__device__ __forceinline__ void store_unset(bf16_t *p) { st_coh(p, bf16_t{(uint16_t)0xffffu}); }
__device__ __forceinline__ void store_unset(float *p) { st_coh(p, u2f(0xffffffffu)); }

// Unit (i, h2) of a batch that starts at (plane, row) pair pr0: byte offset of its 16 bytes in the source
// planes, clamped to a valid address when the unit does not exist (pair beyond the slab rows, row
// without data, K tail); false: it does not exist and counts as zeros.
template <typename T, int SCK>
__device__ __forceinline__ bool slab_unit(const MegaCall &P, const MegaPhase &ph, const ActPlanes<T> &src, int slab, int pr, int h2,
                                          uint32_t &byte_off) {
    constexpr int PER16 = 16 / (int)sizeof(T); // elements per 16-byte unit
    const bool head = ph.kind == PH_HEAD;
    const int rows = P.slab_rows, nrow = Traits<T>::PLANES * rows;
    const int nlive = head ? P.head_rows : P.R;
    const int prc = min(pr, nrow - 1);
    const int r = prc % rows, pl = prc / rows, rc = min(r, nlive - 1);
    const int brow = head ? P.head_row0 + rc * P.head_stride : rc;
    const int x = threadIdx.x + h2 * MEGA_THREADS;
    const int k = slab * (slab_row_bytes(SCK) / (int)sizeof(T)) + x * PER16; // K is a multiple of the unit
    const bool valid = pr < nrow && r < nlive && k < ph.K;
    byte_off = (uint32_t)((pl * src.plane + (size_t)brow * src.ld + (k < ph.K ? k : 0)) * sizeof(T));
    return valid;
}
// All loads of a batch (with_scales: and of the row scales), unconditionally: the number of loads in
// flight is a compile-time constant, so a later wait for them can leave younger loads in flight.
template <typename T, int NPR, int SCK>
__device__ __forceinline__ void slab_issue(const MegaCall &P, const MegaPhase &ph, int slab, int pr0, int G, bool with_scales,
                                           SlabLoads<NPR, SCK> &L) {
    const ActPlanes<T> src = act_planes<T>(P, ph.act_src);
    if (with_scales) scales_issue(P, nsq_set(P, ph.act_src, G), G, false, L.sl);
#pragma unroll
    for (int i = 0; i < NPR; ++i)
#pragma unroll
        for (int h2 = 0; h2 < slab_units(SCK); ++h2) {
            uint32_t off;
            slab_unit<T, SCK>(P, ph, src, slab, pr0 + i, h2, off);
            L.v[i][h2] = ld16_coh_buf(src.base, off);
        }
}
// true: something this lane loaded still shows the "not written yet" pattern
template <typename T, int NPR, int SCK>
__device__ __forceinline__ bool slab_unset(const MegaCall &P, const MegaPhase &ph, int slab, int pr0, int G, bool with_scales,
                                           const SlabLoads<NPR, SCK> &L) {
    const ActPlanes<T> src = act_planes<T>(P, ph.act_src);
    uint32_t m = 0, ms = 0;
#pragma unroll
    for (int i = 0; i < NPR; ++i)
#pragma unroll
        for (int h2 = 0; h2 < slab_units(SCK); ++h2) {
            uint32_t off;
            const bool valid = slab_unit<T, SCK>(P, ph, src, slab, pr0 + i, h2, off);
            const uint32_t um = unset_acc<T>(unset_acc<T>(L.v[i][h2][0], L.v[i][h2][1]), unset_acc<T>(L.v[i][h2][2], L.v[i][h2][3]));
            m = unset_acc<T>(m, valid ? um : 0u);
        }
    if (with_scales) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                int row, i;
                ms = unset_acc<float>(ms, scale_slot(P, G, half, q, row, i) ? f2u(L.sl.t[half][q]) : 0u);
            }
    }
    return unset_seen<T>(m) || unset_seen<float>(ms);
}
// After a first slab_unset() found the pattern: wait (bounded) until nothing this wave loaded shows
// it, loading again what does.  false: gave up (the caller raises the abort flag).
template <typename T, int NPR, int SCK>
__device__ __forceinline__ bool slab_retry(const MegaCall &P, const MegaPhase &ph, int slab, int pr0, int G, bool with_scales,
                                           SlabLoads<NPR, SCK> &L) {
    const ActPlanes<T> src = act_planes<T>(P, ph.act_src);
    for (unsigned spins = 0; spins < P.spin_limit; ++spins) {
        if (__hip_atomic_load(P.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) return false;
        if (with_scales) scales_issue(P, nsq_set(P, ph.act_src, G), G, true, L.sl);
#pragma unroll
        for (int i = 0; i < NPR; ++i)
#pragma unroll
            for (int h2 = 0; h2 < slab_units(SCK); ++h2) {
                uint32_t off;
                if (slab_unit<T, SCK>(P, ph, src, slab, pr0 + i, h2, off) && unit_unset<T>(L.v[i][h2])) L.v[i][h2] = ld16_coh_buf(src.base, off);
            }
        if (!__any(slab_unset<T, NPR, SCK>(P, ph, slab, pr0, G, with_scales, L))) return true;
    }
    return false;
}
template <typename T, int NPR, int SCK>
__device__ __forceinline__ void slab_finish(const MegaCall &P, const MegaPhase &ph, int slab, int pr0, int G, bool with_scales,
                                            const SlabLoads<NPR, SCK> &L, MegaSmem &sm) {
    const ActPlanes<T> src = act_planes<T>(P, ph.act_src);
    const int nrow = Traits<T>::PLANES * P.slab_rows;
    if (with_scales) scales_finish(P, nsq_set(P, ph.act_src, G), G, L.sl, sm);
#pragma unroll
    for (int i = 0; i < NPR; ++i) {
        const int pr = pr0 + i;
        if (pr < nrow) {
#pragma unroll
            for (int h2 = 0; h2 < slab_units(SCK); ++h2) {
                uint32_t off;
                const bool valid = slab_unit<T, SCK>(P, ph, src, slab, pr, h2, off);
                const int x = threadIdx.x + h2 * MEGA_THREADS;
                *reinterpret_cast<u32x4 *>(sm.u + (size_t)pr * slab_pitch(SCK) + x * 16) = valid ? L.v[i][h2] : zero16();
            }
        }
    }
}

// Reset, to the "not written yet" pattern, what this workgroup will write in phase `tp` (a later phase).
// Called in an earlier phase c, once that phase's input is complete, and followed by a wait for the
// store acknowledgements before phase c's own outputs are stored.  Two things must hold:
//  (1) nobody still reads the old contents: they were consumed at the start of a phase before c, and
//      the input of c being complete means that every workgroup has finished the phase before c;
//  (2) every consumer sees the reset before it first looks for the new data: it looks after finishing
//      phase `tp`, whose input it found complete; that input descends, store by store, from the outputs
//      of phase c of EVERY workgroup, which were stored after the resets were acknowledged.
// The schedule that satisfies both (set by the host in MegaPhase::clear_phase): QKV clears what the O
// projection writes, the O projection what gate/up writes, gate/up what the down projection writes, and
// the down projection (the embedding, before the first layer) what the next attention phase writes.
// It needs every workgroup to own part of every GEMM phase, which the host checks (MegaCall::data_sync).
template <typename T>
__device__ __forceinline__ void clear_outputs(const MegaCall &P, const MegaPhase &tp, int wg, int G) {
    constexpr int PL = Traits<T>::PLANES;
    if (tp.kind == PH_RESID || tp.kind == PH_SWIGLU) {
        const Range r = phase_range(tp, wg, G); // columns of the output = rows (pairs) of the weight matrix
        const ActPlanes<T> a = act_planes<T>(P, tp.kind == PH_RESID ? tp.act_dst : ACT_Z);
        const int ncol = r.u1 - r.u0, n = ncol * P.R * PL;
        for (int idx = threadIdx.x; idx < n; idx += MEGA_THREADS) {
            const int col = r.u0 + idx % ncol, rest = idx / ncol, row = rest % P.R, pl = rest / P.R;
            store_unset(a.base + pl * a.plane + (size_t)row * a.ld + col);
        }
        if (tp.kind == PH_RESID && threadIdx.x < 16) store_unset(&nsq_set(P, tp.act_dst, G)[(size_t)threadIdx.x * G + wg]);
    } else if (tp.kind == PH_ATTN) {
        const ActPlanes<T> o = act_planes<T>(P, ACT_O);
        const int units = P.B * P.H * P.nsplit, n = P.M * P.hd * PL;
        for (int u = wg; u < units; u += G) {
            if (u % P.nsplit != 0) continue; // one of the splits of (sequence, head) does it
            const int bh = u / P.nsplit, h = bh % P.H, b = bh / P.H;
            for (int idx = threadIdx.x; idx < n; idx += MEGA_THREADS) {
                const int e = idx % P.hd, rest = idx / P.hd, c = rest % P.M, pl = rest / P.M;
                store_unset(o.base + pl * o.plane + (size_t)(b * P.M + c) * o.ld + h * P.hd + e);
            }
        }
    }
}

// ---------------------------------------------------------------- GEMM chunk + tile epilogue

// What a thread carries from the start of a phase to its epilogue.  A workgroup with a single tile of
// a residual phase (the usual case) fetches its element of h and of the gain while the weights
// stream, instead of paying a memory round trip between the last MFMA and the stores.
struct EpiState {
    float rowsq;       // this thread's share of the row sums of squares of the new hidden rows
    float h_pre, g_pre;
    bool pre;          // h_pre / g_pre hold h[c][n] and gain[n] of this thread's element of tile 0
};
// this thread's element of a residual phase's tile: A-row t >> 4, hidden row t & 15 (see flush_stash)
__device__ __forceinline__ void epi_prefetch(const MegaCall &P, const MegaPhase &ph, const Range &r, EpiState &es) {
    es.pre = ph.kind == PH_RESID && r.ntiles == 1;
    es.h_pre = 0.f;
    es.g_pre = 1.f;
    if (!es.pre) return;
    const int c = threadIdx.x & 15, i = threadIdx.x >> 4;
    bool live;
    const int n = a_row(ph.kind, ph.N, r, P.hd, 0, i, live);
    if (live && c < P.R) {
        es.h_pre = P.h[(size_t)c * P.d + n]; // plain load: see elem_epilogue
        if (ph.gain) es.g_pre = ldf_global(ph.gain + n);
    }
}

// Epilogue of one output element: A-row i (0..15) of tile `tile` for hidden row c.  Paired epilogues
// (gate/up, rotary) are called for i < 8 with `partner` = the value of A-row i + 8.
template <typename T>
__device__ __forceinline__ void elem_epilogue(const MegaCall &P, const MegaPhase &ph, const Range &r, int tile, int i, int c, float sum,
                                              float partner, EpiState &es, MegaSmem &sm) {
    bool live;
    const int n = a_row(ph.kind, ph.N, r, P.hd, tile, i, live);
    if (ph.kind == PH_RESID) {
        if (live && c < P.R) {
            const size_t o = (size_t)c * P.d + n;
            // plain load: these columns of h are only ever written by this workgroup (and, before the
            // first layer, by the embedding phase, which no cache of this XCD has seen yet)
            const float hn = (es.pre ? es.h_pre : P.h[o]) + sum;
            st_coh(&P.h[o], hn);
            const ActPlanes<T> act = act_planes<T>(P, ph.act_dst);
            const float gn = es.pre ? es.g_pre : (ph.gain ? ldf_global(ph.gain + n) : 1.f); // no gain: nothing normalises these rows
            store_act_coh(act, (size_t)c * act.ld + n, ph.gain ? hn * gn : hn);
            es.rowsq += hn * hn;
        }
        return;
    }
    if (ph.kind == PH_HEAD) {
        if (live && c < P.head_rows) P.logits[(size_t)c * P.ldo + n] = sum * sm.t->scale[P.head_row0 + c * P.head_stride];
        return;
    }
    if (!live || c >= P.R) return;
    const float sc = sm.t->scale[c];
    const float x0s = sum * sc, x1s = partner * sc;
    if (ph.kind == PH_SWIGLU) {
        const ActPlanes<T> z = act_planes<T>(P, ACT_Z);
        const float s = x0s / (1.0f + expf(-x0s));
        store_act_coh(z, (size_t)c * z.ld + n, s * x1s); // n = pair index = column of z
        return;
    }
    // PH_QKV: n = hh*hd + j, j in the first half of head hh (heads ordered q | k | v)
    const int hh = n / P.hd, j = n - hh * P.hd;
    const int region = hh / P.H, h = hh - region * P.H;
    const int b = c / P.M, ii = c - b * P.M;
    int pos = sm.t->len[b] + ii;
    if (pos > P.max_pos - 1) pos = P.max_pos - 1; // host validation keeps these from happening
    if (pos > P.S - 1) pos = P.S - 1;
    float x0 = x0s, x1 = x1s;
    if (region < 2) {
        const float2 cs = P.rope[(size_t)pos * (P.hd / 2) + j];
        x0 = x0s * cs.x - x1s * cs.y;
        x1 = x0s * cs.y + x1s * cs.x;
    }
    if (region == 0) {
        const ActPlanes<T> q = act_planes<T>(P, ACT_Q);
        const size_t o = (size_t)c * q.ld + h * P.hd + j;
        store_act_coh(q, o, x0);
        store_act_coh(q, o + P.hd / 2, x1);
    } else if (region == 1) {
        T *kc = reinterpret_cast<T *>(P.kc) + P.layer_elems * ph.layer + (((size_t)b * P.H + h) * P.S + pos) * P.hd + j;
        st_coh(kc, to_storage<T>(x0));
        st_coh(kc + P.hd / 2, to_storage<T>(x1));
    } else {
        T *vc = reinterpret_cast<T *>(P.vc) + P.layer_elems * ph.layer + ((size_t)b * P.H + h) * P.S * P.hd +
                ((size_t)(pos >> 6) * P.hd) * 64 + (pos & 63);
        st_coh(vc + (size_t)j * 64, to_storage<T>(x0));
        st_coh(vc + (size_t)(j + P.hd / 2) * 64, to_storage<T>(x1));
    }
}

// acc0 / acc1 += chunk: the hi and lo planes (bf16) or alternate k-blocks (f32) go to different
// accumulators so that consecutive MFMAs do not wait on each other
__device__ __forceinline__ void mma2(f32x4 &acc0, f32x4 &acc1, u32x4 w, const Act<bf16_t> &b, int) {
    bf16x8 av = __builtin_bit_cast(bf16x8, w);
    acc0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[0]), acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8, b.p[1]), acc1, 0, 0, 0);
}
__device__ __forceinline__ void mma2(f32x4 &acc0, f32x4 &acc1, u32x4 w, const Act<float> &b, int j) {
    if (j & 1) acc1 = mma(acc1, w, b);
    else acc0 = mma(acc0, w, b);
}

// multiply chunk c (weights in wbuf) into the tile accumulators; the B operand comes from the LDS slab
template <typename T, int SCK>
__device__ __forceinline__ void mma_chunk(const Cursor &c, const MegaCall &P, const u32x4 (&wbuf)[2 * CH], f32x4 &acc0, f32x4 &acc1,
                                          MegaSmem &sm) {
    constexpr int PL = Traits<T>::PLANES;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, cc = lane & 15, g = lane >> 4;
    if (c.ck == 0) {
        acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
        acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const bool blive = cc < P.slab_rows;
    const unsigned char *lb = sm.u + (size_t)cc * slab_pitch(SCK) + (c.ck % SCK) * CHUNK_ROW_BYTES + wave * 128 + g * 16;
    const size_t plane_off = (size_t)P.slab_rows * slab_pitch(SCK);
#pragma unroll
    for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            Act<T> av;
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
                av.p[pl] = blive ? *reinterpret_cast<const u32x4 *>(lb + pl * plane_off + i * (MNW * 128) + j * 64) : zero16();
            mma2(acc0, acc1, wbuf[2 * i + j], av, j);
        }
}

// Tile complete: fixed-order sum of the waves' partial tiles by waves 0-3 (register v = wave) into the
// LDS stash.  No global memory is touched here: the epilogues (and their stores) run at flush time,
// outside the chunk loop, because on this ISA a pending store would force every later wait on a
// weight load to vmcnt(0) (loads and stores share the counter and may complete out of order).
__device__ __forceinline__ void finish_tile(int tile, const f32x4 &acc0, const f32x4 &acc1, int &tile_seq, int &nstash,
                                            MegaSmem &sm) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int par = tile_seq & 1;
    ++tile_seq;
#pragma unroll
    for (int v = 0; v < 4; ++v) sm.t->red[par][wave][v][lane] = acc0[v] + acc1[v];
    lds_barrier();
    if (wave < 4) {
        float sum = sm.t->red[par][0][wave][lane];
#pragma unroll
        for (int w2 = 1; w2 < MNW; ++w2) sum += sm.t->red[par][w2][wave][lane];
        sm.t->stash[nstash][wave][lane] = sum;
        if (threadIdx.x == 0) sm.t->stash_tile[nstash] = tile;
    }
    ++nstash;
}

// Epilogues of the stashed tiles, one output element per thread and pass: thread t takes hidden row
// c = t & 15 (which keeps a thread's contribution to the row sums of squares on one row) and A-row
// t >> 4 of a tile (paired epilogues: pair (t >> 4) & 7 of one of two tiles).  Element (i, c) of a
// reduced tile sits in the stash at [register i & 3][lane c + 16 * (i >> 2)] (MFMA output layout).
// A wave-per-accumulator-register split would run the same ~150 instructions six times per wave
// with 10 of 64 lanes doing useful work, which took 2.5 us at every phase end.
template <typename T>
__device__ __forceinline__ void flush_stash(const MegaCall &P, const MegaPhase &ph, const Range &r, int &nstash, EpiState &es,
                                            bool last, MegaSmem &sm) {
    lds_barrier(); // the stash writes of the last tile are visible
    const int c = threadIdx.x & 15, ii = threadIdx.x >> 4;
    if (ph.kind == PH_QKV || ph.kind == PH_SWIGLU) {
        const int i = ii & 7;
        for (int slot = ii >> 3; slot < nstash; slot += MEGA_THREADS / 128) {
            const float sum = sm.t->stash[slot][i & 3][c + 16 * (i >> 2)];
            const float partner = sm.t->stash[slot][i & 3][c + 16 * (i >> 2) + 32];
            elem_epilogue<T>(P, ph, r, sm.t->stash_tile[slot], i, c, sum, partner, es, sm);
        }
    } else {
        for (int slot = 0; slot < nstash; ++slot)
            elem_epilogue<T>(P, ph, r, sm.t->stash_tile[slot], ii, c, sm.t->stash[slot][ii & 3][c + 16 * (ii >> 2)], 0.f, es, sm);
    }
    nstash = 0;
    if (last) return; // end of the phase: the phase boundary synchronises
    stores_done(); // the next segment starts with no store pending
    lds_barrier(); // nobody overwrites the stash before everyone has read it
}

// ---------------------------------------------------------------- the kernel

template <typename T, int SCK>
__global__ __launch_bounds__(MEGA_THREADS) void verify_persistent_kernel(MegaCall P) {
    static_assert(10 * slab_units(SCK) < 31, "one mask bit per unit of a batch, bit 31 for the row scales");
    extern __shared__ __align__(16) unsigned char smem_raw[];
    MegaSmem sm;
    sm.u = smem_raw;
    sm.t = reinterpret_cast<MegaSmemTail *>(smem_raw + P.u_bytes);
    const int wg = blockIdx.x, G = gridDim.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (threadIdx.x < 16) sm.t->len[threadIdx.x] = (int)threadIdx.x < P.B ? P.len[threadIdx.x] : 0; // lengths change in the last phase only
    if (threadIdx.x == 0) sm.t->ok = 1;
    lds_barrier();

    // Weight pipeline: `la` runs RING positions ahead of `cc` (the next chunk to multiply); the loads of
    // those chunks are in flight into the ring slots.  A step multiplies straight out of its
    // slot (which waits for that slot's loads only - later slots stay in flight), then refills the slot
    // with the chunk RING ahead.  A workgroup's positions per phase are padded to a multiple of RING, so
    // each phase starts at slot 0 and the code below exists once.  The last round of a phase does not
    // refill: the ring is empty at a phase boundary and is refilled there with the first round of the
    // next phase, so those loads fly while the boundary's dependencies resolve.
    struct State {
        Cursor cc, la;
        f32x4 acc0, acc1;
        int tile_seq, slab_tag;
        EpiState es;
    } st;
    st.acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
    st.acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
    st.tile_seq = 0;
    st.slab_tag = -1;
    st.es.rowsq = 0.f;
    st.es.pre = false;
    st.es.h_pre = 0.f;
    st.es.g_pre = 1.f;

    u32x4 ring[RING][2 * CH]; // only ever indexed by unrolled constants: lives in registers
    static_assert(MNW >= 4, "waves 0-3 reduce one accumulator register each");

    const char *zeros = reinterpret_cast<const char *>(P.zeros);
    // The empty asm statements are compiler barriers: they pin the slot's loads to this point of the
    // program.  Without them the scheduler sinks each load next to its use (to shorten live ranges),
    // which would leave one 16-byte load in flight per wave instead of a ring of chunks.
    auto fill = [&](u32x4(&slot)[2 * CH]) { // always 2*CH loads
        asm volatile("" ::: "memory");
        issue_chunk(st.la, true, zeros, slot);
        asm volatile("" ::: "memory");
        if (st.la.active) cursor_next<T, SCK>(st.la, P.hd);
    };

    for (int p = 0; p < P.n_phases; ++p) {
        const MegaPhase ph = P.phases[p];
        // Phase boundary.  A workgroup with GEMM work in the phase fills all ring slots here (see below);
        // one without leaves the ring alone.
        cursor_begin<T>(st.cc, ph, P.hd, wg, G);
        st.la = st.cc;
        const unsigned epoch = P.epoch_base + (unsigned)p;
        const int attn_units = P.B * P.H * P.nsplit;
        const bool want_scales = ph.kind == PH_QKV || ph.kind == PH_SWIGLU || ph.kind == PH_HEAD;
        // How this phase's input becomes visible.  Flags: the producers wait for their stores, publish
        // their epoch, and the consumer polls the epochs before it loads anything.  Data: nobody waits
        // for acknowledgements; the consumer loads the first slab at once (together with the weight
        // prefetch) and validates it (slab_unset, slab_retry).  After the attention phase the workgroups without
        // a unit would find nothing for a long time, so they first wait for the units' epochs (a hint:
        // the data is validated all the same).
        const bool polled = P.data_sync && ph.sync != SYNC_FLAGS && st.cc.active;
        const bool hint_first = polled && ph.sync == SYNC_DATA_ATTN && wg >= attn_units;
        const bool spec = polled && !hint_first;
        if (p > 0) {
            if (!polled) stores_done(); // (a workgroup without a share of a data-synchronised phase cannot occur: the host checks)
            grid_arrive(P, epoch, sm);
        }
        // publish this workgroup's partial sums of squares of the new hidden rows: thread t holds a share of row t & 15
        auto publish_rowsq = [&](float rs, int act_dst) {
            rs += __shfl_xor(rs, 16);
            rs += __shfl_xor(rs, 32);
            lds_barrier(); // readers of the previous use are done
            if (lane < 16) sm.t->sq[wave][lane] = rs;
            lds_barrier();
            if (threadIdx.x < 16) {
                float tot = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < MNW; ++w2) tot += sm.t->sq[w2][threadIdx.x];
                st_coh(&nsq_set(P, act_dst, G)[(size_t)threadIdx.x * G + wg], f2u(tot) == 0xffffffffu ? u2f(0xffc00000u) : tot); // the all-ones pattern is reserved
            }
        };
        int nstash = 0;
        const Range my = st.cc.r; // this workgroup's share of the phase
        // One segment: n_fill rounds of RING steps in which each step refills its slot, then (last: the
        // phase ends here) one round that does not.  The loops hold no global memory operation except
        // the pinned ring loads, and nothing else is pending when they start (the wait below costs
        // little: the ring loads it waits for are the ones the first steps need anyway); both are what
        // lets the compiler wait for one slot with an exact count and leave the younger slots in flight.
        auto run_segment = [&](int n_fill, bool last) {
            auto step = [&](auto fill_c, u32x4(&slot)[2 * CH]) {
                const Cursor c = st.cc;
                cursor_next<T, SCK>(st.cc, P.hd);
                if (!c.dummy) mma_chunk<T, SCK>(c, P, slot, st.acc0, st.acc1, sm);
                if (decltype(fill_c)::value) fill(slot);
                if (!c.dummy && c.ck + 1 == c.nck) finish_tile(c.tile, st.acc0, st.acc1, st.tile_seq, nstash, sm);
            };
            stores_done();
            for (int i = 0; i < n_fill; ++i) {
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) step(std::true_type{}, ring[sl]);
            }
            if (last) {
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) step(std::false_type{}, ring[sl]);
            }
        };
        // One K slab of the B operand into LDS, in batches of 10 (plane, row) pairs, one memory round trip
        // each (5 rows of a bf16 model: one batch).
        // false: a bounded wait for the data ran out (every wave of the workgroup returns the same).
        auto load_slab = [&](int slab, bool scales, bool fills, SlabLoads<10, SCK> &L) __attribute__((always_inline)) {
            bool ok = true;
            slab_issue<T, 10, SCK>(P, ph, slab, 0, G, scales, L);
            asm volatile("" ::: "memory"); // keeps the compiler from fusing the two loops (load, wait, store per row)
            // The first look at the data is straight-line code behind the loads (once per branch), so it
            // waits for them with an exact count and leaves the younger weight prefetch in flight.
            bool dirty;
            if (fills) { // the weight prefetch goes out behind the slab: loads return in order, and the slab is needed first
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) fill(ring[sl]);
                dirty = polled && __any(slab_unset<T, 10, SCK>(P, ph, slab, 0, G, scales, L));
            } else {
                dirty = polled && __any(slab_unset<T, 10, SCK>(P, ph, slab, 0, G, scales, L));
            }
            if (dirty) ok = slab_retry<T, 10, SCK>(P, ph, slab, 0, G, scales, L);
            lds_barrier(); // every wave is done with the previous slab
            slab_finish<T, 10, SCK>(P, ph, slab, 0, G, scales, L, sm);
            if (Traits<T>::PLANES * P.slab_rows > 10) {
                slab_issue<T, 10, SCK>(P, ph, slab, 10, G, false, L);
                asm volatile("" ::: "memory");
                if (polled && ok && __any(slab_unset<T, 10, SCK>(P, ph, slab, 10, G, false, L))) ok = slab_retry<T, 10, SCK>(P, ph, slab, 10, G, false, L);
                slab_finish<T, 10, SCK>(P, ph, slab, 10, G, false, L, sm);
            }
            if (!ok && lane == 0) {
                sm.t->ok = 0;
                __hip_atomic_store(P.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (P.timeline && threadIdx.x == 0 && st.cc.idx == 0) P.timeline[(size_t)(5 * p + 2) * G + wg] = wall_clock64();
            lds_barrier();
            return sm.t->ok != 0;
        };
        const bool multi_slab = st.cc.nck > SCK;
        const bool clears = P.data_sync && ph.clear_phase >= 0;
        st.es.rowsq = 0.f;
        if (st.cc.active) {
            // GEMM phase with work: the first slab is loaded (and, with data synchronisation, validated) in the loop below
            epi_prefetch(P, ph, my, st.es);
            // (spec: the ring is filled right behind the first slab's loads, see load_slab)
            if (wave != 0 && !spec) { // wave 0 polls memory in a barrier, which would wait for these loads
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) fill(ring[sl]);
            }
            if (p > 0 && !spec) {
                if (hint_first ? !grid_wait(P, epoch, 0, min(attn_units, G), sm) : !grid_wait(P, epoch, 0, G, sm)) return;
            }
            if (P.timeline && threadIdx.x == 0) P.timeline[(size_t)(5 * p) * G + wg] = wall_clock64();
            if (wave == 0 && !spec) {
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) fill(ring[sl]);
            }
            if (P.timeline && threadIdx.x == 0) P.timeline[(size_t)(5 * p + 1) * G + wg] = wall_clock64();
        } else {
            // No GEMM work in this phase (embedding, attention, length update, or no share of a small
            // GEMM): the weight ring is not used; giving it a constant value here tells the compiler
            // that nothing of it lives across the attention code.
#pragma unroll
            for (int sl = 0; sl < RING; ++sl)
#pragma unroll
                for (int k = 0; k < 2 * CH; ++k) ring[sl][k] = zero16();
            if (p > 0) {
                if (ph.kind == PH_ATTN && attn_units <= G) { // one unit per workgroup at most: wait for its producers only
                    if (wg < attn_units && !grid_wait_qkv_of_head(P, epoch, (wg / P.nsplit) % P.H, G, sm)) return;
                } else if (ph.kind == PH_LEN) {
                    // nothing to wait for: the lengths were read by every workgroup before the first phase
                    // boundary of the launch, which this workgroup has long passed
                } else if (!grid_wait(P, epoch, 0, G, sm)) {
                    return;
                }
            }
            if (P.timeline && threadIdx.x == 0) P.timeline[(size_t)(5 * p) * G + wg] = wall_clock64();
            switch (ph.kind) {
            case PH_EMBED:
                if (clears) clear_outputs<T>(P, P.phases[ph.clear_phase], wg, G);
                publish_rowsq(do_embed<T>(P, ph, wg, G), ACT_A);
                break;
            case PH_ATTN:
                do_attn<T>(P, ph, wg, G, sm);
                st.slab_tag = -1; // the attention area aliases the slab
                break;
            case PH_LEN:
                if (wg == 0 && (int)threadIdx.x < P.B) P.len[threadIdx.x] += P.M;
                break;
            case PH_RESID: // no share of the new hidden rows: this workgroup's partial sums of squares are zero
                if (threadIdx.x < 16) st_coh(&nsq_set(P, ph.act_dst, G)[(size_t)threadIdx.x * G + wg], 0.f);
                break;
            default: break;
            }
            if (P.timeline && threadIdx.x == 0) {
                P.timeline[(size_t)(5 * p + 1) * G + wg] = wall_clock64();
                P.timeline[(size_t)(5 * p + 4) * G + wg] = wall_clock64();
            }
            continue;
        }
        while (st.cc.active) {
            // one segment = rounds that share an LDS slab and fit the stash
            const Cursor &cc = st.cc;
            const bool multi = cc.nck > SCK;
            const int grp_end = min((cc.ck / SCK + 1) * SCK, cc.nck); // multi: end of the slab group
            const int grp_chunks = multi ? grp_end - cc.ck : (cc.r.ntiles - cc.tile) * cc.nck - cc.ck;
            const int grp_rounds = (grp_chunks + RING - 1) / RING;
            const bool last_group = multi ? (cc.tile + 1 == cc.r.ntiles && grp_end == cc.nck) : true;
            // rounds the stash has room for: n rounds from chunk ck of a tile complete at most (ck + n*RING) / nck tiles
            auto stash_room = [&]() { return multi ? STASH_TILES - nstash : ((STASH_TILES - nstash) * cc.nck - cc.ck) / RING; };
            const int n = min(grp_rounds, stash_room()); // >= 1: the stash is flushed below whenever no round fits
            const bool final_round = last_group && n == grp_rounds; // the phase ends with this segment
            const int tag = (p << 8) | (cc.ck / SCK);
            if (st.slab_tag != tag) {
                SlabLoads<10, SCK> L;
                if (!load_slab(cc.ck / SCK, want_scales && cc.idx == 0, spec && cc.idx == 0, L)) return; // first slab of the phase: with the row scales
                st.slab_tag = tag;
                // the whole input has been seen once the first tile's last slab is in; the resets are acknowledged before the rounds start
                if (clears && cc.tile == 0 && (!multi || grp_end == cc.nck)) clear_outputs<T>(P, P.phases[ph.clear_phase], wg, G);
            }
            run_segment(final_round ? n - 1 : n, final_round);
            if (P.timeline && threadIdx.x == 0 && final_round) P.timeline[(size_t)(5 * p + 3) * G + wg] = wall_clock64();
            if (final_round || stash_room() < 1) flush_stash<T>(P, ph, my, nstash, st.es, final_round, sm);
        }
        if (ph.kind == PH_RESID) publish_rowsq(st.es.rowsq, ph.act_dst);
        if (P.timeline && threadIdx.x == 0) P.timeline[(size_t)(5 * p + 4) * G + wg] = wall_clock64();
    }
}

constexpr size_t LDS_BYTES = 160 * 1024;
constexpr size_t ATTN_BYTES = sizeof(AttnSmem<128, MNW>);

// rows the LDS slab can hold (0: use the direct path), the chunks per slab and the size of the slab / attention area
static void smem_plan(int dtype, int rows, bool want_large, int &slab_rows, int &sck, size_t &u_bytes) {
    const size_t planes = dtype ? 2 : 1;
    const size_t avail = LDS_BYTES - sizeof(MegaSmemTail) - 256;
    sck = (want_large && (size_t)rows * planes * slab_pitch(SCK_LARGE) <= avail) ? SCK_LARGE : SCK_SMALL;
    const int max_rows = (int)(avail / (planes * slab_pitch(sck)));
    slab_rows = rows <= max_rows ? rows : 0;
    u_bytes = std::max(ATTN_BYTES, (size_t)slab_rows * planes * slab_pitch(sck));
    u_bytes = (u_bytes + 255) & ~(size_t)255;
}

static const void *mega_fn(int dtype, int sck) {
    if (dtype) return sck == SCK_LARGE ? (const void *)verify_persistent_kernel<bf16_t, SCK_LARGE> : (const void *)verify_persistent_kernel<bf16_t, SCK_SMALL>;
    return sck == SCK_LARGE ? (const void *)verify_persistent_kernel<float, SCK_LARGE> : (const void *)verify_persistent_kernel<float, SCK_SMALL>;
}

static hipError_t ensure_smem_attr(int dtype, int sck) {
    static bool attr_set[2][2] = {{false, false}, {false, false}};
    const int i = dtype ? 1 : 0, j = sck == SCK_LARGE ? 1 : 0;
    if (attr_set[i][j]) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(mega_fn(dtype, sck), hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
    if (e == hipSuccess) attr_set[i][j] = true;
    return e;
}

int mega_max_rows(int dtype) {
    int slab_rows = 0, sck = 0;
    size_t u_bytes = 0;
    for (int rows = 16; rows >= 1; --rows) {
        smem_plan(dtype, rows, false, slab_rows, sck, u_bytes);
        if (slab_rows == rows) return rows;
    }
    return 0;
}

int mega_grid(int dtype, int device) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    const size_t smem = LDS_BYTES - 1024;
    for (int sck : {SCK_SMALL, SCK_LARGE}) { // both variants must fit one workgroup per compute unit
        if (ensure_smem_attr(dtype, sck) != hipSuccess) return 0;
        int per_cu = 0;
        hipError_t e;
        if (dtype) e = sck == SCK_LARGE ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<bf16_t, SCK_LARGE>, MEGA_THREADS, smem)
                                        : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<bf16_t, SCK_SMALL>, MEGA_THREADS, smem);
        else e = sck == SCK_LARGE ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<float, SCK_LARGE>, MEGA_THREADS, smem)
                                  : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<float, SCK_SMALL>, MEGA_THREADS, smem);
        if (e != hipSuccess || per_cu < 1) return 0;
    }
    return prop.multiProcessorCount; // one workgroup per compute unit
}

// One launch of every variant of the kernel with an empty program (a workgroup that finds no phase touches no memory
// and leaves): whatever the runtime sets up at a kernel's first launch (code object, per-lane scratch) then exists
// before a caller freezes allocations, whichever variant its later calls pick.
// Slab trips of a layer's four GEMM phases with either slab size (K in bytes: d_model three times, d_ff once); the
// larger slab moves 1.5 times the bytes per trip.
bool mega_wants_large_slab(int dtype, int d_model, int d_ff) {
    const long esz = dtype ? 2 : 4;
    auto trips = [&](int sck) {
        const long sb = slab_row_bytes(sck);
        return 3 * ((d_model * esz + sb - 1) / sb) + (d_ff * esz + sb - 1) / sb;
    };
    return 3 * trips(SCK_LARGE) < 2 * trips(SCK_SMALL);
}

hipError_t mega_warm(int dtype, hipStream_t st) {
    for (int sck : {SCK_SMALL, SCK_LARGE}) {
        hipError_t e = ensure_smem_attr(dtype, sck);
        if (e != hipSuccess) return e;
        MegaCall c{};
        c.u_bytes = 256;
        void *args[] = {&c};
        e = hipLaunchKernel(mega_fn(dtype, sck), dim3(1), dim3(MEGA_THREADS), args, LDS_BYTES / 2 + 1024, st);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_mega(const MegaCall &call, int grid, hipStream_t st) {
    MegaCall c = call;
    size_t u_bytes;
    int sck;
    smem_plan(c.dtype, std::max(c.R, c.head_rows), c.large_slab != 0, c.slab_rows, sck, u_bytes);
    if (c.slab_rows <= 0) return hipErrorInvalidValue; // the hidden rows must fit the LDS slab (mega_max_rows)
    c.u_bytes = (int)u_bytes;
    void *args[] = {&c};
    const void *fn = mega_fn(call.dtype, sck);
    hipError_t e = ensure_smem_attr(call.dtype, sck);
    if (e != hipSuccess) return e;
    // An ordinary launch: the grid never exceeds the compute units (mega_grid) and a workgroup asks for more than half
    // of a compute unit's LDS, so at most one fits per unit and every workgroup becomes resident as soon as units are
    // free; should another kernel hold units for long, the bounded waits end the launch with the abort flag set
    // instead of hanging.  (A cooperative launch gives the same placement through a separate device queue.)
    const size_t smem = std::max(u_bytes + sizeof(MegaSmemTail), LDS_BYTES / 2 + 1024);
    return hipLaunchKernel(fn, dim3(grid), dim3(MEGA_THREADS), args, smem, st);
}

} // namespace ss
