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
// 8 KB of K per row) into LDS, all loads of the copy in flight together.
#include "attention_core.h"
#include "ss_mega.h"
#include <algorithm>
#include <type_traits>

namespace ss {

constexpr int MNW = MEGA_THREADS / 64; // wavefronts per workgroup
constexpr int CH = 4;                  // 128-byte steps per chunk per wave (8 loads = 8 KB per wave)
constexpr int RING = MEGA_RING;        // chunks in flight per wave (48 KB; the hardware counts at most 63 loads per wave)
constexpr int CHUNK_ROW_BYTES = CH * MNW * 128; // bytes of a weight row one chunk covers (all waves)
constexpr int MAX_SLAB_CK = MEGA_MAX_SLAB_CK; // most chunks an LDS activation slab covers (12 KB of K per row and plane); the launch
                                       // picks MegaCall::slab_ck <= this so that the rows of the call fit the LDS
static_assert(RING + 2 <= MEGA_ROW_WORDS, "a schedule row holds the codes of one round and its action word");
// An LDS slab holds, per hidden row and plane, slab_ck chunks of K = slab_ck * CHUNK_ROW_BYTES bytes, at a pitch padded
// against LDS bank conflicts between rows.
__host__ __device__ constexpr int slab_row_bytes(int slab_ck) { return slab_ck * CHUNK_ROW_BYTES; }
__host__ __device__ constexpr int slab_pitch(int slab_ck) { return slab_ck * CHUNK_ROW_BYTES + 48; }

struct Range {
    int u0, u1, ntiles;
};

// the thread index, opaque to loop-invariant code motion (see thread_index())
__device__ __forceinline__ int tid() { return thread_index(); }

// Phase descriptor i of the program.  The program is written once by the host when the model is created and is read-only
// for every kernel, so it is read through the constant address space: with a uniform index that is a scalar load, which
// the counter of vector memory operations does not see (a vector load here would make the code wait for every weight
// load in flight before it could look at the descriptor).
__device__ __forceinline__ MegaPhase load_phase(const MegaPhase *prog, int i) {
    static_assert(sizeof(MegaPhase) % 4 == 0, "copied word by word");
    typedef const uint32_t __attribute__((address_space(4))) *cptr;
    struct Words {
        uint32_t w[sizeof(MegaPhase) / 4];
    } words;
    cptr src = (cptr)(uintptr_t)(prog + i);
#pragma unroll
    for (size_t j = 0; j < sizeof(MegaPhase) / 4; ++j) words.w[j] = src[j];
    return __builtin_bit_cast(MegaPhase, words);
}

// word `idx` of phase descriptor i's table of schedule offsets (a run-time index into a copy of the descriptor would put the
// copy into scratch memory)
__device__ __forceinline__ int load_sched_off(const MegaPhase *prog, int i, int idx) {
    typedef const int __attribute__((address_space(4))) *cptr;
    return ((cptr)(uintptr_t)(&prog[i].sched_off[0][0]))[idx];
}

// A value that is the same in every lane, said so that the compiler keeps it in a scalar register and
// branches on it with scalar branches (it cannot always prove uniformity through the phase loop).
__device__ __forceinline__ int uni(int x) { return __builtin_amdgcn_readfirstlane(x); }
__device__ __forceinline__ bool uni(bool x) { return __builtin_amdgcn_readfirstlane((int)x) != 0; }

__host__ __device__ __forceinline__ bool is_gemm(int kind) { return kind == PH_QKV || kind == PH_RESID || kind == PH_SWIGLU || kind == PH_HEAD; }

// the share of phase ph owned by workgroup wg: units are tiles (QKV), pairs (SWIGLU) or rows
__host__ __device__ __forceinline__ Range phase_range(const MegaPhase &ph, int wg, int G) {
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

// One round of a phase's chunk schedule (see ss_mega.h), held in scalar registers.
struct Row {
    uint32_t w[MEGA_ROW_WORDS];
};
__device__ __forceinline__ Row load_row(const uint32_t *sched, int off_words) { // the schedule is read-only: scalar loads
    typedef const uint32_t __attribute__((address_space(4))) *cptr;
    cptr src = (cptr)(uintptr_t)(sched + uni(off_words)); // said to be uniform: the loads are scalar, the row lives in scalar registers
    Row r;
#pragma unroll
    for (int j = 0; j < MEGA_ROW_WORDS; ++j) r.w[j] = (uint32_t)uni((int)src[j]);
    return r;
}
__device__ __forceinline__ Row none_row() { // nothing to fetch: every position is padding
    Row r;
#pragma unroll
    for (int j = 0; j < MEGA_ROW_WORDS; ++j) r.w[j] = POS_DUMMY;
    r.w[RING] = ACT_NO_SLAB | ACT_SEG_END | ACT_PHASE_END; // (a consumer that ever ran it would leave its loops at once)
    return r;
}

// Where the weight look-ahead is: the phase its next round belongs to and what it takes to form that phase's addresses.
struct Feed {
    int p;       // program index of the phase the row `nxt` belongs to (-1: before the first)
    int off;     // word offset of that row in the schedule table
    bool active; // `nxt` is a row of phase p's schedule (else: nothing to fetch)
    const char *W;
    int kind, N, kbytes;
    Range rg;
    const char *wp; // this lane's pointer into its weight row of the current tile (+ its wave / lane-group offset)
    bool live;      // the lane's A-row exists
};

// Issue the 2*CH weight loads of the position `code` of the look-ahead's phase.  Every call issues exactly 2*CH loads,
// whatever the position is (real, padding, dead row, K tail): positions without data read a small zero-filled buffer
// instead.  A fixed number of loads per step is what lets the compiler wait for one ring slot with an exact vmcnt(N)
// and leave the younger slots in flight; a conditional load would force vmcnt(0).
__device__ __forceinline__ void issue_chunk(Feed &f, uint32_t code, int hd, const char *zeros, u32x4 (&wbuf)[2 * CH]) {
    const int t = tid(), lane = t & 63, wave = t >> 6, cc = lane & 15, g = lane >> 4;
    if (uni((code & POS_FIRST) != 0)) { // a new tile: this lane's weight row
        const int row = a_row(f.kind, f.N, f.rg, hd, (int)((code >> 8) & 0xfffu), cc, f.live);
        f.wp = f.W + (size_t)row * f.kbytes + wave * 128 + g * 16;
    }
    const int ck = (int)(code & 0xffu);
    const bool real = f.active && !(code & POS_DUMMY) && f.live;
    const char *base = f.wp + (size_t)ck * CHUNK_ROW_BYTES;
    const int kb0 = ck * CHUNK_ROW_BYTES + wave * 128 + g * 16;
#pragma unroll
    for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int off = i * (MNW * 128) + j * 64;
            const char *a = (real && kb0 + off < f.kbytes) ? base + off : zeros;
            wbuf[2 * i + j] = ld16_global(a);
        }
}

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
    if (tid() == 0) __hip_atomic_store(&P.arrive[blockIdx.x], epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ bool grid_wait(const MegaCall &P, unsigned epoch, int lo, int hi, MegaSmem &sm) { // slots lo .. hi-1
    if (tid() < 64) {
        bool ok = true;
        unsigned spins = 0;
        for (;;) {
            bool all = true;
            for (int i = lo + (int)tid(); i < hi; i += 64) {
                const unsigned v = __hip_atomic_load(&P.arrive[i], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((int)(v - epoch) < 0) all = false;
            }
            if (__all(all)) break;
            if (++spins > P.spin_limit || __hip_atomic_load(P.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
                ok = false;
                break;
            }
        }
        if (tid() == 0) {
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
    if (tid() < 64) {
        const int tph = P.hd / 16, units = 3 * P.H * tph; // QKV tiles per head and region, and in total
        bool ok = true;
        unsigned spins = 0;
        for (;;) {
            bool all = true;
            for (int region = 0; region < 3; ++region) {
                const int t_lo = (region * P.H + h) * tph, t_hi = t_lo + tph - 1;
                // owner of tile t under the static split u0(wg) = floor(wg * units / G)
                const int w_lo = (int)(((long long)(t_lo + 1) * G - 1) / units), w_hi = (int)(((long long)(t_hi + 1) * G - 1) / units);
                for (int i = w_lo + (int)tid(); i <= w_hi; i += 64) {
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
        if (tid() == 0) {
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
    const int r = tid() & 15;
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
    for (int e = c0 + (int)(tid() >> 4); e < c1; e += MEGA_THREADS / 16) {
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
            if (tid() == 0) {
                const unsigned old = __hip_atomic_fetch_add(&P.attn_cnt[bh], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                sm.t->flag = old == (unsigned)(P.nsplit - 1);
            }
            __syncthreads();
            merge = sm.t->flag != 0;
        }
        if (merge) {
            for (int idx = tid(); idx < P.M * HD; idx += MEGA_THREADS) {
                const int c = idx / HD, e = idx - c * HD, row = b * P.M + c;
                store_act_coh(out, (size_t)row * a.ld_out + h * HD + e, attn_merge_elem<true>(a, row, h, e));
            }
            if (P.nsplit > 1 && tid() == 0) __hip_atomic_store(&P.attn_cnt[bh], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
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
    row = (tid() >> 5) + half * (MEGA_THREADS / 32);
    i = (tid() & 31) + 32 * q;
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
    const int j = tid() & 31;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
        const int row = (tid() >> 5) + half * (MEGA_THREADS / 32);
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
constexpr int SLAB_UNITS = MAX_SLAB_CK * CHUNK_ROW_BYTES / 16 / MEGA_THREADS; // 16-byte units per thread and slab row (the largest slab)
constexpr int SLAB_BATCH = 10; // (plane, row) pairs per validation mask
static_assert(SLAB_BATCH * SLAB_UNITS <= 32, "one mask bit per unit of a batch");

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

// One 16-byte agent-coherent load per lane (sc0 sc1: performed at the memory side, like ld16_coh_buf) that the memory
// system writes straight into LDS, lane l at lds_wave_base + 16 l: no registers hold the slab.
__device__ __forceinline__ void dma16_coh(const void *src, unsigned char *lds_wave_base) {
    typedef const void __attribute__((address_space(1))) *gptr;
    typedef void __attribute__((address_space(3))) *lptr;
    __builtin_amdgcn_global_load_lds((gptr)src, (lptr)lds_wave_base, 16, 0, 1 | 16);
}
// The 16-byte units of K slab `slab` that this thread handles for the hidden rows r0 .. r0 + SLAB_BATCH / PLANES - 1 (a
// "batch": at most 32 units, one mask bit each).  A slab row is a whole number of 1 KB wave instructions; thread t takes
// unit t + h2 * threads of every (plane, row) pair.  f(bit, valid, byte offset of the unit in the source planes - clamped
// to a valid address when the unit holds no data (row without data, K tail) -, the unit's place in LDS, the LDS base of the
// wave instruction that carries it); valid false: the unit holds no data and counts as zeros.
// (Written without divisions and with the row loop unrolled: this runs at every phase boundary.)
template <typename T, typename F>
__device__ __forceinline__ void slab_units(const MegaCall &P, const MegaPhase &ph, int slab, int r0, MegaSmem &sm, F f) {
    constexpr int PL = Traits<T>::PLANES, BR = SLAB_BATCH / PL, PER16 = 16 / (int)sizeof(T);
    const ActPlanes<T> src = act_planes<T>(P, ph.act_src);
    const bool head = ph.kind == PH_HEAD;
    const int nlive = head ? P.head_rows : P.R;
    const int t = tid(), wave = t >> 6;
    const int srb = slab_row_bytes(P.slab_ck), pitch = slab_pitch(P.slab_ck);
    const int kslab = slab * (srb / (int)sizeof(T));
#pragma unroll
    for (int rr = 0; rr < BR; ++rr) {
        const int r = r0 + rr;
        if (r < P.slab_rows) {
            const int rc = min(r, nlive - 1);
            const int brow = head ? P.head_row0 + rc * P.head_stride : rc;
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                for (int h2 = 0; h2 < SLAB_UNITS; ++h2)
                    if ((wave * 64 + h2 * MEGA_THREADS) * 16 < srb) { // the wave's instruction h2 lies inside the slab row
                        const int x = t + h2 * MEGA_THREADS, k = kslab + x * PER16; // K is a multiple of the unit
                        const bool valid = r < nlive && k < ph.K;
                        const uint32_t off = (uint32_t)((pl * src.plane + (size_t)brow * src.ld + (k < ph.K ? k : 0)) * sizeof(T));
                        unsigned char *row_lds = sm.u + (size_t)(pl * P.slab_rows + r) * pitch;
                        f((rr * PL + pl) * SLAB_UNITS + h2, valid, off, row_lds + x * 16, row_lds + (wave * 64 + h2 * MEGA_THREADS) * 16);
                    }
        }
    }
}
constexpr int slab_batch_rows(int planes) { return SLAB_BATCH / planes; }
// All loads of K slab `slab` (with_scales: and of the row scales, into registers), unconditionally and straight into LDS.
// The caller has made sure that nobody still reads the LDS area.
template <typename T>
__device__ __forceinline__ void slab_issue(const MegaCall &P, const MegaPhase &ph, int slab, int G, bool with_scales, ScaleLoads &sl, MegaSmem &sm) {
    const char *base = reinterpret_cast<const char *>(act_planes<T>(P, ph.act_src).base);
    if (with_scales) scales_issue(P, nsq_set(P, ph.act_src, G), G, false, sl);
    for (int r0 = 0; r0 < P.slab_rows; r0 += slab_batch_rows(Traits<T>::PLANES))
        slab_units<T>(P, ph, slab, r0, sm, [&](int, bool, uint32_t off, unsigned char *, unsigned char *wave_lds) { dma16_coh(base + off, wave_lds); });
}
// Looks at what has arrived in LDS: a bit of the result is set when this thread's unit of that number still shows the
// "not written yet" pattern.  Units without data are ignored (and zeroed when `finish` is set: call it that way once,
// after the first load has landed).  The units of a hidden row are read together, then judged, so that the LDS
// latency is paid once per row and not once per unit.
template <typename T>
__device__ __forceinline__ uint32_t slab_look(const MegaCall &P, const MegaPhase &ph, int slab, int r0, bool finish, MegaSmem &sm) {
    constexpr int PL = Traits<T>::PLANES, BR = SLAB_BATCH / PL, PER16 = 16 / (int)sizeof(T), NU = PL * SLAB_UNITS;
    const int nlive = ph.kind == PH_HEAD ? P.head_rows : P.R;
    const int t = tid(), wave = t >> 6;
    const int srb = slab_row_bytes(P.slab_ck), pitch = slab_pitch(P.slab_ck);
    const int kslab = slab * (srb / (int)sizeof(T));
    uint32_t mask = 0;
#pragma unroll
    for (int rr = 0; rr < BR; ++rr) {
        const int r = r0 + rr;
        if (r < P.slab_rows) {
            u32x4 v[NU];
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                for (int h2 = 0; h2 < SLAB_UNITS; ++h2) { // (a unit outside the slab row reads the thread's first unit instead)
                    const bool in = (wave * 64 + h2 * MEGA_THREADS) * 16 < srb;
                    v[pl * SLAB_UNITS + h2] = *reinterpret_cast<const u32x4 *>(sm.u + (size_t)(pl * P.slab_rows + r) * pitch + (t + (in ? h2 : 0) * MEGA_THREADS) * 16);
                }
#pragma unroll
            for (int pl = 0; pl < PL; ++pl)
#pragma unroll
                for (int h2 = 0; h2 < SLAB_UNITS; ++h2) {
                    const bool in = (wave * 64 + h2 * MEGA_THREADS) * 16 < srb;
                    const int x = t + h2 * MEGA_THREADS, k = kslab + x * PER16;
                    const bool valid = r < nlive && k < ph.K;
                    if (in && valid && unit_unset<T>(v[pl * SLAB_UNITS + h2])) mask |= 1u << ((rr * PL + pl) * SLAB_UNITS + h2);
                    if (in && !valid && finish) *reinterpret_cast<u32x4 *>(sm.u + (size_t)(pl * P.slab_rows + r) * pitch + x * 16) = zero16();
                }
        }
    }
    return mask;
}
__device__ __forceinline__ bool scales_unset(const MegaCall &P, int G, const ScaleLoads &sl) {
    uint32_t ms = 0;
#pragma unroll
    for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            int row, i;
            ms = unset_acc<float>(ms, scale_slot(P, G, half, q, row, i) ? f2u(sl.t[half][q]) : 0u);
        }
    return unset_seen<float>(ms);
}
// After a first look found the pattern: wait (bounded) until nothing this wave loaded shows it, loading again what does.
// false: gave up (the caller raises the abort flag).
template <typename T>
__device__ __forceinline__ bool slab_retry(const MegaCall &P, const MegaPhase &ph, int slab, int r0, int G, bool with_scales, uint32_t mask,
                                           ScaleLoads &sl, MegaSmem &sm, unsigned long long *tl_spins = nullptr) {
    const char *base = reinterpret_cast<const char *>(act_planes<T>(P, ph.act_src).base);
    for (unsigned spins = 0; spins < P.spin_limit; ++spins) {
        const unsigned aborted = __hip_atomic_load(P.abort_flag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); // rides with the loads below: one round trip
        if (with_scales) scales_issue(P, nsq_set(P, ph.act_src, G), G, true, sl);
        slab_units<T>(P, ph, slab, r0, sm, [&](int bit, bool, uint32_t off, unsigned char *, unsigned char *wave_lds) {
            if (__any((mask >> bit & 1u) != 0u)) dma16_coh(base + off, wave_lds); // a wave instruction with a missing unit is issued again as a whole
        });
        stores_done(); // the loads have landed in LDS (and in the registers of the scales)
        if (aborted != 0u) return false;
        mask = slab_look<T>(P, ph, slab, r0, false, sm);
        if (!__any(mask != 0u || (with_scales && scales_unset(P, G, sl)))) {
            if (tl_spins) *tl_spins = spins + 1;
            return true;
        }
    }
    return false;
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
        for (int idx = tid(); idx < n; idx += MEGA_THREADS) {
            const int col = r.u0 + idx % ncol, rest = idx / ncol, row = rest % P.R, pl = rest / P.R;
            store_unset(a.base + pl * a.plane + (size_t)row * a.ld + col);
        }
        if (tp.kind == PH_RESID && tid() < 16) store_unset(&nsq_set(P, tp.act_dst, G)[(size_t)tid() * G + wg]);
    } else if (tp.kind == PH_ATTN) {
        const ActPlanes<T> o = act_planes<T>(P, ACT_O);
        const int units = P.B * P.H * P.nsplit, n = P.M * P.hd * PL;
        for (int u = wg; u < units; u += G) {
            if (u % P.nsplit != 0) continue; // one of the splits of (sequence, head) does it
            const int bh = u / P.nsplit, h = bh % P.H, b = bh / P.H;
            for (int idx = tid(); idx < n; idx += MEGA_THREADS) {
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
    const int c = tid() & 15, i = tid() >> 4;
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

// multiply a chunk (weights in wbuf; sck = its index inside the LDS slab) into the tile accumulators; the B operand
// comes from the LDS slab.  Lanes whose hidden row does not exist read the last row that does (their output columns
// are never looked at), so no LDS read is conditional.
template <typename T>
__device__ __forceinline__ void mma_chunk(int sck, const MegaCall &P, const u32x4 (&wbuf)[2 * CH], f32x4 &acc0, f32x4 &acc1, MegaSmem &sm) {
    constexpr int PL = Traits<T>::PLANES;
    const int t = tid(), lane = t & 63, wave = t >> 6, cc = min(lane & 15, P.slab_rows - 1), g = lane >> 4;
    const unsigned char *lb = sm.u + (size_t)cc * slab_pitch(P.slab_ck) + sck * CHUNK_ROW_BYTES + wave * 128 + g * 16;
    const size_t plane_off = (size_t)P.slab_rows * slab_pitch(P.slab_ck);
#pragma unroll
    for (int i = 0; i < CH; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            Act<T> av;
#pragma unroll
            for (int pl = 0; pl < PL; ++pl) av.p[pl] = *reinterpret_cast<const u32x4 *>(lb + pl * plane_off + i * (MNW * 128) + j * 64);
            mma2(acc0, acc1, wbuf[2 * i + j], av, j);
        }
}

// Tile complete: fixed-order sum of the waves' partial tiles by waves 0-3 (register v = wave) into the
// LDS stash.  No global memory is touched here: the epilogues (and their stores) run at flush time,
// outside the chunk loop, because on this ISA a pending store would force every later wait on a
// weight load to vmcnt(0) (loads and stores share the counter and may complete out of order).
__device__ __forceinline__ void finish_tile(int tile, const f32x4 &acc0, const f32x4 &acc1, int &tile_seq, int &nstash,
                                            MegaSmem &sm) {
    const int lane = tid() & 63, wave = tid() >> 6;
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
        if (tid() == 0) sm.t->stash_tile[nstash] = tile;
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
    const int c = tid() & 15, ii = tid() >> 4;
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

template <typename T>
__global__ __launch_bounds__(MEGA_THREADS) void verify_persistent_kernel(MegaCall P) {
    extern __shared__ __align__(16) unsigned char smem_raw[];
    MegaSmem sm;
    sm.u = smem_raw;
    sm.t = reinterpret_cast<MegaSmemTail *>(smem_raw + P.u_bytes);
    const int wg = uni((int)blockIdx.x), G = uni((int)gridDim.x);
    const int lane = tid() & 63, wave = tid() >> 6;
    if (tid() < 16) sm.t->len[tid()] = (int)tid() < P.B ? P.len[tid()] : 0; // lengths change in the last phase only
    if (tid() == 0) sm.t->ok = 1;
    lds_barrier();

    // Weight pipeline.  The workgroup's chunk positions over all its GEMM phases form one sequence, cut into rounds of
    // RING positions (the phases' schedules, built by the host).  `cur` is the round being multiplied, `nxt` the one
    // after it - possibly the first round of the next GEMM phase: weights depend on nothing.  A step multiplies
    // straight out of its ring slot (which waits for that slot's loads only - later slots stay in flight), then
    // refills the slot with the same position of `nxt`.  So while a phase's epilogue runs and the next phase's input
    // is awaited, the first RING chunks of that phase (48 KB per wave, 192 KB per compute unit) keep the memory
    // system busy, and the O projection's whole share arrives during the attention phase.
    f32x4 acc0 = f32x4{0.f, 0.f, 0.f, 0.f}, acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
    int tile_seq = 0;
    EpiState es;
    es.rowsq = 0.f;
    es.pre = false;
    es.h_pre = 0.f;
    es.g_pre = 1.f;

    u32x4 ring[RING][2 * CH]; // only ever indexed by unrolled constants: lives in registers
    static_assert(MNW >= 4, "waves 0-3 reduce one accumulator register each");
    static_assert(RING * 2 * CH <= 63, "the hardware counts at most 63 vector memory operations in flight per wave");

    const char *zeros = reinterpret_cast<const char *>(P.zeros);
    Feed fd;
    fd.p = -1;
    fd.off = 0;
    fd.active = false;
    fd.W = nullptr;
    fd.kind = PH_LEN;
    fd.N = 0;
    fd.kbytes = 0;
    fd.rg = Range{0, 0, 0};
    fd.wp = zeros;
    fd.live = false;
    Row cur = none_row(), nxt = none_row();
    // `nxt` becomes the round behind it: the next row of its phase's schedule, or the first row of this workgroup's next
    // GEMM phase with work (none left: a row of padding)
    auto advance = [&]() {
        if (uni(fd.active && !(nxt.w[RING] & ACT_PHASE_END))) {
            fd.off = uni(fd.off + MEGA_ROW_WORDS);
            nxt = load_row(P.sched, fd.off);
            return;
        }
        fd.active = false;
        nxt = none_row();
        for (;;) {
            fd.p = uni(fd.p);
            if (fd.p + 1 >= P.n_phases) break;
            const MegaPhase nph = load_phase(P.phases, fd.p + 1);
            ++fd.p;
            if (!uni(is_gemm(nph.kind))) continue;
            const Range rg = phase_range(nph, wg, G);
            if (uni(rg.ntiles <= 0)) continue;
            const int variant = rg.ntiles - nph.ntiles_lo; // shares differ by at most one tile
            if (uni(variant < 0 || variant > 1)) continue;
            const int off = uni(load_sched_off(P.phases, fd.p, 2 * (P.slab_ck - MEGA_MIN_SLAB_CK) + variant));
            if (off < 0) continue;
            fd.active = true;
            fd.W = reinterpret_cast<const char *>(nph.W);
            fd.kind = nph.kind;
            fd.N = nph.N;
            fd.kbytes = nph.K * (int)sizeof(T);
            fd.rg = Range{uni(rg.u0), uni(rg.u1), uni(rg.ntiles)};
            fd.off = off;
            nxt = load_row(P.sched, fd.off);
            return;
        }
    };
    // The empty asm statements are compiler barriers: they pin the slot's loads to this point of the
    // program.  Without them the scheduler sinks each load next to its use (to shorten live ranges),
    // which would leave one 16-byte load in flight per wave instead of a ring of chunks.
    auto fill = [&](u32x4(&slot)[2 * CH], uint32_t code) { // always 2*CH loads
        asm volatile("" ::: "memory");
        issue_chunk(fd, code, P.hd, zeros, slot);
        asm volatile("" ::: "memory");
    };
    // `cur` = the first round of the look-ahead's phase, its loads issued; `nxt` = the round behind it
    auto prime_ring = [&]() {
        advance();
        cur = nxt;
#pragma unroll
        for (int sl = 0; sl < RING; ++sl) fill(ring[sl], cur.w[sl]);
        advance();
    };
    prime_ring(); // the first RING chunks of the first GEMM phase: nothing to wait for

    for (int p = 0; p < P.n_phases; ++p) {
        const MegaPhase ph = load_phase(P.phases, uni(p));
        // Phase boundary.  The ring already holds the first RING chunks of this workgroup's next GEMM phase.
        const Range my = is_gemm(ph.kind) ? phase_range(ph, wg, G) : Range{0, 0, 0}; // this workgroup's share of the phase
        const bool work = my.ntiles > 0;
        const unsigned epoch = P.epoch_base + (unsigned)p;
        const int attn_units = P.B * P.H * P.nsplit;
        const bool want_scales = ph.kind == PH_QKV || ph.kind == PH_SWIGLU || ph.kind == PH_HEAD;
        // How this phase's input becomes visible.  Flags: the producers wait for their stores, publish
        // their epoch, and the consumer polls the epochs before it loads anything.  Data: nobody waits
        // for acknowledgements; the consumer loads the first slab at once and validates it (slab_look,
        // slab_retry).  After the attention phase the workgroups without
        // a unit would find nothing for a long time, so they first wait for the units' epochs (a hint:
        // the data is validated all the same).
        const bool polled = P.data_sync && ph.sync != SYNC_FLAGS && work;
        const bool hint_first = polled && ph.sync == SYNC_DATA_ATTN && wg >= attn_units;
        const bool spec = polled && !hint_first;
        const int t = tid(), lane = t & 63, wave = t >> 6;
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
            if (t < 16) {
                float tot = 0.f;
#pragma unroll
                for (int w2 = 0; w2 < MNW; ++w2) tot += sm.t->sq[w2][t];
                st_coh(&nsq_set(P, act_dst, G)[(size_t)t * G + wg], f2u(tot) == 0xffffffffu ? u2f(0xffc00000u) : tot); // the all-ones pattern is reserved
            }
        };
        int nstash = 0;
        // One K slab of the B operand into LDS: all its loads in flight together (one memory round trip), straight into
        // LDS; then, with data synchronisation, a look at what arrived and more loads for whatever is still missing.
        // false: a bounded wait for the data ran out (every wave of the workgroup returns the same).
        auto load_slab = [&](int slab, bool scales) __attribute__((always_inline)) {
            bool ok = true;
            ScaleLoads sl;
            // Loads return to a wave in the order it issued them, so a slab requested now would come back behind the weight
            // chunks in flight - late, and showing memory as it was when the request went out.  The wave lets its ring land
            // first (those bytes are this phase's first rounds: the wait is streaming time, not idle time) and asks then.
            stores_done();
            lds_barrier(); // every wave is done with the previous slab (or with the attention area, which it aliases)
            slab_issue<T>(P, ph, slab, G, scales, sl, sm);
            stores_done();
            if (P.timeline && t == 0 && scales) P.timeline[(size_t)(MEGA_TL_SLOTS * p + 1) * G + wg] = wall_clock64();
            for (int pr0 = 0; pr0 < P.slab_rows; pr0 += slab_batch_rows(Traits<T>::PLANES)) { // batches of hidden rows
                const bool sc = scales && pr0 == 0;
                const uint32_t mask = slab_look<T>(P, ph, slab, pr0, true, sm); // units without data become zeros
                if (P.timeline && t == 0 && scales && pr0 == 0) P.timeline[(size_t)(MEGA_TL_SLOTS * p + 5) * G + wg] = wall_clock64(); // first look done
                if (polled && ok && __any(mask != 0u || (sc && scales_unset(P, G, sl))))
                    ok = slab_retry<T>(P, ph, slab, pr0, G, sc, mask, sl, sm, (P.timeline && t == 0 && scales) ? &P.timeline[(size_t)(MEGA_TL_SLOTS * p + 6) * G + wg] : nullptr);
            }
            if (scales) scales_finish(P, nsq_set(P, ph.act_src, G), G, sl, sm);
            if (!ok && lane == 0) {
                sm.t->ok = 0;
                __hip_atomic_store(P.abort_flag, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            if (P.timeline && t == 0 && scales) P.timeline[(size_t)(MEGA_TL_SLOTS * p + 2) * G + wg] = wall_clock64();
            lds_barrier();
            return sm.t->ok != 0;
        };
        const bool clears = P.data_sync && ph.clear_phase >= 0;
        es.rowsq = 0.f;
        if (!work) {
            // No GEMM work in this phase (embedding, attention, length update, or no share of a small GEMM): the ring
            // keeps the chunks of the next GEMM phase, which arrive meanwhile.
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
            if (P.timeline && t == 0) P.timeline[(size_t)(MEGA_TL_SLOTS * p) * G + wg] = wall_clock64();
            switch (ph.kind) {
            case PH_EMBED:
                if (clears) clear_outputs<T>(P, load_phase(P.phases, uni(ph.clear_phase)), wg, G);
                publish_rowsq(do_embed<T>(P, ph, wg, G), ACT_A);
                break;
            case PH_ATTN: // (the ring stays live across it: the O projection's chunks arrive meanwhile)
                do_attn<T>(P, ph, wg, G, sm);
                break;
            case PH_LEN:
                if (wg == 0 && t < P.B) P.len[t] += P.M;
                break;
            case PH_RESID: // no share of the new hidden rows: this workgroup's partial sums of squares are zero
                if (t < 16) st_coh(&nsq_set(P, ph.act_dst, G)[(size_t)t * G + wg], 0.f);
                break;
            default: break;
            }
            if (P.timeline && t == 0) {
                P.timeline[(size_t)(MEGA_TL_SLOTS * p + 1) * G + wg] = wall_clock64();
                P.timeline[(size_t)(MEGA_TL_SLOTS * p + 4) * G + wg] = wall_clock64();
            }
            continue;
        }
        // GEMM phase with work: the first slab is loaded (and, with data synchronisation, validated) by its first segment
        epi_prefetch(P, ph, my, es);
        if (p > 0 && !spec) {
            if (hint_first ? !grid_wait(P, epoch, 0, min(attn_units, G), sm) : !grid_wait(P, epoch, 0, G, sm)) return;
        }
        if (P.timeline && t == 0) P.timeline[(size_t)(MEGA_TL_SLOTS * p) * G + wg] = wall_clock64();
        bool first_segment = true;
        for (;;) {
            // One segment: rounds that share an LDS slab and fit the stash.  Its loop holds no global memory operation
            // except the pinned ring loads (the schedule is read with scalar loads), and nothing else is pending when
            // it starts; both are what lets the compiler wait for one slot with an exact count and leave the younger
            // slots in flight.
            const uint32_t act0 = cur.w[RING];
            if (uni((act0 & 0xffu) != ACT_NO_SLAB)) {
                if (!load_slab((int)(act0 & 0xffu), want_scales && first_segment)) return; // first slab of the phase: with the row scales
                // the whole input has been seen once the first tile's last slab is in; the resets are acknowledged before the rounds start
                if (clears && (act0 & ACT_CLEAR)) clear_outputs<T>(P, load_phase(P.phases, uni(ph.clear_phase)), wg, G);
            }
            first_segment = false;
            stores_done();
            uint32_t act;
            do {
                act = cur.w[RING];
#pragma unroll
                for (int sl = 0; sl < RING; ++sl) {
                    const uint32_t code = cur.w[sl];
                    const bool real = uni(!(code & POS_DUMMY));
                    if (real) {
                        if (uni((code & POS_FIRST) != 0)) {
                            acc0 = f32x4{0.f, 0.f, 0.f, 0.f};
                            acc1 = f32x4{0.f, 0.f, 0.f, 0.f};
                        }
                        mma_chunk<T>((int)((code >> 20) & 7u), P, ring[sl], acc0, acc1, sm);
                    }
                    fill(ring[sl], nxt.w[sl]);
                    if (uni(real && (code & POS_LAST))) finish_tile((int)((code >> 8) & 0xfffu), acc0, acc1, tile_seq, nstash, sm);
                }
                cur = nxt;
                advance();
            } while (uni(!(act & ACT_SEG_END)));
            const bool phase_end = (act & ACT_PHASE_END) != 0;
            if (P.timeline && t == 0 && phase_end) P.timeline[(size_t)(MEGA_TL_SLOTS * p + 3) * G + wg] = wall_clock64();
            if (act & ACT_FLUSH) flush_stash<T>(P, ph, my, nstash, es, phase_end, sm);
            if (phase_end) break;
        }
        if (ph.kind == PH_RESID) publish_rowsq(es.rowsq, ph.act_dst);
        if (P.timeline && t == 0) P.timeline[(size_t)(MEGA_TL_SLOTS * p + 4) * G + wg] = wall_clock64();
    }
}

// ---------------------------------------------------------------- host: chunk schedules

// The schedule of one GEMM phase shape for a share of `ntiles` tiles and `slab_ck` chunks per LDS slab (format: ss_mega.h).
static void build_schedule(int K, int esz, int ntiles, int slab_ck, std::vector<uint32_t> &out) {
    const int nck = (K * esz + CHUNK_ROW_BYTES - 1) / CHUNK_ROW_BYTES; // chunks per tile
    const bool multi = nck > slab_ck; // K spans several LDS slabs: a tile's chunks come in slab groups
    struct Pos {
        uint32_t code;
        int slab;       // K slab the position multiplies with
        bool first_of_group;
    };
    std::vector<Pos> pos;
    auto pad = [&]() {
        while (pos.size() % RING) pos.push_back(Pos{POS_DUMMY, -1, false});
    };
    for (int tile = 0; tile < ntiles; ++tile)
        for (int ck = 0; ck < nck; ++ck) {
            const int slab = multi ? ck / slab_ck : 0, sck = multi ? ck % slab_ck : ck;
            const bool group_start = multi ? sck == 0 : (tile == 0 && ck == 0);
            if (group_start) pad(); // a slab group starts a round
            uint32_t code = (uint32_t)ck | ((uint32_t)tile << 8) | ((uint32_t)sck << 20);
            if (ck == 0) code |= POS_FIRST;
            if (ck == nck - 1) code |= POS_LAST;
            pos.push_back(Pos{code, slab, group_start});
        }
    pad();
    const int nrounds = (int)pos.size() / RING;
    std::vector<uint32_t> action(nrounds, ACT_NO_SLAB);
    int nstash = 0;
    for (int r = 0; r < nrounds; ++r) {
        const Pos &p0 = pos[(size_t)r * RING];
        int completes = 0;
        bool last_slab_of_first_tile = false;
        for (int sl = 0; sl < RING; ++sl) {
            const Pos &q = pos[(size_t)r * RING + sl];
            if (!(q.code & POS_DUMMY) && (q.code & POS_LAST)) ++completes;
        }
        if (p0.first_of_group) { // the round starts a slab group: the segment before it ends, the slab is loaded
            if (r > 0) action[r - 1] |= ACT_SEG_END;
            action[r] = (action[r] & ~0xffu) | (uint32_t)p0.slab;
            const int tile = (int)((p0.code >> 8) & 0xfffu);
            last_slab_of_first_tile = tile == 0 && (!multi || (p0.slab + 1) * slab_ck >= nck);
            if (last_slab_of_first_tile) action[r] |= ACT_CLEAR; // from here on the whole input of the phase has been seen
        }
        if (nstash + completes > STASH_TILES) { // the stash cannot take this round's tiles: flush behind the previous round
            action[r - 1] |= ACT_SEG_END | ACT_FLUSH;
            nstash = 0;
        }
        nstash += completes;
    }
    action[nrounds - 1] |= ACT_SEG_END | ACT_FLUSH | ACT_PHASE_END;
    for (int r = 0; r < nrounds; ++r) {
        for (int sl = 0; sl < RING; ++sl) out.push_back(pos[(size_t)r * RING + sl].code);
        out.push_back(action[r]);
        for (int j = RING + 1; j < MEGA_ROW_WORDS; ++j) out.push_back(0u);
    }
}

std::vector<uint32_t> mega_build_schedules(std::vector<MegaPhase> &prog, int grid, int dtype, int head_dim) {
    (void)head_dim;
    const int esz = dtype ? 2 : 4;
    std::vector<uint32_t> table;
    struct Key {
        int kind, N, K;
        int ntiles_lo, off[MEGA_MAX_SLAB_CK - MEGA_MIN_SLAB_CK + 1][2];
    };
    std::vector<Key> done;
    for (MegaPhase &ph : prog) {
        if (!is_gemm(ph.kind)) continue;
        const Key *hit = nullptr;
        for (const Key &k : done)
            if (k.kind == ph.kind && k.N == ph.N && k.K == ph.K) hit = &k;
        if (!hit) {
            Key k{};
            k.kind = ph.kind; k.N = ph.N; k.K = ph.K;
            int lo = 1 << 30, hi = 0;
            for (int wg = 0; wg < grid; ++wg) {
                const int nt = phase_range(ph, wg, grid).ntiles;
                if (nt > 0) lo = std::min(lo, nt);
                hi = std::max(hi, nt);
            }
            if (hi == 0) lo = 1; // nobody has a share (cannot happen for N >= 1)
            k.ntiles_lo = lo;
            // shares differ by at most one unit, hence by at most one tile
            for (int i = 0; i <= MEGA_MAX_SLAB_CK - MEGA_MIN_SLAB_CK; ++i)
                for (int j = 0; j < 2; ++j) {
                    k.off[i][j] = -1;
                    if (lo + j > hi) continue;
                    k.off[i][j] = (int)table.size();
                    build_schedule(ph.K, esz, lo + j, MEGA_MIN_SLAB_CK + i, table);
                }
            done.push_back(k);
            hit = &done.back();
        }
        ph.ntiles_lo = hit->ntiles_lo;
        for (int i = 0; i <= MEGA_MAX_SLAB_CK - MEGA_MIN_SLAB_CK; ++i)
            for (int j = 0; j < 2; ++j) ph.sched_off[i][j] = hit->off[i][j];
    }
    if (table.empty()) table.push_back(0u);
    return table;
}

constexpr size_t LDS_BYTES = 160 * 1024;
constexpr size_t ATTN_BYTES = sizeof(AttnSmem<128, MNW>);

// chunks of K per LDS slab for a call of `rows` hidden rows (0: the rows do not fit) and the size of the slab / attention area
static void smem_plan(int dtype, int rows, int &slab_ck, size_t &u_bytes) {
    const size_t planes = dtype ? 2 : 1;
    const size_t avail = LDS_BYTES - sizeof(MegaSmemTail) - 256;
    slab_ck = 0;
    for (int ck = MAX_SLAB_CK; ck >= 1; --ck) {
        if ((size_t)rows * planes * slab_pitch(ck) <= avail && ck >= MEGA_MIN_SLAB_CK) { // (schedules exist for these sizes)
            slab_ck = ck;
            break;
        }
    }
    u_bytes = std::max(ATTN_BYTES, (size_t)rows * planes * slab_pitch(std::max(slab_ck, 1)));
    u_bytes = (u_bytes + 255) & ~(size_t)255;
}

static hipError_t ensure_smem_attr(int dtype) {
    static bool attr_set[2] = {false, false};
    const int i = dtype ? 1 : 0;
    if (attr_set[i]) return hipSuccess;
    const void *fn = dtype ? (const void *)verify_persistent_kernel<bf16_t> : (const void *)verify_persistent_kernel<float>;
    hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS_BYTES);
    if (e == hipSuccess) attr_set[i] = true;
    return e;
}

int mega_max_rows(int dtype) {
    int slab_ck = 0;
    size_t u_bytes = 0;
    for (int rows = 16; rows >= 1; --rows) {
        smem_plan(dtype, rows, slab_ck, u_bytes);
        if (slab_ck > 0) return rows;
    }
    return 0;
}

int mega_grid(int dtype, int device) {
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, device) != hipSuccess) return 0;
    if (ensure_smem_attr(dtype) != hipSuccess) return 0;
    int per_cu = 0;
    const size_t smem = LDS_BYTES - 1024;
    hipError_t e = dtype ? hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<bf16_t>, MEGA_THREADS, smem)
                         : hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, verify_persistent_kernel<float>, MEGA_THREADS, smem);
    if (e != hipSuccess || per_cu < 1) return 0;
    return prop.multiProcessorCount; // one workgroup per compute unit
}

hipError_t launch_mega(const MegaCall &call, int grid, hipStream_t st) {
    MegaCall c = call;
    size_t u_bytes;
    c.slab_rows = std::max(c.R, c.head_rows);
    smem_plan(c.dtype, c.slab_rows, c.slab_ck, u_bytes);
    if (c.slab_ck <= 0) return hipErrorInvalidValue; // the hidden rows must fit the LDS slab (mega_max_rows)
    c.u_bytes = (int)u_bytes;
    void *args[] = {&c};
    const void *fn = call.dtype ? (const void *)verify_persistent_kernel<bf16_t> : (const void *)verify_persistent_kernel<float>;
    hipError_t e = ensure_smem_attr(call.dtype);
    if (e != hipSuccess) return e;
    // An ordinary launch: the grid never exceeds the compute units (mega_grid) and a workgroup asks for more than half
    // of a compute unit's LDS, so at most one fits per unit and every workgroup becomes resident as soon as units are
    // free; should another kernel hold units for long, the bounded waits end the launch with the abort flag set
    // instead of hanging.  (A cooperative launch gives the same placement through a separate device queue.)
    const size_t smem = std::max(u_bytes + sizeof(MegaSmemTail), LDS_BYTES / 2 + 1024);
    return hipLaunchKernel(fn, dim3(grid), dim3(MEGA_THREADS), args, smem, st);
}

} // namespace ss
