// Program description of the persistent verify kernel: a list of phases (built once per model) and
// the per-call parameters.  Plain data shared by the host API and the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include <vector>

namespace ss {

enum PhaseKind : int {
    PH_EMBED = 0, // hidden rows from the embedding table (or from given rows), packed for the first norm
    PH_QKV,       // QKV projection + row scale + rotary + cache append
    PH_ATTN,      // multi-row decode attention (+ merge by the last split to finish)
    PH_RESID,     // O projection / down projection: h += ..., repack for the next norm
    PH_SWIGLU,    // gate/up projection + row scale + SwiGLU
    PH_HEAD,      // LM head + row scale
    PH_LEN        // cache lengths += M
};

// ACT_A / ACT_A1: the packed hidden rows alternate between two buffers (the down projection and the
// embedding write ACT_A, the O projection writes ACT_A1), so that one can be cleared while the other is read
enum ActBuf : int { ACT_A = 0, ACT_Q = 1, ACT_O = 2, ACT_Z = 3, ACT_A1 = 4, ACT_COUNT = 5 };

// How the inputs of a phase become visible to a workgroup (MegaPhase::sync)
enum PhaseSync : int {
    SYNC_FLAGS = 0,     // device-wide barrier on the arrival flags, producers wait for their stores first
    SYNC_DATA = 1,      // self-validating data: the consumer polls the activation slab itself
    SYNC_DATA_ATTN = 2  // same; the producers are the attention units (workgroups without a unit wait for their flags first)
};

// activation planes: element (row, col) of plane pl lives at base[pl*plane + row*ld + col]
struct ActDesc {
    void *base;
    size_t plane; // elements between planes
    int ld;       // elements between rows
};

// ---- chunk schedule of a GEMM phase (built on the host, read by the kernel through scalar loads) -------------
// A workgroup walks its share of a weight matrix in "chunks" (8 loads = 8 KB per wavefront) through a ring of
// MEGA_RING register slots; one "round" = MEGA_RING consecutive positions, slot s of the ring always holds position
// s of a round.  The schedule of a phase is a list of rounds of MEGA_ROW_WORDS 32-bit words:
//   words 0 .. MEGA_RING-1: one position code each
//       bits 0-7 chunk index inside the tile's K range, bits 8-19 tile index inside the workgroup's share,
//       bits 20-22 chunk index inside the LDS activation slab, POS_DUMMY: padding (no data, no arithmetic),
//       POS_FIRST / POS_LAST: first / last chunk of its tile (clear the accumulators / reduce and stash the tile)
//   word MEGA_RING: what surrounds the round
//       bits 0-7 K slab to load into LDS before the round (ACT_NO_SLAB: none), ACT_CLEAR: the resets of the phase's
//       clear_phase follow that load, ACT_SEG_END: a segment (rounds without any other memory operation) ends behind
//       the round, ACT_FLUSH: the stashed tiles' epilogues run behind it, ACT_PHASE_END: the phase is over.
// Padding makes every slab group a whole number of rounds.  The schedule depends on the phase's shape, the chunks per
// LDS slab of the call (MegaCall::slab_ck) and the number of tiles of the workgroup's share, nothing else.
constexpr int MEGA_RING = 6;
constexpr int MEGA_ROW_WORDS = 8;
constexpr uint32_t POS_DUMMY = 1u << 23, POS_FIRST = 1u << 24, POS_LAST = 1u << 25;
constexpr uint32_t ACT_NO_SLAB = 0xffu, ACT_SEG_END = 1u << 8, ACT_FLUSH = 1u << 9, ACT_PHASE_END = 1u << 10, ACT_CLEAR = 1u << 11;
constexpr int MEGA_MIN_SLAB_CK = 4, MEGA_MAX_SLAB_CK = 6; // chunks of K per LDS slab a launch may choose from

struct MegaPhase {
    int kind, layer;
    const void *W;     // weights of a GEMM phase, row-major [rows][K]
    int N;             // QKV: 3*H*hd rows; SWIGLU: F (pairs of gate/up rows); RESID, HEAD: rows
    int K;
    int act_src;       // activation planes read (B operand)
    const float *gain; // EMBED / RESID: gain of the NEXT RMSNorm, folded in when the new rows are packed
    int act_dst;       // EMBED / RESID: activation planes written (ACT_A or ACT_A1); the norm partials use the same parity
    int sync;          // PhaseSync, honoured when MegaCall::data_sync is set
    int clear_phase;   // index of the later phase whose outputs this phase resets to the "not written yet" pattern (-1: none)
    // GEMM phases: word offsets into MegaCall::sched of the schedules for slab_ck = MEGA_MIN_SLAB_CK + i and a share of
    // ntiles_lo + j tiles (-1: no such share)
    int ntiles_lo;
    int sched_off[MEGA_MAX_SLAB_CK - MEGA_MIN_SLAB_CK + 1][2];
};

struct MegaCall {
    const MegaPhase *phases;
    int n_phases;
    int dtype;
    int d, H, hd, F, V;
    int R, B, M;
    float eps;
    // embedding / residual stream
    const int32_t *tokens; // NULL: rows are taken from h as given
    const void *embed;
    float *h;              // [R][d] residual stream (in/out)
    ActDesc act_a, act_q, act_o, act_z, act_a1; // activation planes, one named field per ActBuf (an array here would be indexed at run time,
                                                // which makes the compiler keep a copy of the whole argument in scratch memory)
    float *nsq;            // [2][16][G] per-workgroup partial sums of squares of the rows of h (index 0 goes with ACT_A, 1 with ACT_A1)
    // LM head: output row r reads activation row head_row0 + r*head_stride
    float *logits;
    int ldo, head_rows, head_row0, head_stride;
    // cache
    void *kc, *vc;
    size_t layer_elems;
    int32_t *len;
    int S, max_pos;
    const float2 *rope;
    // attention
    int nsplit, chunk;
    float *part_o, *part_m, *part_l;
    unsigned *attn_cnt; // [B*H] arrival counters (zero between launches)
    float scale_log2e;
    // device-wide barrier: arrive[G] slots hold the last epoch each workgroup reached
    unsigned *arrive;
    unsigned *abort_flag;
    unsigned epoch_base;
    unsigned spin_limit;
    int32_t *status;
    int data_sync;     // 1: phases marked SYNC_DATA* poll their input data instead of waiting at a barrier
    const void *zeros; // >= 64 zero bytes: the target of weight loads that have no data to fetch
    const uint32_t *sched; // chunk schedules of the GEMM phases (MegaPhase::sched_off)
    int slab_rows, slab_ck, u_bytes; // set by launch_mega: rows held in the LDS slab, chunks of K per slab, size of the slab area
    unsigned long long *timeline; // optional [MEGA_TL_SLOTS*n_phases][G] device clock samples of every workgroup (NULL: off)
};

constexpr int MEGA_THREADS = 256;
constexpr int MEGA_TL_SLOTS = 8; // timeline samples per phase and workgroup

// number of workgroups a launch may use (all resident at once), the largest number of hidden rows a
// launch can take (they must fit the LDS activation slab), and the launch itself
int mega_grid(int dtype, int device);
// Builds the chunk schedules of every GEMM phase of `prog` for a grid of `grid` workgroups (fills ntiles_lo and
// sched_off; phases of the same shape share their schedules) and returns the table to upload as MegaCall::sched.
std::vector<uint32_t> mega_build_schedules(std::vector<MegaPhase> &prog, int grid, int dtype, int head_dim);
int mega_max_rows(int dtype);
hipError_t launch_mega(const MegaCall &call, int grid, hipStream_t st);

} // namespace ss
