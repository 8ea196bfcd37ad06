// Program description of the persistent verify kernel: a list of phases (built once per model) and
// the per-call parameters.  Plain data shared by the host API and the kernel.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

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
    int slab_rows, u_bytes;       // set by launch_mega: rows held in the LDS slab, size of the slab area
    int large_slab;               // host to launch_mega only: 12 KB of K per slab row pays for this model's shapes (if the rows fit LDS)
    unsigned long long *timeline; // optional [5*n_phases][G] device clock samples of every workgroup (NULL: off)
};

constexpr int MEGA_THREADS = 256;

// number of workgroups a launch may use (all resident at once), the largest number of hidden rows a
// launch can take (they must fit the LDS activation slab), and the launch itself
int mega_grid(int dtype, int device);
int mega_max_rows(int dtype);
hipError_t launch_mega(const MegaCall &call, int grid, hipStream_t st);
hipError_t mega_warm(int dtype, hipStream_t st); // launches every kernel variant once with an empty program
bool mega_wants_large_slab(int dtype, int d_model, int d_ff); // 12 KB instead of 8 KB of K per slab row saves slab trips for these shapes

} // namespace ss
