// C ABI of the library (declared in include/specverify.h): argument validation, handle bookkeeping
// and the order in which the kernels of one verify pass / draft step / rejection step are enqueued.
// No arithmetic of the method lives here.
#include "../../include/specverify.h"
#include "ss_kernels.h"
#include "ss_mega.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <set>
#include <string>
#include <algorithm>
#include <atomic>
#include <vector>

using namespace ss;

static thread_local std::string g_err;

static int fail(int code, const char *fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    g_err = buf;
    return code;
}

#define HIP_TRY(expr)                                                                              \
    do {                                                                                           \
        hipError_t e_ = (expr);                                                                    \
        if (e_ != hipSuccess) return fail(SS_EHIP, "%s: %s", #expr, hipGetErrorString(e_));        \
    } while (0)

static int check_launch() {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(SS_EHIP, "kernel launch: %s", hipGetErrorString(e));
    return SS_OK;
}

static inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

struct ss_model {
    ss_model_cfg cfg;
    std::vector<ss_layer_weights> layers;
    const void *embed, *lm_head;
    const float *gf;
    const float *s_head = nullptr; // row scales of an int8 LM head
    int planes, esz, W; // activation planes, storage element size, H*hd
    int R16;            // max_rows rounded up to 16
    float *h;           // [max_rows][d] residual stream
    void *act_a;        // planes [R16][d]   normalised hidden rows
    void *act_a1 = nullptr; // second buffer of the same shape (persistent kernel: rows packed by the O projection)
    void *act_q;        // planes [R16][W]   rotated queries
    void *act_o;        // planes [R16][W]   attention output
    void *act_z;        // planes [R16][F]   SwiGLU output
    float *part_o, *part_m, *part_l;
    float *logits_ws; // [max_rows][vocab] (draft step)
    float2 *stats_ws; // [max_rows]
    float *nsq_ws = nullptr;       // per-tile sums of squares of a deferred RMSNorm (calls of at most 16 rows): [16][d_model / 16]
    float *splitk_ws = nullptr;    // partial tiles of split-K GEMM launches (models that take more than 16 rows per call)
    size_t splitk_ws_bytes = 0;
    unsigned *stats_cnt = nullptr; // [max_rows] arrival counters of the segmented row statistics (zero between launches)
    float2 *stats_part = nullptr;  // per-segment partial statistics
    void *ws = nullptr;            // workspace of the softmax / rejection kernels of ss_speculative_step (layout: see workspace section)
    size_t ws_bytes = 0;
    unsigned long long *timeline = nullptr; // development aid: caller's buffer of device clock samples (ss_model_set_timeline)
    size_t timeline_entries = 0;
    float2 *rope;     // [max_pos][hd/2]
    int32_t *status;
    std::vector<void *> owned;
    // persistent verify kernel: phase programs (device), barrier state, norm partials
    int mega_G = 0;                 // workgroups per launch (0: persistent path unavailable)
    int mega_G_max = 0;             // one per compute unit: what the barrier arrays are sized for
    int mega_rows = 0;              // most rows (batch * M) a persistent launch takes
    int mega_min_units = 0;         // fewest ownership units of any GEMM phase: data synchronisation needs a grid no larger
    bool data_sync = true;          // persistent kernel: self-validating activations instead of barriers where possible
    unsigned spin_limit = 1u << 20; // persistent kernel: polls of a bounded wait before the workgroup gives up
    MegaPhase *prog_full = nullptr; // [embed, layers, head, len]
    MegaPhase *prog_nohead = nullptr; // [embed, layers, len]
    int n_full = 0, n_nohead = 0;
    float *nsq = nullptr;
    unsigned *arrive = nullptr, *abort_flag = nullptr, *attn_cnt = nullptr;
    void *zeros = nullptr;
    unsigned epoch = 1;
    bool persistent = false; // forward path: false = one launch per phase (default), true = the persistent kernel where the rows fit
    // optional per-kernel-class timing (ss_profile_*): event pairs recorded around launches
    bool prof = false;
    std::vector<hipEvent_t> ev;
    std::vector<int> ev_tag;
    size_t ev_used = 0;
};

enum ProfTag { PT_NORM = 0, PT_QKV, PT_ATTN, PT_OPROJ, PT_GATEUP, PT_DOWN, PT_HEAD, PT_OTHER, PT_PERSISTENT, PT_COUNT };

// records an event pair around the launches issued while it is alive (only when profiling is on)
struct ProfScope {
    ss_model *m;
    hipStream_t st;
    bool on;
    ProfScope(ss_model *m_, int tag, hipStream_t st_) : m(m_), st(st_), on(m_->prof) {
        if (!on) return;
        if (m->ev_used + 2 > m->ev.size()) {
            for (int i = 0; i < 2; ++i) {
                hipEvent_t e;
                if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
                m->ev.push_back(e);
            }
        }
        m->ev_tag.resize(m->ev.size() / 2);
        m->ev_tag[m->ev_used / 2] = tag;
        (void)hipEventRecord(m->ev[m->ev_used], st);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(m->ev[m->ev_used + 1], st);
        m->ev_used += 2;
    }
};

struct ss_kv_cache {
    int n_layers, H, hd, dtype, esz;
    int B, max_seq, S;
    void *k, *v; // [n_layers][B][H][S][hd] each (V block-transposed): the two halves of one buffer
    bool owns_buf; // the buffer was allocated by ss_kv_cache_alloc (else it is the caller's)
    int32_t *len_dev;
    std::vector<int32_t> len_ub; // host upper bound of every length
    size_t layer_elems;
};

static const int MAX_SPLITS = 16;

extern "C" const char *ss_last_error(void) { return g_err.c_str(); }

// Live handles.  ss_shutdown() destroys whatever is still alive while the HIP runtime is up; destroy / free calls
// on a handle that is no longer registered do nothing, so a binding may release its objects in any order.
static std::mutex g_reg_mu;
static std::set<ss_model *> g_models;
static std::set<ss_kv_cache *> g_caches;
static bool reg_take(ss_model *m) {
    std::lock_guard<std::mutex> lk(g_reg_mu);
    return g_models.erase(m) != 0;
}
static bool reg_take(ss_kv_cache *kv) {
    std::lock_guard<std::mutex> lk(g_reg_mu);
    return g_caches.erase(kv) != 0;
}

// ------------------------------------------------------------------------------------------ model

// ss_freeze_allocations: while set, every path of the library that would allocate device memory fails instead
static std::atomic<int> g_alloc_frozen{0};
static hipError_t lib_malloc(void **p, size_t bytes) {
    if (g_alloc_frozen.load()) return hipErrorOutOfMemory;
    return hipMalloc(p, bytes);
}

static int dev_alloc(ss_model *m, void **p, size_t bytes, bool zero) {
    if (g_alloc_frozen.load()) return fail(SS_EHIP, "device allocations are frozen (ss_freeze_allocations)");
    HIP_TRY(hipMalloc(p, bytes ? bytes : 16));
    m->owned.push_back(*p);
    if (zero) HIP_TRY(hipMemset(*p, 0, bytes ? bytes : 16));
    return SS_OK;
}

static void model_release(ss_model *m) {
    for (void *p : m->owned) (void)hipFree(p);
    for (hipEvent_t e : m->ev) (void)hipEventDestroy(e);
    delete m;
}

extern "C" int ss_model_destroy(ss_model *m) {
    if (!m || !reg_take(m)) return SS_OK;
    model_release(m);
    return SS_OK;
}

extern "C" int ss_model_create(const ss_model_cfg *cfg, const ss_weights *w, ss_model **out) {
    if (!cfg || !w || !out) return fail(SS_EINVAL, "ss_model_create: NULL argument");
    const ss_model_cfg &c = *cfg;
    if (c.dtype != SS_DTYPE_F32 && c.dtype != SS_DTYPE_BF16) return fail(SS_EINVAL, "dtype must be f32 or bf16");
    const int E = c.dtype == SS_DTYPE_BF16 ? 8 : 4;
    if (c.n_layers < 0 || c.d_model <= 0 || c.n_heads <= 0 || c.d_ff <= 0 || c.vocab <= 0 || c.max_rows <= 0 || c.max_pos <= 0)
        return fail(SS_EINVAL, "non-positive shape");
    if (c.head_dim != 32 && c.head_dim != 64 && c.head_dim != 128) return fail(SS_EINVAL, "head_dim must be 32, 64 or 128");
    if (c.d_model % E || c.d_ff % E) return fail(SS_EINVAL, "d_model and d_ff must be multiples of %d", E);
    if (!w->layers && c.n_layers) return fail(SS_EINVAL, "weights->layers is NULL");
    for (int l = 0; l < c.n_layers; ++l) {
        const ss_layer_weights &L = w->layers[l];
        if (!L.wqkv || !L.wo || !L.wgu || !L.wd || !L.g1 || !L.g2) return fail(SS_EINVAL, "layer %d has a NULL weight", l);
        if (c.weight_quant && (!L.sqkv || !L.so || !L.sgu || !L.sd)) return fail(SS_EINVAL, "layer %d of a quantised model has a NULL scale array", l);
    }
    if (c.weight_quant) {
        if (c.weight_quant != SS_QUANT_INT8 && c.weight_quant != SS_QUANT_INT4_G128) return fail(SS_EINVAL, "weight_quant must be SS_QUANT_NONE, SS_QUANT_INT8 or SS_QUANT_INT4_G128");
        if (c.dtype != SS_DTYPE_BF16) return fail(SS_EINVAL, "quantised weights need bf16 storage for activations and cache");
        const int mult = c.weight_quant == SS_QUANT_INT4_G128 ? 128 : 16;
        if (c.d_model % mult || (c.n_heads * c.head_dim) % mult || c.d_ff % mult)
            return fail(SS_EINVAL, "quantised weights: d_model, n_heads*head_dim and d_ff must be multiples of %d", mult);
        if (w->lm_head && !w->s_head) return fail(SS_EINVAL, "quantised LM head without scales");
    }
    ss_model *m = new ss_model();
    m->cfg = c;
    m->layers.assign(w->layers, w->layers + c.n_layers);
    m->embed = w->embed;
    m->lm_head = w->lm_head;
    m->gf = w->gf;
    m->s_head = c.weight_quant ? w->s_head : nullptr;
    m->planes = c.dtype == SS_DTYPE_BF16 ? 2 : 1;
    m->esz = c.dtype == SS_DTYPE_BF16 ? 2 : 4;
    m->W = c.n_heads * c.head_dim;
    m->R16 = round_up(c.max_rows, 16);
    const size_t pe = (size_t)m->planes * m->esz * m->R16;
    int rc = SS_OK;
    auto A = [&](void **p, size_t bytes, bool zero) {
        if (rc == SS_OK) rc = dev_alloc(m, p, bytes, zero);
    };
    A((void **)&m->h, sizeof(float) * (size_t)c.max_rows * c.d_model, true);
    A(&m->act_a, pe * c.d_model, true);
    A(&m->act_q, pe * m->W, true);
    A(&m->act_o, pe * m->W, true);
    A(&m->act_z, pe * c.d_ff, true);
    A((void **)&m->part_o, sizeof(float) * (size_t)MAX_SPLITS * c.max_rows * m->W, true);
    A((void **)&m->part_m, sizeof(float) * (size_t)MAX_SPLITS * c.max_rows * c.n_heads, true);
    A((void **)&m->part_l, sizeof(float) * (size_t)MAX_SPLITS * c.max_rows * c.n_heads, true);
    A((void **)&m->logits_ws, sizeof(float) * (size_t)c.max_rows * c.vocab, true);
    A((void **)&m->stats_ws, sizeof(float2) * (size_t)c.max_rows, true);
    if (c.max_rows > 16) {
        const size_t cols = (size_t)std::max(std::max(3 * m->W, 2 * c.d_ff), c.d_model);
        m->splitk_ws_bytes = 4 * cols * (size_t)((c.max_rows + 15) / 16) * 64;
        A((void **)&m->splitk_ws, m->splitk_ws_bytes, false);
    }
    A((void **)&m->stats_cnt, sizeof(unsigned) * (size_t)c.max_rows, true);
    if (c.d_model % 256 == 0 && c.d_model / 16 <= NSQ_MAX_TILES) A((void **)&m->nsq_ws, sizeof(float) * 16 * (size_t)(c.d_model / 16), true);
    A((void **)&m->stats_part, row_stats_partial_bytes(c.max_rows, c.vocab) + 16, true);
    m->ws_bytes = ss_workspace_bytes(2 * (int64_t)c.max_rows, c.vocab); // target rows + draft rows of a step
    A(&m->ws, m->ws_bytes, true);
    A((void **)&m->rope, sizeof(float2) * (size_t)c.max_pos * (c.head_dim / 2), false);
    A((void **)&m->status, sizeof(int32_t), true);
    if (rc != SS_OK) {
        model_release(m);
        return rc;
    }
    // phase programs of the persistent verify kernel
    {
        int dev = 0;
        (void)hipGetDevice(&dev);
        m->mega_G = m->mega_G_max = c.weight_quant ? 0 : mega_grid(c.dtype, dev); // the persistent kernel streams storage-type matrices only
        m->mega_rows = mega_max_rows(c.dtype);
        if (m->mega_G > 0 && mega_warm(c.dtype, nullptr) != hipSuccess) m->mega_G = m->mega_G_max = 0; // (first-launch set-up of both kernel variants happens here, where allocating is allowed)
        if (m->mega_G > 0 && c.n_layers >= 0) {
            std::vector<MegaPhase> prog;
            auto gain_after = [&](int l) { return l + 1 < c.n_layers ? m->layers[l + 1].g1 : m->gf; };
            MegaPhase e{};
            e.kind = PH_EMBED;
            e.gain = c.n_layers ? m->layers[0].g1 : m->gf;
            e.act_dst = ACT_A;
            e.clear_phase = -1;
            prog.push_back(e);
            // Program layout: phase 0 = embedding, layer l = phases 1 + 5*l .. 5 + 5*l (QKV, attention, O, gate/up, down).
            // sync: how a phase's input is synchronised when the launch runs with data synchronisation;
            // clear_phase: whose outputs a phase resets (see clear_outputs() in the kernel source).
            for (int l = 0; l < c.n_layers; ++l) {
                const ss_layer_weights &L = m->layers[l];
                const int p0 = 1 + 5 * l;
                MegaPhase q{}; q.kind = PH_QKV; q.layer = l; q.W = L.wqkv; q.N = 3 * m->W; q.K = c.d_model; q.act_src = ACT_A;
                q.sync = l ? SYNC_DATA : SYNC_FLAGS; q.clear_phase = p0 + 2; prog.push_back(q);
                MegaPhase a{}; a.kind = PH_ATTN; a.layer = l; a.sync = SYNC_FLAGS; a.clear_phase = -1; prog.push_back(a);
                MegaPhase o{}; o.kind = PH_RESID; o.layer = l; o.W = L.wo; o.N = c.d_model; o.K = m->W; o.act_src = ACT_O; o.gain = L.g2;
                o.act_dst = ACT_A1; o.sync = SYNC_DATA_ATTN; o.clear_phase = p0 + 3; prog.push_back(o);
                MegaPhase u{}; u.kind = PH_SWIGLU; u.layer = l; u.W = L.wgu; u.N = c.d_ff; u.K = c.d_model; u.act_src = ACT_A1;
                u.sync = SYNC_DATA; u.clear_phase = p0 + 4; prog.push_back(u);
                MegaPhase dn{}; dn.kind = PH_RESID; dn.layer = l; dn.W = L.wd; dn.N = c.d_model; dn.K = c.d_ff; dn.act_src = ACT_Z; dn.gain = gain_after(l);
                dn.act_dst = ACT_A; dn.sync = SYNC_DATA; dn.clear_phase = l + 1 < c.n_layers ? p0 + 5 + 1 : -1; prog.push_back(dn);
            }
            if (c.n_layers) prog[0].clear_phase = 2; // the embedding clears what the first attention phase writes
            MegaPhase ln{}; ln.kind = PH_LEN; ln.sync = SYNC_FLAGS; ln.clear_phase = -1;
            std::vector<MegaPhase> nohead = prog;
            nohead.push_back(ln);
            if (m->lm_head && m->gf) {
                MegaPhase hd{}; hd.kind = PH_HEAD; hd.W = m->lm_head; hd.N = c.vocab; hd.K = c.d_model; hd.act_src = ACT_A;
                hd.sync = c.n_layers ? SYNC_DATA : SYNC_FLAGS; hd.clear_phase = -1; prog.push_back(hd);
            }
            prog.push_back(ln);
            m->mega_min_units = c.vocab;
            for (const MegaPhase &ph : prog) {
                if (ph.kind == PH_QKV) m->mega_min_units = std::min(m->mega_min_units, ph.N / 16);
                if (ph.kind == PH_RESID || ph.kind == PH_SWIGLU || ph.kind == PH_HEAD) m->mega_min_units = std::min(m->mega_min_units, ph.N);
            }
            {
                m->n_full = (int)prog.size();
                m->n_nohead = (int)nohead.size();
                A((void **)&m->prog_full, sizeof(MegaPhase) * prog.size(), false);
                A((void **)&m->prog_nohead, sizeof(MegaPhase) * nohead.size(), false);
                A((void **)&m->nsq, sizeof(float) * 2 * 16 * (size_t)m->mega_G, true);
                A(&m->act_a1, pe * c.d_model, true);
                A((void **)&m->arrive, sizeof(unsigned) * (size_t)m->mega_G, true);
                A((void **)&m->abort_flag, sizeof(unsigned), true);
                A(&m->zeros, 256, true);
                A((void **)&m->attn_cnt, sizeof(unsigned) * (size_t)c.max_rows * c.n_heads, true);
                if (rc == SS_OK) {
                    hipError_t e1 = hipMemcpy(m->prog_full, prog.data(), sizeof(MegaPhase) * prog.size(), hipMemcpyHostToDevice);
                    hipError_t e2 = hipMemcpy(m->prog_nohead, nohead.data(), sizeof(MegaPhase) * nohead.size(), hipMemcpyHostToDevice);
                    if (e1 != hipSuccess || e2 != hipSuccess) rc = fail(SS_EHIP, "program upload failed");
                }
                if (rc != SS_OK) {
                    model_release(m);
                    return rc;
                }
            }
        }
    }
    // rotary table: angle(pos, j) = pos * base^(-2j/hd), evaluated in double, stored as fp32 (cos, sin)
    {
        const int half = c.head_dim / 2;
        std::vector<float2> tab((size_t)c.max_pos * half);
        for (int j = 0; j < half; ++j) {
            const double inv = std::pow((double)c.rope_base, -2.0 * j / (double)c.head_dim);
            for (int p = 0; p < c.max_pos; ++p) {
                const double ang = (double)p * inv;
                tab[(size_t)p * half + j] = make_float2((float)std::cos(ang), (float)std::sin(ang));
            }
        }
        hipError_t e = hipMemcpy(m->rope, tab.data(), tab.size() * sizeof(float2), hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            model_release(m);
            return fail(SS_EHIP, "rope table upload: %s", hipGetErrorString(e));
        }
    }
    m->persistent = false; // one launch per phase unless ss_model_set_persistent asks for the persistent kernel (measured: as fast or faster at most shapes)
    {
        std::lock_guard<std::mutex> lk(g_reg_mu);
        g_models.insert(m);
    }
    *out = m;
    return SS_OK;
}

extern "C" int ss_device_status(ss_model *m, ss_stream stream, int32_t *status_host) {
    if (!m || !status_host) return fail(SS_EINVAL, "ss_device_status: NULL argument");
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(status_host, m->status, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    HIP_TRY(hipMemsetAsync(m->status, 0, sizeof(int32_t), st));
    if (m->abort_flag) {
        unsigned ab = 0;
        HIP_TRY(hipMemcpyAsync(&ab, m->abort_flag, sizeof(unsigned), hipMemcpyDeviceToHost, st));
        HIP_TRY(hipStreamSynchronize(st));
        if (ab) {
            // a device-wide barrier gave up: reset the barrier state so that later launches start clean
            *status_host |= 2;
            HIP_TRY(hipMemsetAsync(m->abort_flag, 0, sizeof(unsigned), st));
            HIP_TRY(hipMemsetAsync(m->arrive, 0, sizeof(unsigned) * (size_t)m->mega_G_max, st));
            HIP_TRY(hipMemsetAsync(m->attn_cnt, 0, sizeof(unsigned) * (size_t)m->cfg.max_rows * m->cfg.n_heads, st));
            HIP_TRY(hipStreamSynchronize(st));
            m->epoch = 1;
        }
    }
    return SS_OK;
}

extern "C" int ss_profile_enable(ss_model *m, int32_t on) {
    if (!m) return fail(SS_EINVAL, "ss_profile_enable: NULL model");
    m->prof = on != 0;
    m->ev_used = 0;
    return SS_OK;
}

extern "C" int ss_profile_read(ss_model *m, int32_t n_classes, double *total_ms_host, int64_t *launches_host) {
    if (!m || !total_ms_host || !launches_host || n_classes < PT_COUNT) return fail(SS_EINVAL, "ss_profile_read: bad argument (need %d classes)", (int)PT_COUNT);
    for (int i = 0; i < n_classes; ++i) {
        total_ms_host[i] = 0.0;
        launches_host[i] = 0;
    }
    for (size_t i = 0; i + 1 < m->ev_used; i += 2) {
        HIP_TRY(hipEventSynchronize(m->ev[i + 1]));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, m->ev[i], m->ev[i + 1]));
        total_ms_host[m->ev_tag[i / 2]] += ms;
        launches_host[m->ev_tag[i / 2]] += 1;
    }
    m->ev_used = 0;
    return SS_OK;
}

extern "C" int ss_quantize_rows_int8(const void *w_dev, int32_t dtype, int64_t rows, int64_t K, int8_t *q_dev, float *scale_dev,
                                     ss_stream stream) {
    if (!w_dev || !q_dev || !scale_dev) return fail(SS_EINVAL, "ss_quantize_rows_int8: NULL argument");
    if (dtype != SS_DTYPE_F32 && dtype != SS_DTYPE_BF16) return fail(SS_EINVAL, "ss_quantize_rows_int8: dtype must be f32 or bf16");
    if (rows < 1 || K < 1 || rows > 0x7fffffffLL) return fail(SS_EINVAL, "ss_quantize_rows_int8: rows %lld, K %lld out of range", (long long)rows, (long long)K);
    launch_quantize_rows_int8(dtype, w_dev, rows, K, q_dev, scale_dev, (hipStream_t)stream);
    return check_launch();
}

extern "C" int ss_quantize_rows_int4(const void *w_dev, int32_t dtype, int64_t rows, int64_t K, uint8_t *q_dev, float *scale_dev,
                                     ss_stream stream) {
    if (!w_dev || !q_dev || !scale_dev) return fail(SS_EINVAL, "ss_quantize_rows_int4: NULL argument");
    if (dtype != SS_DTYPE_F32 && dtype != SS_DTYPE_BF16) return fail(SS_EINVAL, "ss_quantize_rows_int4: dtype must be f32 or bf16");
    if (rows < 1 || K < 128 || K % 128 || rows > 0x7fffffffLL) return fail(SS_EINVAL, "ss_quantize_rows_int4: rows %lld, K %lld (K must be a multiple of 128)", (long long)rows, (long long)K);
    launch_quantize_rows_int4(dtype, w_dev, rows, K, q_dev, scale_dev, (hipStream_t)stream);
    return check_launch();
}

extern "C" int ss_probe_read_bandwidth(const void *buf_dev, size_t bytes, int32_t iters, uint32_t *sink_dev, double *gbps_host,
                                       ss_stream stream) {
    if (!buf_dev || !sink_dev || !gbps_host) return fail(SS_EINVAL, "ss_probe_read_bandwidth: NULL argument");
    if (bytes < ((size_t)1 << 20) || (bytes & 15) || ((uintptr_t)buf_dev & 15) || iters < 1 || iters > 10000)
        return fail(SS_EINVAL, "ss_probe_read_bandwidth: need a 16-byte aligned buffer of >= 1 MiB in 16-byte units and 1..10000 launches");
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    HIP_TRY(hipEventCreate(&e0));
    hipError_t err = hipEventCreate(&e1);
    float ms = 0.f;
    if (err == hipSuccess) {
        ss::launch_read_probe(buf_dev, bytes, sink_dev, st);   // untimed first launch
        err = hipEventRecord(e0, st);
        for (int i = 0; i < iters && err == hipSuccess; ++i) {
            ss::launch_read_probe(buf_dev, bytes, sink_dev, st);
            err = hipGetLastError();
        }
        if (err == hipSuccess) err = hipEventRecord(e1, st);
        if (err == hipSuccess) err = hipEventSynchronize(e1);
        if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    }
    (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (err != hipSuccess) return fail(SS_EHIP, "ss_probe_read_bandwidth: %s", hipGetErrorString(err));
    *gbps_host = ms > 0.f ? (double)bytes * iters / (ms * 1e-3) / 1e9 : 0.0;
    return SS_OK;
}

// ------------------------------------------------------------------------------------------ cache

extern "C" size_t ss_kv_cache_bytes(const ss_model *m, int32_t batch, int32_t max_seq) {
    if (!m || batch <= 0 || max_seq <= 0) return 0;
    const size_t S = round_up(max_seq, 64);
    return 2 * (size_t)m->cfg.n_layers * batch * m->W * S * m->esz;
}

static void cache_release(ss_kv_cache *kv) {
    if (kv->owns_buf && kv->k) (void)hipFree(kv->k);
    if (kv->len_dev) (void)hipFree(kv->len_dev);
    delete kv;
}

extern "C" int ss_kv_cache_free(ss_kv_cache *kv) {
    if (!kv || !reg_take(kv)) return SS_OK;
    cache_release(kv);
    return SS_OK;
}

// handle over the caller's buffer (or one allocated here when buf is NULL): keys in the first half, values in the second
static int cache_create(const ss_model *m, int32_t batch, int32_t max_seq, void *buf, size_t buf_bytes, hipStream_t st, ss_kv_cache **out,
                        const char *who) {
    if (!m || !out) return fail(SS_EINVAL, "%s: NULL argument", who);
    if (batch <= 0 || max_seq <= 0) return fail(SS_EINVAL, "%s: batch and max_seq must be positive", who);
    if (max_seq > m->cfg.max_pos) return fail(SS_EINVAL, "%s: max_seq %d exceeds the model's rotary table (%d)", who, max_seq, m->cfg.max_pos);
    const size_t need = ss_kv_cache_bytes(m, batch, max_seq);
    if (buf && buf_bytes < need) return fail(SS_ECAPACITY, "%s: the buffer has %zu bytes, the cache needs %zu", who, buf_bytes, need);
    if (buf && ((uintptr_t)buf & 15)) return fail(SS_EINVAL, "%s: the buffer must be 16-byte aligned", who);
    ss_kv_cache *kv = new ss_kv_cache();
    kv->n_layers = m->cfg.n_layers;
    kv->H = m->cfg.n_heads;
    kv->hd = m->cfg.head_dim;
    kv->dtype = m->cfg.dtype;
    kv->esz = m->esz;
    kv->B = batch;
    kv->max_seq = max_seq;
    kv->S = round_up(max_seq, 64);
    kv->layer_elems = (size_t)batch * kv->H * kv->S * kv->hd;
    kv->k = kv->v = nullptr;
    kv->len_dev = nullptr;
    kv->owns_buf = buf == nullptr;
    kv->len_ub.assign(batch, 0);
    hipError_t e = hipSuccess;
    if (!buf) e = lib_malloc(&buf, need ? need : 16);
    if (e == hipSuccess) {
        kv->k = buf;
        kv->v = (char *)buf + need / 2;
        e = lib_malloc((void **)&kv->len_dev, sizeof(int32_t) * batch);
    }
    // zero fill: attention multiplies the (masked) value entries past a length inside its last block by zero weights,
    // so they must hold finite numbers
    if (e == hipSuccess && need) e = hipMemsetAsync(buf, 0, need, st);
    if (e == hipSuccess) e = hipMemsetAsync(kv->len_dev, 0, sizeof(int32_t) * batch, st);
    if (e != hipSuccess) {
        cache_release(kv);
        return fail(SS_EHIP, "%s: %s", who, hipGetErrorString(e));
    }
    {
        std::lock_guard<std::mutex> lk(g_reg_mu);
        g_caches.insert(kv);
    }
    *out = kv;
    return SS_OK;
}

extern "C" int ss_kv_cache_create(const ss_model *m, int32_t batch, int32_t max_seq, void *buf_dev, size_t buf_bytes, ss_stream stream,
                                  ss_kv_cache **out) {
    if (!buf_dev) return fail(SS_EINVAL, "ss_kv_cache_create: buf_dev is NULL");
    return cache_create(m, batch, max_seq, buf_dev, buf_bytes, (hipStream_t)stream, out, "ss_kv_cache_create");
}

extern "C" int ss_kv_cache_alloc(const ss_model *m, int32_t batch, int32_t max_seq, ss_kv_cache **out) {
    int rc = cache_create(m, batch, max_seq, nullptr, 0, nullptr, out, "ss_kv_cache_alloc");
    if (rc == SS_OK) HIP_TRY(hipStreamSynchronize(nullptr));
    return rc;
}

extern "C" int ss_kv_cache_append(ss_kv_cache *kv, int32_t layer, int32_t seq, int32_t pos0, const void *k_dev,
                                  const void *v_dev, int32_t n_rows, ss_stream stream) {
    if (!kv || !k_dev || !v_dev) return fail(SS_EINVAL, "ss_kv_cache_append: NULL argument");
    if (layer < 0 || layer >= kv->n_layers || seq < 0 || seq >= kv->B || n_rows < 0 || pos0 < 0)
        return fail(SS_EINVAL, "ss_kv_cache_append: layer/seq/rows out of range");
    if ((int64_t)pos0 + n_rows > kv->max_seq) return fail(SS_ECAPACITY, "append of %d rows at %d exceeds max_seq %d", n_rows, pos0, kv->max_seq);
    char *kc = (char *)kv->k + kv->layer_elems * layer * kv->esz;
    char *vc = (char *)kv->v + kv->layer_elems * layer * kv->esz;
    launch_kv_append(kv->dtype, kc, vc, k_dev, v_dev, seq, pos0, n_rows, kv->H, kv->hd, kv->S, (hipStream_t)stream);
    return check_launch();
}

extern "C" int ss_kv_cache_set_len(ss_kv_cache *kv, const int32_t *len_host, ss_stream stream) {
    if (!kv || !len_host) return fail(SS_EINVAL, "ss_kv_cache_set_len: NULL argument");
    for (int b = 0; b < kv->B; ++b)
        if (len_host[b] < 0 || len_host[b] > kv->max_seq) return fail(SS_EINVAL, "length %d of sequence %d outside [0, %d]", len_host[b], b, kv->max_seq);
    hipStream_t st = (hipStream_t)stream;
    // the source must stay valid until the copy ran: synchronise (this call is off the hot path)
    HIP_TRY(hipMemcpyAsync(kv->len_dev, len_host, sizeof(int32_t) * kv->B, hipMemcpyHostToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    kv->len_ub.assign(len_host, len_host + kv->B);
    return SS_OK;
}

extern "C" int ss_kv_cache_truncate(ss_kv_cache *kv, const int32_t *new_len_dev, const int32_t *new_len_host, int32_t *status_dev,
                                    ss_stream stream) {
    if (!kv || !new_len_dev) return fail(SS_EINVAL, "ss_kv_cache_truncate: NULL argument");
    launch_len_truncate(kv->len_dev, new_len_dev, kv->B, status_dev, (hipStream_t)stream);
    if (new_len_host)
        for (int b = 0; b < kv->B; ++b) kv->len_ub[b] = std::min(kv->len_ub[b], std::max(new_len_host[b], 0));
    return check_launch();
}

extern "C" int ss_kv_cache_get_len(ss_kv_cache *kv, int32_t *len_host, ss_stream stream) {
    if (!kv || !len_host) return fail(SS_EINVAL, "ss_kv_cache_get_len: NULL argument");
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(len_host, kv->len_dev, sizeof(int32_t) * kv->B, hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    kv->len_ub.assign(len_host, len_host + kv->B);
    return SS_OK;
}

extern "C" int ss_kv_cache_rollback(ss_kv_cache *kv, const int32_t *n_accepted_dev, const int32_t *n_accepted_host,
                                    int32_t M, ss_stream stream) {
    if (!kv || !n_accepted_dev) return fail(SS_EINVAL, "ss_kv_cache_rollback: NULL argument");
    if (M < 1 || M > SS_MAX_ROWS_PER_SEQ) return fail(SS_EINVAL, "M must be in [1, %d]", SS_MAX_ROWS_PER_SEQ);
    for (int b = 0; b < kv->B; ++b)
        if (kv->len_ub[b] < M) return fail(SS_EINVAL, "sequence %d is shorter than the %d rows to roll back over", b, M);
    launch_len_rollback(kv->len_dev, n_accepted_dev, kv->B, M, (hipStream_t)stream);
    // without the host copy the bound keeps the unrolled length; ss_kv_cache_get_len tightens it
    if (n_accepted_host)
        for (int b = 0; b < kv->B; ++b) {
            const int a = std::min(std::max(n_accepted_host[b], 0), M - 1);
            kv->len_ub[b] -= M - 1 - a;
        }
    return check_launch();
}

// ------------------------------------------------------------------------------------------ forward

static int check_pair(const ss_model *m, const ss_kv_cache *kv, int batch, int M, const char *who) {
    if (!m || !kv) return fail(SS_EINVAL, "%s: NULL handle", who);
    // a model may run on the leading layers of a deeper cache of the same head geometry (an early-exit draft
    // working in the target's cache)
    if (kv->n_layers < m->cfg.n_layers || kv->H != m->cfg.n_heads || kv->hd != m->cfg.head_dim || kv->dtype != m->cfg.dtype)
        return fail(SS_EINVAL, "%s: cache was allocated for a different model shape", who);
    if (batch != kv->B) return fail(SS_EINVAL, "%s: batch %d != cache batch %d", who, batch, kv->B);
    if (M < 1 || M > SS_MAX_ROWS_PER_SEQ) return fail(SS_EINVAL, "%s: rows per sequence must be in [1, %d]", who, SS_MAX_ROWS_PER_SEQ);
    if ((int64_t)batch * M > m->cfg.max_rows) return fail(SS_EINVAL, "%s: %d rows exceed the model's max_rows %d", who, batch * M, m->cfg.max_rows);
    for (int b = 0; b < batch; ++b)
        if (kv->len_ub[b] + M > kv->max_seq || kv->len_ub[b] + M > m->cfg.max_pos)
            return fail(SS_ECAPACITY, "%s: sequence %d at length <= %d has no room for %d rows (max_seq %d)", who, b, kv->len_ub[b], M, kv->max_seq);
    return SS_OK;
}

// all layers over the R = batch*M rows in m->h
static void run_layers(ss_model *m, ss_kv_cache *kv, int batch, int M, hipStream_t st) {
    const ss_model_cfg &c = m->cfg;
    const int R = batch * M, d = c.d_model, W = m->W, F = c.d_ff;
    const size_t pl = (size_t)m->R16;
    int Lmax = 0;
    for (int b = 0; b < batch; ++b) Lmax = std::max(Lmax, kv->len_ub[b] + M);
    // KV splits per (sequence, head): about 512 workgroups in all, but a single split (no partials, no merge launch)
    // once the units alone give every compute unit a workgroup (8 sequences x 32 heads at 4096 positions: 104 us per
    // layer against 109 - 112 with two splits and the merge)
    const int units = batch * c.n_heads;
    int want = units >= 256 ? 1 : (512 + units - 1) / units;
    if (Lmax <= 192) want = 1; // up to about 200 positions one workgroup per unit beats splits + merge launch (measured at 100, 145, 250 positions: -1.3 %, -0.9 %, +0.4 % of a pass)
    int nsplit = std::max(1, std::min(std::min(want, (Lmax + 63) / 64), MAX_SPLITS));
    const int chunk = round_up((Lmax + nsplit - 1) / nsplit, 64);
    nsplit = (Lmax + chunk - 1) / chunk;

    const int wbits = c.weight_quant == SS_QUANT_INT4_G128 ? 4 : 8;
    // The two residual projections name the RMSNorm that follows them.  A launcher that has a row-wise last launch
    // anyway (split K, more than 16 rows) writes the normalised planes there (1); the kernels of at most 16 rows write
    // h * gain as planes and per-tile sums of squares, and the GEMM that consumes the planes multiplies its sums by the
    // row scale (2: the norm is deferred; no launch of its own either way).  0: the norm is still to be launched.
    int normed = 0;
    const int T = d / 16;
    const bool defer_ok = R <= 16 && m->nsq_ws != nullptr;
    auto with_norm = [&](GemmArgs &g, const float *gain) {
        g.norm_gain = gain; g.norm_act = m->act_a; g.norm_act_plane = pl * d; g.norm_ld = d; g.norm_eps = c.rms_eps;
        if (defer_ok) { g.nsq_out = m->nsq_ws; g.nsq_ld = T; }
    };
    auto consumes_norm = [&](GemmArgs &g) { // the GEMM reads act_a: tell it when the row scale is still missing
        if (normed == 2) { g.act_nsq = m->nsq_ws; g.act_nsq_tiles = T; g.act_nsq_ld = T; g.norm_eps = c.rms_eps; }
    };
    for (int l = 0; l < c.n_layers; ++l) {
        const ss_layer_weights &L = m->layers[l];
        char *kc = (char *)kv->k + kv->layer_elems * l * kv->esz;
        char *vc = (char *)kv->v + kv->layer_elems * l * kv->esz;
        if (!normed) {
            ProfScope ps(m, PT_NORM, st);
            launch_rmsnorm_pack(c.dtype, m->h, L.g1, R, d, c.rms_eps, m->act_a, pl * d, d, st);
        }
        GemmArgs g{};
        g.splitk_ws = m->splitk_ws; g.splitk_ws_bytes = m->splitk_ws_bytes;
        g.W = L.wqkv; g.N = 3 * W; g.K = d; g.wscale = c.weight_quant ? L.sqkv : nullptr; g.wbits = wbits;
        g.act = m->act_a; g.act_plane = pl * d; g.ld_act = d; g.R = R;
        g.act_out = m->act_q; g.act_out_plane = pl * W; g.ld_act_out = W;
        g.H = c.n_heads; g.hd = c.head_dim; g.M = M; g.S = kv->S; g.max_pos = c.max_pos;
        g.len = kv->len_dev; g.rope = m->rope; g.kcache = kc; g.vcache = vc;
        consumes_norm(g);
        {
            ProfScope ps(m, PT_QKV, st);
            launch_gemm(c.dtype, EPI_QKV, g, st);
        }

        AttnArgs a{};
        a.q = m->act_q; a.q_plane = pl * W; a.ldq = W;
        a.kcache = kc; a.vcache = vc; a.len = kv->len_dev;
        a.B = batch; a.M = M; a.H = c.n_heads; a.hd = c.head_dim; a.S = kv->S; a.R = R;
        a.nsplit = nsplit; a.chunk = chunk;
        a.part_o = m->part_o; a.part_m = m->part_m; a.part_l = m->part_l;
        a.act_out = m->act_o; a.act_out_plane = pl * W; a.ld_out = W;
        a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)c.head_dim));
        {
            ProfScope ps(m, PT_ATTN, st);
            launch_attention(c.dtype, a, st);
        }

        GemmArgs o{};
        o.splitk_ws = m->splitk_ws; o.splitk_ws_bytes = m->splitk_ws_bytes;
        o.W = L.wo; o.N = d; o.K = W; o.wscale = c.weight_quant ? L.so : nullptr; o.wbits = wbits;
        o.act = m->act_o; o.act_plane = pl * W; o.ld_act = W; o.R = R;
        o.out = m->h; o.resid = m->h; o.ldo = d;
        with_norm(o, L.g2);
        {
            ProfScope ps(m, PT_OPROJ, st);
            normed = launch_gemm(c.dtype, EPI_RESID, o, st);
        }
        if (!normed) {
            ProfScope ps(m, PT_NORM, st);
            launch_rmsnorm_pack(c.dtype, m->h, L.g2, R, d, c.rms_eps, m->act_a, pl * d, d, st);
        }
        GemmArgs u{};
        u.splitk_ws = m->splitk_ws; u.splitk_ws_bytes = m->splitk_ws_bytes;
        u.W = L.wgu; u.N = F; u.K = d; u.wscale = c.weight_quant ? L.sgu : nullptr; u.wbits = wbits;
        u.act = m->act_a; u.act_plane = pl * d; u.ld_act = d; u.R = R;
        u.act_out = m->act_z; u.act_out_plane = pl * F; u.ld_act_out = F;
        consumes_norm(u);
        {
            ProfScope ps(m, PT_GATEUP, st);
            launch_gemm(c.dtype, EPI_SWIGLU, u, st);
        }

        GemmArgs dn{};
        dn.splitk_ws = m->splitk_ws; dn.splitk_ws_bytes = m->splitk_ws_bytes;
        dn.W = L.wd; dn.N = d; dn.K = F; dn.wscale = c.weight_quant ? L.sd : nullptr; dn.wbits = wbits;
        dn.act = m->act_z; dn.act_plane = pl * F; dn.ld_act = F; dn.R = R;
        dn.out = m->h; dn.resid = m->h; dn.ldo = d;
        if (l + 1 < c.n_layers) with_norm(dn, m->layers[l + 1].g1); // (the final norm belongs to the head: it may gather rows)
        {
            ProfScope ps(m, PT_DOWN, st);
            normed = launch_gemm(c.dtype, EPI_RESID, dn, st);
        }
    }
    launch_len_add(kv->len_dev, batch, M, st);
    for (int b = 0; b < batch; ++b) kv->len_ub[b] += M;
}

// logits[r][:] = RMSNorm(h[row0 + r*stride], gf) . W_lm^T for r < nrows
static void run_head(ss_model *m, int nrows, int row0, int stride, float *logits, hipStream_t st) {
    const ss_model_cfg &c = m->cfg;
    const size_t pl = (size_t)m->R16;
    {
        ProfScope ps(m, PT_NORM, st);
        launch_rmsnorm_pack_rows(c.dtype, m->h, m->gf, nrows, row0, stride, c.d_model, c.rms_eps, m->act_a, pl * c.d_model, c.d_model, st);
    }
    ProfScope ps(m, PT_HEAD, st);
    GemmArgs g{};
    g.W = m->lm_head; g.N = c.vocab; g.K = c.d_model; g.wscale = m->s_head; g.wbits = c.weight_quant == SS_QUANT_INT4_G128 ? 4 : 8;
    g.act = m->act_a; g.act_plane = pl * c.d_model; g.ld_act = c.d_model; g.R = nrows;
    g.out = logits; g.ldo = c.vocab;
    launch_gemm(c.dtype, EPI_STORE, g, st);
}

static bool use_persistent(const ss_model *m, int R) { return m->persistent && m->mega_G > 0 && R <= m->mega_rows; }

extern "C" int ss_model_set_persistent(ss_model *m, int32_t on) {
    if (!m) return fail(SS_EINVAL, "ss_model_set_persistent: NULL model");
    if (on && m->mega_G <= 0) return fail(SS_EINVAL, "the persistent verify kernel is not available for this model on this device");
    m->persistent = on != 0;
    return SS_OK;
}

extern "C" int ss_model_set_persistent_options(ss_model *m, int32_t workgroups, int32_t data_sync) {
    if (!m) return fail(SS_EINVAL, "ss_model_set_persistent_options: NULL model");
    if (m->mega_G_max <= 0) return fail(SS_EINVAL, "the persistent verify kernel is not available for this model on this device");
    if (workgroups < 0 || workgroups > m->mega_G_max)
        return fail(SS_EINVAL, "ss_model_set_persistent_options: workgroups %d outside 0..%d", workgroups, m->mega_G_max);
    m->mega_G = workgroups ? workgroups : m->mega_G_max;
    m->data_sync = data_sync != 0;
    return SS_OK;
}

extern "C" int ss_model_set_timeline(ss_model *m, unsigned long long *buf_dev, size_t entries) {
    if (!m) return fail(SS_EINVAL, "ss_model_set_timeline: NULL model");
    m->timeline = buf_dev;
    m->timeline_entries = buf_dev ? entries : 0;
    return SS_OK;
}

extern "C" int ss_model_set_wait_limit(ss_model *m, uint32_t polls) {
    if (!m) return fail(SS_EINVAL, "ss_model_set_wait_limit: NULL model");
    if (polls < 1) return fail(SS_EINVAL, "ss_model_set_wait_limit: at least one poll");
    m->spin_limit = polls;
    return SS_OK;
}

// One launch of the persistent kernel: [embedding | given rows] -> layers -> [LM head] -> lengths += M.
static int run_persistent(ss_model *m, ss_kv_cache *kv, const int32_t *tokens, float *h, int batch, int M, float *logits,
                          int head_rows, int head_row0, int head_stride, hipStream_t st) {
    const ss_model_cfg &c = m->cfg;
    const size_t pl = (size_t)m->R16;
    MegaCall P{};
    const bool with_head = logits != nullptr;
    P.phases = with_head ? m->prog_full : m->prog_nohead;
    P.n_phases = with_head ? m->n_full : m->n_nohead;
    P.dtype = c.dtype;
    P.large_slab = mega_wants_large_slab(c.dtype, c.d_model, c.d_ff) ? 1 : 0;
    P.d = c.d_model; P.H = c.n_heads; P.hd = c.head_dim; P.F = c.d_ff; P.V = c.vocab;
    P.R = batch * M; P.B = batch; P.M = M;
    P.eps = c.rms_eps;
    P.tokens = tokens; P.embed = m->embed; P.h = h;
    P.act_a = ActDesc{m->act_a, pl * c.d_model, c.d_model};
    P.act_q = ActDesc{m->act_q, pl * m->W, m->W};
    P.act_o = ActDesc{m->act_o, pl * m->W, m->W};
    P.act_z = ActDesc{m->act_z, pl * c.d_ff, c.d_ff};
    P.act_a1 = ActDesc{m->act_a1, pl * c.d_model, c.d_model};
    P.nsq = m->nsq;
    // self-validating activations need every workgroup to own part of every GEMM phase (and the norm partials of at most 256)
    P.data_sync = m->data_sync && m->mega_G <= m->mega_min_units && m->mega_G <= 256;
    P.logits = logits; P.ldo = c.vocab; P.head_rows = head_rows; P.head_row0 = head_row0; P.head_stride = head_stride;
    P.kc = kv->k; P.vc = kv->v; P.layer_elems = kv->layer_elems; P.len = kv->len_dev; P.S = kv->S; P.max_pos = c.max_pos;
    P.rope = m->rope;
    int Lmax = 0;
    for (int b = 0; b < batch; ++b) Lmax = std::max(Lmax, kv->len_ub[b] + M);
    // One (sequence, head, split) unit per workgroup when possible.  Splitting the KV range costs a merge
    // through memory (about 3 us), which pays once a unit would otherwise walk more than ~400 positions;
    // from there on as many splits as there are idle workgroups is best (measured at 512, 1024 and 4000
    // positions: 8 splits beat 1, 2 and 4; below 300 positions one unit per head wins).
    const int fit = std::max(1, m->mega_G / (batch * c.n_heads));
    int nsplit = Lmax <= 384 ? 1 : std::max(1, std::min(std::min((Lmax + 127) / 128, fit), MAX_SPLITS));
    const int chunk = round_up((Lmax + nsplit - 1) / nsplit, 64);
    nsplit = (Lmax + chunk - 1) / chunk;
    P.nsplit = nsplit; P.chunk = chunk;
    P.part_o = m->part_o; P.part_m = m->part_m; P.part_l = m->part_l; P.attn_cnt = m->attn_cnt;
    P.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)c.head_dim));
    P.arrive = m->arrive; P.abort_flag = m->abort_flag; P.epoch_base = m->epoch;
    P.spin_limit = m->spin_limit;
    P.status = m->status;
    P.zeros = m->zeros;
    m->epoch += (unsigned)P.n_phases + 1;
    // development aid: device clock samples of every workgroup, into the caller's buffer when it is large enough
    if (m->timeline && m->timeline_entries >= (size_t)5 * P.n_phases * m->mega_G) P.timeline = m->timeline;
    {
        ProfScope ps(m, PT_PERSISTENT, st);
        hipError_t e = launch_mega(P, m->mega_G, st);
        if (e != hipSuccess) return fail(SS_EHIP, "persistent verify kernel launch: %s", hipGetErrorString(e));
    }
    for (int b = 0; b < batch; ++b) kv->len_ub[b] += M;
    return SS_OK;
}

extern "C" int ss_decoder_layers_forward(ss_model *m, ss_kv_cache *kv, float *h_dev, int32_t batch, int32_t M, ss_stream stream) {
    int rc = check_pair(m, kv, batch, M, "ss_decoder_layers_forward");
    if (rc) return rc;
    if (!h_dev) return fail(SS_EINVAL, "ss_decoder_layers_forward: h_dev is NULL");
    hipStream_t st = (hipStream_t)stream;
    if (use_persistent(m, batch * M)) {
        rc = run_persistent(m, kv, nullptr, h_dev, batch, M, nullptr, 0, 0, 1, st);
        return rc ? rc : check_launch();
    }
    const size_t bytes = sizeof(float) * (size_t)batch * M * m->cfg.d_model;
    HIP_TRY(hipMemcpyAsync(m->h, h_dev, bytes, hipMemcpyDeviceToDevice, st));
    run_layers(m, kv, batch, M, st);
    HIP_TRY(hipMemcpyAsync(h_dev, m->h, bytes, hipMemcpyDeviceToDevice, st));
    return check_launch();
}

extern "C" int ss_verify_forward(ss_model *m, ss_kv_cache *kv, const int32_t *tokens_dev, int32_t batch, int32_t M,
                                 float *logits_dev, ss_stream stream) {
    int rc = check_pair(m, kv, batch, M, "ss_verify_forward");
    if (rc) return rc;
    if (!tokens_dev) return fail(SS_EINVAL, "ss_verify_forward: tokens_dev is NULL");
    if (!m->embed || (logits_dev && (!m->lm_head || !m->gf))) return fail(SS_EINVAL, "ss_verify_forward: model has no embedding / LM head");
    hipStream_t st = (hipStream_t)stream;
    if (use_persistent(m, batch * M)) {
        rc = run_persistent(m, kv, tokens_dev, m->h, batch, M, logits_dev, batch * M, 0, 1, st);
        return rc ? rc : check_launch();
    }
    launch_embed(m->cfg.dtype, m->embed, tokens_dev, batch * M, m->cfg.d_model, m->cfg.vocab, m->h, m->status, st);
    run_layers(m, kv, batch, M, st);
    if (logits_dev) run_head(m, batch * M, 0, 1, logits_dev, st);
    return check_launch();
}

// top_p on the 2^-24 grid the filter works on; 0 = no filtering (top_p >= 1)
static int top_p_grid(float top_p, unsigned *P24, const char *who) {
    if (!(top_p > 0.f)) return fail(SS_EINVAL, "%s: top_p must be > 0 (>= 1 switches the filter off)", who);
    if (top_p >= 1.f) {
        *P24 = 0;
        return SS_OK;
    }
    const double g = std::nearbyint((double)top_p * 16777216.0); // to nearest, ties to even
    *P24 = g < 1.0 ? 1u : (g > 16777216.0 ? 16777216u : (unsigned)g);
    return SS_OK;
}

extern "C" int ss_top_p_filter(const float *probs_dev, int32_t rows, int32_t vocab, float top_p, float *out_dev, ss_stream stream) {
    if (!probs_dev || !out_dev) return fail(SS_EINVAL, "ss_top_p_filter: NULL argument");
    if (rows < 0 || vocab <= 0) return fail(SS_EINVAL, "ss_top_p_filter: bad shape");
    unsigned P24 = 0;
    int rc = top_p_grid(top_p, &P24, "ss_top_p_filter");
    if (rc) return rc;
    if (rows == 0) return SS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (P24 == 0) {
        if (out_dev != probs_dev) HIP_TRY(hipMemcpyAsync(out_dev, probs_dev, sizeof(float) * (size_t)rows * vocab, hipMemcpyDeviceToDevice, st));
        return SS_OK;
    }
    launch_top_p_filter(probs_dev, vocab, rows, vocab, P24, out_dev, vocab, st);
    return check_launch();
}

// top_k as the filter takes it: 0 = no filtering (0 and >= vocab switch it off)
static int top_k_arg(int32_t top_k, int vocab, int *k, const char *who) {
    if (top_k < 0) return fail(SS_EINVAL, "%s: top_k must be >= 0 (0 and >= vocab switch the filter off)", who);
    *k = top_k >= vocab ? 0 : top_k;
    return SS_OK;
}

extern "C" int ss_top_k_filter(const float *probs_dev, int32_t rows, int32_t vocab, int32_t top_k, float *out_dev, ss_stream stream) {
    if (!probs_dev || !out_dev) return fail(SS_EINVAL, "ss_top_k_filter: NULL argument");
    if (rows < 0 || vocab <= 0) return fail(SS_EINVAL, "ss_top_k_filter: bad shape");
    if (top_k < 1) return fail(SS_EINVAL, "ss_top_k_filter: top_k must be >= 1 (>= vocab copies the rows unchanged)");
    if (rows == 0) return SS_OK;
    hipStream_t st = (hipStream_t)stream;
    if (top_k >= vocab) {
        if (out_dev != probs_dev) HIP_TRY(hipMemcpyAsync(out_dev, probs_dev, sizeof(float) * (size_t)rows * vocab, hipMemcpyDeviceToDevice, st));
        return SS_OK;
    }
    launch_top_k_filter(probs_dev, vocab, rows, vocab, top_k, out_dev, vocab, st);
    return check_launch();
}

extern "C" int ss_draft_step(ss_model *m, ss_kv_cache *kv, const int32_t *tokens_dev, int32_t batch, int32_t mrows,
                             float temperature, float top_p, int32_t top_k, const float *u_dev, float *q_rows_dev, int64_t ldq,
                             int32_t *token_out_dev, ss_stream stream) {
    int rc = check_pair(m, kv, batch, mrows, "ss_draft_step");
    if (rc) return rc;
    unsigned P24 = 0;
    rc = top_p_grid(top_p, &P24, "ss_draft_step");
    if (rc) return rc;
    int kk = 0;
    rc = top_k_arg(top_k, m->cfg.vocab, &kk, "ss_draft_step");
    if (rc) return rc;
    if (!tokens_dev || !token_out_dev) return fail(SS_EINVAL, "ss_draft_step: NULL argument");
    if (!m->embed || !m->lm_head || !m->gf) return fail(SS_EINVAL, "ss_draft_step: model has no embedding / LM head");
    if (!(temperature >= 0.f)) return fail(SS_EINVAL, "ss_draft_step: temperature must be >= 0");
    if (temperature > 0.f && (!u_dev || !q_rows_dev || ldq < m->cfg.vocab)) return fail(SS_EINVAL, "ss_draft_step: sampling needs u_dev, q_rows_dev and ldq >= vocab");
    hipStream_t st = (hipStream_t)stream;
    const int V = m->cfg.vocab;
    if (use_persistent(m, batch * mrows)) {
        rc = run_persistent(m, kv, tokens_dev, m->h, batch, mrows, m->logits_ws, batch, mrows - 1, mrows, st);
        if (rc) return rc;
    } else {
        launch_embed(m->cfg.dtype, m->embed, tokens_dev, batch * mrows, m->cfg.d_model, V, m->h, m->status, st);
        run_layers(m, kv, batch, mrows, st);
        run_head(m, batch, mrows - 1, mrows, m->logits_ws, st);
    }
    if (temperature > 0.f) {
        const float inv_t = 1.0f / temperature;
        launch_row_stats(m->logits_ws, batch, V, inv_t, m->stats_ws, m->stats_cnt, m->stats_part, st);
        launch_softmax_write(m->logits_ws, batch, V, inv_t, m->stats_ws, q_rows_dev, ldq, st);
        if (kk) launch_top_k_filter(q_rows_dev, ldq, batch, V, kk, q_rows_dev, ldq, st); // top-k first, top-p on its output
        if (P24) launch_top_p_filter(q_rows_dev, ldq, batch, V, P24, q_rows_dev, ldq, st);
        launch_sample_rows(q_rows_dev, ldq, batch, V, u_dev, token_out_dev, st);
    } else {
        launch_argmax_rows(m->logits_ws, V, batch, V, token_out_dev, st);
    }
    return check_launch();
}

// ------------------------------------------------------------------------------------------ softmax / accept

// Workspace of the softmax / accept entry points (row statistics, per-segment sums, row argmax, status word): device
// memory of the caller (or of a model, for ss_speculative_step), cleared once by ss_workspace_init.
// Layout: [0, 256) device status word; [256, SCR_DATA) arrival counters of the segmented row statistics, a
// zone no call uses for anything else, so that they are zero whenever a launch starts (the kernels leave
// them zero); [SCR_DATA, ...) per-call data.
constexpr size_t SCR_CNT_ROWS = 16384, SCR_DATA = 256 + sizeof(unsigned) * SCR_CNT_ROWS;
static unsigned *scr_cnt(void *ws) { return (unsigned *)((char *)ws + 256); }
static void *scr_data(void *ws) { return (char *)ws + SCR_DATA; }

// rows per launch of the row statistics: the counter zone, and the grid's y extent
static size_t stats_rows_per_launch(int V) { return row_stats_segments(V) > 1 ? SCR_CNT_ROWS : (size_t)65535; }

// what each call keeps behind SCR_DATA
static size_t softmax_need(size_t rows, int V) {
    return SCR_DATA + sizeof(float2) * rows + row_stats_partial_bytes((int)std::min(rows, stats_rows_per_launch(V)), V) + 16;
}
static size_t accept_need(int B, int V) { return SCR_DATA + accept_workspace_bytes(B, V) + 16; }
static size_t accept_logits_need(int B, int K, int V) {
    const size_t rows = (size_t)B * (2 * K + 1);
    return SCR_DATA + sizeof(float2) * rows + ((accept_workspace_bytes(B, V) + 15) & ~(size_t)15) +
           row_stats_partial_bytes((int)std::min(rows, stats_rows_per_launch(V)), V) + 16;
}
static size_t greedy_need(int B, int K) { return SCR_DATA + sizeof(int32_t) * (size_t)B * (K + 1) + 16; }

extern "C" size_t ss_workspace_bytes(int64_t rows, int32_t vocab) {
    if (rows < 0 || vocab <= 0) return 0;
    const size_t r = (size_t)std::max<int64_t>(rows, 1);
    // an upper bound of the four calls' needs when they touch `rows` rows in total (a batch is at most `rows` sequences)
    const size_t acc = sizeof(unsigned long long) * r * 16; // per-segment sums of the rejection step: at most 16 segments per sequence
    return SCR_DATA + sizeof(float2) * r + ((acc + 15) & ~(size_t)15) + row_stats_partial_bytes((int)std::min(r, stats_rows_per_launch(vocab)), vocab) +
           sizeof(int32_t) * r + 64;
}

static int check_ws(const void *ws, size_t have, size_t need, const char *who) {
    if (!ws) return fail(SS_EINVAL, "%s: ws_dev is NULL", who);
    if ((uintptr_t)ws & 15) return fail(SS_EINVAL, "%s: the workspace must be 16-byte aligned", who);
    if (have < need) return fail(SS_ECAPACITY, "%s: the workspace has %zu bytes, this call needs %zu (ss_workspace_bytes)", who, have, need);
    return SS_OK;
}

extern "C" int ss_workspace_init(void *ws_dev, size_t ws_bytes, ss_stream stream) {
    int rc = check_ws(ws_dev, ws_bytes, SCR_DATA, "ss_workspace_init");
    if (rc) return rc;
    launch_fill_u32((uint32_t *)ws_dev, ws_bytes / 4, 0u, (hipStream_t)stream);
    return check_launch();
}

extern "C" int ss_workspace_status(void *ws_dev, size_t ws_bytes, ss_stream stream, int32_t *status_host) {
    int rc = check_ws(ws_dev, ws_bytes, SCR_DATA, "ss_workspace_status");
    if (rc) return rc;
    if (!status_host) return fail(SS_EINVAL, "ss_workspace_status: status_host is NULL");
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(hipMemcpyAsync(status_host, ws_dev, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (*status_host) launch_fill_u32((uint32_t *)ws_dev, 1, 0u, st);
    return check_launch();
}

// statistics of `rows` rows with the workspace's counters; part: room for stats_rows_per_launch(V) rows
static void stats_rows(const float *logits, size_t rows, int V, float inv_t, float2 *stats, void *ws, float2 *part, hipStream_t st) {
    const size_t step = stats_rows_per_launch(V);
    for (size_t r0 = 0; r0 < rows; r0 += step)
        launch_row_stats(logits + r0 * (size_t)V, (int)std::min(step, rows - r0), V, inv_t, stats + r0, scr_cnt(ws), part, st);
}

extern "C" int ss_softmax(const float *logits_dev, int32_t rows, int32_t vocab, float temperature, float *probs_dev,
                          void *ws, size_t ws_bytes, ss_stream stream) {
    if (!logits_dev || !probs_dev) return fail(SS_EINVAL, "ss_softmax: NULL argument");
    if (rows < 0 || vocab <= 0 || !(temperature > 0.f)) return fail(SS_EINVAL, "ss_softmax: bad rows/vocab/temperature");
    int rc = check_ws(ws, ws_bytes, softmax_need((size_t)rows, vocab), "ss_softmax");
    if (rc) return rc;
    hipStream_t st = (hipStream_t)stream;
    const float inv_t = 1.0f / temperature;
    float2 *stats = (float2 *)scr_data(ws);
    stats_rows(logits_dev, (size_t)rows, vocab, inv_t, stats, ws, stats + rows, st);
    launch_softmax_write(logits_dev, rows, vocab, inv_t, stats, probs_dev, vocab, st);
    return check_launch();
}

static int check_accept(const void *p, const void *q, const void *d, const void *u, int B, int K, int V, const void *na,
                        const void *nx, const char *who) {
    if (B < 0 || K < 0 || V <= 0) return fail(SS_EINVAL, "%s: bad batch/K/vocab", who);
    if (K > SS_MAX_ROWS_PER_SEQ - 1) return fail(SS_EINVAL, "%s: K must be <= %d", who, SS_MAX_ROWS_PER_SEQ - 1);
    if (!p || !u || !na || !nx || (K > 0 && (!q || !d))) return fail(SS_EINVAL, "%s: NULL argument", who);
    return SS_OK;
}

// the rejection step on materialised probabilities; status: device status word, partial: accept_workspace_bytes(B, V) bytes
static void accept_probs(const float *p, const float *q, const int32_t *d, const float *u, int B, int K, int V, int32_t *na, int32_t *nx,
                         int32_t *status, unsigned long long *partial, hipStream_t st) {
    AcceptArgs a{};
    a.p = p; a.q = q; a.from_logits = 0; a.inv_t = 1.f;
    a.draft = d; a.u = u; a.B = B; a.K = K; a.V = V;
    a.n_accepted = na; a.next_token = nx; a.status = status;
    launch_accept(a, partial, st);
}

extern "C" int ss_speculative_accept(const float *p_dev, const float *q_dev, const int32_t *draft_tokens_dev,
                                     const float *uniforms_dev, int32_t batch, int32_t K, int32_t vocab,
                                     int32_t *n_accepted_dev, int32_t *next_token_dev, void *ws, size_t ws_bytes, ss_stream stream) {
    int rc = check_accept(p_dev, q_dev, draft_tokens_dev, uniforms_dev, batch, K, vocab, n_accepted_dev, next_token_dev, "ss_speculative_accept");
    if (rc) return rc;
    rc = check_ws(ws, ws_bytes, accept_need(batch, vocab), "ss_speculative_accept");
    if (rc) return rc;
    accept_probs(p_dev, q_dev, draft_tokens_dev, uniforms_dev, batch, K, vocab, n_accepted_dev, next_token_dev, (int32_t *)ws,
                 (unsigned long long *)scr_data(ws), (hipStream_t)stream);
    return check_launch();
}

extern "C" int ss_speculative_accept_logits(const float *p_logits_dev, const float *q_logits_dev, float temperature,
                                            const int32_t *draft_tokens_dev, const float *uniforms_dev, int32_t batch,
                                            int32_t K, int32_t vocab, int32_t *n_accepted_dev, int32_t *next_token_dev,
                                            float *p_out_dev, float *q_out_dev, void *ws, size_t ws_bytes, ss_stream stream) {
    int rc = check_accept(p_logits_dev, q_logits_dev, draft_tokens_dev, uniforms_dev, batch, K, vocab, n_accepted_dev, next_token_dev, "ss_speculative_accept_logits");
    if (rc) return rc;
    if (!(temperature > 0.f)) return fail(SS_EINVAL, "ss_speculative_accept_logits: temperature must be > 0");
    rc = check_ws(ws, ws_bytes, accept_logits_need(batch, K, vocab), "ss_speculative_accept_logits");
    if (rc) return rc;
    const size_t np = (size_t)batch * (K + 1), nq = (size_t)batch * K;
    hipStream_t st = (hipStream_t)stream;
    float2 *ps = (float2 *)scr_data(ws), *qs = ps + np;
    unsigned long long *partial = (unsigned long long *)(qs + nq);
    float2 *part = (float2 *)((char *)partial + ((accept_workspace_bytes(batch, vocab) + 15) & ~(size_t)15));
    const float inv_t = 1.0f / temperature;
    AcceptArgs a{};
    a.p = p_logits_dev; a.q = q_logits_dev; a.p_stats = ps; a.q_stats = qs; a.from_logits = 1; a.inv_t = inv_t;
    a.draft = draft_tokens_dev; a.u = uniforms_dev; a.B = batch; a.K = K; a.V = vocab;
    a.n_accepted = n_accepted_dev; a.next_token = next_token_dev; a.status = (int32_t *)ws;
    // Rows behind a sequence's first rejection are never used by the method (Section 3).  When the logits
    // are large enough for their streaming to dominate and nobody asked for the materialised softmax,
    // the statistics are taken in stages that skip those rows; otherwise every row is covered.
    const bool one_launch = np + nq <= stats_rows_per_launch(vocab);
    const bool staged = !p_out_dev && !q_out_dev && K >= 3 && one_launch && (np + nq) * (size_t)vocab * sizeof(float) >= ((size_t)32 << 20);
    if (staged) {
        launch_row_stats_staged(a, ps, qs, scr_cnt(ws), part, st);
    } else if (one_launch) {
        launch_row_stats2(p_logits_dev, (int)np, ps, q_logits_dev, (int)nq, qs, vocab, inv_t, scr_cnt(ws), part, st);
    } else {
        stats_rows(p_logits_dev, np, vocab, inv_t, ps, ws, part, st);
        stats_rows(q_logits_dev, nq, vocab, inv_t, qs, ws, part, st);
    }
    launch_accept(a, partial, st);
    if (p_out_dev) launch_softmax_write(p_logits_dev, (int)np, vocab, inv_t, ps, p_out_dev, vocab, st);
    if (q_out_dev) launch_softmax_write(q_logits_dev, (int)nq, vocab, inv_t, qs, q_out_dev, vocab, st);
    return check_launch();
}

extern "C" int ss_greedy_accept(const float *p_logits_dev, const int32_t *draft_tokens_dev, int32_t batch, int32_t K,
                                int32_t vocab, int32_t *n_accepted_dev, int32_t *next_token_dev, void *ws, size_t ws_bytes, ss_stream stream) {
    if (batch < 0 || K < 0 || K > SS_MAX_ROWS_PER_SEQ - 1 || vocab <= 0) return fail(SS_EINVAL, "ss_greedy_accept: bad batch/K/vocab");
    if (!p_logits_dev || !n_accepted_dev || !next_token_dev || (K > 0 && !draft_tokens_dev)) return fail(SS_EINVAL, "ss_greedy_accept: NULL argument");
    int rc = check_ws(ws, ws_bytes, greedy_need(batch, K), "ss_greedy_accept");
    if (rc) return rc;
    launch_greedy_accept(p_logits_dev, draft_tokens_dev, batch, K, vocab, (int32_t *)scr_data(ws), n_accepted_dev, next_token_dev, (hipStream_t)stream);
    return check_launch();
}

// ------------------------------------------------------------------------------------------ rejection step without a workspace argument

// Scratch of ss_speculative_accept_noalloc: the status word ([0, 256)) and the per-segment weight sums of the
// rejection step, in a device array that is part of the library's code object (every device the library runs
// on holds its own copy at its own address until the process ends).  In host code the array's name is only a
// handle for hipGetSymbolAddress: the address the kernels get is the one that call returns, kept per device.
constexpr size_t NOALLOC_SCRATCH_BYTES = 64 * 1024;
static __device__ __align__(256) unsigned char noalloc_scratch[NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static std::mutex g_noalloc_mu;
static void *g_noalloc_ptr[NOALLOC_MAX_DEVICES];

// device address of the scratch array on the current device (resolved once per device)
static int noalloc_scratch_ptr(void **out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return fail(SS_EINVAL, "ss_speculative_accept_noalloc: device index %d is not supported", dev);
    std::lock_guard<std::mutex> lk(g_noalloc_mu);
    if (!g_noalloc_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(noalloc_scratch)));
        if (!p) return fail(SS_EHIP, "ss_speculative_accept_noalloc: the scratch array has no address on device %d", dev);
        g_noalloc_ptr[dev] = p;
    }
    *out = g_noalloc_ptr[dev];
    return SS_OK;
}

extern "C" int ss_freeze_allocations(int32_t on) {
    if (on) {
        // set-up that a later call would otherwise do on its first use: the built-in scratch array is given its
        // address on the current device now (loading the code object that holds it is what takes device memory)
        void *scratch = nullptr;
        int rc = noalloc_scratch_ptr(&scratch);
        if (rc) return rc;
    }
    g_alloc_frozen.store(on != 0);
    return SS_OK;
}

extern "C" int ss_speculative_accept_noalloc(const float *p_dev, const float *q_dev, const int32_t *draft_tokens_dev,
                                             const float *uniforms_dev, int32_t batch, int32_t K, int32_t vocab,
                                             int32_t *n_accepted_dev, int32_t *next_token_dev, int32_t *status_dev, ss_stream stream) {
    int rc = check_accept(p_dev, q_dev, draft_tokens_dev, uniforms_dev, batch, K, vocab, n_accepted_dev, next_token_dev, "ss_speculative_accept_noalloc");
    if (rc) return rc;
    const size_t need = 256 + accept_workspace_bytes(batch, vocab);
    if (need > NOALLOC_SCRATCH_BYTES)
        return fail(SS_ECAPACITY, "ss_speculative_accept_noalloc: batch %d at vocabulary %d needs %zu bytes of scratch, the built-in array has %zu "
                    "(use ss_speculative_accept with a workspace)", batch, vocab, need, NOALLOC_SCRATCH_BYTES);
    void *scratch = nullptr;
    rc = noalloc_scratch_ptr(&scratch);
    if (rc) return rc;
    // nothing here has to start at zero: every per-segment sum the finish kernel reads is written by this call's first
    // kernel, and the status word only ever accumulates flags
    accept_probs(p_dev, q_dev, draft_tokens_dev, uniforms_dev, batch, K, vocab, n_accepted_dev, next_token_dev,
                 status_dev ? status_dev : (int32_t *)scratch, (unsigned long long *)((char *)scratch + 256), (hipStream_t)stream);
    return check_launch();
}

// ------------------------------------------------------------------------------------------ one speculative step

extern "C" int ss_speculative_step(ss_model *target, ss_kv_cache *tkv, ss_model *draft, ss_kv_cache *dkv, int32_t K,
                                   float temperature, float top_p, int32_t top_k, int32_t *feed_dev, int32_t *n_feed, const float *u_draft_dev,
                                   const float *u_accept_dev, int32_t *vt, float *q_rows_dev, float *logits_dev, float *p_dev,
                                   int32_t *result_dev, int32_t *out_host, ss_stream stream) {
    if (!target || !tkv || !draft || !dkv || !feed_dev || !n_feed || !vt || !logits_dev || !result_dev || !out_host)
        return fail(SS_EINVAL, "ss_speculative_step: NULL argument");
    if (K < 1 || K > SS_MAX_ROWS_PER_SEQ - 1) return fail(SS_EINVAL, "ss_speculative_step: K must be in [1, %d]", SS_MAX_ROWS_PER_SEQ - 1);
    const bool shared = dkv == tkv; // the draft works in the leading layers of the target's cache
    if (*n_feed != 1 && *n_feed != 2) return fail(SS_EINVAL, "ss_speculative_step: *n_feed must be 1 or 2");
    if (shared && *n_feed != 1) return fail(SS_EINVAL, "ss_speculative_step: a shared cache never needs a two-token feed");
    if (tkv->B != 1 || dkv->B != 1) return fail(SS_EINVAL, "ss_speculative_step: one sequence per cache");
    if (target->cfg.vocab != draft->cfg.vocab) return fail(SS_EINVAL, "ss_speculative_step: the two models have different vocabularies");
    if (!(temperature >= 0.f)) return fail(SS_EINVAL, "ss_speculative_step: temperature must be >= 0");
    unsigned P24 = 0;
    if (int rc0 = top_p_grid(top_p, &P24, "ss_speculative_step")) return rc0;
    int kk = 0;
    if (int rc0 = top_k_arg(top_k, target->cfg.vocab, &kk, "ss_speculative_step")) return rc0;
    const bool sample = temperature > 0.f;
    if (sample && (!u_draft_dev || !u_accept_dev || !q_rows_dev || !p_dev)) return fail(SS_EINVAL, "ss_speculative_step: sampling needs uniforms, q_rows_dev and p_dev");
    hipStream_t st = (hipStream_t)stream;
    const int V = target->cfg.vocab, M = K + 1;
    // everything the calls below would refuse is refused here, before the first of them changes a cache
    int rc = check_pair(target, tkv, 1, M, "ss_speculative_step (target)");
    if (rc) return rc;
    rc = check_pair(draft, dkv, 1, *n_feed, "ss_speculative_step (draft)");
    if (rc) return rc;
    const int draft_rows = *n_feed + K - 1;
    if (dkv->len_ub[0] + draft_rows > dkv->max_seq || dkv->len_ub[0] + draft_rows > draft->cfg.max_pos)
        return fail(SS_ECAPACITY, "ss_speculative_step: the draft cache at length <= %d has no room for %d rows (max_seq %d, max_pos %d)",
                    dkv->len_ub[0], draft_rows, dkv->max_seq, draft->cfg.max_pos);
    const int t_len0 = tkv->len_ub[0], d_len0 = dkv->len_ub[0];
    for (int i = 0; i < K; ++i) {
        rc = ss_draft_step(draft, dkv, i ? vt + i : feed_dev, 1, i ? 1 : *n_feed, temperature, top_p, top_k, sample ? u_draft_dev + i : nullptr,
                           sample ? q_rows_dev + (size_t)i * V : nullptr, V, vt + i + 1, stream);
        if (rc) return rc;
    }
    HIP_TRY(hipMemcpyAsync(vt, feed_dev + (*n_feed - 1), sizeof(int32_t), hipMemcpyDeviceToDevice, st)); // the last committed token
    if (shared) { // the K positions the draft appended are rewritten, for every layer, by the verify pass
        launch_len_add(tkv->len_dev, 1, -K, st);
        tkv->len_ub[0] -= K;
    }
    rc = ss_verify_forward(target, tkv, vt, 1, M, logits_dev, stream);
    if (rc) return rc;
    // the softmax and the rejection step work in the target model's own workspace
    if (sample) {
        rc = ss_softmax(logits_dev, M, V, temperature, p_dev, target->ws, target->ws_bytes, stream);
        if (rc) return rc;
        if (kk) launch_top_k_filter(p_dev, V, M, V, kk, p_dev, V, st); // the draft's rows were filtered by its own calls
        if (P24) launch_top_p_filter(p_dev, V, M, V, P24, p_dev, V, st);
        rc = ss_speculative_accept(p_dev, q_rows_dev, vt + 1, u_accept_dev, 1, K, V, result_dev, result_dev + 1, target->ws, target->ws_bytes, stream);
    } else {
        rc = ss_greedy_accept(logits_dev, vt + 1, 1, K, V, result_dev, result_dev + 1, target->ws, target->ws_bytes, stream);
    }
    if (rc) return rc;
    launch_len_rollback(tkv->len_dev, result_dev, 1, M, st);
    if (!shared) launch_len_rollback(dkv->len_dev, result_dev, 1, K, st); // a == K leaves the draft cache one row short of the target's
    HIP_TRY(hipMemcpyAsync(out_host, result_dev, 2 * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(out_host + 2, vt + 1, K * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    // the abort flags of the persistent kernel travel with the result: a wait that gave up must not go unnoticed
    unsigned ab[2] = {0u, 0u};
    if (target->abort_flag) HIP_TRY(hipMemcpyAsync(&ab[0], target->abort_flag, sizeof(unsigned), hipMemcpyDeviceToHost, st));
    if (draft->abort_flag && draft != target) HIP_TRY(hipMemcpyAsync(&ab[1], draft->abort_flag, sizeof(unsigned), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (ab[0] | ab[1]) {
        int32_t dummy = 0;
        if (ab[0]) (void)ss_device_status(target, stream, &dummy); // resets the synchronisation state
        if (ab[1]) (void)ss_device_status(draft, stream, &dummy);
        const int32_t tl = t_len0, dl = d_len0;
        (void)ss_kv_cache_set_len(tkv, &tl, stream);
        if (!shared) (void)ss_kv_cache_set_len(dkv, &dl, stream);
        return fail(SS_EABORTED, "ss_speculative_step: a bounded wait of the persistent kernel gave up (%s model); cache lengths restored",
                    ab[0] ? "target" : "draft");
    }
    const int a = std::min(std::max(out_host[0], 0), K);
    tkv->len_ub[0] -= M - 1 - a;
    if (!shared) dkv->len_ub[0] -= K - 1 - std::min(a, K - 1);
    // the next step's draft feed: [y], or [d_K, y] after a fully accepted step of the two-cache scheme
    if (a < K || shared) {
        HIP_TRY(hipMemcpyAsync(feed_dev, result_dev + 1, sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        *n_feed = 1;
    } else {
        HIP_TRY(hipMemcpyAsync(feed_dev, vt + K, sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        HIP_TRY(hipMemcpyAsync(feed_dev + 1, result_dev + 1, sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        *n_feed = 2;
    }
    return check_launch();
}

// ------------------------------------------------------------------------------------------ one speculative step, many sequences

extern "C" int ss_speculative_step_batched(ss_model *target, ss_kv_cache *tkv, ss_model *draft, ss_kv_cache *dkv, int32_t batch, int32_t K,
                                           float temperature, float top_p, int32_t top_k, int32_t *feed_dev, const float *u_draft_dev,
                                           const float *u_accept_dev, int32_t *draft_tokens_dev, int32_t *vt, float *q_rows_dev,
                                           float *logits_dev, float *p_dev, int32_t *result_dev, int32_t *out_host, ss_stream stream) {
    if (!target || !tkv || !draft || !dkv || !feed_dev || !draft_tokens_dev || !vt || !logits_dev || !result_dev || !out_host)
        return fail(SS_EINVAL, "ss_speculative_step_batched: NULL argument");
    if (K < 1 || K > SS_MAX_ROWS_PER_SEQ - 1) return fail(SS_EINVAL, "ss_speculative_step_batched: K must be in [1, %d]", SS_MAX_ROWS_PER_SEQ - 1);
    if (dkv == tkv) return fail(SS_EINVAL, "ss_speculative_step_batched: two caches (the shared-cache scheme is single-sequence)");
    if (batch < 1 || tkv->B != batch || dkv->B != batch) return fail(SS_EINVAL, "ss_speculative_step_batched: both caches must hold `batch` sequences");
    if (target->cfg.vocab != draft->cfg.vocab) return fail(SS_EINVAL, "ss_speculative_step_batched: the two models have different vocabularies");
    if (!(temperature >= 0.f)) return fail(SS_EINVAL, "ss_speculative_step_batched: temperature must be >= 0");
    unsigned P24 = 0;
    if (int rc0 = top_p_grid(top_p, &P24, "ss_speculative_step_batched")) return rc0;
    int kk = 0;
    if (int rc0 = top_k_arg(top_k, target->cfg.vocab, &kk, "ss_speculative_step_batched")) return rc0;
    const bool sample = temperature > 0.f;
    if (sample && (!u_draft_dev || !u_accept_dev || !q_rows_dev || !p_dev)) return fail(SS_EINVAL, "ss_speculative_step_batched: sampling needs uniforms, q_rows_dev and p_dev");
    hipStream_t st = (hipStream_t)stream;
    const int V = target->cfg.vocab, M = K + 1;
    // everything the calls below would refuse is refused here, before the first of them changes a cache
    int rc = check_pair(target, tkv, batch, M, "ss_speculative_step_batched (target)");
    if (rc) return rc;
    rc = check_pair(draft, dkv, batch, 2, "ss_speculative_step_batched (draft)");
    if (rc) return rc;
    for (int b = 0; b < batch; ++b)
        if (dkv->len_ub[b] + M > dkv->max_seq || dkv->len_ub[b] + M > draft->cfg.max_pos)
            return fail(SS_ECAPACITY, "ss_speculative_step_batched: the draft cache of sequence %d at length <= %d has no room for %d rows (max_seq %d, max_pos %d)",
                        b, dkv->len_ub[b], M, dkv->max_seq, draft->cfg.max_pos);
    if (ss_workspace_bytes((int64_t)batch * (2 * K + 1), V) > target->ws_bytes)
        return fail(SS_ECAPACITY, "ss_speculative_step_batched: the target model's workspace (sized for max_rows) is too small for %d sequences", batch);
    const std::vector<int32_t> t_len0 = tkv->len_ub, d_len0 = dkv->len_ub;
    int32_t *dbk = draft_tokens_dev + (size_t)K * batch; // the draft's tokens, sequence-major
    for (int i = 0; i < K; ++i) {
        rc = ss_draft_step(draft, dkv, i ? draft_tokens_dev + (size_t)(i - 1) * batch : feed_dev, batch, i ? 1 : 2, temperature, top_p, top_k,
                           sample ? u_draft_dev + (size_t)i * batch : nullptr, sample ? q_rows_dev + (size_t)i * V : nullptr, (int64_t)K * V,
                           draft_tokens_dev + (size_t)i * batch, stream);
        if (rc) return rc;
    }
    launch_step_pack_tokens(feed_dev, draft_tokens_dev, batch, K, vt, dbk, st);
    rc = ss_verify_forward(target, tkv, vt, batch, M, logits_dev, stream);
    if (rc) return rc;
    if (sample) {
        rc = ss_softmax(logits_dev, batch * M, V, temperature, p_dev, target->ws, target->ws_bytes, stream);
        if (rc) return rc;
        if (kk) launch_top_k_filter(p_dev, V, batch * M, V, kk, p_dev, V, st); // the draft's rows were filtered by its own calls
        if (P24) launch_top_p_filter(p_dev, V, batch * M, V, P24, p_dev, V, st);
        rc = ss_speculative_accept(p_dev, q_rows_dev, dbk, u_accept_dev, batch, K, V, result_dev, result_dev + batch, target->ws, target->ws_bytes, stream);
    } else {
        rc = ss_greedy_accept(logits_dev, dbk, batch, K, V, result_dev, result_dev + batch, target->ws, target->ws_bytes, stream);
    }
    if (rc) return rc;
    // both caches grew by K + 1 rows per sequence and keep a_b + 1 of them: the target then holds n'_b - 1 positions, the draft n'_b - 2
    launch_len_rollback(tkv->len_dev, result_dev, batch, M, st);
    launch_len_rollback(dkv->len_dev, result_dev, batch, M, st);
    launch_step_next_feed(vt, result_dev, result_dev + batch, batch, K, feed_dev, st);
    std::vector<int32_t> res(2 * (size_t)batch), dt((size_t)batch * K);
    HIP_TRY(hipMemcpyAsync(res.data(), result_dev, res.size() * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipMemcpyAsync(dt.data(), dbk, dt.size() * sizeof(int32_t), hipMemcpyDeviceToHost, st));
    unsigned ab[2] = {0u, 0u};
    if (target->abort_flag) HIP_TRY(hipMemcpyAsync(&ab[0], target->abort_flag, sizeof(unsigned), hipMemcpyDeviceToHost, st));
    if (draft->abort_flag && draft != target) HIP_TRY(hipMemcpyAsync(&ab[1], draft->abort_flag, sizeof(unsigned), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (ab[0] | ab[1]) {
        int32_t dummy = 0;
        if (ab[0]) (void)ss_device_status(target, stream, &dummy); // resets the synchronisation state
        if (ab[1]) (void)ss_device_status(draft, stream, &dummy);
        (void)ss_kv_cache_set_len(tkv, t_len0.data(), stream);
        (void)ss_kv_cache_set_len(dkv, d_len0.data(), stream);
        return fail(SS_EABORTED, "ss_speculative_step_batched: a bounded wait of the persistent kernel gave up (%s model); cache lengths restored, the feed is stale",
                    ab[0] ? "target" : "draft");
    }
    for (int b = 0; b < batch; ++b) {
        const int a = std::min(std::max(res[b], 0), K);
        tkv->len_ub[b] -= K - a;
        dkv->len_ub[b] -= K - a;
        int32_t *o = out_host + (size_t)b * (K + 2);
        o[0] = a;
        o[1] = res[batch + b];
        for (int i = 0; i < K; ++i) o[2 + i] = dt[(size_t)b * K + i];
    }
    return check_launch();
}

// ------------------------------------------------------------------------------------------ shutdown

extern "C" int ss_shutdown(void) {
    std::set<ss_model *> models;
    std::set<ss_kv_cache *> caches;
    {
        std::lock_guard<std::mutex> lk(g_reg_mu);
        models.swap(g_models);
        caches.swap(g_caches);
    }
    if (models.empty() && caches.empty()) return SS_OK;
    (void)hipDeviceSynchronize();
    for (ss_kv_cache *kv : caches) cache_release(kv);
    for (ss_model *m : models) model_release(m);
    return SS_OK;
}
