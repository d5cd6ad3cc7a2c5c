// C ABI of the RPO suffix-rollout library: handles, argument checks, and the
// launch sequences of prefill, fork, decode and the teacher-forced log-prob pass.
// Host code only; every kernel lives in the other translation units.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/rpo.h"
#include "../../include/rpo_kernels.h"
#include "kernels.hpp"

using namespace rpo;

// ---------------------------------------------------------------------------
// errors
// ---------------------------------------------------------------------------
static thread_local char g_err[512] = "";
static int g_kernel_path = 0;  // 0 = pick the fastest kernel, 1 = generic kernels only

static int fail(int code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
#define HIP_TRY(expr)                                                                         \
    do {                                                                                      \
        hipError_t e_ = (expr);                                                               \
        if (e_ != hipSuccess)                                                                 \
            return fail(RPO_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, \
                        __LINE__);                                                            \
    } while (0)

extern "C" const char* rpo_last_error(void) { return g_err; }

extern "C" int rpo_probe_peaks(const void* src_dev, void* dst_dev, size_t bytes, float* scratch_dev,
                               double* copy_gbps, double* mfma_tflops, void* stream) {
    if (!src_dev || !dst_dev || !scratch_dev || !copy_gbps || !mfma_tflops)
        return fail(RPO_EINVAL, "rpo_probe_peaks: NULL argument");
    if (bytes < ((size_t)1 << 20) || bytes % 16 != 0)
        return fail(RPO_EINVAL, "rpo_probe_peaks: bytes must be a multiple of 16 and at least 1 MiB");
    HIP_TRY(probe_copy(src_dev, dst_dev, bytes, 3, copy_gbps, (hipStream_t)stream));
    HIP_TRY(probe_mfma(scratch_dev, 300000, 2, mfma_tflops, (hipStream_t)stream));
    return RPO_OK;
}

extern "C" int rpo_set_kernel_path(int path) {
    if (path != 0 && path != 1 && path != 2 && path != 17 && !(path >= 19 && path <= 22) && path != 27 && path != 29)
        return fail(RPO_EINVAL, "kernel path must be 0, 1, 2, 17, 19..22, 27 or 29");
    g_kernel_path = path;
    return RPO_OK;
}

// ---------------------------------------------------------------------------
// per-kernel timing: HIP event pairs around the launches of chosen kernels
// ---------------------------------------------------------------------------
namespace {
struct Profile {
    bool on = false;
    std::vector<hipEvent_t> events;  // pool, reused across sessions
    size_t used = 0;
    double flops = 0.0, bytes = 0.0;
    int every = 1;      // time every n-th launch of the kernel only
    int64_t seen = 0;   // launches of the kernel since rpo_profile_start
    hipError_t mark(hipStream_t s) {
        if (used == events.size()) {
            hipEvent_t e;
            hipError_t r = hipEventCreate(&e);
            if (r != hipSuccess) return r;
            events.push_back(e);
        }
        return hipEventRecord(events[used++], s);
    }
};
Profile g_prof[kKidCount];  // one slot per kernel id; several may be active at once

// Runs `launch` and, when kernel `id` is being timed, brackets it with events.
template <typename F>
hipError_t timed(int id, double flops, double bytes, hipStream_t s, F&& launch) {
    Profile& p = g_prof[(id > 0 && id < kKidCount) ? id : 0];
    const bool on = p.on && (p.seen++ % p.every) == 0;
    if (on) {
        hipError_t e = p.mark(s);
        if (e != hipSuccess) return e;
    }
    hipError_t e = launch();
    if (e != hipSuccess) return e;
    if (on) {
        e = p.mark(s);
        p.flops += flops;
        p.bytes += bytes;
    }
    return e;
}
}  // namespace

extern "C" int rpo_profile_start(int kernel_id, int every) {
    if (kernel_id <= 0 || kernel_id >= kKidCount) return fail(RPO_EINVAL, "rpo_profile_start: unknown kernel id");
    if (every < 1) return fail(RPO_EINVAL, "rpo_profile_start: every must be >= 1");
    Profile& p = g_prof[kernel_id];
    p.on = true;
    p.used = 0;
    p.flops = p.bytes = 0.0;
    p.every = every;
    p.seen = 0;
    return RPO_OK;
}

extern "C" int rpo_profile_stop(int kernel_id, int64_t* n_launches, double* total_ms, double* total_flops,
                                double* total_bytes) {
    if (kernel_id <= 0 || kernel_id >= kKidCount) return fail(RPO_EINVAL, "rpo_profile_stop: unknown kernel id");
    if (!n_launches || !total_ms || !total_flops || !total_bytes)
        return fail(RPO_EINVAL, "rpo_profile_stop: NULL argument");
    Profile& p = g_prof[kernel_id];
    double ms = 0.0;
    const size_t n = p.used / 2;
    if (n) HIP_TRY(hipEventSynchronize(p.events[p.used - 1]));
    for (size_t i = 0; i < n; ++i) {
        float t = 0.f;
        HIP_TRY(hipEventElapsedTime(&t, p.events[2 * i], p.events[2 * i + 1]));
        ms += t;
    }
    *n_launches = (int64_t)n;
    *total_ms = ms;
    *total_flops = p.flops;
    *total_bytes = p.bytes;
    p.on = false;
    p.used = 0;
    return RPO_OK;
}

// ---------------------------------------------------------------------------
// handles
// ---------------------------------------------------------------------------
struct rpo_model {
    rpo_model_desc d;
    const void *embed, *lm_head, *final_norm;
    std::vector<const void*> attn_norm, wqkv, wo, ffn_norm, w_gate_up, w_down;
    int qkv_width() const { return (d.n_q_heads + 2 * d.n_kv_heads) * d.head_dim; }
};

namespace {

constexpr size_t kAlign = 256;
constexpr size_t kSplitKBytes = (size_t)96 << 20;
size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

struct BatchDims {
    int n_groups, G, B, max_prefix, max_suffix, pt, max_rows;
    int ppg;         // pages of one group's prefix
    int ppr;         // private pages of one rollout
    int table_len;   // entries of one rollout's page table
    int max_pos;
    int lm_rows;     // rows of one LM-head pass
    int64_t n_pages;
};

bool make_dims(const rpo_model* m, int n_groups, int G, int max_prefix, int max_suffix, int pt,
               int max_rows, BatchDims* o) {
    if (!m || n_groups < 1 || G < 1 || max_prefix < 1 || max_suffix < 0 || pt < 16 || (pt & (pt - 1)))
        return false;
    if ((int64_t)n_groups * G > (1 << 24)) return false;
    o->n_groups = n_groups;
    o->G = G;
    o->B = n_groups * G;
    o->max_prefix = max_prefix;
    o->max_suffix = max_suffix;
    o->pt = pt;
    o->max_rows = max_rows;
    o->ppg = ceil_div(max_prefix, pt);
    o->ppr = ceil_div(pt - 1 + max_suffix, pt);
    if (o->ppr < 1) o->ppr = 1;
    o->table_len = o->ppg + o->ppr;
    o->max_pos = max_prefix + max_suffix;
    o->n_pages = (int64_t)n_groups * o->ppg + (int64_t)o->B * o->ppr;
    o->lm_rows = std::max(std::max(o->B, n_groups), std::min(max_rows, 1024));
    return true;
}

// Workspace carve-up (byte offsets, each 256-aligned).
struct WsLayout {
    size_t x, h, qkv, attn, gu, act, hl, logits, blkmax, partial, rope, tables, group_desc, rollout_desc,
        chunk_desc, row_seq, tok_index, lm_idx, shared_pages, fork_src, fork_dst, last_idx, live, row_of, count, total;
};

WsLayout make_layout(const rpo_model* m, const BatchDims& bd) {
    const rpo_model_desc& d = m->d;
    const size_t es = dtype_size(d.dtype);
    const size_t R = (size_t)bd.max_rows;
    WsLayout L;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L.x = take((R + bd.n_groups) * d.d_model * 4);  // rows [R, R + n_groups) keep each group's last prefix row
    L.h = take(R * d.d_model * es);
    L.qkv = take(R * m->qkv_width() * es);
    L.attn = take(R * (size_t)d.n_q_heads * d.head_dim * es);
    L.gu = take(kSplitKBytes);  // fp32 partial sums of K-split GEMMs
    L.act = take(R * (size_t)d.d_ffn * es);
    L.hl = take((size_t)bd.lm_rows * d.d_model * es);
    L.logits = take((size_t)std::min(bd.max_rows, 1024) * d.vocab * 4);
    L.blkmax = take((size_t)bd.B * ((size_t)ceil_div(d.vocab, 256) * 4) * 4);  // row maxima per column block
    L.partial = take(attn_decode_partial_floats(bd.B, d.n_q_heads, d.head_dim, bd.ppg) * 4);
    L.rope = take((size_t)bd.max_pos * d.head_dim * 4);
    L.tables = take(((size_t)bd.n_groups * bd.ppg + (size_t)bd.B * bd.table_len) * 4);
    L.group_desc = take((size_t)bd.n_groups * sizeof(SeqDesc));
    L.rollout_desc = take((size_t)bd.B * sizeof(SeqDesc));
    L.chunk_desc = take((size_t)std::max(bd.B, bd.n_groups) * sizeof(SeqDesc));
    L.row_seq = take(R * 4);
    L.tok_index = take(R * 4);
    L.lm_idx = take((R + bd.B) * 4);
    L.shared_pages = take((size_t)bd.n_groups * 4);
    L.fork_src = take((size_t)bd.B * 4);
    L.fork_dst = take((size_t)bd.B * 4);
    L.last_idx = take((size_t)bd.n_groups * 4);
    L.live = take((size_t)bd.B * 4);     // compacted decode: query row -> rollout
    L.row_of = take((size_t)bd.B * 4);   //                   rollout -> query row
    L.count = take(4);
    L.total = off;
    return L;
}

enum State { kEmpty = 0, kPrefilled = 1, kForked = 2 };

}  // namespace

struct rpo_batch {
    const rpo_model* m;
    BatchDims bd;
    WsLayout L;
    KvGeom geom;
    char* ws;
    void* kv;
    int state;
    int step;
    std::vector<int> prefix_len;  // S_g
    // Compacted decode: the compaction kernel reports (generation << 32 | live rows) into this
    // pinned host word; the host sizes the next launches from the latest report of the current
    // generation (the number of live rows never grows inside a rollout, so a late report is
    // still an upper bound).  A new generation starts at every fork.
    volatile uint64_t* mailbox = nullptr;   // host address (hipHostMalloc)
    uint64_t* mailbox_dev = nullptr;        // the same word as the device sees it
    uint32_t generation = 0;
    ~rpo_batch() {
        if (mailbox) (void)hipHostFree((void*)mailbox);
    }
    // host staging that must outlive the enqueue of its copy
    std::vector<std::vector<int32_t>> stage_i32;
    std::vector<std::vector<SeqDesc>> stage_desc;

    template <typename T>
    T* at(size_t off) const {
        return (T*)(ws + off);
    }
    int group_table_off(int g) const { return g * bd.ppg; }
    int rollout_table_off(int b) const { return bd.n_groups * bd.ppg + b * bd.table_len; }
    int64_t group_page(int g, int k) const { return (int64_t)g * bd.ppg + k; }
    int64_t rollout_page(int b, int k) const {
        return (int64_t)bd.n_groups * bd.ppg + (int64_t)b * bd.ppr + k;
    }
};

// ---------------------------------------------------------------------------
extern "C" int rpo_model_create(const rpo_model_desc* desc, const rpo_weights* w, rpo_model** out) {
    if (!desc || !w || !out) return fail(RPO_EINVAL, "rpo_model_create: NULL argument");
    const rpo_model_desc& d = *desc;
    if (d.n_layers < 1 || d.d_model < 1 || d.n_q_heads < 1 || d.n_kv_heads < 1 || d.head_dim < 2 ||
        d.d_ffn < 1 || d.vocab < 2)
        return fail(RPO_EINVAL, "rpo_model_create: non-positive size");
    if (d.n_q_heads % d.n_kv_heads) return fail(RPO_EINVAL, "n_q_heads must be a multiple of n_kv_heads");
    if (d.head_dim % 2 || d.head_dim > 256) return fail(RPO_EINVAL, "head_dim must be even and <= 256");
    if (d.dtype != RPO_F32 && d.dtype != RPO_BF16) return fail(RPO_EINVAL, "unknown dtype %d", d.dtype);
    if (!(d.rope_base > 0.f) || !(d.rms_eps >= 0.f)) return fail(RPO_EINVAL, "bad rope_base / rms_eps");
    if (!w->embed || !w->lm_head || !w->final_norm || !w->attn_norm || !w->wqkv || !w->wo || !w->ffn_norm ||
        !w->w_gate_up || !w->w_down)
        return fail(RPO_EINVAL, "rpo_model_create: NULL weight pointer");
    rpo_model* m = new (std::nothrow) rpo_model();
    if (!m) return fail(RPO_ENOMEM, "host allocation failed");
    m->d = d;
    m->embed = w->embed;
    m->lm_head = w->lm_head;
    m->final_norm = w->final_norm;
    for (int l = 0; l < d.n_layers; ++l) {
        if (!w->attn_norm[l] || !w->wqkv[l] || !w->wo[l] || !w->ffn_norm[l] || !w->w_gate_up[l] ||
            !w->w_down[l]) {
            delete m;
            return fail(RPO_EINVAL, "rpo_model_create: NULL weight pointer in layer %d", l);
        }
        m->attn_norm.push_back(w->attn_norm[l]);
        m->wqkv.push_back(w->wqkv[l]);
        m->wo.push_back(w->wo[l]);
        m->ffn_norm.push_back(w->ffn_norm[l]);
        m->w_gate_up.push_back(w->w_gate_up[l]);
        m->w_down.push_back(w->w_down[l]);
    }
    *out = m;
    return RPO_OK;
}

extern "C" void rpo_model_destroy(rpo_model* m) { delete m; }

extern "C" size_t rpo_kv_pool_bytes(const rpo_model* m, int32_t n_groups, int32_t G, int32_t max_prefix,
                                    int32_t max_suffix, int32_t page_tokens) {
    BatchDims bd;
    if (!make_dims(m, n_groups, G, max_prefix, max_suffix, page_tokens, 1, &bd)) return 0;
    const rpo_model_desc& d = m->d;
    return (size_t)d.n_layers * bd.n_pages * 2 * d.n_kv_heads * page_tokens * d.head_dim * dtype_size(d.dtype);
}

static bool rows_ok(const BatchDims& bd) {
    return bd.max_rows >= bd.max_prefix && bd.max_rows >= bd.B && bd.max_rows >= bd.max_suffix;
}

extern "C" size_t rpo_workspace_bytes(const rpo_model* m, int32_t n_groups, int32_t G, int32_t max_prefix,
                                      int32_t max_suffix, int32_t page_tokens, int32_t max_rows) {
    BatchDims bd;
    if (!make_dims(m, n_groups, G, max_prefix, max_suffix, page_tokens, max_rows, &bd) || !rows_ok(bd))
        return 0;
    return make_layout(m, bd).total;
}

extern "C" int rpo_batch_create(const rpo_model* m, int32_t n_groups, int32_t G, int32_t max_prefix,
                                int32_t max_suffix, int32_t page_tokens, int32_t max_rows, void* kv_pool,
                                size_t kv_bytes, void* workspace, size_t ws_bytes, void* stream,
                                rpo_batch** out) {
    if (!m || !out || !kv_pool || !workspace) return fail(RPO_EINVAL, "rpo_batch_create: NULL argument");
    BatchDims bd;
    if (!make_dims(m, n_groups, G, max_prefix, max_suffix, page_tokens, max_rows, &bd))
        return fail(RPO_EINVAL, "rpo_batch_create: bad sizes (page_tokens must be a power of two >= 16)");
    if (!rows_ok(bd))
        return fail(RPO_EINVAL, "rpo_batch_create: max_rows must be >= max_prefix, >= max_suffix and >= n_groups * G");
    if (((uintptr_t)kv_pool | (uintptr_t)workspace) % kAlign)
        return fail(RPO_EINVAL, "rpo_batch_create: buffers must be 256-byte aligned");
    const size_t need_kv = rpo_kv_pool_bytes(m, n_groups, G, max_prefix, max_suffix, page_tokens);
    const WsLayout L = make_layout(m, bd);
    if (kv_bytes < need_kv) return fail(RPO_ENOMEM, "kv pool: %zu bytes given, %zu needed", kv_bytes, need_kv);
    if (ws_bytes < L.total) return fail(RPO_ENOMEM, "workspace: %zu bytes given, %zu needed", ws_bytes, L.total);

    rpo_batch* b = new (std::nothrow) rpo_batch();
    if (!b) return fail(RPO_ENOMEM, "host allocation failed");
    b->m = m;
    b->bd = bd;
    b->L = L;
    b->ws = (char*)workspace;
    b->kv = kv_pool;
    b->state = kEmpty;
    b->step = 0;
    b->geom.n_kv_heads = m->d.n_kv_heads;
    b->geom.head_dim = m->d.head_dim;
    b->geom.page_tokens = page_tokens;
    b->geom.n_pages = bd.n_pages;
    hipStream_t s = (hipStream_t)stream;
    {
        void* host = nullptr;
        void* dev = nullptr;
        hipError_t em = hipHostMalloc(&host, 64, hipHostMallocDefault);
        if (em == hipSuccess) em = hipHostGetDevicePointer(&dev, host, 0);
        if (em != hipSuccess) {
            if (host) (void)hipHostFree(host);
            delete b;
            return fail(RPO_EHIP, "rpo_batch_create: pinned mailbox: %s", hipGetErrorString(em));
        }
        b->mailbox = (volatile uint64_t*)host;
        b->mailbox_dev = (uint64_t*)dev;
        *b->mailbox = 0;
    }

    // Rotary table in fp64 on the host: angle = pos * base^(-2 i / dh).
    const int half = m->d.head_dim / 2;
    std::vector<float> rope((size_t)bd.max_pos * half * 2);
    for (int p = 0; p < bd.max_pos; ++p)
        for (int i = 0; i < half; ++i) {
            const double theta = pow((double)m->d.rope_base, -2.0 * i / (double)m->d.head_dim);
            const double ang = (double)p * theta;
            rope[((size_t)p * half + i) * 2] = (float)cos(ang);
            rope[((size_t)p * half + i) * 2 + 1] = (float)sin(ang);
        }
    // Group page tables never change (static page ownership).
    std::vector<int32_t> gt((size_t)bd.n_groups * bd.ppg);
    for (int g = 0; g < bd.n_groups; ++g)
        for (int k = 0; k < bd.ppg; ++k) gt[(size_t)g * bd.ppg + k] = (int32_t)b->group_page(g, k);
    hipError_t e = hipMemcpyAsync(b->at<float>(L.rope), rope.data(), rope.size() * 4, hipMemcpyHostToDevice, s);
    if (e == hipSuccess)
        e = hipMemcpyAsync(b->at<int32_t>(L.tables), gt.data(), gt.size() * 4, hipMemcpyHostToDevice, s);
    // Stale page contents are masked by length, but they are multiplied by a zero
    // probability: they must be finite.  Clear the pool once.
    if (e == hipSuccess) e = hipMemsetAsync(kv_pool, 0, need_kv, s);
    if (e == hipSuccess) e = hipStreamSynchronize(s);  // the host vectors above go out of scope
    if (e != hipSuccess) {
        delete b;
        return fail(RPO_EHIP, "rpo_batch_create: %s", hipGetErrorString(e));
    }
    *out = b;
    return RPO_OK;
}

extern "C" void rpo_batch_destroy(rpo_batch* b) { delete b; }

// ---------------------------------------------------------------------------
// the layer stack on `rows` packed rows already embedded in x
// ---------------------------------------------------------------------------
namespace {

struct PassCfg {
    int rows;
    const int32_t* row_seq;  // device
    const SeqDesc* seqs;     // device
    int n_seqs, max_seq_rows;
    int pos_add;
    const uint8_t* active;
    bool decode;             // one row per rollout against the shared-prefix cache
    int max_shared_pages;
    double attn_flops = 0.0;  // algorithmic work of ONE layer's attention launch (for timing reports)
    double attn_bytes = 0.0;
    void* final_norm_out = nullptr;  // if set: final RMSNorm of all rows is written here by the last layer
    // compacted decode step: rows are query rows, row_seq maps them to rollouts (< 0: padding),
    // row_of is the inverse map, n_rollouts the rollout rows covered
    const int32_t* row_of = nullptr;
    int n_rollouts = 0;
};

#define RET_IF(expr)                       \
    do {                                   \
        hipError_t e__ = (expr);           \
        if (e__ != hipSuccess) return e__; \
    } while (0)

GemmArgs gemm_args(rpo_batch* b, const void* A, int64_t lda, const void* W, int64_t ldw, void* C, int64_t ldc,
                   int M, int N, int K, int epi) {
    GemmArgs g;
    g.A = A;
    g.lda = lda;
    g.W = W;
    g.ldw = ldw;
    g.C = C;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.dtype = b->m->d.dtype;
    g.epilogue = epi;
    g.path = g_kernel_path;
    g.ws = b->at<void>(b->L.gu);
    g.ws_bytes = kSplitKBytes;
    g.norm_eps = b->m->d.rms_eps;
    return g;
}

hipError_t gemm(rpo_batch* b, const void* A, int64_t lda, const void* W, int64_t ldw, void* C,
                int64_t ldc, int M, int N, int K, int epi, hipStream_t s, const void* norm_gain = nullptr,
                void* norm_out = nullptr, const RopeKvArgs* rope = nullptr) {
    const rpo_model* m = b->m;
    GemmArgs g;
    g.A = A;
    g.lda = lda;
    g.W = W;
    g.ldw = ldw;
    g.C = C;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.dtype = m->d.dtype;
    g.epilogue = epi;
    g.path = g_kernel_path;
    g.ws = b->at<void>(b->L.gu);
    g.ws_bytes = kSplitKBytes;
    g.norm_gain = norm_gain;
    g.norm_out = norm_out;
    g.norm_eps = m->d.rms_eps;
    g.rope = rope;
    const double es = (double)dtype_size(g.dtype);
    const double out_bytes = epi == kEpiStore ? (double)M * N * es
                             : epi == kEpiStoreF32 ? (double)M * N * 4.0
                             : epi == kEpiAddF32 ? (double)M * N * 8.0
                                                 : (double)M * (N / 2) * es;
    return timed(gemm_kernel_id(g), 2.0 * M * N * K, ((double)M * K + (double)N * K) * es + out_bytes, s,
                 [&] { return launch_gemm(g, s); });
}

// Algorithmic flops of one layer's causal attention over packed chunks: every row multiplies its
// query heads with the keys and with the values of the positions it sees (2 * 2 * dh per pair).
double chunk_attn_flops(const std::vector<SeqDesc>& descs, const rpo_model_desc& d) {
    double pairs = 0.0;
    for (const SeqDesc& sd : descs)
        pairs += (double)sd.n_rows * sd.pos0 + 0.5 * (double)sd.n_rows * ((double)sd.n_rows + 1.0);
    return 4.0 * pairs * d.n_q_heads * d.head_dim;
}

hipError_t run_layers(rpo_batch* b, const PassCfg& pc, hipStream_t s) {
    const rpo_model* m = b->m;
    const rpo_model_desc& d = m->d;
    const WsLayout& L = b->L;
    float* x = b->at<float>(L.x);
    void* h = b->at<void>(L.h);
    void* qkv = b->at<void>(L.qkv);
    void* attn = b->at<void>(L.attn);
    void* act = b->at<void>(L.act);
    const int qw = m->qkv_width();
    const int qd = d.n_q_heads * d.head_dim;
    // Every RMSNorm but the first rides on the projection that produces its input (the
    // residual-adding O and down GEMMs write the normalised rows too).
    RET_IF(launch_rmsnorm(x, nullptr, m->attn_norm[0], d.dtype, d.d_model, d.rms_eps, h, pc.rows, s));
    for (int l = 0; l < d.n_layers; ++l) {
        RopeKvArgs ra;
        ra.qkv = qkv;
        ra.dtype = d.dtype;
        ra.rows = pc.rows;
        ra.Hq = d.n_q_heads;
        ra.Hkv = d.n_kv_heads;
        ra.dh = d.head_dim;
        ra.rope = b->at<float>(L.rope);
        ra.row_seq = pc.row_seq;
        ra.seqs = pc.seqs;
        ra.pos_add = pc.pos_add;
        ra.single_row = pc.row_of ? 1 : 0;
        ra.tables = b->at<int32_t>(L.tables);
        ra.active = pc.active;
        ra.kv_pool = b->kv;
        ra.geom = b->geom;
        ra.layer = l;
        // QKV projection; the rotation + KV page write ride on it (fused when the GEMM is K-split)
        RET_IF(gemm(b, h, d.d_model, m->wqkv[l], d.d_model, qkv, qw, pc.rows, qw, d.d_model, kEpiStore, s, nullptr,
                    nullptr, &ra));
        AttnArgs aa;
        aa.q = qkv;
        aa.q_stride = qw;
        aa.out = attn;
        aa.dtype = d.dtype;
        aa.rows = pc.rows;
        aa.Hq = d.n_q_heads;
        aa.Hkv = d.n_kv_heads;
        aa.dh = d.head_dim;
        aa.row_seq = pc.row_seq;
        aa.seqs = pc.seqs;
        aa.n_seqs = pc.n_seqs;
        aa.max_seq_rows = pc.max_seq_rows;
        aa.pos_add = pc.pos_add;
        aa.single_row = pc.row_of ? 1 : 0;
        aa.tables = b->at<int32_t>(L.tables);
        aa.active = pc.active;
        aa.kv_pool = b->kv;
        aa.geom = b->geom;
        aa.layer = l;
        aa.scale = 1.0f / sqrtf((float)d.head_dim);
        aa.path = g_kernel_path;
        if (pc.decode) {
            DecodeAttnArgs da;
            da.base = aa;
            da.n_rollouts = pc.row_of ? pc.n_rollouts : pc.rows;
            da.row_of = pc.row_of;
            da.G = b->bd.G;
            da.shared_pages = b->at<int32_t>(L.shared_pages);
            da.max_shared_pages = pc.max_shared_pages;
            da.max_own_pages = b->bd.ppr;
            da.partial = b->at<float>(L.partial);
            da.partial_floats = attn_decode_partial_floats(b->bd.B, d.n_q_heads, d.head_dim, b->bd.ppg);
            RET_IF(timed(attn_uses_mfma(aa) ? kKidAttnDecode : 0, pc.attn_flops, pc.attn_bytes, s,
                         [&] { return launch_attn_decode(da, s); }));
        } else {
            RET_IF(timed(attn_uses_mfma(aa) ? kKidAttnChunk : 0, pc.attn_flops, pc.attn_bytes, s,
                         [&] { return launch_attn_chunk(aa, s); }));
        }
        RET_IF(gemm(b, attn, qd, m->wo[l], qd, x, d.d_model, pc.rows, d.d_model, qd, kEpiAddF32, s,
                    m->ffn_norm[l], h));
        RET_IF(gemm(b, h, d.d_model, m->w_gate_up[l], d.d_model, act, d.d_ffn, pc.rows, 2 * d.d_ffn, d.d_model,
                    kEpiSwiglu, s));
        const bool last = l + 1 == d.n_layers;
        const void* next_gain = last ? (pc.final_norm_out ? m->final_norm : nullptr) : m->attn_norm[l + 1];
        void* next_out = last ? pc.final_norm_out : h;
        RET_IF(gemm(b, act, d.d_ffn, m->w_down[l], d.d_ffn, x, d.d_model, pc.rows, d.d_model, d.d_ffn,
                    kEpiAddF32, s, next_gain, next_gain ? next_out : nullptr));
    }
    return hipSuccess;
}

// final RMSNorm of selected rows of x (row_idx device, or NULL = rows 0..n) + LM head -> fp32 logits
hipError_t lm_head_rows(rpo_batch* b, const int32_t* row_idx, int n, float* logits, hipStream_t s) {
    const rpo_model* m = b->m;
    const rpo_model_desc& d = m->d;
    void* hl = b->at<void>(b->L.hl);
    RET_IF(launch_rmsnorm(b->at<float>(b->L.x), row_idx, m->final_norm, d.dtype, d.d_model, d.rms_eps, hl, n,
                          s));
    return gemm(b, hl, d.d_model, m->lm_head, d.d_model, logits, d.vocab, n, d.vocab, d.d_model,
                kEpiStoreF32, s);
}

// final RMSNorm of selected rows + LM head + log-softmax value of each row's target token.
// On the MFMA path the log-sum-exp is taken in the GEMM epilogue (the logits never reach memory);
// `scratch` (the logits staging area) then holds the per-block pieces.
hipError_t lm_head_logprob_rows(rpo_batch* b, const int32_t* row_idx, int n, const int32_t* target, float inv_t,
                                float* out, float* scratch, hipStream_t s) {
    const rpo_model* m = b->m;
    const rpo_model_desc& d = m->d;
    void* hl = b->at<void>(b->L.hl);
    RET_IF(launch_rmsnorm(b->at<float>(b->L.x), row_idx, m->final_norm, d.dtype, d.d_model, d.rms_eps, hl, n,
                          s));
    GemmArgs g;
    g.A = hl;
    g.lda = d.d_model;
    g.W = m->lm_head;
    g.ldw = d.d_model;
    g.C = scratch;
    g.ldc = d.vocab;
    g.M = n;
    g.N = d.vocab;
    g.K = d.d_model;
    g.dtype = d.dtype;
    g.epilogue = kEpiStoreF32;
    g.path = g_kernel_path;
    const int blocks = gemm_fuses_lse(g);
    if (blocks <= 0) {
        RET_IF(gemm(b, hl, d.d_model, m->lm_head, d.d_model, scratch, d.vocab, n, d.vocab, d.d_model, kEpiStoreF32,
                    s));
        return launch_lse_gather(scratch, d.vocab, d.vocab, target, inv_t, out, n, s);
    }
    LseFuse lf;
    lf.part = scratch;                                   // [n, blocks, 2]
    lf.target_logit = scratch + (size_t)n * blocks * 2;  // [n]
    lf.target = target;
    lf.k2 = inv_t * 1.4426950408889634f;
    g.lse = &lf;
    const double es = (double)dtype_size(g.dtype);
    RET_IF(timed(gemm_kernel_id(g), 2.0 * n * (double)d.vocab * d.d_model,
                 ((double)n * d.d_model + (double)d.vocab * d.d_model) * es, s, [&] { return launch_gemm(g, s); }));
    return launch_lse_combine(lf.part, lf.blocks, lf.target_logit, target, d.vocab, inv_t, out, n, s);
}

template <typename T>
hipError_t upload(rpo_batch* b, std::vector<std::vector<T>>& keep, const std::vector<T>& v, size_t off,
                  hipStream_t s) {
    if (v.empty()) return hipSuccess;
    keep.push_back(v);
    return hipMemcpyAsync(b->ws + off, keep.back().data(), v.size() * sizeof(T), hipMemcpyHostToDevice, s);
}

}  // namespace

// ---------------------------------------------------------------------------
extern "C" int rpo_prefill_prefix(rpo_batch* b, const int32_t* tokens_dev, const int32_t* cu_len_host,
                                  float* last_logits_dev, void* stream) {
    if (!b || !tokens_dev || !cu_len_host || !last_logits_dev)
        return fail(RPO_EINVAL, "rpo_prefill_prefix: NULL argument");
    const BatchDims& bd = b->bd;
    if (cu_len_host[0] != 0) return fail(RPO_EINVAL, "rpo_prefill_prefix: cu_len[0] must be 0");
    for (int g = 0; g < bd.n_groups; ++g) {
        const int len = cu_len_host[g + 1] - cu_len_host[g];
        if (len < 1 || len > bd.max_prefix)
            return fail(RPO_EINVAL, "rpo_prefill_prefix: group %d has prefix length %d, allowed 1..%d", g, len,
                        bd.max_prefix);
    }
    hipStream_t s = (hipStream_t)stream;
    const rpo_model_desc& d = b->m->d;
    const WsLayout& L = b->L;
    b->stage_i32.clear();
    b->stage_desc.clear();
    b->state = kEmpty;
    b->prefix_len.assign(bd.n_groups, 0);
    for (int g = 0; g < bd.n_groups; ++g) b->prefix_len[g] = cu_len_host[g + 1] - cu_len_host[g];

    int g0 = 0;
    while (g0 < bd.n_groups) {
        int g1 = g0, rows = 0;
        while (g1 < bd.n_groups && rows + b->prefix_len[g1] <= bd.max_rows) rows += b->prefix_len[g1++];
        std::vector<SeqDesc> descs;
        std::vector<int32_t> row_seq((size_t)rows), last_idx;
        int r = 0, max_seq = 0;
        for (int g = g0; g < g1; ++g) {
            SeqDesc sd{r, b->prefix_len[g], 0, b->group_table_off(g)};
            descs.push_back(sd);
            for (int i = 0; i < sd.n_rows; ++i) row_seq[(size_t)r + i] = g - g0;
            r += sd.n_rows;
            last_idx.push_back(r - 1);
            max_seq = std::max(max_seq, sd.n_rows);
        }
        HIP_TRY(upload(b, b->stage_desc, descs, L.chunk_desc, s));
        HIP_TRY(upload(b, b->stage_i32, row_seq, L.row_seq, s));
        HIP_TRY(upload(b, b->stage_i32, last_idx, L.last_idx, s));
        HIP_TRY(launch_embed(tokens_dev + cu_len_host[g0], nullptr, b->m->embed, d.dtype, d.vocab, d.d_model,
                             b->at<float>(L.x), rows, s));
        PassCfg pc;
        pc.rows = rows;
        pc.row_seq = b->at<int32_t>(L.row_seq);
        pc.seqs = b->at<SeqDesc>(L.chunk_desc);
        pc.n_seqs = g1 - g0;
        pc.max_seq_rows = max_seq;
        pc.pos_add = 0;
        pc.active = nullptr;
        pc.decode = false;
        pc.max_shared_pages = 0;
        pc.attn_flops = chunk_attn_flops(descs, d);
        HIP_TRY(run_layers(b, pc, s));
        // keep each group's last residual row (rows [max_rows + g0, max_rows + g1) of x)
        HIP_TRY(launch_gather_rows(b->at<float>(L.x), b->at<int32_t>(L.last_idx), d.d_model,
                                   b->at<float>(L.x) + ((size_t)bd.max_rows + g0) * d.d_model, g1 - g0, s));
        g0 = g1;
    }
    // logits of the last prefix rows
    std::vector<int32_t> idx(bd.n_groups);
    for (int g = 0; g < bd.n_groups; ++g) idx[g] = bd.max_rows + g;
    HIP_TRY(upload(b, b->stage_i32, idx, L.lm_idx, s));
    HIP_TRY(lm_head_rows(b, b->at<int32_t>(L.lm_idx), bd.n_groups, last_logits_dev, s));
    b->state = kPrefilled;
    b->step = 0;
    return RPO_OK;
}

// ---------------------------------------------------------------------------
extern "C" int rpo_kv_fork(rpo_batch* b, void* stream) {
    if (!b) return fail(RPO_EINVAL, "rpo_kv_fork: NULL batch");
    if (b->state != kPrefilled) return fail(RPO_ESTATE, "rpo_kv_fork: call rpo_prefill_prefix first");
    const BatchDims& bd = b->bd;
    const WsLayout& L = b->L;
    hipStream_t s = (hipStream_t)stream;
    std::vector<int32_t> tables((size_t)bd.B * bd.table_len, 0), shared(bd.n_groups), src(bd.B), dst(bd.B);
    std::vector<SeqDesc> descs(bd.B);
    for (int g = 0; g < bd.n_groups; ++g) {
        const int S = b->prefix_len[g];
        const int n_full = S / bd.pt;
        shared[g] = n_full;
        for (int i = 0; i < bd.G; ++i) {
            const int r = g * bd.G + i;
            int32_t* t = &tables[(size_t)r * bd.table_len];
            for (int k = 0; k < n_full; ++k) t[k] = (int32_t)b->group_page(g, k);
            for (int k = 0; k < bd.ppr && n_full + k < bd.table_len; ++k)
                t[n_full + k] = (int32_t)b->rollout_page(r, k);
            src[r] = (S % bd.pt) ? (int32_t)b->group_page(g, n_full) : -1;
            dst[r] = (int32_t)b->rollout_page(r, 0);
            descs[r] = SeqDesc{r, 1, S, b->rollout_table_off(r)};
        }
    }
    HIP_TRY(upload(b, b->stage_i32, tables, L.tables + (size_t)bd.n_groups * bd.ppg * 4, s));
    HIP_TRY(upload(b, b->stage_i32, shared, L.shared_pages, s));
    HIP_TRY(upload(b, b->stage_i32, src, L.fork_src, s));
    HIP_TRY(upload(b, b->stage_i32, dst, L.fork_dst, s));
    HIP_TRY(upload(b, b->stage_desc, descs, L.rollout_desc, s));
    HIP_TRY(launch_fork_copy(b->kv, b->m->d.dtype, b->geom, b->m->d.n_layers, b->at<int32_t>(L.fork_src),
                             b->at<int32_t>(L.fork_dst), bd.B, s));
    b->state = kForked;
    b->step = 0;
    b->generation += 1;
    *b->mailbox = ((uint64_t)b->generation << 32) | (uint32_t)bd.B;
    return RPO_OK;
}

// ---------------------------------------------------------------------------
namespace {
// One decode step on `rows` query rows.  Plain: query row = rollout row, rows = n_rollouts.
// Compacted: query row c belongs to rollout live[c] (padding rows: -1), row_of is the inverse map.
int decode_step_body(rpo_batch* b, const int32_t* tokens_dev, int rows, int n_rollouts, const uint8_t* active_dev,
                     const int32_t* live, const int32_t* row_of, float* logits_dev, float* row_max_out_dev,
                     hipStream_t s) {
    const BatchDims& bd = b->bd;
    const rpo_model_desc& d = b->m->d;
    const WsLayout& L = b->L;
    HIP_TRY(launch_embed(tokens_dev, live, b->m->embed, d.dtype, d.vocab, d.d_model, b->at<float>(L.x), rows, s));
    int max_shared = 0;
    for (int g = 0; g < ceil_div(n_rollouts, bd.G); ++g) max_shared = std::max(max_shared, b->prefix_len[g] / bd.pt);
    PassCfg pc;
    pc.rows = rows;
    pc.row_seq = live;
    pc.seqs = b->at<SeqDesc>(L.rollout_desc);
    pc.n_seqs = n_rollouts;
    pc.max_seq_rows = 1;
    pc.pos_add = b->step;
    pc.active = live ? nullptr : active_dev;
    pc.decode = true;
    pc.max_shared_pages = max_shared;
    pc.row_of = row_of;
    pc.n_rollouts = n_rollouts;
    {
        // Algorithmic work of one layer's decode attention: the shared prefix pages of every live
        // group are read ONCE per group, each rollout's private tokens once per rollout (a
        // compacted step is priced as if every covered rollout were live).
        const double tok_bytes = 2.0 * d.n_kv_heads * d.head_dim * dtype_size(d.dtype);
        double toks = 0.0, qk = 0.0;
        for (int r = 0; r < n_rollouts; ++r) {
            const int g = r / bd.G;
            const int ctx = b->prefix_len[g] + b->step + 1;
            const int shared_tok = (b->prefix_len[g] / bd.pt) * bd.pt;
            toks += ctx - shared_tok;
            if (r % bd.G == 0) toks += shared_tok;
            qk += ctx;
        }
        pc.attn_bytes = toks * tok_bytes;
        pc.attn_flops = 4.0 * qk * d.n_q_heads * d.head_dim;
    }
    pc.final_norm_out = b->at<void>(L.hl);
    HIP_TRY(run_layers(b, pc, s));
    if (!row_max_out_dev) {
        HIP_TRY(gemm(b, b->at<void>(L.hl), d.d_model, b->m->lm_head, d.d_model, logits_dev, d.vocab, rows, d.vocab,
                     d.d_model, kEpiStoreF32, s));
    } else {
        // the LM-head epilogue leaves each row's maximum per column block where it can
        GemmArgs g = gemm_args(b, b->at<void>(L.hl), d.d_model, b->m->lm_head, d.d_model, logits_dev, d.vocab, rows,
                               d.vocab, d.d_model, kEpiStoreF32);
        LseFuse bm;
        bm.part = b->at<float>(L.blkmax);
        g.block_max = &bm;
        // A handful of rows streams the LM-head weights either way: keep the 256-wide tile whose
        // epilogue knows the maxima rather than sweep the logits again.
        if (g.path == 0 && gemm_fuses_max(g) == 0) {
            g.path = 16 + kKidGemm256;
            if (gemm_fuses_max(g) == 0) g.path = 0;
        }
        const bool fused = gemm_fuses_max(g) > 0;
        const double es = (double)dtype_size(g.dtype);
        HIP_TRY(timed(gemm_kernel_id(g), 2.0 * rows * (double)d.vocab * d.d_model,
                      ((double)rows * d.d_model + (double)d.vocab * d.d_model) * es + (double)rows * d.vocab * 4.0,
                      s, [&] { return launch_gemm(g, s); }));
        if (fused)
            HIP_TRY(launch_row_max_blocks(bm.part, bm.blocks, row_max_out_dev, rows, s));
        else
            HIP_TRY(launch_row_max(logits_dev, d.vocab, d.vocab, row_max_out_dev, rows, s));
    }
    b->step += 1;
    return RPO_OK;
}
}  // namespace

extern "C" int rpo_decode_step(rpo_batch* b, const int32_t* tokens_dev, int32_t n_rows,
                               const uint8_t* active_dev, float* logits_dev, float* row_max_out_dev,
                               void* stream) {
    if (!b || !tokens_dev || !logits_dev) return fail(RPO_EINVAL, "rpo_decode_step: NULL argument");
    if (b->state != kForked) return fail(RPO_ESTATE, "rpo_decode_step: call rpo_kv_fork first");
    const BatchDims& bd = b->bd;
    if (n_rows < 1 || n_rows > bd.B) return fail(RPO_EINVAL, "rpo_decode_step: n_rows %d not in 1..%d", n_rows, bd.B);
    if (b->step >= bd.max_suffix)
        return fail(RPO_ESTATE, "rpo_decode_step: step %d would exceed max_suffix %d", b->step, bd.max_suffix);
    return decode_step_body(b, tokens_dev, n_rows, n_rows, active_dev, nullptr, nullptr, logits_dev, row_max_out_dev,
                            (hipStream_t)stream);
}

extern "C" int rpo_decode_step_compact(rpo_batch* b, const int32_t* tokens_dev, int32_t n_rows,
                                       const uint8_t* active_dev, float* logits_dev, float* row_max_out_dev,
                                       int32_t* row_of_out_dev, int32_t* n_logit_rows_out, void* stream) {
    if (!b || !tokens_dev || !logits_dev || !active_dev || !row_of_out_dev || !n_logit_rows_out)
        return fail(RPO_EINVAL, "rpo_decode_step_compact: NULL argument");
    if (b->state != kForked) return fail(RPO_ESTATE, "rpo_decode_step_compact: call rpo_kv_fork first");
    const BatchDims& bd = b->bd;
    if (n_rows < 1 || n_rows > bd.B)
        return fail(RPO_EINVAL, "rpo_decode_step_compact: n_rows %d not in 1..%d", n_rows, bd.B);
    if (b->step >= bd.max_suffix)
        return fail(RPO_ESTATE, "rpo_decode_step_compact: step %d would exceed max_suffix %d", b->step, bd.max_suffix);
    hipStream_t s = (hipStream_t)stream;
    const WsLayout& L = b->L;
    // latest report of this rollout's compaction kernel: an upper bound of the rows still live
    const uint64_t report = *b->mailbox;
    int rows = n_rows;
    if ((uint32_t)(report >> 32) == b->generation) rows = std::min(rows, (int)(uint32_t)report);
    HIP_TRY(launch_compact_rows(active_dev, n_rows, b->at<int32_t>(L.live), row_of_out_dev, b->at<int32_t>(L.count),
                                b->mailbox_dev, b->generation, s));
    *n_logit_rows_out = rows;
    if (rows == 0) {  // every rollout has finished: nothing to compute, the step still counts
        b->step += 1;
        return RPO_OK;
    }
    return decode_step_body(b, tokens_dev, rows, n_rows, active_dev, b->at<int32_t>(L.live), row_of_out_dev,
                            logits_dev, row_max_out_dev, s);
}

// ---------------------------------------------------------------------------
extern "C" int rpo_attn_decode(rpo_batch* b, int32_t layer, const void* q_dev, int32_t n_rows, int32_t n_suffix,
                               const uint8_t* active_dev, void* out_dev, void* stream) {
    if (!b || !q_dev || !out_dev) return fail(RPO_EINVAL, "rpo_attn_decode: NULL argument");
    if (b->state != kForked) return fail(RPO_ESTATE, "rpo_attn_decode: call rpo_kv_fork first");
    const BatchDims& bd = b->bd;
    const rpo_model_desc& d = b->m->d;
    if (layer < 0 || layer >= d.n_layers) return fail(RPO_EINVAL, "rpo_attn_decode: layer %d not in 0..%d", layer, d.n_layers - 1);
    if (n_rows < 1 || n_rows > bd.B) return fail(RPO_EINVAL, "rpo_attn_decode: n_rows %d not in 1..%d", n_rows, bd.B);
    if (n_suffix < 0 || n_suffix > bd.max_suffix)
        return fail(RPO_EINVAL, "rpo_attn_decode: n_suffix %d not in 0..%d", n_suffix, bd.max_suffix);
    for (int g = 0; g < ceil_div(n_rows, bd.G); ++g)
        if (b->prefix_len[g] + n_suffix < 1) return fail(RPO_EINVAL, "rpo_attn_decode: empty context");
    const WsLayout& L = b->L;
    hipStream_t s = (hipStream_t)stream;
    AttnArgs aa;
    aa.q = q_dev;
    aa.q_stride = (int64_t)d.n_q_heads * d.head_dim;
    aa.out = out_dev;
    aa.dtype = d.dtype;
    aa.rows = n_rows;
    aa.Hq = d.n_q_heads;
    aa.Hkv = d.n_kv_heads;
    aa.dh = d.head_dim;
    aa.row_seq = nullptr;
    aa.seqs = b->at<SeqDesc>(L.rollout_desc);
    aa.n_seqs = n_rows;
    aa.max_seq_rows = 1;
    aa.pos_add = n_suffix - 1;  // a row sees positions [0, prefix_len + n_suffix)
    aa.tables = b->at<int32_t>(L.tables);
    aa.active = active_dev;
    aa.kv_pool = b->kv;
    aa.geom = b->geom;
    aa.layer = layer;
    aa.scale = 1.0f / sqrtf((float)d.head_dim);
    aa.path = g_kernel_path;
    DecodeAttnArgs da;
    da.base = aa;
    da.n_rollouts = n_rows;
    da.G = bd.G;
    da.shared_pages = b->at<int32_t>(L.shared_pages);
    int max_shared = 0;
    double toks = 0.0, qk = 0.0;
    for (int r = 0; r < n_rows; ++r) {
        const int g = r / bd.G;
        const int shared_tok = (b->prefix_len[g] / bd.pt) * bd.pt, ctx = b->prefix_len[g] + n_suffix;
        max_shared = std::max(max_shared, b->prefix_len[g] / bd.pt);
        toks += ctx - shared_tok;
        if (r % bd.G == 0) toks += shared_tok;
        qk += ctx;
    }
    da.max_shared_pages = max_shared;
    da.max_own_pages = bd.ppr;
    da.partial = b->at<float>(L.partial);
    da.partial_floats = attn_decode_partial_floats(bd.B, d.n_q_heads, d.head_dim, bd.ppg);
    HIP_TRY(timed(attn_uses_mfma(aa) ? kKidAttnDecode : 0, 4.0 * qk * d.n_q_heads * d.head_dim,
                  toks * 2.0 * d.n_kv_heads * d.head_dim * dtype_size(d.dtype), s,
                  [&] { return launch_attn_decode(da, s); }));
    return RPO_OK;
}

// ---------------------------------------------------------------------------
extern "C" int rpo_suffix_logprobs(rpo_batch* b, const int32_t* suffix_tokens_dev,
                                   const int32_t* cu_suffix_host, float temperature, float* logprobs_out_dev,
                                   void* stream) {
    if (!b || !suffix_tokens_dev || !cu_suffix_host || !logprobs_out_dev)
        return fail(RPO_EINVAL, "rpo_suffix_logprobs: NULL argument");
    if (b->state != kForked) return fail(RPO_ESTATE, "rpo_suffix_logprobs: call rpo_kv_fork first");
    if (!(temperature > 0.f)) return fail(RPO_EINVAL, "rpo_suffix_logprobs: temperature must be > 0");
    const BatchDims& bd = b->bd;
    if (cu_suffix_host[0] != 0) return fail(RPO_EINVAL, "rpo_suffix_logprobs: cu_suffix[0] must be 0");
    for (int r = 0; r < bd.B; ++r) {
        const int len = cu_suffix_host[r + 1] - cu_suffix_host[r];
        if (len < 0 || len > bd.max_suffix)
            return fail(RPO_EINVAL, "rpo_suffix_logprobs: rollout %d has suffix length %d, allowed 0..%d", r, len,
                        bd.max_suffix);
    }
    hipStream_t s = (hipStream_t)stream;
    const rpo_model_desc& d = b->m->d;
    const WsLayout& L = b->L;
    const float inv_t = 1.0f / temperature;
    const int lm_chunk = std::min(bd.max_rows, 1024);
    b->stage_i32.clear();
    b->stage_desc.clear();

    int r0 = 0;
    while (r0 < bd.B) {
        // rollouts [r0, r1): forward rows = suffix tokens 0 .. m-2 of each (the last one scores nothing)
        int r1 = r0, rows = 0;
        while (r1 < bd.B) {
            const int m = cu_suffix_host[r1 + 1] - cu_suffix_host[r1];
            const int fr = m > 0 ? m - 1 : 0;
            if (rows + fr > bd.max_rows) break;
            rows += fr;
            ++r1;
        }
        std::vector<SeqDesc> descs;
        std::vector<int32_t> row_seq((size_t)rows), tok_index((size_t)rows), lm_idx;
        int r = 0, max_seq = 0;
        for (int q = r0; q < r1; ++q) {
            const int m = cu_suffix_host[q + 1] - cu_suffix_host[q];
            const int fr = m > 0 ? m - 1 : 0;
            const int g = q / bd.G;
            descs.push_back(SeqDesc{r, fr, b->prefix_len[g], b->rollout_table_off(q)});
            if (m > 0) lm_idx.push_back(bd.max_rows + g);  // first suffix token: scored by the last prefix row
            for (int i = 0; i < fr; ++i) {
                row_seq[(size_t)r + i] = q - r0;
                tok_index[(size_t)r + i] = cu_suffix_host[q] + i;
                lm_idx.push_back(r + i);
            }
            r += fr;
            max_seq = std::max(max_seq, fr);
        }
        if (rows > 0) {
            HIP_TRY(upload(b, b->stage_desc, descs, L.chunk_desc, s));
            HIP_TRY(upload(b, b->stage_i32, row_seq, L.row_seq, s));
            HIP_TRY(upload(b, b->stage_i32, tok_index, L.tok_index, s));
            HIP_TRY(launch_embed(suffix_tokens_dev, b->at<int32_t>(L.tok_index), b->m->embed, d.dtype, d.vocab,
                                 d.d_model, b->at<float>(L.x), rows, s));
            PassCfg pc;
            pc.rows = rows;
            pc.row_seq = b->at<int32_t>(L.row_seq);
            pc.seqs = b->at<SeqDesc>(L.chunk_desc);
            pc.n_seqs = r1 - r0;
            pc.max_seq_rows = max_seq;
            pc.pos_add = 0;
            pc.active = nullptr;
            pc.decode = false;
            pc.max_shared_pages = 0;
            pc.attn_flops = chunk_attn_flops(descs, d);
            HIP_TRY(run_layers(b, pc, s));
        }
        // LM head + log-softmax gather over the scoring rows of this chunk, lm_chunk rows at a time
        HIP_TRY(upload(b, b->stage_i32, lm_idx, L.lm_idx, s));
        const int n_lm = (int)lm_idx.size();
        const int out0 = cu_suffix_host[r0];
        for (int c0 = 0; c0 < n_lm; c0 += lm_chunk) {
            const int n = std::min(lm_chunk, n_lm - c0);
            HIP_TRY(lm_head_logprob_rows(b, b->at<int32_t>(L.lm_idx) + c0, n, suffix_tokens_dev + out0 + c0, inv_t,
                                         logprobs_out_dev + out0 + c0, b->at<float>(L.logits), s));
        }
        if (r1 == r0) return fail(RPO_EINVAL, "rpo_suffix_logprobs: a suffix does not fit max_rows");
        r0 = r1;
    }
    return RPO_OK;
}

// ---------------------------------------------------------------------------
extern "C" int rpo_sample(const float* logits_dev, int32_t n_logit_rows, int32_t vocab, int64_t row_stride,
                          const int32_t* row_map_dev, int32_t n_out_rows, float temperature, uint64_t seed,
                          const uint64_t* seq_id_dev, uint32_t step, int32_t* tokens_out_dev,
                          float* logprob_out_dev, int32_t eos_id, uint8_t* active_inout_dev,
                          int32_t* lengths_inout_dev, const float* row_max_dev, void* stream) {
    if (!logits_dev || !seq_id_dev || !tokens_out_dev) return fail(RPO_EINVAL, "rpo_sample: NULL argument");
    if (n_logit_rows < 1 || vocab < 1 || vocab > 262144 || row_stride < vocab || n_out_rows < 0)
        return fail(RPO_EINVAL, "rpo_sample: bad sizes (vocab 1..262144, row_stride >= vocab)");
    if (!row_map_dev && n_out_rows > n_logit_rows)
        return fail(RPO_EINVAL, "rpo_sample: more output rows than logits rows without a row map");
    if (!(temperature > 0.f) || isinf(temperature)) return fail(RPO_EINVAL, "rpo_sample: temperature must be finite and > 0");
    SampleArgs a;
    a.logits = logits_dev;
    a.n_logit_rows = n_logit_rows;
    a.vocab = vocab;
    a.row_stride = row_stride;
    a.row_map = row_map_dev;
    a.n_out_rows = n_out_rows;
    a.inv_t = 1.0f / temperature;
    a.seed = seed;
    a.seq_id = seq_id_dev;
    a.step = step;
    a.tokens_out = tokens_out_dev;
    a.logprob_out = logprob_out_dev;
    a.eos_id = eos_id >= vocab ? -1 : eos_id;
    a.active = active_inout_dev;
    a.lengths = lengths_inout_dev;
    a.row_max = row_max_dev;
    HIP_TRY(timed(kKidSample, 0.0, (double)n_out_rows * vocab * 4.0, (hipStream_t)stream,
                  [&] { return launch_sample(a, (hipStream_t)stream); }));
    return RPO_OK;
}

extern "C" int grpo_advantages(const float* rewards_dev, int32_t n_groups, int32_t G, int32_t ddof, float eps,
                               float* adv_out_dev, void* stream) {
    if (!rewards_dev || !adv_out_dev) return fail(RPO_EINVAL, "grpo_advantages: NULL argument");
    if (n_groups < 0 || G < 1) return fail(RPO_EINVAL, "grpo_advantages: bad sizes");
    if ((ddof != 0 && ddof != 1) || ddof >= G) return fail(RPO_EINVAL, "grpo_advantages: ddof must be 0 or 1 and < G");
    if (!(eps >= 0.f)) return fail(RPO_EINVAL, "grpo_advantages: eps must be >= 0");
    HIP_TRY(launch_advantages(rewards_dev, n_groups, G, ddof, eps, adv_out_dev, (hipStream_t)stream));
    return RPO_OK;
}

extern "C" int rpo_objective_forward(const float* lp_new_dev, const float* lp_old_dev, const float* lp_ref_dev,
                                     const int32_t* cu_suffix_dev, const float* adv_dev, int32_t n_groups,
                                     int32_t G, float eps_clip, float beta, float* token_out_dev,
                                     double* rollout_scratch_dev, float* group_out_dev, void* stream) {
    if (!lp_new_dev || !lp_old_dev || !cu_suffix_dev || !adv_dev || !rollout_scratch_dev || !group_out_dev)
        return fail(RPO_EINVAL, "rpo_objective_forward: NULL argument");
    if (n_groups < 0 || G < 1) return fail(RPO_EINVAL, "rpo_objective_forward: bad sizes");
    if (!(eps_clip >= 0.f) || !(beta >= 0.f)) return fail(RPO_EINVAL, "rpo_objective_forward: eps_clip, beta must be >= 0");
    if (beta > 0.f && !lp_ref_dev) return fail(RPO_EINVAL, "rpo_objective_forward: beta > 0 needs reference log-probs");
    HIP_TRY(launch_objective(lp_new_dev, lp_old_dev, beta > 0.f ? lp_ref_dev : nullptr, cu_suffix_dev, adv_dev,
                             n_groups, G, eps_clip, beta, token_out_dev, rollout_scratch_dev, group_out_dev,
                             (hipStream_t)stream));
    return RPO_OK;
}

extern "C" int rpo_shape_rewards(const float* rewards_dev, const int32_t* lengths_dev, int32_t n_groups, int32_t G,
                                 float alpha, float lo, float hi, float* shaped_out_dev, void* stream) {
    if (!rewards_dev || !lengths_dev || !shaped_out_dev) return fail(RPO_EINVAL, "rpo_shape_rewards: NULL argument");
    if (n_groups < 0 || G < 1) return fail(RPO_EINVAL, "rpo_shape_rewards: bad sizes");
    if (!(alpha > 0.f) || !(lo <= hi)) return fail(RPO_EINVAL, "rpo_shape_rewards: need alpha > 0 and lo <= hi");
    HIP_TRY(launch_shape_rewards(rewards_dev, lengths_dev, n_groups, G, alpha, lo, hi, shaped_out_dev,
                                 (hipStream_t)stream));
    return RPO_OK;
}

extern "C" int rpo_cut_pack(const int32_t* prompts_dev, int64_t prompt_stride, const int32_t* prompt_len_dev,
                            const int32_t* pool_dev, int64_t pool_stride, const int32_t* question_dev,
                            const int32_t* cu_len_dev, int32_t n_groups, int32_t* tokens_out_dev, void* stream) {
    if (!prompts_dev || !prompt_len_dev || !pool_dev || !cu_len_dev || !tokens_out_dev)
        return fail(RPO_EINVAL, "rpo_cut_pack: NULL argument");
    if (n_groups < 0 || prompt_stride < 0 || pool_stride < 0) return fail(RPO_EINVAL, "rpo_cut_pack: bad sizes");
    HIP_TRY(launch_cut_pack(prompts_dev, prompt_stride, prompt_len_dev, pool_dev, pool_stride, question_dev,
                            cu_len_dev, n_groups, tokens_out_dev, (hipStream_t)stream));
    return RPO_OK;
}

extern "C" int rpo_cache_update(int32_t* pool_dev, int64_t pool_stride, int32_t* answer_len_dev,
                                const int32_t* question_dev, const int32_t* m_dev, const int32_t* tokens_dev, int64_t tok_stride,
                                const int32_t* lengths_dev, const float* rewards_dev, const float* u_dev,
                                const int32_t* g_prime_dev, int32_t n_groups, int32_t G, float eps,
                                int32_t* chosen_out_dev, void* stream) {
    if (!pool_dev || !answer_len_dev || !m_dev || !tokens_dev || !rewards_dev || !u_dev || !g_prime_dev)
        return fail(RPO_EINVAL, "rpo_cache_update: NULL argument");
    if (n_groups < 0 || G < 1 || pool_stride < 1 || tok_stride < 0)
        return fail(RPO_EINVAL, "rpo_cache_update: bad sizes");
    if (!(eps >= 0.f) || !(eps <= 1.f)) return fail(RPO_EINVAL, "rpo_cache_update: eps must be in [0, 1]");
    HIP_TRY(launch_cache_update(pool_dev, pool_stride, answer_len_dev, question_dev, m_dev, tokens_dev, tok_stride, lengths_dev,
                                rewards_dev, u_dev, g_prime_dev, n_groups, G, eps, chosen_out_dev,
                                (hipStream_t)stream));
    return RPO_OK;
}

// ---------------------------------------------------------------------------
extern "C" int rpo_gemm_nt(const void* a_dev, int64_t lda, const void* w_dev, int64_t ldw, void* c_dev,
                           int64_t ldc, int32_t M, int32_t N, int32_t K, int32_t dtype, int32_t epilogue,
                           void* ws_dev, size_t ws_bytes, void* stream) {
    if (!a_dev || !w_dev || !c_dev) return fail(RPO_EINVAL, "rpo_gemm_nt: NULL argument");
    if (M < 0 || N < 0 || K < 1 || lda < K || ldw < K || ldc < (epilogue == 3 ? N / 2 : N))
        return fail(RPO_EINVAL, "rpo_gemm_nt: bad sizes");
    if (dtype != RPO_F32 && dtype != RPO_BF16) return fail(RPO_EINVAL, "rpo_gemm_nt: unknown dtype");
    if (epilogue < 0 || epilogue > 3) return fail(RPO_EINVAL, "rpo_gemm_nt: unknown epilogue");
    if (epilogue == 3 && (N % 2)) return fail(RPO_EINVAL, "rpo_gemm_nt: SwiGLU needs N = 2F");
    if ((ws_dev == nullptr) != (ws_bytes == 0)) return fail(RPO_EINVAL, "rpo_gemm_nt: ws_dev / ws_bytes mismatch");
    GemmArgs g;
    g.A = a_dev;
    g.lda = lda;
    g.W = w_dev;
    g.ldw = ldw;
    g.C = c_dev;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.dtype = dtype;
    g.epilogue = epilogue;
    g.path = g_kernel_path;
    g.ws = ws_dev;
    g.ws_bytes = ws_bytes;
    const double es = (double)dtype_size(dtype);
    const double out_bytes = epilogue == kEpiStore ? (double)M * N * es
                             : epilogue == kEpiStoreF32 ? (double)M * N * 4.0
                             : epilogue == kEpiAddF32 ? (double)M * N * 8.0
                                                      : (double)M * (N / 2) * es;
    HIP_TRY(timed(gemm_kernel_id(g), 2.0 * M * N * K, ((double)M * K + (double)N * K) * es + out_bytes,
                  (hipStream_t)stream, [&] { return launch_gemm(g, (hipStream_t)stream); }));
    return RPO_OK;
}

// ---------------------------------------------------------------------------
// rpo_gemm_nt without a workspace argument and without any allocation: the K-split partial
// sums go to a fixed device array that is part of the library's code object.
// ---------------------------------------------------------------------------
namespace {
constexpr size_t kScratchBytes = (size_t)16 << 20;
constexpr int kMaxDevices = 64;
}  // namespace
// One copy per GPU the library is loaded on, held until the process ends.  In host code this
// name is only a handle for hipGetSymbolAddress: kernels and copies take the looked-up pointer.
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
namespace {
void* g_scratch_ptr[kMaxDevices] = {};  // device address of `scratch` on each device, looked up once
}

extern "C" int rpo_gemm_nt_noalloc(const void* a_dev, int64_t lda, const void* w_dev, int64_t ldw, void* c_dev,
                                   int64_t ldc, int32_t M, int32_t N, int32_t K, int32_t dtype, int32_t epilogue,
                                   void* stream) {
    if (!a_dev || !w_dev || !c_dev) return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: NULL argument");
    if (M < 0 || N < 0 || K < 1 || lda < K || ldw < K || ldc < (epilogue == 3 ? N / 2 : N))
        return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: bad sizes");
    if (dtype != RPO_F32 && dtype != RPO_BF16) return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: unknown dtype");
    if (epilogue < 0 || epilogue > 3) return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: unknown epilogue");
    if (epilogue == 3 && (N % 2)) return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: SwiGLU needs N = 2F");
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(RPO_EINVAL, "rpo_gemm_nt_noalloc: device index %d not supported", dev);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(RPO_EHIP, "rpo_gemm_nt_noalloc: the scratch array has no device address");
        g_scratch_ptr[dev] = p;
    }
    GemmArgs g;
    g.A = a_dev;
    g.lda = lda;
    g.W = w_dev;
    g.ldw = ldw;
    g.C = c_dev;
    g.ldc = ldc;
    g.M = M;
    g.N = N;
    g.K = K;
    g.dtype = dtype;
    g.epilogue = epilogue;
    g.path = g_kernel_path;
    g.ws = g_scratch_ptr[dev];
    g.ws_bytes = kScratchBytes;
    const size_t need = gemm_splitk_scratch_bytes(g);
    if (need > kScratchBytes)
        return fail(RPO_ENOMEM,
                    "rpo_gemm_nt_noalloc: this problem splits K and needs %zu bytes of partial sums; the static "
                    "scratch holds %zu (use rpo_gemm_nt with a workspace)", need, kScratchBytes);
    HIP_TRY(launch_gemm(g, (hipStream_t)stream));
    return RPO_OK;
}
