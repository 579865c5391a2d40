// C ABI of libspd: model object over caller-owned buffers and the orchestration of
// one decoder forward (verify step / draft step / prefill) out of the HIP kernels.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/spd.h"
#include "launch.h"

using namespace spd;

namespace {

thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
int32_t fail(int32_t code, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                          \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess)                                                                  \
            return fail(SPD_ERR_HIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_),    \
                        __FILE__, __LINE__);                                                   \
    } while (0)

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }


struct Layout {                    // byte offsets inside the three buffers
    // packed
    size_t embed, lm_head, final_norm;
    std::vector<size_t> attn_norm, wqkv, wo, mlp_norm, wgu, wdown;
    size_t packed_total;
    // kv
    size_t kv_layer_stride, kv_k_bytes, kv_v_bytes, kv_total;
    int v_stride;
    // workspace
    size_t h, qkv, xn, xo, xf, rope, logits, ssq_a, ssq_b, d_lens, d_error, qa_count, qa_abort, part, arrive, zero, ws_total;
};

int32_t check_shape(const spd_model_config &c) {
    if (c.n_layers < 1 || c.d_model < 32 || c.n_heads < 1 || c.d_ffn < 8 || c.vocab < 16 ||
        c.max_seqs < 1 || c.max_positions < 1)
        return fail(SPD_ERR_SHAPE, "non-positive dimension in spd_model_config");
    if (c.d_model % 32) return fail(SPD_ERR_SHAPE, "d_model %d must be a multiple of 32", c.d_model);
    if (c.head_dim != 64 && c.head_dim != 128)
        return fail(SPD_ERR_SHAPE, "head_dim %d must be 64 or 128", c.head_dim);
    if ((c.n_heads * c.head_dim) % 32)
        return fail(SPD_ERR_SHAPE, "n_heads*head_dim must be a multiple of 32");
    if (c.d_ffn % 8) return fail(SPD_ERR_SHAPE, "d_ffn %d must be a multiple of 8", c.d_ffn);
    if (c.vocab % 16) return fail(SPD_ERR_SHAPE, "vocab %d must be a multiple of 16", c.vocab);
    if (c.max_seqs > SPD_MAX_ROWS) return fail(SPD_ERR_SHAPE, "max_seqs %d exceeds %d", c.max_seqs, SPD_MAX_ROWS);
    if (!(c.rms_eps >= 0.f) || !(c.rope_theta > 0.f)) return fail(SPD_ERR_SHAPE, "bad rms_eps / rope_theta");
    return SPD_OK;
}

void make_layout(const spd_model_config &c, Layout &L) {
    const int d = c.d_model, HD = c.n_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    L.embed = take((size_t)V * d * 2);
    L.lm_head = take(packed_matrix_bytes(V, d));
    L.final_norm = take((size_t)d * 4);
    for (int l = 0; l < c.n_layers; ++l) {
        L.attn_norm.push_back(take((size_t)d * 4));
        L.wqkv.push_back(take(packed_matrix_bytes(3 * HD, d)));
        L.wo.push_back(take(packed_matrix_bytes(d, HD)));
        L.mlp_norm.push_back(take((size_t)d * 4));
        L.wgu.push_back(take(packed_matrix_bytes(2 * F, d)));
        L.wdown.push_back(take(packed_matrix_bytes(d, F)));
    }
    L.packed_total = off;

    L.v_stride = (c.max_positions + 31) / 32 * 32;         // V is stored transposed, rows padded to 32 positions
    L.kv_k_bytes = (size_t)c.max_seqs * c.n_heads * c.max_positions * c.head_dim * 2;
    L.kv_v_bytes = (size_t)c.max_seqs * c.n_heads * c.head_dim * L.v_stride * 2;
    L.kv_layer_stride = align_up(L.kv_k_bytes, 256) + align_up(L.kv_v_bytes, 256);
    L.kv_total = L.kv_layer_stride * c.n_layers;

    off = 0;
    const size_t KSd = d / 32, KShd = HD / 32, KSf = (F + 31) / 32;
    L.h = take((size_t)kMaxRows * d * 4);
    L.qkv = take((size_t)kMaxRows * 3 * HD * 4);
    L.xn = take((size_t)kMaxGroups * KSd * 1024);
    L.xo = take((size_t)kMaxGroups * KShd * 1024);
    L.xf = take((size_t)kMaxGroups * KSf * 1024);
    L.rope = take((size_t)c.max_positions * (c.head_dim / 2) * 2 * 4);
    L.logits = take((size_t)kMaxRows * V * 4);
    L.d_lens = take((size_t)kMaxRows * 4);
    L.d_error = take(4);
    L.qa_count = take((size_t)c.n_heads * 4);
    L.qa_abort = take(4);
    L.ssq_a = take((size_t)(d / 16) * kMaxRows * 4);
    L.ssq_b = take((size_t)(d / 16) * kMaxRows * 4);
    size_t pb = 0;
    for (size_t b : {gemm_batch_scratch_bytes(3 * HD, d), gemm_batch_scratch_bytes(d, HD), gemm_batch_scratch_bytes(2 * F, d),
                     gemm_batch_scratch_bytes(d, F), gemm_batch_scratch_bytes(V, d)})
        pb = b > pb ? b : pb;
    L.part = take(pb);
    L.arrive = take((size_t)kBatchMaxTileGroups * 4);
    L.zero = take(1024);
    L.ws_total = off;
}

GemmTuning default_tuning(int N, int K) {
    // Measured on MI355X at 5 rows: for K = 4096 (128 K-steps) the activation slice held in
    // registers and one persistent workgroup per CU is fastest, 8 waves x 16 steps for the
    // smaller matrices and 16 x 8 for the larger ones; otherwise fewer tiles -> more waves splitting K.
    int tiles = N / 16, KS = (K + 31) / 32;
    GemmTuning t;
    t.grid_cap = 0;
    t.ring = 8;
    t.no_regb = 0;
    t.no_batch = 0;
    t.force_batch = 0;
    if (KS == 128) t.waves = tiles >= 1024 ? 16 : 8;    // gate|up, LM head: 16 waves x 8 steps measured 1-2 % faster
    else if (KS == 64) t.waves = 8;
    else if (KS == 32) t.waves = 4;
    else if (tiles >= 1024) t.waves = 4;
    else if (tiles >= 512) t.waves = 8;
    else t.waves = 16;
    return t;
}

}  // namespace

struct spd_model {
    spd_model_config cfg;
    Layout L;
    char *packed, *kv, *ws;
    std::vector<int32_t> lens;         // KV lengths (host).  With dev_lens: only an upper bound
    bool dev_lens = false;             // the kernels read the lengths from device memory (ws + L.d_lens)
    bool fuse_qa = false;              // QKV projection + attention as one kernel where the shape allows it
    bool fuse_qa2 = false;             // ... also for 6..8 rows of one sequence
    bool fuse_qa_ok = false, fuse_qa2_ok = false;   // what the shape and the device allow (checked at creation)
    int attn_slices = 0;               // workgroups per head of the stand-alone attention kernel (0: chosen by batch size)
    unsigned spin_limit = 1u << 22;    // polls before a wait between workgroups gives up
    std::vector<float> rope_host;
    GemmTuning t_qkv, t_o, t_gu, t_down, t_lm;
    // optional tracing: HIP events around every launch group of a forward
    struct Span { int kind; hipEvent_t a, b; };
    bool prof_on = false;
    std::vector<Span> spans;
    std::vector<hipEvent_t> pool;
    hipEvent_t take_event() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
    ~spd_model() {
        for (auto &sp : spans) { (void)hipEventDestroy(sp.a); (void)hipEventDestroy(sp.b); }
        for (auto e : pool) (void)hipEventDestroy(e);
    }
};

namespace {
enum ProfKind { PK_QKV = 0, PK_O, PK_GATE_UP, PK_DOWN, PK_LM_HEAD, PK_ATTENTION, PK_EMBED, PK_COUNT };

// Runs one launch group; when tracing is on, brackets it with events on the same stream (the interval
// then includes the dispatch of the group's first kernel).
#define PROF_TRY(kind, expr)                                                                   \
    do {                                                                                       \
        spd_model::Span sp_{(kind), nullptr, nullptr};                                         \
        if (m->prof_on) {                                                                      \
            sp_.a = m->take_event(); sp_.b = m->take_event();                                  \
            if (!sp_.a || !sp_.b) return fail(SPD_ERR_HIP, "hipEventCreate failed");           \
            HIP_TRY(hipEventRecord(sp_.a, st));                                                \
        }                                                                                      \
        HIP_TRY(expr);                                                                         \
        if (m->prof_on) { HIP_TRY(hipEventRecord(sp_.b, st)); m->spans.push_back(sp_); }       \
    } while (0)

// Same for a group that is a single kernel whose launch wrapper can hand the two events to the launch
// itself: they then time the kernel's execution alone, which is what a profiler reports for it.
#define PROF_KERNEL(kind, expr)                                                                \
    do {                                                                                       \
        spd_model::Span sp_{(kind), nullptr, nullptr};                                         \
        LaunchTiming lt_{nullptr, nullptr, false};                                             \
        if (m->prof_on) {                                                                      \
            sp_.a = m->take_event(); sp_.b = m->take_event();                                  \
            if (!sp_.a || !sp_.b) return fail(SPD_ERR_HIP, "hipEventCreate failed");           \
            lt_.start = sp_.a; lt_.stop = sp_.b;                                               \
            launch_timing() = &lt_;                                                            \
        }                                                                                      \
        hipError_t pe_ = (expr);                                                               \
        launch_timing() = nullptr;                                                             \
        HIP_TRY(pe_);                                                                          \
        if (m->prof_on) {                                                                      \
            if (!lt_.used) return fail(SPD_ERR_HIP, "internal: the launch did not take its timing events"); \
            m->spans.push_back(sp_);                                                           \
        }                                                                                      \
    } while (0)

// a projection over one row group is a single kernel; more rows may take several passes
#define PROF_GEMM(kind, expr)                                                                  \
    do {                                                                                       \
        if (rows <= kGroupRows) PROF_KERNEL(kind, expr);                                       \
        else PROF_TRY(kind, expr);                                                             \
    } while (0)
}  // namespace



extern "C" {

const char *spd_last_error(void) { return g_err; }

int32_t spd_model_bytes(const spd_model_config *cfg, size_t *packed_bytes, size_t *kv_bytes,
                        size_t *workspace_bytes) {
    if (!cfg) return fail(SPD_ERR_INVALID_ARG, "NULL config");
    int32_t rc = check_shape(*cfg);
    if (rc) return rc;
    Layout L;
    make_layout(*cfg, L);
    if (packed_bytes) *packed_bytes = L.packed_total;
    if (kv_bytes) *kv_bytes = L.kv_total;
    if (workspace_bytes) *workspace_bytes = L.ws_total;
    return SPD_OK;
}

int32_t spd_model_create(const spd_model_config *cfg, const spd_weights *w, void *packed,
                         size_t packed_bytes, void *kv_cache, size_t kv_bytes, void *workspace,
                         size_t workspace_bytes, void *stream, spd_model **out) {
    if (!cfg || !w || !packed || !kv_cache || !workspace || !out)
        return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_model_create");
    int32_t rc = check_shape(*cfg);
    if (rc) return rc;
    if (((uintptr_t)packed | (uintptr_t)kv_cache | (uintptr_t)workspace) & 255)
        return fail(SPD_ERR_INVALID_ARG, "buffers must be 256-byte aligned");
    if (!w->embed || !w->final_norm || !w->attn_norm || !w->wq || !w->wk || !w->wv || !w->wo ||
        !w->mlp_norm || !w->w_gate || !w->w_up || !w->w_down || (!cfg->tied_embeddings && !w->lm_head))
        return fail(SPD_ERR_INVALID_ARG, "NULL weight pointer");
    spd_model *m = new (std::nothrow) spd_model;
    if (!m) return fail(SPD_ERR_INVALID_ARG, "out of host memory");
    m->cfg = *cfg;
    make_layout(*cfg, m->L);
    const Layout &L = m->L;
    if (packed_bytes < L.packed_total || kv_bytes < L.kv_total || workspace_bytes < L.ws_total) {
        delete m;
        return fail(SPD_ERR_CAPACITY, "buffer smaller than spd_model_bytes reports");
    }
    m->packed = (char *)packed;
    m->kv = (char *)kv_cache;
    m->ws = (char *)workspace;
    m->lens.assign(cfg->max_seqs, 0);
    hipStream_t st = (hipStream_t)stream;
    const int d = cfg->d_model, HD = cfg->n_heads * cfg->head_dim, F = cfg->d_ffn, V = cfg->vocab;

#define CREATE_TRY(expr)                                                                      \
    do {                                                                                       \
        hipError_t e_ = (expr);                                                                \
        if (e_ != hipSuccess) {                                                                \
            delete m;                                                                          \
            return fail(SPD_ERR_HIP, "%s failed: %s", #expr, hipGetErrorString(e_));           \
        }                                                                                      \
    } while (0)

    CREATE_TRY(hipMemcpyAsync(m->packed + L.embed, w->embed, (size_t)V * d * 2, hipMemcpyDeviceToDevice, st));
    CREATE_TRY(launch_pack_weight(cfg->tied_embeddings ? w->embed : w->lm_head, nullptr, nullptr, PACK_PLAIN,
                                  V, d, m->packed + L.lm_head, st));
    CREATE_TRY(hipMemcpyAsync(m->packed + L.final_norm, w->final_norm, (size_t)d * 4, hipMemcpyDeviceToDevice, st));
    for (int l = 0; l < cfg->n_layers; ++l) {
        if (!w->attn_norm[l] || !w->wq[l] || !w->wk[l] || !w->wv[l] || !w->wo[l] || !w->mlp_norm[l] ||
            !w->w_gate[l] || !w->w_up[l] || !w->w_down[l]) {
            delete m;
            return fail(SPD_ERR_INVALID_ARG, "NULL weight pointer in layer %d", l);
        }
        CREATE_TRY(hipMemcpyAsync(m->packed + L.attn_norm[l], w->attn_norm[l], (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        CREATE_TRY(launch_pack_weight(w->wq[l], w->wk[l], w->wv[l], PACK_CONCAT3, 3 * HD, d, m->packed + L.wqkv[l], st));
        CREATE_TRY(launch_pack_weight(w->wo[l], nullptr, nullptr, PACK_PLAIN, d, HD, m->packed + L.wo[l], st));
        CREATE_TRY(hipMemcpyAsync(m->packed + L.mlp_norm[l], w->mlp_norm[l], (size_t)d * 4, hipMemcpyDeviceToDevice, st));
        CREATE_TRY(launch_pack_weight(w->w_gate[l], w->w_up[l], nullptr, PACK_GATE_UP, 2 * F, d, m->packed + L.wgu[l], st));
        CREATE_TRY(launch_pack_weight(w->w_down[l], nullptr, nullptr, PACK_PLAIN, d, F, m->packed + L.wdown[l], st));
    }
    // workspace starts cleared: the padding columns of the packed activation buffers must be zero;
    // the KV cache too: the attention kernel reads (and masks) whole 32-position units, so every
    // slot must hold a finite value
    CREATE_TRY(launch_fill_zero(m->ws, L.ws_total, st));
    CREATE_TRY(launch_fill_zero(m->kv, L.kv_total, st));
    // RoPE table: angle(pos, i) = pos * theta^(-2i/head_dim), computed in double
    const int half = cfg->head_dim / 2;
    m->rope_host.resize((size_t)cfg->max_positions * half * 2);
    for (int p = 0; p < cfg->max_positions; ++p)
        for (int i = 0; i < half; ++i) {
            double ang = (double)p * std::pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
            m->rope_host[((size_t)p * half + i) * 2 + 0] = (float)std::cos(ang);
            m->rope_host[((size_t)p * half + i) * 2 + 1] = (float)std::sin(ang);
        }
    CREATE_TRY(hipMemcpyAsync(m->ws + L.rope, m->rope_host.data(), m->rope_host.size() * 4, hipMemcpyHostToDevice, st));
#undef CREATE_TRY

    m->t_qkv = default_tuning(3 * HD, d);
    m->t_o = default_tuning(d, HD);
    m->t_gu = default_tuning(2 * F, d);
    m->t_down = default_tuning(d, F);
    m->t_lm = default_tuning(V, d);
    // QKV projection + attention as one kernel where the shape and the device allow it
    m->fuse_qa_ok = qkv_attention_supported(cfg->d_model, cfg->n_heads, cfg->head_dim, 1, 1, 1);
    m->fuse_qa2_ok = m->fuse_qa_ok && qkv_attention_supported(cfg->d_model, cfg->n_heads, cfg->head_dim, 8, 1, 8);
    m->fuse_qa = m->fuse_qa_ok;
    m->fuse_qa2 = m->fuse_qa2_ok;
    *out = m;
    return SPD_OK;
}

int32_t spd_model_set_tuning(spd_model *m, const spd_tuning *t) {
    if (!m || !t) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_model_set_tuning");
    if (t->batch_kernel < 0 || t->batch_kernel > 2) return fail(SPD_ERR_INVALID_ARG, "batch_kernel must be 0, 1 or 2");
    if (t->separate_qkv_attention != 0 && t->separate_qkv_attention != 1) return fail(SPD_ERR_INVALID_ARG, "separate_qkv_attention must be 0 or 1");
    if (t->attention_slices != 0 && t->attention_slices != 1 && t->attention_slices != 2 && t->attention_slices != 4 &&
        t->attention_slices != 8)
        return fail(SPD_ERR_INVALID_ARG, "attention_slices must be 0, 1, 2, 4 or 8");
    GemmTuning *gt[SPD_N_PROJECTIONS] = {&m->t_qkv, &m->t_o, &m->t_gu, &m->t_down, &m->t_lm};
    for (int i = 0; i < SPD_N_PROJECTIONS; ++i) {
        const int w = t->gemm_waves[i];
        if (w != 0 && w != 4 && w != 8 && w != 16) return fail(SPD_ERR_INVALID_ARG, "gemm_waves must be 0, 4, 8 or 16");
        if (t->gemm_grid_cap[i] < 0 || t->gemm_grid_cap[i] > 65535) return fail(SPD_ERR_INVALID_ARG, "gemm_grid_cap out of range");
        if (t->gemm_ring[i] != 0 && t->gemm_ring[i] != 8 && t->gemm_ring[i] != 16) return fail(SPD_ERR_INVALID_ARG, "gemm_ring must be 0, 8 or 16");
    }
    const spd_model_config &c = m->cfg;
    const int d = c.d_model, HD = c.n_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
    const int Ns[SPD_N_PROJECTIONS] = {3 * HD, d, 2 * F, d, V}, Ks[SPD_N_PROJECTIONS] = {d, HD, d, F, d};
    for (int i = 0; i < SPD_N_PROJECTIONS; ++i) {
        *gt[i] = default_tuning(Ns[i], Ks[i]);
        if (t->gemm_waves[i]) gt[i]->waves = t->gemm_waves[i];
        gt[i]->grid_cap = t->gemm_grid_cap[i];
        if (t->gemm_ring[i]) gt[i]->ring = t->gemm_ring[i];
        gt[i]->no_regb = t->gemm_general_kernel[i] ? 1 : 0;
        gt[i]->no_batch = t->batch_kernel == 2 ? 1 : 0;
        gt[i]->force_batch = t->batch_kernel == 1 ? 1 : 0;
    }
    m->fuse_qa = t->separate_qkv_attention ? false : m->fuse_qa_ok;
    m->fuse_qa2 = t->separate_qkv_attention ? false : m->fuse_qa2_ok;
    m->attn_slices = t->attention_slices;
    m->spin_limit = t->wait_spin_limit ? t->wait_spin_limit : (1u << 22);
    return SPD_OK;
}

int32_t spd_model_destroy(spd_model *m) {
    delete m;
    return SPD_OK;
}

int32_t spd_kv_set_len(spd_model *m, const int32_t *len, int32_t n_seqs) {
    if (!m || !len) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_kv_set_len");
    if (n_seqs < 0 || n_seqs > m->cfg.max_seqs) return fail(SPD_ERR_CAPACITY, "n_seqs %d exceeds max_seqs %d", n_seqs, m->cfg.max_seqs);
    for (int i = 0; i < n_seqs; ++i) {
        if (len[i] < 0) return fail(SPD_ERR_INVALID_ARG, "negative KV length");
        if (len[i] > m->cfg.max_positions) return fail(SPD_ERR_CAPACITY, "KV length %d exceeds max_positions %d", len[i], m->cfg.max_positions);
    }
    if (m->dev_lens) return fail(SPD_ERR_INVALID_ARG, "KV lengths live on the device: call spd_kv_lens_from_device first");
    for (int i = 0; i < n_seqs; ++i) m->lens[i] = len[i];
    return SPD_OK;
}

int32_t spd_kv_lens_to_device(spd_model *m, void *stream) {
    if (!m) return fail(SPD_ERR_INVALID_ARG, "NULL model");
    HIP_TRY(hipMemcpyAsync(m->ws + m->L.d_lens, m->lens.data(), (size_t)m->cfg.max_seqs * 4, hipMemcpyHostToDevice, (hipStream_t)stream));
    HIP_TRY(launch_fill_zero(m->ws + m->L.d_error, 16, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));          // the host array may change right after this call
    m->dev_lens = true;
    return SPD_OK;
}

int32_t spd_kv_lens_from_device(spd_model *m, void *stream) {
    if (!m) return fail(SPD_ERR_INVALID_ARG, "NULL model");
    if (!m->dev_lens) return SPD_OK;
    std::vector<int32_t> tmp((size_t)m->cfg.max_seqs + 1);
    HIP_TRY(hipMemcpyAsync(tmp.data(), m->ws + m->L.d_lens, (size_t)m->cfg.max_seqs * 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipMemcpyAsync(&tmp[m->cfg.max_seqs], m->ws + m->L.d_error, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    m->dev_lens = false;
    const bool overflow = tmp[m->cfg.max_seqs] != 0;
    for (int i = 0; i < m->cfg.max_seqs; ++i) m->lens[i] = std::max(0, std::min(tmp[i], m->cfg.max_positions));
    if (overflow) return fail(SPD_ERR_CAPACITY, "a forward ran with a device KV length that left no room for its rows");
    return SPD_OK;
}

int32_t spd_device_status(spd_model *m, void *stream) {
    if (!m) return fail(SPD_ERR_INVALID_ARG, "NULL model");
    int32_t flags[2] = {0, 0};
    HIP_TRY(hipMemcpyAsync(&flags[0], m->ws + m->L.d_error, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipMemcpyAsync(&flags[1], m->ws + m->L.qa_abort, 4, hipMemcpyDeviceToHost, (hipStream_t)stream));
    HIP_TRY(hipStreamSynchronize((hipStream_t)stream));
    if (flags[1]) return fail(SPD_ERR_HIP, "a wait between workgroups hit its spin limit: results since then are invalid");
    if (flags[0]) return fail(SPD_ERR_CAPACITY, "a forward ran with a device KV length that left no room for its rows");
    return SPD_OK;
}

int32_t spd_kv_export(spd_model *m, int32_t layer, int32_t seq, int32_t pos0, int32_t n, float *k_out, float *v_out, void *stream) {
    if (!m || !k_out || !v_out) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_kv_export");
    const spd_model_config &c = m->cfg;
    if (layer < 0 || layer >= c.n_layers || seq < 0 || seq >= c.max_seqs) return fail(SPD_ERR_INVALID_ARG, "layer / sequence index out of range");
    if (n < 1 || pos0 < 0 || pos0 + n > c.max_positions) return fail(SPD_ERR_CAPACITY, "positions %d..%d outside the cache (%d)", pos0, pos0 + n - 1, c.max_positions);
    const Layout &L = m->L;
    const char *kv_l = m->kv + (size_t)layer * L.kv_layer_stride;
    const char *k = kv_l + (size_t)seq * c.n_heads * c.max_positions * c.head_dim * 2;
    const char *v = kv_l + align_up(L.kv_k_bytes, 256) + (size_t)seq * c.n_heads * c.head_dim * L.v_stride * 2;
    HIP_TRY(launch_kv_export(k, v, c.n_heads, c.head_dim, c.max_positions, pos0, n, k_out, v_out, (hipStream_t)stream));
    return SPD_OK;
}

int32_t spd_kv_get_len(const spd_model *m, int32_t *len, int32_t n_seqs) {
    if (!m || !len) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_kv_get_len");
    if (n_seqs < 0 || n_seqs > m->cfg.max_seqs) return fail(SPD_ERR_CAPACITY, "n_seqs exceeds max_seqs");
    for (int i = 0; i < n_seqs; ++i) len[i] = m->lens[i];
    return SPD_OK;
}

}  // extern "C"

namespace {

// One decoder forward over M new rows for sequences seq0 .. seq0 + n_seqs - 1.
// Input rows come from token ids (embedding gather) or from embedding rows.
// max_m: SPD_MAX_M for the public calls; the prefill feeds one sequence up to 64 rows per pass.
int32_t forward(spd_model *m, const int32_t *tokens, int token_stride, const float *embeds, int seq0, int n_seqs, int M,
                float *logits_out, hipStream_t st, int max_m = SPD_MAX_M) {
    const spd_model_config &c = m->cfg;
    const Layout &L = m->L;
    const int rows = n_seqs * M;
    if (M < 1 || M > max_m) return fail(SPD_ERR_SHAPE, "M = %d must be in 1..%d", M, max_m);
    if (n_seqs < 1 || rows > SPD_MAX_ROWS) return fail(SPD_ERR_SHAPE, "n_seqs * M = %d must be in 1..%d", rows, SPD_MAX_ROWS);
    if (seq0 < 0 || seq0 + n_seqs > c.max_seqs) return fail(SPD_ERR_CAPACITY, "sequence index beyond max_seqs %d", c.max_seqs);
    if (M > c.max_positions) return fail(SPD_ERR_CAPACITY, "M = %d exceeds max_positions %d", M, c.max_positions);
    if (tokens && token_stride < M) return fail(SPD_ERR_INVALID_ARG, "token stride %d below M = %d", token_stride, M);
    AttnArgs at{};
    for (int s = 0; s < n_seqs; ++s) {
        int len = m->lens[seq0 + s];
        // lengths on the device: the host value is an upper bound and the kernels guard themselves
        if (!m->dev_lens && len + M > c.max_positions)
            return fail(SPD_ERR_CAPACITY, "KV cache overflow: sequence %d has %d positions, +%d > %d", seq0 + s, len, M, c.max_positions);
        at.lens.len[s] = len;
    }
    if (m->dev_lens) {
        at.d_lens = (const int32_t *)(m->ws + L.d_lens) + seq0;
        at.d_error = (int32_t *)(m->ws + L.d_error);
    }
    const int d = c.d_model, HD = c.n_heads * c.head_dim, F = c.d_ffn, V = c.vocab;
    float *h = (float *)(m->ws + L.h);
    float *qkv = (float *)(m->ws + L.qkv);
    void *xn = m->ws + L.xn, *xo = m->ws + L.xo, *xf = m->ws + L.xf;

    float *ssq_a = (float *)(m->ws + L.ssq_a), *ssq_b = (float *)(m->ws + L.ssq_b);
    const int d_tiles = d / 16;
    auto gain_of = [&](size_t off) { return (const float *)(m->packed + off); };

    // input rows -> h, packed (h * attn_norm[0]) and sum of squares (one part per row)
    PROF_TRY(PK_EMBED, launch_input_rows(m->packed + L.embed, tokens, M, tokens ? token_stride : M, embeds, rows, d, V,
                                         gain_of(L.attn_norm[0]), h, xn, ssq_b, st));

    at.qkv = qkv;
    at.rope = (const float *)(m->ws + L.rope);
    at.xout = xo;
    at.n_seqs = n_seqs; at.M = M; at.H = c.n_heads; at.dh = c.head_dim; at.max_positions = c.max_positions;
    at.v_stride = L.v_stride;
    at.slices = m->attn_slices;

    const bool fused = m->fuse_qa && n_seqs == 1 && (rows <= kGroupRows || (rows <= 8 && m->fuse_qa2));   // shapes checked at creation
    for (int l = 0; l < c.n_layers; ++l) {
        // RMSNorm is folded into the projections: the producer of h (input rows / O / down
        // epilogue) leaves packed (h * gain) and per-tile sums of squares; the consumer
        // scales its accumulators by 1 / rms.
        char *kv_l = m->kv + (size_t)l * L.kv_layer_stride;
        at.k_cache = kv_l + (size_t)seq0 * c.n_heads * c.max_positions * c.head_dim * 2;
        at.v_cache = kv_l + align_up(L.kv_k_bytes, 256) + (size_t)seq0 * c.n_heads * c.head_dim * L.v_stride * 2;
        GemmArgs g{};
        g.batch_partials = (float *)(m->ws + L.part); g.batch_arrive = (unsigned *)(m->ws + L.arrive); g.batch_zero = m->ws + L.zero;
        if (fused) {
            QkvAttnArgs qa{};
            qa.W = m->packed + L.wqkv[l]; qa.X = xn; qa.K = d; qa.rows = rows;
            qa.ssq_in = ssq_b; qa.ssq_in_parts = (l == 0) ? 1 : d_tiles; qa.eps = c.rms_eps;
            at.m0 = 0; at.Mq = M;
            qa.at = at;
            qa.head_count = (unsigned *)(m->ws + L.qa_count); qa.spin_limit = m->spin_limit;
            qa.abort_flag = (int *)(m->ws + L.qa_abort);
            PROF_KERNEL(PK_QKV, launch_qkv_attention(qa, st));
        } else {
            g.W = m->packed + L.wqkv[l]; g.X = xn; g.N = 3 * HD; g.K = d; g.rows = rows; g.Y = qkv; g.ldy = 3 * HD;
            g.ssq_in = ssq_b; g.ssq_in_parts = (l == 0) ? 1 : d_tiles; g.eps = c.rms_eps;
            PROF_GEMM(PK_QKV, launch_gemm(g, EPI_STORE, m->t_qkv, st));
            for (int m0 = 0; m0 < M; m0 += 8) {         // at most 8 queries per sequence and launch
                at.m0 = m0; at.Mq = std::min(8, M - m0);
                PROF_TRY(PK_ATTENTION, launch_attention(at, st));
            }
        }
        g = GemmArgs{};
        g.batch_partials = (float *)(m->ws + L.part); g.batch_arrive = (unsigned *)(m->ws + L.arrive); g.batch_zero = m->ws + L.zero;
        g.W = m->packed + L.wo[l]; g.X = xo; g.N = d; g.K = HD; g.rows = rows; g.Y = h; g.ldy = d;
        g.gain_next = gain_of(L.mlp_norm[l]); g.Xnext = xn; g.ssq_out = ssq_a;
        PROF_GEMM(PK_O, launch_gemm(g, EPI_RESIDUAL, m->t_o, st));
        g = GemmArgs{};
        g.batch_partials = (float *)(m->ws + L.part); g.batch_arrive = (unsigned *)(m->ws + L.arrive); g.batch_zero = m->ws + L.zero;
        g.W = m->packed + L.wgu[l]; g.X = xn; g.N = 2 * F; g.K = d; g.rows = rows; g.Xout = xf; g.K_out = F;
        g.ssq_in = ssq_a; g.ssq_in_parts = d_tiles; g.eps = c.rms_eps;
        PROF_GEMM(PK_GATE_UP, launch_gemm(g, EPI_SWIGLU, m->t_gu, st));
        g = GemmArgs{};
        g.batch_partials = (float *)(m->ws + L.part); g.batch_arrive = (unsigned *)(m->ws + L.arrive); g.batch_zero = m->ws + L.zero;
        g.W = m->packed + L.wdown[l]; g.X = xf; g.N = d; g.K = F; g.rows = rows; g.Y = h; g.ldy = d;
        g.gain_next = gain_of(l + 1 < c.n_layers ? L.attn_norm[l + 1] : L.final_norm); g.Xnext = xn; g.ssq_out = ssq_b;
        PROF_GEMM(PK_DOWN, launch_gemm(g, EPI_RESIDUAL, m->t_down, st));
    }
    if (logits_out) {
        GemmArgs g{};
        g.batch_partials = (float *)(m->ws + L.part); g.batch_arrive = (unsigned *)(m->ws + L.arrive); g.batch_zero = m->ws + L.zero;
        g.W = m->packed + L.lm_head; g.X = xn; g.N = V; g.K = d; g.rows = rows; g.Y = logits_out; g.ldy = V;
        g.ssq_in = ssq_b; g.ssq_in_parts = d_tiles; g.eps = c.rms_eps;
        PROF_GEMM(PK_LM_HEAD, launch_gemm(g, EPI_STORE, m->t_lm, st));
    }
    if (m->dev_lens) HIP_TRY(launch_lens_add((int32_t *)(m->ws + L.d_lens) + seq0, n_seqs, M, st));
    for (int s = 0; s < n_seqs; ++s) m->lens[seq0 + s] = std::min(m->lens[seq0 + s] + M, c.max_positions);
    return SPD_OK;
}

int32_t prefill_common(spd_model *m, int32_t seq, const float *embeds, const int32_t *tokens, int32_t n_rows,
                       float *last_logits, hipStream_t st) {
    if (!m || (!embeds && !tokens)) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_prefill");
    if (n_rows < 1) return fail(SPD_ERR_INVALID_ARG, "n_rows must be positive");
    if (seq < 0 || seq >= m->cfg.max_seqs) return fail(SPD_ERR_CAPACITY, "sequence index %d beyond max_seqs %d", seq, m->cfg.max_seqs);
    if (m->lens[seq] + n_rows > m->cfg.max_positions)
        return fail(SPD_ERR_CAPACITY, "KV cache overflow in prefill: %d + %d > %d", m->lens[seq], n_rows, m->cfg.max_positions);
    float *scratch = (float *)(m->ws + m->L.logits);
    // rows per pass over the weights: 64 through the batched projection kernel (measured 0.108 ms per row at the 7B
    // shape against 0.128 for passes of 40), 40 (8 row groups) through the K-splitting kernel otherwise
    const bool batched = m->L.part != 0 && !m->t_qkv.no_batch;
    const int pass_rows = batched ? SPD_MAX_ROWS : 8 * kGroupRows;
    for (int r0 = 0; r0 < n_rows; r0 += pass_rows) {
        int M = n_rows - r0 < pass_rows ? n_rows - r0 : pass_rows;
        bool last = r0 + M >= n_rows;
        int32_t rc = forward(m, tokens ? tokens + r0 : nullptr, M, embeds ? embeds + (size_t)r0 * m->cfg.d_model : nullptr,
                             seq, 1, M, (last && last_logits) ? scratch : nullptr, st, pass_rows);
        if (rc) return rc;
        if (last && last_logits)
            HIP_TRY(hipMemcpyAsync(last_logits, scratch + (size_t)(M - 1) * m->cfg.vocab, (size_t)m->cfg.vocab * 4,
                                   hipMemcpyDeviceToDevice, st));
    }
    return SPD_OK;
}

}  // namespace

extern "C" {

int32_t spd_trace_enable(spd_model *m, int32_t enable) {
    if (!m) return fail(SPD_ERR_INVALID_ARG, "NULL model");
    m->prof_on = enable != 0;
    return SPD_OK;
}

int32_t spd_trace_read(spd_model *m, int32_t n_kinds, double *ms_sum, int32_t *count) {
    if (!m || !ms_sum || !count || n_kinds < 1) return fail(SPD_ERR_INVALID_ARG, "bad argument to spd_trace_read");
    for (int i = 0; i < n_kinds; ++i) { ms_sum[i] = 0.0; count[i] = 0; }
    for (auto &sp : m->spans) {
        HIP_TRY(hipEventSynchronize(sp.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, sp.a, sp.b));
        if (sp.kind < n_kinds) { ms_sum[sp.kind] += ms; count[sp.kind] += 1; }
        m->pool.push_back(sp.a);
        m->pool.push_back(sp.b);
    }
    m->spans.clear();
    return SPD_OK;
}

int32_t spd_prefill(spd_model *m, int32_t seq, const float *embeds, int32_t n_rows, float *last_logits, void *stream) {
    if (!embeds) return fail(SPD_ERR_INVALID_ARG, "NULL embeds");
    return prefill_common(m, seq, embeds, nullptr, n_rows, last_logits, (hipStream_t)stream);
}

int32_t spd_prefill_tokens(spd_model *m, int32_t seq, const int32_t *tokens, int32_t n_rows, float *last_logits, void *stream) {
    if (!tokens) return fail(SPD_ERR_INVALID_ARG, "NULL tokens");
    return prefill_common(m, seq, nullptr, tokens, n_rows, last_logits, (hipStream_t)stream);
}

int32_t spd_verify_forward(spd_model *m, const int32_t *tokens, int32_t n_seqs, int32_t M, float *logits_out, void *stream) {
    if (!m || !tokens || !logits_out) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_verify_forward");
    return forward(m, tokens, M, nullptr, 0, n_seqs, M, logits_out, (hipStream_t)stream);
}

int32_t spd_draft_step_strided(spd_model *m, const int32_t *tokens_in, int32_t in_stride, int32_t n_seqs, int32_t n_in,
                               float temperature, const float *u_draft, int32_t u_stride, float *D_row_out,
                               size_t D_stride, int32_t *token_out, int32_t token_stride, void *stream) {
    if (!m || !tokens_in || !u_draft || !D_row_out || !token_out) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_draft_step");
    if (n_in < 1 || n_in > 2) return fail(SPD_ERR_SHAPE, "n_in = %d must be 1 or 2", n_in);
    if (!(temperature >= 0.f)) return fail(SPD_ERR_INVALID_ARG, "temperature must be >= 0");
    if (in_stride < n_in || u_stride < 1 || token_stride < 1 || D_stride < (size_t)m->cfg.vocab)
        return fail(SPD_ERR_INVALID_ARG, "strides must cover one sequence's entries");
    float *scratch = (float *)(m->ws + m->L.logits);
    int32_t rc = forward(m, tokens_in, in_stride, nullptr, 0, n_seqs, n_in, scratch, (hipStream_t)stream);
    if (rc) return rc;
    const size_t V = m->cfg.vocab;
    HIP_TRY(launch_softmax_sample(scratch + (size_t)(n_in - 1) * V, (size_t)n_in * V, n_seqs, (int)V, temperature,
                                  u_draft, u_stride, D_row_out, D_stride, token_out, token_stride, (hipStream_t)stream));
    return SPD_OK;
}

int32_t spd_draft_step(spd_model *m, const int32_t *tokens_in, int32_t n_seqs, int32_t n_in, float temperature,
                       const float *u_draft, float *D_row_out, int32_t *token_out, void *stream) {
    if (!m) return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_draft_step");
    return spd_draft_step_strided(m, tokens_in, n_in, n_seqs, n_in, temperature, u_draft, 1, D_row_out,
                                  (size_t)m->cfg.vocab, token_out, 1, stream);
}

int32_t spd_accept_workspace_bytes(int32_t n_seqs, int32_t gamma, int32_t vocab, size_t *bytes) {
    if (!bytes || n_seqs < 1 || gamma < 1 || vocab < 1) return fail(SPD_ERR_INVALID_ARG, "bad argument to spd_accept_workspace_bytes");
    *bytes = accept_workspace_bytes(n_seqs, gamma);
    return SPD_OK;
}

int32_t spd_speculative_accept(const float *target, const float *draft, const int32_t *draft_tokens, const float *u,
                               int32_t n_seqs, int32_t gamma, int32_t vocab, float temperature, uint32_t flags,
                               int32_t *n_accepted_out, int32_t *next_token_out, float *accept_prob_out,
                               void *workspace, size_t workspace_bytes, void *stream) {
    if (!target || !draft || !draft_tokens || !u || !n_accepted_out || !next_token_out || !workspace)
        return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_speculative_accept");
    if (n_seqs < 1 || gamma < 1 || gamma > 63 || vocab < 1) return fail(SPD_ERR_INVALID_ARG, "n_seqs, vocab >= 1 and 1 <= gamma <= 63 required");
    if (!(temperature >= 0.f)) return fail(SPD_ERR_INVALID_ARG, "temperature must be >= 0");
    if (flags & ~3u) return fail(SPD_ERR_INVALID_ARG, "unknown flag bits");
    if (workspace_bytes < accept_workspace_bytes(n_seqs, gamma)) return fail(SPD_ERR_CAPACITY, "accept workspace too small");
    AcceptArgs a;
    a.target = target; a.draft = draft; a.draft_tokens = draft_tokens; a.u = u;
    a.n_seqs = n_seqs; a.gamma = gamma; a.vocab = vocab; a.temperature = temperature; a.flags = flags;
    a.n_accepted = n_accepted_out; a.next_token = next_token_out; a.accept_prob = accept_prob_out;
    a.token_stride = gamma;
    a.stats = (float *)workspace;
    HIP_TRY(launch_accept(a, (hipStream_t)stream));
    return SPD_OK;
}

}  // extern "C"

// ---- accept / resample for callers that cannot allocate ----------------------------------------
// The row statistics that spd_speculative_accept keeps in a caller-provided workspace live here in a
// fixed array in device memory.  Every GPU the library runs on holds its own copy at its own address;
// in host code the array's name is only a stand-in for it, so the address is looked up once per
// device (with that device current) and only that pointer is ever handed to a kernel.
namespace {
constexpr size_t kStaticAcceptBytes = 64 * 1024;          // 4096 rows of statistics
static __device__ __align__(256) unsigned char scratch[kStaticAcceptBytes];
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch(void **out) {
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(SPD_ERR_HIP, "device index %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(SPD_ERR_HIP, "hipGetSymbolAddress returned a NULL address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return SPD_OK;
}
}  // namespace

extern "C" {

int32_t spd_speculative_accept_static(const float *target, const float *draft, const int32_t *draft_tokens, const float *u,
                                      int32_t n_seqs, int32_t gamma, int32_t vocab, float temperature, uint32_t flags,
                                      int32_t *n_accepted_out, int32_t *next_token_out, float *accept_prob_out, void *stream) {
    if (!target || !draft || !draft_tokens || !u || !n_accepted_out || !next_token_out)
        return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_speculative_accept_static");
    if (n_seqs < 1 || gamma < 1 || gamma > 63 || vocab < 1) return fail(SPD_ERR_INVALID_ARG, "n_seqs, vocab >= 1 and 1 <= gamma <= 63 required");
    if (!(temperature >= 0.f)) return fail(SPD_ERR_INVALID_ARG, "temperature must be >= 0");
    if (flags & ~3u) return fail(SPD_ERR_INVALID_ARG, "unknown flag bits");
    if ((size_t)n_seqs > SPD_STATIC_ACCEPT_MAX_ROWS || accept_workspace_bytes(n_seqs, gamma) > kStaticAcceptBytes)
        return fail(SPD_ERR_CAPACITY, "n_seqs * (2 gamma + 1) = %lld rows exceed the %d rows of the built-in scratch array",
                    (long long)n_seqs * (2 * gamma + 1), SPD_STATIC_ACCEPT_MAX_ROWS);
    void *ws = nullptr;
    int32_t rc = static_scratch(&ws);
    if (rc) return rc;
    AcceptArgs a;
    a.target = target; a.draft = draft; a.draft_tokens = draft_tokens; a.u = u;
    a.n_seqs = n_seqs; a.gamma = gamma; a.vocab = vocab; a.temperature = temperature; a.flags = flags;
    a.n_accepted = n_accepted_out; a.next_token = next_token_out; a.accept_prob = accept_prob_out;
    a.token_stride = gamma;
    a.stats = (float *)ws;            // every entry the kernels read is written by this call first: nothing to clear
    HIP_TRY(launch_accept(a, (hipStream_t)stream));
    return SPD_OK;
}

int32_t spd_block_finish(spd_model *target, spd_model *draft, const float *target_logits, const float *draft_probs,
                         int32_t *verify_tokens, const float *u, int32_t n_seqs, int32_t gamma, float temperature,
                         int32_t *n_accepted_out, int32_t *next_token_out, int32_t *draft_in_out, int32_t *out_tokens,
                         int32_t out_capacity, int32_t *n_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (!target || !draft || !target_logits || !draft_probs || !verify_tokens || !u || !n_accepted_out || !next_token_out ||
        !draft_in_out || !workspace || (out_tokens && !n_out))
        return fail(SPD_ERR_INVALID_ARG, "NULL argument to spd_block_finish");
    if (!target->dev_lens || !draft->dev_lens)
        return fail(SPD_ERR_INVALID_ARG, "spd_block_finish needs both models' KV lengths on the device (spd_kv_lens_to_device)");
    if (n_seqs < 1 || n_seqs > target->cfg.max_seqs || n_seqs > draft->cfg.max_seqs) return fail(SPD_ERR_CAPACITY, "n_seqs exceeds max_seqs");
    if (gamma < 1 || gamma + 1 > SPD_MAX_M) return fail(SPD_ERR_SHAPE, "gamma + 1 must be in 2..%d", SPD_MAX_M);
    if (target->cfg.vocab != draft->cfg.vocab) return fail(SPD_ERR_SHAPE, "target and draft vocabularies differ");
    if (!(temperature >= 0.f)) return fail(SPD_ERR_INVALID_ARG, "temperature must be >= 0");
    if (out_tokens && out_capacity < 1) return fail(SPD_ERR_INVALID_ARG, "out_capacity must be positive");
    if (workspace_bytes < accept_workspace_bytes(n_seqs, gamma)) return fail(SPD_ERR_CAPACITY, "accept workspace too small");
    AcceptArgs a;
    a.target = target_logits; a.draft = draft_probs; a.draft_tokens = verify_tokens + 1; a.token_stride = gamma + 1; a.u = u;
    a.n_seqs = n_seqs; a.gamma = gamma; a.vocab = target->cfg.vocab; a.temperature = temperature; a.flags = SPD_DRAFT_IS_PROBS;
    a.n_accepted = n_accepted_out; a.next_token = next_token_out; a.accept_prob = nullptr;
    a.stats = (float *)workspace;
    HIP_TRY(launch_accept(a, (hipStream_t)stream));
    CommitArgs cm;
    cm.n_accepted = n_accepted_out; cm.next_token = next_token_out; cm.verify_tokens = verify_tokens; cm.draft_in = draft_in_out;
    cm.target_lens = (int32_t *)(target->ws + target->L.d_lens); cm.draft_lens = (int32_t *)(draft->ws + draft->L.d_lens);
    cm.out_tokens = out_tokens; cm.n_out = n_out; cm.n_seqs = n_seqs; cm.gamma = gamma; cm.out_capacity = out_capacity;
    HIP_TRY(launch_block_commit(cm, (hipStream_t)stream));
    // host bounds: at most gamma + 1 positions per sequence were added by the verify call and stay
    return SPD_OK;
}

}  // extern "C"
