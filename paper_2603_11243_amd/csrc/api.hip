// C-ABI layer: argument checks, host-side ragged-batch metadata, workspace carving, launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>

#include "ssd_internal.h"

using namespace ssd;

namespace {

// Pinned host staging for per-call metadata.  A ring of slots, each guarded by an event recorded
// after its upload, lets back-to-back calls proceed without waiting for the device.
struct Stager {
    static constexpr int SLOTS = 8;
    void* buf[SLOTS] = {};
    size_t cap[SLOTS] = {};
    hipEvent_t ev[SLOTS] = {};
    bool used[SLOTS] = {};
    int next = 0;
    hipError_t acquire(size_t bytes, int& slot, void*& p) {
        slot = next;
        next = (next + 1) % SLOTS;
        hipError_t e;
        if (!ev[slot] && (e = hipEventCreateWithFlags(&ev[slot], hipEventDisableTiming)) != hipSuccess) return e;
        if (used[slot] && (e = hipEventSynchronize(ev[slot])) != hipSuccess) return e;
        if (cap[slot] < bytes) {
            if (buf[slot]) (void)hipHostFree(buf[slot]);
            buf[slot] = nullptr;
            cap[slot] = 0;
            const size_t want = std::max<size_t>(bytes * 2, 4096);
            if ((e = hipHostMalloc(&buf[slot], want, hipHostMallocDefault)) != hipSuccess) return e;
            cap[slot] = want;
        }
        p = buf[slot];
        return hipSuccess;
    }
    hipError_t commit(int slot, hipStream_t st) {
        used[slot] = true;
        return hipEventRecord(ev[slot], st);
    }
    void release() {
        for (int i = 0; i < SLOTS; ++i) {
            if (buf[i]) (void)hipHostFree(buf[i]);
            if (ev[i]) (void)hipEventDestroy(ev[i]);
            buf[i] = nullptr; ev[i] = nullptr; cap[i] = 0; used[i] = false;
        }
    }
};

// Optional per-kernel-class timing with HIP events on the context's stream.
struct Profiler {
    int selected = SSD_PROF_OFF;               // SSD_PROF_OFF, SSD_PROF_ALL or one class
    std::vector<hipEvent_t> pool;
    struct Span { int cls; int e0, e1; };
    std::vector<Span> spans;
    int next_event = 0;
    bool wants(int cls) const { return selected == SSD_PROF_ALL || selected == cls; }
    int event(hipStream_t st) {
        if (next_event == (int)pool.size()) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return -1;
            pool.push_back(e);
        }
        if (hipEventRecord(pool[next_event], st) != hipSuccess) return -1;
        return next_event++;
    }
    void release() {
        for (hipEvent_t e : pool) (void)hipEventDestroy(e);
        pool.clear(); spans.clear(); next_event = 0;
    }
};

}  // namespace

struct ssd_ctx {
    hipStream_t stream = nullptr;
    bool has_model = false;
    bool bf16_ops = false;                   // matrix-core operand type of a 16-bit model: bfloat16 instead of IEEE half
    ssd_model_cfg cfg{};
    const void* embed = nullptr;
    const void* lm_head = nullptr;
    const void* norm_final = nullptr;
    std::vector<const void*> wo, w_down, norm_attn, norm_mlp;   // wo / w_down: what the GEMMs read
    std::vector<void*> wqkv, wgu;            // library-owned fused layouts
    // bf16 models: second copy of the four projection matrices in the layout of the few-row kernel (or NULL)
    std::vector<void*> s_qkv, s_o, s_gu, s_down;
    std::vector<void*> owned;                // every device allocation made by ssd_create
    // bf16 models: weights live as f16 * 2^k; these undo the scale in the GEMM epilogues
    std::vector<float> ds_qkv, ds_o, ds_gu, ds_down;
    float ds_lm = 1.f;
    float* rope_tab = nullptr;               // [max_positions][head_dim/2] (cos, sin) pairs
    int32_t* dev_flags = nullptr;            // sticky data-dependent conditions seen by kernels (ssd_device_flags)
    void* ws = nullptr;
    size_t ws_bytes = 0;
    uint16_t* head_w = nullptr;              // CTC output layer, padded with zero rows (bias -inf there)
    float* head_bias = nullptr;
    int head_V = 0, head_V_pad = 0, head_d = 0;
    // projector windows (ssd_set_qformer): fused [scores | values] weight and the output projection, both bf16
    uint16_t* qf_wcat = nullptr;
    uint16_t* qf_wo = nullptr;
    int qf_nq = 0, qf_heads = 0, qf_dh = 0, qf_denc = 0, qf_dout = 0, qf_window = 0;
    void* kv = nullptr;                      // caller-owned K/V cache: [layer][K|V][slots][d_kv] in the activation type
    int64_t kv_slots = 0;
    int64_t inexact_weights = 0;             // weight values the half conversion could not hold exactly
    std::string err;
    Stager stager;
    Profiler prof;
};

namespace {

int fail(ssd_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    return code;
}

#define HIP_TRY(c, expr)                                                                          \
    do {                                                                                          \
        hipError_t e_ = (expr);                                                                   \
        if (e_ != hipSuccess) return fail((c), SSD_EHIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }
size_t elem_size(int dtype) { return dtype == SSD_BF16 ? 2 : 4; }

bool check_cu(const int32_t* cu, int B, bool need_positive) {
    if (cu[0] != 0) return false;
    for (int b = 0; b < B; ++b) {
        if (cu[b + 1] < cu[b]) return false;
        if (need_positive && cu[b + 1] == cu[b]) return false;
    }
    return true;
}

// Stage `bytes` of host data and enqueue its upload to `dev`.
int upload(ssd_ctx* c, const void* host, void* dev, size_t bytes) {
    if (!bytes) return SSD_OK;
    int slot; void* p;
    HIP_TRY(c, c->stager.acquire(bytes, slot, p));
    memcpy(p, host, bytes);
    HIP_TRY(c, hipMemcpyAsync(dev, p, bytes, hipMemcpyHostToDevice, c->stream));
    HIP_TRY(c, c->stager.commit(slot, c->stream));
    return SSD_OK;
}

// Brackets the launches issued during its lifetime with two events when the class is being timed.
struct ProfScope {
    ssd_ctx* c; int cls; int e0 = -1;
    ProfScope(ssd_ctx* ctx, int k) : c(ctx), cls(k) { if (c->prof.wants(cls)) e0 = c->prof.event(c->stream); }
    ~ProfScope() {
        if (e0 >= 0) {
            const int e1 = c->prof.event(c->stream);
            if (e1 >= 0) c->prof.spans.push_back({cls, e0, e1});
        }
    }
};

struct GatePlan { size_t H, arg, cu, total; };
GatePlan plan_gate(int64_t frames, int64_t utts) {
    GatePlan p;
    size_t o = 0;
    p.H = o; o = align_up(o + (size_t)frames * 4);
    p.arg = o; o = align_up(o + (size_t)frames * 4);
    p.cu = o; o = align_up(o + (size_t)(utts + 1) * 4);
    p.total = o;
    return p;
}

struct HeadPlan { size_t H, arg, cu, part, total; };
HeadPlan plan_head(int64_t frames, int64_t utts, int V) {
    HeadPlan p;
    size_t o = 0;
    p.H = o; o = align_up(o + (size_t)frames * 4);
    p.arg = o; o = align_up(o + (size_t)frames * 4);
    p.cu = o; o = align_up(o + (size_t)(utts + 1) * 4);
    p.part = o; o = align_up(o + (size_t)frames * ctc_head_groups(V) * sizeof(float4));
    p.total = o;
    return p;
}

struct QformerPlan { size_t wins, scores, vals, o, total; int64_t max_windows; };
QformerPlan plan_qformer(int64_t frames, int64_t utts, int window, int n_q, int d_h) {
    QformerPlan p;
    p.max_windows = frames / window + utts;                  // every utterance may end in a short window
    size_t o = 0;
    p.wins = o; o = align_up(o + (size_t)p.max_windows * sizeof(QWindow));
    p.scores = o; o = align_up(o + (size_t)frames * QF_SCORE_COLS * 4);
    p.vals = o; o = align_up(o + (size_t)frames * d_h * 2);
    p.o = o; o = align_up(o + (size_t)p.max_windows * n_q * d_h * 2);
    p.total = o;
    return p;
}

int attn_tile_rows(int dtype) { return dtype == SSD_BF16 ? 64 : 4; }

struct VerifyPlan {
    size_t row_src, pos, vrow, row_slot, tiles, meta_bytes;     // metadata block, uploaded in one copy
    size_t x, a, qkv, attn, gu, h, x_c, attn_c, partials, rope_rows, total;   // activations
};
// rows that may go through the few-row GEMM path (split-K scratch): the whole batch, or the
// verification rows of the last layer
int64_t skinny_rows(int64_t M, int64_t Mv) { return M <= SKINNY_MAX_ROWS ? M : (Mv <= SKINNY_MAX_ROWS ? Mv : 0); }
VerifyPlan plan_verify(const ssd_model_cfg& c, int64_t M, int64_t Mv, int64_t utts) {
    VerifyPlan p;
    const size_t es = elem_size(c.dtype);
    const int64_t max_tiles = M / attn_tile_rows(c.dtype) + utts + 1;
    size_t o = 0;
    p.row_src = o; o = align_up(o + (size_t)M * 4);
    p.pos = o; o = align_up(o + (size_t)M * 4);
    p.vrow = o; o = align_up(o + (size_t)Mv * 4);
    p.row_slot = o; o = align_up(o + (size_t)M * 4);
    p.tiles = o; o = align_up(o + (size_t)max_tiles * sizeof(AttnTile));
    p.meta_bytes = o;
    const int64_t d = c.d_model, dq = (int64_t)c.n_q_heads * c.head_dim, dkv = (int64_t)c.n_kv_heads * c.head_dim;
    p.x = o; o = align_up(o + (size_t)(M * d) * 4);
    p.a = o; o = align_up(o + (size_t)(M * d) * es);
    p.qkv = o; o = align_up(o + (size_t)(M * (dq + 2 * dkv)) * es);
    p.attn = o; o = align_up(o + (size_t)(M * dq) * es);
    p.gu = o; if (c.dtype == SSD_F32) o = align_up(o + (size_t)(M * 2 * c.d_ff) * 4);
    p.h = o; o = align_up(o + (size_t)(M * c.d_ff) * es);
    // last layer: only the verification rows go on after attention
    p.x_c = o; if (c.dtype == SSD_BF16) o = align_up(o + (size_t)(Mv * d) * 4);
    p.attn_c = o; if (c.dtype == SSD_BF16) o = align_up(o + (size_t)(Mv * dq) * es);
    p.partials = o;
    if (c.dtype == SSD_BF16) o = align_up(o + (size_t)SKINNY_MAX_SPLITS * skinny_rows(M, Mv) * d * 4);
    // rotary table rows gathered per decoder row once per forward (the positions are the same in every layer)
    p.rope_rows = o;
    if (c.dtype == SSD_BF16 && M > SKINNY_MAX_ROWS) o = align_up(o + (size_t)M * 64 * sizeof(float2));
    p.total = o;
    return p;
}

struct AcceptPlan { size_t cu, part_ms, tgt, part_arg, total; };
AcceptPlan plan_accept(const ssd_model_cfg& c, int64_t Mv, int64_t utts) {
    AcceptPlan p;
    size_t o = 0;
    p.cu = o; o = align_up(o + (size_t)(utts + 1) * 4);
    p.part_ms = p.tgt = p.part_arg = o;
    if (c.dtype == SSD_BF16) {
        const int64_t g = lmhead_col_groups(c.vocab);
        p.part_ms = o; o = align_up(o + (size_t)(g * Mv) * sizeof(float2));
        p.tgt = o; o = align_up(o + (size_t)Mv * 4);
        p.part_arg = o; o = align_up(o + (size_t)(g * Mv) * sizeof(int2));
    }
    p.total = o;
    return p;
}

int check_model(ssd_ctx* c, const ssd_model_cfg& m) {
    if (m.n_layers <= 0 || m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.head_dim <= 0 ||
        m.d_ff <= 0 || m.vocab <= 0 || m.max_positions <= 0 || !(m.rms_eps >= 0.f) || !(m.rope_theta > 0.f))
        return fail(c, SSD_EINVAL, "ssd_create: non-positive model dimension");
    if (m.n_q_heads % m.n_kv_heads) return fail(c, SSD_ESHAPE, "ssd_create: n_q_heads must be a multiple of n_kv_heads");
    const int dq = m.n_q_heads * m.head_dim, dkv = m.n_kv_heads * m.head_dim;
    if (m.dtype == SSD_BF16) {
        if (m.head_dim != 128) return fail(c, SSD_ESHAPE, "ssd_create: bf16 needs head_dim 128 (got %d)", m.head_dim);
        if (m.d_model > 8192) return fail(c, SSD_ESHAPE, "ssd_create: bf16 needs d_model <= 8192");
        if (m.n_q_heads / m.n_kv_heads > 4) return fail(c, SSD_ESHAPE, "ssd_create: bf16 needs at most 4 query heads per KV head");
        if (m.d_model % 256 || m.d_ff % 128 || dq % 128 || dkv % 128 || (dq + 2 * dkv) % 256 || m.vocab % 256)
            return fail(c, SSD_ESHAPE, "ssd_create: bf16 needs d_model, n_q_heads*head_dim + 2*n_kv_heads*head_dim and vocab to be "
                                       "multiples of 256, d_ff a multiple of 128");
    } else if (m.dtype == SSD_F32) {
        if (m.head_dim % 4 || m.head_dim > 128) return fail(c, SSD_ESHAPE, "ssd_create: f32 needs head_dim %% 4 == 0 and <= 128");
        if (m.d_model % 16 || m.d_ff % 16 || dq % 16 || m.d_model > 1024)
            return fail(c, SSD_ESHAPE, "ssd_create: f32 needs d_model, d_ff, n_q_heads*head_dim multiples of 16 and d_model <= 1024");
    } else {
        return fail(c, SSD_EUNSUPPORTED, "ssd_create: dtype %d", m.dtype);
    }
    if (m.operand != SSD_OP_F16 && m.operand != SSD_OP_BF16) return fail(c, SSD_EUNSUPPORTED, "ssd_create: operand type %d", m.operand);
    if (m.operand == SSD_OP_BF16 && m.dtype != SSD_BF16) return fail(c, SSD_EUNSUPPORTED, "ssd_create: bfloat16 operands need dtype SSD_BF16");
    return SSD_OK;
}

}  // namespace

extern "C" {

const char* ssd_last_error(const ssd_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int ssd_create(ssd_ctx** out, const ssd_model_cfg* cfg, const ssd_weights* w, void* hip_stream) {
    if (!out) return SSD_EINVAL;
    *out = nullptr;
    if ((cfg == nullptr) != (w == nullptr)) return SSD_EINVAL;
    ssd_ctx* c = new ssd_ctx();
    c->stream = static_cast<hipStream_t>(hip_stream);
    if (!cfg) { *out = c; return SSD_OK; }
    int rc = check_model(c, *cfg);
    if (rc == SSD_OK) {
        const void* const* per_layer[] = {w->wq, w->wk, w->wv, w->wo, w->w_gate, w->w_up, w->w_down, w->norm_attn, w->norm_mlp};
        bool ok = w->embed && w->lm_head && w->norm_final;
        for (auto arr : per_layer) {
            ok = ok && arr;
            for (int l = 0; ok && l < cfg->n_layers; ++l) ok = arr[l] != nullptr;
        }
        if (!ok) rc = fail(c, SSD_EINVAL, "ssd_create: NULL weight pointer");
    }
    if (rc != SSD_OK) { fprintf(stderr, "ssd_create: %s\n", c->err.c_str()); delete c; return rc; }
    c->cfg = *cfg;
    c->has_model = true;
    c->embed = w->embed; c->lm_head = w->lm_head; c->norm_final = w->norm_final;
    const int L = cfg->n_layers, d = cfg->d_model, dq = cfg->n_q_heads * cfg->head_dim, dkv = cfg->n_kv_heads * cfg->head_dim;
    const int dff = cfg->d_ff;
    const bool half = cfg->dtype == SSD_BF16;                // a 16-bit model (either operand type)
    const bool bf = half && cfg->operand == SSD_OP_BF16;     // bfloat16 operands: the stored weights are the operands
    c->bf16_ops = bf;
    const size_t es = elem_size(cfg->dtype);
    auto bail = [&](hipError_t e, const char* what) {
        fprintf(stderr, "ssd_create: %s: %s\n", what, hipGetErrorString(e));
        ssd_destroy(c);
        return (int)SSD_EHIP;
    };
    hipError_t e;
    auto dev_alloc = [&](void** p, size_t bytes) {
        hipError_t r = hipMalloc(p, bytes);
        if (r == hipSuccess) c->owned.push_back(*p);
        return r;
    };
    // largest magnitude of each weight group -> exact power-of-two scale into the f16 range
    const int n_groups = 4 * L + 1;
    std::vector<float> scale(n_groups, 1.0f);
    if (half && !bf) {
        unsigned int* d_max = nullptr;
        if ((e = dev_alloc((void**)&d_max, (size_t)n_groups * 4)) != hipSuccess) return bail(e, "hipMalloc(absmax)");
        if ((e = hipMemsetAsync(d_max, 0, (size_t)n_groups * 4, c->stream)) != hipSuccess) return bail(e, "hipMemsetAsync");
        for (int l = 0; l < L; ++l) {
            launch_absmax(cfg->dtype, w->wq[l], (int64_t)dq * d, d_max + 4 * l + 0, c->stream);
            launch_absmax(cfg->dtype, w->wk[l], (int64_t)dkv * d, d_max + 4 * l + 0, c->stream);
            launch_absmax(cfg->dtype, w->wv[l], (int64_t)dkv * d, d_max + 4 * l + 0, c->stream);
            launch_absmax(cfg->dtype, w->wo[l], (int64_t)d * dq, d_max + 4 * l + 1, c->stream);
            launch_absmax(cfg->dtype, w->w_gate[l], (int64_t)dff * d, d_max + 4 * l + 2, c->stream);
            launch_absmax(cfg->dtype, w->w_up[l], (int64_t)dff * d, d_max + 4 * l + 2, c->stream);
            launch_absmax(cfg->dtype, w->w_down[l], (int64_t)d * dff, d_max + 4 * l + 3, c->stream);
        }
        launch_absmax(cfg->dtype, w->lm_head, (int64_t)cfg->vocab * d, d_max + 4 * L, c->stream);
        std::vector<float> mx(n_groups);
        if ((e = hipMemcpyAsync(mx.data(), d_max, (size_t)n_groups * 4, hipMemcpyDeviceToHost, c->stream)) != hipSuccess)
            return bail(e, "hipMemcpyAsync(absmax)");
        if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(e, "absmax");
        for (int g = 0; g < n_groups; ++g) {
            if (!(mx[g] > 0.f) || !std::isfinite(mx[g])) continue;
            int ex;
            frexpf(mx[g], &ex);                               // mx < 2^ex
            scale[g] = ldexpf(1.0f, std::max(-60, std::min(60, 14 - ex)));   // largest value lands below 2^14
        }
    }
    // values that the conversion to half cannot hold exactly are counted (ssd_inexact_weights)
    unsigned long long* d_inexact = nullptr;
    if ((e = dev_alloc((void**)&d_inexact, 256)) != hipSuccess) return bail(e, "hipMalloc(inexact)");
    if ((e = hipMemsetAsync(d_inexact, 0, 256, c->stream)) != hipSuccess) return bail(e, "hipMemsetAsync(inexact)");
    for (int l = 0; l < L; ++l) {
        c->norm_attn.push_back(w->norm_attn[l]); c->norm_mlp.push_back(w->norm_mlp[l]);
        void *pq = nullptr, *pg = nullptr;
        if ((e = dev_alloc(&pq, (size_t)(dq + 2 * dkv) * d * es)) != hipSuccess) return bail(e, "hipMalloc(wqkv)");
        c->wqkv.push_back(pq);
        if ((e = dev_alloc(&pg, (size_t)2 * dff * d * es)) != hipSuccess) return bail(e, "hipMalloc(wgu)");
        c->wgu.push_back(pg);
        launch_pack_qkv(cfg->dtype, w->wq[l], w->wk[l], w->wv[l], pq, dq, dkv, d, cfg->head_dim, bf ? 0.f : scale[4 * l + 0], d_inexact, c->stream);
        launch_pack_gate_up(cfg->dtype, w->w_gate[l], w->w_up[l], pg, dff, d, bf ? 0.f : scale[4 * l + 2], d_inexact, c->stream);
        if (half) {
            void *po = nullptr, *pd = nullptr;
            if ((e = dev_alloc(&po, (size_t)d * dq * 2)) != hipSuccess) return bail(e, "hipMalloc(wo)");
            if ((e = dev_alloc(&pd, (size_t)d * dff * 2)) != hipSuccess) return bail(e, "hipMalloc(w_down)");
            launch_convert_weight(cfg->dtype, w->wo[l], po, d, dq, bf ? 0.f : scale[4 * l + 1], d_inexact, c->stream);
            launch_convert_weight(cfg->dtype, w->w_down[l], pd, d, dff, bf ? 0.f : scale[4 * l + 3], d_inexact, c->stream);
            c->wo.push_back(po); c->w_down.push_back(pd);
            struct { const void* src; int N, K; std::vector<void*>* dst; } copies[4] = {
                {pq, dq + 2 * dkv, d, &c->s_qkv}, {po, d, dq, &c->s_o}, {pg, 2 * dff, d, &c->s_gu}, {pd, d, dff, &c->s_down}};
            for (auto& cp : copies) {
                void* ps = nullptr;
                if (stream_layout_supported(cp.N, cp.K)) {
                    if ((e = dev_alloc(&ps, (size_t)cp.N * cp.K * 2)) != hipSuccess) return bail(e, "hipMalloc(stream layout)");
                    launch_stream_layout((const uint16_t*)cp.src, ps, cp.N, cp.K, c->stream);
                }
                cp.dst->push_back(ps);
            }
        } else {
            c->wo.push_back(w->wo[l]); c->w_down.push_back(w->w_down[l]);
        }
        c->ds_qkv.push_back(1.0f / scale[4 * l + 0]); c->ds_o.push_back(1.0f / scale[4 * l + 1]);
        c->ds_gu.push_back(1.0f / scale[4 * l + 2]); c->ds_down.push_back(1.0f / scale[4 * l + 3]);
    }
    if (half) {
        void* pl = nullptr;
        if ((e = dev_alloc(&pl, (size_t)cfg->vocab * d * 2)) != hipSuccess) return bail(e, "hipMalloc(lm_head)");
        launch_convert_weight(cfg->dtype, w->lm_head, pl, cfg->vocab, d, bf ? 0.f : scale[4 * L], d_inexact, c->stream);
        c->lm_head = pl;
        c->ds_lm = 1.0f / scale[4 * L];
    }
    // rotary table, computed in double and rounded once
    const int hd2 = cfg->head_dim / 2;
    std::vector<float> tab((size_t)cfg->max_positions * hd2 * 2);
    for (int p = 0; p < cfg->max_positions; ++p)
        for (int i = 0; i < hd2; ++i) {
            const double ang = (double)p * pow((double)cfg->rope_theta, -2.0 * i / cfg->head_dim);
            tab[((size_t)p * hd2 + i) * 2] = (float)cos(ang);
            tab[((size_t)p * hd2 + i) * 2 + 1] = (float)sin(ang);
        }
    if ((e = dev_alloc((void**)&c->rope_tab, tab.size() * 4)) != hipSuccess) return bail(e, "hipMalloc(rope)");
    if ((e = hipMemcpyAsync(c->rope_tab, tab.data(), tab.size() * 4, hipMemcpyHostToDevice, c->stream)) != hipSuccess)
        return bail(e, "hipMemcpyAsync(rope)");
    if ((e = dev_alloc((void**)&c->dev_flags, 256)) != hipSuccess) return bail(e, "hipMalloc(flags)");
    if ((e = hipMemsetAsync(c->dev_flags, 0, 256, c->stream)) != hipSuccess) return bail(e, "hipMemsetAsync(flags)");
    unsigned long long n_inexact = 0;
    if ((e = hipMemcpyAsync(&n_inexact, d_inexact, 8, hipMemcpyDeviceToHost, c->stream)) != hipSuccess) return bail(e, "hipMemcpyAsync(inexact)");
    if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(e, "weight packing");
    if ((e = hipGetLastError()) != hipSuccess) return bail(e, "weight packing launch");
    c->inexact_weights = (int64_t)n_inexact;
    *out = c;
    return SSD_OK;
}

int64_t ssd_inexact_weights(const ssd_ctx* ctx) { return ctx ? ctx->inexact_weights : -1; }

void ssd_destroy(ssd_ctx* c) {
    if (!c) return;
    (void)hipStreamSynchronize(c->stream);
    for (void* p : c->owned) if (p) (void)hipFree(p);
    c->stager.release();
    c->prof.release();
    delete c;
}

size_t ssd_workspace_bytes(const ssd_ctx* ctx, int64_t max_frames, int64_t max_tokens, int64_t max_verify_rows,
                           int64_t max_utts) {
    if (!ctx || max_frames < 0 || max_tokens < 0 || max_verify_rows < 0 || max_utts < 0) return 0;
    size_t need = plan_gate(max_frames, max_utts).total;
    if (ctx->head_V) need = std::max(need, plan_head(max_frames, max_utts, ctx->head_V).total);
    if (ctx->qf_nq) need = std::max(need, plan_qformer(max_frames, max_utts, ctx->qf_window, ctx->qf_nq, ctx->qf_dh).total);
    if (ctx->has_model) {
        need = std::max(need, plan_verify(ctx->cfg, max_tokens, max_verify_rows, max_utts).total);
        // a smaller batch may take the few-row path, which needs split-K scratch the big plan does not have
        const int64_t few = std::min<int64_t>(max_tokens, SKINNY_MAX_ROWS);
        need = std::max(need, plan_verify(ctx->cfg, few, std::min(max_verify_rows, few), std::min(max_utts, few)).total);
        need = std::max(need, plan_verify(ctx->cfg, max_tokens, std::min<int64_t>(max_verify_rows, SKINNY_MAX_ROWS), max_utts).total);
        need = std::max(need, plan_accept(ctx->cfg, max_verify_rows, max_utts).total);
    }
    return need + 256;
}

int ssd_device_flags(ssd_ctx* ctx, int32_t* flags) {
    if (!ctx || !flags) return SSD_EINVAL;
    *flags = 0;
    if (!ctx->dev_flags) return SSD_OK;
    HIP_TRY(ctx, hipMemcpyAsync(flags, ctx->dev_flags, 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    if (*flags) HIP_TRY(ctx, hipMemsetAsync(ctx->dev_flags, 0, 4, ctx->stream));
    return SSD_OK;
}

int ssd_set_workspace(ssd_ctx* ctx, void* dev_ptr, size_t bytes) {
    if (!ctx) return SSD_EINVAL;
    if (!dev_ptr && bytes) return fail(ctx, SSD_EINVAL, "workspace pointer is NULL");
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 255) return fail(ctx, SSD_EINVAL, "workspace must be 256-byte aligned");
    ctx->ws = dev_ptr;
    ctx->ws_bytes = bytes;
    return SSD_OK;
}

int ssd_profile_select(ssd_ctx* ctx, int kernel_class) {
    if (!ctx) return SSD_EINVAL;
    if (kernel_class < SSD_PROF_OFF || kernel_class >= SSD_PROF_N_CLASSES) return fail(ctx, SSD_EINVAL, "ssd_profile_select: unknown class %d", kernel_class);
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->prof.selected = kernel_class;
    ctx->prof.spans.clear();
    ctx->prof.next_event = 0;
    return SSD_OK;
}

int ssd_profile_read(ssd_ctx* ctx, float* total_ms, int32_t* launches) {
    if (!ctx || !total_ms || !launches) return SSD_EINVAL;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (int k = 0; k < SSD_PROF_N_CLASSES; ++k) { total_ms[k] = 0.f; launches[k] = 0; }
    for (const Profiler::Span& sp : ctx->prof.spans) {
        float ms = 0.f;
        HIP_TRY(ctx, hipEventElapsedTime(&ms, ctx->prof.pool[sp.e0], ctx->prof.pool[sp.e1]));
        total_ms[sp.cls] += ms;
        launches[sp.cls] += 1;
    }
    ctx->prof.spans.clear();
    ctx->prof.next_event = 0;
    return SSD_OK;
}

int ssd_gate_grid(ssd_ctx* ctx, const float* max_entropy, int B, const float* tau_ctc, int n_tau, uint8_t* gate_pass) {
    if (!ctx) return SSD_EINVAL;
    if (!max_entropy || !tau_ctc || !gate_pass || B <= 0 || n_tau <= 0) return fail(ctx, SSD_EINVAL, "ssd_gate_grid: bad argument");
    const size_t need = align_up((size_t)n_tau * 4);
    if (!ctx->ws || ctx->ws_bytes < need) return fail(ctx, SSD_EWORKSPACE, "ssd_gate_grid: workspace of %zu bytes needed", need);
    int rc = upload(ctx, tau_ctc, ctx->ws, (size_t)n_tau * 4);
    if (rc != SSD_OK) return rc;
    launch_gate_grid(max_entropy, B, static_cast<const float*>(ctx->ws), n_tau, gate_pass, ctx->stream);
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_accept_grid(ssd_ctx* ctx, const float* draft_logp, const int32_t* cu_draft, int Bv, const float* tau_slm, int n_tau,
                    int32_t* accept_len, uint8_t* all_accepted) {
    if (!ctx) return SSD_EINVAL;
    if (!cu_draft || !tau_slm || !accept_len || !all_accepted || Bv <= 0 || n_tau <= 0)
        return fail(ctx, SSD_EINVAL, "ssd_accept_grid: bad argument");
    if (!check_cu(cu_draft, Bv, false)) return fail(ctx, SSD_EINVAL, "ssd_accept_grid: cu_draft must start at 0 and be non-decreasing");
    if (cu_draft[Bv] && !draft_logp) return fail(ctx, SSD_EINVAL, "ssd_accept_grid: NULL draft_logp");
    const size_t off_tau = align_up((size_t)(Bv + 1) * 4);
    const size_t need = off_tau + align_up((size_t)n_tau * 4);
    if (!ctx->ws || ctx->ws_bytes < need) return fail(ctx, SSD_EWORKSPACE, "ssd_accept_grid: workspace of %zu bytes needed", need);
    std::vector<char> meta(need);
    memcpy(meta.data(), cu_draft, (size_t)(Bv + 1) * 4);
    float* ln_taus = reinterpret_cast<float*>(meta.data() + off_tau);
    for (int a = 0; a < n_tau; ++a) {
        if (tau_slm[a] != tau_slm[a]) return fail(ctx, SSD_EINVAL, "ssd_accept_grid: tau_slm[%d] is NaN", a);
        ln_taus[a] = tau_slm[a] > 0.f ? (float)log((double)tau_slm[a]) : -INFINITY;
    }
    char* ws = static_cast<char*>(ctx->ws);
    int rc = upload(ctx, meta.data(), ws, need);
    if (rc != SSD_OK) return rc;
    launch_accept_grid(draft_logp, reinterpret_cast<const int32_t*>(ws), Bv, reinterpret_cast<const float*>(ws + off_tau), n_tau,
                       accept_len, all_accepted, ctx->stream);
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_plan_batches(const int32_t* lengths, int n, int64_t max_tokens, int padded, int32_t* order, int32_t* batch_start,
                     int32_t* n_batches) {
    if (!lengths || !order || !batch_start || !n_batches || n <= 0 || max_tokens <= 0) return SSD_EINVAL;
    for (int i = 0; i < n; ++i) {
        if (lengths[i] <= 0) return SSD_EINVAL;
        order[i] = i;
    }
    std::stable_sort(order, order + n, [&](int32_t a, int32_t b) { return lengths[a] > lengths[b]; });   // longest first
    int nb = 0;
    int64_t count = 0, sum = 0, longest = 0;
    batch_start[0] = 0;
    for (int k = 0; k < n; ++k) {
        const int64_t len = lengths[order[k]];
        const int64_t c2 = count + 1, s2 = sum + len, l2 = std::max(longest, len);
        const int64_t cost = padded ? c2 * l2 : s2;
        if (count > 0 && cost > max_tokens) {
            batch_start[++nb] = k;
            count = 1; sum = len; longest = len;
        } else {
            count = c2; sum = s2; longest = l2;
        }
    }
    batch_start[++nb] = n;
    *n_batches = nb;
    return SSD_OK;
}

int ssd_select_unconfident(ssd_ctx* ctx, int B, int n_sel, const int32_t* sel, const int32_t* cu_frames,
                           const int32_t* draft_len, const int32_t* draft_ctc, const int32_t* ctc_to_llm, int V_ctc,
                           const void* speech_all, const int32_t* cu_speech_all, const int32_t* prompt_all,
                           const int32_t* cu_prompt_all, int d_model, int dtype, void* speech_out, int32_t* prompt_out,
                           int32_t* draft_ids_out, int32_t* cu_speech_out, int32_t* cu_prompt_out, int32_t* cu_draft_out) {
    if (!ctx) return SSD_EINVAL;
    if (!sel || !cu_frames || !draft_len || !cu_speech_all || !cu_prompt_all || !cu_speech_out || !cu_prompt_out || !cu_draft_out)
        return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: NULL host array");
    if (B <= 0 || n_sel <= 0 || n_sel > B) return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: need 0 < n_sel <= B");
    if (d_model <= 0 || (dtype != SSD_F32 && dtype != SSD_BF16)) return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: bad d_model or dtype");
    if (ctc_to_llm && V_ctc <= 0) return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: V_ctc must be positive with a table");
    if (!check_cu(cu_frames, B, true) || !check_cu(cu_speech_all, B, false) || !check_cu(cu_prompt_all, B, false))
        return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: malformed cu_* array");
    const size_t row_bytes = (size_t)d_model * elem_size(dtype);
    if (row_bytes % 16) return fail(ctx, SSD_ESHAPE, "ssd_select_unconfident: a speech row must be a multiple of 16 bytes");
    int64_t nS = 0, nP = 0, nU = 0;
    cu_speech_out[0] = cu_prompt_out[0] = cu_draft_out[0] = 0;
    for (int k = 0; k < n_sel; ++k) {
        const int b = sel[k];
        if (b < 0 || b >= B) return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: sel[%d] = %d outside [0, %d)", k, b, B);
        if (draft_len[b] < 0 || draft_len[b] > cu_frames[b + 1] - cu_frames[b])
            return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: draft_len[%d] = %d does not fit the utterance's %d frames", b,
                        draft_len[b], cu_frames[b + 1] - cu_frames[b]);
        nS += cu_speech_all[b + 1] - cu_speech_all[b];
        nP += cu_prompt_all[b + 1] - cu_prompt_all[b];
        nU += draft_len[b];
        if (nS + nP + nU > 0x3fffffff) return fail(ctx, SSD_ESHAPE, "ssd_select_unconfident: too many rows");
        cu_speech_out[k + 1] = (int32_t)nS; cu_prompt_out[k + 1] = (int32_t)nP; cu_draft_out[k + 1] = (int32_t)nU;
    }
    if ((nS && (!speech_all || !speech_out)) || (nP && (!prompt_all || !prompt_out)) || (nU && (!draft_ctc || !draft_ids_out)))
        return fail(ctx, SSD_EINVAL, "ssd_select_unconfident: NULL data pointer");
    const size_t oS = 0, oP = align_up((size_t)nS * 4), oU = oP + align_up((size_t)nP * 4), need = oU + align_up((size_t)nU * 4);
    if (!ctx->ws || ctx->ws_bytes < need) return fail(ctx, SSD_EWORKSPACE, "ssd_select_unconfident: workspace of %zu bytes needed, %zu set", need, ctx->ws_bytes);
    // source index of every packed output row / id
    std::vector<char> meta(need);
    int32_t* iS = reinterpret_cast<int32_t*>(meta.data() + oS);
    int32_t* iP = reinterpret_cast<int32_t*>(meta.data() + oP);
    int32_t* iU = reinterpret_cast<int32_t*>(meta.data() + oU);
    for (int k = 0; k < n_sel; ++k) {
        const int b = sel[k];
        for (int i = cu_speech_all[b]; i < cu_speech_all[b + 1]; ++i) *iS++ = i;
        for (int i = cu_prompt_all[b]; i < cu_prompt_all[b + 1]; ++i) *iP++ = i;
        for (int i = 0; i < draft_len[b]; ++i) *iU++ = cu_frames[b] + i;       // ctc_gate writes utterance b's draft at cu_frames[b]
    }
    char* ws = static_cast<char*>(ctx->ws);
    int rc = upload(ctx, meta.data(), ws, need);
    if (rc != SSD_OK) return rc;
    {
        ProfScope ps(ctx, SSD_PROF_OTHER);
        launch_gather_rows(speech_all, reinterpret_cast<const int32_t*>(ws + oS), (int)nS, (int64_t)row_bytes, speech_out, ctx->stream);
        launch_gather_ids(prompt_all, reinterpret_cast<const int32_t*>(ws + oP), (int)nP, nullptr, 0, prompt_out, ctx->stream);
        launch_gather_ids(draft_ctc, reinterpret_cast<const int32_t*>(ws + oU), (int)nU, ctc_to_llm, V_ctc, draft_ids_out, ctx->stream);
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_gather_i32(ssd_ctx* ctx, const int32_t* src, const int32_t* idx, int n, int32_t* out) {
    if (!ctx) return SSD_EINVAL;
    if (n < 0 || (n && (!src || !idx || !out))) return fail(ctx, SSD_EINVAL, "ssd_gather_i32: bad argument");
    for (int i = 0; i < n; ++i)
        if (idx[i] < 0) return fail(ctx, SSD_EINVAL, "ssd_gather_i32: idx[%d] is negative", i);
    const size_t need = align_up((size_t)n * 4);
    if (n && (!ctx->ws || ctx->ws_bytes < need)) return fail(ctx, SSD_EWORKSPACE, "ssd_gather_i32: workspace of %zu bytes needed", need);
    int rc = upload(ctx, idx, ctx->ws, (size_t)n * 4);
    if (rc != SSD_OK) return rc;
    launch_gather_ids(src, static_cast<const int32_t*>(ctx->ws), n, nullptr, 0, out, ctx->stream);
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_measure_hbm_read(ssd_ctx* ctx, const void* dev_buf, size_t bytes, int iters, float* gbytes_per_s) {
    if (!ctx || !dev_buf || !gbytes_per_s || iters <= 0 || bytes < 16) return SSD_EINVAL;
    if (reinterpret_cast<uintptr_t>(dev_buf) & 15) return fail(ctx, SSD_EINVAL, "ssd_measure_hbm_read: buffer must be 16-byte aligned");
    if (!ctx->ws || ctx->ws_bytes < 256) return fail(ctx, SSD_EWORKSPACE, "ssd_measure_hbm_read: a workspace must be set");
    bytes &= ~(size_t)15;
    uint32_t* sink = static_cast<uint32_t*>(ctx->ws);
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    launch_hbm_read(dev_buf, bytes, sink, ctx->stream);                                   // warm-up
    HIP_TRY(ctx, hipEventRecord(e0, ctx->stream));
    for (int i = 0; i < iters; ++i) launch_hbm_read(dev_buf, bytes, sink, ctx->stream);
    HIP_TRY(ctx, hipEventRecord(e1, ctx->stream));
    HIP_TRY(ctx, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    *gbytes_per_s = (float)((double)bytes * iters / (ms * 1e-3) / 1e9);
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_measure_mfma_ceiling(ssd_ctx* ctx, int iters, float* tflops, float* shader_ghz) {
    if (!ctx || !tflops || !shader_ghz || iters <= 0) return SSD_EINVAL;
    const int n_wg = 256;                                  // one workgroup of eight wavefronts per CU
    const size_t need = (size_t)n_wg * 512 * 4 + 256;
    if (!ctx->ws || ctx->ws_bytes < need) return fail(ctx, SSD_EWORKSPACE, "ssd_measure_mfma_ceiling: workspace of %zu bytes needed", need);
    float* sink = static_cast<float*>(ctx->ws);
    long long* clocks = reinterpret_cast<long long*>(static_cast<char*>(ctx->ws) + (size_t)n_wg * 512 * 4);
    hipEvent_t e0, e1;
    HIP_TRY(ctx, hipEventCreate(&e0));
    HIP_TRY(ctx, hipEventCreate(&e1));
    launch_mfma_ceiling(sink, clocks, n_wg, std::max(1, iters / 20), ctx->stream);       // warm-up
    HIP_TRY(ctx, hipEventRecord(e0, ctx->stream));
    launch_mfma_ceiling(sink, clocks, n_wg, iters, ctx->stream);
    HIP_TRY(ctx, hipEventRecord(e1, ctx->stream));
    HIP_TRY(ctx, hipEventSynchronize(e1));
    float ms = 0.f;
    HIP_TRY(ctx, hipEventElapsedTime(&ms, e0, e1));
    long long hc[2] = {0, 1};
    HIP_TRY(ctx, hipMemcpy(hc, clocks, sizeof hc, hipMemcpyDeviceToHost));
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    const double flops = (double)n_wg * 8 * (double)iters * 16 * 16384.0;    // 16x16x32 MFMA = 16384 flop
    *tflops = (float)(flops / (ms * 1e-3) / 1e12);
    *shader_ghz = (float)((double)hc[0] / ((double)hc[1] * 10.0));            // constant clock ticks at 100 MHz
    return SSD_OK;
}

int ctc_gate(ssd_ctx* ctx, const void* logits, int dtype, const int32_t* cu_frames, int B, int V_ctc, int blank_id,
             float tau_ctc, float* frame_entropy, int32_t* frame_argmax, float* max_entropy, uint8_t* gate_pass,
             int32_t* draft_ctc, int32_t* draft_len) {
    if (!ctx) return SSD_EINVAL;
    if (!logits || !cu_frames || !max_entropy || !gate_pass || !draft_ctc || !draft_len)
        return fail(ctx, SSD_EINVAL, "ctc_gate: NULL argument");
    if (B <= 0) return fail(ctx, SSD_EINVAL, "ctc_gate: B must be positive (got %d)", B);
    if (V_ctc <= 0) return fail(ctx, SSD_EINVAL, "ctc_gate: V_ctc must be positive (got %d)", V_ctc);
    if (blank_id < 0 || blank_id >= V_ctc) return fail(ctx, SSD_EINVAL, "ctc_gate: blank_id %d outside [0, %d)", blank_id, V_ctc);
    if (dtype != SSD_F32 && dtype != SSD_BF16) return fail(ctx, SSD_EUNSUPPORTED, "ctc_gate: dtype %d", dtype);
    if (!check_cu(cu_frames, B, true))
        return fail(ctx, SSD_EINVAL, "ctc_gate: cu_frames must start at 0 and increase strictly (every utterance needs a frame)");
    const int64_t n_rows = cu_frames[B];
    const GatePlan p = plan_gate(n_rows, B);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "ctc_gate: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);
    char* ws = static_cast<char*>(ctx->ws);
    float* H = frame_entropy ? frame_entropy : reinterpret_cast<float*>(ws + p.H);
    int32_t* arg = frame_argmax ? frame_argmax : reinterpret_cast<int32_t*>(ws + p.arg);
    int32_t* cu_dev = reinterpret_cast<int32_t*>(ws + p.cu);
    int rc = upload(ctx, cu_frames, cu_dev, (size_t)(B + 1) * 4);
    if (rc != SSD_OK) return rc;
    {
        ProfScope ps(ctx, SSD_PROF_GATE);
        launch_gate(logits, dtype, n_rows, V_ctc, cu_dev, B, blank_id, tau_ctc, H, arg, max_entropy, gate_pass, draft_ctc,
                    draft_len, ctx->stream);
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ssd_set_ctc_head(ssd_ctx* ctx, const void* w_ctc, const float* bias, int V_ctc, int d_enc) {
    if (!ctx) return SSD_EINVAL;
    if (!w_ctc) return fail(ctx, SSD_EINVAL, "ssd_set_ctc_head: NULL weight");
    if (V_ctc <= 0 || d_enc <= 0) return fail(ctx, SSD_EINVAL, "ssd_set_ctc_head: non-positive size");
    if (d_enc % 64) return fail(ctx, SSD_ESHAPE, "ssd_set_ctc_head: d_enc must be a multiple of 64 (got %d)", d_enc);
    if (V_ctc > 65536) return fail(ctx, SSD_ESHAPE, "ssd_set_ctc_head: at most 65536 symbols");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    auto drop = [&](void* p) {
        if (!p) return;
        for (auto& q : ctx->owned) if (q == p) q = nullptr;
        (void)hipFree(p);
    };
    drop(ctx->head_w); drop(ctx->head_bias);
    ctx->head_w = nullptr; ctx->head_bias = nullptr; ctx->head_V = 0;
    const int V_pad = ctc_head_padded(V_ctc);
    void *w = nullptr, *b = nullptr;
    HIP_TRY(ctx, hipMalloc(&w, (size_t)V_pad * d_enc * 2));
    ctx->owned.push_back(w);
    HIP_TRY(ctx, hipMalloc(&b, (size_t)V_pad * 4));
    ctx->owned.push_back(b);
    launch_ctc_head_pack(static_cast<const uint16_t*>(w_ctc), bias, V_ctc, V_pad, d_enc, static_cast<uint16_t*>(w),
                         static_cast<float*>(b), ctx->stream);
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));     // the caller may release its copies on return
    ctx->head_w = static_cast<uint16_t*>(w);
    ctx->head_bias = static_cast<float*>(b);
    ctx->head_V = V_ctc; ctx->head_V_pad = V_pad; ctx->head_d = d_enc;
    return SSD_OK;
}

int ssd_set_qformer(ssd_ctx* ctx, const void* q_proj, const void* w_k, const void* w_v, const void* w_o, int n_q, int n_heads,
                    int d_h, int d_enc, int d_out, int window) {
    if (!ctx) return SSD_EINVAL;
    if (!q_proj || !w_k || !w_v || !w_o) return fail(ctx, SSD_EINVAL, "ssd_set_qformer: NULL weight");
    if (n_q <= 0 || n_heads <= 0 || d_h <= 0 || d_enc <= 0 || d_out <= 0 || window <= 0)
        return fail(ctx, SSD_EINVAL, "ssd_set_qformer: non-positive size");
    if (n_q > QF_MAX_QUERIES || n_q * n_heads > QF_SCORE_COLS || window > QF_MAX_WINDOW)
        return fail(ctx, SSD_ESHAPE, "ssd_set_qformer: at most %d queries, %d (query, head) pairs and windows of %d frames",
                    QF_MAX_QUERIES, QF_SCORE_COLS, QF_MAX_WINDOW);
    if (d_h % n_heads || (d_h / n_heads) % 4 || d_h % 64 || d_enc % 64 || d_out % 256)
        return fail(ctx, SSD_ESHAPE, "ssd_set_qformer: d_h must be a multiple of 4 * n_heads and of 64, d_enc of 64, d_out of 256");
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    auto drop = [&](void* p) {
        if (!p) return;
        for (auto& q : ctx->owned) if (q == p) q = nullptr;
        (void)hipFree(p);
    };
    drop(ctx->qf_wcat); drop(ctx->qf_wo);
    ctx->qf_wcat = ctx->qf_wo = nullptr; ctx->qf_nq = 0;
    void *wc = nullptr, *wo = nullptr;
    HIP_TRY(ctx, hipMalloc(&wc, (size_t)qformer_cat_rows(d_h) * d_enc * 2));
    ctx->owned.push_back(wc);
    HIP_TRY(ctx, hipMalloc(&wo, (size_t)d_out * d_h * 2));
    ctx->owned.push_back(wo);
    launch_qformer_fold(static_cast<const uint16_t*>(q_proj), static_cast<const uint16_t*>(w_k), static_cast<const uint16_t*>(w_v),
                        n_q, n_heads, d_h, d_enc, static_cast<uint16_t*>(wc), ctx->stream);
    HIP_TRY(ctx, hipMemcpyAsync(wo, w_o, (size_t)d_out * d_h * 2, hipMemcpyDeviceToDevice, ctx->stream));
    HIP_TRY(ctx, hipGetLastError());
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));     // the caller may release its copies on return
    ctx->qf_wcat = static_cast<uint16_t*>(wc); ctx->qf_wo = static_cast<uint16_t*>(wo);
    ctx->qf_nq = n_q; ctx->qf_heads = n_heads; ctx->qf_dh = d_h; ctx->qf_denc = d_enc; ctx->qf_dout = d_out; ctx->qf_window = window;
    return SSD_OK;
}

int qformer_pool(ssd_ctx* ctx, const void* enc_h, const int32_t* cu_frames, int B, void* speech_emb, int32_t* cu_speech) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->qf_nq) return fail(ctx, SSD_EINVAL, "qformer_pool: no projector set (ssd_set_qformer)");
    if (!enc_h || !cu_frames || !speech_emb || !cu_speech) return fail(ctx, SSD_EINVAL, "qformer_pool: NULL argument");
    if (B <= 0) return fail(ctx, SSD_EINVAL, "qformer_pool: B must be positive (got %d)", B);
    if (!check_cu(cu_frames, B, true))
        return fail(ctx, SSD_EINVAL, "qformer_pool: cu_frames must start at 0 and increase strictly (every utterance needs a frame)");
    const int64_t n_rows = cu_frames[B];
    const int window = ctx->qf_window, n_q = ctx->qf_nq, d_h = ctx->qf_dh, d_enc = ctx->qf_denc;
    if (n_rows * (int64_t)std::max(d_enc, d_h) * 2 >= ((int64_t)1 << 32))
        return fail(ctx, SSD_ESHAPE, "qformer_pool: %lld frames exceed the 4 GiB an operand matrix may have; split the batch", (long long)n_rows);
    const QformerPlan p = plan_qformer(n_rows, B, window, n_q, d_h);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "qformer_pool: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);
    std::vector<QWindow> wins;
    wins.reserve((size_t)p.max_windows);
    cu_speech[0] = 0;
    for (int b = 0; b < B; ++b) {
        for (int f = cu_frames[b]; f < cu_frames[b + 1]; f += window)
            wins.push_back(QWindow{f, std::min(window, cu_frames[b + 1] - f)});
        cu_speech[b + 1] = (int32_t)(wins.size() * n_q);
    }
    const int n_windows = (int)wins.size();
    char* ws = static_cast<char*>(ctx->ws);
    int rc = upload(ctx, wins.data(), ws + p.wins, wins.size() * sizeof(QWindow));
    if (rc != SSD_OK) return rc;
    float* scores = reinterpret_cast<float*>(ws + p.scores);
    uint16_t* vals = reinterpret_cast<uint16_t*>(ws + p.vals);
    uint16_t* o = reinterpret_cast<uint16_t*>(ws + p.o);
    const int n_cat = qformer_cat_rows(d_h);
    {
        ProfScope ps(ctx, SSD_PROF_QFORMER);
        launch_gemm_scores_values(static_cast<const uint16_t*>(enc_h), ctx->qf_wcat, scores, vals, (int)n_rows, n_cat, d_enc, d_h,
                                  ctx->dev_flags, true, ctx->stream);
        launch_qformer_pool(scores, vals, reinterpret_cast<const QWindow*>(ws + p.wins), n_windows, n_q, ctx->qf_heads, d_h, o, ctx->stream);
        launch_gemm_store_16(o, ctx->qf_wo, static_cast<uint16_t*>(speech_emb), n_windows * n_q, ctx->qf_dout, d_h, true, ctx->stream);
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int ctc_head_gate(ssd_ctx* ctx, const void* enc_h, const int32_t* cu_frames, int B, int blank_id, float tau_ctc,
                  float* frame_entropy, int32_t* frame_argmax, float* max_entropy, uint8_t* gate_pass,
                  int32_t* draft_ctc, int32_t* draft_len) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->head_V) return fail(ctx, SSD_EINVAL, "ctc_head_gate: no output layer set (ssd_set_ctc_head)");
    if (!enc_h || !cu_frames || !max_entropy || !gate_pass || !draft_ctc || !draft_len)
        return fail(ctx, SSD_EINVAL, "ctc_head_gate: NULL argument");
    if (B <= 0) return fail(ctx, SSD_EINVAL, "ctc_head_gate: B must be positive (got %d)", B);
    const int V = ctx->head_V, d = ctx->head_d;
    if (blank_id < 0 || blank_id >= V) return fail(ctx, SSD_EINVAL, "ctc_head_gate: blank_id %d outside [0, %d)", blank_id, V);
    if (!check_cu(cu_frames, B, true))
        return fail(ctx, SSD_EINVAL, "ctc_head_gate: cu_frames must start at 0 and increase strictly (every utterance needs a frame)");
    const int64_t n_rows = cu_frames[B];
    const HeadPlan p = plan_head(n_rows, B, V);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "ctc_head_gate: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);
    char* ws = static_cast<char*>(ctx->ws);
    float* H = frame_entropy ? frame_entropy : reinterpret_cast<float*>(ws + p.H);
    int32_t* arg = frame_argmax ? frame_argmax : reinterpret_cast<int32_t*>(ws + p.arg);
    int32_t* cu_dev = reinterpret_cast<int32_t*>(ws + p.cu);
    int rc = upload(ctx, cu_frames, cu_dev, (size_t)(B + 1) * 4);
    if (rc != SSD_OK) return rc;
    {
        ProfScope ps(ctx, SSD_PROF_CTC_HEAD);
        // the kernels address the states with 32-bit byte offsets: at most 4 GiB of them per launch
        const int64_t chunk = ((int64_t)0xffffffffu / ((int64_t)d * 2)) / 256 * 256;
        for (int64_t r0 = 0; r0 < n_rows; r0 += chunk) {
            const int rows = (int)std::min<int64_t>(chunk, n_rows - r0);
            launch_ctc_head(static_cast<const uint16_t*>(enc_h) + r0 * d, ctx->head_w, ctx->head_bias, rows, d, V,
                            ctx->head_V_pad, reinterpret_cast<float4*>(ws + p.part), H + r0, arg + r0, ctx->stream);
        }
        launch_gate_utterances(H, arg, cu_dev, n_rows, B, blank_id, tau_ctc, max_entropy, gate_pass, draft_ctc, draft_len,
                               ctx->stream);
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

}  // extern "C"

namespace {

size_t kv_layer_bytes(const ssd_model_cfg& m, int64_t slots) {
    return (size_t)slots * m.n_kv_heads * m.head_dim * elem_size(m.dtype);
}
// K cache and V cache of layer l
void* kv_k(ssd_ctx* c, int l) { return static_cast<char*>(c->kv) + (size_t)(2 * l) * kv_layer_bytes(c->cfg, c->kv_slots); }
void* kv_v(ssd_ctx* c, int l) { return static_cast<char*>(c->kv) + (size_t)(2 * l + 1) * kv_layer_bytes(c->cfg, c->kv_slots); }

int verify_impl(ssd_ctx* ctx, const void* speech_emb, const int32_t* cu_speech, const int32_t* prompt_ids,
                const int32_t* cu_prompt, const int32_t* draft_ids, const int32_t* cu_draft, int Bv,
                const int32_t* kv_start, void* h_verify) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->has_model) return fail(ctx, SSD_EINVAL, "verify_forward: context was created without a model");
    if (!cu_speech || !cu_prompt || !cu_draft) return fail(ctx, SSD_EINVAL, "verify_forward: NULL cu_* array");
    if (Bv <= 0) return fail(ctx, SSD_EINVAL, "verify_forward: Bv must be positive (got %d)", Bv);
    if (!check_cu(cu_speech, Bv, false) || !check_cu(cu_prompt, Bv, false) || !check_cu(cu_draft, Bv, false))
        return fail(ctx, SSD_EINVAL, "verify_forward: cu_* arrays must start at 0 and be non-decreasing");
    const ssd_model_cfg& m = ctx->cfg;
    const int64_t sum_S = cu_speech[Bv], sum_P = cu_prompt[Bv], Mv = cu_draft[Bv];
    const int64_t M = sum_S + sum_P + Mv;
    if ((sum_S && !speech_emb) || (sum_P && !prompt_ids) || (Mv && (!draft_ids || !h_verify)))
        return fail(ctx, SSD_EINVAL, "verify_forward: NULL data pointer");
    if (M > 0x3fffffff) return fail(ctx, SSD_ESHAPE, "verify_forward: too many rows");
    {   // the GEMM loaders address an operand matrix with 32-bit byte offsets: each must stay below 4 GiB
        const int64_t widest = std::max<int64_t>({(int64_t)m.d_ff, (int64_t)(m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim, (int64_t)m.d_model});
        if (M * widest * (int64_t)elem_size(m.dtype) >= ((int64_t)1 << 32))
            return fail(ctx, SSD_ESHAPE, "verify_forward: %lld rows of %lld columns exceed the 4 GiB an activation matrix may have; "
                        "split the batch (ssd_plan_batches)", (long long)M, (long long)widest);
    }
    const int tile_rows = attn_tile_rows(m.dtype);
    for (int b = 0; b < Bv; ++b) {
        const int S = cu_speech[b + 1] - cu_speech[b], P = cu_prompt[b + 1] - cu_prompt[b], U = cu_draft[b + 1] - cu_draft[b];
        if (S + P < 1) return fail(ctx, SSD_EINVAL, "verify_forward: utterance %d has no speech or prompt row", b);
        if (S + P + U > m.max_positions)
            return fail(ctx, SSD_ESHAPE, "verify_forward: utterance %d has %d rows, max_positions is %d", b, S + P + U, m.max_positions);
        if (kv_start && (kv_start[b] < 0 || (int64_t)kv_start[b] + S + P + U > ctx->kv_slots))
            return fail(ctx, SSD_EINVAL, "verify_forward_kv: utterance %d does not fit the K/V cache (start %d, %d rows, %lld slots)",
                        b, kv_start[b], S + P + U, (long long)ctx->kv_slots);
    }
    if (kv_start && !ctx->kv) return fail(ctx, SSD_EINVAL, "verify_forward_kv: no K/V cache set");
    const VerifyPlan p = plan_verify(m, M, Mv, Bv);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "verify_forward: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);

    // ---- host metadata: source of every decoder row, its position, verification rows, attention tiles
    std::vector<char> meta(p.meta_bytes);
    int32_t* row_src = reinterpret_cast<int32_t*>(meta.data() + p.row_src);
    int32_t* pos = reinterpret_cast<int32_t*>(meta.data() + p.pos);
    int32_t* vrow = reinterpret_cast<int32_t*>(meta.data() + p.vrow);
    int32_t* row_slot = reinterpret_cast<int32_t*>(meta.data() + p.row_slot);
    AttnTile* tiles = reinterpret_cast<AttnTile*>(meta.data() + p.tiles);
    int n_tiles = 0;
    int64_t r = 0;
    for (int b = 0; b < Bv; ++b) {
        const int S = cu_speech[b + 1] - cu_speech[b], P = cu_prompt[b + 1] - cu_prompt[b], U = cu_draft[b + 1] - cu_draft[b];
        const int n = S + P + U;
        const int start = (int)r;
        for (int i = 0; i < S; ++i, ++r) { row_src[r] = cu_speech[b] + i; pos[r] = i; }
        for (int i = 0; i < P; ++i, ++r) { row_src[r] = SRC_PROMPT | (cu_prompt[b] + i); pos[r] = S + i; }
        for (int i = 0; i < U; ++i, ++r) { row_src[r] = SRC_DRAFT | (cu_draft[b] + i); pos[r] = S + P + i; }
        // draft token i (1-based) is scored by sequence index S + P + i - 2
        for (int i = 1; i <= U; ++i) vrow[cu_draft[b] + i - 1] = start + S + P + i - 2;
        if (kv_start) for (int i = 0; i < n; ++i) row_slot[start + i] = kv_start[b] + i;
        for (int q = 0; q < n; q += tile_rows) tiles[n_tiles++] = AttnTile{start, n, q, 0};
    }
    char* ws = static_cast<char*>(ctx->ws);
    int rc = upload(ctx, meta.data(), ws, p.meta_bytes);
    if (rc != SSD_OK) return rc;
    const int32_t* d_row_src = reinterpret_cast<const int32_t*>(ws + p.row_src);
    const int32_t* d_pos = reinterpret_cast<const int32_t*>(ws + p.pos);
    const int32_t* d_vrow = reinterpret_cast<const int32_t*>(ws + p.vrow);
    const int32_t* d_row_slot = reinterpret_cast<const int32_t*>(ws + p.row_slot);
    const AttnTile* d_tiles = reinterpret_cast<const AttnTile*>(ws + p.tiles);
    float* x = reinterpret_cast<float*>(ws + p.x);
    void* a = ws + p.a;
    void* qkv = ws + p.qkv;
    void* att = ws + p.attn;
    void* h = ws + p.h;
    hipStream_t st = ctx->stream;
    const int Mi = (int)M, d = m.d_model, dq = m.n_q_heads * m.head_dim, dkv = m.n_kv_heads * m.head_dim;

    { ProfScope ps(ctx, SSD_PROF_OTHER); launch_embed_rows(m.dtype, speech_emb, ctx->embed, prompt_ids, draft_ids, d_row_src, Mi, d, m.vocab, x, ctx->dev_flags, st); }
    float* rope_rows = nullptr;
    if (m.dtype == SSD_BF16 && M > SKINNY_MAX_ROWS) {
        ProfScope ps(ctx, SSD_PROF_OTHER);
        rope_rows = reinterpret_cast<float*>(ws + p.rope_rows);
        launch_gather_rows(ctx->rope_tab, d_pos, Mi, 64 * sizeof(float2), rope_rows, st);
    }
    float* partials = reinterpret_cast<float*>(ws + p.partials);
    const int64_t split_stride = (int64_t)Mi * d;
    int pending = 1;            // K splits of the last residual projection still to be added to x (1: none)
    // Rows that continue after the attention of the last layer: Eq. 5 needs the output distribution at
    // the verification positions only, so the output projection and the MLP of that layer run on those
    // Mv rows (gathered), not on all M.  Exactly the same values: rows do not interact after attention.
    float* x_c = reinterpret_cast<float*>(ws + p.x_c);
    void* att_c = ws + p.attn_c;
    const int Mvi = (int)Mv;
    bool compact = false;
    for (int l = 0; l < m.n_layers; ++l) {
        { ProfScope ps(ctx, SSD_PROF_OTHER); launch_rmsnorm(m.dtype, x, ctx->norm_attn[l], nullptr, Mi, d, m.rms_eps, a, partials, pending, split_stride, ctx->dev_flags, ctx->bf16_ops, st); }
        pending = 1;
        if (m.dtype == SSD_BF16) {
            { ProfScope ps(ctx, SSD_PROF_GEMM_QKV); launch_gemm_qkv_rope((const uint16_t*)a, (const uint16_t*)ctx->wqkv[l], ctx->s_qkv[l], (uint16_t*)qkv, d_pos, ctx->rope_tab, Mi, d, dq, dkv, ctx->ds_qkv[l],
                                                                         kv_start ? d_row_slot : nullptr, kv_start ? (uint16_t*)kv_k(ctx, l) : nullptr, kv_start ? (uint16_t*)kv_v(ctx, l) : nullptr, rope_rows, ctx->dev_flags, ctx->bf16_ops, st); }
            { ProfScope ps(ctx, SSD_PROF_ATTN); launch_attn_mfma((const uint16_t*)qkv, (uint16_t*)att, d_tiles, n_tiles, m.n_q_heads, m.n_kv_heads, ctx->bf16_ops, st); }
            float* xr = x; const void* attr = att; int rows = Mi;
            if (l == m.n_layers - 1) {
                ProfScope ps(ctx, SSD_PROF_OTHER);
                launch_gather_rows(att, d_vrow, Mvi, (int64_t)dq * 2, att_c, st);
                launch_gather_rows(x, d_vrow, Mvi, (int64_t)d * 4, x_c, st);
                xr = x_c; attr = att_c; rows = Mvi; compact = true;
            }
            const int64_t stride = (int64_t)rows * d;
            { ProfScope ps(ctx, SSD_PROF_GEMM_O); pending = launch_gemm_residual((const uint16_t*)attr, (const uint16_t*)ctx->wo[l], ctx->s_o[l], xr, partials, rows, d, dq, ctx->ds_o[l], ctx->bf16_ops, st); }
            { ProfScope ps(ctx, SSD_PROF_OTHER); launch_rmsnorm(m.dtype, xr, ctx->norm_mlp[l], nullptr, rows, d, m.rms_eps, a, partials, pending, stride, ctx->dev_flags, ctx->bf16_ops, st); }
            pending = 1;
            { ProfScope ps(ctx, SSD_PROF_GEMM_GATE_UP); launch_gemm_swiglu((const uint16_t*)a, (const uint16_t*)ctx->wgu[l], ctx->s_gu[l], (uint16_t*)h, rows, m.d_ff, d, ctx->ds_gu[l], ctx->dev_flags, ctx->bf16_ops, st); }
            { ProfScope ps(ctx, SSD_PROF_GEMM_DOWN); pending = launch_gemm_residual((const uint16_t*)h, (const uint16_t*)ctx->w_down[l], ctx->s_down[l], xr, partials, rows, d, m.d_ff, ctx->ds_down[l], ctx->bf16_ops, st); }
        } else {
            float* gu = reinterpret_cast<float*>(ws + p.gu);
            launch_gemm_f32((const float*)a, (const float*)ctx->wqkv[l], (float*)qkv, Mi, dq + 2 * dkv, d, F32_STORE, st);
            launch_rope_f32((float*)qkv, d_pos, ctx->rope_tab, Mi, m.n_q_heads + m.n_kv_heads, m.head_dim, dq + 2 * dkv, st);
            if (kv_start) launch_kv_store(m.dtype, qkv, d_row_slot, Mi, dq, dkv, kv_k(ctx, l), kv_v(ctx, l), st);
            launch_attn_f32((const float*)qkv, (float*)att, d_tiles, n_tiles, m.n_q_heads, m.n_kv_heads, m.head_dim, st);
            launch_gemm_f32((const float*)att, (const float*)ctx->wo[l], x, Mi, d, dq, F32_ADD, st);
            launch_rmsnorm(m.dtype, x, ctx->norm_mlp[l], nullptr, Mi, d, m.rms_eps, a, nullptr, 1, 0, ctx->dev_flags, ctx->bf16_ops, st);
            launch_gemm_f32((const float*)a, (const float*)ctx->wgu[l], gu, Mi, 2 * m.d_ff, d, F32_STORE, st);
            launch_swiglu_f32(gu, (float*)h, Mi, m.d_ff, st);
            launch_gemm_f32((const float*)h, (const float*)ctx->w_down[l], x, Mi, d, m.d_ff, F32_ADD, st);
        }
    }
    // final RMSNorm of the positions that score a draft token
    if (compact) {
        ProfScope ps(ctx, SSD_PROF_OTHER);
        launch_rmsnorm(m.dtype, x_c, ctx->norm_final, nullptr, Mvi, d, m.rms_eps, h_verify, partials, pending, (int64_t)Mvi * d, ctx->dev_flags, ctx->bf16_ops, st);
    } else {
        ProfScope ps(ctx, SSD_PROF_OTHER);
        launch_rmsnorm(m.dtype, x, ctx->norm_final, d_vrow, Mvi, d, m.rms_eps, h_verify, partials, pending, split_stride, ctx->dev_flags, ctx->bf16_ops, st);
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

struct ArPlan {
    size_t row_src, kv_start, pos, n_ctx, slot, meta_bytes;       // uploaded once: [Br], [Br], [steps][Br] x 3
    size_t x, a, qkv, attn, gu, h, partials, qkv_part, hfin, logp, part_ms, tgt, part_arg, total;
};
ArPlan plan_ar(const ssd_model_cfg& c, int64_t Br, int64_t steps) {
    ArPlan p;
    const size_t es = elem_size(c.dtype);
    const int64_t d = c.d_model, dq = (int64_t)c.n_q_heads * c.head_dim, dkv = (int64_t)c.n_kv_heads * c.head_dim;
    size_t o = 0;
    p.row_src = o; o = align_up(o + (size_t)Br * 4);
    p.kv_start = o; o = align_up(o + (size_t)Br * 4);
    p.pos = o; o = align_up(o + (size_t)(steps * Br) * 4);
    p.n_ctx = o; o = align_up(o + (size_t)(steps * Br) * 4);
    p.slot = o; o = align_up(o + (size_t)(steps * Br) * 4);
    p.meta_bytes = o;
    p.x = o; o = align_up(o + (size_t)(Br * d) * 4);
    p.a = o; o = align_up(o + (size_t)(Br * d) * es);
    p.qkv = o; o = align_up(o + (size_t)(Br * (dq + 2 * dkv)) * es);
    p.attn = o; o = align_up(o + (size_t)(Br * dq) * es);
    p.gu = o; if (c.dtype == SSD_F32) o = align_up(o + (size_t)(Br * 2 * c.d_ff) * 4);
    p.h = o; o = align_up(o + (size_t)(Br * c.d_ff) * es);
    p.partials = o; if (c.dtype == SSD_BF16 && Br <= SKINNY_MAX_ROWS) o = align_up(o + (size_t)SKINNY_MAX_SPLITS * Br * d * 4);
    // K-split partial sums of the QKV projection (finished inside the decode attention, few rows only)
    p.qkv_part = o; if (c.dtype == SSD_BF16 && Br <= 32) o = align_up(o + (size_t)SKINNY_MAX_SPLITS * Br * (dq + 2 * dkv) * 4);
    p.hfin = o; o = align_up(o + (size_t)(Br * d) * es);
    p.logp = o; o = align_up(o + (size_t)Br * 4);
    p.part_ms = p.tgt = p.part_arg = o;
    if (c.dtype == SSD_BF16) {
        const int64_t g = lmhead_col_groups(c.vocab);
        p.part_ms = o; o = align_up(o + (size_t)(g * Br) * sizeof(float2));
        p.tgt = o; o = align_up(o + (size_t)Br * 4);
        p.part_arg = o; o = align_up(o + (size_t)(g * Br) * sizeof(int2));
    }
    p.total = o;
    return p;
}

}  // namespace

extern "C" {

int verify_forward(ssd_ctx* ctx, const void* speech_emb, const int32_t* cu_speech, const int32_t* prompt_ids,
                   const int32_t* cu_prompt, const int32_t* draft_ids, const int32_t* cu_draft, int Bv, void* h_verify) {
    return verify_impl(ctx, speech_emb, cu_speech, prompt_ids, cu_prompt, draft_ids, cu_draft, Bv, nullptr, h_verify);
}

int verify_forward_kv(ssd_ctx* ctx, const void* speech_emb, const int32_t* cu_speech, const int32_t* prompt_ids,
                      const int32_t* cu_prompt, const int32_t* draft_ids, const int32_t* cu_draft, int Bv,
                      const int32_t* kv_start, void* h_verify) {
    if (ctx && !kv_start) return fail(ctx, SSD_EINVAL, "verify_forward_kv: NULL kv_start");
    return verify_impl(ctx, speech_emb, cu_speech, prompt_ids, cu_prompt, draft_ids, cu_draft, Bv, kv_start, h_verify);
}

size_t ssd_kv_cache_bytes(const ssd_ctx* ctx, int64_t slots) {
    if (!ctx || !ctx->has_model || slots <= 0) return 0;
    return (size_t)2 * ctx->cfg.n_layers * kv_layer_bytes(ctx->cfg, slots);
}

int ssd_set_kv_cache(ssd_ctx* ctx, void* dev_ptr, size_t bytes, int64_t slots) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->has_model) return fail(ctx, SSD_EINVAL, "ssd_set_kv_cache: context was created without a model");
    if (!dev_ptr || slots <= 0) { ctx->kv = nullptr; ctx->kv_slots = 0; return SSD_OK; }
    if (reinterpret_cast<uintptr_t>(dev_ptr) & 255) return fail(ctx, SSD_EINVAL, "K/V cache must be 256-byte aligned");
    if (bytes < ssd_kv_cache_bytes(ctx, slots)) return fail(ctx, SSD_EWORKSPACE, "K/V cache of %zu bytes needed for %lld slots, %zu given",
                                                            ssd_kv_cache_bytes(ctx, slots), (long long)slots, bytes);
    ctx->kv = dev_ptr;
    ctx->kv_slots = slots;
    return SSD_OK;
}

size_t ssd_ar_workspace_bytes(const ssd_ctx* ctx, int max_utts, int max_steps) {
    if (!ctx || !ctx->has_model || max_utts <= 0 || max_steps <= 0) return 0;
    return plan_ar(ctx->cfg, max_utts, max_steps).total + 256;
}

int ar_fallback(ssd_ctx* ctx, int Br, const int32_t* kv_start, const int32_t* ctx_len, const int32_t* first_tok,
                int n_steps, int32_t* out_tokens) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->has_model) return fail(ctx, SSD_EINVAL, "ar_fallback: context was created without a model");
    if (!kv_start || !ctx_len || !first_tok || !out_tokens) return fail(ctx, SSD_EINVAL, "ar_fallback: NULL argument");
    if (Br <= 0 || n_steps <= 0) return fail(ctx, SSD_EINVAL, "ar_fallback: Br and n_steps must be positive");
    if (!ctx->kv) return fail(ctx, SSD_EINVAL, "ar_fallback: no K/V cache set");
    const ssd_model_cfg& m = ctx->cfg;
    if (m.head_dim % 8) return fail(ctx, SSD_ESHAPE, "ar_fallback: head_dim must be a multiple of 8 (got %d)", m.head_dim);
    for (int b = 0; b < Br; ++b) {
        if (ctx_len[b] < 1) return fail(ctx, SSD_EINVAL, "ar_fallback: utterance %d has an empty context", b);
        if (ctx_len[b] + n_steps > m.max_positions)
            return fail(ctx, SSD_ESHAPE, "ar_fallback: utterance %d would reach position %d, max_positions is %d", b, ctx_len[b] + n_steps, m.max_positions);
        if (kv_start[b] < 0 || (int64_t)kv_start[b] + ctx_len[b] + n_steps > ctx->kv_slots)
            return fail(ctx, SSD_EINVAL, "ar_fallback: utterance %d does not fit the K/V cache", b);
    }
    const ArPlan p = plan_ar(m, Br, n_steps);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "ar_fallback: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);
    std::vector<char> meta(p.meta_bytes);
    int32_t* row_src = reinterpret_cast<int32_t*>(meta.data() + p.row_src);
    int32_t* h_kvs = reinterpret_cast<int32_t*>(meta.data() + p.kv_start);
    int32_t* pos = reinterpret_cast<int32_t*>(meta.data() + p.pos);
    int32_t* nctx = reinterpret_cast<int32_t*>(meta.data() + p.n_ctx);
    int32_t* slot = reinterpret_cast<int32_t*>(meta.data() + p.slot);
    for (int b = 0; b < Br; ++b) {
        row_src[b] = SRC_DRAFT | b;
        h_kvs[b] = kv_start[b];
        for (int t = 0; t < n_steps; ++t) {
            pos[(size_t)t * Br + b] = ctx_len[b] + t;               // position of the token fed at step t
            nctx[(size_t)t * Br + b] = ctx_len[b] + t + 1;          // rows it attends to, itself included
            slot[(size_t)t * Br + b] = kv_start[b] + ctx_len[b] + t;
        }
    }
    char* ws = static_cast<char*>(ctx->ws);
    int rc = upload(ctx, meta.data(), ws, p.meta_bytes);
    if (rc != SSD_OK) return rc;
    const int32_t* d_row_src = reinterpret_cast<const int32_t*>(ws + p.row_src);
    const int32_t* d_kvs = reinterpret_cast<const int32_t*>(ws + p.kv_start);
    float* x = reinterpret_cast<float*>(ws + p.x);
    void* a = ws + p.a; void* qkv = ws + p.qkv; void* att = ws + p.attn; void* h = ws + p.h; void* hfin = ws + p.hfin;
    float* partials = reinterpret_cast<float*>(ws + p.partials);
    float* qkv_part = reinterpret_cast<float*>(ws + p.qkv_part);
    float* logp = reinterpret_cast<float*>(ws + p.logp);
    hipStream_t st = ctx->stream;
    const int d = m.d_model, dq = m.n_q_heads * m.head_dim, dkv = m.n_kv_heads * m.head_dim;
    const int64_t split_stride = (int64_t)Br * d;
    ProfScope ps_all(ctx, SSD_PROF_AR);
    for (int t = 0; t < n_steps; ++t) {
        const int32_t* tok_in = t == 0 ? first_tok : out_tokens + (size_t)(t - 1) * Br;
        const int32_t* d_pos = reinterpret_cast<const int32_t*>(ws + p.pos) + (size_t)t * Br;
        const int32_t* d_nctx = reinterpret_cast<const int32_t*>(ws + p.n_ctx) + (size_t)t * Br;
        const int32_t* d_slot = reinterpret_cast<const int32_t*>(ws + p.slot) + (size_t)t * Br;
        launch_embed_rows(m.dtype, nullptr, ctx->embed, nullptr, tok_in, d_row_src, Br, d, m.vocab, x, ctx->dev_flags, st);
        int pending = 1;
        for (int l = 0; l < m.n_layers; ++l) {
            launch_rmsnorm(m.dtype, x, ctx->norm_attn[l], nullptr, Br, d, m.rms_eps, a, partials, pending, split_stride, ctx->dev_flags, ctx->bf16_ops, st);
            pending = 1;
            if (m.dtype == SSD_BF16) {
                // few rows, head_dim 128: the QKV projection stays K-split and the decode attention finishes it
                const int qsplits = (Br <= 32 && m.head_dim == 128)
                    ? launch_gemm_qkv_partial((const uint16_t*)a, ctx->s_qkv[l], qkv_part, Br, d, dq + 2 * dkv, ctx->ds_qkv[l], ctx->bf16_ops, st) : 0;
                if (qsplits) {
                    launch_decode_attn_fused(qkv_part, qsplits, ctx->rope_tab, kv_k(ctx, l), kv_v(ctx, l), d_kvs, d_nctx, Br,
                                             m.n_q_heads, m.n_kv_heads, att, ctx->dev_flags, ctx->bf16_ops, st);
                } else {
                    launch_gemm_qkv_rope((const uint16_t*)a, (const uint16_t*)ctx->wqkv[l], ctx->s_qkv[l], (uint16_t*)qkv, d_pos, ctx->rope_tab, Br, d, dq, dkv, ctx->ds_qkv[l],
                                         d_slot, (uint16_t*)kv_k(ctx, l), (uint16_t*)kv_v(ctx, l), nullptr, ctx->dev_flags, ctx->bf16_ops, st);
                    launch_decode_attn(m.dtype, qkv, kv_k(ctx, l), kv_v(ctx, l), d_kvs, d_nctx, Br, m.n_q_heads, m.n_kv_heads, m.head_dim, att, ctx->bf16_ops, st);
                }
                pending = launch_gemm_residual((const uint16_t*)att, (const uint16_t*)ctx->wo[l], ctx->s_o[l], x, partials, Br, d, dq, ctx->ds_o[l], ctx->bf16_ops, st);
                launch_rmsnorm(m.dtype, x, ctx->norm_mlp[l], nullptr, Br, d, m.rms_eps, a, partials, pending, split_stride, ctx->dev_flags, ctx->bf16_ops, st);
                pending = 1;
                launch_gemm_swiglu((const uint16_t*)a, (const uint16_t*)ctx->wgu[l], ctx->s_gu[l], (uint16_t*)h, Br, m.d_ff, d, ctx->ds_gu[l], ctx->dev_flags, ctx->bf16_ops, st);
                pending = launch_gemm_residual((const uint16_t*)h, (const uint16_t*)ctx->w_down[l], ctx->s_down[l], x, partials, Br, d, m.d_ff, ctx->ds_down[l], ctx->bf16_ops, st);
            } else {
                float* gu = reinterpret_cast<float*>(ws + p.gu);
                launch_gemm_f32((const float*)a, (const float*)ctx->wqkv[l], (float*)qkv, Br, dq + 2 * dkv, d, F32_STORE, st);
                launch_rope_f32((float*)qkv, d_pos, ctx->rope_tab, Br, m.n_q_heads + m.n_kv_heads, m.head_dim, dq + 2 * dkv, st);
                launch_kv_store(m.dtype, qkv, d_slot, Br, dq, dkv, kv_k(ctx, l), kv_v(ctx, l), st);
                launch_decode_attn(m.dtype, qkv, kv_k(ctx, l), kv_v(ctx, l), d_kvs, d_nctx, Br, m.n_q_heads, m.n_kv_heads, m.head_dim, att, ctx->bf16_ops, st);
                launch_gemm_f32((const float*)att, (const float*)ctx->wo[l], x, Br, d, dq, F32_ADD, st);
                launch_rmsnorm(m.dtype, x, ctx->norm_mlp[l], nullptr, Br, d, m.rms_eps, a, nullptr, 1, 0, ctx->dev_flags, ctx->bf16_ops, st);
                launch_gemm_f32((const float*)a, (const float*)ctx->wgu[l], gu, Br, 2 * m.d_ff, d, F32_STORE, st);
                launch_swiglu_f32(gu, (float*)h, Br, m.d_ff, st);
                launch_gemm_f32((const float*)h, (const float*)ctx->w_down[l], x, Br, d, m.d_ff, F32_ADD, st);
            }
        }
        launch_rmsnorm(m.dtype, x, ctx->norm_final, nullptr, Br, d, m.rms_eps, hfin, partials, pending, split_stride, ctx->dev_flags, ctx->bf16_ops, st);
        int32_t* tok_out = out_tokens + (size_t)t * Br;
        if (m.dtype == SSD_BF16) {
            float2* part_ms = reinterpret_cast<float2*>(ws + p.part_ms);
            float* tgt = reinterpret_cast<float*>(ws + p.tgt);
            int2* part_arg = reinterpret_cast<int2*>(ws + p.part_arg);
            launch_lmhead_mfma((const uint16_t*)hfin, (const uint16_t*)ctx->lm_head, tok_in, Br, d, m.vocab, part_ms, tgt, part_arg, true, ctx->ds_lm, ctx->bf16_ops, st);
            launch_lmhead_finalize(part_ms, tgt, part_arg, lmhead_col_groups(m.vocab), Br, logp, tok_out, ctx->dev_flags, st);
        } else {
            launch_lmhead_f32((const float*)hfin, (const float*)ctx->lm_head, tok_in, Br, d, m.vocab, logp, tok_out, st);
        }
    }
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

int accept_prefix(ssd_ctx* ctx, const void* h_verify, const int32_t* draft_ids, const int32_t* cu_draft, int Bv,
                  float tau_slm, float* draft_logp, int32_t* accept_len, uint8_t* all_accepted, int32_t* greedy_tok) {
    if (!ctx) return SSD_EINVAL;
    if (!ctx->has_model) return fail(ctx, SSD_EINVAL, "accept_prefix: context was created without a model");
    if (!cu_draft || !accept_len || !all_accepted) return fail(ctx, SSD_EINVAL, "accept_prefix: NULL argument");
    if (Bv <= 0) return fail(ctx, SSD_EINVAL, "accept_prefix: Bv must be positive (got %d)", Bv);
    if (!check_cu(cu_draft, Bv, false)) return fail(ctx, SSD_EINVAL, "accept_prefix: cu_draft must start at 0 and be non-decreasing");
    if (tau_slm != tau_slm) return fail(ctx, SSD_EINVAL, "accept_prefix: tau_slm is NaN");
    const int64_t Mv = cu_draft[Bv];
    if (Mv && (!h_verify || !draft_ids || !draft_logp)) return fail(ctx, SSD_EINVAL, "accept_prefix: NULL data pointer");
    const ssd_model_cfg& m = ctx->cfg;
    if (Mv * (int64_t)m.d_model * (int64_t)elem_size(m.dtype) >= ((int64_t)1 << 32))
        return fail(ctx, SSD_ESHAPE, "accept_prefix: %lld rows exceed the 4 GiB the hidden rows may have; split the batch", (long long)Mv);
    const AcceptPlan p = plan_accept(m, Mv, Bv);
    if (!ctx->ws || ctx->ws_bytes < p.total)
        return fail(ctx, SSD_EWORKSPACE, "accept_prefix: workspace of %zu bytes needed, %zu set", p.total, ctx->ws_bytes);
    char* ws = static_cast<char*>(ctx->ws);
    int32_t* cu_dev = reinterpret_cast<int32_t*>(ws + p.cu);
    int rc = upload(ctx, cu_draft, cu_dev, (size_t)(Bv + 1) * 4);
    if (rc != SSD_OK) return rc;
    hipStream_t st = ctx->stream;
    ProfScope ps_all(ctx, SSD_PROF_LMHEAD);
    if (m.dtype == SSD_BF16) {
        float2* part_ms = reinterpret_cast<float2*>(ws + p.part_ms);
        float* tgt = reinterpret_cast<float*>(ws + p.tgt);
        int2* part_arg = reinterpret_cast<int2*>(ws + p.part_arg);
        launch_lmhead_mfma((const uint16_t*)h_verify, (const uint16_t*)ctx->lm_head, draft_ids, (int)Mv, m.d_model, m.vocab,
                           part_ms, tgt, part_arg, greedy_tok != nullptr, ctx->ds_lm, ctx->bf16_ops, st);
        launch_lmhead_finalize(part_ms, tgt, part_arg, lmhead_col_groups(m.vocab), (int)Mv, draft_logp, greedy_tok, ctx->dev_flags, st);
    } else {
        launch_lmhead_f32((const float*)h_verify, (const float*)ctx->lm_head, draft_ids, (int)Mv, m.d_model, m.vocab,
                          draft_logp, greedy_tok, st);
    }
    // ln(tau) in double, rounded once to fp32; tau <= 0 accepts every token
    const float ln_tau = tau_slm > 0.f ? (float)log((double)tau_slm) : -INFINITY;
    launch_accept_scan(draft_logp, cu_dev, Bv, ln_tau, accept_len, all_accepted, st);
    HIP_TRY(ctx, hipGetLastError());
    return SSD_OK;
}

}  // extern "C"
