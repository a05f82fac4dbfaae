// Host side of the specverify library: context, HBM residency plan, host->HBM layer streamer,
// the verify / draft / prefill passes (kernel enqueue order) and the C ABI.
//
// Streams: `compute` runs target passes, `copy` runs weight copies into the staging ring, `draft`
// runs the draft model.  All hand-offs are HIP events; the host thread never blocks inside the
// draft/verify loop.
#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <deque>
#include <string>
#include <vector>

#include "common.h"

using namespace sv;

namespace {

thread_local std::string g_err;

struct Layout {                // element offsets inside a layer blob
    int64_t g1, wqkv, wo, g2, wr, w1, w3, w2, expert_stride, total, attn_total;
};
struct GlobalLayout { int64_t emb, gf, head, total; };

inline int64_t align128(int64_t n) { return (n + 127) / 128 * 128; }

bool shape_ok(const spec_model_shape* s) {
    if (!s) return false;
    if (s->n_layers < 0 || s->d_model <= 0 || s->n_q_heads <= 0 || s->n_kv_heads <= 0 ||
        s->head_dim <= 0 || s->vocab <= 0)
        return false;
    if (s->n_q_heads % s->n_kv_heads) return false;
    if (s->head_dim % 2 || s->head_dim > 256) return false;
    if (s->dtype != SPEC_F32 && s->dtype != SPEC_BF16) return false;
    if (!s->attn_only) {
        if (s->d_ff <= 0) return false;
        if (s->n_experts < 0 || s->n_experts == 1 || s->n_experts > 8) return false;
        if (s->n_experts > 0 && s->top_k != 2) return false;
    }
    return true;
}

Layout make_layout(const spec_model_shape& s) {
    Layout L{};
    int64_t d = s.d_model, F = s.d_ff, o = 0;
    L.g1 = o; o += align128(d);
    L.wqkv = o; o += align128((int64_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim * d);
    L.wo = o; o += align128(d * (int64_t)s.n_q_heads * s.head_dim);
    L.attn_total = o;
    if (!s.attn_only) {
        L.g2 = o; o += align128(d);
        if (s.n_experts > 0) { L.wr = o; o += align128((int64_t)s.n_experts * d); }
        L.w1 = o;
        L.w3 = L.w1 + align128(F * d);
        L.w2 = L.w3 + align128(F * d);
        L.expert_stride = 2 * align128(F * d) + align128(d * F);
        o = L.w1 + L.expert_stride * std::max(1, s.n_experts);
    }
    L.total = o;
    return L;
}
GlobalLayout make_global_layout(const spec_model_shape& s) {
    GlobalLayout G{};
    int64_t o = 0;
    G.emb = o; o += align128((int64_t)s.vocab * s.d_model);
    G.gf = o; o += align128(s.d_model);
    G.head = o; o += align128((int64_t)s.vocab * s.d_model);
    G.total = o;
    return G;
}
inline size_t esize(int dtype) { return dtype == SPEC_BF16 ? 2 : 4; }

struct Workspace {
    int t_max = 0;
    float* x = nullptr; void* h = nullptr; float* qkv = nullptr; void* q = nullptr; void* att = nullptr;
    float2* cs = nullptr; int32_t* tok_in = nullptr; int32_t* row_pos = nullptr;
    int32_t* r_ids = nullptr; float* r_wts = nullptr; int32_t* offsets = nullptr; int32_t* perm = nullptr;
    int32_t* slots = nullptr; void* u = nullptr; float* y = nullptr;
};

struct Sub {
    int B = 0;
    bool ready = false;         // sequences loaded
    SeqState st{};
    int32_t* page_table = nullptr;      // shared by target and draft pools (same geometry per seq)
    void* kv_t = nullptr; void* kv_d = nullptr;
    int32_t* draft_tokens = nullptr;    // [B_max, k_max]
    float* q_logits = nullptr;          // [B_max, k_max, V] (sampling)
    float* logits = nullptr;            // [B_max*(k_max+1), V]
    float* draft_logits = nullptr;      // [B_max, V] (greedy draft)
    int32_t* n_acc = nullptr; int32_t* next_tok = nullptr;
    int last_k = 0, last_draft_k = 0;
    uint32_t round = 0, seq_base = 0;
    hipEvent_t ev_drafted = nullptr, ev_committed = nullptr;
    bool drafted = false;
};

}  // namespace

struct spec_ctx {
    spec_model_shape tgt{}, drf{};
    bool has_draft = false;
    spec_runtime_cfg cfg{};
    Layout tl{}, dl{};
    GlobalLayout gl{};
    size_t es = 2;
    hipStream_t s_compute = nullptr, s_copy = nullptr, s_draft = nullptr;
    bool own_compute = false, own_copy = false, own_draft = false;
    std::string err;
    // target weights
    std::vector<const void*> host_layers;
    std::vector<void*> resident;          // per layer, nullptr if streamed
    std::vector<int> streamed;            // layer ids in pass order
    std::vector<void*> ring;
    std::vector<hipEvent_t> ev_ready, ev_free;
    int64_t copies_issued = 0, uses_done = 0;
    // compact staging (default): the two slots overlap except for `look_bytes` at either end, so the
    // ring is one layer plus one look-ahead piece; copies are issued in two parts (see issue_copy)
    bool compact = false;
    size_t look_bytes = 0;
    int64_t looks_issued = 0;
    size_t blob_bytes = 0;
    void* d_globals = nullptr;
    // draft weights
    std::vector<void*> d_draft_layers;
    void* d_draft_globals = nullptr;
    bool draft_globals_shared = false;
    // state
    KvGeom gt{}, gd{};
    Sub sub[2];
    Workspace wv, wd;
    float* acc_stats = nullptr;
    int64_t* d_hist = nullptr;            // [17] + committed at [17]
    // stats
    int64_t bytes_streamed = 0, layers_streamed = 0, rounds = 0, hbm_weight_bytes = 0;
    std::deque<std::pair<hipEvent_t, hipEvent_t>> copy_timers;
    std::vector<hipEvent_t> timer_pool;
    double copy_busy_ms = 0.0;
    // optional per-kernel-class timing (spec_profile_enable)
    uint32_t prof_mask = 0;
    struct ProfRec { int cat; hipEvent_t e0, e1; };
    std::vector<ProfRec> prof_pending;
    double prof_ms[SPEC_PROF_N] = {0};
    int64_t prof_n[SPEC_PROF_N] = {0};
    // interleave
    int cur = 0;
    bool primed = false;
    std::vector<void*> allocs;            // everything to hipFree
};

namespace {

int fail(spec_ctx* c, int code, const char* fmt, ...) {
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (c) c->err = buf;
    g_err = buf;
    return code;
}

#define HIPCHK(c, call)                                                                          \
    do {                                                                                         \
        hipError_t e_ = (call);                                                                  \
        if (e_ != hipSuccess)                                                                    \
            return fail((c), SPEC_ERR_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), \
                        __FILE__, __LINE__);                                                     \
    } while (0)

template <typename P>
int dev_alloc(spec_ctx* c, P** out, size_t bytes) {
    void* p = nullptr;
    if (bytes == 0) bytes = 256;
    HIPCHK(c, hipMalloc(&p, bytes));
    c->allocs.push_back(p);
    *out = (P*)p;
    return SPEC_OK;
}

int alloc_workspace(spec_ctx* c, Workspace& w, const spec_model_shape& s, int t_max) {
    size_t es = esize(s.dtype);
    int64_t d = s.d_model, hd = (int64_t)s.n_q_heads * s.head_dim;
    int64_t qkv_rows = (int64_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
    w.t_max = t_max;
    int rc;
    if ((rc = dev_alloc(c, &w.x, t_max * d * 4))) return rc;
    if ((rc = dev_alloc(c, (char**)&w.h, t_max * d * es))) return rc;
    if ((rc = dev_alloc(c, &w.qkv, t_max * qkv_rows * 4))) return rc;
    if ((rc = dev_alloc(c, (char**)&w.q, t_max * hd * es))) return rc;
    if ((rc = dev_alloc(c, (char**)&w.att, t_max * hd * es))) return rc;
    if ((rc = dev_alloc(c, &w.cs, (size_t)t_max * (s.head_dim / 2) * sizeof(float2)))) return rc;
    if ((rc = dev_alloc(c, &w.tok_in, (size_t)t_max * 4))) return rc;
    if ((rc = dev_alloc(c, &w.row_pos, (size_t)t_max * 4))) return rc;
    if (!s.attn_only) {
        int mult = s.n_experts > 0 ? 2 : 1;
        if ((rc = dev_alloc(c, (char**)&w.u, (size_t)mult * t_max * s.d_ff * es))) return rc;
        if (s.n_experts > 0) {
            if ((rc = dev_alloc(c, &w.r_ids, (size_t)t_max * 8))) return rc;
            if ((rc = dev_alloc(c, &w.r_wts, (size_t)t_max * 8))) return rc;
            if ((rc = dev_alloc(c, &w.offsets, 64))) return rc;
            if ((rc = dev_alloc(c, &w.perm, (size_t)t_max * 8))) return rc;
            if ((rc = dev_alloc(c, &w.slots, (size_t)t_max * 8))) return rc;
            if ((rc = dev_alloc(c, &w.y, (size_t)2 * t_max * d * 4))) return rc;
        }
    }
    return SPEC_OK;
}

// ---- per-kernel-class timing ---------------------------------------------------------------------
struct ProfScope {
    spec_ctx* c; int cat; hipStream_t st; hipEvent_t e0 = nullptr, e1 = nullptr; bool on;
    ProfScope(spec_ctx* c_, int cat_, hipStream_t st_) : c(c_), cat(cat_), st(st_) {
        on = c && (c->prof_mask >> cat & 1u);
        if (!on) return;
        auto get = [&](hipEvent_t* e) {
            if (!c->timer_pool.empty()) { *e = c->timer_pool.back(); c->timer_pool.pop_back(); }
            else if (hipEventCreate(e) != hipSuccess) *e = nullptr;
        };
        get(&e0); get(&e1);
        if (!e0 || !e1) { on = false; return; }
        hipEventRecord(e0, st);
    }
    ~ProfScope() {
        if (!on) return;
        hipEventRecord(e1, st);
        c->prof_pending.push_back({cat, e0, e1});
    }
};

// ---- kernel selection ------------------------------------------------------------------------
hipError_t gemm(spec_ctx* c, const GemmArgs& a, int dtype, hipStream_t st) {
    if (dtype == SPEC_BF16 && !(c && (c->cfg.flags & SPEC_FLAG_SIMPLE_KERNELS)))
        return launch_gemm_mfma_bf16(a, st);
    return launch_gemm_simple(a, dtype, st);
}
hipError_t attention(spec_ctx* c, const AttnArgs& a, int dtype, hipStream_t st) {
    if (dtype == SPEC_BF16 && !(c->cfg.flags & SPEC_FLAG_SIMPLE_KERNELS))
        return launch_attention_mfma_bf16(a, st);
    return launch_attention_simple(a, dtype, st);
}

// ---- weight streamer ---------------------------------------------------------------------------
// Streamed layers are used in a fixed cyclic order (layer order, pass after pass) that does not
// depend on any token value, so copies run ahead of compute by up to n_slots layers, across pass
// boundaries as well.  Copy j goes to slot j % n_slots after the compute stream has released the
// layer that used the slot before (ev_free); compute waits for ev_ready of the slot.
int harvest_timers(spec_ctx* c, bool all) {
    while (!c->copy_timers.empty()) {
        auto pr = c->copy_timers.front();
        if (!all && hipEventQuery(pr.second) != hipSuccess) break;
        if (all) HIPCHK(c, hipEventSynchronize(pr.second));
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, pr.first, pr.second));
        c->copy_busy_ms += ms;
        c->timer_pool.push_back(pr.first);
        c->timer_pool.push_back(pr.second);
        c->copy_timers.pop_front();
    }
    return SPEC_OK;
}
int get_timer(spec_ctx* c, hipEvent_t* e) {
    if (c->timer_pool.empty()) {
        if (c->copy_timers.size() > 512) { int rc = harvest_timers(c, false); if (rc) return rc; }
    }
    if (!c->timer_pool.empty()) { *e = c->timer_pool.back(); c->timer_pool.pop_back(); return SPEC_OK; }
    HIPCHK(c, hipEventCreate(e));
    return SPEC_OK;
}

// One timed host->HBM copy on the copy stream.
int timed_copy(spec_ctx* c, void* dst, const void* src, size_t bytes) {
    hipEvent_t t0, t1;
    int rc;
    if ((rc = get_timer(c, &t0)) || (rc = get_timer(c, &t1))) return rc;
    HIPCHK(c, hipEventRecord(t0, c->s_copy));
    HIPCHK(c, hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, c->s_copy));
    HIPCHK(c, hipEventRecord(t1, c->s_copy));
    c->copy_timers.emplace_back(t0, t1);
    c->bytes_streamed += (int64_t)bytes;
    return SPEC_OK;
}

// Whole-slot ring: copy j fills slot j % n_slots once the use that held the slot before is released.
int issue_copy(spec_ctx* c, int64_t j) {
    int ns = (int)c->ring.size();
    int slot = (int)(j % ns);
    int layer = c->streamed[(size_t)(j % (int64_t)c->streamed.size())];
    if (j >= ns) HIPCHK(c, hipStreamWaitEvent(c->s_copy, c->ev_free[slot], 0));
    int rc = timed_copy(c, c->ring[slot], c->host_layers[layer], c->blob_bytes);
    if (rc) return rc;
    HIPCHK(c, hipEventRecord(c->ev_ready[slot], c->s_copy));
    c->layers_streamed += 1;
    return SPEC_OK;
}

// Compact ring (the placeholders of Section 4.2 at sub-layer granularity): slot A = [0, blob), slot B
// = [look, look + blob) of one allocation of blob + look bytes; use j lives in slot j % 2.  The piece
// of a slot that the other slot does not cover (A's head, B's tail: `look` bytes) is the look-ahead
// part of a copy: it only needs the slot's own previous use (j - 2) to be released, so it crosses the
// link while use j - 1 is still being computed.  The rest of the copy overlaps the other slot and
// needs use j - 1 released.  The link therefore stays busy as long as a layer's compute is shorter
// than the look-ahead piece's transfer, with as little as 1 + 1/8 layers of HBM instead of 2 (the
// piece is sized from what the budget leaves; at a whole layer the slots are disjoint).
int issue_look(spec_ctx* c, int64_t j) {
    int par = (int)(j & 1);
    int layer = c->streamed[(size_t)(j % (int64_t)c->streamed.size())];
    size_t off = par ? c->blob_bytes - c->look_bytes : 0;            // piece of the layer blob
    if (j >= 2) HIPCHK(c, hipStreamWaitEvent(c->s_copy, c->ev_free[par], 0));
    return timed_copy(c, (char*)c->ring[par] + off, (const char*)c->host_layers[layer] + off, c->look_bytes);
}
int issue_rest(spec_ctx* c, int64_t j) {
    int par = (int)(j & 1);
    int layer = c->streamed[(size_t)(j % (int64_t)c->streamed.size())];
    size_t off = par ? 0 : c->look_bytes;
    if (j >= 1) HIPCHK(c, hipStreamWaitEvent(c->s_copy, c->ev_free[par ^ 1], 0));
    if (c->blob_bytes > c->look_bytes) {
        int rc = timed_copy(c, (char*)c->ring[par] + off, (const char*)c->host_layers[layer] + off,
                            c->blob_bytes - c->look_bytes);
        if (rc) return rc;
    }
    HIPCHK(c, hipEventRecord(c->ev_ready[par], c->s_copy));
    c->layers_streamed += 1;
    return SPEC_OK;
}

int prefetch(spec_ctx* c) {
    if (c->ring.empty()) return SPEC_OK;
    if (c->cfg.flags & SPEC_FLAG_NO_OVERLAP) return SPEC_OK;
    if (c->compact) {
        // host order: a wait on ev_free[s] must be enqueued after the release that records it.
        // rest(j) needs use j-1 released (j <= uses_done); look(j) needs use j-2 released.
        while (c->copies_issued < c->uses_done + 1) {
            int rc;
            if (c->looks_issued <= c->copies_issued) {
                if ((rc = issue_look(c, c->looks_issued))) return rc;
                c->looks_issued++;
            }
            if ((rc = issue_rest(c, c->copies_issued))) return rc;
            c->copies_issued++;
        }
        while (c->looks_issued < c->uses_done + 2) {
            int rc = issue_look(c, c->looks_issued);
            if (rc) return rc;
            c->looks_issued++;
        }
        return SPEC_OK;
    }
    int ns = (int)c->ring.size();
    while (c->copies_issued < c->uses_done + ns) {
        int rc = issue_copy(c, c->copies_issued);
        if (rc) return rc;
        c->copies_issued++;
    }
    return SPEC_OK;
}

int acquire_layer(spec_ctx* c, int layer, const char** base) {
    if (c->resident[layer]) { *base = (const char*)c->resident[layer]; return SPEC_OK; }
    int ns = (int)c->ring.size();
    int64_t j = c->uses_done;
    int expect = c->streamed[(size_t)(j % (int64_t)c->streamed.size())];
    if (expect != layer)
        return fail(c, SPEC_ERR_STATE, "streamed layer %d used out of pass order (expected %d)", layer, expect);
    if (c->cfg.flags & SPEC_FLAG_NO_OVERLAP) {
        // serial mode: the copy starts only when compute has reached this layer
        hipEvent_t e = c->ev_free[(int)(j % ns)];
        HIPCHK(c, hipEventRecord(e, c->s_compute));
        if (c->copies_issued != j) return fail(c, SPEC_ERR_STATE, "streamer out of step");
        // issue_copy waits on ev_free[slot] for j >= ns; make the wait explicit for all j here
        HIPCHK(c, hipStreamWaitEvent(c->s_copy, e, 0));
        int rc;
        if (c->compact) {
            if ((rc = issue_look(c, j)) || (rc = issue_rest(c, j))) return rc;
            c->looks_issued = j + 1;
        } else if ((rc = issue_copy(c, j))) return rc;
        c->copies_issued++;
    } else {
        int rc = prefetch(c);
        if (rc) return rc;
    }
    int slot = (int)(j % ns);
    HIPCHK(c, hipStreamWaitEvent(c->s_compute, c->ev_ready[slot], 0));
    *base = (const char*)c->ring[slot];
    return SPEC_OK;
}

int release_layer(spec_ctx* c, int layer) {
    if (c->resident[layer]) return SPEC_OK;
    int ns = (int)c->ring.size();
    int slot = (int)(c->uses_done % ns);
    HIPCHK(c, hipEventRecord(c->ev_free[slot], c->s_compute));
    c->uses_done++;
    return prefetch(c);
}

// ---- one decoder layer on T rows ---------------------------------------------------------------
struct RowSet {
    float* x;                 // [T, d] residual stream
    const int32_t* row_pos;   // [T]
    const float2* cs;         // [T, dh/2]
    int T, n_new, B;
};

// `pending`: on entry, true if the previous layer left its MoE output uncombined in ws.y; on exit,
// true if this layer did.  With defer == false the combine is applied before returning.
int layer_body(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* Wb, Workspace& w,
               const RowSet& r, void* kv_layer, const KvGeom& geom, const int32_t* page_table,
               bool* pending, bool defer, hipStream_t st) {
    const int dt = s.dtype;
    const size_t es = esize(dt);
    const int d = s.d_model, T = r.T;
    const int hd = s.n_q_heads * s.head_dim;
    const int qkv_rows = (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
    auto W = [&](int64_t off) { return (const void*)(Wb + off * es); };

    { ProfScope ps(c, SPEC_PROF_NORM, st);
      HIPCHK(c, launch_combine_norm(r.x, *pending ? w.y : nullptr, w.r_wts, w.slots, W(L.g1), w.h, T, d,
                                    s.rms_eps, dt, st)); }
    *pending = false;
    GemmArgs g{};
    g.A = w.h; g.lda = d; g.W = W(L.wqkv); g.C = w.qkv; g.ldc = qkv_rows; g.M = T; g.N = qkv_rows; g.K = d;
    // bf16 MFMA path with 128-wide heads: rotation, q store and KV append happen in the projection's
    // epilogue (no f32 qkv round trip); otherwise projection to f32, then the rope/append kernel
    const bool fused_rope = dt == SPEC_BF16 && !(c->cfg.flags & SPEC_FLAG_SIMPLE_KERNELS) && s.head_dim == 128 &&
                            d % 64 == 0;
    if (fused_rope) {
        g.epilogue = EPI_ROPE_KV;
        g.C = w.q; g.ldc = qkv_rows;       // unused by the epilogue; kept valid for the launcher's checks
        g.rope.cs = r.cs; g.rope.row_pos = r.row_pos; g.rope.page_table = page_table; g.rope.q_out = w.q;
        g.rope.kv_layer = kv_layer; g.rope.geom = geom; g.rope.n_new = r.n_new; g.rope.n_q_heads = s.n_q_heads;
        { ProfScope ps(c, SPEC_PROF_QKV, st); HIPCHK(c, gemm(c, g, dt, st)); }
    } else {
        g.epilogue = EPI_STORE_F32;
        { ProfScope ps(c, SPEC_PROF_QKV, st); HIPCHK(c, gemm(c, g, dt, st)); }
        { ProfScope ps(c, SPEC_PROF_ROPE, st);
          HIPCHK(c, launch_rope_kv(w.qkv, r.cs, r.row_pos, page_table, w.q, kv_layer, geom, T, r.n_new,
                                   s.n_q_heads, dt, st)); }
    }
    AttnArgs a{};
    a.q = w.q; a.out = w.att; a.kv_layer = kv_layer; a.page_table = page_table; a.row_pos = r.row_pos;
    a.geom = geom; a.B = r.B; a.n_new = r.n_new; a.n_q_heads = s.n_q_heads;
    a.scale = 1.0f / sqrtf((float)s.head_dim);
    { ProfScope ps(c, SPEC_PROF_ATTN, st); HIPCHK(c, attention(c, a, dt, st)); }
    g = GemmArgs{};
    g.A = w.att; g.lda = hd; g.W = W(L.wo); g.C = r.x; g.ldc = d; g.M = T; g.N = d; g.K = hd;
    g.epilogue = EPI_ADD_F32;
    { ProfScope ps(c, SPEC_PROF_OPROJ, st); HIPCHK(c, gemm(c, g, dt, st)); }
    if (s.attn_only) return SPEC_OK;

    // post-attention norm; for MoE layers the router logits are taken in the same kernel while the
    // normalised row is still in registers (the plain-kernel mode keeps the two-kernel form)
    const bool fused_route = s.n_experts > 0 && !(c->cfg.flags & SPEC_FLAG_SIMPLE_KERNELS) &&
                             norm_route_supported(d, s.n_experts);
    { ProfScope ps(c, SPEC_PROF_NORM, st);
      if (fused_route)
          HIPCHK(c, launch_norm_route(r.x, W(L.g2), w.h, W(L.wr), w.r_ids, w.r_wts, T, d, s.n_experts, s.rms_eps, dt, st));
      else
          HIPCHK(c, launch_combine_norm(r.x, nullptr, nullptr, nullptr, W(L.g2), w.h, T, d, s.rms_eps, dt, st)); }
    if (s.n_experts > 0) {
        { ProfScope ps(c, SPEC_PROF_ROUTE, st);
          if (!fused_route) HIPCHK(c, launch_router(w.h, W(L.wr), w.r_ids, w.r_wts, T, d, s.n_experts, dt, st));
          HIPCHK(c, launch_moe_sort(w.r_ids, w.offsets, w.perm, w.slots, T, s.n_experts, st)); }
        g = GemmArgs{};
        g.A = w.h; g.lda = d; g.a_rows = w.perm; g.W = W(L.w1); g.W3 = W(L.w3); g.C = w.u; g.ldc = s.d_ff;
        g.M = 2 * T; g.N = s.d_ff; g.K = d; g.epilogue = EPI_SWIGLU_T;
        g.group_offsets = w.offsets; g.n_groups = s.n_experts; g.w_group_stride = L.expert_stride;
        g.m_upper = 2 * T;
        { ProfScope ps(c, SPEC_PROF_MOE1, st); HIPCHK(c, gemm(c, g, dt, st)); }
        g = GemmArgs{};
        g.A = w.u; g.lda = s.d_ff; g.W = W(L.w2); g.C = w.y; g.ldc = d; g.M = 2 * T; g.N = d; g.K = s.d_ff;
        g.epilogue = EPI_STORE_F32;
        g.group_offsets = w.offsets; g.n_groups = s.n_experts; g.w_group_stride = L.expert_stride;
        g.m_upper = 2 * T;
        { ProfScope ps(c, SPEC_PROF_MOE2, st); HIPCHK(c, gemm(c, g, dt, st)); }
        *pending = true;
        if (!defer) {
            ProfScope ps(c, SPEC_PROF_NORM, st);
            HIPCHK(c, launch_combine_norm(r.x, w.y, w.r_wts, w.slots, nullptr, nullptr, T, d, s.rms_eps, dt, st));
            *pending = false;
        }
    } else {
        g = GemmArgs{};
        g.A = w.h; g.lda = d; g.W = W(L.w1); g.W3 = W(L.w3); g.C = w.u; g.ldc = s.d_ff; g.M = T; g.N = s.d_ff;
        g.K = d; g.epilogue = EPI_SWIGLU_T;
        { ProfScope ps(c, SPEC_PROF_MOE1, st); HIPCHK(c, gemm(c, g, dt, st)); }
        g = GemmArgs{};
        g.A = w.u; g.lda = s.d_ff; g.W = W(L.w2); g.C = r.x; g.ldc = d; g.M = T; g.N = d; g.K = s.d_ff;
        g.epilogue = EPI_ADD_F32;
        { ProfScope ps(c, SPEC_PROF_MOE2, st); HIPCHK(c, gemm(c, g, dt, st)); }
    }
    return SPEC_OK;
}

inline void* kv_layer_ptr(void* pool, const KvGeom& g, int layer, size_t es) {
    return (char*)pool + (size_t)layer * (size_t)g.layer_elems() * es;
}

// target pass over rows already embedded in w.x (tok_in/row_pos/cs set); leaves normalised final
// state in w.h when want_head
int target_layers(spec_ctx* c, Sub& sb, Workspace& w, int T, int n_new, bool want_final_norm) {
    RowSet r{w.x, w.row_pos, w.cs, T, n_new, sb.B};
    bool pending = false;
    for (int l = 0; l < c->tgt.n_layers; ++l) {
        const char* Wb;
        int rc = acquire_layer(c, l, &Wb);
        if (rc) return rc;
        rc = layer_body(c, c->tgt, c->tl, Wb, w, r, kv_layer_ptr(sb.kv_t, c->gt, l, c->es), c->gt,
                        sb.page_table, &pending, true, c->s_compute);
        if (rc) return rc;
        if ((rc = release_layer(c, l))) return rc;
    }
    const char* G = (const char*)c->d_globals;
    if (want_final_norm || pending)
        HIPCHK(c, launch_combine_norm(w.x, pending ? w.y : nullptr, w.r_wts, w.slots,
                                      want_final_norm ? G + c->gl.gf * c->es : nullptr, w.h, T,
                                      c->tgt.d_model, c->tgt.rms_eps, c->tgt.dtype, c->s_compute));
    return SPEC_OK;
}

int draft_layers(spec_ctx* c, Sub& sb, Workspace& w, int T, int n_new, bool want_final_norm, hipStream_t st) {
    RowSet r{w.x, w.row_pos, w.cs, T, n_new, sb.B};
    bool pending = false;
    for (int l = 0; l < c->drf.n_layers; ++l) {
        int rc = layer_body(c, c->drf, c->dl, (const char*)c->d_draft_layers[l], w, r,
                            kv_layer_ptr(sb.kv_d, c->gd, l, c->es), c->gd, sb.page_table, &pending, true, st);
        if (rc) return rc;
    }
    const char* G = (const char*)c->d_draft_globals;
    if (want_final_norm || pending)
        HIPCHK(c, launch_combine_norm(w.x, pending ? w.y : nullptr, w.r_wts, w.slots,
                                      want_final_norm ? G + c->gl.gf * c->es : nullptr, w.h, T,
                                      c->drf.d_model, c->drf.rms_eps, c->drf.dtype, st));
    return SPEC_OK;
}

int check_sub(spec_ctx* c, int sub) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    if (sub < 0 || sub >= c->cfg.n_sub_batches) return fail(c, SPEC_ERR_ARG, "sub-batch %d out of range", sub);
    return SPEC_OK;
}

// look-ahead piece of the compact staging ring: an eighth of a layer, 256-byte aligned
int64_t look_ahead_bytes(int64_t blob) { return ((blob / 8) + 255) & ~(int64_t)255; }

// n_slots <= 0: compact ring (one layer + look-ahead piece); otherwise n_slots whole-layer slots
int64_t ring_bytes(int64_t blob, int n_slots) {
    return n_slots <= 0 ? blob + look_ahead_bytes(blob) : (int64_t)n_slots * blob;
}

int64_t plan_residency(const spec_model_shape& t, const spec_model_shape* d, int64_t budget, int n_slots,
                       int64_t* streamed_bytes, int64_t* fixed_bytes_out) {
    size_t es = esize(t.dtype);
    Layout tl = make_layout(t);
    GlobalLayout gl = make_global_layout(t);
    int64_t blob = tl.total * (int64_t)es;
    int64_t fixed = gl.total * (int64_t)es;
    if (d) fixed += (int64_t)d->n_layers * make_layout(*d).total * (int64_t)esize(d->dtype);
    if (fixed_bytes_out) *fixed_bytes_out = fixed;
    int64_t R;
    if (budget <= 0 || fixed + (int64_t)t.n_layers * blob <= budget) R = t.n_layers;
    else {
        int64_t avail = budget - fixed - ring_bytes(blob, n_slots);
        if (avail < 0) return -1;
        R = std::min<int64_t>(avail / blob, t.n_layers);
    }
    if (streamed_bytes) *streamed_bytes = (t.n_layers - R) * blob;
    return R;
}

}  // namespace

// =================================================================================================
// C ABI
// =================================================================================================
extern "C" {

const char* spec_last_error(const spec_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

int64_t spec_layer_blob_elems(const spec_model_shape* s) {
    if (!shape_ok(s)) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported model shape");
    return make_layout(*s).total;
}
int64_t spec_global_blob_elems(const spec_model_shape* s) {
    if (!shape_ok(s)) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported model shape");
    return make_global_layout(*s).total;
}
int64_t spec_plan_residency(const spec_model_shape* target, const spec_model_shape* draft, int64_t budget,
                            int32_t n_ring_slots, int64_t* streamed_bytes_per_pass) {
    if (!shape_ok(target) || (draft && !shape_ok(draft))) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported model shape");
    int64_t R = plan_residency(*target, draft, budget, n_ring_slots, streamed_bytes_per_pass, nullptr);
    if (R < 0) return fail(nullptr, SPEC_ERR_BUDGET, "budget cannot hold globals + draft + the staging ring (n_ring_slots %d)", n_ring_slots);
    return R;
}

int spec_host_alloc(size_t bytes, void** out_host) {
    if (!out_host || bytes == 0) return fail(nullptr, SPEC_ERR_ARG, "spec_host_alloc: bad arguments");
    HIPCHK(nullptr, hipHostMalloc(out_host, bytes, hipHostMallocDefault));
    return SPEC_OK;
}
int spec_host_free(void* host) {
    if (!host) return SPEC_OK;
    HIPCHK(nullptr, hipHostFree(host));
    return SPEC_OK;
}

void spec_destroy(spec_ctx* c) {
    if (!c) return;
    hipDeviceSynchronize();
    for (auto& p : c->copy_timers) { hipEventDestroy(p.first); hipEventDestroy(p.second); }
    for (auto e : c->timer_pool) hipEventDestroy(e);
    for (auto e : c->ev_ready) hipEventDestroy(e);
    for (auto e : c->ev_free) hipEventDestroy(e);
    for (int s = 0; s < 2; ++s) {
        if (c->sub[s].ev_drafted) hipEventDestroy(c->sub[s].ev_drafted);
        if (c->sub[s].ev_committed) hipEventDestroy(c->sub[s].ev_committed);
    }
    for (void* p : c->allocs) hipFree(p);
    if (c->own_compute) hipStreamDestroy(c->s_compute);
    if (c->own_copy) hipStreamDestroy(c->s_copy);
    if (c->own_draft) hipStreamDestroy(c->s_draft);
    delete c;
}

static int init_impl(spec_ctx* c, const spec_host_weights* tw, const spec_host_weights* dw) {
    const spec_model_shape& t = c->tgt;
    const spec_runtime_cfg& cfg = c->cfg;
    c->es = esize(t.dtype);
    c->tl = make_layout(t);
    c->gl = make_global_layout(t);
    c->blob_bytes = (size_t)c->tl.total * c->es;
    if (c->has_draft) c->dl = make_layout(c->drf);

    auto mk_stream = [&](void* given, hipStream_t* s, bool* own) -> int {
        if (given) { *s = (hipStream_t)given; *own = false; return SPEC_OK; }
        HIPCHK(c, hipStreamCreateWithFlags(s, hipStreamNonBlocking));
        *own = true;
        return SPEC_OK;
    };
    int rc;
    if ((rc = mk_stream(cfg.compute_stream, &c->s_compute, &c->own_compute))) return rc;
    if ((rc = mk_stream(cfg.copy_stream, &c->s_copy, &c->own_copy))) return rc;
    if ((rc = mk_stream(cfg.draft_stream, &c->s_draft, &c->own_draft))) return rc;

    // residency plan under the HBM weight budget
    int n_slots = cfg.n_ring_slots;
    int64_t fixed = 0, streamed_bytes = 0;
    int64_t R = plan_residency(t, c->has_draft ? &c->drf : nullptr, cfg.hbm_weight_budget_bytes, n_slots,
                               &streamed_bytes, &fixed);
    if (R < 0)
        return fail(c, SPEC_ERR_BUDGET, "HBM weight budget %lld B cannot hold globals+draft (%lld B) and %d staging slots of %zu B",
                    (long long)cfg.hbm_weight_budget_bytes, (long long)fixed, n_slots, c->blob_bytes);
    c->host_layers.assign(tw->layer_blobs, tw->layer_blobs + t.n_layers);
    c->resident.assign(t.n_layers, nullptr);
    for (int l = 0; l < t.n_layers; ++l) {
        if (!c->host_layers[l]) return fail(c, SPEC_ERR_ARG, "target layer blob %d is NULL", l);
        if (l < R) {
            char* p;
            if ((rc = dev_alloc(c, &p, c->blob_bytes))) return rc;
            HIPCHK(c, hipMemcpy(p, c->host_layers[l], c->blob_bytes, hipMemcpyHostToDevice));
            c->resident[l] = p;
        } else c->streamed.push_back(l);
    }
    c->hbm_weight_bytes = fixed + R * (int64_t)c->blob_bytes;
    if (!c->streamed.empty()) {
        c->compact = n_slots <= 0;
        const int ns = c->compact ? 2 : n_slots;
        c->ring.resize(ns);
        c->ev_ready.resize(ns);
        c->ev_free.resize(ns);
        if (c->compact) {
            // the look-ahead piece takes whatever the budget leaves after the resident layers (at least
            // an eighth of a layer, at most a whole one: then the two slots no longer overlap)
            int64_t left = cfg.hbm_weight_budget_bytes - fixed - (R + 1) * (int64_t)c->blob_bytes;
            left = std::min<int64_t>(left, (int64_t)c->blob_bytes) & ~(int64_t)255;
            c->look_bytes = (size_t)std::max<int64_t>(left, look_ahead_bytes((int64_t)c->blob_bytes));
            char* p;
            if ((rc = dev_alloc(c, &p, c->blob_bytes + c->look_bytes))) return rc;
            c->ring[0] = p;
            c->ring[1] = p + c->look_bytes;
        }
        for (int i = 0; i < ns; ++i) {
            if (!c->compact) {
                char* p;
                if ((rc = dev_alloc(c, &p, c->blob_bytes))) return rc;
                c->ring[i] = p;
            }
            HIPCHK(c, hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming));
            HIPCHK(c, hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
        }
        c->hbm_weight_bytes += c->compact ? (int64_t)(c->blob_bytes + c->look_bytes)
                                          : ring_bytes((int64_t)c->blob_bytes, n_slots);
    }
    {
        char* p;
        size_t gb = (size_t)c->gl.total * c->es;
        if ((rc = dev_alloc(c, &p, gb))) return rc;
        HIPCHK(c, hipMemcpy(p, tw->global_blob, gb, hipMemcpyHostToDevice));
        c->d_globals = p;
    }
    if (c->has_draft) {
        size_t lb = (size_t)c->dl.total * c->es;
        for (int l = 0; l < c->drf.n_layers; ++l) {
            if (!dw->layer_blobs[l]) return fail(c, SPEC_ERR_ARG, "draft layer blob %d is NULL", l);
            char* p;
            if ((rc = dev_alloc(c, &p, lb))) return rc;
            HIPCHK(c, hipMemcpy(p, dw->layer_blobs[l], lb, hipMemcpyHostToDevice));
            c->d_draft_layers.push_back(p);
        }
        if (dw->global_blob == tw->global_blob) { c->d_draft_globals = c->d_globals; c->draft_globals_shared = true; }
        else {
            char* p;
            size_t gb = (size_t)c->gl.total * c->es;
            if ((rc = dev_alloc(c, &p, gb))) return rc;
            HIPCHK(c, hipMemcpy(p, dw->global_blob, gb, hipMemcpyHostToDevice));
            c->d_draft_globals = p;
            c->hbm_weight_bytes += (int64_t)gb;
        }
    }

    // KV pools, sequence state, buffers
    int pt = cfg.page_tokens;
    int cap_tokens = cfg.ctx_max + cfg.k_max + 2;
    int pps = (cap_tokens + pt - 1) / pt;
    c->gt = KvGeom{t.n_kv_heads, t.head_dim, pt, pps, (int64_t)cfg.batch_max * pps};
    if (c->has_draft) c->gd = KvGeom{c->drf.n_kv_heads, c->drf.head_dim, pt, pps, (int64_t)cfg.batch_max * pps};
    int Bm = cfg.batch_max, km = cfg.k_max, V = t.vocab;
    for (int s = 0; s < cfg.n_sub_batches; ++s) {
        Sub& sb = c->sub[s];
        sb.st.tok_cap = cap_tokens;
        if ((rc = dev_alloc(c, &sb.st.tokens, (size_t)Bm * cap_tokens * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.st.len, (size_t)Bm * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.st.n_new, (size_t)Bm * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.st.max_new, (size_t)Bm * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.page_table, (size_t)Bm * pps * 4))) return rc;
        std::vector<int32_t> tab((size_t)Bm * pps);
        for (int b = 0; b < Bm; ++b)
            for (int p = 0; p < pps; ++p) tab[(size_t)b * pps + p] = p * Bm + b;   // pages of a sequence are scattered
        HIPCHK(c, hipMemcpy(sb.page_table, tab.data(), tab.size() * 4, hipMemcpyHostToDevice));
        // pools start zeroed: slots of a page beyond a sequence's length are read (and masked) by the
        // attention kernel, so they must hold finite numbers
        size_t kvt_bytes = (size_t)t.n_layers * (size_t)c->gt.layer_elems() * c->es;
        if ((rc = dev_alloc(c, (char**)&sb.kv_t, kvt_bytes))) return rc;
        HIPCHK(c, hipMemset(sb.kv_t, 0, kvt_bytes));
        if (c->has_draft) {
            size_t kvd_bytes = (size_t)c->drf.n_layers * (size_t)c->gd.layer_elems() * c->es;
            if ((rc = dev_alloc(c, (char**)&sb.kv_d, kvd_bytes))) return rc;
            HIPCHK(c, hipMemset(sb.kv_d, 0, kvd_bytes));
        }
        if ((rc = dev_alloc(c, &sb.draft_tokens, (size_t)Bm * std::max(1, km) * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.logits, (size_t)Bm * (km + 1) * V * 4))) return rc;
        if (c->has_draft) {
            if (cfg.mode == SPEC_SAMPLE) { if ((rc = dev_alloc(c, &sb.q_logits, (size_t)Bm * std::max(1, km) * V * 4))) return rc; }
            else if ((rc = dev_alloc(c, &sb.draft_logits, (size_t)Bm * V * 4))) return rc;
        }
        if ((rc = dev_alloc(c, &sb.n_acc, (size_t)Bm * 4))) return rc;
        if ((rc = dev_alloc(c, &sb.next_tok, (size_t)Bm * 4))) return rc;
        HIPCHK(c, hipEventCreateWithFlags(&sb.ev_drafted, hipEventDisableTiming));
        HIPCHK(c, hipEventCreateWithFlags(&sb.ev_committed, hipEventDisableTiming));
        sb.seq_base = (uint32_t)(s * Bm);
    }
    int chunk = cfg.prefill_chunk;
    int t_max = Bm * std::max(km + 1, chunk);
    if ((rc = alloc_workspace(c, c->wv, t, t_max))) return rc;
    if (c->has_draft && (rc = alloc_workspace(c, c->wd, c->drf, Bm * std::max(2, chunk)))) return rc;
    if ((rc = dev_alloc(c, &c->d_hist, 18 * 8))) return rc;
    HIPCHK(c, hipMemset(c->d_hist, 0, 18 * 8));
    HIPCHK(c, hipDeviceSynchronize());
    return SPEC_OK;
}

int spec_init(const spec_model_shape* target, const spec_model_shape* draft, const spec_host_weights* target_w,
              const spec_host_weights* draft_w, const spec_runtime_cfg* cfg_in, spec_ctx** out) {
    if (!target || !target_w || !cfg_in || !out) return fail(nullptr, SPEC_ERR_ARG, "spec_init: NULL argument");
    *out = nullptr;
    if (!shape_ok(target) || target->attn_only) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported target shape");
    if (!target_w->layer_blobs || !target_w->global_blob) return fail(nullptr, SPEC_ERR_ARG, "target weights missing");
    bool has_draft = draft != nullptr;
    if (has_draft) {
        if (!draft_w || !draft_w->layer_blobs || !draft_w->global_blob) return fail(nullptr, SPEC_ERR_ARG, "draft weights missing");
        if (!shape_ok(draft)) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported draft shape");
        if (draft->vocab != target->vocab || draft->d_model != target->d_model || draft->dtype != target->dtype ||
            draft->head_dim != target->head_dim)
            return fail(nullptr, SPEC_ERR_SHAPE, "draft must share vocab, width, head size and dtype with the target");
    }
    spec_runtime_cfg cfg = *cfg_in;
    if (cfg.n_sub_batches != 1 && cfg.n_sub_batches != 2) return fail(nullptr, SPEC_ERR_ARG, "n_sub_batches must be 1 or 2");
    if (cfg.batch_max <= 0 || cfg.k_max < 0 || cfg.k_max > 16 || cfg.ctx_max <= 0)
        return fail(nullptr, SPEC_ERR_ARG, "batch_max/k_max/ctx_max out of range");
    if (cfg.page_tokens == 0) cfg.page_tokens = 64;
    if (cfg.page_tokens < 16 || cfg.page_tokens % 16) return fail(nullptr, SPEC_ERR_ARG, "page_tokens must be a multiple of 16");
    if (cfg.n_ring_slots < 0 || cfg.n_ring_slots > 8) return fail(nullptr, SPEC_ERR_ARG, "n_ring_slots must be 0..8");
    if (cfg.mode != SPEC_GREEDY && cfg.mode != SPEC_SAMPLE) return fail(nullptr, SPEC_ERR_ARG, "bad mode");
    if (cfg.mode == SPEC_SAMPLE && !(cfg.temperature > 0.f)) return fail(nullptr, SPEC_ERR_ARG, "temperature must be > 0");
    if (cfg.prefill_chunk == 0) {
        int g = target->n_q_heads / target->n_kv_heads;
        cfg.prefill_chunk = std::max(1, std::min(16, 64 / g));
    }
    if (cfg.prefill_chunk < 1 || cfg.prefill_chunk > 64) return fail(nullptr, SPEC_ERR_ARG, "prefill_chunk must be 1..64");
    spec_ctx* c = new spec_ctx();
    c->tgt = *target;
    c->has_draft = has_draft;
    if (has_draft) c->drf = *draft;
    c->cfg = cfg;
    int rc = init_impl(c, target_w, draft_w);
    if (rc) { g_err = c->err; spec_destroy(c); return rc; }
    *out = c;
    return SPEC_OK;
}

int spec_reset(spec_ctx* c, int sub) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    HIPCHK(c, hipDeviceSynchronize());
    Sub& sb = c->sub[sub];
    sb.ready = false; sb.drafted = false; sb.B = 0; sb.round = 0; sb.last_k = sb.last_draft_k = 0;
    c->primed = false; c->cur = 0;
    return SPEC_OK;
}

static int load_sequences(spec_ctx* c, Sub& sb, const int32_t* tokens, const int32_t* cu, int B, int max_new) {
    int cap = sb.st.tok_cap;
    std::vector<int32_t> buf((size_t)B * cap, 0), len(B), zero(B, 0), mx(B, max_new);
    for (int b = 0; b < B; ++b) {
        int n = cu[b + 1] - cu[b];
        if (n < 1) return fail(c, SPEC_ERR_ARG, "prompt %d is empty", b);
        if (n + max_new > c->cfg.ctx_max) return fail(c, SPEC_ERR_CAPACITY, "prompt %d: %d + %d new tokens exceed ctx_max %d", b, n, max_new, c->cfg.ctx_max);
        for (int i = 0; i < n; ++i) {
            int tk = tokens[cu[b] + i];
            if (tk < 0 || tk >= c->tgt.vocab) return fail(c, SPEC_ERR_ARG, "prompt %d token %d out of vocabulary", b, i);
            buf[(size_t)b * cap + i] = tk;
        }
        len[b] = n;
    }
    HIPCHK(c, hipMemcpy(sb.st.tokens, buf.data(), buf.size() * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(sb.st.len, len.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(sb.st.n_new, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(sb.st.max_new, mx.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    sb.B = B;
    return SPEC_OK;
}

int spec_prefill(spec_ctx* c, int sub, const int32_t* tokens, const int32_t* cu_lens, int B, int max_new) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (!tokens || !cu_lens || B <= 0 || max_new < 0) return fail(c, SPEC_ERR_ARG, "spec_prefill: bad arguments");
    if (B > c->cfg.batch_max) return fail(c, SPEC_ERR_CAPACITY, "B %d > batch_max %d", B, c->cfg.batch_max);
    HIPCHK(c, hipDeviceSynchronize());
    Sub& sb = c->sub[sub];
    if ((rc = load_sequences(c, sb, tokens, cu_lens, B, max_new))) return rc;
    int pmax = 0;
    for (int b = 0; b < B; ++b) pmax = std::max(pmax, cu_lens[b + 1] - cu_lens[b] - 1);
    const int Q = c->cfg.prefill_chunk;
    const int n_chunks = (pmax + Q - 1) / Q;
    const int T = B * Q;
    if (n_chunks > 0) {
        const int d = c->tgt.d_model, half = c->tgt.head_dim / 2;
        float* xall = nullptr; int32_t* pos_all = nullptr; float2* cs_all = nullptr;
        hipStream_t st = c->s_compute;
        HIPCHK(c, hipMalloc(&xall, (size_t)n_chunks * T * d * 4));
        hipError_t e1 = hipMalloc(&pos_all, (size_t)n_chunks * T * 4);
        hipError_t e2 = hipMalloc(&cs_all, (size_t)n_chunks * T * half * sizeof(float2));
        auto cleanup = [&]() { hipFree(xall); hipFree(pos_all); hipFree(cs_all); };
        if (e1 != hipSuccess || e2 != hipSuccess) { cleanup(); return fail(c, SPEC_ERR_HIP, "prefill scratch allocation failed"); }
        auto run_model = [&](bool is_draft) -> int {
            const spec_model_shape& s = is_draft ? c->drf : c->tgt;
            Workspace& w = is_draft ? c->wd : c->wv;
            const char* G = (const char*)(is_draft ? c->d_draft_globals : c->d_globals);
            int hf = s.head_dim / 2;
            for (int ch = 0; ch < n_chunks; ++ch) {
                int32_t* rp = pos_all + (size_t)ch * T;
                HIPCHK(c, launch_prefill_prep(sb.st.tokens, sb.st.len, sb.st.tok_cap, B, ch * Q, Q, w.tok_in, rp, st));
                HIPCHK(c, launch_embed(G + c->gl.emb * c->es, w.tok_in, xall + (size_t)ch * T * d, T, d, s.vocab, s.dtype, st));
                HIPCHK(c, launch_rope_table(rp, cs_all + (size_t)ch * T * hf, T, hf, s.rope_theta, st));
            }
            for (int l = 0; l < s.n_layers; ++l) {
                const char* Wb;
                if (is_draft) Wb = (const char*)c->d_draft_layers[l];
                else { int r2 = acquire_layer(c, l, &Wb); if (r2) return r2; }
                for (int ch = 0; ch < n_chunks; ++ch) {
                    RowSet r{xall + (size_t)ch * T * d, pos_all + (size_t)ch * T, cs_all + (size_t)ch * T * hf, T, Q, B};
                    bool pending = false;
                    int r2 = layer_body(c, s, is_draft ? c->dl : c->tl, Wb, w, r,
                                        kv_layer_ptr(is_draft ? sb.kv_d : sb.kv_t, is_draft ? c->gd : c->gt, l, c->es),
                                        is_draft ? c->gd : c->gt, sb.page_table, &pending, false, st);
                    if (r2) return r2;
                }
                if (!is_draft) { int r2 = release_layer(c, l); if (r2) return r2; }
            }
            return SPEC_OK;
        };
        rc = run_model(false);
        if (!rc && c->has_draft) rc = run_model(true);
        hipError_t es_ = hipStreamSynchronize(st);
        cleanup();
        if (rc) return rc;
        if (es_ != hipSuccess) return fail(c, SPEC_ERR_HIP, "prefill failed: %s", hipGetErrorString(es_));
    }
    sb.ready = true; sb.drafted = false; sb.round = 0;
    return SPEC_OK;
}

int spec_kv_import(spec_ctx* c, int sub, int layer, const void* k_ctx, const void* v_ctx, int B, int ctx_len) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (((!k_ctx || !v_ctx) && ctx_len > 0) || B <= 0 || B > c->cfg.batch_max || layer < 0 ||
        layer >= c->tgt.n_layers || ctx_len < 0)
        return fail(c, SPEC_ERR_ARG, "spec_kv_import: bad arguments");
    if (ctx_len + 1 > c->cfg.ctx_max) return fail(c, SPEC_ERR_CAPACITY, "ctx_len %d + 1 > ctx_max %d", ctx_len, c->cfg.ctx_max);
    Sub& sb = c->sub[sub];
    HIPCHK(c, hipDeviceSynchronize());
    HIPCHK(c, launch_kv_import(k_ctx, v_ctx, kv_layer_ptr(sb.kv_t, c->gt, layer, c->es), sb.page_table, c->gt, B, ctx_len,
                               c->tgt.dtype, c->s_compute));
    std::vector<int32_t> len(B, ctx_len + 1), zero(B, 0), big(B, 1 << 30);
    HIPCHK(c, hipMemcpy(sb.st.len, len.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(sb.st.n_new, zero.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(sb.st.max_new, big.data(), (size_t)B * 4, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemset(sb.st.tokens, 0, (size_t)c->cfg.batch_max * sb.st.tok_cap * 4));
    HIPCHK(c, hipDeviceSynchronize());
    sb.B = B; sb.ready = true;
    return SPEC_OK;
}

int spec_draft(spec_ctx* c, int sub, int k, int32_t* out_tokens) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (!c->has_draft) return fail(c, SPEC_ERR_STATE, "context has no draft model");
    Sub& sb = c->sub[sub];
    if (!sb.ready) return fail(c, SPEC_ERR_STATE, "spec_draft before spec_prefill");
    if (k < 1 || k > c->cfg.k_max) return fail(c, SPEC_ERR_CAPACITY, "k %d outside 1..k_max %d", k, c->cfg.k_max);
    hipStream_t st = c->s_draft;
    Workspace& w = c->wd;
    const spec_model_shape& s = c->drf;
    const char* G = (const char*)c->d_draft_globals;
    const int B = sb.B, d = s.d_model, V = s.vocab, half = s.head_dim / 2;
    const bool sample = c->cfg.mode == SPEC_SAMPLE;
    HIPCHK(c, hipStreamWaitEvent(st, sb.ev_committed, 0));
    uint32_t saved_mask = c->prof_mask;
    ProfScope ps_draft(c, SPEC_PROF_DRAFT, st);
    c->prof_mask &= (1u << SPEC_PROF_DRAFT);        // the draft pass is timed as one class
    for (int step = 1; step <= k; ++step) {
        int n_new = step == 1 ? 2 : 1, T = B * n_new;
        HIPCHK(c, launch_draft_prep(sb.st, sb.draft_tokens, k, step, w.tok_in, w.row_pos, B, st));
        HIPCHK(c, launch_embed(G + c->gl.emb * c->es, w.tok_in, w.x, T, d, V, s.dtype, st));
        HIPCHK(c, launch_rope_table(w.row_pos, w.cs, T, half, s.rope_theta, st));
        if ((rc = draft_layers(c, sb, w, T, n_new, true, st))) return rc;
        GemmArgs g{};
        g.A = (const char*)w.h + (size_t)(n_new - 1) * d * c->es; g.lda = (int64_t)n_new * d;
        g.W = G + c->gl.head * c->es; g.M = B; g.N = V; g.K = d; g.epilogue = EPI_STORE_F32;
        float* z; int64_t ld;
        if (sample) { z = sb.q_logits + (size_t)(step - 1) * V; ld = (int64_t)k * V; }
        else { z = sb.draft_logits; ld = V; }
        g.C = z; g.ldc = ld;
        HIPCHK(c, gemm(c, g, s.dtype, st));
        HIPCHK(c, launch_draft_pick(z, ld, V, B, c->cfg.mode, 1.0f / (sample ? c->cfg.temperature : 1.0f),
                                    c->cfg.seed, sb.round, sb.seq_base, step, sb.draft_tokens, k, st));
    }
    c->prof_mask = saved_mask;
    if (out_tokens) HIPCHK(c, hipMemcpyAsync(out_tokens, sb.draft_tokens, (size_t)B * k * 4, hipMemcpyDeviceToDevice, st));
    HIPCHK(c, hipEventRecord(sb.ev_drafted, st));
    sb.drafted = true; sb.last_draft_k = k;
    return SPEC_OK;
}

int spec_verify(spec_ctx* c, int sub, const int32_t* draft_tokens, int k, int32_t* n_accepted, int32_t* next_token) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!sb.ready) return fail(c, SPEC_ERR_STATE, "spec_verify before spec_prefill");
    if (k < 0 || k > c->cfg.k_max) return fail(c, SPEC_ERR_CAPACITY, "k %d outside 0..k_max %d", k, c->cfg.k_max);
    const bool sample = c->cfg.mode == SPEC_SAMPLE;
    hipStream_t st = c->s_compute;
    if (draft_tokens) {
        if (sample) return fail(c, SPEC_ERR_ARG, "caller-supplied candidates need draft probabilities: greedy mode only");
        if (k > 0) HIPCHK(c, hipMemcpyAsync(sb.draft_tokens, draft_tokens, (size_t)sb.B * k * 4, hipMemcpyDeviceToDevice, st));
    } else if (k > 0) {
        if (!sb.drafted || sb.last_draft_k != k) return fail(c, SPEC_ERR_STATE, "no candidates from spec_draft(k=%d) for this sub-batch", k);
        HIPCHK(c, hipStreamWaitEvent(st, sb.ev_drafted, 0));
    }
    if (sample && k == 0) return fail(c, SPEC_ERR_ARG, "sampling mode needs k >= 1");
    Workspace& w = c->wv;
    const spec_model_shape& s = c->tgt;
    const char* G = (const char*)c->d_globals;
    const int B = sb.B, d = s.d_model, V = s.vocab, T = B * (k + 1);
    HIPCHK(c, launch_verify_prep(sb.st, sb.draft_tokens, k, w.tok_in, w.row_pos, B, st));
    HIPCHK(c, launch_embed(G + c->gl.emb * c->es, w.tok_in, w.x, T, d, V, s.dtype, st));
    HIPCHK(c, launch_rope_table(w.row_pos, w.cs, T, s.head_dim / 2, s.rope_theta, st));
    if ((rc = target_layers(c, sb, w, T, k + 1, true))) return rc;
    GemmArgs g{};
    g.A = w.h; g.lda = d; g.W = G + c->gl.head * c->es; g.C = sb.logits; g.ldc = V; g.M = T; g.N = V; g.K = d;
    g.epilogue = EPI_STORE_F32;
    { ProfScope ps(c, SPEC_PROF_HEAD, st); HIPCHK(c, gemm(c, g, s.dtype, st)); }
    AcceptArgs a{};
    a.p_logits = sb.logits; a.q_logits = sample ? sb.q_logits : nullptr; a.draft_tokens = sb.draft_tokens;
    a.inv_tau = 1.0f / (sample ? c->cfg.temperature : 1.0f);
    a.seed = c->cfg.seed; a.round = sb.round; a.seq_base = sb.seq_base;
    a.B = B; a.k = k; a.V = V; a.n_accepted = sb.n_acc; a.next_token = sb.next_tok;
    { ProfScope ps(c, SPEC_PROF_ACCEPT, st); HIPCHK(c, launch_accept(a, st)); }
    HIPCHK(c, launch_commit(sb.st, sb.draft_tokens, k, sb.n_acc, sb.next_tok, c->d_hist, c->d_hist + 17, B, st));
    if (n_accepted) HIPCHK(c, hipMemcpyAsync(n_accepted, sb.n_acc, (size_t)B * 4, hipMemcpyDeviceToDevice, st));
    if (next_token) HIPCHK(c, hipMemcpyAsync(next_token, sb.next_tok, (size_t)B * 4, hipMemcpyDeviceToDevice, st));
    HIPCHK(c, hipEventRecord(sb.ev_committed, st));
    sb.round++; sb.last_k = k; sb.drafted = false;
    c->rounds++;
    return SPEC_OK;
}

int spec_sync(spec_ctx* c, int sub) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    (void)sub;
    HIPCHK(c, hipStreamSynchronize(c->s_draft));
    HIPCHK(c, hipStreamSynchronize(c->s_compute));
    if (sub < 0) HIPCHK(c, hipStreamSynchronize(c->s_copy));
    return SPEC_OK;
}

int spec_step(spec_ctx* c, int k) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    int rc;
    if (k == 0) {       // plain decoding (no candidates): one verify pass per sub-batch in turn
        int cur = c->cfg.n_sub_batches == 1 ? 0 : c->cur;
        if ((rc = spec_verify(c, cur, nullptr, 0, nullptr, nullptr))) return rc;
        if (c->cfg.n_sub_batches == 2) c->cur = 1 - cur;
        return SPEC_OK;
    }
    if (c->cfg.n_sub_batches == 1) {
        if ((rc = spec_draft(c, 0, k, nullptr))) return rc;
        return spec_verify(c, 0, nullptr, k, nullptr, nullptr);
    }
    int cur = c->cur, other = 1 - cur;
    if (!c->primed) { if ((rc = spec_draft(c, cur, k, nullptr))) return rc; c->primed = true; }
    // the draft stream works on `other` while the compute/copy streams verify `cur`
    if ((rc = spec_draft(c, other, k, nullptr))) return rc;
    if ((rc = spec_verify(c, cur, nullptr, k, nullptr, nullptr))) return rc;
    c->cur = other;
    return SPEC_OK;
}

int spec_get_lengths(spec_ctx* c, int sub, int32_t* out_host) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (!out_host) return fail(c, SPEC_ERR_ARG, "out is NULL");
    if ((rc = spec_sync(c, sub))) return rc;
    HIPCHK(c, hipMemcpy(out_host, c->sub[sub].st.len, (size_t)c->sub[sub].B * 4, hipMemcpyDeviceToHost));
    return SPEC_OK;
}

int spec_get_tokens(spec_ctx* c, int sub, int seq, int32_t* out_host, int cap, int* out_len) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!out_host || seq < 0 || seq >= sb.B || cap < 0) return fail(c, SPEC_ERR_ARG, "spec_get_tokens: bad arguments");
    if ((rc = spec_sync(c, sub))) return rc;
    int32_t len = 0;
    HIPCHK(c, hipMemcpy(&len, sb.st.len + seq, 4, hipMemcpyDeviceToHost));
    int n = std::min(len, cap);
    if (n > 0) HIPCHK(c, hipMemcpy(out_host, sb.st.tokens + (size_t)seq * sb.st.tok_cap, (size_t)n * 4, hipMemcpyDeviceToHost));
    if (out_len) *out_len = len;
    return SPEC_OK;
}

int spec_get_stats(spec_ctx* c, spec_stats* out) {
    if (!c || !out) return fail(c, SPEC_ERR_ARG, "spec_get_stats: NULL argument");
    HIPCHK(c, hipDeviceSynchronize());
    int rc = harvest_timers(c, true);
    if (rc) return rc;
    int64_t h[18];
    HIPCHK(c, hipMemcpy(h, c->d_hist, sizeof h, hipMemcpyDeviceToHost));
    memset(out, 0, sizeof *out);
    out->bytes_streamed = c->bytes_streamed;
    out->layers_streamed = c->layers_streamed;
    out->resident_layers = (int64_t)c->tgt.n_layers - (int64_t)c->streamed.size();
    out->hbm_weight_bytes = c->hbm_weight_bytes;
    out->rounds = c->rounds;
    out->committed_tokens = h[17];
    for (int i = 0; i < 17; ++i) out->accept_hist[i] = h[i];
    out->copy_busy_ms = c->copy_busy_ms;
    return SPEC_OK;
}

int spec_reset_stats(spec_ctx* c) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    HIPCHK(c, hipDeviceSynchronize());
    int rc = harvest_timers(c, true);
    if (rc) return rc;
    HIPCHK(c, hipMemset(c->d_hist, 0, 18 * 8));
    HIPCHK(c, hipDeviceSynchronize());
    c->bytes_streamed = 0; c->layers_streamed = 0; c->rounds = 0; c->copy_busy_ms = 0.0;
    return SPEC_OK;
}

int spec_profile_enable(spec_ctx* c, uint32_t category_mask) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    c->prof_mask = category_mask & ((1u << SPEC_PROF_N) - 1u);
    return SPEC_OK;
}

int spec_profile_read(spec_ctx* c, double* ms_out, int64_t* launches_out, int reset) {
    if (!c || !ms_out || !launches_out) return fail(c, SPEC_ERR_ARG, "spec_profile_read: NULL argument");
    HIPCHK(c, hipDeviceSynchronize());
    for (auto& p : c->prof_pending) {
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, p.e0, p.e1));
        c->prof_ms[p.cat] += ms;
        c->prof_n[p.cat] += 1;
        c->timer_pool.push_back(p.e0);
        c->timer_pool.push_back(p.e1);
    }
    c->prof_pending.clear();
    for (int i = 0; i < SPEC_PROF_N; ++i) { ms_out[i] = c->prof_ms[i]; launches_out[i] = c->prof_n[i]; }
    if (reset) for (int i = 0; i < SPEC_PROF_N; ++i) { c->prof_ms[i] = 0.0; c->prof_n[i] = 0; }
    return SPEC_OK;
}

int spec_debug_logits(spec_ctx* c, int sub, float* out_dev) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!out_dev) return fail(c, SPEC_ERR_ARG, "out is NULL");
    if ((rc = spec_sync(c, sub))) return rc;
    HIPCHK(c, hipMemcpy(out_dev, sb.logits, (size_t)sb.B * (sb.last_k + 1) * c->tgt.vocab * 4, hipMemcpyDeviceToDevice));
    return SPEC_OK;
}

int spec_debug_draft_logits(spec_ctx* c, int sub, float* out_dev) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!out_dev || !sb.q_logits) return fail(c, SPEC_ERR_ARG, "draft logits are kept in sampling mode only");
    if ((rc = spec_sync(c, sub))) return rc;
    HIPCHK(c, hipMemcpy(out_dev, sb.q_logits, (size_t)sb.B * sb.last_draft_k * c->tgt.vocab * 4, hipMemcpyDeviceToDevice));
    return SPEC_OK;
}

int spec_debug_routing(spec_ctx* c, int sub, int32_t* ids_dev, float* weights_dev, int T) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (T < 0 || T > c->wv.t_max || !c->wv.r_ids) return fail(c, SPEC_ERR_ARG, "spec_debug_routing: bad arguments");
    if ((rc = spec_sync(c, sub))) return rc;
    if (ids_dev) HIPCHK(c, hipMemcpy(ids_dev, c->wv.r_ids, (size_t)T * 8, hipMemcpyDeviceToDevice));
    if (weights_dev) HIPCHK(c, hipMemcpy(weights_dev, c->wv.r_wts, (size_t)T * 8, hipMemcpyDeviceToDevice));
    return SPEC_OK;
}

int spec_layer_forward(spec_ctx* c, int sub, int layer, const void* x_in, int n_new, float* x_out) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!sb.ready) return fail(c, SPEC_ERR_STATE, "spec_layer_forward before spec_kv_import / spec_prefill");
    if (!x_in || !x_out || layer < 0 || layer >= c->tgt.n_layers) return fail(c, SPEC_ERR_ARG, "spec_layer_forward: bad arguments");
    if (n_new < 1 || n_new > c->cfg.k_max + 1) return fail(c, SPEC_ERR_CAPACITY, "n_new %d outside 1..k_max+1", n_new);
    if (!c->resident[layer]) return fail(c, SPEC_ERR_STATE, "layer %d is not resident in HBM", layer);
    const spec_model_shape& s = c->tgt;
    Workspace& w = c->wv;
    hipStream_t st = c->s_compute;
    const int T = sb.B * n_new;
    HIPCHK(c, launch_verify_prep(sb.st, sb.draft_tokens, n_new - 1, w.tok_in, w.row_pos, sb.B, st));
    HIPCHK(c, launch_cast_to_f32(x_in, x_out, (int64_t)T * s.d_model, s.dtype, st));
    HIPCHK(c, launch_rope_table(w.row_pos, w.cs, T, s.head_dim / 2, s.rope_theta, st));
    RowSet r{x_out, w.row_pos, w.cs, T, n_new, sb.B};
    bool pending = false;
    return layer_body(c, s, c->tl, (const char*)c->resident[layer], w, r, kv_layer_ptr(sb.kv_t, c->gt, layer, c->es),
                      c->gt, sb.page_table, &pending, false, st);
}

int spec_accept(const float* p_logits, const float* q_logits, const int32_t* draft_tokens, const float* u_accept,
                const float* u_resample, float temperature, uint64_t seed, uint32_t round, uint32_t seq_base, int B,
                int k, int V, int32_t* n_accepted, int32_t* next_token, void* stream) {
    if (!p_logits || (k > 0 && !draft_tokens) || B < 0 || k < 0 || k > 16 || V <= 0)
        return fail(nullptr, SPEC_ERR_ARG, "spec_accept: bad arguments");
    if (q_logits && (!(temperature > 0.f) || k < 1)) return fail(nullptr, SPEC_ERR_ARG, "spec_accept: sampling needs temperature > 0 and k >= 1");
    if ((u_accept == nullptr) != (u_resample == nullptr)) return fail(nullptr, SPEC_ERR_ARG, "spec_accept: give both uniform arrays or neither");
    AcceptArgs a{};
    a.p_logits = p_logits; a.q_logits = q_logits; a.draft_tokens = draft_tokens; a.u_accept = u_accept;
    a.u_resample = u_resample; a.inv_tau = q_logits ? 1.0f / temperature : 1.0f; a.seed = seed; a.round = round;
    a.seq_base = seq_base; a.B = B; a.k = k; a.V = V; a.n_accepted = n_accepted; a.next_token = next_token;
    HIPCHK(nullptr, launch_accept(a, (hipStream_t)stream));
    return SPEC_OK;
}

int spec_philox_uniforms(uint64_t seed, uint32_t round, uint32_t seq_base, int B, int k, float* out_dev, void* stream) {
    if (!out_dev || B < 0 || k < 0) return fail(nullptr, SPEC_ERR_ARG, "spec_philox_uniforms: bad arguments");
    HIPCHK(nullptr, launch_philox_uniforms(seed, round, seq_base, B, k, out_dev, (hipStream_t)stream));
    return SPEC_OK;
}

int spec_gemm(const void* A, const void* W, float* C, int M, int N, int K, int dtype, int flags, void* stream) {
    if (!A || !W || !C || M <= 0 || N <= 0 || K <= 0 || (dtype != SPEC_F32 && dtype != SPEC_BF16))
        return fail(nullptr, SPEC_ERR_ARG, "spec_gemm: bad arguments");
    GemmArgs g{};
    g.A = A; g.lda = K; g.W = W; g.C = C; g.ldc = N; g.M = M; g.N = N; g.K = K; g.epilogue = EPI_STORE_F32;
    hipError_t e = (dtype == SPEC_BF16 && !(flags & SPEC_FLAG_SIMPLE_KERNELS)) ? launch_gemm_mfma_bf16(g, (hipStream_t)stream)
                                                                              : launch_gemm_simple(g, dtype, (hipStream_t)stream);
    HIPCHK(nullptr, e);
    return SPEC_OK;
}

int spec_measure_link(size_t bytes, int reps, double* gbps) {
    if (!gbps || bytes == 0 || reps <= 0) return fail(nullptr, SPEC_ERR_ARG, "spec_measure_link: bad arguments");
    void *h = nullptr, *d = nullptr;
    hipStream_t st;
    hipEvent_t e0, e1;
    HIPCHK(nullptr, hipHostMalloc(&h, bytes, hipHostMallocDefault));
    memset(h, 1, bytes);
    if (hipMalloc(&d, bytes) != hipSuccess) { hipHostFree(h); return fail(nullptr, SPEC_ERR_HIP, "hipMalloc failed"); }
    hipStreamCreateWithFlags(&st, hipStreamNonBlocking);
    hipEventCreate(&e0); hipEventCreate(&e1);
    hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, st);     // warm-up
    hipEventRecord(e0, st);
    for (int i = 0; i < reps; ++i) hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, st);
    hipEventRecord(e1, st);
    hipError_t e = hipStreamSynchronize(st);
    float ms = 0.f;
    hipEventElapsedTime(&ms, e0, e1);
    hipEventDestroy(e0); hipEventDestroy(e1); hipStreamDestroy(st); hipFree(d); hipHostFree(h);
    if (e != hipSuccess) return fail(nullptr, SPEC_ERR_HIP, "link measurement failed: %s", hipGetErrorString(e));
    *gbps = (double)bytes * reps / (ms * 1e-3) / 1e9;
    return SPEC_OK;
}

}  // extern "C"
