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

// Activation workspace of spec_layer_forward_static: device memory that exists from the moment the
// library's code object is loaded on a GPU, so that entry point never has to allocate.  Host code must
// not use the array's name as an address (on the host it only stands for the symbol): the address on
// each GPU is looked up once with hipGetSymbolAddress and kept in g_scratch_ptr.  (File scope, outside
// any unnamed namespace: only then is the device symbol visible to the runtime's lookup.)
constexpr size_t SCRATCH_BYTES = (size_t)SPEC_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
static void* g_scratch_ptr[MAX_DEVICES] = {nullptr};

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

struct Piece { size_t off, bytes; };               // byte range of a layer blob
struct Item { int layer, piece; bool last; };      // `last`: last streamed piece of its layer

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
    // testing aid (spec_debug_force_routing): expert ids [n_layers, forced_rows, 2] that the next target
    // pass of this sub-batch uses instead of its own top-2; cleared when that pass has been enqueued
    const int32_t* forced_ids = nullptr;
    int forced_rows = 0;
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
    hipStream_t s_copy2 = nullptr;        // second copy stream (see copy_stream_of)
    bool own_compute = false, own_copy = false, own_draft = false;
    std::string err;
    // target weights
    std::vector<const void*> host_layers;
    std::vector<void*> resident;          // per layer: HBM copy of the whole blob, nullptr otherwise
    // Staging granularity: a layer blob is cut into `pieces` (byte ranges).  One piece = whole-layer
    // staging; piece staging cuts it into the attention part and one piece per expert, and then a
    // layer that is not wholly resident may still have some of its pieces pinned (piece_ptr).
    std::vector<Piece> pieces;
    std::vector<std::vector<void*>> piece_ptr;   // [layer][piece]: HBM address if pinned, else nullptr
    std::vector<Item> items;              // the pieces that stream, in the order one pass uses them
    int64_t pinned_piece_bytes = 0;       // pinned pieces of layers that are not wholly resident
    std::vector<void*> ring;
    size_t slot_bytes = 0;
    std::vector<hipEvent_t> ev_ready, ev_free;
    int64_t copies_issued = 0, uses_done = 0;
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
    hipEvent_t prev_copy_end = nullptr;   // end event of the last harvested copy (see harvest_timers)
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
    // set when a target pass failed after it had started to take streamed pieces: the streamer's cursor
    // is then in the middle of a pass and later passes would use pieces out of order; every hot-path call
    // refuses with SPEC_ERR_STATE until the context is destroyed
    bool broken = false;
    std::vector<void*> allocs;            // everything to hipFree
    int device = 0;
    void* scratch_ptr = nullptr;          // this device's copy of the static scratch array
    std::string scratch_err;              // why its address could not be looked up, if it could not
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
// Streamed pieces (whole layers, or the attention part and the experts of a layer) are used in a
// fixed cyclic order (layer order, pass after pass) that does not depend on any token value, so
// copies run ahead of compute by up to n_slots pieces, across pass boundaries as well.  Copy j goes
// to slot j % n_slots after the compute stream has released the piece that used the slot before
// (ev_free); compute waits for ev_ready of the slot.
// copy_busy_ms is the time at least one copy was in flight: consecutive copies run on different
// streams and overlap, so a copy counts from the later of its own start and the previous copy's end
int harvest_timers(spec_ctx* c, bool all) {
    while (!c->copy_timers.empty()) {
        auto pr = c->copy_timers.front();
        if (!all && hipEventQuery(pr.second) != hipSuccess) break;
        if (all) HIPCHK(c, hipEventSynchronize(pr.second));
        float ms = 0.f;
        HIPCHK(c, hipEventElapsedTime(&ms, pr.first, pr.second));
        if (c->prev_copy_end) {
            float ov = 0.f;                    // how long after this copy's start the previous one ended
            HIPCHK(c, hipEventSynchronize(c->prev_copy_end));
            if (hipEventElapsedTime(&ov, pr.first, c->prev_copy_end) != hipSuccess) { (void)hipGetLastError(); ov = 0.f; }
            if (ov > 0.f) ms -= std::min(ov, ms);
            c->timer_pool.push_back(c->prev_copy_end);
        }
        c->copy_busy_ms += ms;
        c->timer_pool.push_back(pr.first);
        c->prev_copy_end = pr.second;
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

// Copies alternate between two streams: the events that order a copy against compute (ready, free,
// timing) are packets of their own between two copies of one stream and leave the link idle for
// 0.1-0.2 ms each time, 3 % of a pass at one expert per copy; with the next copy already queued on the
// other stream the link never waits (measured: 55.2 -> 56.5 GB/s of a 57.3 GB/s link).
inline hipStream_t copy_stream_of(spec_ctx* c, int64_t j) { return (j & 1) ? c->s_copy2 : c->s_copy; }

// One timed host->HBM copy on a copy stream.
int timed_copy(spec_ctx* c, void* dst, const void* src, size_t bytes, hipStream_t cs) {
    hipEvent_t t0, t1;
    int rc;
    if ((rc = get_timer(c, &t0)) || (rc = get_timer(c, &t1))) return rc;
    HIPCHK(c, hipEventRecord(t0, cs));
    HIPCHK(c, hipMemcpyAsync(dst, src, bytes, hipMemcpyHostToDevice, cs));
    HIPCHK(c, hipEventRecord(t1, cs));
    c->copy_timers.emplace_back(t0, t1);
    c->bytes_streamed += (int64_t)bytes;
    return SPEC_OK;
}

// Copy j of the cyclic item sequence fills slot j % n_slots once the use that held the slot before is
// released.  With piece staging (the placeholders of Section 4.2 at the granularity of the placement
// policy, Section 4.2 "Adaptive Tensor Placement") a slot holds one expert or the attention part, so a
// handful of slots of an eighth of a layer replace two whole-layer buffers and the HBM they free pins
// more of the target.
int issue_copy(spec_ctx* c, int64_t j) {
    const int ns = (int)c->ring.size();
    const int slot = (int)(j % ns);
    const Item& it = c->items[(size_t)(j % (int64_t)c->items.size())];
    const Piece& pc = c->pieces[it.piece];
    hipStream_t cs = copy_stream_of(c, j);
    if (j >= ns) HIPCHK(c, hipStreamWaitEvent(cs, c->ev_free[slot], 0));
    int rc = timed_copy(c, c->ring[slot], (const char*)c->host_layers[it.layer] + pc.off, pc.bytes, cs);
    if (rc) return rc;
    HIPCHK(c, hipEventRecord(c->ev_ready[slot], cs));
    if (it.last) c->layers_streamed += 1;
    return SPEC_OK;
}

// host order: a wait on ev_free[s] must be enqueued after the release that records it, so copies run
// at most n_slots items ahead of the uses the host has enqueued
int prefetch(spec_ctx* c) {
    if (c->ring.empty()) return SPEC_OK;
    if (c->cfg.flags & SPEC_FLAG_NO_OVERLAP) return SPEC_OK;
    const int ns = (int)c->ring.size();
    while (c->copies_issued < c->uses_done + ns) {
        int rc = issue_copy(c, c->copies_issued);
        if (rc) return rc;
        c->copies_issued++;
    }
    return SPEC_OK;
}

// HBM address of piece `piece` of `layer` for the kernels enqueued next on the compute stream: the
// pinned copy, or the staging slot once its copy has landed (the compute stream waits, not the host)
int acquire_piece(spec_ctx* c, int layer, int piece, const char** base) {
    if (c->piece_ptr[layer][piece]) { *base = (const char*)c->piece_ptr[layer][piece]; return SPEC_OK; }
    const int ns = (int)c->ring.size();
    const int64_t j = c->uses_done;
    const Item& expect = c->items[(size_t)(j % (int64_t)c->items.size())];
    if (expect.layer != layer || expect.piece != piece)
        return fail(c, SPEC_ERR_STATE, "streamed piece %d.%d used out of pass order (expected %d.%d)", layer, piece,
                    expect.layer, expect.piece);
    if (c->cfg.flags & SPEC_FLAG_NO_OVERLAP) {
        // serial mode: the copy starts only when compute has reached this piece
        hipEvent_t e = c->ev_free[(int)(j % ns)];
        HIPCHK(c, hipEventRecord(e, c->s_compute));
        if (c->copies_issued != j) return fail(c, SPEC_ERR_STATE, "streamer out of step");
        // issue_copy waits on ev_free[slot] for j >= ns; make the wait explicit for all j here
        HIPCHK(c, hipStreamWaitEvent(copy_stream_of(c, j), e, 0));
        int rc = issue_copy(c, j);
        if (rc) return rc;
        c->copies_issued++;
    } else {
        int rc = prefetch(c);
        if (rc) return rc;
    }
    const int slot = (int)(j % ns);
    HIPCHK(c, hipStreamWaitEvent(c->s_compute, c->ev_ready[slot], 0));
    *base = (const char*)c->ring[slot];
    return SPEC_OK;
}

int release_piece(spec_ctx* c, int layer, int piece) {
    if (c->piece_ptr[layer][piece]) return SPEC_OK;
    const int ns = (int)c->ring.size();
    const int slot = (int)(c->uses_done % ns);
    // checking aid: a released slot is overwritten with NaN patterns before the next copy may land in it,
    // so a kernel that still read from it (a release enqueued too early, a wait on the wrong event) shows
    // up as NaNs in the output instead of passing on stale but plausible weights
    if (c->cfg.flags & SPEC_FLAG_POISON_RELEASED)
        HIPCHK(c, launch_fill_words(c->ring[slot], c->slot_bytes / 4, 0xFFFFFFFFu, c->s_compute));
    HIPCHK(c, hipEventRecord(c->ev_free[slot], c->s_compute));
    c->uses_done++;
    return prefetch(c);
}

// a layer runs as one unit (grouped expert products) when it is staged whole or wholly resident
inline bool layer_is_whole(const spec_ctx* c, int layer) { return c->pieces.size() == 1 || c->resident[layer]; }

// ---- one decoder layer on T rows ---------------------------------------------------------------
struct RowSet {
    float* x;                 // [T, d] residual stream
    const int32_t* row_pos;   // [T]
    const float2* cs;         // [T, dh/2]
    int T, n_new, B;
    const int32_t* forced = nullptr;   // [T, 2] expert ids forced on these rows in this layer, or null
};

inline void* kv_layer_ptr(void* pool, const KvGeom& g, int layer, size_t es) {
    return (char*)pool + (size_t)layer * (size_t)g.layer_elems() * es;
}

// A layer is enqueued in three parts so that a streamed layer can take its weights piece by piece:
// layer_front (attention block, post-attention norm, routing: the weights before the experts),
// the expert products (all experts in two grouped launches, or one expert at a time) and the combine.
//
// `pending`: on entry, true if the previous layer left its MoE output uncombined in ws.y.
int layer_attn(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* Wb, Workspace& w,
               const RowSet& r, void* kv_layer, const KvGeom& geom, const int32_t* page_table,
               bool* pending, hipStream_t st) {
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
    return SPEC_OK;
}

// post-attention norm of rows r.x into w.h and, for MoE layers, routing and the expert-sorted row order
int layer_route(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* Wb, Workspace& w,
                const RowSet& r, hipStream_t st) {
    if (s.attn_only) return SPEC_OK;
    const int dt = s.dtype;
    const size_t es = esize(dt);
    const int d = s.d_model, T = r.T;
    auto W = [&](int64_t off) { return (const void*)(Wb + off * es); };
    // post-attention norm; for MoE layers the router logits are taken in the same kernel while the
    // normalised row is still in registers (the plain-kernel mode keeps the two-kernel form)
    const bool fused_route = s.n_experts > 0 && !(c->cfg.flags & SPEC_FLAG_SIMPLE_KERNELS) &&
                             norm_route_supported(d, s.n_experts);
    { ProfScope ps(c, SPEC_PROF_NORM, st);
      if (fused_route)
          HIPCHK(c, launch_norm_route(r.x, W(L.g2), w.h, W(L.wr), w.r_ids, w.r_wts, T, d, s.n_experts, s.rms_eps, r.forced, r.row_pos, dt, st));
      else
          HIPCHK(c, launch_combine_norm(r.x, nullptr, nullptr, nullptr, W(L.g2), w.h, T, d, s.rms_eps, dt, st)); }
    if (s.n_experts > 0) {
        ProfScope ps(c, SPEC_PROF_ROUTE, st);
        if (!fused_route) HIPCHK(c, launch_router(w.h, W(L.wr), w.r_ids, w.r_wts, T, d, s.n_experts, r.forced, r.row_pos, dt, st));
        HIPCHK(c, launch_moe_sort(w.r_ids, w.offsets, w.perm, w.slots, T, s.n_experts, st));
    }
    return SPEC_OK;
}

int layer_front(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* Wb, Workspace& w,
                const RowSet& r, void* kv_layer, const KvGeom& geom, const int32_t* page_table,
                bool* pending, hipStream_t st) {
    int rc = layer_attn(c, s, L, Wb, w, r, kv_layer, geom, page_table, pending, st);
    return rc ? rc : layer_route(c, s, L, Wb, w, r, st);
}

// Expert products of a layer.  `We` points at the gate matrix of expert `first` (expert-major blob:
// gate, up, down of one expert are contiguous); n_exp experts starting there are applied, each to its
// own rows of the expert-sorted order, so any split into launches gives the same result.  A dense FFN
// (n_experts == 0) is the single "expert" 0 and adds straight into the residual stream.
int layer_experts(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* We, int first, int n_exp,
                  Workspace& w, const RowSet& r, hipStream_t st) {
    const int dt = s.dtype;
    const size_t es = esize(dt);
    const int d = s.d_model, T = r.T;
    const void* W1 = We;
    const void* W3 = We + (L.w3 - L.w1) * es;
    const void* W2 = We + (L.w2 - L.w1) * es;
    GemmArgs g{};
    if (s.n_experts > 0) {
        g.A = w.h; g.lda = d; g.a_rows = w.perm; g.W = W1; g.W3 = W3; g.C = w.u; g.ldc = s.d_ff;
        g.M = 2 * T; g.N = s.d_ff; g.K = d; g.epilogue = EPI_SWIGLU_T;
        g.group_offsets = w.offsets + first; g.n_groups = n_exp; g.w_group_stride = L.expert_stride;
        g.m_upper = 2 * T; g.m_expected = std::max(1, 2 * T / s.n_experts);
        { ProfScope ps(c, SPEC_PROF_MOE1, st); HIPCHK(c, gemm(c, g, dt, st)); }
        g = GemmArgs{};
        g.A = w.u; g.lda = s.d_ff; g.W = W2; g.C = w.y; g.ldc = d; g.M = 2 * T; g.N = d; g.K = s.d_ff;
        g.epilogue = EPI_STORE_F32;
        g.group_offsets = w.offsets + first; g.n_groups = n_exp; g.w_group_stride = L.expert_stride;
        g.m_upper = 2 * T; g.m_expected = std::max(1, 2 * T / s.n_experts);
        { ProfScope ps(c, SPEC_PROF_MOE2, st); HIPCHK(c, gemm(c, g, dt, st)); }
    } else {
        g.A = w.h; g.lda = d; g.W = W1; g.W3 = W3; g.C = w.u; g.ldc = s.d_ff; g.M = T; g.N = s.d_ff;
        g.K = d; g.epilogue = EPI_SWIGLU_T;
        { ProfScope ps(c, SPEC_PROF_MOE1, st); HIPCHK(c, gemm(c, g, dt, st)); }
        g = GemmArgs{};
        g.A = w.u; g.lda = s.d_ff; g.W = W2; g.C = r.x; g.ldc = d; g.M = T; g.N = d; g.K = s.d_ff;
        g.epilogue = EPI_ADD_F32;
        { ProfScope ps(c, SPEC_PROF_MOE2, st); HIPCHK(c, gemm(c, g, dt, st)); }
    }
    return SPEC_OK;
}

// weighted sum of the two expert outputs of every row into the residual stream (when it is not left
// to the next layer's first norm)
int layer_combine(spec_ctx* c, const spec_model_shape& s, Workspace& w, const RowSet& r, hipStream_t st) {
    ProfScope ps(c, SPEC_PROF_NORM, st);
    HIPCHK(c, launch_combine_norm(r.x, w.y, w.r_wts, w.slots, nullptr, nullptr, r.T, s.d_model, s.rms_eps, s.dtype, st));
    return SPEC_OK;
}

// whole layer from one contiguous blob.  On exit *pending is true if the MoE output is left
// uncombined in ws.y (defer == true); with defer == false the combine is applied before returning.
int layer_body(spec_ctx* c, const spec_model_shape& s, const Layout& L, const char* Wb, Workspace& w,
               const RowSet& r, void* kv_layer, const KvGeom& geom, const int32_t* page_table,
               bool* pending, bool defer, hipStream_t st) {
    int rc = layer_front(c, s, L, Wb, w, r, kv_layer, geom, page_table, pending, st);
    if (rc || s.attn_only) return rc;
    if ((rc = layer_experts(c, s, L, Wb + L.w1 * esize(s.dtype), 0, std::max(1, s.n_experts), w, r, st))) return rc;
    if (s.n_experts > 0) {
        *pending = true;
        if (!defer) {
            if ((rc = layer_combine(c, s, w, r, st))) return rc;
            *pending = false;
        }
    }
    return SPEC_OK;
}

// one target layer of a pass: as a whole (staged whole, or resident), or piece by piece, each piece
// released as soon as its kernels are enqueued so that its slot can take the next copy
int target_layer(spec_ctx* c, int l, Workspace& w, const RowSet& r, void* kv_layer, const int32_t* page_table,
                 bool* pending, bool defer) {
    const spec_model_shape& s = c->tgt;
    hipStream_t st = c->s_compute;
    const char* Wb;
    int rc;
    if (layer_is_whole(c, l)) {
        if ((rc = acquire_piece(c, l, 0, &Wb))) return rc;
        if ((rc = layer_body(c, s, c->tl, Wb, w, r, kv_layer, c->gt, page_table, pending, defer, st))) return rc;
        return release_piece(c, l, 0);
    }
    if ((rc = acquire_piece(c, l, 0, &Wb))) return rc;
    if ((rc = layer_front(c, s, c->tl, Wb, w, r, kv_layer, c->gt, page_table, pending, st))) return rc;
    if ((rc = release_piece(c, l, 0))) return rc;
    const int ne = std::max(1, s.n_experts);
    for (int e = 0; e < ne; ++e) {
        if ((rc = acquire_piece(c, l, 1 + e, &Wb))) return rc;
        if ((rc = layer_experts(c, s, c->tl, Wb, e, 1, w, r, st))) return rc;
        if ((rc = release_piece(c, l, 1 + e))) return rc;
    }
    if (s.n_experts > 0) {
        *pending = true;
        if (!defer) {
            if ((rc = layer_combine(c, s, w, r, st))) return rc;
            *pending = false;
        }
    }
    return SPEC_OK;
}


// target pass over rows already embedded in w.x (tok_in/row_pos/cs set); leaves normalised final
// state in w.h when want_head
int target_layers(spec_ctx* c, Sub& sb, Workspace& w, int T, int n_new, bool want_final_norm) {
    RowSet r{w.x, w.row_pos, w.cs, T, n_new, sb.B};
    bool pending = false;
    const int32_t* forced = sb.forced_ids;
    const int64_t forced_rows = sb.forced_rows;
    sb.forced_ids = nullptr;
    if (forced && forced_rows < T) return fail(c, SPEC_ERR_ARG, "forced routing covers %lld rows per layer, the pass has %d", (long long)forced_rows, T);
    for (int l = 0; l < c->tgt.n_layers; ++l) {
        r.forced = forced ? forced + (int64_t)l * forced_rows * 2 : nullptr;
        int rc = target_layer(c, l, w, r, kv_layer_ptr(sb.kv_t, c->gt, l, c->es), sb.page_table, &pending, true);
        if (rc) return rc;
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

// `hot`: the call enqueues model passes (refused on a context whose streamer is out of step)
int check_sub(spec_ctx* c, int sub, bool hot = false) {
    if (!c) return fail(nullptr, SPEC_ERR_ARG, "ctx is NULL");
    if (hot && c->broken) return fail(c, SPEC_ERR_STATE, "context unusable: an earlier target pass failed part-way (destroy it)");
    if (sub < 0 || sub >= c->cfg.n_sub_batches) return fail(c, SPEC_ERR_ARG, "sub-batch %d out of range", sub);
    return SPEC_OK;
}

// pieces of a layer blob: the whole blob, or the weights before the experts and one piece per expert
// (a dense FFN counts as one expert)
std::vector<Piece> make_pieces(const spec_model_shape& s, const Layout& L, bool split) {
    const size_t es = esize(s.dtype);
    std::vector<Piece> v;
    if (!split || s.attn_only) { v.push_back({0, (size_t)L.total * es}); return v; }
    v.push_back({0, (size_t)L.w1 * es});
    for (int e = 0; e < std::max(1, s.n_experts); ++e)
        v.push_back({(size_t)(L.w1 + e * L.expert_stride) * es, (size_t)L.expert_stride * es});
    return v;
}

constexpr int DEFAULT_PIECE_SLOTS = 3;

// Placement of the target's parameters under the HBM weight budget (Section 4.2, "Adaptive Tensor
// Placement": what the current and the next use need comes first, the draft model is resident during
// decoding, spare memory pins further target parameters).  The draft model and the globals are
// `fixed`; the staging ring is what "current and next" need; what is left pins whole layers from the
// first one on and, with piece staging, the leading pieces of one more layer.
struct Placement {
    bool split = false;            // piece staging
    bool front_all = false;        // the weights in front of the experts of EVERY layer are pinned first
    int n_slots = 0;               // staging slots (0: nothing streams)
    int64_t slot_bytes = 0, ring_bytes = 0, fixed = 0;
    int64_t R = 0;                 // wholly resident layers
    int partial_pieces = 0;        // leading pieces of layer R that are pinned as well
    int64_t partial_bytes = 0;     // pinned pieces of layers that are not wholly resident
    int64_t streamed_bytes = 0;
};

// n_ring_slots == 0: piece staging with n_piece_slots slots (0 = default); n >= 1: n whole-layer slots.
// false if the budget cannot hold the fixed part and the ring.
//
// SPEC_FLAG_PIN_ATTENTION (piece staging only) is the decode-phase placement of the paper itself
// (Section 4.1.2; Appendix A.1 "only the MoE FFN parameters ... are loaded into GPU memory"): the
// attention part of every layer is resident and only expert parameters cross the link; what is left of
// the budget pins whole expert sets from the first layer on, then leading experts of one more layer.
bool plan_placement(const spec_model_shape& t, const spec_model_shape* d, int64_t budget, int n_ring_slots,
                    int n_piece_slots, int flags, Placement* out) {
    Placement P;
    const size_t es = esize(t.dtype);
    const Layout tl = make_layout(t);
    const GlobalLayout gl = make_global_layout(t);
    const int64_t blob = tl.total * (int64_t)es;
    P.fixed = gl.total * (int64_t)es;
    if (d) P.fixed += (int64_t)d->n_layers * make_layout(*d).total * (int64_t)esize(d->dtype);
    if (budget <= 0 || P.fixed + (int64_t)t.n_layers * blob <= budget) {
        P.R = t.n_layers;
        *out = P;
        return true;
    }
    P.split = n_ring_slots <= 0 && !t.attn_only;
    P.front_all = P.split && (flags & SPEC_FLAG_PIN_ATTENTION);
    const std::vector<Piece> pieces = make_pieces(t, tl, P.split);
    const int first_staged = P.front_all ? 1 : 0;          // pieces that can ever sit in a staging slot
    for (size_t q = first_staged; q < pieces.size(); ++q) P.slot_bytes = std::max<int64_t>(P.slot_bytes, (int64_t)pieces[q].bytes);
    P.slot_bytes = (P.slot_bytes + 255) & ~(int64_t)255;
    P.n_slots = P.split ? (n_piece_slots > 0 ? n_piece_slots : DEFAULT_PIECE_SLOTS) : std::max(1, n_ring_slots);
    P.ring_bytes = P.n_slots * P.slot_bytes;
    const int64_t front = P.front_all ? (int64_t)pieces[0].bytes : 0;
    const int64_t avail = budget - P.fixed - P.ring_bytes - (int64_t)t.n_layers * front;
    if (avail < 0) { *out = P; return false; }
    P.R = std::min<int64_t>(avail / (blob - front), t.n_layers);
    int64_t left = avail - P.R * (blob - front);
    P.partial_pieces = first_staged;
    if (P.split && P.R < t.n_layers)
        for (size_t q = first_staged; q < pieces.size(); ++q) {
            if ((int64_t)pieces[q].bytes > left) break;
            left -= (int64_t)pieces[q].bytes;
            P.partial_bytes += (int64_t)pieces[q].bytes;
            P.partial_pieces++;
        }
    P.partial_bytes += (t.n_layers - P.R) * front;
    P.streamed_bytes = (t.n_layers - P.R) * blob - P.partial_bytes;
    *out = P;
    return true;
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
    Placement pl;
    if (!plan_placement(*target, draft, budget, n_ring_slots, 0, 0, &pl))
        return fail(nullptr, SPEC_ERR_BUDGET, "budget cannot hold globals + draft (%lld B) + the staging ring (%d slots of %lld B)",
                    (long long)pl.fixed, pl.n_slots, (long long)pl.slot_bytes);
    if (streamed_bytes_per_pass) *streamed_bytes_per_pass = pl.streamed_bytes;
    return pl.R;
}

int spec_plan_placement(const spec_model_shape* target, const spec_model_shape* draft, const spec_runtime_cfg* cfg,
                        spec_placement* out) {
    if (!target || !cfg || !out) return fail(nullptr, SPEC_ERR_ARG, "spec_plan_placement: NULL argument");
    if (!shape_ok(target) || (draft && !shape_ok(draft))) return fail(nullptr, SPEC_ERR_SHAPE, "unsupported model shape");
    Placement pl;
    const bool ok = plan_placement(*target, draft, cfg->hbm_weight_budget_bytes, cfg->n_ring_slots, cfg->n_piece_slots,
                                   cfg->flags, &pl);
    out->resident_layers = pl.R;
    out->pinned_piece_bytes = pl.partial_bytes;
    out->streamed_bytes_per_pass = pl.streamed_bytes;
    out->ring_bytes = pl.ring_bytes;
    out->fixed_bytes = pl.fixed;
    out->n_slots = pl.n_slots;
    out->piece_staging = pl.split;
    if (!ok)
        return fail(nullptr, SPEC_ERR_BUDGET, "budget cannot hold globals + draft (%lld B), the staging ring (%d slots of %lld B)%s",
                    (long long)pl.fixed, pl.n_slots, (long long)pl.slot_bytes,
                    pl.front_all ? " and the attention part of every layer" : "");
    return SPEC_OK;
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
    if (c->prev_copy_end) hipEventDestroy(c->prev_copy_end);
    for (auto e : c->ev_ready) hipEventDestroy(e);
    for (auto e : c->ev_free) hipEventDestroy(e);
    for (int s = 0; s < 2; ++s) {
        if (c->sub[s].ev_drafted) hipEventDestroy(c->sub[s].ev_drafted);
        if (c->sub[s].ev_committed) hipEventDestroy(c->sub[s].ev_committed);
    }
    for (void* p : c->allocs) hipFree(p);
    if (c->own_compute) hipStreamDestroy(c->s_compute);
    if (c->own_copy) hipStreamDestroy(c->s_copy);
    if (c->s_copy2) hipStreamDestroy(c->s_copy2);
    if (c->own_draft) hipStreamDestroy(c->s_draft);
    delete c;
}

static int init_impl(spec_ctx* c, const spec_host_weights* tw, const spec_host_weights* dw) {
    const spec_model_shape& t = c->tgt;
    const spec_runtime_cfg& cfg = c->cfg;
    // the static scratch array's address on this device (each GPU holds its own copy of the array)
    HIPCHK(c, hipGetDevice(&c->device));
    if (c->device < 0 || c->device >= MAX_DEVICES) return fail(c, SPEC_ERR_ARG, "device index %d not supported", c->device);
    if (!g_scratch_ptr[c->device]) {
        // a failed lookup only disables spec_layer_forward_static (which reports it); nothing else uses the array
        void* p = nullptr;
        hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e == hipSuccess) g_scratch_ptr[c->device] = p;
        else { c->scratch_err = hipGetErrorString(e); (void)hipGetLastError(); }
    }
    c->scratch_ptr = g_scratch_ptr[c->device];
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
    HIPCHK(c, hipStreamCreateWithFlags(&c->s_copy2, hipStreamNonBlocking));
    if ((rc = mk_stream(cfg.draft_stream, &c->s_draft, &c->own_draft))) return rc;

    // placement under the HBM weight budget
    Placement pl;
    if (!plan_placement(t, c->has_draft ? &c->drf : nullptr, cfg.hbm_weight_budget_bytes, cfg.n_ring_slots,
                        cfg.n_piece_slots, cfg.flags, &pl))
        return fail(c, SPEC_ERR_BUDGET, "HBM weight budget %lld B cannot hold globals+draft (%lld B) and %d staging slots of %lld B%s",
                    (long long)cfg.hbm_weight_budget_bytes, (long long)pl.fixed, pl.n_slots, (long long)pl.slot_bytes,
                    pl.front_all ? " and the attention part of every layer" : "");
    c->pieces = make_pieces(t, c->tl, pl.split);
    const int np = (int)c->pieces.size();
    c->host_layers.assign(tw->layer_blobs, tw->layer_blobs + t.n_layers);
    c->resident.assign(t.n_layers, nullptr);
    c->piece_ptr.assign(t.n_layers, std::vector<void*>(np, nullptr));
    for (int l = 0; l < t.n_layers; ++l) {
        if (!c->host_layers[l]) return fail(c, SPEC_ERR_ARG, "target layer blob %d is NULL", l);
        if (l < pl.R) {
            char* p;
            if ((rc = dev_alloc(c, &p, c->blob_bytes))) return rc;
            HIPCHK(c, hipMemcpy(p, c->host_layers[l], c->blob_bytes, hipMemcpyHostToDevice));
            c->resident[l] = p;
            for (int q = 0; q < np; ++q) c->piece_ptr[l][q] = p + c->pieces[q].off;
            continue;
        }
        for (int q = 0; q < np; ++q) {
            if ((l == pl.R && q < pl.partial_pieces) || (pl.front_all && q == 0)) {
                char* p;
                if ((rc = dev_alloc(c, &p, c->pieces[q].bytes))) return rc;
                HIPCHK(c, hipMemcpy(p, (const char*)c->host_layers[l] + c->pieces[q].off, c->pieces[q].bytes,
                                    hipMemcpyHostToDevice));
                c->piece_ptr[l][q] = p;
            } else {
                if (!c->items.empty() && c->items.back().layer == l) c->items.back().last = false;
                c->items.push_back(Item{l, q, true});
            }
        }
    }
    c->pinned_piece_bytes = pl.partial_bytes;
    c->hbm_weight_bytes = pl.fixed + pl.R * (int64_t)c->blob_bytes + pl.partial_bytes;
    if (!c->items.empty()) {
        c->slot_bytes = (size_t)pl.slot_bytes;
        c->ring.resize(pl.n_slots);
        c->ev_ready.resize(pl.n_slots);
        c->ev_free.resize(pl.n_slots);
        for (int i = 0; i < pl.n_slots; ++i) {
            char* p;
            if ((rc = dev_alloc(c, &p, c->slot_bytes))) return rc;
            c->ring[i] = p;
            HIPCHK(c, hipEventCreateWithFlags(&c->ev_ready[i], hipEventDisableTiming));
            HIPCHK(c, hipEventCreateWithFlags(&c->ev_free[i], hipEventDisableTiming));
        }
        c->hbm_weight_bytes += pl.ring_bytes;
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
    if (cfg.n_piece_slots < 0 || cfg.n_piece_slots == 1 || cfg.n_piece_slots > 16)
        return fail(nullptr, SPEC_ERR_ARG, "n_piece_slots must be 0 (default) or 2..16");
    if (cfg.mode != SPEC_GREEDY && cfg.mode != SPEC_SAMPLE) return fail(nullptr, SPEC_ERR_ARG, "bad mode");
    if (cfg.mode == SPEC_SAMPLE && !(cfg.temperature > 0.f)) return fail(nullptr, SPEC_ERR_ARG, "temperature must be > 0");
    if (cfg.prefill_chunk == 0) {
        // the MFMA attention kernel takes the query rows of a chunk in blocks of 64, any number of them; the
        // plain kernel is written for the few rows of a verify pass
        const bool mfma_attn = target->dtype == SPEC_BF16 && !(cfg.flags & SPEC_FLAG_SIMPLE_KERNELS) && target->head_dim == 128 &&
                               cfg.page_tokens >= 32 && (cfg.page_tokens & (cfg.page_tokens - 1)) == 0;
        int g = target->n_q_heads / target->n_kv_heads;
        cfg.prefill_chunk = mfma_attn ? 64 : std::max(1, std::min(16, 64 / g));
    }
    if (cfg.prefill_chunk < 1 || cfg.prefill_chunk > 64) return fail(nullptr, SPEC_ERR_ARG, "prefill_chunk must be 1..64");
    if (cfg.prefill_group_rows == 0) cfg.prefill_group_rows = 32768;
    if (cfg.prefill_group_rows < 1) return fail(nullptr, SPEC_ERR_ARG, "prefill_group_rows must be positive");
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
    int rc = check_sub(c, sub, true);
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
        // The attention block runs chunk by chunk (Q prompt positions of every sequence); the feed-forward
        // part runs on groups of chunks so that an expert sees thousands of rows per launch.  A layer that
        // streams piece by piece holds each piece for all groups before the next piece arrives, so what a
        // group carries from the routing to its experts and on to the combine (normalised rows, routing,
        // expert outputs) is then kept per group.
        const int G = std::max(1, std::min(n_chunks, c->cfg.prefill_group_rows / T));
        const int n_grp = (n_chunks + G - 1) / G;
        std::vector<void*> temps;
        const int32_t* forced = sb.forced_ids;
        const int64_t forced_rows = sb.forced_rows;
        sb.forced_ids = nullptr;
        auto cleanup = [&]() { hipFree(xall); hipFree(pos_all); hipFree(cs_all); for (void* p : temps) hipFree(p); };
        // The prefill lays its rows out in its own order of the sequences: longest prompt first.  In chunk
        // ch only the first n_act[ch] sequences still have prompt positions, so the attention part of a
        // chunk (norm, QKV, attention, O-projection) runs on that prefix of the chunk's rows and skips the
        // padding of finished prompts (the feed-forward part already leaves inactive rows out through the
        // routing).  seq_of maps a row block to its sequence for the token gather, and the page table handed
        // to the kernels is the context's with its rows in the same order.  (Forced routing, a test hook whose
        // ids come in sequence order, keeps the sequences in their own order.)
        std::vector<int32_t> order(B);
        for (int b = 0; b < B; ++b) order[b] = b;
        if (!forced)
            std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
                return cu_lens[x + 1] - cu_lens[x] > cu_lens[y + 1] - cu_lens[y]; });
        std::vector<int> n_act(n_chunks, 0);
        for (int ch = 0; ch < n_chunks; ++ch)
            for (int v = 0; v < B; ++v)
                if (cu_lens[order[v] + 1] - cu_lens[order[v]] - 1 > ch * Q) n_act[ch] = v + 1;
        const int pps = c->gt.pages_per_seq, Bm = c->cfg.batch_max;
        int32_t* seq_of = nullptr; int32_t* pt_v = nullptr;
        {
            std::vector<int32_t> tab((size_t)B * pps);
            for (int v = 0; v < B; ++v)
                for (int p = 0; p < pps; ++p) tab[(size_t)v * pps + p] = p * Bm + order[v];
            hipError_t e3 = hipMalloc(&seq_of, (size_t)B * 4);
            if (e3 == hipSuccess) temps.push_back(seq_of);
            hipError_t e4 = hipMalloc(&pt_v, tab.size() * 4);
            if (e4 == hipSuccess) temps.push_back(pt_v);
            if (e3 == hipSuccess && e4 == hipSuccess) {
                e3 = hipMemcpy(seq_of, order.data(), (size_t)B * 4, hipMemcpyHostToDevice);
                e4 = hipMemcpy(pt_v, tab.data(), tab.size() * 4, hipMemcpyHostToDevice);
            }
            if (e3 != hipSuccess || e4 != hipSuccess) { cleanup(); return fail(c, SPEC_ERR_HIP, "prefill scratch allocation failed"); }
        }
        if (forced && forced_rows < (int64_t)n_chunks * T) {
            cleanup();
            return fail(c, SPEC_ERR_ARG, "forced routing covers %lld rows per layer, the prefill has %lld", (long long)forced_rows,
                        (long long)n_chunks * T);
        }
        if (e1 != hipSuccess || e2 != hipSuccess) { cleanup(); return fail(c, SPEC_ERR_HIP, "prefill scratch allocation failed"); }
        auto run_model = [&](bool is_draft) -> int {
            const spec_model_shape& s = is_draft ? c->drf : c->tgt;
            const Layout& L = is_draft ? c->dl : c->tl;
            const KvGeom& geom = is_draft ? c->gd : c->gt;
            Workspace& w = is_draft ? c->wd : c->wv;
            const char* G_ = (const char*)(is_draft ? c->d_draft_globals : c->d_globals);
            const int hf = s.head_dim / 2;
            const bool ffn = !s.attn_only, moe = s.n_experts > 0;
            bool piecewise = false;
            if (!is_draft) for (int l = 0; l < s.n_layers; ++l) piecewise = piecewise || !layer_is_whole(c, l);
            std::vector<Workspace> wg(piecewise ? n_grp : 1, w);
            if (ffn) {
                auto al = [](size_t n) { return (n + 255) & ~(size_t)255; };
                const size_t Tg = (size_t)G * T;
                const size_t b_h = al(Tg * d * c->es), b_y = moe ? al(2 * Tg * d * 4) : 0, b_t8 = moe ? al(Tg * 8) : 0,
                             b_off = moe ? 256 : 0, b_u = al((moe ? 2 : 1) * Tg * s.d_ff * c->es);
                const size_t per = b_h + b_y + 4 * b_t8 + b_off;
                char* base = nullptr;
                if (hipMalloc(&base, per * wg.size() + b_u) != hipSuccess)
                    return fail(c, SPEC_ERR_HIP, "prefill scratch allocation failed");
                temps.push_back(base);
                for (size_t i = 0; i < wg.size(); ++i) {
                    char* p = base + per * i;
                    Workspace& x = wg[i];
                    x.u = base + per * wg.size();
                    x.h = p; p += b_h;
                    if (moe) {
                        x.y = (float*)p; p += b_y;
                        x.r_ids = (int32_t*)p; p += b_t8;
                        x.r_wts = (float*)p; p += b_t8;
                        x.perm = (int32_t*)p; p += b_t8;
                        x.slots = (int32_t*)p; p += b_t8;
                        x.offsets = (int32_t*)p;
                    }
                }
            }
            for (int ch = 0; ch < n_chunks; ++ch) {
                int32_t* rp = pos_all + (size_t)ch * T;
                HIPCHK(c, launch_prefill_prep(sb.st.tokens, sb.st.len, seq_of, sb.st.tok_cap, B, ch * Q, Q, w.tok_in, rp, st));
                HIPCHK(c, launch_embed(G_ + c->gl.emb * c->es, w.tok_in, xall + (size_t)ch * T * d, T, d, s.vocab, s.dtype, st));
                HIPCHK(c, launch_rope_table(rp, cs_all + (size_t)ch * T * hf, T, hf, s.rope_theta, st));
            }
            int cur_layer = 0;
            auto rows_of = [&](int ch, int n_ch) {     // n_ch consecutive chunks as one row set
                RowSet r{xall + (size_t)ch * T * d, pos_all + (size_t)ch * T, cs_all + (size_t)ch * T * hf, n_ch * T, Q, B};
                if (forced && !is_draft) r.forced = forced + ((int64_t)cur_layer * forced_rows + (int64_t)ch * T) * 2;
                return r;
            };
            auto attn_of_group = [&](int g, const char* Wb, void* kvl) -> int {
                for (int ch = g * G; ch < std::min(n_chunks, (g + 1) * G); ++ch) {
                    bool pending = false;
                    RowSet ra = rows_of(ch, 1);
                    ra.T = n_act[ch] * Q; ra.B = n_act[ch];          // the sequences that still have prompt positions
                    if (ra.T == 0) continue;
                    int r2 = layer_attn(c, s, L, Wb, w, ra, kvl, geom, pt_v, &pending, st);
                    if (r2) return r2;
                }
                return SPEC_OK;
            };
            auto group_rows = [&](int g) { return rows_of(g * G, std::min(G, n_chunks - g * G)); };
            const int ne = std::max(1, s.n_experts);
            for (int l = 0; l < s.n_layers; ++l) {
                const char* Wb;
                int r2;
                cur_layer = l;
                void* kvl = kv_layer_ptr(is_draft ? sb.kv_d : sb.kv_t, geom, l, c->es);
                if (is_draft || layer_is_whole(c, l)) {
                    if (is_draft) Wb = (const char*)c->d_draft_layers[l];
                    else if ((r2 = acquire_piece(c, l, 0, &Wb))) return r2;
                    for (int g = 0; g < n_grp; ++g) {
                        if ((r2 = attn_of_group(g, Wb, kvl))) return r2;
                        if (!ffn) continue;
                        const RowSet rg = group_rows(g);
                        if ((r2 = layer_route(c, s, L, Wb, wg[0], rg, st))) return r2;
                        if ((r2 = layer_experts(c, s, L, Wb + L.w1 * c->es, 0, ne, wg[0], rg, st))) return r2;
                        if (moe && (r2 = layer_combine(c, s, wg[0], rg, st))) return r2;
                    }
                    if (!is_draft && (r2 = release_piece(c, l, 0))) return r2;
                    continue;
                }
                // piece by piece: every group through the attention part and the routing, then every group
                // through expert 0, expert 1, ...; the arithmetic of a row is that of the whole-layer order
                if ((r2 = acquire_piece(c, l, 0, &Wb))) return r2;
                for (int g = 0; g < n_grp; ++g) {
                    if ((r2 = attn_of_group(g, Wb, kvl))) return r2;
                    if ((r2 = layer_route(c, s, L, Wb, wg[g], group_rows(g), st))) return r2;
                }
                if ((r2 = release_piece(c, l, 0))) return r2;
                for (int e = 0; e < ne; ++e) {
                    if ((r2 = acquire_piece(c, l, 1 + e, &Wb))) return r2;
                    for (int g = 0; g < n_grp; ++g)
                        if ((r2 = layer_experts(c, s, L, Wb, e, 1, wg[g], group_rows(g), st))) return r2;
                    if ((r2 = release_piece(c, l, 1 + e))) return r2;
                }
                if (moe)
                    for (int g = 0; g < n_grp; ++g)
                        if ((r2 = layer_combine(c, s, wg[g], group_rows(g), st))) return r2;
            }
            return SPEC_OK;
        };
        rc = run_model(false);
        if (rc && !c->items.empty() && c->uses_done % (int64_t)c->items.size() != 0) c->broken = true;   // stopped mid-pass
        if (!rc && c->has_draft) rc = run_model(true);
        hipError_t es_ = hipStreamSynchronize(st);
        cleanup();
        if (rc) return rc;
        if (es_ != hipSuccess) return fail(c, SPEC_ERR_HIP, "prefill failed: %s", hipGetErrorString(es_));
    }
    // a fresh set of sequences: nothing drafted for them, rounds count from 0, and the rotation of
    // spec_step starts over (it drafts for its first sub-batch again before the first verify)
    sb.ready = true; sb.drafted = false; sb.round = 0; sb.last_k = sb.last_draft_k = 0; sb.forced_ids = nullptr;
    c->primed = false; c->cur = 0;
    return SPEC_OK;
}

int spec_kv_import(spec_ctx* c, int sub, int layer, const void* k_ctx, const void* v_ctx, int B, int ctx_len) {
    int rc = check_sub(c, sub, true);
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
    int rc = check_sub(c, sub, true);
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
    ProfScope ps_draft(c, SPEC_PROF_DRAFT, st);
    // the draft pass is timed as one class: its kernels' own classes are masked until this call returns,
    // on the error paths as well
    struct MaskGuard {
        spec_ctx* c; uint32_t saved;
        ~MaskGuard() { c->prof_mask = saved; }
    } mask_guard{c, c->prof_mask};
    c->prof_mask &= (1u << SPEC_PROF_DRAFT);
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
    if (out_tokens) HIPCHK(c, hipMemcpyAsync(out_tokens, sb.draft_tokens, (size_t)B * k * 4, hipMemcpyDeviceToDevice, st));
    HIPCHK(c, hipEventRecord(sb.ev_drafted, st));
    sb.drafted = true; sb.last_draft_k = k;
    return SPEC_OK;
}

int spec_verify(spec_ctx* c, int sub, const int32_t* draft_tokens, int k, int32_t* n_accepted, int32_t* next_token) {
    int rc = check_sub(c, sub, true);
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
    if ((rc = target_layers(c, sb, w, T, k + 1, true))) {
        if (!c->items.empty() && c->uses_done % (int64_t)c->items.size() != 0) c->broken = true;   // stopped mid-pass
        return rc;
    }
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
    if (sub < 0) { HIPCHK(c, hipStreamSynchronize(c->s_copy)); HIPCHK(c, hipStreamSynchronize(c->s_copy2)); }
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
    out->resident_layers = 0;
    for (void* p : c->resident) out->resident_layers += p != nullptr;
    out->pinned_piece_bytes = c->pinned_piece_bytes;
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

int spec_debug_force_routing(spec_ctx* c, int sub, const int32_t* ids_dev, int rows_per_layer) {
    int rc = check_sub(c, sub);
    if (rc) return rc;
    if (ids_dev && rows_per_layer <= 0) return fail(c, SPEC_ERR_ARG, "spec_debug_force_routing: rows_per_layer must be positive");
    if (c->tgt.n_experts == 0) return fail(c, SPEC_ERR_STATE, "the target has no router");
    c->sub[sub].forced_ids = ids_dev;
    c->sub[sub].forced_rows = ids_dev ? rows_per_layer : 0;
    return SPEC_OK;
}

static int layer_forward_impl(spec_ctx* c, int sub, int layer, const void* x_in, int n_new, float* x_out, Workspace& w) {
    Sub& sb = c->sub[sub];
    const spec_model_shape& s = c->tgt;
    hipStream_t st = c->s_compute;
    const int T = sb.B * n_new;
    HIPCHK(c, launch_verify_prep(sb.st, sb.draft_tokens, n_new - 1, w.tok_in, w.row_pos, sb.B, st));
    HIPCHK(c, launch_cast_to_f32(x_in, x_out, (int64_t)T * s.d_model, s.dtype, st));
    HIPCHK(c, launch_rope_table(w.row_pos, w.cs, T, s.head_dim / 2, s.rope_theta, st));
    RowSet r{x_out, w.row_pos, w.cs, T, n_new, sb.B};
    if (sb.forced_ids) {
        if (sb.forced_rows < T) return fail(c, SPEC_ERR_ARG, "forced routing covers %d rows per layer, the pass has %d", sb.forced_rows, T);
        r.forced = sb.forced_ids + (int64_t)layer * sb.forced_rows * 2;
        sb.forced_ids = nullptr;
    }
    bool pending = false;
    return layer_body(c, s, c->tl, (const char*)c->resident[layer], w, r, kv_layer_ptr(sb.kv_t, c->gt, layer, c->es),
                      c->gt, sb.page_table, &pending, false, st);
}

static int layer_forward_check(spec_ctx* c, int sub, int layer, const void* x_in, int n_new, float* x_out) {
    int rc = check_sub(c, sub, true);
    if (rc) return rc;
    Sub& sb = c->sub[sub];
    if (!sb.ready) return fail(c, SPEC_ERR_STATE, "spec_layer_forward before spec_kv_import / spec_prefill");
    if (!x_in || !x_out || layer < 0 || layer >= c->tgt.n_layers) return fail(c, SPEC_ERR_ARG, "spec_layer_forward: bad arguments");
    if (n_new < 1 || n_new > c->cfg.k_max + 1) return fail(c, SPEC_ERR_CAPACITY, "n_new %d outside 1..k_max+1", n_new);
    if (!c->resident[layer]) return fail(c, SPEC_ERR_STATE, "layer %d is not resident in HBM", layer);
    return SPEC_OK;
}

int spec_layer_forward(spec_ctx* c, int sub, int layer, const void* x_in, int n_new, float* x_out) {
    int rc = layer_forward_check(c, sub, layer, x_in, n_new, x_out);
    if (rc) return rc;
    return layer_forward_impl(c, sub, layer, x_in, n_new, x_out, c->wv);
}

// The same layer pass with its activation workspace carved out of the static scratch array instead of
// the context's workspace.  Nothing is allocated here or below: the kernels are the ones
// spec_layer_forward launches and take the scratch addresses as arguments.
int spec_layer_forward_static(spec_ctx* c, int sub, int layer, const void* x_in, int n_new, float* x_out) {
    int rc = layer_forward_check(c, sub, layer, x_in, n_new, x_out);
    if (rc) return rc;
    const spec_model_shape& s = c->tgt;
    const size_t es = c->es;
    const size_t T = (size_t)c->sub[sub].B * n_new;
    const size_t d = s.d_model, hd = (size_t)s.n_q_heads * s.head_dim;
    const size_t qkv_rows = (size_t)(s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim;
    if (!c->scratch_ptr)
        return fail(c, SPEC_ERR_HIP, "spec_layer_forward_static: the static scratch array has no address on device %d (%s)",
                    c->device, c->scratch_err.c_str());
    char* base = (char*)c->scratch_ptr;
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = base + off; off += (bytes + 255) & ~(size_t)255; return p; };
    Workspace w;
    w.t_max = (int)T;
    w.h = take(T * d * es);
    w.qkv = (float*)take(T * qkv_rows * 4);
    w.q = take(T * hd * es);
    w.att = take(T * hd * es);
    w.cs = (float2*)take(T * (s.head_dim / 2) * sizeof(float2));
    w.tok_in = (int32_t*)take(T * 4);
    w.row_pos = (int32_t*)take(T * 4);
    const size_t mult = s.n_experts > 0 ? 2 : 1;
    w.u = take(mult * T * s.d_ff * es);
    if (s.n_experts > 0) {
        w.r_ids = (int32_t*)take(T * 8);
        w.r_wts = (float*)take(T * 8);
        w.offsets = (int32_t*)take(64);
        w.perm = (int32_t*)take(T * 8);
        w.slots = (int32_t*)take(T * 8);
        w.y = (float*)take(2 * T * d * 4);
    }
    if (off > SCRATCH_BYTES)
        return fail(c, SPEC_ERR_CAPACITY, "spec_layer_forward_static: %zu rows of this model need %zu bytes of workspace, the static "
                    "scratch holds %zu (use spec_layer_forward)", T, off, SCRATCH_BYTES);
    // per-class timing would create events on first use: this entry point runs untimed
    struct MaskGuard {
        spec_ctx* c; uint32_t saved;
        ~MaskGuard() { c->prof_mask = saved; }
    } guard{c, c->prof_mask};
    c->prof_mask = 0;
    // nothing in the workspace has to start at zero: every buffer is written by the pass before it is read
    return layer_forward_impl(c, sub, layer, x_in, n_new, x_out, w);
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

int spec_debug_gemm(const void* A, const void* W, float* C, int M, int N, int K, int tile_rows, int tile_cols,
                    void* stream) {
    if (!A || !W || !C || M <= 0 || N <= 0 || K <= 0 || tile_rows < 32 || tile_rows > 256 || tile_rows % 32 != 0 ||
        (tile_cols != 128 && tile_cols != 256))
        return fail(nullptr, SPEC_ERR_ARG, "spec_debug_gemm: bad arguments");
    GemmArgs g{};
    g.A = A; g.lda = K; g.W = W; g.C = C; g.ldc = N; g.M = M; g.N = N; g.K = K; g.epilogue = EPI_STORE_F32;
    g.force_max_rows = tile_rows; g.force_wn_t = tile_cols / 64;
    HIPCHK(nullptr, launch_gemm_mfma_bf16(g, (hipStream_t)stream));
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
