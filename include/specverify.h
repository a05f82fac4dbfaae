/*
 * specverify — C ABI of the MI355X (gfx950) speculative draft/verify library.
 *
 * The library implements the decode-phase hot path of SpecOffload (arXiv 2505.10259):
 * a small draft model resident in HBM proposes k candidate tokens per sequence, the
 * large target model scores all k+1 positions in ONE forward pass while its layer
 * weights stream from pinned host memory into a capped HBM budget, and an accept/reject
 * kernel keeps the longest valid prefix plus one token from the target (Section 2.2;
 * Appendix A.1 "Generated Tokens").  Two sub-batches can be interleaved so that one is
 * drafted while the other is verified (Section 4.1.2).
 *
 * Conventions
 *   - Every function returns SPEC_OK (0) or a negative spec_status; nothing throws or
 *     aborts.  spec_last_error() returns a message for the last failure (ctx may be NULL
 *     for failures of spec_init and of the context-free calls).
 *   - "host" pointers are ordinary CPU pointers, "device" pointers are HBM addresses on
 *     the current HIP device.  The library never takes ownership of caller buffers.
 *   - One context is driven from one host thread.  spec_draft / spec_verify only ENQUEUE
 *     work on the context's streams; results are valid after spec_sync().
 *   - There is no CPU fallback: every step runs in HIP kernels of this library.
 *
 * Host weight format.  All matrices are row-major [out_features, in_features] (the
 * contraction dimension is contiguous); elements are IEEE f32 or bf16 bit patterns
 * (spec_model_shape.dtype); every tensor starts at a multiple of 128 elements.
 *   layer blob:  g1[d] | wqkv[(Hq+2Hkv)*dh, d] (q rows, k rows, v rows) | wo[d, Hq*dh]
 *                | g2[d] | wr[E, d] (only if E > 0)
 *                | per expert e (once if E == 0): w1_e[F, d] (gate) | w3_e[F, d] (up) | w2_e[d, F]
 *                (an attn_only shape ends after wo)
 *   global blob: emb[V, d] | gf[d] | head[V, d]
 * spec_layer_blob_elems() / spec_global_blob_elems() give the sizes.
 */
#ifndef SPECVERIFY_H
#define SPECVERIFY_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spec_ctx spec_ctx;

typedef enum {
    SPEC_OK = 0,
    SPEC_ERR_ARG = -1,       /* NULL pointer, value out of range */
    SPEC_ERR_SHAPE = -2,     /* model shape not supported / draft does not match target */
    SPEC_ERR_BUDGET = -3,    /* HBM weight budget cannot hold draft + globals + staging ring */
    SPEC_ERR_CAPACITY = -4,  /* batch, k, context or KV pages exceed what spec_init sized */
    SPEC_ERR_HIP = -5,       /* a HIP runtime call failed (message has the HIP error) */
    SPEC_ERR_STATE = -6      /* call order violated (e.g. verify before prefill), or the context is unusable
                                because an earlier target pass failed part-way through its streamed layers */
} spec_status;

enum { SPEC_F32 = 0, SPEC_BF16 = 1 };
enum { SPEC_GREEDY = 0, SPEC_SAMPLE = 1 };
enum {
    SPEC_FLAG_NO_OVERLAP = 1,      /* serialise weight copies and compute (time-breakdown runs) */
    SPEC_FLAG_SIMPLE_KERNELS = 2,  /* use the plain (non-MFMA) kernels also for bf16 (debugging) */
    SPEC_FLAG_POISON_RELEASED = 4, /* checking aid for the streamer: a staging slot is overwritten with NaN
                                      bit patterns (by a kernel on the compute stream) as soon as the piece
                                      in it has been released, before the next copy may land there; results
                                      must not change */
    SPEC_FLAG_PIN_ATTENTION = 8    /* piece staging only: placement of the paper's own decoding phase
                                      (Section 4.1.2; Appendix A.1, decoding-phase memory: "only the MoE
                                      FFN parameters" of the target cross the link): the attention part
                                      (norm gains, QKV, O, router) of EVERY layer is resident, the rest of
                                      the budget pins whole expert sets from layer 0 on, and only expert
                                      parameters stream.  The budget must hold them: else SPEC_ERR_BUDGET */
};

/* Limits of this build (checked by spec_init / the size functions, SPEC_ERR_SHAPE or SPEC_ERR_ARG):
 *   n_experts 0 or 2..8 (the routing and sorting kernels keep one counter set per expert id 0..7),
 *   top_k 2, head_dim even and <= 256 (the MFMA attention and the fused rotary epilogue need 128),
 *   k_max <= 16 (spec_stats.accept_hist has 17 bins), n_sub_batches 1 or 2.
 *
 * KV pages are owned statically: spec_init sizes each (model, sub-batch) pool for batch_max sequences of
 * ctx_max + k_max + 2 positions and gives sequence b the fixed pages {p * batch_max + b}; there is no
 * page allocator, so no call can run out of pages at run time.  A sequence cannot outgrow its pages
 * either: spec_prefill refuses prompt + max_new > ctx_max (SPEC_ERR_CAPACITY), commits are clipped to
 * max_new, and a verify pass writes at most k_max positions past the committed length.
 *
 * Workspaces: a context has ONE activation workspace for target passes and ONE for draft passes, shared
 * by both sub-batches.  This is safe because every target pass of either sub-batch is enqueued on the
 * compute stream and every draft pass on the draft stream, each in call order; callers that pass their
 * own streams must not enqueue work of their own that touches library buffers. */

typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    int32_t n_experts;   /* 0 = dense SwiGLU FFN */
    int32_t top_k;       /* must be 2 when n_experts > 0 */
    int32_t attn_only;   /* 1: layers are attention-only (draft truncation) */
    int32_t dtype;       /* SPEC_F32 | SPEC_BF16: weight storage and GEMM input type */
    float rope_theta, rms_eps;
} spec_model_shape;

typedef struct {
    const void* const* layer_blobs; /* host, [n_layers] pointers, format above */
    const void* global_blob;        /* host */
} spec_host_weights;

typedef struct {
    int64_t hbm_weight_budget_bytes; /* cap on target layers held in HBM + staging ring + draft +
                                        globals; 0 = no cap (everything resident) */
    int32_t n_sub_batches;           /* 1 or 2 */
    int32_t batch_max;               /* sequences per sub-batch */
    int32_t k_max;                   /* largest k of spec_draft / spec_verify */
    int32_t ctx_max;                 /* largest prompt + new tokens of a sequence */
    int32_t page_tokens;             /* KV page size in tokens, a multiple of 16 (0 = default 64); the MFMA
                                        attention kernel takes powers of two from 32 on, other sizes
                                        run on the plain kernel */
    int32_t mode;                    /* SPEC_GREEDY | SPEC_SAMPLE */
    float temperature;               /* SPEC_SAMPLE: divides draft and target logits alike */
    uint64_t seed;                   /* SPEC_SAMPLE: Philox key */
    int32_t n_ring_slots;            /* staging for streamed parameters.  0 (default): piece staging: a
                                        layer crosses the link as its attention part and one piece per
                                        expert through n_piece_slots slots of one expert each, and the
                                        HBM this frees pins more layers plus the leading pieces of one
                                        further layer (Section 4.2, Adaptive Tensor Placement).
                                        n >= 1: n whole-layer slots, whole layers pinned only */
    int32_t flags;                   /* SPEC_FLAG_* */
    int32_t prefill_chunk;           /* prompt positions of every sequence per attention launch of the prefill,
                                        1..64 (0 = default: 64 on the MFMA path, fewer on the plain kernels) */
    void* compute_stream;            /* hipStream_t handles, or NULL to let the library create */
    void* copy_stream;               /* weight copies alternate between this stream and a second one
                                        that the library creates (keeps the link busy between copies) */
    void* draft_stream;
    int32_t n_piece_slots;           /* piece staging: slots in the ring, 2..16 (0 = default, 3) */
    int32_t prefill_group_rows;      /* prefill: rows (chunks x sequences x prefill_chunk) whose feed-forward part
                                        runs as one set of expert launches (0 = default, 32768; temporary
                                        HBM grows with it) */
} spec_runtime_cfg;

typedef struct {
    int64_t bytes_streamed;          /* host->HBM weight bytes copied since init/reset_stats */
    int64_t layers_streamed;         /* layer uses whose last streamed piece has been copied */
    int64_t resident_layers;         /* target layers held in HBM for good */
    int64_t hbm_weight_bytes;        /* resident layers + ring + draft + globals */
    int64_t rounds;                  /* spec_verify calls */
    int64_t committed_tokens;        /* tokens appended to sequences by spec_verify */
    int64_t accept_hist[17];         /* accept_hist[n]: sequence-rounds that kept n candidates */
    double copy_busy_ms;             /* time with at least one weight copy in flight (event-timed) */
    int64_t pinned_piece_bytes;      /* piece staging: bytes of the partly resident layer held in HBM */
} spec_stats;

/* ---- sizes (pure host arithmetic; usable without a GPU) -------------------------------- */
int64_t spec_layer_blob_elems(const spec_model_shape* s);   /* <0 on bad shape */
int64_t spec_global_blob_elems(const spec_model_shape* s);
/* Number of target layers that stay wholly resident under `budget` bytes given the draft shape
 * (may be NULL) and the staging ring (n_ring_slots as in spec_runtime_cfg: 0 = piece staging with
 * the default number of slots); writes the bytes that cross the link per pass to
 * *streamed_bytes_per_pass if not NULL (with piece staging the leading pieces of the first streamed
 * layer that still fit are pinned too and do not count).  Mirrors the decoding-phase memory
 * constraint (Appendix A.1, "Memory constraint"): resident target parameters + draft parameters
 * must fit the GPU budget.  <0 on error. */
int64_t spec_plan_residency(const spec_model_shape* target, const spec_model_shape* draft,
                            int64_t budget, int32_t n_ring_slots, int64_t* streamed_bytes_per_pass);

/* What spec_init would place where for `cfg` (hbm_weight_budget_bytes, n_ring_slots, n_piece_slots and
 * flags are read): the adaptive tensor placement of Section 4.2 at piece granularity.  Host arithmetic. */
typedef struct {
    int64_t resident_layers;         /* target layers wholly in HBM */
    int64_t pinned_piece_bytes;      /* pieces of the other layers held in HBM (leading pieces of the first
                                        streamed layer; with SPEC_FLAG_PIN_ATTENTION every attention part) */
    int64_t streamed_bytes_per_pass; /* what crosses the host link in one target pass */
    int64_t ring_bytes;              /* staging slots */
    int64_t fixed_bytes;             /* globals + draft layers */
    int32_t n_slots;                 /* staging slots (0: nothing streams) */
    int32_t piece_staging;           /* 1: pieces, 0: whole layers */
} spec_placement;
/* Errors: SPEC_ERR_SHAPE, SPEC_ERR_BUDGET (out is still filled with the sizes that did not fit). */
int spec_plan_placement(const spec_model_shape* target, const spec_model_shape* draft,
                        const spec_runtime_cfg* cfg, spec_placement* out);

/* ---- pinned host memory ----------------------------------------------------------------- */
/* Weights handed to spec_init must live in page-locked memory for the copies to run
 * asynchronously at link rate (the paper pins host tensors for the same reason, Section 4.2).
 * These allocate/free such memory (hipHostMalloc). */
int spec_host_alloc(size_t bytes, void** out_host);
int spec_host_free(void* host);

/* ---- lifetime --------------------------------------------------------------------------- */
/* Creates a context on the current device.  `draft` / `draft_w` may be NULL (no draft model: only
 * spec_verify with caller-supplied candidates, spec_layer_forward, spec_accept are usable).  The
 * target's host blobs are NOT copied: streamed layers are read from them on every pass, so they
 * must outlive the context.  Draft layers (their attention part, or whole layers) and the global
 * blob are copied to HBM once; if draft_w->global_blob == target_w->global_blob the copy is shared.
 * Errors: SPEC_ERR_ARG, SPEC_ERR_SHAPE, SPEC_ERR_BUDGET, SPEC_ERR_HIP. */
int spec_init(const spec_model_shape* target, const spec_model_shape* draft,
              const spec_host_weights* target_w, const spec_host_weights* draft_w,
              const spec_runtime_cfg* cfg, spec_ctx** out);
void spec_destroy(spec_ctx* ctx);
const char* spec_last_error(const spec_ctx* ctx);

/* ---- sequence set-up -------------------------------------------------------------------- */
/* Loads B prompts (host, ragged: tokens[cu_lens[b] .. cu_lens[b+1])), each >= 1 token, into
 * sub-batch `sub`, and fills the target and draft KV caches for all prompt tokens but the last
 * one, layer by layer (each streamed layer is fetched once for the whole batch — the
 * load-once/run-many-micro-batches order of the prefill phase, Section 4.1.1).  Every sequence
 * will stop after `max_new` new tokens.  Blocks until done.
 * Errors: SPEC_ERR_CAPACITY if B > batch_max or a prompt + max_new > ctx_max. */
int spec_prefill(spec_ctx* ctx, int sub, const int32_t* tokens, const int32_t* cu_lens, int B,
                 int max_new);
/* Layer microbenchmark set-up: declares B sequences whose layer-`layer` target KV cache already
 * holds `ctx_len` positions, copied from device arrays k_ctx, v_ctx [B, Hkv, ctx_len, dh] (model
 * dtype; keys already rotated).  Sets every sequence length to ctx_len + 1. */
int spec_kv_import(spec_ctx* ctx, int sub, int layer, const void* k_ctx_dev, const void* v_ctx_dev,
                   int B, int ctx_len);
int spec_reset(spec_ctx* ctx, int sub);

/* ---- the hot path ----------------------------------------------------------------------- */
/* Draft k candidates for every sequence of sub-batch `sub` with the HBM-resident draft model
 * (k sequential decode steps on the draft stream; the first step also re-feeds the previous
 * token so that the draft cache catches up after a fully accepted round).  Candidates are kept
 * inside the context for the following spec_verify and, if draft_tokens_dev != NULL, also
 * written there ([B, k] int32, device).  In SPEC_SAMPLE mode candidates are inverse-CDF draws
 * from softmax(z/temperature) and the draft logits are kept for the acceptance test. */
int spec_draft(spec_ctx* ctx, int sub, int k, int32_t* draft_tokens_dev);

/* Verify: one target forward over B x (k+1) tokens — [last committed token, candidates] per
 * sequence — streaming non-resident layers through the staging ring, then accept/reject:
 *   greedy: n = longest prefix with candidate_i == argmax(target logits at i-1) (lowest id wins
 *           ties), next = argmax at n                       (Section 2.2; Appendix A.1);
 *   sample: candidate_i kept iff u*q_i(c_i) < p_{i-1}(c_i); on the first rejection next is drawn
 *           from max(0, p_n - q_{n+1}) renormalised, after k kept from p_k (the rule of the
 *           speculative-sampling works the paper cites in Section 2.2).
 * Then commits min(n+1, remaining) tokens per sequence and rolls both KV caches back to the
 * committed length.  draft_tokens_dev == NULL uses the candidates of the last spec_draft(sub);
 * otherwise [B, k] int32 device candidates supplied by the caller (greedy mode only).
 * n_accepted_dev / next_token_dev: [B] int32 device outputs, may be NULL. */
int spec_verify(spec_ctx* ctx, int sub, const int32_t* draft_tokens_dev, int k,
                int32_t* n_accepted_dev, int32_t* next_token_dev);

/* Blocks until all work enqueued for `sub` (sub < 0: everything) is complete. */
int spec_sync(spec_ctx* ctx, int sub);

/* One time slot of the interleaved schedule (Section 4.1.2, model level): verify the current
 * sub-batch with the candidates drafted for it in the previous slot while the draft model
 * proposes candidates for the other sub-batch; then the roles swap.  With one sub-batch it is
 * draft followed by verify.  k = 0 (greedy mode only) is plain decoding, the baseline without
 * speculation: one verify pass of the current sub-batch with no candidates, one token per
 * sequence, sub-batches taking turns.  Enqueue only. */
int spec_step(spec_ctx* ctx, int k);

/* ---- results / introspection ------------------------------------------------------------ */
/* Lengths (prompt + committed new tokens) of the B sequences of `sub` -> host [B].  Syncs. */
int spec_get_lengths(spec_ctx* ctx, int sub, int32_t* out_host);
/* Tokens of sequence `seq` (prompt included) -> host; writes min(length, cap). Syncs. */
int spec_get_tokens(spec_ctx* ctx, int sub, int seq, int32_t* out_host, int cap, int* out_len);
int spec_get_stats(spec_ctx* ctx, spec_stats* out);
int spec_reset_stats(spec_ctx* ctx);
/* Target logits of the last spec_verify(sub): device float [B, k+1, V] copied to out_dev. */
int spec_debug_logits(spec_ctx* ctx, int sub, float* out_dev);
/* Draft logits of the last spec_draft(sub) in SPEC_SAMPLE mode: device float [B, k, V]. */
int spec_debug_draft_logits(spec_ctx* ctx, int sub, float* out_dev);

/* ---- per-kernel-class timing ------------------------------------------------------------------ */
/* Kernel classes of the verify pass (the steps of one target layer, the LM head, accept/reject)
 * and the draft pass as a whole.  With a class enabled, its launches are bracketed by HIP events on
 * the stream they run on; spec_profile_read synchronises and returns accumulated milliseconds and
 * launch counts per class (arrays of SPEC_PROF_N), optionally resetting them. */
enum {
    SPEC_PROF_NORM = 0, SPEC_PROF_QKV, SPEC_PROF_ROPE, SPEC_PROF_ATTN, SPEC_PROF_OPROJ, SPEC_PROF_ROUTE,
    SPEC_PROF_MOE1, SPEC_PROF_MOE2, SPEC_PROF_HEAD, SPEC_PROF_ACCEPT, SPEC_PROF_DRAFT, SPEC_PROF_N
};
int spec_profile_enable(spec_ctx* ctx, uint32_t category_mask);
int spec_profile_read(spec_ctx* ctx, double* ms_out, int64_t* launches_out, int reset);

/* ---- stand-alone pieces (tests, microbenchmarks) ----------------------------------------- */
/* The accept/reject rule on given logits (all device pointers):
 *   p_logits [B, k+1, V] float; q_logits [B, k, V] float or NULL (NULL = greedy rule);
 *   draft_tokens [B, k] int32; u_accept [B, k] and u_resample [B, k+1] float uniforms in [0,1)
 *   (sampling only; both NULL = draw them from Philox4x32-10 with key `seed`, counter
 *   (round, seq_base + b, position, 0), word 1 -> accept, word 2 -> resample);
 *   outputs n_accepted [B], next_token [B] int32.  Runs on `stream` (hipStream_t or NULL). */
int spec_accept(const float* p_logits, const float* q_logits, const int32_t* draft_tokens,
                const float* u_accept, const float* u_resample, float temperature, uint64_t seed,
                uint32_t round, uint32_t seq_base, int B, int k, int V, int32_t* n_accepted,
                int32_t* next_token, void* stream);
/* Philox4x32-10 uniforms exactly as the sampling path draws them: out_dev [B, k+1, 3] float
 * (draft, accept, resample uniform of position i). */
int spec_philox_uniforms(uint64_t seed, uint32_t round, uint32_t seq_base, int B, int k,
                         float* out_dev, void* stream);
/* One decoder layer of the verify pass (the in-HBM layer microbenchmark): residual-stream rows
 * x_in_dev [B*n_new, d] (model dtype) for n_new new tokens per sequence at positions
 * length-1 .. length-2+n_new -> x_out_dev float [B*n_new, d]; appends the rows' K/V to the cache
 * but does not change sequence lengths.  Layer `layer` must be resident (no weight budget). */
int spec_layer_forward(spec_ctx* ctx, int sub, int layer, const void* x_in_dev, int n_new,
                       float* x_out_dev);
/* spec_layer_forward for callers that cannot allocate device memory or have it allocated under them
 * (code running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same
 * pass with the same kernels and the same results, but its activation workspace (normalised rows, q,
 * attention output, rotary table, routing and sort order, expert intermediates and outputs) lives in a
 * static device array of SPEC_STATIC_SCRATCH_BYTES that every GPU the library is loaded on holds until
 * the process ends, instead of in the context's workspace.  The call allocates nothing (no hipMalloc,
 * hipFree, events or library allocations) and runs without per-class timing.  Inputs, output, weights,
 * KV pages and sequence state are the context's and the caller's as before.
 * Limit: the workspace of B * n_new rows of the context's model must fit the array, otherwise
 * SPEC_ERR_CAPACITY and nothing is enqueued (a Mixtral-8x7B-shaped layer takes about 140 KB per row:
 * some 470 rows).  All contexts on one GPU share the array and it keeps the last call's contents (no
 * part of it needs clearing: a pass writes everything it reads); calls that overlap on one GPU — from
 * two contexts or two streams — race.  Other errors as spec_layer_forward. */
#define SPEC_STATIC_SCRATCH_BYTES (64u << 20)
int spec_layer_forward_static(spec_ctx* ctx, int sub, int layer, const void* x_in_dev, int n_new,
                              float* x_out_dev);
/* Router decisions of the last spec_layer_forward / verify layer pass: expert ids [T, 2] int32
 * and weights [T, 2] float copied to device buffers (either may be NULL). */
int spec_debug_routing(spec_ctx* ctx, int sub, int32_t* ids_dev, float* weights_dev, int T);
/* Testing aid for parity runs of MoE models: the NEXT target pass of sub-batch `sub` (spec_prefill,
 * spec_verify or spec_layer_forward) takes the two experts of every row from ids_dev instead of its own
 * top-2; the mixing weights still come from the pass's own router logits of those two experts.  A
 * reference run and this library then follow the same experts even where two router logits are closer
 * than the arithmetic noise between the two, and everything downstream stays comparable.
 *   ids_dev: device int32 [n_layers, rows_per_layer, 2]; it must stay valid until the pass has completed
 *            (spec_sync).  A row whose pair is not two distinct ids in [0, n_experts) keeps its own top-2.
 *   row index inside a layer: verify / layer_forward: b * n_new + i;
 *                             prefill: (chunk * B + b) * prefill_chunk + q for prompt position
 *                             chunk * prefill_chunk + q (spec_layer_forward reads layer index `layer`).
 * The setting is consumed by that pass; NULL cancels it.  Errors: SPEC_ERR_ARG (rows_per_layer smaller
 * than the rows of the pass, reported by the pass), SPEC_ERR_STATE (dense target). */
int spec_debug_force_routing(spec_ctx* ctx, int sub, const int32_t* ids_dev, int rows_per_layer);
/* Plain GEMM entry for kernel tests and roofline runs: C[M,N] (float) = A[M,K] * W[N,K]^T with
 * A, W device arrays of `dtype`; uses the same kernels as the layer.  */
int spec_gemm(const void* A_dev, const void* W_dev, float* C_dev, int M, int N, int K, int dtype,
              int flags, void* stream);
/* Tests only: the bf16 MFMA kernel of spec_gemm with the tile shape given instead of chosen: rows of A are
 * cut into the fewest equal tiles of at most tile_rows rows (32, 64, ... 256) and the columns into tiles
 * of tile_cols (128 or 256), so that a test can visit every tile variant of the kernel.  A, W: device
 * bf16 [M,K] and [N,K]; C: device float [M,N].  Shapes the MFMA kernel does not take (K not a multiple
 * of 64, N not a multiple of 4, ...) fall to the plain kernel as in spec_gemm.  Errors: SPEC_ERR_ARG. */
int spec_debug_gemm(const void* A_dev, const void* W_dev, float* C_dev, int M, int N, int K, int tile_rows,
                    int tile_cols, void* stream);
/* Measures host->HBM copy bandwidth of pinned memory: copies `bytes` from a pinned buffer `reps`
 * times with hipMemcpyAsync and returns GB/s (1e9) in *gbps — the denominator of the link
 * fraction (the paper's planner likewise profiles the CPU-GPU channel first, Section 3). */
int spec_measure_link(size_t bytes, int reps, double* gbps);

/* ---- ParaSpec planner (Section 4.3; Appendix A.1 "ParaSpec Planner") ----------------------- */
/* Host arithmetic only; usable without a GPU.  The profile holds the quantities the appendix's cost
 * model is written in; times in seconds, sizes in bytes, all measured or computed by the caller.
 * The fields after v_draft_kv generalise the appendix's per-batch constants and are 0 for the
 * relations exactly as printed. */
typedef struct {
    int32_t n_layer;              /* target decoder layers */
    int32_t n_layer_streamed;     /* of which this many stream their weights every pass (the rest are
                                     resident: no transfer time) */
    int32_t l_input;              /* prompt tokens per sequence */
    int32_t n_generate;           /* tokens to generate per sequence */
    int32_t bs_max;               /* search bound: batch size 1..bs_max */
    int32_t n_cand_max;           /* search bound: candidates per round 1..n_cand_max */
    double p_accept;              /* probability that one candidate token is accepted, 0 <= p < 1 */
    double t_c2g_para;            /* prefill: streaming the whole target once */
    double t_gpu_prefill_comp;    /* prefill: GPU compute of one prefill batch */
    double t_ffn_c2g;             /* decoding: streaming one layer's weights */
    double t_ffn_gpu;             /* decoding: GPU compute of one layer in one verify pass */
    double t_attention_unit;      /* decoding: attention time per (sequence, candidate) per layer when
                                     attention is not hidden behind the transfer (the paper's CPU
                                     attention term) */
    double t_draft_prefill;       /* first draft step of one draft batch */
    double t_draft_decoding;      /* each further draft step of one draft batch */
    double gpu_mem_capacity;
    double v_target_prefill;      /* target parameters on the GPU during prefill */
    double v_target_kv;           /* target KV bytes per token held on the GPU during prefill */
    double v_target_ffn;          /* target parameters on the GPU during decoding */
    double v_draft;               /* draft parameters */
    double v_draft_kv;            /* draft KV bytes per token */
    double t_ffn_gpu_per_token;   /* + per verified token (bs * (n_cand + 1)) on t_ffn_gpu */
    double t_draft_per_seq;       /* + per sequence of the draft batch on both draft step times */
    double t_prefill_comp_per_seq;/* + per sequence of the prefill batch on t_gpu_prefill_comp */
    double v_target_kv_decoding;  /* target KV bytes per token held on the GPU during decoding */
} spec_planner_profile;

typedef struct {
    int32_t feasible;             /* 0: no point of the search space satisfies both memory constraints */
    int32_t bs, bs_prefill, bs_draft, n_cand;   /* the chosen parameters */
    int32_t n_iter;               /* rounds: ceil(n_generate / expected_tokens) */
    double throughput;            /* N_generated / T_generation, tokens per second */
    double expected_tokens;       /* E[n_generated] per sequence per round */
    double t_prefill, t_round, t_target_decoding, t_draft;   /* seconds; t_round = max of the last two */
    double v_prefill, v_decoding; /* bytes at the chosen parameters */
} spec_plan;

/* Chooses (bs, bs_prefill, bs_draft, n_cand) maximising
 *     throughput = bs * n_iter * E[n_generated] / (T_prefill + n_iter * max(T_target_decoding, T_draft))
 * subject to V_prefill <= gpu_mem_capacity and V_decoding <= gpu_mem_capacity, with every term as in
 * Appendix A.1 (E[n_generated] is the sum over the appendix's probability mass function, i.e.
 * (1 - p^(n_cand+1)) / (1 - p); the closed form printed there does not equal that sum).  Equal
 * throughputs: smallest bs, then smallest n_cand, then largest bs_prefill, then largest bs_draft.
 * Returns SPEC_ERR_ARG for NULL pointers, non-positive sizes or bounds, p outside [0, 1) or negative
 * times; an infeasible problem is SPEC_OK with out->feasible = 0. */
int spec_plan_paraspec(const spec_planner_profile* profile, spec_plan* out);
/* The cost model at one point (same relations, no search): fills *out for the given parameters;
 * out->feasible tells whether both memory constraints hold there. */
int spec_plan_evaluate(const spec_planner_profile* profile, int32_t bs, int32_t bs_prefill,
                       int32_t bs_draft, int32_t n_cand, spec_plan* out);

#ifdef __cplusplus
}
#endif
#endif /* SPECVERIFY_H */
