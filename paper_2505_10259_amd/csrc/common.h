// Internal declarations shared by the HIP sources of the specverify library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/specverify.h"

namespace sv {

// ---- bf16 storage type ------------------------------------------------------------------
struct bf16 {
    uint16_t bits;
};

__host__ __device__ inline float bf16_to_f32(bf16 v) {
    union { uint32_t u; float f; } c;
    c.u = (uint32_t)v.bits << 16;
    return c.f;
}
// round to nearest even; NaN stays NaN
__host__ __device__ inline bf16 f32_to_bf16(float f) {
    union { uint32_t u; float f; } c;
    c.f = f;
    uint32_t u = c.u;
    bf16 r;
    if ((u & 0x7fffffffu) > 0x7f800000u) { r.bits = (uint16_t)((u >> 16) | 0x40u); return r; }
    u += 0x7fffu + ((u >> 16) & 1u);
    r.bits = (uint16_t)(u >> 16);
    return r;
}

template <typename T> __host__ __device__ inline float to_f32(T v);
template <> __host__ __device__ inline float to_f32<float>(float v) { return v; }
template <> __host__ __device__ inline float to_f32<bf16>(bf16 v) { return bf16_to_f32(v); }
template <typename T> __host__ __device__ inline T from_f32(float v);
template <> __host__ __device__ inline float from_f32<float>(float v) { return v; }
template <> __host__ __device__ inline bf16 from_f32<bf16>(float v) { return f32_to_bf16(v); }

constexpr int WAVE = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
    return v;
}

// ---- KV page pool geometry -----------------------------------------------------------------
// One pool per (model, sub-batch).  A (layer, page, kv_head) block holds the page's tokens in
// sub-blocks of 32 (see sub_tokens); each sub-block is its keys followed by its values:
//   keys   [slot][dim]   -- a key row is contiguous (the contraction dimension of q.k)
//   values [dim][slot]   -- TRANSPOSED, so that consecutive positions of one dimension are
//                           contiguous (the contraction dimension of p.v): both MFMA operands of
//                           the attention kernel are then 16-byte pieces of memory rows.
// A sequence owns pages_per_seq logical pages listed in its page-table row.
struct KvGeom {
    int n_kv_heads, head_dim, page_tokens, pages_per_seq;
    int64_t n_pages;        // physical pages per layer
    __host__ __device__ int64_t layer_elems() const {
        return n_pages * (int64_t)n_kv_heads * 2 * page_tokens * head_dim;
    }
    __host__ __device__ int64_t block(int64_t page, int kvh) const {
        return (page * n_kv_heads + kvh) * 2 * (int64_t)page_tokens * head_dim;
    }
    // Inside a (page, kv head) block the tokens are cut into sub-blocks of 32 (the attention kernel's
    // key tile; the whole page if its size is not a multiple of 32), and each sub-block holds its keys
    // [slot][dim] followed by its values transposed [dim][slot]: one key tile of K and V is then one
    // contiguous run of 2 * 32 * head_dim elements in HBM.
    __host__ __device__ int sub_tokens() const { return page_tokens % 32 == 0 ? 32 : page_tokens; }
    __host__ __device__ int64_t sub_block(int64_t page, int kvh, int slot) const {
        return block(page, kvh) + (int64_t)(slot / sub_tokens()) * 2 * sub_tokens() * head_dim;
    }
    __host__ __device__ int64_t k_off(int64_t page, int kvh, int slot) const {
        return sub_block(page, kvh, slot) + (int64_t)(slot % sub_tokens()) * head_dim;
    }
    __host__ __device__ int64_t v_off(int64_t page, int kvh, int slot, int dim) const {
        return sub_block(page, kvh, slot) + (int64_t)sub_tokens() * head_dim + (int64_t)dim * sub_tokens() +
               slot % sub_tokens();
    }
};

// ---- GEMM problem description -------------------------------------------------------------
// C[M,N] (+)= A[M,K] * W[N,K]^T ; all row-major; optional row gather on A; optional grouping:
// rows are split into groups by `group_offsets` (device, [n_groups+1]) and group g uses weights
// W + g * w_group_stride (elements).
enum GemmEpilogue {
    EPI_STORE_F32 = 0,   // C float = acc
    EPI_ADD_F32 = 1,     // C float += acc           (residual accumulate; one writer per element)
    EPI_STORE_T = 2,     // C (model dtype) = acc
    EPI_SWIGLU_T = 3,    // C (model dtype)[M, N] = silu(A W^T) * (A W3^T)   (W3 = second weight)
    EPI_ROPE_KV = 4      // QKV projection (bf16 MFMA kernel, head_dim 128 only): columns are
                         // [q heads | k heads | v heads]; q and k are rotated (pair (i, i + 64)) with the
                         // row's cos/sin table, q goes to rope.q_out, k and v to the row's KV page slot
};

struct RopeKvArgs {               // EPI_ROPE_KV: what rope_kv_kernel takes, minus the f32 qkv buffer
    const float2* cs;             // [M, 64] (cos, sin) per row
    const int32_t* row_pos;       // [M] absolute position of each row (< 0: row inactive)
    const int32_t* page_table;    // [B, pages_per_seq]
    void* q_out;                  // [M, n_q_heads * 128] model dtype
    void* kv_layer;               // KV pool of this layer
    KvGeom geom;
    int n_new, n_q_heads;
};

struct GemmArgs {
    const void* A; int64_t lda;
    const int32_t* a_rows;          // nullable: A row of output row m is a_rows[m]
    const void* W; const void* W3;  // [N,K] each, ld = K
    void* C; int64_t ldc;
    int M, N, K;
    int epilogue;
    const int32_t* group_offsets;   // nullable
    int n_groups;
    int64_t w_group_stride;         // elements between consecutive groups' W (and W3)
    int m_upper;                    // grouped: upper bound on total rows (grid sizing)
    int m_expected;                 // grouped: expected rows per group if known (tile-height choice), else 0
    RopeKvArgs rope;                // EPI_ROPE_KV only
    int force_max_rows, force_wn_t; // tests: tile height limit (multiple of 32, <= 256) and width (2 or 4 x 64 columns); 0 = the launcher's choice
};

// launchers (kernels_*.hip) -------------------------------------------------------------------
hipError_t launch_gemm_simple(const GemmArgs& a, int dtype, hipStream_t st);
hipError_t launch_gemm_mfma_bf16(const GemmArgs& a, hipStream_t st);   // gemm_mfma.hip

struct AttnArgs {
    const void* q;            // [T, Hq*dh] model dtype
    void* out;                // [T, Hq*dh] model dtype
    const void* kv_layer;     // pool base of this layer
    const int32_t* page_table;// [B, pages_per_seq]
    const int32_t* row_pos;   // [T] absolute position of each row (<0: row inactive)
    KvGeom geom;
    int B, n_new, n_q_heads;
    float scale;
};
hipError_t launch_attention_simple(const AttnArgs& a, int dtype, hipStream_t st);
hipError_t launch_attention_mfma_bf16(const AttnArgs& a, hipStream_t st);   // attn_mfma.hip

hipError_t launch_embed(const void* emb, const int32_t* tok, float* x, int T, int d, int vocab,
                        int dtype, hipStream_t st);
hipError_t launch_cast_to_f32(const void* in, float* out, int64_t n, int dtype, hipStream_t st);
hipError_t launch_fill_words(void* p, size_t n_words, uint32_t value, hipStream_t st);
// x[t] += w[t,0]*y[slot[t,0]] + w[t,1]*y[slot[t,1]]  (if y), then h[t] = rmsnorm(x[t]) * g (if g)
hipError_t launch_combine_norm(float* x, const float* y, const float* wts, const int32_t* slots,
                               const void* g, void* h, int T, int d, float eps, int dtype,
                               hipStream_t st);
// RMSNorm + router in one kernel (see kernels_basic.hip); norm_route_supported tells whether it applies
bool norm_route_supported(int d, int E);
// `forced` (nullable): [T, 2] expert ids to use instead of the top-2 (weights still from the logits);
// `row_pos` (nullable): rows with a negative position are inactive and get no experts (ids -1, weights 0)
hipError_t launch_norm_route(const float* x, const void* g, void* h, const void* wr, int32_t* ids, float* wts,
                             int T, int d, int E, float eps, const int32_t* forced, const int32_t* row_pos, int dtype,
                             hipStream_t st);
hipError_t launch_rope_table(const int32_t* row_pos, float2* cs, int T, int half, float theta,
                             hipStream_t st);
hipError_t launch_rope_kv(const float* qkv, const float2* cs, const int32_t* row_pos,
                          const int32_t* page_table, void* q_out, void* kv_layer, KvGeom geom,
                          int T, int n_new, int n_q_heads, int dtype, hipStream_t st);
hipError_t launch_router(const void* h, const void* wr, int32_t* ids, float* wts, int T, int d,
                         int E, const int32_t* forced, const int32_t* row_pos, int dtype, hipStream_t st);
// counting sort of the 2T (token, choice) pairs by expert: offsets[E+1], perm[2T] (sorted row ->
// token), slots[T,2] (token choice -> sorted row)
hipError_t launch_moe_sort(const int32_t* ids, int32_t* offsets, int32_t* perm, int32_t* slots,
                           int T, int E, hipStream_t st);
hipError_t launch_kv_import(const void* k_ctx, const void* v_ctx, void* kv_layer,
                            const int32_t* page_table, KvGeom geom, int B, int ctx_len, int dtype,
                            hipStream_t st);

// sequence-state kernels (kernels_state.hip)
struct SeqState {
    int32_t* tokens;     // [B, tok_cap] committed tokens (prompt included)
    int32_t* len;        // [B] committed length
    int32_t* n_new;      // [B] new tokens so far
    int32_t* max_new;    // [B]
    int tok_cap;
};
hipError_t launch_verify_prep(SeqState s, const int32_t* draft_tokens, int k, int32_t* tok_in,
                              int32_t* row_pos, int B, hipStream_t st);
hipError_t launch_draft_prep(SeqState s, const int32_t* draft_tokens, int k, int step,
                             int32_t* tok_in, int32_t* row_pos, int B, hipStream_t st);
// seq_of (nullable): sequence whose tokens row block b of the chunk carries (the prefill's own order)
hipError_t launch_prefill_prep(const int32_t* tokens_dev, const int32_t* plen, const int32_t* seq_of, int tok_cap, int B,
                               int chunk0, int Q, int32_t* tok_in, int32_t* row_pos, hipStream_t st);
hipError_t launch_commit(SeqState s, const int32_t* draft_tokens, int k, const int32_t* n_acc,
                         const int32_t* next_tok, int64_t* hist, int64_t* committed, int B,
                         hipStream_t st);

// accept / sampling kernels (kernels_accept.hip)
struct AcceptArgs {
    const float* p_logits;   // [B, k+1, V]
    const float* q_logits;   // [B, k, V] or null (greedy)
    const int32_t* draft_tokens;  // [B, k]
    const float* u_accept;   // [B, k] or null -> philox
    const float* u_resample; // [B, k+1] or null -> philox
    float inv_tau;
    uint64_t seed; uint32_t round, seq_base;
    int B, k, V;
    int32_t* n_accepted; int32_t* next_token;
    float* row_stats;        // workspace [B, 2k+1, 2] floats (max, sumexp) — sampling only
};
hipError_t launch_accept(const AcceptArgs& a, hipStream_t st);
// draft token choice from logits rows z[b] (row stride ld): greedy argmax or inverse-CDF sample
hipError_t launch_draft_pick(const float* z, int64_t ld, int V, int B, int mode, float inv_tau,
                             uint64_t seed, uint32_t round, uint32_t seq_base, int step /*1-based*/,
                             int32_t* draft_tokens, int k, hipStream_t st);
hipError_t launch_philox_uniforms(uint64_t seed, uint32_t round, uint32_t seq_base, int B, int k,
                                  float* out, hipStream_t st);

}  // namespace sv
