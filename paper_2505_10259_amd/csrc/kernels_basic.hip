// Element-wise / gather / normalisation / routing kernels and the plain (non-MFMA) GEMM and
// attention used for f32 models.  All are HBM- or latency-bound; they are written for 64-wide
// wavefronts with coalesced row accesses.
#include <algorithm>

#include "common.h"

namespace sv {

#define DISPATCH_DTYPE(dtype, ...)                                     \
    do {                                                               \
        if ((dtype) == SPEC_F32) { using T = float; __VA_ARGS__; }     \
        else { using T = bf16; __VA_ARGS__; }                          \
    } while (0)

// ---------------------------------------------------------------------------------------------
// embedding gather: x[t,:] = Emb[tok[t],:]
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_kernel(const T* __restrict__ emb, const int32_t* __restrict__ tok,
                             float* __restrict__ x, int d, int vocab) {
    int t = blockIdx.x;
    int id = tok[t];
    id = id < 0 ? 0 : (id >= vocab ? vocab - 1 : id);
    const T* src = emb + (int64_t)id * d;
    float* dst = x + (int64_t)t * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) dst[c] = to_f32<T>(src[c]);
}

hipError_t launch_embed(const void* emb, const int32_t* tok, float* x, int T_, int d, int vocab,
                        int dtype, hipStream_t st) {
    if (T_ <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(embed_kernel<T>, dim3(T_), dim3(256), 0, st,
                                             (const T*)emb, tok, x, d, vocab));
    return hipGetLastError();
}

// fill n 32-bit words with one value (grid-stride; used to clear or poison buffers on a stream without
// a memset node, which must stay out of captured graphs)
__global__ void fill_words_kernel(uint32_t* __restrict__ p, size_t n, uint32_t v) {
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = v;
}
hipError_t launch_fill_words(void* p, size_t n_words, uint32_t v, hipStream_t st) {
    if (n_words == 0) return hipSuccess;
    const size_t blocks = std::min<size_t>((n_words + 255) / 256, 4096);
    hipLaunchKernelGGL(fill_words_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (uint32_t*)p, n_words, v);
    return hipGetLastError();
}

// 8 elements per thread (one 16-byte load of bf16 / two of f32, two 16-byte stores); the tail and
// unaligned buffers go element by element
template <typename T>
__global__ void cast_kernel(const T* __restrict__ in, float* __restrict__ out, int64_t n, int vec) {
    const int64_t i = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) * 8;
    if (i >= n) return;
    if (vec && i + 8 <= n) {
        T v[8];
        if (sizeof(T) == 2) *(uint4*)v = *(const uint4*)(in + i);
        else { *(uint4*)v = *(const uint4*)(in + i); *(uint4*)(v + 4) = *(const uint4*)(in + i + 4); }
        *(float4*)(out + i) = make_float4(to_f32<T>(v[0]), to_f32<T>(v[1]), to_f32<T>(v[2]), to_f32<T>(v[3]));
        *(float4*)(out + i + 4) = make_float4(to_f32<T>(v[4]), to_f32<T>(v[5]), to_f32<T>(v[6]), to_f32<T>(v[7]));
    } else {
        for (int64_t j = i; j < n && j < i + 8; ++j) out[j] = to_f32<T>(in[j]);
    }
}
hipError_t launch_cast_to_f32(const void* in, float* out, int64_t n, int dtype, hipStream_t st) {
    if (n <= 0) return hipSuccess;
    const int vec = (((uintptr_t)in | (uintptr_t)out) & 15) == 0;
    const int64_t threads = (n + 7) / 8;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(cast_kernel<T>, dim3((unsigned)((threads + 255) / 256)),
                                             dim3(256), 0, st, (const T*)in, out, n, vec));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// (MoE combine) + RMSNorm.  One 256-thread workgroup per row.
//   if y:  x[t] += w[t,0] * y[slot[t,0]] + w[t,1] * y[slot[t,1]]      (first choice first)
//   if g:  h[t]  = x[t] * rsqrt(mean(x[t]^2) + eps) * g               (stored in the model dtype)
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void combine_norm_kernel(float* __restrict__ x, const float* __restrict__ y,
                                    const float* __restrict__ wts, const int32_t* __restrict__ slots,
                                    const T* __restrict__ g, T* __restrict__ h, int d, float eps) {
    __shared__ float red[4];
    int t = blockIdx.x;
    float* xr = x + (int64_t)t * d;
    float ss = 0.f;
    if (y && (wts[2 * t] != 0.f || wts[2 * t + 1] != 0.f)) {       // (a row without experts has weights 0)
        float w0 = wts[2 * t], w1 = wts[2 * t + 1];
        const float* y0 = y + (int64_t)slots[2 * t] * d;
        const float* y1 = y + (int64_t)slots[2 * t + 1] * d;
        for (int c = threadIdx.x; c < d; c += blockDim.x) {
            float v = xr[c] + (w0 * y0[c] + w1 * y1[c]);
            xr[c] = v;
            ss += v * v;
        }
    } else if (g) {
        for (int c = threadIdx.x; c < d; c += blockDim.x) { float v = xr[c]; ss += v * v; }
    }
    if (!g) return;
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = red[0] + red[1] + red[2] + red[3];
    float r = 1.0f / sqrtf(tot / (float)d + eps);
    T* hr = h + (int64_t)t * d;
    for (int c = threadIdx.x; c < d; c += blockDim.x) hr[c] = from_f32<T>(xr[c] * r * to_f32<T>(g[c]));
}

// Same operation with the row held in registers (8 consecutive elements per thread and chunk, 16-byte
// loads and stores, one pass): for d % 8 == 0 and d <= 8 * 256 * COMBINE_CHUNKS.
constexpr int COMBINE_CHUNKS = 4;
template <typename T>
__global__ void __launch_bounds__(256)
combine_norm_vec_kernel(float* __restrict__ x, const float* __restrict__ y, const float* __restrict__ wts,
                        const int32_t* __restrict__ slots, const T* __restrict__ g, T* __restrict__ h, int d,
                        float eps) {
    __shared__ float red[4];
    const int t = blockIdx.x, tid = threadIdx.x;
    float* xr = x + (int64_t)t * d;
    float v[COMBINE_CHUNKS][8];
    float ss = 0.f;
    float w0 = 0.f, w1 = 0.f;
    const float* y0 = nullptr;
    const float* y1 = nullptr;
    if (y) {
        w0 = wts[2 * t]; w1 = wts[2 * t + 1];
        if (w0 == 0.f && w1 == 0.f) y = nullptr;                   // a row without experts: nothing to add
        else { y0 = y + (int64_t)slots[2 * t] * d; y1 = y + (int64_t)slots[2 * t + 1] * d; }
    }
#pragma unroll
    for (int q = 0; q < COMBINE_CHUNKS; ++q) {
        const int c = (q * 256 + tid) * 8;
        if (c < d) {
            const float4 a = *(const float4*)(xr + c), b = *(const float4*)(xr + c + 4);
            v[q][0] = a.x; v[q][1] = a.y; v[q][2] = a.z; v[q][3] = a.w;
            v[q][4] = b.x; v[q][5] = b.y; v[q][6] = b.z; v[q][7] = b.w;
            if (y) {
                const float4 p0 = *(const float4*)(y0 + c), p1 = *(const float4*)(y0 + c + 4);
                const float4 q0 = *(const float4*)(y1 + c), q1 = *(const float4*)(y1 + c + 4);
                const float e0[8] = {p0.x, p0.y, p0.z, p0.w, p1.x, p1.y, p1.z, p1.w};
                const float e1[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
                for (int e = 0; e < 8; ++e) v[q][e] = v[q][e] + (w0 * e0[e] + w1 * e1[e]);
                *(float4*)(xr + c) = make_float4(v[q][0], v[q][1], v[q][2], v[q][3]);
                *(float4*)(xr + c + 4) = make_float4(v[q][4], v[q][5], v[q][6], v[q][7]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[q][e] * v[q][e];
        }
    }
    if (!g) return;
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float r = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    T* hr = h + (int64_t)t * d;
#pragma unroll
    for (int q = 0; q < COMBINE_CHUNKS; ++q) {
        const int c = (q * 256 + tid) * 8;
        if (c < d) {
            T gv[8], hv[8];
            if (sizeof(T) == 2) *(uint4*)gv = *(const uint4*)(g + c);
            else { *(uint4*)gv = *(const uint4*)(g + c); *(uint4*)(gv + 4) = *(const uint4*)(g + c + 4); }
#pragma unroll
            for (int i = 0; i < 8; ++i) hv[i] = from_f32<T>(v[q][i] * r * to_f32<T>(gv[i]));
            if (sizeof(T) == 2) *(uint4*)(hr + c) = *(const uint4*)hv;
            else { *(uint4*)(hr + c) = *(const uint4*)hv; *(uint4*)(hr + c + 4) = *(const uint4*)(hv + 4); }
        }
    }
}

hipError_t launch_combine_norm(float* x, const float* y, const float* wts, const int32_t* slots,
                               const void* g, void* h, int T_, int d, float eps, int dtype,
                               hipStream_t st) {
    if (T_ <= 0) return hipSuccess;
    if (d % 8 == 0 && d <= 8 * 256 * COMBINE_CHUNKS) {
        DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(combine_norm_vec_kernel<T>, dim3(T_), dim3(256), 0, st, x, y,
                                                 wts, slots, (const T*)g, (T*)h, d, eps));
    } else {
        DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(combine_norm_kernel<T>, dim3(T_), dim3(256), 0, st, x, y,
                                                 wts, slots, (const T*)g, (T*)h, d, eps));
    }
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// RoPE: cos/sin table per row (positions are the same for every layer of a pass), computed in
// double so that large positions lose nothing; then rotate q,k (pair (i, i+dh/2)) and append
// k,v to the sequence's KV pages.
// ---------------------------------------------------------------------------------------------
__global__ void rope_table_kernel(const int32_t* __restrict__ row_pos, float2* __restrict__ cs,
                                  int T_, int half, double theta) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= T_ * half) return;
    int t = idx / half, i = idx % half;
    double inv = pow(theta, -(double)i / (double)half);      // theta^(-2i/dh)
    double a = (double)row_pos[t] * inv;
    double s, c;
    sincos(a, &s, &c);
    cs[idx] = make_float2((float)c, (float)s);
}
hipError_t launch_rope_table(const int32_t* row_pos, float2* cs, int T_, int half, float theta,
                             hipStream_t st) {
    int n = T_ * half;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(rope_table_kernel, dim3((n + 255) / 256), dim3(256), 0, st, row_pos, cs, T_, half,
                       (double)theta);
    return hipGetLastError();
}

template <typename T>
__global__ void rope_kv_kernel(const float* __restrict__ qkv, const float2* __restrict__ cs,
                               const int32_t* __restrict__ row_pos,
                               const int32_t* __restrict__ page_table, T* __restrict__ q_out,
                               T* __restrict__ kv_layer, KvGeom geom, int n_new, int n_q_heads) {
    int t = blockIdx.x;
    int dh = geom.head_dim, half = dh >> 1, Hkv = geom.n_kv_heads;
    int n_heads = n_q_heads + 2 * Hkv;
    int pos = row_pos[t];
    int b = t / n_new;
    const float* row = qkv + (int64_t)t * n_heads * dh;
    int64_t page = -1;
    int slot = 0;
    if (pos >= 0) {
        int lp = pos / geom.page_tokens;
        if (lp < geom.pages_per_seq) { page = page_table[b * geom.pages_per_seq + lp]; slot = pos % geom.page_tokens; }
    }
    for (int idx = threadIdx.x; idx < n_heads * half; idx += blockDim.x) {
        int hd = idx / half, i = idx % half;
        float a = row[hd * dh + i], bb = row[hd * dh + i + half];
        if (hd < n_q_heads + Hkv) {
            float2 c = cs[t * half + i];
            float ra = a * c.x - bb * c.y, rb = bb * c.x + a * c.y;
            a = ra; bb = rb;
        }
        if (hd < n_q_heads) {
            T* dst = q_out + (int64_t)t * n_q_heads * dh + hd * dh;
            dst[i] = from_f32<T>(a); dst[i + half] = from_f32<T>(bb);
        } else if (page >= 0) {
            if (hd < n_q_heads + Hkv) {
                T* dst = kv_layer + geom.k_off(page, hd - n_q_heads, slot);
                dst[i] = from_f32<T>(a); dst[i + half] = from_f32<T>(bb);
            } else {
                int kvh = hd - n_q_heads - Hkv;
                kv_layer[geom.v_off(page, kvh, slot, i)] = from_f32<T>(a);
                kv_layer[geom.v_off(page, kvh, slot, i + half)] = from_f32<T>(bb);
            }
        }
    }
}
hipError_t launch_rope_kv(const float* qkv, const float2* cs, const int32_t* row_pos,
                          const int32_t* page_table, void* q_out, void* kv_layer, KvGeom geom, int T_,
                          int n_new, int n_q_heads, int dtype, hipStream_t st) {
    if (T_ <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(rope_kv_kernel<T>, dim3(T_), dim3(256), 0, st, qkv, cs,
                                             row_pos, page_table, (T*)q_out, (T*)kv_layer, geom, n_new,
                                             n_q_heads));
    return hipGetLastError();
}

template <typename T>
__global__ void kv_import_kernel(const T* __restrict__ k_ctx, const T* __restrict__ v_ctx,
                                 T* __restrict__ kv_layer, const int32_t* __restrict__ page_table,
                                 KvGeom geom, int ctx_len) {
    // one workgroup per (b, kv head, position)
    int64_t id = blockIdx.x;
    int pos = (int)(id % ctx_len);
    int kvh = (int)((id / ctx_len) % geom.n_kv_heads);
    int b = (int)(id / ctx_len / geom.n_kv_heads);
    int64_t page = page_table[b * geom.pages_per_seq + pos / geom.page_tokens];
    int slot = pos % geom.page_tokens;
    const T* ks = k_ctx + id * geom.head_dim;
    const T* vs = v_ctx + id * geom.head_dim;
    T* kd = kv_layer + geom.k_off(page, kvh, slot);
    for (int c = threadIdx.x; c < geom.head_dim; c += blockDim.x) {
        kd[c] = ks[c];
        kv_layer[geom.v_off(page, kvh, slot, c)] = vs[c];
    }
}
hipError_t launch_kv_import(const void* k_ctx, const void* v_ctx, void* kv_layer,
                            const int32_t* page_table, KvGeom geom, int B, int ctx_len, int dtype,
                            hipStream_t st) {
    int64_t n = (int64_t)B * geom.n_kv_heads * ctx_len;
    if (n <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(kv_import_kernel<T>, dim3((unsigned)n), dim3(64), 0, st,
                                             (const T*)k_ctx, (const T*)v_ctx, (T*)kv_layer, page_table,
                                             geom, ctx_len));
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Router: r = h Wr^T (E <= 8 logits, f32 accumulate), top-2 (lowest id wins ties), weights =
// softmax over the two chosen logits.  One wavefront per token.
// ---------------------------------------------------------------------------------------------
// Top-2 of E router logits (lowest id wins ties) and the softmax over the two chosen logits.  With
// `forced` (two expert ids of this token, a testing aid: the routing of a reference run) the two given
// experts are taken instead, if they are valid and distinct, and only the weights come from the logits.
// An inactive row (a padding row of a prefill chunk, beyond its sequence's prompt) is given no expert at
// all: ids -1 and weights 0, so that the sort leaves it out of every expert's rows.
__device__ inline void pick_top2(const float* lg, int E, const int32_t* forced, bool active, int32_t* ids, float* wts) {
    if (!active) { ids[0] = -1; ids[1] = -1; wts[0] = 0.f; wts[1] = 0.f; return; }
    int i0 = 0;
    for (int e = 1; e < E; ++e) if (lg[e] > lg[i0]) i0 = e;
    int i1 = i0 == 0 ? 1 : 0;
    for (int e = 0; e < E; ++e) if (e != i0 && lg[e] > lg[i1]) i1 = e;
    if (forced) {
        const int f0 = forced[0], f1 = forced[1];
        if (f0 >= 0 && f0 < E && f1 >= 0 && f1 < E && f0 != f1) { i0 = f0; i1 = f1; }
    }
    float l0 = lg[0], l1 = lg[0];
    for (int e = 0; e < E; ++e) { if (e == i0) l0 = lg[e]; if (e == i1) l1 = lg[e]; }
    const float w0 = 1.0f / (1.0f + expf(l1 - l0));
    ids[0] = i0; ids[1] = i1;
    wts[0] = w0; wts[1] = 1.0f - w0;
}
template <typename T>
__global__ void router_kernel(const T* __restrict__ h, const T* __restrict__ wr,
                              int32_t* __restrict__ ids, float* __restrict__ wts, int T_, int d, int E,
                              const int32_t* __restrict__ forced, const int32_t* __restrict__ row_pos) {
    int t = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (t >= T_) return;
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    const T* hr = h + (int64_t)t * d;
    constexpr int VEC = 16 / sizeof(T);                 // 16-byte loads
    if (d % VEC == 0) {
        // unrolled so that the loads of four column blocks are in flight together (the kernel is
        // bound by the latency of these loads, not by their bytes)
#pragma unroll 4
        for (int c = lane * VEC; c < d; c += 64 * VEC) {
            alignas(16) T hv[VEC];
            *(uint4*)hv = *(const uint4*)(hr + c);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < E) {
                    alignas(16) T wv[VEC];
                    *(uint4*)wv = *(const uint4*)(wr + (int64_t)e * d + c);
#pragma unroll
                    for (int q = 0; q < VEC; ++q) acc[e] += to_f32<T>(hv[q]) * to_f32<T>(wv[q]);
                }
        }
    } else {
        for (int c = lane; c < d; c += 64) {
            float hv = to_f32<T>(hr[c]);
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < E) acc[e] += hv * to_f32<T>(wr[(int64_t)e * d + c]);
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = wave_sum(acc[e]);
    if (lane == 0) pick_top2(acc, E, forced ? forced + 2 * t : nullptr, !row_pos || row_pos[t] >= 0, ids + 2 * t, wts + 2 * t);
}
hipError_t launch_router(const void* h, const void* wr, int32_t* ids, float* wts, int T_, int d, int E,
                         const int32_t* forced, const int32_t* row_pos, int dtype, hipStream_t st) {
    if (T_ <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(router_kernel<T>, dim3((T_ + 3) / 4), dim3(256), 0, st,
                                             (const T*)h, (const T*)wr, ids, wts, T_, d, E, forced, row_pos));
    return hipGetLastError();
}

// RMSNorm fused with the router (the post-attention norm of an MoE layer): one 256-thread workgroup
// per row keeps the row in registers, writes h = norm(x) * g in the model dtype and multiplies the
// rounded h by the E router rows on the way (same values the stand-alone router reads back from
// memory), then reduces the E logits over the workgroup and picks top-2 as router_kernel does.
// Needs d % 8 == 0 and d <= 8 * 256 * NORM_ROUTE_CHUNKS.
constexpr int NORM_ROUTE_CHUNKS = 4;
template <typename T>
__global__ void __launch_bounds__(256)
norm_route_kernel(const float* __restrict__ x, const T* __restrict__ g, T* __restrict__ h,
                  const T* __restrict__ wr, int32_t* __restrict__ ids, float* __restrict__ wts, int d, int E,
                  float eps, const int32_t* __restrict__ forced, const int32_t* __restrict__ row_pos) {
    __shared__ float red[4];
    __shared__ float part[4][8];
    const int t = blockIdx.x, tid = threadIdx.x;
    const float* xr = x + (int64_t)t * d;
    float v[NORM_ROUTE_CHUNKS][8];
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < NORM_ROUTE_CHUNKS; ++q) {
        const int c = (q * 256 + tid) * 8;
        if (c < d) {
            const float4 a = *(const float4*)(xr + c), b = *(const float4*)(xr + c + 4);
            v[q][0] = a.x; v[q][1] = a.y; v[q][2] = a.z; v[q][3] = a.w;
            v[q][4] = b.x; v[q][5] = b.y; v[q][6] = b.z; v[q][7] = b.w;
#pragma unroll
            for (int e = 0; e < 8; ++e) ss += v[q][e] * v[q][e];
        }
    }
    ss = wave_sum(ss);
    if ((tid & 63) == 0) red[tid >> 6] = ss;
    __syncthreads();
    const float r = 1.0f / sqrtf((red[0] + red[1] + red[2] + red[3]) / (float)d + eps);
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
    T* hr = h + (int64_t)t * d;
#pragma unroll
    for (int q = 0; q < NORM_ROUTE_CHUNKS; ++q) {
        const int c = (q * 256 + tid) * 8;
        if (c < d) {
            T gv[8], hv[8];
            if (sizeof(T) == 2) *(uint4*)gv = *(const uint4*)(g + c);
            else { *(uint4*)gv = *(const uint4*)(g + c); *(uint4*)(gv + 4) = *(const uint4*)(g + c + 4); }
            float hf[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) { hv[i] = from_f32<T>(v[q][i] * r * to_f32<T>(gv[i])); hf[i] = to_f32<T>(hv[i]); }
            if (sizeof(T) == 2) *(uint4*)(hr + c) = *(const uint4*)hv;
            else { *(uint4*)(hr + c) = *(const uint4*)hv; *(uint4*)(hr + c + 4) = *(const uint4*)(hv + 4); }
#pragma unroll
            for (int e = 0; e < 8; ++e)
                if (e < E) {
                    T wv[8];
                    const T* wp = wr + (int64_t)e * d + c;
                    if (sizeof(T) == 2) *(uint4*)wv = *(const uint4*)wp;
                    else { *(uint4*)wv = *(const uint4*)wp; *(uint4*)(wv + 4) = *(const uint4*)(wp + 4); }
#pragma unroll
                    for (int i = 0; i < 8; ++i) acc[e] += hf[i] * to_f32<T>(wv[i]);
                }
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = wave_sum(acc[e]);
    if ((tid & 63) == 0) {
#pragma unroll
        for (int e = 0; e < 8; ++e) part[tid >> 6][e] = acc[e];
    }
    __syncthreads();
    if (tid == 0) {
        float lg[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) lg[e] = (part[0][e] + part[1][e]) + (part[2][e] + part[3][e]);
        pick_top2(lg, E, forced ? forced + 2 * t : nullptr, !row_pos || row_pos[t] >= 0, ids + 2 * t, wts + 2 * t);
    }
}
bool norm_route_supported(int d, int E) { return d % 8 == 0 && d <= 8 * 256 * NORM_ROUTE_CHUNKS && E >= 2 && E <= 8; }
hipError_t launch_norm_route(const float* x, const void* g, void* h, const void* wr, int32_t* ids, float* wts,
                             int T_, int d, int E, float eps, const int32_t* forced, const int32_t* row_pos, int dtype,
                             hipStream_t st) {
    if (T_ <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(norm_route_kernel<T>, dim3(T_), dim3(256), 0, st, x, (const T*)g, (T*)h,
                                             (const T*)wr, ids, wts, d, E, eps, forced, row_pos));
    return hipGetLastError();
}

// Stable counting sort of the 2T (token, choice) pairs by expert id, one 1024-thread workgroup.  Pairs
// of rows without experts (id < 0: inactive rows) are left out: offsets[E] is the number of routed pairs.
__global__ void __launch_bounds__(1024)
moe_sort_kernel(const int32_t* __restrict__ ids, int32_t* __restrict__ offsets,
                int32_t* __restrict__ perm, int32_t* __restrict__ slots, int n_pairs, int E) {
    __shared__ int cnt[8][1024];
    __shared__ int base[9];
    int tid = threadIdx.x;
    int chunk = (n_pairs + 1023) / 1024;
    int p0 = tid * chunk, p1 = min(p0 + chunk, n_pairs);
    int local[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) local[e] = 0;
    for (int p = p0; p < p1; ++p) {
        int e = ids[p];
#pragma unroll
        for (int q = 0; q < 8; ++q) local[q] += (q == e);
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) cnt[e][tid] = local[e];
    __syncthreads();
    // inclusive Hillis-Steele scan of each expert's per-thread counts
    for (int off = 1; off < 1024; off <<= 1) {
        int v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = tid >= off ? cnt[e][tid - off] : 0;
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 8; ++e) cnt[e][tid] += v[e];
        __syncthreads();
    }
    if (tid == 0) {
        int run = 0;
        for (int e = 0; e < E; ++e) { base[e] = run; offsets[e] = run; run += cnt[e][1023]; }
        base[E] = run; offsets[E] = run;
    }
    __syncthreads();
    int start[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) start[e] = (e < E ? base[e] : 0) + cnt[e][tid] - local[e];
    for (int p = p0; p < p1; ++p) {
        int e = ids[p];
        if (e < 0) { slots[p] = 0; continue; }
        int row = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) if (q == e) { row = start[q]; start[q] += 1; }
        perm[row] = p >> 1;
        slots[p] = row;
    }
}
hipError_t launch_moe_sort(const int32_t* ids, int32_t* offsets, int32_t* perm, int32_t* slots, int T_,
                           int E, hipStream_t st) {
    hipLaunchKernelGGL(moe_sort_kernel, dim3(1), dim3(1024), 0, st, ids, offsets, perm, slots, 2 * T_, E);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Plain tiled GEMM (any dtype, any size): 64x64 output tile, 256 threads, 4x4 outputs each.
// Used for f32 models; bf16 models use the MFMA kernels.
// ---------------------------------------------------------------------------------------------
template <typename T, bool SWIGLU>
__global__ void __launch_bounds__(256)
gemm_simple_kernel(GemmArgs a) {
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float As[BK][BM + 1];
    __shared__ float Ws[BK][BN + 1];
    __shared__ float W3s[SWIGLU ? BK : 1][BN + 1];
    int row_begin = 0, row_end = a.M, group = 0;
    int tile_m = blockIdx.y;
    if (a.group_offsets) {
        int acc_tiles = 0;
        bool found = false;
        for (int g = 0; g < a.n_groups; ++g) {
            int b0 = a.group_offsets[g], b1 = a.group_offsets[g + 1];
            int nt = (b1 - b0 + BM - 1) / BM;
            if (!found && tile_m < acc_tiles + nt) {
                group = g; row_begin = b0 + (tile_m - acc_tiles) * BM; row_end = b1; found = true;
            }
            acc_tiles += nt;
        }
        if (!found) return;
    } else {
        row_begin = tile_m * BM;
        if (row_begin >= a.M) return;
    }
    const T* A = (const T*)a.A;
    const T* W = (const T*)a.W + (int64_t)group * a.w_group_stride;
    const T* W3 = SWIGLU ? (const T*)a.W3 + (int64_t)group * a.w_group_stride : nullptr;
    int col0 = blockIdx.x * BN;
    int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4], acc3[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) { acc[i][j] = 0.f; acc3[i][j] = 0.f; }
    // loader mapping: thread loads (row = tid/4, k = (tid%4)*4 .. +3)
    int lr = tid >> 2, lk = (tid & 3) * 4;
    int arow = row_begin + lr;
    int64_t asrc = -1;
    if (arow < row_end) asrc = a.a_rows ? a.a_rows[arow] : arow;
    int wrow = col0 + lr;
    for (int k0 = 0; k0 < a.K; k0 += BK) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            int kk = k0 + lk + q;
            As[lk + q][lr] = (asrc >= 0 && kk < a.K) ? to_f32<T>(A[asrc * a.lda + kk]) : 0.f;
            bool wv = wrow < a.N && kk < a.K;
            Ws[lk + q][lr] = wv ? to_f32<T>(W[(int64_t)wrow * a.K + kk]) : 0.f;
            if (SWIGLU) W3s[lk + q][lr] = wv ? to_f32<T>(W3[(int64_t)wrow * a.K + kk]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < BK; ++kk) {
            float av[4], wv[4], w3v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) av[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) { wv[j] = Ws[kk][tx * 4 + j]; if (SWIGLU) w3v[j] = W3s[kk][tx * 4 + j]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    acc[i][j] += av[i] * wv[j];
                    if (SWIGLU) acc3[i][j] += av[i] * w3v[j];
                }
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int r = row_begin + ty * 4 + i;
        if (r >= row_end) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int c = col0 + tx * 4 + j;
            if (c >= a.N) continue;
            int64_t o = (int64_t)r * a.ldc + c;
            float v = acc[i][j];
            if (SWIGLU) {
                float s = v / (1.0f + expf(-v));
                ((T*)a.C)[o] = from_f32<T>(s * acc3[i][j]);
            } else if (a.epilogue == EPI_STORE_F32) ((float*)a.C)[o] = v;
            else if (a.epilogue == EPI_ADD_F32) ((float*)a.C)[o] += v;
            else ((T*)a.C)[o] = from_f32<T>(v);
        }
    }
}

hipError_t launch_gemm_simple(const GemmArgs& a, int dtype, hipStream_t st) {
    int rows = a.group_offsets ? a.m_upper : a.M;
    if (rows <= 0 || a.N <= 0) return hipSuccess;
    int tiles_m = (rows + 63) / 64 + (a.group_offsets ? a.n_groups : 0);
    dim3 grid((a.N + 63) / 64, tiles_m);
    bool sw = a.epilogue == EPI_SWIGLU_T;
    DISPATCH_DTYPE(dtype, {
        if (sw) hipLaunchKernelGGL((gemm_simple_kernel<T, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((gemm_simple_kernel<T, false>), grid, dim3(256), 0, st, a);
    });
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Plain paged attention: one wavefront per (row, query head); keys in chunks of 64 with an online
// softmax; lanes own keys for the scores and output dimensions for the value sum.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(64)
attention_simple_kernel(AttnArgs a) {
    __shared__ float qs[256];
    int t = blockIdx.x / a.n_q_heads, hq = blockIdx.x % a.n_q_heads;
    int lane = threadIdx.x;
    int dh = a.geom.head_dim;
    int g = a.n_q_heads / a.geom.n_kv_heads, kvh = hq / g;
    int b = t / a.n_new;
    int pos = a.row_pos[t];
    T* out = (T*)a.out + (int64_t)t * a.n_q_heads * dh + hq * dh;
    if (pos < 0) {
        for (int c = lane; c < dh; c += 64) out[c] = from_f32<T>(0.f);
        return;
    }
    const T* q = (const T*)a.q + (int64_t)t * a.n_q_heads * dh + hq * dh;
    for (int c = lane; c < dh; c += 64) qs[c] = to_f32<T>(q[c]);
    __syncthreads();
    const T* kv = (const T*)a.kv_layer;
    const int32_t* pt = a.page_table + b * a.geom.pages_per_seq;
    int n_keys = pos + 1;
    float m = -INFINITY, l = 0.f;
    float acc[4] = {0.f, 0.f, 0.f, 0.f};
    for (int c0 = 0; c0 < n_keys; c0 += 64) {
        int key = c0 + lane;
        float s = -INFINITY;
        if (key < n_keys) {
            int64_t page = pt[key / a.geom.page_tokens];
            const T* kr = kv + a.geom.k_off(page, kvh, key % a.geom.page_tokens);
            float dot = 0.f;
            for (int c = 0; c < dh; ++c) dot += qs[c] * to_f32<T>(kr[c]);
            s = dot * a.scale;
        }
        float m_new = fmaxf(m, wave_max(s));
        float p = key < n_keys ? expf(s - m_new) : 0.f;
        float corr = expf(m - m_new);       // m = -inf on the first chunk -> 0
        l = l * corr + wave_sum(p);
#pragma unroll
        for (int dd = 0; dd < 4; ++dd) acc[dd] *= corr;
        int nk = min(64, n_keys - c0);
        for (int j = 0; j < nk; ++j) {
            float pj = __shfl(p, j, 64);
            int kj = c0 + j;
            int64_t page = pt[kj / a.geom.page_tokens];
            int sl = kj % a.geom.page_tokens;
#pragma unroll
            for (int dd = 0; dd < 4; ++dd) {
                int c = lane + 64 * dd;
                if (c < dh) acc[dd] += pj * to_f32<T>(kv[a.geom.v_off(page, kvh, sl, c)]);
            }
        }
        m = m_new;
    }
    float inv = 1.0f / l;
#pragma unroll
    for (int dd = 0; dd < 4; ++dd) {
        int c = lane + 64 * dd;
        if (c < dh) out[c] = from_f32<T>(acc[dd] * inv);
    }
}
hipError_t launch_attention_simple(const AttnArgs& a, int dtype, hipStream_t st) {
    int T_ = a.B * a.n_new;
    if (T_ <= 0) return hipSuccess;
    DISPATCH_DTYPE(dtype, hipLaunchKernelGGL(attention_simple_kernel<T>, dim3(T_ * a.n_q_heads), dim3(64),
                                             0, st, a));
    return hipGetLastError();
}

}  // namespace sv
