// Accept/reject kernels of the verify step and the draft's token pick.
//
// Greedy rule (Section 2.2; Appendix A.1 "Generated Tokens"): keep the longest prefix of candidates
// that equal the target's own argmax, then emit the target's argmax at the first mismatch (or after
// all k).  Stochastic rule (the speculative-sampling works cited in Section 2.2): keep candidate i
// while u * q_i(c_i) < p_{i-1}(c_i); then draw from max(0, p_n - q_{n+1}) renormalised, or from p_k
// when all were kept.  All reductions over the vocabulary are wavefront shuffles + one LDS hop;
// running sums for the inverse-CDF draw are taken in ascending token id, 1024 ids per sweep.
#include "common.h"

namespace sv {

// ---- Philox4x32-10 (Salmon et al., SC'11): counter-based, so a draw depends only on
// (seed, round, sequence, position) and not on batch split or thread mapping ------------------
__device__ inline void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t k0,
                                     uint32_t k1, uint32_t out[4]) {
    const uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint32_t h0 = __umulhi(M0, c0), l0 = M0 * c0;
        uint32_t h1 = __umulhi(M1, c2), l1 = M1 * c2;
        uint32_t n0 = h1 ^ c1 ^ k0, n2 = h0 ^ c3 ^ k1;
        c0 = n0; c1 = l1; c2 = n2; c3 = l0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}
__device__ inline float word_to_uniform(uint32_t w) { return (float)(w >> 8) * 5.9604644775390625e-8f; }
// word 0: draft draw, word 1: acceptance test, word 2: residual / bonus draw of position i
__device__ inline float philox_uniform(uint64_t seed, uint32_t round, uint32_t seq, uint32_t i, int word) {
    uint32_t o[4];
    philox4x32_10(round, seq, i, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), o);
    return word_to_uniform(o[word]);
}

__global__ void philox_uniforms_kernel(uint64_t seed, uint32_t round, uint32_t seq_base, int B, int k,
                                       float* __restrict__ out) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * (k + 1)) return;
    int b = idx / (k + 1), i = idx % (k + 1);
    uint32_t o[4];
    philox4x32_10(round, seq_base + b, (uint32_t)i, 0u, (uint32_t)seed, (uint32_t)(seed >> 32), o);
    out[3 * idx + 0] = word_to_uniform(o[0]);
    out[3 * idx + 1] = word_to_uniform(o[1]);
    out[3 * idx + 2] = word_to_uniform(o[2]);
}
hipError_t launch_philox_uniforms(uint64_t seed, uint32_t round, uint32_t seq_base, int B, int k,
                                  float* out, hipStream_t st) {
    int n = B * (k + 1);
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(philox_uniforms_kernel, dim3((n + 255) / 256), dim3(256), 0, st, seed, round,
                       seq_base, B, k, out);
    return hipGetLastError();
}

// ---- 256-thread block helpers -----------------------------------------------------------------
constexpr int ACC_THREADS = 256;

__device__ inline float block_sum(float v, float* sh /*>=4*/) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return sh[0] + sh[1] + sh[2] + sh[3];
}
__device__ inline float block_max(float v, float* sh) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
// argmax with lowest-index tie-break
__device__ inline int block_argmax(const float* __restrict__ z, int V, float* shv, int* shi) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
    for (int c = threadIdx.x; c < V; c += ACC_THREADS) {
        float v = z[c];
        if (v > bv) { bv = v; bi = c; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(bv, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { shv[threadIdx.x >> 6] = bv; shi[threadIdx.x >> 6] = bi; }
    __syncthreads();
    bv = shv[0]; bi = shi[0];
#pragma unroll
    for (int w = 1; w < 4; ++w)
        if (shv[w] > bv || (shv[w] == bv && shi[w] < bi)) { bv = shv[w]; bi = shi[w]; }
    return bi;
}

// Smallest id whose running sum of w(id) (ascending ids) exceeds target; if rounding leaves none,
// the largest id with positive weight.
template <typename F>
__device__ inline int block_inverse_cdf(F w, int V, float target, float* shf, int* shi) {
    float run = 0.f;
    int last_pos = -1;
    int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    for (int base = 0; base < V; base += ACC_THREADS * 4) {
        int id0 = base + threadIdx.x * 4;
        float x[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            x[j] = id0 + j < V ? w(id0 + j) : 0.f;
            if (x[j] > 0.f) last_pos = id0 + j;
        }
        float local = (x[0] + x[1]) + (x[2] + x[3]);
        float incl = local;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            float up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        __syncthreads();
        if (lane == 63) shf[wv] = incl;
        __syncthreads();
        float wave_base = 0.f;
        for (int q = 0; q < wv; ++q) wave_base += shf[q];
        float seg_total = shf[0] + shf[1] + shf[2] + shf[3];
        incl += wave_base;
        bool over = run + incl > target;
        // lowest thread over the target
        unsigned long long bal = __ballot(over);
        __syncthreads();
        if (lane == 0) shi[wv] = bal ? (wv * 64 + (int)__ffsll((long long)bal) - 1) : 0x7fffffff;
        __syncthreads();
        int first = min(min(shi[0], shi[1]), min(shi[2], shi[3]));
        if (first != 0x7fffffff) {
            __syncthreads();
            if ((int)threadIdx.x == first) {
                float c = run + (incl - local);
                int pick = -1, lastp = -1;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    c += x[j];
                    if (x[j] > 0.f) lastp = id0 + j;
                    if (pick < 0 && c > target && x[j] > 0.f) pick = id0 + j;
                }
                shi[4] = pick >= 0 ? pick : (lastp >= 0 ? lastp : id0);
            }
            __syncthreads();
            return shi[4];
        }
        run += seg_total;
    }
    // no crossing found (target >= total after rounding): largest id of positive weight
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) last_pos = max(last_pos, __shfl_xor(last_pos, o, 64));
    __syncthreads();
    if (lane == 0) shi[wv] = last_pos;
    __syncthreads();
    int r = max(max(shi[0], shi[1]), max(shi[2], shi[3]));
    return r < 0 ? 0 : r;
}

// max and sum of exp((z - max) * inv_tau) of one row
__device__ inline void block_row_stats(const float* __restrict__ z, int V, float inv_tau, float* sh,
                                       float* out_max, float* out_sum) {
    float m = -INFINITY;
    for (int c = threadIdx.x; c < V; c += ACC_THREADS) m = fmaxf(m, z[c]);
    m = block_max(m, sh);
    float s = 0.f;
    for (int c = threadIdx.x; c < V; c += ACC_THREADS) s += expf((z[c] - m) * inv_tau);
    s = block_sum(s, sh);
    *out_max = m; *out_sum = s;
}

// ---- greedy accept, any vocabulary size: one 256-thread workgroup per sequence, early exit at the
// first mismatch ---------------------------------------------------------------------------------
__global__ void __launch_bounds__(ACC_THREADS)
accept_greedy_generic_kernel(AcceptArgs a) {
    __shared__ float shv[4];
    __shared__ int shi[4];
    int b = blockIdx.x;
    const float* P = a.p_logits + (int64_t)b * (a.k + 1) * a.V;
    int n = 0, am;
    while (true) {
        am = block_argmax(P + (int64_t)n * a.V, a.V, shv, shi);
        if (n < a.k && a.draft_tokens[b * a.k + n] == am) ++n; else break;
    }
    if (threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[b] = n;
        if (a.next_token) a.next_token[b] = am;
    }
}

// ---- stochastic accept, any vocabulary size (rows re-read for every reduction) ------------------
__global__ void __launch_bounds__(ACC_THREADS)
accept_sample_generic_kernel(AcceptArgs a) {
    __shared__ float shf[4];
    __shared__ int shi[5];
    __shared__ int sh_stop;
    int b = blockIdx.x, k = a.k, V = a.V;
    const float* P = a.p_logits + (int64_t)b * (k + 1) * V;
    const float* Q = a.q_logits + (int64_t)b * k * V;
    float it = a.inv_tau;
    int n = 0;
    float pm = 0.f, ps = 1.f, qm = 0.f, qs = 1.f;
    // candidates are tested in order; each test needs the softmax normalisers of two rows
    while (true) {
        block_row_stats(P + (int64_t)n * V, V, it, shf, &pm, &ps);
        if (n == k) break;
        block_row_stats(Q + (int64_t)n * V, V, it, shf, &qm, &qs);
        if (threadIdx.x == 0) {
            int c = a.draft_tokens[b * k + n];
            if (c < 0 || c >= V) sh_stop = 1;       // an id outside the vocabulary is a rejected candidate
            else {
                float pv = expf((P[(int64_t)n * V + c] - pm) * it) / ps;
                float qv = expf((Q[(int64_t)n * V + c] - qm) * it) / qs;
                float u = a.u_accept ? a.u_accept[b * k + n]
                                     : philox_uniform(a.seed, a.round, a.seq_base + b, (uint32_t)(n + 1), 1);
                sh_stop = !(u * qv < pv);
            }
        }
        __syncthreads();
        int stop = sh_stop;
        __syncthreads();
        if (stop) break;
        ++n;
    }
    const float* pr = P + (int64_t)n * V;
    const float* qr = n < k ? Q + (int64_t)n * V : nullptr;
    float ipn = 1.0f / ps, iqn = 1.0f / qs;
    auto wres = [&](int id) -> float {
        float pv = expf((pr[id] - pm) * it) * ipn;
        if (!qr) return pv;
        float qv = expf((qr[id] - qm) * it) * iqn;
        return fmaxf(0.f, pv - qv);
    };
    auto wp = [&](int id) -> float { return expf((pr[id] - pm) * it) * ipn; };
    float tot = 0.f;
    for (int c = threadIdx.x; c < V; c += ACC_THREADS) tot += wres(c);
    tot = block_sum(tot, shf);
    float u = a.u_resample ? a.u_resample[b * (k + 1) + n]
                           : philox_uniform(a.seed, a.round, a.seq_base + b, (uint32_t)n, 2);
    int nxt;
    if (tot > 0.f) nxt = block_inverse_cdf(wres, V, u * tot, shf, shi);
    else {                                  // p == q everywhere: fall back to the target row
        float tp = 0.f;
        for (int c = threadIdx.x; c < V; c += ACC_THREADS) tp += wp(c);
        tp = block_sum(tp, shf);
        nxt = block_inverse_cdf(wp, V, u * tp, shf, shi);
    }
    if (threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[b] = n;
        if (a.next_token) a.next_token[b] = nxt;
    }
}

// =================================================================================================
// Fast path: vocabularies of up to 32768 ids (a multiple of 4, rows 16-byte aligned).  One workgroup
// of 1024 threads per sequence; a logits row is loaded once, 32 values per thread as 8 float4 (thread
// t of sweep s holds ids 4096 s + 4 t .. + 3, so running sums stay in ascending id order), and every
// reduction of that row (max, normaliser, residual total, inverse CDF) runs on the registers.  With
// early exit at the first rejected candidate a round reads each row it needs exactly once: the rule's
// HBM traffic is the logit bytes up to the first rejection, (2 n + 2) rows of V floats per sequence.
// =================================================================================================
constexpr int FAST_THREADS = 1024, FAST_WAVES = FAST_THREADS / 64, FAST_SWEEPS = 8;
constexpr int FAST_MAX_V = FAST_THREADS * 4 * FAST_SWEEPS;

struct FastShared {
    float red[FAST_WAVES];
    int redi[FAST_WAVES];
    float tot[FAST_SWEEPS * FAST_WAVES];     // wave totals of every sweep, then their exclusive prefix
    float total;
    int pick, last, stop;
};

__device__ inline void fast_load_row(const float* __restrict__ row, int V, float4 (&v)[FAST_SWEEPS]) {
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) {
        const int id = (s * FAST_THREADS + (int)threadIdx.x) * 4;
        v[s] = id < V ? *(const float4*)(row + id) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
    }
}
__device__ inline float fast_block_sum(float v, FastShared& sh) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = 0.f;
#pragma unroll
    for (int w = 0; w < FAST_WAVES; ++w) t += sh.red[w];
    return t;
}
__device__ inline float fast_block_max(float v, FastShared& sh) {
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sh.red[threadIdx.x >> 6] = v;
    __syncthreads();
    float t = sh.red[0];
#pragma unroll
    for (int w = 1; w < FAST_WAVES; ++w) t = fmaxf(t, sh.red[w]);
    return t;
}
// max and sum of exp((z - max) * inv_tau) of a row held in registers (padding is -inf: adds 0)
__device__ inline void fast_row_stats(const float4 (&v)[FAST_SWEEPS], float inv_tau, FastShared& sh, float* out_max,
                                      float* out_sum) {
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) m = fmaxf(fmaxf(fmaxf(m, v[s].x), fmaxf(v[s].y, v[s].z)), v[s].w);
    m = fast_block_max(m, sh);
    float sum = 0.f;
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s)
        sum += (expf((v[s].x - m) * inv_tau) + expf((v[s].y - m) * inv_tau)) +
               (expf((v[s].z - m) * inv_tau) + expf((v[s].w - m) * inv_tau));
    *out_max = m;
    *out_sum = fast_block_sum(sum, sh);
}
// argmax of a row held in registers, lowest id on ties
__device__ inline int fast_argmax(const float4 (&v)[FAST_SWEEPS], FastShared& sh) {
    float bv = -INFINITY;
    int bi = 0x7fffffff;
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) {
        const int id = (s * FAST_THREADS + (int)threadIdx.x) * 4;
        const float x[4] = {v[s].x, v[s].y, v[s].z, v[s].w};
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (x[j] > bv) { bv = x[j]; bi = id + j; }
    }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        float ov = __shfl_xor(bv, o, 64);
        int oi = __shfl_xor(bi, o, 64);
        if (ov > bv || (ov == bv && oi < bi)) { bv = ov; bi = oi; }
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) { sh.red[threadIdx.x >> 6] = bv; sh.redi[threadIdx.x >> 6] = bi; }
    __syncthreads();
    bv = sh.red[0]; bi = sh.redi[0];
#pragma unroll
    for (int w = 1; w < FAST_WAVES; ++w)
        if (sh.red[w] > bv || (sh.red[w] == bv && sh.redi[w] < bi)) { bv = sh.red[w]; bi = sh.redi[w]; }
    return bi;
}
// Inverse CDF over non-negative weights held in registers: the smallest id whose running sum (ascending
// ids) exceeds u * total, where total is the same running sum at the end; if rounding leaves none, the
// largest id of positive weight.  *total_out receives the total (0: no positive weight; result invalid).
__device__ inline int fast_inverse_cdf(const float4 (&wt)[FAST_SWEEPS], float u, FastShared& sh, float* total_out) {
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    float local[FAST_SWEEPS], excl[FAST_SWEEPS];
    __syncthreads();
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) {
        local[s] = (wt[s].x + wt[s].y) + (wt[s].z + wt[s].w);
        float incl = local[s];
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            float up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        excl[s] = incl - local[s];
        if (lane == 63) sh.tot[s * FAST_WAVES + wv] = incl;
    }
    if (threadIdx.x == 0) { sh.pick = 0x7fffffff; sh.last = -1; }
    __syncthreads();
    if (wv == 0) {      // exclusive prefix of the 128 (sweep, wavefront) totals, two per lane
        float v0 = sh.tot[2 * lane], v1 = sh.tot[2 * lane + 1];
        float pair = v0 + v1, incl = pair;
#pragma unroll
        for (int o = 1; o < 64; o <<= 1) {
            float up = __shfl_up(incl, o, 64);
            if (lane >= o) incl += up;
        }
        sh.tot[2 * lane] = incl - pair;
        sh.tot[2 * lane + 1] = (incl - pair) + v0;
        if (lane == 63) sh.total = incl;
    }
    __syncthreads();
    const float total = sh.total, target = u * total;
    int found = 0x7fffffff, lastp = -1;
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) {
        const int id = (s * FAST_THREADS + (int)threadIdx.x) * 4;
        float c = sh.tot[s * FAST_WAVES + wv] + excl[s];
        const float x[4] = {wt[s].x, wt[s].y, wt[s].z, wt[s].w};
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            c += x[j];
            if (x[j] > 0.f) {
                lastp = id + j;
                if (c > target && found == 0x7fffffff) found = id + j;
            }
        }
    }
    if (found != 0x7fffffff) atomicMin(&sh.pick, found);
    if (lastp >= 0) atomicMax(&sh.last, lastp);
    __syncthreads();
    *total_out = total;
    return sh.pick != 0x7fffffff ? sh.pick : (sh.last >= 0 ? sh.last : 0);
}
__device__ inline float4 fast_softmax_weights(const float4& z, float m, float inv_tau, float inv_norm) {
    return make_float4(expf((z.x - m) * inv_tau) * inv_norm, expf((z.y - m) * inv_tau) * inv_norm,
                       expf((z.z - m) * inv_tau) * inv_norm, expf((z.w - m) * inv_tau) * inv_norm);
}

__global__ void __launch_bounds__(FAST_THREADS)
accept_greedy_kernel(AcceptArgs a) {
    __shared__ FastShared sh;
    const int b = blockIdx.x;
    const float* P = a.p_logits + (int64_t)b * (a.k + 1) * a.V;
    int n = 0, am;
    while (true) {
        float4 z[FAST_SWEEPS];
        fast_load_row(P + (int64_t)n * a.V, a.V, z);
        am = fast_argmax(z, sh);
        if (n < a.k && a.draft_tokens[b * a.k + n] == am) ++n; else break;
    }
    if (threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[b] = n;
        if (a.next_token) a.next_token[b] = am;
    }
}

__global__ void __launch_bounds__(FAST_THREADS)
accept_sample_kernel(AcceptArgs a) {
    __shared__ FastShared sh;
    const int b = blockIdx.x, k = a.k, V = a.V;
    const float* P = a.p_logits + (int64_t)b * (k + 1) * V;
    const float* Q = a.q_logits + (int64_t)b * k * V;
    const float it = a.inv_tau;
    int n = 0;
    float pm = 0.f, ps = 1.f, qm = 0.f, qs = 1.f;
    float4 pz[FAST_SWEEPS], qz[FAST_SWEEPS];
    // candidates are tested in order; each test needs the softmax normalisers of two rows, which stay
    // in registers for the draw that follows the first rejection
    while (true) {
        fast_load_row(P + (int64_t)n * V, V, pz);
        if (n < k) fast_load_row(Q + (int64_t)n * V, V, qz);
        fast_row_stats(pz, it, sh, &pm, &ps);
        if (n == k) break;
        fast_row_stats(qz, it, sh, &qm, &qs);
        if (threadIdx.x == 0) {
            int c = a.draft_tokens[b * k + n];
            if (c < 0 || c >= V) sh.stop = 1;       // an id outside the vocabulary is a rejected candidate
            else {
                float pv = expf((P[(int64_t)n * V + c] - pm) * it) / ps;
                float qv = expf((Q[(int64_t)n * V + c] - qm) * it) / qs;
                float u = a.u_accept ? a.u_accept[b * k + n]
                                     : philox_uniform(a.seed, a.round, a.seq_base + b, (uint32_t)(n + 1), 1);
                sh.stop = !(u * qv < pv);
            }
        }
        __syncthreads();
        const int stop = sh.stop;
        __syncthreads();
        if (stop) break;
        ++n;
    }
    const float ipn = 1.0f / ps, iqn = 1.0f / qs;
    float4 w[FAST_SWEEPS];
#pragma unroll
    for (int s = 0; s < FAST_SWEEPS; ++s) {
        w[s] = fast_softmax_weights(pz[s], pm, it, ipn);
        if (n < k) {
            const float4 q = fast_softmax_weights(qz[s], qm, it, iqn);
            w[s] = make_float4(fmaxf(0.f, w[s].x - q.x), fmaxf(0.f, w[s].y - q.y), fmaxf(0.f, w[s].z - q.z),
                               fmaxf(0.f, w[s].w - q.w));
        }
    }
    const float u = a.u_resample ? a.u_resample[b * (k + 1) + n]
                                 : philox_uniform(a.seed, a.round, a.seq_base + b, (uint32_t)n, 2);
    float tot;
    int nxt = fast_inverse_cdf(w, u, sh, &tot);
    if (!(tot > 0.f)) {                     // p == q everywhere: fall back to the target row
#pragma unroll
        for (int s = 0; s < FAST_SWEEPS; ++s) w[s] = fast_softmax_weights(pz[s], pm, it, ipn);
        nxt = fast_inverse_cdf(w, u, sh, &tot);
    }
    if (threadIdx.x == 0) {
        if (a.n_accepted) a.n_accepted[b] = n;
        if (a.next_token) a.next_token[b] = nxt;
    }
}

static inline bool fast_rows_ok(const float* base, int V) {
    return V % 4 == 0 && V <= FAST_MAX_V && ((uintptr_t)base & 15) == 0;
}

hipError_t launch_accept(const AcceptArgs& a, hipStream_t st) {
    if (a.B <= 0) return hipSuccess;
    const bool fast = fast_rows_ok(a.p_logits, a.V) && (!a.q_logits || fast_rows_ok(a.q_logits, a.V));
    if (a.q_logits) {
        if (fast) hipLaunchKernelGGL(accept_sample_kernel, dim3(a.B), dim3(FAST_THREADS), 0, st, a);
        else hipLaunchKernelGGL(accept_sample_generic_kernel, dim3(a.B), dim3(ACC_THREADS), 0, st, a);
    } else {
        if (fast) hipLaunchKernelGGL(accept_greedy_kernel, dim3(a.B), dim3(FAST_THREADS), 0, st, a);
        else hipLaunchKernelGGL(accept_greedy_generic_kernel, dim3(a.B), dim3(ACC_THREADS), 0, st, a);
    }
    return hipGetLastError();
}

// ---- draft token pick ---------------------------------------------------------------------------
__global__ void __launch_bounds__(ACC_THREADS)
draft_pick_generic_kernel(const float* __restrict__ z, int64_t ld, int V, int mode, float inv_tau, uint64_t seed,
                          uint32_t round, uint32_t seq_base, int step, int32_t* __restrict__ draft_tokens, int k) {
    __shared__ float shf[4];
    __shared__ int shi[5];
    int b = blockIdx.x;
    const float* row = z + (int64_t)b * ld;
    int pick;
    if (mode == SPEC_GREEDY) {
        pick = block_argmax(row, V, shf, shi);
    } else {
        float m, s;
        block_row_stats(row, V, inv_tau, shf, &m, &s);
        auto w = [&](int id) -> float { return expf((row[id] - m) * inv_tau); };
        float u = philox_uniform(seed, round, seq_base + b, (uint32_t)step, 0);
        pick = block_inverse_cdf(w, V, u * s, shf, shi);
    }
    if (threadIdx.x == 0) draft_tokens[b * k + step - 1] = pick;
}
// fast path (see above): the row is read once
__global__ void __launch_bounds__(FAST_THREADS)
draft_pick_kernel(const float* __restrict__ z, int64_t ld, int V, int mode, float inv_tau, uint64_t seed,
                  uint32_t round, uint32_t seq_base, int step, int32_t* __restrict__ draft_tokens, int k) {
    __shared__ FastShared sh;
    const int b = blockIdx.x;
    float4 row[FAST_SWEEPS];
    fast_load_row(z + (int64_t)b * ld, V, row);
    int pick;
    if (mode == SPEC_GREEDY) {
        pick = fast_argmax(row, sh);
    } else {
        float m, s, tot;
        fast_row_stats(row, inv_tau, sh, &m, &s);
#pragma unroll
        for (int q = 0; q < FAST_SWEEPS; ++q) row[q] = fast_softmax_weights(row[q], m, inv_tau, 1.0f);
        const float u = philox_uniform(seed, round, seq_base + b, (uint32_t)step, 0);
        pick = fast_inverse_cdf(row, u, sh, &tot);
    }
    if (threadIdx.x == 0) draft_tokens[b * k + step - 1] = pick;
}
hipError_t launch_draft_pick(const float* z, int64_t ld, int V, int B, int mode, float inv_tau,
                             uint64_t seed, uint32_t round, uint32_t seq_base, int step,
                             int32_t* draft_tokens, int k, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    if (fast_rows_ok(z, V) && ld % 4 == 0)
        hipLaunchKernelGGL(draft_pick_kernel, dim3(B), dim3(FAST_THREADS), 0, st, z, ld, V, mode, inv_tau, seed,
                           round, seq_base, step, draft_tokens, k);
    else
        hipLaunchKernelGGL(draft_pick_generic_kernel, dim3(B), dim3(ACC_THREADS), 0, st, z, ld, V, mode, inv_tau,
                           seed, round, seq_base, step, draft_tokens, k);
    return hipGetLastError();
}

}  // namespace sv
