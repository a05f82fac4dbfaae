// Sequence-state kernels: they build the token / position rows of each pass from the committed
// tokens kept in HBM and commit accepted tokens, so that the host never has to read results back
// inside the draft/verify loop.
#include "common.h"

namespace sv {

// Verify rows of sequence b: [last committed token, candidate 1..k] at positions len-1 .. len-1+k
// (Section 2.2: all candidates are scored by the target in one forward pass).
__global__ void verify_prep_kernel(SeqState s, const int32_t* __restrict__ d, int k,
                                   int32_t* __restrict__ tok_in, int32_t* __restrict__ row_pos, int B) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * (k + 1)) return;
    int b = idx / (k + 1), i = idx % (k + 1);
    int len = s.len[b];
    tok_in[idx] = i == 0 ? s.tokens[(int64_t)b * s.tok_cap + len - 1] : d[b * k + i - 1];
    row_pos[idx] = len - 1 + i;
}
hipError_t launch_verify_prep(SeqState s, const int32_t* draft_tokens, int k, int32_t* tok_in,
                              int32_t* row_pos, int B, hipStream_t st) {
    int n = B * (k + 1);
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(verify_prep_kernel, dim3((n + 255) / 256), dim3(256), 0, st, s, draft_tokens, k,
                       tok_in, row_pos, B);
    return hipGetLastError();
}

// Draft rows.  Step 1 feeds TWO rows per sequence, the tokens at positions len-2 and len-1: after a
// round in which every candidate was kept the draft cache lacks position len-2, otherwise that entry
// is recomputed to the same value, so the cache always covers [0, len-1) before candidate 1 is
// produced.  Step i >= 2 feeds candidate i-1 at position len-2+i.
__global__ void draft_prep_kernel(SeqState s, const int32_t* __restrict__ d, int k, int step,
                                  int32_t* __restrict__ tok_in, int32_t* __restrict__ row_pos, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int len = s.len[b];
    const int32_t* toks = s.tokens + (int64_t)b * s.tok_cap;
    if (step == 1) {
        tok_in[2 * b] = len >= 2 ? toks[len - 2] : 0;
        row_pos[2 * b] = len >= 2 ? len - 2 : -1;
        tok_in[2 * b + 1] = toks[len - 1];
        row_pos[2 * b + 1] = len - 1;
    } else {
        tok_in[b] = d[b * k + step - 2];
        row_pos[b] = len - 2 + step;
    }
}
hipError_t launch_draft_prep(SeqState s, const int32_t* draft_tokens, int k, int step, int32_t* tok_in,
                             int32_t* row_pos, int B, hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(draft_prep_kernel, dim3((B + 255) / 256), dim3(256), 0, st, s, draft_tokens, k, step,
                       tok_in, row_pos, B);
    return hipGetLastError();
}

// Prefill rows of one chunk: positions chunk0 .. chunk0+Q-1 of every prompt; only positions before
// the last prompt token are active (the last token is fed by the first verify pass).
__global__ void prefill_prep_kernel(const int32_t* __restrict__ tokens, const int32_t* __restrict__ plen,
                                    const int32_t* __restrict__ seq_of, int tok_cap, int B, int chunk0, int Q,
                                    int32_t* __restrict__ tok_in, int32_t* __restrict__ row_pos) {
    int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= B * Q) return;
    int b = idx / Q, pos = chunk0 + idx % Q;
    if (seq_of) b = seq_of[b];            // rows are laid out in the prefill's own order of the sequences
    bool on = pos < plen[b] - 1;
    tok_in[idx] = on ? tokens[(int64_t)b * tok_cap + pos] : 0;
    row_pos[idx] = on ? pos : -1;
}
hipError_t launch_prefill_prep(const int32_t* tokens_dev, const int32_t* plen, const int32_t* seq_of, int tok_cap, int B,
                               int chunk0, int Q, int32_t* tok_in, int32_t* row_pos, hipStream_t st) {
    int n = B * Q;
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(prefill_prep_kernel, dim3((n + 255) / 256), dim3(256), 0, st, tokens_dev, plen,
                       seq_of, tok_cap, B, chunk0, Q, tok_in, row_pos);
    return hipGetLastError();
}

// Commit: append candidates 1..n and the target's token, clipped to the sequence's remaining quota
// (a round emits between 1 and k+1 tokens, Appendix A.1 "Generated Tokens").  The KV caches need no
// work: entries beyond the new length are simply overwritten by the next pass.
__global__ void commit_kernel(SeqState s, const int32_t* __restrict__ d, int k,
                              const int32_t* __restrict__ n_acc, const int32_t* __restrict__ next_tok,
                              unsigned long long* __restrict__ hist,
                              unsigned long long* __restrict__ committed, int B) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    int remaining = s.max_new[b] - s.n_new[b];
    if (remaining <= 0) return;
    int n = n_acc[b];
    int c = min(n + 1, remaining);
    int len = s.len[b];
    int32_t* toks = s.tokens + (int64_t)b * s.tok_cap;
    for (int j = 0; j < c; ++j) toks[len + j] = j < n ? d[b * k + j] : next_tok[b];
    s.len[b] = len + c;
    s.n_new[b] += c;
    atomicAdd(&hist[n], 1ull);
    atomicAdd(committed, (unsigned long long)c);
}
hipError_t launch_commit(SeqState s, const int32_t* draft_tokens, int k, const int32_t* n_acc,
                         const int32_t* next_tok, int64_t* hist, int64_t* committed, int B,
                         hipStream_t st) {
    if (B <= 0) return hipSuccess;
    hipLaunchKernelGGL(commit_kernel, dim3((B + 255) / 256), dim3(256), 0, st, s, draft_tokens, k, n_acc,
                       next_tok, (unsigned long long*)hist, (unsigned long long*)committed, B);
    return hipGetLastError();
}

}  // namespace sv
