"""Oracle speculative decoding: the draft-then-verify loop and its accept/reject rule.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Greedy form (Section 2.2 and the "Generated Tokens" paragraph of Appendix A.1): each
round the draft proposes k candidate tokens, the target scores all of them in one
forward pass, the longest prefix of candidates that the target itself would have
produced is kept, and the target contributes one further token; a round therefore emits
between 1 and k+1 tokens.  By construction the emitted sequence equals plain greedy
decoding with the target.

Stochastic form.  The paper only cites the speculative-sampling works for it, so the
standard rule is written out here: candidate d_i ~ q_i is kept when u * q_i(d_i) <
p_{i-1}(d_i); at the first rejection (after n kept) the next token is drawn from
max(0, p_n - q_{n+1}) renormalised; when all k are kept it is drawn from p_k.  The
emitted tokens are then distributed exactly as plain sampling from the target.

Readings fixed here (the paper is silent on all of them):
  * argmax ties: lowest token id wins;
  * temperature tau divides target and draft logits alike before softmax;
  * inverse-CDF draw: the smallest id whose running sum (ascending id order) exceeds
    u * total, total being the actual sum of the weights;
  * acceptance is the strict inequality u * q < p;
  * if max(0, p - q) sums to zero the draw falls back to p;
  * a sequence stops at exactly max_new emitted tokens (the last round is clipped).

State per sequence: committed tokens s[0..len); the target cache covers [0, len-1); the
draft cache covers [0, m) with m <= len-1.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from . import philox


# ----------------------------------------------------------------------------------------
# rule on given logits
# ----------------------------------------------------------------------------------------
def argmax_lowest(z: np.ndarray) -> int:
    return int(np.argmax(z))               # numpy returns the first (lowest-id) maximum


def softmax_t(z: np.ndarray, tau: float) -> np.ndarray:
    y = np.asarray(z, dtype=np.float64) / tau
    y = y - y.max()
    e = np.exp(y)
    return e / e.sum()


def sample_inverse_cdf(w: np.ndarray, u: float) -> int:
    c = np.cumsum(np.asarray(w, dtype=np.float64))
    return int(np.searchsorted(c, u * c[-1], side="right"))


def accept_greedy(p_logits: np.ndarray, d: Sequence[int]):
    """p_logits [k+1, V] (row i-1 scores the slot candidate d_i fills), d [k].
    Returns (n kept, next token)."""
    k = len(d)
    n = 0
    while n < k and int(d[n]) == argmax_lowest(p_logits[n]):
        n += 1
    return n, argmax_lowest(p_logits[n])


def accept_sample(p_logits: np.ndarray, q_logits: np.ndarray, d: Sequence[int],
                  u_accept: Sequence[float], u_resample: Sequence[float], tau: float,
                  margins: Optional[list] = None):
    """p_logits [k+1, V], q_logits [k, V] (row i-1 is the draft distribution candidate d_i
    was drawn from), u_accept[i-1] tests d_i, u_resample[n] draws the token after n kept.
    Returns (n, next).  ``margins`` collects |u*q - p| of every test made."""
    k = len(d)
    n = 0
    while n < k:
        p = softmax_t(p_logits[n], tau)
        q = softmax_t(q_logits[n], tau)
        lhs, rhs = u_accept[n] * q[int(d[n])], p[int(d[n])]
        if margins is not None:
            margins.append(abs(lhs - rhs) / max(rhs, 1e-300))
        if not lhs < rhs:
            break
        n += 1
    p = softmax_t(p_logits[n], tau)
    if n < k:
        r = np.maximum(0.0, p - softmax_t(q_logits[n], tau))
        if r.sum() <= 0.0:
            r = p
    else:
        r = p
    return n, sample_inverse_cdf(r, u_resample[n])


def expected_generated(p: float, k: int) -> float:
    """Mean tokens emitted per round when each candidate is kept independently with
    probability p (Appendix A.1, "Generated Tokens").  Summing the paper's own
    distribution, P[j] = p^(j-1) (1-p) for j <= k and P[k+1] = p^k, gives
    (1 - p^(k+1)) / (1 - p); the closed form printed there does not equal that sum (at k = 1
    it gives 1 + p - p^2 where the sum is 1 + p), so the sum is used."""
    if p == 1.0:
        return float(k + 1)
    return (1.0 - p ** (k + 1)) / (1.0 - p)


# ----------------------------------------------------------------------------------------
# decoding loops
# ----------------------------------------------------------------------------------------
@dataclass
class RoundTrace:
    seq: int
    rnd: int
    length_before: int
    draft_tokens: np.ndarray
    p_logits: np.ndarray
    q_logits: Optional[np.ndarray]
    n_accepted: int
    next_token: int
    committed: List[int]
    router_gap: float = float("inf")   # smallest 2nd-vs-3rd router logit gap of the target pass
    route_ids: Optional[List[np.ndarray]] = None   # per target layer, expert ids [k+1, 2] of the pass


@dataclass
class SeqState:
    tokens: List[int]
    n_prompt: int
    target_cache: object
    draft_cache: object
    m: int = 0                      # valid draft-cache positions
    n_new: int = 0


class ModelDraft:
    """Draft = a (small) Decoder with its own cache; proposes k tokens autoregressively."""

    def __init__(self, decoder):
        self.dec = decoder

    def new_cache(self, cap):
        return self.dec.new_cache(cap)

    def prefill(self, states):
        self.dec.forward([s.draft_cache for s in states], [np.asarray(s.tokens[:-1]) for s in states],
                         [0] * len(states), want_logits=False)
        for s in states:
            s.m = len(s.tokens) - 1

    def propose(self, states, k, mode, tau, u_draft):
        """Returns (tokens [B,k], logits [B,k,V]).  u_draft[b][i] draws candidate i (1-based)."""
        B = len(states)
        caches = [s.draft_cache for s in states]
        # catch-up: committed tokens the draft has not seen, except the last one
        tail = [np.asarray(s.tokens[s.m:len(s.tokens) - 1]) for s in states]
        if any(t.size for t in tail):
            self.dec.forward(caches, tail, [s.m for s in states], want_logits=False)
        for s in states:
            s.m = len(s.tokens) - 1
        prev = [s.tokens[-1] for s in states]
        toks = np.zeros((B, k), dtype=np.int64)
        logits = None
        for i in range(1, k + 1):
            z = self.dec.forward(caches, [np.asarray([t]) for t in prev],
                                 [len(s.tokens) - 2 + i for s in states])
            z = np.stack([zz[0] for zz in z])
            if logits is None:
                logits = np.zeros((B, k, z.shape[1]))
            logits[:, i - 1, :] = z
            for b in range(B):
                if mode == "greedy":
                    toks[b, i - 1] = argmax_lowest(z[b])
                else:
                    toks[b, i - 1] = sample_inverse_cdf(softmax_t(z[b], tau), u_draft[b][i])
            prev = [int(t) for t in toks[:, i - 1]]
        for s in states:
            s.m = len(s.tokens) - 1 + k            # positions len-1 .. len+k-2 written
        return toks, logits


class FixedDraft:
    """A 'draft' that proposes whatever ``fn(seq_tokens, k, rnd)`` returns (for the
    invariant that greedy output does not depend on the draft)."""

    def __init__(self, fn: Callable):
        self.fn = fn

    def new_cache(self, cap):
        return None

    def prefill(self, states):
        pass

    def propose(self, states, k, mode, tau, u_draft):
        assert mode == "greedy"
        toks = np.stack([np.asarray(self.fn(list(s.tokens), k), dtype=np.int64) for s in states])
        return toks, None


def speculative_decode(target, draft, prompts: Sequence[np.ndarray], k: int, max_new: int,
                       mode: str = "greedy", tau: float = 1.0, seed: int = 0,
                       seq_ids: Optional[Sequence[int]] = None,
                       trace: Optional[List[RoundTrace]] = None, keep_logits: bool = True):
    """Run the draft/verify loop to ``max_new`` new tokens per sequence.
    Returns (list of generated-token lists, stats dict)."""
    B = len(prompts)
    seq_ids = list(range(B)) if seq_ids is None else list(seq_ids)
    cap = max(len(p) for p in prompts) + max_new + k + 2
    states = [SeqState([int(t) for t in p], len(p), target.new_cache(cap), draft.new_cache(cap))
              for p in prompts]
    # prefill: the target cache covers all but the last committed token
    target.forward([s.target_cache for s in states], [np.asarray(s.tokens[:-1]) for s in states],
                   [0] * B, want_logits=False)
    prefill_gap = list(getattr(target, "last_min_gap", [])) or [float("inf")] * B
    prefill_routes = list(getattr(target, "last_route_ids", [])) or [[] for _ in range(B)]
    draft.prefill(states)
    hist = np.zeros(k + 1, dtype=np.int64)
    rnd = 0
    while True:
        live = [b for b in range(B) if states[b].n_new < max_new]
        if not live:
            break
        st = [states[b] for b in live]
        uni = [philox.round_uniforms(seed, rnd, seq_ids[b], k) for b in live] if mode == "sample" else None
        d, qz = draft.propose(st, k, mode, tau, [u[0] for u in uni] if uni else None)
        feed = [np.concatenate([[s.tokens[-1]], d[i]]) for i, s in enumerate(st)]
        pz = target.forward([s.target_cache for s in st], feed, [len(s.tokens) - 1 for s in st])
        gaps = list(getattr(target, "last_min_gap", [])) or [float("inf")] * len(st)
        routes = list(getattr(target, "last_route_ids", [])) or [None] * len(st)
        for i, s in enumerate(st):
            if mode == "greedy":
                n, nxt = accept_greedy(pz[i], d[i])
            else:
                n, nxt = accept_sample(pz[i], qz[i], d[i], uni[i][1][1:], uni[i][2], tau)
            new = [int(t) for t in d[i][:n]] + [nxt]
            new = new[:max_new - s.n_new]
            if trace is not None:
                trace.append(RoundTrace(seq_ids[live[i]], rnd, len(s.tokens), d[i].copy(),
                                        pz[i].copy() if keep_logits else None,
                                        None if qz is None or not keep_logits else qz[i].copy(),
                                        n, nxt, new, gaps[i], routes[i]))
            hist[n] += 1
            s.tokens += new
            s.n_new += len(new)
            # rollback: caches keep only positions of committed tokens but the last
            s.target_cache.length = len(s.tokens) - 1
            s.m = min(s.m, len(s.tokens) - 1)
        rnd += 1
    out = [s.tokens[s.n_prompt:] for s in states]
    return out, {"rounds": rnd, "accept_hist": hist, "prefill_router_gap": prefill_gap,
                 "prefill_route_ids": prefill_routes}


def plain_decode(target, prompts: Sequence[np.ndarray], max_new: int, mode: str = "greedy",
                 tau: float = 1.0, uniforms: Optional[np.ndarray] = None):
    """The definition the speculative loop must reproduce: one token per target forward.
    ``uniforms`` [B, max_new] drive sampling mode."""
    B = len(prompts)
    cap = max(len(p) for p in prompts) + max_new + 1
    caches = [target.new_cache(cap) for _ in range(B)]
    toks = [[int(t) for t in p] for p in prompts]
    target.forward(caches, [np.asarray(t[:-1]) for t in toks], [0] * B, want_logits=False)
    for step in range(max_new):
        z = target.forward(caches, [np.asarray([t[-1]]) for t in toks], [len(t) - 1 for t in toks])
        for b in range(B):
            if mode == "greedy":
                toks[b].append(argmax_lowest(z[b][0]))
            else:
                toks[b].append(sample_inverse_cdf(softmax_t(z[b][0], tau), float(uniforms[b, step])))
    return [t[len(p):] for t, p in zip(toks, prompts)]
