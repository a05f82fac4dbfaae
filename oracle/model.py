"""Oracle decoder: the network the target and draft models compute, in float64 NumPy.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper runs stock Mixtral / Mistral decoder stacks (Section 5.1) and prints no
equations for them, so this file writes the standard pre-norm decoder out directly:

    x   = Emb[token]
    per layer:
        h      = RMSNorm(x; g1)
        q,k,v  = h Wq^T, h Wk^T, h Wv^T            (rows of wqkv: q heads, k heads, v heads)
        q,k    = RoPE(q,k; position)               (half-split pairing (i, i + dh/2))
        cache  += (k, v)
        a_j    = softmax(q_j K_{j//g}^T / sqrt(dh), causal) V_{j//g}      (g = Hq / Hkv)
        x     += a Wo^T
        -- attention-only draft layers stop here --
        h2     = RMSNorm(x; g2)
        MoE :  r = h2 Wr^T ; top-2 experts (lowest id wins ties);
               w = softmax over the two chosen logits;
               x += sum_e w_e * ( silu(h2 W1_e^T) * (h2 W3_e^T) ) W2_e^T
        dense: x += ( silu(h2 W1^T) * (h2 W3^T) ) W2^T
    logits = RMSNorm(x; gf) Whead^T

Weight matrices are [out_features, in_features] float32 arrays (bf16 models: the
bf16 values widened, i.e. exactly the numbers the accelerator reads).

Precision.  All arithmetic is float64.  With ``act="bf16"`` the activations are
rounded to bf16 at the points where a bf16 model stores them (h, q, k, v, attention
output, the SwiGLU product, the final normalised state); the residual stream x, the
softmax, the router logits and all accumulations stay unrounded.  With ``act="f64"``
nothing is rounded.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np


def round_bf16(a: np.ndarray) -> np.ndarray:
    """float64 -> float32 -> bf16 (both nearest-even) -> float64."""
    u = np.asarray(a, dtype=np.float64).astype(np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16 << 16
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * g


def rope(v: np.ndarray, positions: np.ndarray, theta: float) -> np.ndarray:
    """v: [n, H, dh]; rotate pair (i, i + dh/2) of every head by positions[n] * theta^(-2i/dh)."""
    n, H, dh = v.shape
    half = dh // 2
    inv = theta ** (-(np.arange(half, dtype=np.float64) * 2.0) / dh)
    ang = positions.astype(np.float64)[:, None] * inv[None, :]          # [n, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = v[..., :half], v[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


class KVCache:
    """Per-sequence cache as plain arrays: k[l], v[l] are [Hkv, capacity, dh]; ``length``
    is the number of valid positions."""

    def __init__(self, n_layers: int, n_kv: int, dh: int, capacity: int):
        self.k = [np.zeros((n_kv, capacity, dh)) for _ in range(n_layers)]
        self.v = [np.zeros((n_kv, capacity, dh)) for _ in range(n_layers)]
        self.length = 0
        self.capacity = capacity


class Decoder:
    def __init__(self, shape, layers: List[Dict[str, np.ndarray]], glob: Dict[str, np.ndarray],
                 act: str = "f64"):
        assert act in ("f64", "bf16")
        self.s = shape
        self.layers = layers
        self.glob = glob
        self.r = round_bf16 if act == "bf16" else (lambda a: a)
        self._gap23 = None             # last route() call: 2nd-minus-3rd router logit gap per row
        self._ids = None               # last route() call: chosen expert ids per row
        self.last_min_gap: List[float] = []   # last forward(): smallest such gap per sequence
        # last forward(): per sequence, per layer, the chosen expert ids [n_b, 2] (a record only; tests
        # hand it to the accelerator's forced-routing aid)
        self.last_route_ids: List[List[np.ndarray]] = []
        assert len(layers) == shape.n_layers

    # -- pieces ------------------------------------------------------------------------
    def new_cache(self, capacity: int) -> KVCache:
        s = self.s
        return KVCache(s.n_layers, s.n_kv_heads, s.head_dim, capacity)

    def embed(self, tokens: np.ndarray) -> np.ndarray:
        return self.glob["emb"][np.asarray(tokens, dtype=np.int64)].astype(np.float64)

    def attention_part(self, l: int, x: np.ndarray, cache: KVCache, pos0: int) -> np.ndarray:
        """x: [n, d] residual rows of ONE sequence at positions pos0..pos0+n-1; appends to the
        cache (positions >= pos0 already there are overwritten) and returns x + attention."""
        s, W = self.s, self.layers[l]
        n = x.shape[0]
        Hq, Hkv, dh = s.n_q_heads, s.n_kv_heads, s.head_dim
        g = Hq // Hkv
        h = self.r(rmsnorm(x, W["g1"].astype(np.float64), s.rms_eps))
        qkv = h @ W["wqkv"].astype(np.float64).T
        q = qkv[:, :Hq * dh].reshape(n, Hq, dh)
        k = qkv[:, Hq * dh:(Hq + Hkv) * dh].reshape(n, Hkv, dh)
        v = qkv[:, (Hq + Hkv) * dh:].reshape(n, Hkv, dh)
        pos = pos0 + np.arange(n)
        q = self.r(rope(q, pos, s.rope_theta))
        k = self.r(rope(k, pos, s.rope_theta))
        v = self.r(v)
        assert pos0 + n <= cache.capacity
        cache.k[l][:, pos0:pos0 + n, :] = k.transpose(1, 0, 2)
        cache.v[l][:, pos0:pos0 + n, :] = v.transpose(1, 0, 2)
        tot = pos0 + n
        keypos = np.arange(tot)
        masked = keypos[None, :] > pos[:, None]                       # causal
        a = np.zeros((n, Hq, dh))
        for j in range(Hq):
            K, V = cache.k[l][j // g, :tot, :], cache.v[l][j // g, :tot, :]
            sc = (q[:, j, :] @ K.T) / np.sqrt(dh)
            sc = np.where(masked, -np.inf, sc)
            sc = sc - sc.max(axis=1, keepdims=True)
            p = np.exp(sc)
            p = p / p.sum(axis=1, keepdims=True)
            a[:, j, :] = p @ V
        a = self.r(a.reshape(n, Hq * dh))
        return x + a @ W["wo"].astype(np.float64).T

    def route(self, l: int, h2: np.ndarray):
        """Top-2 routing.  Returns (expert ids [n,2], weights [n,2], router logits [n,E])."""
        rl = h2 @ self.layers[l]["wr"].astype(np.float64).T
        n, E = rl.shape
        ids = np.zeros((n, 2), dtype=np.int64)
        work = rl.copy()
        ids[:, 0] = np.argmax(work, axis=1)                # first maximum = lowest id on ties
        work[np.arange(n), ids[:, 0]] = -np.inf
        ids[:, 1] = np.argmax(work, axis=1)
        l0, l1 = rl[np.arange(n), ids[:, 0]], rl[np.arange(n), ids[:, 1]]
        w0 = 1.0 / (1.0 + np.exp(l1 - l0))
        self._ids = ids
        if E > 2:
            work[np.arange(n), ids[:, 1]] = -np.inf
            self._gap23 = l1 - work.max(axis=1)
        return ids, np.stack([w0, 1.0 - w0], axis=1), rl

    def ffn_part(self, l: int, x: np.ndarray, forced_route=None) -> np.ndarray:
        """x: [n, d] residual rows (any mix of sequences; rows are independent)."""
        s, W = self.s, self.layers[l]
        h2 = self.r(rmsnorm(x, W["g2"].astype(np.float64), s.rms_eps))

        def expert(e: int, rows: np.ndarray) -> np.ndarray:
            gate = rows @ W[f"w1_{e}"].astype(np.float64).T
            up = rows @ W[f"w3_{e}"].astype(np.float64).T
            u = self.r(silu(gate) * up)
            return u @ W[f"w2_{e}"].astype(np.float64).T

        if s.n_experts == 0:
            return x + expert(0, h2)
        ids, wts, _ = self.route(l, h2) if forced_route is None else (*forced_route, None)
        y = np.zeros_like(x)
        for e in range(s.n_experts):                      # fixed expert order
            for slot in range(2):
                rows = np.nonzero(ids[:, slot] == e)[0]
                if rows.size:
                    y[rows] += wts[rows, slot][:, None] * expert(e, h2[rows])
        return x + y

    def head(self, x: np.ndarray) -> np.ndarray:
        hf = self.r(rmsnorm(x, self.glob["gf"].astype(np.float64), self.s.rms_eps))
        return hf @ self.glob["head"].astype(np.float64).T

    # -- whole forward -------------------------------------------------------------------
    def forward(self, caches: Sequence[KVCache], tokens: Sequence[np.ndarray],
                pos0: Sequence[int], want_logits: bool = True) -> Optional[List[np.ndarray]]:
        """Feed ``tokens[b]`` at positions ``pos0[b]..`` to sequence b (cache entries at or
        beyond pos0[b] are dropped first).  Returns per-sequence logits [n_b, V]."""
        B = len(caches)
        xs = [self.embed(t) for t in tokens]
        sizes = [x.shape[0] for x in xs]
        cuts = np.cumsum(sizes)[:-1]
        self.last_min_gap = [np.inf] * B
        self.last_route_ids = [[] for _ in range(B)]
        for l in range(self.s.n_layers):
            for b in range(B):
                if sizes[b]:
                    xs[b] = self.attention_part(l, xs[b], caches[b], pos0[b])
            if not self.s.attn_only:
                self._gap23 = None
                self._ids = None
                cat = self.ffn_part(l, np.concatenate(xs, axis=0))
                xs = list(np.split(cat, cuts, axis=0))
                if self._ids is not None:
                    for b, part in enumerate(np.split(self._ids, cuts)):
                        self.last_route_ids[b].append(part.copy())
                if self._gap23 is not None:         # diagnostics only: how close routing was to a tie
                    for b, gp in enumerate(np.split(self._gap23, cuts)):
                        if gp.size:
                            self.last_min_gap[b] = min(self.last_min_gap[b], float(gp.min()))
        for b in range(B):
            caches[b].length = pos0[b] + sizes[b]
        if not want_logits:
            return None
        return [self.head(x) for x in xs]

    def forward_full(self, tokens: np.ndarray) -> np.ndarray:
        """Logits of every position of one sequence, recomputed from scratch (no reuse)."""
        c = self.new_cache(len(tokens))
        return self.forward([c], [np.asarray(tokens)], [0])[0]


def build(host_model, act: Optional[str] = None) -> Decoder:
    """Decoder over an object exposing ``shape``, ``layer(l)`` and ``globals()`` that return
    name -> float32 arrays (bf16 already widened)."""
    s = host_model.shape
    if act is None:
        act = "bf16" if s.dtype == "bf16" else "f64"
    return Decoder(s, [host_model.layer(l) for l in range(s.n_layers)], host_model.globals(), act)
