"""Helpers shared by the GPU parity tests (device buffers via torch; all compute goes through the
C ABI binding)."""
from __future__ import annotations

import numpy as np
import torch

import paper_2505_10259_amd as P
import synth

DEV = "cuda:0"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def host_model_pinned(shape, seed=0, std=0.02, unique_layers=None, gain_std=0.1):
    """Weights generated straight into pinned host memory (what the streamer reads).  RMSNorm gains are
    1 + N(0, gain_std^2) by default, so that a dropped, swapped or misplaced gain changes the result."""
    arena = P.binding.PinnedArena()
    hm = synth.make_model(shape, seed=seed, alloc=arena.alloc, std=std, unique_layers=unique_layers,
                          gain_std=gain_std)
    hm._arena = arena
    return hm


def forced_prefill_ids(route_ids, prompts, n_layers, Q):
    """Expert ids of a reference run's prefill in the row order spec_debug_force_routing documents:
    route_ids[b][l] is [len_b - 1, 2]; row (chunk * B + b) * Q + q holds prompt position chunk * Q + q."""
    B = len(prompts)
    pmax = max(len(p) - 1 for p in prompts)
    n_chunks = (pmax + Q - 1) // Q
    rows = max(1, n_chunks * B * Q)
    out = np.full((n_layers, rows, 2), -1, dtype=np.int32)
    for b in range(B):
        n = len(prompts[b]) - 1
        if n <= 0:
            continue
        pos = np.arange(n)
        r = (pos // Q * B + b) * Q + pos % Q
        for l in range(n_layers):
            out[l, r] = route_ids[b][l]
    return out


def forced_round_ids(traces, B, k, n_layers):
    """Same for one verify pass: traces maps sequence -> the reference's RoundTrace of this round (absent:
    the row keeps its own routing); row b * (k + 1) + i."""
    out = np.full((n_layers, B * (k + 1), 2), -1, dtype=np.int32)
    for b, t in traces.items():
        if t is not None and t.route_ids:
            for l in range(n_layers):
                out[l, b * (k + 1):(b + 1) * (k + 1)] = t.route_ids[l]
    return out


class GpuDecode:
    """Drives spec_draft / spec_verify round by round and records what the oracle's trace records."""

    def __init__(self, hm, draft_layers, draft_attn_only, prompts, k, max_new, mode="greedy", tau=1.0,
                 seed=0, forced_prefill=None, **cfg):
        self.hm, self.k, self.max_new, self.B = hm, k, max_new, len(prompts)
        self.V = hm.shape.vocab
        dm = hm.draft_view(draft_layers, draft_attn_only) if draft_layers else None
        ctx_max = max(len(p) for p in prompts) + max_new
        self.s = P.Session(hm, dm, batch_max=cfg.pop("batch_max", self.B), k_max=cfg.pop("k_max", k), ctx_max=ctx_max,
                           mode=P.SPEC_SAMPLE if mode == "sample" else P.SPEC_GREEDY, temperature=tau,
                           seed=seed, **cfg)
        self.prompts = prompts
        self._forced = None
        if forced_prefill is not None:        # [n_layers, rows, 2] expert ids of a reference run
            self._forced = dev(forced_prefill)
            P.spec_debug_force_routing(self.s.ctx, 0, self._forced, forced_prefill.shape[1])
        P.spec_prefill(self.s.ctx, 0, prompts, max_new)
        self.d_tok = torch.zeros((self.B, k), dtype=torch.int32, device=DEV)
        self.n_acc = torch.zeros(self.B, dtype=torch.int32, device=DEV)
        self.nxt = torch.zeros(self.B, dtype=torch.int32, device=DEV)
        self.logits = torch.zeros((self.B, k + 1, self.V), dtype=torch.float32, device=DEV)
        self.qlogits = torch.zeros((self.B, k, self.V), dtype=torch.float32, device=DEV)
        self.sample = mode == "sample"

    def round(self, forced_draft=None, want_logits=True, forced_route=None):
        ctx = self.s.ctx
        len_before = P.spec_get_lengths(ctx, 0, self.B)
        if forced_route is not None:
            self._forced = dev(forced_route)
            P.spec_debug_force_routing(ctx, 0, self._forced, forced_route.shape[1])
        if self.k == 0:
            P.spec_verify(ctx, 0, None, 0, self.n_acc, self.nxt)
        elif forced_draft is None:
            P.spec_draft(ctx, 0, self.k, self.d_tok)
            P.spec_verify(ctx, 0, None, self.k, self.n_acc, self.nxt)
        else:
            self.d_tok.copy_(dev(np.asarray(forced_draft, dtype=np.int32)))
            P.spec_verify(ctx, 0, self.d_tok, self.k, self.n_acc, self.nxt)
        P.spec_sync(ctx, 0)
        out = {"len_before": len_before, "draft": self.d_tok.cpu().numpy().copy(),
               "n_acc": self.n_acc.cpu().numpy().copy(), "next": self.nxt.cpu().numpy().copy()}
        if want_logits:
            P.spec_debug_logits(ctx, 0, self.logits)
            out["p_logits"] = self.logits.cpu().numpy().copy()
            if self.sample:
                P.spec_debug_draft_logits(ctx, 0, self.qlogits)
                out["q_logits"] = self.qlogits.cpu().numpy().copy()
        return out

    def run(self, max_rounds=10_000, want_logits=True, route_of_round=None):
        """route_of_round(r) -> forced expert ids of round r ([n_layers, B*(k+1), 2]) or None."""
        rounds = []
        for r in range(max_rounds):
            lens = P.spec_get_lengths(self.s.ctx, 0, self.B)
            if all(lens[b] - len(self.prompts[b]) >= self.max_new for b in range(self.B)):
                break
            rounds.append(self.round(want_logits=want_logits,
                                     forced_route=route_of_round(r) if route_of_round else None))
        return rounds

    def generated(self):
        return [P.spec_get_tokens(self.s.ctx, 0, b, len(self.prompts[b]) + self.max_new + 1)[len(self.prompts[b]):].tolist()
                for b in range(self.B)]

    def close(self):
        self.s.close()


def top2_gap(z: np.ndarray) -> np.ndarray:
    """Gap between the largest and second largest entry along the last axis."""
    part = np.partition(z, -2, axis=-1)
    return part[..., -1] - part[..., -2]
