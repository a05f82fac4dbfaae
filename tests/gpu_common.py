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


def host_model_pinned(shape, seed=0, std=0.02, unique_layers=None):
    """Weights generated straight into pinned host memory (what the streamer reads)."""
    arena = P.binding.PinnedArena()
    hm = synth.make_model(shape, seed=seed, alloc=arena.alloc, std=std, unique_layers=unique_layers)
    hm._arena = arena
    return hm


class GpuDecode:
    """Drives spec_draft / spec_verify round by round and records what the oracle's trace records."""

    def __init__(self, hm, draft_layers, draft_attn_only, prompts, k, max_new, mode="greedy", tau=1.0,
                 seed=0, **cfg):
        self.hm, self.k, self.max_new, self.B = hm, k, max_new, len(prompts)
        self.V = hm.shape.vocab
        dm = hm.draft_view(draft_layers, draft_attn_only) if draft_layers else None
        ctx_max = max(len(p) for p in prompts) + max_new
        self.s = P.Session(hm, dm, batch_max=self.B, k_max=k, ctx_max=ctx_max,
                           mode=P.SPEC_SAMPLE if mode == "sample" else P.SPEC_GREEDY, temperature=tau,
                           seed=seed, **cfg)
        self.prompts = prompts
        P.spec_prefill(self.s.ctx, 0, prompts, max_new)
        self.d_tok = torch.zeros((self.B, k), dtype=torch.int32, device=DEV)
        self.n_acc = torch.zeros(self.B, dtype=torch.int32, device=DEV)
        self.nxt = torch.zeros(self.B, dtype=torch.int32, device=DEV)
        self.logits = torch.zeros((self.B, k + 1, self.V), dtype=torch.float32, device=DEV)
        self.qlogits = torch.zeros((self.B, k, self.V), dtype=torch.float32, device=DEV)
        self.sample = mode == "sample"

    def round(self, forced_draft=None, want_logits=True):
        ctx = self.s.ctx
        len_before = P.spec_get_lengths(ctx, 0, self.B)
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

    def run(self, max_rounds=10_000, want_logits=True):
        rounds = []
        for _ in range(max_rounds):
            lens = P.spec_get_lengths(self.s.ctx, 0, self.B)
            if all(lens[b] - len(self.prompts[b]) >= self.max_new for b in range(self.B)):
                break
            rounds.append(self.round(want_logits=want_logits))
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
