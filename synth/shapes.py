"""Model shapes, the host weight-blob format, and the benchmark workloads.

The five workloads are the configurations this build is measured on.  The paper's
targets are Mixtral-8x7B and Mixtral-8x22B (Section 5.1, "Implementation"/"Models");
only their *shapes* are used here, with random-init weights.

Host weight format (what ``make_model`` writes and the HIP library's ``spec_init``
reads).  All tensors are row-major ``[out_features, in_features]`` (so the
contraction dimension is contiguous), elements are f32 or bf16 bit patterns, and
every tensor starts at a multiple of ``ALIGN_ELEMS`` elements inside its blob.

  layer blob (one per decoder layer), in this order:
      g1    [d]                    attention RMSNorm gain
      wqkv  [(Hq + 2*Hkv)*dh, d]   query rows, then key rows, then value rows
      wo    [d, Hq*dh]
      -- the bytes up to here are the "attention part" (all an attention-only
         draft layer needs) --
      g2    [d]                    post-attention RMSNorm gain
      wr    [E, d]                 router (MoE only, E > 0)
      per expert e = 0..E-1 (or once, for a dense FFN with E == 0):
          w1_e [F, d]  gate projection
          w3_e [F, d]  up projection
          w2_e [d, F]  down projection
  global blob:
      emb   [V, d]                 token embedding
      gf    [d]                    final RMSNorm gain
      head  [V, d]                 LM head
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Tuple

ALIGN_ELEMS = 128


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    n_experts: int = 0          # 0 = dense SwiGLU FFN
    top_k: int = 2              # experts per token when n_experts > 0
    rope_theta: float = 1.0e4
    rms_eps: float = 1.0e-5
    dtype: str = "bf16"         # storage + GEMM-input type: "bf16" or "f32"
    attn_only: bool = False     # draft truncation: layers have no g2 / FFN / MoE

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def qkv_rows(self) -> int:
        return (self.n_q_heads + 2 * self.n_kv_heads) * self.head_dim

    def layer_tensors(self) -> List[Tuple[str, Tuple[int, ...]]]:
        d, F = self.d_model, self.d_ff
        t: List[Tuple[str, Tuple[int, ...]]] = [
            ("g1", (d,)),
            ("wqkv", (self.qkv_rows, d)),
            ("wo", (d, self.n_q_heads * self.head_dim)),
        ]
        if self.attn_only:
            return t
        t.append(("g2", (d,)))
        if self.n_experts > 0:
            t.append(("wr", (self.n_experts, d)))
            for e in range(self.n_experts):
                t += [(f"w1_{e}", (F, d)), (f"w3_{e}", (F, d)), (f"w2_{e}", (d, F))]
        else:
            t += [("w1_0", (F, d)), ("w3_0", (F, d)), ("w2_0", (d, F))]
        return t

    def global_tensors(self) -> List[Tuple[str, Tuple[int, ...]]]:
        return [("emb", (self.vocab, self.d_model)), ("gf", (self.d_model,)),
                ("head", (self.vocab, self.d_model))]

    @staticmethod
    def _layout(tensors) -> Tuple[Dict[str, Tuple[int, Tuple[int, ...]]], int]:
        off, out = 0, {}
        for name, shp in tensors:
            n = 1
            for s in shp:
                n *= s
            out[name] = (off, shp)
            off += (n + ALIGN_ELEMS - 1) // ALIGN_ELEMS * ALIGN_ELEMS
        return out, off

    def layer_layout(self):
        """name -> (element offset, shape); total elements of one layer blob."""
        return self._layout(self.layer_tensors())

    def global_layout(self):
        return self._layout(self.global_tensors())

    def attn_part_elems(self) -> int:
        """Elements of the blob prefix holding g1, wqkv, wo."""
        return replace(self, attn_only=True).layer_layout()[1]

    def n_params(self) -> int:
        n = 0
        for _, shp in self.layer_tensors():
            m = 1
            for s in shp:
                m *= s
            n += m
        n *= self.n_layers
        for _, shp in self.global_tensors():
            m = 1
            for s in shp:
                m *= s
            n += m
        return n

    def draft(self, n_layers: int, attn_only: bool) -> "ModelShape":
        """Shape of a draft that is the first ``n_layers`` layers of this model."""
        return replace(self, n_layers=n_layers, attn_only=attn_only)


@dataclass(frozen=True)
class Workload:
    name: str
    target: ModelShape
    draft_layers: int
    draft_attn_only: bool
    batch: int                   # total sequences
    k: int                       # draft tokens per round
    prompt_len: Tuple[int, int]  # inclusive range; equal ends = fixed length
    max_new: int
    mode: str = "greedy"         # "greedy" | "sample"
    temperature: float = 1.0
    hbm_weight_budget: int = 0   # bytes; 0 = everything resident
    n_sub_batches: int = 1
    ctx: int = 0                 # layer microbenchmark: tokens already in the KV cache
    note: str = ""

    @property
    def draft(self) -> ModelShape:
        return self.target.draft(self.draft_layers, self.draft_attn_only)


_MIXTRAL_8X7B = ModelShape(n_layers=32, d_model=4096, n_q_heads=32, n_kv_heads=8, head_dim=128,
                           d_ff=14336, vocab=32000, n_experts=8, top_k=2, rope_theta=1.0e6)
_MIXTRAL_8X22B = ModelShape(n_layers=56, d_model=6144, n_q_heads=48, n_kv_heads=8, head_dim=128,
                            d_ff=16384, vocab=32768, n_experts=8, top_k=2, rope_theta=1.0e6)
_TINY = ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=4, head_dim=64, d_ff=1024,
                   vocab=512, n_experts=0, rope_theta=1.0e4, dtype="f32")

GB = 10 ** 9

WORKLOADS: Dict[str, Workload] = {
    "cfg1": Workload("cfg1", _TINY, draft_layers=1, draft_attn_only=False, batch=4, k=4,
                     prompt_len=(32, 32), max_new=16,
                     note="tiny fp32 greedy; whole run is compared with the oracle"),
    "cfg2": Workload("cfg2", replace(_MIXTRAL_8X7B, n_layers=1), draft_layers=0,
                     draft_attn_only=True, batch=256, k=8, prompt_len=(0, 0), max_new=0, ctx=2048,
                     note="one Mixtral-8x7B-shaped layer, weights in HBM, T = 256*9 = 2304"),
    "cfg3": Workload("cfg3", _MIXTRAL_8X7B, draft_layers=4, draft_attn_only=True, batch=64, k=4,
                     prompt_len=(512, 512), max_new=256, hbm_weight_budget=24 * GB,
                     note="Mixtral-8x7B-shaped target streamed from pinned host memory"),
    "cfg4": Workload("cfg4", _MIXTRAL_8X22B, draft_layers=6, draft_attn_only=True, batch=128, k=6,
                     prompt_len=(256, 1024), max_new=128, hbm_weight_budget=64 * GB,
                     note="Mixtral-8x22B-shaped target streamed from pinned host memory"),
    "cfg5": Workload("cfg5", _MIXTRAL_8X7B, draft_layers=4, draft_attn_only=True, batch=256, k=6,
                     prompt_len=(512, 512), max_new=128, mode="sample", temperature=0.8,
                     hbm_weight_budget=24 * GB, n_sub_batches=2,
                     note="stochastic speculative sampling, two interleaved sub-batches"),
}


def workload(name: str) -> Workload:
    return WORKLOADS[name]


def mini_moe_shape(n_layers: int = 2, d_model: int = 256, n_q_heads: int = 4, n_kv_heads: int = 2,
                   head_dim: int = 128, d_ff: int = 512, vocab: int = 1024, n_experts: int = 8,
                   dtype: str = "bf16") -> ModelShape:
    """A small model with the structure of the Mixtral shapes (GQA, head_dim 128, top-2 of 8
    experts) that the CPU oracle can run end to end in seconds."""
    return ModelShape(n_layers=n_layers, d_model=d_model, n_q_heads=n_q_heads,
                      n_kv_heads=n_kv_heads, head_dim=head_dim, d_ff=d_ff, vocab=vocab,
                      n_experts=n_experts, top_k=2, rope_theta=1.0e6, dtype=dtype)
