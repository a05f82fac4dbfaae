"""Closed-form sizes of a decoder shape and the planner's memory / latency model.

TEST INFRASTRUCTURE ONLY.  Formulas written from the architecture, independently of the
blob-layout code the product uses, so that each can check the other.
"""
from __future__ import annotations


def attention_params(s) -> int:
    """Wq, Wk, Wv, Wo of one layer."""
    return s.d_model * (s.n_q_heads + 2 * s.n_kv_heads) * s.head_dim + s.n_q_heads * s.head_dim * s.d_model


def expert_params(s) -> int:
    """One SwiGLU expert: gate, up, down."""
    return 3 * s.d_model * s.d_ff


def layer_params(s) -> int:
    n = attention_params(s) + s.d_model                       # + attention norm gain
    if s.attn_only:
        return n
    n += s.d_model                                            # post-attention norm gain
    if s.n_experts > 0:
        n += s.n_experts * s.d_model + s.n_experts * expert_params(s)
    else:
        n += expert_params(s)
    return n


def model_params(s) -> int:
    return s.n_layers * layer_params(s) + 2 * s.vocab * s.d_model + s.d_model


def kv_bytes_per_token_per_layer(s) -> int:
    return 2 * s.n_kv_heads * s.head_dim * s.elem_bytes


def verify_flops_per_token_per_layer(s, ctx: int) -> float:
    """Multiply-add = 2 FLOP.  Projections + top-k experts + attention over ctx keys."""
    proj = 2.0 * attention_params(s)
    act = s.top_k if s.n_experts > 0 else 1
    ffn = 2.0 * act * expert_params(s)
    attn = 4.0 * s.n_q_heads * s.head_dim * ctx
    return proj + ffn + attn


def v_decoding(v_target_resident: int, v_draft: int, bs_draft: int, l_input: int, n_generated: int,
               v_draft_kv_per_token: int) -> int:
    """GPU memory in the decoding phase (Appendix A.1, "Memory constraint"): target
    parameters held on the GPU + draft parameters + the draft's KV cache for bs_draft
    sequences of l_input + n_generated tokens."""
    return v_target_resident + v_draft + bs_draft * (l_input + n_generated) * v_draft_kv_per_token


def t_decoding(t_target: float, t_draft: float) -> float:
    """Decode latency of one interleaved slot: the slower of verify and draft
    (Section 4.3, "Inference Latency")."""
    return max(t_target, t_draft)
