"""TEST INFRASTRUCTURE ONLY (imported by tests/, never by the library or its binding).

ParaSpec planner (Section 4.3 and Appendix A.1, "ParaSpec Planner"), written out as the paper states
it: maximise  throughput = N_generated / T_generation  subject to the prefill- and decoding-phase
GPU memory constraints, by exhaustive search over the four parameters the paper names (batch size
bs, prefill batch bs_prefill, draft batch bs_draft, candidates per round n_cand).

Every quantity of the cost model is one function that follows one numbered relation of the appendix:

  * expected tokens per round  E[n] = sum_{k=1}^{n_cand+1} k P[n = k]  with the appendix's PMF
    (P = p^(k-1)(1-p) for k <= n_cand, p^n_cand for k = n_cand+1).  The closed form PRINTED in the
    appendix does not equal that sum (at n_cand = 1 it gives 1 + p - p^2 instead of 1 + p); the sum
    is taken as the definition, and it equals (1 - p^(n_cand+1)) / (1 - p).
  * N_generated = bs * n_iter * E[n]                       ("Generated Tokens")
  * T_generation = T_prefill + T_decoding                  ("Inference Latency")
  * T_prefill = ceil(bs / bs_prefill) * (T_c2g_para + T_gpu_comp)
  * per round  T_round = max(T_target_decoding, T_draft)
  * T_draft = ceil(bs / bs_draft) * (T_draft_prefill + (n_cand - 1) T_draft_decoding)
  * T_target_decoding = sum over layers of  max(T_attention, T_ffn_c2g) + T_ffn_gpu,
    T_attention = n_cand * bs * t_attention_unit
  * V_prefill  = V_target_prefill + bs_prefill * l_input * v_target_kv        <= capacity
  * V_decoding = V_target_ffn + V_draft + bs_draft * (l_input + n_generate) * v_draft_kv  <= capacity

Readings (the paper leaves these open):
  * n_iter: rounds needed for n_generate tokens per sequence = ceil(n_generate / E[n]); T_decoding =
    n_iter * T_round.
  * The appendix treats the per-batch times as constants measured by a profiling run.  Optional linear
    terms (per sequence / per verified token) generalise them; with the defaults (0) the relations are
    exactly the appendix's.
  * Layers whose weights are resident in GPU memory have T_ffn_c2g = 0 (n_layer_streamed of the
    n_layer layers are streamed).
  * Where the target's KV cache is kept in GPU memory during decoding (this build's layout, not the
    paper's), v_target_kv_decoding > 0 adds bs * (l_input + n_generate) * v_target_kv_decoding to
    V_decoding; 0 reproduces the appendix.
  * Ties in throughput: the first candidate in the order bs ascending, n_cand ascending, bs_prefill
    descending, bs_draft descending wins.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, asdict
from typing import Optional


@dataclass
class Profile:
    # workload
    n_layer: int
    n_layer_streamed: int
    l_input: int
    n_generate: int
    p_accept: float
    # search space
    bs_max: int
    n_cand_max: int
    # prefill phase (seconds)
    t_c2g_para: float               # streaming the target once
    t_gpu_prefill_comp: float       # GPU compute of one prefill batch
    # decoding phase (seconds)
    t_ffn_c2g: float                # streaming one layer's weights
    t_ffn_gpu: float                # GPU FFN compute of one layer for one verify pass
    t_attention_unit: float         # attention time per (sequence, candidate) per layer
    t_draft_prefill: float          # first draft step of a draft batch
    t_draft_decoding: float         # each further draft step of a draft batch
    # memory (bytes)
    gpu_mem_capacity: float
    v_target_prefill: float
    v_target_kv: float              # per token, prefill phase
    v_target_ffn: float
    v_draft: float
    v_draft_kv: float               # per token
    # optional generalisations (0 = the appendix as printed)
    t_ffn_gpu_per_token: float = 0.0        # added to t_ffn_gpu per verified token (bs * (n_cand + 1))
    t_draft_per_seq: float = 0.0            # added to both draft step times per sequence of the draft batch
    t_prefill_comp_per_seq: float = 0.0     # added to t_gpu_prefill_comp per sequence of the prefill batch
    v_target_kv_decoding: float = 0.0       # per token, decoding phase, target KV held on the GPU


@dataclass
class Plan:
    feasible: bool
    bs: int = 0
    bs_prefill: int = 0
    bs_draft: int = 0
    n_cand: int = 0
    throughput: float = 0.0
    expected_tokens: float = 0.0
    n_iter: int = 0
    t_prefill: float = 0.0
    t_round: float = 0.0
    t_target_decoding: float = 0.0
    t_draft: float = 0.0
    v_prefill: float = 0.0
    v_decoding: float = 0.0


def expected_generated(p: float, n_cand: int) -> float:
    """E[n_generated] as the sum over the appendix's probability mass function."""
    e = 0.0
    for k in range(1, n_cand + 1):
        e += k * p ** (k - 1) * (1.0 - p)
    e += (n_cand + 1) * p ** n_cand
    return e


def t_prefill(pr: Profile, bs: int, bs_prefill: int) -> float:
    per_batch = pr.t_c2g_para + pr.t_gpu_prefill_comp + pr.t_prefill_comp_per_seq * bs_prefill
    return math.ceil(bs / bs_prefill) * per_batch


def t_draft(pr: Profile, bs: int, bs_draft: int, n_cand: int) -> float:
    first = pr.t_draft_prefill + pr.t_draft_per_seq * bs_draft
    later = pr.t_draft_decoding + pr.t_draft_per_seq * bs_draft
    return math.ceil(bs / bs_draft) * (first + (n_cand - 1) * later)


def t_target_decoding(pr: Profile, bs: int, n_cand: int) -> float:
    t_att = n_cand * bs * pr.t_attention_unit
    t_gpu = pr.t_ffn_gpu + pr.t_ffn_gpu_per_token * bs * (n_cand + 1)
    total = 0.0
    for layer in range(pr.n_layer):
        c2g = pr.t_ffn_c2g if layer < pr.n_layer_streamed else 0.0
        total += max(t_att, c2g) + t_gpu
    return total


def v_prefill(pr: Profile, bs_prefill: int) -> float:
    return pr.v_target_prefill + bs_prefill * pr.l_input * pr.v_target_kv


def v_decoding(pr: Profile, bs: int, bs_draft: int) -> float:
    ctx = pr.l_input + pr.n_generate
    return pr.v_target_ffn + pr.v_draft + bs_draft * ctx * pr.v_draft_kv + bs * ctx * pr.v_target_kv_decoding


def evaluate(pr: Profile, bs: int, bs_prefill: int, bs_draft: int, n_cand: int) -> Plan:
    """Cost model at one point of the search space (feasible = both memory constraints hold)."""
    vp, vd = v_prefill(pr, bs_prefill), v_decoding(pr, bs, bs_draft)
    e = expected_generated(pr.p_accept, n_cand)
    n_iter = math.ceil(pr.n_generate / e)
    tt, td = t_target_decoding(pr, bs, n_cand), t_draft(pr, bs, bs_draft, n_cand)
    t_round = max(tt, td)
    tp = t_prefill(pr, bs, bs_prefill)
    n_gen = bs * n_iter * e
    return Plan(feasible=vp <= pr.gpu_mem_capacity and vd <= pr.gpu_mem_capacity, bs=bs, bs_prefill=bs_prefill,
                bs_draft=bs_draft, n_cand=n_cand, throughput=n_gen / (tp + n_iter * t_round), expected_tokens=e,
                n_iter=n_iter, t_prefill=tp, t_round=t_round, t_target_decoding=tt, t_draft=td, v_prefill=vp,
                v_decoding=vd)


def plan(pr: Profile) -> Plan:
    """Exhaustive search, in the tie-breaking order stated in the module header."""
    best: Optional[Plan] = None
    for bs in range(1, pr.bs_max + 1):
        for n_cand in range(1, pr.n_cand_max + 1):
            for bs_prefill in range(bs, 0, -1):
                for bs_draft in range(bs, 0, -1):
                    cand = evaluate(pr, bs, bs_prefill, bs_draft, n_cand)
                    if cand.feasible and (best is None or cand.throughput > best.throughput):
                        best = cand
    return best if best is not None else Plan(feasible=False)


def as_dict(pr: Profile) -> dict:
    return asdict(pr)
