"""ParaSpec planner (Section 4.3; Appendix A.1): pins of the oracle's cost model against what the
paper and the mathematics fix, then the library's planner (C ABI, host arithmetic, no GPU needed)
against the oracle's exhaustive search."""
import itertools
import math

import numpy as np
import pytest

from oracle import planner as op
from oracle import spec as ospec


def _profile(**over):
    base = dict(n_layer=6, n_layer_streamed=4, l_input=40, n_generate=24, p_accept=0.6, bs_max=9, n_cand_max=5,
                t_c2g_para=1.0, t_gpu_prefill_comp=0.1, t_ffn_c2g=0.05, t_ffn_gpu=0.004, t_attention_unit=0.002,
                t_draft_prefill=0.03, t_draft_decoding=0.02, gpu_mem_capacity=1000.0, v_target_prefill=400.0,
                v_target_kv=0.5, v_target_ffn=300.0, v_draft=100.0, v_draft_kv=1.25)
    base.update(over)
    return op.Profile(**base)


# ---- pins of the oracle -------------------------------------------------------------------------
def test_expected_tokens_is_the_sum_of_the_pmf_and_has_the_geometric_closed_form():
    for p, n in itertools.product([0.0, 0.1, 0.5, 0.9, 0.99], [1, 2, 5, 8, 16]):
        pmf = [p ** (k - 1) * (1 - p) for k in range(1, n + 1)] + [p ** n]
        assert abs(sum(pmf) - 1.0) < 1e-12                      # the appendix's PMF is a distribution
        e = op.expected_generated(p, n)
        assert abs(e - sum((k + 1) * q for k, q in enumerate(pmf))) < 1e-12
        assert abs(e - (1 - p ** (n + 1)) / (1 - p)) < 1e-11    # geometric series
        assert abs(e - ospec.expected_generated(p, n)) < 1e-11  # the decode oracle's formula
    # the form printed in the appendix is NOT that sum: at n_cand = 1 it gives 1 + p - p^2
    p = 0.5
    printed = (1 * p ** 3 - 2 * p ** 2 + 1) / (1 - p)
    assert abs(printed - (1 + p - p * p)) < 1e-12 and abs(op.expected_generated(p, 1) - (1 + p)) < 1e-12


def test_expected_tokens_matches_simulation_of_the_acceptance_process():
    rng = np.random.default_rng(0)
    p, n = 0.7, 6
    ok = rng.random((200_000, n)) < p
    first_reject = np.where(ok.all(axis=1), n, np.argmin(ok, axis=1))
    assert abs((first_reject + 1).mean() - op.expected_generated(p, n)) < 0.02


def test_latency_terms_reduce_to_the_printed_relations():
    pr = _profile()
    # T_prefill = ceil(bs / bs_prefill) * (T_c2g + T_comp)
    assert op.t_prefill(pr, 7, 3) == pytest.approx(3 * 1.1)
    assert op.t_prefill(pr, 6, 3) == pytest.approx(2 * 1.1)
    # T_draft = ceil(bs / bs_draft) * (T_draft_prefill + (n_cand - 1) T_draft_decoding)
    assert op.t_draft(pr, 8, 3, 4) == pytest.approx(3 * (0.03 + 3 * 0.02))
    assert op.t_draft(pr, 8, 8, 1) == pytest.approx(0.03)
    # T_target: attention below the transfer time -> streamed layers cost the transfer, resident ones
    # the attention; above it every layer costs the attention
    t_att = 2 * 5 * 0.002                                        # n_cand * bs * unit = 0.02 < 0.05
    assert op.t_target_decoding(pr, 5, 2) == pytest.approx(4 * 0.05 + 2 * t_att + 6 * 0.004)
    t_att = 5 * 9 * 0.002                                        # 0.09 > 0.05
    assert op.t_target_decoding(pr, 9, 5) == pytest.approx(6 * (t_att + 0.004))
    # memory: V_prefill = V_target + bs_prefill * l_input * v_kv; V_decoding = V_ffn + V_draft + bs_draft * (l_in + n_gen) * v
    assert op.v_prefill(pr, 4) == pytest.approx(400 + 4 * 40 * 0.5)
    assert op.v_decoding(pr, 9, 4) == pytest.approx(300 + 100 + 4 * 64 * 1.25)


def test_throughput_definition_and_special_cases():
    pr = _profile()
    pl = op.evaluate(pr, 6, 3, 2, 3)
    e = op.expected_generated(0.6, 3)
    n_iter = math.ceil(24 / e)
    assert pl.n_iter == n_iter and pl.expected_tokens == pytest.approx(e)
    assert pl.throughput == pytest.approx(6 * n_iter * e / (pl.t_prefill + n_iter * max(pl.t_target_decoding, pl.t_draft)))
    # no acceptance: one token per round whatever n_cand, so the planner takes the fewest candidates
    best = op.plan(_profile(p_accept=0.0))
    assert best.n_cand == 1 and best.expected_tokens == 1.0 and best.n_iter == 24
    # memory never binding, cost independent of the batch: throughput grows with bs, planner takes bs_max
    free = _profile(gpu_mem_capacity=1e30, t_attention_unit=0.0, t_draft_prefill=0.0, t_draft_decoding=0.0)
    best = op.plan(free)
    assert best.bs == free.bs_max and best.bs_prefill == free.bs_max and best.bs_draft == free.bs_max
    # capacity below the fixed parts: infeasible
    assert not op.plan(_profile(gpu_mem_capacity=350.0)).feasible


def test_memory_constraints_bind_where_the_formulas_say():
    pr = _profile(gpu_mem_capacity=500.0)      # prefill: 400 + bp*20 <= 500 -> bp <= 5; decoding: 400 + bd*80 <= 500 -> bd <= 1
    best = op.plan(pr)
    assert best.feasible and best.bs_prefill <= 5 and best.bs_draft == 1
    for bs, bp, bd, nc in itertools.product(range(1, 8), range(1, 8), range(1, 8), [1, 3]):
        if bp <= bs and bd <= bs:
            assert op.evaluate(pr, bs, bp, bd, nc).feasible == (bp <= 5 and bd <= 1)


def test_plan_is_the_argmax_over_an_independent_enumeration():
    """The search is checked against a vectorised enumeration written separately from it."""
    pr = _profile()
    best = op.plan(pr)
    grid = [(bs, nc, bp, bd) for bs in range(1, pr.bs_max + 1) for nc in range(1, pr.n_cand_max + 1)
            for bp in range(1, bs + 1) for bd in range(1, bs + 1)]
    g = np.array(grid, dtype=np.float64)
    bs, nc, bp, bd = g.T
    e = (1 - pr.p_accept ** (nc + 1)) / (1 - pr.p_accept)
    n_iter = np.ceil(pr.n_generate / e - 1e-12)
    t_att = nc * bs * pr.t_attention_unit
    tt = pr.n_layer_streamed * np.maximum(t_att, pr.t_ffn_c2g) + (pr.n_layer - pr.n_layer_streamed) * t_att + pr.n_layer * pr.t_ffn_gpu
    td = np.ceil(bs / bd) * (pr.t_draft_prefill + (nc - 1) * pr.t_draft_decoding)
    tp = np.ceil(bs / bp) * (pr.t_c2g_para + pr.t_gpu_prefill_comp)
    ok = (pr.v_target_prefill + bp * pr.l_input * pr.v_target_kv <= pr.gpu_mem_capacity) & \
         (pr.v_target_ffn + pr.v_draft + bd * (pr.l_input + pr.n_generate) * pr.v_draft_kv <= pr.gpu_mem_capacity)
    thr = np.where(ok, bs * n_iter * e / (tp + n_iter * np.maximum(tt, td)), -1.0)
    assert best.throughput == pytest.approx(thr.max(), rel=1e-12)
    assert thr[grid.index((best.bs, best.n_cand, best.bs_prefill, best.bs_draft))] == pytest.approx(thr.max(), rel=1e-12)


# ---- the library against the oracle ----------------------------------------------------------------
def _rand_profile(rng):
    n_layer = int(rng.integers(1, 9))
    return _profile(n_layer=n_layer, n_layer_streamed=int(rng.integers(0, n_layer + 1)), l_input=int(rng.integers(1, 200)),
                    n_generate=int(rng.integers(1, 60)), p_accept=float(rng.choice([0.0, 0.3, 0.62, 0.9, 0.97])),
                    bs_max=int(rng.integers(1, 11)), n_cand_max=int(rng.integers(1, 7)),
                    t_c2g_para=float(rng.uniform(0, 2)), t_gpu_prefill_comp=float(rng.uniform(0, 0.5)),
                    t_ffn_c2g=float(rng.uniform(0, 0.1)), t_ffn_gpu=float(rng.uniform(0, 0.01)),
                    t_attention_unit=float(rng.choice([0.0, 0.001, 0.004])), t_draft_prefill=float(rng.uniform(0, 0.1)),
                    t_draft_decoding=float(rng.uniform(0, 0.05)), gpu_mem_capacity=float(rng.uniform(300, 2000)),
                    v_target_kv=float(rng.uniform(0, 2)), v_draft_kv=float(rng.uniform(0, 3)),
                    t_ffn_gpu_per_token=float(rng.choice([0.0, 1e-4])), t_draft_per_seq=float(rng.choice([0.0, 2e-3])),
                    t_prefill_comp_per_seq=float(rng.choice([0.0, 0.05])), v_target_kv_decoding=float(rng.choice([0.0, 0.4])))


def test_library_planner_matches_oracle_search():
    import paper_2505_10259_amd as P
    rng = np.random.default_rng(7)
    n_feasible = 0
    for _ in range(60):
        pr = _rand_profile(rng)
        want = op.plan(pr)
        got = P.spec_plan_paraspec(op.as_dict(pr))
        assert bool(got["feasible"]) == want.feasible
        if not want.feasible:
            continue
        n_feasible += 1
        # the optimum value is unique; the parameters may differ only between exact ties
        assert got["throughput"] == pytest.approx(want.throughput, rel=1e-12)
        at = op.evaluate(pr, got["bs"], got["bs_prefill"], got["bs_draft"], got["n_cand"])
        assert at.feasible and at.throughput == pytest.approx(want.throughput, rel=1e-12)
        if (got["bs"], got["bs_prefill"], got["bs_draft"], got["n_cand"]) == (want.bs, want.bs_prefill, want.bs_draft, want.n_cand):
            for f in ("n_iter", "expected_tokens", "t_prefill", "t_round", "t_target_decoding", "t_draft", "v_prefill", "v_decoding"):
                assert got[f] == pytest.approx(getattr(want, f), rel=1e-12), f
    assert n_feasible >= 30


def test_library_cost_model_matches_oracle_pointwise():
    import paper_2505_10259_amd as P
    rng = np.random.default_rng(11)
    for _ in range(40):
        pr = _rand_profile(rng)
        bs = int(rng.integers(1, 12)); bp = int(rng.integers(1, bs + 1)); bd = int(rng.integers(1, bs + 1)); nc = int(rng.integers(1, 9))
        want = op.evaluate(pr, bs, bp, bd, nc)
        got = P.spec_plan_evaluate(op.as_dict(pr), bs, bp, bd, nc)
        assert bool(got["feasible"]) == want.feasible and got["n_iter"] == want.n_iter
        for f in ("throughput", "expected_tokens", "t_prefill", "t_round", "t_target_decoding", "t_draft", "v_prefill", "v_decoding"):
            assert got[f] == pytest.approx(getattr(want, f), rel=1e-13), f


def test_library_planner_rejects_bad_arguments():
    import paper_2505_10259_amd as P
    good = op.as_dict(_profile())
    for field, bad in [("p_accept", 1.0), ("p_accept", -0.1), ("n_layer", 0), ("n_layer_streamed", 99), ("bs_max", 0),
                       ("t_ffn_c2g", -1.0), ("gpu_mem_capacity", float("nan")), ("n_generate", 0)]:
        d = dict(good); d[field] = bad
        with pytest.raises(P.SpecError) as ei:
            P.spec_plan_paraspec(d)
        assert ei.value.code == -1
    with pytest.raises(P.SpecError):
        P.spec_plan_evaluate(good, 0, 1, 1, 1)
