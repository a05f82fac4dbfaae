"""GPU parity: the whole draft/verify loop through the C ABI against the CPU oracle, round by
round, on the tiny fp32 workload and on small MoE models (f32 and bf16)."""
import numpy as np
import pytest

import synth
from oracle import model as omodel, spec as ospec

pytestmark = pytest.mark.gpu


def _cdf_boundary(w, u):
    """Relative distance of the inverse-CDF target u * total from the nearest running-sum boundary."""
    c = np.cumsum(np.asarray(w, dtype=np.float64))
    return float(np.abs(c - u * c[-1]).min() / c[-1])


def _compare_run(hm, draft_layers, attn_only, prompts, k, max_new, logit_tol, gap_tol, min_frac,
                 route_tol=5e-3, force_routing=False, mode="greedy", tau=1.0, seed=0, **cfg):
    """Runs oracle and GPU, walks the rounds of each sequence in order and compares candidates, draft and
    target logits, kept count and next token; a sequence is dropped from the comparison (and all its
    later rounds) at the first decision that differs AND is a near-tie in the oracle: a top-2 logit gap
    below gap_tol (greedy), an acceptance margin |u q - p| / p below 1e-4 or an inverse-CDF target within
    1e-5 of a running-sum boundary (sampling).  Any other difference fails.

    Routing.  A flipped expert changes a row by O(1), and only near-ties may flip.  Without
    force_routing a sequence is also dropped at the first pass in which the ORACLE's router saw a
    2nd-vs-3rd logit gap below route_tol; since that depends on the oracle alone, the number of
    sequence-rounds that can be compared at all (`possible`) is known before the GPU runs, and the GPU
    must reach min_frac of it.  With force_routing the GPU takes every row's two experts from the
    oracle's run (spec_debug_force_routing), no sequence is dropped for routing, and min_frac is of all
    sequence-rounds.  Returns (worst logit difference, compared, denominator)."""
    from gpu_common import GpuDecode, top2_gap, forced_prefill_ids, forced_round_ids
    from oracle import philox
    sample = mode == "sample"
    tgt = omodel.build(hm)
    drf = ospec.ModelDraft(omodel.build(hm.draft_view(draft_layers, attn_only)))
    trace = []
    out_o, st_o = ospec.speculative_decode(tgt, drf, prompts, k, max_new, mode=mode, tau=tau, seed=seed, trace=trace)
    by = {(t.seq, t.rnd): t for t in trace}
    B, L = len(prompts), hm.shape.n_layers
    if force_routing:
        Q = cfg.setdefault("prefill_chunk", 8)
        cfg["forced_prefill"] = forced_prefill_ids(st_o["prefill_route_ids"], prompts, L, Q)
    g = GpuDecode(hm, draft_layers, attn_only, prompts, k, max_new, mode=mode, tau=tau, seed=seed, **cfg)
    try:
        route = (lambda r: forced_round_ids({b: by.get((b, r)) for b in range(B)}, B, k, L)) if force_routing else None
        rounds = g.run(route_of_round=route)
        out_g = g.generated()
    finally:
        g.close()
    tol_r = -1.0 if force_routing else route_tol
    alive = [g_ >= tol_r for g_ in st_o["prefill_router_gap"]]
    possible = 0
    ok_route = list(alive)
    for t in sorted(trace, key=lambda t: (t.rnd, t.seq)):       # what the oracle's own router gaps allow
        ok_route[t.seq] = ok_route[t.seq] and t.router_gap >= tol_r
        possible += ok_route[t.seq]
    compared = total = 0
    worst = 0.0
    for r, rd in enumerate(rounds):
        for b in range(B):
            t = by.get((b, r))
            if t is None:
                continue
            total += 1
            if not alive[b]:
                continue
            assert rd["len_before"][b] == t.length_before
            if t.router_gap < tol_r:
                alive[b] = False
                continue
            if sample:
                ud, ua, ur = philox.round_uniforms(seed, r, b, k)
            if not np.array_equal(rd["draft"][b], t.draft_tokens):
                i = int(np.nonzero(rd["draft"][b] != t.draft_tokens)[0][0])
                if sample:
                    near = _cdf_boundary(ospec.softmax_t(t.q_logits[i], tau), ud[i + 1]) < 1e-5
                else:
                    near = top2_gap(t.q_logits[i]) < gap_tol
                assert near, f"draft token differs at seq {b} round {r} pos {i}"
                alive[b] = False
                continue
            if sample:
                dq = float(np.abs(rd["q_logits"][b] - t.q_logits).max())
                assert dq <= logit_tol, f"draft logits differ by {dq} at seq {b} round {r}"
            diff = float(np.abs(rd["p_logits"][b] - t.p_logits).max())
            worst = max(worst, diff)
            assert diff <= logit_tol, f"logits differ by {diff} at seq {b} round {r}"
            if rd["n_acc"][b] != t.n_accepted or rd["next"][b] != t.next_token:
                n = min(int(rd["n_acc"][b]), t.n_accepted)
                if not sample:
                    near = top2_gap(t.p_logits[n]) < gap_tol
                elif rd["n_acc"][b] != t.n_accepted:           # the acceptance test of candidate n+1
                    margins = []
                    ospec.accept_sample(t.p_logits, t.q_logits, t.draft_tokens, ua[1:], ur, tau, margins=margins)
                    near = margins[n] < 1e-4
                else:                                             # same count, other draw
                    p = ospec.softmax_t(t.p_logits[n], tau)
                    w = np.maximum(0.0, p - ospec.softmax_t(t.q_logits[n], tau)) if n < k else p
                    near = _cdf_boundary(w if w.sum() > 0 else p, ur[n]) < 1e-5
                assert near, f"decision differs at seq {b} round {r}: gpu ({rd['n_acc'][b]}, {rd['next'][b]}) " \
                             f"oracle ({t.n_accepted}, {t.next_token})"
                alive[b] = False
                continue
            compared += 1
    denom = total if force_routing else possible
    print(f"compared {compared} of {total} sequence-rounds ({possible} possible given the oracle's router gaps)")
    assert compared >= min_frac * max(1, denom), (compared, possible, total)
    for b in range(B):
        if alive[b]:
            assert out_g[b] == out_o[b]
        assert len(out_g[b]) == max_new
    return worst, compared, denom


def test_cfg1_whole_run_matches_oracle():
    from gpu_common import host_model_pinned
    w = synth.workload("cfg1")
    hm = host_model_pinned(w.target, seed=0, gain_std=0.0)       # the configuration as given: gains 1
    prompts = synth.make_prompts(w.batch, w.prompt_len, w.target.vocab, seed=0)
    worst, compared, total = _compare_run(hm, w.draft_layers, w.draft_attn_only, prompts, w.k, w.max_new,
                                          logit_tol=1e-4, gap_tol=1e-3, min_frac=0.9)
    print(f"cfg1: worst logit diff {worst:.2e}, compared {compared}/{total} sequence-rounds")


@pytest.mark.parametrize("dtype,tol", [("f32", 2e-4), ("bf16", 3e-2)])
@pytest.mark.parametrize("simple", [False, True])
def test_mini_moe_run_matches_oracle(dtype, tol, simple):
    """The library's own routing in the loop.  In bf16 about half of the sequence-rounds are beyond a
    router near-tie of the oracle (2nd-vs-3rd logit gap below the 2e-3 that bf16 noise in the residual
    stream can bridge) and cannot be compared; of those that can, at least half must be compared to the
    end (f32: 90 %): the others stop at a token-level near-tie, which the comparison checks is one."""
    import paper_2505_10259_amd as P
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype=dtype, n_layers=3)
    hm = host_model_pinned(shp, seed=5, std=0.05)
    prompts = synth.make_prompts(6, (3, 40), shp.vocab, seed=9)
    worst, compared, possible = _compare_run(hm, 2, True, prompts, 3, 12, logit_tol=tol, gap_tol=1e-2,
                                             min_frac=0.9 if dtype == "f32" else 0.5,
                                             route_tol=1e-5 if dtype == "f32" else 2e-3,
                                             flags=P.SPEC_FLAG_SIMPLE_KERNELS if simple else 0,
                                             page_tokens=16 if simple else 32)
    print(f"mini moe {dtype} simple={simple}: worst logit diff {worst:.2e}, compared {compared}/{possible}")
    assert possible >= 12


@pytest.mark.parametrize("simple", [False, True])
def test_mini_moe_bf16_run_with_oracle_routing(simple):
    """bf16 whole-loop parity with the routing of every target pass (prefill included) taken from the
    oracle's run: no sequence is lost to a router near-tie, so at least 80 % of ALL sequence-rounds are
    compared.  What still ends a sequence is a token-level near-tie: with bf16 noise of about 1 % of the
    logit scale, each argmax decision (three of the draft, one or two of the target per round) flips
    with a probability of about 2 %, some 10 % per round, whatever the weights; the run is therefore 24
    sequences of four new tokens rather than a few long ones (every exemption is checked to be a
    near-tie of the oracle's logits)."""
    import paper_2505_10259_amd as P
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=3)
    hm = host_model_pinned(shp, seed=5, std=0.05)
    prompts = synth.make_prompts(24, (3, 70), shp.vocab, seed=9)
    worst, compared, total = _compare_run(hm, 2, True, prompts, 3, 4, logit_tol=3e-2, gap_tol=1e-2,
                                          min_frac=0.8, force_routing=True,
                                          flags=P.SPEC_FLAG_SIMPLE_KERNELS if simple else 0,
                                          page_tokens=16 if simple else 32)
    print(f"mini moe bf16, oracle routing, simple={simple}: worst logit diff {worst:.2e}, compared {compared}/{total}")
    assert total >= 70


@pytest.mark.parametrize("draft_layers,attn_only,k,page_tokens", [
    (1, False, 1, 32),       # the draft keeps its layer's experts; one candidate per round
    (2, True, 8, 64),        # nine verify tokens per sequence, 64-token pages (the library's default)
    (3, True, 16, 32),       # the largest k: 17 verify tokens, 34 query rows per KV head (a draft with experts of
                             # its own is left to the first case: its routing is not forced, and at 16 draft steps
                             # per round some bf16 router near-tie of the draft always ends the comparison)
])
def test_mini_moe_bf16_draft_and_k_variants(draft_layers, attn_only, k, page_tokens):
    """bf16 whole-loop parity (routing from the oracle) over the corners of the draft and round shapes.  Runs
    of three new tokens (about three rounds): with k argmax decisions of the draft per round, each a near-tie with a probability
    of about 2 % under bf16 noise, long runs at large k lose most sequences to (verified) near-ties."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=3)
    hm = host_model_pinned(shp, seed=21, std=0.05)
    prompts = synth.make_prompts(10, (3, 90), shp.vocab, seed=22)
    worst, compared, total = _compare_run(hm, draft_layers, attn_only, prompts, k, 3, logit_tol=3e-2,
                                          gap_tol=1e-2, min_frac=0.5, force_routing=True, page_tokens=page_tokens)
    print(f"bf16 draft {draft_layers} layers attn_only={attn_only} k={k} pages of {page_tokens}: worst logit diff "
          f"{worst:.2e}, compared {compared}/{total}")
    assert total >= 10


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_prompts_at_the_edges_of_the_prefill_chunks(dtype):
    """Prompts of 1 and 2 tokens (nothing, or one position, to prefill), of exactly one chunk of 64 positions
    plus the token the first verify feeds (65), one more (66), and two chunks (129), in one batch."""
    from gpu_common import host_model_pinned
    f32 = dtype == "f32"
    shp = synth.mini_moe_shape(dtype=dtype, n_layers=2)
    hm = host_model_pinned(shp, seed=16, std=0.05)
    rng = np.random.default_rng(17)
    prompts = [rng.integers(0, shp.vocab, n).astype(np.int32) for n in (1, 66, 2, 129, 65, 1, 64, 33)]
    worst, compared, possible = _compare_run(hm, 1, True, prompts, 3, 5, logit_tol=2e-4 if f32 else 3e-2,
                                             gap_tol=1e-4 if f32 else 1e-2, min_frac=0.9 if f32 else 0.6,
                                             route_tol=1e-5, force_routing=not f32, page_tokens=0 if f32 else 32,
                                             **({} if f32 else {"prefill_chunk": 64}))
    print(f"edge prompts ({dtype}): worst logit diff {worst:.2e}, compared {compared}/{possible}")
    assert possible >= 12


@pytest.mark.parametrize("simple", [False, True])
def test_dense_ffn_bf16_run_matches_oracle(simple):
    """A bf16 target whose layers have one dense SwiGLU feed-forward block instead of experts (the
    ungrouped SwiGLU product of the MFMA kernel, or the plain kernels): whole run against the oracle."""
    import paper_2505_10259_amd as P
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=3, n_experts=0)
    hm = host_model_pinned(shp, seed=14, std=0.05)
    prompts = synth.make_prompts(16, (3, 70), shp.vocab, seed=15)
    worst, compared, possible = _compare_run(hm, 2, True, prompts, 3, 4, logit_tol=3e-2, gap_tol=1e-2, min_frac=0.75,
                                             flags=P.SPEC_FLAG_SIMPLE_KERNELS if simple else 0,
                                             page_tokens=16 if simple else 32)
    print(f"dense bf16 simple={simple}: worst logit diff {worst:.2e}, compared {compared}/{possible}")
    assert possible >= 40


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_context_larger_than_the_batch_it_serves(dtype):
    """A context made for 9 sequences and k up to 6 that serves 5 sequences with k = 3 (the static page map
    and the candidate buffers are laid out for the maxima): whole run against the oracle; f32 with the
    model's own routing, bf16 (MFMA kernels) with the oracle's."""
    from gpu_common import host_model_pinned
    f32 = dtype == "f32"
    shp = synth.mini_moe_shape(dtype=dtype, n_layers=2)
    hm = host_model_pinned(shp, seed=8, std=0.05)
    prompts = synth.make_prompts(5, (3, 40), shp.vocab, seed=12)
    worst, compared, possible = _compare_run(hm, 1, True, prompts, 3, 6, logit_tol=2e-4 if f32 else 3e-2,
                                             gap_tol=1e-4 if f32 else 1e-2, min_frac=0.9 if f32 else 0.6,
                                             route_tol=1e-5, force_routing=not f32, batch_max=9, k_max=6,
                                             page_tokens=0 if f32 else 32)
    print(f"batch_max 9 / k_max 6 serving 5 sequences with k 3 ({dtype}): worst logit diff {worst:.2e}, compared {compared}/{possible}")
    assert possible >= 8


@pytest.mark.parametrize("chunk", [16, 64])
def test_prefill_chunk_sizes_match_oracle(chunk):
    """The logits that follow a prefill in chunks of 16 and of 64 prompt positions (64: the MFMA attention
    kernel takes a chunk's query rows in two blocks of 64, each over the keys it may see) against the
    oracle, which knows no chunks: prompts of 70-150 tokens (several chunks, the last one ragged), routing
    taken from the oracle so that every sequence is compared."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=3)
    hm = host_model_pinned(shp, seed=6, std=0.05)
    prompts = synth.make_prompts(12, (70, 150), shp.vocab, seed=10)
    worst, compared, total = _compare_run(hm, 2, True, prompts, 3, 3, logit_tol=3e-2, gap_tol=1e-2,
                                          min_frac=0.75, force_routing=True, page_tokens=32, prefill_chunk=chunk)
    print(f"prefill in chunks of {chunk}: worst logit diff {worst:.2e}, compared {compared}/{total}")
    assert total >= 12


@pytest.mark.parametrize("k", [3, 5])
def test_sampling_loop_matches_oracle_token_for_token(k):
    """Sampling mode, whole loop, f32 model with a vocabulary of 8192 (two register sweeps of the
    token-pick and accept kernels), device Philox: candidates, draft and target logits, kept counts and
    drawn tokens equal the oracle's trace round by round (same seed, same stream layout)."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="f32", n_layers=2, vocab=8192, head_dim=64)
    hm = host_model_pinned(shp, seed=13, std=0.1)
    prompts = synth.make_prompts(6, (3, 20), shp.vocab, seed=2)
    worst, compared, possible = _compare_run(hm, 1, True, prompts, k, 10, logit_tol=3e-4, gap_tol=0.0,
                                             min_frac=0.9, route_tol=1e-5, mode="sample", tau=0.8, seed=4242)
    print(f"sampling loop k={k}: worst logit diff {worst:.2e}, compared {compared}/{possible}")
    assert possible >= 10


def test_greedy_equals_plain_on_gpu_any_draft():
    """Invariant on the GPU itself: candidates supplied by the caller (random ids) still give the
    plain greedy decode (k = 0 rounds) of the same library."""
    from gpu_common import GpuDecode, host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16")
    hm = host_model_pinned(shp, seed=2, std=0.05)
    prompts = synth.make_prompts(4, (5, 40), shp.vocab, seed=1)
    plain = GpuDecode(hm, 0, True, prompts, 0, 10)
    plain.run(want_logits=False)
    ref = plain.generated()
    plain.close()
    rng = np.random.default_rng(0)
    g = GpuDecode(hm, 0, True, prompts, 4, 10)
    for _ in range(10):
        g.round(forced_draft=rng.integers(0, shp.vocab, (4, 4)), want_logits=False)
    got = g.generated()
    g.close()
    # feed the plain continuation as candidates: every round keeps all four
    g2 = GpuDecode(hm, 0, True, prompts, 4, 10)
    import paper_2505_10259_amd as P
    for r in range(2):
        lens = P.spec_get_lengths(g2.s.ctx, 0, 4)
        cand = np.array([ref[b][lens[b] - len(prompts[b]):][:4] for b in range(4)])
        rd = g2.round(forced_draft=cand, want_logits=False)
        assert (rd["n_acc"] == 4).all()
    got2 = g2.generated()
    g2.close()
    assert got == ref and got2 == ref


def test_step_with_no_candidates_is_plain_decoding():
    """spec_step(k = 0) on two sub-batches (the no-speculation baseline of the schedule) gives the
    same tokens as verify-only rounds on one batch, and as the oracle's plain greedy decode where the
    oracle's decisions are not near ties."""
    import paper_2505_10259_amd as P
    from gpu_common import GpuDecode, host_model_pinned
    shp = synth.mini_moe_shape(dtype="f32")
    hm = host_model_pinned(shp, seed=3, std=0.05)
    prompts = synth.make_prompts(6, (5, 30), shp.vocab, seed=4)
    max_new = 8
    plain = GpuDecode(hm, 0, True, prompts, 0, max_new)
    plain.run(want_logits=False)
    ref = plain.generated()
    plain.close()
    s = P.Session(hm, hm.draft_view(1, True), n_sub_batches=2, batch_max=3, k_max=2,
                  ctx_max=max(len(p) for p in prompts) + max_new)
    try:
        for sb in range(2):
            P.spec_prefill(s.ctx, sb, prompts[sb * 3:(sb + 1) * 3], max_new)
        for _ in range(2 * max_new):
            P.spec_step(s.ctx, 0)
        P.spec_sync(s.ctx)
        got = [P.spec_get_tokens(s.ctx, b // 3, b % 3, 64)[len(prompts[b]):].tolist() for b in range(6)]
        st = P.spec_get_stats(s.ctx)
    finally:
        s.close()
    assert got == ref
    assert st["committed_tokens"] == 6 * max_new and st["accept_hist"][0] == 6 * max_new
    out_o = ospec.plain_decode(omodel.build(hm), prompts, max_new)
    same = sum(got[b] == list(out_o[b]) for b in range(6))
    print(f"plain decoding through spec_step(k=0): {same}/6 sequences equal to the oracle's")
    assert same >= 4
