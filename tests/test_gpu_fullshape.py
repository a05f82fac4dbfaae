"""GPU tests at the per-layer shapes of the streamed Mixtral-8x7B configuration (d 4096, 32/8 heads x
128, 8 experts of 14336, vocabulary 32000) with few layers: oracle parity of the whole draft/verify
loop, the streamer and the greedy invariant in the benchmark's launch configuration, and the
distribution of the sampling path end to end."""
import numpy as np
import pytest

import synth
from oracle import model as omodel, spec as ospec

pytestmark = pytest.mark.gpu


def _shape(n_layers):
    from dataclasses import replace
    return replace(synth.workload("cfg3").target, n_layers=n_layers)


def test_8x7b_shape_two_layers_matches_oracle():
    from gpu_common import GpuDecode, host_model_pinned, top2_gap
    shp = _shape(2)
    hm = host_model_pinned(shp, seed=0)
    prompts = synth.make_prompts(2, (20, 24), shp.vocab, seed=5)
    k, max_new = 4, 3
    tgt = omodel.build(hm)
    drf = ospec.ModelDraft(omodel.build(hm.draft_view(1, True)))
    trace = []
    out_o, st_o = ospec.speculative_decode(tgt, drf, prompts, k, max_new, trace=trace)
    by = {(t.seq, t.rnd): t for t in trace}
    g = GpuDecode(hm, 1, True, prompts, k, max_new)
    rounds = g.run()
    out_g = g.generated()
    g.close()
    alive = [gp >= 1e-3 for gp in st_o["prefill_router_gap"]]
    worst, compared = 0.0, 0
    for r, rd in enumerate(rounds):
        for b in range(2):
            t = by.get((b, r))
            if t is None or not alive[b]:
                continue
            if t.router_gap < 1e-3 or not np.array_equal(rd["draft"][b], t.draft_tokens):
                alive[b] = False
                continue
            delta = rd["p_logits"][b] - t.p_logits
            diff = float(np.abs(delta).max())
            worst = max(worst, diff)
            # Two independent bf16 evaluations of a d=4096 model (different accumulation order, so
            # activations near a rounding boundary round differently) differ by about 0.8 % of the
            # logit scale (std 1.28) per logit: rms 1e-2, and 5.5 sigma over 160 000 logits is 5.5e-2.
            # The 3e-2 max-abs bound that holds for the small models is therefore checked here as
            # rms <= 2e-2 and max-abs <= 1e-1 (measured: 9.9e-3 and 5.5e-2).
            assert float(np.sqrt((delta ** 2).mean())) <= 2e-2 and diff <= 1e-1, \
                f"logits differ by {diff} (seq {b}, round {r})"
            if rd["n_acc"][b] != t.n_accepted or rd["next"][b] != t.next_token:
                assert top2_gap(t.p_logits[min(int(rd["n_acc"][b]), t.n_accepted)]) < 1e-2
                alive[b] = False
                continue
            compared += 1
    print(f"8x7B-shaped 2 layers: worst logit diff {worst:.3e} over {compared} sequence-rounds")
    assert compared >= 1
    for b in range(2):
        if alive[b]:
            assert out_g[b] == out_o[b]


def test_8x7b_shape_streamed_equals_resident_and_greedy_invariant():
    import paper_2505_10259_amd as P
    from gpu_common import GpuDecode, host_model_pinned
    shp = _shape(4)
    hm = host_model_pinned(shp, seed=1)
    prompts = synth.make_prompts(8, (40, 48), shp.vocab, seed=6)
    k, max_new = 4, 6
    blob = P.spec_layer_blob_elems(shp) * 2
    draft = shp.draft(2, True)
    fixed = P.spec_global_blob_elems(shp) * 2 + 2 * P.spec_layer_blob_elems(draft) * 2
    res = GpuDecode(hm, 2, True, prompts, k, max_new)
    r_res = res.run()
    out_res = res.generated()
    res.close()
    stm = GpuDecode(hm, 2, True, prompts, k, max_new, hbm_weight_budget_bytes=fixed + 2 * blob + blob // 2)
    r_stm = stm.run()
    out_stm = stm.generated()
    st = P.spec_get_stats(stm.s.ctx)
    stm.close()
    # three staging slots of one expert (3/8 of a layer): two layers and the front piece of a third stay
    assert st["resident_layers"] == 2 and 0 < st["pinned_piece_bytes"] < blob // 8
    assert st["bytes_streamed"] >= (1 + len(r_stm)) * (2 * blob - st["pinned_piece_bytes"])
    assert out_stm == out_res
    for a, b in zip(r_stm, r_res):
        assert np.array_equal(a["p_logits"], b["p_logits"])
    plain = GpuDecode(hm, 0, True, prompts, 0, max_new)
    plain.run(want_logits=False)
    out_plain = plain.generated()
    plain.close()
    assert out_res == out_plain, "speculative greedy differs from plain greedy decoding on the GPU"


def test_sampling_end_to_end_distribution_on_gpu():
    """Toy model with a 16-token vocabulary, 256 sequences with the same prompt, device Philox: the
    first emitted token must follow the target's next-token distribution computed by the oracle."""
    from scipy import stats
    import paper_2505_10259_amd as P
    from gpu_common import host_model_pinned
    shp = synth.ModelShape(n_layers=2, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ff=64, vocab=16,
                           n_experts=4, dtype="f32")
    hm = host_model_pinned(shp, seed=21, std=0.6)
    prompt = np.array([3, 7, 1, 12], dtype=np.int32)
    tau = 0.8
    p = ospec.softmax_t(omodel.build(hm).forward_full(prompt)[-1], tau)
    B, obs, n_hist = 256, np.zeros(16), np.zeros(3)
    for seed in range(12):
        s = P.Session(hm, hm.draft_view(1, True), batch_max=B, k_max=2, ctx_max=8, mode=P.SPEC_SAMPLE,
                      temperature=tau, seed=1000 + seed)
        try:
            P.spec_prefill(s.ctx, 0, [prompt] * B, 1)
            P.spec_step(s.ctx, 2)
            P.spec_sync(s.ctx)
            for b in range(B):
                obs[P.spec_get_tokens(s.ctx, 0, b, 8)[4]] += 1
            n_hist += np.array(P.spec_get_stats(s.ctx)["accept_hist"][:3])
        finally:
            s.close()
    chi2, pval = stats.chisquare(obs, p * obs.sum())
    print(f"first-token chi-square p-value {pval:.3f}; kept-count histogram {n_hist.tolist()}")
    assert pval > 0.01, (chi2, pval)
    assert n_hist.sum() == obs.sum() and n_hist[1:].sum() > 0      # some candidates are kept
