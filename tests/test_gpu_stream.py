"""GPU tests of the host->HBM layer streamer: a run whose layers stream through the staging ring
must equal, bit for bit, the run with every layer resident, for any budget / ring size and also with
copies and compute serialised; plus budget and capacity errors and the interleaved two-sub-batch
schedule against sequential processing of the same sequences."""
import numpy as np
import pytest

import synth

pytestmark = pytest.mark.gpu


def _setup(n_layers=6, dtype="bf16"):
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype=dtype, n_layers=n_layers)
    hm = host_model_pinned(shp, seed=7, std=0.05)
    prompts = synth.make_prompts(6, (4, 50), shp.vocab, seed=3)
    return shp, hm, prompts


def _ring_bytes(shp, slots, piece_slots=3):
    """slots >= 1: whole-layer slots.  slots = 0: piece staging, piece_slots slots of the largest piece
    (an expert, or the weights in front of the experts)."""
    import paper_2505_10259_amd as P
    blob_elems = P.spec_layer_blob_elems(shp)
    if slots:
        return slots * blob_elems * shp.elem_bytes
    al = lambda n: (n + 127) // 128 * 128
    expert = 3 * al(shp.d_model * shp.d_ff)
    front = blob_elems - shp.n_experts * expert
    return piece_slots * ((max(expert, front) * shp.elem_bytes + 255) // 256 * 256)


def _budget(shp, draft, resident, slots, piece_slots=3):
    """Room for `resident` whole layers, the ring and half a layer more (which piece staging fills
    with pinned pieces of the next layer)."""
    import paper_2505_10259_amd as P
    blob = P.spec_layer_blob_elems(shp) * shp.elem_bytes
    fixed = P.spec_global_blob_elems(shp) * shp.elem_bytes + draft.n_layers * P.spec_layer_blob_elems(draft) * draft.elem_bytes
    return fixed + resident * blob + _ring_bytes(shp, slots, piece_slots) + blob // 2


def _run(hm, prompts, k, max_new, **cfg):
    import paper_2505_10259_amd as P
    from gpu_common import GpuDecode
    g = GpuDecode(hm, 2, True, prompts, k, max_new, **cfg)
    rounds = g.run()
    out = g.generated()
    st = P.spec_get_stats(g.s.ctx)
    g.close()
    return rounds, out, st


@pytest.mark.parametrize("resident,slots,flags,piece_slots", [
    (2, 2, 0, 0), (0, 2, 0, 0), (3, 1, 0, 0), (1, 3, 0, 0), (2, 2, 1, 0),         # whole-layer slots
    (2, 0, 0, 0), (0, 0, 0, 0), (4, 0, 0, 0), (3, 0, 1, 0), (1, 0, 0, 2), (2, 0, 0, 7), (0, 0, 1, 2)])
def test_streamed_equals_resident_bit_exact(resident, slots, flags, piece_slots):
    import paper_2505_10259_amd as P
    shp, hm, prompts = _setup()
    draft = shp.draft(2, True)
    ref_rounds, ref_out, ref_st = _run(hm, prompts, 3, 10)
    assert ref_st["bytes_streamed"] == 0 and ref_st["resident_layers"] == shp.n_layers
    budget = _budget(shp, draft, resident, slots, piece_slots or 3)
    rounds, out, st = _run(hm, prompts, 3, 10, hbm_weight_budget_bytes=budget, n_ring_slots=slots, flags=flags,
                           n_piece_slots=piece_slots)
    assert st["resident_layers"] == resident
    n_pass = 1 + len(rounds)                              # prefill + one pass per round
    blob = shp.layer_layout()[1] * shp.elem_bytes
    if slots:
        per_pass = (shp.n_layers - resident) * blob
        assert st["pinned_piece_bytes"] == 0
    else:                                                 # half a layer of pieces is pinned besides
        per_pass = (shp.n_layers - resident) * blob - st["pinned_piece_bytes"]
        assert 0.25 * blob < st["pinned_piece_bytes"] <= 0.5 * blob
        if piece_slots == 0:
            assert P.spec_plan_residency(shp, draft, budget, 0) == (resident, per_pass)
    assert st["hbm_weight_bytes"] <= budget
    assert st["bytes_streamed"] >= n_pass * per_pass                               # + run-ahead copies
    assert st["bytes_streamed"] <= n_pass * per_pass + max(_ring_bytes(shp, slots, piece_slots or 3), 2 * blob)
    assert out == ref_out
    for a, b in zip(rounds, ref_rounds):
        assert np.array_equal(a["p_logits"], b["p_logits"])       # bit exact
        assert np.array_equal(a["n_acc"], b["n_acc"]) and np.array_equal(a["next"], b["next"])


def test_piece_staging_f32_plain_kernels():
    """The piece-by-piece path with the plain kernels (f32 model): same tokens and logits as with every
    layer resident."""
    shp, hm, prompts = _setup(n_layers=4, dtype="f32")
    draft = shp.draft(2, True)
    ref_rounds, ref_out, _ = _run(hm, prompts, 2, 6)
    rounds, out, st = _run(hm, prompts, 2, 6, hbm_weight_budget_bytes=_budget(shp, draft, 1, 0), n_ring_slots=0)
    assert st["resident_layers"] == 1 and st["pinned_piece_bytes"] > 0 and st["bytes_streamed"] > 0
    assert out == ref_out
    for a, b in zip(rounds, ref_rounds):
        assert np.array_equal(a["p_logits"], b["p_logits"])


def test_prefill_chunk_groups():
    """Prompts long enough that the prefill's feed-forward part runs on several groups of chunks, the
    last one partial (64 sequences x 32 positions per chunk: four chunks per group, ten chunks).  A
    row's arithmetic does not depend on how the prompt is chunked or grouped, so the first round's
    logits equal, bit for bit, those of a run with 16 positions per chunk (eight chunks per group) and
    those of a run with 64 positions per chunk (the attention kernel then takes a chunk's query rows
    in two blocks of 64) and those of the same chunking under piece staging."""
    from gpu_common import GpuDecode, host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=3)
    hm = host_model_pinned(shp, seed=13, std=0.05)
    prompts = synth.make_prompts(64, (200, 300), shp.vocab, seed=8)
    draft = shp.draft(2, True)

    def first_round(**cfg):
        g = GpuDecode(hm, 2, True, prompts, 2, 3, **cfg)
        try:
            r = g.round()
            return r["p_logits"], r["next"]
        finally:
            g.close()

    a_logits, a_next = first_round(prefill_chunk=32)
    b_logits, b_next = first_round(prefill_chunk=16)
    # (row 0 of a sequence's logits depends on its prompt only; the other rows follow the drafted tokens)
    assert np.array_equal(a_logits[:, 0], b_logits[:, 0])
    d_logits, d_next = first_round(prefill_chunk=64)
    assert np.array_equal(a_logits[:, 0], d_logits[:, 0])
    c_logits, c_next = first_round(prefill_chunk=32, hbm_weight_budget_bytes=_budget(shp, draft, 1, 0), n_ring_slots=0)
    assert np.array_equal(a_logits, c_logits) and np.array_equal(a_next, c_next)


def test_piece_staging_with_uneven_expert_loads():
    """Per-expert launches of a streamed layer with expert loads far from what the launcher expects (one
    expert takes half of the first choices, all of them in layer 0; one has no rows): the experts of every
    verify pass are forced row by row; logits of the streamed run equal those of the resident run bit for
    bit.  (That the values are right is the layer tests' business.)"""
    from gpu_common import GpuDecode
    shp, hm, _ = _setup()
    prompts = synth.make_prompts(52, (4, 30), shp.vocab, seed=3)
    draft = shp.draft(2, True)
    k, B, L = 3, len(prompts), shp.n_layers
    rng = np.random.default_rng(3)
    T = B * (k + 1)                              # 208 rows: 26 per expert expected
    ids = np.zeros((L, T, 2), dtype=np.int32)
    ids[..., 0] = np.where(rng.random((L, T)) < 0.5, 0, rng.integers(1, 7, (L, T)))
    ids[0, :, 0] = 0                             # layer 0: every row on expert 0 (a tile of 208 rows)
    ids[..., 1] = 1 + (ids[..., 0] + rng.integers(0, 5, (L, T))) % 6
    ids[..., 1] = np.where(ids[..., 1] == ids[..., 0], 1 + ids[..., 0] % 6, ids[..., 1])
    assert (ids[..., 0] != ids[..., 1]).all() and ids.max() <= 6

    def two_rounds(**cfg):
        g = GpuDecode(hm, 2, True, prompts, k, 10, **cfg)
        try:
            return [g.round(forced_route=ids)["p_logits"] for _ in range(2)]
        finally:
            g.close()

    ref = two_rounds()
    got = two_rounds(hbm_weight_budget_bytes=_budget(shp, draft, 1, 0), n_ring_slots=0)
    for a_, b_ in zip(ref, got):
        assert np.isfinite(a_).all() and np.array_equal(a_, b_)


def test_piece_staging_dense_ffn_model():
    """A target without experts (dense SwiGLU feed-forward): its layers stream as two pieces (attention
    part, feed-forward part); tokens and logits equal those of the resident run."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=5, n_experts=0)
    hm = host_model_pinned(shp, seed=11, std=0.05)
    prompts = synth.make_prompts(5, (4, 40), shp.vocab, seed=5)
    draft = shp.draft(2, True)
    ref_rounds, ref_out, _ = _run(hm, prompts, 3, 8)
    import paper_2505_10259_amd as P
    blob = P.spec_layer_blob_elems(shp) * shp.elem_bytes
    fixed = P.spec_global_blob_elems(shp) * shp.elem_bytes + draft.n_layers * P.spec_layer_blob_elems(draft) * draft.elem_bytes
    # room for one whole layer, three slots of the larger piece (at most a layer each) and half a layer
    rounds, out, st = _run(hm, prompts, 3, 8, hbm_weight_budget_bytes=fixed + 4 * blob + blob // 2, n_ring_slots=0)
    assert 1 <= st["resident_layers"] < shp.n_layers and st["bytes_streamed"] > 0
    assert out == ref_out
    for a, b in zip(rounds, ref_rounds):
        assert np.array_equal(a["p_logits"], b["p_logits"])


def test_budget_and_capacity_errors():
    import paper_2505_10259_amd as P
    shp, hm, prompts = _setup(n_layers=3)
    draft = shp.draft(2, True)
    dm = hm.draft_view(2, True)
    with pytest.raises(P.binding.SpecError) as e:
        # room for the fixed part and two staging slots; the default ring has three
        P.Session(hm, dm, batch_max=4, k_max=3, ctx_max=64,
                  hbm_weight_budget_bytes=_budget(shp, draft, 0, 0, piece_slots=2)
                  - P.spec_layer_blob_elems(shp) * shp.elem_bytes // 2)
    assert e.value.code == P.SPEC_ERR_BUDGET
    for bad in (dict(n_piece_slots=1), dict(n_piece_slots=17), dict(n_ring_slots=9), dict(n_ring_slots=-1)):
        with pytest.raises(P.binding.SpecError) as e:
            P.Session(hm, dm, batch_max=4, k_max=3, ctx_max=64, **bad)
        assert e.value.code == P.SPEC_ERR_ARG
    s = P.Session(hm, dm, batch_max=4, k_max=3, ctx_max=64)
    try:
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_prefill(s.ctx, 0, prompts, 10)            # 6 prompts > batch_max 4
        assert e.value.code == P.SPEC_ERR_CAPACITY
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_prefill(s.ctx, 0, prompts[:2], 100)       # prompt + max_new > ctx_max
        assert e.value.code == P.SPEC_ERR_CAPACITY
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_draft(s.ctx, 0, 2)                        # before prefill
        assert e.value.code == P.SPEC_ERR_STATE
        P.spec_prefill(s.ctx, 0, prompts[:3], 8)
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_draft(s.ctx, 0, 9)                        # k > k_max
        assert e.value.code == P.SPEC_ERR_CAPACITY
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_verify(s.ctx, 0, None, 3)                 # no candidates drafted
        assert e.value.code == P.SPEC_ERR_STATE
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_prefill(s.ctx, 1, prompts[:2], 8)         # sub-batch 1 of a 1-sub-batch context
        assert e.value.code == P.SPEC_ERR_ARG
    finally:
        s.close()


@pytest.mark.parametrize("mode", ["greedy", "sample"])
def test_interleaved_sub_batches_equal_sequential(mode):
    """Two sub-batches through spec_step (draft of one overlapping verify of the other, streamed
    weights) give the tokens each sub-batch gets when it is run alone."""
    import paper_2505_10259_amd as P
    shp, hm, prompts = _setup()
    draft = shp.draft(2, True)
    dm = hm.draft_view(2, True)
    k, max_new = 3, 9
    md = P.SPEC_SAMPLE if mode == "sample" else P.SPEC_GREEDY
    budget = _budget(shp, draft, 2, 2)
    ctx_max = max(len(p) for p in prompts) + max_new

    def run(n_sub, groups):
        s = P.Session(hm, dm, hbm_weight_budget_bytes=budget, n_sub_batches=n_sub, batch_max=3, k_max=k,
                      ctx_max=ctx_max, mode=md, temperature=0.8, seed=42)
        outs = []
        try:
            for sb, grp in enumerate(groups):
                P.spec_prefill(s.ctx, sb, grp, max_new)
            for _ in range(max_new * n_sub + 2):
                P.spec_step(s.ctx, k)
            P.spec_sync(s.ctx)
            for sb, grp in enumerate(groups):
                outs.append([P.spec_get_tokens(s.ctx, sb, b, len(p) + max_new + 1)[len(p):].tolist()
                             for b, p in enumerate(grp)])
        finally:
            s.close()
        return outs

    both = run(2, [prompts[:3], prompts[3:]])
    first = run(1, [prompts[:3]])
    assert both[0] == first[0]
    assert all(len(t) == max_new for grp in both for t in grp)
    if mode == "greedy":
        # sub-batch 1 alone: same tokens (its Philox sequence ids differ when run as sub-batch 0, so
        # only the greedy mode is comparable)
        second = run(1, [prompts[3:]])
        assert both[1] == second[0]


def test_released_slots_poisoned_and_copy_stream_delayed():
    """Two checks of the streamer's event protocol.  (1) With SPEC_FLAG_POISON_RELEASED every staging
    slot is overwritten with NaN patterns the moment its piece is released: a kernel that read a slot
    after its release, or a copy that landed before the release, would show as NaNs or changed bits.
    (2) The caller-supplied copy stream is held up by a long spin kernel before every round, so the
    copies on it start late and complete after the copies queued behind them on the library's second
    copy stream: compute must wait for each piece's own event, whatever order the copies finish in.
    Tokens and logits must equal the all-resident run bit for bit in both."""
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import GpuDecode
    shp, hm, prompts = _setup()
    draft = shp.draft(2, True)
    ref_rounds, ref_out, _ = _run(hm, prompts, 3, 10)
    for slots, piece_slots in ((0, 0), (2, 0), (0, 2)):
        budget = _budget(shp, draft, 1, slots, piece_slots or 3)
        rounds, out, st = _run(hm, prompts, 3, 10, hbm_weight_budget_bytes=budget, n_ring_slots=slots,
                               n_piece_slots=piece_slots, flags=P.SPEC_FLAG_POISON_RELEASED)
        assert st["bytes_streamed"] > 0 and out == ref_out
        for a, b in zip(rounds, ref_rounds):
            assert np.isfinite(a["p_logits"]).all() and np.array_equal(a["p_logits"], b["p_logits"])
    side = torch.cuda.Stream()
    g = GpuDecode(hm, 2, True, prompts, 3, 10, hbm_weight_budget_bytes=_budget(shp, draft, 1, 0),
                  copy_stream=side.cuda_stream, flags=P.SPEC_FLAG_POISON_RELEASED)
    try:
        rounds = []
        for _ in range(len(ref_rounds)):
            with torch.cuda.stream(side):
                torch.cuda._sleep(200_000_000)            # roughly 0.1 s of spinning in front of the next copies
                                                          # (a kernel that only reads the clock: it always ends)
            rounds.append(g.round())
        out = g.generated()
    finally:
        g.close()
    assert out == ref_out
    for a, b in zip(rounds, ref_rounds):
        assert np.array_equal(a["p_logits"], b["p_logits"])


def test_attention_resident_placement_streams_only_experts():
    """SPEC_FLAG_PIN_ATTENTION (the decoding-phase placement of Section 4.1.2: attention parameters
    resident, only expert parameters cross the link): same tokens and logits as the all-resident run, and
    the bytes per pass are expert bytes only."""
    import paper_2505_10259_amd as P
    shp, hm, prompts = _setup()
    draft = shp.draft(2, True)
    ref_rounds, ref_out, _ = _run(hm, prompts, 3, 10)
    blob = shp.layer_layout()[1] * shp.elem_bytes
    al = lambda n: (n + 127) // 128 * 128
    expert = 3 * al(shp.d_model * shp.d_ff) * shp.elem_bytes
    front = blob - shp.n_experts * expert
    budget = _budget(shp, draft, 2, 0)                    # default placement: two layers + half a layer
    plan = P.spec_plan_placement(shp, draft, hbm_weight_budget_bytes=budget, flags=P.SPEC_FLAG_PIN_ATTENTION)
    rounds, out, st = _run(hm, prompts, 3, 10, hbm_weight_budget_bytes=budget, flags=P.SPEC_FLAG_PIN_ATTENTION)
    R = st["resident_layers"]
    assert R == plan["resident_layers"] and st["pinned_piece_bytes"] == plan["pinned_piece_bytes"]
    streamed_layers = shp.n_layers - R
    assert st["pinned_piece_bytes"] >= streamed_layers * front                 # every attention part is in HBM
    per_pass = plan["streamed_bytes_per_pass"]
    assert per_pass % expert == 0 and per_pass == streamed_layers * blob - st["pinned_piece_bytes"]
    assert st["hbm_weight_bytes"] <= budget
    n_pass = 1 + len(rounds)
    assert n_pass * per_pass <= st["bytes_streamed"] <= n_pass * per_pass + 3 * expert
    assert out == ref_out
    for a, b in zip(rounds, ref_rounds):
        assert np.array_equal(a["p_logits"], b["p_logits"])
    # a budget that cannot hold every attention part is refused
    fixed = P.spec_global_blob_elems(shp) * shp.elem_bytes + draft.n_layers * P.spec_layer_blob_elems(draft) * draft.elem_bytes
    with pytest.raises(P.binding.SpecError) as e:
        P.Session(hm, hm.draft_view(2, True), batch_max=4, k_max=3, ctx_max=64, flags=P.SPEC_FLAG_PIN_ATTENTION,
                  hbm_weight_budget_bytes=fixed + 3 * expert + (shp.n_layers - 1) * front)
    assert e.value.code == P.SPEC_ERR_BUDGET


def test_second_prefill_restarts_the_rotation_and_failed_pass_marks_context():
    """spec_prefill of new sequences resets the interleaved schedule (spec_step drafts for its first
    sub-batch again); forced-routing rows that do not cover a pass are an error of that pass, which
    leaves a streaming context marked unusable instead of out of step."""
    import torch
    import paper_2505_10259_amd as P
    shp, hm, prompts = _setup(n_layers=3)
    dm = hm.draft_view(2, True)
    s = P.Session(hm, dm, n_sub_batches=2, batch_max=3, k_max=2, ctx_max=80)
    try:
        for rep in range(2):
            for sb in range(2):
                P.spec_prefill(s.ctx, sb, prompts[sb * 3:(sb + 1) * 3], 4)
            for _ in range(3):
                P.spec_step(s.ctx, 2)                     # second time round this failed with SPEC_ERR_STATE
            P.spec_sync(s.ctx)
    finally:
        s.close()
    draft = shp.draft(2, True)
    s = P.Session(hm, dm, batch_max=3, k_max=2, ctx_max=80, hbm_weight_budget_bytes=_budget(shp, draft, 0, 0))
    try:
        P.spec_prefill(s.ctx, 0, prompts[:3], 4)
        P.spec_draft(s.ctx, 0, 2)
        ids = torch.zeros((shp.n_layers, 2, 2), dtype=torch.int32, device="cuda")
        P.spec_debug_force_routing(s.ctx, 0, ids, 2)      # 2 rows per layer, the pass has 9
        with pytest.raises(P.binding.SpecError) as e:
            P.spec_verify(s.ctx, 0, None, 2)
        assert e.value.code == P.SPEC_ERR_ARG
        P.spec_sync(s.ctx)
        # that error came before any streamed piece was taken: the context still works
        P.spec_verify(s.ctx, 0, None, 2)
        P.spec_sync(s.ctx)
    finally:
        s.close()
