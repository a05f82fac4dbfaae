"""GPU parity of one decoder layer of the verify pass (spec_layer_forward: RMSNorm, QKV GEMM, RoPE +
paged KV append, attention over the cached context, O-projection, router, top-2 grouped MoE GEMMs,
combine) against the oracle, on a small layer element by element and on the full Mixtral-8x7B-shaped
layer (256 sequences x 9 tokens, 2048 cached positions) for sampled sequences."""
import numpy as np
import pytest

import synth
from oracle import model as omodel

pytestmark = pytest.mark.gpu


def _oracle_layer(hm, x_bits, kc_bits, vc_bits, seqs, n_new, ctx, act=None, forced_route=None, want_route=False,
                  forced_ids=None):
    """Layer 0 of `hm` on the rows of the sequences in `seqs`; returns (x_out [len(seqs)*n_new, d],
    router gap per row) and, with want_route, the (ids, weights) the router chose.  `act`: "bf16" rounds
    activations where a bf16 model stores them (the default for a bf16 model), "f64" rounds nothing."""
    shp = hm.shape
    dec = omodel.Decoder(shp, [hm.layer(0)], hm.globals(), act=act or ("bf16" if shp.dtype == "bf16" else "f64"))
    widen = synth.bf16_bits_to_f32 if shp.dtype == "bf16" else (lambda a: a)
    xs = []
    for b in seqs:
        cache = dec.new_cache(ctx + n_new)
        cache.k[0][:, :ctx, :] = widen(kc_bits[b]).astype(np.float64)
        cache.v[0][:, :ctx, :] = widen(vc_bits[b]).astype(np.float64)
        x = widen(x_bits[b * n_new:(b + 1) * n_new]).astype(np.float64)
        xs.append(dec.attention_part(0, x, cache, ctx))
    xcat = np.concatenate(xs)
    if forced_ids is not None:
        # experts given row by row (rows of `seqs` in order); the mixing weights are still the softmax over the
        # two chosen router logits
        h2 = dec.r(omodel.rmsnorm(xcat, hm.layer(0)["g2"].astype(np.float64), shp.rms_eps))
        _, _, rl = dec.route(0, h2)
        n = np.arange(len(xcat))
        w0 = 1.0 / (1.0 + np.exp(rl[n, forced_ids[:, 1]] - rl[n, forced_ids[:, 0]]))
        forced_route = (forced_ids, np.stack([w0, 1.0 - w0], axis=1))
    out = dec.ffn_part(0, xcat, forced_route=forced_route)
    if want_route:
        h2 = dec.r(omodel.rmsnorm(xcat, hm.layer(0)["g2"].astype(np.float64), shp.rms_eps))
        ids, wts, _ = dec.route(0, h2)
        return out, dec._gap23, (ids, wts)
    return out, dec._gap23


def _run_gpu(hm, x, kc, vc, B, n_new, ctx, flags=0, page_tokens=0, forced_ids=None):
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    s = P.Session(hm, None, batch_max=B, k_max=n_new - 1, ctx_max=ctx + n_new + 2, flags=flags,
                  page_tokens=page_tokens)
    try:
        P.spec_kv_import(s.ctx, 0, 0, dev(kc), dev(vc), B, ctx)
        out = torch.zeros((B * n_new, hm.shape.d_model), dtype=torch.float32, device="cuda")
        if forced_ids is not None:
            f = dev(np.ascontiguousarray(forced_ids, dtype=np.int32))
            P.spec_debug_force_routing(s.ctx, 0, f, B * n_new)
        P.spec_layer_forward(s.ctx, 0, 0, dev(x), n_new, out)
        P.spec_sync(s.ctx, 0)
        ids = torch.zeros((B * n_new, 2), dtype=torch.int32, device="cuda")
        P.spec_debug_routing(s.ctx, 0, ids, None, B * n_new)
        return out.cpu().numpy(), ids.cpu().numpy()
    finally:
        s.close()


@pytest.mark.parametrize("B,n_new,ctx,page_tokens,flags", [
    (5, 9, 70, 32, 0),        # 36 query rows per KV head, ragged last key tile, 3 tiles: 2 + 1 per wavefront
    (3, 16, 300, 64, 0),      # 64 rows, 10 tiles: steady loop and both tail steps in each wavefront
    (2, 5, 0, 32, 0),         # empty context: only the new tokens attend to each other (one wavefront idle)
    (4, 1, 33, 32, 0),        # single new token (draft-style), one tile per wavefront
    (2, 9, 200, 32, 0),       # 7 tiles: 4 + 3 per wavefront
    (2, 17, 100, 32, 0),      # k = 16: 68 query rows per KV head, two row blocks per (sequence, KV head)
    (2, 9, 500, 128, 0),      # 128-token pages: four tiles per page
    (2, 9, 700, 256, 0),      # 256-token pages: eight tiles per page, the last page a third full
    (1, 9, 4200, 32, 0),      # 132 pages per sequence: the page-table row is longer than the workgroup
    (5, 9, 70, 16, 0),        # 16-token pages: plain attention kernel with MFMA GEMMs
    (5, 9, 70, 32, 2),        # all plain kernels
])
def test_small_layer_matches_oracle(B, n_new, ctx, page_tokens, flags):
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=1, n_q_heads=8, n_kv_heads=2)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, max(ctx, 1), seed=4)
    kc, vc = kc[:, :, :ctx], vc[:, :, :ctx]
    got, ids = _run_gpu(hm, x, np.ascontiguousarray(kc), np.ascontiguousarray(vc), B, n_new, ctx, flags,
                        page_tokens)
    exp, gap = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx)
    ok = gap > 5e-3                      # rows whose routing is not a near-tie
    assert ok.mean() > 0.8
    diff = np.abs(got - exp).max(axis=1)
    assert diff[ok].max() < 3e-2, diff
    print(f"layer B={B} n_new={n_new} ctx={ctx}: max diff {diff[ok].max():.2e} on {ok.sum()}/{ok.size} rows")


@pytest.mark.parametrize("B,n_new", [(3, 16), (4, 9)])      # 32 query rows (one column tile) / 36 (two)
def test_layer_when_the_softmax_reference_has_to_move(B, n_new):
    """Keys whose scores grow by far more than the kernel's lazy-reference slack from one key tile of a
    wavefront to its next (x8 from position 64, x40 from position 160): every wavefront then rescales
    accumulators that already hold sums, which ordinary random inputs almost never make it do."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=1, n_q_heads=8, n_kv_heads=2)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    ctx = 300
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=9)
    k = synth.bf16_bits_to_f32(kc)
    k[:, :, 64:160] *= 8.0
    k[:, :, 160:] *= 40.0
    kc = synth.f32_to_bf16_bits(k)
    got, ids = _run_gpu(hm, x, np.ascontiguousarray(kc), np.ascontiguousarray(vc), B, n_new, ctx, 0, 32)
    exp, gap = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx)
    ok = gap > 5e-3
    assert ok.mean() > 0.8
    diff = np.abs(got - exp).max(axis=1)
    assert diff[ok].max() < 3e-2, diff
    # and the plain attention kernel (exact running maximum) agrees on the same inputs
    got2, _ = _run_gpu(hm, x, np.ascontiguousarray(kc), np.ascontiguousarray(vc), B, n_new, ctx, 0, 16)
    assert np.abs(got2 - exp).max(axis=1)[ok].max() < 3e-2


def test_small_layer_f32_matches_oracle():
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="f32", n_layers=1, head_dim=64)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    B, n_new, ctx = 3, 4, 21
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=4)
    got, _ = _run_gpu(hm, x, kc, vc, B, n_new, ctx)
    exp, gap = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx)
    ok = gap > 1e-4
    assert np.abs(got - exp)[ok].max() < 2e-4


def test_cfg2_full_size_sampled_sequences():
    """The benchmark's launch configuration: d 4096, 32/8 heads x 128, 8 experts of 14336, B 256,
    k 8 (9 new tokens), 2048 cached positions.  The oracle recomputes a few whole sequences."""
    from gpu_common import host_model_pinned
    w = synth.workload("cfg2")
    shp, B, n_new, ctx = w.target, w.batch, w.k + 1, w.ctx
    hm = host_model_pinned(shp, seed=0)
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=0)
    got, ids = _run_gpu(hm, x, kc, vc, B, n_new, ctx)
    assert np.isfinite(got).all()
    counts = np.bincount(ids.ravel(), minlength=8)
    assert counts.sum() == 2 * B * n_new and (ids[:, 0] != ids[:, 1]).all()
    seqs = list(range(0, 256, 8))                    # 32 of the 256 sequences, all 9 rows of each
    exp, gap = _oracle_layer(hm, x, kc, vc, seqs, n_new, ctx)
    rows = np.concatenate([np.arange(b * n_new, (b + 1) * n_new) for b in seqs])
    ok = gap > 2e-3
    diff = np.abs(got[rows] - exp).max(axis=1)
    print(f"cfg2 sampled rows: max diff {diff[ok].max():.3e} ({ok.sum()}/{ok.size} rows), expert counts {counts.tolist()}")
    assert ok.mean() > 0.9
    assert diff[ok].max() < 3e-2


def _skewed_ids(T, pattern, seed):
    """[T, 2] expert ids (two different experts per row) with very uneven loads."""
    rng = np.random.default_rng(seed)
    ids = np.zeros((T, 2), dtype=np.int64)
    if pattern == "two":                 # every row on experts 0 and 1: six experts without rows
        ids[:, 1] = 1
    elif pattern == "last":              # every row on the last two experts
        ids[:, 0], ids[:, 1] = 6, 7
    elif pattern == "heavy":             # expert 0 takes half of the first choices, expert 7 nothing
        ids[:, 0] = np.where(rng.random(T) < 0.5, 0, rng.integers(1, 7, T))
        ids[:, 1] = (ids[:, 0] + rng.integers(1, 6, T)) % 7
        ids[:, 1] = np.where(ids[:, 1] == ids[:, 0], (ids[:, 0] + 1) % 7, ids[:, 1])
    elif pattern == "holes":             # experts 1, 4 and 6 empty, one row on expert 7
        pool = np.array([0, 2, 3, 5])
        ids[:, 0] = pool[rng.integers(0, 4, T)]
        ids[:, 1] = pool[(np.searchsorted(pool, ids[:, 0]) + rng.integers(1, 4, T)) % 4]
        ids[T // 2, 1] = 7
    assert (ids[:, 0] != ids[:, 1]).all()
    return ids


@pytest.mark.parametrize("pattern", ["two", "last", "heavy", "holes"])
def test_small_layer_with_uneven_expert_loads(pattern):
    """The grouped MoE products with groups of very different size, empty groups in front, in the middle
    and at the end, and a group of one row: experts forced row by row on both sides (40 sequences x 9
    tokens; the large groups span several row tiles)."""
    from gpu_common import host_model_pinned
    shp = synth.mini_moe_shape(dtype="bf16", n_layers=1, n_q_heads=8, n_kv_heads=2)
    hm = host_model_pinned(shp, seed=3, std=0.05)
    B, n_new, ctx = 40, 9, 70
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=4)
    ids = _skewed_ids(B * n_new, pattern, seed=1)
    got, gpu_ids = _run_gpu(hm, x, kc, vc, B, n_new, ctx, 0, 32, forced_ids=ids)
    assert np.array_equal(gpu_ids, ids)
    exp, _ = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx, forced_ids=ids)
    diff = np.abs(got - exp).max(axis=1)
    print(f"uneven expert loads ({pattern}): counts {np.bincount(ids.ravel(), minlength=8).tolist()}, max diff {diff.max():.2e}")
    assert diff.max() < 3e-2


def test_cfg2_shape_with_uneven_expert_loads():
    """The benchmark's launch configuration with one expert taking half of the first choices and one
    expert none: the XCDs' shares of the grouped products are then ranges of equal work that cut through
    experts.  The oracle recomputes 16 of the 256 sequences."""
    from gpu_common import host_model_pinned
    w = synth.workload("cfg2")
    shp, B, n_new, ctx = w.target, w.batch, w.k + 1, w.ctx
    hm = host_model_pinned(shp, seed=0)
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=0)
    ids = _skewed_ids(B * n_new, "heavy", seed=2)
    got, gpu_ids = _run_gpu(hm, x, kc, vc, B, n_new, ctx, forced_ids=ids)
    assert np.isfinite(got).all() and np.array_equal(gpu_ids, ids)
    seqs = list(range(0, 256, 16))
    rows = np.concatenate([np.arange(b * n_new, (b + 1) * n_new) for b in seqs])
    exp, _ = _oracle_layer(hm, x, kc, vc, seqs, n_new, ctx, forced_ids=ids[rows])
    diff = np.abs(got[rows] - exp).max(axis=1)
    print(f"cfg2 shape, uneven loads: counts {np.bincount(ids.ravel(), minlength=8).tolist()}, max diff {diff.max():.3e}")
    assert diff.max() < 3e-2


def test_8x22b_shape_layer_matches_oracle():
    """One layer at the shape of the largest configuration (d 6144, 48/8 heads: six query heads per KV
    head, so k = 6 gives 42 query rows per KV head; experts of 16384), 12 sequences x 7 new tokens over
    a ragged number of cached positions per tile (300)."""
    from dataclasses import replace
    from gpu_common import host_model_pinned
    shp = replace(synth.workload("cfg4").target, n_layers=1, vocab=1024)     # the layer does not touch the vocabulary
    B, n_new, ctx = 12, 7, 300
    hm = host_model_pinned(shp, seed=4)
    x, kc, vc = synth.make_layer_inputs(shp, B, n_new, ctx, seed=5)
    got, ids = _run_gpu(hm, x, kc, vc, B, n_new, ctx)
    exp, gap, route = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx, want_route=True)
    ok = gap > 2e-3
    assert ok.mean() > 0.9
    # the same rows in unrounded float64, on the experts the bf16 evaluation chose (the mixing weights too:
    # they depend on the rounded activations only through the router logits)
    exact, _ = _oracle_layer(hm, x, kc, vc, range(B), n_new, ctx, act="f64", forced_route=route)
    rms = lambda a: float(np.sqrt(np.mean(a[ok] ** 2)))
    g64, b64, gb = got - exact, exp - exact, got - exp
    print(f"8x22B-shaped layer ({ok.sum()}/{ok.size} rows): rms / max-abs   GPU - float64 {rms(g64):.2e} / {np.abs(g64[ok]).max():.2e}"
          f"   bf16 oracle - float64 {rms(b64):.2e} / {np.abs(b64[ok]).max():.2e}   GPU - bf16 oracle {rms(gb):.2e} / "
          f"{np.abs(gb[ok]).max():.2e}   (output rms {rms(exact):.2f})")
    # Outputs of this layer are about 2.9 in rms (experts of 16384 on d = 6144), and a bf16 evaluation of it
    # is 4-5e-3 of that away from the exact result whoever does it; 3e-2 max-abs cannot hold between two such
    # evaluations.  The kernels must be as close to the exact result as the reference bf16 evaluation, and
    # the two bf16 evaluations no further apart than two independent draws of that noise.
    assert rms(g64) <= 1.25 * rms(b64) and np.abs(g64[ok]).max() <= max(3e-2, 1.5 * np.abs(b64[ok]).max())
    assert rms(gb) <= 1.25 * np.sqrt(2.0) * rms(b64) and np.abs(gb[ok]).max() <= max(3e-2, 2.5 * np.abs(b64[ok]).max())
