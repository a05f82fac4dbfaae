"""Pins for the oracle's network code (CPU only): special cases, invariants, and an
independent formulation built from library routines (torch SDPA / topk / softmax)."""
import numpy as np
import pytest
import torch

import synth
from oracle import counts, model


def _mini(dtype="f32", **kw):
    shp = synth.mini_moe_shape(dtype=dtype, **kw)
    hm = synth.make_model(shp, seed=3)
    return shp, hm


def test_round_bf16_matches_torch():
    rng = np.random.default_rng(0)
    a = rng.standard_normal(10000) * np.exp(rng.uniform(-20, 20, 10000))
    ref = torch.from_numpy(a.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(model.round_bf16(a), ref)
    # ties go to even: 1 + 2^-8 is halfway between bf16 neighbours 1 and 1 + 2^-7
    assert model.round_bf16(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert model.round_bf16(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6


def test_rmsnorm_unit_rms_and_gain():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 64)) * 7
    y = model.rmsnorm(x, np.ones(64), 0.0)
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0)
    g = rng.standard_normal(64)
    assert np.allclose(model.rmsnorm(x, g, 0.0), y * g)
    # eps enters under the root, added to the mean square
    x1 = np.full((1, 4), 2.0)
    assert np.allclose(model.rmsnorm(x1, np.ones(4), 5.0), 2.0 / 3.0)


def test_rope_properties():
    rng = np.random.default_rng(2)
    q = rng.standard_normal((6, 3, 16))
    k = rng.standard_normal((6, 3, 16))
    pos = np.arange(6)
    # position 0 is the identity; the rotation preserves norms
    assert np.allclose(model.rope(q[:1], np.array([0]), 1e4), q[:1])
    assert np.allclose(np.linalg.norm(model.rope(q, pos, 1e4), axis=-1), np.linalg.norm(q, axis=-1))
    # <rope(q,m), rope(k,n)> depends on m-n only
    a = (model.rope(q[:1], np.array([9]), 1e4) * model.rope(k[:1], np.array([4]), 1e4)).sum()
    b = (model.rope(q[:1], np.array([25]), 1e4) * model.rope(k[:1], np.array([20]), 1e4)).sum()
    assert np.isclose(a, b)
    # explicit pair (i, i+dh/2), angle pos * theta^(-2i/dh)
    v = np.zeros((1, 1, 8)); v[0, 0, 1] = 1.0            # pair (1, 5), i = 1
    out = model.rope(v, np.array([3]), 100.0)[0, 0]
    ang = 3 * 100.0 ** (-2 * 1 / 8)
    exp = np.zeros(8); exp[1] = np.cos(ang); exp[5] = np.sin(ang)
    assert np.allclose(out, exp)


def test_silu_closed_form():
    z = np.array([-3.0, 0.0, 2.0])
    assert np.allclose(model.silu(z), z * (1 / (1 + np.exp(-z))))
    assert model.silu(np.array([0.0]))[0] == 0.0
    # against the library's routine, and what follows from sigma(z) + sigma(-z) = 1 without naming sigma:
    # silu(z) - silu(-z) = z; silu(z) -> z for large z and -> 0 for large negative z
    zz = np.linspace(-12.0, 12.0, 97)
    assert np.allclose(model.silu(zz), torch.nn.functional.silu(torch.from_numpy(zz)).numpy(), atol=1e-15)
    assert np.allclose(model.silu(zz) - model.silu(-zz), zz, atol=1e-14)
    assert abs(model.silu(np.array([40.0]))[0] - 40.0) < 1e-12 and abs(model.silu(np.array([-40.0]))[0]) < 1e-12


def test_attention_single_key_returns_value():
    shp, hm = _mini()
    dec = model.build(hm)
    c = dec.new_cache(4)
    x = dec.embed(np.array([5]))
    y = dec.attention_part(0, x, c, 0)
    W = hm.layer(0)
    h = model.rmsnorm(x, W["g1"], shp.rms_eps)
    v = (h @ W["wqkv"].astype(np.float64).T)[:, (shp.n_q_heads + shp.n_kv_heads) * shp.head_dim:]
    g = shp.n_q_heads // shp.n_kv_heads
    a = np.repeat(v.reshape(shp.n_kv_heads, shp.head_dim), g, axis=0).reshape(1, -1)
    assert np.allclose(y, x + a @ W["wo"].astype(np.float64).T, atol=1e-12)


def test_incremental_equals_block_equals_full():
    for shp, hm in (_mini(), (synth.workload("cfg1").target, synth.make_model(synth.workload("cfg1").target))):
        dec = model.build(hm)
        toks = synth.make_prompts(1, (11, 11), shp.vocab, seed=4)[0]
        full = dec.forward_full(toks)
        c = dec.new_cache(16)
        inc = np.concatenate([dec.forward([c], [toks[i:i + 1]], [i])[0] for i in range(len(toks))])
        c2 = dec.new_cache(16)
        blk = np.concatenate([dec.forward([c2], [toks[:4]], [0])[0], dec.forward([c2], [toks[4:]], [4])[0]])
        assert np.allclose(full, inc, atol=1e-10) and np.allclose(full, blk, atol=1e-10)
        # rewriting positions (rollback then other tokens) leaves earlier positions untouched
        c3 = dec.new_cache(16)
        dec.forward([c3], [np.concatenate([toks[:6], [1, 2, 3]])], [0])
        again = dec.forward([c3], [toks[6:]], [6])[0]
        assert np.allclose(full[6:], again, atol=1e-10)


def test_batch_rows_are_independent():
    shp, hm = _mini()
    dec = model.build(hm)
    ps = synth.make_prompts(3, (5, 9), shp.vocab, seed=5)
    cs = [dec.new_cache(12) for _ in ps]
    together = dec.forward(cs, ps, [0, 0, 0])
    for p, z in zip(ps, together):
        assert np.allclose(dec.forward_full(p), z, atol=1e-10)


def test_moe_two_identical_experts_reduce_to_dense():
    shp = synth.mini_moe_shape(n_experts=2, dtype="f32")
    hm = synth.make_model(shp, seed=6)
    L = hm.layer(0)
    for nm in ("w1", "w3", "w2"):
        L[f"{nm}_1"][...] = L[f"{nm}_0"]
    dec = model.Decoder(shp, [L, hm.layer(1)], hm.globals())
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, shp.d_model))
    h2 = model.rmsnorm(x, L["g2"], shp.rms_eps)
    dense = x + (model.silu(h2 @ L["w1_0"].T.astype(np.float64)) * (h2 @ L["w3_0"].T.astype(np.float64))) @ L["w2_0"].T.astype(np.float64)
    assert np.allclose(dec.ffn_part(0, x), dense, atol=1e-12)


def test_router_top2_tie_break_and_weights():
    shp, hm = _mini()
    dec = model.build(hm)
    dec.layers[0]["wr"][...] = 0.0                      # all logits equal -> experts 0 and 1, weights 1/2
    ids, w, _ = dec.route(0, np.ones((2, shp.d_model)))
    assert ids.tolist() == [[0, 1], [0, 1]] and np.allclose(w, 0.5)
    dec.layers[0]["wr"][5, 0] = 1.0
    dec.layers[0]["wr"][2, 0] = np.log(3.0).astype(np.float32)
    ids, w, _ = dec.route(0, np.eye(1, shp.d_model))
    assert ids.tolist() == [[2, 5]] and np.allclose(w, [[3 / (3 + np.e), np.e / (3 + np.e)]], atol=1e-6)


def _torch_reference_logits(shp, hm, toks):
    """Same network from library pieces: SDPA(is_causal), topk, softmax over all experts then
    renormalise, every expert evaluated densely and masked."""
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    G = {k: t(v) for k, v in hm.globals().items()}
    x = G["emb"][torch.from_numpy(toks.astype(np.int64))]
    n = len(toks)
    Hq, Hkv, dh = shp.n_q_heads, shp.n_kv_heads, shp.head_dim
    half = dh // 2
    inv = torch.tensor(shp.rope_theta, dtype=torch.float64) ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * inv[None]
    cos, sin = torch.cat([ang.cos(), ang.cos()], -1), torch.cat([ang.sin(), ang.sin()], -1)

    def rot(v):                                          # rotate_half formulation
        v1, v2 = v[..., :half], v[..., half:]
        return v * cos[:, None, :] + torch.cat([-v2, v1], -1) * sin[:, None, :]

    def norm(v, g):
        return v * torch.rsqrt(v.pow(2).mean(-1, keepdim=True) + shp.rms_eps) * g

    for l in range(shp.n_layers):
        W = {k: t(v) for k, v in hm.layer(l).items()}
        h = norm(x, W["g1"])
        qkv = torch.nn.functional.linear(h, W["wqkv"])
        q, k, v = qkv.split([Hq * dh, Hkv * dh, Hkv * dh], dim=-1)
        q, k, v = rot(q.view(n, Hq, dh)), rot(k.view(n, Hkv, dh)), v.view(n, Hkv, dh)
        k = k.repeat_interleave(Hq // Hkv, dim=1)
        v = v.repeat_interleave(Hq // Hkv, dim=1)
        a = torch.nn.functional.scaled_dot_product_attention(q.transpose(0, 1), k.transpose(0, 1),
                                                             v.transpose(0, 1), is_causal=True)
        x = x + torch.nn.functional.linear(a.transpose(0, 1).reshape(n, Hq * dh), W["wo"])
        h2 = norm(x, W["g2"])
        if shp.n_experts:
            probs = torch.softmax(torch.nn.functional.linear(h2, W["wr"]), dim=-1)
            top, idx = torch.topk(probs, 2, dim=-1)
            top = top / top.sum(-1, keepdim=True)
            gate = torch.zeros_like(probs).scatter(1, idx, top)
            for e in range(shp.n_experts):
                y = torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(h2, W[f"w1_{e}"]))
                                               * torch.nn.functional.linear(h2, W[f"w3_{e}"]), W[f"w2_{e}"])
                x = x + gate[:, e:e + 1] * y
        else:
            x = x + torch.nn.functional.linear(torch.nn.functional.silu(torch.nn.functional.linear(h2, W["w1_0"]))
                                               * torch.nn.functional.linear(h2, W["w3_0"]), W["w2_0"])
    return torch.nn.functional.linear(norm(x, G["gf"]), G["head"]).numpy()


@pytest.mark.parametrize("which", ["moe", "dense"])
def test_forward_matches_library_formulation(which):
    if which == "moe":
        shp, hm = _mini()
    else:
        shp = synth.workload("cfg1").target
        hm = synth.make_model(shp)
    toks = synth.make_prompts(1, (13, 13), shp.vocab, seed=7)[0]
    ours = model.build(hm).forward_full(toks)
    ref = _torch_reference_logits(shp, hm, toks)
    assert np.abs(ours - ref).max() < 1e-9


def test_draft_is_truncation_of_target():
    shp, hm = _mini()
    dm = hm.draft_view(1, attn_only=True)
    dd = model.build(dm)
    toks = synth.make_prompts(1, (6, 6), shp.vocab, seed=8)[0]
    z = dd.forward_full(toks)
    # by hand: one attention-only layer then final norm and head
    t = model.build(hm)
    c = t.new_cache(8)
    x = t.attention_part(0, t.embed(toks), c, 0)
    assert np.allclose(z, t.head(x), atol=1e-12)


def test_param_counts_against_paper():
    facts = {}
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/paper_facts.txt"):
        if line.strip() and not line.startswith("#"):
            name, val, *_ = line.split()
            facts[name] = float(val)
    s7, s22 = synth.workload("cfg3").target, synth.workload("cfg4").target
    assert abs(counts.model_params(s7) / 1e9 - facts["mixtral_8x7b_params_B"]) < 0.05
    assert abs(counts.model_params(s22) / 1e9 - facts["mixtral_8x22b_params_B"]) < 0.5
    assert abs(counts.model_params(s22) * 2 / 1e9 - facts["mixtral_8x22b_bytes_GB"]) < 1.0
    # the layout code of the input format agrees with the closed forms
    for s in (s7, s22, synth.workload("cfg1").target, s7.draft(4, True)):
        assert s.n_params() == counts.model_params(s)
    # one 8x22B FFN layer (8 experts) in 240 ms must be a plausible PCIe 4.0 x16 rate (< 32 GB/s)
    gbps = 8 * counts.expert_params(s22) * 2 / 1e9 / (facts["ffn_layer_8x22b_load_ms"] * 1e-3)
    assert 15.0 < gbps < 32.0


def test_generator_kat_and_determinism():
    from synth.weights import philox4x32_10, fill_normal
    for line in open(__file__.rsplit("/", 1)[0] + "/golden/philox4x32_10_kat.txt"):
        if line.strip() and not line.startswith("#"):
            w = [int(x, 16) for x in line.split()]
            assert philox4x32_10(w[:4], w[4:6]).tolist() == w[6:]
    a = np.empty(70001, dtype=np.float32); b = np.empty(70001, dtype=np.float32)
    fill_normal(a, 1, 2, n_threads=1); fill_normal(b, 1, 2, n_threads=5)
    assert np.array_equal(a, b) and abs(a.std() - 0.02) < 3e-4 and abs(a.mean()) < 3e-4
