"""Pins for the oracle's speculative-decoding logic (CPU only)."""
import itertools

import numpy as np
import pytest
from scipy import stats

import synth
from oracle import model, philox, spec

GOLD = __file__.rsplit("/", 1)[0] + "/golden/"


def test_oracle_philox_known_answers():
    for line in open(GOLD + "philox4x32_10_kat.txt"):
        if line.strip() and not line.startswith("#"):
            w = [int(x, 16) for x in line.split()]
            assert list(philox.philox4x32_10(w[:4], w[4:6])) == w[6:]
    assert philox.word_to_uniform(0xFFFFFFFF) == 1.0 - 2.0 ** -24
    assert philox.word_to_uniform(0x000000FF) == 0.0


def test_expected_generated_is_sum_of_paper_pmf():
    # Appendix A.1: P[j] = p^(j-1)(1-p) for j <= k, P[k+1] = p^k
    for p in (0.0, 0.3, 0.8, 0.99):
        for k in (1, 2, 4, 8):
            pmf = [p ** (j - 1) * (1 - p) for j in range(1, k + 1)] + [p ** k]
            assert abs(sum(pmf) - 1.0) < 1e-12
            mean = sum(j * pj for j, pj in zip(range(1, k + 2), pmf))
            assert abs(spec.expected_generated(p, k) - mean) < 1e-12
    assert spec.expected_generated(1.0, 5) == 6.0
    # the closed form as printed disagrees with that sum already at k = 1
    p, k = 0.5, 1
    printed = (k * p ** (k + 2) - (k + 1) * p ** (k + 1) + 1) / (1 - p)
    assert abs(printed - (1 + p)) > 0.1


def test_inverse_cdf_convention():
    w = np.array([0.0, 2.0, 0.0, 1.0, 1.0])
    assert spec.sample_inverse_cdf(w, 0.0) == 1          # never an id of zero weight
    assert spec.sample_inverse_cdf(w, 0.4999) == 1
    assert spec.sample_inverse_cdf(w, 0.5) == 3          # running sum must EXCEED u*total
    assert spec.sample_inverse_cdf(w, 0.75) == 4
    assert spec.sample_inverse_cdf(w, 1 - 2.0 ** -24) == 4


def test_accept_greedy_cases():
    V = 6
    z = np.full((4, V), -1.0)
    for i, t in enumerate([2, 5, 1, 3]):
        z[i, t] = 1.0
    assert spec.accept_greedy(z, [2, 5, 1]) == (3, 3)
    assert spec.accept_greedy(z, [2, 4, 1]) == (1, 5)
    assert spec.accept_greedy(z, [0, 5, 1]) == (0, 2)
    z[0, 1] = 1.0                                        # tie at row 0 between ids 1 and 2 -> 1
    assert spec.accept_greedy(z, [2, 5, 1]) == (0, 1)
    assert spec.accept_greedy(z[:1], []) == (0, 1)       # k = 0 is plain decoding


# -- invariant: greedy speculative decoding == plain greedy decoding, whatever the draft ------
@pytest.fixture(scope="module")
def cfg1():
    w = synth.workload("cfg1")
    hm = synth.make_model(w.target, seed=0)
    prompts = synth.make_prompts(w.batch, w.prompt_len, w.target.vocab, seed=0)
    tgt = model.build(hm)
    plain = spec.plain_decode(tgt, prompts, w.max_new + 9)
    return w, hm, prompts, tgt, plain


@pytest.mark.parametrize("k", [1, 2, 3, 4, 5, 6, 7, 8])
def test_greedy_spec_equals_plain_cfg1(cfg1, k):
    w, hm, prompts, tgt, plain = cfg1
    drf = spec.ModelDraft(model.build(hm.draft_view(w.draft_layers, w.draft_attn_only)))
    out, st = spec.speculative_decode(tgt, drf, prompts, k, w.max_new)
    assert out == [p[:w.max_new] for p in plain]
    assert st["rounds"] <= st["accept_hist"].sum() <= st["rounds"] * w.batch
    assert all(len(o) == w.max_new for o in out)


def test_greedy_spec_any_draft(cfg1):
    w, hm, prompts, tgt, plain = cfg1
    rng = np.random.default_rng(0)
    rand = spec.FixedDraft(lambda toks, k: rng.integers(0, w.target.vocab, k))
    out, st = spec.speculative_decode(tgt, rand, prompts, 4, w.max_new)
    assert out == [p[:w.max_new] for p in plain]
    # a draft that always agrees with the target: every round keeps all k
    by_prompt = {tuple(p.tolist()): pl for p, pl in zip(prompts, plain)}

    def perfect(toks, k):
        for p, pl in by_prompt.items():
            if tuple(toks[:len(p)]) == p:
                done = len(toks) - len(p)
                return pl[done:done + k]
        raise AssertionError
    trace = []
    out, st = spec.speculative_decode(tgt, spec.FixedDraft(perfect), prompts, 4, w.max_new, trace=trace)
    assert out == [p[:w.max_new] for p in plain]
    assert all(t.n_accepted == 4 for t in trace)
    assert st["rounds"] == -(-w.max_new // 5)             # ceil(16 / (k+1))
    # emitted per round always within 1..k+1, clipped only in the last round
    assert all(1 <= len(t.committed) <= 5 for t in trace)


def test_greedy_spec_equals_plain_moe_bf16():
    shp = synth.mini_moe_shape(dtype="bf16")
    hm = synth.make_model(shp, seed=11)
    prompts = synth.make_prompts(3, (5, 12), shp.vocab, seed=2)
    tgt = model.build(hm)
    drf = spec.ModelDraft(model.build(hm.draft_view(1, attn_only=True)))
    out, st = spec.speculative_decode(tgt, drf, prompts, 3, 10)
    assert out == spec.plain_decode(tgt, prompts, 10)


# -- stochastic rule -----------------------------------------------------------------------
def _toy(V, seed):
    rng = np.random.default_rng(seed)
    return rng.standard_normal(V) * 1.5, rng.standard_normal(V) * 1.5


def _round_on_fixed(pz, qz, k, tau, ud, ua, ur):
    """One round with context-free target logits pz and draft logits qz."""
    q = spec.softmax_t(qz, tau)
    d = [spec.sample_inverse_cdf(q, ud[i]) for i in range(k)]
    n, nxt = spec.accept_sample(np.tile(pz, (k + 1, 1)), np.tile(qz, (k, 1)), d, ua, ur, tau)
    return d[:n] + [nxt], n


def test_chi_square_emitted_tokens_follow_target():
    V, k, tau = 12, 4, 0.8
    pz, qz = _toy(V, 1)
    p = spec.softmax_t(pz, tau)
    rng = np.random.default_rng(123)
    emitted, ns = [], []
    while len(emitted) < 100_000:
        toks, n = _round_on_fixed(pz, qz, k, tau, rng.random(k), rng.random(k), rng.random(k + 1))
        emitted += toks
        ns.append(n)
    emitted = np.array(emitted[:100_000])
    obs = np.bincount(emitted, minlength=V)
    chi2, pval = stats.chisquare(obs, p * len(emitted))
    assert pval > 0.01, (chi2, pval)
    # consecutive emitted tokens are independent: chi-square on pairs against p (x) p
    pairs = np.bincount(emitted[:-1:2] * V + emitted[1::2], minlength=V * V)
    exp = np.outer(p, p).ravel() * pairs.sum()
    keep = exp > 5
    chi2, pval2 = stats.chisquare(pairs[keep], exp[keep] * pairs[keep].sum() / exp[keep].sum())
    assert pval2 > 0.01, (chi2, pval2)
    # acceptance law: per-candidate keep probability alpha = sum min(p, q); mean emitted per
    # round = (1 - alpha^(k+1)) / (1 - alpha)
    q = spec.softmax_t(qz, tau)
    alpha = np.minimum(p, q).sum()
    ns = np.array(ns)
    mean_emit = (ns + 1).mean()
    sd = (ns + 1).std() / np.sqrt(len(ns))
    assert abs(mean_emit - spec.expected_generated(alpha, k)) < 4 * sd
    for j in range(k):                                  # truncated-geometric counts
        assert abs((ns == j).mean() - alpha ** j * (1 - alpha)) < 4 * np.sqrt(0.25 / len(ns))


def test_chi_square_context_dependent_first_token():
    """Vocabulary-16 toy model: the first emitted token after a prompt has the target's
    next-token distribution (draft = a different model)."""
    shp = synth.ModelShape(n_layers=2, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ff=64,
                           vocab=16, n_experts=4, dtype="f32")
    hm = synth.make_model(shp, seed=21, std=0.6)
    tgt = model.build(hm)
    drf = model.build(hm.draft_view(1, attn_only=True))
    prompt = np.array([3, 7, 1, 12])
    pz = tgt.forward_full(prompt)[-1]
    tau = 0.8
    p = spec.softmax_t(pz, tau)
    c = drf.new_cache(8)
    drf.forward([c], [prompt[:-1]], [0], want_logits=False)
    qz1 = drf.forward([c], [prompt[-1:]], [3])[0][0]
    q1 = spec.softmax_t(qz1, tau)
    rng = np.random.default_rng(5)
    N = 40_000
    obs = np.zeros(16)
    for _ in range(N):                                   # k = 1 rounds; only the first token is context-exact
        d1 = spec.sample_inverse_cdf(q1, rng.random())
        n, nxt = spec.accept_sample(np.stack([pz, pz]), qz1[None], [d1], [rng.random()], rng.random(2), tau)
        obs[d1 if n == 1 else nxt] += 1
    chi2, pval = stats.chisquare(obs, p * N)
    assert pval > 0.01, (chi2, pval)


def test_sampling_special_cases():
    V, k, tau = 9, 3, 0.7
    pz, qz = _toy(V, 3)
    rng = np.random.default_rng(0)
    # q == p: every candidate kept (u*q < p holds for every u < 1)
    for _ in range(200):
        toks, n = _round_on_fixed(pz, pz, k, tau, rng.random(k), rng.random(k), rng.random(k + 1))
        assert n == k
    # draft puts all its mass where the target has none: nothing kept, next ~ p
    pz2 = pz.copy(); pz2[4] = -1e9
    qz2 = np.full(V, -1e9); qz2[4] = 0.0
    p2 = spec.softmax_t(pz2, tau)
    obs = np.zeros(V)
    for _ in range(20000):
        toks, n = _round_on_fixed(pz2, qz2, k, tau, rng.random(k), rng.random(k), rng.random(k + 1))
        assert n == 0
        obs[toks[0]] += 1
    keep = p2 > 0
    assert obs[~keep].sum() == 0
    assert stats.chisquare(obs[keep], p2[keep] * 20000 / p2[keep].sum())[1] > 0.01
    # tiny temperature: the sampling rule makes the greedy decisions
    for seed in range(20):
        pzs = np.random.default_rng(seed).standard_normal((k + 1, V))
        qzs = np.random.default_rng(seed + 99).standard_normal((k, V))
        d = [int(np.argmax(z)) for z in qzs]
        g = spec.accept_greedy(pzs, d)
        s = spec.accept_sample(pzs, qzs, d, rng.random(k), rng.random(k + 1), 1e-4)
        assert g == s


def test_brute_force_k2_exact_law():
    """V = 3, k = 2, probabilities on the 1/12 grid: integrating the oracle's rule over a
    12-point midpoint grid per uniform is exact, and the emitted stream must be i.i.d. p."""
    p = np.array([1 / 2, 1 / 3, 1 / 6]); q = np.array([1 / 4, 1 / 4, 1 / 2])
    pz, qz = np.log(p), np.log(q)
    M = 12
    grid = (np.arange(M) + 0.5) / M
    first = np.zeros(3)                  # law of the first emitted token
    joint = np.zeros((3, 3))             # P(n >= 1, x1 = a, x2 = b)
    rej = np.zeros(3)                    # P(n = 0, x1 = a)
    wgt = 1.0 / M ** 5
    for ud1, ud2, ua1, ua2, ur in itertools.product(grid, repeat=5):
        toks, n = _round_on_fixed(pz, qz, 2, 1.0, [ud1, ud2], [ua1, ua2], [ur, ur, ur])
        first[toks[0]] += wgt
        if n >= 1:
            joint[toks[0], toks[1]] += wgt
        else:
            rej[toks[0]] += wgt
    assert np.allclose(first, p, atol=1e-12)
    # second stream token: either emitted in this round, or the first token of the next round (~p)
    assert np.allclose(joint + np.outer(rej, p), np.outer(p, p), atol=1e-12)


def test_sampled_spec_decode_runs_and_is_reproducible():
    shp = synth.mini_moe_shape(dtype="f32", vocab=64)
    hm = synth.make_model(shp, seed=1, std=0.3)
    prompts = synth.make_prompts(2, (4, 6), shp.vocab, seed=3)
    tgt = model.build(hm)
    mk = lambda: spec.ModelDraft(model.build(hm.draft_view(1, attn_only=True)))
    a, sa = spec.speculative_decode(tgt, mk(), prompts, 3, 9, mode="sample", tau=0.8, seed=77)
    b, sb = spec.speculative_decode(tgt, mk(), prompts, 3, 9, mode="sample", tau=0.8, seed=77)
    c, _ = spec.speculative_decode(tgt, mk(), prompts[::-1], 3, 9, mode="sample", tau=0.8, seed=77, seq_ids=[1, 0])
    assert a == b and all(len(x) == 9 for x in a)
    assert c == a[::-1]                                  # results do not depend on batch order
    assert sa["accept_hist"].sum() >= sa["rounds"]


# -- the sampling LOOP (speculative_decode(mode="sample"), ModelDraft.propose, round_uniforms) ------
def _chi2_merged(obs, expected_p):
    """Chi-square of counts against probabilities with the bins of expected count < 5 merged into one."""
    exp = expected_p * obs.sum()
    small = exp < 5
    o = np.append(obs[~small], obs[small].sum())
    e = np.append(exp[~small], exp[small].sum())
    if e[-1] == 0:
        o, e = o[:-1], e[:-1]
    return stats.chisquare(o, e * o.sum() / e.sum())[1]


@pytest.fixture(scope="module")
def toy16():
    """Vocabulary-16 MoE target, one-layer attention-only draft, one prompt; the exact laws of the first
    two tokens of PLAIN sampling from the target (the definition the loop has to reproduce): p1 = softmax
    of the target's logits after the prompt, p2 = sum over t1 of p1(t1) * softmax(logits after prompt+t1)."""
    shp = synth.ModelShape(n_layers=2, d_model=32, n_q_heads=2, n_kv_heads=1, head_dim=16, d_ff=64,
                           vocab=16, n_experts=4, dtype="f32")
    hm = synth.make_model(shp, seed=21, std=0.6, gain_std=0.1)
    tgt = model.build(hm)
    prompt, tau = np.array([3, 7, 1, 12]), 0.8
    p1 = spec.softmax_t(tgt.forward_full(prompt)[-1], tau)
    p2 = np.zeros(16)
    for t1 in range(16):
        p2 += p1[t1] * spec.softmax_t(tgt.forward_full(np.append(prompt, t1))[-1], tau)
    mk = lambda: spec.ModelDraft(model.build(hm.draft_view(1, attn_only=True)))
    return tgt, mk, prompt, tau, p1, p2


def _loop_counts(toy16, n_seeds, B, k):
    tgt, mk, prompt, tau, _, _ = toy16
    c1, c2, hist = np.zeros(16), np.zeros(16), np.zeros(k + 1)
    for seed in range(n_seeds):
        out, st = spec.speculative_decode(tgt, mk(), [prompt] * B, k, 2, mode="sample", tau=tau, seed=1000 + seed)
        for o in out:
            c1[o[0]] += 1
            c2[o[1]] += 1
        hist += st["accept_hist"]
    return c1, c2, hist


def test_sampled_loop_emits_the_targets_distribution(toy16):
    """The whole sampling loop — Philox stream, draft draws, the hand-over of acceptance and resample
    uniforms, catch-up, the second round after a rejection — against plain sampling: first- and
    second-token marginals over 4096 independent sequences (distinct sequence ids and seeds)."""
    _, _, _, _, p1, p2 = toy16
    c1, c2, hist = _loop_counts(toy16, 32, 128, 3)
    assert hist[1:].sum() > 100 and hist[0] > 100          # both branches (kept, rejected) are exercised
    assert _chi2_merged(c1, p1) > 0.01
    assert _chi2_merged(c2, p2) > 0.01


@pytest.mark.parametrize("mutant", ["accept_reuses_draft_uniform", "resample_reuses_accept_uniform"])
def test_sampled_loop_pin_detects_shared_uniforms(toy16, monkeypatch, mutant):
    """The pin above has the power to catch the mistakes it is there for: an oracle whose acceptance
    test reuses the uniform that drew the candidate, or whose residual draw reuses the acceptance
    uniform, fails the same chi-square by many orders of magnitude."""
    _, _, _, _, p1, p2 = toy16
    orig = philox.round_uniforms

    def shared(seed, rnd, seq, k):
        ud, ua, ur = orig(seed, rnd, seq, k)
        return (ud, ud.copy(), ur) if mutant == "accept_reuses_draft_uniform" else (ud, ua, ua.copy())
    monkeypatch.setattr(philox, "round_uniforms", shared)
    c1, c2, _ = _loop_counts(toy16, 16, 128, 3)
    assert min(_chi2_merged(c1, p1), _chi2_merged(c2, p2)) < 1e-6


def test_round_uniforms_stream_layout():
    """Word order of a Philox block (the all-zero known-answer vector gives round 0, sequence 0,
    position 0 under seed 0), the counter fields, and independence of the three streams."""
    for line in open(GOLD + "philox4x32_10_kat.txt"):
        if line.strip() and not line.startswith("#"):
            w = [int(x, 16) for x in line.split()]
            if not any(w[:6]):
                ud, ua, ur = philox.round_uniforms(0, 0, 0, 0)
                assert (ud[0], ua[0], ur[0]) == tuple(philox.word_to_uniform(x) for x in w[6:9])
    # each counter field and each key half changes every word; position i only moves entry i
    base = np.concatenate(philox.round_uniforms(5, 2, 3, 4))
    for args in ((6, 2, 3, 4), (5 + (1 << 32), 2, 3, 4), (5, 3, 3, 4), (5, 2, 4, 4)):
        assert (np.concatenate(philox.round_uniforms(*args)) != base).all()
    longer = philox.round_uniforms(5, 2, 3, 6)
    for a, b in zip(philox.round_uniforms(5, 2, 3, 4), longer):
        assert np.array_equal(a, b[:5])
    # the three purposes are independent uniform streams: moments and cross-correlations over 20000 draws
    u = np.array([np.stack(philox.round_uniforms(9, r, s, 9)) for r in range(40) for s in range(50)])  # [2000,3,10]
    u = u.transpose(1, 0, 2).reshape(3, -1)
    assert np.abs(u.mean(axis=1) - 0.5).max() < 4 / np.sqrt(12 * u.shape[1])
    cc = np.corrcoef(u)
    assert np.abs(cc[np.triu_indices(3, 1)]).max() < 4 / np.sqrt(u.shape[1])
    assert stats.kstest(u[1], "uniform")[1] > 0.01
