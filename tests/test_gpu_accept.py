"""GPU parity of the accept/reject kernels and the device Philox stream against the oracle, fed
identical logits and uniforms through the C ABI."""
import numpy as np
import pytest

import synth
from oracle import philox as ophilox, spec as ospec

pytestmark = pytest.mark.gpu


def _logits(B, k, V, seed, agree=0.6):
    rng = np.random.default_rng(seed)
    p = (rng.standard_normal((B, k + 1, V)) * 2.0).astype(np.float32)
    q = (p[:, :k] + rng.standard_normal((B, k, V)).astype(np.float32) * 1.0).astype(np.float32)
    d = np.argmax(p[:, :k], axis=-1).astype(np.int32)
    flip = rng.random((B, k)) > agree
    d[flip] = rng.integers(0, V, flip.sum())
    return p, q, d


# vocabularies of up to 32768 ids that are a multiple of 4 take the register-resident kernels (each row
# read once); 33 and 40000 take the general ones
@pytest.mark.parametrize("B,k,V", [(7, 4, 512), (3, 8, 32000), (1, 1, 33), (5, 0, 100), (64, 6, 32768),
                                   (4, 3, 40000), (3, 2, 12), (5, 16, 32768), (3, 16, 1001), (300, 2, 256)])
def test_accept_greedy(B, k, V):
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    p, _, d = _logits(B, k, V, seed=B * 100 + k)
    if k > 0 and B > 2:                          # exact ties: lowest id must win on both sides
        p[0, 0, 5] = p[0, 0].max() + 1; p[0, 0, 9] = p[0, 0, 5]; d[0, 0] = 5
        p[1, 0, 11] = p[1, 0].max() + 1; p[1, 0, 3] = p[1, 0, 11]; d[1, 0] = 11
    n = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    nx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    P.spec_accept(dev(p), None, dev(d) if k else None, None, None, 1.0, 0, 0, 0, B, k, V, n, nx)
    torch.cuda.synchronize()
    exp = [ospec.accept_greedy(p[b], d[b]) for b in range(B)]
    assert n.cpu().tolist() == [e[0] for e in exp]
    assert nx.cpu().tolist() == [e[1] for e in exp]


@pytest.mark.parametrize("B,k,V,tau", [(16, 4, 512, 0.8), (6, 6, 32000, 0.8), (4, 1, 17, 1.3), (32, 3, 1000, 0.5),
                                       (8, 3, 32768, 0.8), (4, 2, 40000, 0.8), (5, 1, 256, 1.0),
                                       (4, 16, 32768, 0.8), (4, 16, 1001, 0.9)])
def test_accept_sample_given_uniforms(B, k, V, tau):
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    p, q, _ = _logits(B, k, V, seed=7 * B + k)
    ud = synth.make_uniforms((B, k), seed=1)
    ua = synth.make_uniforms((B, k), seed=2)
    ur = synth.make_uniforms((B, k + 1), seed=3)
    # candidates are genuine draws from the draft rows
    d = np.array([[ospec.sample_inverse_cdf(ospec.softmax_t(q[b, i], tau), ud[b, i]) for i in range(k)]
                  for b in range(B)], dtype=np.int32)
    if B >= 4:
        q[0] = p[0, :k]                          # q == p: everything kept, bonus token from p_k
        d[0] = [ospec.sample_inverse_cdf(ospec.softmax_t(q[0, i], tau), ud[0, i]) for i in range(k)]
    n = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    nx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
    P.spec_accept(dev(p), dev(q), dev(d), dev(ua), dev(ur), tau, 0, 0, 0, B, k, V, n, nx)
    torch.cuda.synchronize()
    n, nx = n.cpu().numpy(), nx.cpu().numpy()
    exempt = 0
    for b in range(B):
        margins = []
        en, enx = ospec.accept_sample(p[b], q[b], d[b], ua[b], ur[b], tau, margins=margins)
        if n[b] != en:
            assert min(margins) < 1e-4, f"kept count differs at row {b} without a near-tie"
            exempt += 1
            continue
        if nx[b] != enx:
            # only a CDF-boundary near-tie may move the draw, and then only to a neighbouring id
            pr = ospec.softmax_t(p[b, en], tau)
            r = np.maximum(0, pr - ospec.softmax_t(q[b, en], tau)) if en < k else pr
            if r.sum() <= 0:
                r = pr
            c = np.cumsum(r) / r.sum()
            assert np.abs(c - ur[b, en]).min() < 1e-5, f"next token differs at row {b} away from a CDF edge"
            exempt += 1
    assert exempt <= max(1, B // 8)
    if B >= 4:
        assert n[0] == k


def test_accept_sample_internal_philox_matches_oracle_stream():
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    B, k, V, tau, seed, rnd, base = 9, 5, 700, 0.8, 0x1234567ABCDEF, 3, 40
    out = torch.zeros((B, k + 1, 3), dtype=torch.float32, device="cuda")
    P.spec_philox_uniforms(seed, rnd, base, B, k, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for b in range(B):
        ud, ua, ur = ophilox.round_uniforms(seed, rnd, base + b, k)
        assert np.array_equal(got[b, :, 0], ud.astype(np.float32))
        assert np.array_equal(got[b, :, 1], ua.astype(np.float32))
        assert np.array_equal(got[b, :, 2], ur.astype(np.float32))
    p, q, _ = _logits(B, k, V, seed=5)
    d = np.zeros((B, k), dtype=np.int32)
    exp = []
    for b in range(B):
        ud, ua, ur = ophilox.round_uniforms(seed, rnd, base + b, k)
        d[b] = [ospec.sample_inverse_cdf(ospec.softmax_t(q[b, i], tau), ud[i + 1]) for i in range(k)]
        exp.append(ospec.accept_sample(p[b], q[b], d[b], ua[1:], ur, tau))
    n = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    P.spec_accept(dev(p), dev(q), dev(d), None, None, tau, seed, rnd, base, B, k, V, n, nx)
    torch.cuda.synchronize()
    agree = sum(int(a == e[0] and c == e[1]) for a, c, e in zip(n.cpu().tolist(), nx.cpu().tolist(), exp))
    assert agree >= B - 1


def test_accept_sample_distribution_chi_square():
    """Tiny vocabulary, context-free p and q, device Philox: emitted tokens follow the target."""
    import torch
    from scipy import stats
    import paper_2505_10259_amd as P
    from gpu_common import dev
    V, k, tau, B = 12, 4, 0.8, 20000
    rng = np.random.default_rng(1)
    pz, qz = rng.standard_normal(V) * 1.5, rng.standard_normal(V) * 1.5
    pr, qr = ospec.softmax_t(pz, tau), ospec.softmax_t(qz, tau)
    p = np.tile(pz.astype(np.float32), (B, k + 1, 1))
    q = np.tile(qz.astype(np.float32), (B, k, 1))
    d = rng.choice(V, size=(B, k), p=ospec.softmax_t(qz.astype(np.float32), tau)).astype(np.int32)
    n = torch.zeros(B, dtype=torch.int32, device="cuda")
    nx = torch.zeros(B, dtype=torch.int32, device="cuda")
    P.spec_accept(dev(p), dev(q), dev(d), None, None, tau, 99, 0, 0, B, k, V, n, nx)
    torch.cuda.synchronize()
    n, nx = n.cpu().numpy(), nx.cpu().numpy()
    emitted = np.concatenate([np.concatenate([d[b, :n[b]], [nx[b]]]) for b in range(B)])
    obs = np.bincount(emitted, minlength=V)
    chi2, pval = stats.chisquare(obs, pr * len(emitted))
    assert pval > 0.01, (chi2, pval)
    alpha = np.minimum(pr, qr).sum()
    assert abs((n + 1).mean() - ospec.expected_generated(alpha, k)) < 4 * (n + 1).std() / np.sqrt(B)


@pytest.mark.parametrize("V", [512, 40000])        # register-resident and general kernels
def test_candidate_outside_the_vocabulary_is_rejected(V):
    """An id that is no token (V, a negative number) must never index the probability rows: the
    sampling rule treats it as rejected at its position, the greedy rule as a mismatch."""
    import torch
    import paper_2505_10259_amd as P
    from gpu_common import dev
    B, k, tau = 4, 3, 0.8
    p, q, _ = _logits(B, k, V, seed=V)
    q[:] = p[:, :k]                              # q == p: every genuine candidate is kept
    ud = synth.make_uniforms((B, k), seed=11)
    d = np.array([[ospec.sample_inverse_cdf(ospec.softmax_t(q[b, i], tau), ud[b, i]) for i in range(k)]
                  for b in range(B)], dtype=np.int32)
    d[0, 1], d[1, 0], d[2, 2] = V, -7, V + 12345
    ua = synth.make_uniforms((B, k), seed=12)
    ur = synth.make_uniforms((B, k + 1), seed=13)
    for q_dev in (dev(q), None):
        n = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        nx = torch.full((B,), -1, dtype=torch.int32, device="cuda")
        if q_dev is None:
            dd = np.argmax(p[:, :k], axis=-1).astype(np.int32)      # greedy: the target's own choices ...
            dd[0, 1], dd[1, 0], dd[2, 2] = V, -7, V + 12345         # ... except the invalid ids
            P.spec_accept(dev(p), None, dev(dd), None, None, 1.0, 0, 0, 0, B, k, V, n, nx)
        else:
            P.spec_accept(dev(p), q_dev, dev(d), dev(ua), dev(ur), tau, 0, 0, 0, B, k, V, n, nx)
        torch.cuda.synchronize()
        assert n.cpu().tolist() == [1, 0, 2, 3]
        assert all(0 <= t < V for t in nx.cpu().tolist())
