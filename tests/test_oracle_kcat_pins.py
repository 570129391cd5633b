"""Pins for the oracle's causal reading of Eq. 2 (CaP tokens attend to their own keys as well): a hand-worked
example, closed forms, a torch witness that builds the mask from the full-sequence causal mask, brute force with
scalar loops, and the limit in which the CaP keys vanish.  None of them re-types the oracle's formula."""
import math

import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_hand_worked_example():
    """Queries are unit vectors and keys are logs, so every exp(logit) is a chosen integer.
    Query 0 sees context weights a = (1,2,1,4) and CaP key 0 with weight 8:      row sum 16.
    Query 1 sees context weights b = (3,1,2,2) and CaP keys 0, 1 with 4 and 4:   row sum 16.
    u = (a + b) / 16.  CaP key 1 has weight 16 under query 0 - it is in that query's future and must not count."""
    a, b = np.array([1.0, 2, 1, 4]), np.array([3.0, 1, 2, 2])
    K = np.stack([np.log(a), np.log(b)], axis=1)
    Q = np.array([[1.0, 0.0], [0.0, 1.0]])
    K_cap = np.array([[math.log(8), math.log(4)], [math.log(16), math.log(4)]])
    u = O.cap_scores(Q, K, 1.0, K_cap)
    np.testing.assert_allclose(u * 16, [4, 3, 3, 6], rtol=1e-13)
    # the other readings of the mask give other numbers (so the pin above tells them apart)
    for wrong in ([1 / 8 + 3 / 12, 2 / 8 + 1 / 12, 1 / 8 + 2 / 12, 4 / 8 + 2 / 12],            # strictly causal
                  [1 / 32 + 3 / 16, 2 / 32 + 1 / 16, 1 / 32 + 2 / 16, 4 / 32 + 2 / 16]):       # no mask
        assert np.abs(u - np.array(wrong)).max() > 1e-3


@pytest.mark.parametrize("G,P,n,d", [(1, 1, 5, 4), (3, 4, 17, 8), (4, 64, 300, 16)])
def test_zero_queries_give_harmonic_sums(G, P, n, d):
    """All logits equal: CaP token i spreads its mass evenly over n + i + 1 visible keys."""
    r = _rng(1)
    K, K_cap = r.standard_normal((n, d)), r.standard_normal((P, d))
    u = O.cap_scores(np.zeros((G * P, d)), K, 0.37, K_cap)
    expect = G * sum(1.0 / (n + i + 1) for i in range(P))
    np.testing.assert_allclose(u, np.full(n, expect), rtol=1e-13)


@pytest.mark.parametrize("G,P,n,d,seed", [(1, 3, 9, 4, 2), (2, 5, 40, 8, 3), (4, 16, 130, 32, 4)])
def test_torch_witness_full_sequence_causal_mask(G, P, n, d, seed):
    """The CaP rows of a causal attention over the sequence [context, CaP], masked with the lower triangle of the
    full (n + P) x (n + P) matrix, summed over rows and heads, context columns kept."""
    r = _rng(seed)
    Q, K, K_cap = r.standard_normal((G, P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    scale = 1.0 / math.sqrt(d)
    keys = torch.from_numpy(np.concatenate([K, K_cap], axis=0))
    causal = torch.ones(n + P, n + P, dtype=torch.bool).tril()[n:]           # rows of the CaP tokens
    total = torch.zeros(n, dtype=torch.float64)
    for g in range(G):
        logits = torch.from_numpy(Q[g]) @ keys.T * scale
        attn = torch.softmax(logits.masked_fill(~causal, float("-inf")), dim=-1)
        total += attn[:, :n].sum(dim=0)
    u = O.cap_scores(Q.reshape(G * P, d), K, scale, K_cap)
    np.testing.assert_allclose(u, total.numpy(), rtol=1e-12, atol=1e-300)


def test_brute_force_scalar_loops():
    r = _rng(5)
    G, P, n, d, scale = 2, 3, 6, 3, 0.8
    Q, K, K_cap = r.standard_normal((G * P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    u = [0.0] * n
    cap_mass = 0.0
    for g in range(G):
        for i in range(P):
            q = Q[g * P + i]
            w_ctx = [math.exp(scale * sum(q[c] * K[t][c] for c in range(d))) for t in range(n)]
            w_cap = [math.exp(scale * sum(q[c] * K_cap[j][c] for c in range(d))) for j in range(i + 1)]
            z = sum(w_ctx) + sum(w_cap)
            for t in range(n):
                u[t] += w_ctx[t] / z
            cap_mass += sum(w_cap) / z
    got = O.cap_scores(Q, K, scale, K_cap)
    np.testing.assert_allclose(got, u, rtol=1e-12)
    # probability mass: what the context does not get, the visible CaP keys got
    assert abs(got.sum() + cap_mass - G * P) < 1e-12


def test_cap_keys_only_take_mass_and_vanish_in_the_limit():
    r = _rng(6)
    G, P, n, d = 2, 8, 50, 16
    Q = np.abs(r.standard_normal((G * P, d)))                  # positive queries: a negative key is far away
    K = r.standard_normal((n, d))
    plain = O.cap_scores(Q, K, 0.25)
    with_cap = O.cap_scores(Q, K, 0.25, r.standard_normal((P, d)))
    assert np.all(with_cap < plain)
    far = O.cap_scores(Q, K, 0.25, np.full((P, d), -1.0e3))
    np.testing.assert_allclose(far, plain, rtol=1e-13)


def test_a_cap_key_only_reaches_later_queries():
    """Changing CaP key j leaves the rows of queries i < j untouched: with one query per call, the score of CaP
    position i does not depend on the keys after it."""
    r = _rng(7)
    P, n, d = 5, 12, 8
    Q, K, K_cap = r.standard_normal((P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    changed = K_cap.copy()
    changed[3] += 1.0
    # split the sum over queries: put one query at a time on its CaP position, zero rows elsewhere contribute a
    # known harmonic term that cancels in the difference
    def per_query(kc):
        out = []
        for i in range(P):
            Qi = np.zeros((P, d)); Qi[i] = Q[i]
            out.append(O.cap_scores(Qi, K, 0.5, kc))
        return np.array(out)
    a, b = per_query(K_cap), per_query(changed)
    np.testing.assert_array_equal(a[:3], b[:3])
    assert np.all(np.abs(a[3:] - b[3:]).max(axis=1) > 1e-6)


def test_compress_threads_the_cap_keys_per_unit():
    """A unit whose CaP keys are far away scores as without them; the other units change."""
    from paper_2410_01518_amd import synth
    cfg = synth.CCDConfig(name="t", B=1, L=2, Hq=4, Hkv=2, d=64, N=96, k=40, P=4, T=10, w=3, dtype="fp32", keys="normal", seed=8)
    inp = synth.make_inputs(cfg)
    r = _rng(9)
    K_cap = r.standard_normal((cfg.B, cfg.L, cfg.Hkv, cfg.P, cfg.d)).astype(np.float32)
    Qabs = np.abs(inp["Q_cat"])
    K_cap[0, 1, 0] = -1.0e3
    kw = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w)
    plain = O.compress(Qabs, inp["K"], inp["V"], inp["novelty"], **kw)
    causal = O.compress(Qabs, inp["K"], inp["V"], inp["novelty"], K_cap=K_cap, **kw)
    np.testing.assert_array_equal(plain["scores"][0, 1, 0], causal["scores"][0, 1, 0])
    for (l, h) in [(0, 0), (0, 1), (1, 1)]:
        fin = np.isfinite(plain["scores"][0, l, h])
        assert np.all(causal["scores"][0, l, h][fin] <= plain["scores"][0, l, h][fin])
        assert np.any(causal["scores"][0, l, h][fin] < plain["scores"][0, l, h][fin])
