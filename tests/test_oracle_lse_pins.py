"""Pins for the oracle's score from handed-in log-sum-exps: it must reproduce the two self-normalising readings when it is
given THEIR normalisers (computed here with scipy / torch, not with the oracle), a hand-worked example, and brute force."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import ccd_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_hand_worked_example():
    """exp(logit) are chosen integers; with lse = log(row sum) the score is the plain one, with a larger lse (the row
    also spent mass elsewhere) every probability shrinks by the same factor."""
    a, b = np.array([1.0, 2, 1, 4]), np.array([3.0, 1, 2, 2])
    K = np.stack([np.log(a), np.log(b)], axis=1)
    Q = np.array([[1.0, 0.0], [0.0, 1.0]])
    u = O.cap_scores_given_lse(Q, K, 1.0, np.log([8.0, 8.0]))
    np.testing.assert_allclose(u * 8, a + b, rtol=1e-13)
    u = O.cap_scores_given_lse(Q, K, 1.0, np.log([16.0, 32.0]))
    np.testing.assert_allclose(u, a / 16 + b / 32, rtol=1e-13)
    u = O.cap_scores_given_lse(Q, K, 1.0, np.log([8.0, 5.0]), P=2, window=5)      # query 1 does not see token 0
    np.testing.assert_allclose(u, [1 / 8, 2 / 8 + 1 / 5, 1 / 8 + 2 / 5, 4 / 8 + 2 / 5], rtol=1e-13)


@pytest.mark.parametrize("G,P,n,d,seed", [(1, 3, 9, 4, 2), (2, 5, 40, 8, 3), (4, 16, 130, 32, 4)])
def test_with_the_rows_own_normalisers_it_is_the_plain_score(G, P, n, d, seed):
    r = _rng(seed)
    Q, K = r.standard_normal((G * P, d)), r.standard_normal((n, d))
    scale = 1.0 / math.sqrt(d)
    lse = logsumexp(scale * (Q @ K.T), axis=1)
    np.testing.assert_allclose(O.cap_scores_given_lse(Q, K, scale, lse), O.cap_scores(Q, K, scale), rtol=1e-12)


@pytest.mark.parametrize("window", [0, 45])
def test_with_the_models_causal_normalisers_it_is_the_causal_score(window):
    """lse over the cached tokens AND the visible CaP keys, from torch on the full sequence."""
    r = _rng(5)
    G, P, n, d = 2, 8, 40, 16
    Q, K, K_cap = r.standard_normal((G * P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    scale = 0.25
    pos = torch.arange(n + P)
    allowed = pos[None, :] <= pos[:, None]
    if window:
        allowed &= pos[:, None] - pos[None, :] < window
    rows = allowed[n:].repeat(G, 1)                                    # row g*P + i -> CaP position i
    logits = torch.from_numpy(Q) @ torch.from_numpy(np.concatenate([K, K_cap])).T * scale
    lse = torch.logsumexp(logits.masked_fill(~rows, float("-inf")), dim=-1).numpy()
    got = O.cap_scores_given_lse(Q, K, scale, lse, P=P, window=window)
    np.testing.assert_allclose(got, O.cap_scores(Q, K, scale, K_cap, window=window), rtol=1e-12)


def test_brute_force_scalar_loops():
    r = _rng(6)
    GP, n, d, scale = 5, 7, 3, 0.7
    Q, K, lse = r.standard_normal((GP, d)), r.standard_normal((n, d)), r.standard_normal(GP) + 2.0
    u = [sum(math.exp(scale * sum(Q[q][c] * K[t][c] for c in range(d)) - lse[q]) for q in range(GP)) for t in range(n)]
    np.testing.assert_allclose(O.cap_scores_given_lse(Q, K, scale, lse), u, rtol=1e-12)


def test_compress_threads_the_normalisers_per_query_head():
    from paper_2410_01518_amd import synth
    cfg = synth.CCDConfig(name="t", B=2, L=2, Hq=4, Hkv=2, d=64, N=96, k=40, P=6, T=10, w=3, dtype="fp32", keys="normal", seed=8)
    inp = synth.make_inputs(cfg)
    scale = O.default_scale(cfg.d)
    Q64, K64 = inp["Q_cat"].astype(np.float64), inp["K"].astype(np.float64)
    lse = np.empty((cfg.B, cfg.L, cfg.Hq, cfg.P), dtype=np.float32)
    for b in range(cfg.B):
        for l in range(cfg.L):
            for hq in range(cfg.Hq):
                lse[b, l, hq] = logsumexp(scale * (Q64[b, l, hq] @ K64[b, l, hq // cfg.G].T), axis=1)
    kw = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w)
    a = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], **kw)
    b_ = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], lse=lse, **kw)
    fin = np.isfinite(a["scores"])
    np.testing.assert_allclose(b_["scores"][fin], a["scores"][fin], rtol=2e-6)
    np.testing.assert_array_equal(np.isposinf(a["scores"]), np.isposinf(b_["scores"]))
