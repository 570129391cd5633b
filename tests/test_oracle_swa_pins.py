"""Pins for the oracle's sliding-window reading of the CaP attention rows: a hand-worked example, a closed form, a torch
witness built from the full-sequence band mask, scalar brute force and the limit of a window that hides nothing."""
import math

import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O


def _rng(seed):
    return np.random.default_rng(seed)


def test_hand_worked_example():
    """n = 4 cached tokens, 2 CaP tokens at positions 4 and 5, window 5: position 4 sees 0..4, position 5 sees 1..5.
    Query 0 has weights a = (1,2,1,4) on the context: row sum 8.  Query 1 has b = (3,1,2,2) but token 0 is out of
    its window: row sum 5."""
    a, b = np.array([1.0, 2, 1, 4]), np.array([3.0, 1, 2, 2])
    K = np.stack([np.log(a), np.log(b)], axis=1)
    Q = np.array([[1.0, 0.0], [0.0, 1.0]])
    u = O.cap_scores(Q, K, 1.0, P=2, window=5)
    np.testing.assert_allclose(u, [1 / 8, 2 / 8 + 1 / 5, 1 / 8 + 2 / 5, 4 / 8 + 2 / 5], rtol=1e-13)
    # a window one wider hides nothing, one narrower hides token 0 from query 0 as well and token 1 from query 1
    np.testing.assert_allclose(O.cap_scores(Q, K, 1.0, P=2, window=6), (a + b) / 8, rtol=1e-13)
    np.testing.assert_allclose(O.cap_scores(Q, K, 1.0, P=2, window=4), [0, 2 / 7, 1 / 7 + 2 / 4, 4 / 7 + 2 / 4], rtol=1e-13)
    # with the CaP keys in the softmax: query 0 also sees CaP key 0 (weight 8), query 1 CaP keys 0, 1 (weights 3, 2)
    K_cap = np.array([[math.log(8), math.log(3)], [math.log(100), math.log(2)]])
    u = O.cap_scores(Q, K, 1.0, K_cap, window=5)
    np.testing.assert_allclose(u, [1 / 16, 2 / 16 + 1 / 10, 1 / 16 + 2 / 10, 4 / 16 + 2 / 10], rtol=1e-13)


@pytest.mark.parametrize("G,P,n,W", [(1, 4, 20, 20), (3, 8, 50, 52), (2, 16, 100, 40), (2, 5, 30, 5)])
def test_zero_queries_spread_evenly_over_the_window(G, P, n, W):
    r = _rng(1)
    K = r.standard_normal((n, 8))
    u = O.cap_scores(np.zeros((G * P, 8)), K, 0.3, P=P, window=W)
    expect = np.zeros(n)
    for i in range(P):
        first = max(0, n + i + 1 - W)
        if first < n:
            expect[first:] += G / (n - first)
    np.testing.assert_allclose(u, expect, rtol=1e-13)


@pytest.mark.parametrize("with_cap", [False, True])
@pytest.mark.parametrize("G,P,n,d,W,seed", [(1, 3, 9, 4, 9, 2), (2, 5, 40, 8, 41, 3), (4, 16, 130, 32, 64, 4), (2, 6, 30, 8, 100, 5)])
def test_torch_witness_band_mask_of_the_full_sequence(with_cap, G, P, n, d, W, seed):
    """Causal sliding-window mask of the whole sequence [context, CaP]: entry (r, c) allowed iff c <= r < c + W.
    The CaP rows of it, restricted to the keys that exist in the variant (context only, or context and CaP)."""
    r = _rng(seed)
    Q, K, K_cap = r.standard_normal((G, P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    scale = 1.0 / math.sqrt(d)
    pos = torch.arange(n + P)
    band = (pos[None, :] <= pos[:, None]) & (pos[:, None] - pos[None, :] < W)
    rows = band[n:]
    keys = np.concatenate([K, K_cap], axis=0) if with_cap else K
    rows = rows if with_cap else rows[:, :n]
    total = torch.zeros(n, dtype=torch.float64)
    for g in range(G):
        logits = torch.from_numpy(Q[g]) @ torch.from_numpy(keys).T * scale
        attn = torch.softmax(logits.masked_fill(~rows, float("-inf")), dim=-1)
        total += attn[:, :n].sum(dim=0)
    u = O.cap_scores(Q.reshape(G * P, d), K, scale, K_cap if with_cap else None, P=P, window=W)
    np.testing.assert_allclose(u, total.numpy(), rtol=1e-12, atol=1e-300)


def test_brute_force_scalar_loops():
    r = _rng(6)
    G, P, n, d, scale, W = 2, 3, 7, 3, 0.9, 6
    Q, K, K_cap = r.standard_normal((G * P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    for with_cap in (False, True):
        u = [0.0] * n
        for g in range(G):
            for i in range(P):
                q, p_q = Q[g * P + i], n + i
                w_ctx = [math.exp(scale * sum(q[c] * K[t][c] for c in range(d))) if p_q - t < W else 0.0 for t in range(n)]
                w_cap = [math.exp(scale * sum(q[c] * K_cap[j][c] for c in range(d))) for j in range(i + 1)] if with_cap else []
                z = sum(w_ctx) + sum(w_cap)
                for t in range(n):
                    u[t] += w_ctx[t] / z
        got = O.cap_scores(Q, K, scale, K_cap if with_cap else None, P=P, window=W)
        np.testing.assert_allclose(got, u, rtol=1e-12)


def test_a_window_that_hides_nothing_changes_nothing():
    r = _rng(7)
    G, P, n, d = 2, 8, 60, 16
    Q, K, K_cap = r.standard_normal((G * P, d)), r.standard_normal((n, d)), r.standard_normal((P, d))
    np.testing.assert_array_equal(O.cap_scores(Q, K, 0.25), O.cap_scores(Q, K, 0.25, P=P, window=n + P))
    np.testing.assert_array_equal(O.cap_scores(Q, K, 0.25, K_cap), O.cap_scores(Q, K, 0.25, K_cap, window=n + P))
    hidden = O.cap_scores(Q, K, 0.25, P=P, window=n)      # CaP token i no longer sees tokens 0 .. i
    assert hidden[0] == 0.0 and np.all(hidden[P:] > O.cap_scores(Q, K, 0.25)[P:])


def test_compress_threads_the_window():
    from paper_2410_01518_amd import synth
    cfg = synth.CCDConfig(name="t", B=1, L=1, Hq=4, Hkv=2, d=64, N=96, k=40, P=6, T=10, w=1, dtype="fp32", keys="normal", seed=8)
    inp = synth.make_inputs(cfg)
    kw = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w)
    a = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], window=cfg.N, **kw)
    for h in range(cfg.Hkv):
        Qu = O.to_f64(inp["Q_cat"][0, 0, h * cfg.G:(h + 1) * cfg.G].reshape(cfg.G * cfg.P, cfg.d))
        u = O.cap_scores(Qu, O.to_f64(inp["K"][0, 0, h]), O.default_scale(cfg.d), P=cfg.P, window=cfg.N)
        fin = np.isfinite(a["scores"][0, 0, h])
        np.testing.assert_allclose(a["scores"][0, 0, h][fin], u[fin].astype(np.float32), rtol=1e-6)
        assert a["scores"][0, 0, h][0] in (0.0, np.inf)       # token 0 is outside every window
