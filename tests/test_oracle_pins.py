"""Pins for the CPU oracle: closed forms, invariants, a hand-worked example, library witnesses
(torch CPU ops used as a second, independent implementation) and brute force on tiny inputs.
None of these re-type the oracle's own formulas."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import synth


def _rng(seed):
    return np.random.default_rng(seed)


# ---------------------------------------------------------------- hand-worked example (tests/golden)

def _read_golden(path):
    out = {}
    with open(path) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            key, *vals = line.split()
            out[key] = [float(v) for v in vals]
    return out


def test_worked_example(golden_dir):
    g = _read_golden(os.path.join(golden_dir, "worked_example.txt"))
    a, b = np.array(g["a"]), np.array(g["b"])
    K = np.stack([np.log(a), np.log(b)], axis=1)            # [4, 2]
    Q = np.array([[1.0, 0.0], [0.0, 1.0]])
    u = O.cap_scores(Q, K, 1.0)
    np.testing.assert_allclose(u * 8, g["u_times8"], rtol=1e-13)
    ubar = O.pool(u, 3, O.POOL_MAX)
    np.testing.assert_allclose(ubar * 8, g["pooled_times8"], rtol=1e-13)
    nov = np.array(g["novelty"], dtype=np.float32)
    nuc = O.nuc_slots(nov, int(g["T"][0]))
    assert nuc.tolist() == [1]
    s = O.combine(ubar, nuc)
    assert s[1] == np.inf
    assert O.select(s, 2).tolist() == [int(v) for v in g["keep_k2"]]
    assert O.select(s, 3).tolist() == [int(v) for v in g["keep_k3"]]
    s0 = O.combine(O.pool(u, 1, O.POOL_MAX), O.nuc_slots(nov, 0))
    assert O.select(s0, 2).tolist() == [int(v) for v in g["keep_k2_nopool_T0"]]


# ---------------------------------------------------------------- closed forms

@pytest.mark.parametrize("GP,n,d", [(1, 7, 4), (12, 33, 8), (64, 100, 16)])
def test_uniform_when_keys_equal_or_queries_zero(GP, n, d):
    r = _rng(0)
    Q = r.standard_normal((GP, d))
    K = np.tile(r.standard_normal((1, d)), (n, 1))
    np.testing.assert_allclose(O.cap_scores(Q, K, 0.3), np.full(n, GP / n), rtol=1e-12)
    K2 = r.standard_normal((n, d))
    np.testing.assert_allclose(O.cap_scores(np.zeros((GP, d)), K2, 0.3), np.full(n, GP / n), rtol=1e-12)


def test_one_hot_key_closed_form():
    # one key with <q,k> = c, all others orthogonal to q: p_hot = e^{c s}/(e^{c s} + n - 1)
    n, d, scale, c = 50, 6, 0.25, 7.0
    q = np.zeros((1, d)); q[0, 2] = 1.0
    K = np.zeros((n, d)); K[17, 2] = c; K[:, 0] = 3.0        # the component along axis 0 is invisible to q
    u = O.cap_scores(q, K, scale)
    hot = math.exp(c * scale) / (math.exp(c * scale) + n - 1)
    assert abs(u[17] - hot) < 1e-14
    np.testing.assert_allclose(np.delete(u, 17), (1 - hot) / (n - 1), rtol=1e-12)


def test_scale_enters_the_logits():
    # two keys, logits (ln 3)*scale apart: doubling scale squares the odds
    q = np.array([[1.0]]); K = np.array([[0.0], [math.log(3.0)]])
    u1 = O.cap_scores(q, K, 1.0); u2 = O.cap_scores(q, K, 2.0)
    assert abs(u1[1] / u1[0] - 3.0) < 1e-12 and abs(u2[1] / u2[0] - 9.0) < 1e-12


# ---------------------------------------------------------------- invariants

@pytest.mark.parametrize("seed", range(4))
def test_score_invariants(seed):
    r = _rng(seed)
    GP, n, d = 24, 97, 16
    Q, K = r.standard_normal((GP, d)), r.standard_normal((n, d)) * 2
    u = O.cap_scores(Q, K, 0.25)
    assert abs(u.sum() - GP) < 1e-9 * GP and (u > 0).all()           # every query's probabilities sum to 1
    v = r.standard_normal((1, d)) * 5
    np.testing.assert_allclose(O.cap_scores(Q, K + v, 0.25), u, rtol=1e-9)   # softmax shift invariance
    perm = r.permutation(n)
    np.testing.assert_allclose(O.cap_scores(Q, K[perm], 0.25), u[perm], rtol=1e-12)  # token equivariance
    qperm = r.permutation(GP)
    np.testing.assert_allclose(O.cap_scores(Q[qperm], K, 0.25), u, rtol=1e-12)       # query order irrelevant
    # additivity over query rows (the GQA group is summed exactly like the CaP rows)
    np.testing.assert_allclose(O.cap_scores(Q[:10], K, 0.25) + O.cap_scores(Q[10:], K, 0.25), u, rtol=1e-12)


def test_large_logits_do_not_overflow():
    Q = np.array([[1.0, 0.0]]); K = np.array([[2000.0, 0.0], [1999.0, 0.0], [-3000.0, 1.0]])
    u = O.cap_scores(Q, K, 1.0)
    assert np.isfinite(u).all() and abs(u[0] / u[1] - math.e) < 1e-12 and u[2] == 0.0


# ---------------------------------------------------------------- library witnesses (torch CPU, fp64)

@pytest.mark.parametrize("seed", range(3))
def test_matches_torch_softmax_sum(seed):
    r = _rng(10 + seed)
    GP, n, d = 20, 300, 32
    Q, K = r.standard_normal((GP, d)), r.standard_normal((n, d))
    ref = torch.softmax(torch.from_numpy(Q) @ torch.from_numpy(K).T / math.sqrt(d), dim=-1).sum(0).numpy()
    np.testing.assert_allclose(O.cap_scores(Q, K, O.default_scale(d)), ref, rtol=1e-12)


@pytest.mark.parametrize("w", [1, 3, 7, 9])
def test_pool_matches_torch(w):
    u = _rng(w).random(61)
    t = torch.from_numpy(u)[None, None]
    mx = torch.nn.functional.max_pool1d(t, kernel_size=w, stride=1, padding=w // 2)[0, 0].numpy()
    av = torch.nn.functional.avg_pool1d(t, kernel_size=w, stride=1, padding=w // 2)[0, 0].numpy()
    np.testing.assert_array_equal(O.pool(u, w, O.POOL_MAX), mx)
    np.testing.assert_allclose(O.pool(u, w, O.POOL_AVG), av, rtol=1e-13)
    np.testing.assert_array_equal(O.pool(u, w, O.POOL_NONE), u)
    assert (O.pool(u, w, O.POOL_MAX) >= u).all()


def test_pool_window_longer_than_input():
    u = np.array([1.0, 5.0, 2.0])
    np.testing.assert_array_equal(O.pool(u, 7, O.POOL_MAX), [5.0, 5.0, 5.0])
    np.testing.assert_allclose(O.pool(u, 7, O.POOL_AVG), [8 / 7] * 3)


@pytest.mark.parametrize("seed", range(3))
def test_select_matches_torch_topk_on_distinct_scores(seed):
    s = _rng(20 + seed).permutation(500).astype(np.float32)       # all distinct
    for k in (1, 37, 250, 499, 500):
        ref = torch.topk(torch.from_numpy(s), k).indices.sort().values.numpy()
        got = O.select(s, k)
        np.testing.assert_array_equal(got, ref)
        assert got.dtype == np.int32


def test_compact_matches_index_select():
    r = _rng(5)
    X = r.integers(0, 65535, size=(40, 8)).astype(np.uint16)
    keep = np.sort(r.choice(40, 13, replace=False)).astype(np.int32)
    ref = torch.index_select(torch.from_numpy(X.view(np.int16)), 0, torch.from_numpy(keep).long()).numpy().view(np.uint16)
    np.testing.assert_array_equal(O.compact(X, keep), ref)


# ---------------------------------------------------------------- selection rules and ties

def test_append_puts_the_chunk_behind_the_cached_tokens():
    """Hand example: a pot of 5 slots with 2 cached tokens takes a chunk of 2; torch's slice assignment as witness;
    novelty of a token goes to every head; a chunk that does not fit is refused."""
    pot = np.arange(2 * 1 * 2 * 5 * 3, dtype=np.float32).reshape(2, 1, 2, 5, 3)
    chunk = -np.arange(2 * 1 * 2 * 2 * 3, dtype=np.float32).reshape(2, 1, 2, 2, 3) - 1.0
    got = O.append(pot, 2, chunk)
    assert got[1, 0, 1, 2].tolist() == chunk[1, 0, 1, 0].tolist() == [-19.0, -20.0, -21.0]      # first new row of the last unit
    assert got[1, 0, 1, 3].tolist() == [-22.0, -23.0, -24.0]
    assert np.array_equal(got[..., :2, :], pot[..., :2, :]) and np.array_equal(got[..., 4:, :], pot[..., 4:, :])
    want = torch.from_numpy(pot.copy())
    want[:, :, :, 2:4] = torch.from_numpy(chunk)
    assert np.array_equal(got, want.numpy())
    assert np.array_equal(pot, np.arange(60, dtype=np.float32).reshape(2, 1, 2, 5, 3))         # the input is not modified
    nov = np.zeros((2, 1, 2, 5), dtype=np.float32)
    got_n = O.append(nov, 3, np.array([[1.0, 2.0], [3.0, 4.0]], dtype=np.float32)[:, None, None, :])
    assert got_n[0, 0, 0].tolist() == got_n[0, 0, 1].tolist() == [0, 0, 0, 1, 2] and got_n[1, 0, 1].tolist() == [0, 0, 0, 3, 4]
    assert np.array_equal(O.append(nov[:, 0, 0], 0, np.ones((2, 5), np.float32)), np.ones((2, 5), np.float32))   # shared [B, n]
    with pytest.raises(ValueError):
        O.append(pot, 4, chunk)


def test_select_tie_break_and_order():
    s = np.array([1, 3, 3, 2, 3, 1, 3], dtype=np.float32)
    assert O.select(s, 1).tolist() == [1]
    assert O.select(s, 3).tolist() == [1, 2, 4]
    assert O.select(s, 5).tolist() == [1, 2, 3, 4, 6]
    assert O.select(s, 6).tolist() == [0, 1, 2, 3, 4, 6]
    assert O.select(s, 7).tolist() == list(range(7))


def test_select_special_values():
    s = np.array([np.nan, -np.inf, 0.0, -0.0, np.inf, 1e-45, -1.0], dtype=np.float32)
    assert O.select(s, 1).tolist() == [4]
    assert O.select(s, 2).tolist() == [4, 5]
    assert O.select(s, 4).tolist() == [2, 3, 4, 5]            # +0 and -0 tie; lower index first
    assert O.select(s, 6).tolist() == [0, 2, 3, 4, 5, 6]      # NaN ranks with -inf, index 0 < 1


def test_nuc_slots_rules():
    nov = np.array([0.5, 0.9, 0.9, -np.inf, np.nan, 0.1, 0.9], dtype=np.float32)
    assert O.nuc_slots(nov, 0).tolist() == []
    assert O.nuc_slots(nov, 2).tolist() == [1, 2]              # ties -> lower indices
    assert O.nuc_slots(nov, 4).tolist() == [0, 1, 2, 6]
    assert O.nuc_slots(nov, 7).tolist() == [0, 1, 2, 5, 6]     # NaN and -inf never take a slot


def test_combine_flushes_subnormals_and_sets_sentinel():
    ubar = np.array([1e-39, 2e-38, 0.25, 1e-300, 3.0])
    s = O.combine(ubar, np.array([2]))
    assert s.dtype == np.float32
    assert s[0] == 0 and s[3] == 0 and s[1] == np.float32(2e-38) and s[2] == np.inf and s[4] == 3.0


# ---------------------------------------------------------------- brute force over the whole unit (pure Python)

def _brute_unit(Q, K, nov, T, k, scale, w, mode):
    GP, d = len(Q), len(Q[0]); n = len(K)
    u = [0.0] * n
    for q in Q:
        logit = [scale * sum(q[c] * K[t][c] for c in range(d)) for t in range(n)]
        top = max(logit)
        e = [math.exp(x - top) for x in logit]
        z = sum(e)
        for t in range(n):
            u[t] += e[t] / z
    r = w // 2
    if mode == O.POOL_MAX and w > 1:
        ub = [max(u[max(0, t - r):t + r + 1]) for t in range(n)]
    elif mode == O.POOL_AVG and w > 1:
        ub = [sum(u[max(0, t - r):t + r + 1]) / w for t in range(n)]
    else:
        ub = list(u)
    cand = [t for t in range(n) if not math.isnan(nov[t]) and nov[t] > -math.inf]
    nuc = sorted(cand, key=lambda t: (-nov[t], t))[:T]
    score = [float(np.float32(x)) for x in ub]
    for t in nuc:
        score[t] = math.inf
    ranked = sorted(range(n), key=lambda t: (-score[t], t))       # full stable sort of all tokens
    return score, sorted(ranked[:k])


@pytest.mark.parametrize("seed,mode,w,T", [(0, O.POOL_MAX, 7, 5), (1, O.POOL_AVG, 3, 0), (2, O.POOL_NONE, 1, 12),
                                           (3, O.POOL_MAX, 5, 12), (4, O.POOL_MAX, 7, 3)])
def test_unit_matches_brute_force(seed, mode, w, T):
    r = _rng(100 + seed)
    G, P, d, n, k = 2, 3, 8, 40, 12
    # few distinct key rows -> many exactly tied scores
    base = r.standard_normal((5, d)).astype(np.float32)
    K = base[r.integers(0, 5, n)]
    Q = r.standard_normal((G * P, d)).astype(np.float32)
    nov = np.round(r.random(n), 1).astype(np.float32)            # tied novelty too
    s = O.score_unit(Q, K, nov, T=T, scale=0.5, pool_w=w, pool_mode=mode)
    keep = O.select(s, k)
    bs, bkeep = _brute_unit(Q.astype(np.float64).tolist(), K.astype(np.float64).tolist(),
                            [float(x) for x in nov], T, k, 0.5, w, mode)
    assert keep.tolist() == bkeep
    fin = np.isfinite(s)
    assert (np.isinf(s) == np.isinf(np.array(bs))).all()
    np.testing.assert_allclose(s[fin], np.array(bs)[fin], rtol=2e-7)


# ---------------------------------------------------------------- whole-call properties (paper Sec. 3.2-3.3)

def _small_cfg(**kw):
    base = dict(name="t", B=2, L=2, Hq=4, Hkv=2, d=16, N=96, k=40, P=5, T=16, w=3, dtype="bf16", keys="normal", seed=7)
    base.update(kw)
    return synth.CCDConfig(**base)


def _run(cfg, inp, **kw):
    args = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=O.POOL_MAX)
    args.update(kw)
    return O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], **args)


def test_compress_properties():
    cfg = _small_cfg()
    inp = synth.make_inputs(cfg)
    out = _run(cfg, inp)
    keep = out["keep_idx"]
    assert keep.shape == (cfg.B, cfg.L, cfg.Hkv, cfg.k)
    assert (np.diff(keep, axis=-1) > 0).all() and keep.min() >= 0 and keep.max() < cfg.N   # order kept, exactly k
    for b in range(cfg.B):
        nuc = O.nuc_slots(inp["novelty"][b], cfg.T)
        assert len(nuc) == cfg.T
        for l, h in itertools.product(range(cfg.L), range(cfg.Hkv)):
            assert set(nuc.tolist()) <= set(keep[b, l, h].tolist())                        # NuC tokens always survive
            np.testing.assert_array_equal(out["K"][b, l, h], inp["K"][b, l, h][keep[b, l, h]])  # bit copies
            np.testing.assert_array_equal(out["V"][b, l, h], inp["V"][b, l, h][keep[b, l, h]])
            assert np.isinf(out["scores"][b, l, h]).sum() == cfg.T
    # heads are selected independently (Sec. 3.3.1): with random data two heads differ
    assert (keep[0, 0, 0] != keep[0, 0, 1]).any()


def test_nuc_only_is_identical_across_heads_and_cap_only_is_plain_topk():
    cfg = _small_cfg()
    inp = synth.make_inputs(cfg)
    out = _run(cfg, inp, T=cfg.k)                                 # alpha = 100 %: every head keeps the same tokens
    for b in range(cfg.B):
        ref = out["keep_idx"][b, 0, 0]
        assert (out["keep_idx"][b] == ref).all()
        np.testing.assert_array_equal(ref, O.nuc_slots(inp["novelty"][b], cfg.k))
    out0 = _run(cfg, inp, T=0, pool_w=1)                          # alpha = 0: per-head top-k of the CaP score
    G = cfg.G
    for b, l, h in itertools.product(range(cfg.B), range(cfg.L), range(cfg.Hkv)):
        Qu = O.to_f64(inp["Q_cat"][b, l, h * G:(h + 1) * G].reshape(G * cfg.P, cfg.d))
        u = torch.softmax(torch.from_numpy(Qu) @ torch.from_numpy(O.to_f64(inp["K"][b, l, h])).T / math.sqrt(cfg.d), -1).sum(0)
        ref = torch.topk(u.float(), cfg.k).indices.sort().values.numpy()
        np.testing.assert_array_equal(out0["keep_idx"][b, l, h], ref)


def test_gqa_group_uses_its_own_query_heads():
    # head h must be scored by query heads h*G .. h*G+G-1 only: zeroing the other heads' queries changes nothing
    cfg = _small_cfg(B=1, L=1)
    inp = synth.make_inputs(cfg)
    out = _run(cfg, inp)
    Q2 = inp["Q_cat"].copy(); Q2[:, :, cfg.G:] = 0              # wipe the queries of KV head 1
    out2 = O.compress(Q2, inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    np.testing.assert_array_equal(out["scores"][0, 0, 0], out2["scores"][0, 0, 0])
    assert (out["scores"][0, 0, 1] != out2["scores"][0, 0, 1]).any()


def test_per_head_novelty_is_carried_and_compacted():
    cfg = _small_cfg(B=1)
    inp = synth.make_inputs(cfg, per_head_novelty=True)
    out = _run(cfg, inp)
    for l, h in itertools.product(range(cfg.L), range(cfg.Hkv)):
        keep = out["keep_idx"][0, l, h]
        np.testing.assert_array_equal(out["novelty"][0, l, h], inp["novelty"][0, l, h][keep])
        assert set(O.nuc_slots(inp["novelty"][0, l, h], cfg.T).tolist()) <= set(keep.tolist())


def test_partial_pot_scores_only_valid_tokens():
    cfg = _small_cfg(B=1, L=1)
    inp = synth.make_inputs(cfg)
    n = 70
    out = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=30, T=10, pool_w=3, n_valid=n)
    assert out["scores"].shape[-1] == n and out["keep_idx"].max() < n
    K2 = {**inp}; K2["K"] = inp["K"].copy(); K2["K"][..., n:, :] = 0x7FC0      # NaN beyond n_valid must not matter
    out2 = O.compress(K2["Q_cat"], K2["K"], K2["V"], K2["novelty"], k=30, T=10, pool_w=3, n_valid=n)
    np.testing.assert_array_equal(out["keep_idx"], out2["keep_idx"])


def test_bf16_inputs_are_read_exactly():
    bits = np.array([0x3F80, 0xC000, 0x3DCC, 0x0001, 0x7F7F], dtype=np.uint16)
    ref = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).double().numpy()
    np.testing.assert_array_equal(O.to_f64(bits), ref)
    x = _rng(3).standard_normal(1000).astype(np.float32)
    np.testing.assert_array_equal(synth.f32_to_bf16_bits(x).view(np.int16),
                                  torch.from_numpy(x).bfloat16().view(torch.int16).numpy())


# ---------------------------------------------------------------- the pins have teeth: planted mistakes are caught

def _suite(mod):
    """A condensed run of the pins above against module-like object `mod`; returns True if all hold."""
    try:
        a, b = np.array([1.0, 2, 3, 2]), np.array([4.0, 1, 1, 2])
        K = np.stack([np.log(a), np.log(b)], axis=1); Q = np.eye(2)
        u = mod.cap_scores(Q, K, 1.0)
        if not np.allclose(u * 8, [5, 3, 4, 4], rtol=1e-12):
            return False
        r = _rng(0); Qr, Kr = r.standard_normal((6, 4)), r.standard_normal((9, 4))
        ref = torch.softmax(torch.from_numpy(Qr) @ torch.from_numpy(Kr).T * 0.5, -1).sum(0).numpy()
        if not np.allclose(mod.cap_scores(Qr, Kr, 0.5), ref, rtol=1e-12):
            return False
        if mod.select(np.array([1, 3, 3, 2, 3], dtype=np.float32), 2).tolist() != [1, 2]:
            return False
        if not np.array_equal(mod.pool(np.array([1.0, 5, 2, 0, 0, 0, 9]), 3, O.POOL_MAX), [5, 5, 5, 2, 0, 9, 9]):
            return False
        if mod.nuc_slots(np.array([0.1, 0.9, 0.9], dtype=np.float32), 1).tolist() != [1]:
            return False
        s = mod.score_unit(np.eye(2), K, np.array([0.1, 0.9, 0.2, 0.3], dtype=np.float32), T=1, scale=1.0,
                           pool_w=3, pool_mode=O.POOL_MAX)
        return bool(np.isinf(s).sum() == 1 and s[1] == np.inf and np.allclose(s[[0, 2, 3]] * 8, [5, 4, 4]))
    except Exception:
        return False


class _Mutant:
    def __init__(self, **over):
        self.__dict__.update({n: getattr(O, n) for n in ("cap_scores", "select", "pool", "nuc_slots", "combine")})
        self.__dict__.update(over)

    def score_unit(self, Q, K, nov, *, T, scale, pool_w, pool_mode):
        u = self.cap_scores(O.to_f64(Q), O.to_f64(K), scale)
        return self.combine(self.pool(u, pool_w, pool_mode), self.nuc_slots(nov, T))


def _softmax_wrong_axis(Q, K, scale):
    S = scale * (Q @ K.T); E = np.exp(S - S.max(0, keepdims=True)); return (E / E.sum(0, keepdims=True)).sum(0)


def _no_scale(Q, K, scale):
    return O.cap_scores(Q, K, 1.0)


def _mean_over_queries(Q, K, scale):
    return O.cap_scores(Q, K, scale) / Q.shape[0]


def _highest_index_ties(s, k):
    s = np.asarray(s, dtype=np.float64); order = np.lexsort((-np.arange(len(s)), -s)); return np.sort(order[:k])


def _pool_off_by_one(u, w, mode):
    return np.array([u[max(0, t - w // 2):t + w // 2].max() for t in range(len(u))]) if w > 1 else u.copy()


def _nuc_smallest(nov, T):
    return np.sort(np.argsort(nov, kind="stable")[:T])


def _combine_no_sentinel(ubar, nuc):
    return ubar.astype(np.float32)


def test_planted_mistakes_are_caught():
    assert _suite(_Mutant())
    for name, over in [("softmax axis", dict(cap_scores=_softmax_wrong_axis)), ("dropped scale", dict(cap_scores=_no_scale)),
                       ("mean not sum", dict(cap_scores=_mean_over_queries)), ("tie-break", dict(select=_highest_index_ties)),
                       ("pool window", dict(pool=_pool_off_by_one)), ("nuc sign", dict(nuc_slots=_nuc_smallest)),
                       ("no sentinel", dict(combine=_combine_no_sentinel))]:
        assert not _suite(_Mutant(**over)), f"pins did not catch: {name}"
