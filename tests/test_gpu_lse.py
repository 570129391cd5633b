"""GPU parity of the score from handed-in log-sum-exps (ccd_score_lse / ccd_compress_lse) through the C ABI."""
import math

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="t", B=1, L=2, Hq=8, Hkv=2, d=128, N=700, k=300, P=9, T=100, w=7, dtype="bf16", keys="normal", seed=91)
    base.update(kw)
    return synth.CCDConfig(**base)


def _row_lse(cfg, inp, K_cap=None, window=0):
    """fp32 [B, L, Hq, P]: natural-log-sum-exp of every CaP query row over the keys it sees (scipy, fp64 logits)."""
    Q, K = O.to_f64(inp["Q_cat"]), O.to_f64(inp["K"])
    Kc = None if K_cap is None else O.to_f64(K_cap)
    scale = O.default_scale(cfg.d)
    out = np.empty((cfg.B, cfg.L, cfg.Hq, cfg.P), dtype=np.float32)
    n = cfg.N
    for b in range(cfg.B):
        for l in range(cfg.L):
            for hq in range(cfg.Hq):
                h = hq // cfg.G
                S = scale * (Q[b, l, hq] @ K[b, l, h].T)                      # [P, n]
                if window:
                    first = n + np.arange(cfg.P) + 1 - window
                    S = np.where(np.arange(n)[None, :] >= first[:, None], S, -np.inf)
                if Kc is not None:
                    C = scale * (Q[b, l, hq] @ Kc[b, l, h].T)                 # [P, P]
                    C = np.where(np.arange(cfg.P)[None, :] <= np.arange(cfg.P)[:, None], C, -np.inf)
                    S = np.concatenate([S, C], axis=1)
                out[b, l, hq] = logsumexp(S, axis=1)
    return out


def _score_lse(cfg, inp, lse, window=0, path=0):
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, window=window, score_path=path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_score_lse(shape, dev["Q_cat"], dev["K"], torch.from_numpy(lse).cuda(), dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    return gu.to_host(scores)


LSE_CASES = [
    dict(),
    dict(P=1, Hq=2, Hkv=2, d=64, N=513, k=100, T=0, w=1),
    dict(P=40, Hq=16, Hkv=2, d=64, N=515, k=200),                                  # G*P = 320: two sweeps
    dict(B=2, L=1, N=1111, k=10, T=3, w=5, keys="zipf"),
    dict(dtype="fp32", d=64, Hq=4, Hkv=4, N=512, k=256, P=16, T=128, w=1),
    dict(dtype="fp32", N=300, k=120, T=30, P=33, w=3),
]


@pytest.mark.parametrize("path", [ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT])
@pytest.mark.parametrize("case", range(len(LSE_CASES)))
@pytest.mark.parametrize("reading", ["cache_only", "causal", "causal_window"])
def test_score_lse_matches_oracle(case, reading, path):
    cfg = _cfg(**LSE_CASES[case])
    if cfg.dtype == "fp32":
        if path == ip.CCD_PATH_MFMA_SLICES:
            path = ip.CCD_PATH_VALU                        # no slice kernels for fp32: the vector ALUs instead
        elif cfg.d != 64 or reading == "causal_window":
            pytest.skip("fp32 caches on the matrix cores: head dimension 64, no window")
    print(f"score_lse case={case} reading={reading} path={path} {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg) if reading != "cache_only" else None
    window = cfg.N - 30 if reading == "causal_window" else 0
    if window and window < cfg.P:
        pytest.skip("window shorter than the CaP")
    lse = _row_lse(cfg, inp, K_cap, window)
    got = _score_lse(cfg, inp, lse, window, path=path)
    kw = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], lse=lse, window=window, **kw)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)
    # the same scores as the self-normalising form of that reading (up to the rounding of lse to fp32)
    self_norm = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], K_cap=K_cap, window=window, **kw)
    fin = np.isfinite(self_norm["scores"])
    np.testing.assert_allclose(ref["scores"][fin], self_norm["scores"][fin], rtol=2e-5, atol=1e-30)


def test_score_lse_on_the_vector_alu_path_for_bf16():
    cfg = _cfg(P=17, N=400, k=150)
    inp = synth.make_inputs(cfg)
    lse = _row_lse(cfg, inp)
    got = _score_lse(cfg, inp, lse, path=1)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, lse=lse)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


def test_shifted_normalisers_scale_every_probability():
    """lse + log 2 halves every finite score: nothing in the call depends on the rows summing to one."""
    cfg = _cfg(N=640, k=200, P=12, T=0, w=1)
    inp = synth.make_inputs(cfg)
    lse = _row_lse(cfg, inp)
    a = _score_lse(cfg, inp, lse)
    b = _score_lse(cfg, inp, (lse.astype(np.float64) + math.log(2.0)).astype(np.float32))
    np.testing.assert_allclose(b, a / 2, rtol=2e-5, atol=1e-30)


@pytest.mark.parametrize("dtype,d,N", [("bf16", 128, 1024), ("fp32", 64, 300), ("bf16", 64, 17000)])
def test_compress_lse_matches_oracle(dtype, d, N):
    cfg = _cfg(dtype=dtype, d=d, N=N, k=N // 2, T=N // 4, P=20, L=1 if N > 10000 else 2)
    print(f"compress_lse {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg)
    lse = _row_lse(cfg, inp, K_cap)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_compress_lse(shape, dev["Q_cat"], dev["K"], dev["V"], torch.from_numpy(lse).cuda(), dev["novelty"], keep, ws,
                               scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, lse=lse)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    idx = kh.astype(np.int64)[..., None]
    np.testing.assert_array_equal(gu.to_host(dev["K"])[..., :cfg.k, :], np.take_along_axis(inp["K"], idx, axis=3))
    np.testing.assert_array_equal(gu.to_host(dev["V"])[..., :cfg.k, :], np.take_along_axis(inp["V"], idx, axis=3))


def test_compress_rope_with_normalisers():
    cfg = _cfg(P=16, N=768, k=384, T=192)
    inp = synth.make_inputs(cfg)
    K_score = synth.make_inputs(cfg, seed=77)["K"]
    cos, sin = synth.rope_tables(cfg.k, cfg.d)
    lse = _row_lse(cfg, dict(inp, K=K_score))
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    K_rot = gu.to_dev(K_score)
    assert ip.ccd_compress_rope(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, gu.to_dev(cos), gu.to_dev(sin),
                                K_rot, ws, scores=scores, K_score=K_rot, lse=torch.from_numpy(lse).cuda()) == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_score=K_score, lse=lse,
                     rope_cos=cos, rope_sin=sin)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
