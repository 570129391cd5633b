"""GPU parity of the causal reading of Eq. 2 (the CaP tokens' own keys in the softmax) through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="t", B=1, L=2, Hq=8, Hkv=2, d=128, N=700, k=300, P=9, T=100, w=7, dtype="bf16", keys="normal", seed=61)
    base.update(kw)
    return synth.CCDConfig(**base)


def _score(cfg, gain=1.0, path=0, K_cap=None):
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg, gain=gain) if K_cap is None else K_cap
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, score_path=path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_score_kcat(shape, dev["Q_cat"], dev["K"], gu.to_dev(K_cap), dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    return inp, K_cap, gu.to_host(scores)


# P: one CaP token, a ragged block, exactly one and two key tiles, one past them, more than two tiles;
# G * P: below one wave's share, one sweep, more than one sweep of 256 query rows
KCAT_CASES = [
    dict(P=1, Hq=2, Hkv=2),
    dict(P=9),
    dict(P=32, Hq=4, Hkv=2),
    dict(P=33, d=64),
    dict(P=64, Hq=8, Hkv=2, N=1100, k=500),
    dict(P=70, Hq=2, Hkv=1, N=333, k=100, T=50),
    dict(P=40, Hq=16, Hkv=2, d=64, N=515, k=200),
    dict(P=5, dtype="fp32", d=64, N=300, k=120, T=30),
    dict(P=37, dtype="fp32", Hq=4, Hkv=2, N=260, k=100, T=10, w=1),
]


MFMA_PATHS = [ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT]     # a workgroup per token slice / per unit


@pytest.mark.parametrize("path", [ip.CCD_PATH_AUTO] + MFMA_PATHS)
@pytest.mark.parametrize("case", KCAT_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_score_kcat_matches_oracle(case, path):
    cfg = _cfg(**case)
    if cfg.dtype == "fp32" and path != ip.CCD_PATH_AUTO:
        pytest.skip("fp32 caches have one path")
    print(f"score_kcat {cfg} path={path}", flush=True)
    inp, K_cap, got = _score(cfg, path=path)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)
    # the CaP keys matter in these cases: without them the scores would be out of tolerance
    plain = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    fin = np.isfinite(ref["scores"])
    assert np.median(plain["scores"][fin] / ref["scores"][fin]) > 1.0 + 0.25 * ((cfg.P + 1) / 2) / (cfg.N + cfg.P)


@pytest.mark.parametrize("path", MFMA_PATHS)
@pytest.mark.parametrize("gain", [0.0, 6.0])
def test_score_kcat_weak_and_dominant_cap_keys(gain, path):
    """gain 0: every CaP key has logit 0; gain 6: a few CaP keys take nearly all of the mass of their queries."""
    cfg = _cfg(P=24, N=640, k=200)
    print(f"score_kcat gain={gain} path={path} {cfg}", flush=True)
    inp, K_cap, got = _score(cfg, gain=gain, path=path)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


def test_score_kcat_on_the_vector_alu_path_for_bf16():
    cfg = _cfg(P=17, N=400, k=150)
    print(f"score_kcat valu path {cfg}", flush=True)
    inp, K_cap, got = _score(cfg, path=ip.CCD_PATH_VALU)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


def test_far_cap_keys_leave_the_plain_scores():
    """CaP keys far from every query (positive queries, large negative keys) take no mass: ccd_score's result."""
    cfg = _cfg(P=12, N=512, k=200)
    inp = synth.make_inputs(cfg)
    q = np.abs(synth.bf16_bits_to_f32(inp["Q_cat"]))
    inp["Q_cat"] = synth.f32_to_bf16_bits(q)
    K_cap = synth.f32_to_bf16_bits(np.full((cfg.B, cfg.L, cfg.Hkv, cfg.P, cfg.d), -100.0, np.float32))
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    a = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], a, ws) == ip.CCD_OK
    assert ip.ccd_score_kcat(shape, dev["Q_cat"], dev["K"], gu.to_dev(K_cap), dev["novelty"], b, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gu.to_host(a), gu.to_host(b))


@pytest.mark.parametrize("dtype,d,N", [("bf16", 128, 1024), ("fp32", 64, 300), ("bf16", 64, 17000)])
def test_compress_kcat_matches_oracle(dtype, d, N):
    cfg = _cfg(dtype=dtype, d=d, N=N, k=N // 2, T=N // 4, P=20, L=1 if N > 10000 else 2)
    print(f"compress_kcat {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_compress_kcat(shape, dev["Q_cat"], dev["K"], dev["V"], gu.to_dev(K_cap), dev["novelty"], keep, ws,
                                scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    Kh, Vh = gu.to_host(dev["K"]), gu.to_host(dev["V"])
    for b in range(cfg.B):
        for l in range(cfg.L):
            for h in range(cfg.Hkv):
                np.testing.assert_array_equal(Kh[b, l, h, :cfg.k], O.compact(inp["K"][b, l, h], kh[b, l, h]))
                np.testing.assert_array_equal(Vh[b, l, h, :cfg.k], O.compact(inp["V"][b, l, h], kh[b, l, h]))


def test_compress_rope_with_cap_keys():
    """The full deployment form: scores on the embedded cache and the embedded CaP keys, CR-RoPE of the kept keys."""
    cfg = _cfg(P=16, N=768, k=384, T=192)
    print(f"compress_rope + K_cap {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg)
    K_score = synth.make_inputs(cfg, seed=77)["K"]
    cos, sin = synth.rope_tables(cfg.k, cfg.d)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    K_rot = gu.to_dev(K_score)                       # the attention cache: read for the scores, then rewritten
    assert ip.ccd_compress_rope(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, gu.to_dev(cos), gu.to_dev(sin),
                                K_rot, ws, scores=scores, K_score=K_rot, K_cap=gu.to_dev(K_cap)) == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap,
                     K_score=K_score, rope_cos=cos, rope_sin=sin)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    rot = gu.to_host(K_rot)
    for l in range(cfg.L):
        for h in range(cfg.Hkv):
            expect = O.cr_rope(O.compact(inp["K"][0, l, h], kh[0, l, h]), cos, sin)
            assert np.mean(rot[0, l, h, :cfg.k] == expect) > 0.999
