"""GPU parity of the sliding-window reading of the CaP attention rows (shape.window) through the C ABI."""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="t", B=1, L=2, Hq=8, Hkv=2, d=128, N=700, k=300, P=9, T=100, w=7, dtype="bf16", keys="normal", seed=81)
    base.update(kw)
    return synth.CCDConfig(**base)


def _score(cfg, window, path=0, with_cap=False, inp=None):
    inp = synth.make_inputs(cfg) if inp is None else inp
    K_cap = synth.cap_keys(cfg) if with_cap else None
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, window=window, score_path=path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    if with_cap:
        rc = ip.ccd_score_kcat(shape, dev["Q_cat"], dev["K"], gu.to_dev(K_cap), dev["novelty"], scores, ws)
    else:
        rc = ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws)
    assert rc == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap,
                     window=window)
    return gu.to_host(scores), ref


# window relative to the pot: hides one token from the last CaP token only; window == pot (CaP token i loses tokens
# 0..i); a few tiles hidden; hidden part reaching into the second token slice; everything but a few tokens hidden
SWA_CASES = [
    dict(cfg=dict(), window=lambda c: c.N + c.P - 1),
    dict(cfg=dict(), window=lambda c: c.N),
    dict(cfg=dict(P=40, Hq=16, Hkv=2, d=64, N=515, k=200), window=lambda c: c.N),            # G*P = 320: two sweeps
    dict(cfg=dict(N=1100, k=500, P=33), window=lambda c: c.N - 100),
    dict(cfg=dict(B=2, L=4, Hq=4, Hkv=4, N=900, k=300, P=16, T=50), window=lambda c: c.N - 300),  # many units: short slices
    dict(cfg=dict(N=333, k=100, T=50, P=20), window=lambda c: c.P + 10),                      # nearly everything hidden
    dict(cfg=dict(N=333, k=100, T=50, P=20), window=lambda c: c.P),                           # the last CaP token sees nothing
    dict(cfg=dict(L=1, N=8192, k=3000, T=500, P=33), window=lambda c: 4096),                  # half of the pot behind the window
    dict(cfg=dict(L=1, Hq=4, Hkv=2, N=5000, k=1000, T=100, P=70), window=lambda c: 1000),     # most of it, and P > 64
    dict(cfg=dict(dtype="fp32", d=64, N=300, k=120, T=30, P=5), window=lambda c: c.N),
    dict(cfg=dict(dtype="fp32", Hq=4, Hkv=2, N=260, k=100, T=10, P=37, w=1), window=lambda c: c.N - 50),
]


@pytest.mark.parametrize("path", [ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT])
@pytest.mark.parametrize("with_cap", [False, True])
@pytest.mark.parametrize("case", range(len(SWA_CASES)))
def test_scores_under_a_sliding_window(case, with_cap, path):
    cfg = _cfg(**SWA_CASES[case]["cfg"])
    window = SWA_CASES[case]["window"](cfg)
    if cfg.dtype == "fp32":
        if path != ip.CCD_PATH_MFMA_SLICES:
            pytest.skip("fp32 caches have one path")
        path = ip.CCD_PATH_AUTO
    print(f"swa case={case} window={window} with_cap={with_cap} path={path} {cfg}", flush=True)
    got, ref = _score(cfg, window, with_cap=with_cap, path=path)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


def test_window_on_the_vector_alu_path_for_bf16():
    cfg = _cfg(N=400, k=150, P=17)
    print(f"swa valu {cfg}", flush=True)
    got, ref = _score(cfg, cfg.N - 40, path=1, with_cap=True)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


def test_a_window_that_hides_nothing_gives_the_same_bits():
    cfg = _cfg(N=640, k=200, P=12)
    inp = synth.make_inputs(cfg)
    a, _ = _score(cfg, 0, inp=inp)
    b, _ = _score(cfg, cfg.N + cfg.P, inp=inp)
    c, _ = _score(cfg, 1 << 30, inp=inp)
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(a, c)


def test_the_first_token_behind_the_window_scores_zero():
    """window == pot: token 0 is outside every CaP token's window - an attention sink there gets no score."""
    cfg = _cfg(N=512, k=200, P=8, T=0, w=1)
    inp = synth.make_inputs(cfg)
    K = synth.bf16_bits_to_f32(inp["K"])
    Q = synth.bf16_bits_to_f32(inp["Q_cat"])
    for h in range(cfg.Hkv):                         # token 0 of every unit points along the mean query of its group
        K[:, :, h, 0, :] = 3.0 * Q[:, :, h * cfg.G:(h + 1) * cfg.G].mean(axis=(2, 3))
    inp["K"] = synth.f32_to_bf16_bits(K)
    got, ref = _score(cfg, cfg.N, inp=inp)
    assert np.all(got[..., 0] == 0.0) and np.all(ref["scores"][..., 0] == 0.0)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("fp32", 64)])
def test_compress_under_a_sliding_window(dtype, d):
    cfg = _cfg(dtype=dtype, d=d, N=1024 if dtype == "bf16" else 320, k=400 if dtype == "bf16" else 120, T=60, P=20)
    window = cfg.N
    print(f"swa compress {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, window=window)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_compress_kcat(shape, dev["Q_cat"], dev["K"], dev["V"], gu.to_dev(K_cap), dev["novelty"], keep, ws,
                                scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap,
                     window=window)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    Kh = gu.to_host(dev["K"])
    for l in range(cfg.L):
        for h in range(cfg.Hkv):
            np.testing.assert_array_equal(Kh[0, l, h, :cfg.k], O.compact(inp["K"][0, l, h], kh[0, l, h]))


def test_window_limits_are_decided_on_the_host():
    cfg = _cfg(N=4096, k=2048, P=16, L=1)
    inp = synth.make_inputs(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    for window, code in ((cfg.P - 1, ip.CCD_EINVAL), (-5, ip.CCD_EINVAL)):
        shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
        ws = ip.alloc_workspace(shape)
        shape.window = window
        rc = ip.lib().ccd_score(__import__("ctypes").byref(shape), dev["Q_cat"].data_ptr(), dev["K"].data_ptr(),
                                dev["novelty"].data_ptr(), scores.data_ptr(), ws.data_ptr(), ws.numel(), None)
        assert rc == code, (window, rc)


def test_more_cap_tokens_under_a_window_than_the_matrix_core_kernels_take():
    """2100 CaP tokens under a window: the hidden head is longer than the matrix-core head kernels take, so the automatic
    choice scores on the vector ALUs (which mask inside their loops); naming a matrix-core path is refused."""
    cfg = _cfg(L=1, Hq=1, Hkv=1, d=64, N=2600, k=900, T=100, P=2100)
    window = 2300
    print(f"swa with {cfg.P} CaP tokens {cfg} window={window}", flush=True)
    got, ref = _score(cfg, window)
    gu.assert_scores_close(got, ref["scores"], cfg.G * cfg.P)
    inp = synth.make_inputs(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, window=window,
                          score_path=ip.CCD_PATH_MFMA_UNIT)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    rc = ip.lib().ccd_score(__import__("ctypes").byref(shape), dev["Q_cat"].data_ptr(), dev["K"].data_ptr(),
                            dev["novelty"].data_ptr(), scores.data_ptr(), ws.data_ptr(), ws.numel(), None)
    assert rc == ip.CCD_EUNSUPPORTED
