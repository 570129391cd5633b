"""Seeded random shapes through the fused call: every combination of cache type, head dimension, grouping, CaP length,
pot size, kept count, NuC slots, pooling, per-head novelty, CaP keys in the softmax and sliding window that the draw
produces is checked against the oracle like the hand-picked cases."""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _draw(seed):
    r = np.random.default_rng(1000 + seed)
    dtype = "bf16" if r.random() < 0.75 else "fp32"
    d = int(r.choice([64, 128]))
    Hkv = int(r.choice([1, 2, 3]))
    G = int(r.choice([1, 2, 4, 8]))
    P = int(r.choice([1, 3, 8, 17, 32, 40, 64]))
    N = int(r.integers(40, 1500 if dtype == "bf16" else 500))
    k = int(r.integers(1, N))
    T = int(r.integers(0, k + 1)) if r.random() < 0.8 else 0
    w = int(r.choice([1, 3, 5, 7, 9]))
    pool_mode = int(r.choice([O.POOL_MAX, O.POOL_AVG]))
    per_head = bool(r.random() < 0.5)
    with_cap = bool(r.random() < 0.5)
    window = 0
    if r.random() < 0.5:
        window = int(r.integers(max(P, N - 200), N + P + 2))
    keys = str(r.choice(["normal", "outlier1pct", "zipf"]))
    cfg = synth.CCDConfig(name=f"r{seed}", B=int(r.choice([1, 2])), L=int(r.choice([1, 2])), Hq=Hkv * G, Hkv=Hkv, d=d, N=N, k=k, P=P,
                          T=T, w=w, dtype=dtype, keys=keys, seed=2000 + seed)
    return cfg, pool_mode, per_head, with_cap, window


def _draw_wide(seed):
    """Long rows on a few units (the selection with 16 or 32 tokens per thread, or the separate kernels above 32768
    tokens), or many units with short rows (one selection + compaction workgroup per unit)."""
    r = np.random.default_rng(5000 + seed)
    dtype = "bf16" if r.random() < 0.8 else "fp32"
    d = int(r.choice([64, 128]))
    if r.random() < 0.5:
        Hkv, G, B, L = int(r.choice([1, 2])), int(r.choice([1, 2])), 1, 1
        N = int(r.integers(4097, 34000 if dtype == "bf16" else 9000))
    else:
        Hkv, G, B, L = int(r.choice([4, 8])), int(r.choice([1, 2])), int(r.choice([1, 2, 3])), int(r.integers(4, 20))
        N = int(r.integers(40, 700))
    P = int(r.choice([1, 3, 8]))
    k = int(r.integers(1, N))
    T = int(r.integers(0, k + 1)) if r.random() < 0.8 else 0
    w = int(r.choice([1, 3, 5, 7, 9]))
    pool_mode = int(r.choice([O.POOL_MAX, O.POOL_AVG]))
    per_head = bool(r.random() < 0.5)
    with_cap = bool(r.random() < 0.3)
    window = int(r.integers(max(P, N - 200), N + P + 2)) if r.random() < 0.3 else 0
    keys = str(r.choice(["normal", "outlier1pct", "zipf"]))
    cfg = synth.CCDConfig(name=f"w{seed}", B=B, L=L, Hq=Hkv * G, Hkv=Hkv, d=d, N=N, k=k, P=P, T=T, w=w, dtype=dtype, keys=keys,
                          seed=7000 + seed)
    return cfg, pool_mode, per_head, with_cap, window


@pytest.mark.parametrize("seed", range(32))
def test_random_shape(seed):
    _run(seed, *_draw(seed))


@pytest.mark.parametrize("seed", range(24))
def test_random_shape_long_rows_or_many_units(seed):
    _run(seed, *_draw_wide(seed))


def _run(seed, cfg, pool_mode, per_head, with_cap, window):
    # bf16 caches: the automatic choice of score kernels, or one of the two matrix-core kernels by force
    path = [ip.CCD_PATH_AUTO, ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT][seed % 3] if cfg.dtype == "bf16" else ip.CCD_PATH_AUTO
    # fp32 caches the matrix-core unit kernel can take (head dimension 64, plain softmax over the cache; not the Zipf key
    # norms, whose largest logits sit where the hi/lo split of the fp32 values is no longer two orders below the bound)
    if cfg.dtype == "fp32" and cfg.d == 64 and not with_cap and not window and cfg.keys != "zipf":
        path = ip.CCD_PATH_MFMA_UNIT
    print(f"random shape {seed}: {cfg} pool_mode={pool_mode} per_head={per_head} with_cap={with_cap} window={window} "
          f"path={path}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    if seed % 5 == 0:                                    # ties and tokens that may not take a NuC slot
        inp["novelty"] = np.round(inp["novelty"], 1)
        inp["novelty"].reshape(-1)[::7] = -np.inf
        inp["novelty"].reshape(-1)[3::11] = np.nan
    K_cap = synth.cap_keys(cfg) if with_cap else None
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=pool_mode,
                          window=window, score_path=path)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    if with_cap:
        rc = ip.ccd_compress_kcat(shape, dev["Q_cat"], dev["K"], dev["V"], gu.to_dev(K_cap), dev["novelty"], keep, ws, scores=scores)
    else:
        rc = ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores)
    torch.cuda.synchronize()
    assert rc == ip.CCD_OK
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=pool_mode,
                     K_cap=K_cap, window=window)
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    idx = kh.astype(np.int64)[..., None]
    np.testing.assert_array_equal(gu.to_host(dev["K"])[..., :cfg.k, :], np.take_along_axis(inp["K"], idx, axis=3))
    np.testing.assert_array_equal(gu.to_host(dev["V"])[..., :cfg.k, :], np.take_along_axis(inp["V"], idx, axis=3))
    if per_head:
        got = gu.to_host(dev["novelty"])[..., :cfg.k]
        want = np.take_along_axis(inp["novelty"], kh.astype(np.int64), axis=3)
        np.testing.assert_array_equal(got.view(np.uint32), want.view(np.uint32))
