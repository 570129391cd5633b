"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _cfg(**kw):
    base = dict(name="t", B=1, L=2, Hq=8, Hkv=2, d=128, N=700, k=300, P=9, T=100, w=7, dtype="bf16", keys="normal", seed=11)
    base.update(kw)
    return synth.CCDConfig(**base)


def _upload(inp):
    return {k: gu.to_dev(v) for k, v in inp.items()}


def _oracle(cfg, inp, pool_mode=O.POOL_MAX, **kw):
    args = dict(k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=pool_mode)
    args.update(kw)
    return O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], **args)


# ------------------------------------------------------------------ a7: compaction, bit exact

@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 64), ("fp32", 128)])
@pytest.mark.parametrize("inplace", [True, False])
def test_compact_bit_exact(dtype, d, inplace):
    print(f"compact dtype={dtype} d={d} inplace={inplace}", flush=True)
    cfg = _cfg(d=d, dtype=dtype, N=1500, k=777, B=2, L=2)
    inp = synth.make_inputs(cfg, per_head_novelty=True)
    rng = np.random.default_rng(3)
    keep = np.stack([np.sort(rng.choice(cfg.N, cfg.k, replace=False)) for _ in range(cfg.units)]).astype(np.int32)
    keep[0, :50] = np.arange(50)                      # a unit whose first rows stay where they are
    keep = keep.reshape(cfg.B, cfg.L, cfg.Hkv, cfg.k)
    dev = _upload(inp)
    dk = gu.to_dev(keep)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=0)
    if inplace:
        Kd, Vd = dev["K"], dev["V"]
    else:
        Kd, Vd = torch.zeros_like(dev["K"]), torch.zeros_like(dev["V"])
    assert ip.ccd_compact(shape, dev["K"], dev["V"], dk, Kd, Vd, dev["novelty"]) == ip.CCD_OK
    torch.cuda.synchronize()
    Kh, Vh, nh = gu.to_host(Kd), gu.to_host(Vd), gu.to_host(dev["novelty"])
    for b in range(cfg.B):
        for l in range(cfg.L):
            for h in range(cfg.Hkv):
                kp = keep[b, l, h]
                np.testing.assert_array_equal(Kh[b, l, h, :cfg.k], O.compact(inp["K"][b, l, h], kp))
                np.testing.assert_array_equal(Vh[b, l, h, :cfg.k], O.compact(inp["V"][b, l, h], kp))
                np.testing.assert_array_equal(nh[b, l, h, :cfg.k], O.compact(inp["novelty"][b, l, h], kp))
    if inplace:   # rows beyond k are left as they were
        np.testing.assert_array_equal(Kh[..., cfg.k:, :], inp["K"][..., cfg.k:, :])


# ------------------------------------------------------------------ a6: selection, bit exact

def _special_scores(rng, units, n):
    s = rng.standard_normal((units, n)).astype(np.float32)
    s[0] = np.round(s[0], 1)                                           # heavy ties
    if units > 1:
        s[1] = 0.25                                                    # everything ties
    if units > 2:
        s[2, rng.choice(n, n // 3, replace=False)] = np.inf            # many sentinels
        s[2, rng.choice(n, min(n, 5), replace=False)] = np.nan
        s[2, rng.choice(n, min(n, 5), replace=False)] = -np.inf
        s[2, rng.choice(n, min(n, 7), replace=False)] = 0.0
        s[2, rng.choice(n, min(n, 7), replace=False)] = -0.0
    if units > 3:
        s[3] = np.abs(s[3]) * 1e-38                                    # subnormals
    return s


@pytest.mark.parametrize("n,k", [(1, 1), (5, 2), (64, 64), (1000, 1), (1024, 512), (1025, 513), (4096, 2048), (5000, 4999),
                                 (33000, 4096)])
def test_select_bit_exact(n, k):
    print(f"select n={n} k={k}", flush=True)
    rng = np.random.default_rng(n * 7 + k)
    B, L, Hkv = 1, 2, 3
    s = _special_scores(rng, B * L * Hkv, n).reshape(B, L, Hkv, n)
    shape = ip.ccd_shape_t()
    shape.B, shape.L, shape.Hkv, shape.n_valid, shape.k = B, L, Hkv, n, k
    ds = gu.to_dev(s)
    keep = torch.full((B, L, Hkv, k), -1, dtype=torch.int32, device="cuda")
    assert ip.ccd_select(shape, ds, keep) == ip.CCD_OK
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gu.to_host(keep), gu.replay_select(s, k))


# ------------------------------------------------------------------ a1-a5: scores

SCORE_CASES = [
    dict(),                                                                       # bf16, d 128, ragged n and G*P
    dict(d=64, N=513, k=100, P=1, T=0, w=1),                                      # one query token, no pooling, CaP only
    dict(dtype="fp32", d=64, Hq=4, Hkv=4, N=512, k=256, P=16, T=128, w=1),        # config-1 shape
    dict(dtype="fp32", d=128, N=300, k=299, P=33, T=299, w=3),                    # NuC only
    dict(keys="outlier1pct", Hq=8, Hkv=2, N=2048, k=1024, P=32, T=512),           # config-2 shape, fewer heads
    dict(B=2, L=1, Hq=16, Hkv=2, N=1111, k=10, P=40, T=3, w=5),                   # G*P = 320 > one workgroup of queries
    dict(keys="zipf", B=2, L=1, N=900, k=128, P=16, T=64),
    dict(dtype="fp32", d=64, B=2, L=1, Hq=16, Hkv=2, N=1111, k=10, P=40, T=3, w=5),   # fp32, two query sweeps, ragged
    dict(dtype="fp32", d=64, keys="zipf", N=2600, k=900, T=100),                   # fp32, many tiles per wave
]


# the kernels of Eq. 2: vector ALUs, matrix cores with a workgroup per token slice, matrix cores with a workgroup per unit
SCORE_PATHS = [ip.CCD_PATH_VALU, ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT]


def _path_for(cfg, score_path):
    """fp32 caches: the vector ALUs, and the matrix-core unit kernel for head dimension 64."""
    if cfg.dtype == "fp32":
        if score_path == ip.CCD_PATH_VALU or (score_path == ip.CCD_PATH_MFMA_UNIT and cfg.d == 64):
            return score_path
        pytest.skip("fp32 caches: no such path")
    return score_path


@pytest.mark.parametrize("case", range(len(SCORE_CASES)))
@pytest.mark.parametrize("pool_mode", [O.POOL_MAX, O.POOL_AVG])
@pytest.mark.parametrize("score_path", SCORE_PATHS)
def test_scores_and_staged_calls(case, pool_mode, score_path):
    cfg = _cfg(**SCORE_CASES[case])
    score_path = _path_for(cfg, score_path)
    print(f"score case={case} cfg={cfg} pool_mode={pool_mode} path={score_path}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=(case % 2 == 1))
    ref = _oracle(cfg, inp, pool_mode)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=pool_mode,
                          score_path=score_path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
    assert ip.ccd_select(shape, scores, keep) == ip.CCD_OK
    torch.cuda.synchronize()
    sh, kh = gu.to_host(scores), gu.to_host(keep)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)                      # (A) scores
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)             # (B) selection up to threshold ties
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))                # (C) replay on the GPU's scores


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
@pytest.mark.parametrize("G,P", [(1, 64), (1, 65), (4, 32), (3, 43), (4, 33), (2, 96), (8, 33)])
def test_unit_kernel_sweep_widths(G, P, dtype, d):
    """The unit score kernel is built for sweeps of 64, 128 and 256 query rows: G * P at and around the limits (64, 65,
    128, 129, 132, 192) and beyond one sweep (264), with K_cap for bf16 (the CaP block is computed by the waves that
    own query rows)."""
    cfg = _cfg(dtype=dtype, d=d, B=1, L=2, Hq=2 * G, Hkv=2, P=P, N=777, k=300, T=50, w=3, seed=100 + G * P)
    print(f"sweep widths G*P={G * P} {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K_cap = synth.cap_keys(cfg) if dtype == "bf16" else None
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, K_cap=K_cap)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w,
                          score_path=ip.CCD_PATH_MFMA_UNIT)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    if K_cap is not None:
        rc = ip.ccd_score_kcat(shape, dev["Q_cat"], dev["K"], gu.to_dev(K_cap), dev["novelty"], scores, ws)
    else:
        rc = ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws)
    assert rc == ip.CCD_OK
    torch.cuda.synchronize()
    gu.assert_scores_close(gu.to_host(scores), ref["scores"], cfg.G * cfg.P)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("score_path", SCORE_PATHS)
@pytest.mark.parametrize("N", [1, 2, 31, 32, 33, 97, 128, 129])
def test_rows_of_a_few_tokens(N, score_path, dtype):
    """Rows shorter than, equal to and just beyond one 32-token tile and one tile per wave: waves without tokens, a
    ragged tile only, one full tile and a ragged one."""
    cfg = _cfg(dtype=dtype, d=64, L=1, N=N, k=max(1, N // 2), T=N // 4, P=5, w=3, seed=91 + N)
    score_path = _path_for(cfg, score_path)
    print(f"short rows {cfg} path={score_path}", flush=True)
    inp = synth.make_inputs(cfg)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, score_path=score_path) if N > cfg.k else (None, None, None, None)
    if rc is None:                                   # k = n (N = 1): nothing to drop, the fused call is a no-op; score only
        dev = _upload(inp)
        shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, score_path=score_path)
        ws = ip.alloc_workspace(shape)
        scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
        assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
        torch.cuda.synchronize()
        gu.assert_scores_close(gu.to_host(scores), ref["scores"], cfg.G * cfg.P)
        return
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, False)


@pytest.mark.parametrize("per_head", [False, True])
@pytest.mark.parametrize("score_path", SCORE_PATHS)
@pytest.mark.parametrize("T", [1, 37, 200, 699])
def test_nuc_slots_with_ties_and_non_finite_novelty(per_head, score_path, T):
    """Sec. 3.3.3 step 1 on novelty rows full of equal values, NaN and -inf: the +inf entries of the scores must
    sit exactly on the oracle's NuC slots (lowest index wins ties; NaN and -inf never take a slot)."""
    cfg = _cfg(T=T, k=max(300, T))
    print(f"nuc ties per_head={per_head} path={score_path} T={T}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    rng = np.random.default_rng(1234 + T)
    nov = np.round(inp["novelty"] * 4) / 4            # a handful of distinct levels -> many ties
    nov = nov.astype(np.float32)
    bad = rng.random(nov.shape) < 0.15
    nov[bad] = rng.choice(np.array([np.nan, -np.inf, np.inf], dtype=np.float32), size=int(bad.sum()))
    if T == 699:
        nov[..., 5:] = np.where(rng.random(nov[..., 5:].shape) < 0.9, -np.inf, nov[..., 5:])   # fewer eligible than T
    inp["novelty"] = nov
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=T, pool_w=cfg.w, pool_mode=O.POOL_MAX,
                          score_path=score_path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    sh = gu.to_host(scores)
    for b in range(cfg.B):
        for l in range(cfg.L):
            for h in range(cfg.Hkv):
                row = nov[b, l, h] if per_head else nov[b]
                want = O.nuc_slots(row, T)
                got = np.flatnonzero(np.isposinf(sh[b, l, h]))
                np.testing.assert_array_equal(got, want)


# ------------------------------------------------------------------ fused ccd_compress

def _run_fused(cfg, inp, pool_mode=O.POOL_MAX, per_head=False, want_scores=True, score_path=ip.CCD_PATH_AUTO):
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=pool_mode,
                          score_path=score_path)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda") if want_scores else None
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    rc = ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores)
    torch.cuda.synchronize()
    return rc, dev, scores, keep


def _check_fused(cfg, inp, ref, dev, scores, keep, per_head):
    kh = gu.to_host(keep)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    if scores is not None:
        sh = gu.to_host(scores)
        gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
        np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    frac = gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    Kh, Vh = gu.to_host(dev["K"]), gu.to_host(dev["V"])
    idx = kh.astype(np.int64)[..., None]
    np.testing.assert_array_equal(Kh[..., :cfg.k, :], np.take_along_axis(inp["K"], idx, axis=3))   # bit copies
    np.testing.assert_array_equal(Vh[..., :cfg.k, :], np.take_along_axis(inp["V"], idx, axis=3))
    if per_head:
        np.testing.assert_array_equal(gu.to_host(dev["novelty"])[..., :cfg.k],
                                      np.take_along_axis(inp["novelty"], kh.astype(np.int64), axis=3))
    return frac


@pytest.mark.parametrize("name", ["c1", "c2"])
def test_fused_compress_configs(name):
    cfg = synth.CONFIGS[name]
    print(f"fused {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp)
    assert rc == ip.CCD_OK
    frac = _check_fused(cfg, inp, ref, dev, scores, keep, False)
    print(f"  exact keep_idx units: {frac:.3f}", flush=True)
    # the NuC slots survive in every head (Sec. 3.3.3)
    kh = gu.to_host(keep)
    nuc = O.nuc_slots(inp["novelty"][0], cfg.T)
    for h in range(cfg.Hkv):
        assert set(nuc.tolist()) <= set(kh[0, 0, h].tolist())


@pytest.mark.parametrize("score_path", [ip.CCD_PATH_AUTO, ip.CCD_PATH_MFMA_UNIT])
@pytest.mark.parametrize("per_head,want_scores", [(True, False), (False, False), (True, True)])
def test_fused_compress_small(per_head, want_scores, score_path):
    cfg = _cfg(B=2, L=2, N=640, k=320, T=160)
    print(f"fused small per_head={per_head} want_scores={want_scores} path={score_path}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, per_head=per_head, want_scores=want_scores, score_path=score_path)
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, per_head)


@pytest.mark.parametrize("per_head", [False, True])
def test_fused_compress_fp32_cache_on_the_matrix_cores(per_head):
    """An fp32 cache of head dimension 64 on the unit kernel (every value as hi + lo bf16, three products each)."""
    cfg = _cfg(dtype="fp32", d=64, B=2, L=2, Hq=8, Hkv=2, P=20, N=1300, k=500, T=120, seed=37)
    print(f"fused fp32 on the matrix cores per_head={per_head} {cfg}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, per_head=per_head, score_path=ip.CCD_PATH_MFMA_UNIT)
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, per_head)


def test_fp32_cache_that_fills_the_chip_takes_the_matrix_cores_by_itself():
    """192 units of an fp32 cache (d = 64, 32 query rows per unit): the automatic choice is the unit kernel (seen in
    the per-kernel timing), and the result is the oracle's."""
    cfg = _cfg(dtype="fp32", d=64, B=1, L=24, Hq=32, Hkv=8, P=8, N=420, k=200, T=50, w=5, seed=41)
    print(f"fp32 automatic path {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    ref = _oracle(cfg, inp)
    ip.ccd_profile_enable(True)
    try:
        rc, dev, scores, keep = _run_fused(cfg, inp)
        stage_ms, calls = ip.ccd_profile_collect()
    finally:
        ip.ccd_profile_enable(False)
    assert rc == ip.CCD_OK and calls == 1
    assert stage_ms["score_unit"] > 0 and stage_ms["score_stats"] == 0 and stage_ms["score_prob"] == 0
    _check_fused(cfg, inp, ref, dev, scores, keep, False)


@pytest.mark.parametrize("per_head", [False, True])
def test_fused_compress_many_units(per_head):
    """More units than half the chip's compute units: one selection + compaction workgroup per unit (calls with
    fewer units split a unit's rows over several workgroups), novelty shared or carried per head."""
    cfg = _cfg(B=1, L=17, Hq=16, Hkv=8, P=4, N=520, k=250, T=60, w=5, seed=53)
    print(f"fused many units per_head={per_head} {cfg}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, per_head=per_head)
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, per_head)


@pytest.mark.parametrize("score_path", [ip.CCD_PATH_AUTO, ip.CCD_PATH_MFMA_UNIT])
@pytest.mark.parametrize("per_head,N", [(False, 6000), (True, 4100), (False, 16384), (True, 20000), (False, 32768)])
def test_fused_compress_rows_of_several_thousand_tokens(per_head, N, score_path):
    """Rows between 4097 and 32768 tokens: the one-workgroup selection + compaction with 16 or 32 tokens per thread."""
    cfg = _cfg(B=1, L=1, Hq=4, Hkv=2, P=8, N=N, k=N // 3, T=N // 8)
    print(f"fused N={N} per_head={per_head} path={score_path} {cfg}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=per_head)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, per_head=per_head, score_path=score_path)
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, per_head)


@pytest.mark.parametrize("dtype,d", [("bf16", 128), ("bf16", 64), ("fp32", 64)])
@pytest.mark.parametrize("fused", [True, False])
def test_strided_layouts(dtype, d, fused):
    """K and V stored head-major with padding rows ([B, Hkv + 1, L, n_cap + 8, d], seen as [B, L, Hkv, n_cap, d] through
    strides: layer stride below head stride), Q_cat cut out of a longer prompt buffer, per-head novelty with padded
    rows: results as for dense tensors, and nothing outside the views is written."""
    cfg = _cfg(B=2, L=3, Hq=6, Hkv=3, d=d, dtype=dtype, N=600, k=250, P=7, T=90, w=5, seed=61)
    print(f"strided {cfg} fused={fused}", flush=True)
    inp = synth.make_inputs(cfg, per_head_novelty=True)
    ref = _oracle(cfg, inp)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    fill = 3.0

    def embed(x, extra_heads, extra_rows):            # [B, L, H, n, d] -> view of a [B, H + eh, L, n + er, d] buffer
        B, L, H, n, dd = x.shape
        big = torch.full((B, H + extra_heads, L, n + extra_rows, dd), fill, dtype=tdt, device="cuda")
        view = big.permute(0, 2, 1, 3, 4)[:, :, :H, :n]
        view.copy_(gu.to_dev(x))
        return big, view

    Kbig, K = embed(inp["K"], 1, 8)
    Vbig, V = embed(inp["V"], 1, 8)
    Qbig = torch.full((cfg.B, cfg.L, cfg.Hq, cfg.P + 3, d), fill, dtype=tdt, device="cuda")
    Q = Qbig[:, :, :, :cfg.P]
    Q.copy_(gu.to_dev(inp["Q_cat"]))
    novbig = torch.full((cfg.B, cfg.L, cfg.Hkv, cfg.N + 5), fill, dtype=torch.float32, device="cuda")
    nov = novbig[..., :cfg.N]
    nov.copy_(gu.to_dev(inp["novelty"]))
    assert not K.is_contiguous() and not Q.is_contiguous() and not nov.is_contiguous()
    shape = ip.make_shape(Q, K, nov, k=cfg.k, T=cfg.T, pool_w=cfg.w)
    assert shape.kv_stride_l < shape.kv_stride_h
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    if fused:
        assert ip.ccd_compress(shape, Q, K, V, nov, keep, ws, scores=scores) == ip.CCD_OK
    else:
        assert ip.ccd_score(shape, Q, K, nov, scores, ws) == ip.CCD_OK
        assert ip.ccd_select(shape, scores, keep) == ip.CCD_OK
        assert ip.ccd_compact(shape, K, V, keep, K, V, nov) == ip.CCD_OK
    torch.cuda.synchronize()
    sh, kh = gu.to_host(scores), gu.to_host(keep)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    idx = kh.astype(np.int64)
    np.testing.assert_array_equal(gu.to_host(K.contiguous())[..., :cfg.k, :], np.take_along_axis(inp["K"], idx[..., None], axis=3))
    np.testing.assert_array_equal(gu.to_host(V.contiguous())[..., :cfg.k, :], np.take_along_axis(inp["V"], idx[..., None], axis=3))
    np.testing.assert_array_equal(gu.to_host(nov.contiguous())[..., :cfg.k], np.take_along_axis(inp["novelty"], idx, axis=3))
    # the padding: the extra head, the extra rows, the rest of the prompt buffer, the novelty tails
    for big in (Kbig, Vbig):
        assert bool((big[:, cfg.Hkv:] == fill).all()) and bool((big[:, :, :, cfg.N:] == fill).all())
    assert bool((Qbig[:, :, :, cfg.P:] == fill).all()) and bool((novbig[..., cfg.N:] == fill).all())


def test_not_full_pot_is_left_untouched():
    cfg = _cfg()
    inp = synth.make_inputs(cfg)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, n_valid=cfg.N - 1)
    ws = ip.alloc_workspace(shape)
    keep = torch.full((cfg.B, cfg.L, cfg.Hkv, cfg.k), -7, dtype=torch.int32, device="cuda")
    assert ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws) == ip.CCD_NOOP
    torch.cuda.synchronize()
    np.testing.assert_array_equal(gu.to_host(dev["K"]), inp["K"])
    np.testing.assert_array_equal(gu.to_host(dev["V"]), inp["V"])
    assert (gu.to_host(keep) == -7).all()


def test_partial_pot_staged_scoring_ignores_rows_beyond_n_valid():
    cfg = _cfg(N=600, k=200, T=50)
    inp = synth.make_inputs(cfg)
    n = 555
    inp["K"][..., n:, :] = 0x7FC0                                   # NaN rows beyond n_valid must never be read into a score
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, n_valid=n)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, n_valid=n)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, n), dtype=torch.float32, device="cuda")
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    gu.assert_scores_close(gu.to_host(scores), ref["scores"], cfg.G * cfg.P)


def test_non_finite_keys_keep_indices_valid():
    cfg = _cfg(N=400, k=150, T=40)
    inp = synth.make_inputs(cfg)
    inp["K"][0, 0, 0, 17, :] = 0x7FC0                               # NaN key row
    inp["K"][0, 1, 1, 5, 3] = 0x7F80                                # +inf element
    inp["novelty"][0, 3] = np.nan
    rc, dev, scores, keep = _run_fused(cfg, inp)
    assert rc == ip.CCD_OK
    gu.check_keep_valid(gu.to_host(keep), cfg.N, cfg.k)


@pytest.mark.parametrize("where", ["late_tokens", "second_slice", "second_sweep", "tail_tile"])
def test_logits_far_above_those_of_the_first_tile(where):
    """The matrix-core statistics pass sums 2^(x - reference) with the reference taken from the first tile of a slice
    and redoes a slice whose sums leave the fp32 range.  Keys whose logits outgrow the first tile's by hundreds of
    binary orders force that; the result must be the oracle's all the same."""
    cfg = _cfg(B=1, L=1, Hq=16, Hkv=2, P=40, N=2500 if where == "second_slice" else 1000, k=300, T=50, w=3, seed=71)
    print(f"far logits {where} {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K = synth.bf16_bits_to_f32(inp["K"])
    Q = synth.bf16_bits_to_f32(inp["Q_cat"])
    K[..., :64, :] *= 0.01                                           # a quiet first tile
    if where == "late_tokens":
        K[..., 300:, :] *= 30.0
        Q *= 3.0
    elif where == "second_slice":                                    # 2500 tokens: slices of 2048 or shorter
        K[..., 2100:, :] *= 30.0
        Q *= 3.0
    elif where == "second_sweep":                                    # G * P = 320: only query rows >= 256 grow
        K[..., 300:, :] *= 30.0
        Q[:, :, cfg.G - 1::cfg.G, 20:, :] *= 30.0                    # the last query head of each group, CaP rows 20..
        Q[:, :, : cfg.G - 1, :, :] *= 0.01
    else:                                                            # only the ragged last tile (1000 = 31 * 32 + 8)
        K[..., 992:, :] *= 90.0
        Q *= 3.0
    inp["K"], inp["Q_cat"] = synth.f32_to_bf16_bits(K), synth.f32_to_bf16_bits(Q)
    ref = _oracle(cfg, inp)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    gu.assert_scores_close(gu.to_host(scores), ref["scores"], cfg.G * cfg.P)


@pytest.mark.parametrize("gain", [2.0, 4.0])
def test_fp32_cache_on_the_matrix_cores_keeps_the_bound_as_logits_grow(gain):
    """Q and K of N(0,1) scaled by `gain`: the largest log2-domain logits reach about 23 and 93; the scores of the
    hi/lo form stay within the 1e-3 bound (measured: 6e-5 and 4e-4)."""
    cfg = _cfg(dtype="fp32", d=64, B=1, L=2, Hq=8, Hkv=2, N=1500, k=500, P=16, T=0, w=1, seed=5)
    print(f"fp32 on the matrix cores, gain {gain} {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    inp["Q_cat"], inp["K"] = inp["Q_cat"] * np.float32(gain), inp["K"] * np.float32(gain)
    ref = _oracle(cfg, inp)
    rc, dev, scores, keep = _run_fused(cfg, inp, score_path=ip.CCD_PATH_MFMA_UNIT)
    assert rc == ip.CCD_OK
    _check_fused(cfg, inp, ref, dev, scores, keep, False)


@pytest.mark.parametrize("where", ["late_tokens", "tail_tile"])
def test_logits_far_above_those_of_the_first_tile_fp32_on_the_matrix_cores(where):
    """The same redo of a wave's tokens on the fp32 form of the unit kernel.  Logits that overflow a sum are more than 127
    binary orders above the reference, and at that size the hi/lo split of the fp32 values (logits good to about 2^-16
    of sum |q k|) no longer resolves a probability to 1e-3: the bound here is 5e-2, the point is the redo itself."""
    cfg = _cfg(dtype="fp32", d=64, B=1, L=1, Hq=16, Hkv=2, P=40, N=1000, k=300, T=50, w=3, seed=73)
    print(f"far logits fp32 {where} {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    K, Q = inp["K"].copy(), inp["Q_cat"].copy()
    K[..., :64, :] *= 0.01
    if where == "late_tokens":
        K[..., 300:, :] *= 40.0
    else:
        K[..., 992:, :] *= 60.0
    Q *= 4.0
    inp["K"], inp["Q_cat"] = K, Q
    ref = _oracle(cfg, inp)
    dev = _upload(inp)
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w,
                          score_path=ip.CCD_PATH_MFMA_UNIT)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_score(shape, dev["Q_cat"], dev["K"], dev["novelty"], scores, ws) == ip.CCD_OK
    torch.cuda.synchronize()
    got, want = gu.to_host(scores), ref["scores"]
    fin = np.isfinite(want)
    assert np.array_equal(np.isposinf(got), np.isposinf(want)) and not np.isnan(got).any()
    np.testing.assert_allclose(got[fin], want[fin], rtol=5e-2, atol=2 * cfg.G * cfg.P * np.finfo(np.float32).tiny)
    assert (want[fin] > 0).sum() > 100          # not a row of zeros


@pytest.mark.parametrize("score_path", SCORE_PATHS)
def test_heavy_tailed_key_norms_saturate_the_softmax(score_path):
    """Key rows scaled by sqrt(z_t), z_t ~ Zipf(1.1) capped at 2^16 instead of the benchmark's 64 (gains up to 256, logits
    up to 1600 binary orders): nearly every attention row is one-hot, nine scores in ten are exactly zero and fewer
    than k are positive, so the selection is decided by the ties at zero.  (The cap keeps the logits where fp32 still
    resolves their exponent to 1e-3: one unit in the last place of 1600 is 1.2e-4.)"""
    cfg = _cfg(B=2, L=1, Hq=8, Hkv=2, N=1200, k=400, P=16, T=0, w=1, seed=83)
    print(f"heavy-tailed key norms {cfg} path={score_path}", flush=True)
    inp = synth.make_inputs(cfg)
    rng = np.random.default_rng(83)
    z = np.minimum(rng.zipf(1.1, size=(cfg.B, cfg.N)).astype(np.float64), 2.0 ** 16)
    K = synth.bf16_bits_to_f32(inp["K"]) * np.sqrt(z).astype(np.float32)[:, None, None, :, None]
    inp["K"] = synth.f32_to_bf16_bits(K)
    ref = _oracle(cfg, inp)
    assert (ref["scores"] == 0).mean() > 0.8 and ((ref["scores"] > 0).sum(axis=-1) < cfg.k).all()
    rc, dev, scores, keep = _run_fused(cfg, inp, score_path=score_path)
    assert rc == ip.CCD_OK
    sh = gu.to_host(scores)
    assert (sh == 0).mean() > 0.8
    np.testing.assert_allclose(sh.sum(axis=-1, dtype=np.float64), cfg.G * cfg.P, rtol=1e-3)   # every query row sums to one
    _check_fused(cfg, inp, ref, dev, scores, keep, False)


# ------------------------------------------------------------------ run-to-run behaviour

def test_repeated_calls_give_identical_bits():
    """Nothing in the path depends on scheduling order (no float atomics, fixed reduction trees): two calls on the same
    inputs give the same bits in scores, keep_idx, K' and V'."""
    cfg = _cfg(L=4, N=1500, k=700, T=200)
    inp = synth.make_inputs(cfg)
    outs = []
    for rep in range(3):
        rc, dev, scores, keep = _run_fused(cfg, inp)
        assert rc == ip.CCD_OK
        outs.append((gu.to_host(scores).view(np.uint32), gu.to_host(keep), gu.to_host(dev["K"]), gu.to_host(dev["V"])))
    for o in outs[1:]:
        for a, b in zip(outs[0], o):
            np.testing.assert_array_equal(a, b)


def test_compress_in_a_captured_graph_replays_exactly():
    """The call launches kernels only (no allocation, no memset, no host sync): it can be captured into a HIP graph.
    Every replay, with eager work and synchronisations in between, must reproduce the eager result."""
    cfg = _cfg(L=2, N=1100, k=500, T=100)
    inp = synth.make_inputs(cfg)
    rc, dev_e, scores_e, keep_e = _run_fused(cfg, inp)
    assert rc == ip.CCD_OK
    want = (gu.to_host(scores_e).view(np.uint32), gu.to_host(keep_e), gu.to_host(dev_e["K"]), gu.to_host(dev_e["V"]))
    dev = _upload(inp)
    pristine = {k: v.clone() for k, v in dev.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, pool_mode=O.POOL_MAX)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            assert ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores,
                                   stream=side) == ip.CCD_OK
    torch.cuda.synchronize()
    for rep in range(3):
        for k_, v in pristine.items():                      # eager work between the replays: restore the pot
            dev[k_].copy_(v)
        scores.zero_()
        keep.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = (gu.to_host(scores).view(np.uint32), gu.to_host(keep), gu.to_host(dev["K"]), gu.to_host(dev["V"]))
        for a, b in zip(want, got):
            np.testing.assert_array_equal(a, b)


def test_interleaved_calls_with_different_score_paths_do_not_affect_each_other():
    """The score path is an argument of the call (shape.score_path), not a setting of the library: calls that ask for
    different paths, issued alternately from two host threads on two streams, each give the bits the same call gives
    when it runs alone."""
    import threading
    cfgs = [_cfg(L=3, N=1300, k=600, T=150, seed=61), _cfg(L=2, N=900, k=400, T=90, seed=62),
            _cfg(L=2, N=1100, k=512, T=128, seed=63)]
    paths = [ip.CCD_PATH_VALU, ip.CCD_PATH_MFMA_SLICES, ip.CCD_PATH_MFMA_UNIT]
    inps = [synth.make_inputs(c) for c in cfgs]
    alone = []
    for cfg, inp, path in zip(cfgs, inps, paths):
        rc, dev, scores, keep = _run_fused(cfg, inp, score_path=path)
        assert rc == ip.CCD_OK
        alone.append((gu.to_host(scores).view(np.uint32), gu.to_host(keep), gu.to_host(dev["K"]), gu.to_host(dev["V"])))
    # two paths on the same inputs differ in rounding order, so the check below can tell them apart
    rc, _, s_other, _ = _run_fused(cfgs[0], inps[0], score_path=paths[2])
    assert rc == ip.CCD_OK and not np.array_equal(gu.to_host(s_other).view(np.uint32), alone[0][0])

    reps, errors = 4, []
    results = [[None] * reps for _ in cfgs]

    def worker(i):
        try:
            cfg, inp, path = cfgs[i], inps[i], paths[i]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for rep in range(reps):
                    dev = _upload(inp)
                    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w,
                                          pool_mode=O.POOL_MAX, score_path=path)
                    ws = ip.alloc_workspace(shape)
                    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
                    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
                    rc = ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores,
                                         stream=stream)
                    assert rc == ip.CCD_OK
                    stream.synchronize()
                    results[i][rep] = (gu.to_host(scores).view(np.uint32), gu.to_host(keep), gu.to_host(dev["K"]),
                                       gu.to_host(dev["V"]))
        except Exception as e:                                # pragma: no cover - reported by the assert below
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=worker, args=(i,)) for i in range(len(cfgs))]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors
    for i in range(len(cfgs)):
        for rep in range(reps):
            for a, b in zip(alone[i], results[i][rep]):
                np.testing.assert_array_equal(a, b)
