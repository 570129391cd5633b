"""Parity at the benchmark's own sizes and launch configuration, and the streaming use of the step."""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from paper_2410_01518_amd.pot import MemoryPot
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _sample_units(cfg, n, seed=0):
    rng = np.random.default_rng(seed)
    ids = sorted(set([0, cfg.units - 1] + rng.choice(cfg.units, n, replace=False).tolist()))
    return [(u // (cfg.L * cfg.Hkv), (u // cfg.Hkv) % cfg.L, u % cfg.Hkv) for u in ids]


def test_headline_config_fused_full_size():
    """32 layers x 8 KV heads x 128, pot 4096 -> 2048, exactly the call bench.py times: the fp64 oracle, the replay of the
    selection and the bit-exact compaction on all 256 units."""
    cfg = synth.CONFIGS["c3"]
    print(f"full size {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    assert ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    sh, kh = gu.to_host(scores), gu.to_host(keep)
    print("  gpu done", flush=True)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))                      # every unit, bit exact
    nuc = O.nuc_slots(inp["novelty"][0], cfg.T)
    assert len(nuc) == cfg.T and np.isin(nuc, kh.reshape(-1, cfg.k)).all()
    assert (np.isposinf(sh).sum(axis=-1) == cfg.T).all()
    assert (np.isin(kh.reshape(cfg.units, cfg.k), nuc).sum(axis=1) == cfg.T).all()      # the NuC slots survive in every head
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)    # every unit
    print("  oracle done", flush=True)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    frac = gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
    print(f"  units with keep_idx identical to the fp64 oracle: {frac * cfg.units:.0f}/{cfg.units}", flush=True)
    Kh, Vh = gu.to_host(dev["K"]), gu.to_host(dev["V"])
    idx = kh.astype(np.int64)[..., None]
    np.testing.assert_array_equal(Kh[..., :cfg.k, :], np.take_along_axis(inp["K"], idx, axis=3))
    np.testing.assert_array_equal(Vh[..., :cfg.k, :], np.take_along_axis(inp["V"], idx, axis=3))
    np.testing.assert_array_equal(Kh[..., cfg.k:, :], inp["K"][..., cfg.k:, :])


def test_large_pot_shape_on_sampled_units():
    """The stress configuration's per-unit shape (pot 32768 -> 4096, 8 query heads per KV head, 128 CaP tokens,
    Zipf-skewed key norms, 4 sequences) on a few layers; oracle on sampled units."""
    cfg = synth.scaled(synth.CONFIGS["c5"], L=2)
    print(f"large pot {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    shape = ip.make_shape(dev["Q_cat"], dev["K"], dev["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    assert ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], dev["novelty"], keep, ws, scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    sh, kh = gu.to_host(scores), gu.to_host(keep)
    gu.check_keep_valid(kh, cfg.N, cfg.k)
    np.testing.assert_array_equal(kh, gu.replay_select(sh, cfg.k))
    units = _sample_units(cfg, 2, seed=1)
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], inp["novelty"], k=cfg.k, T=cfg.T, pool_w=cfg.w, units=units)
    for (b, l, h) in units:
        gu.assert_scores_close(sh[b, l, h], ref["scores"][b, l, h], cfg.G * cfg.P)
        gu.assert_keep_matches(kh[b, l, h], ref["keep_idx"][b, l, h], ref["scores"][b, l, h], cfg.k)
    Kh = gu.to_host(dev["K"])
    np.testing.assert_array_equal(Kh[..., :cfg.k, :], np.take_along_axis(inp["K"], kh.astype(np.int64)[..., None], axis=3))


def test_stress_config_full_size_drawn_on_device():
    """The whole stress configuration in one call: 4 sequences x 80 layers x 8 KV heads = 2560 units, pot 32768 -> 4096,
    1024 query rows per unit; K and V are 21.5 GB each (element offsets beyond 2^32, a 3 GB workspace).  The inputs
    are drawn on the device with the recipe of the configuration (keys N(0,1) x sqrt(min(z_t, 64)), z_t ~ Zipf(1.1) per
    (sequence, token)); the oracle scores 16 sampled units, the selection is replayed on them, and every unit's
    keep_idx and compacted rows are checked on the device."""
    cfg = synth.CONFIGS["c5"]
    free = torch.cuda.mem_get_info()[0]
    pot_bytes = 2 * cfg.units * cfg.N * cfg.d * 2
    if free < 2.4 * pot_bytes:
        pytest.skip(f"needs {2.4 * pot_bytes / 2**30:.0f} GiB of device memory, {free / 2**30:.0f} GiB free")
    print(f"stress, full size {cfg}", flush=True)
    g = torch.Generator(device="cuda").manual_seed(5005)
    rng = np.random.default_rng(5005)
    z = np.minimum(rng.zipf(1.1, size=(cfg.B, cfg.N)), 64).astype(np.float32)
    gain = torch.from_numpy(np.sqrt(z)).cuda()[:, None, None, :, None]                  # [B,1,1,N,1]
    K = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N, cfg.d), dtype=torch.bfloat16, device="cuda")
    for b in range(cfg.B):                                                              # (fp32 draw, one sequence at a time)
        K[b] = (torch.randn(K[b].shape, generator=g, device="cuda", dtype=torch.float32) * gain[b]).to(torch.bfloat16)
    V = torch.empty_like(K).normal_(generator=g)
    Q = torch.randn((cfg.B, cfg.L, cfg.Hq, cfg.P, cfg.d), generator=g, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    nov = torch.rand((cfg.B, cfg.N), generator=g, device="cuda", dtype=torch.float32)
    K0, V0 = K.clone(), V.clone()
    shape = ip.make_shape(Q, K, nov, k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    print(f"  inputs drawn, workspace {ws.numel() * ws.element_size() / 2**30:.2f} GiB", flush=True)
    t0 = torch.cuda.Event(enable_timing=True); t1 = torch.cuda.Event(enable_timing=True)
    t0.record()
    assert ip.ccd_compress(shape, Q, K, V, nov, keep, ws, scores=scores) == ip.CCD_OK
    t1.record()
    torch.cuda.synchronize()
    print(f"  ccd_compress: {t0.elapsed_time(t1):.1f} ms", flush=True)
    # every unit, on the device: ascending in-range keep_idx, T NuC slots lifted, rows bit-exact, tail untouched
    k64 = keep.to(torch.int64)
    assert int(k64.min()) >= 0 and int(k64.max()) < cfg.N and bool((k64[..., 1:] > k64[..., :-1]).all())
    assert bool((torch.isposinf(scores).sum(dim=-1) == cfg.T).all()) and not bool(torch.isnan(scores).any())
    for b in range(cfg.B):
        idx = k64[b][..., None].expand(-1, -1, -1, cfg.d)
        for T_new, T_old in ((K, K0), (V, V0)):
            got, src = T_new[b].view(torch.int16), T_old[b].view(torch.int16)
            assert torch.equal(got[..., :cfg.k, :], torch.gather(src, 2, idx))
            assert torch.equal(got[..., cfg.k:, :], src[..., cfg.k:, :])
    print("  all units checked on the device", flush=True)
    # sampled units: replay of the selection, fp64 oracle
    units = _sample_units(cfg, 14, seed=2)
    nov_h = gu.to_host(nov)
    for (b, l, h) in units:
        sh, kh = gu.to_host(scores[b, l, h]), gu.to_host(keep[b, l, h])
        np.testing.assert_array_equal(kh, O.select(sh, cfg.k))
        Qu = gu.to_host(Q[b, l, h * cfg.G:(h + 1) * cfg.G])[None, None]
        Ku, Vu = gu.to_host(K0[b, l, h])[None, None, None], gu.to_host(V0[b, l, h])[None, None, None]
        ref = O.compress(Qu, Ku, Vu, nov_h[b:b + 1], k=cfg.k, T=cfg.T, pool_w=cfg.w)
        gu.assert_scores_close(sh, ref["scores"][0, 0, 0], cfg.G * cfg.P)
        gu.assert_keep_matches(kh, ref["keep_idx"][0, 0, 0], ref["scores"][0, 0, 0], cfg.k)
        print(f"  unit {(b, l, h)} matches the oracle", flush=True)
    assert len(units) >= 16


def test_streaming_pot_teacher_forced():
    """Continual distillation (Sec. 3.2): a context streamed through a small pot in chunks; every compression is
    checked against the oracle run on the pot's own state just before the call (K, V, carried per-head novelty)."""
    B, L, Hq, Hkv, d, n_cap, k, T, P, chunk = 1, 2, 4, 2, 128, 512, 256, 128, 8, 256
    rng = np.random.default_rng(4)
    pot = MemoryPot(B, L, Hkv, d, n_cap, k, T, pool_w=7)
    n_chunks, calls = 10, 0
    for c in range(n_chunks):
        if pot.room < chunk:                       # the pot is full on arrival of the next chunk: distill first
            Q = synth.f32_to_bf16_bits(rng.standard_normal((B, L, Hq, P, d), dtype=np.float32))
            pre = {"K": gu.to_host(pot.K), "V": gu.to_host(pot.V), "nov": gu.to_host(pot.novelty)}
            scores = torch.empty((B, L, Hkv, n_cap), dtype=torch.float32, device="cuda")
            assert pot.distill(gu.to_dev(Q), scores=scores) == ip.CCD_OK
            torch.cuda.synchronize()
            calls += 1
            ref = O.compress(Q, pre["K"], pre["V"], pre["nov"], k=k, T=T, pool_w=7)
            sh, kh = gu.to_host(scores), gu.to_host(pot.keep_idx)
            gu.assert_scores_close(sh, ref["scores"], (Hq // Hkv) * P)
            gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], k)
            np.testing.assert_array_equal(kh, gu.replay_select(sh, k))
            idx = kh.astype(np.int64)
            np.testing.assert_array_equal(gu.to_host(pot.K)[..., :k, :], np.take_along_axis(pre["K"], idx[..., None], axis=3))
            np.testing.assert_array_equal(gu.to_host(pot.V)[..., :k, :], np.take_along_axis(pre["V"], idx[..., None], axis=3))
            np.testing.assert_array_equal(gu.to_host(pot.novelty)[..., :k], np.take_along_axis(pre["nov"], idx, axis=3))
            assert pot.n_valid == k
        Kc = synth.f32_to_bf16_bits(rng.standard_normal((B, L, Hkv, chunk, d), dtype=np.float32))
        Vc = synth.f32_to_bf16_bits(rng.standard_normal((B, L, Hkv, chunk, d), dtype=np.float32))
        nv = rng.random((B, chunk), dtype=np.float32)
        pot.append(gu.to_dev(Kc), gu.to_dev(Vc), gu.to_dev(nv))
    assert calls == n_chunks - n_cap // chunk and pot.calls == calls     # compress-on-arrival: chunks 3.. each trigger one
    # a pot that is not full is left alone
    pot2 = MemoryPot(B, L, Hkv, d, n_cap, k, T)
    pot2.append(gu.to_dev(Kc), gu.to_dev(Vc), gu.to_dev(nv))
    assert pot2.distill(gu.to_dev(Q)) == ip.CCD_NOOP and pot2.n_valid == chunk
