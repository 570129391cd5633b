"""GPU parity of the NuC score from logits (Eq. 3) through the C ABI, and the chain logits -> novelty -> compression.

Tolerance (derived from the arithmetic): the library sums V terms 2^((z - m) log2 e) in fp32 (1-ulp exp2, exact
differences z - m, pairwise merging of 256 partial sums) and takes one fast log2: the log-sum-exp carries a relative
error of a few 2^-24 in the sum, i.e. an ABSOLUTE error of about 1e-6 in natural-log units, plus 2^-24 relative
rounding of m + log(s) and of the final subtraction.  |delta| <= 4e-6 + 3 * 2^-24 * (|lse| + |z_label|).
"""
import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip
from paper_2410_01518_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _logits(rows, V, dtype, seed, scale=4.0):
    """Synthetic next-token logits: a flat N(0, scale) background with a few strong candidates per row."""
    rng = np.random.default_rng(seed)
    z = (rng.standard_normal((rows, V)) * scale).astype(np.float32)
    hot = rng.integers(0, V, (rows, 3))
    z[np.arange(rows)[:, None], hot] += rng.uniform(5, 25, (rows, 3)).astype(np.float32)
    labels = np.where(rng.random(rows) < 0.5, hot[:, 0], rng.integers(0, V, rows)).astype(np.int32)
    if dtype == "bf16":
        return synth.f32_to_bf16_bits(z), labels
    return z, labels


def _tol(z_store, labels, ref):
    z = O.to_f64(z_store)
    rows = z.shape[0]
    lab = np.clip(labels, 0, z.shape[1] - 1)
    zl = np.abs(z[np.arange(rows), lab])
    lse = np.abs(ref.astype(np.float64) + z[np.arange(rows), lab])
    return 4e-6 + 3 * 2.0 ** -24 * (lse + zl)


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
@pytest.mark.parametrize("rows,V", [(1, 1), (3, 7), (5, 1000), (64, 32000), (9, 32008), (4, 128256), (2, 2056)])
def test_nuc_from_logits(dtype, rows, V):
    print(f"nuc_from_logits {dtype} rows={rows} V={V}", flush=True)
    esz = 2 if dtype == "bf16" else 4
    z, labels = _logits(rows, V, dtype, seed=rows * 1000 + V)
    if rows >= 3:
        labels[1] = -100                          # a token without a prediction
        labels[2] = V                             # out of range above
    stride = (V * esz + 15) // 16 * 16 // esz     # rows 16-byte aligned: padding columns are never read
    buf = np.zeros((rows, stride), dtype=z.dtype)
    buf[:, :V] = z
    if stride > V:
        buf[:, V:] = synth.f32_to_bf16_bits(np.full((rows, stride - V), 1e30, np.float32)) if dtype == "bf16" else 1e30
    dev = gu.to_dev(buf)
    nov = torch.full((rows,), 123.0, dtype=torch.float32, device="cuda")
    assert ip.ccd_nuc_from_logits(dev[:, :V], torch.from_numpy(labels).cuda(), nov) == ip.CCD_OK
    torch.cuda.synchronize()
    got = nov.cpu().numpy()
    ref = O.nuc_from_logits(z, labels)
    bad = (labels < 0) | (labels >= V)
    assert np.all(np.isneginf(got[bad])) and np.all(np.isneginf(ref[bad]))
    ok = ~bad
    err = np.abs(got[ok].astype(np.float64) - ref[ok].astype(np.float64))
    tol = _tol(z, labels, ref)[ok]
    assert np.all(err <= tol), f"max err {err.max():.3e} (tol {tol[err.argmax()]:.3e})"


def test_nuc_from_logits_extreme_rows():
    """Rows with -inf entries (masked vocabulary), a single survivor, huge spreads and ties."""
    V = 4096
    z = np.zeros((5, V), dtype=np.float32)
    z[0, :] = -np.inf; z[0, 17] = 3.0                         # one survivor: CE of it is 0, of others +inf
    z[1, :] = -80.0; z[1, 5] = 80.0                           # spread of 160: the background underflows
    z[2, :] = 1e4                                             # all equal and large: log V
    z[3, : V // 2] = -np.inf                                  # half masked
    z[4, :] = np.linspace(-50, 50, V, dtype=np.float32)
    labels = np.array([17, 5, 100, V - 1, 0], dtype=np.int32)
    nov = torch.empty(5, dtype=torch.float32, device="cuda")
    assert ip.ccd_nuc_from_logits(torch.from_numpy(z).cuda(), torch.from_numpy(labels).cuda(), nov) == ip.CCD_OK
    torch.cuda.synchronize()
    got = nov.cpu().numpy().astype(np.float64)
    ref = O.nuc_from_logits(z, labels).astype(np.float64)
    assert np.all(np.abs(got - ref) <= _tol(z, labels, ref.astype(np.float32)))
    assert abs(got[0]) <= 4e-6 and abs(got[2] - np.log(V)) <= 2e-3


def test_logits_to_novelty_to_compression():
    """App. B end to end: token losses from the logits give the NuC slots of the compression."""
    cfg = synth.CCDConfig(name="t", B=2, L=2, Hq=4, Hkv=2, d=64, N=512, k=200, P=4, T=60, w=7, dtype="bf16", keys="normal", seed=51)
    print(f"logits -> novelty -> compress {cfg}", flush=True)
    inp = synth.make_inputs(cfg)
    V = 5000
    z, labels = _logits(cfg.B * cfg.N, V, "bf16", seed=52)
    labels[0] = -100                                          # the first token of a sequence has no predictor
    dev = {k: gu.to_dev(v) for k, v in inp.items()}
    nov = torch.empty((cfg.B, cfg.N), dtype=torch.float32, device="cuda")
    logits_dev = gu.to_dev(z).reshape(cfg.B, cfg.N, V)
    assert ip.ccd_nuc_from_logits(logits_dev, torch.from_numpy(labels).cuda().reshape(cfg.B, cfg.N), nov) == ip.CCD_OK
    shape = ip.make_shape(dev["Q_cat"], dev["K"], nov, k=cfg.k, T=cfg.T, pool_w=cfg.w)
    ws = ip.alloc_workspace(shape)
    keep = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.k), dtype=torch.int32, device="cuda")
    scores = torch.empty((cfg.B, cfg.L, cfg.Hkv, cfg.N), dtype=torch.float32, device="cuda")
    assert ip.ccd_compress(shape, dev["Q_cat"], dev["K"], dev["V"], nov, keep, ws, scores=scores) == ip.CCD_OK
    torch.cuda.synchronize()
    nov_ref = O.nuc_from_logits(z, labels).reshape(cfg.B, cfg.N)
    nov_gpu = nov.cpu().numpy()
    kh, sh = gu.to_host(keep), gu.to_host(scores)
    # the NuC slots the library lifted are the top-T of ITS novelty; they agree with the oracle's unless two losses
    # near the T-th one swap within the tolerance above
    for b in range(cfg.B):
        slots_gpu = O.nuc_slots(nov_gpu[b], cfg.T)
        for l in range(cfg.L):
            for h in range(cfg.Hkv):
                np.testing.assert_array_equal(np.flatnonzero(np.isposinf(sh[b, l, h])), slots_gpu)
                assert np.isin(slots_gpu, kh[b, l, h]).all()
        slots_ref = O.nuc_slots(nov_ref[b], cfg.T)
        diff = np.setxor1d(slots_gpu, slots_ref)
        thr = np.sort(nov_ref[b][np.isfinite(nov_ref[b])])[-cfg.T]
        assert np.all(np.abs(nov_ref[b][diff] - thr) <= 1e-4), "NuC slots differ beyond a threshold tie"
    ref = O.compress(inp["Q_cat"], inp["K"], inp["V"], nov_gpu, k=cfg.k, T=cfg.T, pool_w=cfg.w)
    gu.assert_scores_close(sh, ref["scores"], cfg.G * cfg.P)
    gu.assert_keep_matches(kh, ref["keep_idx"], ref["scores"], cfg.k)
