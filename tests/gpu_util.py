"""Helpers for the GPU parity tests: host <-> device marshalling and the three-part parity protocol."""
import numpy as np
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import infinipot as ip

FLT_MIN = float(np.finfo(np.float32).tiny)


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy fp32 / int32 / bf16-bit (uint16) array -> CUDA tensor (bf16 bits become torch.bfloat16)."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def score_tolerance(ref: np.ndarray, GP: int) -> np.ndarray:
    """|gpu - oracle| bound: 1e-3 relative (the stated bar) plus the magnitude at which fp32 probabilities
    of single queries are flushed to zero (G*P terms, each below the smallest normal)."""
    return 1e-3 * np.abs(ref.astype(np.float64)) + 2.0 * GP * FLT_MIN


def assert_scores_close(gpu: np.ndarray, ref: np.ndarray, GP: int):
    inf_r, inf_g = np.isposinf(ref), np.isposinf(gpu)
    assert (inf_r == inf_g).all(), "NuC (+inf) positions differ"
    fin = ~inf_r
    err = np.abs(gpu[fin].astype(np.float64) - ref[fin].astype(np.float64))
    tol = score_tolerance(ref[fin], GP)
    bad = ~(err <= tol)                      # NaN on the GPU side counts as a failure
    if bad.any():
        where = np.argwhere(fin)[bad][:6].tolist()
        raise AssertionError(f"{bad.sum()} scores off (NaN: {np.isnan(gpu).sum()}); first at {where}: "
                             f"gpu {gpu[fin][bad][:6]} ref {ref[fin][bad][:6]}")


def assert_keep_matches(gpu_keep, ref_keep, ref_scores, k):
    """Exact match, else every index in the symmetric difference must sit within 1e-3 (relative) of the
    oracle's k-th largest score - the only place where fp32 vs fp64 scoring may legitimately differ.
    Returns the fraction of units that matched exactly."""
    units = gpu_keep.reshape(-1, k).shape[0]
    g, r, s = gpu_keep.reshape(units, k), ref_keep.reshape(units, k), ref_scores.reshape(units, -1)
    exact = 0
    for i in range(units):
        if np.array_equal(g[i], r[i]):
            exact += 1
            continue
        kth = np.sort(s[i].astype(np.float64))[::-1][k - 1]
        diff = np.setxor1d(g[i], r[i])
        vals = s[i][diff].astype(np.float64)
        assert np.all(np.abs(vals - kth) <= 1e-3 * abs(kth) + 1e-30), \
            f"unit {i}: keep_idx differs away from the threshold: idx {diff[:8]} scores {vals[:8]} kth {kth}"
    return exact / units


def check_keep_valid(keep, n, k):
    keep = keep.reshape(-1, k)
    assert keep.min() >= 0 and keep.max() < n
    assert (np.diff(keep, axis=1) > 0).all(), "keep_idx not strictly ascending"


def replay_select(gpu_scores, k):
    """Oracle selection run on the GPU's own fp32 scores (must equal the GPU's keep_idx bit for bit)."""
    flat = gpu_scores.reshape(-1, gpu_scores.shape[-1])
    return np.stack([O.select(row, k) for row in flat]).reshape(gpu_scores.shape[:-1] + (k,))
