"""Pins for the oracle's CR-RoPE step (Sec. 3.5): the rotation against what the mathematics fixes.

Every expected value here comes from a closed form, an invariant of rotations, or an independent formulation
(complex multiplication in torch) - never from the oracle itself or from the GPU path.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O
from paper_2410_01518_amd import synth


def _rand(n, d, seed):
    return np.random.default_rng(seed).standard_normal((n, d))


def test_tables_are_the_rope_frequencies():
    # angle[p, i] = p * base^(-2i/d): spot values written out by hand
    cos, sin = synth.rope_tables(5, 8, base=10000.0)
    assert cos.shape == (5, 4) and cos.dtype == np.float32
    for p, i in [(0, 0), (1, 0), (3, 1), (4, 3)]:
        ang = p * 10000.0 ** (-2.0 * i / 8)
        assert cos[p, i] == np.float32(math.cos(ang)) and sin[p, i] == np.float32(math.sin(ang))
    assert np.all(cos[0] == 1) and np.all(sin[0] == 0)


def test_d2_is_a_plane_rotation():
    # d = 2: one pair, y = R(angle) x with R = [[c, -s], [s, c]]
    ang = np.array([0.0, 0.3, -1.1, math.pi / 2])
    X = np.array([[1.0, 0.0], [2.0, -1.0], [0.5, 0.25], [3.0, 4.0]])
    Y = O.rope_rotate(X, np.cos(ang)[:, None], np.sin(ang)[:, None])
    for a, x, y in zip(ang, X, Y):
        R = np.array([[math.cos(a), -math.sin(a)], [math.sin(a), math.cos(a)]])
        np.testing.assert_allclose(y, R @ x, rtol=0, atol=1e-15)
    np.testing.assert_allclose(Y[3], [-4.0, 3.0], atol=1e-15)       # quarter turn of (3, 4)


def test_position_zero_is_identity_and_pair_norms_are_kept():
    X = _rand(7, 16, 1)
    cos, sin = synth.rope_tables(7, 16)
    Y = O.rope_rotate(X, cos, sin)
    np.testing.assert_array_equal(Y[0], X[0])
    h = 8
    np.testing.assert_allclose(Y[:, :h] ** 2 + Y[:, h:] ** 2, X[:, :h] ** 2 + X[:, h:] ** 2, rtol=1e-6)


def test_against_complex_multiplication_in_torch():
    # independent formulation: the pair (x_i, x_{i+d/2}) as a complex number times exp(i * angle)
    n, d = 33, 64
    X = _rand(n, d, 2)
    i = torch.arange(d // 2, dtype=torch.float64)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * 10000.0 ** (-2.0 * i / d)[None, :]
    z = torch.complex(torch.from_numpy(X[:, :d // 2]), torch.from_numpy(X[:, d // 2:])) * torch.polar(torch.ones_like(ang), ang)
    want = torch.cat([z.real, z.imag], dim=1).numpy()
    got = O.rope_rotate(X, np.cos(ang.numpy()), np.sin(ang.numpy()))
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-13)


def test_inner_products_depend_on_the_position_difference_only():
    # the defining property of the rotary embedding: <R_p q, R_s k> = <R_{p-s} q, k>
    d = 32
    q, k = _rand(1, d, 3), _rand(1, d, 4)
    i = np.arange(d // 2)
    freq = 10000.0 ** (-2.0 * i / d)

    def rot(x, p):
        return O.rope_rotate(x, np.cos(p * freq)[None], np.sin(p * freq)[None])[0]

    for p, s in [(5, 2), (100, 97), (7, 7), (0, 9)]:
        np.testing.assert_allclose(rot(q, p) @ rot(k, s), rot(q, p - s) @ k[0], rtol=1e-10, atol=1e-10)


def test_rotations_compose_by_adding_positions():
    d = 16
    x = _rand(1, d, 5)
    freq = 10000.0 ** (-2.0 * np.arange(d // 2) / d)
    r = lambda v, p: O.rope_rotate(v, np.cos(p * freq)[None], np.sin(p * freq)[None])
    np.testing.assert_allclose(r(r(x, 3), 11), r(x, 14), rtol=0, atol=1e-12)


def test_bf16_rounding_against_torch():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 6, 20000),
                        # exact ties between neighbouring bf16 values, both parities
                        np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(2.0 + 2.0 ** -7), 0.0, -0.0, 255.5, 256.5 * 2])])
    x32 = x.astype(np.float32)                       # torch rounds from fp32: compare on fp32-representable inputs
    want = torch.from_numpy(x32).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.round_bf16_bits(x32.astype(np.float64))
    np.testing.assert_array_equal(got, want)


def test_cr_rope_uses_the_new_positions_not_the_old_ones():
    # Sec. 3.5: after distillation the kept entries are re-embedded at 0 .. |C|-1
    n, d, k = 40, 16, 9
    K = np.random.default_rng(7).standard_normal((n, d)).astype(np.float32)
    keep = np.array([1, 4, 5, 11, 17, 18, 30, 31, 39])
    cos, sin = synth.rope_tables(n, d)
    got = O.cr_rope(K[keep], cos, sin)
    want = O.rope_rotate(K[keep].astype(np.float64), cos[np.arange(k)], sin[np.arange(k)]).astype(np.float32)
    np.testing.assert_array_equal(got, want)
    old = O.rope_rotate(K[keep].astype(np.float64), cos[keep], sin[keep]).astype(np.float32)
    assert not np.array_equal(got[1:], old[1:])      # positions 4, 5, ... would give something else
    np.testing.assert_array_equal(got[0], K[keep[0]])  # new position 0: unrotated


def test_compress_returns_rotated_kept_keys():
    rng = np.random.default_rng(8)
    B, L, Hq, Hkv, P, d, n, k = 1, 1, 2, 1, 3, 8, 12, 5
    Q = rng.standard_normal((B, L, Hq, P, d)).astype(np.float32)
    K = rng.standard_normal((B, L, Hkv, n, d)).astype(np.float32)
    V = rng.standard_normal((B, L, Hkv, n, d)).astype(np.float32)
    nov = rng.random((B, n)).astype(np.float32)
    cos, sin = synth.rope_tables(k, d)
    out = O.compress(Q, K, V, nov, k=k, T=2, rope_cos=cos, rope_sin=sin)
    keep = out["keep_idx"][0, 0, 0]
    np.testing.assert_array_equal(out["K"][0, 0, 0], K[0, 0, 0][keep])          # the pot keeps pre-RoPE keys
    np.testing.assert_array_equal(out["K_rot"][0, 0, 0], O.cr_rope(K[0, 0, 0][keep], cos, sin))
    assert O.compress(Q, K, V, nov, k=k, T=2)["K_rot"] is None


@pytest.mark.parametrize("mistake", ["sign", "interleaved", "old_positions", "swapped_tables"])
def test_planted_mistakes_fail_the_pins(mistake):
    """A plausible slip in the rotation must break at least one of the pins above."""
    def bad_rotate(X, cos, sin):
        X = np.asarray(X, dtype=np.float64)
        h = X.shape[-1] // 2
        if mistake == "sign":
            return np.concatenate([X[..., :h] * cos + X[..., h:] * sin, X[..., h:] * cos - X[..., :h] * sin], axis=-1)
        if mistake == "interleaved":                  # pairs (2i, 2i+1) instead of (i, i + d/2)
            Y = np.empty_like(X)
            Y[..., 0::2] = X[..., 0::2] * cos - X[..., 1::2] * sin
            Y[..., 1::2] = X[..., 1::2] * cos + X[..., 0::2] * sin
            return Y
        if mistake == "swapped_tables":
            return O.rope_rotate(X, sin, cos)
        return O.rope_rotate(X, cos, sin)

    n, d = 6, 8
    X = _rand(n, d, 9)
    i = torch.arange(d // 2, dtype=torch.float64)
    ang = torch.arange(n, dtype=torch.float64)[:, None] * 10000.0 ** (-2.0 * i / d)[None, :]
    if mistake == "old_positions":
        keep = np.array([0, 2, 3, 5])
        got = bad_rotate(X[keep], np.cos(ang.numpy())[keep], np.sin(ang.numpy())[keep])
        want_rows = ang[: len(keep)]
        Xs = X[keep]
    else:
        got = bad_rotate(X, np.cos(ang.numpy()), np.sin(ang.numpy()))
        want_rows, Xs = ang, X
    z = torch.complex(torch.from_numpy(Xs[:, :d // 2].copy()), torch.from_numpy(Xs[:, d // 2:].copy())) * torch.polar(torch.ones_like(want_rows), want_rows)
    want = torch.cat([z.real, z.imag], dim=1).numpy()
    assert not np.allclose(got, want, atol=1e-9)
