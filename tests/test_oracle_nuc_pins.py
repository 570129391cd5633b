"""Pins for the oracle's NuC-from-logits step (Sec. 3.3.2, Eq. 3): per-token cross entropy.

Expected values come from closed forms, invariants and torch's cross_entropy on the CPU - never from the oracle
itself or from the GPU path.
"""
import math

import numpy as np
import pytest
import torch

from oracle import ccd_oracle as O


def test_uniform_logits_give_log_vocabulary():
    for V in (1, 2, 7, 1000):
        z = np.full((3, V), 2.5, dtype=np.float32)
        np.testing.assert_allclose(O.nuc_from_logits(z, np.array([0, V - 1, V // 2])), math.log(V), rtol=1e-6, atol=1e-7)


def test_two_way_closed_form():
    # softmax over (a, b): -log(e^a / (e^a + e^b)) = log(1 + e^(b - a))
    z = np.array([[1.0, 3.0], [0.0, -4.0], [10.0, 10.0]], dtype=np.float32)
    got = O.nuc_from_logits(z, np.array([0, 0, 1]))
    want = [math.log1p(math.exp(2.0)), math.log1p(math.exp(-4.0)), math.log(2.0)]
    np.testing.assert_allclose(got, want, rtol=1e-6)


def test_against_torch_cross_entropy():
    rng = np.random.default_rng(0)
    z = (rng.standard_normal((50, 333)) * 5).astype(np.float32)
    y = rng.integers(0, 333, 50)
    want = torch.nn.functional.cross_entropy(torch.from_numpy(z).double(), torch.from_numpy(y), reduction="none").numpy()
    np.testing.assert_allclose(O.nuc_from_logits(z, y), want.astype(np.float32), rtol=1e-6, atol=1e-6)


def test_shift_of_a_row_changes_nothing_and_huge_logits_do_not_overflow():
    rng = np.random.default_rng(1)
    z = rng.standard_normal((4, 64))
    y = np.array([3, 0, 63, 17])
    a = O.nuc_from_logits(z.astype(np.float32), y)
    b = O.nuc_from_logits((z + 1000.0), y)                      # fp64 input path
    np.testing.assert_allclose(a, b, rtol=1e-5, atol=1e-5)
    big = np.array([[3.0e4, 0.0, -3.0e4]], dtype=np.float32)    # exp would overflow without the max shift
    np.testing.assert_allclose(O.nuc_from_logits(big, np.array([1])), [3.0e4], rtol=1e-6)


def test_bf16_inputs_are_taken_at_their_exact_value():
    bits = np.array([[0x3F80, 0x4000, 0xBF80]], dtype=np.uint16)   # 1.0, 2.0, -1.0
    want = math.log(math.e + math.e ** 2 + 1 / math.e) - 2.0
    np.testing.assert_allclose(O.nuc_from_logits(bits, np.array([1])), [want], rtol=1e-6)


def test_label_outside_the_vocabulary_gives_minus_infinity():
    z = np.zeros((3, 5), dtype=np.float32)
    got = O.nuc_from_logits(z, np.array([-100, 5, 2]))
    assert got[0] == -np.inf and got[1] == -np.inf and np.isclose(got[2], math.log(5))
    # such a token never takes a NuC slot (Sec. 3.3.3 step 1)
    assert 0 not in O.nuc_slots(got, 3) and 1 not in O.nuc_slots(got, 3)


def test_rare_token_is_more_novel_than_a_likely_one():
    # the meaning of Eq. 3: low probability under the model = high novelty
    z = np.array([[5.0, 0.0, 0.0, 0.0]] * 2, dtype=np.float32)
    got = O.nuc_from_logits(z, np.array([0, 3]))
    assert got[1] > got[0] > 0


@pytest.mark.parametrize("mistake", ["no_minus", "softmax_over_rows", "label_off_by_one", "mean_not_sum"])
def test_planted_mistakes_fail_the_pins(mistake):
    rng = np.random.default_rng(2)
    z = (rng.standard_normal((6, 9)) * 3).astype(np.float64)
    y = np.array([1, 0, 8, 4, 4, 2])
    if mistake == "no_minus":
        bad = z[np.arange(6), y] - np.log(np.exp(z).sum(axis=1))
    elif mistake == "softmax_over_rows":
        bad = np.log(np.exp(z).sum(axis=0))[y] - z[np.arange(6), y]
    elif mistake == "label_off_by_one":
        bad = np.log(np.exp(z).sum(axis=1)) - z[np.arange(6), (y + 1) % 9]
    else:
        bad = np.log(np.exp(z).mean(axis=1)) - z[np.arange(6), y]
    want = torch.nn.functional.cross_entropy(torch.from_numpy(z), torch.from_numpy(y), reduction="none").numpy()
    assert not np.allclose(bad, want, atol=1e-6)
    np.testing.assert_allclose(O.nuc_from_logits(z, y), want.astype(np.float32), rtol=1e-6, atol=1e-6)
