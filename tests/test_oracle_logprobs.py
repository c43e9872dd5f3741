"""Pins for the float64 log-probability checker (CPU only): closed forms, invariants, a
library routine and a hand-derived fixture (the paper prints no value for this step)."""
import math
import os
from fractions import Fraction

import numpy as np
import torch

from oracle import reference as ref
from tests.helpers import bf16_round, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def lp(x, tok, T=1.0):
    return ref.token_logprobs(to_bf16_bits(np.atleast_2d(x)), np.atleast_1d(tok), T)


def test_golden_powers_of_two():
    rec = {l.split()[0]: l.split()[1:] for l in open(os.path.join(GOLD, "logprob_powers_of_two.txt"))
           if l.strip() and not l.startswith("#")}
    logits = np.array([[float(v) for v in rec["logits"]]] * 4, np.float32)
    got = ref.token_logprobs(to_bf16_bits(logits), np.arange(4), 1.0 / math.log(2.0))
    want = [math.log(Fraction(p)) for p in rec["prob"]]
    assert np.abs(got - want).max() <= 1e-14


def test_probabilities_sum_to_one_small_vocab():
    rng = np.random.default_rng(1)
    V = 37
    x = bf16_round(rng.standard_normal((1, V)) * 3)
    rows = np.repeat(x, V, 0)
    got = ref.token_logprobs(to_bf16_bits(rows), np.arange(V), 0.7)
    assert abs(np.exp(got).sum() - 1.0) <= 1e-13


def test_uniform_logits():
    for V in (1, 2, 4096, 152064):
        x = np.full((1, V), 2.5, np.float32)
        assert abs(lp(x, V - 1, 3.0)[0] + math.log(V)) <= 1e-12


def test_shift_invariance_and_temperature():
    rng = np.random.default_rng(2)
    x = bf16_round(rng.integers(-40, 40, (3, 501)) / 8.0)      # multiples of 1/8: shifts stay exact
    tok = np.array([0, 500, 77])
    base = lp(x, tok, 1.0)
    assert np.abs(lp(x + 16.0, tok, 1.0) - base).max() <= 1e-12
    # dividing by a power-of-two temperature equals pre-dividing the logits, exactly
    assert np.array_equal(lp(x, tok, 4.0), lp(x / 4.0, tok, 1.0))
    assert np.array_equal(lp(x, tok, 0.5), lp(x * 2.0, tok, 1.0))


def test_library_log_softmax_float64():
    rng = np.random.default_rng(3)
    x = bf16_round(rng.standard_normal((5, 1000)) * 3)
    tok = rng.integers(0, 1000, 5)
    for T in (1.0, 0.5, 2.0, 1.3):
        want = torch.log_softmax(torch.from_numpy(x).double() / T, dim=-1).gather(
            1, torch.from_numpy(tok)[:, None])[:, 0].numpy()
        assert np.abs(lp(x, tok, T) - want).max() <= 1e-12


def test_one_dominant_logit_and_large_values():
    x = np.zeros((1, 300), np.float32); x[0, 17] = 200.0
    assert abs(lp(x, 17)[0]) <= 1e-30 + 299 * math.exp(-200)
    assert abs(lp(x, 3)[0] + 200.0) <= 1e-12
    big = np.full((1, 8), 3.0e4, np.float32)          # exp would overflow without the max shift
    assert abs(lp(big, 0)[0] + math.log(8)) <= 3.0e4 * 2 ** -50   # rounding of 3e4 - lse
