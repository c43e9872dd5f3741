"""Pins for the inverse-CDF sampling reference (CPU only)."""
import math
import os
from fractions import Fraction

import numpy as np

from oracle import reference as ref
from tests.helpers import bf16_round, to_bf16_bits

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_golden_powers_of_two_cdf():
    """logits 0..3 at T = 1/ln 2 have probabilities 1/15, 2/15, 4/15, 8/15 (the fixture of the
    log-prob pins): the CDF steps are 1/15, 3/15, 7/15, 1."""
    rec = {l.split()[0]: l.split()[1:] for l in open(os.path.join(GOLD, "logprob_powers_of_two.txt"))
           if l.strip() and not l.startswith("#")}
    x = to_bf16_bits(np.array([[float(v) for v in rec["logits"]]] * 6, np.float32))
    u = [0.0, 0.066, 0.067, 0.19, 0.21, 0.999]
    tok, lp = ref.sample_tokens(x, u, 1.0 / math.log(2.0))
    assert list(tok) == [0, 0, 1, 1, 2, 3]
    want = [math.log(Fraction(rec["prob"][t])) for t in tok]
    assert np.abs(lp - want).max() <= 1e-14


def test_uniform_logits_give_floor_of_u_times_vocab():
    V = 1000
    x = to_bf16_bits(np.full((5, V), 1.5, np.float32))
    u = np.array([0.0, 0.0004, 0.5003, 0.7314, 0.99999])       # away from the CDF steps k/V
    tok, lp = ref.sample_tokens(x, u, 2.0)
    assert list(tok) == [math.floor(v * V + 1e-9) for v in u]
    assert np.abs(lp + math.log(V)).max() <= 1e-12


def test_frequencies_follow_the_probabilities():
    """A fine grid of uniforms lands on token t exactly round(p_t * N) +- 1 times."""
    rng = np.random.default_rng(3)
    x = to_bf16_bits(bf16_round(rng.standard_normal((1, 12)) * 2))
    N = 20000
    u = (np.arange(N) + 0.5) / N
    tok, _ = ref.sample_tokens(np.repeat(x, N, 0), u, 0.8)
    p, _ = ref.softmax_cdf(x[0], 0.8)
    counts = np.bincount(tok, minlength=12)
    assert np.abs(counts - p * N).max() <= 1.0 + 1e-9


def test_masked_entries_and_edges():
    x = np.zeros((3, 8), np.float32); x[:, [0, 7]] = -np.inf       # first and last token impossible
    xb = to_bf16_bits(x)
    tok, lp = ref.sample_tokens(xb, [0.0, 0.9999999, 1.0], 1.0)
    assert list(tok) == [1, 6, 6]                                   # u = 1: nothing exceeds it -> last possible token
    assert np.abs(lp + math.log(6)).max() <= 1e-12
    tok, lp = ref.sample_tokens(to_bf16_bits(np.full((1, 4), -np.inf, np.float32)), [0.3], 1.0)
    assert tok[0] == -1 and np.isnan(lp[0])


def test_logprob_agrees_with_the_logprob_checker():
    rng = np.random.default_rng(4)
    x = to_bf16_bits(bf16_round(rng.standard_normal((6, 300)) * 3))
    tok, lp = ref.sample_tokens(x, rng.random(6), 1.3)
    assert np.abs(lp - ref.token_logprobs(x, tok, 1.3)).max() <= 1e-12
