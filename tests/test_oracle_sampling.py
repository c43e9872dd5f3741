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


# ---- top-p (nucleus) sampling -------------------------------------------------------------------
def _pow2_row():
    rec = {l.split()[0]: l.split()[1:] for l in open(os.path.join(GOLD, "logprob_powers_of_two.txt"))
           if l.strip() and not l.startswith("#")}
    return to_bf16_bits(np.array([[float(v) for v in rec["logits"]]], np.float32)), 1.0 / math.log(2.0)


def test_top_p_on_the_powers_of_two_row():
    """Probabilities 1/15, 2/15, 4/15, 8/15 for tokens 0..3: the ranking is 3, 2, 1, 0 with running
    mass 8/15, 12/15, 14/15, 1."""
    x, T = _pow2_row()
    p, _ = ref.softmax_cdf(x[0], T)
    assert list(ref.nucleus(p, 0.5)) == [False, False, False, True]          # 8/15 >= 0.5
    assert list(ref.nucleus(p, 0.54)) == [False, False, True, True]          # needs 12/15
    assert list(ref.nucleus(p, 0.81)) == [False, True, True, True]           # needs 14/15
    assert list(ref.nucleus(p, 0.9334)) == [True, True, True, True]          # 14/15 = 0.93333 is not enough
    # nucleus {2, 3} has mass 12/15; in index order token 2 covers u < 1/3, token 3 the rest
    tok, lp = ref.sample_tokens_top_p(np.repeat(x, 4, 0), [0.0, 0.33, 0.34, 0.999], T, 0.6)
    assert list(tok) == [2, 2, 3, 3]
    want = [math.log(4 / 15), math.log(4 / 15), math.log(8 / 15), math.log(8 / 15)]   # of the full distribution
    assert np.abs(lp - want).max() <= 1e-14


def test_top_p_one_is_plain_sampling_and_tiny_top_p_is_argmax():
    rng = np.random.default_rng(8)
    x = to_bf16_bits(bf16_round(rng.standard_normal((30, 200)) * 3))
    u = rng.random(30)
    t1, l1 = ref.sample_tokens_top_p(x, u, 0.9, 1.0)
    t0, l0 = ref.sample_tokens(x, u, 0.9)
    assert np.array_equal(t1, t0) and np.array_equal(l1, l0)
    ta, _ = ref.sample_tokens_top_p(x, u, 0.9, 1e-9)
    assert np.array_equal(ta, ref.bf16_bits_to_f64(x).argmax(axis=1))        # argmax: first index among equals


def test_top_p_ties_keep_the_lower_indices():
    x = to_bf16_bits(np.full((1, 4), 0.75, np.float32))                      # four tokens of probability 1/4
    p, _ = ref.softmax_cdf(x[0], 1.0)
    assert list(ref.nucleus(p, 0.5)) == [True, True, False, False]
    assert list(ref.nucleus(p, 0.51)) == [True, True, True, False]
    tok, _ = ref.sample_tokens_top_p(np.repeat(x, 3, 0), [0.1, 0.6, 0.99], 1.0, 0.5)
    assert list(tok) == [0, 1, 1]


def test_nucleus_is_sufficient_minimal_and_made_of_the_most_probable_tokens():
    rng = np.random.default_rng(12)
    for top_p in (0.1, 0.5, 0.9, 0.999):
        x = to_bf16_bits(bf16_round(rng.standard_normal((1, 500)) * 2.5))
        p, _ = ref.softmax_cdf(x[0], 1.0)
        keep = ref.nucleus(p, top_p)
        assert p[keep].sum() >= top_p
        assert p[keep].sum() - p[keep].min() < top_p                          # dropping its smallest member breaks it
        assert p[keep].min() >= p[~keep].max()


def test_top_p_frequencies_are_the_renormalised_probabilities():
    rng = np.random.default_rng(5)
    x = to_bf16_bits(bf16_round(rng.standard_normal((1, 12)) * 2))
    N = 20000
    u = (np.arange(N) + 0.5) / N
    tok, _ = ref.sample_tokens_top_p(np.repeat(x, N, 0), u, 0.8, 0.7)
    p, _ = ref.softmax_cdf(x[0], 0.8)
    keep = ref.nucleus(p, 0.7)
    counts = np.bincount(tok, minlength=12)
    assert (counts[~keep] == 0).all()
    assert np.abs(counts - np.where(keep, p, 0) / p[keep].sum() * N).max() <= 1.0 + 1e-9


def test_top_p_never_draws_a_masked_token():
    x = np.zeros((2, 8), np.float32); x[:, [0, 7]] = -np.inf
    x[1] = -np.inf
    tok, lp = ref.sample_tokens_top_p(to_bf16_bits(x), [0.9999999, 0.5], 1.0, 0.999)
    assert tok[0] == 6 and tok[1] == -1 and np.isnan(lp[1])
