"""Pins for the float64 attention checker (CPU only).

The paper prints no value for the decode step (black-box backend, Section 7), so the
checker is pinned by what mathematics fixes: an independently written brute force, a library
routine, closed forms, invariants, and a hand-derived rational fixture."""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

from oracle import reference as ref
from tests.helpers import (D, PAGE, Paged, bf16_round, bits_to_f64, brute_force, random_logical,
                           to_bf16_bits)

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def run_oracle(pg: Paged, q, scale, Hq):
    return ref.decode_attn(to_bf16_bits(q), pg.k_bits, pg.v_bits, pg.ptab, pg.stab, pg.plens,
                           pg.slens, pg.gos, scale, Hq, pg.Hkv)


def make(rng, NG=2, G=3, P=(19, 32), S=None, Hq=4, Hkv=2, **kw):
    NS = NG * G
    S = S if S is not None else [int(x) for x in rng.integers(0, 40, NS)]
    lg = random_logical(rng, NG, G, list(P), list(S), Hq, Hkv)
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng, **kw)
    return lg, pg


def test_brute_force_tiny_odd_lengths():
    rng = np.random.default_rng(11)
    for trial in range(4):
        NG, G = 2, 3
        P = [int(x) for x in rng.integers(0, 37, NG)]
        S = [int(x) for x in rng.integers(0, 40, NG * G)]
        S[0] = 0
        if trial == 0:
            P[0] = 0      # a sequence with no token at all -> zeros
        Hq, Hkv = (6, 2) if trial % 2 else (4, 4)
        lg, pg = make(rng, NG, G, P, S, Hq, Hkv)
        scale = 1 / math.sqrt(D)
        got = run_oracle(pg, lg["q"], scale, Hq)
        want = brute_force(lg["q"], lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], scale, Hq, Hkv)
        assert np.abs(got - want).max() <= 1e-12
        if trial == 0:
            assert np.all(got[0] == 0.0)


def test_library_sdpa_float64():
    rng = np.random.default_rng(5)
    Hq, Hkv = 8, 2
    lg, pg = make(rng, 2, 2, (33, 7), [5, 16, 1, 23], Hq, Hkv)
    scale = 0.11
    got = run_oracle(pg, lg["q"], scale, Hq)
    for s in range(4):
        g = int(lg["gos"][s])
        K = torch.from_numpy(np.concatenate([lg["pk"][g], lg["sk"][s]])).double()  # [L,Hkv,D]
        V = torch.from_numpy(np.concatenate([lg["pv"][g], lg["sv"][s]])).double()
        K = K.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)                 # [Hq,L,D]
        V = V.repeat_interleave(Hq // Hkv, dim=1).permute(1, 0, 2)
        Q = torch.from_numpy(lg["q"][s]).double()[:, None, :]                      # [Hq,1,D]
        o = torch.nn.functional.scaled_dot_product_attention(Q, K, V, scale=scale)[:, 0, :]
        assert np.abs(got[s] - o.numpy()).max() <= 1e-12


def test_golden_rational_weights():
    lines = [l.split() for l in open(os.path.join(GOLD, "attn_rational_weights.txt"))
             if l.strip() and not l.startswith("#")]
    rec = {l[0]: l[1:] for l in lines}
    dots = [int(x) for x in rec["dots"]]
    k = np.zeros((3, 1, D), np.float32); v = np.zeros((3, 1, D), np.float32)
    for j in range(3):
        k[j, 0, 0] = dots[j]
        v[j, 0, :4] = [float(x) for x in rec[f"v{j}"]]
    q = np.zeros((1, 1, D), np.float32); q[0, 0, 0] = 1.0
    rng = np.random.default_rng(0)
    pg = Paged([np.zeros((0, 1, D), np.float32)], [np.zeros((0, 1, D), np.float32)], [k], [v], [0], 1, rng)
    w, out = ref.attn_weights(0, 0, to_bf16_bits(q), pg.k_bits, pg.v_bits, pg.ptab, pg.stab,
                              pg.plens, pg.slens, pg.gos, math.log(2.0), 1, 1)
    want_w = [float(Fraction(x)) for x in rec["weights"]]
    want_o = [float(Fraction(x)) for x in rec["out"]]
    assert np.abs(w - want_w).max() <= 1e-15
    assert np.abs(out[:4] - want_o).max() <= 1e-14
    assert np.all(out[4:] == 0)
    full = run_oracle(pg, q, math.log(2.0), 1)
    assert np.array_equal(full[0, 0], out)


def test_page_permutation_is_bit_identical():
    rng = np.random.default_rng(3)
    lg = random_logical(rng, 2, 2, [21, 48], [9, 0, 31, 16], 4, 2)
    a = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, np.random.default_rng(1))
    b = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, np.random.default_rng(2), spare=9)
    c = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, rng, order="identity")
    assert not np.array_equal(a.ptab, b.ptab)
    oa, ob, oc = (run_oracle(x, lg["q"], 0.09, 4) for x in (a, b, c))
    assert np.array_equal(oa, ob) and np.array_equal(oa, oc)


def test_private_prefix_copies_give_same_result():
    """Sharing is only a storage matter: giving every sequence its own copy of the prefix
    pages (group_of_seq = identity) must not change anything."""
    rng = np.random.default_rng(8)
    NG, G = 2, 3
    lg = random_logical(rng, NG, G, [18, 35], [4, 17, 0, 8, 33, 1], 4, 2)
    shared = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, rng)
    pk = [lg["pk"][g] for g in lg["gos"]]; pv = [lg["pv"][g] for g in lg["gos"]]
    private = Paged(pk, pv, lg["sk"], lg["sv"], np.arange(NG * G), 2, rng)
    assert np.array_equal(run_oracle(shared, lg["q"], 0.1, 4), run_oracle(private, lg["q"], 0.1, 4))


def test_identical_samples_give_identical_rows_and_gqa_rows():
    rng = np.random.default_rng(9)
    G, Hq, Hkv = 4, 4, 2
    lg = random_logical(rng, 1, G, [27], [13] * G, Hq, Hkv)
    for s in range(1, G):   # same query, same generated tokens
        lg["q"][s] = lg["q"][0]; lg["sk"][s] = lg["sk"][0]; lg["sv"][s] = lg["sv"][0]
    lg["q"][:, 1] = lg["q"][:, 0]          # heads 0,1 share KV head 0 and now share the query
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng)
    o = run_oracle(pg, lg["q"], 0.2, Hq)
    for s in range(1, G):
        assert np.array_equal(o[s], o[0])
    assert np.array_equal(o[:, 0], o[:, 1])
    assert not np.array_equal(o[:, 0], o[:, 2])   # a different KV head differs


def test_softmax_weights_sum_to_one_and_hull():
    rng = np.random.default_rng(2)
    lg, pg = make(rng, 2, 2, (40, 5), [12, 3, 30, 0], 4, 2)
    qb = to_bf16_bits(lg["q"])
    for s in range(4):
        for h in range(4):
            w, out = ref.attn_weights(s, h, qb, pg.k_bits, pg.v_bits, pg.ptab, pg.stab, pg.plens,
                                      pg.slens, pg.gos, 0.3, 4, 2)
            L = len(w)
            assert L == pg.plens[pg.gos[s]] + pg.slens[s]
            assert abs(w.sum() - 1.0) <= 1e-14 * L and (w >= 0).all()
            g = int(lg["gos"][s]); kh = h // 2
            Vc = np.concatenate([lg["pv"][g], lg["sv"][s]])[:, kh, :].astype(np.float64)
            assert (out <= Vc.max(0) + 1e-12).all() and (out >= Vc.min(0) - 1e-12).all()
            assert np.abs(out - w @ Vc).max() <= 1e-13


def test_closed_forms():
    rng = np.random.default_rng(4)
    Hq, Hkv, P, S = 2, 1, 20, 11
    lg = random_logical(rng, 1, 1, [P], [S], Hq, Hkv)
    # all keys equal -> uniform weights -> mean of values
    lg2 = dict(lg); krow = lg["pk"][0][0:1]
    lg2["pk"] = [np.repeat(krow, P, 0)]; lg2["sk"] = [np.repeat(krow, S, 0)]
    pg = Paged(lg2["pk"], lg["pv"], lg2["sk"], lg["sv"], lg["gos"], Hkv, rng)
    o = run_oracle(pg, lg["q"], 0.5, Hq)
    mean = np.concatenate([lg["pv"][0], lg["sv"][0]])[:, 0, :].astype(np.float64).mean(0)
    assert np.abs(o[0] - mean[None, :]).max() <= 1e-14
    # q = 0 -> mean of values
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng)
    o = run_oracle(pg, np.zeros_like(lg["q"]), 0.5, Hq)
    assert np.abs(o[0] - mean[None, :]).max() <= 1e-14
    # constant values -> that constant
    cv = bf16_round(np.linspace(-2, 2, D))[None, None, :]
    pg = Paged(lg["pk"], [np.repeat(cv, P, 0)], lg["sk"], [np.repeat(cv, S, 0)], lg["gos"], Hkv, rng)
    o = run_oracle(pg, lg["q"], 0.5, Hq)
    assert np.abs(o[0] - cv[0]).max() <= 1e-14
    # a single token -> its value row, exactly
    one = random_logical(rng, 1, 1, [0], [1], Hq, Hkv)
    pg = Paged(one["pk"], one["pv"], one["sk"], one["sv"], one["gos"], Hkv, rng)
    o = run_oracle(pg, one["q"], 0.5, Hq)
    assert np.array_equal(o[0, 0], one["sv"][0][0, 0].astype(np.float64))
    # one key far ahead of the rest -> (almost) its value row
    dom = random_logical(rng, 1, 1, [9], [6], 1, 1)
    dom["q"][:] = 0; dom["q"][0, 0, 0] = 1.0
    for arr in dom["pk"] + dom["sk"]:
        arr[:, :, 0] = 0.0
    dom["sk"][0][3, 0, 0] = 64.0       # score 64*scale=... ahead by 64 with scale 1
    pg = Paged(dom["pk"], dom["pv"], dom["sk"], dom["sv"], dom["gos"], 1, rng)
    o = run_oracle(pg, dom["q"], 1.0, 1)
    assert np.abs(o[0, 0] - dom["sv"][0][3, 0].astype(np.float64)).max() <= 1e-20 + 14 * math.exp(-64) * 8


def test_poison_never_read():
    rng = np.random.default_rng(6)
    lg = random_logical(rng, 2, 2, [17, 30], [5, 19, 0, 33], 4, 2)
    outs = []
    for poison in (np.nan, np.inf, 0.0, 123.0):
        pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 2, np.random.default_rng(1),
                   spare=4, poison=poison)
        outs.append(run_oracle(pg, lg["q"], 0.1, 4))
    assert np.isfinite(outs[0]).all()
    for o in outs[1:]:
        assert np.array_equal(o, outs[0])
    # padding of the tables is never dereferenced: any value behind the valid pages is fine
    pg.ptab[pg.ptab < 0] = 10 ** 9
    pg.stab[pg.stab < 0] = -12345
    assert np.array_equal(run_oracle(pg, lg["q"], 0.1, 4), outs[0])


def test_split_and_merge_algebra():
    """Cutting the token range anywhere, summarising each piece by (max, sum, weighted values)
    and merging gives the unsplit result."""
    rng = np.random.default_rng(12)
    P, S = 37, 58
    lg = random_logical(rng, 1, 1, [P], [S], 1, 1)
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], 1, rng)
    scale = 0.17
    want = run_oracle(pg, lg["q"], scale, 1)[0, 0]
    Kc = np.concatenate([lg["pk"][0], lg["sk"][0]])[:, 0].astype(np.float64)
    Vc = np.concatenate([lg["pv"][0], lg["sv"][0]])[:, 0].astype(np.float64)
    x = scale * (Kc @ lg["q"][0, 0].astype(np.float64))
    for cuts in ([0, P, P + S], [0, 1, 2, 50, 95], [0, 0, 33, 33, 95], list(range(0, 96, 5)) + [95]):
        parts = [ref.slice_summary(x[a:b], Vc[a:b]) for a, b in zip(cuts[:-1], cuts[1:])]
        got = ref.merge_summaries(parts)
        assert np.abs(got - want).max() <= 1e-12
    assert np.all(ref.merge_summaries([ref.slice_summary(x[:0], Vc[:0])]) == 0)


def test_scale_invariance_power_of_two():
    rng = np.random.default_rng(13)
    lg, pg = make(rng, 1, 2, (25,), [7, 30], 2, 1)
    a = run_oracle(pg, lg["q"], 0.25, 2)
    b = run_oracle(pg, lg["q"] * 4.0, 0.0625, 2)     # exact rescaling in bf16 and float64
    assert np.array_equal(a, b)


def test_layout_is_the_documented_one():
    """K is [page][kv_head][slot][channel]; V is [page][kv_head][channel][slot]: build the
    arrays by hand (not through the helper) for a single page."""
    Hkv = 2
    K = np.zeros((1, Hkv, PAGE, D), np.float32); V = np.zeros((1, Hkv, D, PAGE), np.float32)
    # two tokens in the suffix; head 1 (kv head 1) only
    K[0, 1, 0, 5] = 1.0; K[0, 1, 1, 5] = 2.0
    V[0, 1, 7, 0] = 3.0; V[0, 1, 7, 1] = 1.0
    q = np.zeros((1, 2, D), np.float32); q[0, 1, 5] = 1.0
    out = ref.decode_attn(to_bf16_bits(q), to_bf16_bits(K), to_bf16_bits(V), np.zeros((1, 1), np.int32),
                          np.zeros((1, 1), np.int32), [0], [2], [0], math.log(3.0), 2, Hkv)
    # weights (e^{ln3*1}, e^{ln3*2}) = (3, 9)/12
    assert abs(out[0, 1, 7] - (3 * 3.0 + 9 * 1.0) / 12) <= 1e-15
    assert np.count_nonzero(out) == 1
