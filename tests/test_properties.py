"""Property tests (hypothesis) of the CPU-side pieces: the work-list reference covers every
token exactly once for arbitrary shapes, and the checker equals the brute force on random tiny
problems."""
import math

import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import plan_ref
from oracle import reference as ref
from tests.helpers import D, Paged, brute_force, random_logical, to_bf16_bits


@settings(max_examples=40, deadline=None)
@given(st.integers(1, 6), st.integers(1, 5), st.sampled_from([(4, 4), (8, 2), (28, 4), (16, 1)]),
       st.sampled_from([32, 64, 96, 256]), st.sampled_from([32, 128]), st.integers(0, 2 ** 31 - 1))
def test_plan_covers_every_token_once(NG, Gmax, heads, Cs, Cp, seed):
    Hq, Hkv = heads
    rng = np.random.default_rng(seed)
    sizes = rng.integers(0, Gmax + 1, NG)
    gos = rng.permutation(np.repeat(np.arange(NG), sizes))
    pl = rng.integers(0, 300, NG); sl = rng.integers(0, 400, len(gos))
    p = plan_ref.build_plan(pl, sl, gos, Hq, Hkv, 19, 25, Cs, Cp)
    assert p.flags == 0
    tok = np.zeros(len(gos), int)
    for (s, a, b, _) in p.suffix_items:
        assert 0 <= a < b <= sl[s] and b - a <= Cs and a % Cs == 0
        tok[s] += b - a
    assert np.array_equal(tok, sl)
    R = Hq // Hkv
    QB = plan_ref.rows_per_qblock(len(gos), NG, Hq, Hkv)
    for g in range(NG):
        rows = int(sizes[g]) * R
        cover = np.zeros((rows, int(pl[g])), int)
        for (gg, a, b, r) in p.prefix_items:
            if gg == g:
                cover[r:r + QB, a:b] += 1
        assert (cover == 1).all()
    assert p.num_long_suffix_items == sum(1 for it in p.suffix_items if it[2] - it[1] > 128)
    for s in range(len(gos)):
        assert p.seq_chunks[s] == (math.ceil(pl[gos[s]] / Cp) | (math.ceil(sl[s] / Cs) << 16))


@settings(max_examples=15, deadline=None)
@given(st.integers(1, 3), st.integers(1, 3), st.sampled_from([(4, 2), (3, 3), (8, 1)]), st.integers(0, 2 ** 31 - 1))
def test_checker_equals_brute_force_on_random_tiny_problems(NG, G, heads, seed):
    Hq, Hkv = heads
    rng = np.random.default_rng(seed)
    P = [int(x) for x in rng.integers(0, 40, NG)]
    S = [int(x) for x in rng.integers(0, 40, NG * G)]
    lg = random_logical(rng, NG, G, P, S, Hq, Hkv)
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng)
    scale = float(rng.uniform(0.02, 0.3))
    got = ref.decode_attn(to_bf16_bits(lg["q"]), pg.k_bits, pg.v_bits, pg.ptab, pg.stab, pg.plens, pg.slens,
                          pg.gos, scale, Hq, Hkv)
    want = brute_force(lg["q"], lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], scale, Hq, Hkv)
    assert np.abs(got - want).max() <= 1e-12
