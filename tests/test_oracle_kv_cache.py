"""Pins for the KV-cache maintenance reference (CPU only): appending through the reference and
then reading through the attention checker must equal brute-force attention over the logical
token lists with the new tokens added; a forked sequence must see its parent's tokens."""
import numpy as np

from oracle import reference as ref
from tests.helpers import D, PAGE, Paged, bf16_round, brute_force, random_logical, to_bf16_bits


def test_append_then_attend_equals_logical_append():
    rng = np.random.default_rng(31)
    Hq, Hkv, NG, G = 4, 2, 2, 2
    S = [15, 16, 0, 33]                      # next token lands in slot 15, on a new page, first ever, slot 1
    lg = random_logical(rng, NG, G, [20, 7], S, Hq, Hkv)
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng, spare=8)
    stab = np.full((4, 4), -1, np.int32); stab[:, :pg.stab.shape[1]] = pg.stab
    free = [p for p in range(pg.num_pages) if p not in set(pg.ptab.ravel()) | set(pg.stab.ravel())]
    for s in range(4):                       # the scheduler's part: a page for a token that starts one
        if S[s] % PAGE == 0:
            stab[s, S[s] // PAGE] = free.pop()
    k_new = bf16_round(rng.standard_normal((4, Hkv, D))); v_new = bf16_round(rng.standard_normal((4, Hkv, D)))
    k2, v2, lens2, flags = ref.kv_append(pg.k_bits, pg.v_bits, stab, pg.slens, to_bf16_bits(k_new), to_bf16_bits(v_new))
    assert flags == 0 and list(lens2) == [s + 1 for s in S]
    got = ref.decode_attn(to_bf16_bits(lg["q"]), k2, v2, pg.ptab, stab, pg.plens, lens2, pg.gos, 0.1, Hq, Hkv)
    sk = [np.concatenate([lg["sk"][s], k_new[s][None]]) for s in range(4)]
    sv = [np.concatenate([lg["sv"][s], v_new[s][None]]) for s in range(4)]
    want = brute_force(lg["q"], lg["pk"], lg["pv"], sk, sv, lg["gos"], 0.1, Hq, Hkv)
    assert np.abs(got - want).max() <= 1e-12
    # nothing but the four target slots changed
    changed_k = np.argwhere((k2 != pg.k_bits).any(axis=(1, 3)))
    assert len(changed_k) <= 4 and len({tuple(x) for x in changed_k.tolist()}) == len(changed_k)


def test_append_skips_full_rows_and_bad_pages():
    K = np.zeros((3, 1, PAGE, D), np.uint16); V = np.zeros((3, 1, D, PAGE), np.uint16)
    stab = np.array([[0], [7], [2]], np.int32)
    lens = np.array([16, 3, 5], np.int32)              # row full / page id out of range / fine
    kn = np.full((3, 1, D), 9, np.uint16); vn = np.full((3, 1, D), 8, np.uint16)
    k2, v2, l2, flags = ref.kv_append(K, V, stab, lens, kn, vn)
    assert flags == 6 and list(l2) == [16, 3, 6]
    assert (k2[2, 0, 5] == 9).all() and (v2[2, 0, :, 5] == 8).all()
    assert k2.sum() == 9 * D and v2.sum() == 8 * D


def test_fork_by_page_copy_sees_the_parents_tokens():
    rng = np.random.default_rng(33)
    Hq, Hkv = 4, 2
    lg = random_logical(rng, 1, 1, [10], [21], Hq, Hkv)
    pg = Paged(lg["pk"], lg["pv"], lg["sk"], lg["sv"], lg["gos"], Hkv, rng, spare=6)
    used = set(pg.ptab.ravel()) | set(pg.stab.ravel())
    free = [p for p in range(pg.num_pages) if p not in used]
    # child: shares the parent's full first suffix page, gets a copy of the partial second one
    src, dst = [int(pg.stab[0, 1])], [free[0]]
    k2, v2, flags = ref.kv_copy_pages(pg.k_bits, pg.v_bits, src, dst)
    assert flags == 0
    stab = np.array([pg.stab[0], [pg.stab[0, 0], free[0]]], np.int32)
    q2 = np.concatenate([lg["q"], lg["q"]])
    out = ref.decode_attn(to_bf16_bits(q2), k2, v2, pg.ptab, stab, pg.plens, [21, 21], [0, 0], 0.2, Hq, Hkv)
    assert np.array_equal(out[0], out[1])
    _, _, flags = ref.kv_copy_pages(pg.k_bits, pg.v_bits, [0, 99], [1, 2])
    assert flags == 4
