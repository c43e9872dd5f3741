"""The host reference of the work list: coverage and ordering properties (CPU only)."""
import numpy as np

from oracle import plan_ref


def test_every_token_is_covered_exactly_once():
    rng = np.random.default_rng(0)
    NG, G, Hq, Hkv = 5, 3, 8, 2
    pl = rng.integers(0, 700, NG); sl = rng.integers(0, 900, NG * G); sl[2] = 0; pl[1] = 0
    gos = rng.permutation(np.repeat(np.arange(NG), G))
    mpp, msp = 44, 57
    p = plan_ref.build_plan(pl, sl, gos, Hq, Hkv, mpp, msp, suffix_chunk=128, prefix_chunk=96)
    assert p.flags == 0
    for s in range(NG * G):
        spans = sorted((a, b) for (i, a, b, _) in p.suffix_items if i == s)
        assert [a for a, _ in spans] == list(range(0, int(sl[s]), 128))
        assert sum(b - a for a, b in spans) == sl[s]
        assert all(0 < b - a <= 128 for a, b in spans)
    R = Hq // Hkv
    for g in range(NG):
        rows = int(p.group_count[g]) * R
        items = [(a, b, r) for (i, a, b, r) in p.prefix_items if i == g]
        cover = np.zeros((max(rows, 1), max(int(pl[g]), 1)), int)
        for a, b, r in items:
            cover[r:min(rows, r + plan_ref.rows_per_qblock(NG * G, NG, Hq, Hkv)), a:b] += 1
        if rows and pl[g]:
            assert (cover == 1).all()
        else:
            assert not items
    for g in range(NG):
        seg = p.group_seqs[p.group_start[g]:p.group_start[g + 1]]
        assert list(seg) == sorted(np.nonzero(gos == g)[0])


def test_clamping_and_bad_group_flags():
    p = plan_ref.build_plan([40, -3], [10, 9999, 5], [0, 7, 1], 4, 2, 2, 3, 32, 32)
    assert p.flags == 3
    assert sorted(p.suffix_items) == [(0, 0, 10, 0), (1, 0, 32, 0), (1, 32, 48, 0), (2, 0, 5, 0)]
    assert sorted(p.prefix_items) == [(0, 0, 32, 0)]
    assert list(p.group_count) == [1, 1]


def test_default_chunk_rule():
    assert plan_ref.default_chunks(2048, 256, 28, 4, 128, 512) == (8192, 8192)
    assert plan_ref.default_chunks(16, 4, 8, 2, 16, 8) == (256, 256)
    assert plan_ref.default_chunks(256, 64, 64, 8, 512, 1536) == (8192, 8192)
    assert plan_ref.default_chunks(2048, 64, 28, 4, 256, 4) == (8192, 8192)      # 224 rows: two row blocks
    assert plan_ref.default_chunks(64, 8, 8, 2, 256, 512) == (512, 256)
    assert plan_ref.default_chunks(16, 4, 8, 2, 16, 8, 64, 96) == (64, 96)


def test_long_and_short_item_counts_on_a_hand_worked_list():
    """Chunks of 256 tokens; short = at most 128 tokens.  Own tokens 600 -> items 256, 256, 88 (the 88
    is short and belongs to a sequence with several chunks); 100 -> one short item that is the whole
    sequence; 256 -> one long item; 260 -> 256 and 4 (short, several chunks); 0 -> nothing."""
    p = plan_ref.build_plan([10], [600, 100, 256, 260, 0], [0] * 5, 4, 2, 1, 64, suffix_chunk=256, prefix_chunk=32)
    assert len(p.suffix_items) == 7
    assert p.num_long_suffix_items == 4
    assert p.num_short_partial_items == 2
    # chunks no longer than a short item: every chunk of a sequence with several chunks counts
    p = plan_ref.build_plan([10], [200, 64, 70], [0] * 3, 4, 2, 1, 64, suffix_chunk=64, prefix_chunk=32)
    assert p.num_long_suffix_items == 0
    assert p.num_short_partial_items == 4 + 0 + 2
