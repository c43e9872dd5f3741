"""The device-built work list against its host reference: integer work, compared exactly."""
import numpy as np
import pytest
import torch

from oracle import plan_ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

pytestmark = pytest.mark.gpu


def read_plan(shape, prefix_lens, suffix_lens, gos):
    L = B.marl_attn_plan_layout_for(shape)
    ws = B.alloc_workspace(L.total_bytes, "cuda")
    ws.fill_(0xAB)
    t = lambda a: torch.as_tensor(np.asarray(a, np.int32), device="cuda")
    B.marl_attn_plan(shape, ws, t(prefix_lens), t(suffix_lens), t(gos))
    torch.cuda.synchronize()
    host = ws.cpu().numpy()
    i32 = lambda off, n: host[off:off + 4 * n].view(np.int32).copy()
    ctr = i32(L.counters_off, 64)
    NS, NG = shape.num_seqs, shape.num_groups
    return dict(L=L, ctr=ctr, count=i32(L.group_count_off, NG), start=i32(L.group_start_off, NG + 1),
                seqs=i32(L.group_seqs_off, NS), chunks=i32(L.seq_chunks_off, NS),
                sitems=i32(L.suffix_items_off, 4 * ctr[0]).reshape(-1, 4),
                pitems=i32(L.prefix_items_off, 4 * ctr[1]).reshape(-1, 4))


def compare(shape, pl, sl, gos, Hq, Hkv):
    got = read_plan(shape, pl, sl, gos)
    want = plan_ref.build_plan(pl, sl, gos, Hq, Hkv, shape.max_prefix_pages, shape.max_suffix_pages,
                               shape.suffix_chunk_tokens, shape.prefix_chunk_tokens)
    L = got["L"]
    assert (L.suffix_chunk_tokens, L.prefix_chunk_tokens) == (want.Cs, want.Cp)
    assert (L.suffix_slots, L.prefix_slots) == (want.suffix_slots, want.prefix_slots)
    assert np.array_equal(got["count"], want.group_count)
    assert np.array_equal(got["start"], want.group_start)
    n = int(want.group_start[-1])
    assert np.array_equal(got["seqs"][:n], want.group_seqs[:n])
    assert got["ctr"][B.CTR_FLAGS] == want.flags
    assert np.array_equal(got["chunks"], want.seq_chunks)
    assert got["ctr"][B.CTR_SUFFIX_CURSOR] == 0 and got["ctr"][B.CTR_PREFIX_CURSOR] == 0
    assert got["ctr"][B.CTR_SHORT_CURSOR] == 0
    nlong = got["ctr"][B.CTR_NUM_LONG_SUFFIX_ITEMS]
    assert nlong == want.num_long_suffix_items
    assert got["ctr"][B.CTR_NUM_SHORT_PARTIAL_ITEMS] == want.num_short_partial_items
    assert all(it[2] - it[1] > plan_ref.SHORT_TOKENS for it in got["sitems"][:nlong].tolist())
    assert all(it[2] - it[1] <= plan_ref.SHORT_TOKENS for it in got["sitems"][nlong:].tolist())
    for items, ref_items, chunk in ((got["sitems"], want.suffix_items, want.Cs),
                                    (got["pitems"], want.prefix_items, want.Cp)):
        assert sorted(map(tuple, items.tolist())) == sorted(ref_items)
        cls = [plan_ref.cost_class(it, chunk) for it in items.tolist()]
        assert cls == sorted(cls)            # longest first
    return got


@pytest.mark.parametrize("name,pdiv,ldiv", [("tiny", 1, 1), ("qwen7b", 1, 1), ("skew", 1, 1), ("prefix", 1, 1),
                                            ("long32b", 1, 1), ("qwen7b", 8, 4)])
def test_plan_matches_reference(name, pdiv, ldiv):
    print("case: plan", name, flush=True)
    w = I.WORKLOADS[name].scaled(pdiv, ldiv)
    L = I.draw_lengths(w, np.random.default_rng(w.seed))
    mpp = int(-(-L.prefix_lens.max() // 16)); msp = int(-(-L.suffix_lens.max() // 16))
    shape = B.make_shape(len(L.suffix_lens), len(L.prefix_lens), w.Hq, w.Hkv, 10, mpp, msp)
    compare(shape, L.prefix_lens, L.suffix_lens, L.group_of_seq, w.Hq, w.Hkv)


@pytest.mark.parametrize("NS,S", [(2048, 40), (1000, 200), (333, 300), (64 * 9 + 1, 0)])
def test_plan_equal_lengths(NS, S):
    """Every sequence at the same decode step: one cost class (or none) takes every item."""
    print("case: plan equal lengths", NS, S, flush=True)
    G = 8
    NG = -(-NS // G)
    gos = (np.arange(NS) // G).astype(np.int32)
    pl = np.full(NG, 700, np.int32)
    sl = np.full(NS, S, np.int32)
    sl[NS // 2] = S + 64          # but for one sequence
    shape = B.make_shape(NS, NG, 28, 4, 10, 44, 32, suffix_chunk_tokens=256)
    got = compare(shape, pl, sl, gos, 28, 4)
    assert len({tuple(it) for it in got["sitems"].tolist()}) == len(got["sitems"])   # no place given twice


def test_plan_shuffled_groups_small_chunks_and_bad_values():
    print("case: plan shuffled", flush=True)
    rng = np.random.default_rng(3)
    NG = 37
    sizes = rng.integers(0, 12, NG)
    gos = rng.permutation(np.repeat(np.arange(NG), sizes)).astype(np.int32)
    pl = rng.integers(0, 900, NG).astype(np.int32)
    sl = rng.integers(0, 1200, len(gos)).astype(np.int32)
    pl[3] = -5; sl[4] = 10 ** 7; gos[7] = NG + 3; gos[9] = -1
    shape = B.make_shape(len(gos), NG, 28, 4, 10, 57, 75, suffix_chunk_tokens=96, prefix_chunk_tokens=64)
    got = compare(shape, pl, sl, gos, 28, 4)
    assert got["ctr"][B.CTR_FLAGS] == 3


def test_plan_large_group_stays_a_valid_set():
    """Groups above 64 sequences are not sorted on the device: compare them as sets."""
    print("case: plan large group", flush=True)
    gos = np.zeros(200, np.int32); gos[100:] = 1
    rng = np.random.default_rng(1); gos = rng.permutation(gos)
    shape = B.make_shape(200, 2, 8, 2, 10, 4, 4)
    got = read_plan(shape, [50, 60], np.full(200, 33), gos)
    assert list(got["count"]) == [100, 100] and list(got["start"]) == [0, 100, 200]
    assert sorted(got["seqs"][:100]) == sorted(np.nonzero(gos == 0)[0])
    assert sorted(got["seqs"][100:]) == sorted(np.nonzero(gos == 1)[0])


def big_case(NG, lo, hi, seed):
    rng = np.random.default_rng(seed)
    sizes = rng.integers(lo, hi, NG)
    gos = rng.permutation(np.repeat(np.arange(NG), sizes)).astype(np.int32)
    pl = rng.integers(0, 400, NG).astype(np.int32)
    sl = rng.integers(0, 700, len(gos)).astype(np.int32)
    shape = B.make_shape(len(gos), NG, 8, 2, 10, 25, 44, suffix_chunk_tokens=256, prefix_chunk_tokens=128)
    return shape, pl, sl, gos


def test_plan_larger_lds_variant():
    """8193 .. 32768 sequences in up to 8192 groups: the LDS-resident plan with 16-bit member ids."""
    print("case: plan medium", flush=True)
    shape, pl, sl, gos = big_case(2500, 1, 8, 11)
    assert 8192 < len(gos) <= 32768
    compare(shape, pl, sl, gos, 8, 2)
    shape, pl, sl, gos = big_case(8192, 4, 5, 12)        # exactly 32768 sequences in 8192 groups
    assert len(gos) == 32768
    compare(shape, pl, sl, gos, 8, 2)


def test_plan_general_kernel_for_shapes_beyond_the_lds_variants():
    """More than 32768 sequences or 8192 groups: the plan kernel that keeps its bookkeeping in
    global memory runs; same contract."""
    print("case: plan big", flush=True)
    shape, pl, sl, gos = big_case(8300, 1, 3, 13)        # too many groups
    compare(shape, pl, sl, gos, 8, 2)
    shape, pl, sl, gos = big_case(4000, 8, 10, 14)       # too many sequences
    assert len(gos) > 32768
    compare(shape, pl, sl, gos, 8, 2)
