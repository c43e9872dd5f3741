"""GPU parity of marl_decode_attn against the float64 checker, element by element, through
the C ABI.  Tolerance: max |delta| <= 4e-3."""
import dataclasses
import math

import numpy as np
import pytest
import torch

from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I
from tests.gpu_common import ATTN_TOL, check_attn, gpu_attn, oracle_attn

pytestmark = pytest.mark.gpu


def custom_inputs(prefix_lens, suffix_lens, group_of_seq, Hq, Hkv, seed, scale=None, poison=True):
    L = I.Lengths(np.asarray(prefix_lens, np.int32), np.asarray(suffix_lens, np.int32),
                  np.asarray(group_of_seq, np.int32), np.zeros(len(prefix_lens), np.int32))
    w = I.Workload("custom", Hq, Hkv, (), seed)
    inp = I.build_attn_inputs(w, "cpu", seed, poison=poison, lengths=L)
    if scale is not None:
        inp.scale = scale
    return inp


@pytest.mark.parametrize("out_dtype", [B.MARL_OUT_F32, B.MARL_OUT_BF16])
def test_tiny_workload(out_dtype):
    print("case: tiny", out_dtype, flush=True)
    err = check_attn(I.build_attn_inputs(I.WORKLOADS["tiny"]), out_dtype)
    print("max err", err)


@pytest.mark.parametrize("name,pdiv,ldiv", [("qwen7b", 16, 4), ("skew", 8, 8), ("prefix", 16, 4),
                                            ("long32b", 8, 8)])
def test_scaled_workloads(name, pdiv, ldiv):
    """The named workloads with fewer prompts and shorter lengths, so the checker finishes in
    seconds; they still span several chunks, several query-row blocks and ragged tails."""
    print("case:", name, pdiv, ldiv, flush=True)
    w = I.WORKLOADS[name].scaled(pdiv, ldiv)
    inp = I.build_attn_inputs(w)
    err = check_attn(inp, B.MARL_OUT_BF16)
    print(name, "seqs", inp.num_seqs, "max err", err)


@pytest.mark.parametrize("cs,cp", [(32, 32), (64, 96), (256, 128)])
def test_small_chunks_many_partials(cs, cp):
    print("case: chunks", cs, cp, flush=True)
    w = I.WORKLOADS["qwen7b"].scaled(32, 8)
    check_attn(I.build_attn_inputs(w), B.MARL_OUT_F32, suffix_chunk_tokens=cs, prefix_chunk_tokens=cp)


def test_edge_lengths_and_ragged_groups():
    """Empty suffixes, empty prefixes, sequences with no token at all, lengths on and around
    page / step / chunk boundaries, groups of different sizes listed in shuffled order."""
    print("case: edge lengths", flush=True)
    rng = np.random.default_rng(7)
    plens = [0, 1, 15, 16, 17, 31, 32, 33, 255, 256, 257, 300]
    sizes = [1, 2, 3, 5, 8, 1, 4, 11, 2, 1, 6, 3]
    gos = np.repeat(np.arange(len(plens)), sizes)
    slens = rng.choice([0, 1, 2, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 513],
                       size=len(gos))
    slens[0] = 0                                  # group 0 has no prefix: this sequence has no token
    perm = rng.permutation(len(gos))
    inp = custom_inputs(plens, slens[perm], gos[perm], 12, 4, seed=3)
    want = oracle_attn(inp)
    got, _ = gpu_attn(inp, B.MARL_OUT_F32)
    assert np.abs(got - want).max() <= ATTN_TOL
    s0 = int(np.nonzero(perm == 0)[0][0])
    assert np.all(got[s0] == 0.0)
    got2, _ = gpu_attn(inp, B.MARL_OUT_F32, suffix_chunk_tokens=64, prefix_chunk_tokens=32)
    assert np.abs(got2 - want).max() <= ATTN_TOL


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (16, 1), (6, 2), (64, 8)])
def test_head_layouts(Hq, Hkv):
    print("case: heads", Hq, Hkv, flush=True)
    inp = custom_inputs([70, 33], [40, 5, 100, 64, 1], [0, 0, 1, 1, 1], Hq, Hkv, seed=5)
    check_attn(inp, B.MARL_OUT_F32)


@pytest.mark.parametrize("sizes", [[21], [40], [60, 2], [17, 19, 1]])
def test_big_groups_and_query_row_blocks(sizes):
    """Groups whose G*R query rows fill one ragged block or several blocks of the prefix
    kernel: 147 rows (8-wave kernel, one block), 280 rows (two blocks of 256), a large and a
    tiny group together (8-wave kernel), groups just under and over 128 rows (4-wave kernel)."""
    print("case: big groups", sizes, flush=True)
    gos = np.repeat(np.arange(len(sizes)), sizes)
    rng = np.random.default_rng(sum(sizes))
    inp = custom_inputs(rng.integers(150, 260, len(sizes)), rng.integers(1, 60, len(gos)), gos, 28, 4, seed=9)
    check_attn(inp, B.MARL_OUT_F32)
    check_attn(inp, B.MARL_OUT_F32, prefix_chunk_tokens=64)


@pytest.mark.parametrize("NG", [2100, 8300])
def test_many_groups_use_the_larger_plan_kernels(NG):
    """More groups than the small LDS-resident plan kernel handles (2048), and more than the
    larger one does (8192: the plan that works in global memory)."""
    print("case: many groups", NG, flush=True)
    rng = np.random.default_rng(21)
    sizes = rng.integers(1, 3, NG)
    gos = np.repeat(np.arange(NG), sizes)
    inp = custom_inputs(rng.integers(0, 40, NG), rng.integers(0, 50, len(gos)), gos, 4, 2, seed=23)
    check_attn(inp, B.MARL_OUT_F32)


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(seed):
    """Seeded random shapes: head counts, group sizes (a few of them beyond one query-row block),
    prefix and generated lengths that mix zeros, page and step boundaries and several chunks,
    sequences in shuffled order, default and small chunks."""
    rng = np.random.default_rng(1000 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    R = int(rng.choice([1, 2, 4, 7, 8, 16]))
    NG = int(rng.integers(1, 9))
    sizes = rng.choice([1, 2, 3, 8, 20, 40], size=NG, p=[0.3, 0.2, 0.2, 0.2, 0.05, 0.05])
    gos = rng.permutation(np.repeat(np.arange(NG), sizes))
    edge = np.array([0, 1, 15, 16, 17, 31, 32, 33, 127, 128, 129])
    plens = np.where(rng.random(NG) < 0.4, rng.choice(edge, NG), rng.integers(0, 700, NG))
    slens = np.where(rng.random(len(gos)) < 0.4, rng.choice(edge, len(gos)), rng.integers(0, 600, len(gos)))
    print("case: random shape", seed, "Hq", Hkv * R, "Hkv", Hkv, "groups", sizes.tolist(), flush=True)
    inp = custom_inputs(plens, slens, gos, Hkv * R, Hkv, seed=seed)
    check_attn(inp, B.MARL_OUT_F32)
    # bf16 output: a sequence of a few tokens can have |out| > 1, where the half ulp of the final
    # rounding alone (|out| 2^-8 at most) exceeds the absolute bar, so it is allowed on top
    want = oracle_attn(inp)
    got, _ = gpu_attn(inp, B.MARL_OUT_BF16, suffix_chunk_tokens=int(rng.choice([32, 96, 256])),
                      prefix_chunk_tokens=int(rng.choice([32, 64, 160])))
    assert np.isfinite(got).all()
    assert np.all(np.abs(got - want) <= ATTN_TOL + np.abs(want) * 2.0 ** -8)


def test_negative_and_zero_scale():
    print("case: scale sign", flush=True)
    for scale in (-0.11, 0.0):
        inp = custom_inputs([50], [20, 7], [0, 0], 8, 2, seed=11, scale=scale)
        check_attn(inp, B.MARL_OUT_F32)


def test_peaked_scores():
    # scale 1 makes the scores ~N(0, 128): nearly one-hot weights, a running maximum that keeps moving
    # (accumulator rescales in most steps), partials whose maxima differ widely at the merge
    print("case: peaked scores", flush=True)
    # the outputs are single value rows here (|out| up to ~4, not the ~0.1 of a mean over hundreds of
    # tokens), so the rounding of a weight to bf16 (2^-9 relative) shows in full: bound 4 * 2^-8
    inp = custom_inputs([300, 40], [700, 33, 129, 5], [0, 0, 1, 1], 28, 4, seed=12, scale=1.0)
    check_attn(inp, B.MARL_OUT_F32, tol=4 * 2.0 ** -8)
    check_attn(inp, B.MARL_OUT_F32, tol=4 * 2.0 ** -8, suffix_chunk_tokens=256, prefix_chunk_tokens=256)


def test_peaked_scores_in_a_big_group():
    """The same with a group of 21 samples (147 query rows: the 8-wave prefix kernel, whose reference
    maximum of a row moves only when a score exceeds it by more than 2^8: with scale 1 that happens
    in many steps, and in most of them for some rows of a wave only)."""
    print("case: peaked scores, big group", flush=True)
    rng = np.random.default_rng(77)
    inp = custom_inputs([900], rng.integers(1, 40, 21), [0] * 21, 28, 4, seed=14, scale=1.0)
    check_attn(inp, B.MARL_OUT_F32, tol=4 * 2.0 ** -8)
    check_attn(inp, B.MARL_OUT_F32, tol=4 * 2.0 ** -8, prefix_chunk_tokens=128)


def test_reruns_and_page_permutations_are_bit_identical():
    print("case: determinism", flush=True)
    w = I.WORKLOADS["qwen7b"].scaled(32, 8)
    a = I.build_attn_inputs(w, seed=100)
    out1, call = gpu_attn(a, B.MARL_OUT_F32)
    dev = a.to("cuda")
    for _ in range(3):
        B.run_attn(dev, call)
        torch.cuda.synchronize()
        assert np.array_equal(call.out.float().cpu().numpy().astype(np.float64), out1)
    # same logical content on differently numbered physical pages
    rng = np.random.default_rng(5)
    perm = torch.from_numpy(rng.permutation(a.num_pages))
    inv = torch.empty_like(perm); inv[perm] = torch.arange(a.num_pages)
    b = I.AttnInputs(a.Hq, a.Hkv, a.num_pages, a.q, a.k_pages[perm], a.v_pages[perm],
                     torch.where(a.prefix_block_table >= 0, inv[a.prefix_block_table.clamp(min=0).long()].int(), -1),
                     torch.where(a.suffix_block_table >= 0, inv[a.suffix_block_table.clamp(min=0).long()].int(), -1),
                     a.prefix_lens, a.suffix_lens, a.group_of_seq, a.scale)
    out2, _ = gpu_attn(b, B.MARL_OUT_F32)
    assert np.array_equal(out1, out2)


def test_poison_value_does_not_matter():
    print("case: poison", flush=True)
    w = I.WORKLOADS["tiny"]
    a = I.build_attn_inputs(w, poison=True)
    b = I.build_attn_inputs(w, poison=False)     # same draws, unused locations hold ordinary numbers
    oa, _ = gpu_attn(a, B.MARL_OUT_F32)
    ob, _ = gpu_attn(b, B.MARL_OUT_F32)
    assert np.isfinite(oa).all() and np.array_equal(oa, ob)


def test_bad_device_contents_are_clamped_and_flagged():
    """Out-of-range lengths, group ids and page ids never leave the buffers: the kernels
    clamp them and set a flag."""
    print("case: flags", flush=True)
    inp = custom_inputs([40, 20], [30, 10, 25], [0, 1, 1], 8, 2, seed=13, poison=False)
    bad = I.AttnInputs(**{**inp.__dict__})
    bad.suffix_lens = inp.suffix_lens.clone(); bad.suffix_lens[0] = 10 ** 6
    bad.group_of_seq = inp.group_of_seq.clone(); bad.group_of_seq[1] = 99
    bad.suffix_block_table = inp.suffix_block_table.clone(); bad.suffix_block_table[2, 0] = 10 ** 8
    got, _ = gpu_attn(bad, B.MARL_OUT_F32,
                      expect_flags=B.FLAG_BAD_GROUP | B.FLAG_LEN_CLAMPED | B.FLAG_BAD_PAGE)
    assert np.isfinite(got).all()


@pytest.mark.parametrize("samples", [3, 21])
def test_bad_prefix_page_ids_are_flagged(samples):
    """A prefix block-table entry outside the pool (4-wave and 8-wave prefix kernels): the flag is
    raised, nothing outside the buffers is read, outputs stay finite, and a group whose table is
    intact is computed as if nothing had happened."""
    print("case: bad prefix page ids", samples, flush=True)
    rng = np.random.default_rng(samples)
    gos = [0] * samples + [1] * samples
    inp = custom_inputs([200, 150], rng.integers(1, 50, 2 * samples), gos, 28, 4, seed=15, poison=False)
    good, _ = gpu_attn(inp, B.MARL_OUT_F32)
    bad = I.AttnInputs(**{**inp.__dict__})
    bad.prefix_block_table = inp.prefix_block_table.clone()
    bad.prefix_block_table[0, 3] = 10 ** 8
    bad.prefix_block_table[0, 7] = -5
    got, _ = gpu_attn(bad, B.MARL_OUT_F32, expect_flags=B.FLAG_BAD_PAGE)
    assert np.isfinite(got).all()
    assert np.array_equal(got[samples:], good[samples:])   # the second group does not touch the bad entries


def _full_size_every_row(name):
    """Full-size workload in the launch configuration the benchmark uses (default chunks, bf16
    output, inputs generated in HBM); the checker recomputes EVERY sequence on the host copy of
    the same bytes, and every output element is compared."""
    w = I.WORKLOADS[name] if isinstance(name, str) else name
    name = w.name
    dev = I.build_attn_inputs(w, device="cuda")
    call = B.prepare_attn(dev, B.MARL_OUT_BF16)
    B.run_attn(dev, call)
    torch.cuda.synchronize()
    assert B.marl_attn_read_flags(call.workspace) == 0
    got = call.out.float().cpu().numpy()
    host = dev.to("cpu")
    del dev, call
    torch.cuda.empty_cache()
    print(name, "checker on", host.num_seqs, "sequences ...", flush=True)
    want = oracle_attn(host)
    assert want.shape == got.shape
    assert np.isfinite(got).all()
    per_seq = np.abs(got - want).reshape(host.num_seqs, -1).max(axis=1)
    err = float(per_seq.max())
    total = (host.prefix_lens[host.group_of_seq.long()] + host.suffix_lens).numpy()
    print(f"{name}: all {host.num_seqs} sequences compared, max |delta| = {err:.3e} "
          f"(worst sequence {int(per_seq.argmax())}, {int(total[per_seq.argmax()])} tokens; "
          f"lengths {int(total.min())}..{int(total.max())})", flush=True)
    assert err <= ATTN_TOL


@pytest.mark.parametrize("name", ["qwen7b", "skew", "prefix", "long32b"])
def test_full_size_every_row(name):
    print("case: full size", name, flush=True)
    _full_size_every_row(name)


def test_full_size_sixteen_samples_per_prompt():
    """The bench workload's shape with 16 samples per prompt instead of 8 (the paper runs a
    parallelism of 4 x 16, Section 8.1): 112 query rows per group and KV head, which is the 4-wave
    prefix kernel with two row tiles per wave at full size.  Every row is compared."""
    print("case: full size, 16 samples per prompt", flush=True)
    w = I.WORKLOADS["qwen7b"]
    agents = tuple(I.Agent(a.prompts // 2, 16, a.prompt_len, a.gen_len) for a in w.agents)
    _full_size_every_row(dataclasses.replace(w, name="qwen7b/G16", agents=agents))
