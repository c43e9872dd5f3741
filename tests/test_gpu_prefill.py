"""GPU parity of marl_prefill_attn and marl_kv_write_prompt against the float64 reference,
through the C ABI.

Tolerance.  The kernel rounds the softmax weights to bf16 before the value product (unit
roundoff 2^-8: bf16 keeps 8 significant bits) and, for bf16 output, rounds the result once more
(another 2^-8, relative).  Unlike a decode query over hundreds of tokens, an early prompt row
averages only a few values, so its output is O(max |V|) and the errors do not average out: the
bound is the worst case, stated relative to the softmax-weighted mean of |V| of the row, which
the reference computes:
    |delta| <= 1e-3 + 2^-8 * sum_j p_j |V_j|      (2^-7 for bf16 output).
Rows over many tokens stay far inside it (their errors average out as in the decode tests)."""
import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

pytestmark = pytest.mark.gpu


def reference(inp):
    qb, kb, vb = I.bf16_bits(inp.q), I.bf16_bits(inp.k_pages), I.bf16_bits(inp.v_pages)
    args = (inp.prefix_block_table.cpu().numpy(), inp.q_start.cpu().numpy(), inp.q_pos0.cpu().numpy(),
            inp.scale, inp.Hq, inp.Hkv)
    return R.prefill_attn(qb, kb, vb, *args), R.prefill_attn(qb, kb, vb & 0x7fff, *args)


def run_gpu(inp_cpu, out_dtype, expect_flags=0):
    dev = inp_cpu.to("cuda")
    shape, ws, out = B.prepare_prefill(dev, out_dtype)
    out.fill_(float("nan"))
    B.run_prefill(dev, shape, ws, out)
    torch.cuda.synchronize()
    assert B.marl_attn_read_flags(ws) == expect_flags
    return out.float().cpu().numpy().astype(np.float64)


def check(inp_cpu, out_dtype=B.MARL_OUT_F32):
    want, want_abs = reference(inp_cpu)
    got = run_gpu(inp_cpu, out_dtype)
    covered = np.isfinite(want)
    assert np.isfinite(got[covered]).all()
    assert np.isnan(got[~covered]).all()          # rows no group covers are left alone
    rel = 2.0 ** -8 if out_dtype == B.MARL_OUT_F32 else 2.0 ** -7
    excess = np.abs(got - want)[covered] - (1e-3 + rel * want_abs[covered])
    assert excess.size == 0 or excess.max() <= 0, f"worst excess over the bound {excess.max()}"


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (28, 4), (64, 8), (4, 4), (16, 1)])
@pytest.mark.parametrize("out_dtype", [B.MARL_OUT_F32, B.MARL_OUT_BF16])
def test_ragged_prompts_match_reference(Hq, Hkv, out_dtype):
    lens = [1, 5, 16, 17, 33, 100, 0, 257]
    check(I.build_prefill_inputs(Hq, Hkv, lens, [0] * len(lens), seed=Hq + Hkv), out_dtype)


@pytest.mark.parametrize("seed", range(12))
def test_random_shapes(seed):
    """Seeded random head counts, prompt lengths (zeros, page and row-block boundaries, a few
    hundred tokens) and context lengths in front of the chunk."""
    rng = np.random.default_rng(500 + seed)
    Hkv = int(rng.choice([1, 2, 4, 8]))
    Rq = int(rng.choice([1, 2, 4, 7, 8, 16]))
    n = int(rng.integers(1, 7))
    edge = np.array([0, 1, 15, 16, 17, 47, 48, 49, 191, 192, 193])
    lens = np.where(rng.random(n) < 0.4, rng.choice(edge, n), rng.integers(1, 420, n))
    pos0 = np.where(rng.random(n) < 0.5, 0, rng.integers(0, 300, n))
    print("case: prefill random shape", seed, Hkv * Rq, Hkv, lens.tolist(), pos0.tolist(), flush=True)
    out_dtype = B.MARL_OUT_F32 if seed % 2 == 0 else B.MARL_OUT_BF16
    check(I.build_prefill_inputs(Hkv * Rq, Hkv, lens.tolist(), pos0.tolist(), seed=seed), out_dtype)


def test_chunked_prefill_with_context():
    # chunks that start in the middle of a page, at a page boundary and deep into the prompt
    check(I.build_prefill_inputs(28, 4, [40, 7, 64, 1, 130], [5, 16, 96, 300, 257], seed=3))
    check(I.build_prefill_inputs(8, 2, [40, 7, 64, 1, 130], [5, 16, 96, 300, 257], seed=4), B.MARL_OUT_BF16)


@pytest.mark.parametrize("scale", [1.0, -0.7, 0.0])
def test_peaked_flat_and_sign_flipped_scores(scale):
    # scale 1 makes the scores ~N(0, 128): nearly one-hot rows whose running maximum keeps moving
    # (the accumulator rescale runs in most steps); a negative scale flips every score; scale 0
    # gives uniform weights (running means of the values)
    from dataclasses import replace
    inp = I.build_prefill_inputs(28, 4, [300, 77, 513], [0, 64, 5], seed=21)
    check(replace(inp, scale=scale))
    check(replace(inp, scale=scale), B.MARL_OUT_BF16)


def test_many_small_groups_and_more_than_one_plan_round():
    rng = np.random.default_rng(0)
    lens = rng.integers(0, 12, size=1500).tolist()      # plan scans 1024 groups per round
    pos0 = rng.integers(0, 20, size=1500).tolist()
    check(I.build_prefill_inputs(8, 2, lens, pos0, seed=5))


def test_long_prompt_sampled_rows_against_the_decode_checker():
    # 3 prompts of 2048 / 1500 / 700 tokens, Qwen-7B head layout; the reference prefill would need
    # minutes, so sampled rows are checked one by one with the C decode checker
    inp = I.build_prefill_inputs(28, 4, [2048, 1500, 700], [0, 0, 512], seed=6)
    got = run_gpu(inp, B.MARL_OUT_F32)
    assert np.isfinite(got).all()
    qs, p0 = inp.q_start.numpy(), inp.q_pos0.numpy()
    rng = np.random.default_rng(1)
    picks = [(0, 0), (0, 2047), (0, 31), (0, 32), (1, 1499), (2, 0), (2, 699)] + \
            [(int(g), int(rng.integers(0, qs[g + 1] - qs[g]))) for g in rng.integers(0, 3, size=25)]
    rows = np.array([qs[g] + tau for g, tau in picks])
    gid = np.array([g for g, _ in picks])
    plens = np.array([p0[g] + tau + 1 for g, tau in picks], dtype=np.int32)
    n = len(picks)
    qb, kb, vb = I.bf16_bits(inp.q)[rows], I.bf16_bits(inp.k_pages), I.bf16_bits(inp.v_pages)
    common = (inp.prefix_block_table.numpy()[gid], np.zeros((n, 1), dtype=np.int32), plens,
              np.zeros(n, dtype=np.int32), np.arange(n, dtype=np.int32), inp.scale, 28, 4)
    want = R.decode_attn(qb, kb, vb, *common)
    want_abs = R.decode_attn(qb, kb, vb & 0x7fff, *common)
    excess = np.abs(got[rows] - want) - (1e-3 + 2.0 ** -8 * want_abs)
    assert excess.max() <= 0, f"worst excess over the bound {excess.max()}"


def test_reruns_are_bit_identical_and_page_placement_does_not_matter():
    a = I.build_prefill_inputs(28, 4, [300, 77], [0, 40], seed=7)
    out1, out2 = run_gpu(a, B.MARL_OUT_F32), run_gpu(a, B.MARL_OUT_F32)
    np.testing.assert_array_equal(out1, out2)
    # same logical contents on other physical pages
    perm = np.random.default_rng(2).permutation(a.num_pages)
    inv = np.argsort(perm)
    tab = a.prefix_block_table.numpy().copy()
    tab[tab >= 0] = perm[tab[tab >= 0]]
    from dataclasses import replace
    b = replace(a, k_pages=a.k_pages[torch.from_numpy(inv)], v_pages=a.v_pages[torch.from_numpy(inv)],
                prefix_block_table=torch.from_numpy(tab))
    np.testing.assert_array_equal(run_gpu(b, B.MARL_OUT_F32), out1)


def test_bad_contents_are_flagged_not_followed():
    from dataclasses import replace
    a = I.build_prefill_inputs(8, 2, [20, 30], [0, 0], seed=8, poison=False)
    # a table entry out of range: reads page 0 instead, flag 4
    tab = a.prefix_block_table.clone()
    tab[1, 0] = a.num_pages + 5
    got = run_gpu(replace(a, prefix_block_table=tab), B.MARL_OUT_F32, expect_flags=B.FLAG_BAD_PAGE)
    assert np.isfinite(got).all()
    # a chunk that does not fit its table row is cut short, flag 2
    pos0 = a.q_pos0.clone()
    pos0[1] = 16          # 30 tokens from position 16 need 46 positions, the row has 32
    got = run_gpu(replace(a, q_pos0=pos0), B.MARL_OUT_F32, expect_flags=B.FLAG_LEN_CLAMPED)
    assert np.isfinite(got[:36]).all() and np.isnan(got[36:]).all()
    # q_start beyond the q array drops the group, flag 1
    qs = a.q_start.clone()
    qs[2] = 60
    got = run_gpu(replace(a, q_start=qs), B.MARL_OUT_F32, expect_flags=B.FLAG_BAD_GROUP)
    assert np.isfinite(got[:20]).all() and np.isnan(got[20:]).all()


def test_prompt_scatter_is_bit_exact_and_feeds_attention():
    inp = I.build_prefill_inputs(28, 4, [37, 0, 16, 130], [0, 3, 16, 21], seed=9)
    dev = inp.to("cuda")
    shape, ws, out = B.prepare_prefill(dev, B.MARL_OUT_F32)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.marl_kv_write_prompt(shape, dev.k_new, dev.v_new, dev.k_pages, dev.v_pages, dev.prefix_block_table,
                           dev.q_start, dev.q_pos0, flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == 0
    kp, vp = R.kv_write_prompt(I.bf16_bits(inp.k_pages), I.bf16_bits(inp.v_pages), inp.prefix_block_table.numpy(),
                               inp.q_start.numpy(), inp.q_pos0.numpy(), I.bf16_bits(inp.k_new), I.bf16_bits(inp.v_new))
    # NaN poison compares by bit pattern
    np.testing.assert_array_equal(I.bf16_bits(dev.k_pages.cpu()), kp)
    np.testing.assert_array_equal(I.bf16_bits(dev.v_pages.cpu()), vp)
    B.run_prefill(dev, shape, ws, out)
    torch.cuda.synchronize()
    args = (inp.prefix_block_table.numpy(), inp.q_start.numpy(), inp.q_pos0.numpy(), inp.scale, 28, 4)
    want = R.prefill_attn(I.bf16_bits(inp.q), kp, vp, *args)
    want_abs = R.prefill_attn(I.bf16_bits(inp.q), kp, vp & 0x7fff, *args)
    excess = np.abs(out.cpu().numpy().astype(np.float64) - want) - (1e-3 + 2.0 ** -8 * want_abs)
    assert excess.max() <= 0


def test_scatter_flags_tokens_it_cannot_place():
    from dataclasses import replace
    inp = I.build_prefill_inputs(8, 2, [20, 30], [0, 0], seed=10, poison=False)
    dev = inp.to("cuda")
    shape, _, _ = B.prepare_prefill(dev, B.MARL_OUT_F32)
    tab = dev.prefix_block_table.clone()
    tab[0, 1] = -1
    before_k = dev.k_pages.clone()
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.marl_kv_write_prompt(shape, dev.k_new, dev.v_new, dev.k_pages, dev.v_pages, tab, dev.q_start, dev.q_pos0, flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == B.FLAG_BAD_PAGE
    # tokens 16..19 of group 0 were skipped: their former page is untouched
    pg = int(inp.prefix_block_table[0, 1])
    assert torch.equal(dev.k_pages[pg], before_k[pg])


def test_last_prompt_row_equals_the_decode_call_on_the_same_cache():
    # the decode entry point with an empty suffix over the same pages must agree with the last
    # prefill row up to the two kernels' rounding
    inp = I.build_prefill_inputs(28, 4, [513, 100], [0, 0], seed=11).to("cuda")
    shape, ws, out = B.prepare_prefill(inp, B.MARL_OUT_F32)
    B.run_prefill(inp, shape, ws, out)
    last = (inp.q_start[1:] - 1).long()
    dshape = B.make_shape(2, 2, 28, 4, inp.num_pages, int(inp.prefix_block_table.shape[1]), 1, B.MARL_OUT_F32)
    lay = B.marl_attn_plan_layout_for(dshape)
    dws = B.alloc_workspace(lay.total_bytes, "cuda")
    dout = torch.empty((2, 28, 128), device="cuda")
    B.marl_decode_attn(dshape, dws, inp.q[last].contiguous(), inp.k_pages, inp.v_pages, inp.prefix_block_table,
                       torch.full((2, 1), -1, dtype=torch.int32, device="cuda"),
                       torch.tensor([513, 100], dtype=torch.int32, device="cuda"),
                       torch.zeros(2, dtype=torch.int32, device="cuda"),
                       torch.arange(2, dtype=torch.int32, device="cuda"), inp.scale, dout)
    torch.cuda.synchronize()
    assert float((out[last] - dout).abs().max()) < 2e-3


def test_overlapping_groups_cannot_overrun_the_item_list():
    # three groups that all claim rows 0..299 of a 300-row q: the workspace is sized for groups
    # that share no rows, so the ones that do not fit are dropped and flagged
    from dataclasses import replace
    a = I.build_prefill_inputs(28, 4, [300, 0, 0], [0, 0, 0], seed=12, poison=False)
    tab = a.prefix_block_table[0:1].expand(3, -1).contiguous()
    qs = torch.tensor([0, 300, 0, 300], dtype=torch.int32)       # group 1 is inconsistent, group 2 overlaps group 0
    # q_start[1..2] = (300, 0): negative count -> flag 1; group 2 = rows 0..299 again
    got = run_gpu(replace(a, prefix_block_table=tab, q_start=qs), B.MARL_OUT_F32, expect_flags=B.FLAG_BAD_GROUP)
    want, want_abs = reference(a)
    assert (np.abs(got - want) <= 1e-3 + 2.0 ** -8 * want_abs).all()


def test_full_size_prompts_of_the_bench_workload_sampled_rows():
    """The prompts bench.py's prefill leg runs (256 prompts of the qwen7b workload, 329 k tokens),
    in the same launch configuration; sampled query rows are checked one by one with the C decode
    checker on a compact copy of the pages that row sees."""
    w = I.WORKLOADS["qwen7b"]
    lens = I.draw_lengths(w, np.random.default_rng(w.seed)).prefix_lens.tolist()
    inp = I.build_prefill_inputs(w.Hq, w.Hkv, lens, [0] * len(lens), device="cuda", seed=w.seed, poison=False)
    shape, ws, out = B.prepare_prefill(inp, B.MARL_OUT_BF16)
    B.run_prefill(inp, shape, ws, out)
    torch.cuda.synchronize()
    assert B.marl_attn_read_flags(ws) == 0
    assert bool(torch.isfinite(out.float()).all())
    qs = inp.q_start.cpu().numpy()
    rng = np.random.default_rng(4)
    longest, shortest = int(np.argmax(lens)), int(np.argmin(lens))
    picks = [(longest, lens[longest] - 1), (longest, 0), (shortest, lens[shortest] - 1), (0, 17), (255, lens[255] // 2)] + \
            [(int(g), int(rng.integers(0, lens[g]))) for g in rng.integers(0, len(lens), size=19)]
    worst = 0.0
    for g, tau in picks:
        npages = tau // 16 + 1
        pages = inp.prefix_block_table[g, :npages].long()
        kb, vb = I.bf16_bits(inp.k_pages[pages].cpu()), I.bf16_bits(inp.v_pages[pages].cpu())
        qb = I.bf16_bits(inp.q[qs[g] + tau:qs[g] + tau + 1].cpu())
        common = (np.arange(npages, dtype=np.int32)[None, :], np.zeros((1, 1), dtype=np.int32),
                  np.array([tau + 1], dtype=np.int32), np.zeros(1, dtype=np.int32), np.zeros(1, dtype=np.int32),
                  inp.scale, w.Hq, w.Hkv)
        want = R.decode_attn(qb, kb, vb, *common)[0]
        want_abs = R.decode_attn(qb, kb, vb & 0x7fff, *common)[0]
        got = out[qs[g] + tau].float().cpu().numpy().astype(np.float64)
        excess = np.abs(got - want) - (1e-3 + 2.0 ** -7 * want_abs)
        assert excess.max() <= 0, (g, tau, excess.max())
        worst = max(worst, float(np.abs(got - want).max()))
    print("prefill full size: worst |delta| over sampled rows", worst, flush=True)
