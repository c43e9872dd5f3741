"""GPU parity of the KV-cache maintenance entry points (bit-exact) and a short decode loop:
append, then attend, several iterations, against the references."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I
from tests.gpu_common import ATTN_TOL, oracle_attn

pytestmark = pytest.mark.gpu


def with_room(inp: I.AttnInputs, extra_cols: int, rng) -> I.AttnInputs:
    """Widens the suffix table and hands every sequence spare pages, as a scheduler would."""
    NS, cols = inp.suffix_block_table.shape
    st = torch.full((NS, cols + extra_cols), -1, dtype=torch.int32)
    st[:, :cols] = inp.suffix_block_table
    used = set(inp.prefix_block_table[inp.prefix_block_table >= 0].tolist()) | set(st[st >= 0].tolist())
    need = NS * extra_cols
    first_new = inp.num_pages
    num_pages = inp.num_pages + need
    grow = lambda t: torch.cat([t, torch.full((need,) + tuple(t.shape[1:]), float("nan"), dtype=t.dtype)])
    k, v = grow(inp.k_pages), grow(inp.v_pages)
    new_ids = torch.from_numpy(rng.permutation(np.arange(first_new, num_pages))).int()
    nxt = 0
    for s in range(NS):
        have = (int(inp.suffix_lens[s]) + 15) // 16
        for c in range(have, min(have + extra_cols, cols + extra_cols)):
            st[s, c] = new_ids[nxt]; nxt += 1
    return I.AttnInputs(inp.Hq, inp.Hkv, num_pages, inp.q, k, v, inp.prefix_block_table, st, inp.prefix_lens,
                        inp.suffix_lens.clone(), inp.group_of_seq, inp.scale)


def test_append_is_bit_exact_and_decode_loop_matches():
    print("case: kv append loop", flush=True)
    rng = np.random.default_rng(3)
    w = I.WORKLOADS["qwen7b"].scaled(32, 16)
    cpu = with_room(I.build_attn_inputs(w, seed=77), 2, rng)
    dev = cpu.to("cuda")
    shape = B.make_shape(cpu.num_seqs, cpu.num_groups, cpu.Hq, cpu.Hkv, cpu.num_pages,
                         cpu.prefix_block_table.shape[1], cpu.suffix_block_table.shape[1], B.MARL_OUT_F32)
    call = B.prepare_attn(dev, B.MARL_OUT_F32)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    kb, vb, lens = I.bf16_bits(cpu.k_pages), I.bf16_bits(cpu.v_pages), cpu.suffix_lens.numpy().copy()
    gen = torch.Generator().manual_seed(5)
    for step in range(18):           # crosses a page boundary for every sequence
        k_new = torch.randn(cpu.num_seqs, cpu.Hkv, 128, generator=gen).to(torch.bfloat16)
        v_new = torch.randn(cpu.num_seqs, cpu.Hkv, 128, generator=gen).to(torch.bfloat16)
        kb, vb, lens, f = ref.kv_append(kb, vb, cpu.suffix_block_table.numpy(), lens, I.bf16_bits(k_new), I.bf16_bits(v_new))
        assert f == 0
        B.marl_kv_append(shape, k_new.cuda(), v_new.cuda(), dev.k_pages, dev.v_pages, dev.suffix_block_table,
                         dev.suffix_lens, flags)
        if step % 6 == 5:
            B.run_attn(dev, call)
            torch.cuda.synchronize()
            want = ref.decode_attn(I.bf16_bits(cpu.q), kb, vb, cpu.prefix_block_table.numpy(),
                                   cpu.suffix_block_table.numpy(), cpu.prefix_lens.numpy(), lens,
                                   cpu.group_of_seq.numpy(), cpu.scale, cpu.Hq, cpu.Hkv)
            assert np.abs(call.out.cpu().numpy().astype(np.float64) - want).max() <= ATTN_TOL
    torch.cuda.synchronize()
    assert int(flags.item()) == 0
    assert np.array_equal(dev.suffix_lens.cpu().numpy(), lens)
    assert np.array_equal(I.bf16_bits(dev.k_pages), kb)      # NaN poison compares as bits
    assert np.array_equal(I.bf16_bits(dev.v_pages), vb)


def test_append_skips_and_flags():
    print("case: kv append flags", flush=True)
    Hkv = 2
    k = torch.zeros(4, Hkv, 16, 128, dtype=torch.bfloat16, device="cuda"); v = torch.zeros(4, Hkv, 128, 16, dtype=torch.bfloat16, device="cuda")
    stab = torch.tensor([[0], [9], [2]], dtype=torch.int32, device="cuda")
    lens = torch.tensor([16, 3, 5], dtype=torch.int32, device="cuda")
    shape = B.make_shape(3, 1, 4, Hkv, 4, 1, 1)
    kn = torch.ones(3, Hkv, 128, dtype=torch.bfloat16, device="cuda"); vn = 2 * kn
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.marl_kv_append(shape, kn, vn, k, v, stab, lens, flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == (B.FLAG_LEN_CLAMPED | B.FLAG_BAD_PAGE)
    assert lens.tolist() == [16, 3, 6]
    assert float(k.float().sum()) == Hkv * 128 and float(v.float().sum()) == 2 * Hkv * 128
    assert bool((k[2, :, 5] == 1).all()) and bool((v[2, :, :, 5] == 2).all())


def test_copy_pages_bit_exact():
    print("case: kv copy pages", flush=True)
    cpu = I.build_attn_inputs(I.WORKLOADS["tiny"])
    dev = cpu.to("cuda")
    shape = B.make_shape(cpu.num_seqs, cpu.num_groups, cpu.Hq, cpu.Hkv, cpu.num_pages, 16, 8)
    rng = np.random.default_rng(2)
    ids = rng.permutation(cpu.num_pages)
    src, dst = ids[:10].astype(np.int32), ids[10:20].astype(np.int32)
    src[3] = cpu.num_pages + 5          # skipped and flagged
    kb, vb, f = ref.kv_copy_pages(I.bf16_bits(cpu.k_pages), I.bf16_bits(cpu.v_pages), src, dst)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.marl_kv_copy_pages(shape, dev.k_pages, dev.v_pages, torch.from_numpy(src).cuda(), torch.from_numpy(dst).cuda(), flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == f == B.FLAG_BAD_PAGE
    assert np.array_equal(I.bf16_bits(dev.k_pages), kb) and np.array_equal(I.bf16_bits(dev.v_pages), vb)
