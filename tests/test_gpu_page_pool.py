"""Fork and copy-on-write end to end: the page pool decides (host), marl_kv_copy_pages and
marl_kv_append act (device), and every sample's logical keys and values must be exactly the
tokens it was given, whatever pages it shares or has left; then attention over the final state."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I
from tests.gpu_common import ATTN_TOL

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
HQ, HKV, MAXP, NUM_PAGES = 8, 2, 6, 40


def test_forked_samples_diverge_without_disturbing_each_other():
    print("case: page pool fork / copy-on-write", flush=True)
    gen = torch.Generator().manual_seed(11)
    rng = np.random.default_rng(11)
    pool = B.PagePool(NUM_PAGES)
    nan = float("nan")
    k_pages = torch.full((NUM_PAGES, HKV, 16, 128), nan, dtype=torch.bfloat16, device=DEV)
    v_pages = torch.full((NUM_PAGES, HKV, 128, 16), nan, dtype=torch.bfloat16, device=DEV)
    # the shared prompt: 40 tokens in 3 pages of their own (written with the prompt scatter's sibling, append)
    P = 40
    rc, ppages = pool.alloc(3)
    assert rc == 0
    prefix_table = np.full((1, 3), -1, dtype=np.int32)
    prefix_table[0] = ppages
    rows = [np.full(MAXP, -1, dtype=np.int32)]     # host mirrors of the suffix table rows
    lens = [0]
    tokens = [[]]                                   # per sample: the (k, v) bits of every token it was given
    flags = torch.zeros(1, dtype=torch.int32, device=DEV)

    def step(new_tokens_for):
        """One decode iteration for the listed samples: host bookkeeping, device copies, device append."""
        ns = len(rows)
        copies = []
        for s in new_tokens_for:
            rc, src, dst = pool.prepare_append(rows[s], lens[s])
            assert rc == 0
            if src >= 0:
                copies.append((src, dst))
        shape = B.make_shape(ns, 1, HQ, HKV, NUM_PAGES, 3, MAXP, B.MARL_OUT_F32)
        if copies:
            src = torch.tensor([c[0] for c in copies], dtype=torch.int32, device=DEV)
            dst = torch.tensor([c[1] for c in copies], dtype=torch.int32, device=DEV)
            B.marl_kv_copy_pages(shape, k_pages, v_pages, src, dst, flags)
        # the append entry point serves every row of the table it is given: it gets the rows that take a token
        sel = list(new_tokens_for)
        sub = B.make_shape(len(sel), 1, HQ, HKV, NUM_PAGES, 3, MAXP, B.MARL_OUT_F32)
        k_new = torch.randn(len(sel), HKV, 128, generator=gen).to(torch.bfloat16)
        v_new = torch.randn(len(sel), HKV, 128, generator=gen).to(torch.bfloat16)
        table = torch.from_numpy(np.stack([rows[s] for s in sel])).to(DEV)
        lens_dev = torch.tensor([lens[s] for s in sel], dtype=torch.int32, device=DEV)
        B.marl_kv_append(sub, k_new.to(DEV), v_new.to(DEV), k_pages, v_pages, table, lens_dev, flags)
        torch.cuda.synchronize()
        for j, s in enumerate(sel):
            tokens[s].append((I.bf16_bits(k_new[j]), I.bf16_bits(v_new[j])))
            lens[s] += 1
        assert lens_dev.cpu().tolist() == [lens[s] for s in sel]
        return len(copies)

    def fork(s):
        child = np.full(MAXP, -1, dtype=np.int32)
        assert pool.fork(rows[s], lens[s], child) == 0
        rows.append(child); lens.append(lens[s]); tokens.append(list(tokens[s]))

    ncopies = 0
    for _ in range(21):
        ncopies += step([0])                 # sample 0 generates 21 tokens: one full page, five tokens in the second
    assert ncopies == 0
    fork(0); fork(0)                         # samples 1 and 2 share both pages with sample 0
    assert pool.refcount(int(rows[0][1])) == 3
    ncopies += step([0, 1])                  # both write into the shared second page: two copies, sample 2 keeps it
    assert ncopies == 2 and len({int(r[1]) for r in rows}) == 3 and pool.refcount(int(rows[2][1])) == 1
    for _ in range(12):
        ncopies += step([0, 1, 2])           # past the page boundary at 32; sample 2's first write is in place
    assert ncopies == 2
    fork(1)                                  # sample 3 forks from 1 at a length of 34: shares three pages
    ncopies += step([3])                     # copy-on-write of the third page only
    ncopies += step([1, 3])                  # sample 1 is the sole holder of its third page again: no copy
    assert ncopies == 3
    assert int(flags.item()) == 0

    # every sample's logical keys and values are exactly what it was given, in order
    kb, vb = I.bf16_bits(k_pages), I.bf16_bits(v_pages)
    for s in range(len(rows)):
        assert lens[s] == len(tokens[s])
        for t, (kt, vt) in enumerate(tokens[s]):
            page, slot = int(rows[s][t // 16]), t % 16
            assert np.array_equal(kb[page, :, slot, :], kt) and np.array_equal(vb[page, :, :, slot], vt), (s, t)
    # reference counts = what the rows hold; dropping everything frees every page
    held = {}
    for s in range(len(rows)):
        for p in rows[s][: -(-lens[s] // 16)]:
            held[int(p)] = held.get(int(p), 0) + 1
    assert all(pool.refcount(p) == c for p, c in held.items())

    # attention over the final state (prompt filled now; its content is independent of the bookkeeping)
    for page in ppages:
        k_pages[page] = torch.randn(HKV, 16, 128, generator=gen).to(torch.bfloat16).to(DEV)
        v_pages[page] = torch.randn(HKV, 128, 16, generator=gen).to(torch.bfloat16).to(DEV)
    ns = len(rows)
    q = torch.randn(ns, HQ, 128, generator=gen).to(torch.bfloat16)
    inp = I.AttnInputs(HQ, HKV, NUM_PAGES, q, k_pages.cpu(), v_pages.cpu(), torch.from_numpy(prefix_table),
                       torch.from_numpy(np.stack(rows)), torch.tensor([P], dtype=torch.int32),
                       torch.tensor(lens, dtype=torch.int32), torch.zeros(ns, dtype=torch.int32), 128 ** -0.5)
    dev = inp.to(DEV)
    call = B.prepare_attn(dev, B.MARL_OUT_F32)
    B.run_attn(dev, call)
    torch.cuda.synchronize()
    want = ref.decode_attn(I.bf16_bits(inp.q), I.bf16_bits(inp.k_pages), I.bf16_bits(inp.v_pages), prefix_table,
                           np.stack(rows), np.array([P], dtype=np.int32), np.array(lens, dtype=np.int32),
                           np.zeros(ns, dtype=np.int32), inp.scale, HQ, HKV)
    assert np.abs(call.out.cpu().numpy().astype(np.float64) - want).max() <= ATTN_TOL
    for s in range(len(rows)):
        assert pool.drop(rows[s], lens[s]) == 0
    assert pool.release(ppages) == 0 and pool.free_pages() == NUM_PAGES
