"""The seeded generators: determinism, structure and poison (CPU only)."""
import numpy as np
import torch

from paper_2602_09578_amd import inputs as I


def test_workload_shapes_match_the_named_configs():
    w = I.WORKLOADS
    assert (w["tiny"].num_seqs, w["tiny"].num_groups) == (16, 4)
    assert (w["qwen7b"].num_seqs, w["qwen7b"].num_groups) == (2048, 256)
    assert (w["skew"].num_seqs, w["skew"].num_groups) == (3840, 480)
    assert (w["prefix"].num_seqs, w["prefix"].num_groups) == (2048, 64)
    assert (w["long32b"].num_seqs, w["long32b"].num_groups) == (256, 64)
    L = I.draw_lengths(w["qwen7b"], np.random.default_rng(w["qwen7b"].seed))
    assert L.prefix_lens.min() >= 512 and L.prefix_lens.max() <= 2048
    assert L.suffix_lens.min() >= 1 and L.suffix_lens.max() <= 8192
    med = [np.median(L.suffix_lens[a * 512:(a + 1) * 512]) for a in range(4)]
    assert med[0] < med[1] < med[2] < med[3]
    L = I.draw_lengths(w["skew"], np.random.default_rng(1))
    assert L.suffix_lens[:256].min() >= 12288 and L.suffix_lens[:256].max() <= 16384
    assert L.suffix_lens[256:].min() >= 16 and L.suffix_lens[256:].max() <= 256


def test_tiny_inputs_deterministic_and_poisoned():
    a = I.build_attn_inputs(I.WORKLOADS["tiny"])
    b = I.build_attn_inputs(I.WORKLOADS["tiny"])
    assert torch.equal(a.q.view(torch.int16), b.q.view(torch.int16))
    assert torch.equal(a.k_pages.view(torch.int16), b.k_pages.view(torch.int16))
    assert torch.equal(a.suffix_block_table, b.suffix_block_table)
    pt, st = a.prefix_block_table.numpy(), a.suffix_block_table.numpy()
    used = np.concatenate([pt[pt >= 0], st[st >= 0]])
    assert len(np.unique(used)) == len(used) and used.max() < a.num_pages
    assert len(used) < a.num_pages                      # spare pages exist
    free = np.setdiff1d(np.arange(a.num_pages), used)
    assert torch.isnan(a.k_pages[free].float()).all() and torch.isnan(a.v_pages[free].float()).all()
    # valid slots are finite, slots past the end of a partial page are NaN
    for s in range(a.num_seqs):
        S = int(a.suffix_lens[s]); last = st[s, (S - 1) // 16]; n = S - (S - 1) // 16 * 16
        assert torch.isfinite(a.k_pages[last, :, :n].float()).all()
        assert torch.isfinite(a.v_pages[last, :, :, :n].float()).all()
        if n < 16:
            assert torch.isnan(a.k_pages[last, :, n:].float()).all()
            assert torch.isnan(a.v_pages[last, :, :, n:].float()).all()


def test_extract_subproblem_preserves_bytes():
    a = I.build_attn_inputs(I.WORKLOADS["tiny"])
    sub = I.extract_subproblem(a, [5, 14])
    assert sub.num_seqs == 2 and sub.num_groups == 2
    for i, s in enumerate([5, 14]):
        S = int(a.suffix_lens[s])
        assert int(sub.suffix_lens[i]) == S
        for p in range((S + 15) // 16):
            old, new = int(a.suffix_block_table[s, p]), int(sub.suffix_block_table[i, p])
            assert torch.equal(a.k_pages[old].view(torch.int16), sub.k_pages[new].view(torch.int16))
            assert torch.equal(a.v_pages[old].view(torch.int16), sub.v_pages[new].view(torch.int16))
        g = int(a.group_of_seq[s]); gi = int(sub.group_of_seq[i])
        assert int(sub.prefix_lens[gi]) == int(a.prefix_lens[g])
        old, new = int(a.prefix_block_table[g, 3]), int(sub.prefix_block_table[gi, 3])
        assert torch.equal(a.k_pages[old].view(torch.int16), sub.k_pages[new].view(torch.int16))
        assert torch.equal(a.q[s].view(torch.int16), sub.q[i].view(torch.int16))


def test_logprob_inputs_forced_rows():
    lp = I.build_logprob_inputs(16, 4096, 2.0, 2049)
    assert int(lp.tokens[0]) == 0 and int(lp.tokens[1]) == 4095
    assert int(lp.tokens[2]) == int(torch.argmax(lp.logits[2].float()))
    assert 1.8 < float(lp.logits.float().std()) < 2.2
