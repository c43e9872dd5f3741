"""Pins of the reference prompt (prefill) attention and prompt scatter.  The reference is
numpy (matrix products + mask); it is pinned against code written differently: the float64 C
loops of the decode checker (a query at position t is a decode query over a prefix of t+1
tokens), explicit Python loops, torch's causal scaled_dot_product_attention, and properties
that any causal attention has."""
import math

import numpy as np
import pytest
import torch

from oracle import reference as R
from paper_2602_09578_amd import inputs as I


def np_bits(t):
    return I.bf16_bits(t)


def build(Hq, Hkv, lens, pos0, seed=0, poison=True):
    return I.build_prefill_inputs(Hq, Hkv, lens, pos0, device="cpu", seed=seed, poison=poison)


def ref(inp):
    return R.prefill_attn(np_bits(inp.q), np_bits(inp.k_pages), np_bits(inp.v_pages), inp.prefix_block_table.numpy(),
                          inp.q_start.numpy(), inp.q_pos0.numpy(), inp.scale, inp.Hq, inp.Hkv)


def test_every_row_is_a_decode_query_over_its_visible_prefix():
    inp = build(8, 2, [19, 1, 0, 40], [0, 33, 5, 7], seed=3)
    out = ref(inp)
    qs, p0 = inp.q_start.numpy(), inp.q_pos0.numpy()
    NT = inp.num_tokens
    # one decode "sequence" per query token: its own group whose prefix is the visible positions
    gid = np.repeat(np.arange(len(p0)), np.diff(qs))
    table = inp.prefix_block_table.numpy()[gid]
    plens = np.concatenate([p0[g] + 1 + np.arange(qs[g + 1] - qs[g]) for g in range(len(p0))]).astype(np.int32)
    dec = R.decode_attn(np_bits(inp.q), np_bits(inp.k_pages), np_bits(inp.v_pages), table,
                        np.zeros((NT, 1), dtype=np.int32), plens, np.zeros(NT, dtype=np.int32),
                        np.arange(NT, dtype=np.int32), inp.scale, inp.Hq, inp.Hkv)
    assert np.isfinite(out).all()
    np.testing.assert_allclose(out, dec, atol=1e-13)


def test_explicit_loops_on_a_tiny_case():
    inp = build(4, 2, [5, 3], [2, 0], seed=9)
    out = ref(inp)
    q = R.bf16_bits_to_f64(np_bits(inp.q))
    kp, vp = R.bf16_bits_to_f64(np_bits(inp.k_pages)), R.bf16_bits_to_f64(np_bits(inp.v_pages))
    tab, qs, p0 = inp.prefix_block_table.numpy(), inp.q_start.numpy(), inp.q_pos0.numpy()
    for g in range(2):
        for tau in range(qs[g + 1] - qs[g]):
            t = p0[g] + tau
            for h in range(4):
                kh = h // 2
                scores = []
                for j in range(t + 1):
                    krow = kp[tab[g, j // 16], kh, j % 16, :]
                    scores.append(inp.scale * sum(float(a) * float(b) for a, b in zip(q[qs[g] + tau, h], krow)))
                mx = max(scores)
                w = [math.exp(x - mx) for x in scores]
                Z = sum(w)
                for c in (0, 17, 127):
                    acc = sum(w[j] * vp[tab[g, j // 16], kh, c, j % 16] for j in range(t + 1))
                    assert abs(acc / Z - out[qs[g] + tau, h, c]) < 1e-13


@pytest.mark.parametrize("Hq,Hkv,P", [(4, 4, 37), (8, 2, 64)])
def test_torch_causal_sdpa_on_the_unpaged_gather(Hq, Hkv, P):
    inp = build(Hq, Hkv, [P], [0], seed=5)
    out = ref(inp)
    K, V = R.gather_group_kv(np_bits(inp.k_pages), np_bits(inp.v_pages), inp.prefix_block_table.numpy()[0], P)
    rep = Hq // Hkv
    q = inp.q.double().permute(1, 0, 2)                                   # [Hq, P, 128]
    k = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(rep, 0)
    v = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(rep, 0)
    lib = torch.nn.functional.scaled_dot_product_attention(q, k, v, is_causal=True, scale=inp.scale)
    np.testing.assert_allclose(out, lib.permute(1, 0, 2).numpy(), atol=1e-12)


def test_first_token_returns_its_own_value_and_later_keys_do_not_matter():
    inp = build(8, 2, [24], [0], seed=2, poison=False)
    out = ref(inp)
    K, V = R.gather_group_kv(np_bits(inp.k_pages), np_bits(inp.v_pages), inp.prefix_block_table.numpy()[0], 24)
    for h in range(8):
        np.testing.assert_allclose(out[0, h], V[0, h // 4], atol=1e-15)
    # overwrite positions 10.. with other data: rows 0..9 must not change at all
    other = build(8, 2, [24], [0], seed=77, poison=False)
    kp, vp = np_bits(inp.k_pages).copy(), np_bits(inp.v_pages).copy()
    tab = inp.prefix_block_table.numpy()[0]
    for pos in range(10, 24):
        kp[tab[pos // 16], :, pos % 16, :] = np_bits(other.k_pages)[0, :, pos % 16, :]
        vp[tab[pos // 16], :, :, pos % 16] = np_bits(other.v_pages)[0, :, :, pos % 16]
    out2 = R.prefill_attn(np_bits(inp.q), kp, vp, inp.prefix_block_table.numpy(), inp.q_start.numpy(),
                          inp.q_pos0.numpy(), inp.scale, 8, 2)
    np.testing.assert_array_equal(out2[:10], out[:10])
    assert np.abs(out2[10:] - out[10:]).max() > 1e-3


def test_chunked_prefill_equals_one_shot():
    whole = build(8, 2, [45], [0], seed=4)
    out = ref(whole)
    kp, vp, tab = np_bits(whole.k_pages), np_bits(whole.v_pages), whole.prefix_block_table.numpy()
    q = np_bits(whole.q)
    for cut in (1, 16, 30):
        first = R.prefill_attn(q[:cut], kp, vp, tab, [0, cut], [0], whole.scale, 8, 2)
        second = R.prefill_attn(q[cut:], kp, vp, tab, [0, 45 - cut], [cut], whole.scale, 8, 2)
        np.testing.assert_allclose(np.concatenate([first, second]), out, atol=1e-14)


def test_uniform_keys_give_running_means_of_the_values():
    inp = build(2, 1, [20], [0], seed=6, poison=False)
    kp = np_bits(inp.k_pages).copy()
    kp[:] = kp[0, 0, 0, :]                      # every key row identical -> uniform weights
    out = R.prefill_attn(np_bits(inp.q), kp, np_bits(inp.v_pages), inp.prefix_block_table.numpy(),
                         inp.q_start.numpy(), inp.q_pos0.numpy(), inp.scale, 2, 1)
    _, V = R.gather_group_kv(kp, np_bits(inp.v_pages), inp.prefix_block_table.numpy()[0], 20)
    means = np.cumsum(V[:, 0, :], axis=0) / np.arange(1, 21)[:, None]
    np.testing.assert_allclose(out[:, 0, :], means, atol=1e-14)
    np.testing.assert_allclose(out[:, 1, :], means, atol=1e-14)


def test_poison_outside_the_written_positions_is_never_read():
    a = build(8, 2, [21, 3], [4, 0], seed=8, poison=True)
    b = build(8, 2, [21, 3], [4, 0], seed=8, poison=False)
    np.testing.assert_array_equal(ref(a), ref(b))


def test_prompt_scatter_then_gather_returns_the_tokens():
    inp = build(8, 2, [21, 0, 3], [4, 2, 0], seed=10)
    kp, vp = R.kv_write_prompt(np_bits(inp.k_pages), np_bits(inp.v_pages), inp.prefix_block_table.numpy(),
                               inp.q_start.numpy(), inp.q_pos0.numpy(), np_bits(inp.k_new), np_bits(inp.v_new))
    K, V = R.gather_group_kv(kp, vp, inp.prefix_block_table.numpy()[0], 25)
    np.testing.assert_array_equal(K[4:], R.bf16_bits_to_f64(np_bits(inp.k_new)[:21]))
    np.testing.assert_array_equal(V[4:], R.bf16_bits_to_f64(np_bits(inp.v_new)[:21]))
    # positions before pos0 and every other page keep their contents
    K0, V0 = R.gather_group_kv(np_bits(inp.k_pages), np_bits(inp.v_pages), inp.prefix_block_table.numpy()[0], 4)
    np.testing.assert_array_equal(K[:4], K0)
    touched = set(inp.prefix_block_table.numpy()[0, :2].tolist()) | {int(inp.prefix_block_table.numpy()[2, 0])}
    for pg in range(inp.num_pages):
        if pg not in touched:
            assert (kp[pg] == np_bits(inp.k_pages)[pg]).all() and (vp[pg] == np_bits(inp.v_pages)[pg]).all()
