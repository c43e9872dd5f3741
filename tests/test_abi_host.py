"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_2602_09578_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "marl_decode.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(marl_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = B.load_library()
    names = declared_symbols()
    assert {"marl_decode_attn", "marl_token_logprobs", "marl_workspace_bytes", "marl_attn_plan"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert lib.marl_version() >= 1


def good_shape(**kw):
    d = dict(num_seqs=16, num_groups=4, num_q_heads=8, num_kv_heads=2, num_pages=100,
             max_prefix_pages=16, max_suffix_pages=8)
    d.update(kw)
    return B.make_shape(**d)


def status_of(fn):
    try:
        fn()
    except B.MarlError as e:
        return e.status
    return 0


def test_layout_and_default_chunks():
    L = B.marl_attn_plan_layout_for(good_shape())
    assert (L.suffix_chunk_tokens, L.prefix_chunk_tokens) == (256, 256)
    assert (L.suffix_slots, L.prefix_slots, L.rows_per_qblock) == (1, 1, 128)
    assert L.total_bytes == B.marl_workspace_bytes(good_shape())
    offs = [L.counters_off, L.group_count_off, L.group_start_off, L.seq_rank_off, L.group_tmp_off, L.group_seqs_off, L.seq_chunks_off,
            L.suffix_items_off, L.prefix_items_off, L.partial_ml_off, L.partial_o_off, L.total_bytes]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs) and offs[0] == 0
    assert L.partial_o_off + 16 * 8 * 2 * 128 * 4 <= L.total_bytes
    big = B.marl_attn_plan_layout_for(good_shape(num_seqs=2048, num_groups=256, num_q_heads=28, num_kv_heads=4,
                                                 max_prefix_pages=128, max_suffix_pages=512))
    assert (big.suffix_chunk_tokens, big.prefix_chunk_tokens, big.suffix_slots, big.prefix_slots) == (8192, 8192, 1, 1)
    ov = B.marl_attn_plan_layout_for(good_shape(suffix_chunk_tokens=64, prefix_chunk_tokens=96))
    assert (ov.suffix_chunk_tokens, ov.prefix_chunk_tokens, ov.suffix_slots, ov.prefix_slots) == (64, 96, 2, 3)


@pytest.mark.parametrize("kw,status", [
    (dict(num_seqs=-1), -1), (dict(num_q_heads=7), -1), (dict(num_kv_heads=0), -1), (dict(num_pages=0), -1),
    (dict(head_dim=64), -2), (dict(page_size=32), -2), (dict(out_dtype=5), -2),
    (dict(suffix_chunk_tokens=48), -2), (dict(prefix_chunk_tokens=16), -2),
    (dict(num_q_heads=34, num_kv_heads=2), -2)])
def test_bad_shapes_are_rejected_on_the_host(kw, status):
    assert status_of(lambda: B.marl_workspace_bytes(good_shape(**kw))) == status


def test_decode_attn_argument_errors_without_gpu():
    lib = B.load_library()
    shape = good_shape()
    need = B.marl_workspace_bytes(shape)
    buf = ctypes.create_string_buffer(need + 512)
    base = (ctypes.addressof(buf) + 255) // 256 * 256
    p = ctypes.c_void_p(base)
    call = lambda ws, nbytes, q, scale: lib.marl_decode_attn(ctypes.byref(shape), ws, nbytes, q, p, p, p, p, p, p, p,
                                                            ctypes.c_float(scale), p, None)
    assert call(None, need, p, 1.0) == -1                      # null workspace
    assert call(ctypes.c_void_p(base + 8), need, p, 1.0) == -1  # misaligned workspace
    assert call(p, need - 1, p, 1.0) == -3                     # too small
    assert call(p, need, None, 1.0) == -1                      # null q
    assert call(p, need, ctypes.c_void_p(base + 2), 1.0) == -1  # q not 16-byte aligned
    odd = ctypes.c_void_p(base + 8)
    for at in range(4):                                        # q, k_pages, v_pages, out in turn
        args = [p, p, p] + [p] * 5 + [ctypes.c_float(1.0), p]
        args[[0, 1, 2, 9][at]] = odd
        assert lib.marl_decode_attn(ctypes.byref(shape), p, need, *args, None) == -1
    assert call(p, need, p, float("nan")) == -1
    assert call(p, need, p, float("inf")) == -1
    assert lib.marl_decode_attn(None, p, need, p, p, p, p, p, p, p, p, ctypes.c_float(1.0), p, None) == -1


def test_logprobs_argument_errors_without_gpu():
    lib = B.load_library()
    buf = ctypes.create_string_buffer(1024)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    f = lambda logits, T, rows, vocab, ws=None, n=0: lib.marl_token_logprobs(logits, p, ctypes.c_float(T), p, rows, vocab, ws, n, None)
    assert f(p, 0.0, 4, 100) == -1 and f(p, -1.0, 4, 100) == -1 and f(p, float("nan"), 4, 100) == -1
    assert f(None, 1.0, 4, 100) == -1
    assert f(p, 1.0, -1, 100) == -1 and f(p, 1.0, 4, 0) == -1
    assert f(p, 1.0, 0, 100) == 0                              # nothing to do
    assert f(p, 1.0, 4, 152064, None, 0) == -1                 # sliced launch needs a workspace
    assert f(p, 1.0, 4, 152064, p, 8) == -3
    assert B.marl_logprobs_workspace_bytes(2048, 152064) == 0
    assert B.marl_logprobs_workspace_bytes(256, 152064) == 256 * 4 * 8        # four vocabulary slices per row
    assert lib.marl_status_string(-3) == b"workspace too small"


def test_profile_argument_errors():
    lib = B.load_library()
    assert lib.marl_profile_begin(0) == -1
    assert lib.marl_profile_end(None, None, None) == -1


def test_kv_cache_argument_errors_without_gpu():
    lib = B.load_library()
    shape = good_shape()
    buf = ctypes.create_string_buffer(1024)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    ap = lambda k_new, lens, sh=shape: lib.marl_kv_append(ctypes.byref(sh), k_new, p, p, p, p, lens, None, None)
    assert ap(None, p) == -1 and ap(p, None) == -1
    assert ap(ctypes.c_void_p(p.value + 4), p) == -1               # k_new not 16-byte aligned
    assert ap(p, p, good_shape(max_suffix_pages=0)) == -1          # no room for any token
    assert ap(p, p, good_shape(head_dim=64)) == -2
    assert ap(p, p, good_shape(num_seqs=0)) == 0                   # nothing to do
    cp = lambda src, n: lib.marl_kv_copy_pages(ctypes.byref(shape), p, p, src, p, n, None, None)
    assert cp(p, -1) == -1 and cp(None, 3) == -1 and cp(p, 0) == 0


def test_plan_entry_argument_errors_without_gpu():
    lib = B.load_library()
    shape = good_shape()
    need = B.marl_workspace_bytes(shape)
    buf = ctypes.create_string_buffer(need + 512)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    assert lib.marl_attn_plan(ctypes.byref(shape), p, need, None, p, p, None) == -1
    assert lib.marl_attn_plan(ctypes.byref(shape), p, need - 256, p, p, p, None) == -3
    assert lib.marl_attn_read_flags(None, None, None) == -1


def test_grpo_argument_errors_without_gpu():
    lib = B.load_library()
    buf = ctypes.create_string_buffer(1024)
    p = ctypes.c_void_p(ctypes.addressof(buf))
    f = lambda r, ng, eps: lib.marl_grpo_advantages(r, p, p, ng, ctypes.c_float(eps), p, None)
    assert f(p, -1, 0.0) == -1 and f(p, 2, -1e-3) == -1 and f(p, 2, float("inf")) == -1
    assert f(None, 2, 0.0) == -1
    assert f(None, 0, 0.0) == 0                                    # nothing to do


def test_prefill_argument_errors_without_gpu():
    lib = B.load_library()
    buf = ctypes.create_string_buffer(2048)
    p = ctypes.c_void_p((ctypes.addressof(buf) + 255) // 256 * 256)
    mk = lambda **kw: B.make_prefill_shape(**{**dict(num_tokens=64, num_groups=2, num_q_heads=28, num_kv_heads=4,
                                                     num_pages=16, max_prefix_pages=4), **kw})
    n = ctypes.c_size_t(0)
    assert lib.marl_prefill_workspace_bytes(ctypes.byref(mk()), ctypes.byref(n)) == 0 and n.value == 768   # header + starts + (64*7/128 + 2) items
    assert lib.marl_prefill_workspace_bytes(ctypes.byref(mk(num_q_heads=30)), ctypes.byref(n)) == -1
    assert lib.marl_prefill_workspace_bytes(ctypes.byref(mk(head_dim=64)), ctypes.byref(n)) == -2
    assert lib.marl_prefill_workspace_bytes(ctypes.byref(mk(num_q_heads=68)), ctypes.byref(n)) == -2   # 17 heads per KV head
    at = lambda sh, ws, nbytes, q, scale=1.0: lib.marl_prefill_attn(ctypes.byref(sh), ws, nbytes, q, p, p, p, p, p,
                                                                     ctypes.c_float(scale), p, None)
    assert at(mk(), p, 768, None) == -1 and at(mk(), None, 768, p) == -1
    assert at(mk(), p, 768, p, float("nan")) == -1
    assert at(mk(), p, 512, p) == -3
    assert at(mk(max_prefix_pages=0), p, 768, p) == -1
    assert at(mk(num_tokens=0), None, 0, None) == 0              # nothing to do
    wr = lambda sh, k_new: lib.marl_kv_write_prompt(ctypes.byref(sh), k_new, p, p, p, p, p, p, None, None)
    assert wr(mk(), None) == -1 and wr(mk(num_groups=0), None) == 0 and wr(mk(page_size=32), p) == -2
    # keys are copied, and whole value pages stored, as 16-byte vectors
    off = ctypes.c_void_p(p.value + 8)
    wr5 = lambda k_new, k_pages, v_pages: lib.marl_kv_write_prompt(ctypes.byref(mk()), k_new, p, k_pages, v_pages,
                                                                   p, p, p, None, None)
    assert wr5(off, p, p) == -1 and wr5(p, off, p) == -1 and wr5(p, p, off) == -1


def test_balancer_takes_sparse_request_ids_and_reports_status_codes():
    """Request ids are arbitrary non-negative int32 values (a hash, say): the id map must not be
    sized by the largest id, and no error may leave the library as an exception."""
    bal = B.Balancer([2, 1], delta=5)
    big = 2 ** 31 - 1
    assert bal.submit(0, big, 3) in (0, 1)
    assert bal.submit(1, 2 ** 30 + 12345, 2) == 2
    assert bal.submit(0, 7, 1) in (0, 1)
    with pytest.raises(B.MarlError) as e:
        bal.submit(0, big, 3)                      # ids are unique
    assert e.value.status == -1
    for _ in range(3):
        bal.step()
    assert bal.request_state(big)[2] == 2          # finished in the third step (0-based step 2)
    assert bal.request_state(7)[2] == 0
    with pytest.raises(B.MarlError):
        bal.request_state(8)                       # unknown id
    assert B.load_library().marl_status_string(-5) == b"out of host memory"
    bal.close()


def test_binding_refuses_wrong_dtypes_and_extents():
    """The kernels reinterpret raw bytes: torch's default int64 for an index tensor, or float32 where
    bf16 is expected, must be an error in the binding, not a wrong result."""
    import torch
    logits = torch.zeros((4, 100), dtype=torch.bfloat16)
    out = torch.zeros(4, dtype=torch.float32)
    with pytest.raises(ValueError, match="tokens: expected dtype torch.int32"):
        B.marl_token_logprobs(logits, torch.zeros(4, dtype=torch.int64), 1.0, out)
    with pytest.raises(ValueError, match="logits: expected dtype torch.bfloat16"):
        B.marl_token_logprobs(logits.float(), torch.zeros(4, dtype=torch.int32), 1.0, out)
    with pytest.raises(ValueError, match="out: expected shape"):
        B.marl_token_logprobs(logits, torch.zeros(4, dtype=torch.int32), 1.0, torch.zeros(5))
    shape = good_shape()
    ws = torch.zeros(256, dtype=torch.uint8)
    q = torch.zeros((16, 8, 128), dtype=torch.bfloat16)
    kv = torch.zeros((100, 2, 16, 128), dtype=torch.bfloat16)
    vv = torch.zeros((100, 2, 128, 16), dtype=torch.bfloat16)
    pt, st = torch.zeros((4, 16), dtype=torch.int32), torch.zeros((16, 8), dtype=torch.int32)
    pl, sl, gos = torch.zeros(4, dtype=torch.int32), torch.zeros(16, dtype=torch.int32), torch.zeros(16, dtype=torch.int32)
    o = torch.zeros((16, 8, 128), dtype=torch.bfloat16)
    call = lambda **kw: B.marl_decode_attn(shape, ws, **{**dict(q=q, k_pages=kv, v_pages=vv, prefix_block_table=pt,
                                                               suffix_block_table=st, prefix_lens=pl, suffix_lens=sl,
                                                               group_of_seq=gos, scale=1.0, out=o), **kw})
    with pytest.raises(ValueError, match="suffix_lens: expected dtype"):
        call(suffix_lens=sl.long())
    with pytest.raises(ValueError, match="v_pages: expected shape"):
        call(v_pages=kv)                       # the key layout passed for the values
    with pytest.raises(ValueError, match="out: expected dtype"):
        call(out=o.float())
    with pytest.raises(ValueError, match="device tensors required"):
        call()                                 # everything right except that these are host tensors


def test_bench_refuses_more_than_one_gpu():
    """The benchmark measures one GPU; asked for more it says so and exits without touching a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)
