"""marl_decode_attn_static (the entry point that allocates nothing: its workspace is a fixed array
inside the library) against marl_decode_attn on the same inputs, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I
from tests.gpu_common import ATTN_TOL, oracle_attn


def _both(inp_cpu, out_dtype):
    dev = inp_cpu.to("cuda")
    call = B.prepare_attn(dev, out_dtype)
    assert call.layout.total_bytes <= B.STATIC_WORKSPACE_BYTES
    B.run_attn(dev, call)
    torch.cuda.synchronize()
    assert B.marl_attn_read_flags(call.workspace) == 0
    want = call.out.clone()
    out = torch.full_like(call.out, 7.0)
    flags = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    # everything the call needs exists before it: from here to the synchronize nothing allocates
    B.marl_decode_attn_static(call.shape, dev.q, dev.k_pages, dev.v_pages, dev.prefix_block_table,
                              dev.suffix_block_table, dev.prefix_lens, dev.suffix_lens, dev.group_of_seq,
                              dev.scale, out, flags)
    torch.cuda.synchronize()
    return want, out, int(flags.item())


@pytest.mark.gpu
def test_static_workspace_entry_matches_the_workspace_entry_on_two_calls_in_a_row():
    """A larger call, then a smaller one on the same (now dirty) array: each must equal
    marl_decode_attn bit for bit (same kernels, fixed summation order) and meet the bar
    against the float64 checker."""
    print("case: static workspace, scaled qwen7b then tiny", flush=True)
    big = I.build_attn_inputs(I.WORKLOADS["qwen7b"].scaled(8, 4))
    small = I.build_attn_inputs(I.WORKLOADS["tiny"])
    for inp, dt in ((big, B.MARL_OUT_BF16), (small, B.MARL_OUT_F32)):
        want, got, flags = _both(inp, dt)
        assert flags == 0
        assert torch.equal(want, got)
        err = float(np.abs(got.float().cpu().numpy().astype(np.float64) - oracle_attn(inp)).max())
        print("seqs", inp.num_seqs, "max |delta| vs checker", err, flush=True)
        assert err <= ATTN_TOL


@pytest.mark.gpu
def test_static_workspace_entry_reports_flags_and_handles_empty_batches():
    print("case: static workspace, flags", flush=True)
    w = I.Workload("custom", 8, 2, (), 13)
    L = I.Lengths(np.array([40, 20], np.int32), np.array([30, 10, 25], np.int32), np.array([0, 1, 1], np.int32),
                  np.zeros(2, np.int32))
    inp = I.build_attn_inputs(w, "cpu", 13, poison=False, lengths=L)
    inp.suffix_block_table = inp.suffix_block_table.clone()
    inp.suffix_block_table[2, 0] = 10 ** 8
    dev = inp.to("cuda")
    call = B.prepare_attn(dev, B.MARL_OUT_F32)
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.marl_decode_attn_static(call.shape, dev.q, dev.k_pages, dev.v_pages, dev.prefix_block_table,
                              dev.suffix_block_table, dev.prefix_lens, dev.suffix_lens, dev.group_of_seq,
                              dev.scale, call.out, flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == B.FLAG_BAD_PAGE
    assert torch.isfinite(call.out).all().item()
    # an empty batch runs no kernel of the path and reports no flag
    empty = B.make_shape(0, 0, 8, 2, 1, 0, 0, B.MARL_OUT_F32)
    flags.fill_(-1)
    no_rows = torch.empty((0, 8, 128), dtype=torch.float32, device="cuda")
    B.marl_decode_attn_static(empty, None, None, None, None, None, None, None, None, 1.0, no_rows, flags)
    torch.cuda.synchronize()
    assert int(flags.item()) == 0


def test_static_workspace_entry_rejects_oversized_shapes_on_the_host():
    """The skew workload's shape needs 160 MiB of workspace: more than the fixed array holds.
    The refusal comes before any HIP call, so this runs without a GPU."""
    lib = B.load_library()
    shape = B.make_shape(3840, 480, 28, 4, 300000, 64, 1024)
    assert B.marl_workspace_bytes(shape) > B.STATIC_WORKSPACE_BYTES
    p = ctypes.c_void_p(4096)
    rc = lib.marl_decode_attn_static(ctypes.byref(shape), p, p, p, p, p, p, p, p, ctypes.c_float(1.0), p, None, None)
    assert rc == -3
    ok = B.make_shape(16, 4, 8, 2, 100, 16, 8)
    assert lib.marl_decode_attn_static(ctypes.byref(ok), None, p, p, p, p, p, p, p, ctypes.c_float(1.0), p, None, None) == -1
    assert lib.marl_decode_attn_static(ctypes.byref(ok), p, p, p, p, p, p, p, p, ctypes.c_float(float("nan")), p, None, None) == -1
    assert lib.marl_decode_attn_static(ctypes.byref(ok), p, p, p, p, p, p, p, p, ctypes.c_float(1.0), p,
                                       ctypes.c_void_p(4098), None) == -1
