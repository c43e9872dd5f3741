"""Host side of the one-copy weight synchronisation: the plan (offsets, chunk counts) against the
definition in oracle/reference.py, which is itself pinned by a hand-written layout."""
import ctypes

import numpy as np
import pytest

from oracle import reference as ref
from paper_2602_09578_amd import binding as B


def test_reference_layout_by_hand():
    # sizes 1, 256, 257, 0, 262145 -> starts 0, 256, 512, 1024 (769 rounded up), 1024; chunks 1, 1, 1, 0, 2
    off, first, total, chunks = ref.pack_layout([1, 256, 257, 0, 262145])
    assert off == [0, 256, 512, 1024, 1024] and first == [0, 1, 2, 3, 3]
    assert total == 1024 + 262145 and chunks == 5
    packed, offsets = ref.pack_tensors([np.arange(3, dtype=np.uint8), np.array([0x0102], dtype=np.uint16)], fill=9)
    assert offsets == [0, 256] and packed.size == 258
    assert list(packed[:4]) == [0, 1, 2, 9] and list(packed[254:258]) == [9, 9, 2, 1]   # little endian


def plan(sizes):
    lib = B.load_library()
    n = len(sizes)
    ent = (B.PackEntry * max(n, 1))()
    for k, s in enumerate(sizes):
        ent[k].ptr = 0x1000 + k if s else None
        ent[k].bytes = s
    nbytes, chunks = ctypes.c_uint64(0), ctypes.c_int64(0)
    rc = lib.marl_pack_plan(ent, n, ctypes.byref(nbytes), ctypes.byref(chunks))
    return rc, [ent[k].offset for k in range(n)], [ent[k].first_chunk for k in range(n)], nbytes.value, chunks.value


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_plan_matches_the_reference_layout(seed):
    rng = np.random.default_rng(seed)
    sizes = [int(x) for x in rng.choice([0, 1, 15, 16, 255, 256, 257, 7168, 262143, 262144, 262145, 3 * 262144 + 5,
                                         50_000_000], size=40)]
    rc, off, first, total, chunks = plan(sizes)
    assert rc == 0
    assert (off, first, total, chunks) == ref.pack_layout(sizes)


def test_plan_and_call_argument_errors():
    lib = B.load_library()
    nbytes, chunks = ctypes.c_uint64(0), ctypes.c_int64(0)
    assert plan([])[0] == 0
    assert lib.marl_pack_plan(None, 1, ctypes.byref(nbytes), ctypes.byref(chunks)) == -1
    assert lib.marl_pack_plan(None, -1, ctypes.byref(nbytes), ctypes.byref(chunks)) == -1
    ent = (B.PackEntry * 1)()
    ent[0].ptr, ent[0].bytes = None, 8          # bytes without an address
    assert lib.marl_pack_plan(ent, 1, ctypes.byref(nbytes), ctypes.byref(chunks)) == -1
    ent[0].ptr, ent[0].bytes = 0x1000, 1 << 50   # more chunks than the kernel's index holds
    assert lib.marl_pack_plan(ent, 1, ctypes.byref(nbytes), ctypes.byref(chunks)) == -1
    # device calls validate before touching the GPU
    assert lib.marl_pack_tensors(None, 0, 0, None, None) == 0
    assert lib.marl_pack_tensors(None, 3, 5, None, None) == -1
    assert lib.marl_unpack_tensors(None, -1, 0, None, None) == -1
    assert lib.marl_pack_tensors(None, 1, -2, None, None) == -1
