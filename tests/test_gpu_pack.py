"""One-copy weight synchronisation on the GPU: marl_pack_tensors / marl_unpack_tensors against the
definition in oracle/reference.py (bit-exact: pure data movement)."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_tensors(seed, sizes_dtypes, misalign=()):
    """Random tensors (bit patterns, not values); those listed in `misalign` start 1 byte into a buffer."""
    g = torch.Generator().manual_seed(seed)
    out = []
    for k, (n, dt) in enumerate(sizes_dtypes):
        nbytes = n * torch.empty(0, dtype=dt).element_size()
        raw = torch.randint(0, 256, (nbytes + 1,), dtype=torch.uint8, generator=g).to(DEV)
        if k in misalign:
            assert dt == torch.uint8
            out.append(raw[1:])
        else:
            out.append(raw[:nbytes].view(dt))
    return out


def host_bytes(t):
    return t.contiguous().view(torch.uint8).cpu().numpy().reshape(-1)


CASES = [
    # sizes around the 16-byte vector, the 256-byte offset alignment and the 262144-byte chunk; empty tensors
    [(1, torch.uint8), (15, torch.uint8), (16, torch.uint8), (17, torch.uint8), (0, torch.float32),
     (131071, torch.bfloat16), (131072, torch.bfloat16), (131073, torch.bfloat16), (65537, torch.float32),
     (0, torch.uint8), (3 * 262144 + 5, torch.uint8), (7, torch.int64)],
    # a small transformer's parameter list: two layers of (q, k, v, o, gate, up, down, 2 norms) + embedding
    [(512 * 896, torch.bfloat16)] + 2 * [(896 * 896, torch.bfloat16), (896, torch.bfloat16), (128 * 896, torch.bfloat16),
                                          (128, torch.bfloat16), (128 * 896, torch.bfloat16), (128, torch.bfloat16),
                                          (896 * 896, torch.bfloat16), (4864 * 896, torch.bfloat16),
                                          (4864 * 896, torch.bfloat16), (896 * 4864, torch.bfloat16),
                                          (896, torch.bfloat16), (896, torch.bfloat16)] + [(896, torch.bfloat16)],
]


@pytest.mark.parametrize("case", range(len(CASES)))
def test_pack_then_unpack_is_the_reference_layout(case):
    print("case: pack", case, flush=True)
    tensors = make_tensors(case, CASES[case])
    table = B.PackTable(tensors)
    want, offsets = ref.pack_tensors([host_bytes(t) for t in tensors], fill=0xAB)
    assert table.offsets == offsets and table.packed_bytes == want.size
    packed = torch.full((table.packed_bytes + 64,), 0xAB, dtype=torch.uint8, device=DEV)
    B.marl_pack_tensors(table, packed)
    torch.cuda.synchronize()
    got = packed.cpu().numpy()
    assert np.array_equal(got[:want.size], want)          # tensors in place, gaps untouched
    assert (got[want.size:] == 0xAB).all()                # nothing written past the end
    # scatter into fresh tensors of the same shapes
    fresh = [torch.zeros_like(t) for t in tensors]
    table2 = B.PackTable(fresh)
    assert table2.offsets == offsets
    B.marl_unpack_tensors(table2, packed)
    torch.cuda.synchronize()
    for a, b in zip(tensors, fresh):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_tensors_that_are_not_16_byte_aligned():
    print("case: pack misaligned", flush=True)
    sizes = [(1000, torch.uint8), (262144 + 33, torch.uint8), (4096, torch.float32), (31, torch.uint8)]
    tensors = make_tensors(7, sizes, misalign=(0, 1, 3))
    assert tensors[1].data_ptr() % 16 != 0
    table = B.PackTable(tensors)
    want, _ = ref.pack_tensors([host_bytes(t) for t in tensors], fill=0)
    packed = torch.zeros(table.packed_bytes, dtype=torch.uint8, device=DEV)
    B.marl_pack_tensors(table, packed)
    torch.cuda.synchronize()
    assert np.array_equal(packed.cpu().numpy(), want)
    fresh = make_tensors(8, sizes, misalign=(0, 1, 3))
    B.marl_unpack_tensors(B.PackTable(fresh), packed)
    torch.cuda.synchronize()
    for a, b in zip(tensors, fresh):
        assert torch.equal(a.view(torch.uint8), b.view(torch.uint8))


def test_empty_table_and_rerun():
    B.marl_pack_tensors(B.PackTable([]), torch.zeros(1, dtype=torch.uint8, device=DEV))
    tensors = make_tensors(3, [(100000, torch.bfloat16)] * 5)
    table = B.PackTable(tensors)
    p1 = torch.zeros(table.packed_bytes, dtype=torch.uint8, device=DEV)
    p2 = torch.zeros(table.packed_bytes, dtype=torch.uint8, device=DEV)
    B.marl_pack_tensors(table, p1)
    B.marl_pack_tensors(table, p2)
    torch.cuda.synchronize()
    assert torch.equal(p1, p2)
