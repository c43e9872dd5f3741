"""Host reference of the decode-attention work list (TEST INFRASTRUCTURE ONLY).

A straightforward Python restatement of what the library's header promises about its plan:
the chunking rule, the group -> sequences CSR, and the set of prefix / suffix work items.
It is integer work, so the GPU plan must match it exactly.  The motivation for a
token-sized, longest-first work list is the paper's observation that rollout load is
heavily skewed across agents (Section 2.2, Observation #2); the paper gives no algorithm
for it, so the rule below is the one written in include/marl_decode.h.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np

PAGE = 16
ROWS_PER_QBLOCK = 128          # query rows of a prefix work item ...
ROWS_PER_QBLOCK_WIDE = 256     # ... when the average group has more than 128 query rows
SHORT_TOKENS = 128     # suffix items above this many tokens head the list


def _ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def rows_per_qblock(NS: int, NG: int, Hq: int, Hkv: int) -> int:
    rows = _ceil_div(NS, NG) * (Hq // Hkv) if NG > 0 else 0
    return ROWS_PER_QBLOCK_WIDE if rows > ROWS_PER_QBLOCK else ROWS_PER_QBLOCK


def default_chunks(NS: int, NG: int, Hq: int, Hkv: int, max_prefix_pages: int, max_suffix_pages: int,
                   suffix_chunk: int = 0, prefix_chunk: int = 0) -> Tuple[int, int]:
    mst, mpt = max_suffix_pages * PAGE, max_prefix_pages * PAGE
    Cs = suffix_chunk
    if Cs == 0:
        Cs = 8192
        while NS * Hkv * _ceil_div(mst, Cs) < 2048 and Cs > 256:
            Cs //= 2
    Cp = prefix_chunk
    if Cp == 0:
        qb = rows_per_qblock(NS, NG, Hq, Hkv)
        rows = _ceil_div(NS, NG) * (Hq // Hkv) if NG > 0 else 0
        qblocks = max(1, _ceil_div(rows, qb))
        Cp = 8192
        want = 256 if qb == ROWS_PER_QBLOCK_WIDE else 512
        while NG * Hkv * qblocks * _ceil_div(mpt, Cp) < want and Cp > 256:
            Cp //= 2
    return Cs, Cp


@dataclass
class PlanRef:
    Cs: int
    Cp: int
    suffix_slots: int
    prefix_slots: int
    group_count: np.ndarray      # int32 [NG]
    group_start: np.ndarray      # int32 [NG+1]
    group_seqs: np.ndarray       # int32 [NS]; within a group ascending sequence id
    suffix_items: List[Tuple[int, int, int, int]]   # (seq, tok_begin, tok_end, 0)
    prefix_items: List[Tuple[int, int, int, int]]   # (group, tok_begin, tok_end, row_begin)
    flags: int
    seq_chunks: np.ndarray = None   # int32 [NS]: prefix chunks | suffix chunks << 16

    @property
    def num_long_suffix_items(self) -> int:
        return sum(1 for it in self.suffix_items if it[2] - it[1] > SHORT_TOKENS)

    @property
    def num_short_partial_items(self) -> int:
        """Suffix items of at most SHORT_TOKENS tokens whose sequence has several suffix chunks
        (counted from the finished item list: how many items name each sequence)."""
        per_seq = {}
        for it in self.suffix_items:
            per_seq[it[0]] = per_seq.get(it[0], 0) + 1
        return sum(1 for it in self.suffix_items
                   if it[2] - it[1] <= SHORT_TOKENS and per_seq[it[0]] >= 2)


def build_plan(prefix_lens, suffix_lens, group_of_seq, Hq: int, Hkv: int, max_prefix_pages: int,
               max_suffix_pages: int, suffix_chunk: int = 0, prefix_chunk: int = 0) -> PlanRef:
    pl = np.asarray(prefix_lens, dtype=np.int64)
    sl = np.asarray(suffix_lens, dtype=np.int64)
    gos = np.asarray(group_of_seq, dtype=np.int64)
    NS, NG = len(sl), len(pl)
    R = Hq // Hkv
    QB = rows_per_qblock(NS, NG, Hq, Hkv)
    Cs, Cp = default_chunks(NS, NG, Hq, Hkv, max_prefix_pages, max_suffix_pages, suffix_chunk, prefix_chunk)
    mst, mpt = max_suffix_pages * PAGE, max_prefix_pages * PAGE
    flags = 0
    members: List[List[int]] = [[] for _ in range(NG)]
    for s in range(NS):
        g = int(gos[s])
        if 0 <= g < NG:
            members[g].append(s)
        else:
            flags |= 1
    count = np.array([len(m) for m in members], dtype=np.int32)
    start = np.zeros(NG + 1, dtype=np.int32)
    start[1:] = np.cumsum(count)
    seqs = np.full(NS, -1, dtype=np.int32)
    for g in range(NG):
        seqs[start[g]:start[g + 1]] = members[g]

    def clamp(v, hi):
        nonlocal flags
        c = min(max(int(v), 0), hi)
        if c != int(v):
            flags |= 2
        return c

    sitems = []
    for s in range(NS):
        S = clamp(sl[s], mst)
        for t0 in range(0, S, Cs):
            sitems.append((s, t0, min(S, t0 + Cs), 0))
    pitems = []
    for g in range(NG):
        P = clamp(pl[g], mpt)
        rows = int(count[g]) * R
        for t0 in range(0, P, Cp):
            for r0 in range(0, rows, QB):
                pitems.append((g, t0, min(P, t0 + Cp), r0))
    chunks = np.zeros(NS, dtype=np.int32)
    for s in range(NS):
        g = int(gos[s])
        P = min(max(int(pl[g]), 0), mpt) if 0 <= g < NG else 0
        S = min(max(int(sl[s]), 0), mst)
        chunks[s] = _ceil_div(P, Cp) | (_ceil_div(S, Cs) << 16)
    return PlanRef(Cs, Cp, max(1, _ceil_div(mst, Cs)), max(1, _ceil_div(mpt, Cp)),
                   count, start, seqs, sitems, pitems, flags, chunks)


def cost_class(item, chunk: int) -> int:
    """Work items are listed by non-decreasing class: class 0 holds full chunks."""
    return (chunk - (item[2] - item[1])) // 32
