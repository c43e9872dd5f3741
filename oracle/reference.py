"""Python face of the reference checker (TEST INFRASTRUCTURE ONLY).

Loads the float64 C loops of `marl_oracle.c` and adds the few pieces that are easier to
state in numpy: the (max, sum, weighted-values) summary of a slice of tokens and the rule
that combines such summaries (the algebra any split-KV scheme relies on).  Only tests, the
smoke check and the CPU-baseline leg of the benchmark import this; it shares nothing with
the GPU library and never imports it.

Definitions are the textbook ones (the paper, Sections 4.1, 5.1 and 7, motivates the decode
step but prints no formula for it); see the header of `marl_oracle.c`.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "marl_oracle.c")
_LIB = os.path.join(_HERE, "libmarl_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C checker with gcc (no GPU toolchain involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        P = ctypes.c_void_p
        I = ctypes.c_int
        lib.oracle_decode_attn.restype = I
        lib.oracle_decode_attn.argtypes = [I, I, I, I, P, P, P, P, I, P, I, P, P, P,
                                           ctypes.c_double, P, I, I, I]
        lib.oracle_attn_weights.restype = I
        lib.oracle_attn_weights.argtypes = [I, I, I, I, P, P, P, P, I, P, I, P, P, P,
                                            ctypes.c_double, P, P]
        lib.oracle_token_logprobs.restype = I
        lib.oracle_token_logprobs.argtypes = [I, I, P, P, ctypes.c_double, P, I]
        _lib = lib
    return _lib


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def decode_attn(q, k_pages, v_pages, prefix_table, suffix_table, prefix_lens, suffix_lens,
                group_of_seq, scale: float, Hq: int, Hkv: int,
                seq_range: Optional[Tuple[int, int]] = None, threads: int = 0,
                return_threads: bool = False):
    """q, k_pages, v_pages: uint16 arrays of bf16 bit patterns in the ABI layout.
    Returns float64 [NS, Hq, 128] (rows outside `seq_range` stay zero)."""
    lib = _load()
    q, k_pages, v_pages = _u16(q), _u16(k_pages), _u16(v_pages)
    pt, st = _i32(prefix_table), _i32(suffix_table)
    pl, sl, gos = _i32(prefix_lens), _i32(suffix_lens), _i32(group_of_seq)
    NS, NG = sl.shape[0], pl.shape[0]
    pt = pt.reshape(NG, -1) if pt.size else pt.reshape(NG, 0)
    st = st.reshape(NS, -1) if st.size else st.reshape(NS, 0)
    out = np.zeros((NS, Hq, 128), dtype=np.float64)
    b, e = (0, NS) if seq_range is None else seq_range
    used = lib.oracle_decode_attn(NS, NG, Hq, Hkv, _ptr(q), _ptr(k_pages), _ptr(v_pages),
                                  _ptr(pt), pt.shape[1], _ptr(st), st.shape[1], _ptr(pl), _ptr(sl),
                                  _ptr(gos), float(scale), _ptr(out), b, e, threads)
    if used < 0:
        raise MemoryError("oracle_decode_attn")
    return (out, used) if return_threads else out


def attn_weights(s: int, h: int, q, k_pages, v_pages, prefix_table, suffix_table, prefix_lens,
                 suffix_lens, group_of_seq, scale: float, Hq: int, Hkv: int):
    """Softmax weights over the logical tokens of one (sequence, head), and its output row."""
    lib = _load()
    q, k_pages, v_pages = _u16(q), _u16(k_pages), _u16(v_pages)
    pt, st = _i32(prefix_table), _i32(suffix_table)
    pl, sl, gos = _i32(prefix_lens), _i32(suffix_lens), _i32(group_of_seq)
    NS, NG = sl.shape[0], pl.shape[0]
    pt, st = pt.reshape(NG, -1), st.reshape(NS, -1)
    L = int(pl[gos[s]]) + int(sl[s])
    w = np.zeros(max(L, 1), dtype=np.float64)
    out = np.zeros(128, dtype=np.float64)
    lib.oracle_attn_weights(s, h, Hq, Hkv, _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(pt),
                            pt.shape[1], _ptr(st), st.shape[1], _ptr(pl), _ptr(sl), _ptr(gos),
                            float(scale), _ptr(out), _ptr(w))
    return w[:L], out


def token_logprobs(logits, tokens, temperature: float, threads: int = 0,
                   return_threads: bool = False):
    """logits: uint16 bf16 bit patterns [rows, vocab].  Returns float64 [rows]."""
    lib = _load()
    logits = _u16(logits)
    rows, vocab = logits.shape
    tok = _i32(tokens)
    out = np.zeros(rows, dtype=np.float64)
    used = lib.oracle_token_logprobs(rows, vocab, _ptr(logits), _ptr(tok), float(temperature),
                                     _ptr(out), threads)
    return (out, used) if return_threads else out


# ------------------------------------------------------------------------------------------
# The summary of a slice of tokens and the rule that merges summaries.  For scores x_j and
# value rows v_j of a slice:  m = max_j x_j,  l = sum_j exp(x_j - m),  O = sum_j exp(x_j - m) v_j.
# Two slices combine as  m* = max(m1, m2),  l* = l1 e^{m1-m*} + l2 e^{m2-m*},
# O* = O1 e^{m1-m*} + O2 e^{m2-m*};  the attention output of the union is O*/l*.
# ------------------------------------------------------------------------------------------
def slice_summary(scores: np.ndarray, values: np.ndarray):
    """scores float64 [n], values float64 [n, d] -> (m, l, O[d]); an empty slice gives
    (-inf, 0, 0)."""
    if scores.shape[0] == 0:
        return -np.inf, 0.0, np.zeros(values.shape[1])
    m = float(scores.max())
    w = np.exp(scores - m)
    return m, float(w.sum()), w @ values


def merge_summaries(parts):
    """Combine [(m, l, O), ...] in list order; returns the normalised output O*/l* (zeros if
    every slice is empty)."""
    ms = [p[0] for p in parts]
    mstar = max(ms) if ms else -np.inf
    if not np.isfinite(mstar):
        d = parts[0][2].shape[0] if parts else 128
        return np.zeros(d)
    l = 0.0
    O = np.zeros_like(parts[0][2])
    for (m, li, Oi) in parts:
        if li == 0.0:
            continue
        f = np.exp(m - mstar)
        l += li * f
        O = O + Oi * f
    return O / l


def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns (uint16) to float64."""
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


# ------------------------------------------------------------------------------------------
# KV-cache maintenance of the decode loop, as plain scatter / copy on the ABI layouts
# (K [page][kv_head][slot][128], V [page][kv_head][128][slot]).  The paper says only that rollout
# manages large KV caches (Section 4.1); these are the definitions written in the library header.
# ------------------------------------------------------------------------------------------
def kv_append(k_pages, v_pages, suffix_table, suffix_lens, k_new, v_new):
    """Appends one token per sequence.  Arrays of bf16 bit patterns (uint16): k_pages
    [num_pages, Hkv, 16, 128], v_pages [num_pages, Hkv, 128, 16], k_new / v_new [NS, Hkv, 128].
    Returns (k_pages, v_pages, suffix_lens, flags) as new arrays; a sequence whose table row is
    full (flag 2) or whose page id is out of range (flag 4) is left untouched."""
    k_pages, v_pages = k_pages.copy(), v_pages.copy()
    lens = np.array(suffix_lens, dtype=np.int32).copy()
    table = np.asarray(suffix_table, dtype=np.int32)
    num_pages = k_pages.shape[0]
    flags = 0
    for s in range(lens.shape[0]):
        pos = int(lens[s])
        if pos < 0 or pos >= table.shape[1] * 16:
            flags |= 2
            continue
        page = int(table[s, pos // 16])
        if page < 0 or page >= num_pages:
            flags |= 4
            continue
        slot = pos % 16
        for kh in range(k_pages.shape[1]):
            for c in range(128):
                k_pages[page, kh, slot, c] = k_new[s, kh, c]
                v_pages[page, kh, c, slot] = v_new[s, kh, c]
        lens[s] = pos + 1
    return k_pages, v_pages, lens, flags


def kv_copy_pages(k_pages, v_pages, src, dst):
    """dst[i] <- src[i], whole pages of K and V; pairs with an id out of range are skipped
    (flag 4).  Returns (k_pages, v_pages, flags)."""
    k_pages, v_pages = k_pages.copy(), v_pages.copy()
    n = k_pages.shape[0]
    flags = 0
    for a, b in zip(np.asarray(src).tolist(), np.asarray(dst).tolist()):
        if not (0 <= a < n and 0 <= b < n):
            flags |= 4
            continue
        k_pages[b] = k_pages[a]
        v_pages[b] = v_pages[a]
    return k_pages, v_pages, flags


# ------------------------------------------------------------------------------------------
# Inverse-CDF sampling from softmax(logits / T) with a caller-supplied uniform number, and the
# drawn token's log-probability (textbook definitions; the paper trains with GRPO, Section 8.1,
# which consumes the log-probabilities of sampled tokens, and prints no formula).
# ------------------------------------------------------------------------------------------
def softmax_cdf(logit_bits_row: np.ndarray, temperature: float):
    """Probabilities and their running sum for one row of bf16 bit patterns, in float64."""
    y = bf16_bits_to_f64(logit_bits_row) / float(temperature)
    m = y.max()
    w = np.exp(y - m) if np.isfinite(m) else np.zeros_like(y)
    Z = w.sum()
    p = w / Z if Z > 0 else w
    return p, np.cumsum(p)


def sample_tokens(logit_bits: np.ndarray, uniforms, temperature: float):
    """token[r] = first t whose cumulative probability exceeds uniforms[r] (the last token
    with non-zero probability if none does), and log p of that token.  Rows without a finite
    logit give (-1, nan)."""
    rows = logit_bits.shape[0]
    tokens = np.full(rows, -1, dtype=np.int64)
    logprobs = np.full(rows, np.nan)
    for r in range(rows):
        p, cdf = softmax_cdf(logit_bits[r], temperature)
        if not (p > 0).any():
            continue
        hit = np.nonzero(cdf > float(uniforms[r]))[0]
        t = int(hit[0]) if hit.size else int(np.nonzero(p > 0)[0][-1])
        tokens[r] = t
        logprobs[r] = np.log(p[t])
    return tokens, logprobs


def nucleus(p: np.ndarray, top_p: float) -> np.ndarray:
    """Boolean mask of the top-p nucleus: tokens ranked by probability (ties: lower index first),
    the shortest head of the ranking whose mass is >= top_p; tokens of zero probability are never
    in it.  If rounding keeps the total below top_p, every token of non-zero probability."""
    order = np.argsort(-p, kind="stable")            # stable: equal p keep index order
    csum = np.cumsum(p[order])
    hit = np.nonzero(csum >= top_p)[0]
    k = int(hit[0]) + 1 if hit.size else len(p)
    mask = np.zeros(len(p), dtype=bool)
    mask[order[:k]] = True
    return mask & (p > 0)


def sample_tokens_top_p(logit_bits: np.ndarray, uniforms, temperature: float, top_p: float):
    """Inverse-CDF draw inside the nucleus, in index order, with the uniform number scaled to the
    nucleus mass; log p of the drawn token under the untruncated distribution."""
    rows = logit_bits.shape[0]
    tokens = np.full(rows, -1, dtype=np.int64)
    logprobs = np.full(rows, np.nan)
    for r in range(rows):
        p, _ = softmax_cdf(logit_bits[r], temperature)
        if not np.isfinite(p).all() or not (p > 0).any():
            continue
        keep = nucleus(p, top_p)
        q = np.where(keep, p, 0.0)
        cdf = np.cumsum(q)
        hit = np.nonzero(cdf > float(uniforms[r]) * q.sum())[0]
        t = int(hit[0]) if hit.size else int(np.nonzero(keep)[0][-1])
        tokens[r] = t
        logprobs[r] = np.log(p[t])
    return tokens, logprobs


# ------------------------------------------------------------------------------------------
# GRPO's group-normalised advantage (Shao et al. 2024, the algorithm the paper trains with,
# Section 8.1): reward minus the group mean, over the group's standard deviation (the root of
# the mean squared deviation) plus eps.
# ------------------------------------------------------------------------------------------
def grpo_advantages(rewards, group_of_seq, num_groups: int, eps: float):
    """rewards [NS], group_of_seq [NS] (ids outside [0, num_groups) belong to no group and
    give nan) -> float64 [NS]."""
    r = np.asarray(rewards, dtype=np.float64)
    g = np.asarray(group_of_seq)
    out = np.full(r.shape, np.nan)
    for k in range(num_groups):
        idx = np.nonzero(g == k)[0]
        if idx.size == 0:
            continue
        dev = r[idx] - r[idx].mean()
        std = np.sqrt((dev * dev).mean())
        for i, d in zip(idx, dev):
            out[i] = 0.0 if d == 0.0 else d / (std + eps)
    return out


# ------------------------------------------------------------------------------------------
# Prompt (prefill) attention: textbook causal attention over the logical positions of a
# group's pages, and the scatter of a prompt chunk into the pages (the step that creates the
# prefix all samples of a prompt share, Section 5.1 of the paper, which prints no formula).
# ------------------------------------------------------------------------------------------
def gather_group_kv(k_pages, v_pages, table_row, length: int):
    """Logical K and V of one block-table row as float64 [length, Hkv, 128]."""
    Hkv = k_pages.shape[1]
    K = np.zeros((length, Hkv, 128))
    V = np.zeros((length, Hkv, 128))
    for t in range(length):
        page, slot = int(table_row[t // 16]), t % 16
        K[t] = bf16_bits_to_f64(k_pages[page, :, slot, :])
        V[t] = bf16_bits_to_f64(v_pages[page, :, :, slot])
    return K, V


def prefill_attn(q, k_pages, v_pages, prefix_table, q_start, q_pos0, scale: float, Hq: int, Hkv: int):
    """q uint16 [NT, Hq, 128] (bf16 bits); returns float64 [NT, Hq, 128].  Query token tau of group g
    sits at position q_pos0[g] + tau and attends to positions 0 .. its own (inclusive).  Rows no
    group covers are nan."""
    q, k_pages, v_pages = _u16(q), _u16(k_pages), _u16(v_pages)
    NT = q.shape[0]
    R = Hq // Hkv
    out = np.full((NT, Hq, 128), np.nan)
    qs = np.asarray(q_start, dtype=np.int64)
    for g in range(len(q_pos0)):
        b, e, p0 = int(qs[g]), int(qs[g + 1]), int(q_pos0[g])
        n = e - b
        if n <= 0:
            continue
        L = p0 + n
        K, V = gather_group_kv(k_pages, v_pages, np.asarray(prefix_table)[g], L)
        Q = bf16_bits_to_f64(q[b:e])                          # [n, Hq, 128]
        visible = np.arange(L)[None, :] <= (p0 + np.arange(n))[:, None]
        for h in range(Hq):
            x = float(scale) * (Q[:, h, :] @ K[:, h // R, :].T)     # [n, L]
            x = np.where(visible, x, -np.inf)
            w = np.exp(x - x.max(axis=1, keepdims=True))
            out[b:e, h, :] = (w / w.sum(axis=1, keepdims=True)) @ V[:, h // R, :]
    return out


def kv_write_prompt(k_pages, v_pages, prefix_table, q_start, q_pos0, k_new, v_new):
    """Token q_start[g] + tau goes to position q_pos0[g] + tau of group g.  Returns new arrays."""
    k_pages, v_pages = k_pages.copy(), v_pages.copy()
    table = np.asarray(prefix_table)
    for g in range(len(q_pos0)):
        for tau in range(int(q_start[g + 1]) - int(q_start[g])):
            pos = int(q_pos0[g]) + tau
            page, slot = int(table[g, pos // 16]), pos % 16
            tok = int(q_start[g]) + tau
            k_pages[page, :, slot, :] = k_new[tok]
            v_pages[page, :, :, slot] = v_new[tok]
    return k_pages, v_pages


# ------------------------------------------------------------------------------------------
# Weight synchronisation as one copy (the paper's Discussion, "Hardware-Aware Abstraction": the
# weights are aggregated into a single contiguous buffer).  The definition written out: the
# tensors' bytes one after the other in table order, every start rounded up to 256 bytes.
# ------------------------------------------------------------------------------------------
PACK_ALIGN = 256
PACK_CHUNK = 262144


def pack_layout(sizes):
    """(offsets, first_chunk, packed_bytes, total_chunks) for tensors of the given byte sizes."""
    offsets, first_chunk = [], []
    off = chunks = 0
    for n in sizes:
        off = -(-off // PACK_ALIGN) * PACK_ALIGN
        offsets.append(off)
        first_chunk.append(chunks)
        off += int(n)
        chunks += -(-int(n) // PACK_CHUNK)
    return offsets, first_chunk, off, chunks


def pack_tensors(arrays, fill: int = 0):
    """uint8 buffer holding every array's bytes at its offset; the gaps hold `fill`."""
    raw = [np.ascontiguousarray(a).view(np.uint8).reshape(-1) for a in arrays]
    offsets, _, total, _ = pack_layout([r.size for r in raw])
    out = np.full(total, fill, dtype=np.uint8)
    for r, o in zip(raw, offsets):
        out[o:o + r.size] = r
    return out, offsets
