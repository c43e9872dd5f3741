"""Thin ctypes binding of libmarl_decode.so (include/marl_decode.h): argument marshalling
only.  PyTorch supplies device memory and the stream; every step runs in the library's
kernels.  There is no fallback: if the library is missing or a call fails, this raises."""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import numpy as np
import torch

from .build import LIB_PATH, build_library

I32 = ctypes.c_int32
SZ = ctypes.c_size_t
VP = ctypes.c_void_p

MARL_OUT_BF16, MARL_OUT_F32 = 0, 1
STAGES = ("plan", "prefix", "suffix", "merge", "logprob", "logprob_finish")
CTR_NUM_SUFFIX_ITEMS, CTR_NUM_PREFIX_ITEMS, CTR_SUFFIX_CURSOR, CTR_PREFIX_CURSOR, CTR_FLAGS, \
    CTR_NUM_LONG_SUFFIX_ITEMS, CTR_SHORT_CURSOR, CTR_NUM_SHORT_PARTIAL_ITEMS = range(8)
FLAG_BAD_GROUP, FLAG_LEN_CLAMPED, FLAG_BAD_PAGE = 1, 2, 4


class AttnShape(ctypes.Structure):
    _fields_ = [(n, I32) for n in (
        "num_seqs", "num_groups", "num_q_heads", "num_kv_heads", "head_dim", "page_size",
        "num_pages", "max_prefix_pages", "max_suffix_pages", "out_dtype",
        "suffix_chunk_tokens", "prefix_chunk_tokens")]


class PlanLayout(ctypes.Structure):
    _fields_ = [(n, I32) for n in (
        "suffix_chunk_tokens", "prefix_chunk_tokens", "suffix_slots", "prefix_slots",
        "rows_per_qblock", "max_suffix_items", "max_prefix_items", "reserved")] + \
        [(n, SZ) for n in (
            "counters_off", "group_count_off", "group_start_off", "seq_rank_off", "group_tmp_off", "group_seqs_off",
            "seq_chunks_off",
            "suffix_items_off", "prefix_items_off", "partial_ml_off", "partial_o_off", "total_bytes")]


class PrefillShape(ctypes.Structure):
    _fields_ = [(n, I32) for n in (
        "num_tokens", "num_groups", "num_q_heads", "num_kv_heads", "head_dim", "page_size",
        "num_pages", "max_prefix_pages", "out_dtype", "reserved")]


class BalancerConfig(ctypes.Structure):
    _fields_ = [(n, I32) for n in ("num_agents", "delta", "slots_per_instance", "poll_interval", "migration_delay")]


class BalancerStats(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("now", "submitted", "completed", "migrations")]


class PackEntry(ctypes.Structure):
    _fields_ = [("ptr", ctypes.c_void_p), ("offset", ctypes.c_uint64), ("bytes", ctypes.c_uint64),
                ("first_chunk", ctypes.c_uint64)]


class MarlError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


_lib = None


def load_library(build_if_missing: bool = True):
    """Loads the in-tree shared library; builds it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    path = os.environ.get("MARL_DECODE_LIB", LIB_PATH)   # an explicitly chosen build, if any
    if not os.path.exists(path):
        if not build_if_missing or path != LIB_PATH:
            raise FileNotFoundError(path)
        build_library()
    lib = ctypes.CDLL(path)
    PS, PL = ctypes.POINTER(AttnShape), ctypes.POINTER(PlanLayout)
    lib.marl_version.restype = ctypes.c_int
    lib.marl_status_string.restype = ctypes.c_char_p
    lib.marl_status_string.argtypes = [ctypes.c_int]
    lib.marl_last_hip_error.restype = ctypes.c_char_p
    lib.marl_attn_plan_layout_for.argtypes = [PS, PL]
    lib.marl_workspace_bytes.argtypes = [PS, ctypes.POINTER(SZ)]
    lib.marl_decode_attn.argtypes = [PS, VP, SZ, VP, VP, VP, VP, VP, VP, VP, VP, ctypes.c_float, VP, VP]
    lib.marl_decode_attn_static.argtypes = [PS, VP, VP, VP, VP, VP, VP, VP, VP, ctypes.c_float, VP, VP, VP]
    lib.marl_attn_plan.argtypes = [PS, VP, SZ, VP, VP, VP, VP]
    lib.marl_attn_read_flags.argtypes = [VP, ctypes.POINTER(I32), VP]
    lib.marl_logprobs_workspace_bytes.argtypes = [I32, I32, ctypes.POINTER(SZ)]
    lib.marl_token_logprobs.argtypes = [VP, VP, ctypes.c_float, VP, I32, I32, VP, SZ, VP]
    lib.marl_kv_append.argtypes = [PS, VP, VP, VP, VP, VP, VP, VP, VP]
    lib.marl_kv_copy_pages.argtypes = [PS, VP, VP, VP, VP, I32, VP, VP]
    lib.marl_kv_append.restype = lib.marl_kv_copy_pages.restype = ctypes.c_int
    lib.marl_sample_workspace_bytes.argtypes = [I32, I32, ctypes.POINTER(SZ)]
    lib.marl_sample_tokens.argtypes = [VP, VP, ctypes.c_float, VP, VP, I32, I32, VP, SZ, VP]
    lib.marl_sample_workspace_bytes.restype = lib.marl_sample_tokens.restype = ctypes.c_int
    lib.marl_sample_tokens_top_p.argtypes = [VP, VP, ctypes.c_float, ctypes.c_float, VP, VP, I32, I32, VP]
    lib.marl_sample_tokens_top_p.restype = ctypes.c_int
    lib.marl_grpo_advantages.argtypes = [VP, VP, VP, I32, ctypes.c_float, VP, VP]
    I64P, I32P = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(I32)
    lib.marl_balancer_create.argtypes = [ctypes.POINTER(BalancerConfig), I32P, ctypes.POINTER(VP)]
    lib.marl_balancer_destroy.argtypes = [VP]
    lib.marl_balancer_destroy.restype = None
    lib.marl_balancer_submit.argtypes = [VP, I32, I32, I32, I32P]
    lib.marl_balancer_step.argtypes = [VP, ctypes.POINTER(BalancerStats)]
    lib.marl_balancer_agent_state.argtypes = [VP, I32, I32P, I64P, I64P]
    lib.marl_balancer_instance_batch.argtypes = [VP, I32, I32P, I32P, I32P, I32, I32P]
    lib.marl_balancer_request_state.argtypes = [VP, I32, I32P, I32P, I64P]
    PP = ctypes.POINTER(PrefillShape)
    lib.marl_prefill_workspace_bytes.argtypes = [PP, ctypes.POINTER(SZ)]
    lib.marl_prefill_attn.argtypes = [PP, VP, SZ, VP, VP, VP, VP, VP, VP, ctypes.c_float, VP, VP]
    lib.marl_kv_write_prompt.argtypes = [PP, VP, VP, VP, VP, VP, VP, VP, VP, VP]
    lib.marl_prefill_workspace_bytes.restype = lib.marl_prefill_attn.restype = ctypes.c_int
    lib.marl_kv_write_prompt.restype = ctypes.c_int
    lib.marl_grpo_advantages.restype = ctypes.c_int
    lib.marl_page_pool_create.argtypes = [I32, ctypes.POINTER(VP)]
    lib.marl_page_pool_destroy.argtypes = [VP]
    lib.marl_page_pool_destroy.restype = None
    lib.marl_page_pool_alloc.argtypes = [VP, I32, I32P]
    lib.marl_page_pool_retain.argtypes = [VP, I32P, I32]
    lib.marl_page_pool_release.argtypes = [VP, I32P, I32]
    lib.marl_page_pool_fork.argtypes = [VP, I32P, I32, I32P]
    lib.marl_page_pool_prepare_append.argtypes = [VP, I32P, I32, I32, I32P, I32P]
    lib.marl_page_pool_drop.argtypes = [VP, I32P, I32]
    lib.marl_page_pool_query.argtypes = [VP, I32, I32P, I32P]
    PE = ctypes.POINTER(PackEntry)
    lib.marl_pack_plan.argtypes = [PE, I32, ctypes.POINTER(ctypes.c_uint64), I64P]
    lib.marl_pack_tensors.argtypes = [VP, I32, ctypes.c_int64, VP, VP]
    lib.marl_unpack_tensors.argtypes = [VP, I32, ctypes.c_int64, VP, VP]
    lib.marl_pack_plan.restype = lib.marl_pack_tensors.restype = lib.marl_unpack_tensors.restype = ctypes.c_int
    lib.marl_profile_begin.argtypes = [I32]
    lib.marl_profile_end.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(I32), ctypes.POINTER(I32)]
    for f in ("marl_attn_plan_layout_for", "marl_workspace_bytes", "marl_decode_attn", "marl_decode_attn_static",
              "marl_attn_plan",
              "marl_attn_read_flags", "marl_logprobs_workspace_bytes", "marl_token_logprobs",
              "marl_profile_begin", "marl_profile_end"):
        getattr(lib, f).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc: int, where: str):
    if rc != 0:
        lib = load_library()
        detail = lib.marl_status_string(rc).decode()
        if rc == -4:
            detail += ": " + lib.marl_last_hip_error().decode()
        raise MarlError(rc, where, detail)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(device) -> ctypes.c_void_p:
    return ctypes.c_void_p(torch.cuda.current_stream(device).cuda_stream)


def make_shape(num_seqs, num_groups, num_q_heads, num_kv_heads, num_pages, max_prefix_pages,
               max_suffix_pages, out_dtype=MARL_OUT_BF16, suffix_chunk_tokens=0, prefix_chunk_tokens=0,
               head_dim=128, page_size=16) -> AttnShape:
    return AttnShape(num_seqs, num_groups, num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
                     max_prefix_pages, max_suffix_pages, out_dtype, suffix_chunk_tokens, prefix_chunk_tokens)


def marl_attn_plan_layout_for(shape: AttnShape) -> PlanLayout:
    L = PlanLayout()
    _check(load_library().marl_attn_plan_layout_for(ctypes.byref(shape), ctypes.byref(L)), "marl_attn_plan_layout_for")
    return L


def marl_workspace_bytes(shape: AttnShape) -> int:
    n = SZ(0)
    _check(load_library().marl_workspace_bytes(ctypes.byref(shape), ctypes.byref(n)), "marl_workspace_bytes")
    return int(n.value)


def alloc_workspace(nbytes: int, device) -> torch.Tensor:
    """Device bytes, 256-byte aligned (torch's allocator aligns to 512)."""
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def _require_cuda(*tensors):
    for t in tensors:
        if t is not None and not t.is_cuda:
            raise ValueError("device tensors required: the library has no CPU path")
        if t is not None and not t.is_contiguous():
            raise ValueError("contiguous tensors required")


def _require(t: Optional[torch.Tensor], name: str, dtype, shape=None):
    """The kernels reinterpret raw bytes, so a wrong dtype (torch's default int64 for an index tensor,
    float32 for bf16 data) or a wrong extent would give wrong results without any error: refuse it here.
    `shape`: expected sizes, None entries are free."""
    if t is None:
        return
    if t.dtype != dtype:
        raise ValueError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if shape is not None:
        if t.dim() != len(shape) or any(e is not None and int(g) != int(e) for g, e in zip(t.shape, shape)):
            raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


def _require_attn_operands(shape: AttnShape, q, k_pages, v_pages, prefix_block_table, suffix_block_table,
                           prefix_lens, suffix_lens, group_of_seq, out):
    NS, NG, Hq, Hkv = shape.num_seqs, shape.num_groups, shape.num_q_heads, shape.num_kv_heads
    bf, i32 = torch.bfloat16, torch.int32
    _require(q, "q", bf, (NS, Hq, 128))
    _require(k_pages, "k_pages", bf, (shape.num_pages, Hkv, 16, 128))
    _require(v_pages, "v_pages", bf, (shape.num_pages, Hkv, 128, 16))
    if shape.max_prefix_pages > 0:
        _require(prefix_block_table, "prefix_block_table", i32, (NG, shape.max_prefix_pages))
    if shape.max_suffix_pages > 0:
        _require(suffix_block_table, "suffix_block_table", i32, (NS, shape.max_suffix_pages))
    _require(prefix_lens, "prefix_lens", i32, (NG,))
    _require(suffix_lens, "suffix_lens", i32, (NS,))
    _require(group_of_seq, "group_of_seq", i32, (NS,))
    _require(out, "out", bf if shape.out_dtype == MARL_OUT_BF16 else torch.float32, (NS, Hq, 128))


def marl_decode_attn(shape: AttnShape, workspace: torch.Tensor, q, k_pages, v_pages, prefix_block_table,
                     suffix_block_table, prefix_lens, suffix_lens, group_of_seq, scale: float,
                     out: torch.Tensor) -> torch.Tensor:
    _require_attn_operands(shape, q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens,
                           suffix_lens, group_of_seq, out)
    _require_cuda(workspace, q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens,
                  suffix_lens, group_of_seq, out)
    rc = load_library().marl_decode_attn(
        ctypes.byref(shape), _ptr(workspace), workspace.numel(), _ptr(q), _ptr(k_pages), _ptr(v_pages),
        _ptr(prefix_block_table), _ptr(suffix_block_table), _ptr(prefix_lens), _ptr(suffix_lens),
        _ptr(group_of_seq), float(scale), _ptr(out), _stream(out.device))
    _check(rc, "marl_decode_attn")
    return out


STATIC_WORKSPACE_BYTES = 64 << 20   # MARL_STATIC_WORKSPACE_BYTES of the header


def marl_decode_attn_static(shape: AttnShape, q, k_pages, v_pages, prefix_block_table, suffix_block_table,
                            prefix_lens, suffix_lens, group_of_seq, scale: float, out: torch.Tensor,
                            flags: Optional[torch.Tensor] = None) -> torch.Tensor:
    """marl_decode_attn on the library's own fixed workspace (no allocation in the call)."""
    _require_cuda(q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens, suffix_lens,
                  group_of_seq, out, flags)
    _require_attn_operands(shape, q, k_pages, v_pages, prefix_block_table, suffix_block_table, prefix_lens,
                           suffix_lens, group_of_seq, out)
    _require(flags, "flags", torch.int32)
    rc = load_library().marl_decode_attn_static(
        ctypes.byref(shape), _ptr(q), _ptr(k_pages), _ptr(v_pages), _ptr(prefix_block_table),
        _ptr(suffix_block_table), _ptr(prefix_lens), _ptr(suffix_lens), _ptr(group_of_seq), float(scale),
        _ptr(out), _ptr(flags), _stream(out.device))
    _check(rc, "marl_decode_attn_static")
    return out


def marl_attn_plan(shape: AttnShape, workspace: torch.Tensor, prefix_lens, suffix_lens, group_of_seq):
    _require_cuda(workspace, prefix_lens, suffix_lens, group_of_seq)
    _require(prefix_lens, "prefix_lens", torch.int32, (shape.num_groups,))
    _require(suffix_lens, "suffix_lens", torch.int32, (shape.num_seqs,))
    _require(group_of_seq, "group_of_seq", torch.int32, (shape.num_seqs,))
    rc = load_library().marl_attn_plan(ctypes.byref(shape), _ptr(workspace), workspace.numel(),
                                       _ptr(prefix_lens), _ptr(suffix_lens), _ptr(group_of_seq),
                                       _stream(workspace.device))
    _check(rc, "marl_attn_plan")


def marl_attn_read_flags(workspace: torch.Tensor) -> int:
    _require_cuda(workspace)
    f = I32(0)
    _check(load_library().marl_attn_read_flags(_ptr(workspace), ctypes.byref(f), _stream(workspace.device)),
           "marl_attn_read_flags")
    return int(f.value)


def marl_logprobs_workspace_bytes(rows: int, vocab: int) -> int:
    n = SZ(0)
    _check(load_library().marl_logprobs_workspace_bytes(rows, vocab, ctypes.byref(n)), "marl_logprobs_workspace_bytes")
    return int(n.value)


def marl_token_logprobs(logits: torch.Tensor, tokens: torch.Tensor, temperature: float, out: torch.Tensor,
                        workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    _require(logits, "logits", torch.bfloat16, (None, None))
    rows, vocab = logits.shape
    _require(tokens, "tokens", torch.int32, (rows,))
    _require(out, "out", torch.float32, (rows,))
    _require_cuda(logits, tokens, out, workspace)
    rc = load_library().marl_token_logprobs(
        _ptr(logits), _ptr(tokens), float(temperature), _ptr(out), rows, vocab, _ptr(workspace),
        0 if workspace is None else workspace.numel(), _stream(logits.device))
    _check(rc, "marl_token_logprobs")
    return out


def marl_kv_append(shape: AttnShape, k_new, v_new, k_pages, v_pages, suffix_block_table, suffix_lens,
                   flags: Optional[torch.Tensor] = None):
    _require_cuda(k_new, v_new, k_pages, v_pages, suffix_block_table, suffix_lens, flags)
    NS, Hkv = shape.num_seqs, shape.num_kv_heads
    _require(k_new, "k_new", torch.bfloat16, (NS, Hkv, 128))
    _require(v_new, "v_new", torch.bfloat16, (NS, Hkv, 128))
    _require(k_pages, "k_pages", torch.bfloat16, (shape.num_pages, Hkv, 16, 128))
    _require(v_pages, "v_pages", torch.bfloat16, (shape.num_pages, Hkv, 128, 16))
    _require(suffix_block_table, "suffix_block_table", torch.int32, (NS, shape.max_suffix_pages))
    _require(suffix_lens, "suffix_lens", torch.int32, (NS,))
    _require(flags, "flags", torch.int32)
    rc = load_library().marl_kv_append(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(k_pages), _ptr(v_pages),
                                       _ptr(suffix_block_table), _ptr(suffix_lens), _ptr(flags),
                                       _stream(k_pages.device))
    _check(rc, "marl_kv_append")


def marl_kv_copy_pages(shape: AttnShape, k_pages, v_pages, src, dst, flags: Optional[torch.Tensor] = None):
    _require_cuda(k_pages, v_pages, src, dst, flags)
    _require(k_pages, "k_pages", torch.bfloat16, (shape.num_pages, shape.num_kv_heads, 16, 128))
    _require(v_pages, "v_pages", torch.bfloat16, (shape.num_pages, shape.num_kv_heads, 128, 16))
    _require(src, "src", torch.int32, (None,))
    _require(dst, "dst", torch.int32, (int(src.numel()),))
    _require(flags, "flags", torch.int32)
    rc = load_library().marl_kv_copy_pages(ctypes.byref(shape), _ptr(k_pages), _ptr(v_pages), _ptr(src), _ptr(dst),
                                           int(src.numel()), _ptr(flags), _stream(k_pages.device))
    _check(rc, "marl_kv_copy_pages")


def marl_sample_workspace_bytes(rows: int, vocab: int) -> int:
    n = SZ(0)
    _check(load_library().marl_sample_workspace_bytes(rows, vocab, ctypes.byref(n)), "marl_sample_workspace_bytes")
    return int(n.value)


def marl_sample_tokens(logits: torch.Tensor, uniforms: torch.Tensor, temperature: float, out_tokens: torch.Tensor,
                       out_logprobs: torch.Tensor, workspace: torch.Tensor):
    _require_cuda(logits, uniforms, out_tokens, out_logprobs, workspace)
    _require(logits, "logits", torch.bfloat16, (None, None))
    rows, vocab = logits.shape
    _require(uniforms, "uniforms", torch.float32, (rows,))
    _require(out_tokens, "out_tokens", torch.int32, (rows,))
    _require(out_logprobs, "out_logprobs", torch.float32, (rows,))
    rc = load_library().marl_sample_tokens(_ptr(logits), _ptr(uniforms), float(temperature), _ptr(out_tokens),
                                           _ptr(out_logprobs), rows, vocab, _ptr(workspace), workspace.numel(),
                                           _stream(logits.device))
    _check(rc, "marl_sample_tokens")
    return out_tokens, out_logprobs


def marl_sample_tokens_top_p(logits: torch.Tensor, uniforms: torch.Tensor, temperature: float, top_p: float,
                             out_tokens: torch.Tensor, out_logprobs: torch.Tensor):
    _require_cuda(logits, uniforms, out_tokens, out_logprobs)
    _require(logits, "logits", torch.bfloat16, (None, None))
    rows, vocab = logits.shape
    _require(uniforms, "uniforms", torch.float32, (rows,))
    _require(out_tokens, "out_tokens", torch.int32, (rows,))
    _require(out_logprobs, "out_logprobs", torch.float32, (rows,))
    rc = load_library().marl_sample_tokens_top_p(_ptr(logits), _ptr(uniforms), float(temperature), float(top_p),
                                                 _ptr(out_tokens), _ptr(out_logprobs), rows, vocab,
                                                 _stream(logits.device))
    _check(rc, "marl_sample_tokens_top_p")
    return out_tokens, out_logprobs


def marl_grpo_advantages(rewards: torch.Tensor, group_start: torch.Tensor, group_seqs: torch.Tensor, eps: float,
                         out: torch.Tensor):
    _require_cuda(rewards, group_start, group_seqs, out)
    _require(rewards, "rewards", torch.float32, (None,))
    _require(group_start, "group_start", torch.int32, (None,))
    _require(group_seqs, "group_seqs", torch.int32, (None,))
    _require(out, "out", torch.float32, (int(rewards.numel()),))
    rc = load_library().marl_grpo_advantages(_ptr(rewards), _ptr(group_start), _ptr(group_seqs),
                                             int(group_start.numel()) - 1, float(eps), _ptr(out),
                                             _stream(rewards.device))
    _check(rc, "marl_grpo_advantages")
    return out


def make_prefill_shape(num_tokens, num_groups, num_q_heads, num_kv_heads, num_pages, max_prefix_pages,
                       out_dtype=MARL_OUT_BF16, head_dim=128, page_size=16) -> PrefillShape:
    return PrefillShape(num_tokens, num_groups, num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
                        max_prefix_pages, out_dtype, 0)


def marl_prefill_workspace_bytes(shape: PrefillShape) -> int:
    n = SZ(0)
    _check(load_library().marl_prefill_workspace_bytes(ctypes.byref(shape), ctypes.byref(n)),
           "marl_prefill_workspace_bytes")
    return int(n.value)


def marl_prefill_attn(shape: PrefillShape, workspace, q, k_pages, v_pages, prefix_block_table, q_start, q_pos0,
                      scale: float, out):
    _require_cuda(workspace, q, k_pages, v_pages, prefix_block_table, q_start, q_pos0, out)
    NT, NG, Hq, Hkv = shape.num_tokens, shape.num_groups, shape.num_q_heads, shape.num_kv_heads
    _require(q, "q", torch.bfloat16, (NT, Hq, 128))
    _require(k_pages, "k_pages", torch.bfloat16, (shape.num_pages, Hkv, 16, 128))
    _require(v_pages, "v_pages", torch.bfloat16, (shape.num_pages, Hkv, 128, 16))
    _require(prefix_block_table, "prefix_block_table", torch.int32, (NG, shape.max_prefix_pages))
    _require(q_start, "q_start", torch.int32, (NG + 1,))
    _require(q_pos0, "q_pos0", torch.int32, (NG,))
    _require(out, "out", torch.bfloat16 if shape.out_dtype == MARL_OUT_BF16 else torch.float32, (NT, Hq, 128))
    rc = load_library().marl_prefill_attn(ctypes.byref(shape), _ptr(workspace), workspace.numel(), _ptr(q),
                                          _ptr(k_pages), _ptr(v_pages), _ptr(prefix_block_table), _ptr(q_start),
                                          _ptr(q_pos0), float(scale), _ptr(out), _stream(q.device))
    _check(rc, "marl_prefill_attn")
    return out


def marl_kv_write_prompt(shape: PrefillShape, k_new, v_new, k_pages, v_pages, prefix_block_table, q_start, q_pos0,
                         flags=None):
    _require_cuda(k_new, v_new, k_pages, v_pages, prefix_block_table, q_start, q_pos0, flags)
    NT, NG, Hkv = shape.num_tokens, shape.num_groups, shape.num_kv_heads
    _require(k_new, "k_new", torch.bfloat16, (NT, Hkv, 128))
    _require(v_new, "v_new", torch.bfloat16, (NT, Hkv, 128))
    _require(k_pages, "k_pages", torch.bfloat16, (shape.num_pages, Hkv, 16, 128))
    _require(v_pages, "v_pages", torch.bfloat16, (shape.num_pages, Hkv, 128, 16))
    _require(prefix_block_table, "prefix_block_table", torch.int32, (NG, shape.max_prefix_pages))
    _require(q_start, "q_start", torch.int32, (NG + 1,))
    _require(q_pos0, "q_pos0", torch.int32, (NG,))
    _require(flags, "flags", torch.int32)
    rc = load_library().marl_kv_write_prompt(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(k_pages),
                                             _ptr(v_pages), _ptr(prefix_block_table), _ptr(q_start), _ptr(q_pos0),
                                             _ptr(flags) if flags is not None else None, _stream(k_new.device))
    _check(rc, "marl_kv_write_prompt")


def prepare_prefill(inp, out_dtype=MARL_OUT_BF16):
    """(shape, workspace, out) for an inputs.PrefillInputs resident on a GPU."""
    shape = make_prefill_shape(inp.num_tokens, inp.num_groups, inp.Hq, inp.Hkv, inp.num_pages,
                               int(inp.prefix_block_table.shape[1]), out_dtype)
    ws = alloc_workspace(marl_prefill_workspace_bytes(shape), inp.q.device)
    out = torch.empty((inp.num_tokens, inp.Hq, 128), device=inp.q.device,
                      dtype=torch.bfloat16 if out_dtype == MARL_OUT_BF16 else torch.float32)
    return shape, ws, out


def run_prefill(inp, shape, ws, out):
    return marl_prefill_attn(shape, ws, inp.q, inp.k_pages, inp.v_pages, inp.prefix_block_table, inp.q_start,
                             inp.q_pos0, inp.scale, out)


class Balancer:
    """Handle of the host-side load-balancing simulation (marl_balancer_* in the header)."""

    def __init__(self, instances_per_agent, delta=5, slots_per_instance=1, poll_interval=1, migration_delay=0):
        self._lib = load_library()
        cfg = BalancerConfig(len(instances_per_agent), delta, slots_per_instance, poll_interval, migration_delay)
        arr = (I32 * len(instances_per_agent))(*instances_per_agent)
        h = VP()
        _check(self._lib.marl_balancer_create(ctypes.byref(cfg), arr, ctypes.byref(h)), "marl_balancer_create")
        self._h = h
        self.num_instances = int(sum(instances_per_agent))
        self.slots = slots_per_instance

    def close(self):
        if self._h:
            self._lib.marl_balancer_destroy(self._h)
            self._h = None

    __del__ = close

    def submit(self, agent: int, request_id: int, gen_len: int) -> int:
        inst = I32(-1)
        _check(self._lib.marl_balancer_submit(self._h, agent, request_id, gen_len, ctypes.byref(inst)),
               "marl_balancer_submit")
        return int(inst.value)

    def step(self) -> BalancerStats:
        st = BalancerStats()
        _check(self._lib.marl_balancer_step(self._h, ctypes.byref(st)), "marl_balancer_step")
        return st

    def agent_state(self, agent: int):
        n, w, a = I32(0), ctypes.c_int64(0), ctypes.c_int64(0)
        _check(self._lib.marl_balancer_agent_state(self._h, agent, ctypes.byref(n), ctypes.byref(w), ctypes.byref(a)),
               "marl_balancer_agent_state")
        return int(n.value), int(w.value), int(a.value)

    def instance_batch(self, instance: int):
        ids, gen = (I32 * self.slots)(), (I32 * self.slots)()
        owner, n = I32(0), I32(0)
        _check(self._lib.marl_balancer_instance_batch(self._h, instance, ctypes.byref(owner), ids, gen, self.slots,
                                                      ctypes.byref(n)), "marl_balancer_instance_batch")
        return int(owner.value), list(ids[:n.value]), list(gen[:n.value])

    def request_state(self, request_id: int):
        inst, gen, done = I32(0), I32(0), ctypes.c_int64(0)
        _check(self._lib.marl_balancer_request_state(self._h, request_id, ctypes.byref(inst), ctypes.byref(gen),
                                                     ctypes.byref(done)), "marl_balancer_request_state")
        return int(inst.value), int(gen.value), int(done.value)


class PagePool:
    """Host-side page bookkeeping (marl_page_pool_*).  Rows are numpy int32 arrays owned by the caller;
    methods return the library's status code (0 = ok) so that error paths can be tested."""

    def __init__(self, num_pages: int):
        self._lib = load_library()
        self._h = VP()
        _check(self._lib.marl_page_pool_create(num_pages, ctypes.byref(self._h)), "marl_page_pool_create")

    def __del__(self):
        if getattr(self, "_h", None):
            self._lib.marl_page_pool_destroy(self._h)
            self._h = None

    @staticmethod
    def _p(a: np.ndarray):
        assert a.dtype == np.int32 and a.flags.c_contiguous
        return a.ctypes.data_as(ctypes.POINTER(I32))

    def alloc(self, n: int):
        out = np.empty(max(n, 1), dtype=np.int32)
        rc = self._lib.marl_page_pool_alloc(self._h, n, self._p(out))
        return rc, (out[:n] if rc == 0 else None)

    def retain(self, pages) -> int:
        a = np.ascontiguousarray(pages, dtype=np.int32)
        return self._lib.marl_page_pool_retain(self._h, self._p(a), len(a))

    def release(self, pages) -> int:
        a = np.ascontiguousarray(pages, dtype=np.int32)
        return self._lib.marl_page_pool_release(self._h, self._p(a), len(a))

    def fork(self, parent_row: np.ndarray, length: int, child_row: np.ndarray) -> int:
        return self._lib.marl_page_pool_fork(self._h, self._p(parent_row), length, self._p(child_row))

    def prepare_append(self, row: np.ndarray, length: int):
        src, dst = I32(-1), I32(-1)
        rc = self._lib.marl_page_pool_prepare_append(self._h, self._p(row), len(row), length, ctypes.byref(src),
                                                     ctypes.byref(dst))
        return rc, src.value, dst.value

    def drop(self, row: np.ndarray, length: int) -> int:
        return self._lib.marl_page_pool_drop(self._h, self._p(row), length)

    def refcount(self, page: int) -> int:
        c = I32(0)
        _check(self._lib.marl_page_pool_query(self._h, page, ctypes.byref(c), None), "marl_page_pool_query")
        return c.value

    def free_pages(self) -> int:
        c = I32(0)
        _check(self._lib.marl_page_pool_query(self._h, 0, None, ctypes.byref(c)), "marl_page_pool_query")
        return c.value


class PackTable:
    """The table marl_pack_tensors / marl_unpack_tensors read: planned on the host, kept on the device."""

    def __init__(self, tensors):
        self.n = len(tensors)
        self.host = (PackEntry * max(self.n, 1))()
        for k, t in enumerate(tensors):
            self.host[k].ptr = t.data_ptr() if t.numel() else None
            self.host[k].bytes = t.numel() * t.element_size()
        nbytes, chunks = ctypes.c_uint64(0), ctypes.c_int64(0)
        _check(load_library().marl_pack_plan(self.host, self.n, ctypes.byref(nbytes), ctypes.byref(chunks)),
               "marl_pack_plan")
        self.packed_bytes, self.total_chunks = nbytes.value, chunks.value
        self.offsets = [self.host[k].offset for k in range(self.n)]
        self.device = None
        if self.n:
            raw = np.frombuffer(bytes(self.host), dtype=np.uint8)[: self.n * ctypes.sizeof(PackEntry)].copy()
            self.device = torch.from_numpy(raw).to(tensors[0].device)


def marl_pack_tensors(table: PackTable, packed: torch.Tensor):
    if table.n == 0:
        return packed
    _require_cuda(table.device, packed)
    assert packed.numel() * packed.element_size() >= table.packed_bytes
    _check(load_library().marl_pack_tensors(_ptr(table.device), table.n, table.total_chunks, _ptr(packed),
                                            _stream(packed.device)), "marl_pack_tensors")
    return packed


def marl_unpack_tensors(table: PackTable, packed: torch.Tensor):
    if table.n == 0:
        return
    _require_cuda(table.device, packed)
    assert packed.numel() * packed.element_size() >= table.packed_bytes
    _check(load_library().marl_unpack_tensors(_ptr(table.device), table.n, table.total_chunks, _ptr(packed),
                                              _stream(packed.device)), "marl_unpack_tensors")


def marl_profile_begin(max_calls: int):
    _check(load_library().marl_profile_begin(max_calls), "marl_profile_begin")


def marl_profile_end():
    ms = (ctypes.c_float * len(STAGES))()
    na, nl = I32(0), I32(0)
    _check(load_library().marl_profile_end(ms, ctypes.byref(na), ctypes.byref(nl)), "marl_profile_end")
    return {s: float(ms[i]) for i, s in enumerate(STAGES)}, int(na.value), int(nl.value)


# ---- conveniences over the raw calls (allocation + marshalling only) ---------------------------
@dataclass
class AttnCall:
    shape: AttnShape
    layout: PlanLayout
    workspace: torch.Tensor
    out: torch.Tensor


def prepare_attn(inp, out_dtype=MARL_OUT_BF16, suffix_chunk_tokens=0, prefix_chunk_tokens=0) -> AttnCall:
    """Shape, workspace and output tensor for an inputs.AttnInputs resident on a GPU."""
    shape = make_shape(inp.num_seqs, inp.num_groups, inp.Hq, inp.Hkv, inp.num_pages,
                       int(inp.prefix_block_table.shape[1]) if inp.prefix_block_table.dim() == 2 else 0,
                       int(inp.suffix_block_table.shape[1]) if inp.suffix_block_table.dim() == 2 else 0,
                       out_dtype, suffix_chunk_tokens, prefix_chunk_tokens)
    layout = marl_attn_plan_layout_for(shape)
    dev = inp.q.device
    ws = alloc_workspace(layout.total_bytes, dev)
    out = torch.empty((inp.num_seqs, inp.Hq, 128), device=dev,
                      dtype=torch.bfloat16 if out_dtype == MARL_OUT_BF16 else torch.float32)
    return AttnCall(shape, layout, ws, out)


def run_attn(inp, call: AttnCall) -> torch.Tensor:
    return marl_decode_attn(call.shape, call.workspace, inp.q, inp.k_pages, inp.v_pages,
                            inp.prefix_block_table, inp.suffix_block_table, inp.prefix_lens,
                            inp.suffix_lens, inp.group_of_seq, inp.scale, call.out)
