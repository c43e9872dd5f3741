"""Shared pieces of the GPU parity tests: run the library through its C ABI and the float64
checker on the same bytes."""
from __future__ import annotations

import numpy as np
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

ATTN_TOL = 4e-3      # max |delta| for attention outputs (the bar this library is built to)
LOGPROB_TOL = 1e-3   # max |delta| for log-probabilities


def oracle_attn(inp: I.AttnInputs, threads: int = 0) -> np.ndarray:
    return ref.decode_attn(I.bf16_bits(inp.q), I.bf16_bits(inp.k_pages), I.bf16_bits(inp.v_pages),
                           inp.prefix_block_table.cpu().numpy(), inp.suffix_block_table.cpu().numpy(),
                           inp.prefix_lens.cpu().numpy(), inp.suffix_lens.cpu().numpy(),
                           inp.group_of_seq.cpu().numpy(), inp.scale, inp.Hq, inp.Hkv, threads=threads)


def gpu_attn(inp_cpu: I.AttnInputs, out_dtype=B.MARL_OUT_F32, expect_flags=0, **chunks):
    dev = inp_cpu.to("cuda")
    call = B.prepare_attn(dev, out_dtype, **chunks)
    B.run_attn(dev, call)
    torch.cuda.synchronize()
    assert B.marl_attn_read_flags(call.workspace) == expect_flags
    return call.out.float().cpu().numpy().astype(np.float64), call


def check_attn(inp_cpu: I.AttnInputs, out_dtype=B.MARL_OUT_F32, tol=ATTN_TOL, **chunks) -> float:
    want = oracle_attn(inp_cpu)
    got, _ = gpu_attn(inp_cpu, out_dtype, **chunks)
    assert np.isfinite(got).all()
    err = float(np.abs(got - want).max()) if want.size else 0.0
    assert err <= tol, f"max |delta| = {err}"
    return err
