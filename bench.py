#!/usr/bin/env python3
"""Benchmark of the rollout decode step on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic input that is already
resident in HBM: marl_decode_attn (plan, prefix, suffix, merge kernels) followed by
marl_token_logprobs, on the Qwen-7B-shaped workload (2048 sequences, vocabulary 152064).
Prints ONE JSON line.  The CPU baseline leg times the float64 checker on a bounded sample.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2602_09578_amd import binding as B  # noqa: E402
from paper_2602_09578_amd import inputs as I   # noqa: E402

HBM_PEAK_GBPS = 8000.0

# HBM bytes one suffix_kernel launch moves on this workload, from hardware counters
# (profiles/decode_step_qwen7b_hbm_counters.txt: FETCH_SIZE x 2.000 + WRITE_SIZE x 1.000, the
# factors that the one-launch copy of the weight_pack leg, a copy kernel of known size in the same
# run, gives).  Valid only for the kernel source and flags it was taken
# with: reported as null when either has changed since.
SUFFIX_TRAFFIC = {"workload": "qwen7b", "bytes": 5556.8e6 + 14.1e6,
                  "kernel_sources_sha256": "1911bcbbe2344da1a3d4c8ea5234d8c7c91938043a3d9f26a3d6da4ede0b65c2"}
SUFFIX_SOURCES = ("attn_kernels.hip", "wave_ops.h")


def suffix_kernel_hash():
    """Hash of what the suffix kernel is built from: its sources and its compiler flags (include paths aside)."""
    from paper_2602_09578_amd.build import FLAGS, FILE_FLAGS
    h = hashlib.sha256()
    for name in SUFFIX_SOURCES:
        h.update(open(os.path.join(ROOT, "paper_2602_09578_amd", "csrc", name), "rb").read())
    h.update(" ".join(f for f in FLAGS + FILE_FLAGS.get("attn_kernels.hip", []) if not f.startswith("-I")).encode())
    return h.hexdigest()


def suffix_traffic(workload: str):
    """Counter-measured HBM bytes per suffix_kernel launch, or None when they do not apply."""
    try:
        digest = suffix_kernel_hash()
    except OSError:
        return None
    if workload != SUFFIX_TRAFFIC["workload"] or digest != SUFFIX_TRAFFIC["kernel_sources_sha256"]:
        return None
    return SUFFIX_TRAFFIC["bytes"]


def cpu_baseline(attn_dev: I.AttnInputs, lp_dev: I.LogprobInputs, seq_stride: int, lp_rows: int):
    """Times the float64 checker (as it stands, all host threads) on every `seq_stride`-th
    sequence and on the first `lp_rows` logit rows of the same workload."""
    from oracle import reference as ref
    pick = list(range(0, attn_dev.num_seqs, seq_stride))
    sub = I.extract_subproblem(attn_dev, pick)
    args = (I.bf16_bits(sub.q), I.bf16_bits(sub.k_pages), I.bf16_bits(sub.v_pages),
            sub.prefix_block_table.numpy(), sub.suffix_block_table.numpy(), sub.prefix_lens.numpy(),
            sub.suffix_lens.numpy(), sub.group_of_seq.numpy(), sub.scale, sub.Hq, sub.Hkv)
    t0 = time.perf_counter()
    _, threads = ref.decode_attn(*args, return_threads=True)
    t_attn = time.perf_counter() - t0
    rows = min(lp_rows, lp_dev.logits.shape[0])
    lg = I.bf16_bits(lp_dev.logits[:rows])
    tk = lp_dev.tokens[:rows].cpu().numpy()
    t0 = time.perf_counter()
    ref.token_logprobs(lg, tk, lp_dev.temperature)
    t_lp = time.perf_counter() - t0
    per_seq = t_attn / len(pick) + t_lp / rows      # one sequence's attention + its log-prob row
    return {"value": 1.0 / per_seq, "unit": "sequences*steps/s", "cores": int(threads), "kind": "oracle",
            "sample": f"every sequence with index divisible by {seq_stride} ({len(pick)} of {attn_dev.num_seqs}) for attention "
                      f"({t_attn:.2f} s) and {rows} of {lp_dev.logits.shape[0]} logit rows ({t_lp:.2f} s)",
            "attn_seqs_per_s": len(pick) / t_attn, "logprob_rows_per_s": rows / t_lp}


def dominant_kernel_roofline(w, attn, call, stage_ms):
    """Roofline entry of the attention kernel that takes the most time of a call."""
    bpt = attn.kv_bytes_per_token()
    # the suffix kernel processes the suffix items of more than 128 tokens (the shorter ones are taken
    # by the workgroups of the merge and prefix kernels): its algorithmic bytes per launch
    S = attn.suffix_lens.cpu().numpy().astype(np.int64)
    Cs = call.layout.suffix_chunk_tokens
    tail = S % Cs
    long_tok = int(((S // Cs) * Cs * (Cs > 128) + tail * (tail > 128)).sum())
    if long_tok and stage_ms["suffix"] >= stage_ms["prefix"]:
        gbps = long_tok * bpt / (stage_ms["suffix"] * 1e-3) / 1e9
        return {"kernel": "suffix_kernel", "bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": gbps / HBM_PEAK_GBPS, "traffic": suffix_traffic(w.name),
                "algorithmic_bytes_per_launch": long_tok * bpt, "avg_launch_ms": stage_ms["suffix"]}
    # the prefix kernel dominates (prefix-dominated group sampling): its QK^T and PV products against the
    # dense bf16 matrix peak, and its unique prefix bytes against the HBM peak
    counts = np.bincount(attn.group_of_seq.cpu().numpy(), minlength=attn.num_groups)
    P = attn.prefix_lens.cpu().numpy().astype(np.int64)
    flops = int(4 * 128 * w.Hq * (P * counts).sum())
    tf = flops / (stage_ms["prefix"] * 1e-3) / 1e12
    pbytes = int(P.sum()) * bpt
    return {"kernel": "prefix_kernel", "bound": "mfma", "achieved": tf, "peak": 2500.0, "unit": "TFLOP/s",
            "frac": tf / 2500.0, "traffic": None, "algorithmic_flops_per_launch": flops,
            "avg_launch_ms": stage_ms["prefix"],
            "hbm_frac_on_unique_prefix_bytes": pbytes / (stage_ms["prefix"] * 1e-3) / 1e9 / HBM_PEAK_GBPS}


def measure_workload(name: str, dev, iters: int = 20, warmup: int = 3):
    """One workload's decode attention (and its log-prob call where the workload names one), outside the
    headline timed region: per-call times from events around each call, then per-kernel averages from
    the library's own event timing over `iters` further calls."""
    w = I.WORKLOADS[name]
    attn = I.build_attn_inputs(w, device=dev)
    call = B.prepare_attn(attn, B.MARL_OUT_BF16)
    for _ in range(warmup):
        B.run_attn(attn, call)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for e0, e1 in evs:
        e0.record()
        B.run_attn(attn, call)
        e1.record()
    torch.cuda.synchronize()
    t = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    med = t[len(t) // 2]
    B.marl_profile_begin(iters)
    for _ in range(iters):
        B.run_attn(attn, call)
    torch.cuda.synchronize()
    stage_ms, n_attn, _ = B.marl_profile_end()
    assert n_attn == iters and B.marl_attn_read_flags(call.workspace) == 0
    assert torch.isfinite(call.out.float()).all().item()
    ptok, stok = attn.unique_kv_tokens()
    ubytes = (ptok + stok) * attn.kv_bytes_per_token()
    r = {"num_seqs": w.num_seqs, "unique_kv_bytes": ubytes, "attn_ms_median": med, "attn_ms_min": t[0],
         "unique_kv_GBps": ubytes / (med * 1e-3) / 1e9,
         "pct_of_hbm_peak": ubytes / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS * 100,
         "seq_steps_per_s": w.num_seqs / (med * 1e-3),
         "kernel_ms": {k: stage_ms[k] for k in ("plan", "prefix", "suffix", "merge")},
         "dominant_kernel": dominant_kernel_roofline(w, attn, call, stage_ms)}
    r["dominant_kernel"].pop("traffic", None)
    del attn, call
    if w.vocab:
        lp = I.build_logprob_inputs(w.num_seqs, w.vocab, w.logit_sigma, w.seed, device=dev)
        nws = B.marl_logprobs_workspace_bytes(w.num_seqs, w.vocab)
        ws = B.alloc_workspace(nws, dev) if nws else None
        out = torch.empty(w.num_seqs, dtype=torch.float32, device=dev)
        for _ in range(warmup):
            B.marl_token_logprobs(lp.logits, lp.tokens, lp.temperature, out, ws)
        for e0, e1 in evs:
            e0.record()
            B.marl_token_logprobs(lp.logits, lp.tokens, lp.temperature, out, ws)
            e1.record()
        torch.cuda.synchronize()
        t = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
        med = t[len(t) // 2]
        assert torch.isfinite(out).all().item()
        r["logprob"] = {"rows": w.num_seqs, "vocab": w.vocab, "ms_median": med,
                        "rows_per_s": w.num_seqs / (med * 1e-3),
                        "GBps": w.num_seqs * w.vocab * 2 / (med * 1e-3) / 1e9,
                        "frac_of_hbm_peak": w.num_seqs * w.vocab * 2 / (med * 1e-3) / 1e9 / HBM_PEAK_GBPS}
        del lp, ws, out
    torch.cuda.empty_cache()
    return r


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="qwen7b", choices=sorted(I.WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-workloads", action="store_true", help="skip the per-workload block")
    ap.add_argument("--cpu-seq-stride", type=int, default=1, help="CPU baseline: every n-th sequence")
    ap.add_argument("--cpu-logprob-rows", type=int, default=1 << 30, help="CPU baseline: first n logit rows")
    ap.add_argument("--suffix-chunk", type=int, default=0)
    ap.add_argument("--prefix-chunk", type=int, default=0)
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: this library has no multi-GPU path (run with --gpus 1)")
    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU: the library has no CPU path")

    w = I.WORKLOADS[a.workload]
    dev = torch.device("cuda:0")
    attn = I.build_attn_inputs(w, device=dev)
    call = B.prepare_attn(attn, B.MARL_OUT_BF16, a.suffix_chunk, a.prefix_chunk)
    vocab = w.vocab or 152064
    sigma = w.logit_sigma or 3.0
    lp = I.build_logprob_inputs(w.num_seqs, vocab, sigma, w.seed, device=dev)
    nws = B.marl_logprobs_workspace_bytes(w.num_seqs, vocab)
    lp_ws = B.alloc_workspace(nws, dev) if nws else None
    lp_out = torch.empty(w.num_seqs, dtype=torch.float32, device=dev)

    def step():
        B.run_attn(attn, call)
        B.marl_token_logprobs(lp.logits, lp.tokens, lp.temperature, lp_out, lp_ws)

    for _ in range(a.warmup):
        step()
    # timed region 1: exactly K steps, nothing else on the stream -> `value`
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # the same K steps once more, each bracketed by its own pair of events: median and minimum
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(a.steps)]
    for e0, e1 in evs:
        e0.record()
        step()
        e1.record()
    torch.cuda.synchronize()
    per_step = sorted(e0.elapsed_time(e1) for e0, e1 in evs)
    # timed region 2: the same K steps with the library recording HIP events around every
    # kernel on the call's stream -> per-kernel durations (the events cost a few us per kernel)
    B.marl_profile_begin(a.steps)
    t1 = time.perf_counter()
    for _ in range(a.steps):
        step()
    torch.cuda.synchronize()
    dt_prof = time.perf_counter() - t1
    stage_ms, n_attn, n_lp = B.marl_profile_end()
    assert n_attn == a.steps and n_lp == a.steps
    assert B.marl_attn_read_flags(call.workspace) == 0
    assert torch.isfinite(lp_out).all().item() and torch.isfinite(call.out.float()).all().item()

    # the same step captured once into a HIP graph and replayed K times (the entry points only
    # enqueue kernels, so they can be captured): what a launch-bound decode loop would run
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    graph.replay()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(a.steps):
        graph.replay()
    torch.cuda.synchronize()
    ms_per_step_graph = (time.perf_counter() - t2) / a.steps * 1e3
    del graph

    ms_per_step = dt / a.steps * 1e3
    ptok, stok = attn.unique_kv_tokens()
    bpt = attn.kv_bytes_per_token()
    attn_ms = stage_ms["plan"] + stage_ms["prefix"] + stage_ms["suffix"] + stage_ms["merge"]
    lp_ms = stage_ms["logprob"] + stage_ms["logprob_finish"]
    roofline = dominant_kernel_roofline(w, attn, call, stage_ms)
    res = {
        "metric": "rollout decode step throughput (paged shared-prefix decode attention + token log-probs)",
        "value": w.num_seqs / (ms_per_step * 1e-3),
        "unit": "sequences*steps/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.num_seqs} seqs, {w.num_groups} prompts, Hq {w.Hq}/Hkv {w.Hkv}, "
                               f"d 128, page 16, vocab {vocab}",
                   "unique_kv_bytes": (ptok + stok) * bpt, "prefix_tokens": ptok, "suffix_tokens": stok,
                   "suffix_chunk_tokens": call.layout.suffix_chunk_tokens,
                   "prefix_chunk_tokens": call.layout.prefix_chunk_tokens},
        "stage_ms": stage_ms,
        "ms_per_step_median": per_step[len(per_step) // 2], "ms_per_step_min": per_step[0],
        "ms_per_step_graph_replay": ms_per_step_graph,
        "ms_per_step_with_stage_events": dt_prof / a.steps * 1e3,
        "attn_unique_kv_GBps": (ptok + stok) * bpt / (attn_ms * 1e-3) / 1e9,
        "attn_pct_of_hbm_peak": (ptok + stok) * bpt / (attn_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS * 100,
        "attn_seq_steps_per_s": w.num_seqs / (attn_ms * 1e-3),
        "logprob_rows_per_s": w.num_seqs / (lp_ms * 1e-3),
        "logprob_GBps": w.num_seqs * vocab * 2 / (lp_ms * 1e-3) / 1e9,
        "roofline": roofline,
    }
    # KV append (the cache maintenance that precedes attention in a decode iteration), timed
    # after everything else because it overwrites each sequence's last token
    k_new = I.randn_bf16((w.num_seqs, w.Hkv, 128), 1.0, torch.Generator(device=dev).manual_seed(1), dev)
    v_new = I.randn_bf16((w.num_seqs, w.Hkv, 128), 1.0, torch.Generator(device=dev).manual_seed(2), dev)
    lens_before = (attn.suffix_lens - 1).clamp(min=0)
    lens_work = lens_before.clone()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_app = 20
    tot = 0.0
    for it in range(n_app + 2):
        lens_work.copy_(lens_before)
        ev0.record()
        B.marl_kv_append(call.shape, k_new, v_new, attn.k_pages, attn.v_pages, attn.suffix_block_table, lens_work)
        ev1.record()
        torch.cuda.synchronize()
        if it >= 2:
            tot += ev0.elapsed_time(ev1)
    res["kv_append"] = {"us_per_call": tot / n_app * 1e3, "tokens": w.num_seqs,
                        "bytes_written": w.num_seqs * w.Hkv * 128 * 2 * 2}
    # sampling fused with the log-probability (one more row beyond the timed step)
    uniforms = torch.rand(w.num_seqs, device=dev, generator=torch.Generator(device=dev).manual_seed(3))
    s_ws = B.alloc_workspace(B.marl_sample_workspace_bytes(w.num_seqs, vocab), dev)
    s_tok = torch.empty(w.num_seqs, dtype=torch.int32, device=dev)
    s_lp = torch.empty(w.num_seqs, dtype=torch.float32, device=dev)
    tot = 0.0
    for it in range(12):
        ev0.record()
        B.marl_sample_tokens(lp.logits, uniforms, lp.temperature, s_tok, s_lp, s_ws)
        ev1.record()
        torch.cuda.synchronize()
        if it >= 2:
            tot += ev0.elapsed_time(ev1)
    res["sample_tokens"] = {"us_per_call": tot / 10 * 1e3, "rows": w.num_seqs,
                            "GBps": w.num_seqs * vocab * 2 / (tot / 10 * 1e-3) / 1e9}
    tot = 0.0
    for it in range(7):
        ev0.record()
        B.marl_sample_tokens_top_p(lp.logits, uniforms, lp.temperature, 0.9, s_tok, s_lp)
        ev1.record()
        torch.cuda.synchronize()
        if it >= 2:
            tot += ev0.elapsed_time(ev1)
    res["sample_tokens_top_p"] = {"us_per_call": tot / 5 * 1e3, "rows": w.num_seqs, "top_p": 0.9,
                                  "GBps_of_one_read": w.num_seqs * vocab * 2 / (tot / 5 * 1e-3) / 1e9}
    del s_ws, uniforms
    # training-side log-probs: one micro-batch of 16 responses x 1024 positions at once (the
    # same entry point on 8 x the rows: 5 GB of logits)
    if vocab >= 32768:
        t_rows = 16 * 1024
        tl = I.build_logprob_inputs(t_rows, vocab, sigma, w.seed + 1, device=dev)
        t_need = B.marl_logprobs_workspace_bytes(t_rows, vocab)
        t_ws = B.alloc_workspace(t_need, dev) if t_need else None
        t_out = torch.empty(t_rows, dtype=torch.float32, device=dev)
        tot = 0.0
        for it in range(7):
            ev0.record()
            B.marl_token_logprobs(tl.logits, tl.tokens, tl.temperature, t_out, t_ws)
            ev1.record()
            torch.cuda.synchronize()
            if it >= 2:
                tot += ev0.elapsed_time(ev1)
        assert torch.isfinite(t_out).all().item()
        res["logprobs_training_shape"] = {"ms_per_call": tot / 5, "rows": t_rows,
                                          "GBps": t_rows * vocab * 2 / (tot / 5 * 1e-3) / 1e9}
        del tl, t_ws, t_out
    # prompt (prefill) attention over the workload's prompts: the step that creates the shared
    # prefixes; dense causal MFMA work, reported against the bf16 matrix peak
    pf = I.build_prefill_inputs(w.Hq, w.Hkv, attn.prefix_lens.cpu().tolist(), [0] * w.num_groups, device=dev,
                                seed=w.seed, poison=False)
    pshape, pws, pout = B.prepare_prefill(pf, B.MARL_OUT_BF16)
    pflags = torch.zeros(1, dtype=torch.int32, device=dev)
    t_attn = t_write = 0.0
    for it in range(7):
        ev0.record()
        B.marl_kv_write_prompt(pshape, pf.k_new, pf.v_new, pf.k_pages, pf.v_pages, pf.prefix_block_table,
                               pf.q_start, pf.q_pos0, pflags)
        ev1.record()
        ev2 = torch.cuda.Event(enable_timing=True)
        B.run_prefill(pf, pshape, pws, pout)
        ev2.record()
        torch.cuda.synchronize()
        if it >= 2:
            t_write += ev0.elapsed_time(ev1)
            t_attn += ev1.elapsed_time(ev2)
    assert int(pflags.item()) == 0 and B.marl_attn_read_flags(pws) == 0
    pf_flops = pf.causal_pairs() * w.Hq * 4 * 128
    res["prefill"] = {"ms_per_call": t_attn / 5, "prompt_tokens": pf.num_tokens, "TFLOPps": pf_flops / (t_attn / 5 * 1e-3) / 1e12,
                      "frac_of_bf16_mfma_peak": pf_flops / (t_attn / 5 * 1e-3) / 1e12 / 2500.0,
                      "kv_write_prompt_us": t_write / 5 * 1e3}
    del pf, pws, pout
    # weight synchronisation as one copy: a parameter list of the workload's model shape (bf16)
    # gathered into one contiguous buffer by one launch, against one device copy per parameter
    params = [torch.zeros(n, dtype=torch.bfloat16, device=dev) for n in I.model_param_sizes(w.Hq, w.Hkv, vocab)]
    table = B.PackTable(params)
    packed = torch.empty(table.packed_bytes, dtype=torch.uint8, device=dev)
    views = [packed[o:o + p_.numel() * 2].view(torch.bfloat16) for o, p_ in zip(table.offsets, params)]
    t_pack = t_each = 0.0
    for it in range(5):
        ev0.record()
        B.marl_pack_tensors(table, packed)
        ev1.record()
        ev2 = torch.cuda.Event(enable_timing=True)
        for v_, p_ in zip(views, params):
            v_.copy_(p_)
        ev2.record()
        torch.cuda.synchronize()
        if it >= 2:
            t_pack += ev0.elapsed_time(ev1)
            t_each += ev1.elapsed_time(ev2)
    moved = sum(p_.numel() * 2 for p_ in params)
    res["weight_pack"] = {"ms_per_call": t_pack / 3, "tensors": len(params), "bytes": moved,
                          "GBps_read_plus_write": 2 * moved / (t_pack / 3 * 1e-3) / 1e9,
                          "one_copy_per_tensor_ms": t_each / 3}
    del params, packed, views, table
    # every named workload's attention call (and log-prob call), outside the timed step
    if not a.no_workloads:
        torch.cuda.empty_cache()
        res["workloads"] = {name: measure_workload(name, dev) for name in I.WORKLOADS}
    if not a.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(attn, lp, seq_stride=a.cpu_seq_stride, lp_rows=a.cpu_logprob_rows)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
