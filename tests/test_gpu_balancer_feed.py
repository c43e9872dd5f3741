"""The load balancer's per-step batch composition fed to the decode-attention call: the
requests an instance decodes at some step become one marl_decode_attn batch (samples of the
same prompt that landed on the same instance share their prefix), checked against the float64
checker like any other batch."""
import numpy as np
import pytest

from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I
from tests.gpu_common import ATTN_TOL, check_attn

pytestmark = pytest.mark.gpu


def test_instance_batches_of_a_skewed_rollout_run_through_decode_attention():
    rng = np.random.default_rng(7)
    G = 4
    bal = B.Balancer([2, 2, 2], delta=5, slots_per_instance=24, poll_interval=4, migration_delay=6)
    prompt_len, rid = {}, 0
    checked = 0
    for t in range(120):
        if t < 60:
            for agent, rate in enumerate((0.8, 0.15, 0.1)):        # agent 0 is the hot one
                if rng.random() < rate:
                    plen = int(rng.integers(20, 200))
                    for _ in range(G):                              # the G samples of one prompt
                        prompt_len[rid] = (rid // G, plen)
                        bal.submit(agent, rid, int(rng.integers(5, 90)))
                        rid += 1
        st = bal.step()
        if t in (30, 70, 100):
            for inst in range(bal.num_instances):
                owner, ids, generated = bal.instance_batch(inst)
                live = [(r, g) for r, g in zip(ids, generated) if g > 0]   # a request's first token has no cache yet
                if owner < 0 or not live:
                    continue
                prompts = sorted({prompt_len[r][0] for r, _ in live})
                gmap = {p: k for k, p in enumerate(prompts)}
                lens = I.Lengths(
                    np.array([next(prompt_len[r][1] for r, _ in live if prompt_len[r][0] == p) for p in prompts], dtype=np.int32),
                    np.array([g for _, g in live], dtype=np.int32),
                    np.array([gmap[prompt_len[r][0]] for r, _ in live], dtype=np.int32),
                    np.zeros(len(prompts), dtype=np.int32))
                w = I.Workload("instance batch", 8, 2, (), seed=100 + inst)
                inp = I.build_attn_inputs(w, "cpu", lengths=lens)
                assert check_attn(inp) <= ATTN_TOL
                checked += 1
    assert st.migrations > 0 and checked >= 6
    bal.close()
