"""GPU parity of marl_sample_tokens.  The token is an integer decided by float32 sums on the
GPU and float64 sums in the reference, so a drawn token is accepted when the reference CDF
brackets the uniform within 2e-6 (the kernel adds the few dozen chunk sums in double precision;
what is left is the float32 rounding inside a 4096-logit chunk); it must equal the reference
token whenever the uniform is further than that from every CDF step, which at the 152064-token
vocabulary is the case for about nine draws in ten.  Its log-probability must match the
reference's for that token to 1e-3."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

pytestmark = pytest.mark.gpu
CDF_TOL = 2e-6


def run(lp: I.LogprobInputs, u: np.ndarray):
    d = lp.to("cuda") if not lp.logits.is_cuda else lp
    rows, vocab = d.logits.shape
    ws = B.alloc_workspace(B.marl_sample_workspace_bytes(rows, vocab), "cuda")
    tok = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    out = torch.zeros(rows, dtype=torch.float32, device="cuda")
    B.marl_sample_tokens(d.logits, torch.from_numpy(u.astype(np.float32)).cuda(), d.temperature, tok, out, ws)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), out.cpu().numpy().astype(np.float64)


def check(lp: I.LogprobInputs, u: np.ndarray):
    tok, out = run(lp, u)
    bits = I.bf16_bits(lp.logits)
    u32 = u.astype(np.float32).astype(np.float64)
    exact = 0
    for r in range(len(u)):
        p, cdf = ref.softmax_cdf(bits[r], lp.temperature)
        t = int(tok[r])
        assert 0 <= t < len(p) and p[t] > 0
        lo = cdf[t - 1] if t > 0 else 0.0
        assert lo - CDF_TOL <= u32[r] <= cdf[t] + CDF_TOL, (r, t, lo, u32[r], cdf[t])
        want_t, _ = ref.sample_tokens(bits[r:r + 1], [u32[r]], lp.temperature)
        if np.abs(cdf - u32[r]).min() > CDF_TOL:
            assert t == want_t[0]
            exact += 1
        assert abs(out[r] - np.log(p[t])) <= 1e-3
    return exact


@pytest.mark.parametrize("rows,vocab,T", [(16, 4096, 1.0), (40, 152064, 1.0), (3, 152064, 0.6), (300, 32000, 1.7),
                                          (7, 4099, 1.0), (5, 7, 1.0), (2, 1, 1.0), (9, 20481, 0.9)])
def test_sampled_tokens_are_valid_and_logprobs_match(rows, vocab, T):
    print("case: sampling", rows, vocab, T, flush=True)
    lp = I.build_logprob_inputs(rows, vocab, 3.0, 29, temperature=T)
    rng = np.random.default_rng(rows * 7 + vocab)
    u = rng.random(rows)
    u[0] = 0.0
    if rows > 1:
        u[1] = np.nextafter(np.float32(1.0), np.float32(0.0))
    exact = check(lp, u)
    if 64 <= vocab <= 8192:      # CDF steps are far apart compared with the tolerance: nearly every draw is decidable
        assert exact >= rows - 2
    if rows >= 40:               # also at the real vocabulary most draws are decided, and decided right
        assert exact >= 0.85 * rows, (exact, rows)


def test_uniform_logits_and_masked_vocabulary():
    print("case: sampling special", flush=True)
    V = 10000
    lp = I.LogprobInputs(torch.full((4, V), 0.5, dtype=torch.bfloat16), torch.zeros(4, dtype=torch.int32), 1.0)
    u = np.array([0.00005, 0.25003, 0.5, 0.99996])
    tok, out = run(lp, u)
    assert np.abs(tok - np.floor(u.astype(np.float32).astype(np.float64) * V)).max() <= 1
    assert np.abs(out + np.log(V)).max() <= 1e-3
    x = torch.zeros(3, 5000, dtype=torch.bfloat16); x[:, :100] = float("-inf"); x[:, 4000:] = float("-inf")
    x[2, :] = float("-inf")
    tok, out = run(I.LogprobInputs(x, torch.zeros(3, dtype=torch.int32), 1.0), np.array([0.0, 0.9999999, 0.5]))
    assert tok[0] == 100 and tok[1] == 3999 and tok[2] == -1 and np.isnan(out[2])


def test_full_size_rows_and_rerun_identical():
    print("case: sampling full size", flush=True)
    w = I.WORKLOADS["qwen7b"]
    lp = I.build_logprob_inputs(w.num_seqs, w.vocab, w.logit_sigma, w.seed, device="cuda")
    u = np.random.default_rng(9).random(w.num_seqs)
    tok1, out1 = run(lp, u)
    tok2, out2 = run(lp, u)
    assert np.array_equal(tok1, tok2) and np.array_equal(out1, out2)
    sample = list(range(0, w.num_seqs, 64))
    sub = I.LogprobInputs(lp.logits[sample].cpu(), lp.tokens[sample].cpu(), lp.temperature)
    bits = I.bf16_bits(sub.logits)
    for k, r in enumerate(sample):
        p, cdf = ref.softmax_cdf(bits[k], lp.temperature)
        t = int(tok1[r]); lo = cdf[t - 1] if t > 0 else 0.0
        uf = float(np.float32(u[r]))
        assert lo - CDF_TOL <= uf <= cdf[t] + CDF_TOL and abs(out1[r] - np.log(p[t])) <= 1e-3
