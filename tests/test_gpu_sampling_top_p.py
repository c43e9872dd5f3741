"""GPU parity of marl_sample_tokens_top_p.  Two integers are decided by floating-point sums
(float32 on the GPU, float64 in the reference): which value is the nucleus threshold, and
which token passes the scaled uniform.  A drawn token is accepted when it is what the
reference draws for top_p and u moved by at most 4e-6 (relative) / 2e-6 (of the nucleus mass);
it must EQUAL the reference token whenever no nucleus boundary lies within 4e-6 of top_p and
no CDF step within 2e-6 of u.  The log-probability must match the reference's for that token
to 1e-3."""
import numpy as np
import pytest
import torch

from oracle import reference as ref
from paper_2602_09578_amd import binding as B
from paper_2602_09578_amd import inputs as I

pytestmark = pytest.mark.gpu
P_TOL, CDF_TOL = 4e-6, 2e-6


def run(logits: torch.Tensor, u: np.ndarray, T: float, top_p: float):
    d = logits.cuda()
    rows = d.shape[0]
    tok = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    out = torch.zeros(rows, dtype=torch.float32, device="cuda")
    B.marl_sample_tokens_top_p(d, torch.from_numpy(u.astype(np.float32)).cuda(), T, top_p, tok, out)
    torch.cuda.synchronize()
    return tok.cpu().numpy(), out.cpu().numpy().astype(np.float64)


def check(logits: torch.Tensor, u: np.ndarray, T: float, top_p: float, rows_to_check=None):
    tok, out = run(logits, u, T, top_p)
    u32 = u.astype(np.float32).astype(np.float64)
    tp = float(np.float32(top_p))
    exact = 0
    for r in (range(len(u)) if rows_to_check is None else rows_to_check):
        p, _ = ref.softmax_cdf(I.bf16_bits(logits[r:r + 1])[0], T)
        t = int(tok[r])
        assert 0 <= t < len(p) and p[t] > 0, (r, t)
        masks = [ref.nucleus(p, min(1.0, tp * f)) for f in (1 - P_TOL, 1.0, 1 + P_TOL)]
        ok = False
        for keep in masks:
            if not keep[t]:
                continue
            q = np.where(keep, p, 0.0)
            cdf, mass = np.cumsum(q), q.sum()
            lo = cdf[t] - q[t]
            ok |= lo - CDF_TOL * mass <= u32[r] * mass <= cdf[t] + CDF_TOL * mass
        assert ok, (r, t, top_p)
        decidable = all(np.array_equal(masks[0], m) for m in masks[1:])
        if decidable:
            q = np.where(masks[1], p, 0.0)
            cdf, mass = np.cumsum(q), q.sum()
            steps = cdf[masks[1]]
            if np.abs(steps - u32[r] * mass).min() > CDF_TOL * mass:
                want, _ = ref.sample_tokens_top_p(I.bf16_bits(logits[r:r + 1]), [u32[r]], T, tp)
                assert t == want[0], (r, t, want[0])
                exact += 1
        assert abs(out[r] - np.log(p[t])) <= 1e-3
    return exact


@pytest.mark.parametrize("rows,vocab,T,top_p", [
    (16, 4096, 1.0, 0.9), (12, 152064, 1.0, 0.95), (3, 152064, 0.6, 0.5), (100, 32000, 1.7, 0.8),
    (7, 4099, 1.0, 0.99), (5, 7, 1.0, 0.6), (2, 1, 1.0, 0.3), (9, 20481, 0.9, 0.1), (6, 8192, 1.0, 1.0),
    (6, 8193, 1.3, 1e-4),
    # rows longer than the register-resident variant holds (163840 logits): every pass re-reads memory
    (3, 200003, 1.0, 0.9), (2, 262144, 0.7, 0.97),
    # the two sides of that limit
    (2, 163840, 1.0, 0.8), (2, 163841, 1.0, 0.8)])
def test_tokens_match_the_reference(rows, vocab, T, top_p):
    print("case: top-p", rows, vocab, T, top_p, flush=True)
    lp = I.build_logprob_inputs(rows, vocab, 3.0, 31, temperature=T)
    rng = np.random.default_rng(rows * 11 + vocab)
    u = rng.random(rows)
    u[0] = 0.0
    if rows > 1:
        u[1] = np.nextafter(np.float32(1.0), np.float32(0.0))
    exact = check(lp.logits, u, T, top_p)
    # where the steps of the ranking's running mass and of the CDF are far apart compared with the
    # tolerances, nearly every draw is decidable (with top_p = 0.99 the boundary lies among tail
    # tokens of probability ~1e-5 and is rarely decidable)
    if 64 <= vocab <= 8192 and top_p <= 0.9:
        assert exact >= rows - 2
    if rows >= 100:   # a vocabulary of 32000: most draws are decided, and decided right
        assert exact >= 0.7 * rows, (exact, rows)


def test_flat_rows_ties_and_masks():
    print("case: top-p special", flush=True)
    V = 10000
    flat = torch.full((4, V), 0.5, dtype=torch.bfloat16)        # every token ties: the first ceil(top_p V) are kept
    u = np.array([0.00005, 0.25003, 0.5, 0.99996])
    tok, out = run(flat, u, 1.0, 0.3)
    assert np.abs(tok - np.floor(u.astype(np.float32).astype(np.float64) * 3000)).max() <= 1
    assert tok.max() < 3001 and np.abs(out + np.log(V)).max() <= 1e-3
    x = torch.zeros(3, 5000, dtype=torch.bfloat16); x[:, :100] = float("-inf"); x[:, 4000:] = float("-inf")
    x[2, :] = float("-inf")
    tok, out = run(x, np.array([0.0, 0.9999999, 0.5]), 1.0, 0.5)  # 3900 equal tokens, half of them kept
    assert tok[0] == 100 and abs(tok[1] - (100 + 1949)) <= 1 and tok[2] == -1 and np.isnan(out[2])
    # the same on a row that is re-read from memory for every pass
    V2 = 170000
    flat2 = torch.full((2, V2), -1.25, dtype=torch.bfloat16)
    u2 = np.array([0.25003, 0.99996])
    tok, out = run(flat2, u2, 1.0, 0.3)
    assert np.abs(tok - np.floor(u2.astype(np.float32).astype(np.float64) * 51000)).max() <= 1
    assert tok.max() < 51001 and np.abs(out + np.log(V2)).max() <= 1e-3
    # +0 and -0 are different bit patterns of the same probability: they tie, by index
    z = torch.zeros(2, 1000, dtype=torch.bfloat16); z[:, ::2] = -0.0
    tok, _ = run(z, np.array([0.5003, 0.99996]), 1.0, 0.25)
    assert list(tok) == [125, 249]
    # a peaked row: one token holds 99 %: any top_p up to that returns it whatever u is
    y = torch.zeros(2, 3000, dtype=torch.bfloat16); y[:, 1234] = 12.5
    tok, _ = run(y, np.array([0.0, 0.999]), 1.0, 0.9)
    assert list(tok) == [1234, 1234]


def test_nucleus_below_the_first_window_of_values():
    # logits spread over a wide range with top_p close to 1: the threshold value lies more than
    # 32768 bf16 values below the maximum (beyond the first histogram window)
    rng = np.random.default_rng(3)
    x = torch.from_numpy(rng.uniform(-0.9, 0.3, size=(6, 6000)).astype(np.float32)).to(torch.bfloat16)
    u = rng.random(6)
    assert check(x, u, 1.0, 0.98) >= 4
    assert check(x, u, 1.0, 0.999999) >= 0


def test_full_size_rows_rerun_identical_and_sampled_check():
    print("case: top-p full size", flush=True)
    w = I.WORKLOADS["qwen7b"]
    lp = I.build_logprob_inputs(w.num_seqs, w.vocab, w.logit_sigma, w.seed, device="cuda")
    u = np.random.default_rng(9).random(w.num_seqs)
    tok1, out1 = run(lp.logits, u, 1.0, 0.9)
    tok2, out2 = run(lp.logits, u, 1.0, 0.9)
    assert np.array_equal(tok1, tok2) and np.array_equal(out1, out2)
    sample = list(range(0, w.num_seqs, 128))
    sub = lp.logits[sample].cpu()
    tok_s, out_s = run(sub, u[sample], 1.0, 0.9)
    assert np.array_equal(tok_s, tok1[sample])                 # a row's result does not depend on the batch
    check(sub, u[sample], 1.0, 0.9)
