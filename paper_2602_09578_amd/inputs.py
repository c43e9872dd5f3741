"""Seeded synthetic inputs for the rollout decode step.

This module only *draws and arranges* data: sequence-length mixes, block tables,
random bf16 tensors, NaN poison.  It contains none of the arithmetic of attention or
of log-probabilities, so that both the checker and the GPU library can consume the
same bytes without sharing any of the method.

Workload structure follows the paper's description of multi-agent rollout:
every prompt is expanded into several candidate samples that share its prefix
(Parallel Sampling, Section 5.1; the evaluation uses intra-query parallelism 16 and
inter-query parallelism 4, Section 8.1), agents see heavily skewed load (Observation
#2, Section 2.2), responses are capped at 8192 tokens (Section 8.1) and the policy
models are Qwen2.5-class GQA transformers (Section 8.1).  The paper's own datasets
are confidential, so these draws stand in for them.

Physical KV layout produced here (it is the library's ABI):
  k_pages  bf16 [num_pages, Hkv, PAGE, D]   (one token's key is D contiguous values)
  v_pages  bf16 [num_pages, Hkv, D, PAGE]   (one channel's PAGE slots are contiguous)
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional, Sequence, Tuple

import numpy as np
import torch

PAGE = 16
D = 128


# --------------------------------------------------------------------------------------
# length distributions
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class LenDist:
    kind: str                 # "const" | "uniform" | "lognormal"
    a: float = 0.0            # const value / uniform low / lognormal median
    b: float = 0.0            # uniform high (inclusive) / lognormal sigma
    cap: int = 0              # lognormal clamp (0 = none)

    def draw(self, rng: np.random.Generator, n: int) -> np.ndarray:
        if self.kind == "const":
            return np.full(n, int(self.a), dtype=np.int64)
        if self.kind == "uniform":
            return rng.integers(int(self.a), int(self.b) + 1, size=n, dtype=np.int64)
        if self.kind == "lognormal":
            z = rng.standard_normal(n)
            v = np.rint(np.exp(math.log(self.a) + self.b * z)).astype(np.int64)
            hi = self.cap if self.cap > 0 else np.iinfo(np.int64).max
            return np.clip(v, 1, hi)
        raise ValueError(self.kind)

    def scaled(self, div: int) -> "LenDist":
        """Same shape of distribution with every length divided by `div` (at least 1)."""
        if div == 1:
            return self
        s = lambda x: max(1, int(round(x / div)))
        if self.kind == "const":
            return LenDist("const", s(self.a))
        if self.kind == "uniform":
            return LenDist("uniform", s(self.a), max(s(self.a), s(self.b)))
        return LenDist("lognormal", max(1.0, self.a / div), self.b, max(1, self.cap // div))


def const(v): return LenDist("const", v)
def uniform(lo, hi): return LenDist("uniform", lo, hi)
def lognormal(median, sigma, cap): return LenDist("lognormal", median, sigma, cap)


@dataclass(frozen=True)
class Agent:
    prompts: int              # number of prompts (= shared-prefix groups) of this agent
    G: int                    # samples per prompt
    prompt_len: LenDist
    gen_len: LenDist


@dataclass(frozen=True)
class Workload:
    name: str
    Hq: int
    Hkv: int
    agents: Tuple[Agent, ...]
    seed: int
    vocab: int = 0            # 0 = the workload names no log-prob pass
    logit_sigma: float = 0.0
    temperature: float = 1.0

    @property
    def num_groups(self) -> int:
        return sum(a.prompts for a in self.agents)

    @property
    def num_seqs(self) -> int:
        return sum(a.prompts * a.G for a in self.agents)

    def scaled(self, prompts_div: int = 1, len_div: int = 1, vocab: Optional[int] = None,
               name: Optional[str] = None) -> "Workload":
        """A smaller workload with the same structure: fewer prompts per agent and/or
        shorter lengths, used where the float64 checker must finish in seconds."""
        ags = tuple(Agent(max(1, a.prompts // prompts_div), a.G,
                          a.prompt_len.scaled(len_div), a.gen_len.scaled(len_div))
                    for a in self.agents)
        return replace(self, agents=ags, vocab=self.vocab if vocab is None else vocab,
                       name=name or f"{self.name}/p{prompts_div}l{len_div}")


_K = 1024
_SEED0 = 2048   # the paper fixes its seed to 2048 (Section 8.1); one seed per workload from there

WORKLOADS = {
    # 2 agents x 2 prompts x G=4, 8 q heads / 2 kv heads
    "tiny": Workload("tiny", 8, 2,
                     tuple(Agent(2, 4, const(256), uniform(1, 128)) for _ in range(2)),
                     seed=_SEED0 + 1, vocab=4096, logit_sigma=2.0),
    # Qwen-7B-shaped layer: 4 agents x 64 prompts x G=8
    "qwen7b": Workload("qwen7b", 28, 4,
                       tuple(Agent(64, 8, uniform(512, 2048), lognormal(med, 0.8, 8192))
                             for med in (256, 512, 1024, 2048)),
                       seed=_SEED0 + 2, vocab=152064, logit_sigma=3.0),
    # inter-agent skew: one reasoner agent with very long generations, seven short ones
    "skew": Workload("skew", 28, 4,
                     (Agent(32, 8, const(1024), uniform(12 * _K, 16 * _K)),)
                     + tuple(Agent(64, 8, const(1024), uniform(16, 256)) for _ in range(7)),
                     seed=_SEED0 + 3),
    # prefix-dominated group sampling
    "prefix": Workload("prefix", 28, 4, (Agent(64, 32, const(4096), uniform(1, 64)),),
                       seed=_SEED0 + 4),
    # Qwen-32B-shaped layer, long context
    "long32b": Workload("long32b", 64, 8,
                        tuple(Agent(16, 4, const(8192), uniform(8 * _K, 24 * _K))
                              for _ in range(4)),
                        seed=_SEED0 + 5, vocab=152064, logit_sigma=3.0),
}


# --------------------------------------------------------------------------------------
# lengths and block tables
# --------------------------------------------------------------------------------------
@dataclass
class Lengths:
    prefix_lens: np.ndarray    # int32 [NG]
    suffix_lens: np.ndarray    # int32 [NS]
    group_of_seq: np.ndarray   # int32 [NS]
    agent_of_group: np.ndarray  # int32 [NG]


def draw_lengths(w: Workload, rng: np.random.Generator) -> Lengths:
    pl, sl, gos, aog = [], [], [], []
    g0 = 0
    for ai, a in enumerate(w.agents):
        p = a.prompt_len.draw(rng, a.prompts)
        s = a.gen_len.draw(rng, a.prompts * a.G)
        pl.append(p)
        sl.append(s)
        gos.append(np.repeat(np.arange(g0, g0 + a.prompts), a.G))
        aog.append(np.full(a.prompts, ai))
        g0 += a.prompts
    return Lengths(np.concatenate(pl).astype(np.int32), np.concatenate(sl).astype(np.int32),
                   np.concatenate(gos).astype(np.int32), np.concatenate(aog).astype(np.int32))


def _pages_for(lens: np.ndarray) -> np.ndarray:
    return (lens.astype(np.int64) + PAGE - 1) // PAGE


def build_block_tables(lens: Lengths, rng: np.random.Generator, spare_frac: float = 0.05,
                       min_cols: int = 1):
    """Assign every logical page a distinct physical page from a random permutation.

    Returns (prefix_table [NG, max_prefix_pages], suffix_table [NS, max_suffix_pages],
    num_pages, used_mask[num_pages]).  Unused table entries are -1.  A suffix always
    starts on a fresh page (slot 0), also when the prefix ends in a partial page.
    """
    npp, nsp = _pages_for(lens.prefix_lens), _pages_for(lens.suffix_lens)
    total = int(npp.sum() + nsp.sum())
    num_pages = max(1, int(math.ceil(total * (1.0 + spare_frac))) + (1 if spare_frac > 0 else 0))
    perm = rng.permutation(num_pages).astype(np.int32)
    mpp = max(min_cols, int(npp.max()) if len(npp) else 0)
    msp = max(min_cols, int(nsp.max()) if len(nsp) else 0)
    ptab = np.full((len(npp), mpp), -1, dtype=np.int32)
    stab = np.full((len(nsp), msp), -1, dtype=np.int32)
    cur = 0
    for g, n in enumerate(npp):
        ptab[g, :n] = perm[cur:cur + n]
        cur += int(n)
    for s, n in enumerate(nsp):
        stab[s, :n] = perm[cur:cur + n]
        cur += int(n)
    used = np.zeros(num_pages, dtype=bool)
    used[perm[:cur]] = True
    return ptab, stab, num_pages, used


# --------------------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------------------
def randn_bf16(shape, sigma: float, gen: torch.Generator, device, chunk_elems: int = 1 << 27):
    """N(0, sigma) drawn in fp32 and rounded once (RNE) to bf16, in bounded chunks."""
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=torch.bfloat16, device=device)
    for o in range(0, n, chunk_elems):
        m = min(chunk_elems, n - o)
        x = torch.randn(m, generator=gen, device=device, dtype=torch.float32)
        if sigma != 1.0:
            x.mul_(sigma)
        out[o:o + m] = x.to(torch.bfloat16)
    return out.view(*shape)


@dataclass
class AttnInputs:
    Hq: int
    Hkv: int
    num_pages: int
    q: torch.Tensor                    # bf16 [NS, Hq, D]
    k_pages: torch.Tensor              # bf16 [num_pages, Hkv, PAGE, D]
    v_pages: torch.Tensor              # bf16 [num_pages, Hkv, D, PAGE]
    prefix_block_table: torch.Tensor   # int32 [NG, max_prefix_pages]
    suffix_block_table: torch.Tensor   # int32 [NS, max_suffix_pages]
    prefix_lens: torch.Tensor          # int32 [NG]
    suffix_lens: torch.Tensor          # int32 [NS]
    group_of_seq: torch.Tensor         # int32 [NS]
    scale: float
    agent_of_group: Optional[np.ndarray] = None

    @property
    def num_seqs(self): return int(self.suffix_lens.shape[0])
    @property
    def num_groups(self): return int(self.prefix_lens.shape[0])

    def unique_kv_tokens(self) -> Tuple[int, int]:
        """(prefix tokens counted once per group, suffix tokens counted once per sequence)."""
        return int(self.prefix_lens.sum().item()), int(self.suffix_lens.sum().item())

    def kv_bytes_per_token(self) -> int:
        return 2 * self.Hkv * D * 2

    def to(self, device) -> "AttnInputs":
        kw = {}
        for f in ("q", "k_pages", "v_pages", "prefix_block_table", "suffix_block_table",
                  "prefix_lens", "suffix_lens", "group_of_seq"):
            kw[f] = getattr(self, f).to(device)
        return replace(self, **kw)


def poison_unused(k_pages, v_pages, ptab, stab, plens, slens, used_mask, value=float("nan")):
    """Overwrite every KV location no valid token owns (free pages, and the slots past the
    end of a partially filled last page) so that any read of them shows up in the result."""
    dev = k_pages.device
    free = torch.from_numpy(np.nonzero(~used_mask)[0]).to(dev)
    if free.numel():
        k_pages[free] = value
        v_pages[free] = value
    for tab, lens in ((ptab, plens), (stab, slens)):
        lens = np.asarray(lens, dtype=np.int64)
        rem = lens % PAGE
        rows = np.nonzero(rem)[0]
        if rows.size == 0:
            continue
        pages = tab[rows, lens[rows] // PAGE]
        assert (pages >= 0).all()
        pg = torch.from_numpy(pages.astype(np.int64)).to(dev)
        keep = (torch.arange(PAGE, device=dev)[None, :]
                < torch.from_numpy(rem[rows]).to(dev)[:, None])          # [n, PAGE]
        kk = k_pages[pg]
        kk[~keep[:, None, :, None].expand_as(kk)] = value
        k_pages[pg] = kk
        vv = v_pages[pg]
        vv[~keep[:, None, None, :].expand_as(vv)] = value
        v_pages[pg] = vv


def build_attn_inputs(w: Workload, device="cpu", seed: Optional[int] = None, poison: bool = True,
                      spare_frac: float = 0.05, lengths: Optional[Lengths] = None) -> AttnInputs:
    seed = w.seed if seed is None else seed
    rng = np.random.default_rng(seed)
    lens = lengths if lengths is not None else draw_lengths(w, rng)
    ptab, stab, num_pages, used = build_block_tables(lens, rng, spare_frac)
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    NS = len(lens.suffix_lens)
    q = randn_bf16((NS, w.Hq, D), 1.0, gen, device)
    k_pages = randn_bf16((num_pages, w.Hkv, PAGE, D), 1.0, gen, device)
    v_pages = randn_bf16((num_pages, w.Hkv, D, PAGE), 1.0, gen, device)
    if poison:
        poison_unused(k_pages, v_pages, ptab, stab, lens.prefix_lens, lens.suffix_lens, used)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return AttnInputs(w.Hq, w.Hkv, num_pages, q, k_pages, v_pages, t(ptab), t(stab),
                      t(lens.prefix_lens), t(lens.suffix_lens), t(lens.group_of_seq),
                      scale=1.0 / math.sqrt(D), agent_of_group=lens.agent_of_group)


def extract_subproblem(inp: AttnInputs, seq_ids: Sequence[int]) -> AttnInputs:
    """A self-contained CPU copy of the chosen sequences: their groups, their pages
    (renumbered compactly, in first-use order) and their queries.  Pure indexing; used to
    hand a sample of a large GPU-resident workload to the CPU checker."""
    seq_ids = [int(s) for s in seq_ids]
    gos = inp.group_of_seq.cpu().numpy()
    plens = inp.prefix_lens.cpu().numpy()
    slens = inp.suffix_lens.cpu().numpy()
    groups = sorted({int(gos[s]) for s in seq_ids})
    gmap = {g: i for i, g in enumerate(groups)}
    ptab_rows = inp.prefix_block_table[torch.tensor(groups, device=inp.prefix_block_table.device)].cpu().numpy()
    stab_rows = inp.suffix_block_table[torch.tensor(seq_ids, device=inp.suffix_block_table.device)].cpu().numpy()
    new_ptab = np.full_like(ptab_rows, -1)
    new_stab = np.full_like(stab_rows, -1)
    phys = []
    for i, g in enumerate(groups):
        n = (int(plens[g]) + PAGE - 1) // PAGE
        new_ptab[i, :n] = np.arange(len(phys), len(phys) + n)
        phys.extend(ptab_rows[i, :n].tolist())
    for i, s in enumerate(seq_ids):
        n = (int(slens[s]) + PAGE - 1) // PAGE
        new_stab[i, :n] = np.arange(len(phys), len(phys) + n)
        phys.extend(stab_rows[i, :n].tolist())
    if not phys:
        phys = [0]
    idx = torch.tensor(phys, dtype=torch.int64, device=inp.k_pages.device)
    t = lambda a, dt=np.int32: torch.from_numpy(np.ascontiguousarray(a.astype(dt)))
    sid = torch.tensor(seq_ids, dtype=torch.int64, device=inp.q.device)
    return AttnInputs(inp.Hq, inp.Hkv, len(phys), inp.q[sid].cpu(), inp.k_pages[idx].cpu(),
                      inp.v_pages[idx].cpu(), t(new_ptab), t(new_stab),
                      t(plens[groups]), t(slens[seq_ids]),
                      t(np.array([gmap[int(gos[s])] for s in seq_ids])), inp.scale)


# --------------------------------------------------------------------------------------
# log-probability inputs
# --------------------------------------------------------------------------------------
@dataclass
class LogprobInputs:
    logits: torch.Tensor       # bf16 [rows, vocab], row stride = vocab
    tokens: torch.Tensor       # int32 [rows]
    temperature: float

    def to(self, device):
        return replace(self, logits=self.logits.to(device), tokens=self.tokens.to(device))


def build_logprob_inputs(rows: int, vocab: int, sigma: float, seed: int, device="cpu",
                         temperature: float = 1.0) -> LogprobInputs:
    """Random logits; token ids uniform over the vocabulary except three forced rows:
    row 0 picks id 0, row 1 picks the last id, row 2 picks that row's largest logit."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed + 7919)
    logits = randn_bf16((rows, vocab), sigma, gen, device)
    rng = np.random.default_rng(seed + 104729)
    tok = rng.integers(0, vocab, size=rows, dtype=np.int64)
    if rows > 0:
        tok[0] = 0
    if rows > 1:
        tok[1] = vocab - 1
    if rows > 2:
        tok[2] = int(torch.argmax(logits[2].float()).item())
    return LogprobInputs(logits, torch.from_numpy(tok.astype(np.int32)).to(device), temperature)


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """The raw 16-bit patterns of a bf16 tensor as a uint16 numpy array (CPU copy)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


# --------------------------------------------------------------------------------------
# prompt (prefill) inputs
# --------------------------------------------------------------------------------------
@dataclass
class PrefillInputs:
    Hq: int
    Hkv: int
    num_pages: int
    q: torch.Tensor                    # bf16 [NT, Hq, D]: the query tokens of all groups, group after group
    k_new: torch.Tensor                # bf16 [NT, Hkv, D]: keys of the same tokens (for the prompt scatter)
    v_new: torch.Tensor                # bf16 [NT, Hkv, D]
    k_pages: torch.Tensor              # bf16 [num_pages, Hkv, PAGE, D]; every position < pos0 + n holds data
    v_pages: torch.Tensor              # bf16 [num_pages, Hkv, D, PAGE]
    prefix_block_table: torch.Tensor   # int32 [NG, max_prefix_pages]
    q_start: torch.Tensor              # int32 [NG + 1]
    q_pos0: torch.Tensor               # int32 [NG]
    scale: float

    @property
    def num_tokens(self): return int(self.q.shape[0])
    @property
    def num_groups(self): return int(self.q_pos0.shape[0])

    def to(self, device) -> "PrefillInputs":
        kw = {f: getattr(self, f).to(device) for f in ("q", "k_new", "v_new", "k_pages", "v_pages",
                                                       "prefix_block_table", "q_start", "q_pos0")}
        return replace(self, **kw)

    def causal_pairs(self) -> int:
        """Number of (query token, visible key) pairs: the unit of the operation's work."""
        n = np.diff(self.q_start.cpu().numpy().astype(np.int64))
        p0 = self.q_pos0.cpu().numpy().astype(np.int64)
        return int((n * p0 + n * (n + 1) // 2).sum())


def build_prefill_inputs(Hq: int, Hkv: int, chunk_lens: Sequence[int], pos0: Sequence[int], device="cpu",
                         seed: int = 0, poison: bool = True, spare_frac: float = 0.05,
                         extra_cols: int = 0) -> PrefillInputs:
    """Group g brings chunk_lens[g] query tokens at positions pos0[g] .. of its prompt.  Pages are
    a random permutation; every cache position below pos0[g] + chunk_lens[g] holds N(0,1) data
    (so attention can be run without the scatter), everything else NaN when `poison`."""
    rng = np.random.default_rng(seed)
    n = np.asarray(chunk_lens, dtype=np.int64)
    p0 = np.asarray(pos0, dtype=np.int64)
    NG = len(n)
    total = p0 + n
    npages = (total + PAGE - 1) // PAGE
    used_pages = int(npages.sum())
    num_pages = max(1, int(math.ceil(used_pages * (1.0 + spare_frac))) + (1 if spare_frac > 0 else 0))
    perm = rng.permutation(num_pages).astype(np.int32)
    mpp = max(1, int(npages.max()) if NG else 1) + extra_cols
    ptab = np.full((NG, mpp), -1, dtype=np.int32)
    cur = 0
    for g in range(NG):
        ptab[g, :npages[g]] = perm[cur:cur + npages[g]]
        cur += int(npages[g])
    used = np.zeros(num_pages, dtype=bool)
    used[perm[:cur]] = True
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    NT = int(n.sum())
    q = randn_bf16((NT, Hq, D), 1.0, gen, device)
    k_new = randn_bf16((NT, Hkv, D), 1.0, gen, device)
    v_new = randn_bf16((NT, Hkv, D), 1.0, gen, device)
    k_pages = randn_bf16((num_pages, Hkv, PAGE, D), 1.0, gen, device)
    v_pages = randn_bf16((num_pages, Hkv, D, PAGE), 1.0, gen, device)
    if poison:
        empty = np.zeros((0, 1), dtype=np.int32)
        poison_unused(k_pages, v_pages, ptab, empty, total, np.zeros(0, dtype=np.int64), used)
    q_start = np.zeros(NG + 1, dtype=np.int32)
    q_start[1:] = np.cumsum(n)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(device)
    return PrefillInputs(Hq, Hkv, num_pages, q, k_new, v_new, k_pages, v_pages, t(ptab), t(q_start),
                         t(p0.astype(np.int32)), scale=1.0 / math.sqrt(D))


def model_param_sizes(Hq: int, Hkv: int, vocab: int, head_dim: int = 128):
    """Element counts of the parameter tensors of a decoder of the workload's attention shape, in
    checkpoint order: embedding, per layer (q, k, v projections with biases, output projection,
    gate / up / down projections, two norms), final norm, output head.  Hidden size Hq * head_dim;
    the layer count and MLP width are those of the 7B (Hq 28) and 32B (Hq 64 -> hidden 5120 there,
    kept at Hq * head_dim here) members of the model family the paper trains; other shapes scale them."""
    hidden = Hq * head_dim
    kv = Hkv * head_dim
    layers, mlp = (28, 18944) if Hq <= 28 else (64, 27648)
    sizes = [vocab * hidden]
    for _ in range(layers):
        sizes += [hidden * hidden, hidden, kv * hidden, kv, kv * hidden, kv, hidden * hidden,
                  mlp * hidden, mlp * hidden, hidden * mlp, hidden, hidden]
    sizes += [hidden, vocab * hidden]
    return sizes
