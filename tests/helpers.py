"""Test-side helpers: turn logical (unpaged) K/V lists into the paged ABI layout, and an
independently written brute-force attention used to pin the checker."""
from __future__ import annotations

import numpy as np
import torch

PAGE = 16
D = 128


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_f64(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


class Paged:
    """Pages logical K/V (already bf16-representable float arrays) with a random physical
    page order, extra free pages and NaN in every location no token owns."""

    def __init__(self, prefixK, prefixV, sufK, sufV, group_of_seq, Hkv, rng, spare=3,
                 poison=np.nan, order="random"):
        # prefixK[g]: [P_g, Hkv, D]; sufK[s]: [S_s, Hkv, D]
        NG, NS = len(prefixK), len(sufK)
        npp = [(-(-k.shape[0] // PAGE)) for k in prefixK]
        nsp = [(-(-k.shape[0] // PAGE)) for k in sufK]
        total = sum(npp) + sum(nsp)
        self.num_pages = total + spare
        if order == "random":
            perm = rng.permutation(self.num_pages)
        elif order == "identity":
            perm = np.arange(self.num_pages)
        else:
            perm = np.asarray(order)
        K = np.full((self.num_pages, Hkv, PAGE, D), poison, dtype=np.float32)
        V = np.full((self.num_pages, Hkv, D, PAGE), poison, dtype=np.float32)
        mpp, msp = max([1] + npp), max([1] + nsp)
        ptab = np.full((NG, mpp), -1, dtype=np.int32)
        stab = np.full((NS, msp), -1, dtype=np.int32)
        cur = 0
        for tab, Ks, Vs, cnt in ((ptab, prefixK, prefixV, npp), (stab, sufK, sufV, nsp)):
            for i, (k, v) in enumerate(zip(Ks, Vs)):
                for p in range(cnt[i]):
                    page = int(perm[cur]); cur += 1
                    tab[i, p] = page
                    n = min(PAGE, k.shape[0] - p * PAGE)
                    K[page, :, :n, :] = np.transpose(k[p * PAGE:p * PAGE + n], (1, 0, 2))
                    V[page, :, :, :n] = np.transpose(v[p * PAGE:p * PAGE + n], (1, 2, 0))
        self.k_bits, self.v_bits = to_bf16_bits(K), to_bf16_bits(V)
        self.ptab, self.stab = ptab, stab
        self.plens = np.array([k.shape[0] for k in prefixK], dtype=np.int32)
        self.slens = np.array([k.shape[0] for k in sufK], dtype=np.int32)
        self.gos = np.asarray(group_of_seq, dtype=np.int32)
        self.Hkv = Hkv


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float array -> nearest bf16 values, returned as float32."""
    return bits_to_f64(to_bf16_bits(x)).astype(np.float32)


def random_logical(rng, NG, G, P_list, S_list, Hq, Hkv, sigma=1.0):
    """Random bf16-representable logical problem.  Returns dict of lists/arrays."""
    NS = NG * G
    pk = [bf16_round(rng.standard_normal((P_list[g], Hkv, D)) * sigma) for g in range(NG)]
    pv = [bf16_round(rng.standard_normal((P_list[g], Hkv, D)) * sigma) for g in range(NG)]
    sk = [bf16_round(rng.standard_normal((S_list[s], Hkv, D)) * sigma) for s in range(NS)]
    sv = [bf16_round(rng.standard_normal((S_list[s], Hkv, D)) * sigma) for s in range(NS)]
    q = bf16_round(rng.standard_normal((NS, Hq, D)))
    gos = np.repeat(np.arange(NG), G).astype(np.int32)
    return dict(pk=pk, pv=pv, sk=sk, sv=sv, q=q, gos=gos)


def brute_force(q, pk, pv, sk, sv, gos, scale, Hq, Hkv):
    """Unpaged softmax attention written with whole-array numpy float64 operations."""
    NS = q.shape[0]
    R = Hq // Hkv
    out = np.zeros((NS, Hq, D))
    for s in range(NS):
        g = int(gos[s])
        Kc = np.concatenate([pk[g], sk[s]], axis=0).astype(np.float64)   # [L, Hkv, D]
        Vc = np.concatenate([pv[g], sv[s]], axis=0).astype(np.float64)
        if Kc.shape[0] == 0:
            continue
        Kh = np.repeat(Kc, R, axis=1)                                    # [L, Hq, D]
        Vh = np.repeat(Vc, R, axis=1)
        logits = np.einsum("hc,lhc->hl", q[s].astype(np.float64), Kh) * scale
        logits -= logits.max(axis=1, keepdims=True)
        w = np.exp(logits)
        w /= w.sum(axis=1, keepdims=True)
        out[s] = np.einsum("hl,lhc->hc", w, Vh)
    return out
