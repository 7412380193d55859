"""Seeded synthetic inputs for the KV delta-coding path.

This module only *draws inputs*: candidate KV vectors, top-k next-token
probabilities, the sampled true candidate and the noisy actual KV vectors.  It
contains none of the coding path's arithmetic (no prediction, residual,
quantiser, histogram or entropy coder) and imports neither the device library
nor the CPU oracle, so that both can be fed the very same bits.

The recipe follows the five benchmark configurations: candidates ~ N(0,1)
stored as fp16; one probability row per (session, position) taken from the
head of a Zipf(s = 1.1) distribution over a 50,000-token vocabulary whose
temperature is set so that the *full* distribution has the requested
perplexity; the true candidate is sampled from the renormalised top-k row; the
actual vector is that candidate plus N(0, sigma^2) noise, rounded to fp16.

A configuration with `misses` also draws positions whose true token is none of
the k candidates, with the probability the top k leave (1 - their sum): there
`chosen` is -1 and the actual vectors are fresh N(0,1) draws in every layer and
head (plus the same noise).
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np
import torch

VOCAB = 50_000
ZIPF_S = 1.1

CONFIGS = {
    # name: sessions, layers, KV heads, head dim, positions, candidates, perplexity, noise, step, seed
    "tiny":    dict(S=1,  L=2,  H=4,  d=64,  n=512,   k=4, pp=12.0, sigma=0.05, delta=0.02, seed=0),
    "llama8b": dict(S=1,  L=32, H=8,  d=128, n=4096,  k=8, pp=15.0, sigma=0.05, delta=0.02, seed=1),
    "long":    dict(S=1,  L=32, H=8,  d=128, n=32768, k=4, pp=10.0, sigma=0.03, delta=0.02, seed=2),
    "70b":     dict(S=1,  L=80, H=64, d=128, n=2048,  k=4, pp=20.0, sigma=0.08, delta=0.03, seed=3),
    "batched": dict(S=64, L=32, H=8,  d=128, n=2048,  k=8, pp=(5.0, 40.0), sigma=(0.01, 0.2),
                    delta=0.02, seed=4),
    # the paper's suggested k = 20 (Sec. 7.1), with the top-k misses a real model would have
    "miss20":  dict(S=1,  L=32, H=8,  d=128, n=4096,  k=20, pp=15.0, sigma=0.05, delta=0.02, seed=5,
                    misses=True),
}


def zipf_topk_probs(perplexity: float, k: int, vocab: int = VOCAB, s: float = ZIPF_S) -> np.ndarray:
    """Head of the distribution p_j ~ j^(-s/T), j = 1..vocab, with T chosen by
    bisection so that exp(entropy) equals `perplexity`.  Returns the k largest
    probabilities, raw (they sum to less than one)."""
    ranks = np.arange(1, vocab + 1, dtype=np.float64)
    logr = np.log(ranks)

    def dist(T):
        logits = -(s / T) * logr
        logits -= logits.max()
        p = np.exp(logits)
        return p / p.sum()

    def ppl(T):
        p = dist(T)
        nz = p > 0
        return float(np.exp(-(p[nz] * np.log(p[nz])).sum()))

    lo, hi = 0.02, 200.0
    if not (ppl(lo) < perplexity < ppl(hi)):
        raise ValueError(f"perplexity {perplexity} out of reach for vocab {vocab}")
    for _ in range(200):
        mid = 0.5 * (lo + hi)
        if ppl(mid) < perplexity:
            lo = mid
        else:
            hi = mid
    return dist(0.5 * (lo + hi))[:k].copy()


@dataclasses.dataclass
class Workload:
    name: str
    S: int
    L: int
    H: int
    n: int
    k: int
    d: int
    delta: float
    qmax: int
    sigma: np.ndarray          # [S] noise level of each session
    perplexity: np.ndarray     # [S]
    probs: torch.Tensor        # fp32 [S, n, k], raw top-k probabilities
    chosen: torch.Tensor       # int64 [S, n], index of the true candidate (-1: none of them)
    cand_k: torch.Tensor       # fp16, logical [S, L, H, n, k, d] (any strides, d contiguous)
    cand_v: torch.Tensor
    act_k: torch.Tensor        # fp16 [S, L, H, n, d]
    act_v: torch.Tensor

    @property
    def n_streams(self) -> int:
        return self.S * self.L * self.H

    @property
    def syms_per_stream(self) -> int:
        return 2 * self.n * self.d

    @property
    def kv_bytes(self) -> int:
        """Size of the fp16 KV cache being coded (K and V)."""
        return 2 * self.n_streams * self.n * self.d * 2


def _alloc_cand(S, L, H, n, k, d, layout, device):
    if layout == "lhnkd":      # storage order = logical order
        return torch.empty((S, L, H, n, k, d), dtype=torch.float16, device=device)
    if layout == "lnkhd":      # heads innermost but one, as some KV caches store them
        return torch.empty((S, L, n, k, H, d), dtype=torch.float16, device=device).permute(0, 1, 4, 2, 3, 5)
    raise ValueError(layout)


def make_workload(name: str = "tiny", device="cpu", layout: str = "lhnkd",
                  overrides: Optional[dict] = None, one_hot: bool = False,
                  random_rows: bool = False) -> Workload:
    """Draw one configuration.  `overrides` replaces entries of CONFIGS[name]
    (e.g. a smaller S or n for a test).  `one_hot` puts all probability on the
    chosen candidate and sets the noise to zero.  `random_rows` replaces the
    (position-independent) Zipf row by an independent random row per position,
    so that a row-broadcasting mistake cannot hide."""
    cfg = dict(CONFIGS[name])
    if overrides:
        cfg.update(overrides)
    S, L, H, n, k, d = (cfg[x] for x in ("S", "L", "H", "n", "k", "d"))
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(cfg["seed"]))
    host = np.random.default_rng(int(cfg["seed"]))

    def per_session(v):
        if isinstance(v, tuple):
            return host.uniform(v[0], v[1], size=S)
        return np.full(S, float(v))

    pp = per_session(cfg["pp"])
    sigma = per_session(cfg["sigma"])

    rows = np.stack([zipf_topk_probs(float(pp[s]), k) for s in range(S)])       # [S, k]
    probs = torch.from_numpy(rows.astype(np.float32)).to(dev)[:, None, :].expand(S, n, k).contiguous()
    if random_rows:
        g = torch.rand((S, n, k), generator=gen, device=dev, dtype=torch.float32)
        probs = (-torch.log1p(-g)) * probs          # exponential variates scaled by the Zipf head
        probs = probs / probs.sum(-1, keepdim=True) * float(rows[0].sum())
        probs = probs.contiguous()
    sel = probs / probs.sum(-1, keepdim=True)
    chosen = torch.multinomial(sel.reshape(S * n, k), 1, generator=gen).reshape(S, n)
    miss = None
    if cfg.get("misses"):
        left = (1.0 - probs.sum(-1)).clamp_(0.0, 1.0)                                  # [S, n]
        miss = torch.rand((S, n), generator=gen, device=dev, dtype=torch.float32) < left
    if one_hot:
        probs = torch.zeros_like(probs).scatter_(2, chosen[..., None], 1.0)
        sigma = np.zeros(S)

    cand_k = _alloc_cand(S, L, H, n, k, d, layout, dev)
    cand_v = _alloc_cand(S, L, H, n, k, d, layout, dev)
    act_k = torch.empty((S, L, H, n, d), dtype=torch.float16, device=dev)
    act_v = torch.empty((S, L, H, n, d), dtype=torch.float16, device=dev)
    for s in range(S):
        idx = chosen[s][None, :, None, None].expand(H, n, 1, d)
        for l in range(L):
            for cand, act in ((cand_k, act_k), (cand_v, act_v)):
                c = torch.randn((H, n, k, d), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                z = torch.randn((H, n, d), generator=gen, device=dev, dtype=torch.float32)
                true = c.gather(2, idx).squeeze(2).to(torch.float32)
                if miss is not None:
                    fresh = torch.randn((H, n, d), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
                    true = torch.where(miss[s][None, :, None], fresh.to(torch.float32), true)
                cand[s, l].copy_(c)
                act[s, l].copy_((true + float(sigma[s]) * z).to(torch.float16))
    if miss is not None:
        chosen = torch.where(miss, torch.full_like(chosen, -1), chosen)
    return Workload(name=name, S=S, L=L, H=H, n=n, k=k, d=d, delta=float(cfg["delta"]), qmax=127,
                    sigma=sigma, perplexity=pp, probs=probs, chosen=chosen,
                    cand_k=cand_k, cand_v=cand_v, act_k=act_k, act_v=act_v)


def random_bytes(n_streams: int, syms_per_stream: int, seed: int, kind: str = "gauss",
                 device="cpu") -> torch.Tensor:
    """Byte streams for exercising the histogram / table / rANS calls on their own.
    kind: 'gauss' (discretised normal around 127, like quantised residuals),
    'uniform' (all 256 values), 'constant', 'two' (one rare symbol)."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    shape = (n_streams, syms_per_stream)
    if kind == "gauss":
        x = torch.randn(shape, generator=gen, device=device) * 20.0 + 127.0
        return x.round().clamp_(0, 255).to(torch.uint8)
    if kind == "uniform":
        return torch.randint(0, 256, shape, generator=gen, device=device, dtype=torch.int32).to(torch.uint8)
    if kind == "constant":
        return torch.full(shape, 127, dtype=torch.uint8, device=device)
    if kind == "two":
        r = torch.rand(shape, generator=gen, device=device)
        return torch.where(r < 1e-3, 255, 127).to(torch.uint8)
    raise ValueError(kind)


# ------------------------------------------------------------------------------------------------
# Inputs of the linear-embedding predictor: a full-vocabulary distribution per position, an embedding
# table, one matrix per layer and a bias of the KV cache's shape; the actual vectors are linear in the
# true token's embedding plus noise.

LINEAR_CONFIGS = {
    # name: sessions, layers, KV heads, head dim, positions, embedding dim, vocabulary, perplexity, noise, step, seed
    "tiny":    dict(S=1, L=2,  H=2, d=64,  n=256,  m=256,  V=1024,  pp=12.0, sigma=0.05, delta=0.02, seed=10),
    "llama8b": dict(S=1, L=32, H=8, d=128, n=4096, m=4096, V=50016, pp=15.0, sigma=0.05, delta=0.02, seed=11),
}


@dataclasses.dataclass
class LinearWorkload:
    name: str
    S: int
    L: int
    H: int
    n: int
    d: int
    m: int
    V: int
    delta: float
    qmax: int
    sigma: float
    probs_full: torch.Tensor   # fp16 [S*n, V]
    embed_t: torch.Tensor      # fp16 [m, V]
    A: torch.Tensor            # fp16 [L, H, 2, d, m]
    bias_k: torch.Tensor       # fp16 [S, L, H, n, d]
    bias_v: torch.Tensor
    act_k: torch.Tensor        # fp16 [S, L, H, n, d]
    act_v: torch.Tensor
    token: torch.Tensor        # int64 [S*n] the true token of every position

    @property
    def kv_bytes(self) -> int:
        return 2 * self.S * self.L * self.H * self.n * self.d * 2


def zipf_full_probs(perplexity: float, vocab: int, s: float = ZIPF_S) -> np.ndarray:
    """The whole distribution p_j ~ j^(-s/T) with exp(entropy) = perplexity (see zipf_topk_probs)."""
    return zipf_topk_probs(perplexity, vocab, vocab=vocab, s=s)


def make_linear_workload(name: str = "tiny", device="cpu", overrides: Optional[dict] = None,
                         one_hot: bool = False) -> LinearWorkload:
    """`one_hot` puts all probability on the true token and sets the noise to zero."""
    cfg = dict(LINEAR_CONFIGS[name])
    if overrides:
        cfg.update(overrides)
    S, L, H, d, n, m, V = (cfg[x] for x in ("S", "L", "H", "d", "n", "m", "V"))
    dev = torch.device(device)
    gen = torch.Generator(device=dev)
    gen.manual_seed(int(cfg["seed"]))
    sigma = 0.0 if one_hot else float(cfg["sigma"])
    zipf = torch.from_numpy(zipf_full_probs(float(cfg["pp"]), V).astype(np.float32)).to(dev)
    rows = S * n
    # every position ranks the vocabulary its own way: a per-position rotation of the Zipf row
    shift = torch.randint(0, V, (rows,), generator=gen, device=dev)
    probs_full = torch.empty((rows, V), dtype=torch.float16, device=dev)
    token = torch.empty(rows, dtype=torch.int64, device=dev)
    ar = torch.arange(V, device=dev)
    for r0 in range(0, rows, 512):
        idx = (ar[None, :] + shift[r0:r0 + 512, None]) % V
        p = zipf[idx]
        token[r0:r0 + 512] = torch.multinomial(p, 1, generator=gen).squeeze(1)
        if one_hot:
            p = torch.zeros_like(p).scatter_(1, token[r0:r0 + 512, None], 1.0)
        probs_full[r0:r0 + 512] = p.to(torch.float16)
    embed_t = torch.randn((m, V), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
    A = (torch.randn((L, H, 2, d, m), generator=gen, device=dev, dtype=torch.float32) / float(np.sqrt(m))).to(torch.float16)
    bias_k = torch.randn((S, L, H, n, d), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
    bias_v = torch.randn((S, L, H, n, d), generator=gen, device=dev, dtype=torch.float32).to(torch.float16)
    act_k = torch.empty_like(bias_k)
    act_v = torch.empty_like(bias_v)
    e_true = embed_t[:, token].t().to(torch.float32).reshape(S, n, m)              # [S, n, m]
    for s in range(S):
        for l in range(L):
            lin = e_true[s] @ A[l].reshape(2 * H * d, m).to(torch.float32).t()      # [n, 2Hd]
            lin = lin.reshape(n, H, 2, d).permute(1, 2, 0, 3)                       # [H, 2, n, d]
            for c, (bias, act) in enumerate(((bias_k, act_k), (bias_v, act_v))):
                z = torch.randn((H, n, d), generator=gen, device=dev, dtype=torch.float32)
                act[s, l].copy_((bias[s, l].to(torch.float32) + lin[:, c] + sigma * z).to(torch.float16))
    return LinearWorkload(name=name, S=S, L=L, H=H, n=n, d=d, m=m, V=V, delta=float(cfg["delta"]), qmax=127,
                          sigma=sigma, probs_full=probs_full, embed_t=embed_t, A=A, bias_k=bias_k, bias_v=bias_v,
                          act_k=act_k, act_v=act_v, token=token)
