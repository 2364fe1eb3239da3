"""Seeded synthetic inputs for the replayed MoE layer.

This module only draws random tensors of the right shape and distribution and
rounds them once to the layer's activation dtype.  It holds none of the
method's arithmetic: logits, records, gates and everything after them are
computed by whoever consumes these tensors.

The shapes stand in for one MoE layer of the 128-expert / top-8 model the paper
trains (arxiv 2510.11370, Sections 3.1 and 5.1); its weights and rollouts are
not available, so value distributions are synthetic:
x ~ N(0,1), W_r ~ N(0,1/d) (logits ~ N(0,1)), expert weights ~ N(0,0.02^2),
inference-logit noise ~ N(0,sigma^2), upstream gradient dy ~ N(0,1), and an
optional router bias b_e = -s*ln(rank_e) with seeded ranks, which skews expert
popularity towards a Zipf(s) law.
"""
from dataclasses import dataclass, replace
from typing import Optional

import torch


@dataclass(frozen=True)
class LayerShape:
    T: int
    d: int
    E: int
    K: int
    F: int
    act: str = "bf16"          # "bf16" or "f32": dtype the tensors are rounded to
    sigma: float = 0.01        # std of the inference-logit noise
    zipf_s: Optional[float] = None
    seed: int = 0
    layers: int = 1

    def with_(self, **kw):
        return replace(self, **kw)


# The five benchmark configurations, smallest first (the second and third are the ones throughput is quoted on).
CONFIGS = {
    "tiny_f32": LayerShape(T=256, d=128, E=8, K=2, F=256, act="f32", sigma=0.05, seed=0),
    "fwd_4k": LayerShape(T=4096, d=2048, E=128, K=8, F=768, sigma=0.01, seed=1),
    "fwdbwd_16k": LayerShape(T=16384, d=2048, E=128, K=8, F=768, sigma=0.01, seed=2),
    "stack48_128k": LayerShape(T=131072, d=2048, E=128, K=8, F=768, sigma=0.01, seed=3,
                               layers=48),
    "zipf_64k": LayerShape(T=65536, d=2048, E=128, K=8, F=768, sigma=0.01, zipf_s=1.2,
                           seed=4),
}

_TENSOR_IDS = {"x": 1, "Wr": 2, "Wg": 3, "Wu": 4, "Wd": 5, "noise": 6, "dy": 7, "ranks": 8}


def _gen(shape: LayerShape, name: str, device, layer: int):
    g = torch.Generator(device=device)
    g.manual_seed(1000003 * shape.seed + 101 * layer + _TENSOR_IDS[name])
    return g


def _round(t: torch.Tensor, act: str) -> torch.Tensor:
    """Round once to the activation dtype; the result is float32 holding those values."""
    if act == "bf16":
        return t.to(torch.bfloat16).to(torch.float32)
    return t


def draw(shape: LayerShape, name: str, device="cpu", layer: int = 0) -> Optional[torch.Tensor]:
    """One named tensor of the layer as float32 (values exact in ``shape.act``).

    Names: x [T,d], Wr [d,E], Wg/Wu [E,d,F], Wd [E,F,d], dy [T,d] (rounded to the
    activation dtype); noise [T,E] and bias [E] (float32, never rounded).
    """
    s = shape
    dev = torch.device(device)
    if name == "bias":
        if s.zipf_s is None:
            return None
        ranks = torch.randperm(s.E, generator=_gen(s, "ranks", "cpu", layer)) + 1
        return (-s.zipf_s * torch.log(ranks.to(torch.float64))).to(torch.float32).to(dev)
    dims = {"x": (s.T, s.d), "Wr": (s.d, s.E), "Wg": (s.E, s.d, s.F), "Wu": (s.E, s.d, s.F),
            "Wd": (s.E, s.F, s.d), "noise": (s.T, s.E), "dy": (s.T, s.d)}[name]
    std = {"x": 1.0, "Wr": s.d ** -0.5, "Wg": 0.02, "Wu": 0.02, "Wd": 0.02,
           "noise": s.sigma, "dy": 1.0}[name]
    t = torch.randn(dims, generator=_gen(s, name, dev, layer), device=dev,
                    dtype=torch.float32) * std
    return t if name == "noise" else _round(t, s.act)


def make_layer(shape: LayerShape, device="cpu", layer: int = 0, backward: bool = True):
    """All tensors of one layer as a dict of float32 tensors."""
    names = ["x", "Wr", "Wg", "Wu", "Wd", "noise", "bias"] + (["dy"] if backward else [])
    return {n: draw(shape, n, device, layer) for n in names}


def rollout_batch(T: int, P: int, group: int = 4, prompt_share: float = 0.3, seed: int = 0):
    """Layout of a packed batch of rollouts for the mask cache: sequences in groups of `group` that share
    a prompt (several responses are sampled per prompt), T tokens in all.  Returns numpy arrays
        lens [nseq], shared [nseq] (leading tokens that sit in pages owned by the group's first sequence:
        whole pages of the prompt, 0 for the owner), block_table int32 [nseq, max_blocks] (-1 unused) with
        physical pages dealt in a seeded shuffled order, num_pages.
    Lengths are log-uniform between 1/8 and 8/8 of twice the mean, like a mix of short and long responses.
    Layout only: no ids are drawn here."""
    import numpy as np
    rng = np.random.default_rng(seed)
    mean = max(P * 4, min(2048, T // 8 if T >= 64 else T))
    lens, owner_prompt = [], []
    left = T
    while left > 0:
        prompt = int(mean * prompt_share * rng.uniform(0.5, 1.5))
        for g in range(group):
            if left <= 0:
                break
            n = int(np.exp(rng.uniform(np.log(mean / 4), np.log(mean * 2))))
            n = max(1, min(n, left))
            lens.append(n)
            owner_prompt.append((g, prompt))
            left -= n
    nseq = len(lens)
    lens = np.array(lens, np.int64)
    shared = np.zeros(nseq, np.int64)
    blocks = (lens + P - 1) // P
    max_blocks = int(blocks.max())
    table = -np.ones((nseq, max_blocks), np.int32)
    logical, owner = 0, 0
    for s in range(nseq):
        g, prompt = owner_prompt[s]
        if g == 0:
            owner = s
        else:
            full = min(prompt, int(lens[owner]), int(lens[s])) // P          # whole pages of the common prompt
            shared[s] = full * P
            table[s, :full] = table[owner, :full]
        first = int(shared[s]) // P
        table[s, first:blocks[s]] = np.arange(logical, logical + blocks[s] - first)
        logical += int(blocks[s]) - first
    deal = rng.permutation(logical).astype(np.int32)
    table = np.where(table >= 0, deal[np.maximum(table, 0)], -1).astype(np.int32)
    return lens, shared, table, logical
