"""Seeded synthetic workloads for the TSLT hot path.

This module only manufactures inputs (logit rows, uniforms, tree shapes).  It
holds none of the method's arithmetic: no softmax, no truncation, no sampling,
no verification.  Both the HIP path and the CPU oracle are fed from here so
that they see identical bits; neither of them is imported here.

The paper measures on Llama-68M / Llama-7B logits (Section 5, Table 1); those
weights are not available, so rows are synthetic: Gaussian noise plus a
Zipf-shaped rank bias through a per-row random permutation (a small head that
carries most of the mass, which is the property Section 5.1 relies on).

Recipe (every config):
  * one torch.Generator per call, seeded with (seed, config id);
  * base row (fp32) = N(0, sigma^2) + bias (+ `shift`, 0 in every benchmark configuration); bias is either
      - `boost`: n distinct random indices per row get +amount, or
      - `zipf`:  -a * ln(rank + 1), rank 0-based through a random permutation
                 drawn per row;
  * draft  = round-to-nearest-even(base) in the storage dtype;
  * target = round(base + N(0, noise_t^2)), rounded independently;
  * rows that have no draft partner (the bonus row of a chain, the leaves of a
    tree) are an independent base row + the same target noise;
  * uniforms are fp32 in [0, 1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field, replace
from typing import Optional, Tuple

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    V: int
    dtype: str                 # "f32" | "bf16" | "f16"
    sigma: float               # std of the Gaussian part of a base row
    noise_t: float             # std of target - draft noise
    T: float                   # temperature (draft and target)
    k_cap: int                 # width of the sparse representation
    top_k: int = 0             # 0 = off
    top_p: float = 0.0         # 0 = off
    gamma: int = 0             # chain: draft positions per sequence
    zipf: float = 0.0          # Zipf exponent a (0 = no rank bias)
    boost: Tuple[int, float] = (0, 0.0)   # (n indices, amount)
    expansion: Tuple[int, ...] = ()       # tree: k_1..k_L
    without_replacement: bool = False     # tree: how candidates are drawn
    shift: float = 0.0                    # added to every logit (a softmax does not see it; the number format does)
    config_id: int = 0


# The five benchmark configurations (configuration 2 has two truncation settings).
WORKLOADS = {
    "tiny": Workload("tiny", B=1, gamma=4, V=32000, dtype="f32", sigma=2.0, boost=(8, 8.0),
                     noise_t=0.5, T=1.0, top_k=16, k_cap=16, config_id=1),
    "chain_topk": Workload("chain_topk", B=64, gamma=8, V=32000, dtype="bf16", sigma=3.0, zipf=1.1,
                           noise_t=1.0, T=0.8, top_k=64, k_cap=64, config_id=2),
    "chain_topp": Workload("chain_topp", B=64, gamma=8, V=32000, dtype="bf16", sigma=3.0, zipf=1.1,
                           noise_t=1.0, T=0.8, top_p=0.95, k_cap=256, config_id=2),
    "large_vocab": Workload("large_vocab", B=256, gamma=8, V=128256, dtype="bf16", sigma=2.0, zipf=1.0,
                            noise_t=0.7, T=0.7, top_p=0.9, k_cap=256, config_id=3),
    "tree": Workload("tree", B=128, V=151936, dtype="f32", sigma=2.5, zipf=1.0, noise_t=0.8, T=1.0,
                     top_k=32, k_cap=32, expansion=(4, 4, 4, 4, 4), without_replacement=True,
                     config_id=4),
    "stress": Workload("stress", B=1024, gamma=16, V=256000, dtype="bf16", sigma=1.5, zipf=1.2,
                       noise_t=0.5, T=1.0, top_p=0.99, k_cap=1024, config_id=5),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller B or V for tests)."""
    return replace(w, **kw)


def torch_dtype(name: str) -> torch.dtype:
    return {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[name]


def _generator(device, seed: int, config_id: int, stream: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + config_id * 101 + stream) & 0x7FFFFFFFFFFFFFFF)
    return g


def _base_rows(w: Workload, n_rows: int, g: torch.Generator, device) -> torch.Tensor:
    """fp32 base rows [n_rows, V] = Gaussian noise + head bias."""
    V = w.V
    base = torch.randn(n_rows, V, generator=g, device=device, dtype=torch.float32) * w.sigma
    if w.zipf > 0.0:
        keys = torch.rand(n_rows, V, generator=g, device=device, dtype=torch.float32)
        rank = torch.argsort(torch.argsort(keys, dim=1), dim=1)   # a permutation per row
        del keys
        base -= w.zipf * torch.log(rank.to(torch.float32) + 1.0)
        del rank
    n_boost, amount = w.boost
    if n_boost > 0:
        keys = torch.rand(n_rows, V, generator=g, device=device, dtype=torch.float32)
        hot = torch.topk(keys, n_boost, dim=1).indices            # n distinct indices per row
        base.scatter_add_(1, hot, torch.full_like(hot, amount, dtype=torch.float32))
    if w.shift != 0.0:
        base += w.shift
    return base


def make_rows(w: Workload, n_paired: int, n_unpaired: int, seed: int, device="cpu", stream: int = 0,
              chunk_rows: int = 256):
    """Draft rows [n_paired, V] and target rows [n_paired + n_unpaired, V] in the storage dtype.

    target[i] for i < n_paired is draft[i]'s base + noise; the remaining target rows are
    independent base rows + noise.
    """
    dt = torch_dtype(w.dtype)
    g = _generator(device, seed, w.config_id, stream)
    draft = torch.empty(n_paired, w.V, dtype=dt, device=device)
    target = torch.empty(n_paired + n_unpaired, w.V, dtype=dt, device=device)
    total = n_paired + n_unpaired
    for r0 in range(0, total, chunk_rows):
        r1 = min(total, r0 + chunk_rows)
        base = _base_rows(w, r1 - r0, g, device)
        n_p = max(0, min(r1, n_paired) - r0)
        if n_p > 0:
            draft[r0:r0 + n_p] = base[:n_p].to(dt)
        noise = torch.randn(r1 - r0, w.V, generator=g, device=device, dtype=torch.float32) * w.noise_t
        target[r0:r1] = (base + noise).to(dt)
        del base, noise
    return draft, target


def uniforms(shape, seed: int, config_id: int, stream: int, device="cpu") -> torch.Tensor:
    """fp32 uniforms in [0, 1) (torch.rand never returns 1.0)."""
    g = _generator(device, seed, config_id, 1000 + stream)
    return torch.rand(*shape, generator=g, device=device, dtype=torch.float32)


def make_chain(w: Workload, seed: int, device="cpu"):
    """Inputs of one single-candidate round (Algorithms 2 and 3 of the paper).

    Returns a dict with
      draft  [B, gamma, V]      draft logits
      target [B, gamma + 1, V]  target logits; row gamma is the bonus row
      u_sample [B, gamma], u_accept [B, gamma], u_resample [B, gamma + 1]
    """
    B, G, V = w.B, w.gamma, w.V
    dt = torch_dtype(w.dtype)
    draft = torch.empty(B, G, V, dtype=dt, device=device)
    target = torch.empty(B, G + 1, V, dtype=dt, device=device)
    # sequences are generated in groups so that peak memory stays bounded
    per = max(1, 256 // (G + 1))
    for b0 in range(0, B, per):
        b1 = min(B, b0 + per)
        nb = b1 - b0
        d, t = make_rows(w, nb * G, nb, seed, device, stream=10 + b0)
        draft[b0:b1] = d.view(nb, G, V)
        target[b0:b1, :G] = t[:nb * G].view(nb, G, V)
        target[b0:b1, G] = t[nb * G:]
    return {
        "draft": draft, "target": target,
        "u_sample": uniforms((B, G), seed, w.config_id, 1, device),
        "u_accept": uniforms((B, G), seed, w.config_id, 2, device),
        "u_resample": uniforms((B, G + 1), seed, w.config_id, 3, device),
    }


def tree_shape(expansion):
    """Layer widths W_l, node counts and layer offsets of an expansion-configured token tree
    stored breadth-first (Section 4.1: W_l = prod_{j<=l} k_j; node (l, i)'s children are the
    k_{l+1} consecutive nodes starting at (l+1, i*k_{l+1}), 0-based)."""
    widths = [1]
    for k in expansion:
        widths.append(widths[-1] * int(k))
    offsets = [0]
    for wd in widths:
        offsets.append(offsets[-1] + wd)
    n_nodes = offsets[-1]
    n_internal = offsets[-2]
    return {"widths": widths, "offsets": offsets, "n_nodes": n_nodes, "n_internal": n_internal,
            "depth": len(expansion)}


def make_tree(w: Workload, seed: int, device="cpu"):
    """Inputs of one multi-candidate round (Algorithms 7 and 8).

    draft  [B, N_int, V]   draft logits of every non-leaf node, breadth-first
    target [B, N_nodes, V] target logits of every node; internal node n pairs with draft node n,
                           leaves are independent rows
    u_sample [B, N_int, k_max], u_accept [B, N_nodes - 1], u_resample [B, N_nodes]
    Candidate tokens are NOT produced here: drawing them is part of the method.
    """
    sh = tree_shape(w.expansion)
    B, V = w.B, w.V
    n_int, n_nodes = sh["n_internal"], sh["n_nodes"]
    dt = torch_dtype(w.dtype)
    draft = torch.empty(B, n_int, V, dtype=dt, device=device)
    target = torch.empty(B, n_nodes, V, dtype=dt, device=device)
    for b in range(B):
        d, t = make_rows(w, n_int, n_nodes - n_int, seed, device, stream=10 + b)
        draft[b] = d
        target[b] = t
    k_max = max(w.expansion)
    return {
        "draft": draft, "target": target, "shape": sh,
        "u_sample": uniforms((B, n_int, k_max), seed, w.config_id, 1, device),
        "u_accept": uniforms((B, n_nodes - 1), seed, w.config_id, 2, device),
        "u_resample": uniforms((B, n_nodes), seed, w.config_id, 3, device),
    }
