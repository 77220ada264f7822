"""Closed forms of the paper's latency model (Sections 2.2-2.4 and 4.1), as host arithmetic.

Nothing here touches the GPU or the library; the functions only restate the paper's formulas so that the
sizes the wire codec produces (tslt_pack) can be turned into the uplink times and speed-up ratios the paper
reasons with.  All sizes are in bits, rates in bits per second, times in seconds.
"""
from __future__ import annotations

import math
from typing import Sequence


def index_bits(V: int) -> int:
    """b_idx = ceil(log2 |V|), the binary encoding of a token id (Section 2.2)."""
    if V < 1:
        raise ValueError("V must be >= 1")
    return max(0, (V - 1).bit_length())


def dense_bits(V: int, b_prob: int = 16, with_index: bool = False) -> int:
    """Bits of one dense vocabulary distribution.  Section 2.2 writes D_V = |V| (b_prob + b_idx); the
    experiments quote D_V = 0.5 Mbit for |V| = 32K at FP16, which is |V| * b_prob (a dense vector needs no
    ids): `with_index` selects between the two."""
    return V * (b_prob + (index_bits(V) if with_index else 0))


def sparse_bits(K: int, V: int, b_prob: int = 16) -> int:
    """Bits of one truncated distribution: K pairs of a value and a token id (Section 3.1)."""
    return K * (b_prob + index_bits(V))


def t_comm(bits_per_distribution: float, n_distributions: int, R_up: float) -> float:
    """T_comm = D_up / R_up with D_up = L * D_V (Section 2.2); n_distributions is L for a chain and |Q| for
    a token tree."""
    if R_up <= 0:
        raise ValueError("R_up must be > 0")
    return n_distributions * bits_per_distribution / R_up


def n_oracle(alpha: float, L: int) -> float:
    """Expected tokens per oracle call, (1 - alpha^(L+1)) / (1 - alpha) (Section 2.3)."""
    if not 0.0 <= alpha <= 1.0:
        raise ValueError("alpha must be in [0, 1]")
    if alpha == 1.0:
        return float(L + 1)
    return (1.0 - alpha ** (L + 1)) / (1.0 - alpha)


def t_oracle(L: int, T_slm: float, T_comm: float, T_llm: float) -> float:
    """T_oracle = L * T_SLM + T_comm + T_LLM (Section 2.3, and Section 4.1 with L the tree's depth)."""
    return L * T_slm + T_comm + T_llm


def throughput(alpha: float, L: int, T_slm: float, T_comm: float, T_llm: float) -> float:
    """Tokens per second of distributed speculative decoding, N_oracle / T_oracle."""
    return n_oracle(alpha, L) / t_oracle(L, T_slm, T_comm, T_llm)


def speedup(alpha: float, L: int, T_slm: float, T_comm: float, T_llm: float) -> float:
    """S_inf = throughput / (1 / T_LLM) (Section 2.3)."""
    return throughput(alpha, L, T_slm, T_comm, T_llm) * T_llm


def tree_distributions(expansion: Sequence[int]) -> int:
    """|Q| = 1 + sum_{l=1}^{L-1} prod_{i<=l} k_i: one draft distribution per non-leaf node (Section 4.1)."""
    n, width = 1, 1
    for k in list(expansion)[:-1]:
        width *= int(k)
        n += width
    return n


def tree_speedup(alpha: float, expansion: Sequence[int], T_slm: float, bits_per_distribution: float, R_up: float,
                 T_llm: float) -> float:
    """Section 4.1's S_inf = 1 / ((L T_SLM + |Q| T_V) / ((L alpha + 1) T_LLM) + 1), T_V the uplink time of one
    distribution."""
    L = len(expansion)
    T_v = bits_per_distribution / R_up
    return 1.0 / ((L * T_slm + tree_distributions(expansion) * T_v) / ((L * alpha + 1.0) * T_llm) + 1.0)
