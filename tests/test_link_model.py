"""The latency model's closed forms (Sections 2.2-2.4, 4.1) against the paper's printed figures and against
the sums they abbreviate."""
import math

import numpy as np
import pytest

from oracle import tslt_oracle as O
from paper_2512_16273_amd import linkmodel as M


def test_dense_distribution_is_half_a_megabit():
    # Section 5.1 and Table 1: |V| = 32K at FP16 is D_V = 0.5 Mbit
    assert M.dense_bits(32000, 16) == 512000
    assert abs(M.dense_bits(32000, 16) / 1e6 - 0.5) < 0.02
    assert M.dense_bits(32000, 16, with_index=True) == 32000 * (16 + 15)      # Section 2.2's formula as written


def test_index_bits_and_sparse_size():
    for V, b in ((1, 0), (2, 1), (3, 2), (32000, 15), (32768, 15), (32769, 16), (128256, 17), (151936, 18), (256000, 18)):
        assert M.index_bits(V) == b == O.index_bits(V)
    assert M.sparse_bits(64, 32000) == 64 * 31 == O.payload_bits(64, 16, O.index_bits(32000))
    # the packed stream of tslt_pack is this plus a 16-bit count, rounded up to 32-bit words
    assert (16 + M.sparse_bits(64, 32000) + 31) // 32 == 63


def test_expected_tokens_per_call_is_the_geometric_sum():
    for alpha in (0.0, 0.3, 0.8, 0.999, 1.0):
        for L in (1, 4, 8):
            want = sum(alpha ** i for i in range(L + 1))      # 1 + alpha + ... + alpha^L
            assert abs(M.n_oracle(alpha, L) - want) < 1e-9 * want
    # by simulation of Algorithm 3's stopping rule with independent acceptances
    rng = np.random.default_rng(0)
    alpha, L = 0.7, 6
    acc = rng.random((200000, L)) < alpha
    n = np.where(acc.all(1), L, np.argmin(acc, 1)) + 1        # accepted drafts + the one token the server adds
    assert abs(n.mean() - M.n_oracle(alpha, L)) < 0.02


def test_throughput_and_speedup():
    L, T_slm, T_llm, R = 4, 2e-3, 30e-3, 10e6
    tc = M.t_comm(M.dense_bits(32000, 16), L, R)
    assert abs(tc - 4 * 512000 / 10e6) < 1e-15
    assert abs(M.t_oracle(L, T_slm, tc, T_llm) - (4 * 2e-3 + tc + 30e-3)) < 1e-15
    s = M.speedup(0.8, L, T_slm, tc, T_llm)
    assert abs(s - M.n_oracle(0.8, L) * T_llm / (L * T_slm + tc + T_llm)) < 1e-12
    # no drafting or uplink cost: every call yields N_oracle tokens for one LLM run
    assert abs(M.speedup(0.8, L, 0.0, 0.0, T_llm) - M.n_oracle(0.8, L)) < 1e-12
    # a truncated payload shortens the uplink by |V| b_prob / (K (b_prob + b_idx))
    assert abs(M.t_comm(M.sparse_bits(64, 32000), L, R) / tc - 64 * 31 / 512000) < 1e-15
    with pytest.raises(ValueError):
        M.t_comm(1.0, 1, 0.0)
    with pytest.raises(ValueError):
        M.n_oracle(1.5, 3)


def test_tree_distribution_count_and_speedup():
    assert M.tree_distributions((2, 2, 2)) == 7              # Section 5.1's configuration: 1 + 2 + 4
    assert M.tree_distributions((4, 4, 4, 4, 4)) == 341
    assert M.tree_distributions((3,)) == 1
    lay = O.tree_layout((2, 3, 2))
    assert M.tree_distributions((2, 3, 2)) == lay["n_internal"]
    s = M.tree_speedup(0.8, (2, 2, 2), 2e-3, 512000.0, 10e6, 30e-3)
    want = 1.0 / ((3 * 2e-3 + 7 * 0.0512) / ((3 * 0.8 + 1) * 30e-3) + 1.0)
    assert math.isclose(s, want, rel_tol=1e-12)
    # free drafting and uplink: the formula's ceiling is 1 (it counts the LLM run in the denominator)
    assert M.tree_speedup(0.8, (2, 2, 2), 0.0, 0.0, 10e6, 30e-3) == 1.0
