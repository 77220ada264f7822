"""Seeded random token trees: tslt_verify_tree (both verification rules, all nodes and path only) against the
oracle.  Every case is printed before it runs, so that a failure names its shape and seed."""
import numpy as np
import pytest
import torch

from paper_2512_16273_amd import workloads as W
from tests import _parity as P
from tests.test_gpu_tree import oracle_for, run_tree

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("stream", [0, 1, 2])
def test_random_trees(tslt, stream):
    rng = np.random.default_rng(2000 + stream)
    totals = dict(trees=0, near_tie_nodes=0, near_tie_node_mismatches=0, near_tie_sequences=0)
    for case in range(8):
        dtype = ["f32", "bf16", "f16"][rng.integers(3)]
        depth = int(rng.integers(1, 5))
        expansion = tuple(int(rng.integers(1, 5)) for _ in range(depth))
        while int(np.prod(expansion)) > 64:           # keep the oracle's work small
            expansion = expansion[:-1]
        V = int(rng.choice([rng.integers(200, 3000), rng.integers(3000, 30000)]))
        k_cap = int(rng.choice([4, 16, 64, 256]))
        top_k = int(rng.integers(2, k_cap + 1))
        B = int(rng.integers(1, 4))
        T = float(rng.choice([0.7, 1.0, 1.3]))
        wor = bool(rng.integers(2))                   # how the candidates are drawn
        rule = bool(rng.integers(2)) if wor else False   # the renormalised rule is for candidates without replacement
        w = W.scaled(W.WORKLOADS["tree"], B=B, V=V, dtype=dtype, expansion=expansion, top_k=top_k, top_p=0.0, k_cap=k_cap, T=T,
                     without_replacement=wor, noise_t=float(rng.choice([0.3, 0.8, 2.0])))
        seed = int(rng.integers(1 << 30))
        print(f"case {stream}.{case}: {dtype} B={B} V={V} expansion={expansion} top_k={top_k} k_cap={k_cap} T={T} "
              f"drawn_without_replacement={wor} renormalised_rule={rule} seed={seed}", flush=True)
        tree = W.make_tree(w, seed, DEV)
        ref = oracle_for(w, tree, renormalised_rule=rule)
        out = run_tree(tslt, w, tree, ref, all_nodes=True, renormalised_rule=rule)
        path_only = run_tree(tslt, w, tree, ref, all_nodes=False, renormalised_rule=rule)
        torch.cuda.synchronize()
        res = P.compare_tree(out, ref, w.expansion, all_nodes=True, label=f"case {stream}.{case}")
        assert torch.equal(path_only["seq"], out["seq"]) and torch.equal(path_only["len"], out["len"]), case
        for k in totals:
            totals[k] += res[k]
    print(totals)
