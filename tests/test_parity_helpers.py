"""The GPU parity comparers themselves, on the CPU: fed the oracle's own outputs with a planted difference,
they must fail on a difference outside a near-tie window, excuse and count one inside it, and fail when the
oracle flags more items than the stated share (which is what a margin that went to 0 looks like)."""
import copy

import numpy as np
import pytest

from oracle import tslt_oracle as O
from tests import _parity as P


def rows_and_ref(n=40, V=300, seed=2, top_p=0.9, k_cap=64):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 2.5, size=(n, V)).astype(np.float32)
    ref = O.truncate(z, 0.8, 0, top_p, k_cap)
    gpu = {k: ref[k].copy() for k in ("idx", "logit", "prob", "count", "mass", "status")}
    return z, ref, gpu


def test_truncate_comparer_passes_on_identical_outputs_and_counts():
    z, ref, gpu = rows_and_ref()
    res = P.compare_truncate(gpu, z, 0.8, 0, 0.9, 64)
    assert res["rows"] == 40 and res["exact_index_sets"] == 40 and res["top_p_near_tie_mismatches"] == 0


def test_truncate_comparer_fails_on_a_count_difference_outside_the_window():
    z, ref, gpu = rows_and_ref()
    r = int(np.argmax(ref["margin_rho"]))
    gpu["count"][r] -= 1
    with pytest.raises(AssertionError):
        P.compare_truncate(gpu, z, 0.8, 0, 0.9, 64)
    z, ref, gpu = rows_and_ref()
    gpu["idx"][3, 0], gpu["idx"][3, 1] = gpu["idx"][3, 1], gpu["idx"][3, 0]      # order matters
    with pytest.raises(AssertionError):
        P.compare_truncate(gpu, z, 0.8, 0, 0.9, 64)


def test_truncate_comparer_fails_when_margins_flag_too_many_rows(monkeypatch):
    z, ref, gpu = rows_and_ref()
    real = O.truncate

    def zero_margins(*a, **k):
        out = real(*a, **k)
        out["margin_rho"][:] = 0.0
        return out
    monkeypatch.setattr(O, "truncate", zero_margins)
    with pytest.raises(AssertionError, match="near-tie window"):
        P.compare_truncate(gpu, z, 0.8, 0, 0.9, 64)


def chain_case(B=12, G=4, V=200, K=8, seed=4):
    rng = np.random.default_rng(seed)
    draft = rng.normal(0, 2.0, size=(B, G, V)).astype(np.float32)
    target = np.concatenate([draft + rng.normal(0, 1.0, size=(B, G, V)).astype(np.float32),
                             rng.normal(0, 2.0, size=(B, 1, V)).astype(np.float32)], axis=1)
    ref = P.oracle_chain(draft, target, 1.0, K, 0.0, K, rng.random((B, G), dtype=np.float32),
                         rng.random((B, G), dtype=np.float32), rng.random((B, G + 1), dtype=np.float32))
    v = ref["verify"]
    gpu = dict(accept_len=v["accept_len"].copy(), tokens=v["tokens"].copy(), ratio=v["ratio"].astype(np.float32),
               beta=v["beta_hat"].astype(np.float32), status=v["status"].copy())
    return ref, gpu


def test_verify_comparer_window_and_bound():
    ref, gpu = chain_case()
    v = ref["verify"]
    res = P.compare_verify(gpu, v)
    assert res["sequences"] == 12 and res["accept_near_ties"] == 0 and res["exact_sequences"] == 12
    # a different accepted length outside the window fails
    b = int(np.argmax(v["accept_len"] > 0))
    bad = copy.deepcopy(gpu)
    bad["accept_len"][b] -= 1
    with pytest.raises(AssertionError):
        P.compare_verify(bad, v)
    # the same difference is excused, and counted, when the oracle says that decision is inside the window
    v2 = copy.deepcopy(v)
    v2["accept_margin"][b, bad["accept_len"][b]] = 1e-9
    res = P.compare_verify(bad, v2)
    assert res["accept_near_ties"] == 1 and res["accept_near_tie_mismatches"] == 1 and res["exact_sequences"] == 11
    # ... but not when the window belongs to another position
    v3 = copy.deepcopy(v)
    v3["accept_margin"][b, 0 if bad["accept_len"][b] > 0 else 1] = 1e-9
    if bad["accept_len"][b] > 0:
        with pytest.raises(AssertionError):
            P.compare_verify(bad, v3)
    # a flagged sequence in which the GPU took the oracle's decision is compared like any other
    res = P.compare_verify(gpu, v2)
    assert res["accept_near_ties"] == 1 and res["accept_near_tie_mismatches"] == 0
    wrong_token = copy.deepcopy(gpu)
    wrong_token["tokens"][b, 0] += 1
    with pytest.raises(AssertionError):
        P.compare_verify(wrong_token, v2)
    # margins that flag everything fail the comparison even though nothing differs
    v4 = copy.deepcopy(v)
    v4["accept_margin"][:] = 0.0
    with pytest.raises(AssertionError, match="near-tie window"):
        P.compare_verify(gpu, v4)


def tree_case(B=3, V=150, K=6, expansion=(3, 2), seed=6):
    rng = np.random.default_rng(seed)
    lay = O.tree_layout(expansion)
    n_int, n_nodes = lay["n_internal"], lay["n_nodes"]
    draft = rng.normal(0, 2.0, size=(B, n_int, V)).astype(np.float32)
    target = rng.normal(0, 2.0, size=(B, n_nodes, V)).astype(np.float32)
    target[:, :n_int] = draft + rng.normal(0, 1.0, size=(B, n_int, V)).astype(np.float32)
    ref = P.oracle_tree(draft, target, 1.0, K, 0.0, K, expansion, rng.random((B, n_int, max(expansion)), dtype=np.float32),
                        rng.random((B, n_nodes - 1), dtype=np.float32), rng.random((B, n_nodes), dtype=np.float32), False)
    v = ref["verify"]
    gpu = dict(node_token=v["node_token"].copy(), node_slot=v["node_slot"].copy(), seq=v["seq"].copy(), len=v["len"].copy(),
               ratio=v["ratio"].astype(np.float32), beta=v["beta"].astype(np.float32), status=v["status"].copy())
    return ref, gpu, lay


def test_tree_comparer_window_cap_and_bound():
    expansion = (3, 2)
    ref, gpu, lay = tree_case(expansion=expansion)
    res = P.compare_tree(gpu, ref, expansion)
    assert res["near_tie_nodes"] == 0 and res["exact_sequences"] == 3
    # a node off the verified path with another accepted child: fails, unless the oracle flags that node
    b = 0
    off_path = [n for n in range(lay["n_internal"]) if n not in ref["verify"]["path"][b]][0]
    bad = copy.deepcopy(gpu)
    bad["node_slot"][b, off_path] = (bad["node_slot"][b, off_path] + 2) % 3 - 1
    with pytest.raises(AssertionError):
        P.compare_tree(bad, ref, expansion)
    flagged = copy.deepcopy(ref)
    c0 = O.child_node(lay, expansion, off_path, 0)
    flagged["verify"]["accept_margin"][b, c0 - 1] = 1e-9
    res = P.compare_tree(bad, flagged, expansion)
    assert res["near_tie_nodes"] == 1 and res["near_tie_node_mismatches"] == 1 and res["near_tie_sequences"] == 0
    # the factor amp widens the window, but only up to AMP_CAP
    wide = copy.deepcopy(ref)
    wide["verify"]["accept_margin"][b, c0 - 1] = 1e-4
    wide["verify"]["amp"][b, c0 - 1] = 1e6                     # uncapped, 1e-6 * amp would excuse anything
    with pytest.raises(AssertionError):
        P.compare_tree(bad, wide, expansion)
    wide["verify"]["accept_margin"][b, c0 - 1] = 0.5 * 1e-6 * P.AMP_CAP
    assert P.compare_tree(bad, wide, expansion)["near_tie_node_mismatches"] == 1
    # margins that flag every node fail the comparison even though nothing differs
    allz = copy.deepcopy(ref)
    allz["verify"]["accept_margin"][:] = 0.0
    with pytest.raises(AssertionError, match="near-tie window"):
        P.compare_tree(gpu, allz, expansion)
