"""GPU parity: tslt_verify_tree through the C ABI against the CPU oracle (Algorithms 5 and 8)."""
import numpy as np
import pytest
import torch

from oracle import tslt_oracle as O
from paper_2512_16273_amd import workloads as W
from tests import _parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def t32(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def run_tree(tslt, w, tree, ref, all_nodes=True, renormalised_rule=False):
    return tslt.verify_tree(tree["target"], w.T, w.expansion, t32(ref["q_idx"]), t32(ref["q_logit"]),
                            t32(ref["q_count"]), t32(ref["cands"]), tree["u_accept"], tree["u_resample"],
                            all_nodes=all_nodes, without_replacement=renormalised_rule)


def oracle_for(w, tree, renormalised_rule=False):
    return P.oracle_tree(P.to_np(tree["draft"]), P.to_np(tree["target"]), w.T, w.top_k, w.top_p, w.k_cap, w.expansion,
                         P.to_np(tree["u_sample"]), P.to_np(tree["u_accept"]), P.to_np(tree["u_resample"]),
                         w.without_replacement, renormalised_rule)


@pytest.mark.parametrize("name,kw", [
    ("f32-322", dict(B=3, V=5003, expansion=(3, 2, 2), top_k=8, k_cap=8)),
    ("f32-iid", dict(B=3, V=7001, expansion=(2, 2, 2), top_k=6, k_cap=8, without_replacement=False)),
    ("bf16-44", dict(B=2, V=20011, dtype="bf16", expansion=(4, 4), top_k=32, k_cap=32, T=0.9)),
    ("bf16-topp", dict(B=2, V=30000, dtype="bf16", expansion=(2, 3), top_k=0, top_p=0.9, k_cap=256, T=0.8)),
    ("f16-topp", dict(B=2, V=30000, dtype="f16", expansion=(2, 3), top_k=0, top_p=0.9, k_cap=256, T=0.8)),
    ("f16-44", dict(B=2, V=20011, dtype="f16", expansion=(4, 4), top_k=32, k_cap=32, T=0.9)),
    ("f32-deep", dict(B=2, V=3000, expansion=(1, 2, 1, 2, 1, 2), top_k=4, k_cap=4)),
])
def test_tree_matches_oracle(tslt, name, kw):
    w = W.scaled(W.WORKLOADS["tree"], **kw)
    tree = W.make_tree(w, 5, DEV)
    ref = oracle_for(w, tree)
    out = run_tree(tslt, w, tree, ref, all_nodes=True)
    torch.cuda.synchronize()
    res = P.compare_tree(out, ref, w.expansion, all_nodes=True, label=name)
    path_only = run_tree(tslt, w, tree, ref, all_nodes=False)
    torch.cuda.synchronize()
    assert torch.equal(path_only["seq"], out["seq"]) and torch.equal(path_only["len"], out["len"])
    print(name, res, "len histogram", np.bincount(ref["verify"]["len"], minlength=len(w.expansion) + 2))


@pytest.mark.parametrize("name,kw", [
    ("f32-332", dict(B=3, V=5003, expansion=(3, 3, 2), top_k=8, k_cap=8)),
    ("bf16-44", dict(B=2, V=20011, dtype="bf16", expansion=(4, 4), top_k=32, k_cap=32, T=0.9)),
    ("bf16-noisy", dict(B=3, V=9000, dtype="bf16", expansion=(4, 3), top_k=6, k_cap=8, noise_t=2.5)),
    ("f32-exhaust", dict(B=2, V=3000, expansion=(4, 4), top_k=3, k_cap=4)),       # more candidates than set entries
])
def test_tree_rule_for_candidates_drawn_without_replacement(tslt, name, kw):
    """The rule with renormalised stage proposals, on candidates drawn without replacement; it must differ
    from the printed rule somewhere (else the flag could be ignored unnoticed)."""
    w = W.scaled(W.WORKLOADS["tree"], without_replacement=True, **kw)
    tree = W.make_tree(w, 7, DEV)
    ref = oracle_for(w, tree, renormalised_rule=True)
    out = run_tree(tslt, w, tree, ref, all_nodes=True, renormalised_rule=True)
    torch.cuda.synchronize()
    res = P.compare_tree(out, ref, w.expansion, all_nodes=True, label=name)
    path_only = run_tree(tslt, w, tree, ref, all_nodes=False, renormalised_rule=True)
    printed = run_tree(tslt, w, tree, ref, all_nodes=True, renormalised_rule=False)
    torch.cuda.synchronize()
    assert torch.equal(path_only["seq"], out["seq"]) and torch.equal(path_only["len"], out["len"])
    r_new, r_old = P.to_np(out["ratio"]), P.to_np(printed["ratio"])
    both = ~np.isnan(r_new) & ~np.isnan(r_old)
    differ = int(np.count_nonzero(np.abs(r_new[both] - r_old[both]) > 1e-3 * np.abs(r_old[both])))
    print(name, res, "ratios that differ between the rules:", differ)
    assert differ > 0 or name == "f32-exhaust"      # (there every later ratio is 0 under both rules)


def test_unary_tree_equals_chain_verify(tslt):
    """k = <1,..,1> reduces Algorithm 8 to Algorithm 3 with a bonus row: same tokens from both entry points."""
    L = 5
    w = W.scaled(W.WORKLOADS["tree"], B=6, V=9001, expansion=(1,) * L, top_k=6, k_cap=8, without_replacement=False)
    tree = W.make_tree(w, 9, DEV)
    ref = oracle_for(w, tree)
    out = run_tree(tslt, w, tree, ref)
    chain = tslt.verify(tree["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(ref["cands"]),
                        tree["u_accept"], tree["u_resample"])
    torch.cuda.synchronize()
    assert torch.equal(out["len"], chain["accept_len"] + 1)
    assert torch.equal(out["seq"], chain["tokens"])
    print(P.compare_tree(out, ref, w.expansion, label="unary"))


@pytest.mark.parametrize("name,kw,rule", [
    ("widest", dict(B=2, V=2500, expansion=(16,), top_k=24, k_cap=32), False),            # TSLT_MAX_BRANCH candidates
    ("widest-wor", dict(B=2, V=2500, expansion=(16, 2), top_k=12, k_cap=16), True),       # more candidates than entries
    ("deepest", dict(B=3, V=600, expansion=(1,) * 16, top_k=0, k_cap=600, without_replacement=False, noise_t=0.02), False),
])
def test_tree_limits(tslt, name, kw, rule):
    """The largest branching factor and depth the library accepts."""
    w = W.scaled(W.WORKLOADS["tree"], **kw)
    tree = W.make_tree(w, 13, DEV)
    ref = oracle_for(w, tree, renormalised_rule=rule)
    out = run_tree(tslt, w, tree, ref, all_nodes=True, renormalised_rule=rule)
    path_only = run_tree(tslt, w, tree, ref, all_nodes=False, renormalised_rule=rule)
    torch.cuda.synchronize()
    print(name, P.compare_tree(out, ref, w.expansion, all_nodes=True, label=name), "lens", ref["verify"]["len"])
    if name == "deepest":
        assert ref["verify"]["len"].max() == 17          # a walk through every layer
    assert torch.equal(path_only["seq"], out["seq"]) and torch.equal(path_only["len"], out["len"])
    too_wide = dict(kw, expansion=(17,))
    with pytest.raises(tslt.TsltError):
        w2 = W.scaled(W.WORKLOADS["tree"], **too_wide)
        t2 = W.make_tree(w2, 1, DEV)
        tslt.verify_tree(t2["target"], w2.T, w2.expansion, t32(ref["q_idx"][:, :1]), t32(ref["q_logit"][:, :1]),
                         t32(ref["q_count"][:, :1]), torch.zeros(w2.B, 17, dtype=torch.int32, device=DEV),
                         t2["u_accept"], t2["u_resample"])


def test_tree_broken_rows_and_missing_candidates(tslt):
    w = W.scaled(W.WORKLOADS["tree"], B=4, V=4000, expansion=(2, 2), top_k=5, k_cap=8)
    tree = W.make_tree(w, 2, DEV)
    target = tree["target"].clone()
    target[1, 0, 7] = float("nan")           # unusable root
    target[2, 5, 9] = float("inf")           # unusable leaf
    target[3, 1, :] = -float("inf")          # fully masked internal node
    tree["target"] = target
    ref = oracle_for(w, tree)
    cands = ref["cands"].copy()
    cands[0, 1] = -1                          # an absent candidate
    outside = int(np.setdiff1d(np.arange(w.V), ref["q_idx"][0, 1])[0])
    cands[0, 2] = outside                     # a candidate that is not in its node's set
    ref["cands"] = cands
    ref["verify"] = O.verify_tree(P.to_np(target), w.T, w.expansion, ref["q_idx"], ref["q_logit"], ref["q_count"], cands,
                                  P.to_np(tree["u_accept"]), P.to_np(tree["u_resample"]))
    out = run_tree(tslt, w, tree, ref)
    torch.cuda.synchronize()
    v = ref["verify"]
    assert v["status"][0] & 4 and v["status"][1] & 1 and v["status"][2] & 1 and v["status"][3] & 2
    print(P.compare_tree(out, ref, w.expansion, label="broken"), v["status"])


def test_tree_argument_errors(tslt):
    w = W.scaled(W.WORKLOADS["tree"], B=1, V=2000, expansion=(2, 2), top_k=4, k_cap=4)
    tree = W.make_tree(w, 2, DEV)
    ref = oracle_for(w, tree)
    args = (tree["target"], w.T, w.expansion, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]),
            t32(ref["cands"]), tree["u_accept"], tree["u_resample"])
    with pytest.raises(tslt.TsltError):
        tslt.verify_tree(*args, workspace=torch.empty(64, dtype=torch.uint8, device=DEV))
    bad = list(args)
    bad[2] = (2, 99)
    with pytest.raises(tslt.TsltError):
        tslt.verify_tree(*bad)


def test_tree_config_shape_few_trees(tslt):
    """Benchmark configuration 4's shape (depth 5, 4 candidates per node, V=151936, fp32, top-k 32, candidates drawn
    without replacement) on 2 trees: 682 draft rows and 2730 target rows, every node evaluated."""
    w = W.scaled(W.WORKLOADS["tree"], B=2)
    tree = W.make_tree(w, 0, DEV)
    B, V, K = w.B, w.V, w.k_cap
    n_int = tree["shape"]["n_internal"]
    # the device side of the round on the GPU, checked against the oracle before it is used
    tr = tslt.truncate(tree["draft"], w.T, w.top_k, w.top_p, K)
    ref = oracle_for(w, tree)
    P.compare_truncate(tr, tree["draft"].reshape(B * n_int, V), w.T, w.top_k, w.top_p, K, label="tree draft")
    smp = tslt.sample(tr["idx"], tr["logit"], tr["count"], tree["u_sample"].reshape(B * n_int, -1), w.without_replacement)
    torch.cuda.synchronize()
    got = P.to_np(smp["token"]).reshape(B, n_int, -1)
    lay = ref["layout"]
    for n in range(n_int):
        layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
        c0 = O.child_node(lay, w.expansion, n, 0)
        assert np.array_equal(got[:, n, :w.expansion[layer]], ref["cands"][:, c0 - 1:c0 - 1 + w.expansion[layer]])
    out = run_tree(tslt, w, tree, ref)
    torch.cuda.synchronize()
    print(P.compare_tree(out, ref, w.expansion, label="config4"), "lens", ref["verify"]["len"])
    # the same trees under the rule that is exact for candidates drawn this way
    ref["verify"] = O.verify_tree(P.to_np(tree["target"]), w.T, w.expansion, ref["q_idx"], ref["q_logit"], ref["q_count"],
                                  ref["cands"], P.to_np(tree["u_accept"]), P.to_np(tree["u_resample"]), True)
    out = run_tree(tslt, w, tree, ref, renormalised_rule=True)
    torch.cuda.synchronize()
    print(P.compare_tree(out, ref, w.expansion, label="config4 renormalised"), "lens", ref["verify"]["len"],
          "nodes that rejected every candidate:", int(np.count_nonzero(ref["verify"]["node_slot"][:, :n_int] < 0)))
