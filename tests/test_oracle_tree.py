"""Pins for the oracle's multi-candidate verification (Algorithm 5) and token-tree verification
(Algorithm 8), no GPU: losslessness for i.i.d. candidates by exhaustive enumeration of candidate
tuples at V <= 8 (and, for candidates drawn without replacement, of the rule with renormalised stage
proposals), the stage acceptance rates beta^(j) and the total rate theta of Section 4.3, the tree
identities of Section 4.1, and reductions to Algorithm 3.
"""
import itertools

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import tslt_oracle as O


def case(seed, V, K, noise=1.0):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 1.5, V).astype(np.float32)
    t = (z + rng.normal(0, noise, V)).astype(np.float32)
    tr = O.truncate_row(z, 1.0, K, 0.0, K)
    p = sp_softmax(t.astype(np.float64))
    qh_sparse = sp_softmax(tr["logit"].astype(np.float64))
    qh = np.zeros(V)
    qh[tr["idx"]] = qh_sparse
    return t, tr, p, qh, qh_sparse


def residual_dist(p, q):
    r = np.maximum(0, p - q)
    return r / r.sum()


@pytest.mark.parametrize("V,K,k", [(6, 3, 2), (8, 4, 3), (7, 7, 2), (5, 2, 3)])
def test_mcveri_output_distribution_is_p_for_iid_candidates(V, K, k):
    t, tr, p, qh, qs = case(40 + V + k, V, K)
    nr = 1500
    gr = (np.arange(nr) + 0.5) / nr
    out = np.zeros(V)
    stage_acc = np.zeros(k)      # P(candidate j accepted and all before rejected)
    stage_reach = np.zeros(k)    # P(all before j rejected)
    for tup in itertools.product(range(K), repeat=k):
        cands = [int(tr["idx"][s]) for s in tup]
        w = float(np.prod([qs[s] for s in tup]))
        # learn the acceptance probabilities along the all-rejected path from the reported ratios
        probe = O.mcveri(p, tr["idx"], qs, cands, [0.99999994] * k, 0.5)
        a = np.minimum(1.0, np.where(np.isnan(probe["ratio"]), 1.0, probe["ratio"]))
        reach = 1.0
        for j in range(k):
            if np.isnan(probe["ratio"][j]):
                break                        # an earlier candidate is accepted for every u
            # force: reject 0..j-1 (u just under 1), accept j (u in the middle of [0, a_j))
            stage_reach[j] += w * reach
            if a[j] > 0:
                u = [0.99999994] * j + [a[j] / 2] + [0.0] * (k - j - 1)
                r = O.mcveri(p, tr["idx"], qs, cands, u, 0.5)
                assert r["slot"] == j and r["token"] == cands[j]
                assert abs(r["ratio"][j] - probe["ratio"][j]) < 1e-15
                out[cands[j]] += w * reach * a[j]
                stage_acc[j] += w * reach * a[j]
            if a[j] < 1:
                # just above the bound rejects (strict <)
                u = [0.99999994] * j + [min(0.99999994, a[j] + (1 - a[j]) / 2)] + [0.0] * (k - j - 1)
                r = O.mcveri(p, tr["idx"], qs, cands, u, 0.5)
                assert r["slot"] != j
            reach *= (1 - a[j])
            if reach == 0:
                break
        if reach > 0:
            res = np.zeros(V)
            for ur in gr:
                r = O.mcveri(p, tr["idx"], qs, cands, [0.99999994] * k, ur)
                assert r["slot"] == -1 and r["token"] not in cands   # never a rejected candidate
                res[r["token"]] += 1
            out += w * reach * res / nr
    np.testing.assert_allclose(out, p, atol=2.0 / nr * V)
    # Section 4.3: beta^(j) = sum min(q, p^(j)), computed here from the printed recursion
    pj = p.copy()
    betas = []
    for j in range(k):
        betas.append(np.minimum(qh, pj).sum())
        pj = residual_dist(pj, qh)
    for j in range(k):
        if stage_reach[j] > 0:
            assert abs(stage_acc[j] / stage_reach[j] - betas[j]) < 1e-12
    theta = betas[0] + sum(betas[i] * np.prod([1 - b for b in betas[:i]]) for i in range(1, k))
    assert abs(stage_acc.sum() - theta) < 1e-12
    # multi-candidate acceptance beats single-candidate (Section 5.2's observation, exact here)
    assert theta >= betas[0] - 1e-15


def mcveri_output_distribution(p, tr, qs, tuples_with_weights, k, V, without_replacement, nr=1500):
    """Output distribution of O.mcveri over the given weighted candidate tuples: the accept branches are
    integrated analytically from the reported ratios, the all-rejected branch over a grid of u_resample."""
    gr = (np.arange(nr) + 0.5) / nr
    out = np.zeros(V)
    for cands, w in tuples_with_weights:
        probe = O.mcveri(p, tr["idx"], qs, cands, [0.99999994] * k, 0.5, without_replacement)
        a = np.minimum(1.0, np.where(np.isnan(probe["ratio"]), 1.0, probe["ratio"]))
        reach = 1.0
        for j in range(k):
            if np.isnan(probe["ratio"][j]):
                break
            out[cands[j]] += w * reach * a[j]
            reach *= (1 - a[j])
            if reach == 0:
                break
        if reach > 0:
            res = np.zeros(V)
            for ur in gr:
                r = O.mcveri(p, tr["idx"], qs, cands, [0.99999994] * k, ur, without_replacement)
                assert r["slot"] == -1 and r["token"] not in cands
                res[r["token"]] += 1
            out += w * reach * res / nr
    return out


@pytest.mark.parametrize("V,K,k", [(6, 3, 2), (8, 4, 3), (7, 5, 2), (5, 3, 3)])
def test_mcveri_without_replacement_rule_is_lossless_and_the_printed_rule_is_not(V, K, k):
    """Candidates drawn one after the other without replacement (every ordered k-tuple of distinct tokens of
    the set, weight prod_i q_hat(x_i) / (1 - sum_{j<i} q_hat(x_j))): with the proposal of every stage
    renormalised over what is left the output is distributed as P; Algorithm 5 as printed (q_hat at every
    stage) is exact only for i.i.d. candidates and misses P on these."""
    t, tr, p, qh, qs = case(70 + V + k, V, K)
    nr = 1500
    tuples = []
    for tup in itertools.permutations(range(K), k):
        w, left = 1.0, 1.0
        for s in tup:
            w *= qs[s] / left
            left -= qs[s]
        tuples.append(([int(tr["idx"][s]) for s in tup], w))
    assert abs(sum(w for _, w in tuples) - 1.0) < 1e-12
    exact = mcveri_output_distribution(p, tr, qs, tuples, k, V, True, nr)
    np.testing.assert_allclose(exact, p, atol=2.0 / nr * V)
    # a target that is far below q_hat on the likeliest token of the set and just above it on the others:
    # after the first rejection those others are over-proposed, later stages still reject, and there the
    # two rules part
    top = int(np.argmax(qs))
    p_c = np.zeros(V)
    p_c[tr["idx"]] = 1.1 * qs
    p_c[tr["idx"][top]] = 0.2 * qs[top]
    off = np.setdiff1d(np.arange(V), tr["idx"])
    assert p_c.sum() < 1.0 and len(off) > 0
    p_c[off] = (1.0 - p_c.sum()) / len(off)
    exact_c = mcveri_output_distribution(p_c, tr, qs, tuples, k, V, True, nr)
    np.testing.assert_allclose(exact_c, p_c, atol=2.0 / nr * V)
    printed = mcveri_output_distribution(p_c, tr, qs, tuples, k, V, False, nr)
    assert np.abs(printed - p_c).max() > 0.01 > 2 * np.abs(exact_c - p_c).max()
    # the first stage is the same in both rules, and a single candidate makes them identical
    c0 = [tuples[0][0][0]]
    for u in (0.1, 0.6, 0.99):
        a = O.mcveri(p, tr["idx"], qs, c0, [u], 0.3, True)
        b = O.mcveri(p, tr["idx"], qs, c0, [u], 0.3, False)
        assert a["token"] == b["token"] and a["slot"] == b["slot"] and a["ratio"][0] == b["ratio"][0]


def test_mcveri_without_replacement_stage_proposal():
    """Stage 2's ratio uses q_hat renormalised without the first candidate: p^(2)(x2) / (q_hat(x2) / (1 - q_hat(x1)))."""
    V, K = 9, 4
    t, tr, p, qh, qs = case(3, V, K)
    order = np.argsort(p[tr["idx"]] / qs)            # most over-proposed first: certainly rejectable
    x1, x2 = int(tr["idx"][order[0]]), int(tr["idx"][order[1]])
    r = O.mcveri(p, tr["idx"], qs, [x1, x2], [0.99999994, 0.99999994], 0.5, True)
    p2 = residual_dist(p, qh)
    q2 = qh.copy(); q2[x1] = 0.0; q2 /= q2.sum()
    assert abs(r["ratio"][1] - p2[x2] / q2[x2]) < 1e-14
    assert abs(r["betas"][1] - np.minimum(q2, p2).sum()) < 1e-14
    # a candidate that was drawn before cannot be drawn again: flagged and rejected
    d = O.mcveri(p, tr["idx"], qs, [x1, x1], [0.99999994, 0.0], 0.5, True)
    assert d["status"] & O.STATUS_TOKEN_NOT_IN_SET and d["slot"] == -1 and d["ratio"][1] == -1.0


def test_mcveri_reports_stage_betas_and_duplicates_are_rejected():
    V, K = 9, 4
    t, tr, p, qh, qs = case(3, V, K)
    worst = int(tr["idx"][np.argmin(p[tr["idx"]] / qs)])          # a candidate with ratio < 1
    r = O.mcveri(p, tr["idx"], qs, [worst, worst, worst], [0.99999994] * 3, 0.25)
    # once rejected, p^(2)(x) = 0 so a repeat has ratio 0 and is rejected for every u
    assert r["ratio"][1] == 0.0 and r["ratio"][2] == 0.0 and r["slot"] == -1
    r2 = O.mcveri(p, tr["idx"], qs, [worst, worst], [0.99999994, 0.0], 0.25)
    assert r2["slot"] == -1
    p2 = residual_dist(p, qh)
    assert abs(r["betas"][0] - np.minimum(qh, p).sum()) < 1e-14
    assert abs(r["betas"][1] - np.minimum(qh, p2).sum()) < 1e-14
    # the same rates by candidate number; an absent candidate has none
    r3 = O.mcveri(p, tr["idx"], qs, [worst, -1, worst], [0.99999994] * 3, 0.25)
    assert r3["beta"][0] == r["betas"][0] and np.isnan(r3["beta"][1]) and r3["beta"][2] == r["betas"][1]


def test_single_candidate_mcveri_is_algorithm_3():
    V, K = 30, 8
    rng = np.random.default_rng(12)
    t, tr, p, qh, qs = case(5, V, K)
    bonus = rng.normal(0, 2, V).astype(np.float32)
    for _ in range(200):
        s = int(rng.integers(K))
        ua, ur = np.float32(rng.random()), np.float32(rng.random())
        a = O.mcveri(O.dense_probs(t, 1.0), tr["idx"], O.sparse_probs(tr["logit"], K), [tr["idx"][s]], [ua], ur)
        b = O.verify_chain_seq(np.stack([t, bonus]), 1.0, tr["idx"][None], tr["logit"][None], [K], [tr["idx"][s]],
                               [ua], [ur, ur])
        assert (a["slot"] == 0) == (b["accept_len"] == 1)
        assert a["token"] == b["tokens"][0]
        assert a["ratio"][0] == b["ratio"][0]


def test_tree_identities_of_section_4_1():
    lay = O.tree_layout((4, 4, 4, 4, 4))
    assert lay["widths"] == [1, 4, 16, 64, 256, 1024]
    assert lay["n_internal"] == 341 == 1 + sum(4 ** l for l in range(1, 5))
    assert lay["n_nodes"] == 1365
    for exp in ((2, 2, 2), (3, 1, 2), (1, 1, 1, 1), (2, 3)):
        lay = O.tree_layout(exp)
        W = [int(np.prod(exp[:l])) for l in range(len(exp) + 1)]
        assert lay["widths"] == W
        assert lay["n_internal"] == 1 + sum(int(np.prod(exp[:l])) for l in range(1, len(exp)))
        # children of consecutive nodes of a layer tile the next layer, in order
        seen = []
        for l in range(len(exp)):
            for i in range(W[l]):
                n = int(lay["offsets"][l]) + i
                kids = [O.child_node(lay, exp, n, s) for s in range(exp[l])]
                assert kids == list(range(int(lay["offsets"][l + 1]) + i * exp[l],
                                          int(lay["offsets"][l + 1]) + (i + 1) * exp[l]))
                seen += kids
        assert seen == list(range(1, lay["n_nodes"]))


def build_tree_inputs(seed, V, K, exp, without_replacement=False):
    rng = np.random.default_rng(seed)
    lay = O.tree_layout(exp)
    n_int, n_nodes = lay["n_internal"], lay["n_nodes"]
    z = rng.normal(0, 2, (n_int, V)).astype(np.float32)
    t = rng.normal(0, 2, (n_nodes, V)).astype(np.float32)
    t[:n_int] = (z + rng.normal(0, 0.8, (n_int, V))).astype(np.float32)
    tr = O.truncate(z, 1.0, K, 0.0, K)
    cands = np.full(n_nodes - 1, -1, np.int32)
    for n in range(n_int):
        layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
        k = exp[layer]
        slots, _ = O.sample_row(tr["logit"][n], K, rng.random(k), without_replacement)
        c0 = O.child_node(lay, exp, n, 0)
        cands[c0 - 1:c0 - 1 + k] = tr["idx"][n][slots]
    return lay, t, tr, cands, rng.random(n_nodes - 1).astype(np.float32), rng.random(n_nodes).astype(np.float32)


def test_unary_tree_is_the_chain_with_a_bonus_row():
    V, K, L = 40, 6, 4
    for seed in range(12):
        lay, t, tr, cands, ua, ur = build_tree_inputs(seed, V, K, (1,) * L)
        tree = O.verify_tree_seq(t, 1.0, (1,) * L, tr["idx"], tr["logit"], tr["count"], cands, ua, ur)
        chain = O.verify_chain_seq(t, 1.0, tr["idx"], tr["logit"], tr["count"], cands, ua, ur)
        assert tree["len"] == chain["accept_len"] + 1
        assert np.array_equal(tree["seq"][:tree["len"]], chain["tokens"][:tree["len"]])


@pytest.mark.parametrize("wo", [False, True])
def test_tree_walk_follows_accepted_children(wo):
    V, K, exp = 50, 8, (3, 2, 2)
    for seed in range(10):
        lay, t, tr, cands, ua, ur = build_tree_inputs(100 + seed, V, K, exp, wo)
        r = O.verify_tree_seq(t, 1.0, exp, tr["idx"], tr["logit"], tr["count"], cands, ua, ur)
        assert 1 <= r["len"] <= len(exp) + 1 and len(r["path"]) == r["len"]
        assert r["path"][0] == 0
        for a, b, tok in zip(r["path"][:-1], r["path"][1:], r["seq"]):
            slot = r["node_slot"][a]
            assert slot >= 0 and b == O.child_node(lay, exp, a, slot)
            assert tok == cands[b - 1] == r["node_token"][a]
        last = r["path"][-1]
        assert r["node_slot"][last] == -1 and r["seq"][r["len"] - 1] == r["node_token"][last]
        assert np.all(r["seq"][r["len"]:] == -1)
        # every node's output is defined: leaves carry a target sample, internal nodes an accepted
        # child or a residual sample
        assert np.all(r["node_token"] >= 0)
        assert np.all(r["node_slot"][lay["n_internal"]:] == -1)
        # per-node result equals a direct call of Algorithm 5 on that node
        n = r["path"][-1]
        if n < lay["n_internal"]:
            layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
            c0 = O.child_node(lay, exp, n, 0)
            k = exp[layer]
            d = O.mcveri(O.dense_probs(t[n], 1.0), tr["idx"][n], O.sparse_probs(tr["logit"][n], K),
                         cands[c0 - 1:c0 - 1 + k], ua[c0 - 1:c0 - 1 + k], ur[n])
            assert d["token"] == r["node_token"][n] and d["slot"] == -1
