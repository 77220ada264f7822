"""Helpers shared by the GPU parity tests: run the oracle on host copies, compare element by element.

Tolerances (from the benchmark spec): index sets, counts, accepted lengths and emitted tokens bit-exact,
except (a) sequences in which an acceptance test lies within 1e-6 of its boundary and (b) rows whose
Top-rho decision lies within 1e-6 (relative to the normaliser) of its boundary; for stage i of the
multi-candidate rule the window of (a) is 1e-6 * min(amp, AMP_CAP).  Every class is counted and returned,
and a comparison FAILS when the items its oracle margins flag exceed max(1, 0.5 %) of the items compared:
the margins are pinned on the CPU (tests/test_oracle_margins.py), and a margin or factor that went wrong
would show here as too many flagged items instead of as a green test.  A flagged item is still compared
wherever the GPU took the oracle's decision; only an actual disagreement inside the window is excused.
Compacted logits are the same fp32 product on both sides (compared exactly); probabilities, masses,
ratios and beta within 1e-5 relative (fp32 outputs of fp64 arithmetic).
"""
import math

import numpy as np
import torch

from oracle import tslt_oracle as O

NEAR_TIE = 1e-6
RTOL = 1e-5
# Stage i of Algorithm 5 divides by the normalisers Z_j of the updates before it, so an absolute error of
# p reaches the stage's ratio multiplied by amp = prod 1/Z_j.  1/Z_j has no upper bound; the window is
# widened by at most this factor (the widest window is then 6.4e-5 of the unit interval), and a node
# whose factor is larger is held to the capped window.
AMP_CAP = 64.0
MAX_FLAGGED_SHARE = 0.005


def allowed_flagged(n_items: int) -> int:
    """How many of n_items a comparison may find inside a near-tie window before it fails."""
    return max(1, int(math.ceil(MAX_FLAGGED_SHARE * n_items)))


def to_np(t):
    if isinstance(t, torch.Tensor):
        t = t.detach()
        if t.dtype in (torch.bfloat16, torch.float16):
            t = t.float()
        return t.cpu().numpy()
    return np.asarray(t)


def compare_truncate(gpu: dict, logits_rows, T, top_k, top_p, k_cap, rows=None, label=""):
    """Oracle on the given rows (host fp32 array [n, V]) against the GPU outputs at the same row numbers.
    Returns a dict of counters."""
    logits_rows = to_np(logits_rows)
    n = logits_rows.shape[0]
    rows = np.arange(n) if rows is None else np.asarray(rows)
    g = {k: to_np(v)[rows] for k, v in gpu.items() if v is not None}
    ref = O.truncate(logits_rows, T, top_k, top_p, k_cap)
    # rows the oracle flags, held against what the sizes of the boundary elements explain: rho * Z falls within
    # 1e-6 * Z of a prefix mass with probability about 2e-6 / (mass of the element at the cut)
    flagged = int(np.count_nonzero(ref["margin_rho"] < NEAR_TIE))
    last = np.maximum(ref["count"] - 1, 0)
    w_cut = ref["prob"][np.arange(n), last] * ref["mass"]
    decided = np.isfinite(ref["margin_rho"]) & (w_cut > 0)
    expected = float(np.sum(np.minimum(1.0, 2.0 * NEAR_TIE / w_cut[decided]))) if decided.any() else 0.0
    assert flagged <= allowed_flagged(n) + 3.0 * expected + 3.0 * math.sqrt(expected), \
        (label, "Top-rho decisions inside the near-tie window", flagged, n, expected)
    differ = 0
    exact_path = int(np.count_nonzero(g["status"] & 256))
    for r in range(n):
        tag = f"{label} row {rows[r]}"
        assert (g["status"][r] & 15) == ref["status"][r], (tag, g["status"][r], ref["status"][r])
        if g["count"][r] != ref["count"][r]:
            # only a Top-rho decision at its boundary may differ, and then by the boundary element
            assert ref["margin_rho"][r] < NEAR_TIE, (tag, g["count"][r], ref["count"][r], ref["margin_rho"][r])
            assert abs(int(g["count"][r]) - int(ref["count"][r])) == 1, (tag, g["count"][r], ref["count"][r])
            differ += 1
            c = min(g["count"][r], ref["count"][r])
            assert np.array_equal(g["idx"][r, :c], ref["idx"][r, :c]), tag
            continue
        c = ref["count"][r]
        assert np.array_equal(g["idx"][r], ref["idx"][r]), (tag, g["idx"][r][:8], ref["idx"][r][:8])
        assert np.array_equal(g["logit"][r, :c], ref["logit"][r, :c]), tag
        assert np.all(np.isneginf(g["logit"][r, c:])), tag
        if "prob" in g:
            np.testing.assert_allclose(g["prob"][r], ref["prob"][r], rtol=RTOL, atol=1e-30, err_msg=tag)
        if "mass" in g:
            np.testing.assert_allclose(g["mass"][r], ref["mass"][r], rtol=RTOL, err_msg=tag)
    assert differ <= allowed_flagged(n), (label, "Top-rho decisions that differ inside the window", differ, n)
    return dict(rows=n, exact_index_sets=n - differ, top_p_near_ties=flagged, top_p_near_tie_mismatches=differ,
                exact_path_rows=exact_path, ref=ref)


def compare_verify(gpu: dict, ref: dict, seqs=None, label=""):
    """GPU tslt_verify outputs against oracle verify_chain outputs (already computed) for the sequences
    `seqs` of the GPU batch.  Returns counters."""
    B = ref["accept_len"].shape[0]
    seqs = np.arange(B) if seqs is None else np.asarray(seqs)
    g = {k: to_np(v)[seqs] for k, v in gpu.items() if v is not None}
    flagged = differ = 0
    gamma = ref["ratio"].shape[1]
    for b in range(B):
        tag = f"{label} seq {seqs[b]}"
        n = int(ref["accept_len"][b])
        examined = min(n + 1, gamma)
        if np.any(ref["accept_margin"][b, :examined] < NEAR_TIE):
            flagged += 1
            if g["accept_len"][b] != n:
                # the decision inside the window went the other way: everything after it differs too
                j = int(min(g["accept_len"][b], n))
                assert j < gamma and ref["accept_margin"][b, j] < NEAR_TIE, (tag, g["accept_len"][b], n)
                differ += 1
                continue
        assert g["accept_len"][b] == n, (tag, g["accept_len"][b], n, ref["ratio"][b], g.get("ratio", [None])[b])
        assert np.array_equal(g["tokens"][b], ref["tokens"][b]), (tag, g["tokens"][b], ref["tokens"][b],
                                                                  ref["cdf_margin"][b])
        assert (g["status"][b] & 15) == ref["status"][b], (tag, g["status"][b], ref["status"][b])
        if "ratio" in g and ref["status"][b] == 0:
            rr = ref["ratio"][b, :examined]
            np.testing.assert_allclose(g["ratio"][b, :examined], rr, rtol=RTOL, atol=1e-30, err_msg=tag)
            np.testing.assert_allclose(g["beta"][b, :examined], ref["beta_hat"][b, :examined], rtol=RTOL, err_msg=tag)
    assert flagged <= allowed_flagged(B), (label, "sequences with an acceptance test inside the near-tie window", flagged, B)
    return dict(sequences=B, exact_sequences=B - differ, accept_near_ties=flagged, accept_near_tie_mismatches=differ)


def oracle_chain(draft_rows, target_rows, T, top_k, top_p, k_cap, u_sample, u_accept, u_resample):
    """The whole single-candidate round on the host: truncate every draft row, sample the draft token,
    verify.  draft_rows [B, gamma, V], target_rows [B, gamma+1, V] as fp32 numpy."""
    B, G, V = draft_rows.shape
    tr = O.truncate(draft_rows.reshape(B * G, V), T, top_k, top_p, k_cap)
    smp = O.sample(tr["idx"], tr["logit"], tr["count"], np.asarray(u_sample).reshape(B * G, 1))
    q_idx = tr["idx"].reshape(B, G, k_cap)
    q_logit = tr["logit"].reshape(B, G, k_cap)
    q_count = tr["count"].reshape(B, G)
    tokens = smp["token"].reshape(B, G)
    ver = O.verify_chain(target_rows, T, q_idx, q_logit, q_count, tokens, np.asarray(u_accept), np.asarray(u_resample))
    return dict(trunc=tr, tokens=tokens, q_idx=q_idx, q_logit=q_logit, q_count=q_count, verify=ver)


def oracle_tree(draft_rows, target_rows, T, top_k, top_p, k_cap, expansion, u_sample, u_accept, u_resample,
                without_replacement, renormalised_rule=False):
    """The whole multi-candidate round on the host (Algorithms 7's sampling and 8): truncate every non-leaf
    node's draft row, draw its k candidates, verify the tree.  draft_rows [B, N_int, V], target_rows
    [B, N_nodes, V] fp32 numpy; u_sample [B, N_int, k_max].  without_replacement says how the candidates are
    drawn, renormalised_rule which verification rule is applied (the printed one, or the one for candidates
    drawn without replacement)."""
    B, n_int, V = draft_rows.shape
    lay = O.tree_layout(expansion)
    n_nodes = lay["n_nodes"]
    tr = O.truncate(draft_rows.reshape(B * n_int, V), T, top_k, top_p, k_cap)
    q_idx = tr["idx"].reshape(B, n_int, k_cap)
    q_logit = tr["logit"].reshape(B, n_int, k_cap)
    q_count = tr["count"].reshape(B, n_int)
    cands = np.full((B, n_nodes - 1), -1, np.int32)
    for b in range(B):
        for n in range(n_int):
            layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
            k = int(expansion[layer])
            slots, _ = O.sample_row(q_logit[b, n], int(q_count[b, n]), np.asarray(u_sample)[b, n, :k], without_replacement)
            c0 = O.child_node(lay, expansion, n, 0)
            ok = slots >= 0
            cands[b, c0 - 1:c0 - 1 + k][ok] = q_idx[b, n][slots[ok]]
    ver = O.verify_tree(target_rows, T, expansion, q_idx, q_logit, q_count, cands, np.asarray(u_accept),
                        np.asarray(u_resample), renormalised_rule)
    return dict(trunc=tr, q_idx=q_idx, q_logit=q_logit, q_count=q_count, cands=cands, verify=ver, layout=lay)


def compare_tree(gpu: dict, ref: dict, expansion, all_nodes=True, label=""):
    """GPU tslt_verify_tree outputs against the oracle's.  A node is flagged when one of its acceptance tests
    lies within 1e-6 * min(amp, AMP_CAP) of its boundary.  A flagged node whose accepted child differs from the
    oracle's is excused (its token then differs too), and so is the verified sequence of a tree whose path
    crosses such a node; every other node and sequence is compared bit for bit.  Flagged nodes, excused nodes
    and excused sequences are counted, and too many of any fail the comparison.
    amp = prod_{j<i} 1/Z_j is the factor by which the i-th candidate's ratio magnifies an error in p (each
    residual update divides by its normaliser Z_j < 1); it is 1 for the first candidate, which is the
    single-candidate rule.  Ratios are compared to the same scale."""
    v = ref["verify"]
    lay = ref["layout"]
    n_int, n_nodes = lay["n_internal"], lay["n_nodes"]
    g = {k: to_np(x) for k, x in gpu.items() if x is not None}
    B = v["seq"].shape[0]
    near_nodes = differ_nodes = differ_seqs = 0
    amp = np.minimum(v["amp"], AMP_CAP)
    for b in range(B):
        tag = f"{label} tree {b}"
        risky = np.zeros(n_nodes, bool)
        for n in range(n_int):
            layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
            c0 = O.child_node(lay, expansion, n, 0)
            sl = slice(c0 - 1, c0 - 1 + expansion[layer])
            if np.any(v["accept_margin"][b, sl] < NEAR_TIE * amp[b, sl]):
                risky[n] = True
        near_nodes += int(risky.sum())
        same_seq = g["len"][b] == v["len"][b] and np.array_equal(g["seq"][b], v["seq"][b])
        if all_nodes:
            excused = risky & (g["node_slot"][b] != v["node_slot"][b])
            okn = ~excused
            assert np.array_equal(g["node_slot"][b][okn], v["node_slot"][b][okn]), tag
            assert np.array_equal(g["node_token"][b][okn], v["node_token"][b][okn]), \
                (tag, np.nonzero(g["node_token"][b] != v["node_token"][b])[0][:8])
            if not excused.any():
                assert (g["status"][b] & 15) == v["status"][b], (tag, g["status"][b], v["status"][b])
            differ_nodes += int(excused.sum())
            seq_excused = any(excused[n] for n in v["path"][b])
        else:
            # only the path is known: a differing sequence is excused if the oracle's path crosses a flagged node
            seq_excused = (not same_seq) and any(risky[n] for n in v["path"][b])
        if seq_excused:
            differ_seqs += 1
            continue
        assert g["len"][b] == v["len"][b], (tag, g["len"][b], v["len"][b])
        assert np.array_equal(g["seq"][b], v["seq"][b]), (tag, g["seq"][b], v["seq"][b])
        if "ratio" in g:
            tested = ~np.isnan(v["ratio"][b])
            for n in range(n_int):
                if risky[n]:
                    layer = int(np.searchsorted(lay["offsets"], n, side="right")) - 1
                    c0 = O.child_node(lay, expansion, n, 0)
                    tested[c0 - 1:c0 - 1 + expansion[layer]] = False
            err = np.abs(g["ratio"][b][tested] - v["ratio"][b][tested])
            bound = RTOL * np.abs(v["ratio"][b][tested]) + NEAR_TIE * amp[b][tested]
            assert np.all(err <= bound), (tag, float(np.max(err / bound)))
            if "beta" in g:
                # stage acceptance rates, to the same scale; NaN exactly where the oracle tested nothing
                assert np.array_equal(np.isnan(g["beta"][b][tested]), np.isnan(v["beta"][b][tested])), tag
                err = np.abs(g["beta"][b][tested] - v["beta"][b][tested])
                bound = RTOL * np.abs(v["beta"][b][tested]) + NEAR_TIE * amp[b][tested]
                assert np.all(err <= bound), (tag, "beta", float(np.max(err / bound)))
    assert near_nodes <= allowed_flagged(B * n_int), (label, "nodes with a test inside the near-tie window", near_nodes, B * n_int)
    assert differ_seqs <= allowed_flagged(B), (label, "trees excused", differ_seqs, B)
    return dict(trees=B, exact_sequences=B - differ_seqs, near_tie_nodes=near_nodes, near_tie_node_mismatches=differ_nodes,
                near_tie_sequences=differ_seqs, amp_max=float(np.max(v["amp"])) if v["amp"].size else 1.0)
