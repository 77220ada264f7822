"""Pins for the oracle outputs that excuse a parity mismatch (no GPU): margin_rho, accept_margin, amp, and
the inverse-CDF margin.

The GPU comparisons leave out a Top-rho decision whose margin is below 1e-6, a sequence whose acceptance
test lies within 1e-6 of its boundary, and a tree node whose stage-i test lies within 1e-6 * amp.  A margin
that came out 0, or an amp that came out huge, would make those comparisons pass on anything, so each of
the three is held here to hand-built cases whose value follows from the definitions of Section 3.1 (Top-rho
prefix masses), Algorithm 3 (the bound min(1, p/q_hat)) and Algorithm 5's residual update (its normaliser
Z_j) by arithmetic on small exact fractions.
"""
import numpy as np
import pytest

from oracle import tslt_oracle as O

NEG = -np.inf


# ----------------------------------------------------------------------------------------------
# margin_rho: distance of rho * Z to the prefix masses on either side of the cut, relative to Z
# ----------------------------------------------------------------------------------------------
def test_margin_rho_equal_logits_closed_form():
    # five logits equal to 0, the rest masked: e = (1,1,1,1,1), Z = 5, prefix masses 1..5.  rho = 0.5:
    # rho*Z = 2.5, the cut is after 3 entries; the nearest prefix masses are 3 and 2: margin = 0.5/5
    z = np.full(12, NEG, np.float32)
    z[[1, 4, 6, 7, 10]] = 0.0
    t = O.truncate_row(z, 1.0, 0, 0.5, 12)
    assert t["count"] == 3 and t["idx"].tolist() == [1, 4, 6]
    assert t["margin_rho"] == 0.1
    # rho = 0.75: rho*Z = 3.75, cut after 4; distances 0.25 and 0.75 -> 0.05
    t = O.truncate_row(z, 1.0, 0, 0.75, 12)
    assert t["count"] == 4 and t["margin_rho"] == 0.05
    # a decision exactly on its boundary: rho*Z = 2.5 with Z = 5 was not; rho = 0.5 over FOUR equal logits is:
    # rho*Z = 2 = C_2, so ">=" keeps 2 entries and the margin is exactly 0
    z4 = np.array([0.0, NEG, 0.0, 0.0, 0.0], np.float32)
    t = O.truncate_row(z4, 1.0, 0, 0.5, 5)
    assert t["count"] == 2 and t["margin_rho"] == 0.0


def test_margin_rho_geometric_weights():
    # logits ln(8), ln(4), ln(2), 0, 0 (fp32): e/e_0 = 1, 1/2, 1/4, 1/8, 1/8, Z = 2, prefix masses
    # 1, 1.5, 1.75, 1.875, 2.  rho = 0.8: rho*Z = 1.6 -> cut after 3; distances 0.15 and 0.1 -> 0.05
    z = np.log(np.array([2.0, 8.0, 1.0, 4.0, 1.0])).astype(np.float32)
    t = O.truncate_row(z, 1.0, 0, 0.8, 5)
    assert t["idx"].tolist() == [1, 3, 0] and t["count"] == 3
    rho32 = float(np.float32(0.8))
    assert abs(t["margin_rho"] - min(1.75 - 2 * rho32, 2 * rho32 - 1.5) / 2.0) < 1e-7
    assert abs(t["margin_rho"] - 0.05) < 1e-7
    # temperature 0.5 squares the weights: 1, 1/4, 1/16, 1/64, 1/64; Z = 1.34375; rho = 0.9 -> 1.209375:
    # cut after 2 (C_2 = 1.25); distances 0.040625 and 0.209375
    t = O.truncate_row(z, 0.5, 0, 0.9, 5)
    assert t["count"] == 2
    rho32 = float(np.float32(0.9))
    assert abs(t["margin_rho"] - (1.25 - rho32 * 1.34375) / 1.34375) < 1e-6


def test_margin_rho_when_the_cap_or_top_k_binds():
    z = np.full(12, NEG, np.float32)
    z[[1, 4, 6, 7, 10]] = 0.0
    # the nucleus wants 3 entries (rho*Z = 2.5), the cap allows 2: the count can only change if the nucleus
    # drops to 2 or fewer, i.e. if rho*Z falls to C_2 = 2 (distance 0.5) or C_1 = 1 (1.5) -> 0.5/5
    t = O.truncate_row(z, 1.0, 0, 0.5, 2)
    assert t["count"] == 2 and t["margin_rho"] == 0.1
    t = O.truncate_row(z, 1.0, 1, 0.5, 12)             # top-k 1 binds: only C_1 = 1 matters, 1.5/5
    assert t["count"] == 1 and t["margin_rho"] == pytest.approx(0.3, abs=1e-15)
    # no nucleus test: nothing to be near
    assert O.truncate_row(z, 1.0, 3, 0.0, 12)["margin_rho"] == np.inf
    assert O.truncate_row(z, 1.0, 0, 1.0, 12)["margin_rho"] == np.inf


def test_margin_rho_tells_a_flipped_decision():
    """The margin is what a relative error in Z has to exceed to change the count: scaling the threshold by
    (1 -+ 2*margin) flips it, by (1 -+ margin/2) does not."""
    rng = np.random.default_rng(5)
    for trial in range(40):
        z = rng.normal(0, 2.5, 200).astype(np.float32)
        rho = float(rng.uniform(0.3, 0.97))
        t = O.truncate_row(z, 1.0, 0, rho, 200)
        mg = t["margin_rho"]
        assert 0 < mg < 1
        s = O.scale(z, 1.0).astype(np.float64)
        e = np.sort(np.exp(s - s.max()))[::-1]
        C, Z = np.cumsum(e), e.sum()
        thr = float(np.float32(rho)) * Z
        def count_at(th):
            return int(np.nonzero(C >= th)[0][0]) + 1
        assert count_at(thr) == t["count"]
        assert count_at(thr + 0.5 * mg * Z) == t["count"] == count_at(thr - 0.5 * mg * Z)
        assert count_at(thr + 2.0 * mg * Z) != t["count"] or count_at(thr - 2.0 * mg * Z) != t["count"]


# ----------------------------------------------------------------------------------------------
# accept_margin: |u - min(1, p(x) / q_hat(x))|
# ----------------------------------------------------------------------------------------------
def chain_one(target_row, q_idx, q_logit, x, u_acc, u_res=0.5):
    V = len(target_row)
    rows = np.stack([np.asarray(target_row, np.float32), np.zeros(V, np.float32)])
    k = len(q_idx)
    return O.verify_chain_seq(rows, 1.0, np.asarray([q_idx]), np.asarray([q_logit], np.float32), [k], [x], [u_acc],
                              [u_res, 0.5])


def test_accept_margin_closed_form():
    # p = (1/4, 1/4, 1/4, 1/4) (four equal target logits), q_hat = (1/2, 1/2) on {0, 1}: ratio 1/2 exactly
    p_row = [0.0, 0.0, 0.0, 0.0]
    for u, accepted in ((0.4999, True), (0.5001, False), (0.25, True), (0.0, True)):
        r = chain_one(p_row, [0, 1], [1.5, 1.5], 0, u)
        assert r["ratio"][0] == 0.5
        assert r["accept_len"] == (1 if accepted else 0)
        assert r["accept_margin"][0] == abs(float(np.float32(u)) - 0.5)
    assert abs(chain_one(p_row, [0, 1], [1.5, 1.5], 0, 0.4999)["accept_margin"][0] - 1e-4) < 5e-8      # u is an fp32 number
    # exactly on the boundary: u = 1/2 is not < 1/2 -> rejected, margin 0
    r = chain_one(p_row, [0, 1], [1.5, 1.5], 1, 0.5)
    assert r["accept_len"] == 0 and r["accept_margin"][0] == 0.0
    # a ratio above 1 is cut to 1: p = (1/2, 1/2, 0, 0), q_hat = 1/4 each on four tokens -> ratio 2, bound 1
    r = chain_one([0.0, 0.0, NEG, NEG], [0, 1, 2, 3], [0.0, 0.0, 0.0, 0.0], 1, 0.75)
    assert r["ratio"][0] == 2.0 and r["accept_len"] == 1 and r["accept_margin"][0] == 0.25
    # p = (1/4, 3/4) and q_hat = (1/2, 1/2): ratios 1/2 and 3/2 (logits ln 3 and 0, rounded to fp32)
    row = np.array([0.0, np.log(3.0)], np.float32)
    r = chain_one(row, [0, 1], [0.0, 0.0], 0, 0.4999)
    assert abs(r["ratio"][0] - 0.5) < 1e-7 and abs(r["accept_margin"][0] - 1e-4) < 1e-7 and r["accept_len"] == 1
    r = chain_one(row, [1, 0], [0.0, 0.0], 1, 0.9)
    assert abs(r["ratio"][0] - 1.5) < 1e-6 and abs(r["accept_margin"][0] - 0.1) < 1e-7


def test_accept_margin_only_for_examined_positions():
    # positions after the first rejection are never examined: their margin stays +inf, and so does that of a
    # token outside its set (no ratio to be near to)
    V = 4
    target = np.zeros((4, V), np.float32)
    q_idx = np.array([[0, 1], [0, 1], [0, 1]])
    q_logit = np.zeros((3, 2), np.float32)
    r = O.verify_chain_seq(target, 1.0, q_idx, q_logit, [2, 2, 2], [0, 1, 0], [0.1, 0.7, 0.1], [0.5] * 4)
    assert r["accept_len"] == 1
    assert r["accept_margin"][0] == pytest.approx(0.4) and r["accept_margin"][1] == pytest.approx(0.2, abs=1e-7)
    assert r["accept_margin"][2] == np.inf
    r = O.verify_chain_seq(target, 1.0, q_idx, q_logit, [2, 2, 2], [3, 1, 0], [0.1, 0.7, 0.1], [0.5] * 4)
    assert r["accept_len"] == 0 and r["status"] & O.STATUS_TOKEN_NOT_IN_SET and r["accept_margin"][0] == np.inf


# ----------------------------------------------------------------------------------------------
# amp: the factor prod_{j<i} 1/Z_j in front of candidate i's ratio (Z_j the normaliser of update j)
# ----------------------------------------------------------------------------------------------
def test_amp_is_the_product_of_inverse_residual_normalisers():
    # p = (.4, .1, .3, .2), q_hat = (.3 on token 0, .7 on token 2).
    # stage 1, candidate 2: ratio .3/.7, rejected at u = .9; residual (.1, .1, 0, .2), Z_1 = .4
    #   -> p2 = (.25, .25, 0, .5)
    # stage 2, candidate 0: ratio .25/.3, rejected at u = .9; residual (0, .25, 0, .5), Z_2 = .75
    #   -> p3 = (0, 1/3, 0, 2/3)
    # stage 3, candidate 2 again: ratio 0
    p = np.array([0.4, 0.1, 0.3, 0.2])
    r = O.mcveri(p, [0, 2], np.array([0.3, 0.7]), [2, 0, 2], [0.9, 0.9, 0.9], 0.5)
    assert r["slot"] == -1
    np.testing.assert_allclose(r["amp"], [1.0, 1 / 0.4, 1 / 0.4 / 0.75], rtol=1e-14)
    np.testing.assert_allclose(r["ratio"], [0.3 / 0.7, 0.25 / 0.3, 0.0], rtol=1e-14, atol=1e-16)
    u9 = float(np.float32(0.9))                             # the uniforms are fp32 numbers
    np.testing.assert_allclose(r["accept_margin"], [u9 - 0.3 / 0.7, u9 - 0.25 / 0.3, u9], rtol=1e-13)
    # the all-rejected output is a sample of p3: u = .5 > 1/3 -> token 3
    assert r["token"] == 3
    # an accepted candidate ends the recursion: later entries keep amp 1, margin inf
    r = O.mcveri(p, [0, 2], np.array([0.3, 0.7]), [2, 0, 2], [0.9, 0.1, 0.9], 0.5)
    assert r["slot"] == 1 and r["token"] == 0
    np.testing.assert_allclose(r["amp"], [1.0, 2.5, 1.0], rtol=1e-14)
    assert r["accept_margin"][2] == np.inf
    # an absent candidate (-1) is no stage: the next one sees the same distribution and the same factor
    r = O.mcveri(p, [0, 2], np.array([0.3, 0.7]), [2, -1, 0], [0.9, 0.9, 0.9], 0.5)
    np.testing.assert_allclose(r["amp"], [1.0, 1.0, 2.5], rtol=1e-14)
    np.testing.assert_allclose(r["ratio"][[0, 2]], [0.3 / 0.7, 0.25 / 0.3], rtol=1e-14)


def test_amp_without_replacement_uses_the_stage_proposal():
    # candidates drawn without replacement: after candidate 2 is rejected the proposal is q_hat without token 2,
    # renormalised: (1 on token 0).  Z_1 = .4 as above; stage 2: ratio .25/1, residual (0, .25, 0, .5) -> Z_2 = .75
    p = np.array([0.4, 0.1, 0.3, 0.2])
    r = O.mcveri(p, [0, 2], np.array([0.3, 0.7]), [2, 0], [0.9, 0.9], 0.2, without_replacement=True)
    np.testing.assert_allclose(r["amp"], [1.0, 2.5], rtol=1e-14)
    np.testing.assert_allclose(r["ratio"], [0.3 / 0.7, 0.25], rtol=1e-14)
    assert r["slot"] == -1 and r["token"] == 1          # p3 = (0, 1/3, 0, 2/3), u = .2 < 1/3


def test_amp_bounds_the_ratio_error_of_a_perturbed_p():
    """What amp is for: an absolute error d in p moves the stage-i ratio by about amp_i * d / q(x).  Checked by
    perturbing p and running the recursion again."""
    rng = np.random.default_rng(3)
    V, K, k = 40, 6, 4
    for trial in range(30):
        p = rng.dirichlet(np.ones(V) * 0.3)
        ids = rng.choice(V, K, replace=False)
        q = rng.dirichlet(np.ones(K))
        cands = rng.choice(ids, k)
        base = O.mcveri(p, ids, q, cands, [1.0] * k, 0.5)           # u = 1 rejects everything: all stages run
        d = 1e-9
        pp = p.copy()
        pp[cands[-1]] += d
        pert = O.mcveri(pp / pp.sum(), ids, q, cands, [1.0] * k, 0.5)
        for i in range(k):
            if base["ratio"][i] > 0 and pert["ratio"][i] > 0:
                qx = q[np.nonzero(ids == cands[i])[0][0]]
                assert abs(pert["ratio"][i] - base["ratio"][i]) <= 4.0 * base["amp"][i] * d / qx + 1e-15
        assert np.all(np.diff(base["amp"]) >= -1e-12)                 # every Z_j <= 1: the factor never shrinks


def test_tree_reports_the_node_margins_and_factors():
    # a depth-1 tree with 3 candidates is one MCVeri call: verify_tree_seq passes its amp and margins through
    V = 4
    target = np.log(np.array([[0.4, 0.1, 0.3, 0.2]] * 4)).astype(np.float32)
    q_idx = np.array([[0, 2]])
    q_logit = np.log(np.array([[0.3, 0.7]])).astype(np.float32)
    q_logit = q_logit[:, ::-1].copy(); q_idx = q_idx[:, ::-1].copy()         # canonical order: larger first
    r = O.verify_tree_seq(target, 1.0, [3], q_idx, q_logit, [2], [2, 0, 2], [0.9, 0.9, 0.9], [0.5] * 4)
    np.testing.assert_allclose(r["amp"], [1.0, 2.5, 2.5 / 0.75], rtol=1e-6)
    np.testing.assert_allclose(r["accept_margin"], [0.9 - 0.3 / 0.7, 0.9 - 0.25 / 0.3, 0.9], rtol=2e-6)
    assert r["node_slot"][0] == -1 and r["len"] == 1


# ----------------------------------------------------------------------------------------------
# cdf_margin: distance of u * total to the nearer edge of the chosen bucket, relative to the total
# ----------------------------------------------------------------------------------------------
def test_cdf_margin_closed_form():
    w = np.array([1.0, 0.0, 2.0, 1.0])                      # edges 0, 1, 1, 3, 4
    for u, bucket, margin in ((0.125, 0, 0.125), (0.25, 2, 0.0), (0.5, 2, 0.25), (0.6875, 2, 0.0625), (0.75, 3, 0.0),
                              (0.875, 3, 0.125)):
        y, mg = O.inverse_cdf(w, u)
        assert (y, mg) == (bucket, margin), (u, y, mg)
    assert O.inverse_cdf(np.zeros(3), 0.3) == (-1, np.inf)
