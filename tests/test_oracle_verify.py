"""Pins for the oracle's single-candidate verification (Algorithm 3), no GPU.

The checks are the paper's guarantees, evaluated independently of the oracle's own arithmetic:
Lemma 1 (acceptance rate = sum min(q_hat, p)), losslessness (the verified token is distributed as
p whatever q_hat is, Section 3.2) by exhaustive enumeration at V <= 16, Theorem 1's sigma = 0 case,
and N_oracle = (1 - a^{L+1}) / (1 - a) of Section 2.3.
"""
import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import tslt_oracle as O


def make_case(seed, V, K, T=1.0, noise=1.0):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 2.0, V).astype(np.float32)
    t = (z + rng.normal(0, noise, V)).astype(np.float32)
    tr = O.truncate_row(z, T, K, 0.0, K)
    p = sp_softmax(O.scale(t, T).astype(np.float64))
    qh = np.zeros(V)
    qh[tr["idx"]] = sp_softmax(tr["logit"].astype(np.float64))
    return z, t, tr, p, qh


def run_one(t_rows, T, tr, x, u_acc, u_res):
    """One-position chain (gamma = 1) through the oracle; t_rows = [row, bonus row]."""
    k = tr["count"]
    return O.verify_chain_seq(np.stack(t_rows), T, tr["idx"][None, :], tr["logit"][None, :], [k], [x],
                              [u_acc], u_res)


@pytest.mark.parametrize("V,K,T", [(12, 5, 1.0), (16, 16, 0.7), (9, 1, 1.0), (16, 3, 1.3)])
def test_output_distribution_is_p_by_enumeration(V, K, T):
    z, t, tr, p, qh = make_case(21 + V + K, V, K, T)
    bonus = np.zeros(V, np.float32)
    na, nr = 400, 2000
    ga, gr = (np.arange(na) + 0.5) / na, (np.arange(nr) + 0.5) / nr
    out = np.zeros(V)
    acc_total = 0.0
    for x in tr["idx"]:
        acc = 0
        for ua in ga:
            r = run_one([t, bonus], T, tr, x, ua, [0.5, 0.5])
            acc += r["accept_len"]
            if r["accept_len"] == 1:
                assert r["tokens"][0] == x
        frac = acc / na
        # Lemma 1's integrand: P(accept | x) = min(1, p/q_hat)
        assert abs(frac - min(1.0, p[x] / qh[x])) <= 1.0 / na
        acc_total += qh[x] * frac
        out[x] += qh[x] * frac
        if frac < 1.0:
            res = np.zeros(V)
            for ur in gr:
                r = run_one([t, bonus], T, tr, x, 0.9999999, [ur, 0.5])
                assert r["accept_len"] == 0
                y = r["tokens"][0]
                assert p[y] > qh[y] and y != x      # a residual sample has p > q_hat there
                res[y] += 1
            out += qh[x] * (1 - frac) * res / nr
    # losslessness: the emitted token is distributed as p
    np.testing.assert_allclose(out, p, atol=3.0 / na)
    # Lemma 1: beta_hat = sum min(q_hat, p) = 1 - TV(q_hat, p)
    beta_hat = np.minimum(qh, p).sum()
    assert abs(acc_total - beta_hat) <= 1.0 / na
    assert abs(beta_hat - (1 - 0.5 * np.abs(qh - p).sum())) < 1e-13
    r = run_one([t, bonus], T, tr, tr["idx"][0], 0.5, [0.5, 0.5])
    assert abs(r["beta_hat"][0] - beta_hat) < 1e-13
    # residual shortcut: sum max(0, p - q_hat) = 1 - sum_S min(p, q_hat)
    assert abs(np.maximum(0, p - qh).sum() - (1 - beta_hat)) < 1e-13


def test_bonus_token_is_a_sample_of_the_last_row():
    V = 10
    z, t, tr, p, qh = make_case(5, V, V)
    bonus = np.random.default_rng(1).normal(0, 2, V).astype(np.float32)
    pb = sp_softmax(bonus.astype(np.float64))
    x = int(tr["idx"][0])
    n = 4000
    cnt = np.zeros(V)
    for ur in (np.arange(n) + 0.5) / n:
        r = run_one([t, bonus], 1.0, tr, x, 0.0, [0.5, ur])     # u_acc = 0 always accepts
        assert r["accept_len"] == 1 and r["tokens"][0] == x
        cnt[r["tokens"][1]] += 1
    np.testing.assert_allclose(cnt / n, pb, atol=2.0 / n * V)


def test_support_covering_truncation_changes_nothing():
    """sigma = 0 when the kept set covers q's support (Theorem 1): beta_hat = beta and the decisions
    with and without truncation coincide."""
    V, S = 64, 6
    rng = np.random.default_rng(3)
    z = np.full(V, -np.inf, np.float32)
    sup = rng.choice(V, S, replace=False)
    z[sup] = rng.normal(0, 2, S).astype(np.float32)
    t = rng.normal(0, 2, V).astype(np.float32)
    bonus = rng.normal(0, 2, V).astype(np.float32)
    small = O.truncate_row(z, 0.9, S, 0.0, S)
    full = O.truncate_row(z, 0.9, 0, 0.0, V)
    assert small["count"] == full["count"] == S and abs(small["mass"] - 1.0) < 1e-15
    assert np.array_equal(small["idx"], full["idx"])
    p = sp_softmax(O.scale(t, 0.9).astype(np.float64))
    q = sp_softmax(O.scale(z, 0.9).astype(np.float64))
    qh = np.zeros(V)
    qh[small["idx"]] = small["prob"]
    assert abs(np.minimum(q, p).sum() - np.minimum(qh, p).sum()) < 1e-14
    for x in small["idx"]:
        for ua, ur in rng.random((40, 2)):
            a = run_one([t, bonus], 0.9, small, x, ua, [ur, ur])
            b = run_one([t, bonus], 0.9, full, x, ua, [ur, ur])
            assert a["accept_len"] == b["accept_len"] and np.array_equal(a["tokens"], b["tokens"])


def test_accept_rule_edges_and_status():
    V = 8
    z, t, tr, p, qh = make_case(8, V, 4)
    bonus = np.zeros(V, np.float32)
    # ratio >= 1 accepts for every u in [0, 1)
    x_hi = [x for x in tr["idx"] if p[x] >= qh[x]]
    if x_hi:
        r = run_one([t, bonus], 1.0, tr, x_hi[0], np.float32(1) - np.float32(2 ** -24), [0.5, 0.5])
        assert r["accept_len"] == 1 and r["ratio"][0] >= 1
    # strictness: u equal to the ratio rejects.  p = (1/4, 3/4), q_hat = (1/2, 1/2) -> ratio 1/2
    t2 = np.log(np.array([1.0, 3.0])).astype(np.float32)
    tr2 = dict(idx=np.array([0, 1]), logit=np.zeros(2, np.float32), count=2)
    r = O.verify_chain_seq(np.stack([t2, t2]), 1.0, tr2["idx"][None], tr2["logit"][None], [2], [0], [0.4999],
                           [0.5, 0.5])
    assert r["accept_len"] == 1 and abs(r["ratio"][0] - 0.5) < 1e-7
    r = O.verify_chain_seq(np.stack([t2, t2]), 1.0, tr2["idx"][None], tr2["logit"][None], [2], [0], [0.5001],
                           [0.5, 0.5])
    assert r["accept_len"] == 0 and r["tokens"][0] == 1 and r["tokens"][1] == -1
    # a draft token outside its set is rejected and flagged; the residual then is max(0, p - q_hat)
    outside = int(np.setdiff1d(np.arange(V), tr["idx"])[0])
    r = run_one([t, bonus], 1.0, tr, outside, 0.0, [0.5, 0.5])
    assert r["accept_len"] == 0 and r["status"] & O.STATUS_TOKEN_NOT_IN_SET
    # broken target row
    tb = t.copy()
    tb[2] = np.nan
    r = run_one([tb, bonus], 1.0, tr, int(tr["idx"][0]), 0.0, [0.5, 0.5])
    assert r["status"] & O.STATUS_NONFINITE and r["tokens"][0] == -1


def test_first_rejection_stops_the_chain_and_batch_wrapper():
    V, G, K = 20, 5, 6
    rng = np.random.default_rng(17)
    z = rng.normal(0, 2, (G, V)).astype(np.float32)
    t = np.concatenate([z + rng.normal(0, 1, (G, V)), rng.normal(0, 2, (1, V))]).astype(np.float32)
    tr = O.truncate(z, 1.0, K, 0.0, K)
    toks = tr["idx"][:, 0]
    u_acc = np.array([0.0, 0.0, 0.9999999, 0.0, 0.0], np.float32)
    u_res = rng.random(G + 1).astype(np.float32)
    ratios = O.verify_chain_seq(t, 1.0, tr["idx"], tr["logit"], tr["count"], toks, np.zeros(G), u_res)["ratio"]
    r = O.verify_chain_seq(t, 1.0, tr["idx"], tr["logit"], tr["count"], toks, u_acc, u_res)
    if ratios[2] < 1:
        assert r["accept_len"] == 2 and list(r["tokens"][:2]) == list(toks[:2])
        assert r["tokens"][2] >= 0 and np.all(r["tokens"][3:] == -1)
        assert np.isnan(r["ratio"][3:]).all()
    all_acc = O.verify_chain_seq(t, 1.0, tr["idx"], tr["logit"], tr["count"], toks, np.zeros(G), u_res)
    assert all_acc["accept_len"] == G and all_acc["tokens"][G] >= 0
    batch = O.verify_chain(np.stack([t, t]), 1.0, np.stack([tr["idx"]] * 2), np.stack([tr["logit"]] * 2),
                           np.stack([tr["count"]] * 2), np.stack([toks, toks]), np.stack([u_acc, np.zeros(G)]),
                           np.stack([u_res, u_res]))
    assert batch["accept_len"].tolist() == [r["accept_len"], G]
    assert np.array_equal(batch["tokens"][0], r["tokens"]) and np.array_equal(batch["tokens"][1], all_acc["tokens"])


def test_expected_tokens_per_round_matches_section_2_3():
    """Identical positions with acceptance rate a: E[emitted tokens] = (1 - a^{L+1}) / (1 - a)."""
    V, K, L = 10, 4, 4
    z, t, tr, p, qh = make_case(33, V, K)
    a = np.minimum(qh, p).sum()
    rng = np.random.default_rng(99)
    trials = 6000
    T_rows = np.stack([t] * (L + 1))
    idx, logit = np.stack([tr["idx"]] * L), np.stack([tr["logit"]] * L)
    emitted = 0
    for _ in range(trials):
        slots, _ = zip(*[O.sample_row(tr["logit"], K, [rng.random()]) for _ in range(L)])
        toks = [tr["idx"][s[0]] for s in slots]
        r = O.verify_chain_seq(T_rows, 1.0, idx, logit, [K] * L, toks, rng.random(L), rng.random(L + 1))
        emitted += r["accept_len"] + 1
    want = (1 - a ** (L + 1)) / (1 - a)
    assert abs(emitted / trials - want) < 0.08, (emitted / trials, want)
