"""Pins of the oracle's truncation statistics (Section 3.2): the dense definition written out, Lemma 1,
Theorem 1's bound, nesting of the prefixes, and agreement with the chain verifier's beta_hat."""
import numpy as np

from oracle import tslt_oracle as O


def softmax64(z):
    z = np.asarray(z, np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def make(seed, V=300, k_cap=64, T=0.8, noise=0.7):
    rng = np.random.default_rng(seed)
    draft = (rng.normal(0, 2.5, V) - 1.0 * np.log(rng.permutation(V) + 1.0)).astype(np.float32)
    target = (draft + rng.normal(0, noise, V)).astype(np.float32)
    tr = O.truncate(draft[None, :], T, k_cap, 0.0, k_cap)
    return draft, target, tr, T


def test_statistics_are_the_dense_definition():
    for seed in range(6):
        draft, target, tr, T = make(seed)
        V = draft.size
        ks = [1, 2, 5, 17, 64, 200]
        got = O.truncation_stats_row(target, T, tr["idx"][0], tr["logit"][0], tr["count"][0], ks)
        s_d = (draft * np.float32(1.0 / T)).astype(np.float32)
        s_t = (target * np.float32(1.0 / T)).astype(np.float32)
        q, p = softmax64(s_d), softmax64(s_t)
        order = np.lexsort((np.arange(V), -draft.astype(np.float64)))          # value descending, index ascending
        cnt = int(tr["count"][0])
        q_set = q[order[:cnt]].sum()
        beta_full = np.minimum(q, p).sum()
        for j, K in enumerate(ks):
            k = min(K, cnt)
            top = order[:k]
            qk = np.zeros(V)
            qk[top] = q[top] / q[top].sum()                                  # the renormalisation of Section 3.1
            beta = np.minimum(qk, p).sum()
            assert abs(got["beta"][j] - beta) < 1e-12
            assert abs(got["beta"][j] - (1.0 - 0.5 * np.abs(qk - p).sum())) < 1e-12          # Lemma 1
            assert abs(got["keep"][j] - q[top].sum() / q_set) < 1e-12
            rho = q[top].sum()
            assert abs(beta - beta_full) <= (1.0 - rho) + 1e-12              # Theorem 1: |beta_hat - beta| <= sigma


def test_prefixes_nest_and_the_whole_set_is_what_verification_reports():
    draft, target, tr, T = make(11, V=500, k_cap=32)
    cnt = int(tr["count"][0])
    ks = list(range(1, cnt + 1)) + [cnt + 5]
    got = O.truncation_stats_row(target, T, tr["idx"][0], tr["logit"][0], cnt, ks)
    assert np.all(np.diff(got["keep"]) >= 0) and abs(got["keep"][cnt - 1] - 1.0) < 1e-15 and got["keep"][-1] == got["keep"][cnt - 1]
    # K = 1: q_hat is a point mass, so beta is p of the top draft token
    p = softmax64((target * np.float32(1.0 / T)).astype(np.float32))
    assert abs(got["beta"][0] - p[tr["idx"][0][0]]) < 1e-15
    # the whole set: the value Algorithm 3's verifier reports for this position
    tgt2 = np.stack([target, target])
    v = O.verify_chain_seq(tgt2, T, tr["idx"], tr["logit"], tr["count"], tr["idx"][:, 0], np.zeros(1, np.float32),
                           np.zeros(2, np.float32))
    assert abs(got["beta"][-1] - v["beta_hat"][0]) < 1e-15


def test_identical_models_and_broken_rows():
    draft, _, tr, T = make(3, V=40, k_cap=64)              # k_cap > V: the set is the whole vocabulary
    got = O.truncation_stats_row(draft, T, tr["idx"][0], tr["logit"][0], tr["count"][0], [40])
    assert abs(got["beta"][0] - 1.0) < 1e-12 and got["status"] == 0          # q_hat = q = p
    bad = draft.copy()
    bad[3] = np.nan
    got = O.truncation_stats_row(bad, T, tr["idx"][0], tr["logit"][0], tr["count"][0], [1, 4])
    assert got["status"] == 1 and np.all(np.isnan(got["beta"]))
    got = O.truncation_stats_row(draft, T, tr["idx"][0], tr["logit"][0], 0, [1])
    assert got["status"] == 2 and np.isnan(got["keep"][0])
    batch = O.truncation_stats(np.stack([draft, bad]), T, np.repeat(tr["idx"], 2, 0), np.repeat(tr["logit"], 2, 0),
                               np.repeat(tr["count"], 2), [1, 8])
    assert batch["status"].tolist() == [0, 1] and batch["keep"].shape == (2, 2)


# ----------------------------------------------------------------------------------------------
# Section 4.3: stage acceptance rates beta^(j) and the total rate theta of multi-candidate verification
# ----------------------------------------------------------------------------------------------
def enumerate_stage_events(p, ids, q, k):
    """P(candidates 1..j-1 rejected and candidate j accepted), j = 1..k, by enumeration of every k-tuple of i.i.d.
    candidates (weight prod q_hat) through the candidate-driven recursion O.mcveri: with u = 1 nothing is
    accepted, so every stage's ratio is reported, and the probability of accepting at that stage is
    min(1, ratio) by the algorithm's test u < min(1, ratio) with u uniform."""
    import itertools
    acc_at = np.zeros(k)
    for tup in itertools.product(range(len(ids)), repeat=k):
        w = float(np.prod([q[i] for i in tup]))
        r = O.mcveri(p, ids, q, [int(ids[i]) for i in tup], [1.0] * k, 0.5)
        reach = 1.0
        for j in range(k):
            a = min(1.0, max(0.0, r["ratio"][j]))
            acc_at[j] += w * reach * a
            reach *= 1.0 - a
    return acc_at


def test_stage_rates_are_the_conditional_acceptance_probabilities():
    rng = np.random.default_rng(11)
    for V, K, k in ((6, 3, 3), (8, 4, 2), (5, 5, 3), (7, 2, 4)):
        p = rng.dirichlet(np.ones(V) * 0.7)
        ids = rng.choice(V, K, replace=False)
        q = rng.dirichlet(np.ones(K))
        got = O.multi_candidate_rates(p, ids, q, k)
        acc_at = enumerate_stage_events(p, ids, q, k)
        reach = 1.0
        for j in range(k):
            # Definition of Section 4.3: beta^(j) = Pr[x^(j) accepted | x^(1..j-1) rejected]
            assert abs(got["beta"][j] - acc_at[j] / reach) < 1e-12, (V, K, k, j)
            reach -= acc_at[j]
        # theta is the probability that one of the k candidates is accepted
        assert abs(got["theta"] - acc_at.sum()) < 1e-12
        assert abs(got["theta"] - (1.0 - np.prod(1.0 - got["beta"]))) < 1e-12


def test_stage_rates_special_cases():
    # one candidate: Lemma 1's rate, 1 - TV(q_hat, p)
    rng = np.random.default_rng(12)
    p = rng.dirichlet(np.ones(9))
    ids = np.array([4, 0, 7])
    q = np.array([0.5, 0.3, 0.2])
    qd = np.zeros(9)
    qd[ids] = q
    one = O.multi_candidate_rates(p, ids, q, 1)
    assert abs(one["beta"][0] - (1.0 - 0.5 * np.abs(qd - p).sum())) < 1e-14 and one["theta"] == one["beta"][0]
    # the worked case of tests/test_oracle_margins.py: p = (.4, .1, .3, .2), q_hat = (.3 on 0, .7 on 2):
    # beta1 = .3 + .3 = .6; p2 = (.25, .25, 0, .5): beta2 = .25; p3 = (0, 1/3, 0, 2/3): beta3 = 0
    r = O.multi_candidate_rates(np.array([0.4, 0.1, 0.3, 0.2]), [0, 2], np.array([0.3, 0.7]), 3)
    np.testing.assert_allclose(r["beta"], [0.6, 0.25, 0.0], atol=1e-15)
    assert abs(r["theta"] - (0.6 + 0.25 * 0.4 + 0.0)) < 1e-15
    # q_hat = p on a full set: the first candidate is always accepted, the later stages are never reached
    r = O.multi_candidate_rates(np.array([0.5, 0.25, 0.25]), [0, 1, 2], np.array([0.5, 0.25, 0.25]), 3)
    assert r["beta"][0] == 1.0 and np.all(np.isnan(r["beta"][1:])) and r["theta"] == 1.0
    # more candidates never lower theta, and every stage rate is what mcveri meets on an all-rejected run
    p = rng.dirichlet(np.ones(12) * 0.5)
    ids = rng.choice(12, 5, replace=False)
    q = rng.dirichlet(np.ones(5))
    thetas = [O.multi_candidate_rates(p, ids, q, k)["theta"] for k in range(1, 6)]
    assert np.all(np.diff(thetas) >= -1e-15)
    met = O.mcveri(p, ids, q, [int(ids[0])] * 5, [1.0] * 5, 0.5)["betas"]
    np.testing.assert_allclose(O.multi_candidate_rates(p, ids, q, 5)["beta"], met, rtol=1e-13)


def test_stage_rates_over_rows_and_broken_rows():
    draft, target, tr, T = make(3)
    rows = np.stack([target, target, target])
    rows[1, 5] = np.nan
    cnt = np.array([tr["count"][0], tr["count"][0], 0])
    got = O.multi_candidate_stats(rows, T, np.repeat(tr["idx"], 3, 0), np.repeat(tr["logit"], 3, 0), cnt, 4)
    assert got["status"].tolist() == [0, O.STATUS_NONFINITE, O.STATUS_EMPTY]
    assert np.all(np.isnan(got["beta"][1:])) and np.all(np.isnan(got["theta"][1:]))
    s_t = (target * np.float32(1.0 / T)).astype(np.float32)
    p = softmax64(s_t)
    qh = softmax64(tr["logit"][0][:cnt[0]].astype(np.float64))
    want = O.multi_candidate_rates(p, tr["idx"][0][:cnt[0]], qh, 4)
    np.testing.assert_allclose(got["beta"][0], want["beta"], rtol=1e-12)
    assert abs(got["theta"][0] - want["theta"]) < 1e-12
    # Section 5.2's qualitative statement, on these synthetic rows: more candidates accept more often
    assert got["theta"][0] > got["beta"][0, 0]
