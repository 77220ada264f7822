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
