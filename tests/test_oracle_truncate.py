"""Pins for the oracle's truncation and sparse sampling (no GPU).

Each test checks the oracle against something other than itself: brute-force order properties,
closed forms of Section 3 (Theorem 1: TV(q_hat, q) = sigma; |beta_hat - beta| <= sigma; Lemma 1;
Lemma 2), scipy's softmax for the K = V special case, and the value of D_V printed in Section 5.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import tslt_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def rng_rows(seed, rows, V, ties=False):
    rng = np.random.default_rng(seed)
    z = rng.normal(0, 2.5, size=(rows, V)).astype(np.float32)
    if ties:  # few distinct values, like bf16 at large V
        z = np.round(z * 2) / 2
    return z.astype(np.float32)


def tv(a, b):
    return 0.5 * np.abs(a - b).sum()


def dense_q(z, T):
    return sp_softmax(O.scale(z, T).astype(np.float64))


def scatter(V, t):
    q = np.zeros(V)
    q[t["idx"]] = t["prob"]
    return q


def test_reciprocal_scaling_is_one_fp32_multiply():
    z = np.array([1.5, -3.25, 7.0, 0.1], np.float32)
    for T in (1.0, 0.7, 0.8, 1.3):
        rT = np.float32(1.0 / np.float64(np.float32(T)))
        s = O.scale(z, T)
        assert s.dtype == np.float32
        # exact product in fp64 (24x24 bits fit), rounded once to fp32
        assert np.array_equal(s, (z.astype(np.float64) * np.float64(rT)).astype(np.float32))
    assert np.array_equal(O.scale(z, 1.0), z)
    with pytest.raises(ValueError):
        O.scale(z, 0.0)


@pytest.mark.parametrize("ties", [False, True])
def test_topk_set_is_the_k_best_in_the_total_order(ties):
    V = 300
    z = rng_rows(3, 6, V, ties)
    for r, K in itertools.product(range(6), (1, 2, 7, 64, 300, 500)):
        t = O.truncate_row(z[r], 1.0, K, 0.0, max(K, 1))
        cnt = t["count"]
        assert cnt == min(K, V)
        sel = t["idx"]
        assert len(set(sel.tolist())) == cnt
        # canonical order: strictly decreasing in (value desc, index asc)
        for a, b in zip(sel[:-1], sel[1:]):
            assert z[r, a] > z[r, b] or (z[r, a] == z[r, b] and a < b)
        # brute force: every excluded token is beaten by the last included one
        last = sel[-1]
        excl = np.setdiff1d(np.arange(V), sel)
        for y in excl:
            assert z[r, last] > z[r, y] or (z[r, last] == z[r, y] and last < y)
        assert np.array_equal(t["logit"], z[r, sel])


def test_all_equal_and_two_valued_rows_break_ties_by_index():
    V = 50
    t = O.truncate_row(np.full(V, 1.25, np.float32), 0.9, 7, 0.0, 7)
    assert t["idx"].tolist() == list(range(7))
    z = np.where(np.arange(V) % 3 == 0, 2.0, -1.0).astype(np.float32)
    t = O.truncate_row(z, 1.0, 20, 0.0, 20)
    hi = [i for i in range(V) if i % 3 == 0]          # 17 of them
    lo = [i for i in range(V) if i % 3 != 0]
    assert t["idx"].tolist() == hi + lo[:3]
    # -0.0 and +0.0 are the same value
    z = np.array([-0.0, 0.0, -1.0, 0.0], np.float32)
    assert O.truncate_row(z, 1.0, 3, 0.0, 3)["idx"].tolist() == [0, 1, 3]


def test_masked_and_broken_rows():
    z = np.array([0.0, -np.inf, 1.0, -np.inf], np.float32)
    t = O.truncate_row(z, 1.0, 4, 0.0, 4)
    assert t["idx"].tolist() == [2, 0] and t["count"] == 2 and t["status"] == 0
    assert np.isclose(t["prob"].sum(), 1.0)
    assert O.truncate_row(np.full(4, -np.inf, np.float32), 1.0, 2, 0.0, 2)["status"] == O.STATUS_EMPTY
    for bad in (np.nan, np.inf):
        z = np.array([0.0, bad, 1.0], np.float32)
        t = O.truncate_row(z, 1.0, 2, 0.0, 2)
        assert t["status"] == O.STATUS_NONFINITE and t["count"] == 0


def test_full_set_reduces_to_textbook_softmax():
    z = rng_rows(5, 3, 200)
    for T in (1.0, 0.7):
        for r in range(3):
            t = O.truncate_row(z[r], T, 0, 0.0, 200)
            q = scatter(200, t)
            np.testing.assert_allclose(q, dense_q(z[r], T), rtol=1e-13, atol=0)
            assert abs(t["mass"] - 1.0) < 1e-14 and t["count"] == 200


@pytest.mark.parametrize("T", [1.0, 0.7])
def test_theorem1_tv_equals_sigma_and_acceptance_bound(T):
    V = 400
    z = rng_rows(7, 5, V, ties=True)
    rng = np.random.default_rng(11)
    for r in range(5):
        q = dense_q(z[r], T)
        p = sp_softmax((z[r] + rng.normal(0, 1.0, V)).astype(np.float64))
        for K in (1, 5, 40, 399):
            t = O.truncate_row(z[r], T, K, 0.0, K)
            qh = scatter(V, t)
            sigma = 1.0 - t["mass"]
            assert abs(qh.sum() - 1.0) < 1e-13
            # Theorem 1: TV(q_hat, q) = sigma exactly; sigma is the mass outside the kept set
            assert abs(tv(qh, q) - sigma) < 1e-13
            assert abs(sigma - np.delete(q, t["idx"]).sum()) < 1e-13
            # Lemma 1 and Theorem 1: beta = sum min(q, p) = 1 - TV, |beta_hat - beta| <= sigma
            beta, beta_hat = np.minimum(q, p).sum(), np.minimum(qh, p).sum()
            assert abs(beta - (1 - tv(q, p))) < 1e-13
            assert abs(beta_hat - beta) <= sigma + 1e-13
            # Lemma 2
            assert abs(tv(qh, p) - tv(q, p)) <= tv(qh, q) + 1e-13
            # renormalisation equation: q_hat = q / rho on the kept set
            np.testing.assert_allclose(qh[t["idx"]], q[t["idx"]] / t["mass"], rtol=1e-12)


def test_nucleus_is_minimal_and_monotone():
    V = 500
    z = rng_rows(9, 4, V)
    for r in range(4):
        q = dense_q(z[r], 0.8)
        prev = 0
        for rho in (0.05, 0.3, 0.5, 0.9, 0.95, 0.999):
            t = O.truncate_row(z[r], 0.8, 0, rho, V)
            cnt = t["count"]
            rho32 = np.float64(np.float32(rho))
            kept = q[t["idx"]]
            assert kept.sum() >= rho32 - 1e-12            # reaches rho
            assert kept[:-1].sum() < rho32 + 1e-12         # and would not without its last element
            assert np.all(np.diff(kept) <= 1e-18)          # a prefix of the descending order
            assert np.delete(q, t["idx"]).max(initial=0.0) <= kept.min() + 1e-18
            assert abs(t["mass"] - kept.sum()) < 1e-12
            assert cnt >= prev
            prev = cnt
            assert np.isfinite(t["margin_rho"]) and t["margin_rho"] >= 0
        # rho >= 1 or 0 switches the nucleus off: everything up to the cap is kept
        assert O.truncate_row(z[r], 0.8, 0, 1.0, V)["count"] == V
        assert O.truncate_row(z[r], 0.8, 0, 0.0, V)["count"] == V


def test_cap_and_topk_combine_with_the_nucleus():
    V = 500
    z = rng_rows(10, 1, V)[0]
    full = O.truncate_row(z, 1.0, 0, 0.9, V)
    m_rho = full["count"]
    assert m_rho > 8
    capped = O.truncate_row(z, 1.0, 0, 0.9, 8)            # cap binds: plain top-8, mass vs full Z
    assert capped["count"] == 8 and capped["idx"].tolist() == full["idx"][:8].tolist()
    q = dense_q(z, 1.0)
    assert abs(capped["mass"] - q[capped["idx"]].sum()) < 1e-13
    both = O.truncate_row(z, 1.0, m_rho + 5, 0.9, V)      # nucleus binds
    assert both["count"] == m_rho
    both = O.truncate_row(z, 1.0, 3, 0.9, V)              # top-k binds
    assert both["count"] == 3


def test_batch_wrapper_pads():
    z = rng_rows(12, 3, 64)
    out = O.truncate(z, 1.0, 5, 0.0, 8)
    assert out["idx"].shape == (3, 8) and np.all(out["idx"][:, 5:] == -1)
    assert np.all(np.isneginf(out["logit"][:, 5:])) and np.all(out["prob"][:, 5:] == 0)
    assert np.all(out["count"] == 5)


def test_sparse_sampling_inverse_cdf():
    logit = np.log(np.array([0.5, 0.25, 0.125, 0.125])).astype(np.float32)
    # buckets [0,.5) [.5,.75) [.75,.875) [.875,1)
    for u, want in ((0.0, 0), (0.49, 0), (0.51, 1), (0.74, 1), (0.76, 2), (0.88, 3), (0.999, 3)):
        s, _ = O.sample_row(logit, 4, [u])
        assert s[0] == want, (u, s)
    # empirical frequencies over a fine grid equal q_hat
    grid = (np.arange(4000) + 0.5) / 4000
    s, _ = O.sample_row(logit, 4, grid)
    np.testing.assert_allclose(np.bincount(s, minlength=4) / 4000, [0.5, 0.25, 0.125, 0.125], atol=1e-3)
    # count restricts the set
    s, _ = O.sample_row(logit, 2, grid)
    np.testing.assert_allclose(np.bincount(s, minlength=4) / 4000, [2 / 3, 1 / 3, 0, 0], atol=1e-3)


def test_sampling_without_replacement_matches_sequential_renormalisation():
    q = np.array([0.4, 0.3, 0.2, 0.1])
    logit = np.log(q).astype(np.float32)
    n = 60
    grid = (np.arange(n) + 0.5) / n
    # P(first = a, second = b) = q_a * q_b / (1 - q_a)
    counts = np.zeros((4, 4))
    for u1 in grid:
        for u2 in grid:
            s, _ = O.sample_row(logit, 4, [u1, u2], without_replacement=True)
            assert s[0] != s[1]
            counts[s[0], s[1]] += 1
    want = np.array([[0 if a == b else q[a] * q[b] / (1 - q[a]) for b in range(4)] for a in range(4)])
    np.testing.assert_allclose(counts / n ** 2, want, atol=2.5 / n)
    # drawing everything returns a permutation
    s, _ = O.sample_row(logit, 4, [0.3, 0.9, 0.1, 0.5], without_replacement=True)
    assert sorted(s.tolist()) == [0, 1, 2, 3]


def test_printed_dense_payload():
    vals = {}
    for line in open(GOLDEN):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            vals[k] = v
    V, b = int(vals["dense_payload_vocab"][0]), int(vals["dense_payload_bits_per_prob"][0])
    mbit = float(vals["dense_payload_mbit"][0])
    assert abs(O.payload_bits(V, b, 0) / 1e6 - mbit) < 0.02       # 0.512 Mbit printed as 0.5
    assert O.index_bits(V) == 15
    # truncated payload for K entries: K * (b_prob + ceil(log2 V))
    assert O.payload_bits(320, 16, O.index_bits(V)) == 9920
    exp = [int(x) for x in vals["expansion"]]
    assert O.tree_layout(exp)["n_internal"] == 1 + 2 + 4


# ----------------------------------------------------------------------------------------------
# 16-bit payloads and the wire format (Section 2.2)
# ----------------------------------------------------------------------------------------------
def test_round_payload_is_round_to_nearest_even_of_the_format():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.normal(0, 8, 4000), [0.0, -0.0, 1.0, 65504.0, 7e4, -7e4, 1e-8, 3e38, 3.4e38]]).astype(np.float32)
    h = O.round_payload(x, "f16")
    # nearest: no other binary16 value is closer; brute force over the two neighbours
    h16 = h.astype(np.float16)
    assert np.array_equal(h16.astype(np.float32), h)                       # representable
    with np.errstate(over="ignore"):
        neighbours = (np.nextafter(h16, np.float16(np.inf)), np.nextafter(h16, np.float16(-np.inf)))
    for nb in neighbours:
        ok = np.isfinite(nb.astype(np.float32))
        xc = np.clip(x, -65504, 65504).astype(np.float64)
        assert np.all(np.abs(h.astype(np.float64) - xc)[ok] <= np.abs(nb.astype(np.float64) - xc)[ok])
    assert h[-5] == 65504.0 and h[-4] == -65504.0                         # 7e4 and -7e4: clamped, never infinite
    b = O.round_payload(x, "bf16")
    assert np.all((b.view(np.uint32) & 0xFFFF) == 0) and np.all(np.isfinite(b))
    err = np.abs(b.astype(np.float64) - x.astype(np.float64))
    ulp = np.ldexp(1.0, np.frexp(np.maximum(np.abs(x.astype(np.float64)), 1e-40))[1] - 8)   # 8 significant bits
    assert np.all(err[:-2] <= ulp[:-2] * 0.5)
    tie = np.array([1.00390625], np.float32)                              # 1 + 2^-8: halfway between 1 and 1 + 2^-7
    assert O.round_payload(tie, "bf16")[0] == 1.0                          # ties to even
    assert O.round_payload(np.array([1.01171875], np.float32), "bf16")[0] == np.float32(1.015625)
    assert np.array_equal(O.round_payload(x, "f32"), x)


@pytest.mark.parametrize("payload", ["f16", "bf16"])
def test_truncate_with_a_16_bit_payload(payload):
    rng = np.random.default_rng(8)
    z = (rng.normal(0, 3, (6, 900)) - 1.1 * np.log(rng.permutation(900)[None, :] + 1.0)).astype(np.float32)
    a = O.truncate(z, 0.8, 0, 0.95, 64)
    b = O.truncate(z, 0.8, 0, 0.95, 64, payload)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(a["count"], b["count"])   # the set does not move
    np.testing.assert_allclose(a["mass"], b["mass"], rtol=0, atol=0)
    for r in range(6):
        c = b["count"][r]
        assert np.array_equal(b["logit"][r, :c], O.round_payload(a["logit"][r, :c], payload))
        # q_hat is the softmax of what is transmitted (scipy's, as an independent routine)
        from scipy.special import softmax as sp_softmax
        np.testing.assert_allclose(b["prob"][r, :c], sp_softmax(b["logit"][r, :c].astype(np.float64)), rtol=1e-13)
        assert abs(b["prob"][r, :c].sum() - 1) < 1e-14


@pytest.mark.parametrize("payload,V", [("f16", 32000), ("bf16", 128256), ("f16", 5), ("bf16", 151936)])
def test_wire_format_round_trip_and_size(payload, V):
    rng = np.random.default_rng(11)
    rows, k_cap = 9, 40
    count = np.array([0, 1, 40, 17, 2, 40, 3, 31, 5])
    idx = np.full((rows, k_cap), -1, np.int32)
    logit = np.full((rows, k_cap), -np.inf, np.float32)
    for r in range(rows):
        c = count[r]
        idx[r, :c] = rng.choice(V, c, replace=c > V) if c <= V else rng.integers(0, V, c)
        logit[r, :c] = O.round_payload(np.sort(rng.normal(0, 5, c))[::-1].astype(np.float32), payload)
    if count.max() <= V or True:
        idx[2, 0], idx[2, 1] = V - 1, 0                                    # the extreme token ids
    pk = O.pack_rows(idx, logit, count, V, payload)
    b_idx = O.index_bits(V)
    assert pk["b_idx"] == b_idx and 2 ** b_idx >= V > 2 ** (b_idx - 1) or V <= 2
    # Section 2.2: D = K (b_prob + b_idx) per position
    assert pk["payload_bits"] == sum(O.payload_bits(int(c), 16, b_idx) for c in count)
    assert pk["row_offset"][-1] == len(pk["words"]) == sum((16 + int(c) * (b_idx + 16) + 31) // 32 for c in count)
    un = O.unpack_rows(pk["words"], pk["row_offset"], rows, k_cap, V, payload)
    assert np.array_equal(un["count"], count) and np.array_equal(un["idx"], idx)
    assert np.array_equal(un["logit"], logit)
    # a hand-built stream: one row, two entries, V = 5 (3 index bits)
    one = O.pack_rows(np.array([[4, 1]]), np.array([[1.0, -2.0]], np.float32), [2], 5, "bf16")
    want = 2 | (4 << 16) | (0x3F80 << 19) | (1 << 35) | (0xC000 << 38)
    assert [int(x) for x in one["words"]] == [want & 0xFFFFFFFF, want >> 32]
