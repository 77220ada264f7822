"""GPU parity: tslt_truncation_stats through the C ABI against the oracle (Section 3.2)."""
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


@pytest.mark.parametrize("name,base,kw,ks", [
    ("bf16-topk", "chain_topk", dict(B=6, V=20011, gamma=3), [1, 2, 8, 33, 64, 500]),
    ("f32", "tiny", dict(B=5, V=5003, gamma=2), [1, 4, 16]),
    ("f16-topp", "chain_topp", dict(B=4, gamma=3, dtype="f16"), [1, 16, 64, 128, 256]),
    ("bf16-k1024", "stress", dict(B=2, gamma=2, V=70000), [3, 320, 1024]),
])
def test_stats_match_oracle(tslt, name, base, kw, ks):
    w = W.scaled(W.WORKLOADS[base], **kw)
    chain = W.make_chain(w, 5, DEV)
    B, G, V = w.B, w.gamma, w.V
    draft = chain["draft"].reshape(B * G, V)
    target = chain["target"][:, :G].reshape(B * G, V)
    tr = O.truncate(P.to_np(draft), w.T, w.top_k, w.top_p, w.k_cap)
    out = tslt.truncation_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(tr["count"]), ks)
    torch.cuda.synchronize()
    ref = O.truncation_stats(P.to_np(target), w.T, tr["idx"], tr["logit"], tr["count"], ks)
    assert np.array_equal(P.to_np(out["status"]) & 7, ref["status"])
    np.testing.assert_allclose(P.to_np(out["keep"]), ref["keep"], rtol=P.RTOL, err_msg=name)
    np.testing.assert_allclose(P.to_np(out["beta"]), ref["beta"], rtol=P.RTOL, err_msg=name)
    # the whole set: what tslt_verify reports for the same positions
    ver = tslt.verify(chain["target"], w.T, t32(tr["idx"]).view(B, G, -1), t32(tr["logit"]).view(B, G, -1),
                      t32(tr["count"]).view(B, G), t32(tr["idx"][:, 0].copy()).view(B, G), chain["u_accept"], chain["u_resample"])
    whole = tslt.truncation_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(tr["count"]), [w.k_cap])
    torch.cuda.synchronize()
    torch.testing.assert_close(whole["beta"].view(B, G), ver["beta"], rtol=1e-6, atol=0)
    print(name, "beta by K (mean over rows):", np.round(ref["beta"].mean(0), 4), "keep:", np.round(ref["keep"].mean(0), 4))


def test_stats_broken_rows_and_errors(tslt):
    w = W.scaled(W.WORKLOADS["chain_topk"], B=4, V=3000, gamma=1)
    chain = W.make_chain(w, 2, DEV)
    draft = chain["draft"].reshape(4, w.V)
    target = chain["target"][:, 0].clone()
    target[1, 7] = float("nan")
    target[2, :] = -float("inf")
    tr = O.truncate(P.to_np(draft), w.T, w.top_k, w.top_p, w.k_cap)
    cnt = tr["count"].copy()
    cnt[3] = 0                                           # an empty set
    out = tslt.truncation_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(cnt), [1, 8])
    torch.cuda.synchronize()
    ref = O.truncation_stats(P.to_np(target), w.T, tr["idx"], tr["logit"], cnt, [1, 8])
    assert (P.to_np(out["status"]) & 7).tolist() == ref["status"].tolist() == [0, 1, 2, 2]
    assert np.array_equal(np.isnan(P.to_np(out["beta"])), np.isnan(ref["beta"]))
    np.testing.assert_allclose(P.to_np(out["beta"])[0], ref["beta"][0], rtol=P.RTOL)
    with pytest.raises(tslt.TsltError):
        tslt.truncation_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(cnt), list(range(40)))      # too many K
    with pytest.raises(tslt.TsltError):
        tslt.truncation_stats(target, 0.0, t32(tr["idx"]), t32(tr["logit"]), t32(cnt), [1])


@pytest.mark.parametrize("name,base,kw,k", [
    ("bf16-topk", "chain_topk", dict(B=6, V=20011, gamma=3), 4),
    ("f32", "tiny", dict(B=5, V=5003, gamma=2), 3),
    ("f16-topp", "chain_topp", dict(B=4, gamma=3, dtype="f16"), 2),
    ("bf16-k1024", "stress", dict(B=2, gamma=2, V=70000), 16),
    ("bf16-one", "chain_topk", dict(B=3, V=9001, gamma=2), 1),
])
def test_multicandidate_rates_match_oracle(tslt, name, base, kw, k):
    """tslt_multicandidate_stats: Section 4.3's beta^(j) and theta against the oracle's dense recursion.  Stage j's
    rate carries the factor prod_{i<j} 1/Z_i = prod 1/(1 - beta^(i)) in front of an error of p, as the ratios of
    the tree kernel do; the tolerance grows with it, up to the comparers' cap."""
    w = W.scaled(W.WORKLOADS[base], **kw)
    chain = W.make_chain(w, 9, DEV)
    B, G, V = w.B, w.gamma, w.V
    draft = chain["draft"].reshape(B * G, V)
    target = chain["target"][:, :G].reshape(B * G, V)
    tr = O.truncate(P.to_np(draft), w.T, w.top_k, w.top_p, w.k_cap)
    out = tslt.multicandidate_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(tr["count"]), k)
    torch.cuda.synchronize()
    ref = O.multi_candidate_stats(P.to_np(target), w.T, tr["idx"], tr["logit"], tr["count"], k)
    got_b, got_t = P.to_np(out["beta"]), P.to_np(out["theta"])
    assert np.array_equal(P.to_np(out["status"]) & 15, ref["status"])
    reached = ~np.isnan(ref["beta"])
    # a stage behind an empty residual: the oracle's Z is exactly 0 there or a rounding error away from it
    amp = np.cumprod(np.concatenate([np.ones((B * G, 1)), 1.0 / np.maximum(1.0 - np.nan_to_num(ref["beta"][:, :-1]), 1e-300)], 1), 1)
    tol = P.RTOL * np.abs(np.nan_to_num(ref["beta"])) + P.NEAR_TIE * np.minimum(amp, P.AMP_CAP)
    firm = reached & (amp < P.AMP_CAP)
    assert firm[:, 0].all()
    assert np.all(np.abs(got_b[firm] - ref["beta"][firm]) <= tol[firm]), name
    np.testing.assert_allclose(got_t, ref["theta"], rtol=P.RTOL, atol=1e-6, err_msg=name)
    # one candidate is Lemma 1's rate, which tslt_truncation_stats reports for the whole set
    whole = tslt.truncation_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(tr["count"]), [w.k_cap])
    torch.cuda.synchronize()
    torch.testing.assert_close(out["beta"][:, 0], whole["beta"][:, 0], rtol=1e-6, atol=0)
    print(name, "mean beta^(j):", np.round(np.nanmean(ref["beta"], 0), 4), "mean theta:", round(float(ref["theta"].mean()), 4))


def test_multicandidate_rates_broken_rows_and_errors(tslt):
    w = W.scaled(W.WORKLOADS["chain_topk"], B=4, V=3000, gamma=1)
    chain = W.make_chain(w, 2, DEV)
    draft = chain["draft"].reshape(4, w.V)
    target = chain["target"][:, 0].clone()
    target[1, 7] = float("nan")
    target[2, :] = -float("inf")
    tr = O.truncate(P.to_np(draft), w.T, w.top_k, w.top_p, w.k_cap)
    cnt = tr["count"].copy()
    cnt[3] = 0
    out = tslt.multicandidate_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(cnt), 3)
    torch.cuda.synchronize()
    ref = O.multi_candidate_stats(P.to_np(target), w.T, tr["idx"], tr["logit"], cnt, 3)
    assert (P.to_np(out["status"]) & 15).tolist() == ref["status"].tolist() == [0, 1, 2, 2]
    assert np.all(np.isnan(P.to_np(out["theta"])[1:])) and np.all(np.isnan(P.to_np(out["beta"])[1:]))
    np.testing.assert_allclose(P.to_np(out["theta"])[0], ref["theta"][0], rtol=P.RTOL)
    for bad_k in (0, 17):
        with pytest.raises(tslt.TsltError):
            tslt.multicandidate_stats(target, w.T, t32(tr["idx"]), t32(tr["logit"]), t32(cnt), bad_k)
