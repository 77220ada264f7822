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
