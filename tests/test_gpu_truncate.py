"""GPU parity: tslt_truncate and tslt_sample through the C ABI against the CPU oracle."""
import numpy as np
import pytest
import torch

from oracle import tslt_oracle as O
from paper_2512_16273_amd import workloads as W
from tests import _parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def rows_like(w, n_rows, seed):
    d, _ = W.make_rows(w, n_rows, 0, seed, DEV)
    return d


@pytest.mark.parametrize("name,V,rows,T,top_k,top_p,k_cap", [
    ("f32-topk16", 5000, 9, 1.0, 16, 0.0, 16),            # 5 tiles of 1024 and a ragged one
    ("f32-odd", 33331, 5, 0.9, 40, 0.0, 64),              # odd V: rows at every 4-byte phase
    ("bf16-odd", 20011, 37, 0.8, 64, 0.0, 64),            # odd V: rows start at every 2-byte phase
    ("bf16-topp", 32000, 24, 0.8, 0, 0.95, 256),
    ("bf16-both", 32000, 8, 0.7, 100, 0.9, 256),
    ("bf16-k1024", 70000, 6, 1.0, 0, 0.99, 1024),
    ("bf16-k1", 9000, 4, 1.0, 1, 0.0, 1),
    ("f32-tinyV", 10, 3, 1.0, 0, 0.0, 16),                # K > V
    ("bf16-smallV", 777, 5, 1.3, 64, 0.0, 64),
    ("f16-odd", 20011, 37, 0.8, 64, 0.0, 64),             # binary16 rows, every 2-byte phase
    ("f16-topp", 32000, 24, 0.8, 0, 0.95, 256),
    ("f16-k1024", 70000, 6, 1.0, 0, 0.99, 1024),
    ("f16-smallV", 777, 5, 1.3, 64, 0.0, 64),
])
def test_truncate_matches_oracle(tslt, name, V, rows, T, top_k, top_p, k_cap):
    w = W.scaled(W.WORKLOADS["chain_topk"], V=V, dtype=name.split("-")[0])
    z = rows_like(w, rows, 3)
    out = tslt.truncate(z, T, top_k, top_p, k_cap)
    torch.cuda.synchronize()
    res = P.compare_truncate(out, z, T, top_k, top_p, k_cap, label=name)
    print(name, {k: v for k, v in res.items() if k != "ref"})


def test_truncate_strided_rows(tslt):
    w = W.scaled(W.WORKLOADS["chain_topk"], V=12001)
    full = rows_like(w, 6, 5)                       # [6, 12001]
    view = full[:, :11000]                          # row stride 12001, V 11000
    out = tslt.truncate(view, 0.8, 32, 0.0, 32)
    torch.cuda.synchronize()
    P.compare_truncate(out, view.contiguous(), 0.8, 32, 0.0, 32, label="strided")


def test_truncate_degenerate_rows(tslt):
    V = 6000
    g = torch.Generator().manual_seed(1)
    base = (torch.randn(13, V, generator=g) * 2).to(torch.bfloat16).float()
    rows = base.clone()
    rows[0] = 1.25                                            # all equal
    rows[1] = torch.where(torch.arange(V) % 3 == 0, 2.0, -1.0)  # two values
    rows[2, 100:] = -float("inf")                              # 100 finite
    rows[3, 5:] = -float("inf")                                # fewer finite than K
    rows[4] = -float("inf")                                    # nothing
    rows[5, 77] = float("nan")
    rows[6, 4321] = float("inf")
    rows[7] = torch.arange(V).float() / 64                     # ascending, many ties in bf16
    rows[8] = -torch.arange(V).float() / 64                    # descending
    rows[9, ::2] = 0.0
    rows[9, 1::2] = -0.0                                       # signed zeros are one value
    rows[10, :3000] = -float("inf")
    rows[11] = base[11].abs() * -50                            # huge spread
    rows[12] = (torch.arange(V) % 3 - 1).float() * 3e-6        # 0 and +-3e-6: subnormal as binary16
    for dt in (torch.float32, torch.bfloat16, torch.float16):
        z = rows.to(dt).to(DEV)
        for (k, p, cap) in ((16, 0.0, 16), (0, 0.9, 256), (300, 0.0, 512)):
            out = tslt.truncate(z, 0.7, k, p, cap)
            torch.cuda.synchronize()
            res = P.compare_truncate(out, z, 0.7, k, p, cap, label=f"degenerate {dt} k={k} p={p}")
            assert res["exact_path_rows"] >= 4


def test_truncate_argument_errors(tslt):
    z = torch.zeros(2, 100, device=DEV)
    for bad in (dict(temperature=0.0), dict(temperature=-1.0), dict(k_cap=0), dict(k_cap=2000), dict(top_k=-1)):
        kw = dict(temperature=1.0, top_k=4, top_p=0.0, k_cap=4)
        kw.update(bad)
        with pytest.raises(tslt.TsltError):
            tslt.truncate(z, **kw)
    with pytest.raises(tslt.TsltError):
        tslt.truncate(z.cpu(), 1.0, 4, 0.0, 4)
    with pytest.raises(tslt.TsltError):
        tslt.truncate(z.double(), 1.0, 4, 0.0, 4)
    out = tslt.truncate(torch.zeros(0, 100, device=DEV), 1.0, 4, 0.0, 4)     # empty batch
    assert out["count"].numel() == 0


@pytest.mark.parametrize("wo", [False, True])
def test_sample_matches_oracle(tslt, wo):
    w = W.scaled(W.WORKLOADS["chain_topp"], V=30000)
    z = rows_like(w, 40, 11)
    for (k, p, cap, n) in ((0, 0.95, 256, 1), (32, 0.0, 32, 4), (0, 0.999, 1024, 3), (3, 0.0, 4, 4)):
        ref = O.truncate(P.to_np(z), 0.8, k, p, cap)
        idx = torch.from_numpy(ref["idx"]).to(DEV)
        logit = torch.from_numpy(ref["logit"]).to(DEV)
        count = torch.from_numpy(ref["count"]).to(DEV)
        u = W.uniforms((40, n), 5, 2, 7, DEV)
        out = tslt.sample(idx, logit, count, u, wo)
        torch.cuda.synchronize()
        want = O.sample(ref["idx"], ref["logit"], ref["count"], P.to_np(u), wo)
        assert np.array_equal(P.to_np(out["slot"]), want["slot"])
        assert np.array_equal(P.to_np(out["token"]), want["token"])
    # an empty set gives -1
    out = tslt.sample(idx, logit, torch.zeros_like(count), u, wo)
    assert torch.all(out["token"] == -1)


@pytest.mark.parametrize("name,V,rows,T,top_k,top_p,k_cap,n", [
    ("bf16-topp-1", 32000, 24, 0.8, 0, 0.95, 256, 1),
    ("bf16-topk-4", 20011, 19, 0.8, 32, 0.0, 32, 4),
    ("f32-topk-3", 5000, 9, 1.0, 16, 0.0, 16, 3),
    ("bf16-k1024-2", 70000, 6, 1.0, 0, 0.999, 1024, 2),
    ("bf16-k3-16", 9000, 5, 1.0, 3, 0.0, 4, 16),
    ("f16-topp-2", 32000, 12, 0.8, 0, 0.95, 256, 2),
    ("f32-topk-4-wor", 151936, 6, 1.0, 32, 0.0, 32, 4),       # benchmark configuration 4's draws
    ("bf16-k3-16-wor", 9000, 5, 1.0, 3, 0.0, 4, 16),           # more draws than entries: the rest give -1
    ("bf16-topp-5-wor", 32000, 12, 0.8, 0, 0.95, 256, 5),
])
def test_truncate_sample_in_one_launch(tslt, name, V, rows, T, top_k, top_p, k_cap, n):
    """tslt_truncate_sample: the truncation against the oracle as for tslt_truncate; the draws against the
    oracle's sampling from the very sets the call returned, and against tslt_sample on those sets."""
    wor = name.endswith("-wor")
    w = W.scaled(W.WORKLOADS["chain_topk"], V=V, dtype=name.split("-")[0])
    z = rows_like(w, rows, 21)
    u = W.uniforms((rows, n), 9, 2, 3, DEV)
    out = tslt.truncate(z, T, top_k, top_p, k_cap, u=u, without_replacement=wor)
    torch.cuda.synchronize()
    P.compare_truncate({k: v for k, v in out.items() if k not in ("token", "slot")}, z, T, top_k, top_p, k_cap, label=name)
    want = O.sample(P.to_np(out["idx"]), P.to_np(out["logit"]), P.to_np(out["count"]), P.to_np(u), wor)
    if name == "bf16-k3-16-wor":
        assert np.all(want["slot"][:, 3:] == -1) and np.all(want["slot"][:, :3] >= 0)
    assert np.array_equal(P.to_np(out["slot"]), want["slot"]), name
    assert np.array_equal(P.to_np(out["token"]), want["token"]), name
    two = tslt.sample(out["idx"], out["logit"], out["count"], u, wor)
    assert torch.equal(two["token"], out["token"]) and torch.equal(two["slot"], out["slot"])


def test_truncate_sample_degenerate_and_errors(tslt):
    V = 3000
    z = torch.randn(4, V, generator=torch.Generator().manual_seed(2)).to(torch.bfloat16)
    z[1] = -float("inf")                      # nothing to draw from
    z[2, 7] = float("nan")
    z[3, 10:] = -float("inf")                 # 10 finite logits, K = 16
    z = z.to(DEV)
    u = torch.tensor([[0.0, 0.999999], [0.5, 0.5], [0.5, 0.5], [0.0, 0.999999]], dtype=torch.float32, device=DEV)
    out = tslt.truncate(z, 1.0, 16, 0.0, 16, u=u)
    torch.cuda.synchronize()
    tok, slot, cnt = P.to_np(out["token"]), P.to_np(out["slot"]), P.to_np(out["count"])
    assert cnt[1] == 0 and cnt[2] == 0 and cnt[3] == 10
    assert np.all(tok[1] == -1) and np.all(tok[2] == -1) and np.all(slot[1] == -1)
    want = O.sample(P.to_np(out["idx"]), P.to_np(out["logit"]), cnt, P.to_np(u), False)
    assert np.array_equal(tok, want["token"]) and np.array_equal(slot, want["slot"])
    assert slot[0, 0] == 0 and slot[3, 1] <= 9
    with pytest.raises(tslt.TsltError):
        tslt.truncate(z, 1.0, 16, 0.0, 16, u=torch.zeros(4, 17, dtype=torch.float32, device=DEV))


def test_tiny_config_end_to_end_truncate(tslt):
    w = W.WORKLOADS["tiny"]
    c = W.make_chain(w, 0, DEV)
    z = c["draft"].reshape(-1, w.V)
    out = tslt.truncate(z, w.T, w.top_k, w.top_p, w.k_cap)
    torch.cuda.synchronize()
    P.compare_truncate(out, z, w.T, w.top_k, w.top_p, w.k_cap, label="tiny")


def test_large_vocab_full_size_sampled_rows(tslt):
    """Benchmark configuration 3 at its full size, in the launch configuration bench.py times: every row is
    truncated on the GPU; a sample of rows is checked against the oracle element by element, all rows
    against properties that hold at any size."""
    w = W.WORKLOADS["large_vocab"]
    c = W.make_chain(w, 0, DEV)
    z = c["draft"].reshape(-1, w.V)
    u = c["u_sample"].reshape(-1, 1)
    out = tslt.truncate(z, w.T, w.top_k, w.top_p, w.k_cap, u=u)          # tslt_truncate_sample, as bench.py calls it
    torch.cuda.synchronize()
    plain = tslt.truncate(z, w.T, w.top_k, w.top_p, w.k_cap)
    for k in plain:
        assert torch.equal(out[k], plain[k]), k
    token, slot = out.pop("token"), out.pop("slot")
    want = O.sample(P.to_np(out["idx"][:96]), P.to_np(out["logit"][:96]), P.to_np(out["count"][:96]), P.to_np(u[:96]), False)
    assert np.array_equal(P.to_np(token[:96]), want["token"]) and np.array_equal(P.to_np(slot[:96]), want["slot"])
    assert torch.equal(token[:, 0], torch.gather(out["idx"], 1, slot.long().clamp(min=0))[:, 0])
    rows = np.random.default_rng(0).choice(z.shape[0], 24, replace=False)
    res = P.compare_truncate(out, z[torch.from_numpy(rows).to(DEV)], w.T, w.top_k, w.top_p, w.k_cap, rows=rows,
                             label="large_vocab")
    print({k: v for k, v in res.items() if k != "ref"})
    cnt, idx, prob = out["count"].long(), out["idx"].long(), out["prob"]
    assert int(cnt.min()) >= 1 and int(cnt.max()) <= w.k_cap
    valid = torch.arange(w.k_cap, device=DEV)[None, :] < cnt[:, None]
    assert torch.all((idx >= 0) == valid)
    vals = torch.gather(z.float(), 1, idx.clamp(min=0))
    vals = torch.where(valid, vals, torch.full_like(vals, -float("inf")))
    assert torch.all(vals[:, :-1] >= vals[:, 1:])                       # canonical order by value
    ties = (vals[:, :-1] == vals[:, 1:]) & valid[:, 1:]
    assert torch.all(idx[:, :-1][ties] < idx[:, 1:][ties])              # ties by ascending index
    # nothing outside the set beats the last kept value when the cap binds
    torch.testing.assert_close(prob.double().sum(1), torch.ones_like(cnt, dtype=torch.double), rtol=0, atol=1e-5)
    frac_exact = float((out["status"] & 256).ne(0).float().mean())
    print("rows on the exact multi-pass path:", frac_exact)
    assert frac_exact < 0.05
