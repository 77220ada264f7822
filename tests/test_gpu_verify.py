"""GPU parity: tslt_verify through the C ABI against the CPU oracle, and the whole single-candidate
round truncate -> sample -> verify."""
import numpy as np
import pytest
import torch

from oracle import tslt_oracle as O
from paper_2512_16273_amd import workloads as W
from tests import _parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def t32(a, dtype=None):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV) if dtype is None else \
        torch.from_numpy(np.ascontiguousarray(a)).to(dtype).to(DEV)


def run_verify_from_oracle_inputs(tslt, w, chain, ref):
    return tslt.verify(chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]),
                       t32(ref["tokens"]), chain["u_accept"], chain["u_resample"])


@pytest.mark.parametrize("name,base,kw", [
    ("tiny", "tiny", {}),
    ("f32-odd", "tiny", dict(B=6, V=5003, gamma=3)),
    ("bf16-topk", "chain_topk", dict(B=12, V=20011)),
    ("bf16-topp", "chain_topp", dict(B=10)),
    ("bf16-k1024", "stress", dict(B=3, gamma=4, V=70000)),
    ("bf16-one-segment", "chain_topk", dict(B=5, V=2000, gamma=2)),
    ("f16-topk", "chain_topk", dict(B=12, V=20011, dtype="f16")),
    ("f16-topp", "chain_topp", dict(B=10, dtype="f16")),
    ("f16-k1024", "stress", dict(B=3, gamma=4, V=70000, dtype="f16")),
    # the bulk of a row moved to 0, where the 16-bit formats have most of their small values: bf16 rows stay
    # inside the exp table, binary16 rows leave it and are swept without it
    ("bf16-centred", "chain_topp", dict(B=8, shift=9.4)),
    ("f16-centred", "chain_topp", dict(B=8, dtype="f16", shift=9.4)),
])
def test_verify_matches_oracle(tslt, name, base, kw):
    w = W.scaled(W.WORKLOADS[base], **kw)
    chain = W.make_chain(w, 7, DEV)
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(chain["u_accept"]), P.to_np(chain["u_resample"]))
    out = run_verify_from_oracle_inputs(tslt, w, chain, ref)
    torch.cuda.synchronize()
    res = P.compare_verify(out, ref["verify"], label=name)
    print(name, res, "accept_len histogram", np.bincount(ref["verify"]["accept_len"], minlength=w.gamma + 1))


def test_round_truncate_sample_verify(tslt):
    """The three calls chained on the GPU reproduce the oracle's round."""
    w = W.scaled(W.WORKLOADS["chain_topp"], B=16)
    chain = W.make_chain(w, 21, DEV)
    B, G, V = w.B, w.gamma, w.V
    tr = tslt.truncate(chain["draft"], w.T, w.top_k, w.top_p, w.k_cap)
    smp = tslt.sample(tr["idx"], tr["logit"], tr["count"], chain["u_sample"].reshape(B * G, 1))
    out = tslt.verify(chain["target"], w.T, tr["idx"].view(B, G, -1), tr["logit"].view(B, G, -1),
                      tr["count"].view(B, G), smp["token"].view(B, G), chain["u_accept"], chain["u_resample"])
    torch.cuda.synchronize()
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(chain["u_accept"]), P.to_np(chain["u_resample"]))
    t = P.compare_truncate(tr, chain["draft"].reshape(B * G, V), w.T, w.top_k, w.top_p, w.k_cap, label="round")
    if t["top_p_near_tie_mismatches"] == 0:
        assert np.array_equal(P.to_np(smp["token"]).reshape(B, G), ref["tokens"])
        print(P.compare_verify(out, ref["verify"], label="round"))


def test_verify_forced_paths_and_broken_rows(tslt):
    """All-accepted (bonus row), immediate rejection, tokens outside their set, NaN / masked rows."""
    w = W.scaled(W.WORKLOADS["chain_topk"], B=8, V=9001, gamma=4)
    chain = W.make_chain(w, 3, DEV)
    target = chain["target"].clone()
    target[4, 1, 17] = float("nan")          # broken row in the middle of sequence 4
    target[5, w.gamma, 5] = float("inf")     # broken bonus row of sequence 5
    target[6, 0, :] = -float("inf")          # fully masked row
    target[7, 2, 100:] = -float("inf")       # mostly masked row
    chain["target"] = target
    u_acc = chain["u_accept"].clone()
    u_acc[0] = 0.0                            # sequence 0: everything accepted -> bonus token
    u_acc[1] = 0.9995                         # sequence 1: rejected wherever ratio < 0.9995 (a uniform within 1e-6 of 1 would
                                              # put every ratio >= 1 inside the near-tie window)
    u_acc[5] = 0.0
    chain["u_accept"] = u_acc
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(target), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    # sequence 2: draft tokens that are not in their sets
    toks = ref["tokens"].copy()
    outside = np.setdiff1d(np.arange(w.V), ref["q_idx"][2, 0])[:w.gamma]
    toks[2] = outside
    ref["tokens"] = toks
    ref["verify"] = O.verify_chain(P.to_np(target), w.T, ref["q_idx"], ref["q_logit"], ref["q_count"], toks,
                                   P.to_np(u_acc), P.to_np(chain["u_resample"]))
    out = run_verify_from_oracle_inputs(tslt, w, chain, ref)
    torch.cuda.synchronize()
    v = ref["verify"]
    assert v["accept_len"][0] == w.gamma and v["status"][2] & 4 and v["status"][4] & 1 and v["status"][5] & 1
    print(P.compare_verify(out, v, label="forced"), v["accept_len"], v["status"])


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_verify_rows_outside_the_exp_table(tslt, dtype):
    """Target rows of 16-bit logits whose values leave the magnitude range that the resampling sweep tabulates:
    tiny values, zeros and subnormals, large ones, and ones whose scaled value is beyond the range in which
    terms may be referenced to 0."""
    w = W.scaled(W.WORKLOADS["chain_topk"], B=6, V=9001, gamma=3, dtype=dtype)
    chain = W.make_chain(w, 11, DEV)
    target = chain["target"].float()
    target[0] *= 1e-3                                  # everything below the table
    target[1, :, ::3] = 0.0
    target[1, :, 1::3] = -0.0
    target[1, :, 2::9] = 3e-6 if dtype == "f16" else 1e-39     # subnormal in the storage type
    target[2] *= 10.0                                  # much of the row above the table
    target[3, :, ::7] = -500.0                         # |s| = 625 > 600
    target[4, :, 5::11] = 490.0
    chain["target"] = target.to(chain["target"].dtype)
    u_acc = chain["u_accept"].clone()
    # reject at once wherever the ratio is below 0.9995 (a uniform within 1e-6 of 1 would put every ratio >= 1
    # inside the near-tie window)
    u_acc[:, 0] = 0.9995
    chain["u_accept"] = u_acc
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    out = run_verify_from_oracle_inputs(tslt, w, chain, ref)
    torch.cuda.synchronize()
    v = ref["verify"]
    assert np.all(v["status"] == 0)
    print(dtype, P.compare_verify(out, v, label="table-edges"), v["accept_len"])


@pytest.mark.parametrize("name,base,kw,first_stage", [
    ("bf16-g8-s1", "chain_topk", dict(B=24, V=20011), 1),       # stages of 1, 1, 2, 4 positions
    ("bf16-g8-s3", "chain_topp", dict(B=16), 3),                # 3, 3, 2 (the last stage is cut at gamma)
    ("f32-g3-s2", "tiny", dict(B=6, V=5003, gamma=3), 2),
    ("f16-g16-s2", "stress", dict(B=4, gamma=16, V=30000, dtype="f16"), 2),
    ("bf16-g8-s8", "chain_topk", dict(B=4, V=9001), 8),         # first_stage = gamma: the plain call
])
def test_verify_in_stages(tslt, name, base, kw, first_stage):
    """tslt_verify_staged: decisions and tokens are those of tslt_verify and of the oracle; ratio and beta
    agree with tslt_verify wherever the staged call evaluated the position and are NaN elsewhere, and a
    position is skipped exactly if an earlier stage holds a rejection."""
    w = W.scaled(W.WORKLOADS[base], **kw)
    chain = W.make_chain(w, 13, DEV)
    u_acc = chain["u_accept"].clone()
    u_acc[0] = 0.0                                    # one sequence that accepts everything
    chain["u_accept"] = u_acc
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    args = [chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(ref["tokens"]),
            u_acc, chain["u_resample"]]
    plain = tslt.verify(*args)
    staged = tslt.verify(*args, first_stage=first_stage)
    torch.cuda.synchronize()
    for k in ("accept_len", "tokens", "status"):
        assert torch.equal(plain[k], staged[k]), (name, k)
    # which positions the staged call looked at
    G = w.gamma
    bounds, j0, ln, k = [], 0, (first_stage if first_stage < G else G), 0
    while j0 < G:
        c = min(ln, G - j0)
        bounds.append((j0, j0 + c))
        j0 += c
        if k > 0:
            ln *= 2
        k += 1
    n = P.to_np(plain["accept_len"])
    pr, sr = P.to_np(plain["ratio"]), P.to_np(staged["ratio"])
    pb, sb = P.to_np(plain["beta"]), P.to_np(staged["beta"])
    skipped = 0
    for b in range(w.B):
        for (a, e) in bounds:
            looked = a <= n[b]                        # no rejection before this stage
            for j in range(a, e):
                if looked:
                    assert np.array_equal(sr[b, j], pr[b, j], equal_nan=True) and np.array_equal(sb[b, j], pb[b, j], equal_nan=True), (name, b, j)
                else:
                    assert np.isnan(sr[b, j]) and np.isnan(sb[b, j]), (name, b, j)
                    skipped += 1
    print(name, P.compare_verify(staged, ref["verify"], label=name), "positions skipped", skipped, "of", w.B * G)
    assert n[0] == G
    if first_stage < G:
        assert skipped > 0


def test_verify_argument_errors(tslt):
    w = W.scaled(W.WORKLOADS["chain_topk"], B=2, V=3000, gamma=2)
    chain = W.make_chain(w, 3, DEV)
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(chain["u_accept"]), P.to_np(chain["u_resample"]))
    args = [chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(ref["tokens"]),
            chain["u_accept"], chain["u_resample"]]
    with pytest.raises(tslt.TsltError):
        tslt.verify(*args, workspace=torch.empty(16, dtype=torch.uint8, device=DEV))   # workspace too small
    bad = list(args)
    bad[1] = 0.0
    with pytest.raises(tslt.TsltError):
        tslt.verify(*bad)


def test_large_vocab_full_size_sampled_sequences(tslt):
    """Benchmark configuration 3 at full size (B=256, gamma=8, V=128256, bf16), the configuration bench.py
    times: the GPU runs the whole batch; sampled sequences are checked against the oracle, which is fed
    its own truncation of those sequences' draft rows."""
    w = W.WORKLOADS["large_vocab"]
    chain = W.make_chain(w, 0, DEV)
    B, G, V = w.B, w.gamma, w.V
    tr = tslt.truncate(chain["draft"], w.T, w.top_k, w.top_p, w.k_cap)
    smp = tslt.sample(tr["idx"], tr["logit"], tr["count"], chain["u_sample"].reshape(B * G, 1))
    q_idx, q_logit = tr["idx"].view(B, G, -1).clone(), tr["logit"].view(B, G, -1).clone()
    q_count, toks = tr["count"].view(B, G).clone(), smp["token"].view(B, G).clone()
    seqs = np.random.default_rng(1).choice(B, 6, replace=False)
    sel = torch.from_numpy(seqs).to(DEV)
    ref = P.oracle_chain(P.to_np(chain["draft"][sel]), P.to_np(chain["target"][sel]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"][sel]), P.to_np(chain["u_accept"][sel]),
                         P.to_np(chain["u_resample"][sel]))
    # the sampled sequences get the oracle's own sparse sets and tokens as inputs
    q_idx[sel], q_logit[sel] = t32(ref["q_idx"]), t32(ref["q_logit"])
    q_count[sel], toks[sel] = t32(ref["q_count"]), t32(ref["tokens"])
    out = tslt.verify(chain["target"], w.T, q_idx, q_logit, q_count, toks, chain["u_accept"], chain["u_resample"])
    torch.cuda.synchronize()
    print(P.compare_verify(out, ref["verify"], seqs=seqs, label="large_vocab"))
    # properties over the whole batch
    n = out["accept_len"].long()
    assert int(n.min()) >= 0 and int(n.max()) <= G
    tk = out["tokens"].long()
    pos = torch.arange(G + 1, device=DEV)[None, :]
    assert torch.all((tk >= 0) == (pos <= n[:, None]))
    assert torch.all(tk[:, :G][pos[:, :G] < n[:, None]] == toks.long()[pos[:, :G] < n[:, None]])
    assert torch.all(out["status"] == 0)
    print("mean accepted length", float(n.float().mean()))


def test_stress_configuration_at_its_own_shape(tslt):
    """Benchmark configuration 5 with its own V = 256000, k_cap = 1024, gamma = 16, bf16, T = 1.0, top-p 0.99 (the
    launch plan of the truncation kernel -- sample fraction, threshold rank, candidate capacity, LDS carve-up --
    follows from V and k_cap, so a smaller V does not reach it), on B = 2 sequences: 32 draft and 34 target
    rows through tslt_truncate_sample, tslt_verify_accept + tslt_verify_resample and tslt_verify_staged, the
    calls `bench.py --workload stress` makes, against the oracle."""
    w = W.scaled(W.WORKLOADS["stress"], B=2)
    assert (w.V, w.k_cap, w.gamma, w.dtype, w.T, w.top_p) == (256000, 1024, 16, "bf16", 1.0, 0.99)
    chain = W.make_chain(w, 5, DEV)
    B, G, V, K = w.B, w.gamma, w.V, w.k_cap
    rows = chain["draft"].view(B * G, V)
    tr = tslt.truncate(rows, w.T, w.top_k, w.top_p, K, u=chain["u_sample"].view(B * G, 1))
    torch.cuda.synchronize()
    res = P.compare_truncate({k: v for k, v in tr.items() if k not in ("token", "slot")}, rows, w.T, w.top_k, w.top_p, K,
                             label="stress")
    print({k: v for k, v in res.items() if k != "ref"}, "counts", P.to_np(tr["count"]).min(), P.to_np(tr["count"]).max())
    # the single-pass selection has to carry this shape: no row on the multi-pass path
    assert res["exact_path_rows"] == 0
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, K,
                         P.to_np(chain["u_sample"]), P.to_np(chain["u_accept"]), P.to_np(chain["u_resample"]))
    if res["top_p_near_tie_mismatches"] == 0:
        assert np.array_equal(P.to_np(tr["token"]).reshape(B, G), ref["tokens"])
    # verification on the GPU's own sets and tokens where they are the oracle's (always, short of a near tie)
    args = [chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(ref["tokens"]),
            chain["u_accept"], chain["u_resample"]]
    ws = torch.empty(tslt.workspace_bytes(tslt.OP_VERIFY, B, G, V, K), dtype=torch.uint8, device=DEV)
    split = tslt.verify(*args, workspace=ws, phase="accept")
    tslt.verify(*args, out=split, workspace=ws, phase="resample")
    whole = tslt.verify(*args)
    torch.cuda.synchronize()
    for k in whole:
        assert torch.equal(whole[k], split[k]) or k in ("ratio", "beta") and torch.allclose(whole[k], split[k], equal_nan=True), k
    print(P.compare_verify(whole, ref["verify"], label="stress"), "accept_len", ref["verify"]["accept_len"])
    for first_stage in (1, G // 2):
        staged = tslt.verify(*args, first_stage=first_stage)
        torch.cuda.synchronize()
        for k in ("accept_len", "tokens", "status"):
            assert torch.equal(whole[k], staged[k]), (first_stage, k)
        P.compare_verify(staged, ref["verify"], label=f"stress staged {first_stage}")
    # a sequence that accepts every position reaches the bonus row at this shape too
    u0 = torch.zeros_like(chain["u_accept"])
    args[6] = u0
    ref_all = O.verify_chain(P.to_np(chain["target"]), w.T, ref["q_idx"], ref["q_logit"], ref["q_count"], ref["tokens"],
                             P.to_np(u0), P.to_np(chain["u_resample"]))
    out_all = tslt.verify(*args, first_stage=1)
    torch.cuda.synchronize()
    assert np.all(ref_all["accept_len"] == G)
    print(P.compare_verify(out_all, ref_all, label="stress all accepted"))


def test_verify_reports_a_malformed_received_set(tslt):
    """A received value that is not finite, or a token index outside the vocabulary, marks the position
    TSLT_ROW_BAD_SET: it counts as unusable (no token from it), the sequences around it are untouched."""
    w = W.scaled(W.WORKLOADS["chain_topk"], B=5, V=9001, gamma=3)
    chain = W.make_chain(w, 17, DEV)
    u_acc = torch.zeros_like(chain["u_accept"])               # every usable position accepts
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    q_idx, q_logit = t32(ref["q_idx"]), t32(ref["q_logit"])
    q_logit[1, 1, 3] = float("inf")
    q_logit[2, 0, 5] = float("nan")
    q_idx[3, 2, 7] = w.V                                       # one past the vocabulary
    out = tslt.verify(chain["target"], w.T, q_idx, q_logit, t32(ref["q_count"]), t32(ref["tokens"]), u_acc, chain["u_resample"])
    torch.cuda.synchronize()
    n, st, tok = P.to_np(out["accept_len"]), P.to_np(out["status"]), P.to_np(out["tokens"])
    assert n.tolist() == [3, 1, 0, 2, 3]
    assert (st & tslt.ROW_BAD_SET != 0).tolist() == [False, True, True, True, False]
    for b, j in ((1, 1), (2, 0), (3, 2)):
        assert tok[b, j] == -1 and np.all(tok[b, :j] == ref["tokens"][b, :j])
    P.compare_verify({k: v[[0, 4]] for k, v in out.items()},
                     {k: v[[0, 4]] for k, v in ref["verify"].items()}, label="untouched")


def test_verify_long_chain(tslt):
    """More draft positions than a wave has lanes: the first rejection is looked for beyond the first 64
    decisions, and the status words of all positions up to it are collected."""
    w = W.scaled(W.WORKLOADS["chain_topk"], B=4, V=3001, gamma=150, top_k=8, k_cap=8)
    chain = W.make_chain(w, 23, DEV)
    u_acc = chain["u_accept"].clone()
    u_acc[0, :70] = 0.0            # sequence 0: the first 70 positions accept whatever the ratio is
    u_acc[1, :] = 0.0              # sequence 1: everything accepted, the bonus row is sampled
    u_acc[2, :130] = 0.0           # sequence 2: the first rejection lies in the third group of 64
    chain["u_accept"] = u_acc
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    # sequence 3: a draft token outside its set far down the chain (its status bit has to reach the output)
    toks = ref["tokens"].copy()
    u3 = P.to_np(u_acc).copy()
    u3[3, :100] = 0.0
    toks[3, 90] = int(np.setdiff1d(np.arange(w.V), ref["q_idx"][3, 90])[0])
    v = O.verify_chain(P.to_np(chain["target"]), w.T, ref["q_idx"], ref["q_logit"], ref["q_count"], toks, u3,
                       P.to_np(chain["u_resample"]))
    out = tslt.verify(chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(toks),
                      t32(u3), chain["u_resample"])
    staged = tslt.verify(chain["target"], w.T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(toks),
                         t32(u3), chain["u_resample"], first_stage=5)
    torch.cuda.synchronize()
    assert v["accept_len"][0] >= 70 and v["accept_len"][1] == 150 and v["accept_len"][2] >= 130
    assert v["accept_len"][3] == 90 and v["status"][3] & 4
    print(P.compare_verify(out, v, label="long chain"), v["accept_len"])
    for k in ("accept_len", "tokens", "status"):
        assert torch.equal(out[k], staged[k]), k


@pytest.mark.parametrize("dtype,V", [("bf16", 3), ("bf16", 9), ("f16", 7), ("f32", 3), ("f32", 70), ("bf16", 130), ("f16", 2100)])
def test_verify_tiny_vocabularies(tslt, dtype, V):
    """Rows shorter than a 16-byte vector (everything is an edge element), of one or two vectors, of one run:
    the sweep has no run, or fewer runs than the resampling workgroup has waves."""
    K = min(V, 4)
    w = W.scaled(W.WORKLOADS["chain_topk"], B=7, V=V, gamma=3, dtype=dtype, top_k=K, k_cap=K, zipf=0.5, sigma=1.0)
    chain = W.make_chain(w, 29, DEV)
    u_acc = chain["u_accept"].clone()
    u_acc[0] = 0.0                                   # one sequence reaches the bonus row
    chain["u_accept"] = u_acc
    ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), w.T, w.top_k, w.top_p, w.k_cap,
                         P.to_np(chain["u_sample"]), P.to_np(u_acc), P.to_np(chain["u_resample"]))
    tr = tslt.truncate(chain["draft"], w.T, w.top_k, w.top_p, K, u=chain["u_sample"].view(-1, 1))
    out = run_verify_from_oracle_inputs(tslt, w, chain, ref)
    torch.cuda.synchronize()
    t = P.compare_truncate({k: v for k, v in tr.items() if k not in ("token", "slot")}, chain["draft"].view(-1, V), w.T, w.top_k,
                           w.top_p, K, label=f"tiny {dtype} {V}")
    assert t["top_p_near_ties"] == 0 and np.array_equal(P.to_np(tr["token"]).reshape(w.B, w.gamma), ref["tokens"])
    res = P.compare_verify(out, ref["verify"], label=f"tiny {dtype} {V}")
    assert res["accept_near_ties"] == 0 and ref["verify"]["accept_len"][0] == w.gamma
