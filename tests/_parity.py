"""Helpers shared by the GPU parity tests: run the oracle on host copies, compare element by element.

Tolerances (from the benchmark spec): index sets, counts, accepted lengths and emitted tokens bit-exact,
except (a) sequences in which an acceptance test lies within 1e-6 of its boundary and (b) rows whose
Top-rho decision lies within 1e-6 (relative to the normaliser) of its boundary; both classes are
counted and returned.  Compacted logits are the same fp32 product on both sides (compared exactly);
probabilities, masses, ratios and beta within 1e-5 relative (fp32 outputs of fp64 arithmetic).
"""
import numpy as np
import torch

from oracle import tslt_oracle as O

NEAR_TIE = 1e-6
RTOL = 1e-5


def to_np(t):
    if isinstance(t, torch.Tensor):
        t = t.detach()
        if t.dtype == torch.bfloat16:
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
    near = 0
    exact_path = int(np.count_nonzero(g["status"] & 256))
    for r in range(n):
        tag = f"{label} row {rows[r]}"
        assert (g["status"][r] & 7) == ref["status"][r], (tag, g["status"][r], ref["status"][r])
        if g["count"][r] != ref["count"][r]:
            # only a Top-rho decision at its boundary may differ, and then by the boundary element
            assert ref["margin_rho"][r] < NEAR_TIE, (tag, g["count"][r], ref["count"][r], ref["margin_rho"][r])
            near += 1
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
    return dict(rows=n, top_p_near_ties=near, exact_path_rows=exact_path, ref=ref)


def compare_verify(gpu: dict, ref: dict, seqs=None, label=""):
    """GPU tslt_verify outputs against oracle verify_chain outputs (already computed) for the sequences
    `seqs` of the GPU batch.  Returns counters."""
    B = ref["accept_len"].shape[0]
    seqs = np.arange(B) if seqs is None else np.asarray(seqs)
    g = {k: to_np(v)[seqs] for k, v in gpu.items() if v is not None}
    near = 0
    gamma = ref["ratio"].shape[1]
    for b in range(B):
        tag = f"{label} seq {seqs[b]}"
        n = int(ref["accept_len"][b])
        examined = min(n + 1, gamma)
        if np.any(ref["accept_margin"][b, :examined] < NEAR_TIE):
            near += 1
            continue
        assert g["accept_len"][b] == n, (tag, g["accept_len"][b], n, ref["ratio"][b], g.get("ratio", [None])[b])
        assert np.array_equal(g["tokens"][b], ref["tokens"][b]), (tag, g["tokens"][b], ref["tokens"][b],
                                                                  ref["cdf_margin"][b])
        assert (g["status"][b] & 7) == ref["status"][b], (tag, g["status"][b], ref["status"][b])
        if "ratio" in g and ref["status"][b] == 0:
            rr = ref["ratio"][b, :examined]
            np.testing.assert_allclose(g["ratio"][b, :examined], rr, rtol=RTOL, atol=1e-30, err_msg=tag)
            np.testing.assert_allclose(g["beta"][b, :examined], ref["beta_hat"][b, :examined], rtol=RTOL, err_msg=tag)
    return dict(sequences=B, accept_near_ties=near)


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
