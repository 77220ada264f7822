"""Seeded random shapes and settings: the chain round (truncate with fused draws, verify, staged verify) against
the oracle.  Every case is printed before it runs, so that a failure names its shape and seed."""
import numpy as np
import pytest
import torch

from oracle import tslt_oracle as O  # noqa: F401  (the helpers in _parity use it)
from paper_2512_16273_amd import workloads as W
from tests import _parity as P

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def t32(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


@pytest.mark.parametrize("stream", [0, 1, 2, 3])
def test_random_chain_rounds(tslt, stream):
    rng = np.random.default_rng(1000 + stream)
    totals = dict(sequences=0, accept_near_ties=0, accept_near_tie_mismatches=0, top_p_near_ties=0, top_p_near_tie_mismatches=0)
    for case in range(12):
        dtype = ["f32", "bf16", "f16"][rng.integers(3)]
        V = int(rng.choice([rng.integers(50, 3000), rng.integers(3000, 40000), rng.integers(40000, 90000)]))
        gamma = int(rng.integers(1, 9))
        B = int(rng.integers(1, 7))
        mode = rng.integers(3)                       # top-k only, top-p only, both
        k_cap = int(rng.choice([1, 4, 16, 64, 256, 1024]))
        top_k = int(rng.integers(1, k_cap + 1)) if mode != 1 else 0
        top_p = float(rng.choice([0.5, 0.9, 0.99, 0.999])) if mode != 0 else 0.0
        T = float(rng.choice([0.3, 0.7, 1.0, 1.5]))
        shift = float(rng.choice([0.0, 0.0, np.log(V) - 1.0]))      # a third of the cases: bulk of a row at 0
        base = ["chain_topk", "large_vocab", "stress"][rng.integers(3)]
        w = W.scaled(W.WORKLOADS[base], B=B, V=V, gamma=gamma, dtype=dtype, top_k=top_k, top_p=top_p, k_cap=k_cap, T=T,
                     shift=shift, noise_t=float(rng.choice([0.3, 0.8, 2.0])))
        seed = int(rng.integers(1 << 30))
        first_stage = int(rng.integers(1, gamma + 1))
        print(f"case {stream}.{case}: {base} {dtype} B={B} gamma={gamma} V={V} top_k={top_k} top_p={top_p} k_cap={k_cap} "
              f"T={T} shift={shift:.2f} seed={seed} first_stage={first_stage}", flush=True)
        chain = W.make_chain(w, seed, DEV)
        rows = chain["draft"].view(B * gamma, V)
        tr = tslt.truncate(rows, T, top_k, top_p, k_cap, u=chain["u_sample"].view(B * gamma, 1))
        torch.cuda.synchronize()
        res = P.compare_truncate({k: v for k, v in tr.items() if k not in ("token", "slot")}, rows, T, top_k, top_p, k_cap,
                                 label=f"case {stream}.{case}")
        ref = P.oracle_chain(P.to_np(chain["draft"]), P.to_np(chain["target"]), T, top_k, top_p, k_cap,
                             P.to_np(chain["u_sample"]), P.to_np(chain["u_accept"]), P.to_np(chain["u_resample"]))
        if res["top_p_near_tie_mismatches"] == 0:
            assert np.array_equal(P.to_np(tr["token"]).reshape(B, gamma), ref["tokens"]), case
        args = [chain["target"], T, t32(ref["q_idx"]), t32(ref["q_logit"]), t32(ref["q_count"]), t32(ref["tokens"]),
                chain["u_accept"], chain["u_resample"]]
        out = tslt.verify(*args)
        staged = tslt.verify(*args, first_stage=first_stage)
        torch.cuda.synchronize()
        r = P.compare_verify(out, ref["verify"], label=f"case {stream}.{case}")
        for k in ("accept_len", "tokens", "status"):
            assert torch.equal(out[k], staged[k]), (case, k)
        totals["sequences"] += B
        for k in ("accept_near_ties", "accept_near_tie_mismatches"):
            totals[k] += r[k]
        totals["top_p_near_tie_mismatches"] += res["top_p_near_tie_mismatches"]
        totals["top_p_near_ties"] += res["top_p_near_ties"]
    print(totals)
