"""tslt_verify_static (the entry point for callers that cannot allocate) against tslt_verify, through the C ABI:
two calls in a row on the same GPU, the second with a smaller input, so that the second call finds the first
call's contents in the library's static scratch array."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2512_16273_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def inputs(tslt, w, seed):
    chain = W.make_chain(w, seed, DEV)
    B, G, V, K = w.B, w.gamma, w.V, w.k_cap
    tr = tslt.truncate(chain["draft"].view(B * G, V), w.T, w.top_k, w.top_p, K, u=chain["u_sample"].view(B * G, 1))
    return [chain["target"], w.T, tr["idx"].view(B, G, K), tr["logit"].view(B, G, K), tr["count"].view(B, G),
            tr["token"].view(B, G), chain["u_accept"], chain["u_resample"]]


def empty_out(B, G):
    i32, f32 = torch.int32, torch.float32
    return {"accept_len": torch.full((B,), -7, dtype=i32, device=DEV), "tokens": torch.full((B, G + 1), -7, dtype=i32, device=DEV),
            "ratio": torch.full((B, G), -7.0, dtype=f32, device=DEV), "beta": torch.full((B, G), -7.0, dtype=f32, device=DEV),
            "status": torch.full((B,), -7, dtype=i32, device=DEV)}


def test_static_scratch_entry_point_matches_verify(tslt):
    big = W.scaled(W.WORKLOADS["chain_topp"], B=24, V=20011, gamma=8)
    small = W.scaled(W.WORKLOADS["chain_topk"], B=5, V=9001, gamma=3, dtype="f32")
    for w, seed in ((big, 31), (small, 32)):
        args = inputs(tslt, w, seed)
        want = tslt.verify(*args)
        torch.cuda.synchronize()
        got = tslt.verify_static(*args, out=empty_out(w.B, w.gamma))
        torch.cuda.synchronize()
        for k in ("accept_len", "tokens", "status"):
            assert torch.equal(got[k], want[k]), (w.name, k)
        for k in ("ratio", "beta"):
            assert torch.equal(got[k].view(torch.int32), want[k].view(torch.int32)), (w.name, k)     # same kernels: same bits
        assert int(want["accept_len"].min()) >= 0
    # both kinds of sequence occurred, so the decisions really travelled through the scratch array
    assert len(set(want["accept_len"].tolist())) > 1


def test_static_scratch_entry_point_rejects_what_does_not_fit(tslt):
    lib = tslt.load()
    vp = ctypes.c_void_p
    one = torch.zeros(64, dtype=torch.float32, device=DEV)
    p = vp(one.data_ptr())
    B, G = 1 << 16, 8                                    # 524288 positions > TSLT_STATIC_MAX_POSITIONS
    assert B * G > tslt.STATIC_MAX_POSITIONS
    rc = lib.tslt_verify_static(p, tslt.F32, B, G, 16, 16, 1.0, p, p, p, 4, p, p, p, p, p, p, p, p, None)
    assert rc == -2 and b"static scratch" in lib.tslt_last_error()
    torch.cuda.synchronize()
