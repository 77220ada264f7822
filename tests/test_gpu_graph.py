"""The library enqueues kernels only (no allocation, no memset, no synchronisation), so a round can be
captured into a HIP graph and replayed.  Every replay is checked against the eager result."""
import pytest
import torch

from paper_2512_16273_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.mark.parametrize("first_stage", [0, 2])        # tslt_verify, and tslt_verify_staged (one launch per stage)
def test_captured_round_replays_like_eager(tslt, first_stage):
    w = W.scaled(W.WORKLOADS["chain_topp"], B=12, V=20011, gamma=4)
    B, G, V, K = w.B, w.gamma, w.V, w.k_cap
    sets = [W.make_chain(w, 20 + i, DEV) for i in range(3)]
    static = {k: v.clone() for k, v in sets[0].items() if torch.is_tensor(v)}
    ws = torch.empty(tslt.workspace_bytes(tslt.OP_VERIFY, B, G, V, K), dtype=torch.uint8, device=DEV)

    def run(c, tr=None, vf=None):
        tr = tslt.truncate(c["draft"], w.T, w.top_k, w.top_p, K, out=tr, u=c["u_sample"].view(B * G, 1), payload="bf16")
        vf = tslt.verify(c["target"], w.T, tr["idx"].view(B, G, K), tr["logit"].view(B, G, K), tr["count"].view(B, G),
                         tr["token"].view(B, G), c["u_accept"], c["u_resample"], out=vf, workspace=ws, first_stage=first_stage)
        return tr, vf

    eager = []
    for c in sets:
        tr, vf = run(c)
        torch.cuda.synchronize()
        eager.append(({k: v.clone() for k, v in tr.items()}, {k: v.clone() for k, v in vf.items()}))

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tr_s, vf_s = run(static)                      # warm-up on the capture stream; allocates the outputs
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run(static, tr_s, vf_s)
    for rep in range(2):
        for i, c in enumerate(sets):
            for k, v in static.items():
                v.copy_(c[k])
            torch.cuda.synchronize()                  # eager work and synchronisation between the replays
            graph.replay()
            torch.cuda.synchronize()
            for k, v in eager[i][0].items():
                assert torch.equal(tr_s[k].nan_to_num(), v.nan_to_num()), (rep, i, k)
            for k, v in eager[i][1].items():
                assert torch.equal(vf_s[k].nan_to_num(), v.nan_to_num()), (rep, i, k)
