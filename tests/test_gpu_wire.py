"""GPU parity: 16-bit payloads in tslt_truncate / tslt_truncate_sample and the wire format (tslt_pack,
tslt_unpack) through the C ABI against the CPU oracle (Section 2.2)."""
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


@pytest.mark.parametrize("payload", ["bf16", "f16"])
@pytest.mark.parametrize("name,V,rows,T,top_k,top_p,k_cap", [
    ("bf16-topp", 32000, 20, 0.8, 0, 0.95, 256),
    ("f32-topk", 5003, 9, 1.0, 16, 0.0, 16),
    ("bf16-k1024", 70000, 5, 1.0, 0, 0.999, 1024),
])
def test_truncate_with_16_bit_payload(tslt, payload, name, V, rows, T, top_k, top_p, k_cap):
    """The set and its mass as without rounding; the emitted values bit for bit the oracle's rounded ones;
    q_hat and the draws from the rounded values."""
    w = W.scaled(W.WORKLOADS["chain_topk"], V=V, dtype="f32" if name.startswith("f32") else "bf16")
    z = rows_like(w, rows, 41)
    u = W.uniforms((rows, 3), 6, 2, 5, DEV)
    out = tslt.truncate(z, T, top_k, top_p, k_cap, u=u, payload=payload)
    plain = tslt.truncate(z, T, top_k, top_p, k_cap)
    torch.cuda.synchronize()
    assert torch.equal(out["idx"], plain["idx"]) and torch.equal(out["count"], plain["count"])
    assert torch.equal(out["mass"], plain["mass"])
    ref = O.truncate(P.to_np(z), T, top_k, top_p, k_cap, payload)
    g = {k: P.to_np(v) for k, v in out.items()}
    for r in range(rows):
        if g["count"][r] != ref["count"][r]:
            assert ref["margin_rho"][r] < P.NEAR_TIE        # a nucleus decision at its boundary
            continue
        c = ref["count"][r]
        assert np.array_equal(g["logit"][r, :c], ref["logit"][r, :c]), (name, r)
        np.testing.assert_allclose(g["prob"][r], ref["prob"][r], rtol=P.RTOL, atol=1e-30)
    want = O.sample(g["idx"], g["logit"], g["count"], P.to_np(u), False)
    assert np.array_equal(g["slot"], want["slot"]) and np.array_equal(g["token"], want["token"])
    two = tslt.sample(out["idx"], out["logit"], out["count"], u, False)        # the receiver's view of q_hat
    assert torch.equal(two["token"], out["token"])


@pytest.mark.parametrize("payload,V,k_cap", [("bf16", 128256, 256), ("f16", 32000, 64), ("f16", 5, 8),
                                             ("bf16", 2 ** 31 - 1, 1024), ("f16", 151936, 32)])
def test_wire_format_matches_oracle_and_round_trips(tslt, payload, V, k_cap):
    rng = np.random.default_rng(V % 1000 + k_cap)
    rows = 37
    count = rng.integers(0, k_cap + 1, rows).astype(np.int32)
    count[:3] = [0, k_cap, 1]
    idx = np.full((rows, k_cap), -1, np.int32)
    logit = np.full((rows, k_cap), -np.inf, np.float32)
    for r in range(rows):
        c = count[r]
        idx[r, :c] = rng.integers(0, V, c)
        logit[r, :c] = np.sort(rng.normal(0, 6, c))[::-1].astype(np.float32)       # not yet rounded
    if count[1] >= 2:
        idx[1, 0], idx[1, 1] = V - 1, 0
    pk = tslt.pack(torch.from_numpy(idx).to(DEV), torch.from_numpy(logit).to(DEV), torch.from_numpy(count).to(DEV), V, payload)
    torch.cuda.synchronize()
    ref = O.pack_rows(idx, logit, count, V, payload)
    offs = P.to_np(pk["row_offset"])
    assert np.array_equal(offs, ref["row_offset"])
    words = P.to_np(pk["words"]).view(np.uint32)[:offs[-1]]
    assert np.array_equal(words, ref["words"])
    un = tslt.unpack(pk["words"], pk["row_offset"], rows, k_cap, V, payload)
    torch.cuda.synchronize()
    want = O.unpack_rows(ref["words"], ref["row_offset"], rows, k_cap, V, payload)
    assert np.array_equal(P.to_np(un["count"]), want["count"]) and np.array_equal(P.to_np(un["idx"]), want["idx"])
    assert np.array_equal(P.to_np(un["logit"]), want["logit"])
    assert np.array_equal(want["logit"][logit > -np.inf], O.round_payload(logit[logit > -np.inf], payload))


def test_device_to_server_round_over_the_wire(tslt):
    """Truncate with a bfloat16 payload, pack, unpack, verify: the receiver's sets are the sender's bit for bit,
    so the verification is the oracle's on the oracle's rounded sets."""
    w = W.scaled(W.WORKLOADS["chain_topp"], B=6, V=30011, gamma=5)
    c = W.make_chain(w, 3, DEV)
    B, G, V, K = w.B, w.gamma, w.V, w.k_cap
    tr = tslt.truncate(c["draft"], w.T, w.top_k, w.top_p, K, u=c["u_sample"].view(B * G, 1), payload="bf16")
    pk = tslt.pack(tr["idx"], tr["logit"], tr["count"], V, "bf16")
    rx = tslt.unpack(pk["words"], pk["row_offset"], B * G, K, V, "bf16")
    torch.cuda.synchronize()
    for k in ("idx", "logit", "count"):
        assert torch.equal(rx[k], tr[k]), k
    sent_bits = 32 * int(pk["row_offset"][-1])
    pairs_bits = int(tr["count"].sum()) * (O.index_bits(V) + 16)
    dense_bits = B * G * O.payload_bits(V, 16, 0)
    print("bits on the wire", sent_bits, "of which pairs", pairs_bits, "dense", dense_bits, "ratio", dense_bits / sent_bits)
    assert pairs_bits <= sent_bits <= pairs_bits + B * G * (16 + 31)
    vf = tslt.verify(c["target"], w.T, rx["idx"].view(B, G, K), rx["logit"].view(B, G, K), rx["count"].view(B, G),
                     tr["token"].view(B, G), c["u_accept"], c["u_resample"])
    torch.cuda.synchronize()
    ref = O.verify_chain(P.to_np(c["target"]), w.T, P.to_np(rx["idx"]).reshape(B, G, K), P.to_np(rx["logit"]).reshape(B, G, K),
                         P.to_np(rx["count"]).reshape(B, G), P.to_np(tr["token"]).reshape(B, G), P.to_np(c["u_accept"]),
                         P.to_np(c["u_resample"]))
    print(P.compare_verify(vf, ref, label="wire"))


def test_calibrate_read_runs_and_checks_its_arguments(tslt):
    """The measurement aid: a read-only launch over a buffer; sizes that do not split into whole rounds are refused."""
    buf = torch.ones(64 * 16384, dtype=torch.uint8, device=DEV)
    sink = torch.zeros(1, dtype=torch.int32, device=DEV)
    tslt.calibrate_read(buf, 64, sink)
    tslt.calibrate_read(buf, 1, sink)
    torch.cuda.synchronize()
    assert int(sink[0]) == 0                                  # the xor-sum of this data is not the constant
    with pytest.raises(tslt.TsltError):
        tslt.calibrate_read(buf, 48, sink)                    # 64 rounds do not split over 48 workgroups
    with pytest.raises(tslt.TsltError):
        tslt.calibrate_read(buf[:1000], 1, sink)
    with pytest.raises(tslt.TsltError):
        tslt.calibrate_read(buf[8:8 + 16384], 1, sink)        # not 16-byte aligned
