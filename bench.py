#!/usr/bin/env python3
"""Benchmark of the TSLT hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic logits already resident in
HBM: tslt_truncate_sample on every draft row (truncation and the draw of the draft token in one launch),
tslt_verify (acceptance tests on every target row, then residual / bonus resampling).  Workload:
BASELINE config "large_vocab" (B=256, gamma=8, V=128256, bf16, T=0.7, top-p 0.9 with K cap 256).  Three
independent input sets (3.4 GB) are rotated so that the 256 MB Infinity Cache cannot serve repeats.

Prints ONE JSON line: positions/s (B*gamma per step), the roofline of the dominant kernel measured with an
event pair per step on the launch stream inside the timed region (an untimed pass with events at every
boundary gives the per-kernel breakdown first), and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def algorithmic_bytes(w):
    """Bytes the method has to move per step: every draft and target logit once, the sparse
    representation once out and once in.  Re-reads (the resampled row) earn no credit."""
    s = 2 if w.dtype == "bf16" else 4
    rows_d, rows_t = w.B * w.gamma, w.B * (w.gamma + 1)
    draft = rows_d * w.V * s
    sparse_w = rows_d * w.k_cap * (4 + 4 + 4)          # idx, logit, prob written by truncate
    sparse_r = rows_d * w.k_cap * (4 + 4)              # idx, logit read by verify
    target = rows_t * w.V * s
    return {"truncate": draft + sparse_w, "verify_accept": (rows_t - w.B) * w.V * s + sparse_r,
            "verify_resample": w.B * w.V * s, "total": draft + target + sparse_w + sparse_r}


def committed_traffic(kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", "large_vocab_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    m = re.search(rf"^traffic_bytes_per_launch\s+{kernel}\s+([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(w, host_set, budget_s=20.0):
    """The oracle as it stands, on the host cores, on a bounded sample of the same workload: whole
    sequences of one of the timed input sets (copied to the host), as many as fit the time budget."""
    from oracle import tslt_oracle as O
    draft, target = host_set["draft"], host_set["target"]
    t0 = time.perf_counter()
    done = 0
    for b in range(w.B):
        rows = draft[b].float().numpy()
        tr = O.truncate(rows, w.T, w.top_k, w.top_p, w.k_cap)
        smp = O.sample(tr["idx"], tr["logit"], tr["count"], host_set["u_sample"][b].numpy().reshape(w.gamma, 1))
        O.verify_chain_seq(target[b].float().numpy(), w.T, tr["idx"], tr["logit"], tr["count"], smp["token"][:, 0],
                           host_set["u_accept"][b].numpy(), host_set["u_resample"][b].numpy())
        done += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = time.perf_counter() - t0
    return {"value": round(done * w.gamma / dt, 2), "unit": "draft positions/s", "cores": 1, "kind": "oracle",
            "sample": f"first {done} of the {w.B} sequences (x gamma={w.gamma} positions) of input set 0 of the same "
                      f"workload: truncate+sample+verify, NumPy fp64, one thread, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--workload", default="large_vocab")
    ap.add_argument("--sets", type=int, default=3, help="independent input sets rotated between steps")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-events", action="store_true", help="time the steps without per-kernel events")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the timed steps run N plain elementwise copies of 1 GiB (read 1 GiB, write 1 GiB): "
                         "the launches that scale a profiler's FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (sequences would shard across GPUs with no exchange); "
              "run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_16273_amd import tslt, workloads as W
    tslt.load()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    dev = "cuda:0"
    w = W.WORKLOADS[args.workload]
    B, G, V, K = w.B, w.gamma, w.V, w.k_cap

    sets = []
    for i in range(args.sets):
        c = W.make_chain(w, 100 + i, dev)
        sets.append(c)
    # preallocated outputs and workspace: nothing is allocated inside the timed region
    tr_out = {"idx": torch.empty(B * G, K, dtype=torch.int32, device=dev),
              "logit": torch.empty(B * G, K, dtype=torch.float32, device=dev),
              "prob": torch.empty(B * G, K, dtype=torch.float32, device=dev),
              "count": torch.empty(B * G, dtype=torch.int32, device=dev),
              "mass": torch.empty(B * G, dtype=torch.float32, device=dev),
              "status": torch.empty(B * G, dtype=torch.int32, device=dev)}
    tr_out["token"] = torch.empty(B * G, 1, dtype=torch.int32, device=dev)
    tr_out["slot"] = torch.empty(B * G, 1, dtype=torch.int32, device=dev)
    vf_out = {"accept_len": torch.empty(B, dtype=torch.int32, device=dev),
              "tokens": torch.empty(B, G + 1, dtype=torch.int32, device=dev),
              "ratio": torch.empty(B, G, dtype=torch.float32, device=dev),
              "beta": torch.empty(B, G, dtype=torch.float32, device=dev),
              "status": torch.empty(B, dtype=torch.int32, device=dev)}
    ws = torch.empty(tslt.workspace_bytes(tslt.OP_VERIFY, B, G, V, K), dtype=torch.uint8, device=dev)
    q_idx, q_logit = tr_out["idx"].view(B, G, K), tr_out["logit"].view(B, G, K)
    q_count, toks = tr_out["count"].view(B, G), tr_out["token"].view(B, G)

    names = ["truncate", "verify_accept", "verify_resample"]

    def step(c, ev=None):
        """One pass of the hot path.  ev maps a boundary 0..3 (before truncate ... after resample) to an event."""
        ev = ev or {}
        if 0 in ev: ev[0].record()
        tslt.truncate(c["draft"], w.T, w.top_k, w.top_p, K, out=tr_out, u=c["u_sample"].view(B * G, 1))
        if 1 in ev: ev[1].record()
        tslt.verify(c["target"], w.T, q_idx, q_logit, q_count, toks, c["u_accept"], c["u_resample"], out=vf_out,
                    workspace=ws, phase="accept")
        if 2 in ev: ev[2].record()
        tslt.verify(c["target"], w.T, q_idx, q_logit, q_count, toks, c["u_accept"], c["u_resample"], out=vf_out,
                    workspace=ws, phase="resample")
        if 3 in ev: ev[3].record()

    def new_events(keys, n):
        return [{k: torch.cuda.Event(enable_timing=True) for k in keys} for _ in range(n)]

    for i in range(args.warmup):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()

    # untimed pass with an event at every boundary: the per-kernel breakdown, and which kernel dominates
    alg = algorithmic_bytes(w)
    kernels = {}
    dom = "truncate"
    if not args.no_events:
        n_prof = max(3, min(args.steps, 24))
        pe = new_events(range(4), n_prof)
        for i in range(n_prof):
            step(sets[i % len(sets)], pe[i])
        torch.cuda.synchronize()
        for k, name in enumerate(names):
            ts = [pe[i][k].elapsed_time(pe[i][k + 1]) for i in range(n_prof)]
            kernels[name] = {"avg_ms": round(sum(ts) / len(ts), 4), "min_ms": round(min(ts), 4)}
        for n in ("truncate", "verify_accept", "verify_resample"):
            kernels[n]["GBps"] = round(alg[n] / (kernels[n]["avg_ms"] * 1e-3) / 1e9, 1)
        dom = max(("truncate", "verify_accept"), key=lambda n: kernels[n]["avg_ms"])

    # the timed region: K steps; one event pair per step brackets the dominant kernel's launch
    events = None
    if not args.no_events:
        k0 = names.index(dom)
        events = new_events((k0, k0 + 1), args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)], events[i] if events else None)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    ms_per_step = dt / args.steps * 1e3
    roofline = None
    if events:
        k0 = names.index(dom)
        ts = [events[i][k0].elapsed_time(events[i][k0 + 1]) for i in range(args.steps)]
        avg_ms = sum(ts) / len(ts)
        kname = {"truncate": "truncate_kernel", "verify_accept": "verify_accept_kernel"}[dom]
        achieved = alg[dom] / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "algorithmic_bytes_per_launch": alg[dom], "avg_launch_ms": round(avg_ms, 4),
                    "traffic": committed_traffic(kname)}

    res = {
        "metric": "draft positions truncated+verified/sec at V=128k; achieved HBM GB/s vs peak",
        "value": round(B * G * args.steps / dt, 1), "unit": "draft positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: B={B} gamma={G} V={V} {w.dtype} logits, T={w.T}, top_p={w.top_p}, "
                               f"k_cap={K}; {args.sets} rotating input sets; truncate_sample+verify per step",
                   "storage_dtype": w.dtype},
        "hbm_GBps_whole_step": round(alg["total"] / (dt / args.steps) / 1e9, 1),
        "hbm_frac_whole_step": round(alg["total"] / (dt / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "kernels_untimed_pass": kernels, "roofline": roofline,
    }
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            torch.mul(src, 1.0, out=dst)          # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        host = {k: v.cpu() for k, v in sets[0].items() if torch.is_tensor(v)}
        res["cpu_baseline"] = cpu_baseline(w, host)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
