#!/usr/bin/env python3
"""Benchmark of the TSLT hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic logits already resident in HBM.
Chain workloads (default: benchmark configuration 3, "large_vocab", B=256, gamma=8, V=128256, bf16, T=0.7, top-p 0.9
with K cap 256): tslt_truncate_sample on every draft row (truncation and the draw of the draft token in
one launch), tslt_verify_accept on every target row, tslt_verify_resample (residual / bonus token).
Tree workload ("tree", benchmark configuration 4): tslt_truncate_sample on the draft row of every non-leaf
node (truncation and the draws of its candidates in one launch), tslt_verify_tree over the whole tree.
Independent input sets are rotated so that the 256 MB Infinity Cache cannot serve repeats.

Prints ONE JSON line: positions/s, the roofline of the dominant kernel measured with an event pair per
step on the launch stream inside the timed region (an untimed pass with events at every boundary gives
the per-kernel breakdown first), and the CPU oracle timed on a bounded sample.
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


def committed_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None
    m = re.search(rf"^traffic_bytes_per_launch\s+{kernel}\s+([0-9.eE+]+)", open(path).read(), re.M)
    return float(m.group(1)) if m else None


class ChainPlan:
    """truncate_sample -> verify_accept -> verify_resample on a chain workload."""

    def __init__(self, w, n_sets, torch, tslt, W, dev, sets=None):
        self.w, self.torch, self.tslt = w, torch, tslt
        B, G, V, K = w.B, w.gamma, w.V, w.k_cap
        self.sets = sets if sets is not None else [W.make_chain(w, 100 + i, dev) for i in range(n_sets)]
        self.first_stage = 0
        i32, f32 = torch.int32, torch.float32
        # preallocated outputs and workspace: nothing is allocated inside the timed region
        self.tr = {"idx": torch.empty(B * G, K, dtype=i32, device=dev), "logit": torch.empty(B * G, K, dtype=f32, device=dev),
                   "prob": torch.empty(B * G, K, dtype=f32, device=dev), "count": torch.empty(B * G, dtype=i32, device=dev),
                   "mass": torch.empty(B * G, dtype=f32, device=dev), "status": torch.empty(B * G, dtype=i32, device=dev),
                   "token": torch.empty(B * G, 1, dtype=i32, device=dev), "slot": torch.empty(B * G, 1, dtype=i32, device=dev)}
        self.vf = {"accept_len": torch.empty(B, dtype=i32, device=dev), "tokens": torch.empty(B, G + 1, dtype=i32, device=dev),
                   "ratio": torch.empty(B, G, dtype=f32, device=dev), "beta": torch.empty(B, G, dtype=f32, device=dev),
                   "status": torch.empty(B, dtype=i32, device=dev)}
        self.ws = torch.empty(tslt.workspace_bytes(tslt.OP_VERIFY, B, G, V, K), dtype=torch.uint8, device=dev)
        self.positions = B * G
        s = 4 if w.dtype == "f32" else 2
        # bytes the method has to move: every draft and target logit once, the sparse representation once out
        # and once in; re-reads (the resampled row) earn no credit
        sparse_w = B * G * K * 12 + B * G * 8
        sparse_r = B * G * K * 8
        self.ops = [("truncate", "truncate_kernel", self.truncate, B * G * V * s + sparse_w),
                    ("verify_accept", "verify_accept_kernel", self.accept, B * G * V * s + sparse_r),
                    ("verify_resample", "verify_resample_kernel", self.resample, B * V * s)]
        self.total_bytes = B * G * V * s + B * (G + 1) * V * s + sparse_w + sparse_r
        self.describe = (f"{w.name}: B={B} gamma={G} V={V} {w.dtype} logits{f' shifted by {w.shift:+g}' if w.shift else ''}, "
                         f"T={w.T}, top_k={w.top_k}, top_p={w.top_p}, "
                         f"k_cap={K}; {n_sets} rotating input sets; truncate_sample+verify per step")

    def _verify(self, c, phase):
        w, t = self.w, self.tr
        B, G, K = w.B, w.gamma, w.k_cap
        self.tslt.verify(c["target"], w.T, t["idx"].view(B, G, K), t["logit"].view(B, G, K), t["count"].view(B, G),
                         t["token"].view(B, G), c["u_accept"], c["u_resample"], out=self.vf, workspace=self.ws, phase=phase,
                         first_stage=self.first_stage)

    def truncate(self, c):
        w = self.w
        self.tslt.truncate(c["draft"], w.T, w.top_k, w.top_p, w.k_cap, out=self.tr, u=c["u_sample"].view(w.B * w.gamma, 1))

    def accept(self, c):
        self._verify(c, "accept")

    def resample(self, c):
        self._verify(c, "resample")

    def cpu_baseline(self, budget_s=20.0):
        """The oracle as it stands, on the host cores, on a bounded sample of the same workload: whole
        sequences of one of the timed input sets (copied to the host), as many as fit the time budget."""
        from oracle import tslt_oracle as O
        w = self.w
        host = {k: v.cpu() for k, v in self.sets[0].items() if self.torch.is_tensor(v)}
        t0 = time.perf_counter()
        done = 0
        for b in range(w.B):
            tr = O.truncate(host["draft"][b].float().numpy(), w.T, w.top_k, w.top_p, w.k_cap)
            smp = O.sample(tr["idx"], tr["logit"], tr["count"], host["u_sample"][b].numpy().reshape(w.gamma, 1))
            O.verify_chain_seq(host["target"][b].float().numpy(), w.T, tr["idx"], tr["logit"], tr["count"], smp["token"][:, 0],
                               host["u_accept"][b].numpy(), host["u_resample"][b].numpy())
            done += 1
            if time.perf_counter() - t0 > budget_s:
                break
        dt = time.perf_counter() - t0
        return {"value": round(done * w.gamma / dt, 2), "unit": "draft positions/s", "cores": 1, "kind": "oracle",
                "sample": f"first {done} of the {w.B} sequences (x gamma={w.gamma} positions) of input set 0 of the same "
                          f"workload: truncate+sample+verify, NumPy fp64, one thread, {dt:.1f} s"}


class TreePlan:
    """truncate -> sample (k candidates per non-leaf node) -> verify_tree on the token-tree workload."""

    def __init__(self, w, n_sets, torch, tslt, W, dev):
        self.w, self.torch, self.tslt = w, torch, tslt
        self.sets = [W.make_tree(w, 100 + i, dev) for i in range(n_sets)]
        sh = self.sets[0]["shape"]
        B, V, K = w.B, w.V, w.k_cap
        self.n_int, self.n_nodes, self.kmax = sh["n_internal"], sh["n_nodes"], max(w.expansion)
        n_int, n_nodes, kmax = self.n_int, self.n_nodes, self.kmax
        i32, f32 = torch.int32, torch.float32
        R = B * n_int
        self.tr = {"idx": torch.empty(R, K, dtype=i32, device=dev), "logit": torch.empty(R, K, dtype=f32, device=dev),
                   "prob": torch.empty(R, K, dtype=f32, device=dev), "count": torch.empty(R, dtype=i32, device=dev),
                   "mass": torch.empty(R, dtype=f32, device=dev), "status": torch.empty(R, dtype=i32, device=dev)}
        self.tr["token"] = torch.empty(R, kmax, dtype=i32, device=dev)
        self.tr["slot"] = torch.empty(R, kmax, dtype=i32, device=dev)
        self.vt = {"seq": torch.empty(B, len(w.expansion) + 1, dtype=i32, device=dev), "len": torch.empty(B, dtype=i32, device=dev),
                   "node_token": None, "node_slot": None, "ratio": torch.empty(B, n_nodes - 1, dtype=f32, device=dev),
                   "status": torch.empty(B, dtype=i32, device=dev)}
        self.ws = torch.empty(tslt.workspace_bytes(tslt.OP_VERIFY_TREE_PATH, B, n_nodes, V, K), dtype=torch.uint8, device=dev)
        if len(set(w.expansion)) != 1:
            raise SystemExit("bench.py: the tree workload needs the same number of candidates at every layer")
        self.positions = B * (n_nodes - 1)                 # candidate nodes
        s = 4 if w.dtype == "f32" else 2
        sparse = R * K * 12
        # the verified path needs at most depth + 1 target rows per tree (uniforms are indexed by node, so the
        # nodes off the path never influence the output); every draft row is needed for its candidates
        path_rows = B * (len(w.expansion) + 1)
        self.ops = [("truncate", "truncate_kernel", self.truncate, R * V * s + sparse),
                    ("verify_tree", "tree_lazy_walk_kernel", self.verify, path_rows * V * s + path_rows * K * 8)]
        self.total_bytes = R * V * s + sparse + path_rows * V * s + path_rows * K * 8
        self.describe = (f"{w.name}: B={B} trees, expansion={tuple(w.expansion)} ({n_int} non-leaf of {n_nodes} nodes), V={V} "
                         f"{w.dtype} logits, T={w.T}, top_k={w.top_k}, k_cap={K}, candidates drawn "
                         f"{'without' if w.without_replacement else 'with'} replacement and verified by the matching rule, only "
                         f"the verified path is sampled; {n_sets} rotating input sets; truncate_sample+verify_tree per step")

    def truncate(self, c):
        # truncation and the draws of every node's candidates in one launch (tslt_truncate_sample)
        w = self.w
        self.tslt.truncate(c["draft"], w.T, w.top_k, w.top_p, w.k_cap, out=self.tr, u=c["u_sample"].view(-1, self.kmax),
                           without_replacement=w.without_replacement)

    def verify(self, c):
        w, t = self.w, self.tr
        B, K, n_int = w.B, w.k_cap, self.n_int
        # children of node n are the kmax consecutive nodes from 1 + n*kmax: the candidates of all non-leaf nodes,
        # node after node, are the tree's candidate array
        self.tslt.verify_tree(c["target"], w.T, w.expansion, t["idx"].view(B, n_int, K), t["logit"].view(B, n_int, K),
                              t["count"].view(B, n_int), t["token"].view(B, n_int * self.kmax), c["u_accept"], c["u_resample"],
                              all_nodes=False, out=self.vt, workspace=self.ws, without_replacement=w.without_replacement)

    def cpu_baseline(self, budget_s=20.0):
        """The oracle on whole trees of input set 0, as many as fit the time budget (at least one)."""
        from oracle import tslt_oracle as O
        import numpy as np
        w = self.w
        c = self.sets[0]
        n_int, n_nodes, kmax = self.n_int, self.n_nodes, self.kmax
        t0 = time.perf_counter()
        done = 0
        for b in range(w.B):
            draft = c["draft"][b].float().cpu().numpy()
            target = c["target"][b].float().cpu().numpy()
            tr = O.truncate(draft, w.T, w.top_k, w.top_p, w.k_cap)
            smp = O.sample(tr["idx"], tr["logit"], tr["count"], c["u_sample"][b].cpu().numpy(), w.without_replacement)
            O.verify_tree_seq(target, w.T, w.expansion, tr["idx"], tr["logit"], tr["count"],
                              smp["token"].reshape(n_int * kmax).astype(np.int32), c["u_accept"][b].cpu().numpy(),
                              c["u_resample"][b].cpu().numpy(), w.without_replacement)
            done += 1
            if time.perf_counter() - t0 > budget_s:
                break
        dt = time.perf_counter() - t0
        return {"value": round(done * (n_nodes - 1) / dt, 2), "unit": "draft positions/s", "cores": 1, "kind": "oracle",
                "sample": f"first {done} of the {w.B} trees ({n_nodes - 1} candidate nodes each) of input set 0 of the same "
                          f"workload, every node evaluated: truncate+sample+verify_tree, NumPy fp64, one thread, {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--workload", default="large_vocab")
    ap.add_argument("--dtype", default="", choices=["", "f32", "bf16", "f16"], help="override the workload's logit storage type")
    ap.add_argument("--shift", type=float, default=0.0, help="constant added to every logit of the workload (the Zipf recipe "
                    "centres a row's bulk near -ln V; a shift of +ln V - 1 centres it on 0, where 16-bit formats are densest)")
    ap.add_argument("--first-stage", type=int, default=0, help="chain workloads: take the acceptance tests in stages "
                    "(tslt_verify_accept_staged) with this many positions in the first stage; 0 = one launch")
    ap.add_argument("--no-staged", action="store_true", help="skip the extra measurement with staged acceptance tests")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's B (sequences or trees)")
    ap.add_argument("--sets", type=int, default=0, help="independent input sets rotated between steps (default 3; 1 for tree)")
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
    if args.batch > 0:
        w = W.scaled(w, B=args.batch)
    if args.dtype:
        w = W.scaled(w, dtype=args.dtype)
    if args.shift != 0.0:
        w = W.scaled(w, shift=args.shift)
    is_tree = len(w.expansion) > 0
    n_sets = args.sets if args.sets > 0 else (1 if is_tree else 3)
    plan = (TreePlan if is_tree else ChainPlan)(w, n_sets, torch, tslt, W, dev)
    if args.first_stage > 0 and not is_tree:
        plan.first_stage = args.first_stage
        plan.describe += f"; acceptance in stages from {args.first_stage} positions"
    sets, ops = plan.sets, plan.ops
    n_ops = len(ops)

    def step(c, ev=None):
        """One pass of the hot path.  ev maps a boundary 0..n_ops (before the first call ... after the last) to an
        event."""
        ev = ev or {}
        for k, (_, _, fn, _) in enumerate(ops):
            if k in ev: ev[k].record()
            fn(c)
        if n_ops in ev: ev[n_ops].record()

    def new_events(keys, n):
        return [{k: torch.cuda.Event(enable_timing=True) for k in keys} for _ in range(n)]

    for i in range(args.warmup):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()

    # untimed pass with an event at every boundary: the per-kernel breakdown, and which call dominates
    kernels = {}
    dom = 0
    if not args.no_events:
        n_prof = max(3, min(args.steps, 24))
        pe = new_events(range(n_ops + 1), n_prof)
        for i in range(n_prof):
            step(sets[i % len(sets)], pe[i])
        torch.cuda.synchronize()
        for k, (name, _, _, nbytes) in enumerate(ops):
            ts = [pe[i][k].elapsed_time(pe[i][k + 1]) for i in range(n_prof)]
            avg = sum(ts) / len(ts)
            kernels[name] = {"avg_ms": round(avg, 4), "min_ms": round(min(ts), 4), "GBps": round(nbytes / (avg * 1e-3) / 1e9, 1)}
        dom = max(range(n_ops), key=lambda k: kernels[ops[k][0]]["avg_ms"])

    # the timed region: K steps; one event pair per step brackets the dominant call
    events = None
    if not args.no_events:
        events = new_events((dom, dom + 1), args.steps)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)], events[i] if events else None)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    roofline = None
    if events:
        ts = [events[i][dom].elapsed_time(events[i][dom + 1]) for i in range(args.steps)]
        avg_ms = sum(ts) / len(ts)
        _, kname, _, nbytes = ops[dom]
        achieved = nbytes / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": round(avg_ms, 4),
                    "traffic": committed_traffic(w.name, kname)}

    res = {
        "metric": "draft positions truncated+verified/sec at V=128k; achieved HBM GB/s vs peak",
        "value": round(plan.positions * args.steps / dt, 1), "unit": "draft positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": plan.describe, "storage_dtype": w.dtype},
        "hbm_GBps_whole_step": round(plan.total_bytes / (dt / args.steps) / 1e9, 1),
        "hbm_frac_whole_step": round(plan.total_bytes / (dt / args.steps) / 1e9 / HBM_PEAK_GBS, 4),
        "kernels_untimed_pass": kernels, "roofline": roofline,
    }
    if not is_tree and plan.first_stage > 0:
        # rows after a rejection are not read: the all-rows byte count does not describe this run
        res["hbm_GBps_whole_step"] = res["hbm_frac_whole_step"] = None
        if "verify_accept" in kernels:
            kernels["verify_accept"]["GBps"] = None
    elif not is_tree and not args.no_staged:
        # beside the headline (every position evaluated): the same steps with the acceptance tests taken in
        # two stages, which does not read the target rows behind a rejection found in the first half
        plan.first_stage = max(1, w.gamma // 2)
        for i in range(3):
            step(sets[i % len(sets)])
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for i in range(args.steps):
            step(sets[i % len(sets)])
        torch.cuda.synchronize()
        dt1 = time.perf_counter() - t1
        plan.first_stage = 0
        res["staged_acceptance"] = {"first_stage": max(1, w.gamma // 2), "ms_per_step": round(dt1 / args.steps * 1e3, 4),
                                    "value": round(plan.positions * args.steps / dt1, 1), "unit": "draft positions/s",
                                    "note": "same outputs (accept_len, tokens); ratio and beta of skipped positions are NaN"}
    if not is_tree and not args.no_staged:
        # beside the headline (one stream, a step starts when the one before it has ended): the same steps
        # issued alternately on two streams, each with its own outputs and workspace, as a server with two
        # batches in flight would; the ramp and the tail of one step's kernels are then covered by the other's
        plans = [plan, ChainPlan(w, n_sets, torch, tslt, W, dev, sets=sets)]
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]         # default priority
        def run2(n):
            for i in range(n):
                with torch.cuda.stream(streams[i % 2]):
                    for (_, _, fn, _) in plans[i % 2].ops:
                        fn(sets[i % len(sets)])
            torch.cuda.synchronize()
        run2(4)
        t2 = time.perf_counter()
        run2(args.steps)
        dt2 = time.perf_counter() - t2
        res["two_streams"] = {"ms_per_step": round(dt2 / args.steps * 1e3, 4),
                              "value": round(plan.positions * args.steps / dt2, 1), "unit": "draft positions/s",
                              "note": "steps alternate between two streams (two batches in flight); every position evaluated"}
        for q in plans:
            q.first_stage = max(1, w.gamma // 2)
        run2(4)
        t3 = time.perf_counter()
        run2(args.steps)
        dt3 = time.perf_counter() - t3
        for q in plans:
            q.first_stage = 0
        res["two_streams"]["with_staged_acceptance"] = {"ms_per_step": round(dt3 / args.steps * 1e3, 4),
                                                        "value": round(plan.positions * args.steps / dt3, 1)}
    if not args.copy_calibration:
        # what this chip delivers to a kernel that only reads (same load shape as the dense passes): the practical
        # ceiling beside the published peak.  2048 chunks of 256 KiB, three buffers in turn, events on this stream
        bufs = [torch.ones(1 << 29, dtype=torch.uint8, device=dev) for _ in range(3)]
        sink = torch.zeros(1, dtype=torch.int32, device=dev)
        for i in range(6):
            tslt.calibrate_read(bufs[i % 3], 2048, sink)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        n_cal = 30
        e0.record()
        for i in range(n_cal):
            tslt.calibrate_read(bufs[i % 3], 2048, sink)
        e1.record()
        torch.cuda.synchronize()
        cal = (1 << 29) * n_cal / (e0.elapsed_time(e1) * 1e-3) / 1e9
        res["read_ceiling"] = {"GBps": round(cal, 1), "frac_of_peak": round(cal / HBM_PEAK_GBS, 4),
                               "dominant_kernel_frac": round(roofline["achieved"] / cal, 4) if roofline else None,
                               "note": "tslt_calibrate_read: read-only kernel, 16-byte nontemporal loads, 512 MiB per launch"}
        del bufs
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            torch.mul(src, 1.0, out=dst)          # one elementwise kernel: 2^30 bytes in, 2^30 bytes out
        torch.cuda.synchronize()
        del src, dst
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = plan.cpu_baseline()
    print(json.dumps(res))


if __name__ == "__main__":
    main()
