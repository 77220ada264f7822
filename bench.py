#!/usr/bin/env python3
"""Benchmark of the TSLT hot path on one MI355X.

One step = one pass of the whole hot path over one batch of synthetic logits already resident in HBM.
Chain workloads (default: benchmark configuration 3, "large_vocab", B=256, gamma=8, V=128256, bf16, T=0.7, top-p 0.9
with K cap 256): tslt_truncate_sample on every draft row (truncation and the draw of the draft token in
one launch), tslt_verify_accept on every target row, tslt_verify_resample (residual / bonus token).
Tree workload ("tree", benchmark configuration 4): tslt_truncate_sample on the draft row of every non-leaf
node (truncation and the draws of its candidates in one launch), tslt_verify_tree over the whole tree.
Independent input sets are rotated so that the 256 MB Infinity Cache cannot serve repeats.

Prints ONE JSON line: positions/s, the roofline of the dominant kernel measured with an event pair on
the launch stream around that kernel in every eighth step of the timed region (an untimed pass with events at every boundary gives
the per-kernel breakdown first), the CPU oracle timed on a bounded sample (one thread, then all cores), and
a parity report: the GPU's outputs for the very sequences the oracle was timed on, compared item by item,
with the near-tie classes counted.

`--stats-sweep` instead prints the synthetic analogue of the paper's Top-K-mass and acceptance-rate figures
(Sections 5.1, 5.2): retained mass and acceptance rate against K, and the multi-candidate rates.
"""
import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


NEAR_TIE = 1e-6          # the near-tie window of the parity report (accept test, Top-rho boundary)
AMP_CAP = 64.0           # widest factor by which the window of a later multi-candidate stage is stretched


def committed_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` from the committed rocprofv3 --pmc summary (not measured in this run:
    counters need the profiler), and a note saying which file and which commit of the kernels it describes."""
    rel = os.path.join("profiles", f"{workload}_hbm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = re.search(rf"^traffic_bytes_per_launch\s+{kernel}\s+([0-9.eE+]+)", text, re.M)
    c = re.search(r"^taken at commit\s+(\S+)", text, re.M)
    note = f"{rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, taken at commit {c.group(1) if c else 'unknown'})"
    return (float(m.group(1)) if m else None), note


def timed_pool(fn, items, threads, budget_s):
    """Runs fn(item) over `items` on `threads` host threads until the time budget is used up.  Returns the
    results of the items that were finished, in order, and the elapsed seconds."""
    t0 = time.perf_counter()
    out = []
    if threads <= 1:
        for it in items:
            out.append(fn(it))
            if time.perf_counter() - t0 > budget_s:
                break
        return out, time.perf_counter() - t0
    with ThreadPoolExecutor(max_workers=threads) as pool:
        pending = []
        it = iter(items)
        for _ in range(threads):
            nxt = next(it, None)
            if nxt is None:
                break
            pending.append(pool.submit(fn, nxt))
        while pending:
            out.append(pending.pop(0).result())
            if time.perf_counter() - t0 <= budget_s:
                nxt = next(it, None)
                if nxt is not None:
                    pending.append(pool.submit(fn, nxt))
    return out, time.perf_counter() - t0


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

    def cpu_baseline_and_parity(self, budget_s=20.0):
        """The oracle as it stands, on the host cores, on a bounded sample of the same workload: whole sequences
        of input set 0 (copied to the host), first on one thread, then on all cores with sequences split across
        threads, as many as fit the time budget.  The GPU's outputs for the same sequences (one more step on
        input set 0, every position evaluated) are then compared with the oracle's, item by item."""
        from oracle import tslt_oracle as O
        import numpy as np
        w, torch = self.w, self.torch
        B, G, K = w.B, w.gamma, w.k_cap
        self.first_stage = 0
        for (_, _, fn, _) in self.ops:
            fn(self.sets[0])
        torch.cuda.synchronize()
        g_tr = {k: v.cpu().numpy() for k, v in self.tr.items()}
        g_vf = {k: v.cpu().numpy() for k, v in self.vf.items()}
        host = {k: v.cpu() for k, v in self.sets[0].items() if torch.is_tensor(v)}

        def one(b):
            t0 = time.perf_counter()
            tr = O.truncate(host["draft"][b].float().numpy(), w.T, w.top_k, w.top_p, K)
            smp = O.sample(tr["idx"], tr["logit"], tr["count"], host["u_sample"][b].numpy().reshape(G, 1))
            t1 = time.perf_counter()
            vr = O.verify_chain_seq(host["target"][b].float().numpy(), w.T, tr["idx"], tr["logit"], tr["count"], smp["token"][:, 0],
                                    host["u_accept"][b].numpy(), host["u_resample"][b].numpy())
            return b, tr, smp, vr, t1 - t0, time.perf_counter() - t1

        host_cores = os.cpu_count() or 1
        threads = max(1, min(16, host_cores))
        r1, dt1 = timed_pool(one, range(B), 1, 0.3 * budget_s)
        r2, dt2 = timed_pool(one, range(len(r1), B), threads, 0.7 * budget_s) if len(r1) < B else ([], 0.0)

        def leg(res, dt, n_threads):
            if not res:
                return None
            pos = len(res) * G
            t_tr, t_vf = sum(r[4] for r in res), sum(r[5] for r in res)
            return {"value": round(pos / dt, 2), "unit": "draft positions/s", "threads": n_threads, "sequences": len(res),
                    "seconds": round(dt, 2),
                    # the two halves, by the share of the thread time each took
                    "truncate_sample_value": round(pos / (dt * t_tr / (t_tr + t_vf)), 2),
                    "verify_value": round(pos / (dt * t_vf / (t_tr + t_vf)), 2)}
        single, allc = leg(r1, dt1, 1), leg(r2, dt2, threads)
        best = allc if allc and allc["value"] > single["value"] else single
        baseline = {"value": best["value"], "unit": "draft positions/s", "cores": best["threads"], "kind": "oracle",
                    "host_cores": host_cores, "single_thread": single, "all_cores": allc,
                    "sample": f"whole sequences (x gamma={G} positions) of input set 0 of the same workload, truncate+sample+verify, "
                              f"NumPy {np.__version__} fp64: sequences 0..{len(r1) - 1} on one thread in {dt1:.1f} s, then sequences "
                              f"{len(r1)}..{len(r1) + len(r2) - 1} split over {threads} threads in {dt2:.1f} s"}

        # ---- parity of the GPU's outputs for those sequences ----
        par = dict(sequences=0, positions=0, exact_index_sets=0, exact_draft_tokens=0, exact_accept_len=0, exact_tokens=0,
                   accept_near_ties=0, accept_near_tie_mismatches=0, top_rho_near_ties=0, top_rho_near_tie_mismatches=0,
                   cdf_edge_near_ties=0, mc_amp_near_ties=0, exact_path_rows=0, unexplained_mismatches=0,
                   max_rel_err_prob=0.0, max_rel_err_mass=0.0, max_rel_err_ratio=0.0)
        for (b, tr, smp, vr, _, _) in r1 + r2:
            par["sequences"] += 1
            par["positions"] += G
            seq_sets_exact = True
            for jj in range(G):
                r = b * G + jj
                near = tr["margin_rho"][jj] < NEAR_TIE
                par["top_rho_near_ties"] += int(near)
                par["exact_path_rows"] += int(g_tr["status"][r] & 256 != 0)
                same = g_tr["count"][r] == tr["count"][jj] and np.array_equal(g_tr["idx"][r], tr["idx"][jj]) and \
                    np.array_equal(g_tr["logit"][r], tr["logit"][jj])
                if same:
                    par["exact_index_sets"] += 1
                    c = int(tr["count"][jj])
                    rel = np.max(np.abs(g_tr["prob"][r, :c] - tr["prob"][jj, :c]) / tr["prob"][jj, :c]) if c else 0.0
                    par["max_rel_err_prob"] = max(par["max_rel_err_prob"], float(rel))
                    if tr["mass"][jj] > 0:
                        par["max_rel_err_mass"] = max(par["max_rel_err_mass"], float(abs(g_tr["mass"][r] - tr["mass"][jj]) / tr["mass"][jj]))
                    par["exact_draft_tokens"] += int(g_tr["token"][r, 0] == smp["token"][jj, 0])
                    if g_tr["token"][r, 0] != smp["token"][jj, 0]:
                        par["unexplained_mismatches"] += 1
                        seq_sets_exact = False
                else:
                    seq_sets_exact = False
                    if near and abs(int(g_tr["count"][r]) - int(tr["count"][jj])) <= 1:
                        par["top_rho_near_tie_mismatches"] += 1
                    else:
                        par["unexplained_mismatches"] += 1
            n = int(vr["accept_len"])
            examined = min(n + 1, G)
            near = bool(np.any(vr["accept_margin"][:examined] < NEAR_TIE))
            par["accept_near_ties"] += int(near)
            par["cdf_edge_near_ties"] += int(vr["cdf_margin"] < 1e-9)
            if not seq_sets_exact:
                continue                       # the GPU verified other sets or tokens than the oracle: nothing to compare
            if g_vf["accept_len"][b] == n:
                par["exact_accept_len"] += 1
                if np.array_equal(g_vf["tokens"][b], vr["tokens"]):
                    par["exact_tokens"] += 1
                else:
                    par["unexplained_mismatches"] += 1
                ok = vr["ratio"][:examined] > 0
                if ok.any():
                    rel = np.max(np.abs(g_vf["ratio"][b, :examined][ok] - vr["ratio"][:examined][ok]) / vr["ratio"][:examined][ok])
                    par["max_rel_err_ratio"] = max(par["max_rel_err_ratio"], float(rel))
            elif near and vr["accept_margin"][min(int(g_vf["accept_len"][b]), n)] < NEAR_TIE:
                par["accept_near_tie_mismatches"] += 1
            else:
                par["unexplained_mismatches"] += 1
        par["max_rel_err_prob"] = float(f"{par['max_rel_err_prob']:.3g}")
        par["max_rel_err_mass"] = float(f"{par['max_rel_err_mass']:.3g}")
        par["max_rel_err_ratio"] = float(f"{par['max_rel_err_ratio']:.3g}")
        par["note"] = ("GPU outputs of the sequences the oracle was timed on; index sets, draft tokens, accepted lengths and emitted "
                       "tokens compared bit for bit; near-tie classes: |u - min(1, p/q)| < 1e-6, Top-rho boundary within 1e-6 of Z, "
                       "inverse-CDF target within 1e-9 of a bucket edge (counted only: it excuses nothing)")
        return baseline, par


class TreePlan:
    """truncate_sample (k candidates per non-leaf node) -> verify_tree on the token-tree workload.  With
    all_nodes every node of every tree is verified (Algorithm 8's parallel form: one target row per node);
    without, only the nodes on each tree's verified path are (depth + 1 target rows per tree)."""

    def __init__(self, w, n_sets, torch, tslt, W, dev, all_nodes=True):
        self.w, self.torch, self.tslt, self.all_nodes = w, torch, tslt, all_nodes
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
                   "node_token": torch.empty(B, n_nodes, dtype=i32, device=dev) if all_nodes else None,
                   "node_slot": torch.empty(B, n_nodes, dtype=i32, device=dev) if all_nodes else None,
                   "ratio": torch.empty(B, n_nodes - 1, dtype=f32, device=dev),
                   "status": torch.empty(B, dtype=i32, device=dev)}
        op = tslt.OP_VERIFY_TREE if all_nodes else tslt.OP_VERIFY_TREE_PATH
        self.ws = torch.empty(tslt.workspace_bytes(op, B, n_nodes, V, K), dtype=torch.uint8, device=dev)
        if len(set(w.expansion)) != 1:
            raise SystemExit("bench.py: the tree workload needs the same number of candidates at every layer")
        self.candidate_nodes = B * (n_nodes - 1)
        s = 4 if w.dtype == "f32" else 2
        sparse = R * K * 12
        if all_nodes:
            # every candidate node is drawn and verified; every target row is read once (non-leaf rows by the
            # multi-candidate kernel, leaf rows by the sampling sweep), the sparse sets once out and once in
            self.positions = self.candidate_nodes
            ver_bytes = B * n_int * V * s + R * K * 8
            leaf_bytes = B * (n_nodes - n_int) * V * s
            self.ops = [("truncate", "truncate_kernel", self.truncate, R * V * s + sparse),
                        ("verify_tree", "tree_mcveri_kernel", self.verify, ver_bytes + leaf_bytes)]
            self.total_bytes = R * V * s + sparse + ver_bytes + leaf_bytes
            mode = "every node verified (one target row per node; leaves sampled from their target rows)"
        else:
            # the verified path needs at most depth + 1 target rows per tree (uniforms are indexed by node, so the
            # nodes off the path never influence the output); every draft row is needed for its candidates.
            # positions is set after a run to the candidates that were actually tested.
            path_rows = B * (len(w.expansion) + 1)
            self.positions = None
            self.ops = [("truncate", "truncate_kernel", self.truncate, R * V * s + sparse),
                        ("verify_tree", "tree_lazy_walk_kernel", self.verify, path_rows * V * s + path_rows * K * 8)]
            self.total_bytes = R * V * s + sparse + path_rows * V * s + path_rows * K * 8
            mode = "only the verified path is verified and sampled (positions = candidates actually tested)"
        self.describe = (f"{w.name}: B={B} trees, expansion={tuple(w.expansion)} ({n_int} non-leaf of {n_nodes} nodes), V={V} "
                         f"{w.dtype} logits, T={w.T}, top_k={w.top_k}, k_cap={K}, candidates drawn "
                         f"{'without' if w.without_replacement else 'with'} replacement and verified by the matching rule, "
                         f"{mode}; {n_sets} rotating input sets; truncate_sample+verify_tree per step")

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
                              all_nodes=self.all_nodes, out=self.vt, workspace=self.ws, without_replacement=w.without_replacement)

    def tested_candidates(self):
        """Candidates whose acceptance test was evaluated in the last run (their ratio is not NaN)."""
        return int((~self.torch.isnan(self.vt["ratio"])).sum().item())

    def cpu_baseline_and_parity(self, budget_s=20.0):
        """The oracle on whole trees of input set 0 (every node evaluated), one thread and then all cores, as many
        trees as fit the time budget (at least one each); the GPU's outputs for those trees compared with it."""
        from oracle import tslt_oracle as O
        import numpy as np
        w, torch = self.w, self.torch
        c = self.sets[0]
        n_int, n_nodes, kmax, K = self.n_int, self.n_nodes, self.kmax, w.k_cap
        for (_, _, fn, _) in self.ops:
            fn(c)
        torch.cuda.synchronize()

        def one(b):
            t0 = time.perf_counter()
            draft = c["draft"][b].float().cpu().numpy()
            target = c["target"][b].float().cpu().numpy()
            t1 = time.perf_counter()
            tr = O.truncate(draft, w.T, w.top_k, w.top_p, K)
            smp = O.sample(tr["idx"], tr["logit"], tr["count"], c["u_sample"][b].cpu().numpy(), w.without_replacement)
            t2 = time.perf_counter()
            vr = O.verify_tree_seq(target, w.T, w.expansion, tr["idx"], tr["logit"], tr["count"],
                                   smp["token"].reshape(n_int * kmax).astype(np.int32), c["u_accept"][b].cpu().numpy(),
                                   c["u_resample"][b].cpu().numpy(), w.without_replacement)
            return b, tr, smp, vr, t2 - t1, time.perf_counter() - t2, t1 - t0

        host_cores = os.cpu_count() or 1
        threads = max(1, min(16, host_cores))
        r1, dt1 = timed_pool(one, range(w.B), 1, 0.4 * budget_s)
        r2, dt2 = timed_pool(one, range(len(r1), w.B), threads, 0.6 * budget_s) if len(r1) < w.B else ([], 0.0)

        def leg(res, dt, n_threads):
            if not res:
                return None
            pos = len(res) * (n_nodes - 1)
            t_tr, t_vf, t_copy = sum(r[4] for r in res), sum(r[5] for r in res), sum(r[6] for r in res)
            busy = t_tr + t_vf + t_copy
            dt_eff = dt * (t_tr + t_vf) / busy            # the copies of the rows to the host are not the oracle's work
            return {"value": round(pos / dt_eff, 2), "unit": "draft positions/s", "threads": n_threads, "trees": len(res),
                    "seconds": round(dt_eff, 2),
                    "truncate_sample_value": round(pos / (dt_eff * t_tr / (t_tr + t_vf)), 2),
                    "verify_value": round(pos / (dt_eff * t_vf / (t_tr + t_vf)), 2)}
        single, allc = leg(r1, dt1, 1), leg(r2, dt2, threads)
        best = allc if allc and allc["value"] > single["value"] else single
        baseline = {"value": best["value"], "unit": "draft positions/s", "cores": best["threads"], "kind": "oracle",
                    "host_cores": host_cores, "single_thread": single, "all_cores": allc,
                    "sample": f"whole trees ({n_nodes - 1} candidate nodes each, every node evaluated) of input set 0 of the same "
                              f"workload, truncate+sample+verify_tree, NumPy {np.__version__} fp64: trees 0..{len(r1) - 1} on one "
                              f"thread, then trees {len(r1)}..{len(r1) + len(r2) - 1} split over {threads} threads"}

        g_tr = {k: v.view(w.B, n_int, -1).cpu().numpy() if v.dim() > 1 else v.view(w.B, n_int).cpu().numpy() for k, v in self.tr.items()}
        g_vt = {k: v.cpu().numpy() for k, v in self.vt.items() if v is not None}
        lay = O.tree_layout(w.expansion)
        par = dict(trees=0, positions=0, exact_index_sets=0, exact_candidates=0, exact_sequences=0, exact_node_outputs=0,
                   nodes_compared=0, mc_amp_near_ties=0, mc_amp_near_tie_mismatches=0, accept_near_ties=0, top_rho_near_ties=0,
                   exact_path_rows=0, unexplained_mismatches=0, amp_max=1.0)
        for (b, tr, smp, vr, _, _, _) in r1 + r2:
            par["trees"] += 1
            par["positions"] += n_nodes - 1
            sets_same = np.array_equal(g_tr["count"][b], tr["count"]) and np.array_equal(g_tr["idx"][b], tr["idx"]) and \
                np.array_equal(g_tr["logit"][b], tr["logit"])
            par["exact_index_sets"] += int(np.sum((g_tr["count"][b] == tr["count"]) & np.all(g_tr["idx"][b] == tr["idx"], axis=1)))
            par["top_rho_near_ties"] += int(np.sum(tr["margin_rho"] < NEAR_TIE))
            par["exact_path_rows"] += int(np.sum(g_tr["status"][b] & 256 != 0))
            cands_same = np.array_equal(g_tr["token"][b], smp["token"])
            par["exact_candidates"] += int(np.sum(g_tr["token"][b] == smp["token"]))
            amp = np.minimum(vr["amp"], AMP_CAP)
            par["amp_max"] = max(par["amp_max"], float(np.max(vr["amp"])))
            flagged_c = vr["accept_margin"] < NEAR_TIE * amp                     # per candidate
            par["accept_near_ties"] += int(np.sum(vr["accept_margin"] < NEAR_TIE))
            risky = np.zeros(n_nodes, bool)
            for n in range(n_int):
                c0 = O.child_node(lay, w.expansion, n, 0)
                risky[n] = bool(np.any(flagged_c[c0 - 1:c0 - 1 + kmax]))
            par["mc_amp_near_ties"] += int(risky.sum())
            if not (sets_same and cands_same):
                par["unexplained_mismatches"] += int(not sets_same) + int(not cands_same)
                continue
            excused = np.zeros(n_nodes, bool)
            if "node_slot" in g_vt:
                differ = (g_vt["node_slot"][b] != vr["node_slot"]) | (g_vt["node_token"][b] != vr["node_token"])
                excused = differ & risky
                par["mc_amp_near_tie_mismatches"] += int(excused.sum())
                par["unexplained_mismatches"] += int((differ & ~risky).sum())
                par["exact_node_outputs"] += int((~differ).sum())
                par["nodes_compared"] += n_nodes
            same_seq = g_vt["len"][b] == vr["len"] and np.array_equal(g_vt["seq"][b], vr["seq"])
            if same_seq:
                par["exact_sequences"] += 1
            elif not any(risky[n] for n in vr["path"]):
                par["unexplained_mismatches"] += 1
        par["note"] = ("GPU outputs of the trees the oracle was timed on; index sets, candidates, node outputs and verified sequences "
                       "compared bit for bit; a node is in the near-tie class when one of its tests lies within 1e-6 * min(amp, 64) of "
                       "its boundary, amp = prod 1/Z_j over the residual updates before that stage")
        return baseline, par


def stats_sweep(torch, tslt, W, dev):
    """The synthetic analogue of the paper's Top-K-mass figure (Section 5.1) and acceptance-rate figure (Section
    5.2): per K, the share of the draft distribution's mass that the Top-K set keeps (rho of Theorem 1) and the
    acceptance rate under truncation beta_hat_K (Section 3.2), for one candidate, and the total rate theta with 2
    and 4 candidates per position (Section 4.3), averaged over the draft/target row pairs of benchmark
    configurations 2 and 3.  One tslt_truncate with k_cap = 1024, then tslt_truncation_stats over the nested
    prefixes and tslt_multicandidate_stats on the sets cut to K."""
    ks = [1, 3, 10, 32, 100, 320, 1024]
    out = {"metric": "retained Top-K mass, acceptance rate under truncation and multi-candidate rate against K", "K": ks,
           "data": "synthetic", "workloads": {}}
    for name in ("chain_topk", "large_vocab"):
        w = W.scaled(W.WORKLOADS[name], B=16)
        c = W.make_chain(w, 100, dev)
        B, G, V = w.B, w.gamma, w.V
        draft = c["draft"].view(B * G, V)
        target = c["target"][:, :G].reshape(B * G, V)
        tr = tslt.truncate(draft, w.T, 1024, 0.0, 1024)
        st = tslt.truncation_stats(target, w.T, tr["idx"], tr["logit"], tr["count"], ks)
        theta = {}
        for k_cand in (2, 4):
            theta[k_cand] = []
            for K in ks:
                cnt = torch.clamp(tr["count"], max=K)
                mc = tslt.multicandidate_stats(target, w.T, tr["idx"], tr["logit"], cnt, k_cand)
                theta[k_cand].append(round(float(mc["theta"].double().mean()), 4))
        torch.cuda.synchronize()
        rho = (st["keep"].double() * tr["mass"].double()[:, None]).mean(0)
        out["workloads"][name] = {
            "rows": B * G, "V": V, "dtype": w.dtype, "T": w.T,
            "top_k_mass_rho": [round(float(x), 4) for x in rho],
            "acceptance_rate_one_candidate": [round(float(x), 4) for x in st["beta"].double().mean(0)],
            "total_rate_two_candidates": theta[2], "total_rate_four_candidates": theta[4]}
    print(json.dumps(out))


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
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle leg (and with it the parity report)")
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of oracle time (one thread, then all cores)")
    ap.add_argument("--tree-mode", default="all", choices=["all", "path"], help="tree workload: verify every node (Algorithm 8's "
                    "parallel form) or only the nodes on each tree's verified path")
    ap.add_argument("--stats-sweep", action="store_true", help="print retained mass and acceptance rate against K, and the "
                    "multi-candidate rates, on rows of benchmark configurations 2 and 3 (no timing)")
    ap.add_argument("--no-events", action="store_true", help="time the steps without per-kernel events")
    ap.add_argument("--event-every", type=int, default=8, help="the event pair around the dominant kernel is recorded in "
                    "every N-th step of the timed region")
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
    if args.stats_sweep:
        stats_sweep(torch, tslt, W, dev)
        return
    w = W.WORKLOADS[args.workload]
    if args.batch > 0:
        w = W.scaled(w, B=args.batch)
    if args.dtype:
        w = W.scaled(w, dtype=args.dtype)
    if args.shift != 0.0:
        w = W.scaled(w, shift=args.shift)
    is_tree = len(w.expansion) > 0
    n_sets = args.sets if args.sets > 0 else (1 if is_tree else 3)
    plan = TreePlan(w, n_sets, torch, tslt, W, dev, all_nodes=args.tree_mode == "all") if is_tree else \
        ChainPlan(w, n_sets, torch, tslt, W, dev)
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
    # (an event pair costs the stream about 4 us, so it brackets the dominant call of every
    # `--event-every`-th timed step, not of all of them)
    events = None
    every = max(1, args.event_every)
    if not args.no_events:
        events = {i: ev for i, ev in zip(range(0, args.steps, every), new_events((dom, dom + 1), (args.steps + every - 1) // every))}
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)], events.get(i) if events else None)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0

    roofline = None
    if events:
        ts = [ev[dom].elapsed_time(ev[dom + 1]) for ev in events.values()]
        avg_ms = sum(ts) / len(ts)
        _, kname, _, nbytes = ops[dom]
        achieved = nbytes / (avg_ms * 1e-3) / 1e9
        traffic, traffic_note = committed_traffic(w.name, kname)
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "algorithmic_bytes_per_launch": nbytes, "avg_launch_ms": round(avg_ms, 4),
                    "launches_measured": len(ts),
                    "traffic": traffic, "traffic_from_profile": traffic_note}
    if plan.positions is None:
        # tree, path only: the candidates whose acceptance test was evaluated in the last step
        plan.positions = plan.tested_candidates()

    res = {
        "metric": "draft positions truncated+verified/sec at V=128k; achieved HBM GB/s vs peak",
        "value": round(plan.positions * args.steps / dt, 1), "unit": "draft positions/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(dt / args.steps * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # the arithmetic type: fp32 terms in the streaming sums, fp64 for the kept sets and the sampling sweeps
        "dtype": "f32",
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
    if is_tree:
        res["candidate_nodes_drawn_per_step"] = plan.candidate_nodes
        res["positions_verified_per_step"] = plan.positions
    if not args.no_cpu_baseline:
        res["cpu_baseline"], res["parity"] = plan.cpu_baseline_and_parity(args.cpu_budget)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
