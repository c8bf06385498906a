#!/usr/bin/env python3
"""Benchmark of the LC-RWMD hot path on one MI355X.

One step = one call of lcrwmd_rwmd over the whole workload (both directions of the bound: first phase,
second phase, swapped pass, transposed maximum), with E, the database and the queries already resident
in HBM.  Prints ONE JSON line: whole-job throughput in query x database pairs per second, the roofline
figures of the dominant kernel (first-phase MFMA contraction, timed with HIP events on its own stream
inside the library) and the CPU oracle timed on a bounded sample of the same workload.

`value` is always the Medium workload in fp32 with the per-entry form (the paper's two phases).  The same
line carries, under "configs", a short run of every other workload family at full size (long documents in
fp32, one batch of the short-text all-pairs sweep in bf16, large-vocabulary k-NN in bf16 with top-16), each
with its own first-phase roofline, second-phase rates, sampled error against the oracle and oracle timing,
and under "variants" the other arithmetics and forms on Medium.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_F32_MFMA_TFLOPS = 157.3     # MI355X, dense fp32 matrix
PEAK_BF16_MFMA_TFLOPS = 2500.0   # MI355X, dense bf16 matrix
PEAK_HBM_GBS = 8000.0
PEAKS = {"f32": PEAK_F32_MFMA_TFLOPS, "bf16": PEAK_BF16_MFMA_TFLOPS, "bf16x3": PEAK_BF16_MFMA_TFLOPS / 3}
# bf16x3 issues three bf16 MFMAs per algorithmic product: its algorithmic rate is held against a third of the peak


def recorded_traffic(workload, compute):
    """HBM bytes per launch of the dominant kernel as recorded by earlier rocprofv3 --pmc runs of this command
    (profiles/traffic.txt); a counter run cannot be part of a timed run.  None when no run is recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.txt")
    try:
        for line in open(path):
            f = line.split()
            if len(f) == 5 and not line.startswith("#") and f[0] == workload and f[1] == compute:
                return (float(f[3]) + float(f[4])) * 1e9
    except OSError:
        pass
    return None


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def wmd_leg(ctx, binding, synth, prob, E, v, m, n_w, q_w, k_w, with_oracle):
    """Top-k exact WMD with the RWMD cut-off on the first n_w database rows x q_w queries; solver rate; oracle rate."""
    import torch
    sub_db = synth.csr_rows(*prob["db"], np.arange(n_w))
    sub_q = synth.csr_rows(*prob["queries"], np.arange(q_w))
    db, qs = binding.Csr.from_numpy(sub_db, v), binding.Csr.from_numpy(sub_q, v)
    hmax = (int(np.max(np.diff(sub_db[0]))), int(np.max(np.diff(sub_q[0]))))
    saved = ctx.get_options()
    ctx.set_options(**{**saved, "dedup": 1})      # the bounds come from the table form here (same values, a tenth of the time)
    ws = binding.alloc_workspace(ctx.wmd_topk_workspace_bytes(v, m, n_w, db.nnz, q_w, qs.nnz, binding.F32, k_w, *hmax))
    R_idx = torch.empty((q_w, k_w), dtype=torch.int32, device="cuda")
    R_dist = torch.empty((q_w, k_w), dtype=torch.float32, device="cuda")
    ev = torch.zeros(q_w, dtype=torch.int64)
    ctx.wmd_topk(qs, db, E, k_w, R_idx, R_dist, ws, ev)
    torch.cuda.synchronize()
    ctx.profile_begin()
    t = time.perf_counter()
    ctx.wmd_topk(qs, db, E, k_w, R_idx, R_dist, ws, ev)
    torch.cuda.synchronize()
    t = time.perf_counter() - t
    pr = ctx.profile_end()
    ctx.set_options(**saved)
    evaluated = int(ev.sum())
    out = {"workload": f"first {n_w} database rows x first {q_w} queries, k = {k_w}", "rwmd_form": "table", "ms": 1e3 * t,
           "wmd_evaluated": evaluated, "evaluated_fraction": evaluated / (n_w * q_w),
           "abandoned_above_cutoff": int(pr["emd_abandoned"]),
           "solver_ms": pr["emd_ms"], "rwmd_first_phase_ms": pr["phase1_ms"],
           "solver_pairs_per_s": pr["emd_pairs"] / max(pr["emd_ms"], 1e-9) * 1e3,
           "equivalent_exhaustive_pairs_per_s": n_w * q_w / t}
    if with_oracle:
        import oracle
        gi = R_idx[:2, :4].cpu().numpy().astype(np.int64).ravel()
        gj = np.repeat(np.arange(2), 4)
        tc = time.perf_counter()
        ref = oracle.wmd_pairs(prob["E"], sub_db, sub_q, gi, gj)
        tc = time.perf_counter() - tc
        got = R_dist[:2, :4].cpu().numpy().astype(np.float64).ravel()
        out["max_rel_err_vs_oracle_8_pairs"] = float(np.max(np.abs(got - ref) / np.maximum(ref, 1e-6)))
        out["cpu_oracle_pairs_per_s"] = 8 / tc
        out["cpu_oracle"] = "LP solve per pair (fp64, one core), 8 of the returned pairs"
    return out


FORM_NAMES = {0: "none", 1: "per-entry", 2: "table", 3: "per-entry and table"}
T_START = time.perf_counter()


def progress(msg):
    """One line per finished piece of work, on stderr (stdout carries the JSON line only)."""
    print(f"[bench {time.perf_counter() - T_START:6.1f} s] {msg}", file=sys.stderr, flush=True)


class Job:
    """One workload resident on the device, and the ways of running it."""

    def __init__(self, workload, compute, permute_vocab=False, batches=1):
        import torch
        from paper_1711_07227_amd import binding, synth
        self.torch, self.binding, self.synth = torch, binding, synth
        self.cfg = cfg = synth.CONFIGS[workload]
        self.bf16_in = cfg.precision == "bf16"
        self.compute = "bf16" if self.bf16_in else compute
        t = time.perf_counter()
        self.prob = prob = synth.make(cfg, permute_vocab=permute_vocab)
        self.t_gen = time.perf_counter() - t
        progress(f"{workload}: inputs generated")
        self.v, self.m, self.n, self.q = prob["v"], cfg.m, prob["n"], prob["q"]
        self.E = torch.from_numpy(prob["E"]).cuda()
        if self.bf16_in:
            self.E = self.E.to(torch.bfloat16)          # the generator already rounded the values to bf16
        self.db = binding.Csr.from_numpy(prob["db"], self.v)
        self.ctx = binding.Context(0)
        self.emb_dtype = binding.BF16 if self.bf16_in else binding.F32
        self.k = cfg.topk
        if cfg.queries_from_db:
            # all-pairs sweep: step i uses database rows [i*q, (i+1)*q) as the queries
            self.batches = []
            for i in range(max(batches, 1)):
                rows = (np.arange(self.q) + i * self.q) % self.n
                self.batches.append(binding.Csr.from_numpy(synth.csr_rows(*prob["db"], rows), self.v))
            self.qs = self.batches[0]
            prob["queries"] = synth.csr_rows(*prob["db"], (np.arange(self.q) + (len(self.batches) - 1) * self.q) % self.n)
        else:
            self.qs = binding.Csr.from_numpy(prob["queries"], self.v)
            self.batches = None
        self.ws = None
        self.D = self.R_idx = self.R_dist = self.sums = None

    def options(self, compute=None, dedup=0):
        b = self.binding
        c = {"f32": b.F32, "bf16": b.BF16, "bf16x3": b.BF16X3}[compute or self.compute]
        self.ctx.set_options(compute=c, dedup=dedup)
        need = self.ctx.workspace_bytes(self.v, self.m, self.n, self.db.nnz, self.q, self.qs.nnz, self.emb_dtype, max(self.k, 16))
        if self.ws is None or self.ws.numel() < need:
            self.ws = None
            self.ws = b.alloc_workspace(need)

    def outputs(self, reduce):
        torch = self.torch
        if reduce:
            k = self.k or 16
            if self.R_idx is None:
                self.R_idx = torch.empty((self.q, k), dtype=torch.int32, device="cuda")
                self.R_dist = torch.empty((self.q, k), dtype=torch.float32, device="cuda")
                self.sums = torch.empty((self.q,), dtype=torch.float64, device="cuda")
        elif self.D is None:
            self.D = torch.empty((self.n, self.q), dtype=torch.float32, device="cuda")

    def step(self, i, reduce):
        qs = self.batches[i % len(self.batches)] if self.batches else self.qs
        if reduce:
            self.ctx.rwmd_reduce(qs, self.db, self.E, self.R_idx.shape[1], self.R_idx, self.R_dist, self.sums, self.ws)
        else:
            self.ctx.rwmd(qs, self.db, self.E, self.D, self.ws)

    def timed(self, steps, warmup, reduce=False):
        """Wall time of `steps` steps between two device synchronisations, with the library's per-kernel events."""
        torch = self.torch
        self.outputs(reduce)
        for i in range(warmup):
            self.step(i, reduce)
        torch.cuda.synchronize()
        self.ctx.profile_begin()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(warmup + i, reduce)
        torch.cuda.synchronize()
        sec = time.perf_counter() - t0
        prof = self.ctx.profile_end()
        progress(f"{self.cfg.name}: {steps} steps of {'lcrwmd_rwmd_reduce' if reduce else 'lcrwmd_rwmd'} timed, "
                 f"{1e3 * sec / steps:.1f} ms each ({FORM_NAMES[self.ctx.forms_ran()]} form)")
        return sec, prof

    def report(self, steps, sec, prof, compute=None):
        compute = compute or self.compute
        n, q = self.n, self.q
        out = {"ms_per_step": 1e3 * sec / steps, "pairs_per_s": n * q * steps / sec, "steps": steps, "compute": compute,
               "form": FORM_NAMES[self.ctx.forms_ran()]}
        if prof["phase1_launches"]:
            ms = prof["phase1_ms"] / prof["phase1_launches"]
            fl = prof["phase1_flops"] / prof["phase1_launches"]
            tf = fl / (ms * 1e-3) / 1e12
            out["phase1"] = {"bound": "mfma", "kernel": f"phase1_{compute}", "achieved": tf, "peak": PEAKS[compute],
                             "unit": "TFLOP/s", "frac": tf / PEAKS[compute],
                             "launches_per_step": prof["phase1_launches"] / steps, "avg_launch_ms": ms,
                             "flops_per_launch": fl, "share_of_step": prof["phase1_ms"] / (1e3 * sec)}
        if prof["phase2_launches"]:
            gbs = prof["phase2_bytes"] / prof["phase2_ms"] / 1e6
            out["phase2"] = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                             "what": "compulsory bytes (CSR arrays, Z once, output once or twice) / kernel time",
                             "gather_GBps": prof["phase2_gather_bytes"] / prof["phase2_ms"] / 1e6,
                             "launches_per_step": prof["phase2_launches"] / steps,
                             "avg_launch_ms": prof["phase2_ms"] / prof["phase2_launches"],
                             "share_of_step": prof["phase2_ms"] / (1e3 * sec)}
        if prof["table_rev_launches"]:
            # table form: the swapped table pass dominates; algorithmic bytes = one table row (4 bytes x distinct query
            # words) per stored database entry, plus the output read and written once
            gbs = prof["table_rev_bytes"] / prof["table_rev_ms"] / 1e6
            out["table_rev"] = {"bound": "hbm", "kernel": "table_rev", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                "frac": gbs / PEAK_HBM_GBS, "launches_per_step": prof["table_rev_launches"] / steps,
                                "avg_launch_ms": prof["table_rev_ms"] / prof["table_rev_launches"],
                                "bytes_per_launch": prof["table_rev_bytes"] / prof["table_rev_launches"],
                                "share_of_step": prof["table_rev_ms"] / (1e3 * sec),
                                "table_fwd_avg_launch_ms": prof["table_fwd_ms"] / max(prof["table_fwd_launches"], 1),
                                "table_fwd_GBps": prof["table_fwd_bytes"] / max(prof["table_fwd_ms"], 1e-9) / 1e6}
        out["time_split_ms_per_step"] = {
            "phase1_forward": (prof["phase1_ms"] - prof["phase1_swapped_ms"]) / steps,
            "phase1_swapped": prof["phase1_swapped_ms"] / steps, "phase2": prof["phase2_ms"] / steps,
            "table_passes": (prof["table_fwd_ms"] + prof["table_rev_ms"]) / steps,
            "rest": 1e3 * sec / steps - (prof["phase1_ms"] + prof["phase2_ms"] + prof["table_fwd_ms"] + prof["table_rev_ms"]) / steps}
        return out

    def check_and_oracle(self, reduce, cpu_queries, check_pairs=512):
        """Sampled outputs of the last step against the oracle's per-pair brute force; the table oracle timed."""
        import oracle
        torch, prob, n, q = self.torch, self.prob, self.n, self.q
        rng = np.random.default_rng(1)
        if reduce:    # the returned neighbours' distances, recomputed pair by pair
            k = self.R_idx.shape[1]
            pj = rng.integers(0, q, check_pairs // 4)
            pr = rng.integers(0, k, check_pairs // 4)
            pi = self.R_idx[torch.from_numpy(pj).cuda(), torch.from_numpy(pr).cuda()].cpu().numpy().astype(np.int64)
            got = self.R_dist[torch.from_numpy(pj).cuda(), torch.from_numpy(pr).cuda()].cpu().numpy().astype(np.float64)
        else:
            pi, pj = rng.integers(0, n, check_pairs), rng.integers(0, q, check_pairs)
            got = self.D[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()].cpu().numpy().astype(np.float64)
        ref = oracle.rwmd_pairs(prob["E"], prob["db"], prob["queries"], pi, pj)
        err = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-6)))
        qn = max(1, min(cpu_queries, q))
        sub = self.synth.csr_rows(*prob["queries"], np.arange(qn))
        tc = time.perf_counter()
        col = oracle.rwmd_table(prob["E"], prob["db"], sub)
        tc = time.perf_counter() - tc
        cpu = {"value": n * qn / tc, "unit": "pairs/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"per-query table oracle (fp64, gcc -O3 -march=x86-64-v3, OpenMP), all {n} database docs x first {qn} "
                         f"queries, {tc:.1f} s", "cpu": cpu_model()}
        progress(f"{self.cfg.name}: oracle sample done ({tc:.1f} s for {qn} queries)")
        extra = {}
        if reduce and self.sums is not None:
            s = self.sums[:qn].cpu().numpy()
            extra["column_sum_max_rel_err_vs_oracle"] = float(np.max(np.abs(s - col.sum(axis=0)) / col.sum(axis=0)))
        return err, cpu, extra

    def quadratic_leg(self, qn):
        """The quadratic-complexity method (Sec. III / Sec. V) against the linear-complexity one on the first qn queries."""
        torch, b = self.torch, self.binding
        sub = b.Csr.from_numpy(self.synth.csr_rows(*self.prob["queries"], np.arange(qn)), self.v)
        saved = self.ctx.get_options()
        self.ctx.set_options(compute=saved["compute"], dedup=0)
        Dq = torch.empty((self.n, qn), dtype=torch.float32, device="cuda")
        Dl = torch.empty_like(Dq)
        wq = b.alloc_workspace(self.ctx.rwmd_quadratic_workspace_bytes(self.v, self.m, self.n, self.db.nnz, qn, sub.nnz, self.emb_dtype))
        wl = b.alloc_workspace(self.ctx.workspace_bytes(self.v, self.m, self.n, self.db.nnz, qn, sub.nnz, self.emb_dtype))
        times = {}
        for name, dedup, fn in (("linear", 0, lambda: self.ctx.rwmd(sub, self.db, self.E, Dl, wl)),
                                ("quadratic", 0, lambda: self.ctx.rwmd_quadratic(sub, self.db, self.E, Dq, wq)),
                                ("linear_auto", 2, lambda: self.ctx.rwmd(sub, self.db, self.E, Dl, wl))):
            self.ctx.set_options(compute=saved["compute"], dedup=dedup)
            if dedup:
                wl = None
                wl = b.alloc_workspace(self.ctx.workspace_bytes(self.v, self.m, self.n, self.db.nnz, qn, sub.nnz, self.emb_dtype))
            torch.cuda.synchronize()
            self.ctx.profile_begin()
            t = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            times[name] = time.perf_counter() - t
            times[name + "_prof"] = self.ctx.profile_end()
            times[name + "_form"] = FORM_NAMES[self.ctx.forms_ran()]
        self.ctx.set_options(**saved)
        pq = times["quadratic_prof"]
        progress(f"{self.cfg.name}: quadratic method on {qn} queries, {1e3 * times['quadratic']:.0f} ms against "
                 f"{1e3 * times['linear']:.0f} ms")
        return {"queries": qn, "quadratic_ms": 1e3 * times["quadratic"], "linear_complexity_ms": 1e3 * times["linear"],
                "speedup_of_linear_complexity": times["quadratic"] / times["linear"],
                "linear_complexity_library_choice_ms": 1e3 * times["linear_auto"], "library_choice_form": times["linear_auto_form"],
                "speedup_of_library_choice": times["quadratic"] / times["linear_auto"],
                "mean_histogram_size": self.db.nnz / self.n,
                "quadratic_first_phase_TFLOPs": pq["phase1_flops"] / max(pq["phase1_ms"], 1e-9) / 1e9,
                "quadratic_flops": pq["phase1_flops"], "linear_complexity_flops": times["linear_prof"]["phase1_flops"],
                "note": "the quadratic method evaluates C = T1 o T2 twice (once per kind of minimum); both in the per-entry form",
                "max_abs_diff": float((Dq - Dl).abs().max())}

    def workload_string(self):
        c = self.cfg
        return f"{c.name}: v={self.v} m={self.m} n={self.n} q={self.q} h={c.h_lo}-{c.h_hi} zipf={c.zipf_s}"

    def close(self):
        self.ctx.close()
        self.ws = self.D = self.R_idx = self.R_dist = self.sums = self.E = self.db = self.qs = self.batches = None
        self.torch.cuda.empty_cache()


def config_leg(name, steps, warmup, cpu_queries, with_cpu, sweep=False, self_sweep=False):
    """A short run of another workload family at full size: the line's `configs` entry for it."""
    job = Job(name, "f32", batches=steps + warmup)
    try:
        reduce = bool(job.k)                 # k-NN: fused top-k, D never formed
        job.options()
        sec, prof = job.timed(steps, warmup, reduce)
        out = {"workload": job.workload_string(), "data_gen_s": round(job.t_gen, 1),
               "step": "lcrwmd_rwmd_reduce (top-%d + column sums, D never formed)" % job.k if reduce else
                       "lcrwmd_rwmd into the full n x q matrix" + (" (one batch of the sweep)" if job.batches else "")}
        out.update(job.report(steps, sec, prof))
        if with_cpu:
            err, cpu, extra = job.check_and_oracle(reduce, cpu_queries)
            out["max_rel_err_vs_oracle_sampled"] = err
            out["cpu_baseline"] = cpu
            out.update(extra)
        if job.batches:
            # the sweep's own step: the batch reduced on the device (top-16 + column sums), D never formed
            sec_r, prof_r = job.timed(steps, warmup, reduce=True)
            red = job.report(steps, sec_r, prof_r)
            if with_cpu:
                err, _, extra = job.check_and_oracle(True, min(cpu_queries, 4))
                red["max_rel_err_vs_oracle_sampled"] = err
                red.update(extra)
            nbatch = (job.n + job.q - 1) // job.q
            red["all_pairs_sweep_s_extrapolated"] = nbatch * sec_r / steps
            out["reduced_on_device"] = red
            if sweep:
                torch = job.torch
                rows_all = np.arange(job.n)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                total = 0.0
                for b in range(nbatch):
                    rows = rows_all[b * job.q:(b + 1) * job.q]
                    qs = job.binding.Csr.from_numpy(job.synth.csr_rows(*job.prob["db"], rows), job.v)
                    nq = qs.rows
                    job.ctx.rwmd_reduce(qs, job.db, job.E, 16, job.R_idx[:nq], job.R_dist[:nq], job.sums[:nq], job.ws)
                    total += float(job.sums[:nq].sum())          # synchronises: the batch is done
                    if b % 20 == 19:
                        progress(f"all-pairs sweep: {b + 1} of {nbatch} batches")
                torch.cuda.synchronize()
                sw = time.perf_counter() - t0
                out["all_pairs_sweep"] = {"batches": nbatch, "seconds": sw, "pairs_per_s": job.n * job.n / sw,
                                          "sum_of_all_distances": total,
                                          "includes": "host-side slicing and upload of every batch of queries"}
            if self_sweep:
                try:
                    # the same job in one call: lcrwmd_rwmd_self evaluates every pair once (the bound is symmetric) and
                    # keeps every document's list and sum on the device; nothing is sliced or uploaded per batch.  In the
                    # largest batches (a power of two up to 65,536) whose workspace fits the free memory - what the entry point
                    # picks by itself in a workspace of that size; with --sweep also in batches of 4,096.
                    torch = job.torch
                    rp = job.prob["db"][0]
                    job.D = job.ws = None
                    torch.cuda.empty_cache()
                    def self_ws_bytes(qb):
                        starts = np.arange(0, job.n, qb)
                        most = int(np.max(rp[np.minimum(starts + qb, job.n)] - rp[starts]))
                        return job.ctx.workspace_bytes(job.v, job.cfg.m, job.n, job.db.nnz, qb, most, job.emb_dtype, 16)
                    big = 65536
                    while big > job.q and self_ws_bytes(big) > 0.85 * torch.cuda.mem_get_info()[0]:
                        big //= 2
                    R_idx = torch.empty((job.n, 16), dtype=torch.int32, device="cuda")
                    R_dist = torch.empty((job.n, 16), dtype=torch.float32, device="cuda")
                    sums = torch.empty((job.n,), dtype=torch.float64, device="cuda")
                    for qb in ((big, job.q) if sweep and big != job.q else (big,)):
                        ws = job.binding.alloc_workspace(self_ws_bytes(qb))
                        torch.cuda.synchronize()
                        t0 = time.perf_counter()
                        job.ctx.rwmd_self(job.db, job.E, qb, 16, R_idx, R_dist, sums, ws)
                        torch.cuda.synchronize()
                        sw = time.perf_counter() - t0
                        del ws
                        progress(f"all-pairs in one call, batches of {qb}: {sw:.1f} s")
                        selfrec = {"seconds": sw, "pairs_per_s": job.n * job.n / sw, "batch": qb, "k": 16,
                                   "sum_of_all_distances": float(sums.sum()),
                                   "entry_point": "lcrwmd_rwmd_self: every pair evaluated once, lists and sums of all documents on the device"}
                        if with_cpu and qb == big:
                            # sampled documents: their lists against the oracle's full columns
                            import oracle
                            pick = np.array([0, job.q - 1, job.q, job.n // 2, job.n - 1])
                            ref = oracle.rwmd_table(job.prob["E"], job.prob["db"], job.synth.csr_rows(*job.prob["db"], pick))
                            _, rdist = oracle.topk(ref, 16)
                            got = R_dist[torch.from_numpy(pick).cuda()].cpu().numpy()
                            selfrec["max_rel_err_of_5_lists_vs_oracle"] = float(np.max(np.abs(got - rdist) / np.maximum(rdist, 1e-6)))
                            selfrec["sum_max_rel_err_vs_oracle"] = float(np.max(np.abs(sums[torch.from_numpy(pick).cuda()].cpu().numpy()
                                                                                       - ref.sum(axis=0)) / ref.sum(axis=0)))
                        out["all_pairs_in_one_call" if qb == big else "all_pairs_in_one_call_batches_of_%d" % qb] = selfrec
                    del R_idx, R_dist, sums
                except Exception as e:      # this leg's failure must not take the per-batch figures with it
                    out["all_pairs_in_one_call"] = {"failed": f"{type(e).__name__}: {str(e)[:300]}"}
        elif not reduce and job.cfg.h_hi > 200:
            # long documents: the form the library picks by itself
            job.options(dedup=2)
            sec_a, prof_a = job.timed(max(1, steps), 1)
            out["auto_form"] = job.report(max(1, steps), sec_a, prof_a)
            job.options()
            out["quadratic_method"] = job.quadratic_leg(16)
        if "auto_form" not in out:
            # short documents, many queries: what the library picks by itself (the same step, option dedup = 2)
            job.options(dedup=2)
            sec_a, prof_a = job.timed(1, 1, reduce or bool(job.batches))
            rep = job.report(1, sec_a, prof_a)
            out["auto_form"] = {"ms_per_step": rep["ms_per_step"], "form": rep["form"], "steps": 1,
                                "step": "reduced on the device" if (reduce or job.batches) else "full matrix"}
            job.options()
        return out
    finally:
        job.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="medium", choices=["tiny", "medium", "long", "short", "knn"],
                    help="medium is the benchmark's workload; the others are the remaining workload families "
                         "(short: one step = one batch of 4,096 database rows used as queries; knn: fused top-16)")
    ap.add_argument("--compute", default="f32", choices=["f32", "bf16", "bf16x3"],
                    help="arithmetic of the first phase: fp32 MFMA (default), bf16 MFMA on rounded embeddings, or the "
                         "split form bf16x3 (three bf16 products per fp32 product, fp32-grade results)")
    ap.add_argument("--dedup", type=int, default=0, choices=[0, 1, 2],
                    help="0: per-entry form (the paper's two phases; default).  1: table form (one word-pair table per "
                         "range of queries, same result).  2: the library picks")
    ap.add_argument("--reduce", action="store_true", help="time lcrwmd_rwmd_reduce (top-16 + column sums) instead of lcrwmd_rwmd")
    ap.add_argument("--permute-vocab", action="store_true",
                    help="stress variant: renumber the vocabulary at random, so that word id is no longer frequency rank")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only", action="store_true",
                    help="only the timed workload: no variants, no other configurations, no WMD leg (keeps a profile to the timed kernels)")
    ap.add_argument("--sweep", action="store_true",
                    help="workload short: also run the whole all-pairs job, batch by batch through lcrwmd_rwmd_reduce (245 "
                         "calls, over a minute) and in one call of lcrwmd_rwmd_self")
    ap.add_argument("--all-pairs", action="store_true",
                    help="workload short: also run the whole all-pairs job in one call of lcrwmd_rwmd_self (half a minute)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy (outside the timed region): a kernel of known "
                         "traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--mfma-probe", action="store_true",
                    help="instead of a workload: bare MFMA loops (lcrwmd_probe_mfma) in fp32 and bf16, on zero and on random "
                         "operands, from registers and with the A operand from LDS; prints their rates and shader clocks")
    ap.add_argument("--gather-probe", action="store_true",
                    help="instead of a workload: the rate at which wavefronts gather row segments as the second phase does "
                         "(lcrwmd_probe_gather), by number of distinct segments and load width")
    ap.add_argument("--cpu-queries", type=int, default=48, help="queries in the CPU oracle's timed sample")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    torch.cuda.set_device(0)
    with_cpu = not args.no_cpu_baseline
    if args.mfma_probe:
        from paper_1711_07227_amd import binding
        ctx = binding.Context(0)
        rows = []
        for dtype, name, peak in ((binding.BF16, "bf16", PEAK_BF16_MFMA_TFLOPS), (binding.F32, "f32", PEAK_F32_MFMA_TFLOPS)):
            for random_data in (False, True):
                for lds in (False, True):
                    ctx.probe_mfma(dtype, random_data, lds, 0.2)                       # warm-up, also of the clock
                    tf, mhz = ctx.probe_mfma(dtype, random_data, lds, 1.0)
                    rows.append({"mfma": name, "operands": "random" if random_data else "zero",
                                 "a_operand": "LDS, one 16-byte read per two MFMAs" if lds else "registers",
                                 "TFLOPs": tf, "of_peak": tf / peak, "shader_MHz": mhz})
                    progress(f"probe {name} {'random' if random_data else 'zero'} {'lds' if lds else 'reg'}: {tf:.1f} TFLOP/s at {mhz:.0f} MHz")
        print(json.dumps({"mfma_probe": rows, "peaks_TFLOPs": {"bf16": PEAK_BF16_MFMA_TFLOPS, "f32": PEAK_F32_MFMA_TFLOPS}}))
        return
    if args.gather_probe:
        from paper_1711_07227_amd import binding
        ctx = binding.Context(0)
        rows = []
        for segments in (128, 2048, 16384, 262144):
            for width in (4, 2, 1):
                tb = ctx.probe_gather(segments, width)
                rows.append({"segments": segments, "distinct_MiB": segments * 64 * width * 4 / 2 ** 20, "bytes_per_lane": 4 * width,
                             "TBps": tb})
                progress(f"gather probe: {segments} segments, {4 * width} bytes per lane: {tb:.1f} TB/s")
        print(json.dumps({"gather_probe": rows, "what": "wavefronts gather 64 x bytes_per_lane consecutive bytes of pseudo-random "
                          "rows (pitch 16 KiB), eight loads in flight per wavefront, eight workgroups per CU"}))
        return
    main_is_default = args.workload == "medium" and args.compute == "f32" and args.dedup == 0 and not args.reduce

    job = Job(args.workload, args.compute, args.permute_vocab, batches=args.steps + args.warmup)
    reduce = bool(job.k) or args.reduce
    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    job.options(dedup=args.dedup)
    sec, prof = job.timed(args.steps, args.warmup, reduce)
    rep = job.report(args.steps, sec, prof)
    check = cpu = None
    extra = {}
    if with_cpu:
        check, cpu, extra = job.check_and_oracle(reduce, args.cpu_queries)

    table = rep.get("table_rev")
    roof = dict(table if table else rep.get("phase1", {}))
    tkey = job.compute + ("-dedup" if table else "")
    roof["traffic"] = recorded_traffic(args.workload, tkey)
    roof["traffic_source"] = ("recorded, not measured in this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                              "profiles/traffic.txt") if roof["traffic"] else None

    variants = {}
    if main_is_default and not args.only:
        # the other forms and arithmetics on the same job (reported, never `value`)
        vsteps = max(1, min(args.steps, 5))
        D_ref = job.D.clone()
        for vname, vcompute, vdedup in (("table_form", "f32", 1), ("auto_form", "f32", 2), ("bf16x3", "bf16x3", 0),
                                        ("bf16", "bf16", 0)):
            try:
                job.options(compute=vcompute, dedup=vdedup)
                vsec, vprof = job.timed(vsteps, 1)
                r = job.report(vsteps, vsec, vprof, vcompute)
                r["max_abs_diff_vs_default"] = float((job.D - D_ref).abs().max())
                variants[vname] = r
            except (RuntimeError, job.binding.LcrwmdError) as e:
                variants[vname] = {"skipped": str(e)[:200]}
        job.D.copy_(D_ref)
        del D_ref
        job.options()
        try:
            variants["quadratic_method"] = job.quadratic_leg(min(job.q, 200))
        except (RuntimeError, job.binding.LcrwmdError) as e:
            variants["quadratic_method"] = {"skipped": str(e)[:200]}

    # Exact WMD behind the bound (reported, never `value`): the k nearest by WMD with the RWMD cut-off, on the first
    # 20,000 database rows and 64 queries of the same workload.
    wmd = None
    cfg = job.cfg
    # (documents of up to 200 words: a transport problem's cost grows with the cube of its size, and so does the oracle's)
    if (not args.only and not job.k and not cfg.queries_from_db and not job.bf16_in and job.n >= 20000 and job.q >= 64
            and cfg.h_hi <= 200 and args.compute == "f32"):
        try:
            wmd = wmd_leg(job.ctx, job.binding, job.synth, job.prob, job.E, job.v, job.m, 20000, 64, 16, with_cpu)
            progress("exact-WMD leg done")
        except (RuntimeError, job.binding.LcrwmdError) as e:
            wmd = {"skipped": str(e)[:200]}

    out = {
        "metric": "query x database RWMD pairs/s on 1 MI355X (both directions + max)",
        "value": rep["pairs_per_s"],
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": rep["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": job.compute,
        "data": "synthetic",
        "config": {"workload": job.workload_string(),
                   "variant": {"per-entry": "per-entry distances (the paper's two phases)", "table": "table form (word-pair table)"}.get(
                       rep["form"], rep["form"]),
                   "step": "lcrwmd_rwmd_reduce (top-k + column sums, D never formed)" if reduce else "lcrwmd_rwmd into the full n x q matrix",
                   "vocabulary": "renumbered at random" if args.permute_vocab else "word id = frequency rank",
                   "nnz_db": job.db.nnz, "nnz_q": job.qs.nnz, "data_gen_s": round(job.t_gen, 1)},
        "roofline": roof,
        "phase1": rep.get("phase1") if table else None,
        "phase2": rep.get("phase2"),
        "cpu_baseline": cpu,
        "time_split_ms_per_step": rep["time_split_ms_per_step"],
        "max_rel_err_vs_oracle_512_pairs": check,
        "variants": variants or None,
        "wmd_topk": wmd,
        "numpy": np.__version__,
        # the paper's own figures for this path (Sec. VI, read off its Figs. 12 and 13): other hardware, other data,
        # one query at a time - context, not a target, and not what vs_baseline refers to
        "paper_context": {"hardware": "NVIDIA Tesla P100 16 GB, CUDA 8 (paper, Sec. VI)", "workload": "one query against the whole resident set",
                          "set_1_1M_docs_mean_107_words": {"one_gpu_ms": 120, "pairs_per_s": 8.3e6, "sixteen_gpus_ms": 8},
                          "set_2_2.8M_docs_mean_27_words": {"one_gpu_ms": 160, "pairs_per_s": 1.75e7, "sixteen_gpus_ms": 10},
                          "note": "approximate values as the paper states them; its datasets are not public"},
    }
    out.update(extra)
    sweep_cfg = None
    if args.workload == "short" and (args.sweep or args.all_pairs):
        job.close()
        sweep_cfg = config_leg("short", args.steps, args.warmup, min(args.cpu_queries, 8), with_cpu, sweep=args.sweep, self_sweep=True)
        out["all_pairs_sweep"] = sweep_cfg.get("all_pairs_sweep")
        for key in sweep_cfg:
            if key.startswith("all_pairs_in_one_call"):
                out[key] = sweep_cfg[key]
    else:
        job.close()

    if main_is_default and not args.only:
        # the other workload families at full size, a few steps each
        configs = {}
        for name, csteps, cwarm, cq in (("long", 2, 1, 2), ("short", 5, 2, 8), ("knn", 2, 1, 1)):
            t = time.perf_counter()
            try:
                configs[name] = config_leg(name, csteps, cwarm, cq, with_cpu, self_sweep=(name == "short"))
            except Exception as e:      # a leg that fails must not take the line with it
                configs[name] = {"failed": f"{type(e).__name__}: {str(e)[:300]}"}
            configs[name]["leg_wall_s"] = round(time.perf_counter() - t, 1)
        out["configs"] = configs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
