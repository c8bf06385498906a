#!/usr/bin/env python3
"""Benchmark of the LC-RWMD hot path on one MI355X.

One step = one call of lcrwmd_rwmd over the whole workload (both directions of the bound: first phase,
second phase, swapped pass, transposed maximum), with E, the database and the queries already resident
in HBM.  Prints ONE JSON line: whole-job throughput in query x database pairs per second, the roofline
figures of the dominant kernel (first-phase fp32 MFMA contraction, timed with HIP events on its own
stream inside the library) and the CPU oracle timed on a bounded sample of the same workload.
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


def recorded_traffic(workload, compute):
    """HBM bytes per launch of the first-phase kernel from the committed rocprofv3 counter runs, or None."""
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
    ctx.set_options(**{**saved, "dedup": 1})      # the bounds come from the de-duplicated form here (same values, a tenth of the time)
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
    out = {"workload": f"first {n_w} database rows x first {q_w} queries, k = {k_w}", "rwmd_form": "dedup", "ms": 1e3 * t,
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
    ap.add_argument("--dedup", action="store_true",
                    help="de-duplicated form: one word-pair table per query batch instead of one distance per stored "
                         "entry (same result); the dominant kernel is then the bandwidth-bound swapped table pass")
    ap.add_argument("--permute-vocab", action="store_true",
                    help="stress variant: renumber the vocabulary at random, so that word id is no longer frequency rank")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-dedup-variant", action="store_true", dest="no_dedup_variant",
                    help="do not time the de-duplicated and split-bf16 forms after the default one (keeps a profile to the timed kernels)")
    ap.add_argument("--no-wmd", action="store_true",
                    help="skip the exact-WMD leg (top-k WMD with the RWMD cut-off on a slice of the same workload)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy (outside the timed region): a kernel of known "
                         "traffic against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--cpu-queries", type=int, default=48, help="queries in the CPU oracle's timed sample")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_1711_07227_amd import binding, synth

    cfg = synth.CONFIGS[args.workload]
    bf16_in = cfg.precision == "bf16"
    if bf16_in:
        args.compute = "bf16"
    t_gen = time.perf_counter()
    prob = synth.make(cfg, permute_vocab=args.permute_vocab)
    t_gen = time.perf_counter() - t_gen
    v, m, n, q = prob["v"], cfg.m, prob["n"], prob["q"]

    torch.cuda.set_device(0)
    E = torch.from_numpy(prob["E"]).cuda()
    if bf16_in:
        E = E.to(torch.bfloat16)          # the generator already rounded the values to bf16
    db = binding.Csr.from_numpy(prob["db"], v)
    ctx = binding.Context(0)
    compute = {"f32": binding.F32, "bf16": binding.BF16, "bf16x3": binding.BF16X3}[args.compute]
    ctx.set_options(compute=compute, dedup=1 if args.dedup else 0)
    emb_dtype = binding.BF16 if bf16_in else binding.F32
    if cfg.queries_from_db:
        # all-pairs sweep: step i uses database rows [i*q, (i+1)*q) as the queries
        nb = max(args.steps + args.warmup, 1)
        batches = []
        for i in range(nb):
            rows = (np.arange(q) + i * q) % n
            batches.append(binding.Csr.from_numpy(synth.csr_rows(*prob["db"], rows), v))
        qs = batches[0]
        prob["queries"] = synth.csr_rows(*prob["db"], (np.arange(q) + (nb - 1) * q) % n)   # the last timed batch
    else:
        qs = binding.Csr.from_numpy(prob["queries"], v)
        batches = None
    k = cfg.topk
    ws = binding.alloc_workspace(ctx.workspace_bytes(v, m, n, db.nnz, q, qs.nnz, emb_dtype, k))
    if k:
        R_idx = torch.empty((q, k), dtype=torch.int32, device="cuda")
        R_dist = torch.empty((q, k), dtype=torch.float32, device="cuda")
        D = None
    else:
        D = torch.empty((n, q), dtype=torch.float32, device="cuda")

    def step(i):
        if k:
            ctx.rwmd_topk(qs, db, E, k, R_idx, R_dist, ws)
        else:
            ctx.rwmd(batches[i] if batches else qs, db, E, D, ws)

    if args.copy_probe:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    ctx.profile_begin()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(args.warmup + i)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    prof = ctx.profile_end()
    sec = t1 - t0
    ms_per_step = 1e3 * sec / args.steps
    pairs_per_s = n * q * args.steps / sec

    p1_ms = prof["phase1_ms"] / max(prof["phase1_launches"], 1)
    p1_flops = prof["phase1_flops"] / max(prof["phase1_launches"], 1)
    achieved_tflops = p1_flops / (p1_ms * 1e-3) / 1e12 if p1_ms > 0 else 0.0
    # bf16x3 issues three bf16 MFMAs per algorithmic product: its algorithmic rate is held against a third of the peak
    peak = {"f32": PEAK_F32_MFMA_TFLOPS, "bf16": PEAK_BF16_MFMA_TFLOPS, "bf16x3": PEAK_BF16_MFMA_TFLOPS / 3}[args.compute]
    p2_ms = prof["phase2_ms"] / max(prof["phase2_launches"], 1)
    p2_gbs = prof["phase2_bytes"] / max(prof["phase2_ms"], 1e-9) / 1e6
    p2_gather_gbs = prof["phase2_gather_bytes"] / max(prof["phase2_ms"], 1e-9) / 1e6

    # The de-duplicated form of the same job, timed next to the default one (reported, never `value`).
    variant = None
    if not args.dedup and not args.no_dedup_variant and not k and not cfg.queries_from_db:
        try:
            ctx.set_options(compute=compute, dedup=1)
            ws2 = binding.alloc_workspace(ctx.workspace_bytes(v, m, n, db.nnz, q, qs.nnz, emb_dtype, 0))
            D2 = torch.empty((n, q), dtype=torch.float32, device="cuda")
            ctx.rwmd(qs, db, E, D2, ws2)
            torch.cuda.synchronize()
            tv = time.perf_counter()
            for _ in range(args.steps):
                ctx.rwmd(qs, db, E, D2, ws2)
            torch.cuda.synchronize()
            tv = (time.perf_counter() - tv) / args.steps
            variant = {"form": "dedup (word-pair table per query batch, same result)", "ms_per_step": 1e3 * tv,
                       "pairs_per_s": n * q / tv, "max_abs_diff_vs_default": float((D2 - D).abs().max())}
            del ws2, D2
        except (RuntimeError, binding.LcrwmdError) as e:      # e.g. not enough device memory for the table
            variant = {"form": "dedup", "skipped": str(e)[:200]}
        finally:
            ctx.set_options(compute=compute, dedup=0)

    # The split-bf16 arithmetic on the same job (fp32-grade results on the bf16 matrix units), timed next to the default.
    x3 = None
    if args.compute == "f32" and not args.dedup and not args.no_dedup_variant and not k and not cfg.queries_from_db and m <= 300:
        ctx.set_options(compute=binding.BF16X3, dedup=0)
        D3 = torch.empty((n, q), dtype=torch.float32, device="cuda")
        ctx.rwmd(qs, db, E, D3, ws)
        torch.cuda.synchronize()
        tv = time.perf_counter()
        for _ in range(args.steps):
            ctx.rwmd(qs, db, E, D3, ws)
        torch.cuda.synchronize()
        tv = (time.perf_counter() - tv) / args.steps
        x3 = {"form": "compute = bf16x3 (hi*hi + hi*lo + lo*hi on the bf16 matrix units, fp32 accumulation)",
              "ms_per_step": 1e3 * tv, "pairs_per_s": n * q / tv, "max_abs_diff_vs_default": float((D3 - D).abs().max())}
        del D3
        ctx.set_options(compute=compute, dedup=0)

    # Exact WMD behind the bound (reported, never `value`): the k nearest by WMD with the RWMD cut-off, on the first
    # 20,000 database rows and 64 queries of the same workload.
    wmd = None
    # (documents of up to 200 words: a transport problem's cost grows with the cube of its size, and so does the oracle's)
    if not args.no_wmd and not k and not cfg.queries_from_db and not bf16_in and n >= 20000 and q >= 64 and cfg.h_hi <= 200:
        wmd = wmd_leg(ctx, binding, synth, prob, E, v, m, 20000, 64, 16, not args.no_cpu_baseline)

    # sampled check of the timed result against the oracle's per-pair brute force
    cpu = None
    check = None
    if not args.no_cpu_baseline:
        import oracle
        rng = np.random.default_rng(1)
        pi = rng.integers(0, n, 512)
        pj = rng.integers(0, q, 512)
        if k:    # the returned neighbours' distances, recomputed pair by pair
            pj = rng.integers(0, q, 128)
            pr = rng.integers(0, k, 128)
            pi = R_idx[torch.from_numpy(pj).cuda(), torch.from_numpy(pr).cuda()].cpu().numpy().astype(np.int64)
            got = R_dist[torch.from_numpy(pj).cuda(), torch.from_numpy(pr).cuda()].cpu().numpy().astype(np.float64)
        else:
            got = D[torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda()].cpu().numpy().astype(np.float64)
        ref = oracle.rwmd_pairs(prob["E"], prob["db"], prob["queries"], pi, pj)
        check = float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), 1e-6)))
        qn = max(1, min(args.cpu_queries, q))
        sub = synth.csr_rows(*prob["queries"], np.arange(qn))
        tc = time.perf_counter()
        oracle.rwmd_table(prob["E"], prob["db"], sub)
        tc = time.perf_counter() - tc
        cpu = {"value": n * qn / tc, "unit": "pairs/s", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"per-query table oracle (fp64), all {n} database docs x first {qn} queries, {tc:.1f} s",
               "cpu": cpu_model()}

    p1_roof = {"bound": "mfma", "kernel": f"phase1_{args.compute}", "achieved": achieved_tflops, "peak": peak,
               "unit": "TFLOP/s", "frac": achieved_tflops / peak,
               "traffic": None if args.dedup else recorded_traffic(args.workload, args.compute),
               "launches_per_step": prof["phase1_launches"] / args.steps, "avg_launch_ms": p1_ms,
               "flops_per_launch": p1_flops,
               "share_of_step": prof["phase1_ms"] / (1e3 * sec)}
    table = None
    if prof["table_rev_launches"] > 0:
        # de-duplicated form: the swapped table pass dominates; algorithmic bytes = one table row (4 bytes x distinct
        # query words) per stored database entry, plus D read and written once
        tr_ms = prof["table_rev_ms"] / prof["table_rev_launches"]
        tr_gbs = prof["table_rev_bytes"] / prof["table_rev_ms"] / 1e6
        tf_ms = prof["table_fwd_ms"] / max(prof["table_fwd_launches"], 1)
        table = {"bound": "hbm", "kernel": "table_rev", "achieved": tr_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                 "frac": tr_gbs / PEAK_HBM_GBS, "traffic": recorded_traffic(args.workload, args.compute + "-dedup"),
                 "launches_per_step": prof["table_rev_launches"] / args.steps, "avg_launch_ms": tr_ms,
                 "bytes_per_launch": prof["table_rev_bytes"] / prof["table_rev_launches"],
                 "share_of_step": prof["table_rev_ms"] / (1e3 * sec),
                 "table_fwd_avg_launch_ms": tf_ms,
                 "table_fwd_GBps": prof["table_fwd_bytes"] / max(prof["table_fwd_ms"], 1e-9) / 1e6}

    out = {
        "metric": "query x database RWMD pairs/s on 1 MI355X (both directions + max)",
        "value": pairs_per_s,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": args.compute,
        "all_pairs_sweep_s": (n / q) * sec / args.steps if cfg.queries_from_db else None,
        "data": "synthetic",
        "config": {"workload": f"{cfg.name}: v={v} m={m} n={n} q={q} h={cfg.h_lo}-{cfg.h_hi} zipf={cfg.zipf_s}",
                   "variant": "dedup (word-pair table)" if table else "per-entry distances (the paper's two phases)",
                   "vocabulary": "renumbered at random" if args.permute_vocab else "word id = frequency rank",
                   "nnz_db": db.nnz, "nnz_q": qs.nnz, "data_gen_s": round(t_gen, 1)},
        "roofline": table if table else p1_roof,
        "phase1": p1_roof if table else None,
        "phase2": {"bound": "hbm", "achieved": p2_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": p2_gbs / PEAK_HBM_GBS,
                   "gather_GBps": p2_gather_gbs, "launches_per_step": prof["phase2_launches"] / args.steps,
                   "avg_launch_ms": p2_ms, "share_of_step": prof["phase2_ms"] / (1e3 * sec)},
        "cpu_baseline": cpu,
        "dedup_variant": variant,
        "bf16x3_variant": x3,
        "wmd_topk": wmd,
        "time_split_ms_per_step": {"phase1": prof["phase1_ms"] / args.steps,
                                   "phase1_forward": (prof["phase1_ms"] - prof["phase1_swapped_ms"]) / args.steps,
                                   "phase1_swapped": prof["phase1_swapped_ms"] / args.steps,
                                   "phase2": prof["phase2_ms"] / args.steps,
                                   "table_passes": (prof["table_fwd_ms"] + prof["table_rev_ms"]) / args.steps,
                                   "rest": ms_per_step - (prof["phase1_ms"] + prof["phase2_ms"] + prof["table_fwd_ms"] +
                                                          prof["table_rev_ms"]) / args.steps},
        "numpy": np.__version__,
        "max_rel_err_vs_oracle_512_pairs": check,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
