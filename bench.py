#!/usr/bin/env python3
"""Benchmark of the batched layer-wise strategy search on one MI355X.

A "step" is one complete solve of the workload through the C ABI: R transpose
and input validation, layer-0 init, one fused min-plus/argmin/shift-add launch
per layer, final reduce -- everything Eq. 3 needs for every budget e and every
instance -- with the inputs already resident in HBM and a reused context (no
allocation inside the timed region).

Prints ONE JSON line.  metric = DP cell-updates/s with the nominal count
sum_b L_b * E * S * S'; `value_executed` uses the count the kernels really
perform, sum_b (L_b - 1) * (E + 1) * S * S' (layer 0 has no contraction), and
that count is what the roofline fraction is based on.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# One plain (non-packed, non-FMA) fp32 VALU instruction retires 64 lanes per CU
# per clock: 256 CU x 64 lanes x 2.4 GHz.  The published 157.3 TFLOP/s vector
# figure is this x2 (packed) x2 (FMA counts as two), neither of which an
# add/min mix can use.
PEAK_PLAIN_FP32_TOPS = 256 * 64 * 2.4e9 / 1e12
PEAK_PUBLISHED_FP32_TFLOPS = 157.3
OPS_PER_UPDATE = 2          # one add + one min: the algorithmic minimum


def solve_steps(g, torch, p, d, steps, warmup, flags=0):
    ctx = None
    for _ in range(max(1, warmup)):
        ctx = g.gbmw_dp_solve_batched(p.L, d[0], d[1], d[2], p.S, p.E, flags=flags, ctx=ctx)
    g.gbmw_synchronize(ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        ctx = g.gbmw_dp_solve_batched(p.L, d[0], d[1], d[2], p.S, p.E, flags=flags, ctx=ctx)
    g.gbmw_synchronize(ctx)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return ctx, dt / steps


def to_device(torch, p):
    return (torch.from_numpy(p.c).cuda(), torch.from_numpy(p.M).cuda(), torch.from_numpy(p.R).cuda())


def cpu_baseline(p, budget_s=12.0):
    """The oracle as it stands, all host threads, on as many leading instances
    of the workload as fit in about budget_s seconds."""
    import oracle
    threads = min(oracle.max_threads(), 16)
    done_nominal = 0
    done_exec = 0
    t_used = 0.0
    n = 0
    b = 0
    while t_used < budget_s:                               # instance after instance, round and round
        o, Lb = int(p.offsets[b % p.B]), int(p.L[b % p.B])
        t0 = time.perf_counter()
        oracle.solve(p.c[o:o + Lb], p.M[o:o + Lb], p.R[o:o + Lb], p.E, keep_C=False, keep_A=True,
                     nthreads=threads)
        t_used += time.perf_counter() - t0
        done_nominal += Lb * p.E * p.S * p.S
        done_exec += (Lb - 1) * (p.E + 1) * p.S * p.S
        n += 1
        b += 1
    # the same oracle on one thread, on the first instance only
    o, Lb = 0, int(p.L[0])
    t0 = time.perf_counter()
    oracle.solve(p.c[o:o + Lb], p.M[o:o + Lb], p.R[o:o + Lb], p.E, keep_C=False, keep_A=True, nthreads=1)
    t1 = time.perf_counter() - t0
    return {"value": done_nominal / t_used, "unit": "cell-updates/s", "cores": threads,
            "kind": "oracle", "value_executed": done_exec / t_used,
            "value_1_thread": Lb * p.E * p.S * p.S / t1,
            "sample": f"{n} instance solves ({n / p.B:.1f} passes over the workload's {p.B} instances in order), "
                      f"{t_used:.1f} s of oracle time, OpenMP over budget rows"}


def kernel_roofline(g, torch, p, d, args, flags, step_sec):
    """The dominant kernel (k_minplus: Eq. 3's inner minimum fused with the shift-add), one launch per
    layer: average duration from HIP event pairs around every launch on the solve's stream (one stream),
    and the work the launches really did from the library's path counters (a second, untimed solve
    with GBMW_FLAG_COUNT_WORK: which waves took the run shortcut depends on the inputs alone).

    achieved = executed lane-ops per launch / average launch duration, with 2 lane-ops (one add, one
    min) per candidate update that a lane or a run really computed; covered / executed updates is
    the shortcut's gain and is reported separately.  HBM bytes are modelled from the same counters.
    """
    dense = bool(flags & g.GBMW_FLAG_DENSE_ARITHMETIC)
    keep = flags & (g.GBMW_FLAG_DENSE_ARITHMETIC | g.GBMW_FLAG_LAZY_ARGMIN)
    records = not (flags & g.GBMW_FLAG_LAZY_ARGMIN)
    reps = max(3, min(args.steps, 10))
    tctx = None
    mp_ms = mp_n = tot_ms = 0.0
    for _ in range(reps + 1):
        tctx = g.gbmw_dp_solve_batched(p.L, d[0], d[1], d[2], p.S, p.E, flags=g.GBMW_FLAG_TIME_KERNELS | keep, ctx=tctx)
        a, b, n = g.gbmw_last_solve_ms(tctx)
        if _ == 0:
            continue                                                      # warm-up of this mode
        tot_ms += a; mp_ms += b; mp_n += n
    # the same launch sequence, untimed, on one stream: the step that the per-kernel times add up to
    octx, one_sec = solve_steps(g, torch, p, d, max(3, args.steps // 2), 1, flags=g.GBMW_FLAG_ONE_STREAM | keep)
    g.gbmw_destroy(octx)
    tctx = g.gbmw_dp_solve_batched(p.L, d[0], d[1], d[2], p.S, p.E, flags=g.GBMW_FLAG_COUNT_WORK | keep, ctx=tctx)
    n_launch = int(mp_n / reps)
    work = [g.gbmw_last_solve_work(tctx, i) for i in range(n_launch)]
    g.gbmw_destroy(tctx)
    S = p.S
    tot = [sum(w[k] for w in work) for k in range(4)]
    upd_runs = (tot[0] + tot[1] + tot[2]) * S * S                          # one column's S x S' updates each
    upd_dense = tot[3] * 64 * S                                            # a row: 64 lanes x S' candidates
    upd_exec = upd_runs + upd_dense
    covered = p.executed_updates()
    # HBM bytes by path (the R tile of an instance's layer, S x (S'+2) floats padded to quads, comes from
    # HBM once per XCD, whose L2 then serves the workgroups):
    #   dense row (wave, s): 64 x 4 B of the previous table read (not in the layer-1 launch), 64 x 4 B of
    #     the new table and 64 x 1 B of records written, one summary word
    #     (with the run shortcut also the byte that says the group's records are in A)
    #   run wave: per strategy M and two summary words read (12 B), one summary word and one record byte
    #     for the group written; if it was recognised only from the loaded values it has read its 64 x 4 B
    #     per strategy too
    #   run workgroup (4 waves): 4 x the reads, four summary words and four record bytes per strategy
    rec = 1 if records else 0
    sumw = 0 if dense else 4
    grp = rec if not dense else 0
    read_b = write_b = 0
    RS = (S + 3) // 4 * 4 + 4                                              # a row of the R tile in floats
    for i, w in enumerate(work):
        read_b += int((p.L > i + 1).sum()) * 8 * S * RS * 4                # launch i is layer i + 1 (one stream)
        read_b += w[3] * (256 if i > 0 else 0) + (w[1] + w[2] + 4 * w[0]) * 12 * S + (w[2] * 256 * S if i > 0 else 0)
        write_b += w[3] * (256 + 64 * rec + sumw + grp) + (w[1] + w[2]) * S * (rec + 4) + w[0] * S * (4 * rec + 16)
    avg_launch_s = mp_ms / mp_n * 1e-3 if mp_n else float("nan")
    ach = OPS_PER_UPDATE * upd_exec / n_launch / avg_launch_s / 1e12 if mp_n else 0.0
    hbm_model = (read_b + write_b) / n_launch if n_launch else 0.0
    traffic, traffic_source = None, None
    tname = f"k_minplus_cfg{args.config}_hbm_traffic.txt"
    tpath = os.path.join(ROOT, "profiles", tname)
    if os.path.exists(tpath):
        key = ("hbm_bytes_per_launch_dense:" if dense else "hbm_bytes_per_launch:" if records
               else "hbm_bytes_per_launch_lazy:")
        for line in open(tpath):
            if line.startswith(key):
                traffic = int(line.split(":")[1])
                traffic_source = (f"profiles/{tname}: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of "
                                  f"this benchmark, scaled by a 1 GiB copy (commands in the file); not measured "
                                  f"in this run")
    return {
        "kernel": "k_minplus (fused min-plus + argmin + shift-add), one launch per layer",
        "mode": "dense arithmetic" if dense else "run shortcut (default)",
        "bound": "alu", "achieved": ach, "peak": PEAK_PLAIN_FP32_TOPS, "unit": "TFLOP/s",
        "frac": ach / PEAK_PLAIN_FP32_TOPS,
        "peak_is": "plain (non-packed, non-FMA) fp32 VALU lane-ops: 256 CU x 64 lanes x 2.4 GHz = 39.3 T/s; "
                   "the published 157.3 TFLOP/s is this x2 packed x2 FMA",
        "frac_of_published_fp32_vector_peak": ach / PEAK_PUBLISHED_FP32_TFLOPS,
        "ops_per_update": OPS_PER_UPDATE,
        "valu_instr_floor_per_update": 1.5,
        "frac_of_instr_floor": ach / OPS_PER_UPDATE * 1.5 / PEAK_PLAIN_FP32_TOPS,
        "note": "achieved = 2 lane-ops (add, min) x candidate updates really computed per launch / average "
                "launch duration; a three-input min folds two candidates, so the instruction floor is 1.5 per "
                "update and frac_of_instr_floor is the share of the VALU issue rate that floor would need",
        "executed_updates_per_launch": upd_exec / n_launch if n_launch else 0,
        "covered_updates_per_launch": covered / n_launch if n_launch else 0,
        "shortcut_gain": covered / upd_exec if upd_exec else None,
        "work_per_solve": {"run_workgroups": tot[0], "run_waves_by_summary": tot[1], "run_waves_by_value": tot[2],
                           "dense_rows": tot[3]},
        "hbm": {"modelled_bytes_per_launch": hbm_model, "achieved_GBps": hbm_model / avg_launch_s / 1e9 if mp_n else 0.0,
                "peak": 8000.0, "frac": hbm_model / avg_launch_s / 8e12 if mp_n else 0.0,
                "dense_formulation_bytes_per_launch": (8.0 + rec) * covered / S / n_launch if n_launch else 0.0},
        "traffic": traffic, "traffic_source": traffic_source,
        "avg_launch_ms": avg_launch_s * 1e3, "launches_per_solve": n_launch,
        "sum_kernel_ms_per_solve": mp_ms / reps, "timed_solve_ms": tot_ms / reps,
        "ms_per_step_one_stream": one_sec * 1e3, "ms_per_step": step_sec * 1e3,
        "kernel_share_of_one_stream_step": (mp_ms / reps) / (one_sec * 1e3) if one_sec else None,
    }


def partition_workload(gi):
    """16 (batch size, PP degree) pairs of a 48-layer, 44-strategy model: batch
    sizes scale the activation memory (x0.5, x1, x2, x4), PP degrees 2, 4, 8, 16."""
    models = []
    for q, act in enumerate((0.5, 1.0, 2.0, 4.0)):
        for P in (2, 4, 8, 16):
            models.append(gi.structured_pipeline_model(500 + q, 48, P, 32768, m=8, act_scale=act,
                                                       name=f"bmw48 act x{act} P={P}"))
    return models


def partition_leg(g, gi, cpu: bool, budget_s=10.0):
    """Algorithm 2's partition loop through gbmw_partition_search, host to host
    (model upload, every round's batched solve of the changed stages, trace
    download), with a reused context; the same with every stage re-solved in
    every round; and the oracle on the first pairs."""
    import numpy as np
    models = partition_workload(gi)
    S, E = models[0].S, models[0].E
    a = dict(P=np.array([m.P for m in models], np.int32), Lm=np.array([m.Lm for m in models], np.int32),
             m=np.array([m.m for m in models], np.int32), c=np.concatenate([m.c for m in models]),
             cns=np.concatenate([m.c_ns for m in models]), R=np.concatenate([m.R for m in models]),
             M=np.concatenate([m.M.reshape(m.P * m.Lm, S) for m in models]),
             p0=np.concatenate([m.p0 for m in models]), p_t=np.concatenate([m.p_t for m in models]))
    # the same pairs with synthetic O_b / O_ms tables, for stage searches with Appendix A's check
    split = [gi.with_memory_split(m, 900 + k) for k, m in enumerate(models)]
    a["O_b"] = np.concatenate([m.Ob.reshape(m.P * m.Lm, S) for m in split])
    a["O_ms"] = np.concatenate([m.Oms.reshape(m.P * m.Lm, S) for m in split])
    out = {"workload": "16 pairs: 48 layers, S=44, E=32768, PP 2/4/8/16 x 4 activation scales, max_iter 32"}
    ctx = None
    for name, flags, overall in (("changed_stages", 0, False), ("resolve_all", g.GBMW_FLAG_RESOLVE_ALL, False),
                                 ("changed_stages_lazy_argmin", g.GBMW_FLAG_LAZY_ARGMIN, False),
                                 ("changed_stages_overall_memory", 0, True),
                                 ("changed_stages_overall_memory_lazy_argmin", g.GBMW_FLAG_LAZY_ARGMIN, True)):
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            res, ctx = g.gbmw_partition_search(a["P"], a["Lm"], a["m"], a["c"], a["cns"], a["R"], a["M"], a["p0"],
                                               a["p_t"], S, E, max_iter=32, flags=flags, ctx=ctx,
                                               O_b=a["O_b"] if overall else None,
                                               O_ms=a["O_ms"] if overall else None)
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        out[name] = {"ms": best * 1e3, "device_ms": res["device_ms"], "rounds": res["rounds"],
                     "stage_solves": res["stage_solves"], "cell_updates": int(res["cell_updates"]),
                     "cell_updates_per_s": res["cell_updates"] / best,
                     "searched_partitions": int(res["n_iter"].sum())}
    g.gbmw_destroy(ctx)
    if cpu:
        import oracle.bmw as bmw
        t_used, n, upd = 0.0, 0, 0
        for mod in models:
            t0 = time.perf_counter()
            ref = bmw.partition_search(mod.as_dict(), mod.p0, mod.E, mod.m, p_t=mod.p_t, max_iter=32)
            t_used += time.perf_counter() - t0
            n += 1
            upd += (len(ref["trace"]) + 1) * (mod.Lm - mod.P) * (E + 1) * S * S
            if t_used > budget_s:
                break
        out["cpu_oracle"] = {"ms_per_pair": t_used / n * 1e3, "pairs": n, "cores": 1,
                             "cell_updates_per_s": upd / t_used,
                             "note": "plain Python over the C oracle, every stage solved in every round"}
    return out


def whole_search_leg(g, gi):
    """The whole search the paper times in its search-time figure (Fig. 5a: 8 GPUs, the
    checkpointing strategy set, 16 GB budget, depth 24..96): batch-size sweep x PP degrees x
    partition loop x stages, here from layer shapes through the library's entry points
    (strategy enumeration, cost model, Algorithm 2), host to host.  Context beside the
    paper's seconds, on different hardware and with this build's own cost model."""
    from paper_2307_02031_amd.plan_example import plan
    hw = gi.default_hardware(unit_mb=1.0)                 # the budget axis in MB: 16 GB = 16384 units
    batches = [8.0, 16.0, 24.0, 32.0, 40.0, 48.0, 56.0, 64.0]
    paper_s = {24: 280.59, 48: 537.91, 72: 825.86, 96: 1104.92}
    out = {"setup": "BERT-Huge layer repeated L times, 8 devices, E = 16384 units of 1 MB, 8 batch sizes "
                    "x PP 1/2/4/8, 8 micro-batches, max_iter 32",
           "stage_searches": "Appendix A, Algorithm 3 (overall-memory check) with the cost model's O_b and O_ms",
           "paper_fig5a_16G_seconds": paper_s, "ours": {}}
    for L in (24, 48, 72, 96):
        layers = gi.table1_layers("BERT-Huge-32", layers=L)
        plan(g, gi, layers, 8, 16384, hw, batches[:2], 8)                 # warm-up: allocations
        t0 = time.perf_counter()
        plan(g, gi, layers, 8, 16384, hw, batches, 8, overall=False)
        dt_fwd = time.perf_counter() - t0
        t0 = time.perf_counter()
        best, _, st = plan(g, gi, layers, 8, 16384, hw, batches, 8)
        dt = time.perf_counter() - t0
        out["ours"][L] = {"seconds": dt, "seconds_without_overall_memory_check": dt_fwd, "device_ms": st["device_ms"], "partitions_searched": st["partitions"],
                          "stage_solves": st["stage_solves"], "cell_updates": st["cell_updates"],
                          "pairs": st["pairs"], "rounds": st["rounds"],
                          "best": None if best is None else {"batch": best["B"], "P": best["P"],
                                                             "partition": best["part"], "tpt": best["tpt"]}}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default: the batched config)")
    ap.add_argument("--streams", type=int, default=0, choices=[0, 1],
                    help="1: keep every launch on one stream (GBMW_FLAG_ONE_STREAM), as the "
                         "per-kernel roofline leg always does; 0: library default")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="instead of the benchmark, run a plain 1 GiB device-to-device copy five times "
                         "(a kernel of known traffic against which HBM byte counters are scaled)")
    ap.add_argument("--dense-arithmetic", action="store_true",
                    help="GBMW_FLAG_DENSE_ARITHMETIC for every solve: no shortcut for waves whose budgets "
                         "share one input column")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true", help="skip the short runs of the other configs")
    ap.add_argument("--no-partition", action="store_true", help="skip the partition-search leg (Algorithm 2)")
    ap.add_argument("--only-partition", action="store_true",
                    help="run the partition-search leg alone and print it (for profiling that leg)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; the search shards by instance with no "
              "communication, but no multi-GPU figure is produced here.", file=sys.stderr)
        sys.exit(2)

    import torch
    import gbmw_inputs as gi
    import paper_2307_02031_amd as g

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)

    if args.copy_calibration:
        n = 1 << 28                                   # 2^28 floats = 1 GiB read + 1 GiB written
        src = torch.ones(n, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": 4 * n,
                          "bytes_written_per_copy": 4 * n, "copies": 5}), flush=True)
        return

    if args.only_partition:
        print(json.dumps({"partition_search": partition_leg(g, gi, cpu=not args.no_cpu_baseline),
                          "whole_search": whole_search_leg(g, gi)}), flush=True)
        return

    p = gi.make_config(args.config)
    d = to_device(torch, p)
    base_flags = g.GBMW_FLAG_ONE_STREAM if args.streams == 1 else 0
    if args.dense_arithmetic:
        base_flags |= g.GBMW_FLAG_DENSE_ARITHMETIC
    ctx, sec = solve_steps(g, torch, p, d, args.steps, args.warmup, flags=base_flags)
    nominal, executed = p.nominal_updates(), p.executed_updates()

    roofline = kernel_roofline(g, torch, p, d, args, base_flags, sec)

    out = {
        "metric": "DP cell-updates/s (B*L*E*S*S')", "value": nominal / sec, "unit": "cell-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": sec * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": p.name, "B": p.B, "S": p.S, "E": p.E, "sum_L": p.sumL,
                   "nominal_updates": nominal, "executed_updates": executed,
                   "streams": "one" if args.streams == 1 else "library default (instance groups)",
                   "library": g.gbmw_version()},
        "value_executed": executed / sec,
        "roofline": roofline,
    }
    # The same solve with every lane computing its own cell (GBMW_FLAG_DENSE_ARITHMETIC): what the
    # arithmetic itself reaches against the ALU roofline, without the shortcut for runs of equal columns.
    if not args.dense_arithmetic:
        dflags = base_flags | g.GBMW_FLAG_DENSE_ARITHMETIC
        dctx, dsec = solve_steps(g, torch, p, d, args.steps, args.warmup, flags=dflags)
        g.gbmw_destroy(dctx)
        dr = kernel_roofline(g, torch, p, d, args, dflags, dsec)
        out["dense_arithmetic"] = dict(dr, ms_per_step=dsec * 1e3, value=nominal / dsec, value_executed=executed / dsec)
        # the VALU fraction of the min-plus kernel when it executes every update of the batched config
        out["roofline"]["frac_with_every_update_executed"] = dr["frac"]
        out["roofline"]["frac_with_every_update_executed_is"] = (
            "roofline.frac of the same solve under GBMW_FLAG_DENSE_ARITHMETIC (object dense_arithmetic): the default "
            "mode's run shortcut executes one update in shortcut_gain, so its launches are short and bound by "
            "neither roofline")
    # The same solve without argmin records (GBMW_FLAG_LAZY_ARGMIN): every layer's fp32 table
    # is kept and the walkers recompute the records they need.  Reported beside the headline,
    # never as it: the headline path materialises every record.
    lflags = base_flags | g.GBMW_FLAG_LAZY_ARGMIN
    lt, lsec = solve_steps(g, torch, p, d, args.steps, args.warmup, flags=lflags)
    # plans through the recomputing walker, same query set as the backtrack leg below
    import numpy as np
    window = min(256, p.E + 1)
    qi = np.repeat(np.arange(p.B, dtype=np.int32), window)
    qe = np.tile(np.arange(p.E - window + 1, p.E + 1, dtype=np.int32), p.B)
    g.gbmw_backtrack(lt, qi, qe)                            # first call: the staging block is allocated
    lbt = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        g.gbmw_backtrack(lt, qi, qe)
        lbt = min(lbt, time.perf_counter() - t0)
    g.gbmw_destroy(lt)
    lr = kernel_roofline(g, torch, p, d, args, lflags, lsec)
    out["lazy_argmin"] = dict(
        lr, ms_per_step=lsec * 1e3, value=nominal / lsec, value_executed=executed / lsec,
        table_bytes_per_cell=4, backtrack_ms=lbt * 1e3, backtrack_queries=int(len(qi)),
        note_lazy="no argmin records written (8 bytes per cell of the dense formulation instead of 9; the "
                  "tables of all layers are kept, 4 B/cell resident instead of 1); a value pass folds two "
                  "candidates per three-input min, so its frac at 2 lane-ops per update can pass 1.0 while "
                  "frac_of_instr_floor cannot")
    # row a4: plans for a window of budgets below E for every instance (the E_fwd window
    # Algorithm 3 inspects), timed end to end through the ABI (upload, walk, download)
    g.gbmw_backtrack(ctx, qi, qe)                           # first call: the staging block is allocated
    bt = float("inf")
    for _ in range(3):
        t0 = time.perf_counter()
        plan, cost, mem = g.gbmw_backtrack(ctx, qi, qe)
        bt = min(bt, time.perf_counter() - t0)
    out["backtrack"] = {"queries": int(len(qi)), "ms": bt * 1e3, "plans_per_s": len(qi) / bt,
                        "note": "host-to-host through gbmw_backtrack, best of 3 after a first call that "
                                "allocates the staging block: query upload, one lane per query walking "
                                "L_b argmin records, plan download"}
    # Algorithm 3's outer loop (overall-memory check over the b_up window, largest valid
    # E_fwd and its plan per instance) on synthetic O_f / O_b / O_ms with O_f + O_ms == M
    Of, Ob, Oms = gi.split_memory(p, 4)
    g.gbmw_select_forward_budget(ctx, Of, Ob, Oms)
    t0 = time.perf_counter()
    e_opt, _, _, _ = g.gbmw_select_forward_budget(ctx, Of, Ob, Oms)
    sb = time.perf_counter() - t0
    out["select_forward_budget"] = {"ms": sb * 1e3, "instances": p.B,
                                    "budgets_checked": int(sum(min(int(Ob[int(o):int(o) + int(n)].max()), p.E + 1)
                                                               for o, n in zip(p.offsets, p.L))),
                                    "note": "host-to-host through the ABI, includes the upload of the three "
                                            "O tables and the host-side O_f + O_ms == M check"}
    g.gbmw_destroy(ctx)
    del d

    if not args.no_others:
        others = {}
        ceiling = PEAK_PLAIN_FP32_TOPS * 1e12 / OPS_PER_UPDATE       # updates/s at 2 plain lane-ops per update
        wide = gi.stack([gi.random_instance(128 + i, 8, 128, 32768, M_rng=(64, 1024), R_rng=(0.0, 5.0))
                         for i in range(16)], "S128")
        wide.name = "S=128 (upper end of the register-blocked range): B=16, L=8, E=32768, c~U[1,10), M~U{64..1024}, R~U[0,5)"
        for k in (1, 2, 3, 5, "S128"):
            if k == args.config:
                continue
            q = wide if k == "S128" else gi.make_config(k)
            name = k if k == "S128" else f"cfg{k}"
            dq = to_device(torch, q)
            n_steps = 5 if k in (5, "S128") else 20
            c2, s2 = solve_steps(g, torch, q, dq, n_steps, 2, flags=base_flags)
            others[name] = {"workload": q.name, "ms_per_step": s2 * 1e3, "value": q.nominal_updates() / s2,
                            "value_executed": q.executed_updates() / s2,
                            "covered_updates_frac_of_alu_ceiling": q.executed_updates() / s2 / ceiling}
            g.gbmw_destroy(c2)
            c3, s3 = solve_steps(g, torch, q, dq, n_steps, 2, flags=base_flags | g.GBMW_FLAG_LAZY_ARGMIN)
            others[name]["lazy_argmin_ms_per_step"] = s3 * 1e3
            others[name]["lazy_argmin_value_executed"] = q.executed_updates() / s3
            g.gbmw_destroy(c3)
            if k in (2, 3, 5, "S128") and not args.dense_arithmetic:
                c4, s4 = solve_steps(g, torch, q, dq, n_steps, 2, flags=base_flags | g.GBMW_FLAG_DENSE_ARITHMETIC)
                others[name]["dense_arithmetic_ms_per_step"] = s4 * 1e3
                others[name]["dense_arithmetic_frac_of_alu_ceiling"] = q.executed_updates() / s4 / ceiling
                g.gbmw_destroy(c4)
            del dq
        others["alu_ceiling_updates_per_s"] = ceiling
        out["other_configs"] = others

    if not args.no_partition:
        out["partition_search"] = partition_leg(g, gi, cpu=not args.no_cpu_baseline)
        out["whole_search"] = whole_search_leg(g, gi)

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(p)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
