"""End-to-end planning example on one MI355X: layer shapes -> candidate strategies
(Section 3.2) -> analytic cost model -> Algorithm 2's partition search for every
PP degree and a range of batch sizes -> the plan with the highest estimated
throughput.

    python -m paper_2307_02031_amd.plan_example --model BERT-Huge-32 --devices 8 --mem-gb 16

Every number comes from the library's kernels; this file only arranges the calls
and prints.  The layer shapes are rows of the paper's model table cut into equal
layers and the hardware figures are round A100-class numbers (gbmw_inputs), so
the output illustrates the planner, it does not predict a real cluster.
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))

KIND = {1: "DP", 2: "SDP", 3: "TP"}


def strategy_name(s) -> str:
    lv = "-".join(f"{KIND[int(k)]}{int(d)}" for k, d in zip(s["kind"][:s["n_levels"]], s["degree"][:s["n_levels"]]))
    return (lv or "single") + ("+CKPT" if s["ckpt"] else "")


def plan(g, gi, layers, devices, E, hw, batches, microbatches, flags=0, max_iter=32, log=None, overall=True):
    """Algorithm 2 over the given batch sizes (in order) and every PP degree 1, 2, 4, ... that
    fits, as ONE call of the partition search: a pair per (batch size, PP degree), grouped by
    batch size, so that the library also runs the outer loops (best degree per batch size,
    stop at the first batch size that fits nowhere, Tpt).  The strategy set depends on the
    group size devices / P; the smaller sets are padded to the largest with forbidden
    strategies (c = +inf), which no plan ever picks.  overall: every stage search checks the
    overall memory of Eq. 2 (Appendix A, Algorithm 3) with the cost model's O_b and O_ms;
    otherwise a stage only has to fit its forward memory.
    Returns (best pair or None, results per (batch, P), stats)."""
    Lm = len(layers)
    degrees = [p for p in (1, 2, 4, 8, 16, 32, 64) if p <= devices and p <= Lm]
    sets = {P: g.gbmw_enumerate_strategies(devices // P) for P in degrees}
    S = max(len(v) for v in sets.values())
    Ps, cs, cns, Rs, Ms, Obs, Omss, p0s, pts, bsz, grp, key = [], [], [], [], [], [], [], [], [], [], [], []
    for gi_, B in enumerate(batches):
        for P in degrees:
            n_s = len(sets[P])
            cm = g.gbmw_cost_model(layers, sets[P], hw, B / microbatches, P)
            c = np.full((Lm, S), np.inf, np.float32); c[:, :n_s] = cm["c"]
            cn = np.full((Lm, S), np.inf, np.float32); cn[:, :n_s] = cm["c_nosync"]
            R = np.zeros((Lm, S, S), np.float32); R[:, :n_s, :n_s] = cm["R"]
            M = np.zeros((P, Lm, S), np.int32); M[:, :, :n_s] = cm["M"]
            Ob = np.zeros((P, Lm, S), np.int32); Ob[:, :, :n_s] = cm["O_b"]      # one micro-batch in backward,
            Oms = np.zeros((P, Lm, S), np.int32); Oms[:, :, :n_s] = cm["O_ms"]   # whatever the stage
            Ps.append(P); cs.append(c); cns.append(cn); Rs.append(R); Ms.append(M.reshape(P * Lm, S))
            Obs.append(Ob.reshape(P * Lm, S)); Omss.append(Oms.reshape(P * Lm, S))
            p0s.append(gi.proportional_partition(Lm, 1.0 / np.arange(P, 0, -1)))
            pts.append(gi.proportional_partition(Lm, np.ones(P)))
            bsz.append(B); grp.append(gi_); key.append((B, P))
    n = len(Ps)
    res, ctx = g.gbmw_partition_search(Ps, [Lm] * n, [microbatches] * n, np.concatenate(cs), np.concatenate(cns),
                                       np.concatenate(Rs), np.concatenate(Ms), np.concatenate(p0s),
                                       np.concatenate(pts), S, E, max_iter=max_iter, flags=flags,
                                       batch_size=bsz, batch_group=grp,
                                       O_b=np.concatenate(Obs) if overall else None,
                                       O_ms=np.concatenate(Omss) if overall else None)
    g.gbmw_destroy(ctx)
    stats = dict(device_ms=res["device_ms"], partitions=int(res["n_iter"].sum()), rounds=res["rounds"],
                 cell_updates=int(res["cell_updates"]), stage_solves=int(res["stage_solves"]), pairs=n, S=S)
    found = {}
    for k, (B, P) in enumerate(key):
        j = int(res["n_iter"][k]) - 1
        found[(B, P)] = dict(B=B, P=P, cost=float(res["cost"][k, j]), part=[int(x) for x in res["p"][k, j, :P]],
                             plan=[strategy_name(sets[P][int(s)]) if s != 255 else "-" for s in res["strat"][k, :Lm]],
                             searched=j + 1, alpha_t=float(res["alpha_t"][k, j]),
                             alpha_m=float(res["alpha_m"][k, j]), mem=[int(x) for x in res["O"][k, j, :P]])
    if log:
        for P in degrees:
            log(f"  PP={P:<2d} group of {devices // P:<2d} devices, {len(sets[P]):2d} strategies: " +
                "  ".join(f"B={int(B)}: " + (f"{found[(B, P)]['cost']:.4g}s" if np.isfinite(found[(B, P)]['cost']) else "OOM")
                          for B in batches))
        log(f"  {n} pairs, {stats['partitions']} partitions searched in {stats['rounds']} lockstep rounds, "
            f"{stats['device_ms']:.2f} ms on the GPU")
    if res["tpt_pair"] < 0:
        return None, found, stats
    best = dict(found[key[res["tpt_pair"]]], tpt=float(res["tpt"]))
    return best, found, stats


def main():
    import gbmw_inputs as gi
    import paper_2307_02031_amd as g

    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", default="BERT-Huge-32", choices=sorted(gi.TABLE1))
    ap.add_argument("--devices", type=int, default=8)
    ap.add_argument("--mem-gb", type=float, default=16.0, help="memory budget per device")
    ap.add_argument("--unit-mb", type=float, default=8.0, help="granularity of the budget axis")
    ap.add_argument("--batches", default="8,16,32,64,128", help="global batch sizes to try, in order")
    ap.add_argument("--microbatches", type=int, default=8)
    ap.add_argument("--lazy-argmin", action="store_true", help="GBMW_FLAG_LAZY_ARGMIN for the searches")
    ap.add_argument("--forward-memory-only", action="store_true",
                    help="stages need to fit their forward memory only (no overall-memory check)")
    args = ap.parse_args()

    layers = gi.table1_layers(args.model)
    Lm = len(layers)
    hw = gi.default_hardware(unit_mb=args.unit_mb)
    hw["island"] = min(hw["island"], args.devices)
    E = int(args.mem_gb * 1024 / args.unit_mb)
    batches = [float(b) for b in args.batches.split(",")]
    flags = g.GBMW_FLAG_LAZY_ARGMIN if args.lazy_argmin else 0
    print(f"{args.model}: {Lm} layers on {args.devices} devices, {args.mem_gb:g} GB each "
          f"({E} units of {args.unit_mb:g} MB), micro-batches {args.microbatches}")

    best, _, _ = plan(g, gi, layers, args.devices, E, hw, batches, args.microbatches, flags=flags, log=print,
                      overall=not args.forward_memory_only)
    if best is None:
        print("no feasible plan")
        return
    print(f"best: batch {int(best['B'])}, PP={best['P']}, partition {best['part']}, estimated iteration "
          f"{best['cost']:.4g} s, throughput {best['tpt']:.4g} samples/s")
    print(f"      balance degrees alpha_t={best['alpha_t']:.3f} alpha_m={best['alpha_m']:.3f}, stage memory "
          f"{best['mem']} of {E} units, {best['searched']} partitions searched for this pair")
    a = 0
    for i, cnt in enumerate(best["part"]):
        names = best["plan"][a:a + cnt]
        runs, prev = [], None
        for nm in names:
            if nm == prev:
                runs[-1][1] += 1
            else:
                runs.append([nm, 1]); prev = nm
        print(f"      stage {i}: layers {a}..{a + cnt - 1}: " + ", ".join(f"{c} x {nm}" for nm, c in runs))
        a += cnt


if __name__ == "__main__":
    main()
