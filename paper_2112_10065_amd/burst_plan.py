"""Burst-parallel plan of the VGG-16 chain from a measured time-versus-batch table.

    python bench.py --table table.json                       # dp_profile_layer's comp(i, g): layer time at per-GPU batch B/g
    python -m paper_2112_10065_amd.burst_plan table.json --amp-limit 2

Feeds the table to the library's dp_plan_chain (paper section 4.2, algorithm "Search Linear") together
with the closed-form communication costs of section 4.1 (dp_plan_cost_tables).  The interconnect numbers
cannot be measured on a one-GPU machine; the defaults are the published xGMI figures of an 8-GPU MI355X node
(7 links x 153 GB/s per GPU) and an assumed 10 us propagation delay - pass your own.
Argument marshalling and printing only: the search runs in the library.
"""
import argparse
import json
import math

from . import binding as dp
from . import workloads as W


def chain_inputs(table, global_batch):
    """(layer names, gpu counts, comp[L][G] in seconds, act_bytes[L], param_bytes[L]) for the VGG-16 chain."""
    convs, fcs = W.vgg16_convs(), W.vgg16_linears()
    names = [l.name for l in convs] + [f.name for f in fcs]
    gpus = [g for g in (1, 2, 4, 8, 16, 32, 64) if global_batch % g == 0 and all(str(global_batch // g) in table[n] for n in names)]
    if not gpus or gpus[0] != 1:
        raise SystemExit(f"the table has no row for per-GPU batch {global_batch} (one GPU)")
    comp = [[sum(v for k, v in table[n][str(global_batch // g)].items() if k.endswith("_us")) * 1e-6 for g in gpus] for n in names]
    act = [2.0 * global_batch * l.h * l.w * l.c for l in convs] + [2.0 * global_batch * f.in_f for f in fcs]      # bf16 activations
    par = [4.0 * (l.k * l.r * l.s * l.c + l.k) for l in convs] + [4.0 * (f.in_f * f.out_f + f.out_f) for f in fcs]  # fp32 gradients
    return names, gpus, comp, act, par


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("table", help="JSON written by bench.py --table")
    ap.add_argument("--global-batch", type=int, default=W.GLOBAL_BATCH)
    ap.add_argument("--amp-limit", type=float, default=2.0, help="GPU-sec amplification limit (inf: none)")
    ap.add_argument("--bandwidth", type=float, default=7 * 153e9, help="per-GPU bandwidth, bytes/s")
    ap.add_argument("--delay", type=float, default=10e-6, help="propagation delay, seconds")
    args = ap.parse_args()
    with open(args.table) as f:
        table = json.load(f)
    table = table.get("layers", table)   # bench.py --table: {"source": "dp_profile_layer", "layers": {...}, "kernels": {...}}
    names, gpus, comp, act, par = chain_inputs(table, args.global_batch)
    comm, sync = dp.dp_plan_cost_tables(gpus, act, par, args.bandwidth, args.delay)
    plan = dp.dp_plan_chain(gpus, comp, comm, sync, args.amp_limit)
    one = sum(c[0] for c in comp)
    print(f"global batch {args.global_batch}, GPU counts {gpus}, amplification limit {args.amp_limit}")
    print(f"{'layer':9s} {'gpus':>4s} {'comp us':>9s} {'T us':>9s} {'Amp':>6s}")
    for i, n in enumerate(names):
        a = gpus.index(plan["gpus"][i])
        t = plan["T"][i + 1][a]
        print(f"{n:9s} {plan['gpus'][i]:4d} {comp[i][a] * 1e6:9.1f} {t * 1e6:9.1f} {t * plan['gpus'][i] / comp[i][0]:6.2f}")
    print(f"iteration: {plan['time'] * 1e6:.1f} us planned, {one * 1e6:.1f} us on one GPU "
          f"(speed-up {one / plan['time']:.2f}x on up to {max(plan['gpus'])} GPUs)")
    for a in range(1, len(gpus)):   # plain data parallelism for comparison: every layer on the same g
        dpar = sum(c[a] for c in comp) + sum(s_[a] for s_ in sync)
        print(f"  every layer on {gpus[a]:2d} GPUs: {dpar * 1e6:9.1f} us, amplification {dpar * gpus[a] / one:.2f}")

if __name__ == "__main__":
    main()
