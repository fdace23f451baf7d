"""Supernet profiler: the latency table l_phi(B) of a resident SuperNet and the latency buckets
built on it.

The paper's worker is profiled once, before serving, for every pareto subnet and every power-of-two
batch size ("Supernet Profiler" paragraph of the system architecture section); the scheduler then
searches a one-dimensional set of evenly sized latency buckets instead of the two-dimensional
table, and inside the bucket just under the most urgent query's slack takes the control tuple with
the largest batch ("SlackFit: Online-Scheduling Policy", paragraphs on the monotonic properties
P1-P3 and on slack-based decisions).  This module measures the table with the library's own
kernels and builds those buckets; it does not schedule anything.

Measurement goes through `Supernet.forward` (events on torch's current stream); the bucket logic
is plain host code with no GPU dependency.
"""
from __future__ import annotations

import dataclasses
from typing import List, Sequence, Tuple

import numpy as np

POW2_BATCHES = (1, 2, 4, 8, 16, 32, 64)


def profile_latency(net, spec, cfgs, make_inputs, batches: Sequence[int] = POW2_BATCHES, reps: int = 7,
                    warmup: int = 2) -> np.ndarray:
    """Median forward latency in milliseconds, shape [len(cfgs)][len(batches)].

    make_inputs(cfg, batch) returns the device tensor of `batch` requests for cfg.  Every (cfg,
    batch) is passed through `net.tune` first, so the table describes the tuned kernels a server
    would run.
    """
    torch = net.torch
    table = np.zeros((len(cfgs), len(batches)), np.float64)
    for i, c in enumerate(cfgs):
        cfgs_c = net.prepare_cfgs([c])
        for j, b in enumerate(batches):
            x = make_inputs(c, b)
            route = np.zeros(b, np.int32)
            logits = torch.empty((b, spec.n_classes), dtype=torch.float32, device=x.device)
            net.tune(cfgs_c, route, x)
            for _ in range(warmup):
                net.forward(cfgs_c, route, x, logits=logits)
            times = []
            for _ in range(reps):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                net.forward(cfgs_c, route, x, logits=logits)
                e1.record()
                e1.synchronize()
                times.append(e0.elapsed_time(e1))
            table[i, j] = float(np.median(times))
    return table


def check_properties(table: np.ndarray, slack: float = 0.03) -> dict:
    """The three properties the scheduler relies on, counted on a table whose rows are ordered from
    the smallest to the largest subnet (MACs stand in for accuracy: there are no trained weights).
    P1: latency does not fall when the batch grows; P2: latency does not fall when the subnet grows;
    P3: the latency spread between the smallest and largest batch grows with the subnet.  `slack` is
    the relative measurement noise tolerated before a pair counts as a violation."""
    n, m = table.shape
    p1 = sum(1 for i in range(n) for j in range(m - 1) if table[i, j + 1] < table[i, j] * (1 - slack))
    p2 = sum(1 for j in range(m) for i in range(n - 1) if table[i + 1, j] < table[i, j] * (1 - slack))
    spread = table[:, -1] - table[:, 0]
    p3 = sum(1 for i in range(n - 1) if spread[i + 1] < spread[i] * (1 - slack))
    return {"p1_pairs": n * (m - 1), "p1_violations": p1, "p2_pairs": m * (n - 1), "p2_violations": p2,
            "p3_pairs": n - 1, "p3_violations": p3, "spread_ms": spread.tolist()}


def pareto_subset(table: np.ndarray, col: int = -1) -> List[int]:
    """Rows (ordered from the smallest to the largest subnet) that are pareto-optimal for (size,
    latency at batch column `col`): a row is dropped when a larger subnet is at least as fast.  The
    paper's scheduler works on such a set (found there by architecture search against measured
    latency); seeded random cfgs are not one, so P2 is judged on this subset."""
    keep: List[int] = []
    best = np.inf
    for i in range(table.shape[0] - 1, -1, -1):          # from the largest subnet down
        if table[i, col] < best:
            keep.append(i)
            best = table[i, col]
    return keep[::-1]


@dataclasses.dataclass
class Bucket:
    lo: float                                 # latency range [lo, hi) in ms
    hi: float
    choices: List[Tuple[int, int, float]]     # (batch, cfg index, latency ms), largest batch first


def latency_buckets(table: np.ndarray, batches: Sequence[int], n_buckets: int) -> List[Bucket]:
    """Evenly sized latency buckets over [min latency, max latency]; bucket k holds every control
    tuple (B, phi) whose latency falls in its range.  Inside a bucket the choices are ordered by
    batch size, largest first, ties by the larger subnet."""
    lo, hi = float(table.min()), float(table.max())
    width = (hi - lo) / n_buckets if hi > lo else 1.0
    buckets = [Bucket(lo + k * width, lo + (k + 1) * width, []) for k in range(n_buckets)]
    for i in range(table.shape[0]):
        for j, b in enumerate(batches):
            k = min(int((table[i, j] - lo) / width), n_buckets - 1)
            buckets[k].choices.append((int(b), i, float(table[i, j])))
    for bk in buckets:
        bk.choices.sort(key=lambda t: (-t[0], -t[1]))
    return buckets


def pick(buckets: List[Bucket], slack_ms: float):
    """The control tuple for a most-urgent query with `slack_ms` left: from the non-empty bucket
    whose upper edge is closest to and not above the slack (every choice in it meets the deadline),
    the choice with the largest batch.  None when even the fastest bucket would miss."""
    best = None
    for bk in buckets:
        if bk.choices and bk.hi <= slack_ms:
            best = bk
    return best.choices[0] if best else None


def format_table(table: np.ndarray, batches: Sequence[int], labels: Sequence[str]) -> str:
    out = ["%-34s" % "cfg (GMACs/request, resolution)" + "".join("%9s" % ("B=%d" % b) for b in batches)]
    for lab, row in zip(labels, table):
        out.append("%-34s" % lab + "".join("%9.3f" % v for v in row))
    return "\n".join(out)


def main():
    import argparse
    import os
    import sys

    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    import torch
    import synth
    import paper_2312_16733_amd as sna

    ap = argparse.ArgumentParser(description="latency table l_phi(B) of a synthetic SuperNet on this GPU")
    ap.add_argument("--family", default="resnet", choices=["resnet", "mbv3", "transformer"])
    ap.add_argument("--buckets", type=int, default=12)
    ap.add_argument("--out", default=None, help="also write the report to this file")
    args = ap.parse_args()
    spec = {"resnet": synth.ResNetSpec, "mbv3": synth.MBV3Spec, "transformer": synth.TransformerSpec}[args.family]()
    n_cfgs = 12 if args.family == "transformer" else 16
    batches = POW2_BATCHES if args.family != "transformer" else (1, 2, 4, 8, 16, 32)
    W = synth.make_weights(spec, 2312)
    S = synth.make_stats(spec, n_cfgs, 2312)
    C = synth.enumerate_cfgs(spec, n_cfgs, 16733)
    net = sna.Supernet(spec, W, S, n_cfgs, max(batches))
    table_path = os.path.join(here, "tuned", f"gfx950_{args.family}.txt")
    if os.path.exists(table_path):
        net.tuning_import(open(table_path).read())
    dev = torch.device("cuda:0")

    def make_inputs(c, b):
        return torch.from_numpy(synth.make_inputs(spec, b, c.in_h, c.in_w, 5)).to(torch.bfloat16).to(dev)

    table = profile_latency(net, spec, C, make_inputs, batches)
    labels = ["%2d: %6.3f G, %dx%d" % (i, synth.subnet_macs(spec, c) / 1e9, c.in_h, c.in_w) for i, c in enumerate(C)]
    props = check_properties(table)
    front = pareto_subset(table)
    pprops = check_properties(table[front])
    bks = latency_buckets(table, batches, args.buckets)
    lines = [f"latency profile l_phi(B) in ms, {args.family}-shaped synthetic SuperNet, one MI355X, median of 7 forwards",
             "command: python -m paper_2312_16733_amd.profiler --family %s --buckets %d" % (args.family, args.buckets), "",
             format_table(table, batches, labels), "",
             "P1 (latency rises with batch): %d of %d adjacent pairs fall by more than 3 %%" % (props["p1_violations"], props["p1_pairs"]),
             "P2 (latency rises with subnet size): %d of %d adjacent pairs fall by more than 3 %%" % (props["p2_violations"], props["p2_pairs"]),
             "P3 (spread between batch %d and batch 1 rises with subnet size): %d of %d adjacent pairs fall by more than 3 %%"
             % (batches[-1], props["p3_violations"], props["p3_pairs"]),
             "the seeded cfgs are not a pareto set; on the %d cfgs that are pareto-optimal for (size, latency at batch %d) - cfgs %s -"
             % (len(front), batches[-1], " ".join(str(i) for i in front)),
             "  P2: %d of %d, P3: %d of %d" % (pprops["p2_violations"], pprops["p2_pairs"], pprops["p3_violations"], pprops["p3_pairs"]), "",
             "%d evenly sized latency buckets (control tuples per bucket; first choice = largest batch):" % args.buckets]
    for bk in bks:
        first = "B=%d cfg %d (%.3f ms)" % bk.choices[0] if bk.choices else "-"
        lines.append("  [%7.3f, %7.3f) ms: %3d tuples, first choice %s" % (bk.lo, bk.hi, len(bk.choices), first))
    report = "\n".join(lines) + "\n"
    print(report)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(report)
    net.close()


if __name__ == "__main__":
    main()
