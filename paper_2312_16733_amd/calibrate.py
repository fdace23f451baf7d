"""SubnetNorm calibration of every subnet of a resident SuperNet, as an offline step before serving.

The paper keeps separate normalisation statistics per subnet, computed by forward passes ahead of
serving (section "SubNetAct", SubnetNorm paragraph).  `calibrate_all` does that for a list of
control tuples with the library's calibration entry point: one calibration batch per subnet, the
statistics written in place into the resident table.  The command line below runs it on a seeded
synthetic SuperNet and reports the time per subnet and what the calibration kernels reach.
"""
from __future__ import annotations

import numpy as np


def calibrate_all(net, cfgs, make_inputs, batch: int):
    """Calibrates each cfg on make_inputs(cfg, batch) (a device tensor).  Returns the wall time per cfg
    in milliseconds (events on torch's current stream)."""
    torch = net.torch
    times = []
    for c in cfgs:
        x = make_inputs(c, batch)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        net.calibrate(c, x)
        e1.record()
        e1.synchronize()
        times.append(e0.elapsed_time(e1))
    return times


def main():
    import argparse
    import os
    import sys

    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    import torch
    import synth
    import paper_2312_16733_amd as sna

    ap = argparse.ArgumentParser(description="calibrate every seeded subnet of a synthetic SuperNet on this GPU")
    ap.add_argument("--family", default="resnet", choices=["resnet", "mbv3"])
    ap.add_argument("--batch", type=int, default=8)
    ap.add_argument("--passes", type=int, default=3, help="timed passes over all cfgs; the last one is reported")
    ap.add_argument("--out", default=None, help="also write the report to this file")
    args = ap.parse_args()
    spec = {"resnet": synth.ResNetSpec, "mbv3": synth.MBV3Spec}[args.family]()
    n_cfgs = 16
    W = synth.make_weights(spec, 2312)
    S = synth.make_stats(spec, n_cfgs, 2312)
    C = synth.enumerate_cfgs(spec, n_cfgs, 16733)
    net = sna.Supernet(spec, W, S, n_cfgs, args.batch)
    dev = torch.device("cuda:0")
    inputs = {}

    def make_inputs(c, b):
        if c.in_h not in inputs:
            inputs[c.in_h] = torch.from_numpy(synth.make_inputs(spec, b, c.in_h, c.in_w, 5)).to(torch.bfloat16).to(dev)
        return inputs[c.in_h]

    for _ in range(max(args.passes, 1)):
        times = calibrate_all(net, C, make_inputs, args.batch)
    net.profile_enable(True)                       # one more pass with events around every launch
    calibrate_all(net, C, make_inputs, args.batch)
    torch.cuda.synchronize()
    prof = net.profile_read()
    net.profile_enable(False)
    table = net.stats_table()
    finite = all(np.all(np.isfinite(v)) for v in table.values())
    lines = ["SubnetNorm calibration, %s-shaped synthetic SuperNet, one MI355X, %d cfgs, one batch of %d requests per cfg"
             % (args.family, n_cfgs, args.batch),
             "command: python -m paper_2312_16733_amd.calibrate --family %s --batch %d --passes %d"
             % (args.family, args.batch, args.passes), "",
             "cfg  GMACs/request  resolution  calibration pass ms"]
    for i, (c, t) in enumerate(zip(C, times)):
        lines.append("%3d  %13.3f  %10d  %19.3f" % (i, synth.subnet_macs(spec, c) / 1e9, c.in_h, t))
    lines += ["", "all %d cfgs: %.2f ms; statistics table finite: %s" % (n_cfgs, sum(times), finite), "",
              "kernel classes over one further pass (events around every launch; algorithmic bytes / time):"]
    for k, v in prof.items():
        lines.append("  %-18s %8.3f ms %5d launches %8.1f GB/s" % (k, v["ms"], v["launches"],
                                                                  v["bytes"] / v["ms"] / 1e6 if v["ms"] else 0.0))
    report = "\n".join(lines) + "\n"
    print(report)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(report)
    net.close()


if __name__ == "__main__":
    main()
