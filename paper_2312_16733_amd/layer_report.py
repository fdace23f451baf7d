"""Per-layer roofline table of a subnet forward (python -m paper_2312_16733_amd.layer_report).

Every launch of the forward is bracketed by HIP events on the launch stream (sna_profile_enable) and
graded against its own bound: with the launch's algorithmic flops F and bytes B (active sizes only),
arithmetic intensity AI = F / B, the bound is min(MFMA peak, AI x HBM peak); a launch with
AI below the ridge (peak flops / peak bandwidth) is HBM-bound and is graded on bytes / time, the
others on flops / time.  Times are medians over the repeats and include the gap between two
dependent launches (the events sit on the stream between kernels), so they are an upper bound of
the kernel's own duration by 1-3 us.
"""
import argparse
import sys

import numpy as np

PEAK_TFLOPS = 2500.0      # bf16 dense MFMA, MI355X
PEAK_GBS = 8000.0         # HBM3E
RIDGE = PEAK_TFLOPS * 1e12 / (PEAK_GBS * 1e9)


def grade(flops, nbytes, us):
    """(bound name, achieved in the bound's unit, fraction of the bound's peak)."""
    t = us * 1e-6
    if nbytes <= 0 or t <= 0:
        return "-", 0.0, 0.0
    ai = flops / nbytes
    if ai >= RIDGE:
        ach = flops / t / 1e12
        return "mfma", ach, ach / PEAK_TFLOPS
    ach = nbytes / t / 1e9
    return "hbm", ach, ach / PEAK_GBS


def parse_line(line):
    parts = line.split(" ", 4)
    us, cls = float(parts[0]), parts[1]
    flops = float(parts[2].split("=")[1])
    nbytes = float(parts[3].split("=")[1])
    what = parts[4].strip() if len(parts) > 4 else ""
    return us, cls, flops, nbytes, what


def measure(net, cfgs_c, route, x, logits, reps):
    """Median time per launch index over `reps` profiled forwards; returns list of (us, cls, flops, bytes, what)."""
    import torch
    for _ in range(3):
        net.forward(cfgs_c, route, x, logits=logits)
    torch.cuda.synchronize()
    runs = []
    net.profile_enable(True)
    try:
        for _ in range(reps):
            net.forward(cfgs_c, route, x, logits=logits)
            torch.cuda.synchronize()
            lines = [l for l in net.profile_read_launches().split("\n") if l]
            net.profile_read()
            runs.append([parse_line(l) for l in lines])
    finally:
        net.profile_enable(False)
    n = len(runs[0])
    assert all(len(r) == n for r in runs)
    out = []
    for i in range(n):
        us = float(np.median([r[i][0] for r in runs]))
        out.append((us,) + runs[0][i][1:])
    return out


def report(rows, title, fh):
    """One line per distinct launch (class + shapes), in order of first appearance, with how often the
    forward issues it and its mean time; totals over all launches below."""
    fh.write(f"## {title}\n")
    fh.write(f"{'n':>3} {'us':>7} {'class':<18} {'GFLOP':>8} {'MB':>8} {'AI':>5} {'bound':<5} {'achieved':>13} {'frac':>6}  launch\n")
    tot_us = tot_f = tot_b = ideal_us = 0.0
    merged, order = {}, []
    for us, cls, flops, nbytes, what in rows:
        what = what.replace("chunked=0 ", "").replace(" parts=1", "")
        key = (cls, flops, nbytes, what)
        if key not in merged:
            merged[key] = []
            order.append(key)
        merged[key].append(us)
        tot_us += us
        tot_f += flops
        tot_b += nbytes
        ideal_us += max(flops / (PEAK_TFLOPS * 1e12), nbytes / (PEAK_GBS * 1e9)) * 1e6
    for key in order:
        cls, flops, nbytes, what = key
        us = float(np.mean(merged[key]))
        bound, ach, frac = grade(flops, nbytes, us)
        unit = "TFLOP/s" if bound == "mfma" else "GB/s"
        ai = flops / nbytes if nbytes else 0.0
        fh.write(f"{len(merged[key]):3d} {us:7.2f} {cls:<18} {flops / 1e9:8.3f} {nbytes / 1e6:8.3f} {ai:5.0f} {bound:<5} {ach:7.1f} {unit:<7} {frac:6.3f}  {what}\n")
    fh.write(f"total: {len(rows)} launches, {tot_us:.1f} us, {tot_f / 1e9:.2f} GFLOP ({tot_f / tot_us / 1e6:.0f} TFLOP/s), "
             f"{tot_b / 1e6:.1f} MB ({tot_b / tot_us / 1e3:.0f} GB/s); sum of per-launch roofline times {ideal_us:.1f} us "
             f"= {ideal_us / tot_us:.3f} of the measured time\n\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--family", default="resnet", choices=["resnet", "mbv3", "transformer"])
    ap.add_argument("--cfgs", default="0,8,15", help="indices into the seeded benchmark cfg list")
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--reps", type=int, default=9)
    ap.add_argument("--out", default="-")
    args = ap.parse_args()

    import torch

    import paper_2312_16733_amd as sna
    import synth
    import os

    dev = torch.device("cuda:0")
    spec = {"resnet": synth.ResNetSpec, "mbv3": synth.MBV3Spec, "transformer": synth.TransformerSpec}[args.family]()
    n_cfgs = 12 if args.family == "transformer" else 16
    B = min(args.batch, 32) if args.family == "transformer" else args.batch
    W = synth.make_weights(spec, 2312)
    S = synth.make_stats(spec, n_cfgs, 2312)
    C = synth.enumerate_cfgs(spec, n_cfgs, 16733)
    net = sna.Supernet(spec, W, S, n_cfgs, B)
    table = os.path.join(os.path.dirname(os.path.abspath(sna.__file__)), "tuned", f"gfx950_{args.family}.txt")
    if os.path.exists(table):
        net.tuning_import(open(table).read())
    fh = sys.stdout if args.out == "-" else open(args.out, "w")
    fh.write(f"# per-launch roofline, {args.family}-shaped SuperNet, batch {B}, bf16, one MI355X\n"
             f"# command: python -m paper_2312_16733_amd.layer_report --family {args.family} --cfgs {args.cfgs} "
             f"--batch {args.batch} --reps {args.reps}\n"
             f"# peaks: {PEAK_TFLOPS:.0f} TFLOP/s bf16 MFMA, {PEAK_GBS:.0f} GB/s HBM, ridge {RIDGE:.0f} flop/B; "
             f"times are event-bracketed medians (launch gap included)\n\n")
    route = np.zeros(B, np.int32)
    logits = torch.empty((B, spec.n_classes), dtype=torch.float32, device=dev)
    for ci in [int(v) for v in args.cfgs.split(",")]:
        c = C[ci]
        x = torch.from_numpy(synth.make_inputs(spec, B, c.in_h, c.in_w, 5)).to(torch.bfloat16).to(dev)
        cc = net.prepare_cfgs([c])
        net.tune(cc, route, x)
        rows = measure(net, cc, route, x, logits, args.reps)
        report(rows, f"cfg {ci}: depth {list(c.depth)}, input {c.in_h}, {synth.subnet_macs(spec, c) / 1e9:.2f} GMAC per request", fh)
    net.close()
    if fh is not sys.stdout:
        fh.close()


if __name__ == "__main__":
    main()
