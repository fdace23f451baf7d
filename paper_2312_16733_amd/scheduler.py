"""Host-side control policies on the latency table l_phi(B), an EDF queue, seeded arrival traces and a
discrete-event model of a router with N identical workers.

What the paper defines (section "SlackFit: Online-Scheduling Policy" and the appendix "Policy Design
Space"): the scheduler looks at the remaining slack theta of the most urgent queued query and picks a
control tuple (batch b, subnet s) from the profiled table L(b, s):
  MaxBatch  the largest b with L(b, smallest subnet) < theta, then the largest s with L(b, s) < theta;
  MaxAcc    the largest s with L(1, s) < theta, then the largest b with L(b, s) < theta;
  SlackFit  evenly sized latency buckets over the table; the bucket closest to and not above theta;
            inside it the tuple with the largest batch.
MaxBatch and MaxAcc rely on latency being monotone in b and in s (binary searches), so the table rows
must be a pareto-ordered subnet set (see `profiler.pareto_subset`).

Readings where the paper is silent: the slack test is strict (L < theta) for MaxBatch / MaxAcc as
printed and "bucket upper edge <= theta" for SlackFit; when nothing fits, every policy falls back to
the smallest subnet at the largest profiled batch (the choice that drains the queue fastest); a
batch takes min(b, queued) queries in deadline order and is charged the profiled latency of the
smallest profiled batch that holds them; a query whose deadline has already passed when it reaches
the head of the queue is dropped and counts as a miss.  Subnet index stands in for accuracy (no
trained weights): "accuracy rank" is index / (S - 1).

The policies, traces and event loop are plain host code.  Workers are either modelled by the
measured table or, with `GpuExecutor`, are the library itself: every dispatched batch runs through
the forward entry point and occupies the worker for the time it took.
"""
from __future__ import annotations

import bisect
import heapq
from typing import List, Optional, Sequence, Tuple

import numpy as np

from . import profiler


# ---- policies -----------------------------------------------------------------------------------
def _last_below(values: Sequence[float], theta: float) -> int:
    """Index of the last entry < theta in a non-decreasing sequence, -1 if none (binary search)."""
    return bisect.bisect_left(values, theta) - 1


class Policy:
    name = "policy"

    def __init__(self, table: np.ndarray, batches: Sequence[int]):
        self.table = np.asarray(table, np.float64)
        self.batches = tuple(int(b) for b in batches)
        assert self.table.shape[1] == len(self.batches)

    def fallback(self) -> Tuple[int, int]:
        return len(self.batches) - 1, 0

    def choose(self, theta_ms: float) -> Tuple[int, int]:
        """(batch column, subnet row) for a most urgent query with theta_ms of slack left."""
        raise NotImplementedError


class MaxBatch(Policy):
    name = "MaxBatch"

    def choose(self, theta_ms):
        j = _last_below(self.table[0, :], theta_ms)
        if j < 0:
            return self.fallback()
        i = _last_below(self.table[:, j], theta_ms)
        return j, max(i, 0)


class MaxAcc(Policy):
    name = "MaxAcc"

    def choose(self, theta_ms):
        i = _last_below(self.table[:, 0], theta_ms)
        if i < 0:
            return self.fallback()
        j = _last_below(self.table[i, :], theta_ms)
        return max(j, 0), i


class SlackFit(Policy):
    name = "SlackFit"

    def __init__(self, table, batches, n_buckets: int = 16):
        super().__init__(table, batches)
        self.buckets = profiler.latency_buckets(self.table, self.batches, n_buckets)
        self.edges = [bk.hi for bk in self.buckets]
        # for every bucket the nearest non-empty one at or below it: O(1) at decision time
        self.first_choice: List[Optional[Tuple[int, int]]] = []
        last = None
        for bk in self.buckets:
            if bk.choices:
                b, i, _ = bk.choices[0]
                last = (self.batches.index(b), i)
            self.first_choice.append(last)

    def choose(self, theta_ms):
        k = bisect.bisect_right(self.edges, theta_ms) - 1       # last bucket whose upper edge <= theta
        if k < 0 or self.first_choice[k] is None:
            return self.fallback()
        return self.first_choice[k]


# ---- traces -------------------------------------------------------------------------------------
def gamma_arrivals(rate: float, cv2: float, duration_s: float, rng: np.random.Generator) -> np.ndarray:
    """Arrival times in [0, duration) with gamma inter-arrival times of mean 1 / rate and squared
    coefficient of variation cv2 (cv2 = 0: evenly spaced)."""
    if rate <= 0:
        return np.zeros(0)
    if cv2 == 0:
        return np.arange(0.0, duration_s, 1.0 / rate)
    n = int(rate * duration_s * 1.5) + 64
    t = np.cumsum(rng.gamma(1.0 / cv2, cv2 / rate, size=n))
    while t[-1] < duration_s:
        t = np.concatenate([t, t[-1] + np.cumsum(rng.gamma(1.0 / cv2, cv2 / rate, size=n))])
    return t[t < duration_s]


def bursty_trace(rate_base: float, rate_var: float, cv2: float, duration_s: float, seed: int) -> np.ndarray:
    """The paper's bursty trace: an evenly spaced base stream of rate_base q/s plus a variant stream of
    rate_var q/s with gamma inter-arrivals of squared coefficient of variation cv2."""
    rng = np.random.default_rng(seed)
    return np.sort(np.concatenate([gamma_arrivals(rate_base, 0.0, duration_s, rng),
                                   gamma_arrivals(rate_var, cv2, duration_s, rng)]))


def accelerating_trace(rate1: float, rate2: float, tau: float, cv2: float, duration_s: float, seed: int) -> np.ndarray:
    """The paper's time-varying trace: the mean rate climbs from rate1 to rate2 q/s at tau q/s^2;
    inter-arrival times are gamma with the current mean and a fixed cv2."""
    rng = np.random.default_rng(seed)
    out, t = [], 0.0
    while True:
        rate = min(rate2, rate1 + tau * t)
        t += rng.gamma(1.0 / cv2, cv2 / rate) if cv2 > 0 else 1.0 / rate
        if t >= duration_s:
            break
        out.append(t)
    return np.asarray(out)


# ---- router + workers ---------------------------------------------------------------------------
def simulate(policy: Policy, arrivals_s: np.ndarray, slo_ms: float, n_workers: int = 1, executor=None) -> dict:
    """Discrete-event run: queries arrive at arrivals_s with deadline arrival + slo; whenever a worker
    is free and the EDF queue is not empty the policy picks (b, s) from the head query's slack, the
    batch is dequeued in deadline order and occupies the worker for the profiled latency.  With an
    `executor(subnet row, batch column, queries taken) -> milliseconds` the batch is really run (see
    `GpuExecutor`) and the worker is occupied for the time it took; the policy still decides on the
    profiled table, as the paper's scheduler does.  Returns SLO attainment over all arrivals, the mean
    accuracy rank over served queries and the decision log (time s, slack ms, batch, subnet, queries
    taken)."""
    table, batches = policy.table, policy.batches
    n_sub = table.shape[0]
    slo = slo_ms * 1e-3
    queue: List[Tuple[float, int]] = []                    # (deadline, query id): a heap is an EDF queue
    free_at = [0.0] * n_workers
    heapq.heapify(free_at)
    met = served = dropped = 0
    rank_sum = 0.0
    log = []
    nxt, n = 0, len(arrivals_s)
    now = 0.0
    while nxt < n or queue:
        if not queue:                                       # idle: jump to the next arrival
            now = max(now, float(arrivals_s[nxt]))
        now = max(now, free_at[0])                          # a worker must be free to dispatch
        while nxt < n and arrivals_s[nxt] <= now:
            heapq.heappush(queue, (float(arrivals_s[nxt]) + slo, nxt))
            nxt += 1
        while queue and queue[0][0] <= now:                 # already late at the head: dropped, a miss
            heapq.heappop(queue)
            dropped += 1
        if not queue:
            continue
        theta_ms = (queue[0][0] - now) * 1e3
        j, i = policy.choose(theta_ms)
        take = min(batches[j], len(queue))
        j_eff = bisect.bisect_left(batches, take)           # smallest profiled batch that holds them
        service_ms = table[i, j_eff] if executor is None else executor(i, j_eff, take)
        done = now + service_ms * 1e-3
        for _ in range(take):
            deadline, _qid = heapq.heappop(queue)
            served += 1
            met += done <= deadline
            rank_sum += i / max(n_sub - 1, 1)
        heapq.heapreplace(free_at, done)
        log.append((now, theta_ms, batches[j], i, take))
    return {"queries": n, "served": served, "dropped": dropped, "slo_attainment": met / n if n else 1.0,
            "mean_accuracy_rank": rank_sum / served if served else 0.0, "decisions": log}


class GpuExecutor:
    """Runs the chosen control tuple on the resident SuperNet and returns the time it took (events on
    torch's current stream): the worker of the paper's architecture, driven by `simulate` in virtual
    time.  A batch of `take` queries runs as the first `take` requests of the profiled batch's inputs."""

    def __init__(self, net, spec, cfgs, batches, make_inputs):
        self.net, self.torch, self.batches = net, net.torch, tuple(batches)
        self.cfgs = [net.prepare_cfgs([c]) for c in cfgs]
        self.inputs = [make_inputs(c, self.batches[-1]) for c in cfgs]
        self.logits = self.torch.empty((self.batches[-1], spec.n_classes), dtype=self.torch.float32, device=self.inputs[0].device)
        self.calls = 0
        self.busy_ms = 0.0

    def __call__(self, i: int, j: int, take: int) -> float:
        torch = self.torch
        route = np.zeros(take, np.int32)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        self.net.forward(self.cfgs[i], route, self.inputs[i][:take], logits=self.logits[:take])
        e1.record()
        e1.synchronize()
        ms = float(e0.elapsed_time(e1))
        self.calls += 1
        self.busy_ms += ms
        return ms


def main():
    """Measures the table on this GPU for the pareto subset of the ResNet-shaped cfgs, then runs the three
    policies over bursty and accelerating traces scaled to the measured capacity."""
    import argparse
    import os
    import sys

    here = os.path.dirname(os.path.abspath(__file__))
    sys.path.insert(0, os.path.dirname(here))
    import torch
    import synth
    import paper_2312_16733_amd as sna

    ap = argparse.ArgumentParser(description="SlackFit / MaxBatch / MaxAcc on the measured latency table")
    ap.add_argument("--workers", type=int, default=8)
    ap.add_argument("--duration", type=float, default=2.0, help="seconds of simulated trace")
    ap.add_argument("--live-duration", type=float, default=0.25, help="seconds of trace for the runs that drive the GPU")
    ap.add_argument("--out", default=None)
    args = ap.parse_args()
    spec = synth.ResNetSpec()
    W, S = synth.make_weights(spec, 2312), synth.make_stats(spec, 16, 2312)
    C = synth.enumerate_cfgs(spec, 16, 16733)
    net = sna.Supernet(spec, W, S, 16, 64)
    tp = os.path.join(here, "tuned", "gfx950_resnet.txt")
    if os.path.exists(tp):
        net.tuning_import(open(tp).read())
    dev = torch.device("cuda:0")

    def make_inputs(c, b):
        return torch.from_numpy(synth.make_inputs(spec, b, c.in_h, c.in_w, 5)).to(torch.bfloat16).to(dev)

    batches = profiler.POW2_BATCHES
    full = profiler.profile_latency(net, spec, C, make_inputs, batches)
    # a set ordered in both directions, as the binary searches need: pareto at the largest batch, then
    # rows that break the order at batch 1 are dropped too
    front = profiler.pareto_subset(full)
    front = [front[k] for k in profiler.pareto_subset(full[front], col=0)]
    table = full[front]
    slo_ms = 3.0 * float(table[-1, -1])                   # three times the slowest tuple, as a stand-in for the paper's 36 ms
    cap_small = args.workers * batches[-1] / (table[0, -1] * 1e-3)
    cap_large = args.workers * batches[-1] / (table[-1, -1] * 1e-3)
    lines = ["policies on the measured ResNet-shaped latency table, %d simulated workers, SLO %.2f ms, %.1f s traces"
             % (args.workers, slo_ms, args.duration),
             "command: python -m paper_2312_16733_amd.scheduler --workers %d --duration %g" % (args.workers, args.duration),
             "subnets (pareto-ordered cfg indices): %s" % " ".join(map(str, front)),
             "capacity at batch 64: %.0f q/s with the smallest subnet, %.0f q/s with the largest" % (cap_small, cap_large), "",
             "%-58s %-9s %8s %9s %8s" % ("trace", "policy", "SLO att.", "acc. rank", "dropped")]
    mean_rate = 0.6 * float(np.sqrt(cap_small * cap_large))   # above what the largest subnet sustains, well below the smallest
    traces = [("bursty, mean %.0f q/s, CV2=%g" % (mean_rate, cv2),
               bursty_trace(0.2 * mean_rate, 0.8 * mean_rate, cv2, args.duration, 100 + k))
              for k, cv2 in enumerate((2.0, 4.0, 8.0))]
    traces += [("accelerating %.0f -> %.0f q/s, tau=%.0e q/s2, CV2=8" % (0.3 * cap_large, 0.6 * cap_small, tau),
                accelerating_trace(0.3 * cap_large, 0.6 * cap_small, tau, 8.0, args.duration, 200 + k))
               for k, tau in enumerate((0.25 * cap_small, 5.0 * cap_small))]
    for name, arr in traces:
        for pol in (SlackFit(table, batches), MaxBatch(table, batches), MaxAcc(table, batches)):
            r = simulate(pol, arr, slo_ms, args.workers)
            lines.append("%-58s %-9s %8.4f %9.3f %8d" % (name, pol.name, r["slo_attainment"], r["mean_accuracy_rank"], r["dropped"]))
    # the same policies driving the library on this GPU (one worker): every decision is really run and
    # the worker is busy for the time the forward took, in virtual time
    ex = GpuExecutor(net, spec, [C[k] for k in front], batches, make_inputs)
    for i in range(len(front)):                              # every (cfg, batch) the policies can pick, warmed up
        for j, b in enumerate(batches):
            ex(i, j, b)
    cap1_small = batches[-1] / (table[0, -1] * 1e-3)
    cap1_large = batches[-1] / (table[-1, -1] * 1e-3)
    rate1 = 0.6 * float(np.sqrt(cap1_small * cap1_large))
    lines += ["", "live: one worker = this GPU, every dispatched batch run through sna_subnet_forward and charged the time it took",
              "capacity at batch 64: %.0f q/s with the smallest subnet, %.0f q/s with the largest" % (cap1_small, cap1_large), "",
              "%-58s %-9s %8s %9s %8s %9s" % ("trace", "policy", "SLO att.", "acc. rank", "dropped", "forwards")]
    live = [("bursty, mean %.0f q/s, CV2=%g" % (rate1, cv2), bursty_trace(0.2 * rate1, 0.8 * rate1, cv2, args.live_duration, 300 + k))
            for k, cv2 in enumerate((2.0, 8.0))]
    live += [("accelerating %.0f -> %.0f q/s, tau=%.0e q/s2, CV2=8" % (0.3 * cap1_large, 0.6 * cap1_small, 5.0 * cap1_small),
              accelerating_trace(0.3 * cap1_large, 0.6 * cap1_small, 5.0 * cap1_small, 8.0, args.live_duration, 400))]
    for name, arr in live:
        for pol in (SlackFit(table, batches), MaxBatch(table, batches), MaxAcc(table, batches)):
            ex.calls = 0
            r = simulate(pol, arr, slo_ms, 1, executor=ex)
            lines.append("%-58s %-9s %8.4f %9.3f %8d %9d" % (name, pol.name, r["slo_attainment"], r["mean_accuracy_rank"], r["dropped"], ex.calls))
    net.close()
    report = "\n".join(lines) + "\n"
    print(report)
    if args.out:
        with open(args.out, "w") as fh:
            fh.write(report)


if __name__ == "__main__":
    main()
