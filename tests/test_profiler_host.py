"""Host logic of the supernet profiler (no GPU): latency buckets and the slack rule against their
definitions written out by brute force, and the property counters on hand-made tables."""
import numpy as np

from paper_2312_16733_amd import profiler


def synthetic_table(n=6, batches=profiler.POW2_BATCHES):
    # latency = fixed cost + per-request cost growing with the subnet: P1-P3 hold by construction
    b = np.asarray(batches, np.float64)
    return np.stack([0.3 + 0.05 * i + (0.02 + 0.015 * i) * b for i in range(n)])


def test_properties_hold_on_a_monotone_table_and_violations_are_counted():
    t = synthetic_table()
    p = profiler.check_properties(t)
    assert p["p1_violations"] == p["p2_violations"] == p["p3_violations"] == 0
    assert p["p1_pairs"] == 6 * 6 and p["p2_pairs"] == 7 * 5 and p["p3_pairs"] == 5
    t2 = t.copy()
    t2[2, 3] = t2[2, 2] * 0.5                      # one entry falls with the batch ...
    p = profiler.check_properties(t2)
    assert p["p1_violations"] == 1                  # ... and below its smaller-subnet neighbour
    assert p["p2_violations"] == 1
    t3 = t.copy()
    t3[4, -1] = t3[4, 0] + 0.01                     # spread of subnet 4 collapses
    assert profiler.check_properties(t3)["p3_violations"] == 1
    noisy = t * (1 + 0.01 * np.sin(np.arange(t.size)).reshape(t.shape))
    assert profiler.check_properties(noisy)["p1_violations"] == 0      # 1 % noise is inside the slack


def test_buckets_partition_the_control_space():
    t = synthetic_table()
    batches = profiler.POW2_BATCHES
    for nb in (1, 4, 9):
        bks = profiler.latency_buckets(t, batches, nb)
        assert len(bks) == nb
        assert abs(bks[0].lo - t.min()) < 1e-12 and abs(bks[-1].hi - t.max()) < 1e-9
        seen = set()
        for k, bk in enumerate(bks):
            assert abs((bk.hi - bk.lo) - (t.max() - t.min()) / nb) < 1e-9
            for b, i, lat in bk.choices:
                assert lat == t[i, batches.index(b)]
                assert bk.lo - 1e-12 <= lat and (lat < bk.hi + 1e-12)
                if k < nb - 1:
                    assert lat < bk.hi
                seen.add((b, i))
            assert [c[0] for c in bk.choices] == sorted((c[0] for c in bk.choices), reverse=True)
        assert len(seen) == t.size


def test_pick_is_the_largest_batch_of_the_last_bucket_that_fits():
    t = synthetic_table()
    batches = profiler.POW2_BATCHES
    bks = profiler.latency_buckets(t, batches, 8)
    assert profiler.pick(bks, t.min() * 0.5) is None
    assert profiler.pick(bks, bks[0].hi - 1e-9) is None          # the fastest bucket's edge is above the slack
    for slack in np.linspace(bks[0].hi, t.max() * 1.2, 40):
        got = profiler.pick(bks, slack)
        # brute force: among non-empty buckets whose upper edge fits, the last; its largest batch, then largest subnet
        fitting = [bk for bk in bks if bk.choices and bk.hi <= slack]
        want = max(fitting[-1].choices, key=lambda c: (c[0], c[1]))
        assert got == want
        assert got[2] <= slack


def test_report_table_lists_every_cfg():
    t = synthetic_table(3, (1, 2))
    txt = profiler.format_table(t, (1, 2), ["a", "b", "c"])
    assert txt.count("\n") == 3 and "B=2" in txt


def test_pareto_subset_against_the_definition():
    rng = np.random.default_rng(7)
    for _ in range(20):
        t = rng.uniform(0.2, 3.0, size=(9, 4))
        keep = profiler.pareto_subset(t)
        # definition: row i stays iff no larger subnet (higher index) is at least as fast at the last batch
        want = [i for i in range(9) if all(t[k, -1] > t[i, -1] for k in range(i + 1, 9))]
        assert keep == want
        assert all(t[a, -1] < t[b, -1] for a, b in zip(keep, keep[1:]))
    t = synthetic_table()
    assert profiler.pareto_subset(t) == list(range(6))
