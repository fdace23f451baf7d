"""Host-side policies, traces and the router model (no GPU): each policy against its definition
written out by exhaustive search, trace statistics against their parameters, and the event loop on
cases small enough to work by hand."""
import numpy as np
import pytest

from paper_2312_16733_amd import profiler, scheduler

BATCHES = profiler.POW2_BATCHES


def table(n=7):
    b = np.asarray(BATCHES, np.float64)
    return np.stack([0.3 + 0.07 * i + (0.02 + 0.013 * i) * b for i in range(n)])   # monotone both ways


def brute_maxbatch(t, theta):
    js = [j for j in range(t.shape[1]) if t[0, j] < theta]
    if not js:
        return None
    j = max(js)
    return j, max(i for i in range(t.shape[0]) if t[i, j] < theta)


def brute_maxacc(t, theta):
    rows = [i for i in range(t.shape[0]) if t[i, 0] < theta]
    if not rows:
        return None
    i = max(rows)
    return max(j for j in range(t.shape[1]) if t[i, j] < theta), i


def test_maxbatch_and_maxacc_match_exhaustive_search():
    t = table()
    mb, ma = scheduler.MaxBatch(t, BATCHES), scheduler.MaxAcc(t, BATCHES)
    for theta in np.concatenate([np.linspace(0.0, t.max() * 1.3, 301), t.ravel(), t.ravel() + 1e-9]):
        want = brute_maxbatch(t, theta)
        assert mb.choose(theta) == (want if want else (len(BATCHES) - 1, 0)), theta
        want = brute_maxacc(t, theta)
        assert ma.choose(theta) == (want if want else (len(BATCHES) - 1, 0)), theta
    # the two orders of greed differ: a slack that admits every subnet at batch 1 but few at batch 64
    theta = t[-1, 0] + 1e-6
    assert ma.choose(theta)[1] == t.shape[0] - 1 and mb.choose(theta)[0] > ma.choose(theta)[0]


def test_slackfit_matches_the_bucket_rule():
    t = table()
    for nb in (5, 16):
        sf = scheduler.SlackFit(t, BATCHES, nb)
        bks = profiler.latency_buckets(t, BATCHES, nb)
        for theta in np.linspace(0.0, t.max() * 1.3, 257):
            want = profiler.pick(bks, theta)
            got = sf.choose(theta)
            if want is None:
                assert got == (len(BATCHES) - 1, 0)
            else:
                assert (BATCHES[got[0]], got[1]) == want[:2]
                assert t[got[1], got[0]] <= theta
    # more slack never lowers the chosen latency bucket
    sf = scheduler.SlackFit(t, BATCHES, 16)
    lat = [t[i, j] for j, i in (sf.choose(th) for th in np.linspace(sf.edges[0], t.max() * 1.2, 100))]
    edges = np.asarray(sf.edges)
    assert all(np.searchsorted(edges, a, side="left") <= np.searchsorted(edges, b, side="left") for a, b in zip(lat, lat[1:]))


@pytest.mark.parametrize("cv2", [0.0, 2.0, 8.0])
def test_gamma_arrivals_have_the_requested_rate_and_variation(cv2):
    rng = np.random.default_rng(3)
    a = scheduler.gamma_arrivals(5000.0, cv2, 20.0, rng)
    gaps = np.diff(a)
    assert abs(len(a) / 20.0 - 5000.0) < 5000.0 * 0.05
    assert abs(gaps.mean() - 1 / 5000.0) < 0.05 / 5000.0
    got_cv2 = gaps.var() / gaps.mean() ** 2
    assert abs(got_cv2 - cv2) <= 0.1 * max(cv2, 0.1)
    assert (gaps >= 0).all() and a[-1] < 20.0


def test_traces_are_seeded_sorted_and_shaped():
    a = scheduler.bursty_trace(1500.0, 5550.0, 4.0, 4.0, 11)
    b = scheduler.bursty_trace(1500.0, 5550.0, 4.0, 4.0, 11)
    assert np.array_equal(a, b) and (np.diff(a) >= 0).all()
    assert abs(len(a) / 4.0 - 7050.0) < 7050.0 * 0.08
    t = scheduler.accelerating_trace(2500.0, 7400.0, 5000.0, 8.0, 4.0, 5)
    early = ((t >= 0.0) & (t < 0.2)).sum() / 0.2
    late = ((t >= 2.0) & (t < 4.0)).sum() / 2.0
    assert early < 4500 and abs(late - 7400.0) < 7400.0 * 0.15        # ramp done after (7400 - 2500) / 5000 = 0.98 s
    assert (np.diff(t) >= 0).all()          # shape 1/8 gamma gaps can round to nothing


def test_router_model_on_a_case_worked_by_hand():
    # one subnet, batches 1 and 2: L(1) = 1 ms, L(2) = 1.5 ms; SLO 2 ms; one worker
    t = np.array([[1.0, 1.5]])
    pol = scheduler.MaxBatch(t, (1, 2))
    # queries at 0, 0.1, 0.2 ms.  t=0: queue {q0}, slack 2 -> b=2 but one queued: takes 1, done at 1.0 (met).
    # t=1.0: queue {q1 (deadline 2.1), q2 (2.2)}, slack 1.1 -> b=1 (L(2)=1.5 >= 1.1): q1 done 2.0 (met).
    # t=2.0: q2 slack 0.2 -> nothing fits -> fallback b=2, takes 1, charged L(1): done 3.0 > 2.2 (miss).
    r = scheduler.simulate(pol, np.array([0.0, 0.1e-3, 0.2e-3]), slo_ms=2.0, n_workers=1)
    assert r["served"] == 3 and r["dropped"] == 0
    assert abs(r["slo_attainment"] - 2 / 3) < 1e-12
    assert [(round(d[0] * 1e3, 6), d[2], d[4]) for d in r["decisions"]] == [(0.0, 2, 1), (1.0, 1, 1), (2.0, 2, 1)]
    # two workers: q1 starts at 0.1 on the second worker -> all three meet the deadline
    r2 = scheduler.simulate(pol, np.array([0.0, 0.1e-3, 0.2e-3]), slo_ms=2.0, n_workers=2)
    assert r2["slo_attainment"] == 1.0
    # a query that is already late when a worker frees up is dropped and counted as a miss
    slow = scheduler.MaxBatch(np.array([[5.0, 5.5]]), (1, 2))
    r3 = scheduler.simulate(slow, np.array([0.0, 0.1e-3]), slo_ms=2.0, n_workers=1)
    assert r3["dropped"] == 1 and r3["served"] == 1 and r3["slo_attainment"] == 0.0


def test_every_query_is_served_or_dropped_once_and_batches_follow_deadline_order():
    t = table()
    arr = scheduler.bursty_trace(300.0, 1200.0, 8.0, 1.0, 2)
    for pol in (scheduler.SlackFit(t, BATCHES), scheduler.MaxBatch(t, BATCHES), scheduler.MaxAcc(t, BATCHES)):
        r = scheduler.simulate(pol, arr, slo_ms=4.0, n_workers=2)
        assert r["served"] + r["dropped"] == r["queries"] == len(arr)
        assert 0.0 <= r["slo_attainment"] <= r["served"] / r["queries"]
        assert 0.0 <= r["mean_accuracy_rank"] <= 1.0
        assert all(d[4] <= d[2] for d in r["decisions"])
        times = [d[0] for d in r["decisions"]]
        assert times == sorted(times)


def test_slackfit_trades_accuracy_for_attainment_under_burst():
    """The behaviour the paper reports: with a bursty overload-prone trace SlackFit keeps SLO attainment
    at least as high as MaxAcc, and serves a higher accuracy rank than MaxBatch on a calm one."""
    t = table()
    cap_large = 64 / (t[-1, -1] * 1e-3)
    calm = scheduler.bursty_trace(0.3 * cap_large, 0.0, 0.0, 1.0, 1)
    res = {p.name: scheduler.simulate(p, calm, slo_ms=3 * t[-1, -1], n_workers=1)
           for p in (scheduler.SlackFit(t, BATCHES), scheduler.MaxBatch(t, BATCHES), scheduler.MaxAcc(t, BATCHES))}
    assert res["SlackFit"]["slo_attainment"] > 0.99
    assert res["SlackFit"]["mean_accuracy_rank"] >= res["MaxBatch"]["mean_accuracy_rank"]
    burst = scheduler.bursty_trace(0.3 * cap_large, 1.5 * cap_large, 8.0, 1.0, 4)
    rb = {p.name: scheduler.simulate(p, burst, slo_ms=3 * t[-1, -1], n_workers=1)
          for p in (scheduler.SlackFit(t, BATCHES), scheduler.MaxAcc(t, BATCHES))}
    assert rb["SlackFit"]["slo_attainment"] >= rb["MaxAcc"]["slo_attainment"]


def test_simulate_charges_what_the_executor_reports():
    """With an executor the worker is busy for the returned time, not the table's; decisions still come from the table."""
    table = np.array([[1.0, 2.0], [3.0, 5.0]])
    pol = scheduler.MaxBatch(table, (1, 2))
    arrivals = np.array([0.0, 0.0, 0.0, 0.0])
    calls = []

    def slow(i, j, take):
        calls.append((i, j, take))
        return 10.0 * table[i, j]                       # ten times slower than profiled

    fast = scheduler.simulate(pol, arrivals, slo_ms=8.0, n_workers=1)
    live = scheduler.simulate(pol, arrivals, slo_ms=8.0, n_workers=1, executor=slow)
    # by hand: slack 8 -> batch 2 of the larger subnet (5 ms), done at 5; slack 3 -> batch 2 of the smaller (2 ms), done at 7
    assert fast["slo_attainment"] == 1.0
    assert calls[0] == (1, 1, 2)
    # ten times slower: the first batch ends at 50 ms, past its deadline; the other two are late at the head and dropped
    assert live["slo_attainment"] == 0.0 and live["dropped"] == 2
    assert live["slo_attainment"] < fast["slo_attainment"]
    assert live["decisions"][0][2:] == fast["decisions"][0][2:]
