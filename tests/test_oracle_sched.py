"""Pins for the oracle's Algorithm 1: the paper's timeline example, its batch-size identities,
Eq. 3 / Eq. 4 worked by hand, and the degenerate policies."""
import os

import numpy as np
import pytest

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "timeline_example.txt")
KINDS = {"ROUND": 1, "PROC": 2, "CATCHUP": 3, "CRITERION": 4, "MERGE": 5}


def read_timeline():
    events, samples = [], []
    for line in open(GOLD):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[1] in KINDS:
            events.append((int(tok[0]), KINDS[tok[1]], int(tok[2]), int(tok[3]), int(tok[4])))
        else:
            samples.append(tuple(int(t) for t in tok))
    return events, samples


def test_paper_timeline_example(orc):
    events, samples = read_timeline()
    arrivals = np.array([0, 0, 5, 5, 5, 5, 15], np.int64)
    forced = np.array([s[1] - 1 for s in samples], np.int32)
    lut = np.full((2, 8), 10, np.int64)
    res, st, ev = orc.serve_stream(None, arrivals, None, 8, lut, t_slo_ns=35, forced_exit=forced, n_stages=2, max_events=64)
    got = [(int(e["t_ns"]), int(e["kind"]), int(e["stage"]), int(e["b"]), int(e["aux"])) for e in ev]
    assert got == events
    for (sid, ex, done), r, arr in zip(samples, res, arrivals):
        assert r["exit_idx"] == ex - 1 and r["latency_ns"] == done - arr
    assert st["preemptions"] == 1 and st["criterion_evals"] == 2 and st["rounds"] == 2


def random_case(seed, n=300, n_stages=4, b_max=8, rate=0.02):
    rng = np.random.default_rng(seed)
    arrivals = np.floor(np.cumsum(rng.exponential(1.0 / rate, size=n))).astype(np.int64)
    arrivals -= arrivals[0]
    forced = rng.choice(n_stages, size=n, p=[0.2, 0.2, 0.3, 0.3][:n_stages]).astype(np.int32)
    base = rng.integers(50, 100, size=n_stages)
    lut = (base[:, None] + np.arange(b_max)[None, :] * rng.integers(1, 6, size=(n_stages, 1))).astype(np.int64)
    return arrivals, forced, lut


@pytest.mark.parametrize("seed", range(6))
def test_batch_size_identities(orc, seed):
    b_max = 8
    arrivals, forced, lut = random_case(seed, b_max=b_max)
    res, st, ev = orc.serve_stream(None, arrivals, None, b_max, lut, t_slo_ns=-1, forced_exit=forced, n_stages=4, max_events=100000)
    assert st["n_events"] == len(ev)
    assert np.array_equal(res["exit_idx"], forced)                    # everyone leaves once, where told
    assert np.all(ev["b"][ev["kind"] != 4] <= b_max) and np.all(ev["b"][(ev["kind"] == 2) | (ev["kind"] == 3)] >= 1)
    # B_merged = B_rem + B_incr - B_exit: the MERGE size equals the previous batch + catch-up survivors
    for k in np.nonzero(ev["kind"] == 5)[0]:
        crit = k - 1
        while ev["kind"][crit] != 4:
            crit -= 1
        assert ev["aux"][crit] == 1 and ev["aux"][k] <= ev["b"][crit]           # survivors <= B_incr
        assert ev["b"][k] <= b_max
    # the criterion is only evaluated at intermediate exits, never after the last segment
    assert np.all(ev["stage"][ev["kind"] == 4] < 3)
    # FIFO + no idling while work is queued: a sample never starts before it arrives
    assert np.all(res["latency_ns"] >= lut[0].min())
    # every sample was processed by segment 0 exactly once
    assert st["seg_samples"][0] == len(arrivals)
    for s in range(1, 4):
        assert st["seg_samples"][s] == int(np.count_nonzero(forced >= s))


def test_scheduler_invoked_only_between_segments(orc):
    """One batch, nothing queued behind it: no criterion evaluation at all; with a deep queue
    the scheduler runs at the |E|-1 intermediate exits of a round (Sec. III-B, Preemptible Points)."""
    lut = np.full((4, 8), 10, np.int64)
    forced = np.full(8, 3, np.int32)
    res, st, ev = orc.serve_stream(None, np.zeros(8, np.int64), None, 8, lut, forced_exit=forced, n_stages=4, max_events=100)
    assert st["criterion_evals"] == 0 and st["rounds"] == 1 and np.all(res["latency_ns"] == 40)
    # 16 requests at t=0, the first 8 each lose one sample per exit -> one catch-up per intermediate exit
    forced = np.array([0, 1, 2, 3, 3, 3, 3, 3] + [3] * 8, np.int32)
    res, st, ev = orc.serve_stream(None, np.zeros(16, np.int64), None, 8, lut, forced_exit=forced, n_stages=4, max_events=100)
    first_round = ev[: np.nonzero(ev["kind"] == 1)[0][1]] if np.count_nonzero(ev["kind"] == 1) > 1 else ev
    assert sorted(first_round["stage"][first_round["kind"] == 4].tolist()) == [0, 1, 2]


def test_no_refill_is_model_level_batching(orc):
    arrivals, forced, lut = random_case(11)
    a, sa, _ = orc.serve_stream(None, arrivals, None, 8, lut, refill=0, forced_exit=forced, n_stages=4)
    b, sb, _ = orc.serve_stream(None, arrivals, None, 8, lut, refill=1, t_slo_ns=0, forced_exit=forced, n_stages=4)
    assert sa["preemptions"] == 0 and sb["preemptions"] == 0
    assert np.array_equal(a["latency_ns"], b["latency_ns"])           # an SLO of zero refuses every preemption
    # model-level batching by hand: rounds of <= 8 in FIFO order, each runs all four segments
    now, k, lat = 0, 0, np.zeros(len(arrivals), np.int64)
    n = len(arrivals)
    while k < n:
        now = max(now, arrivals[k])
        batch = [i for i in range(k, min(n, k + 8)) if arrivals[i] <= now]
        k += len(batch)
        alive = batch
        for s in range(4):
            if not alive:
                break
            now += lut[s, len(alive) - 1]
            for i in alive:
                if forced[i] == s or s == 3:
                    lat[i] = now - arrivals[i]
            alive = [i for i in alive if forced[i] > s and s < 3]
    assert np.array_equal(a["latency_ns"], lat)


def test_refill_raises_mean_batch_of_deep_segments(orc):
    arrivals, forced, _ = random_case(5, n=2000, rate=0.2)              # overloaded server
    # a machine whose segment time grows with the batch (as on the paper's NPU): refilling pays
    lut = (20 + 10 * np.arange(1, 9))[None, :].repeat(4, axis=0).astype(np.int64)
    a, sa, _ = orc.serve_stream(None, arrivals, None, 8, lut, refill=0, forced_exit=forced, n_stages=4)
    b, sb, _ = orc.serve_stream(None, arrivals, None, 8, lut, refill=1, forced_exit=forced, n_stages=4)
    mean_b = lambda st: st["seg_samples"][3] / st["seg_runs"][3]
    assert mean_b(sb) > mean_b(sa) * 1.5            # the deep segment runs (almost) full: 7.99 vs 2.51 of 8
    assert mean_b(sb) > 7.5 and sb["preemptions"] > 0


def test_slo_criterion_by_hand(orc):
    """Two samples start at t=0, one exits at E1 (t = T1[2] = 110); four more are queued.  Eq. 4:
    T_overhead = T1[4] + T2[5] = 130 + 250 = 380.  Eq. 3: T_slack = T_SLO - 110."""
    lut = np.array([[100, 110, 120, 130, 140, 150, 160, 170], [210, 220, 230, 240, 250, 260, 270, 280]], np.int64)
    arrivals = np.array([0, 0, 1, 2, 3, 4], np.int64)
    forced = np.array([1, 0, 1, 1, 1, 1], np.int32)
    for slo, accept in ((490, False), (491, True)):
        res, st, ev = orc.serve_stream(None, arrivals, None, 8, lut, t_slo_ns=slo, forced_exit=forced, n_stages=2, max_events=50)
        crit = ev[ev["kind"] == 4][0]
        assert crit["t_ns"] == 110 and crit["b"] == 4 and crit["aux"] == int(accept)
        if accept:
            # upper bound of Eq. 4 holds: the preempted sample still meets its SLO
            assert res["latency_ns"][0] == 110 + 130 + 250 and res["latency_ns"][0] <= slo
        else:
            assert res["latency_ns"][0] == 110 + 210


def test_min_incr_and_errors(orc):
    arrivals, forced, lut = random_case(3)
    _, s1, _ = orc.serve_stream(None, arrivals, None, 8, lut, forced_exit=forced, n_stages=4)
    _, s4, _ = orc.serve_stream(None, arrivals, None, 8, lut, min_incr=4, forced_exit=forced, n_stages=4)
    assert 0 < s4["preemptions"] < s1["preemptions"]
    bad = arrivals.copy()
    bad[10] = bad[9] - 1
    with pytest.raises(orc.OracleError):
        orc.serve_stream(None, bad, None, 8, lut, forced_exit=forced, n_stages=4)


# ---- baselines of the evaluation: SERIAL and adaptive batching <B_max, T_timeout> ------------------------
def test_adaptive_batching_timeline_by_hand(orc):
    """B_max = 4, two segments of 10 each (any batch size), nobody leaves early, T_timeout = 20.
    t=0   request 0 queued; window ends at 20; request 1 joins at 3; nothing else by 20 -> {0,1} issued at 20, done at 40
    t=40  queue empty -> idle until 50; window ends at 70; 51, 52, 53 join: the batch is full at 53 -> issued at 53, done at 73
    t=73  request 6 (arrived 54) has waited 19 < 20 -> issued at 74, done at 94"""
    arrivals = np.array([0, 3, 50, 51, 52, 53, 54], np.int64)
    forced = np.ones(7, np.int32)
    lut = np.full((2, 4), 10, np.int64)
    res, st, ev = orc.serve_stream(None, arrivals, None, 4, lut, refill=0, t_timeout_ns=20, forced_exit=forced, n_stages=2, max_events=64)
    assert res["latency_ns"].tolist() == [40, 37, 23, 22, 21, 20, 40]
    assert [(int(e["t_ns"]), int(e["b"])) for e in ev[ev["kind"] == KINDS["ROUND"]]] == [(20, 2), (53, 4), (74, 1)]
    assert st["rounds"] == 3 and st["end_time_ns"] == 94
    # a request that arrives exactly when the window ends still joins the batch
    res, st, ev = orc.serve_stream(None, np.array([0, 20], np.int64), None, 4, lut, refill=0, t_timeout_ns=20, forced_exit=np.ones(2, np.int32), n_stages=2, max_events=8)
    assert [(int(e["t_ns"]), int(e["b"])) for e in ev[ev["kind"] == KINDS["ROUND"]]] == [(20, 2)]


@pytest.mark.parametrize("seed", range(3))
def test_adaptive_batching_closed_forms(orc, seed):
    b_max = 8
    arrivals, forced, lut = random_case(70 + seed, n=240, b_max=b_max, rate=[0.01, 0.05, 0.3][seed])
    plain = orc.serve_stream(None, arrivals, None, b_max, lut, refill=0, forced_exit=forced, n_stages=4, max_events=10000)
    zero = orc.serve_stream(None, arrivals, None, b_max, lut, refill=0, t_timeout_ns=0, forced_exit=forced, n_stages=4, max_events=10000)
    assert np.array_equal(plain[0], zero[0]) and plain[1] == zero[1]            # no window = model-level batching as it comes
    # an endless window: every batch is full (240 = 30 * 8) and is issued when its last member has arrived and the server is free
    res, st, ev = orc.serve_stream(None, arrivals, None, b_max, lut, refill=0, t_timeout_ns=10**15, forced_exit=forced, n_stages=4, max_events=10000)
    rounds = ev[ev["kind"] == KINDS["ROUND"]]
    assert len(rounds) == 30 and np.all(rounds["b"] == b_max)
    free = 0
    for k in range(30):
        members = np.arange(8 * k, 8 * k + 8)
        start = max(free, int(arrivals[members[-1]]))
        assert int(rounds["t_ns"][k]) == start
        t, alive = start, members
        for s in range(4):                                                       # model-level batching: the batch shrinks, nothing joins
            if len(alive) == 0:
                break
            t += int(lut[s][len(alive) - 1])
            for m in alive[(forced[alive] == s) | (s == 3)]:
                assert res["latency_ns"][m] == t - arrivals[m]
            alive = alive[(forced[alive] > s) & (s < 3)]
        free = t
    # every window in between: nobody is issued before the window allows, nobody waits for batch forming longer than the window
    for window in (50, 400, 3000):
        res, st, ev = orc.serve_stream(None, arrivals, None, b_max, lut, refill=0, t_timeout_ns=window, forced_exit=forced, n_stages=4, max_events=10000)
        rounds = ev[ev["kind"] == KINDS["ROUND"]]
        first = 0
        prev_end = None
        procs = ev[ev["kind"] == KINDS["PROC"]]
        for k, r in enumerate(rounds):
            t, b = int(r["t_ns"]), int(r["b"])
            oldest = int(arrivals[first])
            assert b == b_max or t >= oldest + window                            # an incomplete batch only after the window
            assert b == int(np.count_nonzero(arrivals[first:first + b_max] <= t))   # everyone who had arrived (up to B_max) is in it
            first += b
        assert first == len(arrivals)


@pytest.mark.parametrize("seed", range(2))
def test_serial_is_one_request_at_a_time(orc, seed):
    arrivals, forced, lut = random_case(80 + seed, n=150, b_max=1, rate=0.004)
    res, st, _ = orc.serve_stream(None, arrivals, None, 1, lut, refill=0, forced_exit=forced, n_stages=4)
    done = 0
    for k in range(len(arrivals)):
        done = max(done, int(arrivals[k])) + int(lut[: forced[k] + 1, 0].sum())
        assert res["latency_ns"][k] == done - arrivals[k]
    assert st["rounds"] == len(arrivals)
