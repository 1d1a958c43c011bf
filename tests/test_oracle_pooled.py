"""Pins for the oracle's second serving policy, stage pools (refill = 2): survivors of exit i wait in a
pool in front of segment i+1 and segments run on full batches.  The policy is an extension, so there is
no printed example; it is pinned by a timeline worked by hand, by the closed form it reduces to at
B_max = 1, by a replay that checks every launch against the statement of the policy, and by counting
launches."""
import numpy as np
import pytest

from test_oracle_sched import random_case

PROC, CRITERION = 2, 4


def serve(orc, arrivals, forced, b_max, lut, slo=-1, n_stages=None):
    return orc.serve_stream(None, np.asarray(arrivals, np.int64), None, b_max, np.asarray(lut, np.int64), t_slo_ns=slo, refill=2,
                            forced_exit=np.asarray(forced, np.int32), n_stages=n_stages or len(lut), max_events=200000)


def test_timeline_worked_by_hand(orc):
    """Six requests at t = 0, B_max = 2, three segments with T[s][b] = 10 (s + 1) + b.
    t=0    queue 6            -> segment 1 on {0,1}: 12.  0 leaves at 12.   pool1 = [1]
    t=12   pool1 1, queue 4   -> segment 1 on {2,3}: 12.  nobody leaves.     pool1 = [1,2,3]
    t=24   pool1 3 (full)     -> segment 2 on {1,2}: 22.  1 leaves at 46.   pool1 = [3], pool2 = [2]
    t=46   pools 1/1, queue 2 -> segment 1 on {4,5}: 12.  5 leaves at 58.   pool1 = [3,4]
    t=58   pool1 full         -> segment 2 on {3,4}: 22.  4 leaves at 80.   pool2 = [2,3]
    t=80   pool2 full         -> segment 3 on {2,3}: 32.  both leave at 112."""
    lut = [[10 * (s + 1) + b for b in (1, 2)] for s in range(3)]
    res, st, ev = serve(orc, [0] * 6, [0, 1, 2, 2, 1, 0], 2, lut)
    assert res["latency_ns"].tolist() == [12, 46, 112, 112, 80, 58]
    assert res["exit_idx"].tolist() == [0, 1, 2, 2, 1, 0]
    assert [(int(e["t_ns"]), int(e["stage"]), int(e["b"])) for e in ev[ev["kind"] == PROC]] == \
        [(0, 0, 2), (12, 0, 2), (24, 1, 2), (46, 0, 2), (58, 1, 2), (80, 2, 2)]
    assert st["seg_runs"][:3] == [3, 2, 1] and st["end_time_ns"] == 112 and st["rounds"] == 3


@pytest.mark.parametrize("seed", range(3))
def test_one_slot_is_serial_service(orc, seed):
    """B_max = 1: every pool is full as soon as it holds a sample and the deepest goes first, so a request
    runs to its exit before the next one starts: completion_k = max(completion_{k-1}, arrival_k) + sum of its segments."""
    arrivals, forced, lut = random_case(seed, n=120, b_max=1, rate=0.004)
    res, st, _ = serve(orc, arrivals, forced, 1, lut)
    done = 0
    for k in range(len(arrivals)):
        done = max(done, arrivals[k]) + int(lut[: forced[k] + 1, 0].sum())
        assert res["latency_ns"][k] == done - arrivals[k]
    assert st["end_time_ns"] == done


def replay(arrivals, forced, lut, b_max, ev, slo=-1):
    """Walks the launches in order with pool sizes kept from the forced exits and checks each against the
    statement of the policy: which level is preferred, when another one may override it, the batch taken."""
    E = len(lut)
    cnt = [0] * E
    members = [[] for _ in range(E)]
    taken = 0
    now = None
    overrides = 0
    for e in ev[ev["kind"] == PROC]:
        t, L, b = int(e["t_ns"]), int(e["stage"]), int(e["b"])
        if now is not None:
            assert t >= now
            if t > now:                                     # the server idled: nothing at all was waiting
                assert sum(cnt[1:]) == 0 and int(np.count_nonzero(arrivals <= now)) == taken
        cnt[0] = int(np.count_nonzero(arrivals <= t)) - taken
        full = [i for i in range(E) if cnt[i] >= b_max]
        inflight = [i for i in range(1, E) if cnt[i] > 0]
        pref = max(full) if full else (max(inflight) if inflight else 0)
        assert cnt[L] > 0 and b == min(cnt[L], b_max)

        def urgent(i):
            bi = min(cnt[i], b_max)
            rest = sum(int(lut[s][bi - 1]) for s in range(i, E))
            slack = slo - (t - min(arrivals[m] for m in members[i]))
            return rest < slack <= int(lut[pref][min(cnt[pref], b_max) - 1]) + rest

        candidates = [i for i in range(E - 1, 0, -1)
                      if i != pref and cnt[i] > 0 and slo >= 0 and (i + 1 == E or cnt[i + 1] < b_max) and urgent(i)]
        assert L == (candidates[0] if candidates else pref)  # only an SLO lets another pool go first, the deepest such
        overrides += L != pref
        if L == 0:
            batch = list(range(taken, taken + b))
            taken += b
        else:
            batch, members[L] = members[L][:b], members[L][b:]
        cnt[L] -= b
        stay = [m for m in batch if forced[m] > L and L < E - 1]
        if L + 1 < E:
            members[L + 1] += stay
            cnt[L + 1] += len(stay)
            assert cnt[L + 1] <= 2 * b_max - 1              # a pool never needs more room than this
        now = t + int(lut[L][b - 1])
    assert sum(cnt[1:]) == 0 and taken == len(arrivals)
    return overrides


@pytest.mark.parametrize("seed", range(6))
def test_every_launch_is_the_one_the_policy_names(orc, seed):
    b_max = 8
    arrivals, forced, lut = random_case(seed, n=400, b_max=b_max, rate=[0.02, 0.2, 0.05, 0.5, 0.01, 0.1][seed])
    res, st, ev = serve(orc, arrivals, forced, b_max, lut)
    assert st["n_events"] == len(ev) and st["preemptions"] == 0
    assert np.array_equal(res["exit_idx"], forced)
    assert replay(arrivals, forced, lut, b_max, ev) == 0
    assert st["seg_samples"][0] == len(arrivals)
    for s in range(1, 4):
        assert st["seg_samples"][s] == int(np.count_nonzero(forced >= s))
    # a request completes no earlier than its own segments take at the fastest table entry
    floor = np.array([lut[: f + 1].min(axis=1).sum() for f in forced])
    assert np.all(res["latency_ns"] >= floor)


@pytest.mark.parametrize("seed", range(4))
def test_slo_overrides_are_the_stated_ones(orc, seed):
    b_max = 8
    arrivals, forced, lut = random_case(20 + seed, n=400, b_max=b_max, rate=[0.02, 0.03, 0.2, 0.03][seed])
    slo = [900, 600, 1500, 700][seed]
    res, st, ev = serve(orc, arrivals, forced, b_max, lut, slo=slo)
    assert np.array_equal(res["exit_idx"], forced)
    assert replay(arrivals, forced, lut, b_max, ev, slo=slo) == st["preemptions"]
    assert st["criterion_evals"] == int(np.count_nonzero(ev["kind"] == CRITERION))


def test_slo_override_by_hand(orc):
    """B_max = 4, two segments.  Four requests at t = 0, request 0 survives exit 1 at t = T1[4] = 40 and waits
    alone in the pool; eight more requests have arrived, so the queue is full and preferred.  The pool goes
    first iff T2[1] = 15 < T_slack and not 40 + 15 < T_slack, with T_slack = T_SLO - 40: T_SLO in (55, 95]."""
    lut = [[10, 20, 30, 40], [15, 25, 35, 45]]
    arrivals = [0, 0, 0, 0] + [1] * 8
    forced = [1, 0, 0, 0] + [0] * 8
    for slo, lat0 in ((95, 55), (56, 55), (55, 135), (96, 95), (-1, 135)):
        res, st, ev = serve(orc, arrivals, forced, 4, lut, slo=slo)
        assert res["latency_ns"][0] == lat0, slo
    # T_SLO = 96: not urgent at t = 40 (55 < 56), urgent one step later at t = 80 (slack 16: 15 < 16 <= 55)
    res, st, ev = serve(orc, arrivals, forced, 4, lut, slo=96)
    assert [(int(e["t_ns"]), int(e["stage"]), int(e["b"])) for e in ev[ev["kind"] == PROC]] == [(0, 0, 4), (40, 0, 4), (80, 1, 1), (95, 0, 4)]
    assert st["preemptions"] == 1 and st["criterion_evals"] == 2


def test_full_batches_under_overload(orc):
    """Everything queued at t = 0: all launches but the last few run at B_max, so segment s needs at most
    ceil(N_s / B_max) launches plus the partial ones of the final drain (fewer than |E| per level), and on a
    machine with a fixed cost per launch the job ends earlier than under model-level batching."""
    b_max, E = 8, 4
    _, forced, _ = random_case(7, n=2000)
    lut = (100 + 5 * np.arange(1, b_max + 1))[None, :].repeat(E, axis=0).astype(np.int64)
    zeros = np.zeros(len(forced), np.int64)
    res, st, ev = serve(orc, zeros, forced, b_max, lut)
    proc = ev[ev["kind"] == PROC]
    for s in range(E):
        n_s = int(np.count_nonzero(forced >= s))
        runs = proc[proc["stage"] == s]
        assert -(-n_s // b_max) <= len(runs) <= -(-n_s // b_max) + E
        assert np.count_nonzero(runs["b"] < b_max) <= E
    static, sst, _ = orc.serve_stream(None, zeros, None, b_max, lut, refill=0, forced_exit=forced, n_stages=E)
    assert st["end_time_ns"] < 0.8 * sst["end_time_ns"]


# ---- several steps in flight (lanes) ------------------------------------------------------------------
def serve_lanes(orc, arrivals, forced, b_max, lut, lanes, slo=-1):
    return orc.serve_stream(None, np.asarray(arrivals, np.int64), None, b_max, np.asarray(lut, np.int64), t_slo_ns=slo, refill=2, lanes=lanes,
                            forced_exit=np.asarray(forced, np.int32), n_stages=len(lut), max_events=400000)


def test_two_lanes_timeline_worked_by_hand(orc):
    """The six requests of the one-lane timeline above on two lanes (same table: T[s][b] = 10 (s + 1) + b, B_max = 2).
    t=0    lane 0: segment 1 on {0,1} until 12; lane 1 idle (level 0 is in flight, the pools are empty)
    t=12   0 leaves.  pool1 = [1].  lane 0: segment 1 on {2,3} until 24; lane 1: pool1 is not full, a step is running -> idle
    t=24   nobody leaves.  pool1 = [1,2,3].  lane 0: segment 2 on {1,2} until 46; lane 1: segment 1 on {4,5} until 36
    t=36   5 leaves.  pool1 = [3,4].  lane 1: level 1 is in flight, the queue is empty -> idle
    t=46   1 leaves.  pool2 = [2].  lane 0: segment 2 on {3,4} until 68; lane 1: pool2 is not full -> idle
    t=68   4 leaves.  pool2 = [2,3].  lane 0: segment 3 on {2,3} until 100: both leave."""
    lut = [[10 * (s + 1) + b for b in (1, 2)] for s in range(3)]
    res, st, ev = serve_lanes(orc, [0] * 6, [0, 1, 2, 2, 1, 0], 2, lut, lanes=2)
    assert res["latency_ns"].tolist() == [12, 46, 100, 100, 68, 36]
    assert [(int(e["t_ns"]), int(e["stage"]), int(e["b"]), int(e["aux"])) for e in ev[ev["kind"] == PROC]] == \
        [(0, 0, 2, 0), (12, 0, 2, 0), (24, 1, 2, 0), (24, 0, 2, 1), (46, 1, 2, 0), (68, 2, 2, 0)]
    assert st["end_time_ns"] == 100 and st["seg_runs"][:3] == [3, 2, 1]


def test_idle_lane_starts_when_an_arrival_fills_a_batch(orc):
    """B_max = 2, two segments, T[s][b] = 10 (s + 1) + b.  Requests 0, 1 arrive at 0 and leave at the last exit, requests 2, 3
    arrive at 13 and 15 and leave at the first.  Lane 0 runs segment 1 on {0,1} until 12 and then segment 2 on them until 34.
    At t = 13 the queue holds one request: not a full batch while a step is running, so lane 1 waits; at t = 15 it holds two and
    lane 1 runs segment 1 on {2,3} until 27.  (While lane 0 ran segment 1 itself, lane 1 could not have: one step per level.)"""
    lut = [[11, 12], [21, 22]]
    res, st, ev = serve_lanes(orc, [0, 0, 13, 15], [1, 1, 0, 0], 2, lut, lanes=2)
    assert [(int(e["t_ns"]), int(e["stage"]), int(e["b"]), int(e["aux"])) for e in ev[ev["kind"] == PROC]] == [(0, 0, 2, 0), (12, 1, 2, 0), (15, 0, 2, 1)]
    assert res["latency_ns"].tolist() == [34, 34, 14, 12]
    # one lane: the second batch waits for the first to finish
    res1, _, _ = serve_lanes(orc, [0, 0, 13, 15], [1, 1, 0, 0], 2, lut, lanes=1)
    assert res1["latency_ns"].tolist() == [34, 34, 33, 31]
    # a single-segment network never overlaps: one step per level
    res2, _, ev2 = serve_lanes(orc, [0, 0, 3, 5], [0, 0, 0, 0], 2, [[11, 12]], lanes=2)
    assert [(int(e["t_ns"]), int(e["aux"])) for e in ev2[ev2["kind"] == PROC]] == [(0, 0), (12, 0)]


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("lanes", [2, 3, 4])
def test_lanes_invariants(orc, seed, lanes):
    b_max, E = 8, 4
    arrivals, forced, lut = random_case(40 + seed, n=500, b_max=b_max, rate=[0.05, 0.3, 1.0, 0.02, 0.15][seed])
    res, st, ev = serve_lanes(orc, arrivals, forced, b_max, lut, lanes)
    assert np.array_equal(res["exit_idx"], forced)
    proc = ev[ev["kind"] == PROC]
    t0 = proc["t_ns"].astype(np.int64)
    t1 = t0 + np.array([lut[int(s)][int(b) - 1] for s, b in zip(proc["stage"], proc["b"])])
    order = np.argsort(t0, kind="stable")
    assert np.array_equal(order, np.arange(len(proc)))                       # logged in time order
    for k in range(len(proc)):
        live = (t0[:k] <= t0[k]) & (t1[:k] > t0[k])                          # steps still running when step k starts
        assert np.count_nonzero(live) < lanes
        assert not np.any(proc["stage"][:k][live] == proc["stage"][k])       # one step per level at a time
        assert not np.any(proc["aux"][:k][live] == proc["aux"][k])           # a lane runs one step at a time
        if np.any(live):
            assert proc["b"][k] == b_max                                     # beside a running step only full batches start
    # first in, first out at every level: a level's batches take the samples in the order they reached it
    done_at = res["latency_ns"] + arrivals
    for s in range(E):
        runs = proc[proc["stage"] == s]
        ends = (runs["t_ns"].astype(np.int64) + np.array([lut[s][int(b) - 1] for b in runs["b"]]))
        leavers = np.nonzero(forced == s)[0]
        assert set(done_at[leavers].tolist()) <= set(ends.tolist())           # a sample completes when a step of its exit's segment ends
    assert st["seg_samples"][0] == len(arrivals)
    for s in range(1, E):
        assert st["seg_samples"][s] == int(np.count_nonzero(forced >= s))
    busy = int((t1 - t0).sum())
    assert st["end_time_ns"] - arrivals[0] >= busy / lanes                    # work conservation


@pytest.mark.parametrize("seed", range(3))
def test_one_lane_is_the_plain_policy_and_more_lanes_finish_sooner_under_overload(orc, seed):
    b_max = 8
    _, forced, lut = random_case(60 + seed, n=1500, b_max=b_max)
    zeros = np.zeros(len(forced), np.int64)
    base = serve(orc, zeros, forced, b_max, lut)
    one = serve_lanes(orc, zeros, forced, b_max, lut, 1)
    assert np.array_equal(base[0], one[0]) and base[1] == one[1] and np.array_equal(base[2], one[2])
    two = serve_lanes(orc, zeros, forced, b_max, lut, 2)
    assert two[1]["end_time_ns"] < 0.75 * one[1]["end_time_ns"]               # the second lane is busy most of the time
    assert two[1]["end_time_ns"] >= 0.5 * one[1]["end_time_ns"] - lut.max() * 8  # and cannot more than halve the time (up to the drain)
