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
