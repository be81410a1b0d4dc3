"""Queue simulation of the serving experiment (paper_2310_18813_amd/traffic_sim.py): hand-worked cases, a
time-stepped brute-force server, and the statistics of the arrival generator.  No GPU."""
import numpy as np
import pytest

from paper_2310_18813_amd import traffic_sim as ts


def brute_force_server(arrivals, service_time, choose_s, max_batch, tick):
    """Plain time-stepped version of the server of Sec. 5.3: every tick, if free, take what waits."""
    n = len(arrivals)
    lat = np.zeros(n)
    t, busy_until, i = 0.0, 0.0, 0
    group = None
    while i < n or group is not None:
        if group is not None and t >= busy_until - 1e-12:
            lo, hi = group
            lat[lo:hi] = busy_until - arrivals[lo:hi]
            group = None
        if group is None and i < n:
            j = i
            while j < n and j - i < max_batch and arrivals[j] <= t + 1e-12:
                j += 1
            if j > i:
                B = j - i
                busy_until = t + service_time(B, choose_s(B))
                group = (i, j)
                i = j
        t += tick
    return lat


def test_hand_worked_queue():
    # service 1.0 s whatever the batch; arrivals 0.0, 0.1, 0.2, 2.5: first goes alone, the next two wait and go
    # together at t = 1.0, the last finds the server free
    lat, batches = ts.serve([0.0, 0.1, 0.2, 2.5], lambda b, s: 1.0, lambda b: 3, max_batch=16)
    assert [b for _, b, _ in batches] == [1, 2, 1]
    assert [s for _, _, s in batches] == [3, 3, 3]
    assert lat == pytest.approx([1.0, 1.9, 1.8, 1.0])
    # the batch limit splits a burst: 5 simultaneous requests, at most 2 per batch
    lat, batches = ts.serve([0.0] * 5, lambda b, s: 1.0, lambda b: 0, max_batch=2)
    assert [b for _, b, _ in batches] == [2, 2, 1]
    assert lat == pytest.approx([1.0, 1.0, 2.0, 2.0, 3.0])
    # nothing to serve
    lat, batches = ts.serve([], lambda b, s: 1.0, lambda b: 0)
    assert len(lat) == 0 and batches == []


def test_event_driven_server_matches_time_stepped_one():
    rng = np.random.default_rng(3)
    service = lambda b, s: 0.05 + 0.01 * b + 0.004 * s * b
    policy = lambda b: 4 if b <= 2 else 2
    for trial in range(5):
        arr = np.round(np.cumsum(rng.exponential(0.05, size=60)), 3)     # on the tick grid
        lat, _ = ts.serve(arr, service, policy, max_batch=4)
        ref = brute_force_server(arr, lambda b, s: round(service(b, s), 3), policy, 4, tick=0.001)
        lat2, _ = ts.serve(arr, lambda b, s: round(service(b, s), 3), policy, max_batch=4)
        assert lat2 == pytest.approx(ref, abs=2e-3)
        assert (lat >= 0.05).all()


def test_gamma_arrivals_have_the_requested_mean_and_cv():
    for mean, cv in [(0.3, 0.5), (0.1, 1.0), (0.8, 2.0), (0.2, 5.0)]:
        arr = ts.gamma_arrivals(200000, mean, cv, seed=1)
        gaps = np.diff(np.concatenate([[0.0], arr]))
        assert gaps.mean() == pytest.approx(mean, rel=0.05)
        assert gaps.std() / gaps.mean() == pytest.approx(cv, rel=0.08)
        assert (np.diff(arr) >= 0).all()
    assert np.array_equal(ts.gamma_arrivals(10, 0.3, 1.0, seed=5), ts.gamma_arrivals(10, 0.3, 1.0, seed=5))
    with pytest.raises(ValueError):
        ts.gamma_arrivals(10, 0.0, 1.0, seed=0)


def test_alternating_traffic_switches_rate():
    arr = ts.alternating_arrivals(400.0, [0.2, 1.0], 50.0, 1.0, seed=2)
    dense = ((arr >= 0) & (arr < 50)).sum() + ((arr >= 100) & (arr < 150)).sum()
    sparse = ((arr >= 50) & (arr < 100)).sum() + ((arr >= 150) & (arr < 200)).sum()
    assert dense == pytest.approx(500, rel=0.15) and sparse == pytest.approx(100, rel=0.3)


def test_lut_policy_is_the_rule_of_sec4():
    from oracle import oracle as om
    orc = om.Oracle("f64")
    pb, lut = [1, 2, 4, 8, 16], [6, 7, 5, 5, 3]
    choose = ts.lut_policy(pb, lut)
    for B in range(1, 40):
        assert choose(B) == orc.lut_lookup(pb, lut, B), B


def test_adaptive_wins_when_it_is_faster_for_every_batch_and_load_is_light():
    # light traffic: every request is served alone, so latency is the service time of B = 1
    service = lambda b, s: {0: 1.0, 2: 0.7, 4: 0.6}[s] * (1 + 0.1 * (b - 1) * (1 + s))
    arr = np.arange(50) * 10.0
    means = {s: ts.serve(arr, service, lambda b, s=s: s)[0].mean() for s in (0, 2, 4)}
    assert means[4] < means[2] < means[0]


def brute_force_continuous(arrivals, n_tokens, slots, dt_round, dt_admit, gain, tick):
    """Time-stepped continuous-batching server with constant round time and token gain: a state machine that
    looks at the clock every tick (all event times are multiples of the tick)."""
    n = len(arrivals)
    lat = np.zeros(n)
    who, left = [-1] * slots, [0] * slots
    nxt = done = 0
    busy_until, mode = 0.0, "idle"
    for k in range(10 ** 7):
        if done == n:
            return lat
        t = k * tick
        if t < busy_until - 1e-9:
            continue
        if mode == "round":  # the round that was running ends now
            for i in range(slots):
                if who[i] >= 0:
                    left[i] -= gain
                    if left[i] <= 0:
                        lat[who[i]] = busy_until - arrivals[who[i]]
                        who[i] = -1
                        done += 1
        mode = "idle"
        free = [i for i in range(slots) if who[i] < 0]
        if free and nxt < n and arrivals[nxt] <= t + 1e-9:
            who[free[0]], left[free[0]] = nxt, n_tokens
            nxt += 1
            busy_until, mode = t + dt_admit, "admitting"
        elif any(w >= 0 for w in who):
            busy_until, mode = t + dt_round, "round"
    raise AssertionError("the time-stepped server did not finish")


def test_continuous_server_hand_worked():
    # one slot, rounds of 1 s giving 2 tokens, requests of 4 tokens, admission 0.5 s:
    # request 0 arrives at 0: admitted 0..0.5, rounds end at 1.5 and 2.5 -> latency 2.5
    # request 1 arrives at 0.2, waits for the slot: admitted 2.5..3.0, rounds end at 4.0 and 5.0 -> latency 4.8
    lat, rounds = ts.serve_continuous([0.0, 0.2], 4, 1, lambda s: 1.0, 0.5, lambda s: 2, lambda occ: 3)
    assert lat == pytest.approx([2.5, 4.8])
    assert [r[0] for r in rounds] == pytest.approx([0.5, 1.5, 3.0, 4.0])
    assert all(occ == 1 and s == 3 for _, occ, s in rounds)
    # two slots: the second request joins after the round in progress when it arrived
    # t=0: admit r0 (0.5); round 0.5..1.5 (r0: 2 left); r1 arrived at 0.7 -> admitted 1.5..2.0; round 2.0..3.0
    # finishes r0 (latency 3.0), r1 has 2 left; round 3.0..4.0 finishes r1 (latency 3.3)
    lat, rounds = ts.serve_continuous([0.0, 0.7], 4, 2, lambda s: 1.0, 0.5, lambda s: 2, lambda occ: 0)
    assert lat == pytest.approx([3.0, 3.3])
    assert [occ for _, occ, _ in rounds] == [1, 2, 1]
    # a request that arrives while another is being admitted is admitted right after it, before the first round
    lat, rounds = ts.serve_continuous([0.0, 0.2], 4, 2, lambda s: 1.0, 0.5, lambda s: 2, lambda occ: 0)
    assert lat == pytest.approx([3.0, 2.8])
    assert [occ for _, occ, _ in rounds] == [2, 2]
    # idle gaps: the server waits for the next arrival
    lat, rounds = ts.serve_continuous([0.0, 10.0], 2, 2, lambda s: 1.0, 0.0, lambda s: 2, lambda occ: 0)
    assert lat == pytest.approx([1.0, 1.0])
    lat, rounds = ts.serve_continuous([], 2, 2, lambda s: 1.0, 0.0, lambda s: 2, lambda occ: 0)
    assert len(lat) == 0 and rounds == []


def test_continuous_server_matches_time_stepped_one():
    # every time is a multiple of 1/64 s, so sums of them are exact and "arrived by now" has no rounding to argue about
    rng = np.random.default_rng(11)
    tick = 1.0 / 64
    for trial in range(6):
        arr = np.cumsum(rng.geometric(0.05, size=40)) * tick
        lat, _ = ts.serve_continuous(arr, 6, 3, lambda s: 16 * tick, 4 * tick, lambda s: 2, lambda occ: 2)
        ref = brute_force_continuous(arr, 6, 3, 16 * tick, 4 * tick, 2, tick=tick)
        assert np.array_equal(lat, ref), trial


def test_continuous_server_conservation_and_policy():
    arr = ts.gamma_arrivals(300, 0.2, 2.0, seed=4)
    seen = []

    def policy(occ):
        seen.append(occ)
        return 4 if occ <= 2 else 1
    gains = iter(np.random.default_rng(0).integers(1, 4, size=10 ** 6))
    lat, rounds = ts.serve_continuous(arr, 16, 4, lambda s: 0.05 + 0.01 * s, 0.02, lambda s: int(next(gains)), policy)
    assert (lat > 0).all() and len(lat) == 300
    assert max(seen) <= 4 and min(seen) >= 1
    assert all(s == (4 if occ <= 2 else 1) for _, occ, s in rounds)
    # nobody finishes faster than the rounds it needs at the largest gain
    assert lat.min() >= np.ceil(16 / 3) * 0.05 - 1e-9
