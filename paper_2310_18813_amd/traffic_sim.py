#!/usr/bin/env python3
"""Serving under time-varying traffic (Sec. 5.3 of the paper): a client that sends requests at Gamma-distributed
intervals, a server that merges whatever waits in its queue into one batch (at most `max_batch` requests) and
decodes it with batched speculative decoding, four policies for the speculation length (none, fixed 2, fixed 4,
adaptive = the profiled look-up table).  Latency of a request = finish time of its batch - its arrival time, so
waiting in the queue counts.  Beside the paper's server a continuous-batching one (`serve_continuous`, on
spec_admit): requests join the running batch between rounds and leave when they are done.

The queue is simulated on the host on a virtual clock; the service time of a batch of B requests at speculation
length s is what the library needs on the GPU to generate N tokens for B synthetic prompts (measured once per
(B, s) by `measure_service_table`, through the C ABI).  Run as a program it measures the table on the 7B-shape
workload and prints one JSON line per traffic setting:

    python -m paper_2310_18813_amd.traffic_sim --requests 1000

The paper's intervals (0.1 .. 0.8 s) belong to its GPU and models; here the intervals are given in units of the
measured service time of a single request without speculation (`--intervals`, default 0.25 .. 2.0), which keeps
the load of the server in the same range.
"""
import argparse
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def gamma_arrivals(n, mean_interval, cv, seed):
    """Arrival times of n requests whose gaps are Gamma distributed with the given mean and coefficient of
    variation (shape 1/cv^2, scale mean*cv^2); the first request arrives after the first gap."""
    if n < 0 or mean_interval <= 0 or cv <= 0:
        raise ValueError("n >= 0, mean_interval > 0, cv > 0")
    rng = np.random.default_rng(seed)
    gaps = rng.gamma(shape=1.0 / (cv * cv), scale=mean_interval * cv * cv, size=n)
    return np.cumsum(gaps)


def alternating_arrivals(duration, intervals, period, cv, seed):
    """The timeline experiment: the mean interval switches through `intervals` every `period` seconds."""
    rng = np.random.default_rng(seed)
    t, out = 0.0, []
    while True:
        mean = intervals[int(t // period) % len(intervals)]
        t += rng.gamma(shape=1.0 / (cv * cv), scale=mean * cv * cv)
        if t >= duration:
            return np.array(out)
        out.append(t)


def serve(arrivals, service_time, choose_s, max_batch=16):
    """First-come-first-served batch server.  Whenever it is free and requests wait, it takes the oldest
    min(waiting, max_batch) of them as one batch of size B, asks choose_s(B) for the speculation length and is busy
    for service_time(B, s).  Returns (latencies per request, list of (start, B, s) per batch)."""
    arrivals = np.asarray(arrivals, dtype=np.float64)
    n = len(arrivals)
    lat = np.zeros(n)
    batches = []
    t, i = 0.0, 0
    while i < n:
        if arrivals[i] > t:
            t = arrivals[i]            # idle until the next request
        j = i
        while j < n and j - i < max_batch and arrivals[j] <= t:
            j += 1
        B = j - i
        s = int(choose_s(B))
        done = t + float(service_time(B, s))
        lat[i:j] = done - arrivals[i:j]
        batches.append((t, B, s))
        t, i = done, j
    return lat, batches


def serve_continuous(arrivals, n_tokens, slots, round_time, admit_time, tokens_per_round, choose_s):
    """Continuous batching (beyond the paper's server, which decodes whole batches): the server owns `slots`
    sequence slots and decodes them round after round; a request that waits takes a free slot as soon as the
    current round ends (spec_admit: the server is busy for admit_time per admission, one after the other), and
    leaves when its n_tokens are out.  A round with speculation length s = choose_s(occupied) lasts
    round_time(s) whatever the number of occupied slots (the pass always has slots * (s + 1) rows) and gives
    every occupied slot tokens_per_round(s) tokens (a callable: 1 + the accepted length of that sequence's
    round).  Returns (latencies per request, list of (start, occupied, s) per round)."""
    arrivals = np.asarray(arrivals, dtype=np.float64)
    n = len(arrivals)
    lat = np.zeros(n)
    left = [0] * slots      # tokens still owed to the request in the slot
    who = [-1] * slots      # request index, -1 = free
    rounds = []
    t, nxt, done = 0.0, 0, 0
    while done < n:
        for k in range(slots):  # admissions, oldest request first
            if who[k] < 0 and nxt < n and arrivals[nxt] <= t:
                who[k], left[k] = nxt, int(n_tokens)
                nxt += 1
                t += float(admit_time)
        occupied = sum(1 for w in who if w >= 0)
        if occupied == 0:
            t = max(t, arrivals[nxt])  # idle until the next request
            continue
        s = int(choose_s(occupied))
        rounds.append((t, occupied, s))
        t += float(round_time(s))
        for k in range(slots):
            if who[k] >= 0:
                left[k] -= int(tokens_per_round(s))
                if left[k] <= 0:
                    lat[who[k]] = t - arrivals[who[k]]
                    who[k] = -1
                    done += 1
    return lat, rounds


def lut_policy(profiled_B, lut):
    """The look-up of Sec. 4: exact hit, else the smaller entry of the two nearest profiled sizes; ends clamp."""
    pb, lt = list(profiled_B), list(lut)

    def choose(B):
        if B <= pb[0]:
            return lt[0]
        if B >= pb[-1]:
            return lt[-1]
        hi = next(k for k, b in enumerate(pb) if b >= B)
        return lt[hi] if pb[hi] == B else min(lt[hi - 1], lt[hi])
    return choose


def measure_service_table(ctx, prompts, n_tokens, batch_sizes, s_values, check_every=4):
    """Seconds the library needs to emit n_tokens for each of B sequences at speculation length s, for every
    (B, s): reset (with prefill), rounds until every sequence is done.  Needs a proposal source in the context."""
    import time
    import torch
    table = {}
    for B in batch_sizes:
        for s in s_values:
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.spec_reset(prompts[:B])
            P = prompts.shape[1]
            while True:
                ctx.spec_round(s, check_every)
                n, _, _, _ = ctx.spec_read_state()        # synchronises
                if min(n) - P >= n_tokens:
                    break
            table[(B, s)] = time.perf_counter() - t0
    return table


def measure_continuous(ctx, prompts, n_tokens, s_values, n_admit=4):
    """What the continuous-batching server needs, measured through the C ABI with all slots of the batch busy:
    seconds per round and the distribution of tokens per round and sequence (1 + accepted length) for every s,
    and the seconds one spec_admit takes."""
    import time
    import torch
    B = prompts.shape[0]
    round_s, gain = {}, {}
    for s in s_values:
        rounds = max(1, n_tokens // (s + 1))   # nobody can finish within these
        ctx.spec_reset(prompts)
        ctx.spec_round(s, 1)
        ctx.spec_rewind()
        ctx.spec_read_state()
        t0 = time.perf_counter()
        ctx.spec_round(s, rounds)
        ctx.spec_read_state()                  # synchronises
        round_s[s] = (time.perf_counter() - t0) / rounds
        _, hist = ctx.spec_read_output()
        h = np.array(hist[:s + 1], dtype=np.float64)
        gain[s] = (np.arange(1, s + 2), h / h.sum())
    ctx.spec_reset(prompts)
    ctx.spec_round(0, 1)
    ctx.spec_read_state()
    t0 = time.perf_counter()
    for i in range(n_admit):
        ctx.spec_admit(i % B, prompts[(i + 1) % B])
    ctx.spec_read_state()
    torch.cuda.synchronize()
    admit_s = (time.perf_counter() - t0) / n_admit
    return round_s, gain, admit_s


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--requests", type=int, default=1000)
    ap.add_argument("--tokens", type=int, default=128)
    ap.add_argument("--prompt", type=int, default=128)
    ap.add_argument("--max-batch", type=int, default=16)
    ap.add_argument("--cvs", default="0.5,1,2,5")
    ap.add_argument("--intervals", default="0.25,0.5,0.75,1.0,1.25,1.5,1.75,2.0",
                    help="mean request interval in units of the service time of one request at s = 0")
    ap.add_argument("--workload", default="llama7b_bf16")
    args = ap.parse_args()

    import torch
    import synth_inputs as si
    from paper_2310_18813_amd import binding as B

    dtype, seed, tdesc, ddesc = si.CONFIGS[args.workload]
    P, N, s_max, alpha, mb = args.prompt, args.tokens, 8, 0.7, args.max_batch
    L_max = P + N + s_max
    tdesc, ddesc = dict(tdesc, max_pos=L_max), dict(ddesc, max_pos=L_max)
    wt = si.make_weights(tdesc, dtype, seed, device="cuda:0", tag="tgt.")
    wd = si.make_weights(ddesc, dtype, seed, device="cuda:0", tag="drf.")
    ctx = B.Context(tdesc, wt, ddesc, wd, dtype, mb, s_max, L_max, N, B.PROPOSALS_EXTERNAL, "cuda:0")
    del wt, wd
    prompts = si.make_prompts(mb, P, tdesc["vocab"], seed)
    # proposals as in the benchmark: the target's own greedy continuation, each token replaced with probability 1 - alpha
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    ref, _ = ctx.spec_read_output()
    truth = np.zeros((mb, L_max), dtype=np.int32)
    for b in range(mb):
        truth[b, P:P + N] = ref[b]
    ctx.spec_set_proposal_table(si.make_proposal_table(truth, alpha, tdesc["vocab"], seed + 1))
    prof_B = [b for b in (1, 2, 4, 8, 16, 32, 64) if b <= mb]
    lut, _ = ctx.spec_profile_and_choose_s(prof_B, s_max, prompts, N)
    adaptive = lut_policy(prof_B, lut)
    s_needed = sorted({0, 2, 4} | {adaptive(b) for b in range(1, mb + 1)})
    table = measure_service_table(ctx, prompts, N, range(1, mb + 1), s_needed)
    unit = table[(1, 0)]
    policies = {"s=0": lambda b: 0, "s=2": lambda b: 2, "s=4": lambda b: 4, "adaptive": adaptive}
    print(json.dumps({"lut": {str(b): int(s) for b, s in zip(prof_B, lut)}, "unit_s": round(unit, 4),
                      "service_s": {"%d,%d" % k: round(v, 4) for k, v in sorted(table.items())}}), flush=True)
    for cv in [float(x) for x in args.cvs.split(",")]:
        for rel in [float(x) for x in args.intervals.split(",")]:
            arr = gamma_arrivals(args.requests, rel * unit, cv, seed=int(1000 * cv) + int(100 * rel))
            row = {"cv": cv, "interval_units": rel, "interval_s": round(rel * unit, 4)}
            for name, pol in policies.items():
                lat, batches = serve(arr, lambda b, s: table[(b, s)], pol, mb)
                row[name] = {"mean_latency_s": round(float(lat.mean()), 4),
                             "mean_batch": round(float(np.mean([b for _, b, _ in batches])), 2)}
            row["adaptive_vs_s0"] = round(row["s=0"]["mean_latency_s"] / row["adaptive"]["mean_latency_s"], 3)
            row["adaptive_vs_best_fixed"] = round(min(row["s=2"]["mean_latency_s"], row["s=4"]["mean_latency_s"]) /
                                                  row["adaptive"]["mean_latency_s"], 3)
            print(json.dumps(row), flush=True)
    # continuous batching on the same arrivals: all slots decode every round, waiting requests take free slots
    round_s, gain, admit_s = measure_continuous(ctx, prompts, N, sorted({0, 2, 4, adaptive(mb)}))
    print(json.dumps({"continuous": {"slots": mb, "admit_s": round(admit_s, 4),
                                     "round_s": {str(k): round(v, 5) for k, v in round_s.items()},
                                     "mean_tokens_per_round": {str(k): round(float((g[0] * g[1]).sum()), 3)
                                                               for k, g in gain.items()}}}), flush=True)
    cont = {"s=0": 0, "s=2": 2, "s=4": 4, "adaptive": adaptive(mb)}
    for cv in [float(x) for x in args.cvs.split(",")]:
        for rel in [float(x) for x in args.intervals.split(",")]:
            arr = gamma_arrivals(args.requests, rel * unit, cv, seed=int(1000 * cv) + int(100 * rel))
            row = {"cv": cv, "interval_units": rel, "server": "continuous"}
            for name, sv in cont.items():
                draws = iter(np.random.default_rng(17).choice(gain[sv][0], p=gain[sv][1], size=args.requests * N + 64))
                lat, _ = serve_continuous(arr, N, mb, lambda s_: round_s[s_], admit_s,
                                          lambda s_: next(draws), lambda occ, sv=sv: sv)
                row[name] = round(float(lat.mean()), 4)
            lat_static, _ = serve(arr, lambda b, s_: table[(b, s_)], adaptive, mb)
            row["static_adaptive"] = round(float(lat_static.mean()), 4)
            row["continuous_vs_static"] = round(row["static_adaptive"] / row["adaptive"], 3)
            print(json.dumps(row), flush=True)
    # timeline: intense and sparse traffic alternate every 50 mean-service units, CV = 1
    arr = alternating_arrivals(300 * unit * 5, [0.4 * unit, 2.0 * unit], 50 * unit * 5, 1.0, seed=7)
    row = {"timeline_requests": int(len(arr))}
    for name, pol in policies.items():
        lat, _ = serve(arr, lambda b, s: table[(b, s)], pol, mb)
        row[name] = round(float(lat.mean()), 4)
    print(json.dumps(row), flush=True)
    ctx.close()


if __name__ == "__main__":
    main()
