#!/usr/bin/env python3
"""Benchmark of the batched speculative-decoding hot path on one MI355X.

A step is one round of Alg. 1 over one batch: s draft steps, one target verification pass
over B*(s+1) rows, acceptance and commit.  Headline workload: the 7B-shape synthetic configuration
(32 layers, d=4096, bf16 target; 2-layer d=768 draft; prompt 128; proposals = the target's
own greedy continuation with each token replaced by a random one with probability 0.3) at B = 64.
The speculation length is the one the profiling stage (Sec. 4 of the paper) picks for the
batch size.  The 13B OPT shape (fp16, prompt 256) and the 33B shape (bf16, 2048-token prompts) run
afterwards at their headline batch sizes and are reported as extra objects of the same line.
Prints ONE JSON line.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12        # bytes/s, MI355X published
MFMA_BF16_PEAK = 2.5e15  # flop/s dense bf16 / fp16, MI355X published

# prompt length, tokens per sequence in the profiling stage, longest speculation, acceptance probability, headline batch
WORKLOADS = {"llama7b_bf16": (128, 128, 8, 0.7, 64), "opt13b_fp16": (256, 128, 8, 0.8, 64),
             "llama33b_bf16": (2048, 256, 6, 0.6, 32)}
ARITHMETIC = {"bf16": "bf16 storage (weights, KV cache), fp16 MFMA operands, fp32 accumulate",
              "fp16": "fp16 storage and MFMA operands, fp32 accumulate", "fp32": "f32"}


def pmc_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter passes: rows `| class | workload | M | read MB | written MB |`
    of profiles/hbm_traffic_by_kernel.md -> {(workload, class, M): bytes}."""
    out = {}
    path = os.path.join(ROOT, "profiles", "hbm_traffic_by_kernel.md")
    if not os.path.exists(path):
        return out
    for line in open(path):
        m = re.match(r"\|\s*(gemm_\w+|attention)\s*\|\s*(\w+)\s*\|\s*(\d+)\s*\|\s*([\d.]+)\s*\|\s*([\d.]+)\s*\|", line)
        if m:
            out[(m.group(2), m.group(1), int(m.group(3)))] = (float(m.group(4)) + float(m.group(5))) * 1e6
    return out


def gemm_cost(M, N, K, extra_bytes):
    """Algorithmic bytes and flops of one weight-streaming GEMM launch: every weight byte once,
    the activation rows in, the epilogue's output."""
    return 2 * N * K + 2 * M * K + extra_bytes, 2.0 * M * N * K


def class_costs(desc, M, kv_positions, q):
    d, f, V = desc["d_model"], desc["d_ffn"], desc["vocab"]
    kf = 2 if desc["ffn_kind"] == 0 else 1   # SwiGLU streams gate and up, ReLU one matrix
    return {
        "gemm_qkv": gemm_cost(M, 3 * d, d, 2 * M * 3 * d),
        "gemm_o": gemm_cost(M, d, d, 8 * M * d),
        "gemm_ffn_in": gemm_cost(M, kf * f, d, 2 * M * f),
        "gemm_ffn_out": gemm_cost(M, d, f, 8 * M * d),
        "gemm_head": gemm_cost(M, V, d, 8 * M * ((V + 15) // 16)),
        # K and V rows of every attended position once, queries in, output out
        "attention": (2 * 2 * d * kv_positions + 4 * M * d, 4.0 * d * kv_positions * q),
    }


class Workload:
    """One configuration resident on the GPU: weights, context, prompts, the reference continuation (plain greedy
    decoding on the GPU, s = 0, untimed) and the proposal table built from it."""

    def __init__(self, name, B_list, batch, K, W, keep_host_weights=False, N_profile=None):
        import numpy as np
        import torch
        import synth_inputs as si
        from paper_2310_18813_amd import binding as B
        self.np, self.torch, self.si, self.B = np, torch, si, B
        self.name = name
        self.dtype, self.seed, tdesc, ddesc = si.CONFIGS[name]
        self.P, N, self.s_max, self.alpha, _ = WORKLOADS[name]
        self.N = N_profile or N
        self.B_list = B_list
        self.B_max = max(B_list + [batch])
        self.gen_max = max(self.N + self.s_max + 1, (K + W + 4) * (self.s_max + 1))
        self.L_max = self.P + self.gen_max + self.s_max
        self.tdesc, self.ddesc = dict(tdesc, max_pos=self.L_max), dict(ddesc, max_pos=self.L_max)
        t0 = time.time()
        dev = "cuda:0"
        wt = si.make_weights(self.tdesc, self.dtype, self.seed, device=dev, tag="tgt.")
        wd = si.make_weights(self.ddesc, self.dtype, self.seed, device=dev, tag="drf.")
        self.host_w = (si.weights_to_numpy(wt), si.weights_to_numpy(wd)) if keep_host_weights else None
        self.ctx = B.Context(self.tdesc, wt, self.ddesc, wd, self.dtype, self.B_max, self.s_max, self.L_max, self.gen_max,
                             B.PROPOSALS_EXTERNAL, dev)
        del wt, wd
        torch.cuda.empty_cache()
        self.prompts = si.make_prompts(self.B_max, self.P, self.tdesc["vocab"], self.seed)
        self.ctx.spec_reset(self.prompts)
        self.ctx.spec_round(0, self.gen_max)
        self.ref, _ = self.ctx.spec_read_output()
        truth = np.zeros((self.B_max, self.L_max), dtype=np.int32)
        truth[:, self.P:self.P + self.gen_max] = np.array(self.ref, dtype=np.int32)
        self.ctx.spec_set_proposal_table(si.make_proposal_table(truth, self.alpha, self.tdesc["vocab"], self.seed))
        self.setup_s = time.time() - t0

    def close(self):
        self.ctx.close()
        self.ctx = None
        self.torch.cuda.empty_cache()

    def prefill_timed(self, nB, reps=2):
        """The step in front of the timed path (outside `value`): P - 1 prompt tokens of nB sequences through both
        models in row passes of the verification kernels.  Best of reps."""
        ctx, torch = self.ctx, self.torch
        best = None
        for _ in range(reps):
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ctx.spec_reset(self.prompts[:nB])
            torch.cuda.synchronize()
            dt = time.perf_counter() - t0
            best = dt if best is None else min(best, dt)
        n = nB * (self.P - 1)
        return {"ms": round(best * 1e3, 3), "prompt_tokens": n, "tokens_per_s": round(n / best, 1)}

    def run_timed(self, nB, s, rounds, warm):
        ctx, torch = self.ctx, self.torch
        ctx.spec_reset(self.prompts[:nB])
        ctx.spec_round(s, warm)
        out0, _ = ctx.spec_read_output()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        ctx.spec_round(s, rounds)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        out1, hist = ctx.spec_read_output()
        tokens = sum(len(x) for x in out1) - sum(len(x) for x in out0)
        # what was emitted is the greedy continuation, token for token
        for b in range(nB):
            assert out1[b] == self.ref[b][:len(out1[b])], "speculative output differs from plain greedy decoding"
        return tokens, dt, hist

    def kernel_classes(self, nB, s, W, n_rounds=4):
        """Per-kernel-class durations of n_rounds rounds (HIP event pairs on the library's stream around every launch of the
        target's kernels), with the fraction of the HBM and MFMA roofline each class reaches, and the dominant class."""
        ctx = self.ctx
        ctx.spec_reset(self.prompts[:nB])
        ctx.spec_round(s, W)
        ctx.spec_kernel_timing(True)
        ctx.spec_read_kernel_timing()
        ctx.spec_round(s, n_rounds)
        kt = ctx.spec_read_kernel_timing()
        ctx.spec_kernel_timing(False)
        M = nB * (s + 1)
        n_now, _, _, _ = ctx.spec_read_state()
        kv_positions = int(sum(n_now))  # attended cache positions per layer, summed over the batch (end of the timed rounds)
        costs = class_costs(self.tdesc, M, kv_positions, s + 1)
        per_class = {}
        for name, (cnt, ms) in kt.items():
            if cnt:
                per_class[name] = {"launches": cnt, "avg_us": ms * 1000.0 / cnt}
        dom = max((k for k in per_class if k in costs), key=lambda k: per_class[k]["avg_us"] * per_class[k]["launches"])
        dbytes, dflops = costs[dom]
        dur = per_class[dom]["avg_us"] * 1e-6
        if dom != "attention" and dflops / MFMA_BF16_PEAK > dbytes / HBM_PEAK:
            roof = {"bound": "mfma", "achieved": dflops / dur / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s"}
        else:
            roof = {"bound": "hbm", "achieved": dbytes / dur / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
        roof["frac"] = roof["achieved"] / roof["peak"]
        roof["traffic"] = pmc_traffic().get((self.name, dom, M))
        roof["kernel"] = dom
        roof["avg_us"] = per_class[dom]["avg_us"]
        roof["rows_M"] = M
        roof["algorithmic_bytes"] = dbytes
        roof["algorithmic_flops"] = dflops
        for name, (b_, f_) in costs.items():
            if name in per_class:
                t = per_class[name]["avg_us"] * 1e-6
                per_class[name]["hbm_frac"] = b_ / t / HBM_PEAK
                per_class[name]["mfma_frac"] = f_ / t / MFMA_BF16_PEAK if name != "attention" else None
        return per_class, roof


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=0, help="batch size of the headline number (0: the workload's)")
    ap.add_argument("--workload", default="llama7b_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fixed-s", type=int, default=-1, help="skip the profiling stage and use this s everywhere")
    ap.add_argument("--b-list", default="1,2,4,8,16,32,64", help="batch sizes of the profiling stage / curve / grid")
    ap.add_argument("--b-extra", default="3,6,12,24,48", help="batch sizes the profiling stage does not see (look-up rule)")
    ap.add_argument("--no-curve", action="store_true", help="skip the tokens/s-vs-batch curve")
    ap.add_argument("--no-grid", action="store_true", help="skip the verify-step latency grid")
    ap.add_argument("--no-extras", action="store_true", help="skip the 13B and 33B shapes")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2310_18813_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    K, W = args.steps, args.warmup
    nB = args.batch or WORKLOADS[args.workload][4]
    B_list = sorted(int(b) for b in args.b_list.split(","))
    B_list = [b for b in B_list if b <= max(nB, 1)] or [nB]
    if nB not in B_list:
        B_list = sorted(B_list + [nB])
    wl = Workload(args.workload, B_list, nB, K, W, keep_host_weights=not args.no_cpu_baseline)
    ctx = wl.ctx

    # profiling stage -> LUT (batch size -> speculation length)
    if args.fixed_s >= 0:
        lut, grid = [args.fixed_s] * len(B_list), None
        ctx.spec_set_lut(B_list, lut)
    else:
        lut, grid = ctx.spec_profile_and_choose_s(B_list, wl.s_max, wl.prompts, wl.N)

    s_star = ctx.spec_choose_s(nB)
    tokens, dt, hist = wl.run_timed(nB, s_star, K, W)
    value = tokens / dt
    ms_per_step = dt * 1000.0 / K
    per_class, roof = wl.kernel_classes(nB, s_star, W)
    M = nB * (s_star + 1)
    # the same against what a pure load stream and back-to-back MFMA issue reach on this GPU (spec_measure_peaks)
    hbm_meas, mfma_meas = B.spec_measure_peaks("cuda:0", 1 << 30)
    roof["peak_measured"] = hbm_meas if roof["bound"] == "hbm" else mfma_meas
    roof["frac_of_measured"] = roof["achieved"] / roof["peak_measured"]

    # accepted tokens/s against batch size at the adaptive s (short runs, independent of the profiling stage's timings),
    # with the neighbouring speculation lengths beside it; batch sizes the profiling stage never saw get their s from
    # the look-up rule of Sec. 4 (the smaller entry of the two nearest profiled sizes)
    curve = {}
    extra_B = [] if args.no_curve else [int(b) for b in args.b_extra.split(",") if b and int(b) <= wl.B_max]
    for b in ([] if args.no_curve else sorted(set(B_list + extra_B))):
        s_b = ctx.spec_choose_s(b)
        entry = {"s_star": s_b, "profiled": b in B_list}
        by_s = {}
        for s_try in sorted({max(0, s_b - 1), s_b, min(wl.s_max, s_b + 1)}):
            # enough rounds for a few hundred acceptance draws also at small batches, within what gen_max leaves room for
            n_rounds = max(8, min(wl.gen_max // (s_try + 1) - 2, -(-256 // b)))
            tk, tt, hb = wl.run_timed(b, s_try, n_rounds, 1)
            by_s[str(s_try)] = round(tk / tt, 1)
            if s_try == s_b:
                entry["tokens_per_s"] = tk / tt
                entry["mean_accepted"] = round(sum(l * c for l, c in enumerate(hb)) / max(1, sum(hb)), 3)
        entry["tokens_per_s_by_s"] = by_s
        if grid is not None and b in B_list:
            i = B_list.index(b)
            entry["us_per_token_by_s"] = [round(x, 2) for x in grid[i]]
            entry["best_fixed_s"] = int(np.argmin(grid[i]))
            # the table takes the smaller s among those within 1 % of the minimum (timing noise): never worse than this
            entry["s_star_over_best_fixed"] = round(float(grid[i][s_b] / min(grid[i])), 4) if s_b < len(grid[i]) else None
        curve[str(b)] = entry

    vgrid = None if args.no_grid else verify_grid(ctx, torch, wl.prompts, wl.tdesc, wl.P, B_list, wl.s_max)
    model = None if vgrid is None else model_fit_object(ctx, wl.prompts, B_list, vgrid, wl.alpha, lut)

    cpu = None
    if wl.host_w is not None:
        cpu = cpu_baseline(wl)
    config = {"workload": "%s: %d-layer d=%d target + %d-layer d=%d draft, random init, B=%d, prompt %d, "
                          "acceptance prob %.1f, s=adaptive" % (args.workload, wl.tdesc["n_layers"], wl.tdesc["d_model"],
                                                                  wl.ddesc["n_layers"], wl.ddesc["d_model"], nB, wl.P, wl.alpha),
              "batch": nB, "s_star": s_star, "rows_per_verify": M, "accepted_hist": hist,
              "tokens_per_round_per_seq": tokens / K / nB}
    setup_s = round(wl.setup_s, 1)
    dtype = wl.dtype
    prefill = wl.prefill_timed(nB)
    wl.close()
    del wl, ctx

    extras = []
    if not args.no_extras and args.workload == "llama7b_bf16":
        for name in ("opt13b_fp16", "llama33b_bf16"):
            extras.append(extra_workload(name, min(K, 12), W))

    line = {
        "metric": "accepted tokens/s at adaptive s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": ARITHMETIC[dtype], "data": "synthetic",
        "config": config,
        "roofline": roof,
        "measured_peaks": {"hbm_stream_GBs": round(hbm_meas, 1), "mfma_f16_TFLOPs": round(mfma_meas, 1)},
        "cpu_baseline": cpu,
        "kernels": per_class,
        "lut": {str(b): s for b, s in zip(B_list, lut)},
        "curve": curve,
        "verify_grid": vgrid,
        "model": model,
        "prefill": prefill,
        "other_workloads": extras,
        "setup_s": setup_s,
    }
    print(json.dumps(line))


def extra_workload(name, K, W):
    """Headline cell of another configuration: its own profiling stage at the one batch size, K timed rounds at the s it
    picks, per-class kernel timings and the roofline of the dominant class, one verification pass at M = B and M = 1."""
    import torch
    P, N, s_max, alpha, nB = WORKLOADS[name]
    wl = Workload(name, [nB], nB, K, W, N_profile=64)
    lut, grid = wl.ctx.spec_profile_and_choose_s([nB], wl.s_max, wl.prompts, wl.N)
    s_star = lut[0]
    tokens, dt, hist = wl.run_timed(nB, s_star, K, W)
    per_class, roof = wl.kernel_classes(nB, s_star, W, n_rounds=2)
    vg = verify_grid(wl.ctx, torch, wl.prompts, wl.tdesc, wl.P, [1, nB], wl.s_max, s_list=(0, s_star), iters=4)
    out = {"workload": "%s: %d-layer d=%d target + %d-layer d=%d draft, random init, B=%d, prompt %d, acceptance prob %.1f, "
                       "s=adaptive" % (name, wl.tdesc["n_layers"], wl.tdesc["d_model"], wl.ddesc["n_layers"],
                                       wl.ddesc["d_model"], nB, P, alpha),
           "dtype": ARITHMETIC[wl.dtype], "value": tokens / dt, "unit": "tokens/s", "steps": K, "ms_per_step": dt * 1000.0 / K,
           "s_star": s_star, "us_per_token_by_s": [round(x, 2) for x in grid[0]], "accepted_hist": hist,
           "roofline": roof, "kernels": per_class, "verify_grid": vg, "prefill": wl.prefill_timed(nB),
           "setup_s": round(wl.setup_s, 1)}
    wl.close()
    return out


def verify_grid(ctx, torch, prompts, desc, P, B_list, s_max, s_list=(0, 1, 2, 4, 8), iters=8):
    """Latency of one target verification pass (plus the commit) for every (B, s), with the fraction
    of the HBM and of the bf16 MFMA roofline it reaches.  Algorithmic cost per pass: every weight
    byte once, the attended K/V rows once, the appended K/V rows; 2 flops per weight per row plus
    the attention products."""
    d, f, V, nl = desc["d_model"], desc["d_ffn"], desc["vocab"], desc["n_layers"]
    w_layer = 4 * d * d + (3 if desc["ffn_kind"] == 0 else 2) * d * f
    out = {}
    for nB in B_list:
        for s in sorted({min(x, s_max) for x in s_list}):
            M = nB * (s + 1)
            ctx.spec_reset_noprefill(prompts[:nB])      # cache content is whatever earlier runs left: timing only
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            for it in range(2 + iters):
                if it == 2:
                    e0.record()
                ctx.spec_verify_step(s)
                ctx.spec_accept_commit(s)
            e1.record()
            e1.synchronize()
            us = e0.elapsed_time(e1) * 1000.0 / iters
            kv = nB * (P + 2 + iters)                   # attended positions per layer, summed over the batch
            nbytes = 2 * (nl * w_layer + V * d) + nl * (2 * 2 * d * kv + 2 * 2 * d * M)
            flops = 2.0 * M * (nl * w_layer + V * d) + nl * 4.0 * d * kv * (s + 1)
            out["%d,%d" % (nB, s)] = {"us": round(us, 1), "hbm_frac": round(nbytes / HBM_PEAK / (us * 1e-6), 3),
                                      "mfma_frac": round(flops / MFMA_BF16_PEAK / (us * 1e-6), 3)}
    return out


def model_fit_object(ctx, prompts, B_list, vgrid, alpha, lut):
    """The runtime model of Sec. 3.3 fitted to this run: t_L(B, s) ~ alpha_B s + beta (Sec. 3.3.1) from the verify grid,
    one draft step t_S(B, 1) from the draft passes of a few rounds, l(s) from the workload's acceptance probability
    (Eq. 6 under independence) fitted by c s^gamma (Eq. 5); the root of Eq. 11 next to the measured arg-min and
    the profiled table."""
    from paper_2310_18813_amd import model_fit as mf
    s_list = sorted({int(k.split(",")[1]) for k in vgrid})
    t_L = [[vgrid["%d,%d" % (b, s)]["us"] for s in s_list] for b in B_list]
    t_S = []
    for b in B_list:
        ctx.spec_reset_noprefill(prompts[:b])
        ctx.spec_round(2, 1)
        ctx.spec_kernel_timing(True)
        ctx.spec_read_kernel_timing()
        ctx.spec_round(2, 3)
        cnt, ms = ctx.spec_read_kernel_timing()["draft_pass"]
        ctx.spec_kernel_timing(False)
        t_S.append(ms * 1000.0 / max(cnt, 1))
    l_of_s = [mf.l_iid(alpha, s) for s in range(max(s_list) + 1)]
    res = mf.explain(B_list, s_list, t_L, t_S, l_of_s)
    for row, ts, s_lut in zip(res["rows"], t_S, lut):
        row["t_S_us"] = round(ts, 1)
        row["s_lut"] = int(s_lut)
        for k in ("alpha_b", "alpha_b_with_draft", "beta", "s_opt_model"):
            row[k] = round(row[k], 2)
    res["c"], res["gamma"] = round(res["c"], 3), round(res["gamma"], 3)
    return res


def cpu_baseline(wl):
    """The fp32 oracle as it stands, on the host cores, on a bounded sample of the same
    workload: one sequence, an 8-token prompt, 24 tokens at s=4 (about fifteen seconds of CPU work) on the
    same 7B-shape weights, on every thread the box gives this process; then one single-token decode step on one
    thread.  Prefill is timed apart and left out, as on the GPU side."""
    import ctypes
    import numpy as np
    from oracle import oracle as om
    si, ctx = wl.si, wl.ctx
    orc = om.Oracle("f32")
    code = {"fp32": 0, "bf16": 1, "fp16": 2}[wl.dtype]
    ot = orc.model(wl.tdesc, wl.host_w[0], code)
    od = orc.model(wl.ddesc, wl.host_w[1], code)
    P8, s, n_tok = 8, 4, 24
    prompt = si.make_prompts(1, P8, wl.tdesc["vocab"], wl.seed + 1)
    # true continuation of the short prompt from the GPU, so that acceptance looks like the workload's
    ctx.spec_reset(prompt)
    ctx.spec_round(0, n_tok + s + 2)
    cont, _ = ctx.spec_read_output()
    L = P8 + n_tok + s + 4
    truth = np.zeros((1, max(L, ctx.L_max)), dtype=np.int32)
    truth[0, P8:P8 + len(cont[0])] = cont[0]
    table = si.make_proposal_table(truth, 0.7, wl.tdesc["vocab"], wl.seed)[0]
    t0 = time.perf_counter()
    c1, c2 = ot.cache(L), od.cache(L)
    ot.forward(c1, prompt[0][:P8 - 1], 0, want_logits=False)
    od.forward(c2, prompt[0][:P8 - 1], 0, want_logits=False)
    t_prefill = time.perf_counter() - t0
    t0 = time.perf_counter()
    out, ls = ot.spec_generate(od, prompt[0], n_tok, s, proposal_mode=1, prop_table=table, L_max=L)
    t_all = time.perf_counter() - t0
    t_dec = max(t_all - t_prefill, 1e-9)
    cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
    res = {"value": n_tok / t_dec, "unit": "tokens/s", "cores": cores, "kind": "oracle", "nproc": os.cpu_count(),
           "sample": "fp32 oracle, B=1, s=4, %d tokens (%d rounds) after an 8-token prompt, same 7B-shape weights; "
                     "prefill (%.1f s) excluded" % (n_tok, len(ls), t_prefill)}
    # one thread: plain decoding (s = 0), two tokens on the cache the prefill left
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        t0 = time.perf_counter()
        ot.forward(c1, [int(prompt[0][P8 - 1])], P8 - 1)
        t1 = time.perf_counter() - t0
        gomp.omp_set_num_threads(cores)
        res["one_core"] = {"value": 1.0 / t1, "unit": "tokens/s", "cores": 1,
                           "sample": "the same oracle on one thread: one single-token decode step (s = 0), %.1f s" % t1}
    except OSError:
        res["one_core"] = None
    return res


if __name__ == "__main__":
    main()
