#!/usr/bin/env python3
"""Benchmark of the batched speculative-decoding hot path on one MI355X.

A step is one round of Alg. 1 over one batch: s draft steps, one target verification pass
over B*(s+1) rows, acceptance and commit.  Workload: the 7B-shape synthetic configuration
(32 layers, d=4096, bf16 target; 2-layer d=768 draft; prompt 128; proposals = the target's
own greedy continuation with each token replaced by a random one with probability 0.3).
The speculation length is the one the profiling stage (Sec. 4 of the paper) picks for the
batch size.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12        # bytes/s, MI355X published
MFMA_BF16_PEAK = 2.5e15  # flop/s dense bf16, MI355X published

# HBM bytes per launch from the committed rocprofv3 counter passes (FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00,
# calibrated on a copy of known size in the same run): {(kernel class, rows M): bytes}.  Other cells: null.
PMC_TRAFFIC = {("gemm_ffn_in", 1): 181.0e6 + 0.04e6, ("gemm_ffn_in", 256): 197.4e6 + 5.6e6}


def to_device(w, dev):
    out = {k: (v.to(dev) if v is not None else None) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: (v.to(dev) if v is not None else None) for k, v in L.items()} for L in w["layers"]]
    return out


def gemm_cost(M, N, K, extra_bytes):
    """Algorithmic bytes and flops of one weight-streaming GEMM launch: every weight byte once,
    the activation rows in, the epilogue's output."""
    return 2 * N * K + 2 * M * K + extra_bytes, 2.0 * M * N * K


def class_costs(desc, M, kv_positions, q):
    d, f, V, H = desc["d_model"], desc["d_ffn"], desc["vocab"], desc["n_heads"]
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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=40)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--batch", type=int, default=64, help="batch size of the headline number")
    ap.add_argument("--workload", default="llama7b_bf16")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--fixed-s", type=int, default=-1, help="skip the profiling stage and use this s everywhere")
    ap.add_argument("--b-list", default="1,2,4,8,16,32,64", help="batch sizes of the profiling stage / curve / grid")
    ap.add_argument("--no-curve", action="store_true", help="skip the tokens/s-vs-batch curve")
    ap.add_argument("--no-grid", action="store_true", help="skip the verify-step latency grid")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no cross-GPU part); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth_inputs as si
    from paper_2310_18813_amd import binding as B

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    dtype, seed, tdesc, ddesc = si.CONFIGS[args.workload]
    # prompt length, tokens per sequence in the profiling stage, longest speculation, acceptance probability
    P, N, s_max, alpha = {"llama7b_bf16": (128, 128, 8, 0.7), "opt13b_fp16": (256, 128, 8, 0.8),
                          "llama33b_bf16": (2048, 256, 6, 0.6)}.get(args.workload, (128, 128, 8, 0.7))
    B_list = sorted(int(b) for b in args.b_list.split(","))
    B_max = max(B_list + [args.batch])
    K, W = args.steps, args.warmup
    gen_max = max(N + s_max + 1, (K + W + 4) * (s_max + 1))
    L_max = P + gen_max + s_max
    tdesc = dict(tdesc, max_pos=L_max)
    ddesc = dict(ddesc, max_pos=L_max)

    t_setup = time.time()
    wt = si.make_weights(tdesc, dtype, seed, device=dev, tag="tgt.")
    wd = si.make_weights(ddesc, dtype, seed, device=dev, tag="drf.")
    host_w = None
    if not args.no_cpu_baseline:
        host_w = (si.weights_to_numpy(wt), si.weights_to_numpy(wd))
    ctx = B.Context(tdesc, wt, ddesc, wd, dtype, B_max, s_max, L_max, gen_max, B.PROPOSALS_EXTERNAL, dev)
    del wt, wd
    torch.cuda.empty_cache()
    prompts = si.make_prompts(B_max, P, tdesc["vocab"], seed)

    # reference continuation: plain greedy decoding on the GPU (s = 0), untimed
    ctx.spec_reset(prompts)
    ctx.spec_round(0, gen_max)
    ref, _ = ctx.spec_read_output()
    truth = np.zeros((B_max, L_max), dtype=np.int32)
    truth[:, P:P + gen_max] = np.array(ref, dtype=np.int32)
    table = si.make_proposal_table(truth, alpha, tdesc["vocab"], seed)
    ctx.spec_set_proposal_table(table)
    t_setup = time.time() - t_setup

    # profiling stage -> LUT (batch size -> speculation length)
    if args.fixed_s >= 0:
        lut, grid = [args.fixed_s] * len(B_list), None
        ctx.spec_set_lut(B_list, lut)
    else:
        lut, grid = ctx.spec_profile_and_choose_s(B_list, s_max, prompts, N)

    def run_timed(nB, s, rounds, warm):
        ctx.spec_reset(prompts[:nB])
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
            assert out1[b] == ref[b][:len(out1[b])], "speculative output differs from plain greedy decoding"
        return tokens, dt, hist

    nB = args.batch
    s_star = ctx.spec_choose_s(nB)
    tokens, dt, hist = run_timed(nB, s_star, K, W)
    value = tokens / dt
    ms_per_step = dt * 1000.0 / K

    # per-kernel durations of the same rounds, HIP events around every launch of the target's kernels
    ctx.spec_reset(prompts[:nB])
    ctx.spec_round(s_star, W)
    ctx.spec_kernel_timing(True)
    ctx.spec_read_kernel_timing()
    n_t = 4
    ctx.spec_round(s_star, n_t)
    kt = ctx.spec_read_kernel_timing()
    ctx.spec_kernel_timing(False)
    M = nB * (s_star + 1)
    n_now, _, _, _ = ctx.spec_read_state()
    kv_positions = int(sum(n_now))  # attended cache positions per layer, summed over the batch (end of the timed rounds)
    costs = class_costs(tdesc, M, kv_positions, s_star + 1)
    per_class = {}
    for name, (cnt, ms) in kt.items():
        if cnt:
            per_class[name] = {"launches": cnt, "avg_us": ms * 1000.0 / cnt}
    dom = max((k for k in per_class if k in costs), key=lambda k: per_class[k]["avg_us"] * per_class[k]["launches"])
    dbytes, dflops = costs[dom]
    dur = per_class[dom]["avg_us"] * 1e-6
    if dflops / MFMA_BF16_PEAK > dbytes / HBM_PEAK:
        roof = {"bound": "mfma", "achieved": dflops / dur / 1e12, "peak": MFMA_BF16_PEAK / 1e12, "unit": "TFLOP/s"}
    else:
        roof = {"bound": "hbm", "achieved": dbytes / dur / 1e9, "peak": HBM_PEAK / 1e9, "unit": "GB/s"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    # the same against what a pure load stream and back-to-back MFMA issue reach on this GPU (spec_measure_peaks)
    hbm_meas, mfma_meas = B.spec_measure_peaks("cuda:0", 1 << 30)
    roof["peak_measured"] = hbm_meas if roof["bound"] == "hbm" else mfma_meas
    roof["frac_of_measured"] = roof["achieved"] / roof["peak_measured"]
    roof["traffic"] = PMC_TRAFFIC.get((dom, M))
    roof["kernel"] = dom
    roof["avg_us"] = per_class[dom]["avg_us"]
    roof["rows_M"] = M
    for name, (b_, f_) in costs.items():
        if name in per_class:
            t = per_class[name]["avg_us"] * 1e-6
            per_class[name]["hbm_frac"] = b_ / t / HBM_PEAK
            per_class[name]["mfma_frac"] = f_ / t / MFMA_BF16_PEAK if name != "attention" else None

    # accepted tokens/s against batch size at the adaptive s (short runs)
    curve = {}
    for i, b in enumerate([] if args.no_curve else B_list):
        s_b = ctx.spec_choose_s(b)
        # enough rounds for a few hundred acceptance draws also at small batches, within what gen_max leaves room for
        n_rounds = max(8, min(gen_max // (s_b + 1) - 2, -(-256 // b)))
        tk, tt, hb = run_timed(b, s_b, n_rounds, 1)
        entry = {"s_star": s_b, "tokens_per_s": tk / tt,
                 "mean_accepted": round(sum(l * c for l, c in enumerate(hb)) / max(1, sum(hb)), 3)}
        if grid is not None:
            entry["us_per_token_by_s"] = [round(x, 2) for x in grid[i]]
            entry["best_fixed_s"] = int(np.argmin(grid[i]))
            # the table takes the smaller s among those within 1 % of the minimum (timing noise): never worse than this
            entry["s_star_over_best_fixed"] = round(float(grid[i][s_b] / min(grid[i])), 4) if s_b < len(grid[i]) else None
        curve[str(b)] = entry

    vgrid = None if args.no_grid else verify_grid(ctx, torch, prompts, tdesc, P, B_list)
    model = None if vgrid is None else model_fit_object(ctx, prompts, B_list, vgrid, alpha, lut)

    cpu = None
    if host_w is not None:
        cpu = cpu_baseline(si, tdesc, ddesc, host_w, ctx, dtype, seed)

    line = {
        "metric": "accepted tokens/s at adaptive s", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": K, "warmup": W, "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: %d-layer d=%d target + %d-layer d=%d draft, random init, B=%d, prompt %d, "
                               "acceptance prob %.1f, s=adaptive" % (args.workload, tdesc["n_layers"], tdesc["d_model"],
                                                                       ddesc["n_layers"], ddesc["d_model"], nB, P, alpha),
                   "batch": nB, "s_star": s_star, "rows_per_verify": M, "accepted_hist": hist,
                   "tokens_per_round_per_seq": tokens / K / nB},
        "roofline": roof,
        "measured_peaks": {"hbm_stream_GBs": round(hbm_meas, 1), "mfma_f16_TFLOPs": round(mfma_meas, 1)},
        "cpu_baseline": cpu,
        "kernels": per_class,
        "lut": {str(b): s for b, s in zip(B_list, lut)},
        "curve": curve,
        "verify_grid": vgrid,
        "model": model,
        "setup_s": round(t_setup, 1),
    }
    print(json.dumps(line))


def verify_grid(ctx, torch, prompts, desc, P, B_list, s_list=(0, 1, 2, 4, 8), iters=8):
    """Latency of one target verification pass (plus the commit) for every (B, s), with the fraction
    of the HBM and of the bf16 MFMA roofline it reaches.  Algorithmic cost per pass: every weight
    byte once, the attended K/V rows once, the appended K/V rows; 2 flops per weight per row plus
    the attention products."""
    d, f, V, nl = desc["d_model"], desc["d_ffn"], desc["vocab"], desc["n_layers"]
    w_layer = 4 * d * d + (3 if desc["ffn_kind"] == 0 else 2) * d * f
    out = {}
    for nB in B_list:
        for s in [x for x in s_list if x <= ctx.s_max]:
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
    """The runtime model of Sec. 3.2 fitted to this run: t_L(B, s) ~ alpha_B s + beta from the verify grid, one
    draft step t_S(B, 1) from the draft passes of a few rounds, l(s) from the workload's acceptance probability
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


def cpu_baseline(si, tdesc, ddesc, host_w, ctx, dtype, seed):
    """The fp32 oracle as it stands, on the host cores, on a bounded sample of the same
    workload: one sequence, an 8-token prompt, 24 tokens at s=4 (about fifteen seconds of CPU work) on the
    same 7B-shape weights.  Prefill is timed apart and left out, as on the GPU side."""
    import numpy as np
    from oracle import oracle as om
    orc = om.Oracle("f32")
    code = {"fp32": 0, "bf16": 1, "fp16": 2}[dtype]
    ot = orc.model(tdesc, host_w[0], code)
    od = orc.model(ddesc, host_w[1], code)
    P8, s, n_tok = 8, 4, 24
    prompt = si.make_prompts(1, P8, tdesc["vocab"], seed + 1)
    # true continuation of the short prompt from the GPU, so that acceptance looks like the workload's
    ctx.spec_reset(prompt)
    ctx.spec_round(0, n_tok + s + 2)
    cont, _ = ctx.spec_read_output()
    L = P8 + n_tok + s + 4
    truth = np.zeros((1, max(L, ctx.L_max)), dtype=np.int32)
    truth[0, P8:P8 + len(cont[0])] = cont[0]
    table = si.make_proposal_table(truth, 0.7, tdesc["vocab"], seed)[0]
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
    return {"value": n_tok / t_dec, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "fp32 oracle, B=1, s=4, %d tokens (%d rounds) after an 8-token prompt, same 7B-shape weights; "
                      "prefill (%.1f s) excluded" % (n_tok, len(ls), t_prefill)}


if __name__ == "__main__":
    main()
