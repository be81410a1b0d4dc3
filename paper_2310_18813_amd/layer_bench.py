#!/usr/bin/env python3
"""Verify-step micro-benchmark on LLaMA-7B-shape layers (d=4096, 32 heads x 128, SwiGLU 11008,
LM head 32000, bf16; 512 cached positions per sequence; --shape picks the 13B OPT or the 33B width instead): latency of one target verification
pass for chosen (B, s) cells, per kernel class, against the HBM / MFMA roofline.

The layer stack holds `--layers` distinct weight copies (default 4 = 1.6 GB, far beyond the
256 MB memory-side cache), so every pass streams its weights from HBM as the full model does.

    python -m paper_2310_18813_amd.layer_bench --cells "1,0;8,3;64,3" --iters 20

Few kernel launches per run: this is also the program the rocprofv3 counter passes use.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK, MFMA_PEAK = 8.0e12, 2.5e15


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cells", default="1,0;1,8;8,3;16,3;64,0;64,3;64,8")
    ap.add_argument("--iters", type=int, default=20)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--kv", type=int, default=512)
    ap.add_argument("--shape", default="7b", choices=["7b", "13b", "33b"], help="layer width: 7b d=4096 (bf16), 13b OPT d=5120 (fp16), 33b d=6656 (bf16)")
    ap.add_argument("--tune", default="0,0,0", help="spec_set_gemm_tuning arguments: tile_mtw,tile_nbw,flags")
    ap.add_argument("--attn-shape", type=int, default=0)
    ap.add_argument("--samples", type=int, default=0, help="also time this many single passes, one by one: median, p10, p90")
    args = ap.parse_args()

    import numpy as np
    import torch
    import synth_inputs as si
    from paper_2310_18813_amd import binding as B

    cells = [tuple(int(x) for x in c.split(",")) for c in args.cells.split(";")]
    dtype, seed, desc, _ = si.CONFIGS["layer_bf16"]
    if args.shape == "13b":
        dtype, seed, desc = "fp16", 1003, si.opt_desc(1, 5120, 40, 20480, 50272, 1024)
    elif args.shape == "33b":
        dtype, seed, desc = "bf16", 1004, si.llama_desc(1, 6656, 52, 17920, 32000, 4096)
    B_max, s_max = max(c[0] for c in cells), max(c[1] for c in cells)
    L_max = args.kv + 1 + (max(args.iters, args.samples) + 4) * (s_max + 1) + s_max
    desc = dict(desc, n_layers=args.layers, max_pos=L_max)
    w = si.make_weights(desc, dtype, seed, device="cuda:0", emb_std=1.0, tag="tgt.")
    ctx = B.Context(desc, w, None, None, dtype, B_max, s_max, L_max, L_max - args.kv - 1 - s_max,
                    B.PROPOSALS_EXTERNAL)
    del w
    K, V = si.make_kv(B_max, desc["d_model"], args.kv, dtype, seed, "cuda:0")
    for layer in range(args.layers):
        ctx.spec_kv_import(B.MODEL_TARGET, layer, K, V)
    prompts = si.make_prompts(B_max, args.kv + 1, desc["vocab"], seed)
    ctx.spec_set_proposal_table(np.zeros((B_max, L_max), dtype=np.int32))
    ctx.spec_set_gemm_tuning(*[int(x) for x in args.tune.split(",")])
    ctx.spec_set_attention_shape(args.attn_shape)
    d, f, Vv, nl = desc["d_model"], desc["d_ffn"], desc["vocab"], args.layers
    w_layer = 4 * d * d + (3 if desc["ffn_kind"] == 0 else 2) * d * f
    out = []
    for nB, s in cells:
        M = nB * (s + 1)
        ctx.spec_reset_noprefill(prompts[:nB])
        ctx.spec_round(s, 2)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        ctx.spec_round(s, args.iters)
        e1.record()
        e1.synchronize()
        us = e0.elapsed_time(e1) * 1000.0 / args.iters
        spread = None
        if args.samples > 0:
            # one event pair per pass (each pair adds its own few microseconds): the run-to-run spread of a pass
            ctx.spec_reset_noprefill(prompts[:nB])
            ctx.spec_round(s, 2)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.samples + 1)]
            ev[0].record()
            for i in range(args.samples):
                ctx.spec_round(s, 1)
                ev[i + 1].record()
            ev[-1].synchronize()
            t = np.sort(np.array([ev[i].elapsed_time(ev[i + 1]) * 1000.0 for i in range(args.samples)]))
            spread = {"samples": args.samples, "median_us": round(float(np.median(t)), 1),
                      "p10_us": round(float(np.percentile(t, 10)), 1), "p90_us": round(float(np.percentile(t, 90)), 1)}
            ctx.spec_reset_noprefill(prompts[:nB])
            ctx.spec_round(s, 2 + args.iters)
        ctx.spec_kernel_timing(True)
        ctx.spec_read_kernel_timing()
        ctx.spec_round(s, 2)
        kt = ctx.spec_read_kernel_timing()
        ctx.spec_kernel_timing(False)
        kv = nB * (args.kv + 2 + args.iters // 2)
        nbytes = 2 * (nl * w_layer + Vv * d) + nl * (2 * 2 * d * kv + 2 * 2 * d * M)
        flops = 2.0 * M * (nl * w_layer + Vv * d) + nl * 4.0 * d * kv * (s + 1)
        out.append({"B": nB, "s": s, "M": M, "us_per_pass": round(us, 1),
                    "us_per_layer": round((us - kt["gemm_head"][1] * 1000 / max(1, kt["gemm_head"][0])) / nl, 1),
                    "hbm_frac": round(nbytes / HBM_PEAK / (us * 1e-6), 3),
                    "mfma_frac": round(flops / MFMA_PEAK / (us * 1e-6), 3),
                    "kernels_us": {k: round(v[1] * 1000 / v[0], 1) for k, v in kt.items() if v[0]}})
        if spread:
            out[-1]["pass_spread"] = spread
        print(json.dumps(out[-1]), flush=True)


if __name__ == "__main__":
    main()
