"""Host-side pieces of bench.py (no GPU): the algorithmic byte and flop counts that the roofline fractions rest on,
the table of measured HBM traffic it reads, and the refusal to run on more than one GPU."""
import os
import subprocess
import sys

import bench
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_algorithmic_bytes_and_flops_of_the_7b_gate_up():
    desc = si.CONFIGS["llama7b_bf16"][2]
    d, f = desc["d_model"], desc["d_ffn"]
    costs = bench.class_costs(desc, 256, 64 * 200, 4)
    nbytes, flops = costs["gemm_ffn_in"]
    # every weight byte once (gate and up: 2 f x d fp16 values), 256 activation rows in, 256 x f fp16 outputs
    assert nbytes == 2 * 2 * f * d + 2 * 256 * d + 2 * 256 * f == 188088320
    assert flops == 2.0 * 256 * 2 * f * d
    # one row: the weights alone, to within the two small terms
    b1, _ = bench.class_costs(desc, 1, 200, 1)["gemm_ffn_in"]
    assert abs(b1 - 2 * 2 * f * d) <= 2 * d + 2 * f


def test_traffic_table_is_read_and_holds_the_headline_cell():
    t = bench.pmc_traffic()
    key = ("llama7b_bf16", "gemm_ffn_in", 256)
    assert key in t, "profiles/hbm_traffic_by_kernel.md must carry the dominant kernel of the headline cell"
    algorithmic = 188088320
    assert algorithmic <= t[key] <= 1.15 * algorithmic      # measured HBM bytes: at least the algorithmic ones, little above
    assert ("llama33b_bf16", "attention", 128) in t


def test_more_than_one_gpu_is_refused_with_a_message():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in (r.stdout + r.stderr)
