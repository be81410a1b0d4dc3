"""GPU parity tests of the whole round (draft steps -> verify -> accept/commit) against
the CPU oracle, through the C ABI.  Small models so the oracle finishes in seconds; they
still span several GEMM tiles, a ragged vocabulary and ragged acceptance across a batch."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import LOGIT_TOL, build_pair, top2_margin, truth_table

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

CASES = {
    # the smallest named configuration: fp32 pair, B=1, s=4, P=16, N=32, replacement probability 0.3
    "tiny_fp32": dict(dtype="fp32", seed=1000, B=1, P=16, N=32, s=4, alpha=0.7,
                      tgt=si.CONFIGS["tiny_fp32"][2], drf=si.CONFIGS["tiny_fp32"][3]),
    # bf16 LLaMA shape, head_dim 64 and 128 mixed between target and draft, ragged vocab
    "small_bf16": dict(dtype="bf16", seed=77, B=3, P=9, N=20, s=3, alpha=0.7,
                       tgt=si.llama_desc(2, 256, 2, 416, 1000, 128), drf=si.llama_desc(1, 128, 2, 160, 1000, 128)),
    # fp16 OPT shape: LayerNorm, biases, ReLU, learned positions
    "small_fp16_opt": dict(dtype="fp16", seed=78, B=2, P=5, N=18, s=5, alpha=0.6,
                           tgt=si.opt_desc(2, 256, 4, 384, 777, 64), drf=si.opt_desc(1, 128, 2, 192, 777, 64)),
    # fp16 LLaMA shape: the RMS norm folded into fp16 weights (gain * weight needs the per-matrix scaling too)
    "small_fp16_llama": dict(dtype="fp16", seed=81, B=2, P=7, N=16, s=4, alpha=0.7,
                             tgt=si.llama_desc(2, 256, 4, 448, 900, 64), drf=si.llama_desc(1, 128, 2, 160, 900, 64)),
    # widths whose k dimension splits into two slices (d = 192: 6 steps of 32) and into one (f = 352: 11 steps),
    # three heads, a single-head draft
    "odd_slices_bf16": dict(dtype="bf16", seed=83, B=2, P=6, N=14, s=3, alpha=0.7,
                            tgt=si.llama_desc(2, 192, 3, 352, 500, 64), drf=si.llama_desc(1, 64, 1, 96, 500, 64)),
    # wider bf16 model: 8 k-slices, two row passes (M = 96), two strips per workgroup in the LM head
    "medium_bf16": dict(dtype="bf16", seed=79, B=24, P=12, N=12, s=3, alpha=0.7,
                        tgt=si.llama_desc(1, 512, 4, 1536, 20000, 64), drf=si.llama_desc(1, 256, 4, 512, 20000, 64)),
    # mixed shapes, for the LayerNorm folded into the GEMMs: LayerNorm in front of a bias-free QKV and a gate/up pair
    # (the fold has to bring its own bias arrays and the row sums of the interleaved gate/up rows), with rotary positions
    "ln_swiglu_nobias_fp16": dict(dtype="fp16", seed=84, B=3, P=6, N=14, s=3, alpha=0.7,
                                  tgt=dict(si.llama_desc(2, 256, 4, 448, 900, 64), norm_kind=si.NORM_LAYER),
                                  drf=dict(si.llama_desc(1, 128, 2, 160, 900, 64), norm_kind=si.NORM_LAYER)),
    # ... and with attention biases but none in the feed-forward block, bf16
    "ln_swiglu_bias_bf16": dict(dtype="bf16", seed=85, B=2, P=7, N=12, s=4, alpha=0.7,
                                tgt=dict(si.llama_desc(2, 256, 2, 416, 700, 64), norm_kind=si.NORM_LAYER, has_bias=1),
                                drf=dict(si.llama_desc(1, 128, 2, 160, 700, 64), norm_kind=si.NORM_LAYER, has_bias=1)),
    # context spanning five attention chunks (four of 128 keys, one of 256), ragged against the chunk boundary
    "longctx_bf16": dict(dtype="bf16", seed=80, B=2, P=530, N=12, s=4, alpha=0.8,
                         tgt=si.llama_desc(2, 256, 2, 416, 300, 600), drf=si.llama_desc(1, 128, 2, 160, 300, 600)),
}


@pytest.fixture(scope="module")
def orc():
    from oracle import oracle as om
    return om.Oracle("f64")


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


def setup_case(orc, B, name, proposal_mode=None, s_max=None, B_max=None, random_norms=True):
    c = CASES[name]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV, random_norms=random_norms)
    s_max = c["s"] if s_max is None else s_max
    L_max = c["P"] + c["N"] + s_max + 3
    mode = B.PROPOSALS_EXTERNAL if proposal_mode is None else proposal_mode
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], B_max or c["B"], s_max, L_max, c["N"], mode, DEV)
    prompts = si.make_prompts(c["B"], c["P"], c["tgt"]["vocab"], c["seed"])
    return c, ot, od, ctx, prompts, L_max


def oracle_refs(ot, prompts, n):
    return np.stack([ot.greedy(p, n) for p in prompts])


@pytest.mark.parametrize("name", list(CASES))
def test_teacher_forced_logits_and_commit(orc, B, name):
    """Round by round: the oracle is fed exactly the tokens the GPU verified, logits are
    compared element by element, greedy tokens wherever the oracle's top-2 margin exceeds
    the tolerance, and the commit arithmetic (l, emitted tokens, lengths) bit-exactly."""
    c, ot, od, ctx, prompts, L_max = setup_case(orc, B, name)
    tol = LOGIT_TOL[c["dtype"]]
    nB, P, N, s = c["B"], c["P"], c["N"], c["s"]
    ref = oracle_refs(ot, prompts, N + s + 2)
    table = si.make_proposal_table(truth_table(ref, P, L_max), c["alpha"], c["tgt"]["vocab"], c["seed"])
    ctx.spec_set_proposal_table(table)
    ctx.spec_reset(prompts)
    caches = [ot.cache(L_max) for _ in range(nB)]
    seqs = [list(p) for p in prompts]
    for b in range(nB):
        if P > 1:
            ot.forward(caches[b], prompts[b][:P - 1], 0, want_logits=False)
    # prefill parity: cached K/V rows of layer 0 and the last layer
    for layer in (0, c["tgt"]["n_layers"] - 1):
        K, V = ctx.spec_kv_export(B.MODEL_TARGET, layer, nB, P - 1)
        for b in range(nB):
            assert np.abs(K[b].float().cpu().numpy() - caches[b].k(layer)[:P - 1]).max() < tol
            assert np.abs(V[b].float().cpu().numpy() - caches[b].v(layer)[:P - 1]).max() < tol
    worst = 0.0
    checked = 0
    rounds = 0
    hist = np.zeros(s + 1, dtype=np.int64)
    while min(len(q) for q in seqs) < P + N and rounds < 4 * N:
        rounds += 1
        n_before = [len(q) for q in seqs]
        for j in range(1, s + 1):
            ctx.spec_draft_step(j)
        g_logits = ctx.spec_verify_step(s, want_logits=True).cpu().numpy()
        ctx.spec_accept_commit(s)
        n_g, kd_g, l_g, a_g = ctx.spec_read_state()
        for b in range(nB):
            n = n_before[b]
            t = [int(table[b][n + j]) for j in range(s)]
            o_logits = ot.forward(caches[b], [seqs[b][n - 1]] + t, n - 1)
            err = np.abs(g_logits[b] - o_logits).max()
            worst = max(worst, err)
            assert err <= tol, (name, rounds, b, err)
            marg = top2_margin(o_logits)
            o_arg = o_logits.argmax(-1)
            for i in range(s + 1):
                if marg[i] > 2 * tol:
                    assert a_g[b][i] == o_arg[i], (name, rounds, b, i)
                    checked += 1
            # commit arithmetic on the GPU's own greedy tokens, against the oracle's rule
            l, em = orc.accept(t, a_g[b][:s + 1])
            gen = n - P
            take = min(l + 1, N - gen)
            assert l_g[b] == l
            assert n_g[b] == n + take
            if gen < N:
                hist[l] += 1
            seqs[b] = seqs[b] + em[:take]
            if take == l + 1:
                assert kd_g[b] == n + min(l, s - 1)
    out, g_hist = ctx.spec_read_output()
    for b in range(nB):
        assert out[b] == seqs[b][P:P + N]
    assert list(hist) == g_hist
    assert checked > 0
    print("%s: worst |logit err| %.3g over %d rounds (tol %g)" % (name, worst, rounds, tol))


@pytest.mark.parametrize("shift", [0.0, 1.0, 4.0])
def test_folded_layernorm_on_rows_off_centre(orc, B, shift):
    """The matrix-core path takes a LayerNorm's mean and variance from the fp16 copy of the residual rows and subtracts
    the mean's share after the product, so the rounding of a row to fp16 is relative to its mean, not to its spread.
    Rows whose mean is up to four times their spread must keep the usual tolerance (measured: 7e-4, 9e-4, 1.3e-3 of
    the allowed 1e-2).  The embeddings get a common offset of `shift` standard deviations on every channel."""
    desc = si.opt_desc(2, 256, 4, 384, 777, 64)
    nB, P, s, seed, dtype = 6, 5, 3, 91, "fp16"

    def off_centre(w):
        w["tok_emb"] = (w["tok_emb"].float() + shift * 0.03).to(w["tok_emb"].dtype)   # token + position: std 0.028

    ot, _, gt, _ = build_pair(orc, desc, None, dtype, seed, DEV, random_norms=True, tweak=off_centre)
    L_max = P + s + 4
    ctx = B.Context(desc, gt, None, None, dtype, nB, s, L_max, 1, B.PROPOSALS_EXTERNAL, DEV)
    prompts = si.make_prompts(nB, P, desc["vocab"], seed)
    table = np.random.default_rng(seed).integers(desc["vocab"], size=(nB, L_max)).astype(np.int32)
    ctx.spec_set_proposal_table(table)
    ctx.spec_reset(prompts)
    g_logits = ctx.spec_verify_step(s, want_logits=True).cpu().numpy()
    tol = LOGIT_TOL[dtype]
    worst = 0.0
    for b in range(nB):
        cache = ot.cache(L_max)
        ot.forward(cache, prompts[b][:P - 1], 0, want_logits=False)
        o_logits = ot.forward(cache, [prompts[b][P - 1]] + [int(t) for t in table[b][P:P + s]], P - 1)
        worst = max(worst, np.abs(g_logits[b] - o_logits).max())
    assert worst <= tol, (shift, worst)
    print("shift %.0f sigma: worst |logit err| %.3g (tol %g)" % (shift, worst, tol))
    ctx.close()


@pytest.mark.parametrize("name", list(CASES))
def test_speculative_equals_nonspeculative_on_gpu(orc, B, name):
    """The invariant of Sec. 2 on the GPU itself: every s, every proposal source and every
    batch composition emits exactly the tokens of plain greedy decoding (s = 0)."""
    c, ot, od, ctx, prompts, L_max = setup_case(orc, B, name, s_max=8)
    nB, P, N = c["B"], c["P"], c["N"]
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    base, _ = ctx.spec_read_output()
    assert all(len(x) == N for x in base)
    # vs the oracle: identical up to the first position whose top-2 margin is within tolerance
    tol = LOGIT_TOL[c["dtype"]]
    for b in range(nB):
        cache = ot.cache(L_max)
        lg = ot.forward(cache, list(prompts[b]) + base[b][:-1], 0)[P - 1:]
        for i in range(N):
            if top2_margin(lg[i]) <= 2 * tol:
                break
            assert base[b][i] == int(lg[i].argmax()), (name, b, i)
    truth = np.zeros((nB, L_max), dtype=np.int32)
    for b in range(nB):
        truth[b, P:P + N] = base[b]
    for s in (1, 2, 3, 5, 8):
        for alpha in (1.0, 0.0, c["alpha"]):
            if alpha == 0.0:
                table = (truth + 1) % c["tgt"]["vocab"]
            else:
                table = si.make_proposal_table(truth, alpha, c["tgt"]["vocab"], 31 + s)
            ctx.spec_set_proposal_table(table)
            ctx.spec_rewind()
            max_rounds = N if alpha < 1.0 else -(-N // (s + 1))
            ctx.spec_round(s, max_rounds)
            out, hist = ctx.spec_read_output()
            assert out == base, (name, s, alpha)
            if alpha == 1.0:   # perfect proposals: all s accepted (the last round may run past the known truth)
                assert sum(hist) == nB * max_rounds and hist[s] >= nB * (max_rounds - 1)
            if alpha == 0.0:   # useless proposals: one token per round
                assert hist[0] == nB * N and sum(hist[1:]) == 0
    # a sequence's tokens do not depend on what else is in the batch
    if nB > 1:
        ctx.spec_set_proposal_table(si.make_proposal_table(truth[1:2], c["alpha"], c["tgt"]["vocab"], 5))
        ctx.spec_reset(prompts[1:2])
        ctx.spec_round(3, N)
        solo, _ = ctx.spec_read_output()
        assert solo[0] == base[1]


@pytest.mark.parametrize("name", ["tiny_fp32", "small_bf16"])
def test_draft_model_proposals(orc, B, name):
    """SPEC_PROPOSALS_DRAFT: proposals are the draft model's own greedy tokens.  Output
    must still be the plain greedy output; draft-cache lengths follow the commit rule."""
    c, ot, od, ctx, prompts, L_max = setup_case(orc, B, name, proposal_mode=B.PROPOSALS_DRAFT, s_max=4)
    nB, P, N = c["B"], c["P"], c["N"]
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    base, _ = ctx.spec_read_output()
    for s in (1, 2, 4):
        ctx.spec_reset(prompts)
        for r in range(N):
            n0, _, _, _ = ctx.spec_read_state()
            for j in range(1, s + 1):
                ctx.spec_draft_step(j)
            ctx.spec_verify_step(s)
            ctx.spec_accept_commit(s)
            n1, kd, ll, _ = ctx.spec_read_state()
            for b in range(nB):
                if n1[b] - P < N:
                    assert n1[b] == n0[b] + ll[b] + 1
                    assert kd[b] == n0[b] + min(ll[b], s - 1)
        out, hist = ctx.spec_read_output()
        assert out == base, (name, s)
    # s switches between rounds, including s = 0 rounds that leave the draft cache behind
    ctx.spec_reset(prompts)
    for s in [2, 0, 3, 0, 0, 4, 1] * N:
        ctx.spec_round(s, 1)
    out, _ = ctx.spec_read_output()
    assert out == base


def test_maximum_speculation_length_and_exact_capacity(orc, B):
    """The largest s the library takes (15: 16 rows per sequence in one pass), a workspace sized to the last
    position (L_max = P + gen_max + s_max exactly), every slot of the batch used, rounds that overshoot
    gen_max: output is still the plain greedy output, for perfect, useless and mixed proposals."""
    c = CASES["small_bf16"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV, random_norms=True)
    nB, P, N, s_max = 3, 9, 21, 15
    L_max = P + N + s_max
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s_max, L_max, N, B.PROPOSALS_EXTERNAL, DEV)
    prompts = si.make_prompts(nB, P, c["tgt"]["vocab"], c["seed"])
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    base, _ = ctx.spec_read_output()
    assert all(len(x) == N for x in base)
    truth = np.zeros((nB, L_max), dtype=np.int32)
    for b in range(nB):
        truth[b, P:P + N] = base[b]
    for alpha in (1.0, 0.0, 0.8):
        table = (truth + 1) % c["tgt"]["vocab"] if alpha == 0.0 else si.make_proposal_table(truth, alpha, c["tgt"]["vocab"], 9)
        ctx.spec_set_proposal_table(table)
        ctx.spec_rewind()
        ctx.spec_round(s_max, N)                    # far more rounds than needed: finished sequences stay frozen
        out, hist = ctx.spec_read_output()
        assert out == base, alpha
        n, _, _, _ = ctx.spec_read_state()
        assert list(n) == [P + N] * nB
        if alpha == 1.0:                            # 16 tokens in the first round, the remaining 5 in the second
            assert hist[s_max] >= nB
    with pytest.raises(B.SpecError):
        ctx.spec_round(s_max + 1, 1)
    ctx.close()


def test_kv_import_export_roundtrip(orc, B):
    c, ot, od, ctx, prompts, L_max = setup_case(orc, B, "small_bf16")
    d = c["tgt"]["d_model"]
    K, V = si.make_kv(c["B"], d, 11, c["dtype"], 5, DEV)
    ctx.spec_kv_import(B.MODEL_TARGET, 1, K, V)
    K2, V2 = ctx.spec_kv_export(B.MODEL_TARGET, 1, c["B"], 11)
    assert torch.equal(K, K2) and torch.equal(V, V2)


def test_call_order_and_capacity_errors(orc, B):
    c, ot, od, ctx, prompts, L_max = setup_case(orc, B, "small_bf16")
    with pytest.raises(B.SpecError) as e:
        ctx.spec_verify_step(1)
    assert e.value.code == B.ERR_STATE
    ctx.spec_reset(prompts)
    with pytest.raises(B.SpecError) as e:
        ctx.spec_verify_step(c["s"] + 1)
    assert e.value.code == B.ERR_CAPACITY
    with pytest.raises(B.SpecError) as e:
        ctx.spec_accept_commit(0)
    assert e.value.code == B.ERR_STATE
    with pytest.raises(B.SpecError) as e:
        ctx.spec_draft_step(2)
    assert e.value.code == B.ERR_STATE
    with pytest.raises(B.SpecError) as e:
        ctx.spec_verify_step(2)          # external proposals were never supplied
    assert e.value.code == B.ERR_STATE
    ctx.spec_set_proposals(torch.zeros((c["B"], 2), dtype=torch.int32))
    ctx.spec_verify_step(2)
    with pytest.raises(B.SpecError) as e:
        ctx.spec_accept_commit(1)
    assert e.value.code == B.ERR_STATE
    ctx.spec_accept_commit(2)
    big = si.make_prompts(c["B"] + 1, c["P"], 10, 1)
    with pytest.raises(B.SpecError) as e:
        ctx.spec_reset(big)
    assert e.value.code == B.ERR_CAPACITY
    long = si.make_prompts(1, L_max, 10, 1)
    with pytest.raises(B.SpecError) as e:
        ctx.spec_reset(long)
    assert e.value.code == B.ERR_CAPACITY


@pytest.mark.parametrize("L_max,kv", [(640, 600), (2048, 1990), (3840, 3700)])
def test_attention_launch_shapes_give_identical_bits(orc, B, L_max, kv):
    """The launch shapes of the verify attention (split over chunks + merge kernel; one wave per sequence and
    head; one workgroup per sequence and head) must agree bit for bit: the batch size picks between them."""
    dtype, seed = "bf16", 5
    tdesc = si.llama_desc(1, 256, 2, 416, 300, L_max + 8)
    w = si.make_weights(tdesc, dtype, seed, device=DEV, emb_std=1.0)
    # 600 cached positions: five chunks (four of 128 keys, then 256-key ones), the last one ragged; 1990: ten, more
    # than the one-workgroup shape has waves (they take two chunks each); 3700: seventeen, where that shape hands over
    # to split + merge
    ctx = B.Context(tdesc, w, None, None, dtype, 3, 4, L_max, 4, B.PROPOSALS_EXTERNAL, DEV)
    K, V = si.make_kv(3, 256, kv, dtype, seed, DEV)
    ctx.spec_kv_import(B.MODEL_TARGET, 0, K, V)
    prompts = si.make_prompts(3, kv + 1, 300, seed)
    props = si.make_prompts(3, 4, 300, seed + 1)
    got = []
    for shape in (1, 2, 3, 0):
        ctx.spec_set_attention_shape(shape)
        ctx.spec_reset_noprefill(prompts)
        ctx.spec_set_proposals(torch.tensor(props))
        got.append(ctx.spec_verify_step(4, want_logits=True).clone())
        ctx.spec_accept_commit(4)
    assert all(torch.equal(got[0], g) for g in got[1:])
    with pytest.raises(B.SpecError):
        ctx.spec_set_attention_shape(4)


def test_saturation_counter_reports_activations_beyond_fp16(orc, B):
    """16-bit runs feed fp16 GEMM operands; values beyond +-65504 are clamped and counted.  The workloads never get
    there (count 0); an embedding table scaled into the hundreds of thousands does."""
    c = CASES["small_bf16"]
    for emb_std, expect_clamped in ((0.02, False), (2.0e5, True)):
        w = si.make_weights(c["tgt"], c["dtype"], c["seed"], device=DEV, emb_std=emb_std, tag="tgt.")
        L_max = c["P"] + 4 + 3
        ctx = B.Context(c["tgt"], w, None, None, c["dtype"], c["B"], 2, L_max, 4, B.PROPOSALS_EXTERNAL, DEV)
        assert ctx.spec_read_saturation() == 0
        ctx.spec_reset(si.make_prompts(c["B"], c["P"], c["tgt"]["vocab"], c["seed"]))
        ctx.spec_round(0, 2)
        n = ctx.spec_read_saturation()
        assert (n > 0) == expect_clamped, (emb_std, n)
        ctx.close()
