"""Pins of the CPU oracle against things other than itself (CPU only).

* decoder forward vs the HuggingFace LLaMA / OPT implementations (the model layer
  the paper's prototype ran on, Sec. 3.1), in fp64
* elementary operations vs closed forms and library routines
* Alg. 1 vs plain greedy decoding (the invariant of Sec. 2), vs HF greedy generation
* acceptance rule vs hand-worked cases; acceptance statistics vs Eq. 6 in closed form
* LUT rule (Sec. 4) vs enumerated cases; Eq. 4 estimator; Eq. 7 time model
"""
import math
import os

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as orc_mod

GOLD = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def o64():
    return orc_mod.Oracle("f64")


@pytest.fixture(scope="module")
def o32():
    return orc_mod.Oracle("f32")


# ------------------------------------------------------------------ helpers

def tiny_llama(seed=3, n_layers=2, d=32, heads=2, ffn=48, vocab=61, max_pos=64):
    desc = si.llama_desc(n_layers, d, heads, ffn, vocab, max_pos)
    w = si.make_weights(desc, "fp32", seed, emb_std=0.5)
    for L in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "w1", "w3", "w2"):
            L[k] = L[k] * 10.0  # make attention / FFN matter
    si.randomize_norms(w, desc, "fp32", seed)
    return desc, w


def tiny_opt(seed=5, n_layers=2, d=32, heads=4, ffn=40, vocab=53, max_pos=48):
    desc = si.opt_desc(n_layers, d, heads, ffn, vocab, max_pos)
    w = si.make_weights(desc, "fp32", seed, emb_std=0.5)
    for L in w["layers"]:
        for k in ("wq", "wk", "wv", "wo", "w1", "w2", "bq", "bk", "bv", "bo", "b1", "b2"):
            L[k] = L[k] * 10.0
    w["pos_emb"] = w["pos_emb"] * 10.0
    si.randomize_norms(w, desc, "fp32", seed)
    return desc, w


def hf_llama(desc, w):
    from transformers import LlamaConfig, LlamaForCausalLM
    c = LlamaConfig(vocab_size=desc["vocab"], hidden_size=desc["d_model"], intermediate_size=desc["d_ffn"],
                    num_hidden_layers=desc["n_layers"], num_attention_heads=desc["n_heads"],
                    num_key_value_heads=desc["n_heads"], max_position_embeddings=desc["max_pos"],
                    rms_norm_eps=desc["norm_eps"], rope_theta=desc["rope_theta"], tie_word_embeddings=False,
                    attention_bias=False, mlp_bias=False, hidden_act="silu")
    m = LlamaForCausalLM(c)
    sd = {"model.embed_tokens.weight": w["tok_emb"], "model.norm.weight": w["final_norm_w"],
          "lm_head.weight": w["lm_head"]}
    for i, L in enumerate(w["layers"]):
        p = "model.layers.%d." % i
        sd.update({p + "self_attn.q_proj.weight": L["wq"], p + "self_attn.k_proj.weight": L["wk"],
                   p + "self_attn.v_proj.weight": L["wv"], p + "self_attn.o_proj.weight": L["wo"],
                   p + "mlp.gate_proj.weight": L["w1"], p + "mlp.up_proj.weight": L["w3"],
                   p + "mlp.down_proj.weight": L["w2"], p + "input_layernorm.weight": L["attn_norm_w"],
                   p + "post_attention_layernorm.weight": L["ffn_norm_w"]})
    m.load_state_dict(sd, strict=True)
    return m.double().eval()


def hf_opt(desc, w):
    from transformers import OPTConfig, OPTForCausalLM
    c = OPTConfig(vocab_size=desc["vocab"], hidden_size=desc["d_model"], ffn_dim=desc["d_ffn"],
                  num_hidden_layers=desc["n_layers"], num_attention_heads=desc["n_heads"],
                  max_position_embeddings=desc["max_pos"], do_layer_norm_before=True,
                  word_embed_proj_dim=desc["d_model"], tie_word_embeddings=False, activation_function="relu",
                  enable_bias=True, layer_norm_elementwise_affine=True)
    m = OPTForCausalLM(c)
    # HF's OPT position table carries two leading rows that are never addressed by real positions
    pos = torch.cat([torch.zeros(2, desc["d_model"]), w["pos_emb"]], 0)
    sd = {"model.decoder.embed_tokens.weight": w["tok_emb"], "model.decoder.embed_positions.weight": pos,
          "model.decoder.final_layer_norm.weight": w["final_norm_w"],
          "model.decoder.final_layer_norm.bias": w["final_norm_b"], "lm_head.weight": w["lm_head"]}
    for i, L in enumerate(w["layers"]):
        p = "model.decoder.layers.%d." % i
        sd.update({p + "self_attn.q_proj.weight": L["wq"], p + "self_attn.q_proj.bias": L["bq"],
                   p + "self_attn.k_proj.weight": L["wk"], p + "self_attn.k_proj.bias": L["bk"],
                   p + "self_attn.v_proj.weight": L["wv"], p + "self_attn.v_proj.bias": L["bv"],
                   p + "self_attn.out_proj.weight": L["wo"], p + "self_attn.out_proj.bias": L["bo"],
                   p + "self_attn_layer_norm.weight": L["attn_norm_w"],
                   p + "self_attn_layer_norm.bias": L["attn_norm_b"],
                   p + "fc1.weight": L["w1"], p + "fc1.bias": L["b1"], p + "fc2.weight": L["w2"],
                   p + "fc2.bias": L["b2"], p + "final_layer_norm.weight": L["ffn_norm_w"],
                   p + "final_layer_norm.bias": L["ffn_norm_b"]})
    m.load_state_dict(sd, strict=True)
    return m.double().eval()


def omodel(orc, desc, w, wdtype=orc_mod.W_F32):
    return orc.model(desc, si.weights_to_numpy(w), wdtype)


# ------------------------------------------------------ forward vs HuggingFace

@pytest.mark.parametrize("family", ["llama", "opt"])
def test_forward_matches_huggingface(o64, family):
    desc, w = tiny_llama() if family == "llama" else tiny_opt()
    hf = hf_llama(desc, w) if family == "llama" else hf_opt(desc, w)
    rng = np.random.default_rng(11)
    toks = rng.integers(0, desc["vocab"], size=13).astype(np.int32)
    with torch.no_grad():
        ref = hf(torch.tensor(toks[None].astype(np.int64))).logits[0].numpy()
    m = omodel(o64, desc, w)
    # HF evaluates the rotary angles, cos and sin in float32 whatever the model dtype, so its
    # LLaMA logits carry ~1e-7 of their own error; OPT (no rotary) agrees to fp64 rounding
    tol = (1e-6 if family == "llama" else 1e-9) * max(1.0, np.abs(ref).max())
    # (a) whole sequence in one call, empty cache
    c = m.cache(32)
    got = m.forward(c, toks, 0)
    assert np.abs(got - ref).max() < tol
    # (b) prefix through the cache, then a multi-token verification call, then single steps
    c = m.cache(32)
    m.forward(c, toks[:5], 0, want_logits=False)
    got_b = m.forward(c, toks[5:9], 5)
    assert np.abs(got_b - ref[5:9]).max() < tol
    for i in range(9, 13):
        g = m.forward(c, toks[i:i + 1], i)
        assert np.abs(g[0] - ref[i]).max() < tol
    # (c) roll-back: overwrite positions 5.. with other tokens, then restore -> same logits
    m.forward(c, (toks[5:9] + 1) % desc["vocab"], 5)
    got_c = m.forward(c, toks[5:9], 5)
    assert np.array_equal(got_c, got_b)


def test_greedy_matches_huggingface_generate(o64):
    desc, w = tiny_llama(seed=8)
    hf = hf_llama(desc, w)
    prompt = si.make_prompts(1, 6, desc["vocab"], 21)[0]
    N = 20
    ids = torch.tensor(prompt[None].astype(np.int64))
    with torch.no_grad():
        for _ in range(N):  # plain autoregressive greedy, full recompute every step (brute force)
            nxt = hf(ids).logits[0, -1].argmax().item()
            ids = torch.cat([ids, torch.tensor([[nxt]])], 1)
    ref = ids[0, 6:].numpy().astype(np.int32)
    got = omodel(o64, desc, w).greedy(prompt, N)
    assert np.array_equal(got, ref)


# ---------------------------------------------------- elementary operations

def test_widen_bf16_fp16_exhaustive(o64):
    bits = np.arange(65536, dtype=np.uint16)
    for code, tdt in ((orc_mod.W_BF16, torch.bfloat16), (orc_mod.W_F16, torch.float16)):
        ref = torch.from_numpy(bits.view(np.int16)).view(tdt).to(torch.float64).numpy()
        got = o64.widen(bits, code)
        ok = np.isnan(ref) | (got == ref)
        assert ok.all()
        assert np.isnan(got[np.isnan(ref)]).all()


def test_linear_rmsnorm_layernorm_swiglu_vs_library(o64):
    rng = np.random.default_rng(2)
    x = rng.standard_normal((5, 37))
    W = rng.standard_normal((11, 37)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    y = o64.linear(x, W, b)
    ref = torch.nn.functional.linear(torch.tensor(x), torch.tensor(W).double(), torch.tensor(b).double()).numpy()
    assert np.abs(y - ref).max() < 1e-12
    # a transposed operand or a dropped bias would show here
    assert np.abs(o64.linear(x, W) - (ref - b)).max() < 1e-12
    g = rng.standard_normal(37).astype(np.float32)
    bb = rng.standard_normal(37).astype(np.float32)
    r = o64.rmsnorm(x, g, 1e-5)
    ref = torch.nn.functional.rms_norm(torch.tensor(x), (37,), torch.tensor(g).double(), 1e-5).numpy()
    assert np.abs(r - ref).max() < 1e-12
    ln = o64.layernorm(x, g, bb, 1e-5)
    ref = torch.nn.functional.layer_norm(torch.tensor(x), (37,), torch.tensor(g).double(),
                                         torch.tensor(bb).double(), 1e-5).numpy()
    assert np.abs(ln - ref).max() < 1e-12
    u = rng.standard_normal((5, 37))
    sw = o64.swiglu(x, u)
    ref = (torch.nn.functional.silu(torch.tensor(x)) * torch.tensor(u)).numpy()
    assert np.abs(sw - ref).max() < 1e-12


def test_rope_closed_forms(o64):
    rng = np.random.default_rng(4)
    H, hd = 3, 16
    x = rng.standard_normal(H * hd)
    # position 0 is the identity
    assert np.array_equal(o64.rope(x, H, 0), x)
    # pair norms are preserved; pair i of every head turns by pos * theta^(-2i/hd)
    pos, theta = 7, 10000.0
    y = o64.rope(x, H, pos, theta)
    xv, yv = x.reshape(H, hd), y.reshape(H, hd)
    for i in range(hd // 2):
        zx = xv[:, i] + 1j * xv[:, i + hd // 2]
        zy = yv[:, i] + 1j * yv[:, i + hd // 2]
        ang = pos * theta ** (-2.0 * i / hd)
        assert np.abs(zy - zx * np.exp(1j * ang)).max() < 1e-12
    # relative-position property: <rope(q,m), rope(k,n)> depends on m-n only
    q, k = rng.standard_normal(hd), rng.standard_normal(hd)
    d1 = o64.rope(q, 1, 9) @ o64.rope(k, 1, 4)
    d2 = o64.rope(q, 1, 25) @ o64.rope(k, 1, 20)
    assert abs(d1 - d2) < 1e-10


def test_attention_closed_forms_and_sdpa(o64):
    rng = np.random.default_rng(6)
    H, hd, n = 2, 8, 9
    d = H * hd
    q = rng.standard_normal(d)
    K = rng.standard_normal((n, d))
    V = rng.standard_normal((n, d))
    # one key: the output is that key's value row, whatever the scores
    assert np.abs(o64.attention(q, K[:1], V[:1], H) - V[0]).max() < 1e-14
    # identical keys: uniform weights -> mean of the values
    Ksame = np.repeat(K[:1], n, 0)
    assert np.abs(o64.attention(q, Ksame, V, H) - V.mean(0)).max() < 1e-12
    # general case vs torch's scaled_dot_product_attention (scale 1/sqrt(hd))
    out = o64.attention(q, K, V, H)
    tq = torch.tensor(q).view(1, H, 1, hd)
    tk = torch.tensor(K).view(n, H, hd).permute(1, 0, 2)[None]
    tv = torch.tensor(V).view(n, H, hd).permute(1, 0, 2)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv).reshape(d).numpy()
    assert np.abs(out - ref).max() < 1e-12


def test_argmax_lowest_index_on_ties(o64):
    assert o64.argmax([1.0, 3.0, 3.0, 2.0]) == 1
    assert o64.argmax([5.0, 5.0]) == 0
    assert o64.argmax([-2.0, -1.0, -3.0]) == 1


# ------------------------------------------------------------ acceptance rule

def _ints(s):
    s = s.strip()
    return [] if s == "-" else [int(x) for x in s.split(",")]


def test_accept_hand_worked_cases(o64):
    n = 0
    for line in open(os.path.join(GOLD, "accept_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        t, a, l, em = [p for p in line.split("|")]
        got_l, got_em = o64.accept(_ints(t), _ints(a))
        assert got_l == int(l) and got_em == _ints(em), line
        n += 1
    assert n >= 8


def test_accept_statistics_match_eq6(o64):
    """Under i.i.d. per-token correctness alpha, Eq. 6 gives l(s) = sum_i alpha^i."""
    rng = np.random.default_rng(9)
    alpha, s, n = 0.7, 4, 40000
    ls = []
    for _ in range(n):
        a = rng.integers(0, 1000, size=s + 1)
        ok = rng.random(s) < alpha
        t = np.where(ok, a[:s], a[:s] + 1)  # a wrong proposal never equals the target token here
        l, em = o64.accept(t, a)
        ls.append(l)
        assert len(em) == l + 1
    closed = sum(alpha ** i for i in range(1, s + 1))
    assert abs(closed - alpha * (1 - alpha ** s) / (1 - alpha)) < 1e-12
    assert abs(closed - 1.7731) < 1e-4          # worked value for alpha=0.7, s=4
    assert abs(np.mean(ls) - closed) < 4 * np.std(ls) / math.sqrt(n)
    # Eq. 4 on untruncated run lengths converges to the same number
    geo = rng.geometric(1 - alpha, size=n) - 1   # number of correct tokens before the first wrong one
    assert abs(o64.l_estimate(geo, s) - closed) < 0.02
    assert o64.l_estimate([0, 1, 5, 9], 3) == (0 + 1 + 3 + 3) / 4


# -------------------------------------------------- Alg. 1 == plain greedy

@pytest.fixture(scope="module")
def tiny_pair():
    dt, wt = tiny_llama(seed=12, n_layers=2, d=32, heads=2, ffn=48, vocab=61, max_pos=128)
    dd, wd = tiny_llama(seed=13, n_layers=1, d=16, heads=2, ffn=24, vocab=61, max_pos=128)
    return dt, wt, dd, wd


@pytest.mark.parametrize("s", [0, 1, 2, 3, 4, 8])
def test_speculative_equals_greedy_every_source(o64, tiny_pair, s):
    dt, wt, dd, wd = tiny_pair
    tgt, drf = omodel(o64, dt, wt), omodel(o64, dd, wd)
    P, N = 5, 23
    prompt = si.make_prompts(1, P, dt["vocab"], 33)[0]
    ref = tgt.greedy(prompt, N + 10)
    L = P + N + 10 + s + 1
    truth = np.zeros(L, dtype=np.int32)
    truth[P:P + N + 10] = ref
    # the draft model's own proposals
    out, ls = tgt.spec_generate(drf, prompt, N, s, proposal_mode=0)
    assert np.array_equal(out, ref[:N])
    assert sum(l + 1 for l in ls) >= N and all(0 <= l <= s for l in ls)
    # perfect proposals: every round but the last yields s+1 tokens
    out, ls = tgt.spec_generate(drf, prompt, N, s, proposal_mode=1, prop_table=truth, L_max=L)
    assert np.array_equal(out, ref[:N])
    assert len(ls) == math.ceil(N / (s + 1)) and all(l == s for l in ls)
    # useless proposals: exactly one token per round, still the greedy output (Sec. 2)
    wrong = (truth + 1) % dt["vocab"]
    out, ls = tgt.spec_generate(None, prompt, N, s, proposal_mode=1, prop_table=wrong, L_max=L)
    assert np.array_equal(out, ref[:N])
    assert len(ls) == N and all(l == 0 for l in ls)
    # the replacement scheme of the workloads
    tbl = si.make_proposal_table(truth[None], 0.7, dt["vocab"], 5)[0]
    out, ls = tgt.spec_generate(drf, prompt, N, s, proposal_mode=1, prop_table=tbl, L_max=L)
    assert np.array_equal(out, ref[:N])


@pytest.mark.parametrize("s", [1, 2, 3, 4, 5, 6, 7, 8])
def test_draft_equal_to_target_gets_every_proposal_accepted(o64, tiny_pair, s):
    """Pins the draft side of Alg. 1 (the call speculate(S, kv_SSM, s)): with the target's own weights as the
    draft every proposal is the target's greedy token, so every round accepts all s proposals and emits s + 1
    tokens (Sec. 2: at least one, at most s + 1 per round) -- but only if the draft's cache is exactly the
    committed prefix when a round starts: a wrong cache length after the roll-back, a first step that ingests one
    token where two are due (after l = s the draft never read t_s), or a stale row all change a proposal."""
    dt, wt, _, _ = tiny_pair
    tgt, twin = omodel(o64, dt, wt), omodel(o64, dt, wt)
    for P, N in ((5, 23), (1, 17), (2, 9 * (s + 1))):
        prompt = si.make_prompts(1, P, dt["vocab"], 33 + P)[0]
        ref = tgt.greedy(prompt, N)
        out, ls = tgt.spec_generate(twin, prompt, N, s, proposal_mode=0)
        assert np.array_equal(out, ref)
        assert ls == [s] * math.ceil(N / (s + 1)), (P, N, s, ls)


def _alg1_with_draft_rule(tgt, drf, prompt, N, s, L, keep_rule, first_rule):
    """Alg. 1 written on the oracle's forward alone, the draft-cache bookkeeping left open: keep_rule(n_old, l, s)
    -> draft cache length kept after a round; first_rule(n, kvD) -> how many committed tokens the round's first
    draft step ingests (they end at position n - 1).  Returns the accepted counts per round."""
    ct, cd = tgt.cache(L), drf.cache(L)
    S = list(prompt)
    P = len(S)
    if P > 1:
        tgt.forward(ct, S[:P - 1], 0, want_logits=False)
        drf.forward(cd, S[:P - 1], 0, want_logits=False)
    kvD, ls = P - 1, []
    while len(S) - P < N:
        n, t = len(S), []
        for j in range(1, s + 1):
            if j == 1:
                cnt = first_rule(n, kvD)
                lg = drf.forward(cd, S[n - cnt:n], n - cnt)
            else:
                lg = drf.forward(cd, [t[-1]], n + j - 2)
            t.append(int(lg[-1].argmax()))
        a = tgt.forward(ct, [S[n - 1]] + t, n - 1).argmax(-1)
        l, em = tgt.orc.accept(t, a)
        S += em
        ls.append(l)
        kvD = min(keep_rule(n, l, s), len(S) - 1)
    return ls


def test_draft_equal_to_target_pin_catches_planted_bookkeeping_mistakes(o64, tiny_pair):
    """The pin above has teeth: the same construction run with a planted mistake in the draft bookkeeping (on the
    CPU, through the oracle's own forward) no longer accepts everything."""
    dt, wt, _, _ = tiny_pair
    tgt, twin = omodel(o64, dt, wt), omodel(o64, dt, wt)
    P, N, s, L = 5, 24, 3, 64
    prompt = si.make_prompts(1, P, dt["vocab"], 38)[0]
    right_keep = lambda n, l, s_: n + min(l, s_ - 1)
    right_first = lambda n, kvD: n - kvD
    assert _alg1_with_draft_rule(tgt, twin, prompt, N, s, L, right_keep, right_first) == [s] * (N // (s + 1))
    # forgets that t_s was never ingested (keeps n + l): position n + s - 1 of the draft cache is stale
    ls = _alg1_with_draft_rule(tgt, twin, prompt, N, s, L, lambda n, l, s_: n + l, right_first)
    assert min(ls) < s
    # first step always ingests one token: the draft cache gets a hole after every fully accepted round
    ls = _alg1_with_draft_rule(tgt, twin, prompt, N, s, L, right_keep, lambda n, kvD: 1)
    assert min(ls) < s


def test_verify_logits_equal_single_steps(o64, tiny_pair):
    dt, wt, _, _ = tiny_pair
    m = omodel(o64, dt, wt)
    toks = si.make_prompts(1, 12, dt["vocab"], 44)[0]
    c1, c2 = m.cache(16), m.cache(16)
    m.forward(c1, toks[:7], 0, want_logits=False)
    m.forward(c2, toks[:7], 0, want_logits=False)
    block = m.forward(c1, toks[7:12], 7)
    for i in range(7, 12):
        one = m.forward(c2, toks[i:i + 1], i)[0]
        assert np.abs(one - block[i - 7]).max() < 1e-12


def test_config1_fp32_oracle_agrees_with_fp64(o32, o64):
    dtype, seed, dt, dd = si.CONFIGS["tiny_fp32"]
    wt = si.make_weights(dt, dtype, seed, tag="tgt.")
    wd = si.make_weights(dd, dtype, seed, tag="drf.")
    prompt = si.make_prompts(1, 16, dt["vocab"], seed)[0]
    t64, t32 = omodel(o64, dt, wt), omodel(o32, dt, wt)
    ref = t64.greedy(prompt, 32 + 9)
    c64, c32 = t64.cache(64), t32.cache(64)
    seq = np.concatenate([prompt, ref[:8]])
    l64 = t64.forward(c64, seq, 0)
    l32 = t32.forward(c32, seq, 0)
    assert np.abs(l64 - l32).max() < 1e-4
    # config 1 as specified: B=1, s=4, replacement probability 0.3
    L = 16 + 32 + 9 + 5
    truth = np.zeros(L, dtype=np.int32)
    truth[16:16 + 41] = ref
    tbl = si.make_proposal_table(truth[None], 0.7, dt["vocab"], seed)[0]
    d64 = omodel(o64, dd, wd)
    out, ls = t64.spec_generate(d64, prompt, 32, 4, proposal_mode=1, prop_table=tbl, L_max=L)
    assert np.array_equal(out, ref[:32])
    assert 0 < np.mean(ls) < 4


# ---------------------------------------------------------------- adaptive

def test_lut_lookup_enumerated_cases(o64):
    n = 0
    for line in open(os.path.join(GOLD, "lut_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        pb, lut, B, exp = line.split("|")
        assert o64.lut_lookup(_ints(pb), _ints(lut), int(B)) == int(exp), line
        n += 1
    assert n >= 10


def test_lut_build_argmin_and_ties(o64):
    lat = np.array([[5.0, 4.0, 3.0, 2.5, 2.6],     # clear minimum at s=3
                    [3.0, 2.0, 2.01, 2.5, 3.0],    # s=2 within 1 % of s=1 -> smaller s wins
                    [1.0, 1.2, 1.4, 1.6, 1.8]])    # speculation never pays -> s=0
    assert o64.lut_build(lat, 0.01).tolist() == [3, 1, 0]
    assert o64.lut_build(np.array([[2.0, 1.0, 0.995]]), 0.01).tolist() == [1]
    assert o64.lut_build(np.array([[2.0, 1.0, 0.9]]), 0.01).tolist() == [2]


def test_time_model_eq7(o64):
    # no speculation, nothing accepted: N target steps
    assert o64.time_model(100, 2.0, 0.5, 0, 0.0) == 200.0
    # Eq. 2 + Eq. 3: N/(l+1) rounds, each one target step plus s draft steps
    assert abs(o64.time_model(120, 3.0, 0.25, 4, 2.0) - (120 / 3.0) * (3.0 + 4 * 0.25)) < 1e-12
