"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds no arithmetic of the method: only model shapes, random parameter /
prompt / KV-cache generation and the proposal-replacement table.  Both the CPU
oracle and the GPU library are fed from here; neither is imported here.

Workload recipes (the five synthetic configurations that stand in for the
paper's OPT / LLaMA checkpoints and its prompt dataset, Sec. 5.1):
  * parameters ~ N(0, 0.02) rounded to the model dtype; norm gains 1, LayerNorm
    biases 0; OPT-shape linear biases ~ N(0, 0.02)
  * prompts: uniform-random token ids
  * proposals: the target's own greedy continuation, each token independently
    replaced by a uniform-random token with probability 1 - accept_prob
"""
import zlib

import numpy as np
import torch

FFN_SWIGLU, FFN_RELU = 0, 1
NORM_RMS, NORM_LAYER = 0, 1
POS_ROPE, POS_LEARNED = 0, 1

SLOT_NAMES = ["attn_norm_w", "attn_norm_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
              "ffn_norm_w", "ffn_norm_b", "w1", "b1", "w3", "w2", "b2"]

TORCH_DTYPE = {"fp32": torch.float32, "bf16": torch.bfloat16, "fp16": torch.float16}
DTYPE_CODE = {"fp32": 0, "bf16": 1, "fp16": 2}


def llama_desc(n_layers, d, heads, ffn, vocab, max_pos=4096):
    return dict(n_layers=n_layers, d_model=d, n_heads=heads, d_ffn=ffn, vocab=vocab, max_pos=max_pos,
                ffn_kind=FFN_SWIGLU, norm_kind=NORM_RMS, pos_kind=POS_ROPE, has_bias=0,
                norm_eps=1e-5, rope_theta=10000.0)


def opt_desc(n_layers, d, heads, ffn, vocab, max_pos=2048):
    return dict(n_layers=n_layers, d_model=d, n_heads=heads, d_ffn=ffn, vocab=vocab, max_pos=max_pos,
                ffn_kind=FFN_RELU, norm_kind=NORM_LAYER, pos_kind=POS_LEARNED, has_bias=1,
                norm_eps=1e-5, rope_theta=10000.0)


# name -> (dtype, seed, target desc, draft desc or None)
CONFIGS = {
    "tiny_fp32": ("fp32", 1000, llama_desc(2, 256, 4, 1024, 1024, 256), llama_desc(1, 128, 2, 512, 1024, 256)),
    "layer_bf16": ("bf16", 1001, llama_desc(1, 4096, 32, 11008, 32000, 1024), None),
    "llama7b_bf16": ("bf16", 1002, llama_desc(32, 4096, 32, 11008, 32000, 512),
                     llama_desc(2, 768, 12, 3072, 32000, 512)),
    "opt13b_fp16": ("fp16", 1003, opt_desc(40, 5120, 40, 20480, 50272, 512),
                    opt_desc(12, 768, 12, 3072, 50272, 512)),
    "llama33b_bf16": ("bf16", 1004, llama_desc(60, 6656, 52, 17920, 32000, 2560),
                      llama_desc(4, 1024, 16, 4096, 32000, 2560)),
}


def _gen(seed, name, device):
    g = torch.Generator(device=device)
    g.manual_seed((int(seed) * 1000003 + zlib.crc32(name.encode())) % (2 ** 63))
    return g


def _normal(shape, std, dtype, seed, name, device):
    g = _gen(seed, name, device)
    # draw in chunks so a 500 MB matrix never needs a multi-GB fp32 temporary on the host
    out = torch.empty(shape, dtype=dtype, device=device)
    flat = out.view(-1)
    step = 1 << 26
    for i in range(0, flat.numel(), step):
        n = min(step, flat.numel() - i)
        flat[i:i + n] = (torch.randn(n, generator=g, device=device, dtype=torch.float32) * std).to(dtype)
    return out


def make_weights(desc, dtype, seed, device="cpu", emb_std=0.02, tag=""):
    """Canonical parameter set: dict of torch tensors, every matrix row-major [out][in]."""
    td = TORCH_DTYPE[dtype]
    d, f, V = desc["d_model"], desc["d_ffn"], desc["vocab"]
    ln = desc["norm_kind"] == NORM_LAYER
    hb = bool(desc["has_bias"])
    swi = desc["ffn_kind"] == FFN_SWIGLU

    def N(shape, name, std=0.02):
        return _normal(shape, std, td, seed, tag + name, device)

    def ones(n):
        return torch.ones(n, dtype=td, device=device)

    def zeros(n):
        return torch.zeros(n, dtype=td, device=device)

    w = {"tok_emb": N((V, d), "tok_emb", emb_std),
         "pos_emb": N((desc["max_pos"], d), "pos_emb") if desc["pos_kind"] == POS_LEARNED else None,
         "final_norm_w": ones(d), "final_norm_b": zeros(d) if ln else None,
         "lm_head": N((V, d), "lm_head"), "layers": []}
    for li in range(desc["n_layers"]):
        p = "L%d." % li
        L = {"attn_norm_w": ones(d), "attn_norm_b": zeros(d) if ln else None,
             "wq": N((d, d), p + "wq"), "wk": N((d, d), p + "wk"), "wv": N((d, d), p + "wv"),
             "wo": N((d, d), p + "wo"),
             "bq": N((d,), p + "bq") if hb else None, "bk": N((d,), p + "bk") if hb else None,
             "bv": N((d,), p + "bv") if hb else None, "bo": N((d,), p + "bo") if hb else None,
             "ffn_norm_w": ones(d), "ffn_norm_b": zeros(d) if ln else None,
             "w1": N((f, d), p + "w1"), "b1": N((f,), p + "b1") if (hb and not swi) else None,
             "w3": N((f, d), p + "w3") if swi else None,
             "w2": N((d, f), p + "w2"), "b2": N((d,), p + "b2") if (hb and not swi) else None}
        w["layers"].append(L)
    return w


def randomize_norms(w, desc, dtype, seed, device="cpu"):
    """Non-trivial norm gains/biases (tests only: the workloads keep gain 1 / bias 0)."""
    td = TORCH_DTYPE[dtype]
    d = desc["d_model"]

    def G(name):
        return (1.0 + _normal((d,), 0.1, torch.float32, seed, name, device)).to(td)

    def Bz(name):
        return _normal((d,), 0.1, td, seed, name, device)

    ln = desc["norm_kind"] == NORM_LAYER
    w["final_norm_w"] = G("fnw")
    if ln:
        w["final_norm_b"] = Bz("fnb")
    for li, L in enumerate(w["layers"]):
        L["attn_norm_w"] = G("anw%d" % li)
        L["ffn_norm_w"] = G("fnw%d" % li)
        if ln:
            L["attn_norm_b"] = Bz("anb%d" % li)
            L["ffn_norm_b"] = Bz("fnb%d" % li)
    return w


def to_numpy(t):
    """torch tensor -> numpy: float32 as is, 16-bit types as their uint16 bit patterns."""
    if t is None:
        return None
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.float32:
        return t.numpy()
    return t.view(torch.int16).numpy().view(np.uint16)


def weights_to_numpy(w):
    out = {k: to_numpy(v) for k, v in w.items() if k != "layers"}
    out["layers"] = [{k: to_numpy(v) for k, v in L.items()} for L in w["layers"]]
    return out


def make_prompts(B, P, vocab, seed):
    rng = np.random.default_rng([int(seed), 7])
    return rng.integers(0, vocab, size=(B, P), dtype=np.int32)


def _splitmix64(x):
    x = (x + np.uint64(0x9E3779B97F4A7C15)) & np.uint64(0xFFFFFFFFFFFFFFFF)
    z = x
    z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
    return z ^ (z >> np.uint64(31))


def make_proposal_table(ref, accept_prob, vocab, seed):
    """ref: int32 [B][L] -- the true greedy token at every absolute position (prompt
    positions are never proposed, their content is irrelevant).  Entry [b][pos] is
    what the draft proposes for position pos: ref[b][pos] with probability
    accept_prob, else a uniform-random token (which may happen to be right).
    Draws are keyed on (seed, b, pos) so a position proposed twice gets the same token."""
    ref = np.asarray(ref, dtype=np.int32)
    B, L = ref.shape
    with np.errstate(over="ignore"):
        b = np.arange(B, dtype=np.uint64)[:, None]
        p = np.arange(L, dtype=np.uint64)[None, :]
        key = np.uint64(seed) * np.uint64(0x100000001B3) + b * np.uint64(0x1000193) * np.uint64(1 << 20) + p
        h1 = _splitmix64(key)
        h2 = _splitmix64(h1)
    u = (h1 >> np.uint64(11)).astype(np.float64) / float(1 << 53)
    rnd = (h2 % np.uint64(vocab)).astype(np.int32)
    return np.where(u < accept_prob, ref, rnd).astype(np.int32)


def make_kv(B, d, L, dtype, seed, device="cpu"):
    """Random cache content for the single-layer verify microbenchmark: K and V rows
    ~ N(0,1) rounded to the model dtype, canonical layout [B][L][d_model]."""
    td = TORCH_DTYPE[dtype]
    K = _normal((B, L, d), 1.0, td, seed, "kvK", device)
    V = _normal((B, L, d), 1.0, td, seed, "kvV", device)
    return K, V
