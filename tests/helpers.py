"""Shared helpers of the GPU parity tests: build the same model for the CPU oracle and the
GPU library from one seeded parameter set."""
import numpy as np
import torch

import synth_inputs as si

ORC_WDTYPE = {"fp32": 0, "bf16": 1, "fp16": 2}
# max |logit| error the GPU path may show against the fp64 oracle fed the same rounded
# parameters: fp32 arithmetic 1e-4, bf16 storage of activations 2e-2, fp16 1e-2
LOGIT_TOL = {"fp32": 1e-4, "bf16": 2e-2, "fp16": 1e-2}


def build_pair(orc, tdesc, ddesc, dtype, seed, device, emb_std=0.02, random_norms=False, tweak=None):
    """-> (oracle target, oracle draft or None, gpu weights target, gpu weights draft or None)
    tweak(w): changes the seeded parameter set in place before either side sees it."""
    out = []
    gw = []
    for tag, desc in (("tgt.", tdesc), ("drf.", ddesc)):
        if desc is None:
            out.append(None)
            gw.append(None)
            continue
        w = si.make_weights(desc, dtype, seed, device="cpu", emb_std=emb_std, tag=tag)
        if random_norms:
            si.randomize_norms(w, desc, dtype, seed)
        if tweak:
            tweak(w)
        out.append(orc.model(desc, si.weights_to_numpy(w), ORC_WDTYPE[dtype]))
        wg = {k: (v.to(device) if v is not None else None) for k, v in w.items() if k != "layers"}
        wg["layers"] = [{k: (v.to(device) if v is not None else None) for k, v in L.items()} for L in w["layers"]]
        gw.append(wg)
    return out[0], out[1], gw[0], gw[1]


def truth_table(ref, P, L_max):
    """ref: [B][n] greedy continuation -> [B][L_max] table of true tokens by absolute position."""
    ref = np.asarray(ref)
    B, n = ref.shape
    t = np.zeros((B, L_max), dtype=np.int32)
    m = min(n, L_max - P)
    t[:, P:P + m] = ref[:, :m]
    return t


def top2_margin(logits):
    s = np.sort(np.asarray(logits, dtype=np.float64), axis=-1)
    return s[..., -1] - s[..., -2]


def assert_greedy_matches_oracle(ot, prompt, tokens, dtype):
    """The GPU's plain greedy continuation of one prompt against the oracle: identical token for token in fp32; in the
    16-bit types identical up to the first position where the oracle's own top-2 margin is within twice the logit
    tolerance (from there on the two may legitimately follow different continuations).  The oracle is teacher-forced
    with the GPU's tokens, so every compared position has the same prefix on both sides.  Returns how many tokens
    were compared."""
    tokens = [int(t) for t in tokens]
    if dtype == "fp32":
        assert tokens == [int(t) for t in ot.greedy(prompt, len(tokens))]
        return len(tokens)
    tol = LOGIT_TOL[dtype]
    P = len(prompt)
    seq = [int(t) for t in prompt] + tokens[:-1]
    lg = ot.forward(ot.cache(len(seq) + 1), seq, 0)[P - 1:]
    n = 0
    for i, t in enumerate(tokens):
        if top2_margin(lg[i]) <= 2 * tol:
            break
        assert t == int(lg[i].argmax()), (i, t, int(lg[i].argmax()))
        n += 1
    return n
