"""An end-of-sequence token through the C ABI (spec_set_eos).  By definition the output of a sequence is the
target's greedy continuation of its prompt up to and including the first end token (or gen_max tokens if none
comes): the expected tokens are the library's own non-speculative decode (the CPU oracle's for fp32), cut there.
Speculation must not change that, whichever round the end token falls into and wherever in the round."""
import numpy as np
import pytest

import synth_inputs as si
from helpers import build_pair, assert_greedy_matches_oracle

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

CASES = {
    "tiny_fp32": dict(dtype="fp32", seed=1000, B=4, P=16, N=24, s=4, alpha=0.8,
                      tgt=si.CONFIGS["tiny_fp32"][2], drf=si.CONFIGS["tiny_fp32"][3]),
    "small_bf16": dict(dtype="bf16", seed=77, B=5, P=21, N=24, s=3, alpha=0.8,
                       tgt=si.llama_desc(2, 256, 2, 416, 1000, 128), drf=si.llama_desc(1, 128, 2, 160, 1000, 128)),
    "small_fp16_opt": dict(dtype="fp16", seed=78, B=3, P=5, N=18, s=5, alpha=0.7,
                           tgt=si.opt_desc(2, 256, 4, 384, 777, 64), drf=si.opt_desc(1, 128, 2, 192, 777, 64)),
}


@pytest.fixture(scope="module")
def orc():
    from oracle import oracle as om
    return om.Oracle("f64")


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


def cut(tokens, eos):
    """Up to and including the first end token."""
    hit = np.nonzero(np.asarray(tokens) == eos)[0]
    return np.asarray(tokens) if len(hit) == 0 else np.asarray(tokens)[:hit[0] + 1]


@pytest.mark.parametrize("mode", ["table", "draft"])
@pytest.mark.parametrize("name", list(CASES))
def test_sequences_stop_at_the_end_token(orc, B, name, mode):
    c = CASES[name]
    nB, P, N, s = c["B"], c["P"], c["N"], c["s"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = P + N + s + 3
    pmode = B.PROPOSALS_EXTERNAL if mode == "table" else B.PROPOSALS_DRAFT
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, pmode, DEV)
    vocab = c["tgt"]["vocab"]
    prompts = si.make_prompts(nB, P, vocab, c["seed"])
    if mode == "table":
        ctx.spec_set_proposal_table(np.zeros((nB, L_max), dtype=np.int32))
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    toks, _ = ctx.spec_read_output()
    ref = [np.array(t) for t in toks]
    for b in range(nB):  # the reference itself against the oracle (exact in fp32, margin rule in 16 bits)
        assert_greedy_matches_oracle(ot, prompts[b], ref[b], c["dtype"])
    if mode == "table":
        truth = np.zeros((nB, L_max), dtype=np.int32)
        for b in range(nB):
            truth[b, P:P + N] = ref[b]
        ctx.spec_set_proposal_table(si.make_proposal_table(truth, c["alpha"], vocab, c["seed"] + 5))

    # end tokens taken from the continuations themselves: early, in the middle, the very first token, and one
    # that no sequence emits
    absent = next(t for t in range(vocab) if all(t not in r for r in ref))
    stops = 0
    for eos in (int(ref[0][3]), int(ref[1][N // 2]), int(ref[nB - 1][0]), int(ref[0][N - 1]), absent):
        want = [cut(r, eos) for r in ref]
        for s_round in (s, 0, 1):
            ctx.spec_set_eos(eos)
            ctx.spec_reset(prompts)
            ctx.spec_round(s_round, N + 2)       # more rounds than anyone needs
            toks, _ = ctx.spec_read_output()
            n, _, _, _ = ctx.spec_read_state()
            for b in range(nB):
                assert np.array_equal(np.array(toks[b]), want[b]), (name, mode, eos, s_round, b)
                assert n[b] == P + len(want[b])
            stops += sum(len(w) < N for w in want)
            # a stopped sequence stays stopped when the end token is taken away; a rewind revives it
            ctx.spec_set_eos(None)
            ctx.spec_round(s_round, 2)
            n2, _, _, _ = ctx.spec_read_state()
            for b in range(nB):
                if len(want[b]) < N:
                    assert n2[b] == n[b]
            ctx.spec_rewind()
            ctx.spec_round(s_round, N)
            toks, _ = ctx.spec_read_output()
            for b in range(nB):
                assert np.array_equal(np.array(toks[b]), ref[b])
    assert stops > 0

    # a slot that stopped at its end token takes a new prompt and decodes it to its own end
    eos = int(ref[0][3])
    ctx.spec_set_eos(eos)
    ctx.spec_reset(prompts)
    ctx.spec_round(s, N)
    ctx.spec_admit(0, prompts[1])
    if mode == "table":
        truth[0] = truth[1]
        ctx.spec_set_proposal_table(si.make_proposal_table(truth, c["alpha"], vocab, c["seed"] + 5))
    ctx.spec_round(s, N)
    toks, _ = ctx.spec_read_output()
    assert np.array_equal(np.array(toks[0]), cut(ref[1], eos))
    assert np.array_equal(np.array(toks[1]), cut(ref[1], eos))

    with pytest.raises(B.SpecError):
        ctx.spec_set_eos(vocab)
    with pytest.raises(B.SpecError):
        ctx.spec_set_eos(-2)
    ctx.spec_set_eos(None)
    ctx.spec_reset(prompts)
    ctx.spec_draft_step(1) if mode == "draft" else ctx.spec_verify_step(0)
    with pytest.raises(B.SpecError):
        ctx.spec_set_eos(1)                       # inside a round
    ctx.close()
