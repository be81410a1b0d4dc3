"""A speculation length per sequence through the C ABI (spec_set_seq_s): sequence b verifies at most
caps[b] proposals of a round.  Round by round the accepted length must be the first-mismatch rule of Sec. 2
applied to the capped proposals, and the emitted tokens must stay the target's greedy continuation
(the library decoding the same prompts without speculation; the CPU oracle for the fp32 configuration)."""
import numpy as np
import pytest

import synth_inputs as si
from helpers import build_pair, assert_greedy_matches_oracle

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

CASES = {
    "tiny_fp32": dict(dtype="fp32", seed=1000, B=4, P=16, N=20, s=4, alpha=0.8, caps=[0, 4, 2, 1],
                      tgt=si.CONFIGS["tiny_fp32"][2], drf=si.CONFIGS["tiny_fp32"][3]),
    "small_bf16": dict(dtype="bf16", seed=77, B=5, P=21, N=24, s=3, alpha=0.8, caps=[3, 0, 1, 2, 7],
                       tgt=si.llama_desc(2, 256, 2, 416, 1000, 128), drf=si.llama_desc(1, 128, 2, 160, 1000, 128)),
    "small_fp16_opt": dict(dtype="fp16", seed=78, B=3, P=5, N=18, s=5, alpha=0.7, caps=[2, 5, -1],
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


def greedy_reference(ctx, prompts, N):
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    toks, _ = ctx.spec_read_output()
    return [np.array(t) for t in toks]


@pytest.mark.parametrize("name", list(CASES))
def test_capped_rounds_follow_the_acceptance_rule(orc, B, name):
    """External proposals from a table (so the host knows them): every round, every sequence."""
    c = CASES[name]
    nB, P, N, s, caps = c["B"], c["P"], c["N"], c["s"], c["caps"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = P + N + s + 3
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, B.PROPOSALS_EXTERNAL, DEV)
    prompts = si.make_prompts(nB, P, c["tgt"]["vocab"], c["seed"])
    ctx.spec_set_proposal_table(np.zeros((nB, L_max), dtype=np.int32))
    ref = greedy_reference(ctx, prompts, N)
    for b in range(nB):  # the reference itself against the oracle (exact in fp32, margin rule in 16 bits)
        assert_greedy_matches_oracle(ot, prompts[b], ref[b], c["dtype"])
    truth = np.zeros((nB, L_max), dtype=np.int32)
    for b in range(nB):
        truth[b, P:P + N] = ref[b]
    table = si.make_proposal_table(truth, c["alpha"], c["tgt"]["vocab"], c["seed"] + 9)
    ctx.spec_set_proposal_table(table)
    ctx.spec_reset(prompts)
    ctx.spec_set_seq_s(caps)
    n = [P] * nB
    capped = 0
    for rnd in range(2 * N):
        ctx.spec_round(s, 1)
        n_g, _, l_g, a_g = ctx.spec_read_state()
        for b in range(nB):
            sb = min(s, max(0, caps[b]))
            t = [int(table[b][n[b] + j]) for j in range(sb)]
            l, em = orc.accept(t, a_g[b][:sb + 1])
            take = min(l + 1, N - (n[b] - P))
            assert l_g[b] == l, (name, rnd, b, l_g[b], l)
            assert n_g[b] == n[b] + take, (name, rnd, b)
            # would the uncapped rule have accepted more?  then the cap was what stopped it
            if sb < s and l == sb and int(table[b][n[b] + sb]) == a_g[b][sb]:
                capped += 1
            n[b] = n_g[b]
        if min(n) == P + N:
            break
    assert min(n) == P + N
    assert capped > 0, "no round was ever limited by its cap: the test would pass without the feature"
    toks, hist = ctx.spec_read_output()
    for b in range(nB):
        assert np.array_equal(np.array(toks[b]), ref[b]), (name, b)
    # no sequence ever reported more accepted proposals than the largest cap in use
    top = max(min(s, max(0, x)) for x in caps)
    assert sum(hist[top + 1:]) == 0
    # caps off again: plain rounds
    ctx.spec_set_seq_s(None)
    ctx.spec_reset(prompts)
    ctx.spec_round(s, N)
    toks, _ = ctx.spec_read_output()
    for b in range(nB):
        assert np.array_equal(np.array(toks[b]), ref[b])
    ctx.close()


@pytest.mark.parametrize("name", list(CASES))
def test_capped_rounds_with_the_draft_model(orc, B, name):
    """Proposals from the draft model: the draft's cache must stay consistent when some of its steps are
    skipped for a sequence; emitted tokens, and the draft cache length against the committed length."""
    c = CASES[name]
    nB, P, N, s, caps = c["B"], c["P"], c["N"], c["s"], c["caps"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = P + N + s + 3
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, B.PROPOSALS_DRAFT, DEV)
    prompts = si.make_prompts(nB, P, c["tgt"]["vocab"], c["seed"])
    ref = greedy_reference(ctx, prompts, N)
    # the same draft model, uncapped: accepted lengths of the first round, to compare with
    ctx.spec_reset(prompts)
    ctx.spec_round(s, 1)
    _, _, l_free, _ = ctx.spec_read_state()
    ctx.spec_reset(prompts)
    ctx.spec_set_seq_s(caps)
    ctx.spec_round(s, 1)
    n1, kd1, l1, _ = ctx.spec_read_state()
    for b in range(nB):
        sb = min(s, max(0, caps[b]))
        assert l1[b] == min(l_free[b], sb), (name, b, l1[b], l_free[b], sb)   # same proposals, cut at the cap
        assert 1 <= n1[b] - kd1[b] <= 2, (name, b, n1[b], kd1[b])              # the draft is at most two tokens behind
    ctx.spec_round(s, 2 * N)
    toks, _ = ctx.spec_read_output()
    for b in range(nB):
        assert np.array_equal(np.array(toks[b]), ref[b]), (name, b)
    ctx.close()
