"""The draft side of a round -- the call speculate(S, kv_SSM, s) of Alg. 1, s sequential decode steps of the small
model, charged s * t_S(b, 1) in Eq. 3 -- against the CPU oracle, through the C ABI.

The reference for draft step j of a round is the definition, with no cache bookkeeping in it: the draft model's
logits after reading the whole committed sequence plus the proposals t_1..t_{j-1} of that round, recomputed by
the oracle from an empty cache.  The GPU reaches the same through its draft KV cache, a first step that ingests
whatever the cache is behind by (one token, two after a fully accepted round, more after rounds without
speculation), and a roll-back by length; any slip there shows as a logit difference or a wrong cache row.
"""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import LOGIT_TOL, build_pair, top2_margin

pytestmark = pytest.mark.gpu
DEV = "cuda:0"

PAIRS = {
    "tiny_fp32": ("fp32", 1000, si.CONFIGS["tiny_fp32"][2], si.CONFIGS["tiny_fp32"][3]),
    "small_bf16": ("bf16", 77, si.llama_desc(2, 256, 2, 416, 1000, 128), si.llama_desc(1, 128, 2, 160, 1000, 128)),
    "small_fp16_opt": ("fp16", 78, si.opt_desc(2, 256, 4, 384, 777, 128), si.opt_desc(1, 128, 2, 192, 777, 128)),
}


@pytest.fixture(scope="module")
def orc():
    from oracle import oracle as om
    return om.Oracle("f64")


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


def make(orc, B, name, twin, mode, nB, P, N, s_max):
    """twin: the draft is the target itself (same shape, same parameters)."""
    dtype, seed, tdesc, ddesc = PAIRS[name]
    L_max = P + N + s_max + 3
    tdesc = dict(tdesc, max_pos=max(L_max, tdesc["max_pos"]))
    ddesc = dict(tdesc) if twin else dict(ddesc, max_pos=max(L_max, ddesc["max_pos"]))
    ot, od, gt, gd = build_pair(orc, tdesc, ddesc, dtype, seed, DEV, random_norms=True)
    if twin:
        od, gd = ot, gt
    ctx = B.Context(tdesc, gt, ddesc, gd, dtype, nB, s_max, L_max, N, mode, DEV)
    prompts = si.make_prompts(nB, P, tdesc["vocab"], seed)
    return dtype, tdesc, ddesc, ot, od, ctx, prompts, L_max


@pytest.mark.parametrize("name", list(PAIRS))
def test_draft_equal_to_target_gets_every_proposal_accepted(orc, B, name):
    """With the target's own parameters as the draft every proposal is the target's greedy token (a row's bits do
    not depend on the pass it sits in), so every round accepts all s proposals: rounds = ceil(N / (s + 1)) and the
    whole histogram sits at l = s.  A wrong draft position, a stale draft cache row or a first draft step that
    misses a token would cost acceptances here -- and nowhere else, since the output is the greedy one regardless."""
    nB, P, N, s_max = 3, 7, 30, 8
    dtype, tdesc, ddesc, ot, od, ctx, prompts, L_max = make(orc, B, name, True, B.PROPOSALS_DRAFT, nB, P, N, s_max)
    ctx.spec_reset(prompts)
    ctx.spec_round(0, N)
    base, _ = ctx.spec_read_output()
    for s in range(1, s_max + 1):
        rounds = math.ceil(N / (s + 1))
        ctx.spec_reset(prompts)
        ctx.spec_round(s, rounds)
        out, hist = ctx.spec_read_output()
        assert out == base, (name, s)
        assert sum(hist) == nB * rounds
        frac = hist[s] / float(nB * rounds)
        print("%s s=%d: %d rounds, fraction of rounds with l = s: %.3f" % (name, s, rounds, frac))
        if dtype == "fp32":
            assert hist[s] == nB * rounds, (name, s, hist)
        else:
            assert frac >= 0.95, (name, s, hist)
    # the same with rounds without speculation in between (the draft cache falls behind and catches up)
    ctx.spec_reset(prompts)
    for s in [3, 0, 0, 2, 0, 4, 1, 0, 0, 0, 5]:
        ctx.spec_round(s, 1)
    out, hist = ctx.spec_read_output()
    assert all(o == b[:len(o)] for o, b in zip(out, base))
    assert sum(hist[i] for i in (1, 2, 3, 4, 5)) == 5 * nB and hist[0] == 6 * nB, hist
    ctx.close()


SCHEDULE = [2, 4, 0, 3, 0, 0, 4, 1, 3] + [0] * 19 + [4, 2]   # s per round; 19 rounds without draft steps in a row


@pytest.mark.parametrize("name,twin,external", [
    ("tiny_fp32", False, False), ("tiny_fp32", True, False), ("tiny_fp32", False, True),
    ("small_bf16", False, False), ("small_bf16", True, False), ("small_bf16", False, True),
    ("small_fp16_opt", True, False), ("small_fp16_opt", False, True),
])
def test_draft_steps_match_oracle_round_by_round(orc, B, name, twin, external):
    """Every draft step of every round: logits and proposal against the oracle's draft forward over the committed
    sequence plus the round's earlier proposals; after the commit the draft cache rows the length says are valid
    against the oracle's K/V of the committed sequence.  twin (draft = target): all s proposals are accepted, so the
    next round's first draft step has two tokens to ingest; the schedule's runs of s = 0 leave up to 20."""
    nB, P, s_max = 2, 6, 4
    N = sum(s + 1 for s in SCHEDULE)       # never reached: no sequence freezes
    mode = B.PROPOSALS_EXTERNAL if external else B.PROPOSALS_DRAFT
    dtype, tdesc, ddesc, ot, od, ctx, prompts, L_max = make(orc, B, name, twin, mode, nB, P, N, s_max)
    tol = LOGIT_TOL[dtype]
    V = tdesc["vocab"]
    if external:   # the workloads' proposals: the target's greedy continuation with replacements
        ref = np.stack([ot.greedy(p, L_max - P, L_max=L_max + 1) for p in prompts])
        truth = np.zeros((nB, L_max), dtype=np.int32)
        truth[:, P:] = ref
        table = si.make_proposal_table(truth, 0.7, V, 11)
        ctx.spec_set_proposal_table(table)
    ctx.spec_reset(prompts)
    dump = ctx.spec_set_draft_logits(True)
    nl_d = ddesc["n_layers"]
    worst, worst_kv, checked, two_token_rounds, far_behind = 0.0, 0.0, 0, 0, 0
    _, kd_prev, _, _ = ctx.spec_read_state()
    assert list(kd_prev) == [P - 1] * nB
    for rnd, s in enumerate(SCHEDULE):
        out, _ = ctx.spec_read_output()
        S = [list(prompts[b]) + out[b] for b in range(nB)]
        n0, kd0, _, _ = ctx.spec_read_state()
        assert [len(x) for x in S] == list(n0)
        lag = [n0[b] - kd0[b] for b in range(nB)]
        two_token_rounds += int(s > 0 and max(lag) == 2)
        far_behind += int(s > 0 and max(lag) > 16)
        for j in range(1, s + 1):
            ctx.spec_draft_step(j)
            g = dump[:nB].cpu().numpy()
            t = ctx.spec_read_proposals()
            for b in range(nB):
                toks = S[b] + [int(x) for x in t[b][:j - 1]]
                o = od.forward(od.cache(len(toks) + 1), toks, 0)[-1]
                err = np.abs(g[b] - o).max()
                worst = max(worst, err)
                assert err <= tol, (name, rnd, s, j, b, err)
                if not external and top2_margin(o) > 2 * tol:
                    assert t[b][j - 1] == int(o.argmax()), (name, rnd, s, j, b)
                    checked += 1
        ctx.spec_verify_step(s)
        ctx.spec_accept_commit(s)
        n1, kd1, l1, _ = ctx.spec_read_state()
        out, _ = ctx.spec_read_output()
        for b in range(nB):
            assert n1[b] == n0[b] + l1[b] + 1
            if s == 0:
                assert kd1[b] == kd0[b]                       # no draft step: the draft cache is left alone
            else:
                assert n1[b] - 2 <= kd1[b] <= n1[b] - 1       # at most two tokens to ingest next round
            if twin and not external and (dtype == "fp32"):
                assert l1[b] == s
        # the draft cache rows its length says are valid == the oracle's K/V of the committed prefix
        if s > 0:
            Sn = [list(prompts[b]) + out[b] for b in range(nB)]
            kmax = max(kd1)
            for b in range(nB):
                cache = od.cache(kmax + 1)
                od.forward(cache, Sn[b][:kd1[b]], 0, want_logits=False)
                for layer in range(nl_d):
                    K, Vv = ctx.spec_kv_export(B.MODEL_DRAFT, layer, nB, kmax)
                    for got, want in ((K, cache.k(layer)), (Vv, cache.v(layer))):
                        e = np.abs(got[b, :kd1[b]].float().cpu().numpy() - want[:kd1[b]]).max()
                        worst_kv = max(worst_kv, e)
                        assert e < tol, (name, rnd, s, b, layer, e)
    ctx.spec_set_draft_logits(False)
    assert far_behind >= 1
    if twin and not external:
        assert two_token_rounds >= 3
    if not external:
        assert checked > 0
    print("%s twin=%s external=%s: worst draft |logit err| %.3g, worst draft cache err %.3g (tol %g), %d proposals checked"
          % (name, twin, external, worst, worst_kv, tol, checked))
    ctx.close()
