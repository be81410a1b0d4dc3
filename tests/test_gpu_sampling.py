"""Speculative sampling (the non-greedy acceptance rule that Sec. 2 cites) on the GPU against the numpy oracle,
through the C ABI.

The GPU decides in fp32, the oracle in fp64, and a decision is an integer: where the oracle reports that the random
number fell within MARGIN of a decision boundary, either outcome is legitimate and that row or sequence is left out
of the comparison (and counted: the share must stay tiny).  Everything else must agree exactly.
"""
import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import build_pair, truth_table
from oracle import sampling as osm

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
MARGIN = 1e-5   # fp32 sums over a vocabulary, added chunk by chunk: the cumulative weights are good to about 1e-6 of the total


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


@pytest.mark.parametrize("V,T", [(32000, 0.7), (32000, 1.3), (50272, 1.0), (1003, 0.9), (37, 1.0), (5, 2.0)])
def test_token_draws_match_the_oracle(B, V, T):
    rng = np.random.default_rng(V)
    rows = 48
    z = _peaky(rng, (rows, V))
    u = rng.random(rows).astype(np.float32)
    u[0], u[1] = 0.0, np.float32(1.0 - 2 ** -24)      # the ends of the range
    got = B.spec_sample_tokens(torch.from_numpy(z).to(DEV), torch.from_numpy(u).to(DEV), T).cpu().numpy()
    skipped = 0
    for r in range(rows):
        tok, margin = osm.sample_token(z[r], T, float(u[r]))
        if margin < MARGIN:
            skipped += 1
            continue
        assert got[r] == tok, (r, got[r], tok, margin)
    assert skipped <= 4


def _peaky(rng, shape):
    """Logits with the shape of a language model's: a broad bulk and a few tokens far above it that carry the mass
    (with a flat distribution over 32000 tokens most draws land within rounding of a boundary and say nothing)."""
    z = rng.normal(size=shape) * 2.0
    z += (rng.random(shape) < 24.0 / shape[-1]) * rng.uniform(8.0, 14.0, size=shape)
    return z.astype(np.float32)


def _round_inputs(rng, nB, s, V, point_mass, T):
    tl = _peaky(rng, (nB, s + 1, V))
    u = rng.random((nB, s + 1, 3)).astype(np.float32)
    if point_mass:
        dl = None
        props = np.where(rng.random((nB, s)) < 0.6, tl[:, :s].argmax(-1), rng.integers(V, size=(nB, s))).astype(np.int32)
    else:
        # a draft near the target, so that keeping and rejecting both happen; step-major as the entry point wants it
        dl = (tl[:, :s] + rng.normal(size=(nB, s, V)) * 1.2).astype(np.float32).transpose(1, 0, 2).copy()
        props = np.array([[osm.sample_token(dl[j, b], T, float(u[b, j, 0]))[0] for j in range(s)] for b in range(nB)],
                         dtype=np.int32).reshape(nB, s)
    return tl, dl, props, u


@pytest.mark.parametrize("V", [32000, 1003])
@pytest.mark.parametrize("s", [0, 1, 4, 8])
@pytest.mark.parametrize("point_mass", [False, True])
def test_acceptance_rule_matches_the_oracle(B, V, s, point_mass):
    rng = np.random.default_rng(1000 * s + V + point_mass)
    nB, T = 40, 0.9
    tl, dl, props, u = _round_inputs(rng, nB, s, V, point_mass, T)
    dev = lambda a: None if a is None else torch.from_numpy(a).to(DEV)
    chosen, acc, em = B.spec_sample_accept(dev(tl), dev(dl) if s else None, dev(props) if s else None, dev(u), T)
    chosen, acc, em = chosen.cpu().numpy(), acc.cpu().numpy(), em.cpu().numpy()
    skipped, ls = 0, []
    for b in range(nB):
        l, emitted, margin = osm.spec_sample_round(tl[b], None if dl is None else dl[:, b], props[b], u[b, :s, 1], u[b, :, 2], T)
        if margin < MARGIN:
            skipped += 1
            continue
        ls.append(l)
        assert acc[b] == l, (b, acc[b], l, margin)
        assert list(em[b, :l + 1]) == emitted and all(x == -1 for x in em[b, l + 1:]), (b, em[b], emitted)
        assert list(chosen[b, :l + 1]) == emitted
    assert skipped <= 4
    if s >= 4:
        assert 0 < np.mean(ls) < s, "the inputs should exercise both keeping and rejecting"


def test_identical_draft_keeps_everything_and_bad_arguments_are_refused(B):
    rng = np.random.default_rng(5)
    nB, s, V, T = 16, 5, 2048, 1.1
    tl = (rng.normal(size=(nB, s + 1, V)) * 2).astype(np.float32)
    dl = tl[:, :s].transpose(1, 0, 2).copy()
    u = rng.random((nB, s + 1, 3)).astype(np.float32)
    props = np.array([[osm.sample_token(dl[j, b], T, float(u[b, j, 0]))[0] for j in range(s)] for b in range(nB)], dtype=np.int32)
    dev = lambda a: torch.from_numpy(a).to(DEV)
    _, acc, em = B.spec_sample_accept(dev(tl), dev(dl), dev(props), dev(u), T)
    assert acc.cpu().tolist() == [s] * nB          # p = q bit for bit: the ratio is 1, every u < 1 keeps
    assert np.array_equal(em.cpu().numpy()[:, :s], props)
    with pytest.raises(B.SpecError):
        B.spec_sample_accept(dev(tl), dev(dl), dev(props), dev(u), 0.0)
    with pytest.raises(B.SpecError):
        B.spec_sample_tokens(dev(tl[:, 0]), dev(u[:, 0, 0].copy()), -1.0)


PAIRS = {
    "tiny_fp32": ("fp32", 1000, si.CONFIGS["tiny_fp32"][2], si.CONFIGS["tiny_fp32"][3]),
    "small_bf16": ("bf16", 77, si.llama_desc(2, 256, 2, 416, 1000, 128), si.llama_desc(1, 128, 2, 160, 1000, 128)),
}


def _context(B, name, mode, nB, P, N, s_max, twin=False):
    from oracle import oracle as om
    dtype, seed, tdesc, ddesc = PAIRS[name]
    L_max = P + N + s_max + 3
    tdesc = dict(tdesc, max_pos=max(L_max, tdesc["max_pos"]))
    ddesc = dict(tdesc) if twin else dict(ddesc, max_pos=max(L_max, ddesc["max_pos"]))
    ot, od, gt, gd = build_pair(om.Oracle("f64"), tdesc, ddesc, dtype, seed, DEV, random_norms=True, emb_std=1.0)
    if twin:
        gd = gt
    ctx = B.Context(tdesc, gt, ddesc, gd, dtype, nB, s_max, L_max, N, mode, DEV)
    return ctx, si.make_prompts(nB, P, tdesc["vocab"], seed), L_max, tdesc["vocab"]


@pytest.mark.parametrize("name", list(PAIRS))
@pytest.mark.parametrize("mode", ["draft", "table", "draft_caps"])
def test_rounds_inside_a_context_follow_the_rule_on_their_own_logits(B, name, mode):
    """Sampling switched on in a context: every round's proposals, acceptance count and committed tokens must be
    what the oracle's rule gives on the logits the GPU itself produced in that round (the library leaves them in the
    caller's buffers) and the caller's table of uniform numbers, indexed by sequence and absolute position.  This
    checks the wiring -- which random number decides which token, which draft step's logits meet which target row,
    the hand-over to the commit step -- independently of the models' numerics."""
    nB, P, N, s_max = 5, 9, 40, 4
    T = 0.9 if mode != "table" else 0.2
    ctx, prompts, L_max, V = _context(B, name, B.PROPOSALS_DRAFT if mode != "table" else B.PROPOSALS_EXTERNAL, nB, P, N, s_max)
    rng = np.random.default_rng(3)
    u = rng.random((nB, L_max, 3)).astype(np.float32)
    ctx.spec_reset(prompts)
    if mode == "table":
        # the table holds the target's greedy continuation: at a low temperature the sampled sequences follow it for
        # a while, so proposals are kept as well as rejected
        ctx.spec_round(0, N)
        greedy, _ = ctx.spec_read_output()
        ctx.spec_set_proposal_table(truth_table(np.array(greedy), P, L_max))
        ctx.spec_reset(prompts)
    caps = None
    if mode == "draft_caps":   # a speculation length per sequence: the bonus draw moves to row s_b
        mode, caps = "draft", [0, 1, 2, 3, 4]
        ctx.spec_set_seq_s(caps)
    tl, dl = ctx.spec_set_sampling(T, torch.from_numpy(u).to(DEV))
    skipped, ls, checked = 0, [], 0
    for rnd, s in enumerate([3, 4, 1, 0, 2, 4, 3, 3]):
        n0 = list(ctx.spec_read_state()[0])
        out0, _ = ctx.spec_read_output()
        ctx.spec_round(s, 1)
        n1, _, l_last, _ = ctx.spec_read_state()
        out1, _ = ctx.spec_read_output()
        props = ctx.spec_read_proposals()
        tln = tl[:nB * (s + 1)].view(nB, s + 1, V).cpu().numpy()
        dln = dl.cpu().numpy() if mode == "draft" else None
        s_round = s
        for b in range(nB):
            s = min(s_round, caps[b]) if caps else s_round
            ub = u[b, n0[b]:n0[b] + s + 1]
            margin = 1.0
            if mode == "draft":
                for j in range(s):
                    tok, m = osm.sample_token(dln[j, b], T, float(ub[j, 0]))
                    margin = min(margin, m)
                    if margin >= MARGIN:
                        assert props[b][j] == tok, (rnd, b, j)
            l, emitted, m = osm.spec_sample_round(tln[b][:s + 1], None if dln is None else dln[:s, b], props[b][:s], ub[:s, 1],
                                                  ub[:, 2], T)
            if min(margin, m) < MARGIN:
                skipped += 1
                continue
            checked += 1
            ls.append(l / max(1, s))
            assert l_last[b] == l and n1[b] - n0[b] == l + 1, (rnd, b, l_last[b], l, n1[b] - n0[b])
            assert out1[b][len(out0[b]):] == emitted, (rnd, b)
    assert skipped <= 3 and checked >= 30
    assert 0.0 < np.mean(ls) < 1.0, "the rounds should exercise both keeping and rejecting"
    # back to the greedy rule: the next round's tokens are the arg-max of their rows again
    ctx.spec_set_sampling(0.0, None)
    if caps:
        ctx.spec_set_seq_s(None)
    lg = None
    out0, _ = ctx.spec_read_output()
    if mode == "draft":
        for j in range(1, 3):
            ctx.spec_draft_step(j)
    lg = ctx.spec_verify_step(2, want_logits=True).cpu().numpy()
    a = ctx.spec_read_state()[3]
    assert [list(r[:3]) for r in a] == [list(lg[b].argmax(-1)) for b in range(nB)]
    ctx.spec_accept_commit(2)
    ctx.close()


@pytest.mark.parametrize("name", list(PAIRS))
def test_draft_equal_to_target_keeps_every_proposal_when_sampling(B, name):
    """The draft is the target: a row's bits do not depend on the pass it sits in, so q = p bit for bit, the ratio is
    1 and every proposal is kept whatever the random numbers -- any slip in which draft step's logits meet which
    target row would break it."""
    nB, P, N, s_max, T = 4, 8, 36, 5, 1.0
    ctx, prompts, L_max, V = _context(B, name, B.PROPOSALS_DRAFT, nB, P, N, s_max, twin=True)
    rng = np.random.default_rng(4)
    ctx.spec_reset(prompts)
    ctx.spec_set_sampling(T, torch.from_numpy(rng.random((nB, L_max, 3)).astype(np.float32)).to(DEV))
    for s in (5, 3, 4, 1, 5):
        ctx.spec_round(s, 1)
        assert list(ctx.spec_read_state()[2]) == [s] * nB
    ctx.close()
