"""Continuous batching through the C ABI (spec_admit): a slot of the running batch starts over with a new
prompt while the other sequences go on.  Greedy speculative decoding must still emit, for every prompt,
exactly the target's own greedy continuation (Sec. 2, Alg. 1: the output does not depend on the proposals),
whatever was admitted when; checked against the same library decoding each prompt without speculation, and
for the fp32 configuration against the CPU oracle."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from helpers import build_pair, assert_greedy_matches_oracle

pytestmark = pytest.mark.gpu

DEV = "cuda:0"

CASES = {
    "tiny_fp32": dict(dtype="fp32", seed=1000, B=3, P=16, N=20, s=4, alpha=0.7,
                      tgt=si.CONFIGS["tiny_fp32"][2], drf=si.CONFIGS["tiny_fp32"][3]),
    "small_bf16": dict(dtype="bf16", seed=77, B=4, P=21, N=24, s=3, alpha=0.7,
                       tgt=si.llama_desc(2, 256, 2, 416, 1000, 128), drf=si.llama_desc(1, 128, 2, 160, 1000, 128)),
    # a prompt longer than the pass has rows: two groups of 16 rows of the one sequence in the first pass
    # (they share the slot's cache), a ragged second pass
    "small_bf16_long": dict(dtype="bf16", seed=83, B=4, P=43, N=14, s=7, alpha=0.7,
                            tgt=si.llama_desc(2, 256, 4, 416, 1000, 128), drf=si.llama_desc(1, 128, 2, 160, 1000, 128)),
    "small_fp16_opt": dict(dtype="fp16", seed=78, B=3, P=5, N=18, s=5, alpha=0.6,
                           tgt=si.opt_desc(2, 256, 4, 384, 777, 64), drf=si.opt_desc(1, 128, 2, 192, 777, 64)),
}
EXTRA = 3  # prompts admitted later


@pytest.fixture(scope="module")
def orc():
    from oracle import oracle as om
    return om.Oracle("f64")


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


def greedy_reference(ctx, prompts, nB, N):
    """The library's own non-speculative decode of every prompt, nB at a time."""
    out = []
    for lo in range(0, len(prompts), nB):
        part = prompts[lo:lo + nB]
        ctx.spec_reset(part)
        ctx.spec_round(0, N)
        toks, _ = ctx.spec_read_output()
        assert all(len(toks[b]) == N for b in range(len(part)))
        out.extend(np.array(toks[b]) for b in range(len(part)))
    return out


@pytest.mark.parametrize("mode", ["table", "draft"])
@pytest.mark.parametrize("name", list(CASES))
def test_admitted_sequences_decode_as_if_alone(orc, B, name, mode):
    c = CASES[name]
    nB, P, N, s = c["B"], c["P"], c["N"], c["s"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = P + N + s + 3
    pmode = B.PROPOSALS_EXTERNAL if mode == "table" else B.PROPOSALS_DRAFT
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, pmode, DEV)
    prompts = si.make_prompts(nB + EXTRA, P, c["tgt"]["vocab"], c["seed"])
    if mode == "table":
        ctx.spec_set_proposal_table(np.zeros((nB, L_max), dtype=np.int32))  # unused at s = 0
    ref = greedy_reference(ctx, prompts, nB, N)
    for i, p in enumerate(prompts):  # the reference itself against the oracle (exact in fp32, margin rule in 16 bits)
        assert_greedy_matches_oracle(ot, p, ref[i], c["dtype"])

    # which prompt sits in which slot, and the proposals that go with it (its greedy continuation with
    # a share of the tokens replaced)
    owner = list(range(nB))

    def set_table():
        if mode != "table":
            return
        truth = np.zeros((nB, L_max), dtype=np.int32)
        for b in range(nB):
            truth[b, P:P + N] = ref[owner[b]]
        ctx.spec_set_proposal_table(si.make_proposal_table(truth, c["alpha"], c["tgt"]["vocab"], c["seed"] + 5))

    def admit(b, i):
        owner[b] = i
        ctx.spec_admit(b, prompts[i])
        set_table()

    def check(slots):
        toks, _ = ctx.spec_read_output()
        for b in slots:
            assert len(toks[b]) == N, (b, len(toks[b]))
            assert np.array_equal(np.array(toks[b]), ref[owner[b]]), (name, mode, b, owner[b])

    def prompt_kv(slot):
        """Cached keys and values of a slot's prompt, first and last layer of both models."""
        out = []
        for which, desc in ((B.MODEL_TARGET, c["tgt"]), (B.MODEL_DRAFT, c["drf"])):
            for layer in sorted({0, desc["n_layers"] - 1}):
                K, V = ctx.spec_kv_export(which, layer, nB, P - 1)
                out += [K[slot].clone(), V[slot].clone()]
        return out

    # what a plain reset leaves in slot 1 for the prompt that will be admitted there
    first = [prompts[b] for b in range(nB)]
    first[1] = prompts[nB]
    ctx.spec_reset(np.stack(first))
    kv_reset = prompt_kv(1)

    set_table()
    ctx.spec_reset(prompts[:nB])
    ctx.spec_round(s, 2)
    admit(1, nB)                  # a sequence in mid-flight is replaced
    # the single-sequence prefill leaves the same bits in both caches as the batch prefill does
    for got, want in zip(prompt_kv(1), kv_reset):
        assert torch.equal(got, want)
    ctx.spec_round(s, 3)
    admit(0, nB + 1)              # and another, a few rounds later
    ctx.spec_round(s, N)          # more rounds than anyone needs: finished sequences stay as they are
    check(range(nB))
    n_before, _, _, _ = ctx.spec_read_state()
    admit(nB - 1, nB + 2)         # a finished sequence leaves, a new one takes its slot
    ctx.spec_round(s, N)
    check(range(nB))
    n_after, _, _, _ = ctx.spec_read_state()
    assert list(n_after) == list(n_before)
    ctx.close()


RAGGED = {
    # admitted prompts shorter and longer than the batch's; the longest needs two prefill passes of its own
    "tiny_fp32": dict(lengths=[5, 23, 1]),
    "small_bf16": dict(lengths=[9, 40, 21]),
    "small_fp16_opt": dict(lengths=[12, 2, 7]),
}


@pytest.mark.parametrize("mode", ["table", "draft"])
@pytest.mark.parametrize("name", list(RAGGED))
def test_admitted_prompts_of_other_lengths(orc, B, name, mode):
    """Every slot keeps its own prompt length: emitted tokens are the greedy continuation of that prompt
    (the library decoding it alone, without speculation; the CPU oracle for fp32), the admitted prompt's
    cache rows equal those of a reset with that prompt, and a rewind takes every slot back to its own prompt."""
    c = CASES[name]
    nB, P, N, s = c["B"], c["P"], c["N"], c["s"]
    lengths = RAGGED[name]["lengths"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = max(P, max(lengths)) + N + s + 3
    pmode = B.PROPOSALS_EXTERNAL if mode == "table" else B.PROPOSALS_DRAFT
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, pmode, DEV)
    vocab = c["tgt"]["vocab"]
    base = si.make_prompts(nB, P, vocab, c["seed"])
    extra = [si.make_prompts(1, L, vocab, c["seed"] + 100 + i)[0] for i, L in enumerate(lengths)]
    if mode == "table":
        ctx.spec_set_proposal_table(np.zeros((nB, L_max), dtype=np.int32))
    ref_base = greedy_reference(ctx, base, nB, N)
    ref_extra, kv_extra = [], []
    for p in extra:                      # each admitted prompt alone: its continuation and its cache rows
        ctx.spec_reset(p[None, :])
        kv = []
        if len(p) > 1:
            for which, desc in ((B.MODEL_TARGET, c["tgt"]), (B.MODEL_DRAFT, c["drf"])):
                K, V = ctx.spec_kv_export(which, desc["n_layers"] - 1, 1, len(p) - 1)
                kv += [K[0].clone(), V[0].clone()]
        kv_extra.append(kv)
        ctx.spec_round(0, N)
        toks, _ = ctx.spec_read_output()
        ref_extra.append(np.array(toks[0]))
        assert_greedy_matches_oracle(ot, p, ref_extra[-1], c["dtype"])

    owner = [("base", b) for b in range(nB)]

    def prompt_of(o):
        return base[o[1]] if o[0] == "base" else extra[o[1]]

    def ref_of(o):
        return ref_base[o[1]] if o[0] == "base" else ref_extra[o[1]]

    def set_table():
        if mode != "table":
            return
        truth = np.zeros((nB, L_max), dtype=np.int32)
        for b in range(nB):
            Pb = len(prompt_of(owner[b]))
            truth[b, Pb:Pb + N] = ref_of(owner[b])
        ctx.spec_set_proposal_table(si.make_proposal_table(truth, c["alpha"], vocab, c["seed"] + 5))

    def admit(b, i):
        owner[b] = ("extra", i)
        ctx.spec_admit(b, extra[i])
        set_table()

    def check():
        toks, _ = ctx.spec_read_output()
        n, _, _, _ = ctx.spec_read_state()
        for b in range(nB):
            assert np.array_equal(np.array(toks[b]), ref_of(owner[b])), (name, mode, b, owner[b])
            assert n[b] == len(prompt_of(owner[b])) + N

    set_table()
    ctx.spec_reset(base)
    ctx.spec_round(s, 2)
    admit(0, 0)
    admit(nB - 1, 1)
    if len(extra[1]) > 1:                # same cache bits as the single-sequence reset left
        got = []
        for which, desc in ((B.MODEL_TARGET, c["tgt"]), (B.MODEL_DRAFT, c["drf"])):
            K, V = ctx.spec_kv_export(which, desc["n_layers"] - 1, nB, len(extra[1]) - 1)
            got += [K[nB - 1], V[nB - 1]]
        for g, w in zip(got, kv_extra[1]):
            assert torch.equal(g, w)
    ctx.spec_round(s, 3)
    admit(1, 2)
    ctx.spec_round(s, N)
    check()
    # back to "prompts just given", each slot to its own prompt, and the same tokens again
    ctx.spec_rewind()
    n, _, _, _ = ctx.spec_read_state()
    assert list(n) == [len(prompt_of(o)) for o in owner]
    ctx.spec_round(s, N)
    check()
    # a new batch forgets the admitted lengths
    ctx.spec_reset(base)
    owner[:] = [("base", b) for b in range(nB)]
    set_table()
    ctx.spec_round(s, N)
    check()
    ctx.close()


@pytest.mark.parametrize("mode", ["table", "draft"])
@pytest.mark.parametrize("name", list(RAGGED))
def test_batch_of_prompts_of_different_lengths(orc, B, name, mode):
    """spec_reset_ragged: one batch prefill over prompts of different lengths.  Every sequence emits the greedy
    continuation of its own prompt (the library decoding it alone; the CPU oracle for fp32) and its prompt's
    cache rows carry the bits a reset with that prompt alone leaves."""
    c = CASES[name]
    N, s = c["N"], c["s"]
    lengths = RAGGED[name]["lengths"] + [c["P"]]
    nB = len(lengths)
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    L_max = max(lengths) + N + s + 3
    pmode = B.PROPOSALS_EXTERNAL if mode == "table" else B.PROPOSALS_DRAFT
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, L_max, N, pmode, DEV)
    vocab = c["tgt"]["vocab"]
    prompts = [si.make_prompts(1, L, vocab, c["seed"] + 200 + i)[0] for i, L in enumerate(lengths)]
    if mode == "table":
        ctx.spec_set_proposal_table(np.zeros((nB, L_max), dtype=np.int32))
    ref, kv_ref = [], []
    last = {B.MODEL_TARGET: c["tgt"]["n_layers"] - 1, B.MODEL_DRAFT: c["drf"]["n_layers"] - 1}
    for p in prompts:
        ctx.spec_reset(p[None, :])
        kv = []
        if len(p) > 1:
            for which in (B.MODEL_TARGET, B.MODEL_DRAFT):
                K, V = ctx.spec_kv_export(which, last[which], 1, len(p) - 1)
                kv += [K[0].clone(), V[0].clone()]
        kv_ref.append(kv)
        ctx.spec_round(0, N)
        toks, _ = ctx.spec_read_output()
        ref.append(np.array(toks[0]))
        assert_greedy_matches_oracle(ot, p, ref[-1], c["dtype"])
    if mode == "table":
        truth = np.zeros((nB, L_max), dtype=np.int32)
        for b in range(nB):
            truth[b, lengths[b]:lengths[b] + N] = ref[b]
        ctx.spec_set_proposal_table(si.make_proposal_table(truth, c["alpha"], vocab, c["seed"] + 5))

    ctx.spec_reset_ragged(prompts)
    n, _, _, _ = ctx.spec_read_state()
    assert list(n) == lengths
    for b in range(nB):
        if lengths[b] > 1:
            got = []
            for which in (B.MODEL_TARGET, B.MODEL_DRAFT):
                K, V = ctx.spec_kv_export(which, last[which], nB, lengths[b] - 1)
                got += [K[b], V[b]]
            for g, w in zip(got, kv_ref[b]):
                assert torch.equal(g, w), (name, mode, b)
    for attempt in range(2):             # the second time after a rewind to the prompts
        ctx.spec_round(s, N)
        toks, _ = ctx.spec_read_output()
        n, _, _, _ = ctx.spec_read_state()
        for b in range(nB):
            assert np.array_equal(np.array(toks[b]), ref[b]), (name, mode, attempt, b)
            assert n[b] == lengths[b] + N
        ctx.spec_rewind()
        n, _, _, _ = ctx.spec_read_state()
        assert list(n) == lengths
    # refused: a length outside 1..stride
    rows = torch.zeros((2, 4), dtype=torch.int32, device=DEV)
    import ctypes as C
    for bad in ([0, 4], [5, 1]):
        rc = B.lib.spec_reset_ragged(ctx.h, 2, C.c_void_p(rows.data_ptr()), 4, (C.c_int32 * 2)(*bad))
        assert rc == B.ERR_INVALID_ARG
    ctx.close()


def test_admit_is_refused_where_it_cannot_work(orc, B):
    c = CASES["tiny_fp32"]
    nB, P, N, s = c["B"], c["P"], c["N"], c["s"]
    ot, od, gt, gd = build_pair(orc, c["tgt"], c["drf"], c["dtype"], c["seed"], DEV)
    ctx = B.Context(c["tgt"], gt, c["drf"], gd, c["dtype"], nB, s, P + N + s + 3, N, B.PROPOSALS_DRAFT, DEV)
    prompts = si.make_prompts(nB, P, c["tgt"]["vocab"], c["seed"])
    with pytest.raises(B.SpecError):
        ctx.spec_admit(0, prompts[0])          # no batch yet
    ctx.spec_reset(prompts)
    for bad in (-1, nB):
        with pytest.raises(B.SpecError):
            ctx.spec_admit(bad, prompts[0])    # slot out of range
    with pytest.raises(B.SpecError):           # P + gen_max + s_max would not fit into L_max
        ctx.spec_admit(0, si.make_prompts(1, P + 4, c["tgt"]["vocab"], 5)[0])
    with pytest.raises(B.SpecError):
        ctx.spec_admit(0, np.zeros(0, dtype=np.int32))   # an empty prompt
    ctx.spec_admit(0, si.make_prompts(1, P + 3, c["tgt"]["vocab"], 5)[0])   # the longest that fits
    ctx.spec_draft_step(1)
    with pytest.raises(B.SpecError):
        ctx.spec_admit(0, prompts[0])          # inside a round
    ctx.close()
