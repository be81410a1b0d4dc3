"""spec_greedy_accept: greedy tokens and the acceptance rule of Sec. 2 on logits the caller supplies, against
numpy's arg-max and the oracle's acceptance rule, bit-exactly (integer work)."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth_inputs as si

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_case(nB, s, V, seed, alpha=0.7):
    """Logits ~ N(0, 1) with planted ties and a planted winner per row; proposals agree with the row's arg-max
    with probability alpha (the workloads' replacement scheme)."""
    g = torch.Generator(device="cpu").manual_seed(seed)
    lg = torch.randn((nB, s + 1, V), generator=g, dtype=torch.float32)
    rng = np.random.default_rng(seed)
    win = rng.integers(0, V, size=(nB, s + 1))
    for b in range(nB):
        for i in range(s + 1):
            lg[b, i, win[b, i]] = 9.0
            if (b + i) % 3 == 0:                       # a tie further up the vocabulary: the lower index must win
                lg[b, i, min(V - 1, win[b, i] + 1 + (7 * b + i) % max(1, V - win[b, i] - 1))] = 9.0
    a = lg.numpy().argmax(-1)                           # numpy: first maximum = lowest index
    truth = np.zeros((nB, s + 1), dtype=np.int32)
    truth[:, :s] = a[:, :s]
    t = si.make_proposal_table(truth, alpha, V, seed)[:, :s].astype(np.int32)
    return lg, a, t


@pytest.mark.parametrize("nB,s,V", [(1, 0, 17), (3, 4, 1000), (64, 8, 32000), (5, 15, 50272), (2, 3, 4096), (2, 2, 4097),
                                     (7, 1, 151936)])
def test_greedy_accept_matches_numpy_argmax_and_oracle_rule(nB, s, V):
    from oracle import oracle as om
    from paper_2310_18813_amd import binding as B
    orc = om.Oracle("f64")
    lg, a, t = make_case(nB, s, V, 100 + nB + s)
    acc, em = B.spec_greedy_accept(lg.to(DEV), torch.from_numpy(t).to(DEV) if s else None)
    acc, em = acc.cpu().numpy(), em.cpu().numpy()
    for b in range(nB):
        l, out = orc.accept([int(x) for x in t[b]], [int(x) for x in a[b]])
        assert acc[b] == l, (b, acc[b], l)
        assert list(em[b, :l + 1]) == out and all(x == -1 for x in em[b, l + 1:]), (b, em[b], out)


def test_greedy_accept_rejects_bad_arguments():
    from paper_2310_18813_amd import binding as B
    lg = torch.zeros((2, 3, 100), dtype=torch.float32, device=DEV)
    t = torch.zeros((2, 2), dtype=torch.int32, device=DEV)
    out = torch.zeros((2, 4), dtype=torch.int32, device=DEV)
    ws = torch.zeros(8, dtype=torch.uint8, device=DEV)
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    p = lambda x: C.c_void_p(x.data_ptr())
    assert B.lib.spec_greedy_accept(st, p(lg), p(t), 2, 2, 100, p(ws), 8, p(out), p(out)) == B.ERR_WORKSPACE
    assert B.lib.spec_greedy_accept(st, p(lg), None, 2, 2, 100, p(ws), 1 << 20, p(out), p(out)) == B.ERR_INVALID_ARG
    assert B.lib.spec_greedy_accept(st, p(lg), p(t), 2, 16, 100, p(ws), 1 << 20, p(out), p(out)) == B.ERR_CAPACITY
    assert b"spec_greedy_accept" in B.lib.spec_last_error(None)
