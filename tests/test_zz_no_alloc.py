"""spec_greedy_accept_noalloc (the entry point for callers that cannot allocate: its arg-max partials live in an
array built into the library) against spec_greedy_accept (the same kernels on a caller's workspace), through the
C ABI: identical integers on two calls in a row, the second with a smaller input, so the second call runs over
what the first left in the shared scratch."""
import ctypes as C

import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_pair(B, nB, s, V, seed):
    g = torch.Generator(device="cpu").manual_seed(seed)
    lg = torch.randn((nB, s + 1, V), generator=g, dtype=torch.float32)
    a = lg.numpy().argmax(-1)
    rng = np.random.default_rng(seed)
    t = np.where(rng.random((nB, max(s, 1))) < 0.7, a[:, :max(s, 1)], rng.integers(0, V, size=(nB, max(s, 1))))
    t = torch.from_numpy(t[:, :s].astype(np.int32)).contiguous().to(DEV) if s else None
    lg = lg.to(DEV)
    acc0, em0 = B.spec_greedy_accept(lg, t)
    acc1 = torch.full((nB,), -7, dtype=torch.int32, device=DEV)
    em1 = torch.full((nB, s + 1), -7, dtype=torch.int32, device=DEV)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(DEV)
    B.spec_greedy_accept(lg, t, accepted=acc1, emitted=em1, noalloc=True)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated(DEV) == before
    assert torch.equal(acc0, acc1) and torch.equal(em0, em1), (nB, s, V)
    # and both are the plain definition
    l_ref = [next((j for j in range(s) if int(t[b, j]) != a[b, j]), s) for b in range(nB)]
    assert acc1.cpu().tolist() == l_ref
    for b in range(nB):
        assert int(em1[b, l_ref[b]]) == a[b, l_ref[b]]


def test_noalloc_equals_workspace_variant_on_two_calls_in_a_row():
    from paper_2310_18813_amd import binding as B
    run_pair(B, 64, 8, 32000, 1)      # 576 rows x 8 chunks
    run_pair(B, 3, 2, 5000, 2)        # smaller: 9 rows x 2 chunks over the first call's leftovers
    run_pair(B, 1, 0, 17, 3)
    run_pair(B, 16, 15, 50272, 4)


def test_noalloc_rejects_sizes_beyond_its_scratch():
    from paper_2310_18813_amd import binding as B
    st = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    x = torch.zeros(16, dtype=torch.int32, device=DEV)
    p = C.c_void_p(x.data_ptr())
    # 65535 sequences x 16 rows x 8 chunks of a 32000-token vocabulary: 8.4 M partials against 131072
    rc = B.lib.spec_greedy_accept_noalloc(st, p, p, 65535, 15, 32000, p, p)
    assert rc == B.ERR_CAPACITY and b"built-in scratch" in B.lib.spec_last_error(None)
    # the largest that fits: 16384 rows x 8 chunks
    n = C.c_size_t(0)
    assert B.lib.spec_greedy_accept_workspace_bytes(1024, 15, 32000, C.byref(n)) == B.OK and n.value == 1 << 20
