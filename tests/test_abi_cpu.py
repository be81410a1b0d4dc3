"""CPU-only checks of the C ABI: the library loads, exports every function the header
declares, and rejects bad arguments before any device call (so this runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2310_18813_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "spec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(B):
    names = declared_functions()
    assert len(names) >= 20
    for n in names:
        assert hasattr(B.lib, n), n
    assert sorted(B.EXPORTS) == names


def run_desc(B, **kw):
    d = dict(dtype=B.DTYPE_BF16, B_max=4, s_max=4, L_max=64, gen_max=16, eos_id=-1, proposal_mode=B.PROPOSALS_EXTERNAL)
    d.update(kw)
    return B.RunDesc(**d)


def test_workspace_bytes_and_argument_validation(B):
    tgt = si.llama_desc(2, 256, 4, 512, 1000, 64)
    drf = si.llama_desc(1, 128, 2, 256, 1000, 64)
    n1 = B.spec_workspace_bytes(tgt, None, run_desc(B))
    n2 = B.spec_workspace_bytes(tgt, drf, run_desc(B))
    assert 0 < n1 < n2
    # the two KV caches alone: layers * 2 * B_max * L_max * d * 2 bytes
    assert n1 > 2 * 2 * 4 * 64 * 256 * 2
    assert B.spec_workspace_bytes(tgt, None, run_desc(B, B_max=8)) > n1
    bad = [
        (dict(tgt, n_heads=3), None, run_desc(B), B.ERR_INVALID_ARG),          # d_model % heads
        (dict(tgt, ffn_kind=7), None, run_desc(B), B.ERR_INVALID_ARG),
        (dict(tgt, norm_eps=0.0), None, run_desc(B), B.ERR_INVALID_ARG),
        (tgt, dict(drf, vocab=999), run_desc(B), B.ERR_INVALID_ARG),           # vocabularies differ
        (tgt, None, run_desc(B, dtype=9), B.ERR_INVALID_ARG),
        (tgt, None, run_desc(B, B_max=0), B.ERR_INVALID_ARG),
        (tgt, None, run_desc(B, s_max=16), B.ERR_INVALID_ARG),
        (tgt, None, run_desc(B, L_max=10), B.ERR_INVALID_ARG),                 # < gen_max + s_max + 1
        (tgt, None, run_desc(B, eos_id=-2), B.ERR_INVALID_ARG),
        (tgt, None, run_desc(B, eos_id=1000), B.ERR_INVALID_ARG),              # outside the vocabulary
        (tgt, None, run_desc(B, proposal_mode=5), B.ERR_INVALID_ARG),
    ]
    for t, d, r, code in bad:
        with pytest.raises(B.SpecError) as e:
            B.spec_workspace_bytes(t, d, r)
        assert e.value.code == code, (t, d, code, str(e.value))
        assert str(e.value)


def test_init_rejects_bad_arguments_without_touching_the_device(B):
    tgt = si.llama_desc(1, 64, 1, 128, 100, 64)
    td = B.make_desc(tgt)
    run = run_desc(B, proposal_mode=B.PROPOSALS_EXTERNAL)
    out = C.c_void_p()
    arr = (C.c_void_p * B.T_COUNT)()
    for i in range(B.T_COUNT):
        arr[i] = 4096  # never dereferenced: validation fails first
    w = B.Weights(4096, None, 4096, None, 4096, C.cast(arr, C.POINTER(C.c_void_p)))
    # null workspace
    rc = B.lib.spec_init(C.byref(td), C.byref(w), None, None, C.byref(run), None, 1 << 40, None, C.byref(out))
    assert rc == B.ERR_WORKSPACE and not out.value and b"workspace" in B.lib.spec_last_error(None)
    # misaligned / too small workspace
    rc = B.lib.spec_init(C.byref(td), C.byref(w), None, None, C.byref(run), C.c_void_p(4096 + 8), 1 << 40, None, C.byref(out))
    assert rc == B.ERR_WORKSPACE
    rc = B.lib.spec_init(C.byref(td), C.byref(w), None, None, C.byref(run), C.c_void_p(4096), 1024, None, C.byref(out))
    assert rc == B.ERR_WORKSPACE
    # missing tensors
    w2 = B.Weights(None, None, 4096, None, 4096, C.cast(arr, C.POINTER(C.c_void_p)))
    rc = B.lib.spec_init(C.byref(td), C.byref(w2), None, None, C.byref(run), C.c_void_p(4096), 1 << 40, None, C.byref(out))
    assert rc == B.ERR_INVALID_ARG
    arr[8] = None  # wo of layer 0
    rc = B.lib.spec_init(C.byref(td), C.byref(w), None, None, C.byref(run), C.c_void_p(4096), 1 << 40, None, C.byref(out))
    assert rc == B.ERR_INVALID_ARG and b"layer 0" in B.lib.spec_last_error(None)
    # draft-proposal mode without a draft model
    run2 = run_desc(B, proposal_mode=B.PROPOSALS_DRAFT)
    arr[8] = 4096
    rc = B.lib.spec_init(C.byref(td), C.byref(w), None, None, C.byref(run2), C.c_void_p(4096), 1 << 40, None, C.byref(out))
    assert rc == B.ERR_INVALID_ARG
    # null context everywhere
    assert B.lib.spec_reset(None, 1, None, 1) == B.ERR_INVALID_ARG
    assert B.lib.spec_draft_step(None, 1) == B.ERR_INVALID_ARG
    assert B.lib.spec_verify_step(None, 0, None) == B.ERR_INVALID_ARG
    assert B.lib.spec_accept_commit(None, 0) == B.ERR_INVALID_ARG
    assert B.lib.spec_round(None, 0, 1) == B.ERR_INVALID_ARG
    assert B.lib.spec_choose_s(None, 1, None) == B.ERR_INVALID_ARG
    assert B.lib.spec_destroy(None) == B.OK


def test_greedy_accept_validates_before_any_device_call(B):
    n = C.c_size_t(0)
    assert B.lib.spec_greedy_accept_workspace_bytes(64, 8, 32000, C.byref(n)) == B.OK
    assert n.value == 64 * 9 * 8 * 8          # rows x chunks of 4096 logits x (value, index)
    assert B.lib.spec_greedy_accept_workspace_bytes(0, 8, 32000, C.byref(n)) == B.ERR_INVALID_ARG
    assert B.lib.spec_greedy_accept_workspace_bytes(1, 16, 32000, C.byref(n)) == B.ERR_CAPACITY
    fake = C.c_void_p(4096)                   # never dereferenced: validation fails first
    assert B.lib.spec_greedy_accept(None, None, fake, 1, 1, 10, fake, 64, fake, fake) == B.ERR_INVALID_ARG
    assert B.lib.spec_greedy_accept(None, fake, fake, 1, 1, 10, None, 64, fake, fake) == B.ERR_WORKSPACE
    assert B.lib.spec_greedy_accept(None, fake, fake, 1, 1, 10, fake, 4, fake, fake) == B.ERR_WORKSPACE
    assert B.lib.spec_greedy_accept_noalloc(None, fake, fake, 65535, 15, 32000, fake, fake) == B.ERR_CAPACITY
    assert b"built-in scratch" in B.lib.spec_last_error(None)


def test_sampling_entry_points_validate_before_any_device_call(B):
    fake = C.c_void_p(4096)                   # never dereferenced: validation fails first
    assert B.lib.spec_sample_tokens(None, fake, 4, 100, 0.0, fake, fake) == B.ERR_INVALID_ARG       # temperature
    assert B.lib.spec_sample_tokens(None, fake, -1, 100, 1.0, fake, fake) == B.ERR_INVALID_ARG
    assert B.lib.spec_sample_tokens(None, None, 4, 100, 1.0, fake, fake) == B.ERR_INVALID_ARG
    assert B.lib.spec_sample_tokens(None, fake, 0, 100, 1.0, fake, fake) == B.OK                    # nothing to do
    assert B.lib.spec_sample_accept(None, fake, fake, fake, fake, 2, 16, 100, 1.0, fake, fake, fake) == B.ERR_CAPACITY
    assert B.lib.spec_sample_accept(None, fake, None, None, fake, 2, 3, 100, 1.0, fake, fake, fake) == B.ERR_INVALID_ARG
    assert B.lib.spec_sample_accept(None, fake, None, fake, fake, 2, 3, 100, -2.0, fake, fake, fake) == B.ERR_INVALID_ARG
    assert B.lib.spec_sample_accept(None, fake, None, fake, fake, 0, 3, 100, 1.0, fake, fake, fake) == B.OK
    assert B.lib.spec_set_sampling(None, 1.0, fake, fake, fake) == B.ERR_INVALID_ARG                # no context
