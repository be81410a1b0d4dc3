"""Thin ctypes binding of include/spec.h: the same function names, argument marshalling
only.  PyTorch is used for device memory (tensors -> data_ptr) and the HIP stream; every
step of the method runs inside libspecdec.so.  There is no fallback: a missing library
raises at import of this module.
"""
import ctypes as C
import os

import torch  # must be loaded first: the library binds to the HIP runtime torch already mapped

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspecdec.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libspecdec.so is not built: run `python -m paper_2310_18813_amd.build`")
lib = C.CDLL(LIB_PATH)

OK, ERR_INVALID_ARG, ERR_WORKSPACE, ERR_STATE, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_HIP = range(7)
DTYPE_F32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
PROPOSALS_DRAFT, PROPOSALS_EXTERNAL = 0, 1
MODEL_TARGET, MODEL_DRAFT = 0, 1
T_NAMES = ["attn_norm_w", "attn_norm_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
           "ffn_norm_w", "ffn_norm_b", "w1", "b1", "w3", "w2", "b2"]
T_COUNT = len(T_NAMES)
DTYPE_CODE = {"fp32": DTYPE_F32, "bf16": DTYPE_BF16, "fp16": DTYPE_F16}
TORCH_DTYPE = {DTYPE_F32: torch.float32, DTYPE_BF16: torch.bfloat16, DTYPE_F16: torch.float16}

EXPORTS = ["spec_last_error", "spec_workspace_bytes", "spec_init", "spec_destroy", "spec_reset",
           "spec_reset_noprefill", "spec_reset_ragged", "spec_admit", "spec_set_seq_s", "spec_set_eos", "spec_rewind", "spec_set_proposal_table",
           "spec_set_proposals", "spec_draft_step", "spec_verify_step", "spec_accept_commit", "spec_round",
           "spec_profile_and_choose_s", "spec_set_lut", "spec_choose_s", "spec_read_output",
           "spec_read_state", "spec_kv_import", "spec_kv_export", "spec_kernel_timing",
           "spec_read_kernel_timing", "spec_set_hidden_dump", "spec_set_attention_shape", "spec_measure_peaks",
           "spec_set_draft_logits", "spec_read_proposals", "spec_greedy_accept_workspace_bytes", "spec_greedy_accept",
           "spec_greedy_accept_noalloc", "spec_set_gemm_tuning", "spec_read_saturation", "spec_sample_tokens",
           "spec_sample_accept", "spec_set_sampling"]
KCLASS_NAMES = ["gemm_qkv", "gemm_o", "gemm_ffn_in", "gemm_ffn_out", "gemm_head", "attention", "norm", "other",
                "draft_pass"]


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_ffn", C.c_int32),
                ("vocab", C.c_int32), ("max_pos", C.c_int32), ("ffn_kind", C.c_int32), ("norm_kind", C.c_int32),
                ("pos_kind", C.c_int32), ("has_bias", C.c_int32), ("norm_eps", C.c_float), ("rope_theta", C.c_float)]


class Weights(C.Structure):
    _fields_ = [("d_tok_emb", C.c_void_p), ("d_pos_emb", C.c_void_p), ("d_final_norm_w", C.c_void_p),
                ("d_final_norm_b", C.c_void_p), ("d_lm_head", C.c_void_p), ("layer_tensors", C.POINTER(C.c_void_p))]


class RunDesc(C.Structure):
    _fields_ = [("dtype", C.c_int32), ("B_max", C.c_int32), ("s_max", C.c_int32), ("L_max", C.c_int32),
                ("gen_max", C.c_int32), ("eos_id", C.c_int32), ("proposal_mode", C.c_int32)]


_vp, _i32, _i32p, _f32p, _i64p = C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.POINTER(C.c_float), C.POINTER(C.c_int64)
lib.spec_last_error.restype = C.c_char_p
lib.spec_last_error.argtypes = [_vp]
lib.spec_workspace_bytes.argtypes = [C.POINTER(ModelDesc), C.POINTER(ModelDesc), C.POINTER(RunDesc), C.POINTER(C.c_size_t)]
lib.spec_init.argtypes = [C.POINTER(ModelDesc), C.POINTER(Weights), C.POINTER(ModelDesc), C.POINTER(Weights),
                          C.POINTER(RunDesc), _vp, C.c_size_t, _vp, C.POINTER(_vp)]
lib.spec_destroy.argtypes = [_vp]
lib.spec_reset.argtypes = [_vp, _i32, _vp, _i32]
lib.spec_reset_noprefill.argtypes = [_vp, _i32, _vp, _i32]
lib.spec_reset_ragged.argtypes = [_vp, _i32, _vp, _i32, _i32p]
lib.spec_rewind.argtypes = [_vp]
lib.spec_admit.argtypes = [_vp, _i32, _vp, _i32]
lib.spec_set_seq_s.argtypes = [_vp, _vp]
lib.spec_set_eos.argtypes = [_vp, _i32]
lib.spec_set_proposal_table.argtypes = [_vp, _vp]
lib.spec_set_proposals.argtypes = [_vp, _vp, _i32]
lib.spec_draft_step.argtypes = [_vp, _i32]
lib.spec_verify_step.argtypes = [_vp, _i32, _vp]
lib.spec_accept_commit.argtypes = [_vp, _i32]
lib.spec_round.argtypes = [_vp, _i32, _i32]
lib.spec_profile_and_choose_s.argtypes = [_vp, _i32p, _i32, _i32, _vp, _i32, _i32, _i32p, _f32p]
lib.spec_set_lut.argtypes = [_vp, _i32p, _i32p, _i32]
lib.spec_choose_s.argtypes = [_vp, _i32, _i32p]
lib.spec_read_output.argtypes = [_vp, _i32p, _i32p, _i64p]
lib.spec_read_state.argtypes = [_vp, _i32p, _i32p, _i32p, _i32p]
lib.spec_kv_import.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp]
lib.spec_kv_export.argtypes = [_vp, _i32, _i32, _i32, _i32, _vp, _vp]
lib.spec_set_hidden_dump.argtypes = [_vp, _vp]
lib.spec_set_draft_logits.argtypes = [_vp, _vp]
lib.spec_read_proposals.argtypes = [_vp, _i32p]
lib.spec_read_saturation.argtypes = [_vp, _i64p]
lib.spec_greedy_accept_workspace_bytes.argtypes = [_i32, _i32, _i32, C.POINTER(C.c_size_t)]
lib.spec_greedy_accept.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _vp, C.c_size_t, _vp, _vp]
lib.spec_greedy_accept_noalloc.argtypes = [_vp, _vp, _vp, _i32, _i32, _i32, _vp, _vp]
lib.spec_sample_tokens.argtypes = [_vp, _vp, _i32, _i32, C.c_float, _vp, _vp]
lib.spec_sample_accept.argtypes = [_vp, _vp, _vp, _vp, _vp, _i32, _i32, _i32, C.c_float, _vp, _vp, _vp]
lib.spec_set_sampling.argtypes = [_vp, C.c_float, _vp, _vp, _vp]
lib.spec_set_attention_shape.argtypes = [_vp, _i32]
lib.spec_set_gemm_tuning.argtypes = [_vp, _i32, _i32, _i32]
lib.spec_kernel_timing.argtypes = [_vp, _i32]
lib.spec_read_kernel_timing.argtypes = [_vp, _i64p, C.POINTER(C.c_double)]
lib.spec_measure_peaks.argtypes = [_vp, _vp, C.c_size_t, C.POINTER(C.c_double), C.POINTER(C.c_double)]


class SpecError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("spec error %d: %s" % (code, msg))
        self.code = code


def last_error(ctx=None):
    return (lib.spec_last_error(ctx) or b"").decode()


def _check(rc, ctx=None):
    if rc != OK:
        raise SpecError(rc, last_error(ctx))


def _dp(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def make_desc(d):
    return ModelDesc(**{k: d[k] for k, _ in ModelDesc._fields_})


def make_weights(w):
    """w: dict of device tensors as produced by synth_inputs.make_weights.  Returns the
    struct plus the objects that must stay alive while it is used."""
    nl = len(w["layers"])
    arr = (C.c_void_p * max(1, nl * T_COUNT))()
    for li, L in enumerate(w["layers"]):
        for si, name in enumerate(T_NAMES):
            t = L.get(name)
            arr[li * T_COUNT + si] = None if t is None else t.data_ptr()
    s = Weights(_dp(w["tok_emb"]), _dp(w.get("pos_emb")), _dp(w["final_norm_w"]), _dp(w.get("final_norm_b")),
                _dp(w["lm_head"]), C.cast(arr, C.POINTER(C.c_void_p)))
    return s, arr


def spec_measure_peaks(device="cuda:0", nbytes=1 << 30):
    """-> (HBM stream GB/s, MFMA f16 TFLOP/s) measured on the device, over a scratch tensor of nbytes."""
    dev = torch.device(device)
    buf = torch.arange(nbytes // 8, dtype=torch.int64, device=dev).mul_(0x9E3779B97F4A7C15 - (1 << 64))  # not all zeros
    g, t = C.c_double(0.0), C.c_double(0.0)
    with torch.cuda.device(dev):
        st = torch.cuda.current_stream(dev)
        _check(lib.spec_measure_peaks(C.c_void_p(st.cuda_stream), _dp(buf), buf.numel() * 8, C.byref(g), C.byref(t)))
    return g.value, t.value


def spec_greedy_accept(logits, proposals, accepted=None, emitted=None, workspace=None, noalloc=False):
    """logits [B][s+1][V] fp32 device tensor, proposals [B][s] int32 device tensor (or None when s = 0).
    -> (accepted [B], emitted [B][s+1]) int32 device tensors.  noalloc=True calls spec_greedy_accept_noalloc
    (outputs must then be passed in: this wrapper allocates nothing in that mode)."""
    assert logits.dim() == 3 and logits.dtype == torch.float32 and logits.is_contiguous()
    nB, q, V = logits.shape
    s = q - 1
    if s:
        assert proposals.dtype == torch.int32 and proposals.shape == (nB, s) and proposals.is_contiguous()
    dev = logits.device
    st = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
    if noalloc:
        assert accepted is not None and emitted is not None
        with torch.cuda.device(dev):
            _check(lib.spec_greedy_accept_noalloc(st, _dp(logits), _dp(proposals) if s else None, nB, s, V, _dp(accepted),
                                                  _dp(emitted)))
        return accepted, emitted
    if accepted is None:
        accepted = torch.empty(nB, dtype=torch.int32, device=dev)
    if emitted is None:
        emitted = torch.empty((nB, q), dtype=torch.int32, device=dev)
    n = C.c_size_t(0)
    _check(lib.spec_greedy_accept_workspace_bytes(nB, s, V, C.byref(n)))
    if workspace is None:
        workspace = torch.empty(max(8, n.value), dtype=torch.uint8, device=dev)
    with torch.cuda.device(dev):
        _check(lib.spec_greedy_accept(st, _dp(logits), _dp(proposals) if s else None, nB, s, V, _dp(workspace),
                                      workspace.numel(), _dp(accepted), _dp(emitted)))
    return accepted, emitted


def spec_sample_tokens(logits, uniforms, temperature):
    """logits [rows][V] fp32, uniforms [rows] fp32, device tensors -> tokens [rows] int32."""
    assert logits.dim() == 2 and logits.dtype == torch.float32 and logits.is_contiguous()
    assert uniforms.dtype == torch.float32 and uniforms.shape == (logits.shape[0],) and uniforms.is_contiguous()
    dev = logits.device
    out = torch.empty(logits.shape[0], dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        st = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        _check(lib.spec_sample_tokens(st, _dp(logits), logits.shape[0], logits.shape[1], float(temperature), _dp(uniforms),
                                      _dp(out)))
    return out


def spec_sample_accept(target_logits, draft_logits, proposals, uniforms, temperature):
    """target_logits [B][s+1][V], draft_logits [s][B][V] or None, proposals [B][s] int32 (None when s = 0),
    uniforms [B][s+1][3]: device tensors -> (chosen [B][s+1], accepted [B], emitted [B][s+1]) int32."""
    assert target_logits.dim() == 3 and target_logits.dtype == torch.float32 and target_logits.is_contiguous()
    nB, q, V = target_logits.shape
    s = q - 1
    if draft_logits is not None:
        assert draft_logits.dtype == torch.float32 and draft_logits.shape == (s, nB, V) and draft_logits.is_contiguous()
    if s:
        assert proposals.dtype == torch.int32 and proposals.shape == (nB, s) and proposals.is_contiguous()
    assert uniforms.dtype == torch.float32 and uniforms.shape == (nB, q, 3) and uniforms.is_contiguous()
    dev = target_logits.device
    chosen = torch.empty((nB, q), dtype=torch.int32, device=dev)
    accepted = torch.empty(nB, dtype=torch.int32, device=dev)
    emitted = torch.empty((nB, q), dtype=torch.int32, device=dev)
    with torch.cuda.device(dev):
        st = C.c_void_p(torch.cuda.current_stream(dev).cuda_stream)
        _check(lib.spec_sample_accept(st, _dp(target_logits), _dp(draft_logits) if draft_logits is not None and s else None,
                                      _dp(proposals) if s else None, _dp(uniforms), nB, s, V, float(temperature),
                                      _dp(chosen), _dp(accepted), _dp(emitted)))
    return chosen, accepted, emitted


def spec_workspace_bytes(tgt_desc, drf_desc, run):
    n = C.c_size_t(0)
    t = make_desc(tgt_desc)
    d = make_desc(drf_desc) if drf_desc is not None else None
    _check(lib.spec_workspace_bytes(C.byref(t), C.byref(d) if d is not None else None, C.byref(run), C.byref(n)))
    return n.value


class Context:
    """Owns the workspace tensor and the opaque spec_ctx; methods are the C entry points."""

    def __init__(self, tgt_desc, tgt_w, drf_desc, drf_w, dtype, B_max, s_max, L_max, gen_max,
                 proposal_mode=PROPOSALS_EXTERNAL, device="cuda:0", stream=None):
        self.device = torch.device(device)
        self.dtype_code = DTYPE_CODE[dtype] if isinstance(dtype, str) else dtype
        self.run = RunDesc(self.dtype_code, B_max, s_max, L_max, gen_max, -1, proposal_mode)
        self.tgt_desc, self.drf_desc = dict(tgt_desc), (dict(drf_desc) if drf_desc is not None else None)
        nbytes = spec_workspace_bytes(tgt_desc, drf_desc, self.run)
        self.workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=self.device)
        base = self.workspace.data_ptr()
        off = (-base) % 256
        td = make_desc(tgt_desc)
        tw, self._keep_t = make_weights(tgt_w)
        dd = make_desc(drf_desc) if drf_desc is not None else None
        dw, self._keep_d = make_weights(drf_w) if drf_w is not None else (None, None)
        self.stream = stream if stream is not None else torch.cuda.current_stream(self.device)
        h = C.c_void_p()
        with torch.cuda.device(self.device):
            rc = lib.spec_init(C.byref(td), C.byref(tw), C.byref(dd) if dd is not None else None,
                               C.byref(dw) if dw is not None else None, C.byref(self.run),
                               C.c_void_p(base + off), nbytes, C.c_void_p(self.stream.cuda_stream), C.byref(h))
        _check(rc)
        self.h = h
        self.B_max, self.s_max, self.L_max, self.gen_max = B_max, s_max, L_max, gen_max
        self.B = 0
        self._table = None

    def close(self):
        if getattr(self, "h", None):
            lib.spec_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- one method per C entry point -------------------------------------
    def _prompt(self, prompt):
        p = torch.as_tensor(prompt, dtype=torch.int32).to(self.device).contiguous()
        assert p.dim() == 2
        return p

    def spec_reset(self, prompt):
        p = self._prompt(prompt)
        _check(lib.spec_reset(self.h, p.shape[0], _dp(p), p.shape[1]), self.h)
        self.B = p.shape[0]

    def spec_reset_ragged(self, prompts):
        """prompts: a list of 1-d token arrays of different lengths."""
        lens = [int(len(p)) for p in prompts]
        rows = torch.zeros((len(prompts), max(lens)), dtype=torch.int32)
        for b, p in enumerate(prompts):
            rows[b, :lens[b]] = torch.as_tensor(p, dtype=torch.int32)
        p = rows.to(self.device).contiguous()
        _check(lib.spec_reset_ragged(self.h, p.shape[0], _dp(p), p.shape[1], (C.c_int32 * len(lens))(*lens)), self.h)
        self.B = p.shape[0]

    def spec_reset_noprefill(self, prompt):
        p = self._prompt(prompt)
        _check(lib.spec_reset_noprefill(self.h, p.shape[0], _dp(p), p.shape[1]), self.h)
        self.B = p.shape[0]

    def spec_admit(self, b, prompt):
        p = torch.as_tensor(prompt, dtype=torch.int32).to(self.device).contiguous()
        assert p.dim() == 1
        self._admit_prompt = p  # stays alive until the stream has consumed it
        _check(lib.spec_admit(self.h, int(b), _dp(p), int(p.shape[0])), self.h)

    def spec_set_seq_s(self, caps):
        if caps is None:
            self._seq_s = None
            _check(lib.spec_set_seq_s(self.h, None), self.h)
            return
        t = torch.as_tensor(caps, dtype=torch.int32).to(self.device).contiguous()
        assert t.dim() == 1 and t.shape[0] >= self.B
        self._seq_s = t  # must outlive its use
        _check(lib.spec_set_seq_s(self.h, _dp(t)), self.h)

    def spec_set_eos(self, eos_token):
        _check(lib.spec_set_eos(self.h, -1 if eos_token is None else int(eos_token)), self.h)

    def spec_rewind(self):
        _check(lib.spec_rewind(self.h), self.h)

    def spec_set_proposal_table(self, table):
        if table is None:
            self._table = None
            _check(lib.spec_set_proposal_table(self.h, None), self.h)
            return
        t = torch.as_tensor(table, dtype=torch.int32).to(self.device).contiguous()
        assert t.dim() == 2 and t.shape[1] == self.L_max and t.shape[0] >= 1
        self._table = t  # must outlive its use
        _check(lib.spec_set_proposal_table(self.h, _dp(t)), self.h)

    def spec_set_proposals(self, tok):
        t = torch.as_tensor(tok, dtype=torch.int32).to(self.device).contiguous()
        s = t.shape[1] if t.dim() == 2 else 0
        _check(lib.spec_set_proposals(self.h, _dp(t) if s else None, s), self.h)

    def spec_draft_step(self, j):
        _check(lib.spec_draft_step(self.h, j), self.h)

    def spec_verify_step(self, s, want_logits=False):
        logits = None
        if want_logits:
            logits = torch.empty((self.B, s + 1, self.tgt_desc["vocab"]), dtype=torch.float32, device=self.device)
        _check(lib.spec_verify_step(self.h, s, _dp(logits)), self.h)
        return logits

    def spec_accept_commit(self, s):
        _check(lib.spec_accept_commit(self.h, s), self.h)

    def spec_round(self, s, n_rounds=1):
        _check(lib.spec_round(self.h, s, n_rounds), self.h)

    def spec_profile_and_choose_s(self, batch_sizes, s_max_profile, prompt, gen):
        p = self._prompt(prompt)
        nb = len(batch_sizes)
        bs = (C.c_int32 * nb)(*batch_sizes)
        lut = (C.c_int32 * nb)()
        grid = (C.c_float * (nb * (s_max_profile + 1)))()
        assert p.shape[0] >= max(batch_sizes)
        _check(lib.spec_profile_and_choose_s(self.h, bs, nb, s_max_profile, _dp(p), p.shape[1], gen, lut, grid), self.h)
        self.B = batch_sizes[-1]
        g = [[grid[i * (s_max_profile + 1) + s] for s in range(s_max_profile + 1)] for i in range(nb)]
        return list(lut), g

    def spec_set_lut(self, batch_sizes, lut):
        nb = len(batch_sizes)
        _check(lib.spec_set_lut(self.h, (C.c_int32 * nb)(*batch_sizes), (C.c_int32 * nb)(*lut), nb), self.h)

    def spec_choose_s(self, B):
        s = C.c_int32(-1)
        _check(lib.spec_choose_s(self.h, B, C.byref(s)), self.h)
        return s.value

    def spec_read_output(self):
        """-> (list of per-sequence emitted token lists, histogram of accepted lengths)."""
        tok = (C.c_int32 * (self.B * self.gen_max))()
        ln = (C.c_int32 * self.B)()
        hist = (C.c_int64 * (self.s_max + 1))()
        _check(lib.spec_read_output(self.h, tok, ln, hist), self.h)
        out = [[tok[b * self.gen_max + i] for i in range(ln[b])] for b in range(self.B)]
        return out, list(hist)

    def spec_read_state(self):
        n = (C.c_int32 * self.B)()
        kd = (C.c_int32 * self.B)()
        ll = (C.c_int32 * self.B)()
        am = (C.c_int32 * (self.B * (self.s_max + 1)))()
        _check(lib.spec_read_state(self.h, n, kd, ll, am), self.h)
        a = [[am[b * (self.s_max + 1) + i] for i in range(self.s_max + 1)] for b in range(self.B)]
        return list(n), list(kd), list(ll), a

    def spec_set_hidden_dump(self, on):
        """on=True allocates the dump tensor [n_layers + 1][B_max * 16][d_model] and returns it."""
        if not on:
            self._hidden = None
            _check(lib.spec_set_hidden_dump(self.h, None), self.h)
            return None
        nl, d = self.tgt_desc["n_layers"], self.tgt_desc["d_model"]
        self._hidden = torch.zeros((nl + 1) * self.B_max * 16 * d, dtype=torch.float32, device=self.device)
        _check(lib.spec_set_hidden_dump(self.h, _dp(self._hidden)), self.h)
        return self._hidden

    def spec_set_draft_logits(self, on):
        """on=True allocates [B_max][vocab] fp32 for the draft steps' logits and returns it."""
        if not on:
            self._draft_logits = None
            _check(lib.spec_set_draft_logits(self.h, None), self.h)
            return None
        self._draft_logits = torch.zeros((self.B_max, self.drf_desc["vocab"]), dtype=torch.float32, device=self.device)
        _check(lib.spec_set_draft_logits(self.h, _dp(self._draft_logits)), self.h)
        return self._draft_logits

    def spec_set_sampling(self, temperature, uniforms):
        """uniforms: [B_max][L_max][3] fp32 device tensor (None: back to the greedy rule).  Allocates the logits
        buffers the library needs and returns them: (target [B_max*(s_max+1)][V], draft [s_max][B_max][V] or None)."""
        if uniforms is None:
            _check(lib.spec_set_sampling(self.h, 0.0, None, None, None), self.h)
            self._smp = None
            return None, None
        assert uniforms.dtype == torch.float32 and uniforms.shape == (self.B_max, self.L_max, 3) and uniforms.is_contiguous()
        V = self.tgt_desc["vocab"]
        tl = torch.zeros((self.B_max * (self.s_max + 1), V), dtype=torch.float32, device=self.device)
        dl = None
        if self.drf_desc is not None:
            dl = torch.zeros((max(1, self.s_max), self.B_max, V), dtype=torch.float32, device=self.device)
        _check(lib.spec_set_sampling(self.h, float(temperature), _dp(uniforms), _dp(tl), _dp(dl) if dl is not None else None),
               self.h)
        self._smp = (uniforms, tl, dl)
        return tl, dl

    def spec_read_saturation(self):
        n = C.c_int64(-1)
        _check(lib.spec_read_saturation(self.h, C.byref(n)), self.h)
        return n.value

    def spec_read_proposals(self):
        """-> [B][s_max] proposals of the current round."""
        t = (C.c_int32 * max(1, self.B * self.s_max))()
        _check(lib.spec_read_proposals(self.h, t), self.h)
        return [[t[b * self.s_max + j] for j in range(self.s_max)] for b in range(self.B)]

    def spec_set_attention_shape(self, shape):
        _check(lib.spec_set_attention_shape(self.h, shape), self.h)

    def spec_set_gemm_tuning(self, tile_mtw=0, tile_nbw=0, flags=0):
        _check(lib.spec_set_gemm_tuning(self.h, tile_mtw, tile_nbw, flags), self.h)

    def spec_kernel_timing(self, enable):
        _check(lib.spec_kernel_timing(self.h, 1 if enable else 0), self.h)

    def spec_read_kernel_timing(self):
        """-> {class name: (launch count, total ms)}"""
        n = len(KCLASS_NAMES)
        cnt = (C.c_int64 * n)()
        ms = (C.c_double * n)()
        _check(lib.spec_read_kernel_timing(self.h, cnt, ms), self.h)
        return {KCLASS_NAMES[i]: (cnt[i], ms[i]) for i in range(n)}

    def spec_kv_import(self, which, layer, K, V):
        K, V = K.contiguous(), V.contiguous()
        assert K.dtype == TORCH_DTYPE[self.dtype_code] and K.shape == V.shape and K.dim() == 3
        _check(lib.spec_kv_import(self.h, which, layer, K.shape[0], K.shape[1], _dp(K), _dp(V)), self.h)

    def spec_kv_export(self, which, layer, B, length):
        d = (self.tgt_desc if which == MODEL_TARGET else self.drf_desc)["d_model"]
        K = torch.empty((B, length, d), dtype=TORCH_DTYPE[self.dtype_code], device=self.device)
        V = torch.empty_like(K)
        _check(lib.spec_kv_export(self.h, which, layer, B, length, _dp(K), _dp(V)), self.h)
        return K, V
