"""ctypes front-end of the CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It builds oracle/spec_oracle.c with gcc (twice: fp32 and fp64
arithmetic) and exposes the C functions on numpy arrays.  It imports nothing
from the GPU package.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spec_oracle.c")
_HDR = os.path.join(_HERE, "spec_oracle.h")

W_F32, W_BF16, W_F16 = 0, 1, 2
FFN_SWIGLU, FFN_RELU = 0, 1
NORM_RMS, NORM_LAYER = 0, 1
POS_ROPE, POS_LEARNED = 0, 1

(T_ATTN_NORM_W, T_ATTN_NORM_B, T_WQ, T_BQ, T_WK, T_BK, T_WV, T_BV, T_WO, T_BO,
 T_FFN_NORM_W, T_FFN_NORM_B, T_W1, T_B1, T_W3, T_W2, T_B2, T_COUNT) = range(18)


def lib_path(prec):
    return os.path.join(_HERE, "liboracle_%s.so" % prec)


def build(force=False):
    """Compile both precisions of the oracle (gcc, no fast-math)."""
    for prec, ctype in (("f32", "float"), ("f64", "double")):
        out = lib_path(prec)
        if not force and os.path.exists(out) and os.path.getmtime(out) >= max(
                os.path.getmtime(_SRC), os.path.getmtime(_HDR)):
            continue
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-fno-fast-math",
               "-ffp-contract=off", "-DORC_REAL=" + ctype, "-o", out, _SRC, "-lm"]
        subprocess.check_call(cmd)


class Desc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("max_pos", C.c_int32),
                ("ffn_kind", C.c_int32), ("norm_kind", C.c_int32), ("pos_kind", C.c_int32),
                ("has_bias", C.c_int32), ("norm_eps", C.c_double), ("rope_theta", C.c_double)]


class Weights(C.Structure):
    _fields_ = [("wdtype", C.c_int32), ("tok_emb", C.c_void_p), ("pos_emb", C.c_void_p),
                ("final_norm_w", C.c_void_p), ("final_norm_b", C.c_void_p), ("lm_head", C.c_void_p),
                ("layers", C.POINTER(C.c_void_p))]


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


class Oracle:
    """One precision of the oracle ("f64" is the parity reference, "f32" the fp32 oracle)."""

    def __init__(self, prec="f64"):
        build()
        self.prec = prec
        self.real = np.float64 if prec == "f64" else np.float32
        L = C.CDLL(lib_path(prec))
        self.L = L
        assert L.orc_real_bytes() == np.dtype(self.real).itemsize
        L.orc_model_create.restype = C.c_void_p
        L.orc_cache_create.restype = C.c_void_p
        L.orc_cache_k.restype = C.c_void_p
        L.orc_cache_v.restype = C.c_void_p
        L.orc_l_estimate.restype = C.c_double
        L.orc_time_model.restype = C.c_double
        L.orc_time_model.argtypes = [C.c_double] * 5

    # ---- helpers -------------------------------------------------------
    def _real(self, a):
        return np.ascontiguousarray(a, dtype=self.real)

    @staticmethod
    def wdtype_of(a):
        if a.dtype == np.float32:
            return W_F32
        raise TypeError("pass 16-bit tensors as (uint16 array, wdtype)")

    # ---- elementary operations ----------------------------------------
    def widen(self, bits, wdtype):
        bits = np.ascontiguousarray(bits)
        out = np.empty(bits.shape, dtype=self.real)
        self.L.orc_widen(_ptr(bits), C.c_int(wdtype), C.c_int64(bits.size), _ptr(out))
        return out

    def linear(self, x, W, bias=None, wdtype=W_F32):
        x = self._real(x)
        M, K = x.shape
        W = np.ascontiguousarray(W)
        N = W.shape[0]
        assert W.shape[1] == K
        y = np.empty((M, N), dtype=self.real)
        b = None if bias is None else np.ascontiguousarray(bias)
        self.L.orc_linear(_ptr(x), M, K, _ptr(W), _ptr(b), wdtype, N, _ptr(y))
        return y

    def rmsnorm(self, x, gain, eps, wdtype=W_F32):
        x = self._real(x)
        y = np.empty_like(x)
        g = np.ascontiguousarray(gain)
        self.L.orc_rmsnorm(_ptr(x), x.shape[0], x.shape[1], _ptr(g), wdtype, C.c_double(eps), _ptr(y))
        return y

    def layernorm(self, x, gain, bias, eps, wdtype=W_F32):
        x = self._real(x)
        y = np.empty_like(x)
        g = np.ascontiguousarray(gain)
        b = np.ascontiguousarray(bias)
        self.L.orc_layernorm(_ptr(x), x.shape[0], x.shape[1], _ptr(g), _ptr(b), wdtype, C.c_double(eps), _ptr(y))
        return y

    def rope(self, x, n_heads, pos, theta=10000.0):
        x = self._real(x).copy()
        hd = x.size // n_heads
        self.L.orc_rope(_ptr(x), n_heads, hd, int(pos), C.c_double(theta))
        return x

    def attention(self, q, Kc, Vc, n_heads):
        q = self._real(q)
        Kc = self._real(Kc)
        Vc = self._real(Vc)
        d = q.size
        out = np.empty(d, dtype=self.real)
        self.L.orc_attention(_ptr(q), n_heads, d // n_heads, _ptr(Kc), _ptr(Vc), Kc.shape[0], _ptr(out))
        return out

    def swiglu(self, g, u):
        g = self._real(g)
        u = self._real(u)
        out = np.empty_like(g)
        self.L.orc_swiglu(_ptr(g), _ptr(u), C.c_int64(g.size), _ptr(out))
        return out

    def argmax(self, v):
        v = self._real(v)
        return int(self.L.orc_argmax(_ptr(v), v.size))

    def accept(self, t, a):
        s = len(t)
        t_, tp = _i32(t if s else [0])
        a_, ap = _i32(a)
        em = np.zeros(s + 1, dtype=np.int32)
        l = self.L.orc_accept(tp, s, ap, em.ctypes.data_as(C.POINTER(C.c_int32)))
        return l, em[: l + 1].tolist()

    # ---- adaptive policy -------------------------------------------------
    def lut_build(self, lat, rel_eps=0.01):
        lat = np.ascontiguousarray(lat, dtype=np.float64)
        nB, nS = lat.shape
        lut = np.zeros(nB, dtype=np.int32)
        self.L.orc_lut_build(_ptr(lat), nB, nS, C.c_double(rel_eps), lut.ctypes.data_as(C.POINTER(C.c_int32)))
        return lut

    def lut_lookup(self, profiled_B, lut, B):
        pb, pbp = _i32(profiled_B)
        lt, ltp = _i32(lut)
        return int(self.L.orc_lut_lookup(pbp, ltp, len(pb), int(B)))

    def l_estimate(self, l_i, s):
        li, lip = _i32(l_i)
        return float(self.L.orc_l_estimate(lip, len(li), int(s)))

    def time_model(self, N, tL, tS, s, l):
        return float(self.L.orc_time_model(float(N), float(tL), float(tS), float(s), float(l)))

    # ---- models ----------------------------------------------------------
    def model(self, desc, weights, wdtype):
        return Model(self, desc, weights, wdtype)


class Model:
    """desc: dict of orc_desc fields.  weights: dict with 'tok_emb', 'pos_emb',
    'final_norm_w', 'final_norm_b', 'lm_head' and 'layers' = list of dicts keyed by
    slot name ('attn_norm_w', 'wq', ... see SLOT_NAMES).  Arrays are float32, or
    uint16 bit patterns when wdtype is W_BF16 / W_F16.                            """

    SLOT_NAMES = ["attn_norm_w", "attn_norm_b", "wq", "bq", "wk", "bk", "wv", "bv", "wo", "bo",
                  "ffn_norm_w", "ffn_norm_b", "w1", "b1", "w3", "w2", "b2"]

    def __init__(self, orc, desc, weights, wdtype):
        self.orc = orc
        self.desc = dict(desc)
        self.keep = []  # keep numpy arrays alive

        def hold(a):
            if a is None:
                return None
            a = np.ascontiguousarray(a)
            want = np.float32 if wdtype == W_F32 else np.uint16
            assert a.dtype == want, (a.dtype, want)
            self.keep.append(a)
            return a.ctypes.data

        nl = desc["n_layers"]
        arr = (C.c_void_p * max(1, nl * T_COUNT))()
        for li in range(nl):
            for si, name in enumerate(self.SLOT_NAMES):
                arr[li * T_COUNT + si] = hold(weights["layers"][li].get(name))
        self.arr = arr
        w = Weights(wdtype, hold(weights["tok_emb"]), hold(weights.get("pos_emb")),
                    hold(weights["final_norm_w"]), hold(weights.get("final_norm_b")),
                    hold(weights["lm_head"]), C.cast(arr, C.POINTER(C.c_void_p)))
        d = Desc(**{k: desc[k] for k, _ in Desc._fields_})
        self.h = C.c_void_p(orc.L.orc_model_create(C.byref(d), C.byref(w)))
        assert self.h.value, "orc_model_create rejected the description"

    def __del__(self):
        try:
            self.orc.L.orc_model_destroy(self.h)
        except Exception:
            pass

    def cache(self, L_max):
        return Cache(self, L_max)

    def forward(self, cache, tokens, start_pos, want_logits=True):
        tk, tp = _i32(tokens)
        q = len(tk)
        logits = np.empty((q, self.desc["vocab"]), dtype=self.orc.real) if want_logits else None
        rc = self.orc.L.orc_forward(self.h, cache.h, tp, q, int(start_pos), _ptr(logits))
        if rc:
            raise ValueError("orc_forward rc=%d" % rc)
        return logits

    def greedy(self, prompt, N, L_max=None):
        pr, pp = _i32(prompt)
        L_max = L_max or (len(pr) + N + 1)
        out = np.zeros(N, dtype=np.int32)
        rc = self.orc.L.orc_greedy(self.h, pp, len(pr), N, L_max, out.ctypes.data_as(C.POINTER(C.c_int32)))
        if rc:
            raise ValueError("orc_greedy rc=%d" % rc)
        return out

    def spec_generate(self, draft, prompt, N, s, proposal_mode=0, prop_table=None, L_max=None):
        """Returns (tokens[N], accepted-per-round list)."""
        pr, pp = _i32(prompt)
        L_max = L_max or (len(pr) + N + s + 1)
        out = np.zeros(N, dtype=np.int32)
        stats = np.zeros(max(N, 1), dtype=np.int32)
        rounds = C.c_int32(0)
        tbl = None
        tblp = None
        if prop_table is not None:
            tbl, tblp = _i32(prop_table)
            assert len(tbl) >= L_max
        rc = self.orc.L.orc_spec_generate(self.h, draft.h if draft is not None else None, pp, len(pr), N, int(s),
                                          int(proposal_mode), tblp, L_max,
                                          out.ctypes.data_as(C.POINTER(C.c_int32)),
                                          stats.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(rounds))
        if rc:
            raise ValueError("orc_spec_generate rc=%d" % rc)
        return out, stats[: rounds.value].tolist()


class Cache:
    def __init__(self, model, L_max):
        self.model = model
        self.L_max = L_max
        self.h = C.c_void_p(model.orc.L.orc_cache_create(model.h, L_max))

    def __del__(self):
        try:
            self.model.orc.L.orc_cache_destroy(self.h)
        except Exception:
            pass

    def _view(self, fn, layer):
        d = self.model.desc["d_model"]
        p = fn(self.h, layer)
        n = self.L_max * d
        ct = C.c_double if self.model.orc.real == np.float64 else C.c_float
        buf = (ct * n).from_address(p)
        return np.frombuffer(buf, dtype=self.model.orc.real).reshape(self.L_max, d)

    def k(self, layer):
        """Writable view [L_max][d_model] of the layer's cached keys (post-RoPE)."""
        return self._view(self.model.orc.L.orc_cache_k, layer)

    def v(self, layer):
        return self._view(self.model.orc.L.orc_cache_v, layer)
