"""ctypes front end of the CPU oracle (oracle/specache_oracle.cpp): test infrastructure only.

Marshals numpy arrays to the C functions; holds no arithmetic of its own.
16-bit tensors are passed as raw uint16 bit patterns plus a dtype flag
(0 = binary16, 1 = bfloat16).
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None

FP16, BF16 = 0, 1


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        vp, i32, f32, f64 = C.c_void_p, C.c_int, C.c_float, C.c_double
        L.orc_widen.restype = f32
        L.orc_widen.argtypes = [C.c_uint16, i32]
        L.orc_quantize_group.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp]
        L.orc_quantize_group_form.argtypes = [vp, i32, i32, i32, vp, vp, vp, vp, vp]
        L.orc_derive_scale_zero.argtypes = [f32, f32, i32, vp, vp]
        L.orc_derive_scale_zero_form.argtypes = [f32, f32, i32, i32, vp, vp]
        L.orc_pack_group.argtypes = [vp, i32, i32, vp]
        L.orc_unpack_group.argtypes = [vp, i32, i32, vp]
        L.orc_cache_create.restype = vp
        L.orc_cache_create.argtypes = [i32] * 5
        L.orc_cache_create_form.restype = vp
        L.orc_cache_create_form.argtypes = [i32] * 6
        L.orc_cache_destroy.restype = None
        L.orc_cache_destroy.argtypes = [vp]
        L.orc_cache_append.argtypes = [vp, vp, vp, i32]
        L.orc_cache_counts.argtypes = [vp, vp, vp]
        L.orc_cache_export.argtypes = [vp] * 7
        L.orc_cache_dequant.argtypes = [vp, vp, vp]
        L.orc_cache_history.argtypes = [vp, vp, vp]
        L.orc_scores.argtypes = [vp, vp, i32, i32, f64, vp, vp]
        L.orc_scores_form.argtypes = [vp, vp, i32, i32, f64, i32, vp, vp]
        L.orc_scores_mixed.argtypes = [vp, vp, i32, i32, f64, i32, vp, i32, vp, vp]
        L.orc_topk.argtypes = [vp, i32, i32, vp]
        L.orc_attend.argtypes = [vp, vp, i32, i32, f64, vp, i32, vp, vp, vp]
        L.orc_full_attention.argtypes = [vp, vp, i32, i32, f64, vp, vp, vp, vp]
        L.orc_hit_rate.restype = f64
        L.orc_hit_rate.argtypes = [vp, i32, vp, i32]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def widen(bits, dtype):
    """Exact float32 value of 16-bit patterns."""
    bits = _u16(bits)
    out = np.empty(bits.shape, np.float32)
    L = lib()
    flat_in, flat_out = bits.reshape(-1), out.reshape(-1)
    for i in range(flat_in.size):
        flat_out[i] = L.orc_widen(int(flat_in[i]), dtype)
    return out


SELECT_MAX_LOGIT, SELECT_MAX_LOGPROB = 0, 1   # how the query heads of a KV head share one index set
IMPROVED_1BIT, KIVI_1BIT = 0, 1   # Eq. 3, and Eq. 2 with B = 1 (Section 4.4 / Table 5, "original")


def quantize_group(x, bits, one_bit_form=IMPROVED_1BIT):
    """Eq. 2 / Eq. 3 on one group.  Returns (codes u8[g], mn, mx, s, z) with float32 scalars."""
    x = np.ascontiguousarray(x, np.float32)
    g = x.size
    codes = np.empty(g, np.uint8)
    out = np.empty(4, np.float32)
    _check(lib().orc_quantize_group_form(_p(x), g, bits, one_bit_form, _p(out[0:1]), _p(out[1:2]), _p(out[2:3]),
                                         _p(out[3:4]), _p(codes)), "quantize_group")
    return codes, out[0], out[1], out[2], out[3]


def derive_scale_zero(mn, mx, bits, one_bit_form=IMPROVED_1BIT):
    out = np.empty(2, np.float32)
    _check(lib().orc_derive_scale_zero_form(float(mn), float(mx), bits, one_bit_form, _p(out[0:1]), _p(out[1:2])),
           "derive_scale_zero")
    return out[0], out[1]


def pack_group(codes, bits):
    codes = np.ascontiguousarray(codes, np.uint8)
    packed = np.empty(codes.size * bits // 8, np.uint8)
    _check(lib().orc_pack_group(_p(codes), codes.size, bits, _p(packed)), "pack_group")
    return packed


def unpack_group(packed, g, bits):
    packed = np.ascontiguousarray(packed, np.uint8)
    codes = np.empty(g, np.uint8)
    _check(lib().orc_unpack_group(_p(packed), g, bits, _p(codes)), "unpack_group")
    return codes


class Cache:
    """The SpeCache state of one (batch, KV head): 16-bit history C and low-bit copy C'."""

    def __init__(self, D, bits, g, R, dtype, one_bit_form=IMPROVED_1BIT):
        self.D, self.bits, self.g, self.R, self.dtype = D, bits, g, R, dtype
        self._h = lib().orc_cache_create_form(D, bits, g, R, dtype, one_bit_form)
        if not self._h:
            raise ValueError("oracle cache: invalid configuration")

    def __del__(self):
        if getattr(self, "_h", None) and _lib is not None:   # at interpreter exit the module may be gone already
            _lib.orc_cache_destroy(self._h)
            self._h = None

    def append(self, k_rows, v_rows):
        k_rows, v_rows = _u16(k_rows).reshape(-1, self.D), _u16(v_rows).reshape(-1, self.D)
        assert k_rows.shape == v_rows.shape
        _check(lib().orc_cache_append(self._h, _p(k_rows), _p(v_rows), k_rows.shape[0]), "append")

    def counts(self):
        n, nq = C.c_int(), C.c_int()
        _check(lib().orc_cache_counts(self._h, C.byref(n), C.byref(nq)), "counts")
        return n.value, nq.value

    def export(self):
        """dict of canonical arrays: k_codes [Nq,D], k_mnmx/k_sz [Nq/g,D,2], v_codes [Nq,D], v_mnmx/v_sz [Nq,D/g,2]."""
        _, nq = self.counts()
        D, g = self.D, self.g
        r = dict(k_codes=np.empty((nq, D), np.uint8), k_mnmx=np.empty((nq // g, D, 2), np.float32),
                 k_sz=np.empty((nq // g, D, 2), np.float32), v_codes=np.empty((nq, D), np.uint8),
                 v_mnmx=np.empty((nq, D // g, 2), np.float32), v_sz=np.empty((nq, D // g, 2), np.float32))
        _check(lib().orc_cache_export(self._h, _p(r["k_codes"]), _p(r["k_mnmx"]), _p(r["k_sz"]),
                                      _p(r["v_codes"]), _p(r["v_mnmx"]), _p(r["v_sz"])), "export")
        return r

    def dequant(self):
        _, nq = self.counts()
        k, v = np.empty((nq, self.D)), np.empty((nq, self.D))
        _check(lib().orc_cache_dequant(self._h, _p(k), _p(v)), "dequant")
        return k, v

    def history(self):
        n, _ = self.counts()
        k, v = np.empty((n, self.D)), np.empty((n, self.D))
        _check(lib().orc_cache_history(self._h, _p(k), _p(v)), "history")
        return k, v

    def scores(self, q, sm_scale, select_form=0, P=None):
        """q: uint16 [G, rows, D].  Returns (logits f64 [G, rows, Nq], sigma f64 [Nq]).
        select_form: SELECT_MAX_LOGIT (0) or SELECT_MAX_LOGPROB (1).  P: staged positions (int32, -1 ignored):
        with it the logits are those of the mixed cache (16-bit keys at P), without it pure low-bit."""
        q = _u16(q)
        G, rows, D = q.shape
        assert D == self.D
        _, nq = self.counts()
        logits, sigma = np.empty((G, rows, nq)), np.empty(nq)
        P = np.ascontiguousarray(P, np.int32) if P is not None else np.empty(0, np.int32)
        _check(lib().orc_scores_mixed(self._h, _p(q), G, rows, float(sm_scale), select_form, _p(P) if P.size else None,
                                      int(P.size), _p(logits), _p(sigma)), "scores")
        return logits, sigma

    def attend(self, q, sm_scale, P=None, k_spec=None, v_spec=None):
        """Mixed attention of Eq. 1.  Returns out f64 [G, rows, D]."""
        q = _u16(q)
        G, rows, _ = q.shape
        P = np.ascontiguousarray(P if P is not None else np.empty(0), np.int32)
        ks = _u16(k_spec).reshape(-1) if k_spec is not None else None
        vs = _u16(v_spec).reshape(-1) if v_spec is not None else None
        out = np.empty((G, rows, self.D))
        _check(lib().orc_attend(self._h, _p(q), G, rows, float(sm_scale), _p(P) if P.size else None,
                                P.size, _p(ks), _p(vs), _p(out)), "attend")
        return out

    def full_attention(self, q, sm_scale, k_spec=None, v_spec=None, want_weights=False):
        q = _u16(q)
        G, rows, _ = q.shape
        n, _ = self.counts()
        ks = _u16(k_spec).reshape(-1) if k_spec is not None else None
        vs = _u16(v_spec).reshape(-1) if v_spec is not None else None
        out = np.empty((G, rows, self.D))
        w = np.empty((G, rows, n)) if want_weights else None
        _check(lib().orc_full_attention(self._h, _p(q), G, rows, float(sm_scale), _p(ks), _p(vs),
                                        _p(out), _p(w)), "full_attention")
        return (out, w) if want_weights else out


def topk(sigma, k):
    sigma = np.ascontiguousarray(sigma, np.float64)
    idx = np.empty(k, np.int32)
    _check(lib().orc_topk(_p(sigma), sigma.size, k, _p(idx)), "topk")
    return idx


def hit_rate(weights, idx):
    weights = np.ascontiguousarray(weights, np.float64)
    idx = np.ascontiguousarray(idx, np.int32)
    return lib().orc_hit_rate(_p(weights), weights.size, _p(idx), idx.size)
