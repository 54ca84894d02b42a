"""Thin ctypes binding of libspecache.so: argument marshalling only.

Every step of the decode path runs in the HIP kernels behind the C ABI declared
in include/specache.h; the functions here carry the same names.  Tensors are
PyTorch tensors on the GPU (PyTorch provides device memory and streams) or raw
integer device addresses.  There is no CPU fallback: if the library is missing
or a call fails, an exception is raised.
"""
import ctypes as C
import os

from . import build as _build

FP16, BF16 = 0, 1
OK, EINVAL, ECAPACITY, ENOMEM, EHIP, ESTATE = 0, -1, -2, -3, -4, -5
_NAMES = {EINVAL: "EINVAL", ECAPACITY: "ECAPACITY", ENOMEM: "ENOMEM", EHIP: "EHIP", ESTATE: "ESTATE"}

EXPORTS = ["specache_create", "specache_destroy", "specache_last_error", "specache_counts",
           "specache_plan_append", "specache_quantize_append", "specache_score_topk", "specache_gather",
           "specache_score", "specache_select_gather", "specache_append_score",
           "specache_attend", "specache_score_attend", "specache_append_score_attend", "specache_decode_step", "specache_attend_static", "specache_debug_poison_slot", "specache_debug_fail_alloc", "specache_debug_kernel_choice", "specache_export_quantized", "specache_export_rows", "specache_debug_logits",
           "specache_timing", "specache_measure_hbm_read", "specache_measure_link"]


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "batch", "n_q_heads", "n_kv_heads", "head_dim", "bits",
                                         "group", "residual", "max_seq", "topk", "dtype")] + [("sm_scale", C.c_float),
                                                                                 ("one_bit_form", C.c_int32), ("select_form", C.c_int32),
                                                                                 ("select_cache", C.c_int32), ("async_select", C.c_int32)]


class SpeCacheError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"specache: {_NAMES.get(code, code)}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load libspecache.so.  It is built first if it was never built; a library older than its
    sources is an error (build again: python -m paper_2503_16163_amd.build), so that tests and
    timings never run on a stale build unnoticed."""
    global _lib
    if _lib is None:
        if not os.path.exists(_build.LIB):
            _build.build()
        elif not _build.is_built():
            raise RuntimeError("libspecache.so is older than its sources under csrc/ or include/specache.h: "
                               "run `python -m paper_2503_16163_amd.build` (or __graft_entry__.build())")
        L = C.CDLL(_build.LIB)
        vp, i32 = C.c_void_p, C.c_int32
        L.specache_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
        L.specache_destroy.argtypes = [vp]
        L.specache_last_error.argtypes = [vp]
        L.specache_last_error.restype = C.c_char_p
        L.specache_counts.argtypes = [vp, i32, C.POINTER(i32), C.POINTER(i32)]
        L.specache_plan_append.argtypes = [i32, i32, i32, i32, i32, C.POINTER(i32)]
        L.specache_quantize_append.argtypes = [vp, i32, vp, vp, i32, vp]
        L.specache_score_topk.argtypes = [vp, i32, vp, i32, vp, vp]
        L.specache_gather.argtypes = [vp, i32, vp, i32, vp]
        L.specache_score.argtypes = [vp, i32, vp, i32, vp]
        L.specache_select_gather.argtypes = [vp, i32, vp, i32, vp]
        L.specache_append_score.argtypes = [vp, i32, vp, vp, vp, i32, vp]
        L.specache_attend.argtypes = [vp, i32, vp, i32, vp, vp, i32, vp, vp]
        L.specache_attend_static.argtypes = [vp, i32, vp, i32, vp, vp, i32, vp, vp]
        L.specache_score_attend.argtypes = [vp, i32, vp, i32, vp, vp, i32, vp, vp]
        L.specache_append_score_attend.argtypes = [vp, i32, vp, vp, vp, i32, vp, vp, i32, vp, vp]
        L.specache_decode_step.argtypes = [vp, i32, vp, vp, vp, vp, vp, i32, vp, vp, vp, i32, vp]
        L.specache_debug_poison_slot.argtypes = [vp, i32, i32, vp]
        L.specache_debug_kernel_choice.argtypes = [i32]
        L.specache_debug_fail_alloc.argtypes = [i32]
        L.specache_export_quantized.argtypes = [vp, i32] + [vp] * 6
        L.specache_export_rows.argtypes = [vp, i32, i32, i32, vp]
        L.specache_debug_logits.argtypes = [vp, vp]
        L.specache_timing.argtypes = [vp, i32, vp, vp]
        L.specache_measure_hbm_read.argtypes = [C.c_int64, i32, C.POINTER(C.c_double)]
        L.specache_measure_link.argtypes = [C.c_int64, i32, C.POINTER(C.c_double), C.POINTER(C.c_double)]
        for name in EXPORTS:
            if name != "specache_last_error":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _ptr(x):
    """Device (or host) address of a tensor / numpy array / int / None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return x.ctypes.data


def _stream(s):
    if s is None:
        return None
    if isinstance(s, int):
        return s
    return s.cuda_stream  # torch.cuda.Stream


def plan_append(residual, group, n_tokens, n_quantized, n_new):
    out = C.c_int32()
    rc = lib().specache_plan_append(residual, group, n_tokens, n_quantized, n_new, C.byref(out))
    if rc != OK:
        raise SpeCacheError(rc, "plan_append: inconsistent arguments")
    return out.value


SCORE_ON_VECTOR_ALU, ATTEND_ON_VECTOR_ALU, KEEP_ONE_PASS_LOGITS = 1, 2, 4


def debug_fail_alloc(nth):
    """The nth allocating call of the next specache_create fails (0: off)."""
    rc = lib().specache_debug_fail_alloc(nth)
    if rc != OK:
        raise SpeCacheError(rc, "specache_debug_fail_alloc")


def debug_kernel_choice(flags):
    """Process-wide: send the shapes the integer-matrix-core kernels take to the vector-ALU kernels (A/B timing)."""
    rc = lib().specache_debug_kernel_choice(flags)
    if rc != OK:
        raise SpeCacheError(rc, "debug_kernel_choice: unknown flag")


def measure_hbm_read(nbytes=1 << 30, reps=10):
    """GB/s of a plain 128-bit streaming read of `nbytes` of device memory (median of `reps` launches)."""
    out = C.c_double()
    rc = lib().specache_measure_hbm_read(nbytes, reps, C.byref(out))
    if rc != OK:
        raise SpeCacheError(rc, "measure_hbm_read failed")
    return out.value


def measure_link(nbytes=256 << 20, reps=5):
    """(memcpy GB/s, zero-copy read kernel GB/s) of the host link over `nbytes` of pinned host memory."""
    a, b = C.c_double(), C.c_double()
    rc = lib().specache_measure_link(nbytes, reps, C.byref(a), C.byref(b))
    if rc != OK:
        raise SpeCacheError(rc, "measure_link failed")
    return a.value, b.value


class SpeCache:
    """Owner of a specache_ctx; methods mirror the C calls one to one."""

    def __init__(self, n_layers, batch, n_q_heads, n_kv_heads, bits, group, max_seq, topk, dtype,
                 residual=64, head_dim=128, sm_scale=0.0, one_bit_form=0, select_form=0, select_cache=0, async_select=0):
        self.cfg = Config(n_layers, batch, n_q_heads, n_kv_heads, head_dim, bits, group, residual, max_seq,
                          topk, dtype, sm_scale, one_bit_form, select_form, select_cache, async_select)
        self._ctx = C.c_void_p()
        rc = lib().specache_create(C.byref(self.cfg), C.byref(self._ctx))
        if rc != OK:
            raise SpeCacheError(rc, lib().specache_last_error(None).decode())

    def close(self):
        if getattr(self, "_ctx", None):
            lib().specache_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        self.close()

    def _check(self, rc):
        if rc != OK:
            raise SpeCacheError(rc, lib().specache_last_error(self._ctx).decode())

    def counts(self, layer):
        n, nq = C.c_int32(), C.c_int32()
        self._check(lib().specache_counts(self._ctx, layer, C.byref(n), C.byref(nq)))
        return n.value, nq.value

    def quantize_append(self, layer, k_new, v_new, n_new, stream=None):
        self._check(lib().specache_quantize_append(self._ctx, layer, _ptr(k_new), _ptr(v_new), n_new, _stream(stream)))

    def score_topk(self, layer, q, n_rows, topk_idx_out, stream=None):
        self._check(lib().specache_score_topk(self._ctx, layer, _ptr(q), n_rows, _ptr(topk_idx_out), _stream(stream)))

    def score(self, layer, q, n_rows, stream=None):
        self._check(lib().specache_score(self._ctx, layer, _ptr(q), n_rows, _stream(stream)))

    def append_score(self, layer, k_new, v_new, q, n_rows, stream=None):
        self._check(lib().specache_append_score(self._ctx, layer, _ptr(k_new), _ptr(v_new), _ptr(q), n_rows, _stream(stream)))

    def select_gather(self, layer, topk_idx_out, slot, side_stream=None):
        self._check(lib().specache_select_gather(self._ctx, layer, _ptr(topk_idx_out), slot, _stream(side_stream)))

    def gather(self, layer, idx, slot, side_stream=None):
        self._check(lib().specache_gather(self._ctx, layer, _ptr(idx), slot, _stream(side_stream)))

    def attend(self, layer, q, n_rows, k_spec, v_spec, slot, out, stream=None):
        self._check(lib().specache_attend(self._ctx, layer, _ptr(q), n_rows, _ptr(k_spec), _ptr(v_spec), slot,
                                          _ptr(out), _stream(stream)))

    def score_attend(self, layer, q, n_rows, k_spec, v_spec, slot, out, stream=None):
        self._check(lib().specache_score_attend(self._ctx, layer, _ptr(q), n_rows, _ptr(k_spec), _ptr(v_spec), slot,
                                                _ptr(out), _stream(stream)))

    def append_score_attend(self, layer, k_new, v_new, q, n_rows, k_spec, v_spec, slot, out, stream=None):
        self._check(lib().specache_append_score_attend(self._ctx, layer, _ptr(k_new), _ptr(v_new), _ptr(q), n_rows,
                                                       _ptr(k_spec), _ptr(v_spec), slot, _ptr(out), _stream(stream)))

    def decode_step(self, layer, k_new, v_new, q, k_spec, v_spec, read_slot, out, stream, topk_idx_out, fill_slot, side_stream):
        self._check(lib().specache_decode_step(self._ctx, layer, _ptr(k_new), _ptr(v_new), _ptr(q), _ptr(k_spec), _ptr(v_spec),
                                               read_slot, _ptr(out), _stream(stream), _ptr(topk_idx_out), fill_slot,
                                               _stream(side_stream)))

    def attend_static(self, layer, q, n_rows, k_spec, v_spec, slot, out, stream=None):
        self._check(lib().specache_attend_static(self._ctx, layer, _ptr(q), n_rows, _ptr(k_spec), _ptr(v_spec), slot,
                                                 _ptr(out), _stream(stream)))

    def debug_poison_slot(self, layer, slot, stream=None):
        self._check(lib().specache_debug_poison_slot(self._ctx, layer, slot, _stream(stream)))

    KERNELS = ("flush", "append_copy", "score", "topk", "gather", "attend", "attend_combine", "score_attend")

    def timing(self, enable):
        """Collect and reset per-kernel event timings; returns {kernel: (total_us, launches)}."""
        us = (C.c_double * len(self.KERNELS))()
        n = (C.c_int64 * len(self.KERNELS))()
        self._check(lib().specache_timing(self._ctx, int(bool(enable)), us, n))
        return {k: (us[i], n[i]) for i, k in enumerate(self.KERNELS)}

    # ---- parity hooks (host numpy arrays) ------------------------------------
    def export_quantized(self, layer):
        import numpy as np
        c = self.cfg
        rows, (_, nq), g, D = c.batch * c.n_kv_heads, self.counts(layer), c.group, c.head_dim
        shp = (c.batch, c.n_kv_heads)
        r = dict(k_codes=np.zeros(shp + (nq, D), np.uint8), k_mnmx=np.zeros(shp + (nq // g, D, 2), np.uint16),
                 k_sz=np.zeros(shp + (nq // g, D, 2), np.float32), v_codes=np.zeros(shp + (nq, D), np.uint8),
                 v_mnmx=np.zeros(shp + (nq, D // g, 2), np.uint16), v_sz=np.zeros(shp + (nq, D // g, 2), np.float32))
        self._check(lib().specache_export_quantized(self._ctx, layer, _ptr(r["k_codes"]), _ptr(r["k_mnmx"]),
                                                    _ptr(r["k_sz"]), _ptr(r["v_codes"]), _ptr(r["v_mnmx"]),
                                                    _ptr(r["v_sz"])))
        return r

    def export_rows(self, layer, first, count):
        import numpy as np
        c = self.cfg
        out = np.zeros((c.batch, c.n_kv_heads, count, 2, c.head_dim), np.uint16)
        self._check(lib().specache_export_rows(self._ctx, layer, first, count, _ptr(out)))
        return out

    def debug_logits(self, layer, n_rows):
        import numpy as np
        c = self.cfg
        _, nq = self.counts(layer)
        out = np.zeros((c.batch, c.n_q_heads, n_rows, nq), np.float32)
        self._check(lib().specache_debug_logits(self._ctx, _ptr(out)))
        return out
