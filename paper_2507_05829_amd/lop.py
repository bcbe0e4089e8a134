"""ctypes binding of liblop.so (see include/lop.h). Argument marshalling only: every
step of the path runs inside the library's HIP kernels. There is no fallback: if the
library is not built, importing this module raises.

Module-level functions carry the C names (lop_plan, lop_run_band, lop_run_chain, ...);
``Plan`` is a small convenience wrapper over the same calls. Device and pinned-host
buffers are torch tensors used purely as memory; their ``data_ptr()`` is what crosses the
boundary.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_float, c_int, c_size_t, c_uint, c_void_p
from typing import List, Optional, Sequence, Tuple

import numpy as np
# torch ships its own HIP runtime; it has to be in the process before liblop.so is
# loaded so that both resolve to the same runtime (device pointers and streams are
# shared between them).
import torch  # noqa: F401

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblop.so")

LOP_OK = 0
LOP_ERR_INVALID_ARG, LOP_ERR_UNSUPPORTED, LOP_ERR_SHAPE, LOP_ERR_BAND_RANGE = -1, -2, -3, -4
LOP_ERR_OOM, LOP_ERR_HIP, LOP_ERR_NOT_READY, LOP_ERR_TOO_LARGE = -5, -6, -7, -8
LOP_STATIC_SCRATCH_BYTES = 64 << 20
LOP_CONV2D, LOP_DWCONV2D, LOP_MAXPOOL2D, LOP_ELTWISE = 0, 1, 2, 3
LOP_ACT_NONE, LOP_ACT_RELU, LOP_ACT_RELU6 = 0, 1, 2
LOP_F32, LOP_BF16 = 0, 1
LOP_INPUT, LOP_NO_RESIDUAL = -1, -2
LOP_MAX_BANDS = 64
LOP_FLAG_NO_D2H, LOP_FLAG_PLAN_ONLY, LOP_FLAG_GRAPH, LOP_FLAG_DMA_COPY = 1, 2, 4, 8
LOP_FLAG_REUSE = 16
LOP_FLAG_INDEPENDENT = 0
LOP_FLAG_NO_FUSE = 32
LOP_FLAG_POISON_SCRATCH = 64
LOP_FLAG_BATCH_BANDS = 128
LOP_LINK_INDEPENDENT, LOP_LINK_QUEUED = 0, 1


def LOP_FLAG_LANES(n: int) -> int:
    return (n & 0xFF) << 8


EXPORTS = [
    "lop_plan", "lop_plan_out_desc", "lop_plan_layer_desc", "lop_plan_n_bands",
    "lop_plan_n_layers", "lop_plan_band_out_rows", "lop_plan_band_in_rows",
    "lop_plan_band_layer_rows", "lop_plan_stats", "lop_plan_layer_work", "lop_run_band",
    "lop_run_chain", "lop_synchronize", "lop_time_layer", "lop_plan_destroy", "lop_strerror",
    "lop_last_hip_error", "lop_plan_layer_kernel", "lop_profile_chain", "lop_copy_chain",
    "lop_plan_band_compute_rows", "lop_plan_rowwise", "lop_loss_eval", "lop_loss_solve",
    "lop_run_two_party", "lop_measure_ceilings", "lop_run_chain_static", "lop_debug_guard_check",
]


class lop_layer_t(Structure):
    _fields_ = [("op", c_int), ("c_in", c_int), ("c_out", c_int),
                ("kh", c_int), ("kw", c_int), ("sh", c_int), ("sw", c_int),
                ("ph", c_int), ("pw", c_int), ("dh", c_int), ("dw", c_int),
                ("act", c_int), ("input_from", c_int), ("residual_from", c_int),
                ("weight", c_void_p), ("bias", c_void_p)]


class lop_rowwise_t(Structure):
    _fields_ = [("k", c_int), ("n", c_int), ("act", c_int), ("input_from", c_int),
                ("residual_from", c_int), ("weight", c_void_p), ("bias", c_void_p)]


class lop_loss_layer_t(Structure):
    _fields_ = [("n_ops", c_int), ("input_from", c_int), ("residual_from", c_int),
                ("k", c_int), ("s", c_int), ("p", c_int), ("d", c_int),
                ("cm_fixed", c_double), ("cm_row", c_double), ("cr_fixed", c_double),
                ("cr_row", c_double), ("row_bytes", c_double)]


class lop_loss_alloc_t(Structure):
    _fields_ = [("m_lo", c_int), ("m_hi", c_int), ("r_lo", c_int), ("r_hi", c_int)]


class lop_two_party_stats_t(Structure):
    _fields_ = [("total_ms", c_float), ("bytes_to_m", c_double), ("bytes_to_r", c_double),
                ("transfers", c_int)]


class lop_ceilings_t(Structure):
    _fields_ = [("hbm_copy_gbs", c_double), ("mfma_bf16_tflops", c_double), ("mfma_f32_tflops", c_double),
                ("launch_floor_us", c_double), ("graph_node_floor_us", c_double)]


class lop_tensor_desc_t(Structure):
    _fields_ = [("n", c_int), ("c", c_int), ("h", c_int), ("w", c_int), ("dtype", c_int)]


class lop_rows_t(Structure):
    _fields_ = [("lo", c_int), ("hi", c_int)]


class lop_timing_t(Structure):
    _fields_ = [("n_bands", c_int), ("wall_ms", c_float), ("compute_ms", c_float),
                ("copy_ms", c_float), ("band_compute_ms", c_float * LOP_MAX_BANDS),
                ("band_copy_ms", c_float * LOP_MAX_BANDS),
                ("band_ready_ms", c_float * LOP_MAX_BANDS)]


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2507_05829_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    P = c_void_p
    sig = {
        "lop_plan": (c_int, [POINTER(lop_layer_t), c_int, POINTER(lop_tensor_desc_t), c_int, c_uint,
                             POINTER(P)]),
        "lop_plan_rowwise": (c_int, [POINTER(lop_rowwise_t), c_int, c_int, c_int, c_int, c_int, c_uint,
                                     POINTER(P)]),
        "lop_loss_eval": (c_int, [POINTER(lop_loss_layer_t), c_int, c_int, c_double, c_double, c_double,
                                  POINTER(lop_loss_alloc_t), POINTER(c_double), POINTER(c_double),
                                  POINTER(c_double), POINTER(c_int), c_int]),
        "lop_loss_solve": (c_int, [POINTER(lop_loss_layer_t), c_int, c_int, c_double, c_double, c_double,
                                   c_int, c_int, ctypes.c_ulonglong, POINTER(lop_loss_alloc_t),
                                   POINTER(c_double), POINTER(c_int), c_int]),
        "lop_plan_out_desc": (c_int, [P, POINTER(lop_tensor_desc_t)]),
        "lop_plan_layer_desc": (c_int, [P, c_int, POINTER(lop_tensor_desc_t)]),
        "lop_plan_n_bands": (c_int, [P]),
        "lop_plan_n_layers": (c_int, [P]),
        "lop_plan_band_out_rows": (c_int, [P, c_int, POINTER(lop_rows_t)]),
        "lop_plan_band_in_rows": (c_int, [P, c_int, POINTER(lop_rows_t)]),
        "lop_plan_band_layer_rows": (c_int, [P, c_int, c_int, POINTER(lop_rows_t)]),
        "lop_plan_band_compute_rows": (c_int, [P, c_int, c_int, POINTER(lop_rows_t)]),
        "lop_plan_stats": (c_int, [P, POINTER(c_double), POINTER(c_double), POINTER(c_size_t)]),
        "lop_plan_layer_work": (c_int, [P, c_int, c_int, POINTER(c_double), POINTER(c_double)]),
        "lop_run_band": (c_int, [P, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]),
        "lop_run_chain": (c_int, [P, c_void_p, c_void_p, c_void_p, c_void_p, POINTER(lop_timing_t)]),
        "lop_run_chain_static": (c_int, [P, c_void_p, c_void_p, c_void_p]),
        "lop_synchronize": (c_int, [P]),
        "lop_time_layer": (c_int, [P, c_int, c_int, c_void_p, c_void_p, c_int, POINTER(c_float)]),
        "lop_plan_destroy": (None, [P]),
        "lop_plan_layer_kernel": (c_int, [P, c_int, c_int, ctypes.c_char_p, c_size_t, POINTER(c_int)]),
        "lop_profile_chain": (c_int, [P, c_void_p, c_void_p, c_int, POINTER(c_float), POINTER(c_float)]),
        "lop_copy_chain": (c_int, [P, c_void_p, c_void_p]),
        "lop_run_two_party": (c_int, [P, c_void_p, c_void_p, POINTER(lop_loss_alloc_t), c_int,
                                      POINTER(lop_loss_layer_t), c_double, c_double,
                                      POINTER(lop_two_party_stats_t)]),
        "lop_measure_ceilings": (c_int, [POINTER(lop_ceilings_t)]),
        "lop_debug_guard_check": (c_int, []),
        "lop_strerror": (c_char_p, [c_int]),
        "lop_last_hip_error": (c_int, []),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype, fn.argtypes = res, args
    return lib


_lib = _load()


class LopError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.lop_strerror(code).decode()
        if code == LOP_ERR_HIP:
            msg += f" (hipError_t {_lib.lop_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def _check(code: int, where: str) -> None:
    if code != LOP_OK:
        raise LopError(code, where)


def _ptr(t) -> c_void_p:
    """Raw address of a torch tensor / numpy array / int / None."""
    if t is None:
        return c_void_p(0)
    if isinstance(t, int):
        return c_void_p(t)
    if hasattr(t, "data_ptr"):
        return c_void_p(t.data_ptr())
    return c_void_p(t.ctypes.data)


def _stream(s) -> c_void_p:
    if s is None:
        return c_void_p(0)
    if isinstance(s, int):
        return c_void_p(s)
    return c_void_p(s.cuda_stream)


# ------------------------------------------------------------------ C-named functions

def lop_plan(layers: Sequence[lop_layer_t], in_desc: lop_tensor_desc_t, n_bands: int,
             flags: int = 0) -> c_void_p:
    arr = (lop_layer_t * len(layers))(*layers) if len(layers) else None
    out = c_void_p(0)
    _check(_lib.lop_plan(arr, len(layers), byref(in_desc), n_bands, flags, byref(out)), "lop_plan")
    return out


def lop_plan_rowwise(layers: Sequence[lop_rowwise_t], m: int, k: int, dtype: int, n_bands: int,
                     flags: int = 0) -> c_void_p:
    arr = (lop_rowwise_t * len(layers))(*layers) if len(layers) else None
    out = c_void_p(0)
    _check(_lib.lop_plan_rowwise(arr, len(layers), m, k, dtype, n_bands, flags, byref(out)),
           "lop_plan_rowwise")
    return out


def _loss_layers(layers):
    """lop_loss_layer_t array from objects with the fields of the struct (duck-typed)."""
    return (lop_loss_layer_t * len(layers))(*[
        lop_loss_layer_t(L.n_ops, L.input_from, L.residual_from, L.k, L.s, L.p, L.d,
                         L.cm_fixed, L.cm_row, L.cr_fixed, L.cr_row, L.row_bytes) for L in layers])


def lop_loss_eval(layers, in_rows: int, in_row_bytes: float, bandwidth: float, latency: float,
                  sched: Sequence[Tuple[Tuple[int, int], Tuple[int, int]]], link_model: int = 0):
    """sched: per vertex ((m_lo, m_hi), (r_lo, r_hi)). Returns (T, s_m, s_r, violations)."""
    n = len(layers)
    arr = (lop_loss_alloc_t * n)(*[lop_loss_alloc_t(m[0], m[1], r[0], r[1]) for m, r in sched])
    T, viol = c_double(0.0), c_int(0)
    s_m, s_r = (c_double * (n + 1))(), (c_double * n)()
    _check(_lib.lop_loss_eval(_loss_layers(layers), n, in_rows, in_row_bytes, bandwidth, latency,
                              arr, byref(T), s_m, s_r, byref(viol), link_model), "lop_loss_eval")
    return T.value, list(s_m), list(s_r), viol.value


def lop_loss_solve(layers, in_rows: int, in_row_bytes: float, bandwidth: float, latency: float,
                   population: int = 0, generations: int = 200, seed: int = 1, link_model: int = 0):
    """Returns (schedule as in lop_loss_eval, T, violations)."""
    n = len(layers)
    best = (lop_loss_alloc_t * n)()
    T, viol = c_double(0.0), c_int(0)
    _check(_lib.lop_loss_solve(_loss_layers(layers), n, in_rows, in_row_bytes, bandwidth, latency,
                               population, generations, seed, best, byref(T), byref(viol), link_model),
           "lop_loss_solve")
    return [((a.m_lo, a.m_hi), (a.r_lo, a.r_hi)) for a in best], T.value, viol.value


def lop_plan_destroy(plan) -> None:
    _lib.lop_plan_destroy(plan)


def lop_plan_out_desc(plan) -> lop_tensor_desc_t:
    d = lop_tensor_desc_t()
    _check(_lib.lop_plan_out_desc(plan, byref(d)), "lop_plan_out_desc")
    return d


def lop_plan_layer_desc(plan, layer: int) -> lop_tensor_desc_t:
    d = lop_tensor_desc_t()
    _check(_lib.lop_plan_layer_desc(plan, layer, byref(d)), "lop_plan_layer_desc")
    return d


def lop_plan_n_bands(plan) -> int:
    return _lib.lop_plan_n_bands(plan)


def lop_plan_n_layers(plan) -> int:
    return _lib.lop_plan_n_layers(plan)


def _rows(fn, name, *args) -> Tuple[int, int]:
    r = lop_rows_t()
    _check(fn(*args, byref(r)), name)
    return (r.lo, r.hi)


def lop_plan_band_out_rows(plan, band: int) -> Tuple[int, int]:
    return _rows(_lib.lop_plan_band_out_rows, "lop_plan_band_out_rows", plan, band)


def lop_plan_band_in_rows(plan, band: int) -> Tuple[int, int]:
    return _rows(_lib.lop_plan_band_in_rows, "lop_plan_band_in_rows", plan, band)


def lop_plan_band_layer_rows(plan, band: int, layer: int) -> Tuple[int, int]:
    return _rows(_lib.lop_plan_band_layer_rows, "lop_plan_band_layer_rows", plan, band, layer)


def lop_plan_band_compute_rows(plan, band: int, layer: int) -> Tuple[int, int]:
    return _rows(_lib.lop_plan_band_compute_rows, "lop_plan_band_compute_rows", plan, band, layer)


def lop_plan_stats(plan) -> Tuple[float, float, int]:
    u, e, s = c_double(), c_double(), c_size_t()
    _check(_lib.lop_plan_stats(plan, byref(u), byref(e), byref(s)), "lop_plan_stats")
    return u.value, e.value, s.value


def lop_plan_layer_work(plan, band: int, layer: int) -> Tuple[float, float]:
    f, b = c_double(), c_double()
    _check(_lib.lop_plan_layer_work(plan, band, layer, byref(f), byref(b)), "lop_plan_layer_work")
    return f.value, b.value


def lop_run_band(plan, band: int, d_in, d_out, h_out=None, compute_stream=None,
                 copy_stream=None) -> None:
    _check(_lib.lop_run_band(plan, band, _ptr(d_in), _ptr(d_out), _ptr(h_out),
                             _stream(compute_stream), _stream(copy_stream)), "lop_run_band")


def lop_run_chain(plan, d_in, d_out, h_out=None, compute_stream=None,
                  timing: bool = False) -> Optional[lop_timing_t]:
    t = lop_timing_t() if timing else None
    _check(_lib.lop_run_chain(plan, _ptr(d_in), _ptr(d_out), _ptr(h_out), _stream(compute_stream),
                              byref(t) if timing else None), "lop_run_chain")
    return t


def lop_run_chain_static(plan, d_in, d_out, stream=None) -> None:
    _check(_lib.lop_run_chain_static(plan, _ptr(d_in), _ptr(d_out), _stream(stream)), "lop_run_chain_static")


def lop_synchronize(plan) -> None:
    _check(_lib.lop_synchronize(plan), "lop_synchronize")


def lop_time_layer(plan, band: int, layer: int, d_in, d_out, iters: int = 20) -> float:
    ms = c_float()
    _check(_lib.lop_time_layer(plan, band, layer, _ptr(d_in), _ptr(d_out), iters, byref(ms)),
           "lop_time_layer")
    return ms.value


def lop_plan_layer_kernel(plan, band: int, layer: int) -> Tuple[str, int]:
    """(kernel instance name, number of K slices) of a (band, layer) launch."""
    buf = ctypes.create_string_buffer(128)
    k = c_int(0)
    _check(_lib.lop_plan_layer_kernel(plan, band, layer, buf, 128, byref(k)), "lop_plan_layer_kernel")
    return buf.value.decode(), k.value


def lop_profile_chain(plan, d_in, d_out, iters: int = 5) -> Tuple[np.ndarray, np.ndarray]:
    """Mean ms of every (band, layer) main kernel and of its split-K finish kernel."""
    nb, nl = lop_plan_n_bands(plan), lop_plan_n_layers(plan)
    ms = np.zeros((nb, nl), np.float32)
    fin = np.zeros((nb, nl), np.float32)
    _check(_lib.lop_profile_chain(plan, _ptr(d_in), _ptr(d_out), iters,
                                  ms.ctypes.data_as(POINTER(c_float)),
                                  fin.ctypes.data_as(POINTER(c_float))), "lop_profile_chain")
    return ms, fin


def lop_copy_chain(plan, d_out, h_out) -> None:
    _check(_lib.lop_copy_chain(plan, _ptr(d_out), _ptr(h_out)), "lop_copy_chain")


def lop_run_two_party(plan, d_in, d_out, sched, bandwidth: float, latency: float = 0.0, costs=None):
    """sched: per layer ((m_lo, m_hi), (r_lo, r_hi)); costs: objects with the lop_loss_layer_t
    fields or None. Returns the filled lop_two_party_stats_t."""
    n = len(sched)
    arr = (lop_loss_alloc_t * n)(*[lop_loss_alloc_t(m[0], m[1], r[0], r[1]) for m, r in sched])
    st = lop_two_party_stats_t()
    _check(_lib.lop_run_two_party(plan, _ptr(d_in), _ptr(d_out), arr, n,
                                  _loss_layers(costs) if costs is not None else None,
                                  bandwidth, latency, byref(st)), "lop_run_two_party")
    return st


def lop_measure_ceilings() -> lop_ceilings_t:
    c = lop_ceilings_t()
    _check(_lib.lop_measure_ceilings(byref(c)), "lop_measure_ceilings")
    return c


def lop_debug_guard_check() -> int:
    return _lib.lop_debug_guard_check()


def lop_strerror(code: int) -> str:
    return _lib.lop_strerror(code).decode()


# ------------------------------------------------------------------ chain marshalling

_OPS = {"conv": LOP_CONV2D, "dwconv": LOP_DWCONV2D, "maxpool": LOP_MAXPOOL2D, "eltwise": LOP_ELTWISE}
_ACTS = {"none": LOP_ACT_NONE, "relu": LOP_ACT_RELU, "relu6": LOP_ACT_RELU6}
_DTYPES = {"f32": LOP_F32, "bf16": LOP_BF16}


def _storage(a: np.ndarray, dtype: str) -> np.ndarray:
    """float32 values -> the storage type's bytes (bf16: the upper 16 bits, which is exact
    because the values are already bfloat16-representable)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "f32":
        return a
    u = a.view(np.uint32)
    if np.any(u & 0xFFFF):
        raise ValueError("bf16 plan: values must be bfloat16-representable")
    return (u >> 16).astype(np.uint16)


def layers_from_chain(chain, tensors=None):
    """lop_layer_t list from a chain description (duck-typed: .layers with op, c_in, c_out,
    k, s, p, d, act, input_from, residual_from) and optional host tensors. Returns the list
    and the numpy arrays that must stay alive until lop_plan returns."""
    keep, out = [], []
    for i, L in enumerate(chain.layers):
        d = lop_layer_t(_OPS[L.op], L.c_in, L.c_out, L.k[0], L.k[1], L.s[0], L.s[1],
                        L.p[0], L.p[1], L.d[0], L.d[1], _ACTS[L.act], L.input_from,
                        L.residual_from, None, None)
        if tensors is not None:
            if tensors.weights[i] is not None:
                w = _storage(tensors.weights[i], chain.dtype)
                keep.append(w)
                d.weight = w.ctypes.data
            if tensors.biases[i] is not None:
                b = np.ascontiguousarray(tensors.biases[i], dtype=np.float32)
                keep.append(b)
                d.bias = b.ctypes.data
        out.append(d)
    return out, keep


class Plan:
    """Owns a lop_plan_t handle."""

    def __init__(self, chain, tensors=None, n_bands: Optional[int] = None, flags: int = 0):
        layers, keep = layers_from_chain(chain, tensors)
        n, c, h, w = chain.in_shape
        desc = lop_tensor_desc_t(n, c, h, w, _DTYPES[chain.dtype])
        if tensors is None:
            flags |= LOP_FLAG_PLAN_ONLY
        self.handle = lop_plan(layers, desc, chain.n_bands if n_bands is None else n_bands, flags)
        del keep
        self.n_bands = lop_plan_n_bands(self.handle)
        self.n_layers = lop_plan_n_layers(self.handle)
        self.dtype = chain.dtype

    @classmethod
    def rowwise(cls, chain, tensors=None, n_bands: Optional[int] = None, flags: int = 0) -> "Plan":
        """Plan for a chain of row-wise operators (duck-typed: .m, .k, .dtype, .n_bands and
        .layers with k, n, act, input_from, residual_from) through lop_plan_rowwise."""
        keep, layers = [], []
        for i, L in enumerate(chain.layers):
            d = lop_rowwise_t(L.k, L.n, _ACTS[L.act], L.input_from, L.residual_from, None, None)
            if tensors is not None:
                w = _storage(tensors.weights[i], chain.dtype)
                keep.append(w)
                d.weight = w.ctypes.data
                if tensors.biases[i] is not None:
                    b = np.ascontiguousarray(tensors.biases[i], dtype=np.float32)
                    keep.append(b)
                    d.bias = b.ctypes.data
            layers.append(d)
        if tensors is None:
            flags |= LOP_FLAG_PLAN_ONLY
        self = cls.__new__(cls)
        self.handle = lop_plan_rowwise(layers, chain.m, chain.k, _DTYPES[chain.dtype],
                                       chain.n_bands if n_bands is None else n_bands, flags)
        del keep
        self.n_bands = lop_plan_n_bands(self.handle)
        self.n_layers = lop_plan_n_layers(self.handle)
        self.dtype = chain.dtype
        return self

    def destroy(self) -> None:
        if getattr(self, "handle", None):
            _lib.lop_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:      # interpreter shutdown: the library may already be gone
            pass

    def out_shape(self) -> Tuple[int, int, int, int]:
        d = lop_plan_out_desc(self.handle)
        return (d.n, d.c, d.h, d.w)

    def layer_shape(self, layer: int) -> Tuple[int, int, int, int]:
        d = lop_plan_layer_desc(self.handle, layer)
        return (d.n, d.c, d.h, d.w)

    def band_out_rows(self, b): return lop_plan_band_out_rows(self.handle, b)
    def band_in_rows(self, b): return lop_plan_band_in_rows(self.handle, b)
    def band_layer_rows(self, b, l): return lop_plan_band_layer_rows(self.handle, b, l)
    def band_compute_rows(self, b, l): return lop_plan_band_compute_rows(self.handle, b, l)
    def stats(self): return lop_plan_stats(self.handle)
    def layer_work(self, b, l): return lop_plan_layer_work(self.handle, b, l)

    def run_band(self, band, d_in, d_out, h_out=None, compute_stream=None, copy_stream=None):
        lop_run_band(self.handle, band, d_in, d_out, h_out, compute_stream, copy_stream)

    def run_chain(self, d_in, d_out, h_out=None, compute_stream=None, timing=False):
        return lop_run_chain(self.handle, d_in, d_out, h_out, compute_stream, timing)

    def run_chain_static(self, d_in, d_out, stream=None):
        lop_run_chain_static(self.handle, d_in, d_out, stream)

    def synchronize(self): lop_synchronize(self.handle)

    def layer_kernel(self, b, l): return lop_plan_layer_kernel(self.handle, b, l)
    def profile_chain(self, d_in, d_out, iters=5): return lop_profile_chain(self.handle, d_in, d_out, iters)
    def copy_chain(self, d_out, h_out): lop_copy_chain(self.handle, d_out, h_out)

    def run_two_party(self, d_in, d_out, sched, bandwidth, latency=0.0, costs=None):
        return lop_run_two_party(self.handle, d_in, d_out, sched, bandwidth, latency, costs)

    def time_layer(self, band, layer, d_in, d_out, iters=20):
        return lop_time_layer(self.handle, band, layer, d_in, d_out, iters)
