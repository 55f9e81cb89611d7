"""Thin ctypes binding of libscheinfer.so (see include/scheinfer.h for the contract).

Argument marshalling only: every step of the layer runs in the library's HIP kernels / host
workers.  PyTorch appears only as the owner of device memory and streams in the callers.
The library must have been built (``python paper_2411_15715_amd/build.py`` or
``__graft_entry__.build()``); loading fails loudly otherwise - there is no fallback path.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libscheinfer.so")

SI_OK, SI_EINVAL, SI_ENOMEM, SI_EHIP, SI_ESTATE = 0, -1, -2, -3, -4
SI_AUTO, SI_DECODE, SI_PREFILL = 0, 1, 2
SI_DECODE_AUTO_T, SI_DECODE_MAX_T = 8, 16

EXPORTS = ["si_layer_create", "si_layer_split_info", "si_split_counts", "si_layer_forward", "si_route",
           "si_layer_stats", "si_layer_set_profiling", "si_repack_chunks", "si_cc_compute", "si_layer_destroy", "si_last_error", "si_version"]


class si_layer_desc_t(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("d_ff_shared", ctypes.c_int32), ("r_gg", ctypes.c_float),
                ("r_cg", ctypes.c_float), ("r_cc", ctypes.c_float), ("granule", ctypes.c_int32),
                ("max_tokens", ctypes.c_int32), ("cc_threads", ctypes.c_int32), ("device", ctypes.c_int32),
                ("stage_mib", ctypes.c_int32), ("n_stage", ctypes.c_int32)]


class si_routing_out_t(ctypes.Structure):
    _fields_ = [("idx", ctypes.c_void_p), ("w", ctypes.c_void_p), ("count", ctypes.c_void_p),
                ("off", ctypes.c_void_p), ("perm", ctypes.c_void_p), ("inv", ctypes.c_void_p)]


class si_stats_t(ctypes.Structure):
    _fields_ = [("total_ms", ctypes.c_float), ("copy_ms", ctypes.c_float), ("gpu_ms", ctypes.c_float),
                ("cc_ms", ctypes.c_float), ("route_ms", ctypes.c_float), ("bytes_streamed", ctypes.c_double),
                ("bytes_gg", ctypes.c_double), ("bytes_cc", ctypes.c_double), ("overlap", ctypes.c_float),
                ("n_copies", ctypes.c_int32), ("n_touched", ctypes.c_int32), ("path", ctypes.c_int32),
                ("kernel_ms", ctypes.c_float * 8), ("kernel_launches", ctypes.c_int32 * 8),
                ("staged_ms", ctypes.c_float), ("handoff_ms", ctypes.c_float), ("enqueue_ms", ctypes.c_float)]


SI_K_NAMES = ["route", "decode_gateup", "decode_down", "decode_combine", "prefill_gateup", "prefill_down",
              "prefill_combine", "fill"]


class ScheInferError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("scheinfer error %d: %s" % (code, text))
        self.code = code


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libscheinfer.so is not built: run `python paper_2411_15715_amd/build.py`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_float
        L.si_layer_create.restype = ctypes.c_int
        L.si_layer_create.argtypes = [ctypes.POINTER(si_layer_desc_t), vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        L.si_layer_split_info.restype = ctypes.c_int
        L.si_layer_split_info.argtypes = [vp] + [ctypes.POINTER(i32)] * 6
        L.si_split_counts.restype = ctypes.c_int
        L.si_split_counts.argtypes = [i32, i32, f32, f32] + [ctypes.POINTER(i32)] * 3
        L.si_layer_forward.restype = ctypes.c_int
        L.si_layer_forward.argtypes = [vp, vp, vp, i32, i32, i32, vp, ctypes.POINTER(si_routing_out_t), vp]
        L.si_route.restype = ctypes.c_int
        L.si_route.argtypes = [vp, i32, i32, i32, ctypes.POINTER(si_routing_out_t), vp]
        L.si_layer_stats.restype = ctypes.c_int
        L.si_layer_stats.argtypes = [vp, ctypes.POINTER(si_stats_t)]
        L.si_layer_set_profiling.restype = ctypes.c_int
        L.si_layer_set_profiling.argtypes = [vp, i32]
        L.si_repack_chunks.restype = ctypes.c_int
        L.si_repack_chunks.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp]
        L.si_cc_compute.restype = ctypes.c_int
        L.si_cc_compute.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, ctypes.c_uint64, i32, vp, i32, i32, vp]
        L.si_layer_destroy.restype = None
        L.si_layer_destroy.argtypes = [vp]
        L.si_last_error.restype = ctypes.c_char_p
        L.si_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def si_last_error() -> str:
    return lib().si_last_error().decode()


def si_version() -> str:
    return lib().si_version().decode()


def _check(rc):
    if rc != SI_OK:
        raise ScheInferError(rc, si_last_error())


def _host_ptr(a):
    """Address of a C-contiguous uint16 NumPy array (or None)."""
    if a is None:
        return None
    if a.dtype.itemsize != 2 or not a.flags["C_CONTIGUOUS"]:
        raise ValueError("weights must be C-contiguous 16-bit arrays (bf16 bit patterns)")
    return ctypes.c_void_p(a.ctypes.data)


def si_split_counts(d_ff, granule, r_gg, r_cg):
    """(n_gg, n_cg, n_cc)"""
    n = [ctypes.c_int32(0) for _ in range(3)]
    _check(lib().si_split_counts(d_ff, granule, r_gg, r_cg, *[ctypes.byref(v) for v in n]))
    return tuple(v.value for v in n)


def si_layer_create(d_model, d_ff, n_experts, top_k, w_gate, w_up, w_down, r_gg, r_cg, r_cc, max_tokens,
                    d_ff_shared=0, shared=None, granule=0, cc_threads=0, device=0, stage_mib=0, n_stage=0):
    """Returns the opaque layer handle (an int).  Weights are host NumPy uint16 arrays."""
    desc = si_layer_desc_t(d_model, d_ff, n_experts, top_k, d_ff_shared, r_gg, r_cg, r_cc, granule, max_tokens,
                           cc_threads, device, stage_mib, n_stage)
    sg, su, sd = shared if shared is not None else (None, None, None)
    out = ctypes.c_void_p(None)
    _check(lib().si_layer_create(ctypes.byref(desc), _host_ptr(w_gate), _host_ptr(w_up), _host_ptr(w_down),
                                 _host_ptr(sg), _host_ptr(su), _host_ptr(sd), ctypes.byref(out)))
    return out.value


def si_layer_split_info(layer):
    """dict of hidden-column counts n_gg, n_cg, n_cc (routed) and s_gg, s_cg, s_cc (shared)."""
    n = [ctypes.c_int32(0) for _ in range(6)]
    _check(lib().si_layer_split_info(layer, *[ctypes.byref(v) for v in n]))
    return dict(zip(("n_gg", "n_cg", "n_cc", "s_gg", "s_cg", "s_cc"), (v.value for v in n)))


def _routing(routing_out):
    if routing_out is None:
        return None
    r = si_routing_out_t(*[routing_out.get(k) for k in ("idx", "w", "count", "off", "perm", "inv")])
    return ctypes.byref(r)


def si_layer_forward(layer, x_ptr, logits_ptr, T, n_g, mode, y_ptr, routing_out=None, stream=0):
    """Pointers are device addresses (ints, e.g. tensor.data_ptr()); routing_out: dict name -> address."""
    _check(lib().si_layer_forward(layer, x_ptr, logits_ptr, T, n_g, mode, y_ptr, _routing(routing_out), stream))


def si_route(logits_ptr, T, E, k, routing_out, stream=0):
    _check(lib().si_route(logits_ptr, T, E, k, _routing(routing_out), stream))


def si_layer_set_profiling(layer, on):
    _check(lib().si_layer_set_profiling(layer, int(on)))


def si_layer_stats(layer) -> dict:
    st = si_stats_t()
    _check(lib().si_layer_stats(layer, ctypes.byref(st)))
    d = {name: getattr(st, name) for name, _ in si_stats_t._fields_}
    d["kernel_ms"] = list(st.kernel_ms)
    d["kernel_launches"] = list(st.kernel_launches)
    return d


def si_repack_chunks(w_gate, w_up, w_down, chunk0, n_chunks):
    """Host: chunk-major storage (NumPy uint16, n_chunks*3*64*M elements) of one expert's [H, M] weights."""
    import numpy as np
    H, M = w_gate.shape
    out = np.empty(n_chunks * 3 * 64 * M, np.uint16)
    _check(lib().si_repack_chunks(_host_ptr(w_gate), _host_ptr(w_up), _host_ptr(w_down), H, M, chunk0, n_chunks,
                                  _host_ptr(out)))
    return out


def si_cc_compute(x, idx, w, n_experts, routed, expert_stride, n_cc_chunks, shared=None, s_cc_chunks=0, threads=4):
    """Host: the CC workers' result ycc[T1, M] (float32) for NumPy inputs."""
    import numpy as np
    T1, M = x.shape
    k = idx.shape[1]
    idx = np.ascontiguousarray(idx, np.int32)
    w = np.ascontiguousarray(w, np.float32)
    ycc = np.empty((T1, M), np.float32)
    _check(lib().si_cc_compute(_host_ptr(x), ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(w.ctypes.data), T1, k, M,
                               n_experts, _host_ptr(routed), expert_stride, n_cc_chunks, _host_ptr(shared),
                               s_cc_chunks, threads, ctypes.c_void_p(ycc.ctypes.data)))
    return ycc


def si_layer_destroy(layer):
    lib().si_layer_destroy(layer)
