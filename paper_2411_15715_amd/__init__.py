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
SI_DECODE_AUTO_T, SI_DECODE_AUTO_ROWS, SI_DECODE_MAX_T = 8, 4, 16
SI_ROUTE_NOALLOC_MAX_PAIRS = 131072

EXPORTS = ["si_layer_create", "si_layer_split_info", "si_split_counts", "si_layer_forward", "si_route", "si_route_noalloc",
           "si_layer_stats", "si_layer_set_profiling", "si_repack_chunks", "si_cc_compute", "si_layer_destroy", "si_last_error", "si_version",
           "si_stack_create", "si_stack_forward", "si_stack_destroy",
           "si_layer_create_q4", "si_repack_chunks_q4", "si_cc_compute_q4", "si_layer_create_placed", "si_place_experts", "si_layer_resplit",
           # scheinfer_solver.h
           "si_fit_linear", "si_model_times", "si_simulate", "si_solve_split", "si_model_times_ng", "si_solve_ng",
           "si_assign_gpu_memory", "si_profile", "si_measure_peaks"]
SI_MAX_EDGE_POINTS, SI_PROFILE_MAX_SIZES = 24, 12


class si_layer_desc_t(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("n_experts", ctypes.c_int32),
                ("top_k", ctypes.c_int32), ("d_ff_shared", ctypes.c_int32), ("r_gg", ctypes.c_float),
                ("r_cg", ctypes.c_float), ("r_cc", ctypes.c_float), ("granule", ctypes.c_int32),
                ("max_tokens", ctypes.c_int32), ("cc_threads", ctypes.c_int32), ("device", ctypes.c_int32),
                ("stage_mib", ctypes.c_int32), ("n_stage", ctypes.c_int32), ("deq_mib", ctypes.c_int32)]


class si_q4_weights_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in ("q_gate", "q_up", "q_down", "z_gate", "z_up", "z_down")]


class si_routing_out_t(ctypes.Structure):
    _fields_ = [("idx", ctypes.c_void_p), ("w", ctypes.c_void_p), ("count", ctypes.c_void_p),
                ("off", ctypes.c_void_p), ("perm", ctypes.c_void_p), ("inv", ctypes.c_void_p)]


class si_stats_t(ctypes.Structure):
    _fields_ = [("total_ms", ctypes.c_float), ("copy_ms", ctypes.c_float), ("gpu_ms", ctypes.c_float),
                ("cc_ms", ctypes.c_float), ("route_ms", ctypes.c_float), ("bytes_streamed", ctypes.c_double),
                ("bytes_gg", ctypes.c_double), ("bytes_cc", ctypes.c_double), ("overlap", ctypes.c_float),
                ("n_copies", ctypes.c_int32), ("n_touched", ctypes.c_int32), ("path", ctypes.c_int32),
                ("kernel_ms", ctypes.c_float * 8), ("kernel_launches", ctypes.c_int32 * 8),
                ("staged_ms", ctypes.c_float), ("handoff_ms", ctypes.c_float), ("enqueue_ms", ctypes.c_float),
                ("gg_in_copy", ctypes.c_float)]


class si_perf_model_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("alpha_g", "beta_g", "alpha_c", "beta_c", "alpha_c2g", "beta_c2g", "t_launch")]


class si_problem_t(ctypes.Structure):
    _fields_ = [("n_gemm", ctypes.c_double), ("n_w", ctypes.c_double), ("n_l", ctypes.c_int32)]


class si_task_times_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in ("t_g", "t_c", "t_c2g", "t_l")]


class si_split_solution_t(ctypes.Structure):
    _fields_ = [("r_cg", ctypes.c_double), ("r_cc", ctypes.c_double), ("t_fin", ctypes.c_double),
                ("which_case", ctypes.c_int32), ("n_points", ctypes.c_int32),
                ("x", ctypes.c_double * SI_MAX_EDGE_POINTS), ("y", ctypes.c_double * SI_MAX_EDGE_POINTS)]


class si_ng_solution_t(ctypes.Structure):
    _fields_ = [("n_g", ctypes.c_int32), ("t_fin", ctypes.c_double), ("which_case", ctypes.c_int32),
                ("n_points", ctypes.c_int32), ("x", ctypes.c_double * SI_MAX_EDGE_POINTS),
                ("y", ctypes.c_double * SI_MAX_EDGE_POINTS)]


class si_peaks_t(ctypes.Structure):
    _fields_ = [("hbm_read_gbs", ctypes.c_double), ("hbm_copy_gbs", ctypes.c_double), ("mfma_bf16_tflops", ctypes.c_double),
                ("h2d_gbs", ctypes.c_double), ("n_cu", ctypes.c_int32), ("mfma_bf16_random_tflops", ctypes.c_double)]


class si_profile_desc_t(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("tokens", ctypes.c_int32),
                ("mode", ctypes.c_int32), ("n_sizes", ctypes.c_int32), ("reps", ctypes.c_int32),
                ("cc_threads", ctypes.c_int32), ("device", ctypes.c_int32), ("copy_max_mib", ctypes.c_int32),
                ("seed", ctypes.c_uint32), ("q4", ctypes.c_int32)]


class si_profile_result_t(ctypes.Structure):
    _fields_ = [("model", si_perf_model_t), ("r2_g", ctypes.c_double), ("r2_c", ctypes.c_double),
                ("r2_c2g", ctypes.c_double), ("sigma_launch", ctypes.c_double), ("n_points", ctypes.c_int32)] + \
               [(n, ctypes.c_double * SI_PROFILE_MAX_SIZES) for n in ("n_gemm", "t_g", "t_c", "bytes", "t_c2g")]


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
        L.si_route_noalloc.restype = ctypes.c_int
        L.si_route_noalloc.argtypes = [vp, i32, i32, i32, ctypes.POINTER(si_routing_out_t), vp]
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
        pq = ctypes.POINTER(si_q4_weights_t)
        L.si_layer_create_q4.restype = ctypes.c_int
        L.si_layer_create_q4.argtypes = [ctypes.POINTER(si_layer_desc_t), pq, pq, vp, ctypes.POINTER(vp)]
        L.si_layer_create_placed.restype = ctypes.c_int
        L.si_layer_create_placed.argtypes = [ctypes.POINTER(si_layer_desc_t), vp, vp, vp, vp, vp, vp, vp, ctypes.POINTER(vp)]
        L.si_layer_resplit.restype = ctypes.c_int
        L.si_layer_resplit.argtypes = [vp, f32, f32, f32]
        L.si_place_experts.restype = ctypes.c_int
        L.si_place_experts.argtypes = [vp, i32, i32, ctypes.c_double, vp]
        L.si_repack_chunks_q4.restype = ctypes.c_int
        L.si_repack_chunks_q4.argtypes = [pq, i32, i32, i32, i32, vp]
        L.si_cc_compute_q4.restype = ctypes.c_int
        L.si_cc_compute_q4.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, ctypes.c_uint64, i32, vp, i32, i32, vp]
        L.si_stack_create.restype = ctypes.c_int
        L.si_stack_create.argtypes = [ctypes.POINTER(vp), i32, ctypes.POINTER(vp)]
        L.si_stack_forward.restype = ctypes.c_int
        L.si_stack_forward.argtypes = [vp, vp, ctypes.POINTER(vp), i32, i32, i32, vp, i32, vp]
        L.si_stack_destroy.restype = None
        L.si_stack_destroy.argtypes = [vp]
        L.si_version.restype = ctypes.c_char_p
        f64, pd = ctypes.c_double, ctypes.POINTER(ctypes.c_double)
        pm, pp, pt = ctypes.POINTER(si_perf_model_t), ctypes.POINTER(si_problem_t), ctypes.POINTER(si_task_times_t)
        L.si_fit_linear.restype = ctypes.c_int
        L.si_fit_linear.argtypes = [vp, vp, i32, i32, pd, pd, pd]
        L.si_model_times.restype = ctypes.c_int
        L.si_model_times.argtypes = [pm, pp, f64, f64, pt]
        L.si_simulate.restype = ctypes.c_int
        L.si_simulate.argtypes = [pt, i32, pd, pd, pd]
        L.si_solve_split.restype = ctypes.c_int
        L.si_solve_split.argtypes = [pm, pp, f64, f64, ctypes.POINTER(si_split_solution_t)]
        L.si_model_times_ng.restype = ctypes.c_int
        L.si_model_times_ng.argtypes = [pm, i32, i32, i32, f64, f64, f64, i32, pt]
        L.si_solve_ng.restype = ctypes.c_int
        L.si_solve_ng.argtypes = [pm, i32, i32, i32, f64, i32, f64, f64, ctypes.POINTER(si_ng_solution_t)]
        L.si_assign_gpu_memory.restype = ctypes.c_int
        L.si_assign_gpu_memory.argtypes = [vp, vp, i32, i32, f64, vp]
        L.si_measure_peaks.restype = ctypes.c_int
        L.si_measure_peaks.argtypes = [i32, ctypes.POINTER(si_peaks_t)]
        L.si_profile.restype = ctypes.c_int
        L.si_profile.argtypes = [ctypes.POINTER(si_profile_desc_t), ctypes.POINTER(si_profile_result_t)]
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


def _placement_ptr(placement, n_experts):
    import numpy as np
    if placement is None:
        return None, None
    a = np.ascontiguousarray(placement, np.uint8)
    if a.shape != (n_experts,):
        raise ValueError("placement must have one entry per expert")
    return a, ctypes.c_void_p(a.ctypes.data)


def si_layer_create(d_model, d_ff, n_experts, top_k, w_gate, w_up, w_down, r_gg, r_cg, r_cc, max_tokens,
                    d_ff_shared=0, shared=None, granule=0, cc_threads=0, device=0, stage_mib=0, n_stage=0, placement=None):
    """Returns the opaque layer handle (an int).  Weights are host NumPy uint16 arrays.  placement: None (slice by
    the rates) or one of 0 (GG) / 1 (CG) / 2 (CC) per expert (whole-expert placement)."""
    desc = si_layer_desc_t(d_model, d_ff, n_experts, top_k, d_ff_shared, r_gg, r_cg, r_cc, granule, max_tokens,
                           cc_threads, device, stage_mib, n_stage)
    sg, su, sd = shared if shared is not None else (None, None, None)
    out = ctypes.c_void_p(None)
    keep, pp = _placement_ptr(placement, n_experts)
    if pp is None:
        _check(lib().si_layer_create(ctypes.byref(desc), _host_ptr(w_gate), _host_ptr(w_up), _host_ptr(w_down),
                                     _host_ptr(sg), _host_ptr(su), _host_ptr(sd), ctypes.byref(out)))
    else:
        _check(lib().si_layer_create_placed(ctypes.byref(desc), _host_ptr(w_gate), _host_ptr(w_up), _host_ptr(w_down),
                                            _host_ptr(sg), _host_ptr(su), _host_ptr(sd), pp, ctypes.byref(out)))
    return out.value


def si_place_experts(freq, n_gg, cg_share):
    """Placement (list of 0 / 1 / 2 per expert) from expert frequencies."""
    import numpy as np
    f = np.ascontiguousarray(freq, np.float64)
    out = np.zeros(f.size, np.uint8)
    _check(lib().si_place_experts(ctypes.c_void_p(f.ctypes.data), f.size, int(n_gg), float(cg_share), ctypes.c_void_p(out.ctypes.data)))
    return out.tolist()


def _q4_struct(w, prefix=""):
    """si_q4_weights_t over the NumPy arrays w[prefix + 'q_gate'] ...; returns (struct, keep-alive list)."""
    import numpy as np
    keep = []
    vals = []
    for name, dt in (("q_gate", np.uint8), ("q_up", np.uint8), ("q_down", np.uint8), ("z_gate", np.uint16), ("z_up", np.uint16), ("z_down", np.uint16)):
        a = w[prefix + name]
        if a.dtype != dt or not a.flags["C_CONTIGUOUS"]:
            raise ValueError(prefix + name + " must be a C-contiguous %s array" % dt.__name__)
        keep.append(a)
        vals.append(a.ctypes.data)
    return si_q4_weights_t(*vals), keep


def si_layer_create_q4(d_model, d_ff, n_experts, top_k, wq, r_gg, r_cg, r_cc, max_tokens, d_ff_shared=0, granule=0,
                       cc_threads=0, device=0, stage_mib=0, n_stage=0, placement=None, deq_mib=0):
    """Layer from 4-bit weights: wq holds q_gate, q_up, q_down, z_gate, z_up, z_down (and sq_* / sz_* of the shared
    expert when d_ff_shared > 0) as NumPy arrays.  Returns the opaque layer handle."""
    desc = si_layer_desc_t(d_model, d_ff, n_experts, top_k, d_ff_shared, r_gg, r_cg, r_cc, granule, max_tokens,
                           cc_threads, device, stage_mib, n_stage, deq_mib)
    routed, keep = _q4_struct(wq)
    shared = None
    if d_ff_shared:
        sh, keep2 = _q4_struct(wq, "s")
        shared = ctypes.byref(sh)
    out = ctypes.c_void_p(None)
    keep3, pp = _placement_ptr(placement, n_experts)
    _check(lib().si_layer_create_q4(ctypes.byref(desc), ctypes.byref(routed), shared, pp, ctypes.byref(out)))
    return out.value


def si_layer_resplit(layer, r_gg, r_cg, r_cc):
    """Change the slicing rates of an existing layer (moves chunks between GPU and pinned host memory)."""
    _check(lib().si_layer_resplit(layer, r_gg, r_cg, r_cc))


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


def si_route_noalloc(logits_ptr, T, E, k, routing_out, stream=0):
    """si_route without any device allocation (fixed scratch; T * k <= SI_ROUTE_NOALLOC_MAX_PAIRS)."""
    _check(lib().si_route_noalloc(logits_ptr, T, E, k, _routing(routing_out), stream))


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


def si_repack_chunks_q4(wq, chunk0, n_chunks, prefix=""):
    """Host: library storage (NumPy uint16, n_chunks*51*M units) of one expert's 4-bit arrays wq[prefix + 'q_gate'] ..."""
    import numpy as np
    H, M2 = wq[prefix + "q_gate"].shape
    st, keep = _q4_struct(wq, prefix)
    out = np.empty(n_chunks * 51 * M2 * 2, np.uint16)
    _check(lib().si_repack_chunks_q4(ctypes.byref(st), H, M2 * 2, chunk0, n_chunks, _host_ptr(out)))
    return out


def si_cc_compute(x, idx, w, n_experts, routed, expert_stride, n_cc_chunks, shared=None, s_cc_chunks=0, threads=4, q4=False):
    """Host: the CC workers' result ycc[T1, M] (float32) for NumPy inputs."""
    import numpy as np
    T1, M = x.shape
    k = idx.shape[1]
    idx = np.ascontiguousarray(idx, np.int32)
    w = np.ascontiguousarray(w, np.float32)
    ycc = np.empty((T1, M), np.float32)
    fn = lib().si_cc_compute_q4 if q4 else lib().si_cc_compute
    _check(fn(_host_ptr(x), ctypes.c_void_p(idx.ctypes.data), ctypes.c_void_p(w.ctypes.data), T1, k, M,
              n_experts, _host_ptr(routed), expert_stride, n_cc_chunks, _host_ptr(shared),
              s_cc_chunks, threads, ctypes.c_void_p(ycc.ctypes.data)))
    return ycc


def si_layer_destroy(layer):
    lib().si_layer_destroy(layer)


def si_stack_create(layers):
    """layers: list of layer handles; returns the opaque stack handle."""
    arr = (ctypes.c_void_p * len(layers))(*layers)
    out = ctypes.c_void_p(None)
    _check(lib().si_stack_create(arr, len(layers), ctypes.byref(out)))
    return out.value


def si_stack_forward(stack, x_ptr, logits_ptrs, T, n_g, mode, h_out_ptr, prefetch=1, stream=0):
    """logits_ptrs: None, or one device address (or None) per layer.  prefetch: bit 0 next layer, bit 1 wrap-around."""
    arr = None
    if logits_ptrs is not None:
        arr = (ctypes.c_void_p * len(logits_ptrs))(*logits_ptrs)
    _check(lib().si_stack_forward(stack, x_ptr, arr, T, n_g, mode, h_out_ptr, int(prefetch), stream))


def si_stack_destroy(stack):
    lib().si_stack_destroy(stack)


# ---------------------------------------------------------------- scheinfer_solver.h
_MODEL_KEYS = ("alpha_g", "beta_g", "alpha_c", "beta_c", "alpha_c2g", "beta_c2g", "t_launch")


def _model(m):
    return m if isinstance(m, si_perf_model_t) else si_perf_model_t(*[float(m[k]) for k in _MODEL_KEYS])


def _times(t):
    return {k: getattr(t, k) for k in ("t_g", "t_c", "t_c2g", "t_l")}


def si_fit_linear(n, t, nonneg=False):
    """(alpha, beta, r2) of t = alpha + n*beta."""
    import numpy as np
    n = np.ascontiguousarray(n, np.float64)
    t = np.ascontiguousarray(t, np.float64)
    if n.shape != t.shape or n.ndim != 1:
        raise ValueError("n and t must be 1-d arrays of equal length")
    a, b, r2 = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib().si_fit_linear(ctypes.c_void_p(n.ctypes.data), ctypes.c_void_p(t.ctypes.data), n.size, int(nonneg),
                               ctypes.byref(a), ctypes.byref(b), ctypes.byref(r2)))
    return a.value, b.value, r2.value


def si_model_times(model, n_gemm, n_w, n_l, r_gg, r_cg) -> dict:
    out = si_task_times_t()
    _check(lib().si_model_times(ctypes.byref(_model(model)), ctypes.byref(si_problem_t(n_gemm, n_w, n_l)), r_gg, r_cg,
                                ctypes.byref(out)))
    return _times(out)


def si_simulate(times: dict, n_l) -> dict:
    t = si_task_times_t(times["t_g"], times["t_c"], times["t_c2g"], times["t_l"])
    f, g, c = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    _check(lib().si_simulate(ctypes.byref(t), n_l, ctypes.byref(f), ctypes.byref(g), ctypes.byref(c)))
    return {"t_fin": f.value, "tau_g": g.value, "tau_c": c.value}


def si_solve_split(model, n_gemm, n_w, n_l, r_gg, r_step=0.0) -> dict:
    out = si_split_solution_t()
    _check(lib().si_solve_split(ctypes.byref(_model(model)), ctypes.byref(si_problem_t(n_gemm, n_w, n_l)), r_gg, r_step,
                                ctypes.byref(out)))
    return {"r_cg": out.r_cg, "r_cc": out.r_cc, "t_fin": out.t_fin, "case": out.which_case,
            "X": list(out.x[:out.n_points]), "Y": list(out.y[:out.n_points])}


def si_model_times_ng(model, T, d_model, d_ff, n_w, r_gg, r_cg, n_g) -> dict:
    out = si_task_times_t()
    _check(lib().si_model_times_ng(ctypes.byref(_model(model)), T, d_model, d_ff, n_w, r_gg, r_cg, n_g, ctypes.byref(out)))
    return _times(out)


def si_solve_ng(model, T, d_model, d_ff, n_w, n_l, r_gg, r_cg) -> dict:
    out = si_ng_solution_t()
    _check(lib().si_solve_ng(ctypes.byref(_model(model)), T, d_model, d_ff, n_w, n_l, r_gg, r_cg, ctypes.byref(out)))
    return {"n_g": out.n_g, "t_fin": out.t_fin, "case": out.which_case,
            "X": [int(v) for v in out.x[:out.n_points]], "Y": list(out.y[:out.n_points])}


def si_assign_gpu_memory(t_star, n_m, budget):
    """t_star: [n_layers][n_grid+1]; returns the chosen grid index per layer."""
    import numpy as np
    t = np.ascontiguousarray(t_star, np.float64)
    w = np.ascontiguousarray(n_m, np.float64)
    if t.ndim != 2 or w.shape != (t.shape[0],):
        raise ValueError("t_star must be [n_layers][n_grid+1] and n_m [n_layers]")
    pick = np.zeros(t.shape[0], np.int32)
    _check(lib().si_assign_gpu_memory(ctypes.c_void_p(t.ctypes.data), ctypes.c_void_p(w.ctypes.data), t.shape[0],
                                      t.shape[1] - 1, float(budget), ctypes.c_void_p(pick.ctypes.data)))
    return pick.tolist()


def si_profile(d_model, d_ff, tokens, mode=SI_AUTO, n_sizes=0, reps=0, cc_threads=0, device=0, copy_max_mib=0, seed=1, q4=False) -> dict:
    """Measure this machine and fit Eq. 3; returns the model, the r^2 values and the raw points."""
    desc = si_profile_desc_t(d_model, d_ff, tokens, mode, n_sizes, reps, cc_threads, device, copy_max_mib, seed, int(bool(q4)))
    out = si_profile_result_t()
    _check(lib().si_profile(ctypes.byref(desc), ctypes.byref(out)))
    k = out.n_points
    return {"model": {n: getattr(out.model, n) for n in _MODEL_KEYS}, "r2_g": out.r2_g, "r2_c": out.r2_c,
            "r2_c2g": out.r2_c2g, "sigma_launch": out.sigma_launch, "n_gemm": list(out.n_gemm[:k]),
            "t_g": list(out.t_g[:k]), "t_c": list(out.t_c[:k]), "bytes": list(out.bytes[:k]), "t_c2g": list(out.t_c2g[:k])}


def si_measure_peaks(device=0) -> dict:
    """Measured HBM read / copy GB/s, bf16 MFMA TFLOP/s and host-to-device GB/s of this machine."""
    out = si_peaks_t()
    _check(lib().si_measure_peaks(device, ctypes.byref(out)))
    return {n: getattr(out, n) for n, _ in si_peaks_t._fields_}
