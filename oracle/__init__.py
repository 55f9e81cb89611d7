"""ctypes binding of the CPU oracle (``scheinfer_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, by ``__graft_entry__.smoke()`` and by the
``cpu_baseline`` leg of ``bench.py``.  The GPU library never imports or calls anything here, and
this module imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "scheinfer_oracle.c")
_LIB = os.path.join(_HERE, "libscheinfer_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP for the trivial parallel-for)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        c_i, c_d, c_p = ctypes.c_int, ctypes.c_double, ctypes.c_void_p
        L.so_silu.restype = c_d
        L.so_silu.argtypes = [c_d]
        L.so_set_threads.argtypes = [c_i]
        L.so_get_threads.restype = c_i
        L.so_split_counts.restype = c_i
        L.so_split_counts.argtypes = [c_i, c_i, c_d, c_d, c_p, c_p, c_p]
        L.so_route.restype = c_i
        L.so_route.argtypes = [c_p, c_i, c_i, c_i, c_p, c_p, c_p, c_p, c_p, c_p]
        L.so_layer_forward.restype = c_i
        L.so_layer_forward.argtypes = [c_p, c_i, c_i, c_i, c_i, c_i, c_p, c_p, c_p, c_p, c_i, c_p, c_p, c_p,
                                       c_i, c_i, c_i, c_i, c_i, c_p, c_i, c_p]
        L.so_layer_forward_q4.restype = c_i
        L.so_layer_forward_q4.argtypes = [c_p, c_i, c_i, c_i, c_i, c_i, c_p] + [c_p] * 6 + [c_i] + [c_p] * 6 + \
                                         [c_i, c_i, c_i, c_i, c_i, c_p, c_i, c_p]
        L.so_q4_value.restype = c_d
        L.so_q4_value.argtypes = [c_p, c_p, c_i, c_i, c_i, c_i]
        _lib = L
    return _lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def set_threads(n: int) -> None:
    _load().so_set_threads(int(n))


def get_threads() -> int:
    return int(_load().so_get_threads())


def silu(z: float) -> float:
    return float(_load().so_silu(float(z)))


def split_counts(H: int, granule: int, r_gg: float, r_cg: float):
    """(n_cc, n_cg, n_gg) hidden-column counts for the given rates; rates are taken as float32."""
    n = [ctypes.c_int(0) for _ in range(3)]
    rc = _load().so_split_counts(int(H), int(granule), float(np.float32(r_gg)), float(np.float32(r_cg)),
                                 ctypes.byref(n[0]), ctypes.byref(n[1]), ctypes.byref(n[2]))
    if rc:
        raise ValueError("so_split_counts: invalid arguments")
    return n[0].value, n[1].value, n[2].value


def route(logits: np.ndarray, k: int) -> dict:
    logits = np.ascontiguousarray(logits, dtype=np.float32)
    T, E = logits.shape
    n = max(T * k, 1)
    out = {"idx": np.zeros(n, np.int32), "w": np.zeros(n, np.float64), "count": np.zeros(E, np.int32),
           "off": np.zeros(E + 1, np.int32), "perm": np.zeros(n, np.int32), "inv": np.zeros(n, np.int32)}
    rc = _load().so_route(_ptr(logits), T, E, int(k), _ptr(out["idx"]), _ptr(out["w"]), _ptr(out["count"]),
                          _ptr(out["off"]), _ptr(out["perm"]), _ptr(out["inv"]))
    if rc:
        raise ValueError("so_route failed with code %d" % rc)
    for key in ("idx", "w"):
        out[key] = out[key][:T * k].reshape(T, k)
    for key in ("perm", "inv"):
        out[key] = out[key][:T * k]
    return out


def layer_forward(x, w_gate, w_up, w_down, logits=None, top_k=1, shared=None, counts=(0, 0),
                  shared_counts=(0, 0), n_g=0, sel=None) -> np.ndarray:
    """y[T or len(sel), M] in float64.

    x: uint16 [T, M]; w_*: uint16 [E, H, M]; logits: float32 [T, E] or None (E must be 1);
    shared: None or (s_gate, s_up, s_down) uint16 [Hs, M]; counts = (n_cc, n_cg) hidden columns of
    the CC and CG parts (0, 0 = unsliced); shared_counts likewise for the shared expert.
    """
    x = np.ascontiguousarray(x, dtype=np.uint16)
    T, M = x.shape
    wg = np.ascontiguousarray(w_gate, dtype=np.uint16)
    wu = np.ascontiguousarray(w_up, dtype=np.uint16)
    wd = np.ascontiguousarray(w_down, dtype=np.uint16)
    E, H, M2 = wg.shape
    assert M2 == M and wu.shape == wg.shape and wd.shape == wg.shape
    lg = None
    if logits is not None:
        lg = np.ascontiguousarray(logits, dtype=np.float32)
        assert lg.shape == (T, E)
    Hs, sg, su, sd = 0, None, None, None
    if shared is not None:
        sg, su, sd = (np.ascontiguousarray(a, dtype=np.uint16) for a in shared)
        Hs = sg.shape[0]
        assert sg.shape == (Hs, M) and su.shape == sg.shape and sd.shape == sg.shape
    sel_a = None if sel is None else np.ascontiguousarray(sel, dtype=np.int32)
    n_out = T if sel_a is None else len(sel_a)
    y = np.zeros((n_out, M), np.float64)
    rc = _load().so_layer_forward(_ptr(x), T, M, H, E, int(top_k), _ptr(lg), _ptr(wg), _ptr(wu), _ptr(wd), Hs,
                                  _ptr(sg), _ptr(su), _ptr(sd), int(counts[0]), int(counts[1]),
                                  int(shared_counts[0]), int(shared_counts[1]), int(n_g), _ptr(sel_a),
                                  0 if sel_a is None else len(sel_a), _ptr(y))
    if rc:
        raise ValueError("so_layer_forward failed with code %d" % rc)
    return y


def layer_forward_q4(x, wq: dict, logits=None, top_k=1, counts=(0, 0), shared_counts=(0, 0), n_g=0, sel=None) -> np.ndarray:
    """As layer_forward, for 4-bit weights: wq holds q_gate, q_up, q_down (uint8 [E][H][M/2]), z_gate, z_up
    (uint16 [E][H][M/64]), z_down (uint16 [E][H/64][M]) and optionally the shared expert's sq_* / sz_*."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    T, M = x.shape
    q = [np.ascontiguousarray(wq[k], dtype=np.uint8) for k in ("q_gate", "q_up", "q_down")]
    z = [np.ascontiguousarray(wq[k], dtype=np.uint16) for k in ("z_gate", "z_up", "z_down")]
    E, H, M2 = q[0].shape
    assert M2 * 2 == M and z[0].shape == (E, H, M // 64) and z[2].shape == (E, H // 64, M)
    lg = None
    if logits is not None:
        lg = np.ascontiguousarray(logits, dtype=np.float32)
        assert lg.shape == (T, E)
    Hs, sq, sz = 0, [None] * 3, [None] * 3
    if "sq_gate" in wq:
        sq = [np.ascontiguousarray(wq[k], dtype=np.uint8) for k in ("sq_gate", "sq_up", "sq_down")]
        sz = [np.ascontiguousarray(wq[k], dtype=np.uint16) for k in ("sz_gate", "sz_up", "sz_down")]
        Hs = sq[0].shape[0]
    sel_a = None if sel is None else np.ascontiguousarray(sel, dtype=np.int32)
    n_out = T if sel_a is None else len(sel_a)
    y = np.zeros((n_out, M), np.float64)
    rc = _load().so_layer_forward_q4(_ptr(x), T, M, H, E, int(top_k), _ptr(lg), *[_ptr(a) for a in q + z], Hs,
                                     *[_ptr(a) for a in sq + sz], int(counts[0]), int(counts[1]),
                                     int(shared_counts[0]), int(shared_counts[1]), int(n_g), _ptr(sel_a),
                                     0 if sel_a is None else len(sel_a), _ptr(y))
    if rc:
        raise ValueError("so_layer_forward_q4 failed with code %d" % rc)
    return y


def q4_value(q, z, M, which, j, m) -> float:
    """Dequantised element (which: 0 gate, 1 up, 2 down) of one expert's code / scale arrays."""
    q = np.ascontiguousarray(q, np.uint8)
    z = np.ascontiguousarray(z, np.uint16)
    return float(_load().so_q4_value(_ptr(q), _ptr(z), int(M), int(which), int(j), int(m)))


def round_to_bf16(v: np.ndarray) -> np.ndarray:
    """Round float64 values to the nearest bfloat16 (8 significant bits, ties to even) and return the uint16
    bit patterns.  Normal range only (no subnormals, no overflow): the hidden states of a layer stack."""
    v = np.asarray(v, np.float64)
    m, e = np.frexp(v)                    # v = m * 2^e, 0.5 <= |m| < 1
    q = np.rint(m * 256.0)                # 8 significant bits; rint rounds halves to even
    r = np.ldexp(q / 256.0, e).astype(np.float32)   # exact: 8 bits fit float32
    return (r.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f64(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def stack_forward(x, layers) -> np.ndarray:
    """Layers run back to back with the residual connection around each:
    x_{l+1} = bf16(x_l + Layer_l(x_l)); returns h = x_{n-1} + Layer_{n-1}(x_{n-1}) in float64, not rounded.
    layers: list of dicts with the keyword arguments of layer_forward (w_gate, w_up, w_down, logits, top_k,
    shared)."""
    x = np.ascontiguousarray(x, dtype=np.uint16)
    h = None
    for i, kw in enumerate(layers):
        y = layer_forward(x, **kw)
        h = bf16_to_f64(x) + y
        if i + 1 < len(layers):
            x = round_to_bf16(h)
    return h
