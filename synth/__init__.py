"""Seeded synthetic inputs for the partitioned FFN/MoE layer.

This module only *draws numbers and rounds them to their storage type*; it holds
none of the layer's arithmetic (no routing, no SwiGLU, no slicing).  Both the CPU
oracle's tests and the HIP path's tests/bench take their inputs from here so that
the two sides see byte-identical tensors.

The paper's own workloads are prompts from a public prompt dataset run through
trained Mixtral / LLaMA-2 / Qwen2 / PhiMoE checkpoints (Section V-A).  Neither is
available; for one FFN/MoE layer only the layer shape and the token count matter,
so the tensors below take those shapes and stand in for them.

Every tensor is keyed by ``(seed, tensor_id, chunk)`` so that any chunk can be
regenerated on its own, and large tensors are drawn chunk-wise on a thread pool.
"""
from __future__ import annotations

import dataclasses
import math
from concurrent.futures import ThreadPoolExecutor

import numpy as np

# tensor ids (the second word of the generator key)
TID_X, TID_WG, TID_WU, TID_WD, TID_GATE, TID_SG, TID_SU, TID_SD, TID_PERM = range(9)

_CHUNK = 1 << 22


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even) and return the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return rounded.astype(np.uint16)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float64."""
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.asarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal_chunk(seed: int, tid: int, chunk: int, n: int, std: float, out: np.ndarray) -> None:
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tid, chunk])))
    v = g.standard_normal(n, dtype=np.float32)
    if std != 1.0:
        v *= np.float32(std)
    out[:] = f32_to_bf16_bits(v)


def normal_bf16(seed: int, tid: int, shape, std: float, threads: int = 8) -> np.ndarray:
    """bf16 bit patterns (uint16) of N(0, std^2) samples, shape ``shape``."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    jobs = [(c, min(_CHUNK, n - c * _CHUNK)) for c in range((n + _CHUNK - 1) // _CHUNK)]
    if len(jobs) <= 1 or threads <= 1:
        for c, m in jobs:
            _normal_chunk(seed, tid, c, m, std, out[c * _CHUNK:c * _CHUNK + m])
    else:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(lambda cm: _normal_chunk(seed, tid, cm[0], cm[1], std,
                                                 out[cm[0] * _CHUNK:cm[0] * _CHUNK + cm[1]]), jobs))
    return out.reshape(shape)


@dataclasses.dataclass(frozen=True)
class LayerConfig:
    """Shape of one synthetic layer (model dim M, hidden dim H per expert, as in Section IV-A.2)."""
    name: str
    seed: int
    n_experts: int
    top_k: int
    d_model: int
    d_ff: int
    d_ff_shared: int
    t_decode: int
    t_prefill: int
    split: tuple          # (r_gg, r_cg, r_cc) the config is quoted on
    router: str           # "none" | "gate" | "zipf"
    w_std: float = 0.02

    @property
    def dense(self) -> bool:
        return self.router == "none"


CONFIGS = {
    "tiny_dense": LayerConfig("tiny_dense", 0, 1, 1, 256, 704, 0, 4, 32, (0.4, 0.3, 0.3), "none"),
    "mixtral_8x7b": LayerConfig("mixtral_8x7b", 1, 8, 2, 4096, 14336, 0, 1, 512, (0.5, 0.5, 0.0), "gate"),
    "llama2_70b": LayerConfig("llama2_70b", 2, 1, 1, 8192, 28672, 0, 1, 1024, (0.3, 0.5, 0.2), "none"),
    "qwen_moe": LayerConfig("qwen_moe", 3, 64, 8, 3584, 2560, 20480, 4, 2048, (1.0, 0.0, 0.0), "zipf"),
    "phimoe": LayerConfig("phimoe", 4, 16, 2, 4096, 6400, 0, 1, 4096, (1.0, 0.0, 0.0), "gate"),
    "mixtral_8x22b": LayerConfig("mixtral_8x22b", 5, 8, 2, 6144, 16384, 0, 1, 4096, (1.0, 0.0, 0.0), "gate"),
}

# split sweep used on the PhiMoE / Mixtral-8x22B shaped layers (r_gg, r_cg, r_cc)
SPLIT_SWEEP = [(1.0, 0.0, 0.0), (0.8, 0.2, 0.0), (0.6, 0.3, 0.1), (0.5, 0.5, 0.0),
               (0.4, 0.4, 0.2), (0.3, 0.5, 0.2), (0.2, 0.6, 0.2)]


def scaled(cfg: LayerConfig, **kw) -> LayerConfig:
    """A copy of ``cfg`` with some fields replaced (used for reduced-size test variants)."""
    return dataclasses.replace(cfg, **kw)


def make_weights(cfg: LayerConfig, threads: int = 8) -> dict:
    """Expert weights as bf16 bit patterns, all indexed [expert][d_ff index j][d_model index m]."""
    E, H, M = cfg.n_experts, cfg.d_ff, cfg.d_model
    w = {
        "w_gate": normal_bf16(cfg.seed, TID_WG, (E, H, M), cfg.w_std, threads),
        "w_up": normal_bf16(cfg.seed, TID_WU, (E, H, M), cfg.w_std, threads),
        "w_down": normal_bf16(cfg.seed, TID_WD, (E, H, M), cfg.w_std, threads),
    }
    if cfg.d_ff_shared:
        Hs = cfg.d_ff_shared
        w["s_gate"] = normal_bf16(cfg.seed, TID_SG, (Hs, M), cfg.w_std, threads)
        w["s_up"] = normal_bf16(cfg.seed, TID_SU, (Hs, M), cfg.w_std, threads)
        w["s_down"] = normal_bf16(cfg.seed, TID_SD, (Hs, M), cfg.w_std, threads)
    return w


def _codes_chunk(seed: int, tid: int, chunk: int, n_bytes: int, out: np.ndarray) -> None:
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tid, chunk, 4])))
    # codes of a bell-shaped weight distribution: round(2.4 z) + 8 clipped to 0..15, two per byte
    z = g.standard_normal(2 * n_bytes, dtype=np.float32)
    c = np.clip(np.rint(z * np.float32(2.4)) + 8, 0, 15).astype(np.uint8)
    out[:] = c[0::2] | (c[1::2] << np.uint8(4))


def codes_u4(seed: int, tid: int, shape, threads: int = 8) -> np.ndarray:
    """Packed 4-bit codes (uint8, two per byte, low nibble first) of the given shape (last dim = bytes)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint8)
    jobs = [(c, min(_CHUNK, n - c * _CHUNK)) for c in range((n + _CHUNK - 1) // _CHUNK)]
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(lambda cm: _codes_chunk(seed, tid, cm[0], cm[1], out[cm[0] * _CHUNK:cm[0] * _CHUNK + cm[1]]), jobs))
    return out.reshape(shape)


def scales_bf16(seed: int, tid: int, shape, mean: float) -> np.ndarray:
    """Positive group scales around ``mean`` (uniform in [0.7, 1.3] x mean) as bf16 bit patterns."""
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([seed, tid, 0, 16])))
    return f32_to_bf16_bits((g.uniform(0.7, 1.3, size=shape) * mean).astype(np.float32))


def make_weights_q4(cfg: LayerConfig, threads: int = 8) -> dict:
    """Expert weights in 4-bit storage: codes q_* [E][H][M/2] (uint8, element m in byte m/2, low nibble for even
    m), scales z_gate / z_up [E][H][M/64] and z_down [E][H/64][M] (bf16 bit patterns).  The standard deviation
    of the weights the codes stand for is about cfg.w_std (scale mean = w_std / 2.4)."""
    E, H, M = cfg.n_experts, cfg.d_ff, cfg.d_model
    zm = cfg.w_std / 2.4
    w = {
        "q_gate": codes_u4(cfg.seed, TID_WG, (E, H, M // 2), threads),
        "q_up": codes_u4(cfg.seed, TID_WU, (E, H, M // 2), threads),
        "q_down": codes_u4(cfg.seed, TID_WD, (E, H, M // 2), threads),
        "z_gate": scales_bf16(cfg.seed, TID_WG, (E, H, M // 64), zm),
        "z_up": scales_bf16(cfg.seed, TID_WU, (E, H, M // 64), zm),
        "z_down": scales_bf16(cfg.seed, TID_WD, (E, H // 64, M), zm),
    }
    if cfg.d_ff_shared:
        Hs = cfg.d_ff_shared
        w["sq_gate"] = codes_u4(cfg.seed, TID_SG, (Hs, M // 2), threads)
        w["sq_up"] = codes_u4(cfg.seed, TID_SU, (Hs, M // 2), threads)
        w["sq_down"] = codes_u4(cfg.seed, TID_SD, (Hs, M // 2), threads)
        w["sz_gate"] = scales_bf16(cfg.seed, TID_SG, (Hs, M // 64), zm)
        w["sz_up"] = scales_bf16(cfg.seed, TID_SU, (Hs, M // 64), zm)
        w["sz_down"] = scales_bf16(cfg.seed, TID_SD, (Hs // 64, M), zm)
    return w


def make_tokens(cfg: LayerConfig, T: int, stream: int = 0) -> np.ndarray:
    """Hidden states x[T, M] ~ N(0,1) as bf16 bit patterns.  ``stream`` selects an independent batch."""
    return normal_bf16(cfg.seed + 1000 * stream, TID_X, (T, cfg.d_model), 1.0, threads=1)


def make_router_logits(cfg: LayerConfig, x_bits: np.ndarray):
    """Router logits fp32 [T, E] for the given tokens, or None for a dense layer.

    "gate": logits = x . G with G[M, E] ~ N(0, 1/M) so that logits ~ N(0, 1).
    "zipf": the same plus a per-expert bias b[pi(r)] = -1.1 ln r, r = 1..E, pi a seeded
            permutation, i.e. a prior popularity proportional to r^-1.1.
    The product is formed once in float64 on the host and rounded to fp32; the result is an
    *input* handed to both the oracle and the HIP path.
    """
    if cfg.router == "none":
        return None
    M, E = cfg.d_model, cfg.n_experts
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, TID_GATE])))
    G = g.standard_normal((M, E)) / math.sqrt(M)
    logits = bf16_bits_to_f64(x_bits) @ G
    if cfg.router == "zipf":
        gp = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, TID_PERM])))
        pi = gp.permutation(E)
        b = np.empty(E)
        b[pi] = -1.1 * np.log(np.arange(1, E + 1, dtype=np.float64))
        logits = logits + b[None, :]
    return np.ascontiguousarray(logits.astype(np.float32))
