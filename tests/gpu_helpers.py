"""Helpers for the GPU tests: device tensors come from PyTorch, every computation from the library."""
import numpy as np
import torch

import paper_2411_15715_amd as si

TOL = 2e-2  # max-abs error <= TOL * RMS(oracle output)


class GpuLayer:
    def __init__(self, cfg, w, split, max_tokens, **kw):
        shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
        self.cfg = cfg
        self.h = si.si_layer_create(cfg.d_model, cfg.d_ff, cfg.n_experts, cfg.top_k, w["w_gate"], w["w_up"], w["w_down"],
                                    split[0], split[1], split[2], max_tokens, d_ff_shared=cfg.d_ff_shared, shared=shared, **kw)
        self.info = si.si_layer_split_info(self.h)

    def forward(self, x_bits, logits, n_g=0, mode=si.SI_AUTO, routing=False):
        cfg = self.cfg
        T = x_bits.shape[0]
        dev = torch.device("cuda:0")
        x = torch.from_numpy(np.ascontiguousarray(x_bits).view(np.int16)).to(dev)
        lg = torch.from_numpy(logits).to(dev) if logits is not None else None
        y = torch.full((max(T, 1), cfg.d_model), float("nan"), dtype=torch.float32, device=dev)
        ro = None
        bufs = {}
        if routing:
            n = max(T * cfg.top_k, 1)
            bufs = {"idx": torch.full((n,), -1, dtype=torch.int32, device=dev),
                    "w": torch.zeros(n, dtype=torch.float32, device=dev),
                    "count": torch.full((cfg.n_experts,), -1, dtype=torch.int32, device=dev),
                    "off": torch.full((cfg.n_experts + 1,), -1, dtype=torch.int32, device=dev),
                    "perm": torch.full((n,), -1, dtype=torch.int32, device=dev),
                    "inv": torch.full((n,), -1, dtype=torch.int32, device=dev)}
            ro = {k: v.data_ptr() for k, v in bufs.items()}
        stream = torch.cuda.current_stream().cuda_stream
        si.si_layer_forward(self.h, x.data_ptr(), lg.data_ptr() if lg is not None else None, T, n_g, mode, y.data_ptr(),
                            routing_out=ro, stream=stream)
        torch.cuda.synchronize()
        out = y[:T].cpu().numpy()
        if routing:
            r = {k: v.cpu().numpy() for k, v in bufs.items()}
            r["idx"] = r["idx"][:T * cfg.top_k].reshape(T, cfg.top_k)
            r["w"] = r["w"][:T * cfg.top_k].reshape(T, cfg.top_k)
            r["perm"] = r["perm"][:T * cfg.top_k]
            r["inv"] = r["inv"][:T * cfg.top_k]
            return out, r
        return out

    def close(self):
        if self.h:
            si.si_layer_destroy(self.h)
            self.h = None


def gpu_route(logits, k):
    dev = torch.device("cuda:0")
    T, E = logits.shape
    n = max(T * k, 1)
    lg = torch.from_numpy(np.ascontiguousarray(logits)).to(dev)
    bufs = {"idx": torch.full((n,), -1, dtype=torch.int32, device=dev), "w": torch.zeros(n, dtype=torch.float32, device=dev),
            "count": torch.full((E,), -1, dtype=torch.int32, device=dev), "off": torch.full((E + 1,), -1, dtype=torch.int32, device=dev),
            "perm": torch.full((n,), -1, dtype=torch.int32, device=dev), "inv": torch.full((n,), -1, dtype=torch.int32, device=dev)}
    si.si_route(lg.data_ptr(), T, E, k, {kk: v.data_ptr() for kk, v in bufs.items()}, stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    r = {kk: v.cpu().numpy() for kk, v in bufs.items()}
    r["idx"] = r["idx"][:T * k].reshape(T, k)
    r["w"] = r["w"][:T * k].reshape(T, k)
    r["perm"] = r["perm"][:T * k]
    r["inv"] = r["inv"][:T * k]
    return r


def assert_routing_equal(r_gpu, r_or, T, k):
    """idx, count, off, perm, inv bit-exact; weights to 1e-6 (expf vs exp differ in the last ulp)."""
    for key in ("idx", "count", "off", "perm", "inv"):
        assert np.array_equal(r_gpu[key], r_or[key]), key
    if T:
        assert np.max(np.abs(r_gpu["w"].astype(np.float64) - r_or["w"])) <= 1e-6
        assert np.max(np.abs(r_gpu["w"].sum(axis=1) - 1.0)) <= 1e-6


def assert_parity(y_gpu, y_or, tol=TOL):
    assert y_gpu.shape == y_or.shape
    assert np.all(np.isfinite(y_gpu))
    rms = float(np.sqrt(np.mean(y_or ** 2)))
    err = float(np.max(np.abs(y_gpu.astype(np.float64) - y_or)))
    assert err <= tol * rms, "max-abs error %.3e > %.1e x RMS %.3e" % (err, tol, rms)
    return err / rms
