"""si_route_noalloc (the entry point for callers that cannot allocate) against si_route through the C ABI:
bit-exact tables, two calls in a row on the same GPU, the second with a smaller input, with and without the
caller's own idx / w (without them both tables live in the library's fixed device array)."""
import numpy as np
import pytest
import torch

import paper_2411_15715_amd as si

pytestmark = pytest.mark.gpu

KEYS = ("idx", "w", "count", "off", "perm", "inv")


def _bufs(T, E, k, dev):
    n = max(T * k, 1)
    return {"idx": torch.full((n,), -1, dtype=torch.int32, device=dev), "w": torch.full((n,), -1.0, dtype=torch.float32, device=dev),
            "count": torch.full((E,), -1, dtype=torch.int32, device=dev), "off": torch.full((E + 1,), -1, dtype=torch.int32, device=dev),
            "perm": torch.full((n,), -1, dtype=torch.int32, device=dev), "inv": torch.full((n,), -1, dtype=torch.int32, device=dev)}


def _route(fn, lg, T, E, k, omit=()):
    dev = lg.device
    b = _bufs(T, E, k, dev)
    fn(lg.data_ptr(), T, E, k, {kk: (None if kk in omit else v.data_ptr()) for kk, v in b.items()},
       stream=torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    return {kk: v.cpu().numpy() for kk, v in b.items() if kk not in omit}


def test_noalloc_matches_si_route_on_two_calls_in_a_row():
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(11)
    # second call smaller than the first: what the first left in the fixed array must not leak into it
    for (T, E, k) in [(4096, 64, 8), (37, 8, 2)]:
        logits = rng.standard_normal((T, E)).astype(np.float32)
        logits[::5, 1] = logits[::5, 0]  # ties
        lg = torch.from_numpy(logits).to(dev)
        print("si_route_noalloc T=%d E=%d k=%d" % (T, E, k), flush=True)
        ref = _route(si.si_route, lg, T, E, k)
        got_full = _route(si.si_route_noalloc, lg, T, E, k)
        for key in KEYS:
            assert np.array_equal(ref[key], got_full[key]), key  # same kernels, same inputs: bit-identical, w included
        got = _route(si.si_route_noalloc, lg, T, E, k, omit=("idx", "w"))
        for key in ("count", "off", "perm", "inv"):
            assert np.array_equal(ref[key], got[key]), key


def test_noalloc_rejects_sizes_beyond_its_scratch():
    dev = torch.device("cuda:0")
    lg = torch.zeros((8, 8), dtype=torch.float32, device=dev)
    T = si.SI_ROUTE_NOALLOC_MAX_PAIRS // 8 + 1
    with pytest.raises(si.ScheInferError) as ei:
        si.si_route_noalloc(lg.data_ptr(), T, 8, 8, {"count": lg.data_ptr()})
    assert ei.value.code == si.SI_EINVAL
    assert "exceeds" in str(ei.value)
