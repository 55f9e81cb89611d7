"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.
Routing indices, counts, offsets and permutations bit-exact; outputs within 2e-2 x RMS."""
import numpy as np
import pytest

import paper_2411_15715_amd as si
import synth
from gpu_helpers import GpuLayer, assert_parity, assert_routing_equal, gpu_route

pytestmark = pytest.mark.gpu


def oracle_y(oracle, cfg, w, xb, lg, sel=None):
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
    return oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"], logits=lg, top_k=cfg.top_k, shared=shared, sel=sel)


# ------------------------------------------------------------------ token assignment
@pytest.mark.parametrize("T,E,k", [(1, 8, 2), (4, 64, 8), (7, 3, 3), (512, 8, 2), (1500, 16, 2), (4096, 64, 8),
                                   (2048, 256, 8), (1024, 1, 1), (33, 200, 5)])
def test_route_bit_exact(oracle, T, E, k):
    rng = np.random.default_rng(T * 1000 + E)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    assert_routing_equal(gpu_route(logits, k), oracle.route(logits, k), T, k)


def test_route_ties_and_skew(oracle):
    rng = np.random.default_rng(5)
    # heavy ties: logits quantised to a few values
    logits = np.round(rng.standard_normal((777, 16)) * 2).astype(np.float32) / 2
    assert_routing_equal(gpu_route(logits, 4), oracle.route(logits, 4), 777, 4)
    # all equal
    logits = np.zeros((65, 8), np.float32)
    r = gpu_route(logits, 3)
    assert_routing_equal(r, oracle.route(logits, 3), 65, 3)
    assert np.array_equal(r["idx"][0], [0, 1, 2])
    # everything routed to one expert pair: other experts get no token
    logits = np.zeros((300, 8), np.float32)
    logits[:, 5] = 9.0
    logits[:, 2] = 7.0
    r = gpu_route(logits, 2)
    assert_routing_equal(r, oracle.route(logits, 2), 300, 2)
    assert r["count"].tolist() == [0, 0, 300, 0, 0, 300, 0, 0]
    # Zipf-skewed router of the Qwen-shaped workload
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128)
    xb = synth.make_tokens(cfg, 2048)
    lg = synth.make_router_logits(cfg, xb)
    assert_routing_equal(gpu_route(lg, cfg.top_k), oracle.route(lg, cfg.top_k), 2048, cfg.top_k)


# ------------------------------------------------------------------ config 0 (tiny dense), as specified
def test_tiny_dense_config(oracle):
    cfg = synth.CONFIGS["tiny_dense"]
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, cfg.split, max_tokens=32)
    try:
        assert (L.info["n_gg"], L.info["n_cg"], L.info["n_cc"]) == (256, 256, 192)
        xd = synth.make_tokens(cfg, cfg.t_decode, stream=1)
        assert_parity(L.forward(xd, None), oracle_y(oracle, cfg, w, xd, None))
        for n_g in (0, 2, 4):
            assert_parity(L.forward(xd, None, n_g=n_g, mode=si.SI_DECODE), oracle_y(oracle, cfg, w, xd, None))
        xp = synth.make_tokens(cfg, cfg.t_prefill)
        yo = oracle_y(oracle, cfg, w, xp, None)
        for n_g in (0, 16, 32):
            assert_parity(L.forward(xp, None, n_g=n_g), yo)
        # the prefill kernels on the decode batch and the decode kernels on a 16-token batch
        assert_parity(L.forward(xd, None, mode=si.SI_PREFILL), oracle_y(oracle, cfg, w, xd, None))
        assert_parity(L.forward(xp[:16], None, n_g=5, mode=si.SI_DECODE), yo[:16])
    finally:
        L.close()


SPLITS = [(1.0, 0.0, 0.0), (0.0, 1.0, 0.0), (0.0, 0.0, 1.0), (0.5, 0.5, 0.0), (0.4, 0.3, 0.3), (0.2, 0.6, 0.2)]


@pytest.mark.parametrize("split", SPLITS)
def test_dense_reduced_splits(oracle, split):
    # LLaMA-shaped (dense) at reduced size: several row tiles with a ragged tail, several staged pieces
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=512, d_ff=1792)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, split, max_tokens=300, stage_mib=1)
    try:
        x1 = synth.make_tokens(cfg, 1, stream=2)
        assert_parity(L.forward(x1, None), oracle_y(oracle, cfg, w, x1, None))
        x6 = synth.make_tokens(cfg, 6, stream=3)
        assert_parity(L.forward(x6, None), oracle_y(oracle, cfg, w, x6, None))
        xp = synth.make_tokens(cfg, 300)
        yo = oracle_y(oracle, cfg, w, xp, None)
        for n_g in (0, 100, 300):
            assert_parity(L.forward(xp, None, n_g=n_g), yo)
    finally:
        L.close()


@pytest.mark.parametrize("split", SPLITS)
def test_moe_reduced_splits(oracle, split):
    # Mixtral-shaped at reduced size: 8 experts top-2
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=512, d_ff=1024)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, split, max_tokens=700, stage_mib=1)
    try:
        for T, stream in ((1, 1), (3, 2), (8, 3)):
            xb = synth.make_tokens(cfg, T, stream=stream)
            lg = synth.make_router_logits(cfg, xb)
            y, r = L.forward(xb, lg, routing=True)
            assert_routing_equal(r, oracle.route(lg, cfg.top_k), T, cfg.top_k)
            assert_parity(y, oracle_y(oracle, cfg, w, xb, lg))
        xb = synth.make_tokens(cfg, 16, stream=4)
        lg = synth.make_router_logits(cfg, xb)
        assert_parity(L.forward(xb, lg, n_g=7, mode=si.SI_DECODE), oracle_y(oracle, cfg, w, xb, lg))
        xp = synth.make_tokens(cfg, 700)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle_y(oracle, cfg, w, xp, lg)
        for n_g in (0, 333, 700):
            y, r = L.forward(xp, lg, n_g=n_g, routing=True)
            assert_routing_equal(r, oracle.route(lg, cfg.top_k), 700, cfg.top_k)
            assert_parity(y, yo)
    finally:
        L.close()


@pytest.mark.parametrize("split", [(1.0, 0.0, 0.0), (0.5, 0.5, 0.0), (0.4, 0.3, 0.3), (0.0, 0.0, 1.0)])
def test_shared_expert_zipf_reduced(oracle, split):
    # Qwen-MoE-shaped at reduced size: many experts, top-8, shared expert, Zipf-skewed routing
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=256, d_ff=384, d_ff_shared=1024, n_experts=32)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, split, max_tokens=600, stage_mib=1)
    try:
        xd = synth.make_tokens(cfg, 4, stream=1)
        lg = synth.make_router_logits(cfg, xd)
        assert_parity(L.forward(xd, lg), oracle_y(oracle, cfg, w, xd, lg))
        xp = synth.make_tokens(cfg, 600)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle_y(oracle, cfg, w, xp, lg)
        r_or = oracle.route(lg, cfg.top_k)
        assert r_or["count"].max() > 3 * max(1, r_or["count"].min())
        for n_g in (0, 250):
            y, r = L.forward(xp, lg, n_g=n_g, routing=True)
            assert_routing_equal(r, r_or, 600, cfg.top_k)
            assert_parity(y, yo)
    finally:
        L.close()


def test_split_does_not_change_gpu_output(oracle):
    """Section III-B: the sliced result is identical to the unsliced one.  Same kernels, different
    placement: GPU vs GPU agrees far tighter than GPU vs oracle."""
    cfg = synth.scaled(synth.CONFIGS["phimoe"], d_model=256, d_ff=640, n_experts=16)
    w = synth.make_weights(cfg)
    xb = synth.make_tokens(cfg, 260)
    lg = synth.make_router_logits(cfg, xb)
    yo = oracle_y(oracle, cfg, w, xb, lg)
    rms = float(np.sqrt(np.mean(yo ** 2)))
    ys = []
    for split in synth.SPLIT_SWEEP:
        L = GpuLayer(cfg, w, split, max_tokens=260, stage_mib=1)
        try:
            ys.append((L.forward(xb, lg, n_g=130), L.forward(xb[:2], lg[:2])))
        finally:
            L.close()
        assert_parity(ys[-1][0], yo)
        assert_parity(ys[-1][1], yo[:2])
    for yp, yd in ys[1:]:
        # prefill: the host (CC) keeps the activations in fp32, the GPU rounds them to bf16 once
        assert np.max(np.abs(yp - ys[0][0])) <= 1e-2 * rms
        assert np.max(np.abs(yd - ys[0][1])) <= 1e-4 * rms


def test_max_tokens_beyond_32bit_offsets_is_refused():
    """The prompt-phase GEMMs address operand rows with 32-bit element offsets: a layer whose max_tokens would
    take x (or the activations) to 2^31 elements is refused at creation, before anything large is allocated."""
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=8192, d_ff=64)
    w = synth.make_weights(cfg)
    with pytest.raises(si.ScheInferError) as ei:
        GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=(1 << 31) // 8192)
    assert ei.value.code == si.SI_EINVAL
    L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=1024)  # a sane limit still creates
    L.close()


def test_edge_cases(oracle):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=128, d_ff=256)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (0.5, 0.25, 0.25), max_tokens=64, stage_mib=1)
    try:
        import torch
        # T = 0 is a no-op and leaves y untouched
        y = torch.full((1, cfg.d_model), 7.0, device="cuda:0")
        si.si_layer_forward(L.h, y.data_ptr(), y.data_ptr(), 0, 0, si.SI_AUTO, y.data_ptr())
        torch.cuda.synchronize()
        assert float(y.min()) == 7.0
        xb = synth.make_tokens(cfg, 65)
        lg = synth.make_router_logits(cfg, xb)
        with pytest.raises(si.ScheInferError) as ei:
            L.forward(xb, lg)
        assert ei.value.code == si.SI_ESTATE
        with pytest.raises(si.ScheInferError) as ei:
            L.forward(xb[:17], lg[:17], mode=si.SI_DECODE)
        assert ei.value.code == si.SI_ESTATE
        with pytest.raises(si.ScheInferError) as ei:
            L.forward(xb[:4], lg[:4], n_g=5)
        assert ei.value.code == si.SI_EINVAL
        with pytest.raises(si.ScheInferError) as ei:
            L.forward(xb[:4], None)
        assert ei.value.code == si.SI_EINVAL
        # the layer still works afterwards; repeated calls give identical results (deterministic)
        y1 = L.forward(xb[:64], lg[:64], n_g=10)
        y2 = L.forward(xb[:64], lg[:64], n_g=10)
        assert np.array_equal(y1, y2)
        assert_parity(y1, oracle_y(oracle, cfg, w, xb[:64], lg[:64]))
        d1 = L.forward(xb[:1], lg[:1])
        d2 = L.forward(xb[:1], lg[:1])
        assert np.array_equal(d1, d2)
    finally:
        L.close()


def test_unusual_shapes_and_knobs(oracle):
    """Granule 128, three staging buffers, top_k == n_experts, d_model not a multiple of 256 or 512,
    a hidden size with an odd number of chunks, several forward calls in a row on one layer."""
    cfg = synth.scaled(synth.CONFIGS["phimoe"], d_model=192, d_ff=640, n_experts=4, top_k=4)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (0.4, 0.4, 0.2), max_tokens=300, granule=128, stage_mib=1, n_stage=3, cc_threads=3)
    try:
        assert (L.info["n_gg"], L.info["n_cg"], L.info["n_cc"]) == (256, 256, 128)
        for T, n_g, mode in ((2, 0, si.SI_AUTO), (9, 4, si.SI_DECODE), (9, 4, si.SI_PREFILL), (300, 77, si.SI_AUTO),
                             (130, 130, si.SI_AUTO), (1, 1, si.SI_AUTO)):
            xb = synth.make_tokens(cfg, T, stream=T)
            lg = synth.make_router_logits(cfg, xb)
            y, r = L.forward(xb, lg, n_g=n_g, mode=mode, routing=True)
            assert_routing_equal(r, oracle.route(lg, cfg.top_k), T, cfg.top_k)
            assert np.array_equal(r["count"], np.full(4, T))  # top_k == E: every expert gets every token
            assert_parity(y, oracle_y(oracle, cfg, w, xb, lg))
    finally:
        L.close()
    # many experts, few tokens: most experts receive nothing
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128, d_ff=128, d_ff_shared=0, n_experts=256, top_k=6)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (0.5, 0.5, 0.0), max_tokens=40, stage_mib=1)
    try:
        for T in (3, 40):
            xb = synth.make_tokens(cfg, T, stream=T)
            lg = synth.make_router_logits(cfg, xb)
            y, r = L.forward(xb, lg, routing=True)
            assert_routing_equal(r, oracle.route(lg, cfg.top_k), T, cfg.top_k)
            assert (r["count"] == 0).sum() > 100
            assert_parity(y, oracle_y(oracle, cfg, w, xb, lg))
    finally:
        L.close()


@pytest.mark.parametrize("shape", ["moe", "shared", "dense", "many_experts", "topk_all"])
def test_resident_decode_two_launch_path(oracle, shape):
    """Generation-phase calls of a fully resident layer with at most 4 tokens and 8 (token, expert) pairs derive the
    token assignment inside the gate/up launch instead of by a kernel of its own.  Routing tables bit-exact,
    outputs within the bar; repeated and interleaved calls (more tokens, fewer tokens, calls that take the separate
    assignment kernel because they have more pairs) leave no state behind."""
    if shape == "moe":
        cfg = synth.scaled(synth.CONFIGS["phimoe"], d_model=512, d_ff=1280, n_experts=16)
    elif shape == "shared":
        cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=256, d_ff=384, d_ff_shared=1024, n_experts=64)
    elif shape == "dense":
        cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=512, d_ff=1792)
    elif shape == "many_experts":
        cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128, d_ff=128, d_ff_shared=0, n_experts=256, top_k=6)
    else:
        cfg = synth.scaled(synth.CONFIGS["phimoe"], d_model=192, d_ff=640, n_experts=16, top_k=16)  # 4 x 16 = 64 pairs
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=16)
    try:
        outs = {}
        for T in (4, 1, 3, 7, 2, 4, 16, 1):
            xb = synth.make_tokens(cfg, T, stream=40 + T)
            lg = synth.make_router_logits(cfg, xb)
            if lg is not None and T == 3:
                lg[1] = lg[0]            # two tokens with identical logits
                lg[2, :] = 0.25          # all experts tied: the lowest indices win
            if lg is not None:
                y, r = L.forward(xb, lg, mode=si.SI_DECODE, routing=True)
                assert_routing_equal(r, oracle.route(lg, cfg.top_k), T, cfg.top_k)
            else:
                y = L.forward(xb, None, mode=si.SI_DECODE)
            assert_parity(y, oracle_y(oracle, cfg, w, xb, lg))
            if T in outs:
                assert np.array_equal(outs[T], y)   # same call again after other calls: bit-identical
            outs[T] = y
    finally:
        L.close()
