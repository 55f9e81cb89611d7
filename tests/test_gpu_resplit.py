"""Re-slicing an existing layer: after si_layer_resplit the layer must compute exactly what a layer created at the
new rates computes (same chunks in the same places, same launches: bit-identical), and stay within the parity bar
of the oracle, through a chain of rate changes that crosses every boundary direction (chunks leaving the GPU,
chunks becoming resident, parts appearing and disappearing)."""
import numpy as np
import pytest

import paper_2411_15715_amd as si
import synth
from gpu_helpers import GpuLayer, assert_parity
from test_gpu_parity import oracle_y
from test_gpu_q4 import Q4Layer

pytestmark = pytest.mark.gpu

CHAIN = [(0.4, 0.3, 0.3), (1.0, 0.0, 0.0), (0.0, 0.0, 1.0), (0.0, 1.0, 0.0), (0.7, 0.1, 0.2), (0.2, 0.6, 0.2), (0.4, 0.3, 0.3)]


def _run_chain(make, cfg, cases, oracle_out):
    """cases: list of (x_bits, logits, n_g, mode); oracle_out: matching list of oracle outputs."""
    L = make(CHAIN[0])
    try:
        for split in CHAIN[1:]:
            si.si_layer_resplit(L.h, *split)
            fresh = make(split)
            try:
                assert si.si_layer_split_info(L.h) == fresh.info
                for (xb, lg, n_g, mode), yo in zip(cases, oracle_out):
                    y = L.forward(xb, lg, n_g=n_g, mode=mode)
                    assert_parity(y, yo)
                    # the host workers sum their partial results in an order that depends on thread timing only
                    # through which thread takes which chunk, never within a chunk: outputs are reproducible
                    assert np.array_equal(y, fresh.forward(xb, lg, n_g=n_g, mode=mode)), split
            finally:
                fresh.close()
    finally:
        L.close()


def test_resplit_dense(oracle):
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=512, d_ff=1792)
    w = synth.make_weights(cfg)
    x1, x6, xp = synth.make_tokens(cfg, 1, stream=2), synth.make_tokens(cfg, 6, stream=3), synth.make_tokens(cfg, 300)
    cases = [(x1, None, 0, si.SI_AUTO), (x6, None, 0, si.SI_AUTO), (xp, None, 0, si.SI_AUTO), (xp, None, 120, si.SI_AUTO)]
    outs = [oracle_y(oracle, cfg, w, x, None) for x in (x1, x6, xp)]
    outs.append(outs[2])
    _run_chain(lambda s: GpuLayer(cfg, w, s, max_tokens=300, stage_mib=1), cfg, cases, outs)


def test_resplit_moe_shared(oracle):
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=256, d_ff=256, d_ff_shared=1024, n_experts=16)
    w = synth.make_weights(cfg)
    cases, outs = [], []
    for T, n_g in ((1, 0), (5, 0), (400, 0), (400, 150)):
        xb = synth.make_tokens(cfg, T, stream=T)
        lg = synth.make_router_logits(cfg, xb)
        cases.append((xb, lg, n_g, si.SI_AUTO))
        outs.append(oracle_y(oracle, cfg, w, xb, lg))
    _run_chain(lambda s: GpuLayer(cfg, w, s, max_tokens=400, stage_mib=1), cfg, cases, outs)


def test_resplit_q4(oracle):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=512, d_ff=1024)
    wq = synth.make_weights_q4(cfg)
    cases, outs = [], []
    for T, n_g in ((1, 0), (8, 0), (300, 0), (300, 100)):
        xb = synth.make_tokens(cfg, T, stream=T)
        lg = synth.make_router_logits(cfg, xb)
        cases.append((xb, lg, n_g, si.SI_AUTO))
        outs.append(oracle.layer_forward_q4(xb, wq, logits=lg, top_k=cfg.top_k))
    _run_chain(lambda s: Q4Layer(cfg, wq, s, max_tokens=300, stage_mib=1), cfg, cases, outs)


def test_resplit_errors():
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=256, d_ff=256)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (0.5, 0.25, 0.25), max_tokens=16)
    try:
        before = si.si_layer_split_info(L.h)
        for bad in ((0.5, 0.5, 0.5), (-0.1, 0.6, 0.5), (float("nan"), 0.5, 0.5)):
            with pytest.raises(si.ScheInferError) as ei:
                si.si_layer_resplit(L.h, *bad)
            assert ei.value.code == si.SI_EINVAL
        assert si.si_layer_split_info(L.h) == before
    finally:
        L.close()
    P = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=16, placement=[0, 1, 2, 0, 1, 2, 0, 0])
    try:
        with pytest.raises(si.ScheInferError) as ei:
            si.si_layer_resplit(P.h, 0.5, 0.5, 0.0)
        assert ei.value.code == si.SI_ESTATE
    finally:
        P.close()
