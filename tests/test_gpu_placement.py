"""GPU parity of whole-expert placement (each expert entirely GG, CG or CC): the output is that of the unsliced
layer whatever the placement, so the oracle is called without any slicing."""
import numpy as np
import pytest
import torch

import paper_2411_15715_amd as si
import synth
from gpu_helpers import GpuLayer, assert_parity, assert_routing_equal
from test_gpu_q4 import Q4Layer

pytestmark = pytest.mark.gpu

PLACEMENTS = {
    "mixed": [0, 1, 2, 0, 1, 2, 1, 2],
    "all_gg": [0] * 8,
    "all_cg": [1] * 8,
    "all_cc": [2] * 8,
    "no_gg": [1, 2, 2, 1, 1, 2, 1, 2],
    "one_cc": [0, 0, 0, 2, 0, 0, 0, 0],
}


@pytest.mark.parametrize("name", sorted(PLACEMENTS))
def test_moe_placements(oracle, name):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=512, d_ff=1024)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=700, stage_mib=1, placement=PLACEMENTS[name])
    try:
        for T, stream in ((1, 1), (3, 2), (8, 3)):
            xb = synth.make_tokens(cfg, T, stream=stream)
            lg = synth.make_router_logits(cfg, xb)
            y, r = L.forward(xb, lg, routing=True)
            assert_routing_equal(r, oracle.route(lg, cfg.top_k), T, cfg.top_k)
            assert_parity(y, oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"], logits=lg, top_k=cfg.top_k))
        xb = synth.make_tokens(cfg, 16, stream=4)
        lg = synth.make_router_logits(cfg, xb)
        yo = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"], logits=lg, top_k=cfg.top_k)
        for n_g in (0, 7, 16):
            assert_parity(L.forward(xb, lg, n_g=n_g, mode=si.SI_DECODE), yo)
        xp = synth.make_tokens(cfg, 700)
        lg = synth.make_router_logits(cfg, xp)
        yo = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"], logits=lg, top_k=cfg.top_k)
        for n_g in (0, 333, 700):
            assert_parity(L.forward(xp, lg, n_g=n_g), yo)
        # twice in a row: nothing left over from the previous call (zero-filled rows, slot reuse)
        assert_parity(L.forward(xp[:5], lg[:5]), yo[:5])
        assert_parity(L.forward(xp[:5], lg[:5]), yo[:5])
    finally:
        L.close()


def test_placement_with_shared_expert_and_zipf(oracle):
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=256, d_ff=384, d_ff_shared=1024, n_experts=32)
    w = synth.make_weights(cfg)
    xp = synth.make_tokens(cfg, 600)
    lg = synth.make_router_logits(cfg, xp)
    r = oracle.route(lg, cfg.top_k)
    place = si.si_place_experts(r["count"].astype(np.float64), 8, 0.5)   # the 8 most used experts resident
    assert sorted(set(place)) == [0, 1, 2]
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down"))
    L = GpuLayer(cfg, w, (0.4, 0.3, 0.3), max_tokens=600, stage_mib=1, placement=place)   # the rates slice the shared expert
    try:
        yo = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"], logits=lg, top_k=cfg.top_k, shared=shared)
        for n_g in (0, 250, 600):
            assert_parity(L.forward(xp, lg, n_g=n_g), yo)
        xd = xp[:4]
        assert_parity(L.forward(xd, lg[:4]), yo[:4])
    finally:
        L.close()


def test_placement_q4(oracle):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=512, d_ff=1024)
    wq = synth.make_weights_q4(cfg)
    L = Q4Layer(cfg, wq, (1.0, 0.0, 0.0), max_tokens=300, stage_mib=1, placement=PLACEMENTS["mixed"])
    try:
        for T, n_g in ((2, 0), (300, 100)):
            xb = synth.make_tokens(cfg, T, stream=T)
            lg = synth.make_router_logits(cfg, xb)
            assert_parity(L.forward(xb, lg, n_g=n_g), oracle.layer_forward_q4(xb, wq, logits=lg, top_k=cfg.top_k))
    finally:
        L.close()


def test_placement_argument_checks():
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=128, d_ff=128)
    w = synth.make_weights(cfg)
    with pytest.raises(si.ScheInferError) as ei:
        si.si_layer_create(cfg.d_model, cfg.d_ff, 8, 2, w["w_gate"], w["w_up"], w["w_down"], 1.0, 0.0, 0.0, 8,
                           placement=[0, 1, 2, 3, 0, 0, 0, 0])
    assert ei.value.code == si.SI_EINVAL
    with pytest.raises(ValueError):
        si.si_layer_create(cfg.d_model, cfg.d_ff, 8, 2, w["w_gate"], w["w_up"], w["w_down"], 1.0, 0.0, 0.0, 8, placement=[0, 1])
