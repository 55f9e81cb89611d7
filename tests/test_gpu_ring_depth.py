"""The LDS ring of the prompt-phase GEMMs synchronises with hand-counted waits on outstanding loads, so every
body (64, 128, 192, 256, 320 rows; 3 or 2 stages) is run here with fewer k-tiles than stages, as many, and more, in the
bf16 loop and in the 4-bit loop, against the oracle.  FC1 contracts over d_model (k-tiles = d_model / 64); FC2
over the hidden columns of one k-split (the layer cuts the chunk range of a 1-tile launch into 4 splits, so
d_ff = 64 gives splits of 1, 0, 0, 0 k-tiles and d_ff = 512 / 768 / 1024 gives 2 / 3 / 4 each)."""
import numpy as np
import pytest

import paper_2411_15715_amd as si
import synth
from gpu_helpers import GpuLayer, assert_parity
from test_gpu_q4 import Q4Layer

pytestmark = pytest.mark.gpu

# one row tile each: the 64-, 128-, 192-, 256- and 320-row body (the 4-bit GEMMs take the 300 rows as 256 + 44 in
# two passes of one block)
ROWS = (40, 100, 150, 250, 300)


@pytest.mark.parametrize("d_model", [64, 128, 192, 256])
@pytest.mark.parametrize("d_ff", [64, 512, 768, 1024])
def test_ring_depth_bf16(oracle, d_model, d_ff):
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=d_model, d_ff=d_ff, seed=100 + d_model + d_ff)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=max(ROWS))
    try:
        xp = synth.make_tokens(cfg, max(ROWS))
        yo = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"])
        for T in ROWS:
            print("ring depth bf16 M=%d H=%d T=%d" % (d_model, d_ff, T), flush=True)
            assert_parity(L.forward(xp[:T], None, mode=si.SI_PREFILL), yo[:T])
    finally:
        L.close()


@pytest.mark.parametrize("d_model,d_ff", [(384, 1536), (448, 1792), (512, 2048), (1024, 4096)])
def test_ring_depth_streaming(oracle, d_model, d_ff):
    """Tiles of at most 192 rows run a loop whose weights travel through registers, up to five k-tiles ahead: its
    hand-counted waits reach their steady state only with at least 6 (64 rows), 5 (128) or 3 (192) k-tiles, so
    here FC1 has 6, 7, 8 and 16 k-tiles and a k-split of FC2 as many."""
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=d_model, d_ff=d_ff, seed=300 + d_model)
    w = synth.make_weights(cfg)
    L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=max(ROWS))
    try:
        xp = synth.make_tokens(cfg, max(ROWS))
        yo = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"])
        for T in ROWS:
            print("ring depth streaming M=%d H=%d T=%d" % (d_model, d_ff, T), flush=True)
            assert_parity(L.forward(xp[:T], None, mode=si.SI_PREFILL), yo[:T])
    finally:
        L.close()


@pytest.mark.parametrize("d_model", [64, 128, 192, 256])
@pytest.mark.parametrize("d_ff", [64, 512, 768, 1024])
def test_ring_depth_q4(oracle, d_model, d_ff):
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=d_model, d_ff=d_ff, seed=200 + d_model + d_ff)
    wq = synth.make_weights_q4(cfg)
    # Power-of-two scales (2^-7, about the synthetic mean): (code - 8) * scale is then a bfloat16 exactly, so the one
    # rounding per weight of the 4-bit GEMMs costs nothing and the test measures the ring, not that rounding (which
    # alone reaches 2e-2 x RMS on layers this small: 64 x 64 weights leave nothing to average over)
    for key in ("z_gate", "z_up", "z_down"):
        wq[key] = np.full_like(wq[key], 0x3C00)
    L = Q4Layer(cfg, wq, (1.0, 0.0, 0.0), max_tokens=max(ROWS))
    try:
        xp = synth.make_tokens(cfg, max(ROWS))
        yo = oracle.layer_forward_q4(xp, wq)
        for T in ROWS:
            print("ring depth 4-bit M=%d H=%d T=%d" % (d_model, d_ff, T), flush=True)
            assert_parity(L.forward(xp[:T], None, mode=si.SI_PREFILL), yo[:T])
    finally:
        L.close()


@pytest.mark.parametrize("q4", [False, True])
def test_last_tile_takes_spill_rows(oracle, q4):
    """An expert's last row tile also takes up to 64 rows beyond 256: row counts on both sides of every boundary
    (one tile of 320, 256 + 65, 256 + 320, 256 + 256 + 65)."""
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=256, d_ff=768, seed=77)
    rows = (256, 257, 320, 321, 576, 577)
    xp = synth.make_tokens(cfg, max(rows))
    if q4:
        wq = synth.make_weights_q4(cfg)
        for key in ("z_gate", "z_up", "z_down"):
            wq[key] = np.full_like(wq[key], 0x3C00)  # exact products: see test_ring_depth_q4
        L = Q4Layer(cfg, wq, (1.0, 0.0, 0.0), max_tokens=max(rows))
        yo = oracle.layer_forward_q4(xp, wq)
    else:
        w = synth.make_weights(cfg)
        L = GpuLayer(cfg, w, (1.0, 0.0, 0.0), max_tokens=max(rows))
        yo = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"])
    try:
        for T in rows:
            print("spill rows q4=%s T=%d" % (q4, T), flush=True)
            assert_parity(L.forward(xp[:T], None, mode=si.SI_PREFILL), yo[:T])
    finally:
        L.close()
