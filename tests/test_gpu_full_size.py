"""GPU parity at the full sizes of the workload configurations, in the launch configuration that
bench.py times (default staging, SI_DECODE / SI_PREFILL).  The oracle evaluates a seeded sample of
tokens one by one (tokens are independent given the routing): tokens routed to the least and to the
most loaded expert, tokens on both sides of the X1/X2 boundary, and random ones.  Routing outputs are
compared for all tokens, bit-exact."""
import numpy as np
import pytest

import paper_2411_15715_amd as si
import synth
from gpu_helpers import GpuLayer, assert_parity, assert_routing_equal

pytestmark = pytest.mark.gpu

N_SAMPLE = 48


def pick_tokens(r_or, T, n_g, seed, n=N_SAMPLE):
    rng = np.random.default_rng(seed)
    sel = set(rng.integers(0, T, n // 2).tolist())
    sel |= {0, T - 1}
    if 0 < n_g < T:
        sel |= {T - n_g - 1, T - n_g}
    if r_or is not None:
        cnt = r_or["count"]
        nz = np.nonzero(cnt)[0]
        for e in (nz[np.argmin(cnt[nz])], int(np.argmax(cnt))):
            toks = np.nonzero((r_or["idx"] == e).any(axis=1))[0]
            sel |= set(toks[:4].tolist())
    while len(sel) < n:
        sel.add(int(rng.integers(0, T)))
    return np.array(sorted(sel), np.int32)


def check_config(oracle, name, splits, decode_reps=2, prefill_ng=None, placement=None):
    cfg = synth.CONFIGS[name]
    w = synth.make_weights(cfg, threads=16)
    shared = tuple(w[k] for k in ("s_gate", "s_up", "s_down")) if cfg.d_ff_shared else None
    xp = synth.make_tokens(cfg, cfg.t_prefill)
    lp = synth.make_router_logits(cfg, xp)
    r_or = oracle.route(lp, cfg.top_k) if lp is not None else None
    refs = {}
    for split in splits:
        pl = placement(r_or) if placement is not None else None
        L = GpuLayer(cfg, w, split, max_tokens=max(cfg.t_prefill, cfg.t_decode), placement=pl)
        try:
            for rep in range(decode_reps):
                xd = synth.make_tokens(cfg, cfg.t_decode, stream=200 + rep)
                ld = synth.make_router_logits(cfg, xd)
                key = ("d", rep)
                if key not in refs:
                    refs[key] = oracle.layer_forward(xd, w["w_gate"], w["w_up"], w["w_down"], logits=ld, top_k=cfg.top_k, shared=shared)
                if ld is not None:
                    y, r = L.forward(xd, ld, mode=si.SI_DECODE, routing=True)
                    assert_routing_equal(r, oracle.route(ld, cfg.top_k), cfg.t_decode, cfg.top_k)
                else:
                    y = L.forward(xd, None, mode=si.SI_DECODE)
                e = assert_parity(y, refs[key])
                print("%s split=%s decode rep %d: rel err %.2e" % (name, split, rep, e), flush=True)
            for n_g in (prefill_ng or [0]):
                if n_g < 0:
                    n_g = cfg.t_prefill + n_g
                sel = pick_tokens(r_or, cfg.t_prefill, n_g, seed=cfg.seed)
                key = ("p", tuple(sel.tolist()))
                if key not in refs:
                    refs[key] = oracle.layer_forward(xp, w["w_gate"], w["w_up"], w["w_down"], logits=lp, top_k=cfg.top_k, shared=shared, sel=sel)
                if lp is not None:
                    y, r = L.forward(xp, lp, n_g=n_g, mode=si.SI_PREFILL, routing=True)
                    assert_routing_equal(r, r_or, cfg.t_prefill, cfg.top_k)
                else:
                    y = L.forward(xp, None, n_g=n_g, mode=si.SI_PREFILL)
                e = assert_parity(y[sel], refs[key])
                print("%s split=%s prefill n_g=%d: rel err %.2e on %d sampled tokens" % (name, split, n_g, e, len(sel)), flush=True)
        finally:
            L.close()


def test_mixtral_8x7b_full(oracle):
    check_config(oracle, "mixtral_8x7b", [(0.5, 0.5, 0.0), (1.0, 0.0, 0.0)], decode_reps=3)


def test_llama2_70b_full(oracle):
    # 30/50/20 by d_ff columns; n_g = 0 leaves the whole CC share of all 1024 tokens to the host
    # workers, n_g = T moves it to the GPU through CG'
    check_config(oracle, "llama2_70b", [(0.3, 0.5, 0.2)], prefill_ng=[1024, 0])


def test_qwen_moe_full(oracle):
    check_config(oracle, "qwen_moe", [(1.0, 0.0, 0.0), (0.5, 0.5, 0.0)])


def test_phimoe_full_sweep(oracle):
    # every split of the sweep 100/0/0 ... 20/60/20 at full size: one decode call and one prefill call whose last
    # T - 512 tokens take the CC share to the GPU (CG') while the host computes the first 512; the oracle
    # references are computed once and shared by the seven splits
    check_config(oracle, "phimoe", synth.SPLIT_SWEEP, decode_reps=1, prefill_ng=[-512])


def test_mixtral_8x22b_full_sweep(oracle):
    check_config(oracle, "mixtral_8x22b", synth.SPLIT_SWEEP, decode_reps=1, prefill_ng=[-256])


def test_qwen_moe_full_whole_expert_placement(oracle):
    # the 16 most used of the 64 experts resident, the rest split between CG and CC; the rates slice the shared expert
    def place(r_or):
        pl = si.si_place_experts(r_or["count"].astype(np.float64), 16, 0.5)
        assert pl.count(0) == 16 and pl.count(1) > 0 and pl.count(2) > 0
        return pl
    check_config(oracle, "qwen_moe", [(0.5, 0.3, 0.2)], prefill_ng=[0, 1024], placement=place)
