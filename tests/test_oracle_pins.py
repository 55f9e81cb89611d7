"""Pins for the CPU oracle: things the paper and the mathematics fix, none of which reuse the
oracle's own code.  A dropped term, a wrong sign/index or a transposed operand in the oracle
fails at least one of them.

Pinned here:
  - SiLU closed forms (scalar function)
  - dense SwiGLU MLP: brute-force Python loops, a hand-computed 2x1 case, zero cases, exact
    power-of-two homogeneity, and a NumPy float64 matmul expression (library routine)
  - slicing invariance (Section III-B, Eq. 1-2: the sliced output is identical to the unsliced one)
    for every rate in the sweep and every n_g
  - routing: brute-force full sort, invariants, ties, dominance, k = E
  - MoE: reductions to the dense MLP, expert-permutation invariance, shared-expert special cases
  - rate -> column-count table worked out by hand (tests/golden/split_counts.txt)
"""
import math
import os

import numpy as np
import pytest

import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    """float array -> bf16 bit patterns (uint16), and the exactly representable float64 values."""
    bits = synth.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))
    return bits, synth.bf16_bits_to_f64(bits)


def rand_bits(rng, shape, std):
    return bf16(rng.standard_normal(shape) * std)


def np_silu(z):
    return z / (1.0 + np.exp(-z))


def np_mlp(xv, g, u, d):
    """silu(x Wg^T) * (x Wu^T) Wd in float64 with library matmuls; weights [H, M]."""
    return (np_silu(xv @ g.T) * (xv @ u.T)) @ d


# ---------------------------------------------------------------- scalar function
def test_silu_closed_forms(oracle):
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-16
    assert abs(oracle.silu(1.0) - 0.7310585786300049) < 1e-15
    for z in (0.25, 1.5, 3.0, 7.0, 20.0):
        assert abs(oracle.silu(z) - oracle.silu(-z) - z) < 1e-14 * max(1.0, z)
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12
    assert abs(oracle.silu(-40.0)) < 1e-15
    assert oracle.silu(-1.0) < 0.0  # SiLU dips below zero for negative arguments


# ---------------------------------------------------------------- dense MLP
def brute_mlp(xv, g, u, d):
    """Per-token, per-j, per-m scalar loops on Python floats."""
    T, M = xv.shape
    H = g.shape[0]
    y = [[0.0] * M for _ in range(T)]
    for t in range(T):
        for j in range(H):
            gs = 0.0
            us = 0.0
            for m in range(M):
                gs += float(xv[t, m]) * float(g[j, m])
                us += float(xv[t, m]) * float(u[j, m])
            h = gs / (1.0 + math.exp(-gs)) * us
            for m in range(M):
                y[t][m] += h * float(d[j, m])
    return np.array(y)


def test_dense_bruteforce_tiny(oracle):
    rng = np.random.default_rng(11)
    for (T, M, H) in [(1, 1, 1), (3, 5, 7), (4, 8, 6), (2, 7, 3)]:
        xb, xv = rand_bits(rng, (T, M), 1.0)
        gb, gv = rand_bits(rng, (1, H, M), 0.5)
        ub, uv = rand_bits(rng, (1, H, M), 0.5)
        db, dv = rand_bits(rng, (1, H, M), 0.5)
        y = oracle.layer_forward(xb, gb, ub, db)
        ref = brute_mlp(xv, gv[0], uv[0], dv[0])
        assert np.allclose(y, ref, rtol=1e-13, atol=1e-15)


def test_dense_hand_case(oracle):
    # M = 2, H = 1: x = [1, 2], Wg = [1, 0.5] -> g = 2; Wu = [0.5, -1] -> u = -1.5;
    # h = SiLU(2) * (-1.5); Wd = [2, -4] -> y = h * [2, -4].
    xb, _ = bf16([[1.0, 2.0]])
    gb, _ = bf16([[[1.0, 0.5]]])
    ub, _ = bf16([[[0.5, -1.0]]])
    db, _ = bf16([[[2.0, -4.0]]])
    h = 2.0 / (1.0 + math.exp(-2.0)) * -1.5
    y = oracle.layer_forward(xb, gb, ub, db)
    assert np.allclose(y, [[2.0 * h, -4.0 * h]], rtol=1e-15, atol=0)
    # two hidden columns: contributions add
    gb2, _ = bf16([[[1.0, 0.5], [0.0, 1.0]]])
    ub2, _ = bf16([[[0.5, -1.0], [1.0, 1.0]]])
    db2, _ = bf16([[[2.0, -4.0], [1.0, 1.0]]])
    h2 = 2.0 / (1.0 + math.exp(-2.0)) * 3.0
    y2 = oracle.layer_forward(xb, gb2, ub2, db2)
    assert np.allclose(y2, [[2.0 * h + h2, -4.0 * h + h2]], rtol=1e-15, atol=0)


def test_dense_zero_cases_and_homogeneity(oracle):
    rng = np.random.default_rng(5)
    T, M, H = 3, 24, 40
    xb, _ = rand_bits(rng, (T, M), 1.0)
    gb, _ = rand_bits(rng, (1, H, M), 0.3)
    ub, uv = rand_bits(rng, (1, H, M), 0.3)
    db, dv = rand_bits(rng, (1, H, M), 0.3)
    zero = np.zeros((1, H, M), np.uint16)
    assert np.all(oracle.layer_forward(xb, zero, ub, db) == 0.0)   # g = 0 -> SiLU(0) = 0
    assert np.all(oracle.layer_forward(xb, gb, zero, db) == 0.0)   # u = 0
    assert np.all(oracle.layer_forward(xb, gb, ub, zero) == 0.0)   # Wd = 0
    y = oracle.layer_forward(xb, gb, ub, db)
    assert np.any(y != 0.0)
    d2, _ = bf16(dv * 2.0)
    u2, _ = bf16(uv * 2.0)
    assert np.array_equal(oracle.layer_forward(xb, gb, ub, d2), 2.0 * y)  # exact in binary fp
    assert np.array_equal(oracle.layer_forward(xb, gb, u2, db), 2.0 * y)
    # the gate is NOT homogeneous: doubling it must not simply double y
    g2, _ = bf16(synth.bf16_bits_to_f64(gb) * 2.0)
    assert not np.allclose(oracle.layer_forward(xb, g2, ub, db), 2.0 * y)


def test_dense_matches_numpy_matmul(oracle):
    rng = np.random.default_rng(7)
    T, M, H = 9, 96, 160  # M != H so a transposed operand cannot pass
    xb, xv = rand_bits(rng, (T, M), 1.0)
    gb, gv = rand_bits(rng, (1, H, M), 0.1)
    ub, uv = rand_bits(rng, (1, H, M), 0.1)
    db, dv = rand_bits(rng, (1, H, M), 0.1)
    y = oracle.layer_forward(xb, gb, ub, db)
    ref = np_mlp(xv, gv[0], uv[0], dv[0])
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    # swapping gate and up changes the result (SiLU is applied to the gate only)
    assert not np.allclose(oracle.layer_forward(xb, ub, gb, db), ref, rtol=1e-3)
    # token selection returns the same rows
    sel = [7, 0, 3]
    ys = oracle.layer_forward(xb, gb, ub, db, sel=sel)
    assert np.array_equal(ys, y[sel])


def test_tiny_config_matches_numpy(oracle):
    cfg = synth.CONFIGS["tiny_dense"]
    w = synth.make_weights(cfg)
    xb = synth.make_tokens(cfg, cfg.t_prefill)
    y = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"])
    ref = np_mlp(synth.bf16_bits_to_f64(xb), *(synth.bf16_bits_to_f64(w[k][0]) for k in ("w_gate", "w_up", "w_down")))
    assert np.allclose(y, ref, rtol=1e-11, atol=1e-14)
    rms = math.sqrt(float(np.mean(ref ** 2)))
    assert 1e-3 < rms < 1.0


# ---------------------------------------------------------------- slicing (Eq. 1-2)
def test_split_counts_golden(oracle):
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "split_counts.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) >= 9
    for H, g, rgg, rcg, rcc, ngg, ncg, ncc in rows:
        n_cc, n_cg, n_gg = oracle.split_counts(int(H), int(g), float(rgg), float(rcg))
        assert (n_gg, n_cg, n_cc) == (int(ngg), int(ncg), int(ncc))
        assert abs(float(rgg) + float(rcg) + float(rcc) - 1.0) < 1e-6


def test_split_counts_invariants(oracle):
    for H, g in [(704, 64), (2560, 64), (6400, 128), (28672, 64), (64, 64)]:
        prev = -1
        for i in range(0, 21):
            rgg = i / 20.0
            for jx in range(0, 21 - i):
                rcg = jx / 20.0
                n_cc, n_cg, n_gg = oracle.split_counts(H, g, rgg, rcg)
                assert n_cc + n_cg + n_gg == H
                assert min(n_cc, n_cg, n_gg) >= 0
                assert n_cc % g == 0 and n_cg % g == 0 and n_gg % g == 0
                assert abs(n_gg - rgg * H) <= g / 2 + 1e-3 and abs(n_gg + n_cg - (rgg + rcg) * H) <= g / 2 + 1e-3
            n_gg_only = oracle.split_counts(H, g, rgg, 0.0)[2]
            assert n_gg_only >= prev  # monotone in the rate
            prev = n_gg_only
    with pytest.raises(ValueError):
        oracle.split_counts(700, 64, 0.5, 0.5)  # granule must divide H
    with pytest.raises(ValueError):
        oracle.split_counts(704, 64, 0.8, 0.5)


def test_split_invariance_dense(oracle):
    cfg = synth.CONFIGS["tiny_dense"]
    w = synth.make_weights(cfg)
    T = 8
    xb = synth.make_tokens(cfg, T)
    y0 = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"])
    scale = np.max(np.abs(y0))
    rates = synth.SPLIT_SWEEP + [(0.0, 1.0, 0.0), (0.0, 0.0, 1.0), (0.4, 0.3, 0.3)]
    for rgg, rcg, rcc in rates:
        n_cc, n_cg, n_gg = oracle.split_counts(cfg.d_ff, 64, rgg, rcg)
        for n_g in (0, 1, T // 2, T):
            y = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"], counts=(n_cc, n_cg), n_g=n_g)
            assert np.max(np.abs(y - y0)) <= 1e-12 * scale


# ---------------------------------------------------------------- routing
def brute_route(logits, k):
    T, E = logits.shape
    idx = np.zeros((T, k), np.int32)
    w = np.zeros((T, k))
    for t in range(T):
        order = sorted(range(E), key=lambda e: (-float(logits[t, e]), e))[:k]
        idx[t] = order
        ex = [math.exp(float(logits[t, e]) - float(logits[t, order[0]])) for e in order]
        w[t] = [v / sum(ex) for v in ex]
    pairs = sorted(range(T * k), key=lambda q: (int(idx.reshape(-1)[q]), q))
    return idx, w, np.array(pairs, np.int32)


def check_routing_invariants(r, T, E, k):
    assert r["idx"].shape == (T, k) and r["idx"].min(initial=0) >= 0 and r["idx"].max(initial=0) < E
    for t in range(T):
        assert len(set(r["idx"][t].tolist())) == k
    assert np.all(r["w"] >= 0) and np.allclose(r["w"].sum(axis=1), 1.0, atol=1e-12)
    assert r["count"].sum() == T * k and r["off"][0] == 0 and r["off"][E] == T * k
    assert np.array_equal(np.diff(r["off"]), r["count"])
    assert np.array_equal(np.bincount(r["idx"].reshape(-1), minlength=E), r["count"])
    assert np.array_equal(np.sort(r["perm"]), np.arange(T * k))
    assert np.array_equal(r["inv"][r["perm"]], np.arange(T * k))
    e_of_pos = r["idx"].reshape(-1)[r["perm"]]
    assert np.all(np.diff(e_of_pos) >= 0)  # expert-sorted
    for e in range(E):
        seg = r["perm"][r["off"][e]:r["off"][e + 1]]
        assert np.all(np.diff(seg) > 0)  # stable inside an expert


def test_route_bruteforce_and_invariants(oracle):
    rng = np.random.default_rng(3)
    for (T, E, k) in [(1, 2, 1), (5, 4, 2), (7, 8, 2), (6, 16, 4), (9, 64, 8), (3, 5, 5)]:
        logits = rng.standard_normal((T, E)).astype(np.float32)
        r = oracle.route(logits, k)
        idx, w, perm = brute_route(logits, k)
        assert np.array_equal(r["idx"], idx)
        assert np.allclose(r["w"], w, rtol=1e-14, atol=0)
        assert np.array_equal(r["perm"], perm)
        check_routing_invariants(r, T, E, k)


def test_route_special_cases(oracle):
    # all-equal logits: experts 0..k-1 in order, weight 1/k each
    r = oracle.route(np.full((4, 8), 0.25, np.float32), 3)
    assert np.array_equal(r["idx"], np.tile(np.arange(3, dtype=np.int32), (4, 1)))
    assert np.allclose(r["w"], 1.0 / 3.0, rtol=1e-15)
    # ties between two experts: the lower index comes first
    lg = np.array([[0.0, 2.0, -1.0, 2.0, 1.0]], np.float32)
    r = oracle.route(lg, 3)
    assert r["idx"].tolist() == [[1, 3, 4]]
    e1 = math.exp(-1.0)
    assert np.allclose(r["w"], [[1 / (2 + e1), 1 / (2 + e1), e1 / (2 + e1)]], rtol=1e-15)
    # one dominant logit takes all the weight
    lg = np.zeros((2, 8), np.float32)
    lg[0, 5] = 40.0
    lg[1, 2] = 40.0
    r = oracle.route(lg, 2)
    assert r["idx"][0, 0] == 5 and r["idx"][1, 0] == 2 and r["idx"][0, 1] == 0 and r["idx"][1, 1] == 0
    assert np.all(np.abs(r["w"][:, 0] - 1.0) < 1e-6)
    # k = E: weights are the full softmax
    rng = np.random.default_rng(0)
    lg = rng.standard_normal((5, 6)).astype(np.float32)
    r = oracle.route(lg, 6)
    sm = np.exp(lg.astype(np.float64) - lg.astype(np.float64).max(axis=1, keepdims=True))
    sm /= sm.sum(axis=1, keepdims=True)
    for t in range(5):
        assert np.allclose(r["w"][t], sm[t, r["idx"][t]], rtol=1e-14)
    # empty batch
    r = oracle.route(np.zeros((0, 4), np.float32), 2)
    assert r["count"].tolist() == [0, 0, 0, 0] and r["off"].tolist() == [0] * 5
    with pytest.raises(ValueError):
        oracle.route(np.array([[0.0, np.nan]], np.float32), 1)
    with pytest.raises(ValueError):
        oracle.route(np.zeros((2, 3), np.float32), 4)


def test_route_zipf_config_shape(oracle):
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128)
    xb = synth.make_tokens(cfg, 512)
    lg = synth.make_router_logits(cfg, xb)
    r = oracle.route(lg, cfg.top_k)
    check_routing_invariants(r, 512, cfg.n_experts, cfg.top_k)
    assert r["count"].max() > 4 * max(1, r["count"].min())  # the Zipf bias skews the load


# ---------------------------------------------------------------- MoE
def np_moe(xv, lg, k, gv, uv, dv, shared=None):
    T = xv.shape[0]
    idx, w, _ = brute_route(lg, k)
    y = np.zeros((T, xv.shape[1]))
    for t in range(T):
        for s in range(k):
            e = idx[t, s]
            y[t] += w[t, s] * np_mlp(xv[t:t + 1], gv[e], uv[e], dv[e])[0]
        if shared is not None:
            y[t] += np_mlp(xv[t:t + 1], *shared)[0]
    return y


def moe_case(rng, T, M, H, E, Hs=0):
    xb, xv = rand_bits(rng, (T, M), 1.0)
    gb, gv = rand_bits(rng, (E, H, M), 0.2)
    ub, uv = rand_bits(rng, (E, H, M), 0.2)
    db, dv = rand_bits(rng, (E, H, M), 0.2)
    lg = rng.standard_normal((T, E)).astype(np.float32)
    sh = shv = None
    if Hs:
        parts = [rand_bits(rng, (Hs, M), 0.2) for _ in range(3)]
        sh = tuple(p[0] for p in parts)
        shv = tuple(p[1] for p in parts)
    return xb, xv, gb, gv, ub, uv, db, dv, lg, sh, shv


def test_moe_matches_numpy_and_bruteforce(oracle):
    rng = np.random.default_rng(21)
    for (T, M, H, E, k, Hs) in [(6, 16, 24, 4, 2, 0), (5, 32, 64, 8, 3, 128), (3, 8, 8, 2, 2, 0)]:
        xb, xv, gb, gv, ub, uv, db, dv, lg, sh, shv = moe_case(rng, T, M, H, E, Hs)
        y = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k, shared=sh)
        ref = np_moe(xv, lg, k, gv, uv, dv, shv)
        assert np.allclose(y, ref, rtol=1e-11, atol=1e-13)
    # fully scalar brute force on the smallest case
    xb, xv, gb, gv, ub, uv, db, dv, lg, _, _ = moe_case(rng, 2, 4, 3, 3, 0)
    idx, w, _ = brute_route(lg, 2)
    ref = np.zeros((2, 4))
    for t in range(2):
        for s in range(2):
            ref[t] += w[t, s] * brute_mlp(xv[t:t + 1], gv[idx[t, s]], uv[idx[t, s]], dv[idx[t, s]])[0]
    assert np.allclose(oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=2), ref, rtol=1e-13, atol=1e-15)


def test_moe_reductions(oracle):
    rng = np.random.default_rng(22)
    T, M, H, E, k = 5, 16, 32, 4, 2
    xb, xv, gb, gv, ub, uv, db, dv, lg, _, _ = moe_case(rng, T, M, H, E)
    # E = 1, k = 1 equals the dense MLP exactly
    y_d = oracle.layer_forward(xb, gb[:1], ub[:1], db[:1])
    y_1 = oracle.layer_forward(xb, gb[:1], ub[:1], db[:1], logits=lg[:, :1], top_k=1)
    assert np.array_equal(y_d, y_1)
    # identical experts: the routing weights sum to 1, so the result is the dense MLP
    same = lambda a: np.repeat(a[:1], E, axis=0)
    y_same = oracle.layer_forward(xb, same(gb), same(ub), same(db), logits=lg, top_k=k)
    assert np.allclose(y_same, y_d, rtol=1e-13, atol=1e-15)
    # relabelling experts together with their logit columns leaves y unchanged
    y = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k)
    p = np.array([2, 0, 3, 1])
    y_p = oracle.layer_forward(xb, gb[p], ub[p], db[p], logits=np.ascontiguousarray(lg[:, p]), top_k=k)
    assert np.allclose(y_p, y, rtol=1e-12, atol=1e-15)


def test_shared_expert_cases(oracle):
    rng = np.random.default_rng(23)
    T, M, H, E, k, Hs = 4, 16, 32, 4, 2, 48
    xb, xv, gb, gv, ub, uv, db, dv, lg, sh, shv = moe_case(rng, T, M, H, E, Hs)
    y_routed = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k)
    zs = tuple(np.zeros((Hs, M), np.uint16) for _ in range(3))
    assert np.array_equal(oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k, shared=zs), y_routed)
    z = np.zeros_like(db)
    y_sh = oracle.layer_forward(xb, gb, ub, z, logits=lg, top_k=k, shared=sh)
    assert np.allclose(y_sh, np_mlp(xv, *shv), rtol=1e-12, atol=1e-15)
    y_both = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k, shared=sh)
    assert np.allclose(y_both, y_routed + y_sh, rtol=1e-12, atol=1e-15)


def test_split_invariance_moe_shared(oracle):
    rng = np.random.default_rng(24)
    T, M, H, E, k, Hs = 6, 16, 256, 4, 2, 512
    xb, xv, gb, gv, ub, uv, db, dv, lg, sh, shv = moe_case(rng, T, M, H, E, Hs)
    y0 = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k, shared=sh)
    scale = np.max(np.abs(y0))
    for rgg, rcg, rcc in synth.SPLIT_SWEEP + [(0.0, 1.0, 0.0), (0.0, 0.0, 1.0)]:
        c = oracle.split_counts(H, 64, rgg, rcg)
        cs = oracle.split_counts(Hs, 64, rgg, rcg)
        for n_g in (0, 1, T // 2, T):
            y = oracle.layer_forward(xb, gb, ub, db, logits=lg, top_k=k, shared=sh, counts=c[:2],
                                     shared_counts=cs[:2], n_g=n_g)
            assert np.max(np.abs(y - y0)) <= 1e-12 * scale


def test_threads_do_not_change_result(oracle):
    cfg = synth.CONFIGS["tiny_dense"]
    w = synth.make_weights(cfg)
    xb = synth.make_tokens(cfg, 4)
    n0 = oracle.get_threads()
    oracle.set_threads(1)
    y1 = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"])
    oracle.set_threads(4)
    y4 = oracle.layer_forward(xb, w["w_gate"], w["w_up"], w["w_down"])
    oracle.set_threads(n0)
    assert np.array_equal(y1, y4)  # each j and each m-block is summed by one thread in the same order


# ------------------------------------------------------------------ layer stack (residual chain)
def test_round_to_bf16_against_bit_arithmetic_and_ties(oracle):
    rng = np.random.default_rng(17)
    v32 = (rng.standard_normal(20000) * np.exp(rng.uniform(-8, 8, 20000))).astype(np.float32)
    # float32 inputs: the integer rounding trick on the bit pattern is an independent implementation
    assert np.array_equal(oracle.round_to_bf16(v32.astype(np.float64)), synth.f32_to_bf16_bits(v32))
    # exact ties go to the even mantissa: 1 + 2^-8 -> 1.0, 1 + 3*2^-8 -> 1 + 2^-6
    assert oracle.round_to_bf16(np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -(1.0 + 2.0 ** -8)])).tolist() == \
        [0x3F80, 0x3F82, 0xBF80]
    # a float64 just above a tie rounds up although its float32 rounding would sit on the tie
    assert oracle.round_to_bf16(np.array([1.0 + 2.0 ** -8 + 2.0 ** -40])).tolist() == [0x3F81]
    # representable values are fixed points
    b = np.arange(0x3F00, 0x4100, dtype=np.uint16)
    assert np.array_equal(oracle.round_to_bf16(oracle.bf16_to_f64(b)), b)


def test_stack_reduces_to_layers(oracle):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=64, d_ff=128, n_experts=4)
    w = synth.make_weights(cfg)
    xb = synth.make_tokens(cfg, 5)
    lg = synth.make_router_logits(cfg, xb)
    kw = dict(w_gate=w["w_gate"], w_up=w["w_up"], w_down=w["w_down"], logits=lg, top_k=cfg.top_k)
    x64 = synth.bf16_bits_to_f64(xb)
    y0 = oracle.layer_forward(xb, **kw)
    # one layer: the residual sum, nothing rounded
    assert np.array_equal(oracle.stack_forward(xb, [kw]), x64 + y0)
    # two layers written out by hand
    x1 = synth.f32_to_bf16_bits((x64 + y0).astype(np.float32))   # float32 first: differs from direct rounding only on double-rounding ties
    x1d = oracle.round_to_bf16(x64 + y0)
    assert np.mean(x1 != x1d) < 1e-3
    h2 = synth.bf16_bits_to_f64(x1d) + oracle.layer_forward(x1d, **kw)
    assert np.array_equal(oracle.stack_forward(xb, [kw, kw]), h2)
    # a layer with zero down projection passes the hidden state through unchanged
    kz = dict(kw, w_down=np.zeros_like(w["w_down"]))
    assert np.array_equal(oracle.stack_forward(xb, [kz, kz, kz]), x64)


# ------------------------------------------------------------------ 4-bit weight storage
def _dequant_numpy(q, z, kind):
    """Independent vectorised reading of the storage form: q [.., H, M/2] -> values [.., H, M] in float64."""
    lo = (q & 0x0F).astype(np.float64) - 8.0
    hi = (q >> 4).astype(np.float64) - 8.0
    v = np.stack([lo, hi], axis=-1).reshape(q.shape[:-1] + (q.shape[-1] * 2,))
    zf = synth.bf16_bits_to_f64(z)
    if kind == "fc1":
        return v * np.repeat(zf, 64, axis=-1)
    return v * np.repeat(zf, 64, axis=-2)


def test_q4_values_against_numpy_reading(oracle):
    cfg = synth.scaled(synth.CONFIGS["mixtral_8x7b"], d_model=128, d_ff=192, n_experts=2)
    wq = synth.make_weights_q4(cfg)
    assert wq["q_gate"].shape == (2, 192, 64) and wq["z_gate"].shape == (2, 192, 2) and wq["z_down"].shape == (2, 3, 128)
    codes = np.concatenate([wq["q_gate"] & 15, wq["q_gate"] >> 4]).ravel()
    assert codes.min() == 0 and codes.max() == 15 and abs(codes.mean() - 8.0) < 0.1     # bell shape around 8
    rng = np.random.default_rng(2)
    for which, (qk, zk, kind) in enumerate((("q_gate", "z_gate", "fc1"), ("q_up", "z_up", "fc1"), ("q_down", "z_down", "fc2"))):
        full = _dequant_numpy(wq[qk][1], wq[zk][1], kind)
        for _ in range(300):
            j, m = int(rng.integers(192)), int(rng.integers(128))
            assert oracle.q4_value(wq[qk][1], wq[zk][1], 128, which, j, m) == full[j, m]
    # hand-made bytes: 0x3A holds code 10 (even m) and code 3 (odd m); scale 0.5 -> +1.0 and -2.5
    q = np.zeros((64, 32), np.uint8)
    q[5, 7] = 0x3A
    z = synth.f32_to_bf16_bits(np.full((64, 1), 0.5, np.float32))
    assert oracle.q4_value(q, z, 64, 0, 5, 14) == 1.0 and oracle.q4_value(q, z, 64, 0, 5, 15) == -2.5
    assert oracle.q4_value(q, z, 64, 0, 5, 13) == -4.0                                     # code 0 -> -8 * 0.5
    zd = synth.f32_to_bf16_bits(np.full((1, 64), 0.25, np.float32))
    assert oracle.q4_value(q, zd, 64, 2, 5, 14) == 0.5


def test_q4_layer_equals_bf16_layer_when_values_are_representable(oracle):
    """Power-of-two scales make every (code - 8) * scale exactly a bfloat16: the 4-bit layer must then give the
    bit-identical result of the bf16 layer on those values (pins nibble order, both scale groupings, the offset
    8, expert and shared-expert addressing, slicing and token split)."""
    cfg = synth.scaled(synth.CONFIGS["qwen_moe"], d_model=128, d_ff=192, d_ff_shared=128, n_experts=6, top_k=3)
    wq = synth.make_weights_q4(cfg)
    rng = np.random.default_rng(3)
    for k in list(wq):
        if k.startswith(("z_", "sz_")):
            wq[k] = synth.f32_to_bf16_bits((2.0 ** rng.integers(-9, -4, size=wq[k].shape)).astype(np.float32))
    deq = {}
    for name, qk, zk, kind in (("w_gate", "q_gate", "z_gate", "fc1"), ("w_up", "q_up", "z_up", "fc1"), ("w_down", "q_down", "z_down", "fc2"),
                               ("s_gate", "sq_gate", "sz_gate", "fc1"), ("s_up", "sq_up", "sz_up", "fc1"), ("s_down", "sq_down", "sz_down", "fc2")):
        v = _dequant_numpy(wq[qk], wq[zk], kind)
        bits = synth.f32_to_bf16_bits(v.astype(np.float32))
        assert np.array_equal(synth.bf16_bits_to_f64(bits), v)     # representable, as constructed
        deq[name] = bits
    xb = synth.make_tokens(cfg, 9)
    lg = synth.make_router_logits(cfg, xb)
    shared = (deq["s_gate"], deq["s_up"], deq["s_down"])
    for counts, sc, n_g in (((0, 0), (0, 0), 0), ((64, 64), (64, 0), 4), ((128, 0), (0, 64), 9)):
        a = oracle.layer_forward_q4(xb, wq, logits=lg, top_k=3, counts=counts, shared_counts=sc, n_g=n_g)
        b = oracle.layer_forward(xb, deq["w_gate"], deq["w_up"], deq["w_down"], logits=lg, top_k=3, shared=shared,
                                 counts=counts, shared_counts=sc, n_g=n_g)
        assert np.array_equal(a, b)
    sel = np.array([8, 0, 3], np.int32)
    assert np.array_equal(oracle.layer_forward_q4(xb, wq, logits=lg, top_k=3, sel=sel),
                          oracle.layer_forward_q4(xb, wq, logits=lg, top_k=3)[sel])


def test_q4_layer_against_numpy_matmul(oracle):
    """General scales (not representable in bf16 after multiplication): float64 matmul on the numpy reading."""
    cfg = synth.scaled(synth.CONFIGS["llama2_70b"], d_model=64, d_ff=128)
    wq = synth.make_weights_q4(cfg)
    xb = synth.make_tokens(cfg, 4)
    x = synth.bf16_bits_to_f64(xb)
    Wg = _dequant_numpy(wq["q_gate"][0], wq["z_gate"][0], "fc1")
    Wu = _dequant_numpy(wq["q_up"][0], wq["z_up"][0], "fc1")
    Wd = _dequant_numpy(wq["q_down"][0], wq["z_down"][0], "fc2")
    g = x @ Wg.T
    ref = ((g / (1.0 + np.exp(-g))) * (x @ Wu.T)) @ Wd
    got = oracle.layer_forward_q4(xb, wq)
    assert np.allclose(got, ref, rtol=1e-11, atol=1e-13)
    assert np.std(Wg) == pytest.approx(cfg.w_std, rel=0.15)
