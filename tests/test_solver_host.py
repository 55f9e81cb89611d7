"""The library's Solver (host arithmetic behind the C ABI, include/scheinfer_solver.h) against the
oracle on the same inputs: fit, Eq. 4 / Eq. 15 task times, Eq. 6 recurrence, the r_CG and n_g solves,
the greedy memory assignment, and the argument checks.  No GPU is needed."""
import numpy as np
import pytest

import paper_2411_15715_amd as si
from oracle import solver_oracle as so
from test_solver_oracle_pins import TABLE_I, golden_cases, random_instances

REL = 1e-12


def test_fit_matches_oracle():
    rng = np.random.default_rng(1)
    for _ in range(50):
        k = int(rng.integers(2, 13))
        n = np.sort(np.exp(rng.uniform(10, 22, k))) + np.arange(k)
        t = 1e-6 * rng.uniform(0, 50) + n * 1e-11 * rng.uniform(0.1, 10) * (1 + 0.1 * rng.standard_normal(k))
        a, b, r2 = si.si_fit_linear(n, t)
        ao, bo, r2o = so.fit_linear(n, t)
        assert a == pytest.approx(ao, rel=1e-7, abs=1e-12) and b == pytest.approx(bo, rel=1e-8) and r2 == pytest.approx(r2o, abs=1e-8)


def test_fit_nonneg_is_the_constrained_optimum():
    # a line through points that forces a negative intercept; the constrained fit must beat every other
    # (alpha >= 0, beta) pair on a grid around it
    n = np.array([1.0, 2.0, 3.0, 4.0, 5.0])
    t = np.array([0.0, 0.9, 2.1, 3.0, 4.2])
    a0, _, _ = si.si_fit_linear(n, t)
    assert a0 < 0
    a, b, r2 = si.si_fit_linear(n, t, nonneg=True)
    assert a == 0.0 and b == pytest.approx(float(n @ t) / float(n @ n), rel=1e-14)
    sse = lambda aa, bb: float(np.sum((t - aa - bb * n) ** 2))
    for aa in np.linspace(0, 0.5, 11):
        for bb in np.linspace(b - 0.2, b + 0.2, 41):
            assert sse(a, b) <= sse(aa, bb) + 1e-15
    assert r2 == pytest.approx(1.0 - sse(a, b) / float(np.sum((t - t.mean()) ** 2)), rel=1e-12)
    # where the plain fit is already non-negative the flag changes nothing
    t2 = 3.0 + 2.0 * n
    assert si.si_fit_linear(n, t2, nonneg=True) == pytest.approx(si.si_fit_linear(n, t2), rel=1e-14)


@pytest.mark.parametrize("case", golden_cases())
def test_worked_examples(case):
    T, M, H, n_l, r_gg, r_cg, times, t_fin, which = case
    m = TABLE_I["A_fp16"]
    got = si.si_model_times(m, float(T) * M * H, 2.0 * M * H, n_l, r_gg, r_cg)
    assert (got["t_g"], got["t_c"], got["t_c2g"], got["t_l"]) == pytest.approx(tuple(times), rel=1e-12, abs=1e-18)
    assert si.si_simulate(got, n_l)["t_fin"] == pytest.approx(t_fin, rel=1e-12)
    sol = si.si_solve_split(m, float(T) * M * H, 2.0 * M * H, n_l, r_gg)
    assert sol["t_fin"] <= t_fin * (1 + 1e-12)


def test_times_and_recurrence_match_oracle():
    rng = np.random.default_rng(2)
    for m, T, M, H, n_l, r_gg in random_instances(51, 200):
        r_cg = float(rng.choice([0.0, 1.0 - r_gg, (1.0 - r_gg) * rng.random()]))
        n_gemm, n_w = float(T) * M * H, 2.0 * M * H
        got = si.si_model_times(m, n_gemm, n_w, n_l, r_gg, r_cg)
        want = so.task_times(m, n_gemm, n_w, r_gg, r_cg)
        assert (got["t_g"], got["t_c"], got["t_c2g"], got["t_l"]) == pytest.approx(want, rel=REL, abs=0.0)
        sim = si.si_simulate(got, n_l)
        t_fin, tau = so.simulate(*want, n_l)
        assert sim["t_fin"] == pytest.approx(t_fin, rel=REL)
        assert sim["tau_g"] == pytest.approx(tau["G"][n_l], rel=REL, abs=0.0)
        assert sim["tau_c"] == pytest.approx(tau["C"][n_l], rel=REL, abs=0.0)
        n_g = int(rng.integers(0, T + 1))
        got = si.si_model_times_ng(m, T, M, H, n_w, r_gg, r_cg, n_g)
        want = so.task_times_ng(m, T, M, H, n_w, r_gg, r_cg, n_g)
        assert (got["t_g"], got["t_c"], got["t_c2g"], got["t_l"]) == pytest.approx(want, rel=REL, abs=0.0)


def test_solve_split_matches_oracle():
    cases = set()
    for m, T, M, H, n_l, r_gg in random_instances(61, 400):
        n_gemm, n_w = float(T) * M * H, 2.0 * M * H
        got = si.si_solve_split(m, n_gemm, n_w, n_l, r_gg)
        want = so.solve_split(m, n_gemm, n_w, n_l, r_gg)
        assert got["t_fin"] == pytest.approx(want["t_fin"], rel=1e-11)
        # the minimiser may be one of several equal points: compare it through the oracle's layer time
        assert so.t_fin(m, n_gemm, n_w, n_l, r_gg, got["r_cg"]) == pytest.approx(want["t_fin"], rel=1e-11)
        assert 0.0 <= got["r_cg"] <= 1.0 - r_gg and got["r_cc"] == pytest.approx(1.0 - r_gg - got["r_cg"], abs=1e-15)
        t = so.task_times(m, n_gemm, n_w, r_gg, got["r_cg"])
        assert got["case"] == so.which_case(t[0], t[2], t[3])
        cases.add(got["case"])
        assert len(got["X"]) == len(got["Y"]) >= (1 if r_gg == 1.0 else 2)
    assert cases == {1, 2, 3}


def test_solve_split_on_the_granule_grid():
    """r_step > 0: the answer must be the best multiple of r_step (or the right end), by exhaustive search
    over the grid with the oracle's layer time."""
    for m, T, M, H, n_l, r_gg in random_instances(71, 150):
        if H < 1024:
            continue
        n_gemm, n_w = float(T) * M * H, 2.0 * M * H
        step = 64.0 / H
        R = 1.0 - r_gg
        got = si.si_solve_split(m, n_gemm, n_w, n_l, r_gg, r_step=step)
        grid = [k * step for k in range(int(np.floor(R / step + 1e-9)) + 1) if k * step < R] + [R]
        vals = [so.t_fin(m, n_gemm, n_w, n_l, r_gg, r) for r in grid]
        assert got["t_fin"] == pytest.approx(min(vals), rel=1e-11), (m, T, M, H, n_l, r_gg)
        k = got["r_cg"] / step
        assert got["r_cg"] == R or abs(k - round(k)) < 1e-9


def test_solve_ng_matches_oracle():
    for m, T, M, H, n_l, r_gg in random_instances(81, 300):
        T = min(T, 600)
        for r_cg in (0.0, (1.0 - r_gg) * 0.5):
            n_w = 2.0 * M * H
            got = si.si_solve_ng(m, T, M, H, n_w, n_l, r_gg, r_cg)
            want = so.solve_ng(m, T, M, H, n_w, n_l, r_gg, r_cg)
            assert got["t_fin"] == pytest.approx(want["t_fin"], rel=1e-11)
            assert so.t_fin_ng(m, T, M, H, n_w, n_l, r_gg, r_cg, got["n_g"]) == pytest.approx(want["t_fin"], rel=1e-11)
            if got["n_g"] != want["n_g"]:   # equal minima up to rounding: both must be optimal
                assert so.t_fin_ng(m, T, M, H, n_w, n_l, r_gg, r_cg, want["n_g"]) == pytest.approx(got["t_fin"], rel=1e-11)


def test_greedy_memory_matches_oracle():
    rng = np.random.default_rng(9)
    assert si.si_assign_gpu_memory([[10.0, 6.0, 5.0], [10.0, 9.0, 4.0]], [10.0, 10.0], 15.0) == [1, 2]
    for _ in range(200):
        n_layers, n_G = int(rng.integers(1, 6)), int(rng.integers(1, 9))
        t_star = np.sort(rng.uniform(1.0, 5.0, (n_layers, n_G + 1)), axis=1)[:, ::-1] + rng.uniform(-0.3, 0.3, (n_layers, n_G + 1))
        n_m = rng.uniform(1.0, 4.0, n_layers)
        budget = float(rng.uniform(0.0, n_m.sum() * 1.1))
        assert si.si_assign_gpu_memory(t_star, n_m, budget) == so.greedy_memory(t_star.tolist(), n_m.tolist(), budget)


def test_end_to_end_split_then_memory():
    """Two-stage algorithm of Section IV-A: t_fin*(r_GG = i/n_G) from the first stage feeds the greedy second
    stage; library and oracle must agree on the whole chain."""
    m = TABLE_I["A_fp16"]
    layers = [(4096, 14336), (4096, 14336), (8192, 28672)]
    n_G = 8
    t_lib, t_or, n_m = [], [], []
    for M, H in layers:
        n_gemm, n_w = float(M) * H, 2.0 * M * H
        t_lib.append([si.si_solve_split(m, n_gemm, n_w, 3, i / n_G)["t_fin"] for i in range(n_G + 1)])
        t_or.append([so.solve_split(m, n_gemm, n_w, 3, i / n_G)["t_fin"] for i in range(n_G + 1)])
        n_m.append(3 * n_w)
    assert np.allclose(t_lib, t_or, rtol=1e-11, atol=0)
    for frac in (0.0, 0.2, 0.5, 0.9, 1.0):
        budget = frac * sum(n_m)
        assert si.si_assign_gpu_memory(t_lib, n_m, budget) == so.greedy_memory(t_or, n_m, budget)
    # nothing resident is the slowest choice (Section IV-A.4 notes that the fastest need not be r_GG = 1)
    assert all(t[0] == max(t) for t in t_lib)


def test_argument_checks():
    m = dict(TABLE_I["A_fp16"])
    for bad in (lambda: si.si_fit_linear([1.0], [1.0]),
                lambda: si.si_fit_linear([2.0, 2.0], [1.0, 3.0]),
                lambda: si.si_fit_linear([1.0, 2.0], [1.0, float("nan")]),
                lambda: si.si_model_times(m, 1e6, 2e6, 2, 0.7, 0.4),
                lambda: si.si_model_times(m, 1e6, 2e6, 0, 0.5, 0.4),
                lambda: si.si_model_times(dict(m, beta_c=-1.0), 1e6, 2e6, 2, 0.5, 0.4),
                lambda: si.si_simulate({"t_g": 1.0, "t_c": 1.0, "t_c2g": 1.0, "t_l": 1.0}, 0),
                lambda: si.si_simulate({"t_g": -1.0, "t_c": 1.0, "t_c2g": 1.0, "t_l": 1.0}, 2),
                lambda: si.si_solve_split(m, 1e6, 2e6, 2, 1.5),
                lambda: si.si_solve_split(m, 1e6, 2e6, 2, 0.5, r_step=-0.1),
                lambda: si.si_model_times_ng(m, 10, 64, 64, 8192.0, 0.5, 0.25, 11),
                lambda: si.si_solve_ng(m, 10, 64, 64, 8192.0, 0, 0.5, 0.25),
                lambda: si.si_assign_gpu_memory([[1.0, 0.5]], [0.0], 1.0),
                lambda: si.si_assign_gpu_memory([[1.0, 0.5]], [1.0], -1.0)):
        with pytest.raises(si.ScheInferError) as ei:
            bad()
        assert ei.value.code == si.SI_EINVAL and str(ei.value)


def test_profile_rejects_bad_arguments_before_any_gpu_call():
    for kw in (dict(d_model=100, d_ff=1024, tokens=4), dict(d_model=128, d_ff=64, tokens=4),
               dict(d_model=128, d_ff=1024, tokens=0), dict(d_model=128, d_ff=1024, tokens=64, mode=si.SI_DECODE),
               dict(d_model=128, d_ff=1024, tokens=4, n_sizes=40)):
        with pytest.raises(si.ScheInferError) as ei:
            si.si_profile(**kw)
        assert ei.value.code == si.SI_EINVAL


def test_place_experts_hand_worked_examples():
    """Oracle and library against placements worked by hand (ties, the share hit exactly, the share missed by one
    expert, the extremes): a wrong tie order or a wrong acceptance rule fails here."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "place_experts.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and ln[0] != "#"]
    assert len(rows) >= 6
    for freq, n_gg, share, want in rows:
        freq = [float(v) for v in freq.split(",")]
        want = [int(v) for v in want.split(",")]
        assert so.place_experts(freq, int(n_gg), float(share)) == want, freq
        assert si.si_place_experts(np.array(freq), int(n_gg), float(share)) == want, freq


def test_place_experts_matches_oracle_and_its_contract():
    rng = np.random.default_rng(12)
    for _ in range(200):
        E = int(rng.integers(1, 65))
        freq = rng.zipf(1.5, E).astype(np.float64) if rng.random() < 0.5 else rng.random(E)
        if rng.random() < 0.3:
            freq = np.round(freq, 1)          # ties
        n_gg = int(rng.integers(0, E + 1))
        share = float(rng.choice([0.0, 0.25, 0.5, 0.8, 1.0]))
        got = si.si_place_experts(freq, n_gg, share)
        assert got == so.place_experts(freq.tolist(), n_gg, share)
        # contract: exactly n_gg resident experts and none of the others is more frequent than any of them
        gg = [e for e in range(E) if got[e] == 0]
        rest = [e for e in range(E) if got[e] != 0]
        assert len(gg) == n_gg
        if gg and rest:
            assert min(freq[e] for e in gg) >= max(freq[e] for e in rest)
        # CG's share of the streamed-or-host frequency mass never exceeds cg_share
        mass = sum(freq[e] for e in rest)
        if mass > 0:
            assert sum(freq[e] for e in rest if got[e] == 1) <= share * mass + 1e-12
        if share == 0.0:
            assert all(got[e] == 2 for e in rest if freq[e] > 0)
    with pytest.raises(si.ScheInferError):
        si.si_place_experts([1.0, 2.0], 3, 0.5)
    with pytest.raises(si.ScheInferError):
        si.si_place_experts([1.0, -2.0], 1, 0.5)
