"""Pins of the Profiler & Solver oracle (oracle/solver_oracle.py) to things other than itself:
hand-worked values from the paper's Table I coefficients, a library regression routine, path
enumeration on the task graph, brute-force search over the decision variable, limiting cases."""
import os

import numpy as np
import pytest

from oracle import solver_oracle as so

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "eq6_worked_examples.txt")

# Table I, Testbed A / B / C (seconds); "fp16" and "int4" are the two GEMM column pairs
TABLE_I = {
    "A_fp16": dict(alpha_g=1.0e-7, beta_g=3.2e-12, alpha_c=7.4e-7, beta_c=1.6e-11, alpha_c2g=3.0e-6, beta_c2g=2.6e-11, t_launch=4.4e-5),
    "A_int4": dict(alpha_g=4.7e-6, beta_g=8.1e-13, alpha_c=1.1e-5, beta_c=5.4e-12, alpha_c2g=3.0e-6, beta_c2g=2.6e-11, t_launch=4.4e-5),
    "B_fp16": dict(alpha_g=1.9e-7, beta_g=2.6e-12, alpha_c=3.4e-6, beta_c=1.5e-11, alpha_c2g=5.8e-6, beta_c2g=2.5e-11, t_launch=5.7e-5),
    "B_int4": dict(alpha_g=4.6e-6, beta_g=6.5e-13, alpha_c=1.3e-5, beta_c=6.5e-12, alpha_c2g=5.8e-6, beta_c2g=2.5e-11, t_launch=5.7e-5),
    "C_fp16": dict(alpha_g=1.4e-7, beta_g=3.6e-12, alpha_c=1.8e-6, beta_c=2.5e-11, alpha_c2g=3.7e-6, beta_c2g=4.1e-11, t_launch=5.2e-5),
    "C_int4": dict(alpha_g=6.4e-6, beta_g=9.2e-13, alpha_c=5.6e-7, beta_c=8.4e-12, alpha_c2g=3.7e-6, beta_c2g=4.1e-11, t_launch=5.2e-5),
}


def golden_cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        a, b, c, d = [p.split() for p in line.split("|")]
        out.append((int(a[0]), int(a[1]), int(a[2]), int(a[3]), float(a[4]), float(a[5]),
                    [float(v) for v in b], float(c[0]), int(d[0])))
    return out


# ------------------------------------------------------------------ Eq. 3: fitting
def test_fit_recovers_a_line_exactly():
    n = np.array([1e6, 3e6, 1e7, 5e7, 2e8])
    a, b, r2 = so.fit_linear(n, 4.4e-5 + 3.2e-12 * n)
    assert a == pytest.approx(4.4e-5, rel=1e-9) and b == pytest.approx(3.2e-12, rel=1e-9) and r2 == pytest.approx(1.0, abs=1e-12)


def test_fit_against_library_regression():
    from scipy import stats
    rng = np.random.default_rng(3)
    n = np.geomspace(1e5, 1e9, 23)
    t = 2.0e-6 + 2.6e-11 * n * (1.0 + 0.08 * rng.standard_normal(n.size)) + 1e-6 * rng.standard_normal(n.size)
    a, b, r2 = so.fit_linear(n, t)
    ref = stats.linregress(n, t)
    assert a == pytest.approx(ref.intercept, rel=1e-8, abs=1e-15)
    assert b == pytest.approx(ref.slope, rel=1e-10)
    assert r2 == pytest.approx(ref.rvalue ** 2, rel=1e-10)
    assert 0.9 < r2 < 1.0


def test_fit_r2_of_pure_noise_is_small():
    rng = np.random.default_rng(4)
    n = np.linspace(1.0, 100.0, 400)
    _, _, r2 = so.fit_linear(n, rng.standard_normal(n.size))
    assert abs(r2) < 0.05


# ------------------------------------------------------------------ Eq. 4 + Eq. 6: worked examples
@pytest.mark.parametrize("case", golden_cases())
def test_worked_examples(case):
    T, M, H, n_l, r_gg, r_cg, times, t_fin, which = case
    m = TABLE_I["A_fp16"]
    got = so.task_times(m, float(T) * M * H, 2.0 * M * H, r_gg, r_cg)
    assert got == pytest.approx(tuple(times), rel=1e-12, abs=1e-18)
    assert so.simulate(*got, n_l)[0] == pytest.approx(t_fin, rel=1e-12)
    assert so.t_fin(m, float(T) * M * H, 2.0 * M * H, n_l, r_gg, r_cg) == pytest.approx(t_fin, rel=1e-12)
    assert so.which_case(got[0], got[2], got[3]) == which


def test_task_times_sign_terms():
    m = TABLE_I["B_fp16"]
    n, w = 1e8, 2e8
    # nothing streamed: no copy, no copy launch; only the resident part is launched
    t_g, t_c, t_c2g, t_l = so.task_times(m, n, w, 0.5, 0.0)
    assert t_c2g == 0.0 and t_l == m["t_launch"]
    assert t_g == pytest.approx(m["alpha_g"] + 0.5 * n * m["beta_g"], rel=1e-14)
    assert t_c == pytest.approx(m["alpha_c"] + 0.5 * n * m["beta_c"], rel=1e-14)
    # everything on the CPU
    assert so.task_times(m, n, w, 0.0, 0.0) == pytest.approx((0.0, m["alpha_c"] + n * m["beta_c"], 0.0, 0.0), rel=1e-14)
    # everything streamed: CPU idle, two launches (copy + kernel)
    t_g, t_c, t_c2g, t_l = so.task_times(m, n, w, 0.0, 1.0)
    assert t_c == 0.0 and t_l == 2 * m["t_launch"] and t_c2g == pytest.approx(m["alpha_c2g"] + w * m["beta_c2g"], rel=1e-14)


# ------------------------------------------------------------------ Eq. 6: recurrence vs the task graph
def longest_path(t_g, t_c2g, t_l, n_l):
    """Finish time of the last GPU task by enumerating every chain launch_1..launch_a -> copy_a..copy_b ->
    gemm_b..gemm_{n_l} of the dependency graph the recurrence describes."""
    best = 0.0
    for a in range(1, n_l + 1):
        for b in range(a, n_l + 1):
            best = max(best, a * t_l + (b - a + 1) * t_c2g + (n_l - b + 1) * t_g)
    return best


def test_recurrence_equals_critical_path():
    rng = np.random.default_rng(11)
    for _ in range(300):
        t_g, t_c, t_c2g, t_l = np.exp(rng.uniform(-14, -4, 4))
        n_l = int(rng.integers(1, 9))
        t_fin, tau = so.simulate(t_g, t_c, t_c2g, t_l, n_l)
        assert tau["G"][n_l] == pytest.approx(longest_path(t_g, t_c2g, t_l, n_l), rel=1e-13)
        assert tau["C"][n_l] == pytest.approx(n_l * t_c, rel=1e-13)
        assert t_fin == max(tau["G"][n_l], tau["C"][n_l])
        # the three closed forms of Section IV-A.3: each is a chain, so a lower bound, and the case the
        # conditions Q1-Q3 select is attained
        forms = {1: t_l + n_l * t_c2g + t_g, 2: t_l + t_c2g + n_l * t_g, 3: n_l * t_l + t_c2g + t_g}
        assert tau["G"][n_l] == pytest.approx(max(forms.values()), rel=1e-13)
        assert forms[so.which_case(t_g, t_c2g, t_l)] == pytest.approx(tau["G"][n_l], rel=1e-13)


def test_recurrence_limits():
    assert so.simulate(2.0, 0.0, 0.0, 0.0, 5)[0] == 10.0          # only GPU work: serial GEMMs
    assert so.simulate(0.0, 3.0, 0.0, 0.0, 4)[0] == 12.0          # only CPU work
    assert so.simulate(1.0, 0.5, 2.0, 0.25, 1)[0] == 3.25         # one GEMM: launch, copy, compute in a row
    t_fin, tau = so.simulate(1.0, 0.0, 5.0, 0.1, 3)               # copies back to back, last GEMM after the last copy
    assert tau["C2G"] == pytest.approx([0.0, 5.1, 10.1, 15.1]) and t_fin == pytest.approx(16.1)
    assert tau["L"] == pytest.approx([0.0, 0.1, 0.2, 0.3])


# ------------------------------------------------------------------ Eq. 13: edge points vs brute force
def random_instances(seed, count):
    rng = np.random.default_rng(seed)
    names = sorted(TABLE_I)
    for i in range(count):
        m = dict(TABLE_I[names[i % len(names)]])
        # spread the regimes: scale single coefficients by up to 100x either way
        for key in m:
            if rng.random() < 0.5:
                m[key] *= float(np.exp(rng.uniform(-4.6, 4.6)))
        T = int(rng.choice([1, 1, 2, 8, 64, 512, 4096]))
        M = int(rng.choice([64, 512, 4096, 8192]))
        H = int(rng.choice([64, 1024, 14336, 28672]))
        n_l = int(rng.integers(1, 7))
        r_gg = float(rng.choice([0.0, 0.0, 0.125, 0.5, 0.75, 1.0]))
        yield m, T, M, H, n_l, r_gg


def test_solve_split_equals_grid_search():
    kinds = set()
    for m, T, M, H, n_l, r_gg in random_instances(21, 400):
        n_gemm, n_w = float(T) * M * H, 2.0 * M * H
        sol = so.solve_split(m, n_gemm, n_w, n_l, r_gg)
        R = 1.0 - r_gg
        grid = np.linspace(0.0, R, 4001)
        vals = np.array([so.t_fin(m, n_gemm, n_w, n_l, r_gg, float(r)) for r in grid])
        lo = float(vals.min())
        slope = n_l * (n_w * m["beta_c2g"] + n_gemm * (m["beta_g"] + m["beta_c"]))
        assert sol["t_fin"] <= lo * (1 + 1e-12), (m, T, M, H, n_l, r_gg, sol, lo)
        assert sol["t_fin"] >= lo - slope * (R / 4000) - 1e-18
        assert 0.0 <= sol["r_cg"] <= R
        assert so.t_fin(m, n_gemm, n_w, n_l, r_gg, sol["r_cg"]) == sol["t_fin"]
        kinds.add("end" if sol["r_cg"] in (0.0, R) else "interior")
    assert kinds == {"end", "interior"}


def test_solve_split_known_optima():
    # CPU very slow -> stream (all but a sliver of) what is not resident; link very slow -> stream nothing
    m = dict(TABLE_I["A_fp16"], beta_c=1.0)
    assert so.solve_split(m, 1e8, 2e8, 2, 0.25)["r_cg"] == pytest.approx(0.75, abs=1e-6)
    m = dict(TABLE_I["A_fp16"], beta_c2g=1.0)
    assert so.solve_split(m, 1e8, 2e8, 2, 0.25)["r_cg"] == pytest.approx(0.0, abs=1e-9)
    # no start-up costs, no launch cost, GPU infinitely fast: copy and CPU finish together,
    # r*W = (1-r)*C  =>  r = C/(W+C)
    m = dict(alpha_g=0.0, beta_g=0.0, alpha_c=0.0, beta_c=3e-11, alpha_c2g=0.0, beta_c2g=1e-11, t_launch=0.0)
    sol = so.solve_split(m, 1e8, 2e8, 3, 0.0)
    assert sol["r_cg"] == pytest.approx(3e-3 / (2e-3 + 3e-3), rel=1e-12)
    assert sol["t_fin"] == pytest.approx(3 * 2e-3 * 0.6, rel=1e-12)


def test_optimal_r_cg_grows_as_the_cpu_slows():
    """Section V-E.2 (ablation on slicing rates): with r_GG = 0 the best r_CG rises as CPU threads are
    taken away (0.18 / 0.25 / 0.42 / 0.71 for 16 / 8 / 4 / 2 threads); the per-thread-count coefficients
    are not printed, so only the direction is pinned."""
    M, H = 8192, 28672
    base = TABLE_I["A_int4"]
    prev = -1.0
    rs = []
    for slow in (1.0, 2.0, 4.0, 8.0):
        m = dict(base, beta_c=base["beta_c"] * slow)
        r = so.solve_split(m, float(M) * H, 0.5 * M * H, 2, 0.0)["r_cg"]
        assert r >= prev
        prev = r
        rs.append(r)
    assert rs[-1] > rs[0] + 0.2 and 0.0 < rs[0] < rs[-1] < 1.0


# ------------------------------------------------------------------ Eq. 15: token assignment
def test_ng_zero_reduces_to_eq4():
    for m, T, M, H, n_l, r_gg in random_instances(31, 60):
        r_cg = (1.0 - r_gg) * 0.4
        assert so.task_times_ng(m, T, M, H, 2.0 * M * H, r_gg, r_cg, 0) == \
            pytest.approx(so.task_times(m, float(T) * M * H, 2.0 * M * H, r_gg, r_cg), rel=1e-13, abs=0.0)


def test_ng_all_tokens_on_gpu_idles_the_cpu():
    m = TABLE_I["C_fp16"]
    T, M, H = 256, 4096, 14336
    t_g, t_c, t_c2g, t_l = so.task_times_ng(m, T, M, H, 2.0 * M * H, 0.25, 0.25, T)
    assert t_c == 0.0
    assert t_c2g == pytest.approx(2 * m["alpha_c2g"] + 0.75 * 2.0 * M * H * m["beta_c2g"], rel=1e-13)
    assert t_g == pytest.approx(3 * m["alpha_g"] + T * M * H * m["beta_g"], rel=1e-13)
    assert t_l == pytest.approx(5 * m["t_launch"], rel=1e-13)


def test_solve_ng_equals_exhaustive_search():
    seen = set()
    for m, T, M, H, n_l, r_gg in random_instances(41, 250):
        T = min(T, 600)
        for r_cg in (0.0, (1.0 - r_gg) * 0.5):
            n_w = 2.0 * M * H
            sol = so.solve_ng(m, T, M, H, n_w, n_l, r_gg, r_cg)
            vals = [so.t_fin_ng(m, T, M, H, n_w, n_l, r_gg, r_cg, n) for n in range(T + 1)]
            best = int(np.argmin(vals))
            assert sol["t_fin"] == vals[best]
            assert sol["n_g"] == best
            seen.add("0" if best == 0 else "T" if best == T else "mid")
    assert seen == {"0", "T", "mid"}


# ------------------------------------------------------------------ Eq. 14: greedy GPU memory assignment
def test_greedy_memory_hand_example():
    # importance values worked by hand: layer 0 gains 4 then 1 per half, layer 1 gains 1 then 5
    t_star = [[10.0, 6.0, 5.0], [10.0, 9.0, 4.0]]
    n_m = [10.0, 10.0]
    assert so.greedy_memory(t_star, n_m, 20.0) == [2, 2]   # 0.8 -> layer 0 half; 0.6 -> layer 1 full; 0.2 -> layer 0 full
    assert so.greedy_memory(t_star, n_m, 15.0) == [1, 2]
    assert so.greedy_memory(t_star, n_m, 9.0) == [1, 0]    # after layer 0's first half nothing else fits
    assert so.greedy_memory(t_star, n_m, 4.0) == [0, 0]


def test_greedy_memory_invariants():
    rng = np.random.default_rng(8)
    for _ in range(100):
        n_layers, n_G = int(rng.integers(1, 5)), int(rng.integers(1, 6))
        t_star = [list(np.sort(rng.uniform(1.0, 5.0, n_G + 1))[::-1] + rng.uniform(-0.3, 0.3, n_G + 1)) for _ in range(n_layers)]
        n_m = list(rng.uniform(1.0, 4.0, n_layers))
        budget = float(rng.uniform(0.0, sum(n_m)))
        pick = so.greedy_memory(t_star, n_m, budget)
        used = sum(p / n_G * w for p, w in zip(pick, n_m))
        assert used <= budget + 1e-12
        # never worse than leaving everything off the GPU, and no single affordable raise still helps
        assert sum(t[p] for t, p in zip(t_star, pick)) <= sum(t[0] for t in t_star) + 1e-12
        for j in range(n_layers):
            for i in range(pick[j] + 1, n_G + 1):
                if (i - pick[j]) / n_G * n_m[j] <= budget - used:
                    assert t_star[j][i] >= t_star[j][pick[j]]
        # with room for everything and strictly decreasing times every layer ends fully resident
        dec = [[float(n_G - i) for i in range(n_G + 1)] for _ in range(n_layers)]
        assert so.greedy_memory(dec, n_m, sum(n_m) + 1.0) == [n_G] * n_layers
