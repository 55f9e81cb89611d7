"""CPU oracle of the Profiler & Solver arithmetic (performance models, layer-time recurrence,
slicing-rate and token-assignment optimisation).

TEST INFRASTRUCTURE ONLY: imported by ``tests/`` (and by nothing in the product path).  Plain
Python / NumPy in float64, written from the paper's equations in the paper's notation; it shares no
code with the library's solver and imports nothing from the GPU package.

What each function follows:
  fit_linear        Section IV-A.1, Eq. 3 (t = alpha + n*beta), ordinary least squares, r^2 as in Table I
  task_times        Section IV-A.2, Eq. 4 (with alpha_C2G multiplied by sgn(r_CG), as the case formulas
                    of Section IV-A.3 have it)
  simulate          Section IV-A.2, Eq. 6 (timestamps tau_L, tau_C2G, tau_G, tau_C; tau^0 = 0, i = 1..n_l)
  solve_split       Section IV-A.3 (conditions Q1-Q3, edge points X, Y = t_fin(X), Eq. 13)
  task_times_ng     Section IV-B, Eq. 15 (primed times as functions of n_g), read so that n_g = 0 gives
                    back Eq. 4: the CG' terms carry sgn(n_g) and the copied bytes are (r_CG + r_CC)*n_W
  solve_ng          Section IV-B (same edge-point method on the integer n_g)
  greedy_memory     Section IV-A.4, Eq. 14 (importance s_i^{j,t}, greedy until the memory is used up)

Pins: tests/test_solver_oracle_pins.py.
"""
from __future__ import annotations

import math

import numpy as np


def sgn(v: float) -> float:
    """Sign function of Eq. 4 for non-negative arguments: 1 if v > 0 else 0."""
    return 1.0 if v > 0.0 else 0.0


def fit_linear(n, t):
    """Least-squares alpha, beta of t = alpha + n*beta and the coefficient of determination r^2."""
    n = np.asarray(n, np.float64)
    t = np.asarray(t, np.float64)
    A = np.stack([np.ones_like(n), n], axis=1)
    (alpha, beta), *_ = np.linalg.lstsq(A, t, rcond=None)
    res = t - (alpha + beta * n)
    tot = t - t.mean()
    ss_tot = float(tot @ tot)
    r2 = 1.0 - float(res @ res) / ss_tot if ss_tot > 0.0 else 1.0
    return float(alpha), float(beta), r2


def task_times(model: dict, n_gemm: float, n_w: float, r_gg: float, r_cg: float):
    """Eq. 4: (t_G, t_C, t_C2G, t_L) of one GEMM of the layer for slicing rates r_GG, r_CG, r_CC = 1 - both."""
    r_cc = 1.0 - r_gg - r_cg
    if abs(r_cc) < 1e-15:
        r_cc = 0.0
    t_g = model["alpha_g"] * (sgn(r_cg) + sgn(r_gg)) + (r_cg + r_gg) * n_gemm * model["beta_g"]
    t_c = model["alpha_c"] * sgn(r_cc) + r_cc * n_gemm * model["beta_c"]
    t_c2g = model["alpha_c2g"] * sgn(r_cg) + r_cg * n_w * model["beta_c2g"]
    t_l = (2.0 * sgn(r_cg) + sgn(r_gg)) * model["t_launch"]
    return t_g, t_c, t_c2g, t_l


def simulate(t_g: float, t_c: float, t_c2g: float, t_l: float, n_l: int):
    """Eq. 6: completion timestamps of the n_l GEMMs of a layer; returns (t_fin, tau) with tau a dict of lists
    indexed 0..n_l (entry 0 is the start, 0.0)."""
    tau_l = [0.0]
    tau_c2g = [0.0]
    tau_g = [0.0]
    tau_c = [0.0]
    for i in range(1, n_l + 1):
        tau_l.append(tau_l[i - 1] + t_l)
        tau_c2g.append(max(tau_l[i], tau_c2g[i - 1]) + t_c2g)
        tau_g.append(max(tau_c2g[i], tau_g[i - 1]) + t_g)
        tau_c.append(tau_c[i - 1] + t_c)
    return max(tau_g[n_l], tau_c[n_l]), {"L": tau_l, "C2G": tau_c2g, "G": tau_g, "C": tau_c}


def t_fin(model: dict, n_gemm: float, n_w: float, n_l: int, r_gg: float, r_cg: float) -> float:
    return simulate(*task_times(model, n_gemm, n_w, r_gg, r_cg), n_l)[0]


def which_case(t_g: float, t_c2g: float, t_l: float) -> int:
    """Section IV-A.3: Case 1 (Q1 and Q2), Case 2 (Q1 and not Q2, or not Q1 and Q3), Case 3 (neither Q1 nor Q3)."""
    q1 = t_l < t_c2g
    q2 = t_g < t_c2g
    q3 = t_l < t_g
    if q1 and q2:
        return 1
    if (q1 and not q2) or (not q1 and q3):
        return 2
    return 3


def solve_split(model: dict, n_gemm: float, n_w: float, n_l: int, r_gg: float):
    """Section IV-A.3: the edge points X in [0, 1 - r_GG], Y = t_fin(X), and the minimiser (Eq. 13).
    Returns dict(r_cg, t_fin, X, Y)."""
    R = 1.0 - r_gg
    sg = sgn(r_gg)
    aG, bG = model["alpha_g"], model["beta_g"]
    aC, bC = model["alpha_c"], model["beta_c"]
    aX, bX = model["alpha_c2g"], model["beta_c2g"]
    L = (2.0 + sg) * model["t_launch"]       # t_L for 0 < r_CG
    W = n_w * bX                              # d t_C2G / d r_CG
    G = n_gemm * bG                           # d t_G   / d r_CG
    C = n_gemm * bC                           # -d t_C  / d r_CG
    g0 = aG * (1.0 + sg) + r_gg * G           # t_G at r_CG -> 0+
    c0 = aC + R * C                           # t_C at r_CG -> 0+
    X = [0.0, R]

    def add(num, den):
        if den != 0.0:
            r = num / den
            if 0.0 < r < R:
                X.append(r)

    add(L - aX, W)                            # t_L = t_C2G
    add(g0 - aX, W - G)                       # t_G = t_C2G
    add(L - g0, G)                            # t_L = t_G
    # tau_G^{n_l} = tau_C^{n_l}, with tau_G^{n_l} taken from each of the three cases
    add(n_l * c0 - L - n_l * aX - g0, n_l * W + G + n_l * C)      # Case 1: t_L + n_l t_C2G + t_G
    add(n_l * c0 - L - aX - n_l * g0, W + n_l * G + n_l * C)      # Case 2: t_L + t_C2G + n_l t_G
    add(n_l * c0 - n_l * L - aX - g0, W + G + n_l * C)            # Case 3: n_l t_L + t_C2G + t_G
    Y = [t_fin(model, n_gemm, n_w, n_l, r_gg, r) for r in X]
    i = int(np.argmin(Y))
    return {"r_cg": X[i], "t_fin": Y[i], "X": X, "Y": Y}


# ------------------------------------------------------------------ Section IV-B: token assignment
def task_times_ng(model: dict, T: int, M: int, H: int, n_w: float, r_gg: float, r_cg: float, n_g: int):
    """Eq. 15: primed (t_G', t_C', t_C2G', t_L') of one GEMM when n_g of the T tokens run CC's share on the
    GPU through CG'.  The CG' terms are switched by sgn(n_g) and the copy moves (r_CG + r_CC*sgn(n_g))*n_W
    bytes, so that n_g = 0 reproduces Eq. 4."""
    r_cc = 1.0 - r_gg - r_cg
    if abs(r_cc) < 1e-15:
        r_cc = 0.0
    p = sgn(r_cc) * sgn(n_g)                   # CG' is in use
    t_l = (2.0 * sgn(r_cg) + 2.0 * p + sgn(r_gg)) * model["t_launch"]
    t_c2g = model["alpha_c2g"] * (sgn(r_cg) + p) + (r_cg + r_cc * sgn(n_g)) * n_w * model["beta_c2g"]
    t_g = model["alpha_g"] * (sgn(r_cg) + sgn(r_gg) + p) + (T * (r_cg + r_gg) + n_g * r_cc) * M * H * model["beta_g"]
    t_c = model["alpha_c"] * sgn(r_cc * (T - n_g)) + (T - n_g) * r_cc * M * H * model["beta_c"]
    return t_g, t_c, t_c2g, t_l


def t_fin_ng(model, T, M, H, n_w, n_l, r_gg, r_cg, n_g) -> float:
    return simulate(*task_times_ng(model, T, M, H, n_w, r_gg, r_cg, n_g), n_l)[0]


def solve_ng(model: dict, T: int, M: int, H: int, n_w: float, n_l: int, r_gg: float, r_cg: float):
    """Section IV-B: the best integer n_g in [0, T] from the edge points of the primed model.  Returns
    dict(n_g, t_fin, X, Y); among equal minima the smallest n_g."""
    r_cc = 1.0 - r_gg - r_cg
    if abs(r_cc) < 1e-15:
        r_cc = 0.0
    X = {0, T}
    if r_cc > 0.0 and T > 0:
        X.update({1, T - 1} if T >= 2 else {1})
        # for 1 <= n_g <= T-1: t_L', t_C2G' constant; t_G' = g0 + n_g*G; t_C' = c0 - n_g*C
        t_g1, t_c1, x, L = task_times_ng(model, T, M, H, n_w, r_gg, r_cg, 1)
        G = r_cc * M * H * model["beta_g"]
        C = r_cc * M * H * model["beta_c"]
        g0 = t_g1 - G
        c0 = t_c1 + C
        cand = []
        if G > 0.0:
            cand.append((x - g0) / G)                                   # t_G' = t_C2G'
            cand.append((L - g0) / G)                                   # t_L' = t_G'
        # tau_G^{n_l} = tau_C^{n_l} for the three cases
        cand.append((n_l * c0 - L - n_l * x - g0) / (G + n_l * C))      # Case 1
        cand.append((n_l * c0 - L - x - n_l * g0) / (n_l * G + n_l * C))  # Case 2
        cand.append((n_l * c0 - n_l * L - x - g0) / (G + n_l * C))      # Case 3
        for v in cand:
            if math.isfinite(v):
                for z in (math.floor(v), math.ceil(v)):
                    if 0 <= z <= T:
                        X.add(int(z))
    X = sorted(X)
    Y = [t_fin_ng(model, T, M, H, n_w, n_l, r_gg, r_cg, n) for n in X]
    i = int(np.argmin(Y))
    return {"n_g": X[i], "t_fin": Y[i], "X": X, "Y": Y}


# ------------------------------------------------------------------ Section IV-A.4: GPU memory assignment
def greedy_memory(t_star, n_m, budget: float):
    """Eq. 14.  t_star[j][i] = t_fin*(r_GG = i/n_G) of layer j for i = 0..n_G (Eq. 13 at each grid value);
    n_m[j] = bytes of layer j's sliceable weights; budget = GPU bytes available.  Every iteration computes the
    importance s_i^{j,t} = (t*(v_pre^j) - t*(v_i)) / ((v_i - v_pre^j) * n_m^j) of every grid value above the
    layer's current one that still fits, takes the largest (first in (j, i) order among equals) if it is
    positive, and stops when nothing fits or nothing helps.  Returns the list of grid indices per layer."""
    n_layers = len(t_star)
    n_G = len(t_star[0]) - 1
    cur = [0] * n_layers
    left = float(budget)
    while True:
        best = None
        for j in range(n_layers):
            for i in range(cur[j] + 1, n_G + 1):
                cost = (i - cur[j]) / n_G * n_m[j]
                if cost > left:
                    continue
                s = (t_star[j][cur[j]] - t_star[j][i]) / cost
                if best is None or s > best[0]:
                    best = (s, j, i, cost)
        if best is None or best[0] <= 0.0:
            return cur
        _, j, i, cost = best
        cur[j] = i
        left -= cost


def place_experts(freq, n_gg: int, cg_share: float):
    """Whole-expert placement heuristic (this build's, not the paper's): the n_gg most frequent experts are GG (0);
    the rest, in descending frequency (ties: lower index first), go to CG (1) while CG's share of the frequency
    handed out so far stays <= cg_share, else to CC (2)."""
    order = sorted(range(len(freq)), key=lambda e: (-freq[e], e))
    place = [0] * len(freq)
    cg = total = 0.0
    for r, e in enumerate(order):
        if r < n_gg:
            continue
        if cg + freq[e] <= cg_share * (total + freq[e]):
            place[e] = 1
            cg += freq[e]
        else:
            place[e] = 2
        total += freq[e]
    return place
