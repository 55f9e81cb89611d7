// Solver half of the Profiler & Solver (Section IV): linear performance models, the layer-time
// recurrence, and the O(1) edge-point searches for the slicing rate r_CG and the prompt-phase token
// assignment n_g.  Host-only double arithmetic; no GPU call.
//
// Between the discontinuities of the sign terms every task time of Eq. 4 / Eq. 15 is affine in the
// decision variable, and the last GPU timestamp of Eq. 6 is the largest of three affine chains
// (Section IV-A.3, Cases 1-3).  The layer time is therefore the upper envelope of four lines
// (three GPU chains and the CPU chain) and its minimum sits where two of them cross or at an end
// of the interval.  The crossings are exactly the paper's edge points: C1=C2 <=> t_G = t_C2G,
// C1=C3 <=> t_L = t_C2G, C2=C3 <=> t_L = t_G, and C*=CPU <=> tau_G = tau_C.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <vector>

#include "scheinfer_solver.h"
#include "si_error.h"

namespace {

using si::set_error;

struct Line { double a, b; };  // a + b*v

inline double sgn(double v) { return v > 0.0 ? 1.0 : 0.0; }

int check_model(const si_perf_model_t* m) {
  if (!m) return set_error(SI_EINVAL, "model is NULL");
  const double v[7] = {m->alpha_g, m->beta_g, m->alpha_c, m->beta_c, m->alpha_c2g, m->beta_c2g, m->t_launch};
  for (double x : v)
    if (!std::isfinite(x) || x < 0.0) return set_error(SI_EINVAL, "model coefficients must be finite and >= 0");
  return SI_OK;
}

int check_rates(double r_gg, double r_cg) {
  if (!(r_gg >= 0.0 && r_gg <= 1.0) || !(r_cg >= 0.0 && r_cg <= 1.0) || r_gg + r_cg > 1.0 + 1e-9)
    return set_error(SI_EINVAL, "rates must lie in [0,1] with r_gg + r_cg <= 1 (got %g, %g)", r_gg, r_cg);
  return SI_OK;
}

inline double rest(double r_gg, double r_cg) {
  double r = 1.0 - r_gg - r_cg;
  return std::fabs(r) < 1e-15 || r < 0.0 ? 0.0 : r;
}

void times_eq4(const si_perf_model_t& m, double n_gemm, double n_w, double r_gg, double r_cg, si_task_times_t* o) {
  const double r_cc = rest(r_gg, r_cg);
  o->t_g = m.alpha_g * (sgn(r_cg) + sgn(r_gg)) + (r_cg + r_gg) * n_gemm * m.beta_g;
  o->t_c = m.alpha_c * sgn(r_cc) + r_cc * n_gemm * m.beta_c;
  o->t_c2g = m.alpha_c2g * sgn(r_cg) + r_cg * n_w * m.beta_c2g;
  o->t_l = (2.0 * sgn(r_cg) + sgn(r_gg)) * m.t_launch;
}

void times_eq15(const si_perf_model_t& m, int T, int M, int H, double n_w, double r_gg, double r_cg, int n_g,
                si_task_times_t* o) {
  const double r_cc = rest(r_gg, r_cg);
  const double prime = sgn(r_cc) * sgn((double)n_g);  // CG' in use
  const double mh = (double)M * (double)H;
  o->t_l = (2.0 * sgn(r_cg) + 2.0 * prime + sgn(r_gg)) * m.t_launch;
  o->t_c2g = m.alpha_c2g * (sgn(r_cg) + prime) + (r_cg + r_cc * sgn((double)n_g)) * n_w * m.beta_c2g;
  o->t_g = m.alpha_g * (sgn(r_cg) + sgn(r_gg) + prime) + ((double)T * (r_cg + r_gg) + (double)n_g * r_cc) * mh * m.beta_g;
  o->t_c = m.alpha_c * sgn(r_cc * (double)(T - n_g)) + (double)(T - n_g) * r_cc * mh * m.beta_c;
}

// Eq. 6 with tau^0 = 0
double recurrence(const si_task_times_t& t, int n_l, double* g_end, double* c_end) {
  double tl = 0.0, tx = 0.0, tg = 0.0, tc = 0.0;
  for (int i = 1; i <= n_l; ++i) {
    tl += t.t_l;
    tx = std::max(tl, tx) + t.t_c2g;
    tg = std::max(tx, tg) + t.t_g;
    tc += t.t_c;
  }
  if (g_end) *g_end = tg;
  if (c_end) *c_end = tc;
  return std::max(tg, tc);
}

int case_of(const si_task_times_t& t) {
  const bool q1 = t.t_l < t.t_c2g, q2 = t.t_g < t.t_c2g, q3 = t.t_l < t.t_g;
  if (q1 && q2) return 1;
  if ((q1 && !q2) || (!q1 && q3)) return 2;
  return 3;
}

// the four chains of the envelope from the affine task times L (constant), X, G, C of one GEMM
void chains(double L, Line X, Line G, Line C, int n_l, Line out[4]) {
  const double n = (double)n_l;
  out[0] = {L + n * X.a + G.a, n * X.b + G.b};      // Case 1: t_L + n_l t_C2G + t_G
  out[1] = {L + X.a + n * G.a, X.b + n * G.b};      // Case 2: t_L + t_C2G + n_l t_G
  out[2] = {n * L + X.a + G.a, X.b + G.b};          // Case 3: n_l t_L + t_C2G + t_G
  out[3] = {n * C.a, n * C.b};                      // tau_C^{n_l}
}

void crossings(const Line c[4], std::vector<double>* v) {
  for (int i = 0; i < 4; ++i)
    for (int j = i + 1; j < 4; ++j) {
      const double db = c[i].b - c[j].b;
      if (db == 0.0) continue;
      const double x = (c[j].a - c[i].a) / db;
      if (std::isfinite(x)) v->push_back(x);
    }
}

void sort_unique(std::vector<double>* v) {
  std::sort(v->begin(), v->end());
  v->erase(std::unique(v->begin(), v->end()), v->end());
}

}  // namespace

extern "C" {

int si_fit_linear(const double* n, const double* t, int32_t count, int32_t nonneg, double* alpha, double* beta,
                  double* r2) {
  if (!n || !t || !alpha || !beta) return set_error(SI_EINVAL, "si_fit_linear: NULL pointer");
  if (count < 2) return set_error(SI_EINVAL, "si_fit_linear: need at least 2 points");
  double mn = 0.0, mt = 0.0;
  for (int i = 0; i < count; ++i) {
    if (!std::isfinite(n[i]) || !std::isfinite(t[i])) return set_error(SI_EINVAL, "si_fit_linear: non-finite input");
    mn += n[i];
    mt += t[i];
  }
  mn /= count;
  mt /= count;
  double snn = 0.0, snt = 0.0, stt = 0.0;
  for (int i = 0; i < count; ++i) {
    const double dn = n[i] - mn, dt = t[i] - mt;
    snn += dn * dn;
    snt += dn * dt;
    stt += dt * dt;
  }
  if (snn == 0.0) return set_error(SI_EINVAL, "si_fit_linear: all sizes are equal");
  double b = snt / snn, a = mt - b * mn;
  if (nonneg && a < 0.0) {
    double pnn = 0.0, pnt = 0.0;
    for (int i = 0; i < count; ++i) {
      pnn += n[i] * n[i];
      pnt += n[i] * t[i];
    }
    a = 0.0;
    b = pnt / pnn;
  }
  if (nonneg && b < 0.0) {  // times that fall with size: best non-negative model is the mean
    b = 0.0;
    a = std::max(mt, 0.0);
  }
  *alpha = a;
  *beta = b;
  if (r2) {
    double res = 0.0;
    for (int i = 0; i < count; ++i) {
      const double e = t[i] - (a + b * n[i]);
      res += e * e;
    }
    *r2 = stt > 0.0 ? 1.0 - res / stt : 1.0;
  }
  return SI_OK;
}

int si_model_times(const si_perf_model_t* model, const si_problem_t* p, double r_gg, double r_cg, si_task_times_t* out) {
  if (int rc = check_model(model)) return rc;
  if (!p || !out) return set_error(SI_EINVAL, "si_model_times: NULL pointer");
  if (p->n_l < 1 || !(p->n_gemm >= 0.0) || !(p->n_w >= 0.0)) return set_error(SI_EINVAL, "si_model_times: bad problem");
  if (int rc = check_rates(r_gg, r_cg)) return rc;
  times_eq4(*model, p->n_gemm, p->n_w, r_gg, r_cg, out);
  return SI_OK;
}

int si_simulate(const si_task_times_t* t, int32_t n_l, double* t_fin, double* tau_g_end, double* tau_c_end) {
  if (!t || !t_fin) return set_error(SI_EINVAL, "si_simulate: NULL pointer");
  if (n_l < 1) return set_error(SI_EINVAL, "si_simulate: n_l must be >= 1");
  if (!(t->t_g >= 0.0 && t->t_c >= 0.0 && t->t_c2g >= 0.0 && t->t_l >= 0.0))
    return set_error(SI_EINVAL, "si_simulate: task times must be >= 0");
  *t_fin = recurrence(*t, n_l, tau_g_end, tau_c_end);
  return SI_OK;
}

int si_solve_split(const si_perf_model_t* model, const si_problem_t* p, double r_gg, double r_step,
                   si_split_solution_t* out) {
  if (int rc = check_model(model)) return rc;
  if (!p || !out) return set_error(SI_EINVAL, "si_solve_split: NULL pointer");
  if (p->n_l < 1 || !(p->n_gemm >= 0.0) || !(p->n_w >= 0.0)) return set_error(SI_EINVAL, "si_solve_split: bad problem");
  if (int rc = check_rates(r_gg, 0.0)) return rc;
  if (!(r_step >= 0.0) || r_step > 1.0) return set_error(SI_EINVAL, "si_solve_split: r_step must lie in [0,1]");
  const si_perf_model_t& m = *model;
  const double R = 1.0 - r_gg, sg = sgn(r_gg);

  // affine task times on the open interval 0 < r_CG < R
  const double L = (2.0 + sg) * m.t_launch;
  const Line X = {m.alpha_c2g, p->n_w * m.beta_c2g};
  const Line G = {m.alpha_g * (1.0 + sg) + r_gg * p->n_gemm * m.beta_g, p->n_gemm * m.beta_g};
  const Line C = {m.alpha_c + R * p->n_gemm * m.beta_c, -p->n_gemm * m.beta_c};
  Line env[4];
  chains(L, X, G, C, p->n_l, env);
  std::vector<double> inner;
  crossings(env, &inner);

  std::vector<double> xs = {0.0, R};
  if (r_step > 0.0) {
    const double kmax = std::floor(R / r_step + 1e-9);
    auto on_grid = [&](double k) {
      if (k >= 1.0 && k <= kmax && k * r_step < R) xs.push_back(k * r_step);
    };
    on_grid(1.0);
    on_grid(kmax);
    on_grid(kmax - 1.0);
    for (double v : inner)
      if (v > 0.0 && v < R) {
        on_grid(std::floor(v / r_step));
        on_grid(std::floor(v / r_step) + 1.0);
      }
  } else {
    for (double v : inner)
      if (v > 0.0 && v < R) xs.push_back(v);
  }
  sort_unique(&xs);
  if ((int)xs.size() > SI_MAX_EDGE_POINTS) xs.resize(SI_MAX_EDGE_POINTS);  // cannot happen: <= 2 + 3 + 12

  std::memset(out, 0, sizeof *out);
  int best = -1;
  for (size_t i = 0; i < xs.size(); ++i) {
    si_task_times_t t;
    times_eq4(m, p->n_gemm, p->n_w, r_gg, xs[i], &t);
    out->x[i] = xs[i];
    out->y[i] = recurrence(t, p->n_l, nullptr, nullptr);
    if (best < 0 || out->y[i] < out->y[best]) best = (int)i;
  }
  out->n_points = (int32_t)xs.size();
  out->r_cg = out->x[best];
  out->r_cc = rest(r_gg, out->r_cg);
  out->t_fin = out->y[best];
  si_task_times_t t;
  times_eq4(m, p->n_gemm, p->n_w, r_gg, out->r_cg, &t);
  out->which_case = case_of(t);
  return SI_OK;
}

int si_model_times_ng(const si_perf_model_t* model, int32_t T, int32_t d_model, int32_t d_ff, double n_w, double r_gg,
                      double r_cg, int32_t n_g, si_task_times_t* out) {
  if (int rc = check_model(model)) return rc;
  if (!out) return set_error(SI_EINVAL, "si_model_times_ng: NULL pointer");
  if (T < 0 || d_model < 1 || d_ff < 1 || !(n_w >= 0.0) || n_g < 0 || n_g > T)
    return set_error(SI_EINVAL, "si_model_times_ng: need T >= 0, 0 <= n_g <= T, positive shape");
  if (int rc = check_rates(r_gg, r_cg)) return rc;
  times_eq15(*model, T, d_model, d_ff, n_w, r_gg, r_cg, n_g, out);
  return SI_OK;
}

int si_solve_ng(const si_perf_model_t* model, int32_t T, int32_t d_model, int32_t d_ff, double n_w, int32_t n_l,
                double r_gg, double r_cg, si_ng_solution_t* out) {
  if (int rc = check_model(model)) return rc;
  if (!out) return set_error(SI_EINVAL, "si_solve_ng: NULL pointer");
  if (T < 0 || d_model < 1 || d_ff < 1 || !(n_w >= 0.0) || n_l < 1)
    return set_error(SI_EINVAL, "si_solve_ng: need T >= 0, n_l >= 1, positive shape");
  if (int rc = check_rates(r_gg, r_cg)) return rc;
  const si_perf_model_t& m = *model;
  const double r_cc = rest(r_gg, r_cg);

  std::vector<double> xs = {0.0, (double)T};
  if (r_cc > 0.0 && T >= 1) {
    xs.push_back(1.0);
    xs.push_back((double)(T - 1));
    // affine task times for 1 <= n_g <= T-1 (all sign terms fixed)
    si_task_times_t t1;
    times_eq15(m, T, d_model, d_ff, n_w, r_gg, r_cg, 1, &t1);
    const double mh = (double)d_model * (double)d_ff;
    const double gs = r_cc * mh * m.beta_g, cs = r_cc * mh * m.beta_c;
    const Line X = {t1.t_c2g, 0.0};
    const Line G = {t1.t_g - gs, gs};
    const Line C = {m.alpha_c + (double)T * cs, -cs};
    Line env[4];
    chains(t1.t_l, X, G, C, n_l, env);
    std::vector<double> inner;
    crossings(env, &inner);
    for (double v : inner) {
      const double f = std::floor(v);
      for (double z : {f, f + 1.0})
        if (z >= 0.0 && z <= (double)T) xs.push_back(z);
    }
  }
  sort_unique(&xs);
  if ((int)xs.size() > SI_MAX_EDGE_POINTS) xs.resize(SI_MAX_EDGE_POINTS);  // cannot happen: <= 4 + 12

  std::memset(out, 0, sizeof *out);
  int best = -1;
  for (size_t i = 0; i < xs.size(); ++i) {
    si_task_times_t t;
    times_eq15(m, T, d_model, d_ff, n_w, r_gg, r_cg, (int)xs[i], &t);
    out->x[i] = xs[i];
    out->y[i] = recurrence(t, n_l, nullptr, nullptr);
    if (best < 0 || out->y[i] < out->y[best]) best = (int)i;
  }
  out->n_points = (int32_t)xs.size();
  out->n_g = (int32_t)out->x[best];
  out->t_fin = out->y[best];
  si_task_times_t t;
  times_eq15(m, T, d_model, d_ff, n_w, r_gg, r_cg, out->n_g, &t);
  out->which_case = case_of(t);
  return SI_OK;
}

int si_assign_gpu_memory(const double* t_star, const double* n_m, int32_t n_layers, int32_t n_grid, double budget,
                         int32_t* pick) {
  if (!t_star || !n_m || !pick) return set_error(SI_EINVAL, "si_assign_gpu_memory: NULL pointer");
  if (n_layers < 1 || n_grid < 1 || !(budget >= 0.0)) return set_error(SI_EINVAL, "si_assign_gpu_memory: bad sizes");
  for (int j = 0; j < n_layers; ++j) {
    if (!(n_m[j] > 0.0)) return set_error(SI_EINVAL, "si_assign_gpu_memory: layer sizes must be > 0");
    pick[j] = 0;
  }
  const int stride = n_grid + 1;
  double left = budget;
  for (;;) {
    int bj = -1, bi = -1;
    double bs = 0.0, bcost = 0.0;
    for (int j = 0; j < n_layers; ++j)
      for (int i = pick[j] + 1; i <= n_grid; ++i) {
        const double cost = (double)(i - pick[j]) / (double)n_grid * n_m[j];
        if (cost > left) continue;
        const double s = (t_star[j * stride + pick[j]] - t_star[j * stride + i]) / cost;  // Eq. 14
        if (bj < 0 || s > bs) {
          bj = j;
          bi = i;
          bs = s;
          bcost = cost;
        }
      }
    if (bj < 0 || bs <= 0.0) return SI_OK;
    pick[bj] = bi;
    left -= bcost;
  }
}

int si_place_experts(const double* freq, int32_t n_experts, int32_t n_gg, double cg_share, uint8_t* placement) {
  if (!freq || !placement) return set_error(SI_EINVAL, "si_place_experts: NULL pointer");
  if (n_experts < 1 || n_gg < 0 || n_gg > n_experts || !(cg_share >= 0.0 && cg_share <= 1.0))
    return set_error(SI_EINVAL, "si_place_experts: need n_experts >= 1, 0 <= n_gg <= n_experts, cg_share in [0,1]");
  std::vector<int> order(n_experts);
  for (int e = 0; e < n_experts; ++e) {
    if (!(freq[e] >= 0.0) || !std::isfinite(freq[e])) return set_error(SI_EINVAL, "si_place_experts: freq[%d] must be finite and >= 0", e);
    order[e] = e;
  }
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return freq[a] > freq[b]; });
  double cg = 0.0, all = 0.0;
  for (int r = 0; r < n_experts; ++r) {
    const int e = order[r];
    if (r < n_gg) {
      placement[e] = 0;
      continue;
    }
    if (cg + freq[e] <= cg_share * (all + freq[e])) {
      placement[e] = 1;
      cg += freq[e];
    } else {
      placement[e] = 2;
    }
    all += freq[e];
  }
  return SI_OK;
}

}  // extern "C"
