/*
 * scheinfer_solver.h - C ABI of the Profiler & Solver (Section III-D, Section IV) that chooses the
 * slicing rates and the prompt-phase token assignment of the partitioned layer in scheinfer.h.
 *
 * All arithmetic is host-side double precision.  Times are seconds, copy sizes are bytes, a GEMM's
 * workload is n_GEMM = T*M*H (Section IV-A.2).  Every function returns SI_OK or a negative SI_E*
 * code (text from si_last_error()); pointers are HOST memory owned by the caller.
 */
#ifndef SCHEINFER_SOLVER_H
#define SCHEINFER_SOLVER_H

#include <stdint.h>

#include "scheinfer.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Linear performance models of Section IV-A.1, Eq. 3: t = alpha + n*beta for a GPU GEMM, a CPU
 * GEMM and a host->device copy, and a constant time per launch. */
typedef struct {
  double alpha_g, beta_g;     /* GPU GEMM: s, s per unit of n_GEMM */
  double alpha_c, beta_c;     /* CPU GEMM: s, s per unit of n_GEMM */
  double alpha_c2g, beta_c2g; /* copy: s, s per byte */
  double t_launch;            /* s per launch */
} si_perf_model_t;

/* One layer as the model of Section IV-A.2 sees it: n_l GEMMs of equal workload n_gemm whose
 * weight tensors hold n_w bytes each. */
typedef struct {
  double n_gemm;
  double n_w;
  int32_t n_l;
} si_problem_t;

/* Per-GEMM task times of Eq. 4 (or their primed versions of Eq. 15). */
typedef struct {
  double t_g, t_c, t_c2g, t_l;
} si_task_times_t;

#define SI_MAX_EDGE_POINTS 24

/* Result of the slicing-rate solve (Eq. 13): the minimiser, the layer time there, which of the
 * three cases of Section IV-A.3 holds at the minimiser (1, 2 or 3), and the evaluated edge points
 * x[i] (values of r_CG) with their layer times y[i]. */
typedef struct {
  double r_cg, r_cc, t_fin;
  int32_t which_case;
  int32_t n_points;
  double x[SI_MAX_EDGE_POINTS], y[SI_MAX_EDGE_POINTS];
} si_split_solution_t;

/* Result of the token-assignment solve (Section IV-B): x[i] are the candidate values of n_g. */
typedef struct {
  int32_t n_g;
  double t_fin;
  int32_t which_case;
  int32_t n_points;
  double x[SI_MAX_EDGE_POINTS], y[SI_MAX_EDGE_POINTS];
} si_ng_solution_t;

/*
 * Ordinary least-squares fit of t = alpha + n*beta to `count` >= 2 measured points (Eq. 3), and
 * the coefficient of determination r^2 reported in Table I (1 - SS_res/SS_tot; 1 when all t are
 * equal).  With nonneg != 0 a negative intercept is replaced by the constrained optimum
 * alpha = 0, beta = sum(n t)/sum(n n), which the solver needs (start-up times cannot be negative).
 * Errors: SI_EINVAL (null pointers, count < 2, all n equal, non-finite input).
 */
int si_fit_linear(const double* n, const double* t, int32_t count, int32_t nonneg, double* alpha,
                  double* beta, double* r2);

/*
 * Eq. 4: task times of one GEMM for slicing rates r_gg, r_cg (r_cc = 1 - r_gg - r_cg).  The copy
 * start-up alpha_C2G is multiplied by sgn(r_CG) as in the case formulas of Section IV-A.3.
 * Errors: SI_EINVAL (rates outside [0,1] or r_gg + r_cg > 1 + 1e-9, n_l < 1, negative model terms).
 */
int si_model_times(const si_perf_model_t* model, const si_problem_t* problem, double r_gg, double r_cg,
                   si_task_times_t* out);

/*
 * Eq. 6: the timestamp recurrence for n_l GEMMs (tau^0 = 0, i = 1..n_l) and the layer time
 * t_fin = max(tau_G^{n_l}, tau_C^{n_l}).  tau_g_end / tau_c_end may be NULL.
 */
int si_simulate(const si_task_times_t* times, int32_t n_l, double* t_fin, double* tau_g_end, double* tau_c_end);

/*
 * Section IV-A.3: the r_CG in [0, 1 - r_gg] that minimises t_fin for a fixed r_gg, found in O(1)
 * from the edge points (t_L = t_C2G, t_G = t_C2G, t_L = t_G, tau_G = tau_C under each case, and the
 * two ends of the interval).  r_step = 0: r_CG is continuous.  r_step > 0: r_CG is restricted to
 * multiples of r_step (what the column granule of a real layer allows, granule/d_ff) plus the right
 * end, and each interior edge point contributes its two neighbours on that grid.
 */
int si_solve_split(const si_perf_model_t* model, const si_problem_t* problem, double r_gg, double r_step,
                   si_split_solution_t* out);

/*
 * Section IV-B, Eq. 15: task times when n_g of the T prompt tokens run the CC share on the GPU from
 * the CC addresses (CG').  The CG' terms are switched by sgn(n_g) and the bytes copied are
 * (r_CG + r_CC*sgn(n_g))*n_w, so that n_g = 0 gives Eq. 4 back.
 */
int si_model_times_ng(const si_perf_model_t* model, int32_t T, int32_t d_model, int32_t d_ff, double n_w,
                      double r_gg, double r_cg, int32_t n_g, si_task_times_t* out);

/* The integer n_g in [0, T] that minimises the layer time of the primed model, by the same edge
 * point method; among equal minima the smallest n_g. */
int si_solve_ng(const si_perf_model_t* model, int32_t T, int32_t d_model, int32_t d_ff, double n_w, int32_t n_l,
                double r_gg, double r_cg, si_ng_solution_t* out);

/*
 * Section IV-A.4, Eq. 14: greedy assignment of GPU memory to layers.  t_star[j*(n_grid+1) + i] is
 * the solved layer time t_fin*(r_GG = i/n_grid) of layer j (from si_solve_split), n_m[j] the bytes
 * of layer j's sliceable weights, budget the GPU bytes to hand out.  Each iteration takes the
 * (layer, grid value) of largest importance (time saved per byte) among those that still fit, as
 * long as it saves time.  Writes the chosen grid index of every layer to pick[j].
 */
int si_assign_gpu_memory(const double* t_star, const double* n_m, int32_t n_layers, int32_t n_grid, double budget,
                         int32_t* pick);

/*
 * Profiler (Section V-B, Table I): measures this machine and fits Eq. 3.
 *  - GPU GEMM and CPU GEMM: a dense layer of d_model x h, h = d_ff*i/n_sizes rounded to 64 columns,
 *    entirely resident (GPU) or entirely on the host (CPU), `tokens` rows; time of the three GEMMs
 *    of the layer (gate, up, down) divided by 3 against n_GEMM = tokens*d_model*h;
 *  - copy: hipMemcpyAsync from pinned memory, n_sizes sizes from 256 KiB to copy_max_mib MiB;
 *  - launch: host time per launch of an empty kernel (mean, sigma over batches).
 * Needs a GPU; allocates and frees its own buffers; synchronises the device.
 */
#define SI_PROFILE_MAX_SIZES 12
typedef struct {
  int32_t d_model, d_ff;
  int32_t tokens;       /* rows of the profiled GEMMs */
  int32_t mode;         /* SI_DECODE | SI_PREFILL | SI_AUTO */
  int32_t n_sizes;      /* 2..SI_PROFILE_MAX_SIZES; 0 -> 6 */
  int32_t reps;         /* timed repetitions per size (the median is kept); 0 -> 5 */
  int32_t cc_threads;   /* as in si_layer_desc_t */
  int32_t device;
  int32_t copy_max_mib; /* largest copy; 0 -> 256 */
  uint32_t seed;        /* of the synthetic weights */
  int32_t q4;           /* 0: bf16 layers; 1: layers in the 4-bit storage form (Table I has a column pair for each) */
} si_profile_desc_t;

typedef struct {
  si_perf_model_t model;           /* non-negative fits */
  double r2_g, r2_c, r2_c2g;       /* r^2 of the three fits */
  double sigma_launch;             /* standard deviation of the launch time over batches */
  int32_t n_points;                /* sizes actually measured */
  double n_gemm[SI_PROFILE_MAX_SIZES], t_g[SI_PROFILE_MAX_SIZES], t_c[SI_PROFILE_MAX_SIZES];
  double bytes[SI_PROFILE_MAX_SIZES], t_c2g[SI_PROFILE_MAX_SIZES];
} si_profile_result_t;

int si_profile(const si_profile_desc_t* desc, si_profile_result_t* out);

/*
 * What this machine sustains on the resources that bound the layer, from the simplest kernels that can reach
 * them (each the best of 4 runs): a read-only stream over 2 GiB of device memory, a 1 GiB device-to-device copy
 * (bytes read + written), a register-resident bf16 MFMA loop on every compute unit, one 256 MiB copy from pinned
 * host memory.  The MFMA loop is run twice: on near-constant operands (the most the matrix cores can do) and on
 * pseudo-random ones that change from instruction to instruction (what they sustain on data: the clock the chip
 * grants depends on the power the operands make the multipliers draw).
 * Needs a GPU and ~3.3 GiB of free device memory; allocates and frees its own buffers.
 */
typedef struct {
  double hbm_read_gbs;
  double hbm_copy_gbs;
  double mfma_bf16_tflops;
  double h2d_gbs;
  int32_t n_cu;
  double mfma_bf16_random_tflops;
} si_peaks_t;
int si_measure_peaks(int32_t device, si_peaks_t* out);

#ifdef __cplusplus
}
#endif
#endif /* SCHEINFER_SOLVER_H */
