/*
 * CPU oracle for the partitioned feed-forward layer (dense SwiGLU MLP or routed MoE experts).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain definition of what the layer computes,
 * in double precision, used only to check the GPU library and to give a timed CPU baseline.
 * It shares no code with the GPU library and the GPU library never calls it.
 *
 * What it follows:
 *  - Section III-B, Eq. 1-2: the weights of FC1 are sliced by columns and those of FC2 by rows
 *    into CC / CG / GG parts; the layer output is the sum of the three partial products and is
 *    identical to the unsliced layer.  Tokens are split X -> [X1; X2]; the last n_g tokens (X2)
 *    use the CC weights on the GPU (CG'), the others on the CPU.  Arithmetic is the same.
 *  - Section II-A: the MoE block assigns tokens to experts with a gating function, processes
 *    each token with its experts and aggregates the results.
 *  The paper does not name the activation or the router; the workload definition fixes a SwiGLU
 *  MLP (gate and up projections both play the role of FC1, sliced by the same hidden index j;
 *  down is FC2) and top-k routing on raw logits with a softmax over the selected k
 *  (ties -> lower expert index, slots ordered by descending logit).
 *
 * Storage types: weights and x are bfloat16 bit patterns (uint16), logits are float32.  Every
 * value is widened exactly to double and all arithmetic is double; nothing is rounded in between.
 * Weight layout is [expert][hidden index j][model index m] for gate, up and down alike.
 *
 * Parallelism: "omp parallel for" over independent hidden indices j (step 1) and over blocks of
 * 256 output columns m (step 2: the m loop is cut into blocks only to hand them to threads; every
 * y[m] is still the sum over j in ascending j, so the result does not depend on the block size or
 * the thread count).  No fusion or reordering beyond that.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double bf16_to_double(uint16_t b) {
  uint32_t u = ((uint32_t)b) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

void so_set_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int so_get_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

/* SiLU(z) = z / (1 + exp(-z)) */
double so_silu(double z) { return z / (1.0 + exp(-z)); }

/*
 * Slicing rates -> integer column counts.  The paper gives rates only (Section IV-A: r_CC + r_CG +
 * r_GG = 1); the reading used here rounds the cumulative rates to a granule g of hidden columns:
 *   n_GG = g * floor(r_GG * H/g + 1/2),  n_GG + n_CG = g * floor((r_GG + r_CG) * H/g + 1/2),
 *   n_CC = H - n_GG - n_CG.   Returns 0, or -1 on invalid arguments.
 */
int so_split_counts(int H, int g, double r_gg, double r_cg, int* n_cc, int* n_cg, int* n_gg) {
  if (H <= 0 || g <= 0 || H % g != 0 || r_gg < 0 || r_cg < 0 || r_gg + r_cg > 1.0 + 1e-6) return -1;
  int units = H / g;
  int a = (int)floor(r_gg * units + 0.5);
  int b = (int)floor((r_gg + r_cg) * units + 0.5);
  if (a > units) a = units;
  if (b > units) b = units;
  if (b < a) b = a;
  *n_gg = a * g;
  *n_cg = (b - a) * g;
  *n_cc = H - b * g;
  return 0;
}

/*
 * Token assignment (Section II-A "gating function to assign tokens to their respective experts").
 *  idx[t][s]  : the k experts of token t, ordered by (logit descending, expert index ascending)
 *  w[t][s]    : softmax over the k selected logits (sums to 1 per token)
 *  count[e]   : number of (t,s) pairs routed to expert e
 *  off[e]     : exclusive prefix sum of count, off[E] = T*k
 *  perm[p]    : pair id t*k+s that sits at position p when pairs are sorted by expert, keeping
 *               ascending (t,s) order inside an expert;  inv[t*k+s] = p.
 * Returns 0, -1 on bad arguments, -2 if a logit is not finite.
 */
int so_route(const float* logits, int T, int E, int k, int32_t* idx, double* w, int32_t* count,
             int32_t* off, int32_t* perm, int32_t* inv) {
  if (T < 0 || E <= 0 || k <= 0 || k > E) return -1;
  for (long i = 0; i < (long)T * E; ++i)
    if (!isfinite(logits[i])) return -2;
  char* taken = (char*)malloc((size_t)E);
  for (int t = 0; t < T; ++t) {
    const float* l = logits + (long)t * E;
    memset(taken, 0, (size_t)E);
    for (int s = 0; s < k; ++s) {
      int best = -1;
      for (int e = 0; e < E; ++e) {
        if (taken[e]) continue;
        if (best < 0 || l[e] > l[best]) best = e; /* strict > keeps the lower index on ties */
      }
      taken[best] = 1;
      idx[(long)t * k + s] = best;
    }
    double lmax = (double)l[idx[(long)t * k]];
    double sum = 0.0;
    for (int s = 0; s < k; ++s) sum += exp((double)l[idx[(long)t * k + s]] - lmax);
    for (int s = 0; s < k; ++s) w[(long)t * k + s] = exp((double)l[idx[(long)t * k + s]] - lmax) / sum;
  }
  free(taken);
  for (int e = 0; e < E; ++e) count[e] = 0;
  for (long q = 0; q < (long)T * k; ++q) count[idx[q]] += 1;
  off[0] = 0;
  for (int e = 0; e < E; ++e) off[e + 1] = off[e] + count[e];
  int32_t* fill = (int32_t*)calloc((size_t)E, sizeof(int32_t));
  for (long q = 0; q < (long)T * k; ++q) { /* ascending (t,s) = ascending q */
    int e = idx[q];
    int32_t p = off[e] + fill[e]++;
    perm[p] = (int32_t)q;
    inv[q] = p;
  }
  free(fill);
  return 0;
}

/*
 * Weights of one SwiGLU MLP, [hidden index j][model index m], in one of two storage forms:
 *  kind 0: bfloat16 bit patterns g, u, d.
 *  kind 1: 4-bit codes with group scales (the paper evaluates INT4 models, Section V-A, without naming a
 *          format; this one is the build's own): code c in 0..15 stands for (c - 8) * scale.
 *          qg, qu, qd [H][M/2] bytes: element m of row j is the low nibble of byte m/2 for even m, the high
 *          nibble for odd m.  Scales are bfloat16: sg, su [H][M/64] (one per 64 consecutive m of a row, the
 *          contraction index of FC1), sd [H/64][M] (one per 64 consecutive j of a column, the contraction
 *          index of FC2).  The dequantised value is exact in double and is never rounded.
 */
typedef struct {
  int kind;
  const uint16_t *g, *u, *d;
  const uint8_t *qg, *qu, *qd;
  const uint16_t *sg, *su, *sd;
} mlp_w;

static inline int q4_code(const uint8_t* q, int M, int j, int m) {
  int b = q[(size_t)j * (M / 2) + m / 2];
  return (m & 1) ? (b >> 4) : (b & 15);
}

static inline double w_fc1(const mlp_w* w, int which /* 0 gate, 1 up */, int M, int j, int m) {
  if (w->kind == 0) return bf16_to_double((which ? w->u : w->g)[(size_t)j * M + m]);
  return (double)(q4_code(which ? w->qu : w->qg, M, j, m) - 8) *
         bf16_to_double((which ? w->su : w->sg)[(size_t)j * (M / 64) + m / 64]);
}

static inline double w_fc2(const mlp_w* w, int M, int j, int m) {
  if (w->kind == 0) return bf16_to_double(w->d[(size_t)j * M + m]);
  return (double)(q4_code(w->qd, M, j, m) - 8) * bf16_to_double(w->sd[(size_t)(j / 64) * M + m]);
}

/*
 * One token through the hidden columns j in [j0, j1) of one SwiGLU MLP:
 *   h_j = SiLU(sum_m x_m Wg[j][m]) * (sum_m x_m Wu[j][m]),   y_m += coef * sum_j h_j Wd[j][m].
 * With [j0,j1) = [0,H) this is the unsliced layer; with a sub-range it is one term of Eq. 2.
 */
static void mlp_token_range(int M, const mlp_w* w, int j0, int j1, double coef, double* y, double* h,
                            const double* xd /* the token, widened: xd[m] */) {
  if (j1 <= j0) return;
#pragma omp parallel for schedule(static)
  for (int j = j0; j < j1; ++j) {
    double g = 0.0, u = 0.0;
    for (int m = 0; m < M; ++m) {
      g += xd[m] * w_fc1(w, 0, M, j, m);
      u += xd[m] * w_fc1(w, 1, M, j, m);
    }
    h[j] = so_silu(g) * u;
  }
  const int MB = 256;
#pragma omp parallel for schedule(static)
  for (int m0 = 0; m0 < M; m0 += MB) {
    int m1 = m0 + MB < M ? m0 + MB : M;
    double acc[256];
    for (int m = m0; m < m1; ++m) acc[m - m0] = 0.0;
    for (int j = j0; j < j1; ++j) {
      double hj = h[j];
      for (int m = m0; m < m1; ++m) acc[m - m0] += hj * w_fc2(w, M, j, m);
    }
    for (int m = m0; m < m1; ++m) y[m] += coef * acc[m - m0];
  }
}

/* the MLP of expert e inside [E][H][...] arrays of either storage form */
static mlp_w expert_view(const mlp_w* all, int e, int H, int M) {
  mlp_w v = *all;
  if (all->kind == 0) {
    v.g = all->g + (size_t)e * H * M; v.u = all->u + (size_t)e * H * M; v.d = all->d + (size_t)e * H * M;
  } else {
    v.qg = all->qg + (size_t)e * H * (M / 2); v.qu = all->qu + (size_t)e * H * (M / 2); v.qd = all->qd + (size_t)e * H * (M / 2);
    v.sg = all->sg + (size_t)e * H * (M / 64); v.su = all->su + (size_t)e * H * (M / 64); v.sd = all->sd + (size_t)e * (H / 64) * M;
  }
  return v;
}

/*
 * Layer forward, sliced form (Eq. 1-2).  Hidden columns of every expert are ordered
 * [CC | CG | GG] (Section III-B): j in [0,n_cc) is CC, [n_cc, n_cc+n_cg) CG, the rest GG.
 * The three partial outputs are computed separately and then added.  Tokens t < T - n_g are X1
 * (their CC share is the CPU's), tokens t >= T - n_g are X2 (CG' : same weights, same math).
 * Passing n_cc = n_cg = 0 gives the unsliced layer in one piece.
 *
 *  x        [T][M] bf16;  logits [T][E] fp32 or NULL when E == 1 (dense MLP, weight 1)
 *  wg,wu,wd [E][H][M] bf16;  sg,su,sd [Hs][M] bf16 shared expert (Hs = 0: none), weight 1,
 *  sliced by its own counts (s_cc, s_cg).
 *  sel      token indices to evaluate (n_sel of them) or NULL for all T tokens
 *  y        [n_sel or T][M] double, overwritten.
 * Returns 0 or a negative error code (so_route's, or -1).
 */
static int layer_forward_core(const uint16_t* x, int T, int M, int H, int E, int k, const float* logits,
                              const mlp_w* routed, int Hs, const mlp_w* shared, int n_cc, int n_cg,
                              int s_cc, int s_cg, int n_g, const int32_t* sel, int n_sel, double* y) {
  if (T < 0 || M <= 0 || H <= 0 || E <= 0 || k <= 0 || k > E) return -1;
  if (n_cc < 0 || n_cg < 0 || n_cc + n_cg > H || n_g < 0 || n_g > T) return -1;
  if (Hs > 0 && (s_cc < 0 || s_cg < 0 || s_cc + s_cg > Hs)) return -1;
  if (E > 1 && logits == NULL) return -1;
  if (sel)
    for (int i = 0; i < n_sel; ++i)
      if (sel[i] < 0 || sel[i] >= T) return -1;
  int32_t* idx = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * k);
  double* w = (double*)malloc(sizeof(double) * (size_t)(T > 0 ? T : 1) * k);
  if (logits) {
    int32_t* count = (int32_t*)malloc(sizeof(int32_t) * E);
    int32_t* off = (int32_t*)malloc(sizeof(int32_t) * (E + 1));
    int32_t* perm = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * k);
    int32_t* inv = (int32_t*)malloc(sizeof(int32_t) * (size_t)(T > 0 ? T : 1) * k);
    int rc = so_route(logits, T, E, k, idx, w, count, off, perm, inv);
    free(count); free(off); free(perm); free(inv);
    if (rc) { free(idx); free(w); return rc; }
  } else {
    for (int t = 0; t < T; ++t) { idx[t] = 0; w[t] = 1.0; }
  }
  int n_out = sel ? n_sel : T;
  int Hmax = H > Hs ? H : Hs;
  double* h = (double*)malloc(sizeof(double) * (size_t)Hmax);
  double* xd = (double*)malloc(sizeof(double) * (size_t)M);
  double* part[3];
  for (int p = 0; p < 3; ++p) part[p] = (double*)malloc(sizeof(double) * (size_t)M);
  for (int i = 0; i < n_out; ++i) {
    int t = sel ? sel[i] : i;
    const uint16_t* xt = x + (size_t)t * M;
    for (int m = 0; m < M; ++m) xd[m] = bf16_to_double(xt[m]);
    for (int p = 0; p < 3; ++p) memset(part[p], 0, sizeof(double) * (size_t)M);
    /* part[0]: Y^CC when t is an X1 row (t < T - n_g), Y^CG' when it is an X2 row: the same
       weights and the same arithmetic, only the place of execution differs (Section III-B);
       part[1]: Y^CG; part[2]: Y^GG */
    for (int s = 0; s < k; ++s) {
      int e = idx[(size_t)t * k + s];
      double c = w[(size_t)t * k + s];
      const mlp_w we = expert_view(routed, e, H, M);
      mlp_token_range(M, &we, 0, n_cc, c, part[0], h, xd);
      mlp_token_range(M, &we, n_cc, n_cc + n_cg, c, part[1], h, xd);
      mlp_token_range(M, &we, n_cc + n_cg, H, c, part[2], h, xd);
    }
    if (Hs > 0) {
      mlp_token_range(M, shared, 0, s_cc, 1.0, part[0], h, xd);
      mlp_token_range(M, shared, s_cc, s_cc + s_cg, 1.0, part[1], h, xd);
      mlp_token_range(M, shared, s_cc + s_cg, Hs, 1.0, part[2], h, xd);
    }
    double* yo = y + (size_t)i * M;
    for (int m = 0; m < M; ++m) yo[m] = part[0][m] + part[1][m] + part[2][m];
  }
  for (int p = 0; p < 3; ++p) free(part[p]);
  free(xd); free(h); free(idx); free(w);
  return 0;
}

int so_layer_forward(const uint16_t* x, int T, int M, int H, int E, int k, const float* logits,
                     const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, int Hs,
                     const uint16_t* sg, const uint16_t* su, const uint16_t* sd, int n_cc, int n_cg,
                     int s_cc, int s_cg, int n_g, const int32_t* sel, int n_sel, double* y) {
  mlp_w routed = {0, wg, wu, wd, NULL, NULL, NULL, NULL, NULL, NULL};
  mlp_w shared = {0, sg, su, sd, NULL, NULL, NULL, NULL, NULL, NULL};
  return layer_forward_core(x, T, M, H, E, k, logits, &routed, Hs, &shared, n_cc, n_cg, s_cc, s_cg, n_g, sel, n_sel, y);
}

/*
 * The same layer with 4-bit weights (storage form 1 above): q* are the code arrays, z* the scale arrays of
 * the routed experts ([E] leading) and of the shared expert.  M and H (and Hs) must be multiples of 64.
 */
int so_layer_forward_q4(const uint16_t* x, int T, int M, int H, int E, int k, const float* logits,
                        const uint8_t* qg, const uint8_t* qu, const uint8_t* qd, const uint16_t* zg,
                        const uint16_t* zu, const uint16_t* zd, int Hs, const uint8_t* sqg, const uint8_t* squ,
                        const uint8_t* sqd, const uint16_t* szg, const uint16_t* szu, const uint16_t* szd,
                        int n_cc, int n_cg, int s_cc, int s_cg, int n_g, const int32_t* sel, int n_sel, double* y) {
  if (M % 64 != 0 || H % 64 != 0 || Hs % 64 != 0) return -1;
  mlp_w routed = {1, NULL, NULL, NULL, qg, qu, qd, zg, zu, zd};
  mlp_w shared = {1, NULL, NULL, NULL, sqg, squ, sqd, szg, szu, szd};
  return layer_forward_core(x, T, M, H, E, k, logits, &routed, Hs, &shared, n_cc, n_cg, s_cc, s_cg, n_g, sel, n_sel, y);
}

/* Dequantised value of one element (test hook for the pins): which = 0 gate, 1 up, 2 down. */
double so_q4_value(const uint8_t* q, const uint16_t* z, int M, int which, int j, int m) {
  mlp_w w = {1, NULL, NULL, NULL, q, q, q, z, z, z};
  return which == 2 ? w_fc2(&w, M, j, m) : w_fc1(&w, which, M, j, m);
}
