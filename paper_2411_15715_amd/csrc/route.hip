// Token assignment (Section II-A: a gating function assigns tokens to their experts).
// top-k on raw logits (ties -> lower index), softmax over the selected k, per-expert histogram,
// exclusive prefix sum, stable expert-sorted permutation, and the launch tables derived from them.
// Everything that decides an index is integer or an exact fp32 comparison, so the result does not
// depend on scheduling.
#include "si_internal.h"
#include "route_device.h"

namespace si {

namespace {

constexpr int WAVE = 64;

__global__ __launch_bounds__(256) void k_topk(const float* __restrict__ logits, int T, int E, int k,
                                              int32_t* __restrict__ idx, float* __restrict__ w) {
  __shared__ float sel[4][MAX_EXPERTS];
  int wv = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
  int t = blockIdx.x * 4 + wv;
  if (t >= T) return;
  topk_token(logits + (size_t)t * E, E, k, lane, idx + (size_t)t * k, w + (size_t)t * k, sel[wv]);
}

__global__ void k_dense_assign(int T, int32_t* __restrict__ idx, float* __restrict__ w) {
  int t = blockIdx.x * blockDim.x + threadIdx.x;
  if (t < T) { idx[t] = 0; w[t] = 1.f; }
}

// Single block.  Builds count/off/perm/inv and the launch tables from idx.
__device__ __forceinline__ void assign_body(int T, int E, int k, int has_shared, int n_x1, const Plan& p,
                                            const RouteOut& u) {
  __shared__ int s_count[MAX_EXPERTS + 2];
  __shared__ int s_count1[MAX_EXPERTS + 2];
  __shared__ int s_off[MAX_EXPERTS + 3];
  __shared__ int s_run[MAX_EXPERTS + 2];
  __shared__ int s_wcnt[ROUTE_THREADS / WAVE][MAX_EXPERTS];
  __shared__ int s_tiles[2][MAX_EXPERTS + 3];
  const int tid = threadIdx.x, lane = tid % WAVE, wv = tid / WAVE;
  const int NW = ROUTE_THREADS / WAVE;
  const int EX = E + (has_shared ? 1 : 0);
  const int n_pairs = T * k;

  for (int e = tid; e < EX; e += ROUTE_THREADS) { s_count[e] = 0; s_count1[e] = 0; s_run[e] = 0; }
  __syncthreads();
  for (int q = tid; q < n_pairs; q += ROUTE_THREADS) {
    int e = p.idx[q];
    atomicAdd(&s_count[e], 1);
    if (q / k < n_x1) atomicAdd(&s_count1[e], 1);
  }
  __syncthreads();
  if (tid == 0) {
    if (has_shared) { s_count[E] = T; s_count1[E] = n_x1; }
    int acc = 0;
    for (int e = 0; e < EX; ++e) { s_off[e] = acc; acc += s_count[e]; }
    s_off[EX] = acc;
    // touched list and row-tile tables
    int nt = 0, a = 0, b = 0, single = 3;
    for (int e = 0; e < EX; ++e) {
      if (s_count[e] > 0 && p.touched) p.touched[nt] = e;
      if (s_count[e] > 0) ++nt;
      s_tiles[0][e] = a;
      s_tiles[1][e] = b;
      const int ta = n_row_tiles(s_count[e]), tb = n_row_tiles(s_count[e] - s_count1[e]);
      a += ta;
      b += tb;
      if (e < E) single &= (ta <= 1 ? 1 : 0) | (tb <= 1 ? 2 : 0);
    }
    if (p.tile_flags) *p.tile_flags = single;
    s_tiles[0][EX] = a;
    s_tiles[1][EX] = b;
    if (p.n_touched) *p.n_touched = nt;
    // launches over "all experts" cover the routed experts only (the shared expert, entry E, gets its own)
    if (p.n_tiles) *p.n_tiles = s_tiles[0][E];
    if (p.n_tiles_x2) *p.n_tiles_x2 = s_tiles[1][E];
  }
  __syncthreads();
  for (int e = tid; e < EX; e += ROUTE_THREADS) {
    if (p.count) p.count[e] = s_count[e];
    if (p.count1) p.count1[e] = s_count1[e];
    if (p.off) p.off[e] = s_off[e];
    if (e < E) {
      if (u.count) u.count[e] = s_count[e];
      if (u.off) u.off[e] = s_off[e];
    }
    if (p.tile_e) {
      int n0 = s_tiles[0][e + 1] - s_tiles[0][e];
      for (int r = 0; r < n0; ++r) { p.tile_e[s_tiles[0][e] + r] = e; p.tile_r[s_tiles[0][e] + r] = r; }
    }
    if (p.tile_e_x2) {
      int n1 = s_tiles[1][e + 1] - s_tiles[1][e];
      for (int r = 0; r < n1; ++r) { p.tile_e_x2[s_tiles[1][e] + r] = e; p.tile_r_x2[s_tiles[1][e] + r] = r; }
    }
  }
  if (tid == 0) {
    if (p.off) p.off[EX] = s_off[EX];
    if (u.off) u.off[E] = s_off[E];
  }
  // stable positions: pairs in ascending q, ROUTE_THREADS at a time
  for (int base = 0; base < n_pairs; base += ROUTE_THREADS) {
    for (int i = tid; i < NW * E; i += ROUTE_THREADS) s_wcnt[i / E][i % E] = 0;
    __syncthreads();
    int q = base + tid;
    bool valid = q < n_pairs;
    int e = valid ? p.idx[q] : -1;
    int rank = 0;
    unsigned long long remaining = __ballot(valid);
    const unsigned long long lt = (lane == 0) ? 0ull : (~0ull >> (64 - lane));
    while (remaining) {
      int leader = __ffsll((long long)remaining) - 1;
      int el = __shfl(e, leader, WAVE);
      unsigned long long m = __ballot(valid && e == el);
      if (valid && e == el) {
        rank = __popcll(m & lt);
        if (rank == 0) s_wcnt[wv][e] = __popcll(m);
      }
      remaining &= ~m;
    }
    __syncthreads();
    if (valid) {
      int pos = s_run[e] + rank;
      for (int w2 = 0; w2 < wv; ++w2) pos += s_wcnt[w2][e];
      int row = s_off[e] + pos;
      if (p.perm) p.perm[row] = q;
      if (p.inv) p.inv[q] = row;
      if (u.perm) u.perm[row] = q;
      if (u.inv) u.inv[q] = row;
      if (p.row_token) p.row_token[row] = q / k;
    }
    __syncthreads();
    for (int e2 = tid; e2 < E; e2 += ROUTE_THREADS) {
      int add = 0;
      for (int w2 = 0; w2 < NW; ++w2) add += s_wcnt[w2][e2];
      s_run[e2] += add;
    }
    __syncthreads();
  }
  if (has_shared && p.row_token)
    for (int t = tid; t < T; t += ROUTE_THREADS) p.row_token[n_pairs + t] = t;
}

__global__ __launch_bounds__(ROUTE_THREADS) void k_assign(int T, int E, int k, int has_shared, int n_x1,
                                                          Plan p, RouteOut u) {
  assign_body(T, E, k, has_shared, n_x1, p, u);
}

// Few tokens (generation phase): selection and assignment in one launch.  Wave v of the block takes
// tokens v, v + 16, ...; the assignment then runs on the whole block.
__global__ __launch_bounds__(ROUTE_THREADS) void k_route_small(const float* __restrict__ logits, int T, int E, int k,
                                                               int has_shared, int n_x1, Plan p, RouteOut u) {
  __shared__ float sel[ROUTE_THREADS / WAVE][MAX_EXPERTS];
  const int wv = threadIdx.x / WAVE, lane = threadIdx.x % WAVE;
  if (logits) {
    for (int t = wv; t < T; t += ROUTE_THREADS / WAVE)
      topk_token(logits + (size_t)t * E, E, k, lane, p.idx + (size_t)t * k, p.w + (size_t)t * k, sel[wv]);
  } else {
    for (int t = threadIdx.x; t < T; t += ROUTE_THREADS) { p.idx[t] = 0; p.w[t] = 1.f; }
  }
  __syncthreads();
  if (u.idx || u.w)
    for (int i = threadIdx.x; i < T * k; i += ROUTE_THREADS) {
      if (u.idx) u.idx[i] = p.idx[i];
      if (u.w) u.w[i] = p.w[i];
    }
  assign_body(T, E, k, has_shared, n_x1, p, u);
}

__global__ void k_copy_user(int n, const int32_t* __restrict__ idx, const float* __restrict__ w, int32_t* uidx,
                            float* uw) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) {
    if (uidx) uidx[i] = idx[i];
    if (uw) uw[i] = w[i];
  }
}

}  // namespace

hipError_t launch_route(const float* logits, int T, int E, int k, int has_shared, int n_g,
                        const Plan& plan, const RouteOut& user, hipStream_t stream) {
  if (T <= 0) return hipSuccess;
  if (T <= 64) {
    hipLaunchKernelGGL(k_route_small, dim3(1), dim3(ROUTE_THREADS), 0, stream, logits, T, E, k, has_shared, T - n_g,
                       plan, user);
    return hipGetLastError();
  }
  if (logits) {
    hipLaunchKernelGGL(k_topk, dim3((T + 3) / 4), dim3(256), 0, stream, logits, T, E, k, plan.idx, plan.w);
  } else {
    hipLaunchKernelGGL(k_dense_assign, dim3((T + 255) / 256), dim3(256), 0, stream, T, plan.idx, plan.w);
  }
  if (user.idx || user.w) {
    int n = T * k;
    hipLaunchKernelGGL(k_copy_user, dim3((n + 255) / 256), dim3(256), 0, stream, n, plan.idx, plan.w, user.idx,
                       user.w);
  }
  hipLaunchKernelGGL(k_assign, dim3(1), dim3(ROUTE_THREADS), 0, stream, T, E, k, has_shared, T - n_g, plan,
                     user);
  return hipGetLastError();
}

}  // namespace si
