// Generation-phase expert GEMV (few tokens per expert): bandwidth-bound streaming of bf16 weights
// with fp32 accumulation.  Three kernels per part:
//   gateup : h[row][j] = SiLU(x . Wg[j]) * (x . Wu[j])         (FC1 + activation, Eq. 1)
//   down   : part[slot][row][m] = sum_{j in slot} h[row][j] Wd[j][m]   (FC2, one term of Eq. 2)
//   combine: y[t] = sum_s w[t][s] sum_slots part[..][row(t,s)] (+ shared expert, + Y^CC)
// Every weight byte is read once per pass of up to DECODE_TB tokens, with 128-bit loads that are
// contiguous across the lanes of a wave.
#include "si_internal.h"
#include "route_device.h"

#include <type_traits>

namespace si {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
constexpr int WAVE = 64;
constexpr int GU_THREADS = 256;
constexpr int GU_JPW = 4;                                  // hidden columns per wave
constexpr int GU_JPB = GU_JPW * (GU_THREADS / WAVE);       // hidden columns per block (16)
constexpr int DN_THREADS = 256;

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, WAVE);
  return v;
}

__device__ inline float silu_f(float z) { return z / (1.f + __expf(-z)); }

// expert handled by this block and its row range; returns false when there is nothing to do
__device__ inline bool block_rows(const Plan& p, int expert_sel, int x2_only, int slot, int& e, int& r0, int& r1) {
  if (expert_sel >= 0) {
    e = expert_sel;
  } else {
    if (slot >= *p.n_touched) return false;
    e = p.touched[slot];
    if (e >= p.n_routed) return false;
  }
  r0 = p.off[e] + (x2_only ? p.count1[e] : 0);
  r1 = p.off[e + 1];
  return r1 > r0;
}

// Token assignment of a few tokens inside a block (FusedRoute): the same result as route.hip's kernels, derived
// by every block for itself.  Pairs q = t*k + s in ascending order; the expert-sorted row of pair q is the number of
// pairs with a smaller expert plus the number of earlier pairs with the same expert (stable), which for at most
// FUSED_ROUTE_MAX_PAIRS pairs is a loop over all pairs per thread.
struct BlockRoute {
  int32_t idx[FUSED_ROUTE_MAX_PAIRS];
  float w[FUSED_ROUTE_MAX_PAIRS];
  int32_t row[FUSED_ROUTE_MAX_PAIRS];        // expert-sorted row of pair q
  int32_t row_token[FUSED_ROUTE_MAX_PAIRS + FUSED_ROUTE_MAX_T];  // token of each row (shared expert rows follow)
  int32_t t_expert[FUSED_ROUTE_MAX_PAIRS];   // touched experts, ascending
  int32_t t_off[FUSED_ROUTE_MAX_PAIRS];      // first row of each touched expert
  int32_t t_cnt[FUSED_ROUTE_MAX_PAIRS];
  int32_t n_touched;
  float sel[FUSED_ROUTE_MAX_T][MAX_EXPERTS];
};

__device__ inline void block_route(const FusedRoute& fr, BlockRoute& br, const Plan& p, bool write_tables) {
  const int tid = threadIdx.x, lane = tid % WAVE, wid = tid / WAVE;
  const int T = fr.T, E = fr.E, k = fr.k, n_pairs = T * k;
  if (fr.logits) {
    if (wid < T) topk_token(fr.logits + (size_t)wid * E, E, k, lane, br.idx + wid * k, br.w + wid * k, br.sel[wid]);
  } else if (tid < n_pairs) {
    br.idx[tid] = 0;
    br.w[tid] = 1.f;
  }
  if (tid == 0) br.n_touched = 0;
  __syncthreads();
  int e = -1, row = 0, cnt = 0, first = 0;
  if (tid < n_pairs) {
    e = br.idx[tid];
    first = 1;
    for (int q = 0; q < n_pairs; ++q) {
      const int eq = br.idx[q];
      row += (eq < e) || (eq == e && q < tid);
      cnt += eq == e;
      if (eq == e && q < tid) first = 0;
    }
    br.row[tid] = first;  // (reused as the flag "first pair of its expert" for the next step)
    br.row_token[row] = tid / k;
  }
  if (fr.has_shared && tid < T) br.row_token[n_pairs + tid] = tid;
  __syncthreads();
  if (first) {
    // slot of this expert in the ascending list of touched experts = distinct smaller experts
    int slot = 0;
    for (int q = 0; q < n_pairs; ++q) slot += br.row[q] && br.idx[q] < e;
    br.t_expert[slot] = e;
    br.t_off[slot] = row;
    br.t_cnt[slot] = cnt;
    atomicAdd(&br.n_touched, 1);
  }
  __syncthreads();
  if (!write_tables) return;
  // the tables later launches of this call and the caller read (block (0, 0) only)
  const RouteOut& u = fr.user;
  const int EX = E + (fr.has_shared ? 1 : 0);
  if (tid < n_pairs) {
    const int q = tid;
    p.idx[q] = e; p.w[q] = br.w[q];
    p.perm[row] = q; p.inv[q] = row;
    if (u.idx) u.idx[q] = e;
    if (u.w) u.w[q] = br.w[q];
    if (u.perm) u.perm[row] = q;
    if (u.inv) u.inv[q] = row;
  }
  for (int r = tid; r < n_pairs + (fr.has_shared ? T : 0); r += GU_THREADS) p.row_token[r] = br.row_token[r];
  for (int ex = tid; ex <= EX; ex += GU_THREADS) {
    int c = 0, c1 = 0, o = 0;
    if (ex < E) {
      for (int q = 0; q < n_pairs; ++q) {
        const int eq = br.idx[q];
        c += eq == ex;
        c1 += eq == ex && q / k < fr.n_x1;
        o += eq < ex;
      }
    } else if (ex == E && fr.has_shared) {
      c = T; c1 = fr.n_x1; o = n_pairs;
    } else {
      o = n_pairs + (fr.has_shared ? T : 0);  // the end of the prefix sum
    }
    if (ex < EX) { p.count[ex] = c; p.count1[ex] = c1; }
    p.off[ex] = o;
    if (ex < E) { if (u.count) u.count[ex] = c; }
    if (ex <= E) { if (u.off) u.off[ex] = ex < E ? o : n_pairs; }
  }
  if (tid < br.n_touched) p.touched[tid] = br.t_expert[tid];
  if (tid == 0) {
    int nt = br.n_touched;
    if (fr.has_shared) p.touched[nt++] = E;  // the shared expert always has rows
    *p.n_touched = nt;
  }
}

template <int TB, int FUSED>
__global__ __launch_bounds__(GU_THREADS) void k_decode_gateup(const uint16_t* __restrict__ x, int M, Plan p,
                                                              int expert_sel, int x2_only, WeightView wv,
                                                              float* __restrict__ h, int ldh, FusedRoute fr) {
  extern __shared__ u32x4 s_x[];  // [TB][M/8] bf16 x 8
  __shared__ typename std::conditional<FUSED != 0, BlockRoute, int>::type s_br;  // (4 bytes when the tables are given)
  int e, r0, r1;
  const int* row_token = p.row_token;
  constexpr int X_EARLY_MAX = 4;  // 16-byte pieces per thread: d_model <= 8192
  u32x4 x_reg[X_EARLY_MAX];
  bool x_early = false;
  if constexpr (FUSED != 0) {
    // with a single token every row is token 0
    x_early = TB == 1 && fr.T == 1 && M / 8 <= X_EARLY_MAX * GU_THREADS;
    if (x_early) {
#pragma unroll
      for (int i = 0; i < X_EARLY_MAX; ++i)
        if ((int)threadIdx.x + i * GU_THREADS < M / 8) x_reg[i] = reinterpret_cast<const u32x4*>(x)[threadIdx.x + i * GU_THREADS];
    }
    BlockRoute& br = s_br;
    block_route(fr, br, p, blockIdx.x == 0 && blockIdx.y == 0);
    if (expert_sel >= 0) {
      // one given expert: the routed expert of a dense layer (every pair is its row)
      e = expert_sel;
      r0 = 0;
      r1 = fr.T * fr.k;
    } else {
      if ((int)blockIdx.y >= br.n_touched) return;
      e = br.t_expert[blockIdx.y];
      r0 = br.t_off[blockIdx.y];
      r1 = r0 + br.t_cnt[blockIdx.y];
    }
    row_token = br.row_token;
  } else {
    if (!block_rows(p, expert_sel, x2_only, blockIdx.y, e, r0, r1)) return;
  }
  const int tid = threadIdx.x, lane = tid % WAVE, wid = tid / WAVE;
  const int M8 = M / 8;
  const int blocks_per_chunk = CHUNK_J / GU_JPB;
  const int chunk = wv.chunk0 + blockIdx.x / blocks_per_chunk;
  const int jj0 = (blockIdx.x % blocks_per_chunk) * GU_JPB + wid * GU_JPW;  // first j of this wave in the chunk
  int se;
  if (!storage_index(wv, e, se)) return;
  const uint16_t* cbase = wv.base + (size_t)se * wv.expert_stride + (size_t)chunk * 3 * CHUNK_J * M;
  // gate / up blocks are [M/PW panels][64 j][PW m]: one wave load = 512 contiguous m of one row
  const u32x4* gblk = reinterpret_cast<const u32x4*>(cbase);
  const u32x4* ublk = reinterpret_cast<const u32x4*>(cbase + (size_t)CHUNK_J * M);
  const int PW = panel_width(M), PW8 = PW / 8;
  const int jcol = wv.col0 + (blockIdx.x / blocks_per_chunk) * CHUNK_J + jj0;

  // One-row launches (TB == 1, the generation phase proper): the weights of a wave's first step are fetched before
  // the row of x is staged (and, with a single token, x before the token assignment is derived), so that a block's
  // first bytes are on their way while it waits, not after.  With more rows per pass the peeled first step costs
  // registers, i.e. waves per SIMD, and the plain loop stays.
  constexpr bool EARLY = TB == 1;
  u32x4 wg[GU_JPW], wu[GU_JPW];
  auto wload = [&](int c) {
    const size_t poff = (size_t)(c / PW8) * CHUNK_J * PW8 + (c % PW8);  // panel base + position in the row segment
#pragma unroll
    for (int j = 0; j < GU_JPW; ++j) {
      wg[j] = __builtin_nontemporal_load(gblk + poff + (size_t)(jj0 + j) * PW8);
      wu[j] = __builtin_nontemporal_load(ublk + poff + (size_t)(jj0 + j) * PW8);
    }
  };
  if (EARLY && lane < M8) wload(lane);

  for (int rb = r0; rb < r1; rb += TB) {
    const int nt = min(TB, r1 - rb);
    __syncthreads();
    if (x_early) {
#pragma unroll
      for (int i = 0; i < X_EARLY_MAX; ++i)
        if (tid + i * GU_THREADS < M8) s_x[tid + i * GU_THREADS] = x_reg[i];
    } else {
      for (int i = tid; i < nt * M8; i += GU_THREADS) {
        int tb = i / M8, c = i % M8;
        int tok = row_token[rb + tb];
        s_x[tb * M8 + c] = reinterpret_cast<const u32x4*>(x + (size_t)tok * M)[c];
      }
    }
    __syncthreads();
    float ag[GU_JPW][TB], au[GU_JPW][TB];
#pragma unroll
    for (int j = 0; j < GU_JPW; ++j)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) { ag[j][tb] = 0.f; au[j][tb] = 0.f; }
    auto fma_step = [&](int c) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          u32x4 xv = s_x[tb * M8 + c];
          float xf[8] = {bf_lo(xv.x), bf_hi(xv.x), bf_lo(xv.y), bf_hi(xv.y),
                         bf_lo(xv.z), bf_hi(xv.z), bf_lo(xv.w), bf_hi(xv.w)};
#pragma unroll
          for (int j = 0; j < GU_JPW; ++j) {
            float g = ag[j][tb], u = au[j][tb];
            g = fmaf(xf[0], bf_lo(wg[j].x), g); g = fmaf(xf[1], bf_hi(wg[j].x), g);
            g = fmaf(xf[2], bf_lo(wg[j].y), g); g = fmaf(xf[3], bf_hi(wg[j].y), g);
            g = fmaf(xf[4], bf_lo(wg[j].z), g); g = fmaf(xf[5], bf_hi(wg[j].z), g);
            g = fmaf(xf[6], bf_lo(wg[j].w), g); g = fmaf(xf[7], bf_hi(wg[j].w), g);
            u = fmaf(xf[0], bf_lo(wu[j].x), u); u = fmaf(xf[1], bf_hi(wu[j].x), u);
            u = fmaf(xf[2], bf_lo(wu[j].y), u); u = fmaf(xf[3], bf_hi(wu[j].y), u);
            u = fmaf(xf[4], bf_lo(wu[j].z), u); u = fmaf(xf[5], bf_hi(wu[j].z), u);
            u = fmaf(xf[6], bf_lo(wu[j].w), u); u = fmaf(xf[7], bf_hi(wu[j].w), u);
            ag[j][tb] = g; au[j][tb] = u;
          }
        }
      }
    };
    if constexpr (EARLY) {
      if (lane < M8) {
        if (rb != r0) wload(lane);  // a further pass over the same weights starts over
        fma_step(lane);
      }
      for (int c = lane + WAVE; c < M8; c += WAVE) {
        wload(c);
        fma_step(c);
      }
    } else {
      for (int c = lane; c < M8; c += WAVE) {
        wload(c);
        fma_step(c);
      }
    }
#pragma unroll
    for (int j = 0; j < GU_JPW; ++j)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          float g = wave_sum(ag[j][tb]);
          float u = wave_sum(au[j][tb]);
          if (lane == 0) h[(size_t)(rb + tb) * ldh + jcol + j] = silu_f(g) * u;
        }
      }
  }
}

template <int TB>
__global__ __launch_bounds__(DN_THREADS) void k_decode_down(const float* __restrict__ h, int ldh, int M, Plan p,
                                                            int expert_sel, int x2_only, WeightView wv, int slot0,
                                                            int chunks_per_slot, float* __restrict__ part,
                                                            size_t slot_stride) {
  int e, r0, r1;
  if (!block_rows(p, expert_sel, x2_only, blockIdx.z, e, r0, r1)) return;
  const int s = blockIdx.y;
  const int c_begin = s * chunks_per_slot;
  const int c_end = min(c_begin + chunks_per_slot, wv.n_chunks);
  if (c_begin >= c_end) return;
  const int m = blockIdx.x * DN_THREADS + threadIdx.x;
  const bool active = m < M;
  const int mm = active ? m : 0;
  const int NW = ntile_width(M);
  int se;
  if (!storage_index(wv, e, se)) return;
  const uint16_t* ebase = wv.base + (size_t)se * wv.expert_stride;
  float* out = part + (size_t)(slot0 + s) * slot_stride;

  extern __shared__ float s_h[];  // [TB][n_j] activations of this slot
  const int n_j = (c_end - c_begin) * CHUNK_J;
  const int jbase = wv.col0 + c_begin * CHUNK_J;

  for (int rb = r0; rb < r1; rb += TB) {
    const int nt = min(TB, r1 - rb);
    __syncthreads();
    for (int i = threadIdx.x; i < nt * n_j; i += DN_THREADS) {
      int tb = i / n_j, j = i % n_j;
      s_h[tb * n_j + j] = h[(size_t)(rb + tb) * ldh + jbase + j];
    }
    __syncthreads();
    float acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = 0.f;
    for (int c = c_begin; c < c_end; ++c) {
      const u32x4* dblk = reinterpret_cast<const u32x4*>(ebase + (size_t)(wv.chunk0 + c) * 3 * CHUNK_J * M +
                                                         (size_t)2 * CHUNK_J * M);
      u32x4 wd[8];  // down block [M/NW tiles][8 q][NW m][8 i]: 16 bytes per (q, m)
#pragma unroll
      for (int q = 0; q < 8; ++q) wd[q] = __builtin_nontemporal_load(dblk + ((size_t)(mm / NW) * 8 + q) * NW + (mm % NW));
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          const float4* hr = reinterpret_cast<const float4*>(s_h + tb * n_j + (c - c_begin) * CHUNK_J);
          float a = acc[tb];
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            float4 h0 = hr[q * 2], h1 = hr[q * 2 + 1];
            a = fmaf(h0.x, bf_lo(wd[q].x), a); a = fmaf(h0.y, bf_hi(wd[q].x), a);
            a = fmaf(h0.z, bf_lo(wd[q].y), a); a = fmaf(h0.w, bf_hi(wd[q].y), a);
            a = fmaf(h1.x, bf_lo(wd[q].z), a); a = fmaf(h1.y, bf_hi(wd[q].z), a);
            a = fmaf(h1.z, bf_lo(wd[q].w), a); a = fmaf(h1.w, bf_hi(wd[q].w), a);
          }
          acc[tb] = a;
        }
      }
    }
    if (active) {
#pragma unroll
      for (int tb = 0; tb < TB; ++tb)
        if (tb < nt) out[(size_t)(rb + tb) * M + m] = acc[tb];
    }
  }
}

// One thread per 4 output columns of one token.  The slot partials of a row are independent loads
// (issued together, then summed in slot order, so the result is deterministic).
__global__ __launch_bounds__(64) void k_decode_combine(DecodeCombineArgs a, Plan p, float* __restrict__ y) {
  const int t = blockIdx.y;
  const int m4 = blockIdx.x * 64 + threadIdx.x;
  if (m4 * 4 >= a.M) return;
  const bool is_x2 = t >= a.n_x1;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  const int n_terms = a.k + (a.has_shared ? 1 : 0);
  for (int s = 0; s < n_terms; ++s) {
    int row;
    float wgt;
    if (s < a.k) { row = p.inv[t * a.k + s]; wgt = p.w[t * a.k + s]; }
    else { row = a.T * a.k + t; wgt = 1.f; }
    const int n_part[3] = {s < a.k ? a.n_slots_gg : a.s_slots_gg, s < a.k ? a.n_slots_cg : a.s_slots_cg,
                           is_x2 ? (s < a.k ? a.n_slots_cc : a.s_slots_cc) : 0};
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
    for (int part = 0; part < 3; ++part) {
      const float* base = a.part + (size_t)(part * DOWN_SLOTS) * a.slot_stride + (size_t)row * a.M;
      // eight slots at a time: their loads are issued together, then added in slot order
      for (int q0 = 0; q0 < n_part[part]; q0 += 8) {
        float4 tmp[8];
#pragma unroll
        for (int q = 0; q < 8; ++q)
          tmp[q] = q0 + q < n_part[part] ? reinterpret_cast<const float4*>(base + (size_t)(q0 + q) * a.slot_stride)[m4]
                                         : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int q = 0; q < 8; ++q) { v.x += tmp[q].x; v.y += tmp[q].y; v.z += tmp[q].z; v.w += tmp[q].w; }
      }
    }
    acc.x = fmaf(wgt, v.x, acc.x); acc.y = fmaf(wgt, v.y, acc.y);
    acc.z = fmaf(wgt, v.z, acc.z); acc.w = fmaf(wgt, v.w, acc.w);
  }
  if (!is_x2 && a.ycc) {
    const float4 c = reinterpret_cast<const float4*>(a.ycc + (size_t)t * a.M)[m4];
    acc.x += c.x; acc.y += c.y; acc.z += c.z; acc.w += c.w;
  }
  reinterpret_cast<float4*>(y + (size_t)t * a.M)[m4] = acc;
}

}  // namespace

static int pick_tb(int tb_hint) { return tb_hint <= 1 ? 1 : (tb_hint <= 2 ? 2 : 4); }

hipError_t launch_decode_gateup(const uint16_t* x, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                int max_touched, const WeightView& wv, float* h, int ldh, hipStream_t stream,
                                const FusedRoute* fused_route) {
  if (wv.n_chunks <= 0) return hipSuccess;
  if (wv.q4) {
    if (fused_route) return hipErrorInvalidValue;  // the 4-bit kernels take the assignment from the tables
    return launch_decode_gateup_q4(x, M, plan, tb_hint, expert_sel, x2_only, max_touched, wv, h, ldh, stream);
  }
  dim3 grid(wv.n_chunks * (CHUNK_J / GU_JPB), expert_sel >= 0 ? 1 : max_touched);
  const int tb = pick_tb(tb_hint);
  size_t lds = (size_t)tb * M * 2;
  if (fused_route) {
    const FusedRoute& fr = *fused_route;
    if (fr.T < 1 || fr.T > FUSED_ROUTE_MAX_T || fr.T * fr.k > FUSED_ROUTE_MAX_PAIRS || fr.E > MAX_EXPERTS || x2_only) return hipErrorInvalidValue;
    if (tb == 1) hipLaunchKernelGGL((k_decode_gateup<1, 1>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, fr);
    else if (tb == 2) hipLaunchKernelGGL((k_decode_gateup<2, 1>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, fr);
    else hipLaunchKernelGGL((k_decode_gateup<4, 1>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, fr);
    return hipGetLastError();
  }
  const FusedRoute none{};
  if (tb == 1) hipLaunchKernelGGL((k_decode_gateup<1, 0>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, none);
  else if (tb == 2) hipLaunchKernelGGL((k_decode_gateup<2, 0>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, none);
  else hipLaunchKernelGGL((k_decode_gateup<4, 0>), grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh, none);
  return hipGetLastError();
}

hipError_t launch_decode_down(const float* h, int ldh, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                              int max_touched, const WeightView& wv, int slot0, int chunks_per_slot, float* part,
                              size_t slot_stride, hipStream_t stream) {
  if (wv.n_chunks <= 0) return hipSuccess;
  if (wv.q4)
    return launch_decode_down_q4(h, ldh, M, plan, tb_hint, expert_sel, x2_only, max_touched, wv, slot0, chunks_per_slot, part,
                                 slot_stride, stream);
  int n_slots = (wv.n_chunks + chunks_per_slot - 1) / chunks_per_slot;
  dim3 grid((M + DN_THREADS - 1) / DN_THREADS, n_slots, expert_sel >= 0 ? 1 : max_touched);
  const int tb = pick_tb(tb_hint);
  size_t lds = (size_t)tb * chunks_per_slot * CHUNK_J * sizeof(float);
  if (tb == 1) hipLaunchKernelGGL(k_decode_down<1>, grid, dim3(DN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  else if (tb == 2) hipLaunchKernelGGL(k_decode_down<2>, grid, dim3(DN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  else hipLaunchKernelGGL(k_decode_down<4>, grid, dim3(DN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  return hipGetLastError();
}

hipError_t launch_decode_combine(const DecodeCombineArgs& a, const Plan& plan, float* y, hipStream_t stream) {
  if (a.T <= 0) return hipSuccess;
  dim3 grid((a.M / 4 + 63) / 64, a.T);
  hipLaunchKernelGGL(k_decode_combine, grid, dim3(64), 0, stream, a, plan, y);
  return hipGetLastError();
}

}  // namespace si
