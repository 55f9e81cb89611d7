// Generation-phase expert GEMV (few tokens per expert): bandwidth-bound streaming of bf16 weights
// with fp32 accumulation.  Three kernels per part:
//   gateup : h[row][j] = SiLU(x . Wg[j]) * (x . Wu[j])         (FC1 + activation, Eq. 1)
//   down   : part[slot][row][m] = sum_{j in slot} h[row][j] Wd[j][m]   (FC2, one term of Eq. 2)
//   combine: y[t] = sum_s w[t][s] sum_slots part[..][row(t,s)] (+ shared expert, + Y^CC)
// Every weight byte is read once per pass of up to DECODE_TB tokens, with 128-bit loads that are
// contiguous across the lanes of a wave.
#include "si_internal.h"

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

template <int TB>
__global__ __launch_bounds__(GU_THREADS) void k_decode_gateup(const uint16_t* __restrict__ x, int M, Plan p,
                                                              int expert_sel, int x2_only, WeightView wv,
                                                              float* __restrict__ h, int ldh) {
  extern __shared__ u32x4 s_x[];  // [TB][M/8] bf16 x 8
  int e, r0, r1;
  if (!block_rows(p, expert_sel, x2_only, blockIdx.y, e, r0, r1)) return;
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

  for (int rb = r0; rb < r1; rb += TB) {
    const int nt = min(TB, r1 - rb);
    __syncthreads();
    for (int i = tid; i < nt * M8; i += GU_THREADS) {
      int tb = i / M8, c = i % M8;
      int tok = p.row_token[rb + tb];
      s_x[tb * M8 + c] = reinterpret_cast<const u32x4*>(x + (size_t)tok * M)[c];
    }
    __syncthreads();
    float ag[GU_JPW][TB], au[GU_JPW][TB];
#pragma unroll
    for (int j = 0; j < GU_JPW; ++j)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) { ag[j][tb] = 0.f; au[j][tb] = 0.f; }
    for (int c = lane; c < M8; c += WAVE) {
      u32x4 wg[GU_JPW], wu[GU_JPW];
      const size_t poff = (size_t)(c / PW8) * CHUNK_J * PW8 + (c % PW8);  // panel base + position in the row segment
#pragma unroll
      for (int j = 0; j < GU_JPW; ++j) {
        wg[j] = __builtin_nontemporal_load(gblk + poff + (size_t)(jj0 + j) * PW8);
        wu[j] = __builtin_nontemporal_load(ublk + poff + (size_t)(jj0 + j) * PW8);
      }
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
      float4 tmp[DOWN_SLOTS];
#pragma unroll
      for (int q = 0; q < DOWN_SLOTS; ++q)
        tmp[q] = q < n_part[part] ? reinterpret_cast<const float4*>(base + (size_t)q * a.slot_stride)[m4]
                                  : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
      for (int q = 0; q < DOWN_SLOTS; ++q) { v.x += tmp[q].x; v.y += tmp[q].y; v.z += tmp[q].z; v.w += tmp[q].w; }
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
                                int max_touched, const WeightView& wv, float* h, int ldh, hipStream_t stream) {
  if (wv.n_chunks <= 0) return hipSuccess;
  if (wv.q4) return launch_decode_gateup_q4(x, M, plan, tb_hint, expert_sel, x2_only, max_touched, wv, h, ldh, stream);
  dim3 grid(wv.n_chunks * (CHUNK_J / GU_JPB), expert_sel >= 0 ? 1 : max_touched);
  const int tb = pick_tb(tb_hint);
  size_t lds = (size_t)tb * M * 2;
  if (tb == 1) hipLaunchKernelGGL(k_decode_gateup<1>, grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
  else if (tb == 2) hipLaunchKernelGGL(k_decode_gateup<2>, grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
  else hipLaunchKernelGGL(k_decode_gateup<4>, grid, dim3(GU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
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
