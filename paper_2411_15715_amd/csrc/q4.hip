// Kernels for the 4-bit storage form of the weights (codes 0..15 standing for (code - 8) * scale, bf16 group
// scales; chunk layout in cc_worker.h).
//   k_decode_gateup_q4 / k_decode_down_q4 : the generation-phase GEMVs straight from the codes (fp32, exact
//       products; 4x fewer weight bytes than bf16, so the integer unpacking has to stay below ~2 VALU
//       operations per weight for the kernels to remain bound by HBM)
//   k_dequant_q4 : codes -> bf16 chunks (the layout the MFMA GEMMs read), piece by piece, for the prompt phase
#include "si_internal.h"

namespace si {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
constexpr int WAVE = 64;
constexpr int QGU_THREADS = 256;
constexpr int QGU_JPW = 4;                                   // hidden columns per wave
constexpr int QGU_JPB = QGU_JPW * (QGU_THREADS / WAVE);      // per block (16)
constexpr int QDN_THREADS = 256;

__device__ inline float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ inline float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ inline float bf16_f32(uint16_t b) { return __uint_as_float((uint32_t)b << 16); }
__device__ inline float silu_f(float z) { return z / (1.f + __expf(-z)); }

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, WAVE);
  return v;
}

// expert handled by this block and its row range; false when there is nothing to do
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

// sum over the 32 weights of one 16-byte load of x[m] * (128 + code[m]): the pair (codes 2p, 2p+1) of a word is
// (word >> 4p) & 0x000F000F; putting 0x4300 into the other bits of both halves makes the two bf16 values
// 128 + code (exact: bf16 has 8 significant bits), and one dot-product instruction multiplies them with the bf16
// pair of x.  mask / magic arrive in registers so that select-bits-and-merge is one bit-field-insert
// instruction: shift, insert, dot product = 3 operations per 2 weights.
__device__ inline float dot_codes(const u32x4& w, const uint32_t* xv, uint32_t mask, uint32_t magic) {
  float d = 0.f;
  const uint32_t ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int pp = 0; pp < 4; ++pp) {
      const uint32_t sh = ws[i] >> (4 * pp);
      uint32_t pair;  // (mask & sh) | (~mask & magic)
      asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(pair) : "v"(mask), "v"(sh), "s"(magic));
      d = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), __builtin_bit_cast(bf16x2, xv[i * 4 + pp]), d, false);
    }
  return d;
}

// h[row][j] = SiLU(x . Wg[j]) * (x . Wu[j]) with W = (code - 8) * scale:
//   x . W[j] = sum over groups of 64 m of scale * ( sum x (128 + code) - 136 * sum x ).
// A lane owns 32 consecutive m of a row per pass (one 16-byte load per row), i.e. half a scale group.
template <int TB>
__global__ __launch_bounds__(QGU_THREADS) void k_decode_gateup_q4(const uint16_t* __restrict__ x, int M, Plan p,
                                                                  int expert_sel, int x2_only, WeightView wv,
                                                                  float* __restrict__ h, int ldh) {
  extern __shared__ uint32_t s_xq[];  // [TB][M/2] bf16 pairs of x
  int e, r0, r1;
  if (!block_rows(p, expert_sel, x2_only, blockIdx.y, e, r0, r1)) return;
  const int tid = threadIdx.x, lane = tid % WAVE, wid = tid / WAVE;
  const int M2 = M / 2, M32 = M / 32, MG = M / 64;
  constexpr int blocks_per_chunk = CHUNK_J / QGU_JPB;
  const int chunk = wv.chunk0 + blockIdx.x / blocks_per_chunk;
  const int jj0 = (blockIdx.x % blocks_per_chunk) * QGU_JPB + wid * QGU_JPW;
  int se;
  if (!storage_index(wv, e, se)) return;
  const unsigned char* cb = reinterpret_cast<const unsigned char*>(wv.base + (size_t)se * wv.expert_stride + (size_t)chunk * q4_chunk_u16(M));
  const u32x4* gq = reinterpret_cast<const u32x4*>(cb + q4_off_codes(0, M));
  const u32x4* uq = reinterpret_cast<const u32x4*>(cb + q4_off_codes(1, M));
  const uint16_t* gs = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(0, M));
  const uint16_t* us = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(1, M));
  const int jcol = wv.col0 + (blockIdx.x / blocks_per_chunk) * CHUNK_J + jj0;
  const u32x4* gp = gq + (size_t)jj0 * M32;
  const u32x4* up = uq + (size_t)jj0 * M32;
  const uint16_t* gsp = gs + (size_t)jj0 * MG;
  const uint16_t* usp = us + (size_t)jj0 * MG;
  u32x4 wg[QGU_JPW], wu[QGU_JPW];
  float sg[QGU_JPW], su[QGU_JPW];
  auto load_w = [&](int slot) {
#pragma unroll
    for (int j = 0; j < QGU_JPW; ++j) {
      wg[j] = __builtin_nontemporal_load(gp + j * M32 + slot);
      wu[j] = __builtin_nontemporal_load(up + j * M32 + slot);
      sg[j] = bf16_f32(gsp[j * MG + (slot >> 1)]);
      su[j] = bf16_f32(usp[j * MG + (slot >> 1)]);
    }
  };

  for (int rb = r0; rb < r1; rb += TB) {
    const int nt = min(TB, r1 - rb);
    __syncthreads();
    for (int i = tid; i < nt * (M2 / 4); i += QGU_THREADS) {
      const int tb = i / (M2 / 4), c = i % (M2 / 4);
      const int tok = p.row_token[rb + tb];
      reinterpret_cast<u32x4*>(s_xq)[tb * (M2 / 4) + c] = reinterpret_cast<const u32x4*>(x + (size_t)tok * M)[c];
    }
    __syncthreads();
    float ag[QGU_JPW][TB], au[QGU_JPW][TB];
#pragma unroll
    for (int j = 0; j < QGU_JPW; ++j)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) { ag[j][tb] = 0.f; au[j][tb] = 0.f; }
    // constants kept out of the optimiser's sight (see dot_codes)
    uint32_t mask = 0x000F000Fu, magic = 0x43004300u, ones = 0x3F803F80u;
    asm volatile("" : "+v"(mask), "+s"(magic), "+s"(ones));
    for (int slot = lane; slot < M32; slot += WAVE) {
      load_w(slot);
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          uint32_t xv[16];
          const u32x4* xs4 = reinterpret_cast<const u32x4*>(s_xq + tb * M2 + slot * 16);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const u32x4 v = xs4[i];
            xv[4 * i] = v.x; xv[4 * i + 1] = v.y; xv[4 * i + 2] = v.z; xv[4 * i + 3] = v.w;
          }
          float xsum = 0.f;  // sum of the lane's 32 x values: pairs times (1, 1)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            xsum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, xv[i]), __builtin_bit_cast(bf16x2, ones), xsum, false);
          const float off = 136.f * xsum;
#pragma unroll
          for (int j = 0; j < QGU_JPW; ++j) {
            ag[j][tb] = fmaf(sg[j], dot_codes(wg[j], xv, mask, magic) - off, ag[j][tb]);
            au[j][tb] = fmaf(su[j], dot_codes(wu[j], xv, mask, magic) - off, au[j][tb]);
          }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < QGU_JPW; ++j)
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          const float g = wave_sum(ag[j][tb]);
          const float u = wave_sum(au[j][tb]);
          if (lane == 0) h[(size_t)(rb + tb) * ldh + jcol + j] = silu_f(g) * u;
        }
      }
  }
}

// part[slot][row][m] = sum over the chunks of the slot of scale_c[m] * ( sum_j h_j code[j][m] - 8 * sum_j h_j ).
// One thread per output column; a chunk's 64 codes of a column are two 16-byte loads.
template <int TB>
__global__ __launch_bounds__(QDN_THREADS) void k_decode_down_q4(const float* __restrict__ h, int ldh, int M, Plan p,
                                                                int expert_sel, int x2_only, WeightView wv, int slot0,
                                                                int chunks_per_slot, float* __restrict__ part,
                                                                size_t slot_stride) {
  int e, r0, r1;
  if (!block_rows(p, expert_sel, x2_only, blockIdx.z, e, r0, r1)) return;
  const int s = blockIdx.y;
  const int c_begin = s * chunks_per_slot;
  const int c_end = min(c_begin + chunks_per_slot, wv.n_chunks);
  if (c_begin >= c_end) return;
  const int m = blockIdx.x * QDN_THREADS + threadIdx.x;
  const bool active = m < M;
  const int mm = active ? m : 0;
  const int NW = ntile_width(M);
  int se;
  if (!storage_index(wv, e, se)) return;
  const uint16_t* ebase = wv.base + (size_t)se * wv.expert_stride;
  float* out = part + (size_t)(slot0 + s) * slot_stride;

  extern __shared__ float s_hq[];  // [TB][n_j] activations of this slot, then [TB][n_c] their sums per chunk
  const int n_c = c_end - c_begin, n_j = n_c * CHUNK_J;
  float* s_sum = s_hq + TB * n_j;
  const int jbase = wv.col0 + c_begin * CHUNK_J;

  for (int rb = r0; rb < r1; rb += TB) {
    const int nt = min(TB, r1 - rb);
    __syncthreads();
    for (int i = threadIdx.x; i < nt * n_j; i += QDN_THREADS) {
      const int tb = i / n_j, j = i % n_j;
      s_hq[tb * n_j + j] = h[(size_t)(rb + tb) * ldh + jbase + j];
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nt * n_c; i += QDN_THREADS) {
      const int tb = i / n_c, c = i % n_c;
      float a = 0.f;
      for (int j = 0; j < CHUNK_J; ++j) a += s_hq[tb * n_j + c * CHUNK_J + j];
      s_sum[tb * n_c + c] = a;
    }
    __syncthreads();
    float acc[TB];
#pragma unroll
    for (int tb = 0; tb < TB; ++tb) acc[tb] = 0.f;
    for (int c = c_begin; c < c_end; ++c) {
      const unsigned char* cb = reinterpret_cast<const unsigned char*>(ebase + (size_t)(wv.chunk0 + c) * q4_chunk_u16(M));
      const u32x4* dq = reinterpret_cast<const u32x4*>(cb + q4_off_codes(2, M));
      const size_t i0 = ((size_t)(mm / NW) * 2) * NW + (mm % NW);
      const u32x4 w0 = __builtin_nontemporal_load(dq + i0), w1 = __builtin_nontemporal_load(dq + i0 + NW);
      const float sd = bf16_f32(reinterpret_cast<const uint16_t*>(cb + q4_off_scales(2, M))[mm]);
      const uint32_t ws[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
#pragma unroll
      for (int tb = 0; tb < TB; ++tb) {
        if (tb < nt) {
          const float4* hr = reinterpret_cast<const float4*>(s_hq + tb * n_j + (c - c_begin) * CHUNK_J);
          float a = 0.f;
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const uint32_t lo = ws[q] & 0x0F0F0F0Fu, hi = (ws[q] >> 4) & 0x0F0F0F0Fu;
            const float4 h0 = hr[q * 2], h1 = hr[q * 2 + 1];
            a = fmaf(h0.x, (float)(lo & 0xffu), a); a = fmaf(h0.y, (float)((lo >> 8) & 0xffu), a);
            a = fmaf(h0.z, (float)((lo >> 16) & 0xffu), a); a = fmaf(h0.w, (float)(lo >> 24), a);
            a = fmaf(h1.x, (float)(hi & 0xffu), a); a = fmaf(h1.y, (float)((hi >> 8) & 0xffu), a);
            a = fmaf(h1.z, (float)((hi >> 16) & 0xffu), a); a = fmaf(h1.w, (float)(hi >> 24), a);
          }
          acc[tb] = fmaf(sd, a - 8.f * s_sum[tb * n_c + (c - c_begin)], acc[tb]);
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

__device__ inline uint32_t pack_bf16x2(float a, float b) {
  uint32_t ua = __float_as_uint(a), ub = __float_as_uint(b);
  ua += 0x7fffu + ((ua >> 16) & 1u);  // round to nearest even
  ub += 0x7fffu + ((ub >> 16) & 1u);
  return (ua >> 16) | (ub & 0xffff0000u);
}

// 4-bit chunks [c0, c0+n) of the selected experts -> bf16 chunks 0..n of `dst` (expert e at dst + e*dst_estride),
// value = bf16((code - 8) * scale).  One thread per 32-bit word of codes (8 weights -> one 16-byte store).
// grid: (n * 24, experts): 8 blocks of work per gate block, 8 per up block, 8 per down block of a chunk.
__global__ __launch_bounds__(256) void k_dequant_q4(const uint16_t* __restrict__ src, size_t src_estride,
                                                    const int32_t* __restrict__ e_map, int c0, int M, Plan p,
                                                    int expert_sel, int x2_only, uint16_t* __restrict__ dst,
                                                    size_t dst_estride) {
  int e, de;
  if (expert_sel >= 0) {
    e = expert_sel;
    de = 0;
  } else {
    e = blockIdx.y;
    de = e;
    if (e >= p.n_routed) return;
  }
  if (p.off[e + 1] - p.off[e] - (x2_only ? p.count1[e] : 0) <= 0) return;  // no rows: nobody reads these weights
  const int se = e_map ? e_map[e] : e;
  if (se < 0) return;
  const int c = blockIdx.x / 24, sec = (blockIdx.x % 24) / 8, oct = blockIdx.x % 8;
  const unsigned char* cb = reinterpret_cast<const unsigned char*>(src + (size_t)se * src_estride + (size_t)(c0 + c) * q4_chunk_u16(M));
  uint16_t* ob = dst + (size_t)de * dst_estride + (size_t)c * 3 * CHUNK_J * M + (size_t)sec * CHUNK_J * M;
  const uint32_t* q = reinterpret_cast<const uint32_t*>(cb + q4_off_codes(sec, M));
  const uint16_t* z = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(sec, M));
  float v[8];
  if (sec < 2) {
    // rows oct*8 .. oct*8+7 of the gate / up block; destination [M/PW panels][64 j][PW m]
    const int PW = panel_width(M), M8 = M / 8;
    for (int i = threadIdx.x; i < 8 * M8; i += 256) {
      const int j = oct * 8 + i / M8, m0 = (i % M8) * 8;
      const uint32_t w = q[(size_t)j * M8 + m0 / 8];
      const float sc = bf16_f32(z[(size_t)j * (M / 64) + m0 / 64]);
#pragma unroll
      for (int el = 0; el < 8; ++el) v[el] = (float)((int)((w >> (4 * q4_fc1_nibble(el))) & 15u) - 8) * sc;
      const uint4 o = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
      *reinterpret_cast<uint4*>(ob + gu_off(j, m0, PW)) = o;
    }
  } else {
    // j = oct*8 .. oct*8+7 of the down block for every column m; destination [M/NW][8 q][NW m][8 i]
    const int NW = ntile_width(M);
    for (int m = threadIdx.x; m < M; m += 256) {
      const uint32_t w = q[q4_fc2_word(oct * 8, m, NW)];
      const float sc = bf16_f32(z[m]);
#pragma unroll
      for (int el = 0; el < 8; ++el) v[el] = (float)((int)((w >> (4 * q4_fc2_nibble(el))) & 15u) - 8) * sc;
      const uint4 o = make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
      *reinterpret_cast<uint4*>(ob + dn_off(oct * 8, m, NW)) = o;
    }
  }
}

int pick_tb(int tb_hint) { return tb_hint <= 1 ? 1 : (tb_hint <= 2 ? 2 : 4); }

}  // namespace

hipError_t launch_decode_gateup_q4(const uint16_t* x, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                   int max_touched, const WeightView& wv, float* h, int ldh, hipStream_t stream) {
  if (wv.n_chunks <= 0) return hipSuccess;
  dim3 grid(wv.n_chunks * (CHUNK_J / QGU_JPB), expert_sel >= 0 ? 1 : max_touched);
  const int tb = pick_tb(tb_hint);
  const size_t lds = (size_t)tb * M * 2;
  if (tb == 1) hipLaunchKernelGGL(k_decode_gateup_q4<1>, grid, dim3(QGU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
  else if (tb == 2) hipLaunchKernelGGL(k_decode_gateup_q4<2>, grid, dim3(QGU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
  else hipLaunchKernelGGL(k_decode_gateup_q4<4>, grid, dim3(QGU_THREADS), lds, stream, x, M, plan, expert_sel, x2_only, wv, h, ldh);
  return hipGetLastError();
}

hipError_t launch_decode_down_q4(const float* h, int ldh, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                 int max_touched, const WeightView& wv, int slot0, int chunks_per_slot, float* part,
                                 size_t slot_stride, hipStream_t stream) {
  if (wv.n_chunks <= 0) return hipSuccess;
  const int n_slots = (wv.n_chunks + chunks_per_slot - 1) / chunks_per_slot;
  dim3 grid((M + QDN_THREADS - 1) / QDN_THREADS, n_slots, expert_sel >= 0 ? 1 : max_touched);
  int tb = pick_tb(tb_hint);
  size_t lds = (size_t)tb * chunks_per_slot * (CHUNK_J + 1) * sizeof(float);
  while (lds > 65536 && tb > 1) {  // stay inside the default dynamic LDS limit: fewer tokens per weight pass
    tb >>= 1;
    lds = (size_t)tb * chunks_per_slot * (CHUNK_J + 1) * sizeof(float);
  }
  if (tb == 1) hipLaunchKernelGGL(k_decode_down_q4<1>, grid, dim3(QDN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  else if (tb == 2) hipLaunchKernelGGL(k_decode_down_q4<2>, grid, dim3(QDN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  else hipLaunchKernelGGL(k_decode_down_q4<4>, grid, dim3(QDN_THREADS), lds, stream, h, ldh, M, plan, expert_sel, x2_only, wv, slot0, chunks_per_slot, part, slot_stride);
  return hipGetLastError();
}

hipError_t launch_dequant_q4(const WeightView& wv, int M, const Plan& plan, int expert_sel, int x2_only, int n_experts,
                             uint16_t* dst, size_t dst_estride, hipStream_t stream) {
  if (wv.n_chunks <= 0) return hipSuccess;
  dim3 grid(wv.n_chunks * 24, expert_sel >= 0 ? 1 : n_experts);
  hipLaunchKernelGGL(k_dequant_q4, grid, dim3(256), 0, stream, wv.base, wv.expert_stride, wv.e_map, wv.chunk0, M, plan,
                     expert_sel, x2_only, dst, dst_estride);
  return hipGetLastError();
}

}  // namespace si
