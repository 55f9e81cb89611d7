// Prompt-phase grouped GEMMs on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//   gateup : Hact[row][j] = SiLU(X_e . Wg_e[j]) * (X_e . Wu_e[j])   (FC1 + activation, Eq. 1)
//   down   : Yp[row][m] (+)= Hact[row][:] . Wd_e[:, m]              (FC2, one term of Eq. 2)
//   combine: y[t] = sum_s w[t][s] Yp[row(t,s)] (+ shared expert row) (+ Y^CC for X1 rows)
// Rows are the expert-sorted (token, slot) pairs of the token assignment; a row tile never
// crosses an expert.  The gather of x rows is fused into the A-operand load of the first GEMM.
//
// LDS tiles hold 64 contraction elements (128 bytes) per row; the 16-byte piece c of row r sits
// at piece (c ^ (r & 7)) so that both the 128-bit stores (8 lanes per row) and the 128-bit MFMA
// operand loads (32 rows x 2 pieces per wave) are bank-conflict free.
#include "si_internal.h"

namespace si {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int WAVE = 64;
constexpr int THREADS = 256;
constexpr int BM = PREFILL_BM;  // 128 rows
constexpr int BK = 64;
constexpr int BN2 = 128;        // output columns (m) per block in the down projection

__device__ inline uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ inline float silu_f(float z) { return z / (1.f + __expf(-z)); }

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// swizzled byte offset of 16-byte piece c of row r in a [rows][64] bf16 tile
__device__ inline int swz(int r, int c) { return r * 128 + ((c ^ (r & 7)) << 4); }

// XCD-aware remap: consecutive hardware block ids go round-robin over the 8 XCDs; give each XCD a
// contiguous range of logical ids so that blocks sharing weights share an L2.
__device__ inline int xcd_remap(int b, int total) {
  const int per = (total + 7) / 8;
  return (b % 8) * per + b / 8;
}

struct TileInfo { int e, row0, row_end; };

// logical id L -> (expert, inner index, row tile) with the row tile varying fastest inside an
// expert: L / n_inner indexes the row-tile table, which yields the expert.
__device__ inline bool decode_tile(const Plan& p, int expert_sel, int x2_only, int L, int n_inner, int& inner,
                                   TileInfo& ti) {
  int e, first, nrt, start, end;
  if (expert_sel >= 0) {
    e = expert_sel;
    start = p.off[e] + (x2_only ? p.count1[e] : 0);
    end = p.off[e + 1];
    nrt = (end - start + BM - 1) / BM;
    if (L >= nrt * n_inner) return false;
    first = 0;
  } else {
    const int n_tiles = x2_only ? *p.n_tiles_x2 : *p.n_tiles;
    const int t = L / n_inner;
    if (t >= n_tiles) return false;
    e = x2_only ? p.tile_e_x2[t] : p.tile_e[t];
    if (e >= p.n_routed) return false;
    first = t - (x2_only ? p.tile_r_x2[t] : p.tile_r[t]);
    start = p.off[e] + (x2_only ? p.count1[e] : 0);
    end = p.off[e + 1];
    nrt = (end - start + BM - 1) / BM;
  }
  const int Le = L - first * n_inner;
  inner = Le / nrt;
  const int r = Le % nrt;
  ti.e = e;
  ti.row0 = start + r * BM;
  ti.row_end = end;
  return true;
}

// ---------------------------------------------------------------------------------------------
// FC1 + SwiGLU.  Block: 128 rows x 64 hidden columns (one chunk: 64 gate rows + 64 up rows).
// 4 waves as 2 (rows) x 2 (columns): each wave 64 rows x 32 columns of gate and of up.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(THREADS) void k_prefill_gateup(const uint16_t* __restrict__ x, int M, Plan p,
                                                            int expert_sel, int x2_only, int total_blocks,
                                                            WeightView wv, uint16_t* __restrict__ hact, int ldh) {
  __shared__ __attribute__((aligned(16))) unsigned char s_a[BM * 128];
  __shared__ __attribute__((aligned(16))) unsigned char s_g[CHUNK_J * 128];
  __shared__ __attribute__((aligned(16))) unsigned char s_u[CHUNK_J * 128];
  const int L = xcd_remap(blockIdx.x, total_blocks);
  int cidx;
  TileInfo ti;
  if (!decode_tile(p, expert_sel, x2_only, L, wv.n_chunks, cidx, ti)) return;
  const int tid = threadIdx.x, lane = tid % WAVE, wid = tid / WAVE;
  const int wr = wid >> 1, wc = wid & 1;
  const uint16_t* cbase = wv.base + (size_t)ti.e * wv.expert_stride + (size_t)(wv.chunk0 + cidx) * 3 * CHUNK_J * M;

  // global -> register staging: piece c = tid % 8 of rows tid/8 + 32*i
  const int lc = tid & 7, lr = tid >> 3;
  const uint16_t* a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = ti.row0 + lr + 32 * i;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = x + (size_t)p.row_token[row] * M + lc * 8;
  }
  const uint16_t* g_src = cbase + (size_t)lr * M + lc * 8;
  const uint16_t* u_src = cbase + (size_t)(CHUNK_J + lr) * M + lc * 8;

  f32x16 accg[2], accu[2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) { accg[i][r] = 0.f; accu[i][r] = 0.f; }

  u32x4 ra[4], rg[2], ru[2];
  auto load_tiles = [&](int k0) {
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *reinterpret_cast<const u32x4*>(a_src[i] + k0);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      rg[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(g_src + (size_t)32 * i * M + k0));
      ru[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(u_src + (size_t)32 * i * M + k0));
    }
  };
  load_tiles(0);
  for (int k0 = 0; k0 < M; k0 += BK) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(s_a + swz(lr + 32 * i, lc)) = ra[i];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      *reinterpret_cast<u32x4*>(s_g + swz(lr + 32 * i, lc)) = rg[i];
      *reinterpret_cast<u32x4*>(s_u + swz(lr + 32 * i, lc)) = ru[i];
    }
    __syncthreads();
    if (k0 + BK < M) load_tiles(k0 + BK);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int pc = ks * 2 + (lane >> 5);
      bf16x8 fa[2], fg, fu;
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(s_a + swz(wr * 64 + i * 32 + (lane & 31), pc)));
      fg = as_bf16x8(*reinterpret_cast<const u32x4*>(s_g + swz(wc * 32 + (lane & 31), pc)));
      fu = as_bf16x8(*reinterpret_cast<const u32x4*>(s_u + swz(wc * 32 + (lane & 31), pc)));
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        accg[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fg, accg[i], 0, 0, 0);
        accu[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fu, accu[i], 0, 0, 0);
      }
    }
  }
  // epilogue: element (row 8*(r/4) + 4*(lane/32) + r%4, column lane%32) of each 32x32 tile
  const int col = cidx * CHUNK_J + wv.col0 + wc * 32 + (lane & 31);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int row = ti.row0 + wr * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
      if (row < ti.row_end) hact[(size_t)row * ldh + col] = f32_to_bf16(silu_f(accg[i][r]) * accu[i][r]);
    }
}

// ---------------------------------------------------------------------------------------------
// FC2.  Block: 128 rows x 128 output columns m; contraction over the hidden columns of the launch
// (one chunk = 64 per step).  4 waves as 2 x 2, each 64 x 64.
// B operand: the down block of a chunk is [8 groups][M][8 j], i.e. already "8 consecutive k per
// (group, m)"; the tile is kept in that order in LDS ([group][128 m] x 16 bytes).
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(THREADS) void k_prefill_down(const uint16_t* __restrict__ hact, int ldh, int M, Plan p,
                                                          int expert_sel, int x2_only, int total_blocks, int n_ntiles,
                                                          WeightView wv, float* __restrict__ yp, int accumulate) {
  __shared__ __attribute__((aligned(16))) unsigned char s_a[BM * 128];
  __shared__ __attribute__((aligned(16))) unsigned char s_b[8 * BN2 * 16];
  const int L = xcd_remap(blockIdx.x, total_blocks);
  int nt;
  TileInfo ti;
  if (!decode_tile(p, expert_sel, x2_only, L, n_ntiles, nt, ti)) return;
  const int tid = threadIdx.x, lane = tid % WAVE, wid = tid / WAVE;
  const int wr = wid >> 1, wc = wid & 1;
  const int n0 = nt * BN2;
  const uint16_t* ebase = wv.base + (size_t)ti.e * wv.expert_stride;

  const int lc = tid & 7, lr = tid >> 3;
  const uint16_t* a_src[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int row = ti.row0 + lr + 32 * i;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = hact + (size_t)row * ldh + wv.col0 + lc * 8;
  }
  // B staging: 8 groups x 128 m pieces of 16 bytes; thread handles m = tid % 128, groups tid/128 + 2*i
  const int bn = tid & 127, bg = tid >> 7;
  const int bm_src = min(n0 + bn, M - 1);

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4 ra[4], rb[4];
  auto load_tiles = [&](int c) {
    const uint16_t* dblk = ebase + (size_t)(wv.chunk0 + c) * 3 * CHUNK_J * M + (size_t)2 * CHUNK_J * M;
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *reinterpret_cast<const u32x4*>(a_src[i] + c * CHUNK_J);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      rb[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(dblk + ((size_t)(bg + 2 * i) * M + bm_src) * 8));
  };
  load_tiles(0);
  for (int c = 0; c < wv.n_chunks; ++c) {
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(s_a + swz(lr + 32 * i, lc)) = ra[i];
#pragma unroll
    for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(s_b + ((bg + 2 * i) * BN2 + bn) * 16) = rb[i];
    __syncthreads();
    if (c + 1 < wv.n_chunks) load_tiles(c + 1);
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      const int pc = ks * 2 + (lane >> 5);
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int i = 0; i < 2; ++i)
        fa[i] = as_bf16x8(*reinterpret_cast<const u32x4*>(s_a + swz(wr * 64 + i * 32 + (lane & 31), pc)));
#pragma unroll
      for (int j = 0; j < 2; ++j)
        fb[j] = as_bf16x8(*reinterpret_cast<const u32x4*>(s_b + (pc * BN2 + wc * 64 + j * 32 + (lane & 31)) * 16));
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int m = n0 + wc * 64 + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = ti.row0 + wr * 64 + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < ti.row_end && m < M) {
          float* dst = yp + (size_t)row * M + m;
          *dst = accumulate ? *dst + acc[i][j][r] : acc[i][j][r];
        }
      }
    }
}

__global__ __launch_bounds__(256) void k_prefill_combine(const float* __restrict__ yp, const float* __restrict__ ycc,
                                                         int T, int k, int M, int n_x1, int has_shared, Plan p,
                                                         float* __restrict__ y) {
  const int t = blockIdx.y;
  const int m4 = blockIdx.x * 256 + threadIdx.x;
  if (m4 * 4 >= M) return;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < k; ++s) {
    const float wgt = p.w[t * k + s];
    const float4 v = reinterpret_cast<const float4*>(yp + (size_t)p.inv[t * k + s] * M)[m4];
    acc.x = fmaf(wgt, v.x, acc.x); acc.y = fmaf(wgt, v.y, acc.y);
    acc.z = fmaf(wgt, v.z, acc.z); acc.w = fmaf(wgt, v.w, acc.w);
  }
  if (has_shared) {
    const float4 v = reinterpret_cast<const float4*>(yp + (size_t)(T * k + t) * M)[m4];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  if (ycc && t < n_x1) {
    const float4 v = reinterpret_cast<const float4*>(ycc + (size_t)t * M)[m4];
    acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
  }
  reinterpret_cast<float4*>(y + (size_t)t * M)[m4] = acc;
}

__global__ void k_fill_zero(float* __restrict__ p, size_t n) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n; i += stride) p[i] = 0.f;
}

}  // namespace

hipError_t launch_prefill_gateup(const uint16_t* x, int M, const Plan& plan, int expert_sel, int x2_only,
                                 int n_row_tiles, const WeightView& wv, uint16_t* hact, int ldh,
                                 hipStream_t stream) {
  if (wv.n_chunks <= 0 || n_row_tiles <= 0) return hipSuccess;
  const int total = n_row_tiles * wv.n_chunks;
  hipLaunchKernelGGL(k_prefill_gateup, dim3((total + 7) / 8 * 8), dim3(THREADS), 0, stream, x, M, plan, expert_sel,
                     x2_only, (total + 7) / 8 * 8, wv, hact, ldh);
  return hipGetLastError();
}

hipError_t launch_prefill_down(const uint16_t* hact, int ldh, int M, const Plan& plan, int expert_sel, int x2_only,
                               int n_row_tiles, const WeightView& wv, float* yp, int accumulate,
                               hipStream_t stream) {
  if (wv.n_chunks <= 0 || n_row_tiles <= 0) return hipSuccess;
  const int n_ntiles = (M + BN2 - 1) / BN2;
  const int total = n_row_tiles * n_ntiles;
  hipLaunchKernelGGL(k_prefill_down, dim3((total + 7) / 8 * 8), dim3(THREADS), 0, stream, hact, ldh, M, plan,
                     expert_sel, x2_only, (total + 7) / 8 * 8, n_ntiles, wv, yp, accumulate);
  return hipGetLastError();
}

hipError_t launch_prefill_combine(const float* yp, const float* ycc, int T, int k, int M, int n_x1, int has_shared,
                                  const Plan& plan, float* y, hipStream_t stream) {
  if (T <= 0) return hipSuccess;
  dim3 grid((M / 4 + 255) / 256, T);
  hipLaunchKernelGGL(k_prefill_combine, grid, dim3(256), 0, stream, yp, ycc, T, k, M, n_x1, has_shared, plan, y);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  int blocks = (int)std::min<size_t>((n + 255) / 256, 4096);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

}  // namespace si
