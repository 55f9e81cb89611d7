// Prompt-phase grouped GEMMs on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16), fp32 accumulate.
//   gateup : Hact[row][j] = SiLU(X_e . Wg_e[j]) * (X_e . Wu_e[j])   (FC1 + activation, Eq. 1)
//   down   : Yp[row][m] (+)= Hact[row][:] . Wd_e[:, m]              (FC2, one term of Eq. 2)
//   combine: y[t] = sum_s w[t][s] Yp[row(t,s)] (+ shared expert row) (+ Y^CC for X1 rows)
// Rows are the expert-sorted (token, slot) pairs of the token assignment; a row tile never
// crosses an expert.  The gather of x rows is fused into the A-operand load of the first GEMM.
//
// Both GEMMs: one 512-thread block (8 waves, 2 per SIMD) per BM x 256 output tile, BK = 64, a ring of LDS
// stages filled by direct global->LDS loads (global_load_lds_dwordx4, no VGPR staging), wave tile
// (BM/2) x 64.  A row tile holds up to 256 rows, the last one of an expert up to 320 (si_internal.h: n_row_tiles);
// the block runs the body instantiated for BM = 64, 128, 192, 256 or 320, the smallest that covers the rows the
// tile really has.
// LDS rows hold 64 contraction elements (128 bytes); the 16-byte piece c of row r sits at piece
// c ^ ((r >> 1) & 7): gfx950's LDS has 64 banks, so 16 consecutive rows x 16 bytes must cover 256
// distinct bytes of bank space for the 128-bit MFMA operand reads to be conflict free (measured:
// SQ_LDS_BANK_CONFLICT = 0).
#include "si_internal.h"

namespace si {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define SI_GPTR(p) ((const void __attribute__((address_space(1)))*)(p))
#define SI_LPTR(p) ((void __attribute__((address_space(3)))*)(p))

constexpr int WAVE = 64;
constexpr int THREADS = 512;
constexpr int BN = 256;  // B rows per tile: 128 hidden columns (gate+up) or 256 output columns
constexpr int BK = 64;
constexpr int B_BYTES = BN * BK * 2;  // 32 KB
constexpr int KERNEL_LDS = 144 * 1024;  // the largest body

// Body shapes.  With few rows the GEMM only streams its weights: the smaller A tiles then leave LDS for a
// deeper ring of stages, i.e. more weight bytes in flight per CU.
template <int BM> struct Shape {
  static constexpr int NST = BM >= 192 ? 2 : 3;           // LDS stages
  static constexpr int STAGE = BM * 128 + B_BYTES;        // bytes per stage
  static constexpr int LDS = NST * STAGE;                 // 120, 144, 112, 128, 144 KB for BM = 64, 128, 192, 256, 320
  static constexpr int FA = BM / 64;                      // A fragments (32 rows each) per wave
  static constexpr int ALD = BM / 64;                     // A load instructions per wave per stage
  static constexpr int LPW = ALD + 4;                     // load instructions per wave per stage
  // Invariant behind every wait_vmcnt<N> of the main loops: between two barriers a wave issues exactly these
  // vector-memory instructions, in program order, and no others (no spill, no hoisted table load: everything a
  // loop needs from global memory besides the tiles is fetched before it starts).  ensure_lds_attr() refuses a
  // build whose kernels use scratch memory, and the GPU tests run every body with fewer, as many and more k-tiles
  // than stages.
};

// Ring shapes of the streaming loop, which tiles of at most 192 rows run.  Such a tile is latency bound, not
// matrix-core bound: what it needs is weight bytes in flight, and the LDS ring above holds at most two k-tiles
// of them (64 KB per CU; the chip needs about 25 MB in flight to saturate its HBM, i.e. 100 KB per CU).  Here only
// the A operand keeps a ring of DA stages in LDS; the B operand (the weights) travels through registers, R = DA - 1
// k-tiles of it in flight per wave, and is written into one of two B stages in LDS one iteration before it is read.
template <int BM> struct StreamShape {
  static constexpr int DA = BM <= 64 ? 6 : BM <= 128 ? 5 : 3;  // A stages = prefetch distance in k-tiles
  static constexpr int R = DA - 1;                              // register sets holding B tiles in flight
  static constexpr int A_STAGE = BM * 128;
  static constexpr int B0 = DA * A_STAGE;                       // offset of the two B stages
  static constexpr int LDS = B0 + 2 * B_BYTES;                  // 112, 144, 136 KB for BM = 64, 128, 192
  static constexpr int GL = 4;                                  // B register loads per wave and k-tile
  static constexpr int ALD = BM / 64;                           // A load instructions per wave and k-tile
  // waits of the steady state: a wave issues, per k-tile and in this order, GL register loads (B) and ALD
  // direct-to-LDS loads (A); younger than B of tile t+1 are A of tile t+1 and the tiles t+2 .. t+DA-1
  static constexpr int WAIT_B = (DA - 2) * (GL + ALD) + ALD;
  static constexpr int WAIT_A = (DA - 2) * (GL + ALD);
  static_assert(LDS <= KERNEL_LDS && WAIT_B < 64, "ring does not fit");
};

__device__ inline uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ inline float silu_f(float z) { return z / (1.f + __expf(-z)); }

__device__ inline bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// swizzled byte offset of 16-byte piece c of row r in a [rows][64] bf16 tile
__device__ inline int swz(int r, int c) { return r * 128 + ((c ^ ((r >> 1) & 7)) << 4); }

// s_waitcnt vmcnt(n) only (lgkmcnt / expcnt untouched); n < 64
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 0xf) | (((N >> 4) & 3) << 14));
}

__device__ inline void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xc07f); }  // lgkmcnt(0) only

// Workgroup barrier WITHOUT the memory fence of __syncthreads(): the fence would drain every outstanding
// global->LDS load (s_waitcnt vmcnt(0)) and so defeat the multi-stage ring.  What has to be visible
// after the barrier is (a) each wave's own direct-to-LDS loads of the tile about to be read, which the
// wave itself waited for with wait_vmcnt<> just before, and (b) nothing else: fragments read from the
// slot about to be refilled were consumed by MFMAs earlier in program order.
__device__ inline void block_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Hardware block id -> logical tile id.
//  * XCD-aware remap: consecutive hardware block ids go round-robin over the 8 XCDs; give each XCD a
//    contiguous range of logical ids so that the row tiles that read the same weights share an L2.  The
//    ranges are cut from the number of ids that really have work (known on the device only), so that no
//    XCD is handed a range of empty ids (with ranges cut from the grid's upper bound the remap cost more than
//    it saved on small tiles: the last XCD idled while the others carried its share).
//    When no expert of the launch has more than one row tile nothing is shared through the L2 but the few rows
//    of x, and tiles of different experts differ in cost (a 192-row tile streams its weights a quarter slower than
//    a 128-row one): the ids are then dealt round-robin (`interleave`), every XCD gets the same mix, and the launch
//    takes the mean of the experts' times instead of the slowest XCD's.
//  * Tail split: N tiles on n_cu compute units run in ceil(N / n_cu) rounds; when the last round is at most
//    half full each of its tiles gets two blocks, which share its rows if it has more than 128 (LLaMA-shaped
//    gate/up GEMM: 896 tiles = 3.5 rounds; the last round then costs about half a round).
__device__ inline bool map_block(int b, int N, int n_cu, int interleave, int& L, int& half, int& halves) {
  int r = N % n_cu;
  if (2 * r > n_cu) r = 0;
  const int main_n = N - r;
  const int per = (main_n + 7) / 8;
  if (b < 8 * per) {
    L = interleave ? b : (b % 8) * per + b / 8;
    half = 0;
    halves = 1;
    return L < main_n;
  }
  const int bt = b - 8 * per;
  if (bt >= 2 * r) return false;
  L = main_n + (bt >> 1);
  half = bt & 1;
  halves = 2;
  return true;
}

// se: index of the expert inside the launch's weight storage; solo: the tile holds all rows of its expert, so
// nobody else reads its weight tiles (they come from HBM, not from a sibling's trail in the L2)
struct TileInfo { int e, row0, row_end, se, solo; };

// Number of logical tile ids with work in this launch (row tiles x inner tiles); single: no expert of the launch
// has more than one row tile.
__device__ inline int launch_extent(const Plan& p, int expert_sel, int x2_only, int n_inner, int& single) {
  if (expert_sel >= 0) {
    const int start = p.off[expert_sel] + (x2_only ? p.count1[expert_sel] : 0);
    const int nrt = n_row_tiles(p.off[expert_sel + 1] - start);
    single = nrt <= 1;
    return nrt * n_inner;
  }
  single = (*p.tile_flags >> (x2_only ? 1 : 0)) & 1;
  return (x2_only ? *p.n_tiles_x2 : *p.n_tiles) * n_inner;  // row tiles of the routed experts
}

// logical id L -> (expert, inner index, row tile) with the row tile varying fastest inside an
// expert: L / n_inner indexes the row-tile table, which yields the expert.
__device__ inline bool decode_tile(const Plan& p, int expert_sel, int x2_only, int L, int n_inner, int& inner,
                                   TileInfo& ti) {
  int e, first, nrt, start, end;
  if (expert_sel >= 0) {
    e = expert_sel;
    start = p.off[e] + (x2_only ? p.count1[e] : 0);
    end = p.off[e + 1];
    nrt = n_row_tiles(end - start);
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
    nrt = n_row_tiles(end - start);
  }
  const int Le = L - first * n_inner;
  inner = Le / nrt;
  const int r = Le % nrt;
  ti.e = e;
  ti.row0 = start + r * TILE_ROWS;
  ti.row_end = r == nrt - 1 ? end : ti.row0 + TILE_ROWS;
  ti.solo = nrt == 1;
  return true;
}

// block id -> tile of this block (false: nothing to do)
// spread: deal single-tile launches round-robin over the XCDs (see map_block)
__device__ inline bool block_tile(const Plan& p, int expert_sel, int x2_only, int n_inner, int n_cu, int spread,
                                  int& inner, TileInfo& ti) {
  int L, half, halves, single;
  const int extent = launch_extent(p, expert_sel, x2_only, n_inner, single);
  if (!map_block(blockIdx.x, extent, n_cu, single && spread, L, half, halves)) return false;
  if (!decode_tile(p, expert_sel, x2_only, L, n_inner, inner, ti)) return false;
  if (halves == 2) {
    const int rows = ti.row_end - ti.row0;
    if (rows <= 128) return half == 0;  // too few rows to share: the first block takes them all
    ti.solo = 0;
    const int hs = ((rows + 1) / 2 + 31) / 32 * 32;
    ti.row0 += half * hs;
    ti.row_end = min(ti.row_end, ti.row0 + hs);
    if (ti.row0 >= ti.row_end) return false;
  }
  return true;
}

// ---------------------------------------------------------------------------------------------
// The two GEMM kernels share their main loop.  8 waves as 2 (rows) x 4 (B-row quarters of 64);
// wave tile (BM/2) x 64: FA A-fragments x 2 B-fragments of v_mfma_f32_32x32x16_bf16.
// Ring of NST stages holding k-tiles it .. it+NST-1.  The one barrier of an iteration sits before
// its last k-step: by then every fragment of stage `st` is in registers, so after the barrier the
// stage is refilled (tile it+NST) and the first fragments of the next stage are fetched while the
// last 8 MFMAs of this iteration run; the wait before the barrier leaves the NST-2 youngest tiles in
// flight.
// ---------------------------------------------------------------------------------------------
// accumulators, operand fragments and the two lambdas every variant of the main loop uses
#define SI_GEMM_DECLS(BFRAG_OFF)                                                                                 \
  f32x16 acc[S::FA][2];                                                                                          \
  _Pragma("unroll") for (int i = 0; i < S::FA; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j)                \
      _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;                                         \
  bf16x8 fa[2][S::FA], fb[2][2];                                                                                 \
  auto ldfrag = [&](int stage, int ks, int buf) {                                                                \
    const unsigned char* sa = lds + stage * S::STAGE;                                                            \
    const unsigned char* sb = sa + BM * 128;                                                                     \
    const int pc = ks * 2 + (lane >> 5);                                                                         \
    _Pragma("unroll") for (int i = 0; i < S::FA; ++i) fa[buf][i] = as_bf16x8(                                    \
        *reinterpret_cast<const u32x4*>(sa + swz(wr * (BM / 2) + i * 32 + (lane & 31), pc)));                    \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) fb[buf][j] = as_bf16x8(                                        \
        *reinterpret_cast<const u32x4*>(sb + BFRAG_OFF(wc * 64 + j * 32 + (lane & 31), pc)));                    \
  };                                                                                                             \
  auto mma = [&](int buf) {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < S::FA; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j)              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);         \
  };

// register loads and the dependency tie used by the loops whose B operand travels through registers
__device__ inline void gload_b128(u32x4& q, const void* p) {
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q) : "v"(p) : "memory");
}
__device__ inline void gload_u16(uint32_t& z, const void* p) {
  asm volatile("global_load_ushort %0, %1, off" : "=v"(z) : "v"(p) : "memory");
}
struct BRegs { u32x4 q[4]; };  // one lane's share of a bf16 B tile
__device__ inline void bready(BRegs& r) { asm volatile("" : "+v"(r.q[0]), "+v"(r.q[1]), "+v"(r.q[2]), "+v"(r.q[3])::"memory"); }

#define SI_GEMM_MAIN_LOOP(NK, ISSUE)                                                                  \
  {                                                                                                              \
    const int nk_ = (NK);                                                                                        \
    _Pragma("unroll") for (int s0 = 0; s0 < S::NST; ++s0) if (s0 < nk_) ISSUE(s0, s0);                           \
    if (S::NST - 1 < nk_) wait_vmcnt<(S::NST - 1) * S::LPW>(); else wait_vmcnt<0>();                             \
    block_barrier();                                                                                             \
    ldfrag(0, 0, 0);                                                                                             \
    int st = 0;                                                                                                  \
    for (int it = 0; it < nk_; ++it) {                                                                           \
      const int nx = st + 1 == S::NST ? 0 : st + 1;                                                              \
      ldfrag(st, 1, 1); mma(0);                                                                                  \
      ldfrag(st, 2, 0); mma(1);                                                                                  \
      ldfrag(st, 3, 1); mma(0);                                                                                  \
      /* tile it+1 must have landed for every wave and every read of stage st must be complete before the   */   \
      /* barrier: after it stage nx is read and stage st is refilled with tile it+NST                       */   \
      if (it + S::NST - 1 < nk_) wait_vmcnt<(S::NST - 2) * S::LPW>(); else wait_vmcnt<0>();                      \
      wait_lgkmcnt0();                                                                                           \
      block_barrier();                                                                                           \
      if (it + 1 < nk_) ldfrag(nx, 0, 0);                                                                        \
      if (it + S::NST < nk_) ISSUE(st, it + S::NST);                                                             \
      __builtin_amdgcn_s_setprio(1);                                                                             \
      mma(1);                                                                                                    \
      __builtin_amdgcn_s_setprio(0);                                                                             \
      st = nx;                                                                                                   \
    }                                                                                                            \
  }

struct Q4Regs { u32x4 q; uint32_t z; };  // codes and scale of one lane's share of a B tile

// The streaming loop (StreamShape).  ISSUE_A(a_stage, kt): direct-to-LDS loads of A tile kt; BLOAD(kt, regs): register
// loads of B tile kt; BSTORE(b_stage, regs, i): 16-byte LDS store of the i-th of them.  Iteration `it` computes tile
// `it` (A stage it % DA, B stage it % 2), writes B of tile it+1 (fetched DA-1 iterations earlier) into the other B
// stage between its matrix instructions, and after its barrier fetches tile it+DA into the A stage and the register
// set it has just released.  The loop is unrolled by R so that every register set is named statically.  Near the end
// of the contraction (fewer than DA-1 tiles ahead) the hand-counted waits no longer hold and the loop drains instead.
#define SI_GEMM_DECLS_STREAM(BFRAG_OFF)                                                                          \
  using SS = StreamShape<BM>;                                                                                    \
  f32x16 acc[S::FA][2];                                                                                          \
  _Pragma("unroll") for (int i = 0; i < S::FA; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j)                \
      _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;                                         \
  bf16x8 fa[2][S::FA], fb[2][2];                                                                                 \
  auto ldfrag = [&](int sta, int stb, int ks, int buf) {                                                         \
    const unsigned char* sa = lds + sta * SS::A_STAGE;                                                           \
    const unsigned char* sb = lds + SS::B0 + stb * B_BYTES;                                                      \
    const int pc = ks * 2 + (lane >> 5);                                                                         \
    _Pragma("unroll") for (int i = 0; i < S::FA; ++i) fa[buf][i] = as_bf16x8(                                    \
        *reinterpret_cast<const u32x4*>(sa + swz(wr * (BM / 2) + i * 32 + (lane & 31), pc)));                    \
    _Pragma("unroll") for (int j = 0; j < 2; ++j) fb[buf][j] = as_bf16x8(                                        \
        *reinterpret_cast<const u32x4*>(sb + BFRAG_OFF(wc * 64 + j * 32 + (lane & 31), pc)));                    \
  };                                                                                                             \
  auto mma = [&](int buf) {                                                                                      \
    _Pragma("unroll") for (int i = 0; i < S::FA; ++i) _Pragma("unroll") for (int j = 0; j < 2; ++j)              \
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);         \
  };

#define SI_GEMM_MAIN_LOOP_STREAM(NK, ISSUE_A, BLOAD, BSTORE)                                                     \
  {                                                                                                              \
    const int nk_ = (NK);                                                                                        \
    BRegs rs[SS::R];                                                                                             \
    /* tile 0 goes straight through; then the tiles 1 .. DA-1 are set off */                                     \
    BLOAD(0, rs[0]); ISSUE_A(0, 0);                                                                              \
    wait_vmcnt<SS::ALD>(); bready(rs[0]);                                                                        \
    _Pragma("unroll") for (int i = 0; i < 4; ++i) BSTORE(0, rs[0], i);                                           \
    _Pragma("unroll") for (int t = 1; t < SS::DA; ++t) if (t < nk_) { BLOAD(t, rs[t % SS::R]); ISSUE_A(t, t); }  \
    if (SS::DA - 1 < nk_) wait_vmcnt<(SS::DA - 1) * (SS::GL + SS::ALD)>(); else wait_vmcnt<0>(); /* A of tile 0 */ \
    wait_lgkmcnt0();                                                                                             \
    block_barrier();                                                                                             \
    ldfrag(0, 0, 0, 0);                                                                                          \
    int sta = 0;                                                                                                 \
    auto step = [&](int it, BRegs& rc) { /* rc: B of tile it+1 */                                                \
      const int stb = it & 1;                                                                                    \
      const int nsta = sta + 1 == SS::DA ? 0 : sta + 1;                                                          \
      const bool full = it + SS::DA - 1 < nk_; /* the tiles it+1 .. it+DA-1 have all been set off */             \
      const bool more = it + 1 < nk_;                                                                            \
      ldfrag(sta, stb, 1, 1); mma(0);                                                                            \
      if (full) wait_vmcnt<SS::WAIT_B>(); else wait_vmcnt<0>();                                                  \
      bready(rc);                                                                                                \
      if (more) BSTORE(stb ^ 1, rc, 0);                                                                          \
      ldfrag(sta, stb, 2, 0); mma(1);                                                                            \
      if (more) BSTORE(stb ^ 1, rc, 1);                                                                          \
      ldfrag(sta, stb, 3, 1); mma(0);                                                                            \
      if (more) { BSTORE(stb ^ 1, rc, 2); BSTORE(stb ^ 1, rc, 3); }                                              \
      /* A of tile it+1 landed, B of tile it+1 written, every read of the two stages complete */                 \
      if (full) wait_vmcnt<SS::WAIT_A>(); else wait_vmcnt<0>();                                                  \
      wait_lgkmcnt0();                                                                                           \
      block_barrier();                                                                                           \
      if (more) ldfrag(nsta, stb ^ 1, 0, 0);                                                                     \
      if (it + SS::DA < nk_) { BLOAD(it + SS::DA, rc); ISSUE_A(sta, it + SS::DA); }                              \
      __builtin_amdgcn_s_setprio(1);                                                                             \
      mma(1);                                                                                                    \
      __builtin_amdgcn_s_setprio(0);                                                                             \
      sta = nsta;                                                                                                \
    };                                                                                                           \
    for (int it = 0; it < nk_; it += SS::R) {                                                                    \
      _Pragma("unroll") for (int u = 0; u < SS::R; ++u) if (it + u < nk_) step(it + u, rs[(u + 1) % SS::R]);     \
    }                                                                                                            \
  }


// The same loop for weights in the 4-bit storage form.  The A operand still arrives by direct global->LDS loads;
// the B operand cannot (it has to be turned into bf16 on the way), so every lane fetches 16 bytes of codes (32
// weights) and their group scale into registers one iteration ahead (BLOAD), and turns them into four 16-byte
// pieces of bf16((code - 8) * scale) that it writes into the stage freed by the previous iteration's barrier,
// one piece after each k-step's matrix instructions (BCONV), so that the conversion arithmetic runs under the
// matrix core's work.  A k-tile of 64 is one scale group of either projection.
// Order of the vector-memory operations of a wave, which the wait counts rely on: iteration j issues the
// register loads of tile j+NST (GL instructions, at the top of the iteration) and, after its barrier, the A loads
// of tile j+NST (ALD instructions).  The register loads are inline assembly and their waits explicit: with
// direct-to-LDS loads in flight the compiler's own wait before the first use of a loaded register is vmcnt(0),
// which would drain the ring every iteration; BREADY ties the registers to the explicit wait so that no use is
// scheduled above it.
#define SI_GEMM_MAIN_LOOP_REGB(NK, GLN, BREGS, ISSUE_A, BLOAD, BREADY, BCONV)                                    \
  {                                                                                                              \
    constexpr int GL = (GLN); /* register loads per B tile and lane */                                           \
    const int nk_ = (NK);                                                                                        \
    BREGS ra, rb;                                                                                                \
    _Pragma("unroll") for (int s0 = 0; s0 < S::NST; ++s0) if (s0 < nk_) ISSUE_A(s0, s0);                         \
    _Pragma("unroll") for (int s0 = 0; s0 < S::NST - 1; ++s0) if (s0 < nk_) {                                    \
      BLOAD(s0, ra);                                                                                             \
      wait_vmcnt<0>();                                                                                           \
      BREADY(ra);                                                                                                \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) BCONV(s0, ra, i);                                            \
    }                                                                                                            \
    BLOAD(min(S::NST - 1, nk_ - 1), ra);                                                                         \
    wait_vmcnt<0>();                                                                                             \
    BREADY(ra);                                                                                                  \
    wait_lgkmcnt0();                                                                                             \
    block_barrier();                                                                                             \
    ldfrag(0, 0, 0);                                                                                             \
    int st = 0;                                                                                                  \
    /* one iteration; the registers it converts are rc, those it fetches go to rn: the loop below            */ \
    /* alternates two register sets, so that no fetched register is copied while its load is in flight        */ \
    auto step = [&](int it, BREGS& rc, BREGS& rn) {                                                              \
      const int nx = st + 1 == S::NST ? 0 : st + 1;                                                              \
      const int pv = st == 0 ? S::NST - 1 : st - 1;                                                              \
      const bool fill = it + S::NST - 1 < nk_; /* B of tile it+NST-1 goes into stage pv during this iteration */ \
      /* always issued (index clamped), so that the wait below sees the same number of younger operations */     \
      BLOAD(min(it + S::NST, nk_ - 1), rn);                                                                      \
      ldfrag(st, 1, 1); mma(0);                                                                                  \
      /* rc was fetched at the top of the previous iteration; younger: that iteration's A loads, the          */ \
      /* fetch above.  Past the last tile the conversion runs on whatever the clamped fetch brought and      */ \
      /* writes a stage nobody reads again: straight-line code, so that the scheduler can place the          */ \
      /* conversion arithmetic between the matrix instructions                                               */ \
      wait_vmcnt<S::ALD + GL>(); BREADY(rc); BCONV(pv, rc, 0);                                                   \
      ldfrag(st, 2, 0); mma(1); BCONV(pv, rc, 1);                                                                \
      ldfrag(st, 3, 1); mma(0); BCONV(pv, rc, 2); BCONV(pv, rc, 3);                                              \
      /* the A loads of tile it+1 must have landed, the B pieces written above and every read of stage st  */    \
      /* must be complete before the barrier; younger than those A loads are the operations of NST-2 whole  */    \
      /* iterations and this iteration's register loads                                                     */    \
      if (fill) wait_vmcnt<(S::NST - 2) * (S::ALD + GL) + GL>(); else wait_vmcnt<0>();                           \
      wait_lgkmcnt0();                                                                                           \
      block_barrier();                                                                                           \
      if (it + 1 < nk_) ldfrag(nx, 0, 0);                                                                        \
      if (it + S::NST < nk_) ISSUE_A(st, it + S::NST);                                                           \
      __builtin_amdgcn_s_setprio(1);                                                                             \
      mma(1);                                                                                                    \
      __builtin_amdgcn_s_setprio(0);                                                                             \
      st = nx;                                                                                                   \
    };                                                                                                           \
    for (int it = 0; it < nk_; it += 2) {                                                                        \
      step(it, ra, rb);                                                                                          \
      if (it + 1 < nk_) step(it + 1, rb, ra);                                                                    \
    }                                                                                                            \
  }

// 16-byte LDS store the compiler does not see as one: with a direct-to-LDS load in flight it would otherwise wait
// for ALL vector-memory operations (vmcnt(0)) before any LDS store it cannot prove disjoint from the load's
// target, which would drain the ring every iteration.  Disjointness is by construction here (the stage written is
// not the target of any load in flight), and completion is covered by the loop's own lgkmcnt(0) before each barrier.
__device__ inline void lds_store_b128(unsigned char* p, const u32x4& v) {
  const uint32_t a = (uint32_t)(uintptr_t)SI_LPTR(p);
  asm volatile("ds_write_b128 %0, %1" ::"v"(a), "v"(v) : "memory");
}

// Eight 4-bit codes (as two words of four byte-sized codes each: `lo` holds elements a0 a1 a2 a3 in its bytes
// 0..3 for the byte order given by the caller) -> bf16((code - 8) * scale), exact product, one rounding.
// s8 = -8 * scale.
__device__ inline uint32_t q4_pair(uint32_t bytes, int b0, int b1, float sc, float s8) {
  // (the compiler turns byte extraction + conversion into one v_cvt_f32_ubyteN)
  const float c0 = (float)((bytes >> (8 * b0)) & 0xffu), c1 = (float)((bytes >> (8 * b1)) & 0xffu);
  typedef float f32x2 __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  const f32x2 v = {__builtin_fmaf(c0, sc, s8), __builtin_fmaf(c1, sc, s8)};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));  // round to nearest even
}

#define SI_BOFF_SWZ(row, pc) swz((row), (pc))
#define SI_BOFF_K8(col, pc) (((pc) * BN + (col)) * 16)

// ---------------------------------------------------------------------------------------------
// FC1 + SwiGLU.  Tile: BM rows x 128 hidden columns (two chunks).  B rows in LDS are ordered so
// that wave column wc owns hidden columns [32 wc, 32 wc + 32): LDS B row = wc*64 + f*32 + jj with
// f = 0 the gate row and f = 1 the up row of column 32 wc + jj; SiLU(gate)*up is then formed in
// registers from the two accumulator tiles of a wave.
// ---------------------------------------------------------------------------------------------
template <int BM, bool STREAM>
__device__ __forceinline__ void gateup_body(const uint16_t* __restrict__ x, int M, const Plan& p, int tc, const TileInfo& ti,
                                            const WeightView& wv, uint16_t* __restrict__ hact, int ldh,
                                            unsigned char* lds) {
  using S = Shape<BM>;
  const int tid = threadIdx.x, lane = tid % WAVE, w = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wave index, known to be uniform
  const int wr = w >> 2, wc = w & 3;
  const uint16_t* ebase = wv.base + (size_t)ti.se * wv.expert_stride;

  // loader: a wave instruction fills 8 LDS rows (1 KB); lane/8 is the row, lane%8 the slot inside the
  // 128-byte row, which holds logical piece slot ^ ((row >> 1) & 7)
  const int lrow = lane >> 3, lpp = lane & 7;
  uint32_t a_src[S::ALD];  // element offsets from x (the host checks that x spans less than 2^31 elements)
#pragma unroll
  for (int i = 0; i < S::ALD; ++i) {
    const int lr = w * (BM / 8) + i * 8 + lrow;  // LDS row of the A tile
    int row = ti.row0 + lr;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = (uint32_t)p.row_token[row] * (uint32_t)M + ((lpp ^ ((lr >> 1) & 7)) * 8);
  }
  // B: LDS row w*32 + i*8 + lrow  ->  chunk 2*tc + w/4, f = w%2 (gate / up block), column-in-chunk
  // jc = ((w/2)%2)*32 + i*8 + lrow.  Blocks are [M/PW panels][64 j][PW m] (cc_worker.h).
  const int chunk_rel = min(2 * tc + (w >> 2), wv.n_chunks - 1);
  const uint16_t* b_blk = ebase + (size_t)(wv.chunk0 + chunk_rel) * 3 * CHUNK_J * M + (size_t)(w & 1) * CHUNK_J * M;
  const int jc0 = ((w >> 1) & 1) * 32 + lrow;
  const int PW = panel_width(M);
  const int lc0 = lpp ^ (lrow >> 1);  // B piece for even i; odd i uses lc0 ^ 4

  auto issue = [&](int stage, int kt) {
    unsigned char* sa = lds + stage * S::STAGE + w * (BM / 8) * 128;
    unsigned char* sb = lds + stage * S::STAGE + BM * 128 + w * 4096;
    const int k0 = kt * BK;
#pragma unroll
    for (int i = 0; i < S::ALD; ++i)
      __builtin_amdgcn_global_load_lds(SI_GPTR(x + (a_src[i] + (uint32_t)k0)), SI_LPTR(sa + i * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int m0 = k0 + (((i & 1) ? (lc0 ^ 4) : lc0) * 8);
      __builtin_amdgcn_global_load_lds(SI_GPTR(b_blk + ((size_t)(m0 / PW) * CHUNK_J + jc0 + i * 8) * PW + (m0 % PW)),
                                       SI_LPTR(sb + i * 1024), 16, 0, 0);
    }
  };
  // epilogue: element (row 8*(r/4) + 4*(lane/32) + r%4, column lane%32) of each 32x32 tile;
  // acc[i][0] is the gate tile and acc[i][1] the up tile of the same 32 hidden columns
  auto epilogue = [&](const f32x16 (&acc)[S::FA][2]) {
    const int jl = wc * 32 + (lane & 31);  // hidden column inside the 128-column tile
    if (2 * tc + (jl >> 6) < wv.n_chunks) {
      const int col = wv.col0 + tc * 128 + jl;
#pragma unroll
      for (int i = 0; i < S::FA; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = ti.row0 + wr * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < ti.row_end) hact[(size_t)row * ldh + col] = f32_to_bf16(silu_f(acc[i][0][r]) * acc[i][1][r]);
        }
    }
  };
  if constexpr (STREAM) {
    // the same loads, with B through registers: lane (lrow, lpp) of instruction i fetches the piece that the
    // direct load would have put at byte lane * 16 of the wave's KB i, and stores it there
    auto issue_a = [&](int sta, int kt) {
      unsigned char* sa = lds + sta * StreamShape<BM>::A_STAGE + w * (BM / 8) * 128;
#pragma unroll
      for (int i = 0; i < S::ALD; ++i)
        __builtin_amdgcn_global_load_lds(SI_GPTR(x + (a_src[i] + (uint32_t)(kt * BK))), SI_LPTR(sa + i * 1024), 16, 0, 0);
    };
    auto bload = [&](int kt, BRegs& r) {
      const int k0 = kt * BK;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int m0 = k0 + (((i & 1) ? (lc0 ^ 4) : lc0) * 8);
        gload_b128(r.q[i], b_blk + ((size_t)(m0 / PW) * CHUNK_J + jc0 + i * 8) * PW + (m0 % PW));
      }
    };
    auto bstore = [&](int stb, const BRegs& r, int i) {
      lds_store_b128(lds + StreamShape<BM>::B0 + stb * B_BYTES + w * 4096 + i * 1024 + lane * 16, r.q[i]);
    };
    SI_GEMM_DECLS_STREAM(SI_BOFF_SWZ)
    SI_GEMM_MAIN_LOOP_STREAM(M / BK, issue_a, bload, bstore)
    epilogue(acc);
  } else {
    SI_GEMM_DECLS(SI_BOFF_SWZ)
    SI_GEMM_MAIN_LOOP(M / BK, issue)
    epilogue(acc);
  }
}

// A block picks the body for the rows its tile really has (whole-block branch), so a 40-row tile costs a 64-row
// body and a 140-row tile a 192-row one.  The 320-row body (five A fragments per wave, 144 KB of LDS, every one of
// the 256 registers a wave may have at two waves per SIMD) exists for the last tile of an expert only.  A tile that
// holds all rows of its expert, at most 192, runs the streaming loop (StreamShape): its weights come from HBM.
// (Two spellings of the same choice: with the 320-row body at the very limit of the register file, the order of the
// tests decides where the compiler places what several bodies have in common, and each kernel has one order that
// leaves it without a spill; ensure_lds_attr() refuses a build that has one.)
#define SI_PICK_BODY_GU(ti, CALL)                               \
  {                                                             \
    const int rows_ = (ti).row_end - (ti).row0;                 \
    if (rows_ <= 64) CALL(64, true);                            \
    else if ((ti).solo && rows_ <= 192) {                       \
      if (rows_ <= 128) CALL(128, true);                        \
      else CALL(192, true);                                     \
    } else if (rows_ <= 128) CALL(128, false);                  \
    else if (rows_ <= 192) CALL(192, false);                    \
    else if (rows_ <= 256) CALL(256, false);                    \
    else CALL(320, false);                                      \
  }
#define SI_PICK_BODY_DN(ti, CALL)                               \
  {                                                             \
    const int rows_ = (ti).row_end - (ti).row0;                 \
    if (rows_ > 256) CALL(320, false);                          \
    else if (rows_ > 192) CALL(256, false);                     \
    else if (rows_ <= 64) CALL(64, true);                       \
    else if ((ti).solo) {                                       \
      if (rows_ <= 128) CALL(128, true);                        \
      else CALL(192, true);                                     \
    } else if (rows_ <= 128) CALL(128, false);                  \
    else CALL(192, false);                                      \
  }
// The 4-bit bodies stop at 256 rows (their B operand passes through registers, which leaves no room for a fifth
// A fragment): the rows a last tile holds beyond 256 take a second pass of the same block.  No wave still reads
// the LDS ring when a body returns (its last barrier follows every fragment read), so the next pass may refill it.
#define SI_PICK_BODY_2PASS(ti, CALL)                                  \
  for (const int row_end_all_ = (ti).row_end;;) {                     \
    (ti).row_end = min(row_end_all_, (ti).row0 + TILE_ROWS);          \
    const int rows_ = (ti).row_end - (ti).row0;                       \
    if (rows_ <= 64) CALL(64);                                        \
    else if (rows_ <= 128) CALL(128);                                 \
    else if (rows_ <= 192) CALL(192);                                 \
    else CALL(256);                                                   \
    if ((ti).row_end >= row_end_all_) break;                          \
    (ti).row0 = (ti).row_end;                                         \
  }

__global__ __launch_bounds__(THREADS, 1) void k_prefill_gateup(const uint16_t* __restrict__ x, int M, Plan p,
                                                               int expert_sel, int x2_only, int n_cu,
                                                               int n_ctiles, WeightView wv,
                                                               uint16_t* __restrict__ hact, int ldh) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  int tc;
  TileInfo ti;
  if (!block_tile(p, expert_sel, x2_only, n_ctiles, n_cu, 1, tc, ti)) return;
  if (!storage_index(wv, ti.e, ti.se)) return;
#define SI_CALL_GU(BMV, ST) gateup_body<BMV, ST>(x, M, p, tc, ti, wv, hact, ldh, lds)
  SI_PICK_BODY_GU(ti, SI_CALL_GU)
#undef SI_CALL_GU
}

// ---------------------------------------------------------------------------------------------
// FC2.  Tile: BM rows x 256 output columns m; contraction over the hidden columns of this
// k-split's chunk range (one chunk = 64 per step).  B operand: the down block of a chunk is
// [8 groups][M][8 j], i.e. already "8 consecutive k per (group, m)"; it is kept in that order in
// LDS ([group][256 m] x 16 bytes), read conflict free by consecutive lanes.
// Output slab `split` of yp: rows x M fp32; overwritten or accumulated.
// ---------------------------------------------------------------------------------------------
template <int BM, bool STREAM>
__device__ __forceinline__ void down_body(const uint16_t* __restrict__ hact, int ldh, int M, int inner, const TileInfo& ti,
                                          int n_ntiles, int n_split, const WeightView& wv, float* __restrict__ yp,
                                          size_t slab_stride, int accumulate, unsigned char* lds) {
  using S = Shape<BM>;
  const int nt = inner % n_ntiles, split = inner / n_ntiles;
  const int c_begin = (int)((long)wv.n_chunks * split / n_split), c_end = (int)((long)wv.n_chunks * (split + 1) / n_split);
  if (c_begin >= c_end && accumulate) return;  // nothing to add
  const int tid = threadIdx.x, lane = tid % WAVE, w = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wave index, known to be uniform
  const int wr = w >> 2, wc = w & 3;
  const int n0 = nt * BN;
  const uint16_t* ebase = wv.base + (size_t)ti.se * wv.expert_stride;
  float* out = yp + (size_t)split * slab_stride;

  const int lrow = lane >> 3, lpp = lane & 7;
  uint32_t a_src[S::ALD];  // element offsets from hact (the host checks that it spans less than 2^31 elements)
#pragma unroll
  for (int i = 0; i < S::ALD; ++i) {
    const int lr = w * (BM / 8) + i * 8 + lrow;
    int row = ti.row0 + lr;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = (uint32_t)row * (uint32_t)ldh + wv.col0 + ((lpp ^ ((lr >> 1) & 7)) * 8);
  }
  // B: wave w loads group q = w of the chunk's down block ([M/NW tiles][8 q][NW m][8 i]), 4 x 64 output columns
  const int NW = ntile_width(M);
  const int nw_shift = __builtin_ctz(NW);
  uint32_t b_off[4];  // inside one chunk's down block: below 64 * M elements
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int n = min(n0 + i * 64 + lane, M - 1);
    b_off[i] = (((uint32_t)(n >> nw_shift) * 8 + w) * NW + (n & (NW - 1))) * 8;  // NW is a power of two
  }

  auto issue = [&](int stage, int kt) {
    unsigned char* sa = lds + stage * S::STAGE + w * (BM / 8) * 128;
    unsigned char* sb = lds + stage * S::STAGE + BM * 128 + w * 4096;
    const int c = c_begin + kt;
    const uint16_t* dblk = ebase + (size_t)(wv.chunk0 + c) * 3 * CHUNK_J * M + (size_t)2 * CHUNK_J * M;
#pragma unroll
    for (int i = 0; i < S::ALD; ++i)
      __builtin_amdgcn_global_load_lds(SI_GPTR(hact + (a_src[i] + (uint32_t)(c * CHUNK_J))), SI_LPTR(sa + i * 1024), 16, 0, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i)
      __builtin_amdgcn_global_load_lds(SI_GPTR(dblk + b_off[i]), SI_LPTR(sb + i * 1024), 16, 0, 0);
  };
  auto epilogue = [&](const f32x16 (&acc)[S::FA][2]) {
    // (the lane index is made opaque here so that the output addresses are formed after the main loop: formed
    // ahead of it they are live through it, which the 320-row body has no registers for)
    int el = lane;
    asm volatile("" : "+v"(el));
#pragma unroll
    for (int i = 0; i < S::FA; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = n0 + wc * 64 + j * 32 + (el & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = ti.row0 + wr * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (el >> 5) + (r & 3);
          if (row < ti.row_end && m < M) {
            float* dst = out + (size_t)row * M + m;
            *dst = accumulate ? *dst + acc[i][j][r] : acc[i][j][r];
          }
        }
      }
  };
  if (c_begin < c_end) {
    if constexpr (STREAM) {
      auto issue_a = [&](int sta, int kt) {
        unsigned char* sa = lds + sta * StreamShape<BM>::A_STAGE + w * (BM / 8) * 128;
#pragma unroll
        for (int i = 0; i < S::ALD; ++i)
          __builtin_amdgcn_global_load_lds(SI_GPTR(hact + (a_src[i] + (uint32_t)((c_begin + kt) * CHUNK_J))), SI_LPTR(sa + i * 1024), 16, 0, 0);
      };
      auto bload = [&](int kt, BRegs& r) {
        const uint16_t* dblk = ebase + (size_t)(wv.chunk0 + c_begin + kt) * 3 * CHUNK_J * M + (size_t)2 * CHUNK_J * M;
#pragma unroll
        for (int i = 0; i < 4; ++i) gload_b128(r.q[i], dblk + b_off[i]);
      };
      auto bstore = [&](int stb, const BRegs& r, int i) {
        lds_store_b128(lds + StreamShape<BM>::B0 + stb * B_BYTES + w * 4096 + i * 1024 + lane * 16, r.q[i]);
      };
      SI_GEMM_DECLS_STREAM(SI_BOFF_K8)
      SI_GEMM_MAIN_LOOP_STREAM(c_end - c_begin, issue_a, bload, bstore)
      epilogue(acc);
    } else {
      SI_GEMM_DECLS(SI_BOFF_K8)
      SI_GEMM_MAIN_LOOP(c_end - c_begin, issue)
      epilogue(acc);
    }
  } else {
    // an empty k-split of an overwriting launch still has to define its slab
    for (int i = tid; i < BM * BN; i += THREADS) {
      const int row = ti.row0 + i / BN, m = n0 + i % BN;
      if (row < ti.row_end && m < M) out[(size_t)row * M + m] = 0.f;
    }
  }
}

__global__ __launch_bounds__(THREADS, 1) void k_prefill_down(const uint16_t* __restrict__ hact, int ldh, int M, Plan p,
                                                             int expert_sel, int x2_only, int n_cu,
                                                             int n_ntiles, int n_split, WeightView wv,
                                                             float* __restrict__ yp, size_t slab_stride,
                                                             int accumulate) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  int inner;
  TileInfo ti;
  // (XCD ranges also when every expert has a single row tile: one expert's Hact rows, the A operand, a few MB,
  // then stay in one L2; dealt round-robin every XCD re-reads every expert's rows for each of its column tiles,
  // which measured 3 % slower although the XCDs finish together)
  if (!block_tile(p, expert_sel, x2_only, n_ntiles * n_split, n_cu, 0, inner, ti)) return;
  if (!storage_index(wv, ti.e, ti.se)) return;
#define SI_CALL_DN(BMV, ST) down_body<BMV, ST>(hact, ldh, M, inner, ti, n_ntiles, n_split, wv, yp, slab_stride, accumulate, lds)
  SI_PICK_BODY_DN(ti, SI_CALL_DN)
#undef SI_CALL_DN
}

// ---------------------------------------------------------------------------------------------
// The same two GEMMs on weights in the 4-bit storage form (chunk layout in cc_worker.h), converted on the way
// into the B stage.  Tiles, LDS layouts, fragment reads, matrix instructions and epilogues are those above.
// ---------------------------------------------------------------------------------------------
template <int BM>
__device__ __forceinline__ void gateup_body_q4(const uint16_t* __restrict__ x, int M, const Plan& p, int tc, const TileInfo& ti,
                                               const WeightView& wv, uint16_t* __restrict__ hact, int ldh,
                                               unsigned char* lds) {
  using S = Shape<BM>;
  const int tid = threadIdx.x, lane = tid % WAVE, w = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wave index, known to be uniform
  const int wr = w >> 2, wc = w & 3;
  const unsigned char* ebase = reinterpret_cast<const unsigned char*>(wv.base + (size_t)ti.se * wv.expert_stride);

  const int lrow = lane >> 3, lpp = lane & 7;
  const uint16_t* a_src[S::ALD];
#pragma unroll
  for (int i = 0; i < S::ALD; ++i) {
    const int lr = w * (BM / 8) + i * 8 + lrow;
    int row = ti.row0 + lr;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = x + (size_t)p.row_token[row] * M + ((lpp ^ ((lr >> 1) & 7)) * 8);
  }
  auto issue_a = [&](int stage, int kt) {
    unsigned char* sa = lds + stage * S::STAGE + w * (BM / 8) * 128;
#pragma unroll
    for (int i = 0; i < S::ALD; ++i)
      __builtin_amdgcn_global_load_lds(SI_GPTR(a_src[i] + kt * BK), SI_LPTR(sa + i * 1024), 16, 0, 0);
  };
  // B: wave w fills LDS rows [32 w, 32 w + 32) = (chunk 2*tc + w/4, gate (w even) or up block, columns
  // ((w/2)%2)*32 .. +31 of the chunk); lane = (row lane/2, k-half lane%2): the 32 weights of its half row are
  // 16 bytes of codes, i.e. the pieces 4*(lane%2) .. +3 of the LDS row
  const int chunk_rel = min(2 * tc + (w >> 2), wv.n_chunks - 1);
  const unsigned char* cb = ebase + (size_t)(wv.chunk0 + chunk_rel) * q4_chunk_u16(M) * 2;
  const int jc = ((w >> 1) & 1) * 32 + (lane >> 1), kh = lane & 1;
  const unsigned char* qrow = cb + q4_off_codes(w & 1, M) + (size_t)jc * (M / 2) + kh * 16;
  const uint16_t* zrow = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(w & 1, M)) + (size_t)jc * (M / 64);
  const int brow = w * 32 + (lane >> 1);
  const int bsw = (brow >> 1) & 7;
  auto bload = [&](int kt, Q4Regs& r) {
    gload_b128(r.q, qrow + (size_t)kt * 32);
    gload_u16(r.z, zrow + kt);
  };
  auto bready = [&](Q4Regs& r) { asm volatile("" : "+v"(r.q), "+v"(r.z)::"memory"); };
  // word i of the lane's codes = elements 8i .. 8i+7 of its half row; even nibbles hold elements 0 4 1 5, odd
  // nibbles 2 6 3 7 (cc_worker.h)
  auto bconv = [&](int stage, const Q4Regs& r, int i) {
    const float sc = __uint_as_float(r.z << 16), s8 = -8.f * sc;
    const uint32_t wd = r.q[i], ev = wd & 0x0f0f0f0fu, od = (wd >> 4) & 0x0f0f0f0fu;
    u32x4 o;
    o.x = q4_pair(ev, 0, 2, sc, s8);
    o.y = q4_pair(od, 0, 2, sc, s8);
    o.z = q4_pair(ev, 1, 3, sc, s8);
    o.w = q4_pair(od, 1, 3, sc, s8);
    lds_store_b128(lds + stage * S::STAGE + BM * 128 + brow * 128 + (((kh * 4 + i) ^ bsw) << 4), o);
  };
  SI_GEMM_DECLS(SI_BOFF_SWZ)
  SI_GEMM_MAIN_LOOP_REGB(M / BK, 2, Q4Regs, issue_a, bload, bready, bconv)
  const int jl = wc * 32 + (lane & 31);
  if (2 * tc + (jl >> 6) < wv.n_chunks) {
    const int col = wv.col0 + tc * 128 + jl;
#pragma unroll
    for (int i = 0; i < S::FA; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = ti.row0 + wr * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row < ti.row_end) hact[(size_t)row * ldh + col] = f32_to_bf16(silu_f(acc[i][0][r]) * acc[i][1][r]);
      }
  }
}

__global__ __launch_bounds__(THREADS, 1) void k_prefill_gateup_q4(const uint16_t* __restrict__ x, int M, Plan p,
                                                                  int expert_sel, int x2_only, int n_cu,
                                                                  int n_ctiles, WeightView wv,
                                                                  uint16_t* __restrict__ hact, int ldh) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  int tc;
  TileInfo ti;
  if (!block_tile(p, expert_sel, x2_only, n_ctiles, n_cu, 1, tc, ti)) return;
  if (!storage_index(wv, ti.e, ti.se)) return;
#define SI_CALL_GU(BMV) gateup_body_q4<BMV>(x, M, p, tc, ti, wv, hact, ldh, lds)
  SI_PICK_BODY_2PASS(ti, SI_CALL_GU);
#undef SI_CALL_GU
}

template <int BM>
__device__ __forceinline__ void down_body_q4(const uint16_t* __restrict__ hact, int ldh, int M, int inner, const TileInfo& ti,
                                             int n_ntiles, int n_split, const WeightView& wv, float* __restrict__ yp,
                                             size_t slab_stride, int accumulate, unsigned char* lds) {
  using S = Shape<BM>;
  const int nt = inner % n_ntiles, split = inner / n_ntiles;
  const int c_begin = (int)((long)wv.n_chunks * split / n_split), c_end = (int)((long)wv.n_chunks * (split + 1) / n_split);
  if (c_begin >= c_end && accumulate) return;
  const int tid = threadIdx.x, lane = tid % WAVE, w = __builtin_amdgcn_readfirstlane(tid / WAVE);  // wave index, known to be uniform
  const int wr = w >> 2, wc = w & 3;
  const int n0 = nt * BN;
  const unsigned char* ebase = reinterpret_cast<const unsigned char*>(wv.base + (size_t)ti.se * wv.expert_stride);
  float* out = yp + (size_t)split * slab_stride;

  const int lrow = lane >> 3, lpp = lane & 7;
  const uint16_t* a_src[S::ALD];
#pragma unroll
  for (int i = 0; i < S::ALD; ++i) {
    const int lr = w * (BM / 8) + i * 8 + lrow;
    int row = ti.row0 + lr;
    row = row < ti.row_end ? row : ti.row_end - 1;
    a_src[i] = hact + (size_t)row * ldh + wv.col0 + ((lpp ^ ((lr >> 1) & 7)) * 8);
  }
  auto issue_a = [&](int stage, int kt) {
    unsigned char* sa = lds + stage * S::STAGE + w * (BM / 8) * 128;
#pragma unroll
    for (int i = 0; i < S::ALD; ++i)
      __builtin_amdgcn_global_load_lds(SI_GPTR(a_src[i] + (c_begin + kt) * CHUNK_J), SI_LPTR(sa + i * 1024), 16, 0, 0);
  };
  // B: thread = (output column n0 + (w%4)*64 + lane, j-half w/4): its 16 bytes of codes are the 32 hidden columns
  // of the half for that output column, i.e. the pieces 4*half .. +3 of the column in the [piece][column] B stage
  const int NW = ntile_width(M);
  const int half = w >> 2, col = (w & 3) * 64 + lane;
  const int n = min(n0 + col, M - 1);
  const size_t qoff = q4_off_codes(2, M) + (((size_t)(n / NW) * 2 + half) * NW + (n % NW)) * 16;
  const size_t zoff = q4_off_scales(2, M) + (size_t)n * 2;
  const size_t cbytes = q4_chunk_u16(M) * 2;
  auto bload = [&](int kt, Q4Regs& r) {
    const unsigned char* cb = ebase + (size_t)(wv.chunk0 + c_begin + kt) * cbytes;
    gload_b128(r.q, cb + qoff);
    gload_u16(r.z, cb + zoff);
  };
  auto bready = [&](Q4Regs& r) { asm volatile("" : "+v"(r.q), "+v"(r.z)::"memory"); };
  // word i = hidden columns 8i .. 8i+7 of the half; even nibbles hold elements 0 1 2 3, odd nibbles 4 5 6 7
  auto bconv = [&](int stage, const Q4Regs& r, int i) {
    const float sc = __uint_as_float(r.z << 16), s8 = -8.f * sc;
    const uint32_t wd = r.q[i], ev = wd & 0x0f0f0f0fu, od = (wd >> 4) & 0x0f0f0f0fu;
    u32x4 o;
    o.x = q4_pair(ev, 0, 1, sc, s8);
    o.y = q4_pair(ev, 2, 3, sc, s8);
    o.z = q4_pair(od, 0, 1, sc, s8);
    o.w = q4_pair(od, 2, 3, sc, s8);
    lds_store_b128(lds + stage * S::STAGE + BM * 128 + ((half * 4 + i) * BN + col) * 16, o);
  };
  if (c_begin < c_end) {
    SI_GEMM_DECLS(SI_BOFF_K8)
    SI_GEMM_MAIN_LOOP_REGB(c_end - c_begin, 2, Q4Regs, issue_a, bload, bready, bconv)
#pragma unroll
    for (int i = 0; i < S::FA; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int m = n0 + wc * 64 + j * 32 + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = ti.row0 + wr * (BM / 2) + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
          if (row < ti.row_end && m < M) {
            float* dst = out + (size_t)row * M + m;
            *dst = accumulate ? *dst + acc[i][j][r] : acc[i][j][r];
          }
        }
      }
  } else {
    for (int i = tid; i < BM * BN; i += THREADS) {
      const int row = ti.row0 + i / BN, m = n0 + i % BN;
      if (row < ti.row_end && m < M) out[(size_t)row * M + m] = 0.f;
    }
  }
}

__global__ __launch_bounds__(THREADS, 1) void k_prefill_down_q4(const uint16_t* __restrict__ hact, int ldh, int M, Plan p,
                                                                int expert_sel, int x2_only, int n_cu,
                                                                int n_ntiles, int n_split, WeightView wv,
                                                                float* __restrict__ yp, size_t slab_stride,
                                                                int accumulate) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  int inner;
  TileInfo ti;
  if (!block_tile(p, expert_sel, x2_only, n_ntiles * n_split, n_cu, 0, inner, ti)) return;
  if (!storage_index(wv, ti.e, ti.se)) return;
#define SI_CALL_DN(BMV) down_body_q4<BMV>(hact, ldh, M, inner, ti, n_ntiles, n_split, wv, yp, slab_stride, accumulate, lds)
  SI_PICK_BODY_2PASS(ti, SI_CALL_DN);
#undef SI_CALL_DN
}

__global__ __launch_bounds__(256) void k_prefill_combine(const float* __restrict__ yp, size_t slab_stride, int n_split,
                                                         const float* __restrict__ ycc, int T, int k, int M, int n_x1,
                                                         int has_shared, Plan p, float* __restrict__ y) {
  const int t = blockIdx.y;
  const int m4 = blockIdx.x * 256 + threadIdx.x;
  if (m4 * 4 >= M) return;
  float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int s = 0; s < k; ++s) {
    const float wgt = p.w[t * k + s];
    const float* row = yp + (size_t)p.inv[t * k + s] * M;
    float4 v = reinterpret_cast<const float4*>(row)[m4];
    for (int q = 1; q < n_split; ++q) {
      const float4 v2 = reinterpret_cast<const float4*>(row + (size_t)q * slab_stride)[m4];
      v.x += v2.x; v.y += v2.y; v.z += v2.z; v.w += v2.w;
    }
    acc.x = fmaf(wgt, v.x, acc.x); acc.y = fmaf(wgt, v.y, acc.y);
    acc.z = fmaf(wgt, v.z, acc.z); acc.w = fmaf(wgt, v.w, acc.w);
  }
  if (has_shared) {
    const float* row = yp + (size_t)(T * k + t) * M;
    for (int q = 0; q < n_split; ++q) {
      const float4 v = reinterpret_cast<const float4*>(row + (size_t)q * slab_stride)[m4];
      acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
    }
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

static_assert(Shape<64>::LDS <= KERNEL_LDS && Shape<128>::LDS <= KERNEL_LDS && Shape<192>::LDS <= KERNEL_LDS &&
              Shape<256>::LDS <= KERNEL_LDS, "a body does not fit the launch's LDS");

// compute units of the current device (a round of the tail split)
static int cu_count() {
  static int n = [] {
    int dev = 0, v = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0)
      v = 256;
    return v;
  }();
  return n;
}

// grid of a launch over at most n_tiles logical ids: room for the XCD ranges (rounded up to 8) and for the
// second blocks of a split tail (at most half a round)
static int grid_blocks(int n_tiles) { return (n_tiles + 7) / 8 * 8 + 8 + cu_count() / 2 + 8; }

static hipError_t ensure_lds_attr() {
  static hipError_t st = [] {
    const void* kernels[] = {(const void*)k_prefill_gateup, (const void*)k_prefill_down, (const void*)k_prefill_gateup_q4,
                             (const void*)k_prefill_down_q4};
    for (const void* k : kernels) {
      hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, KERNEL_LDS);
      if (e != hipSuccess) return e;
      // The main loops count their own vector-memory operations (wait_vmcnt<N> against Shape<>::LPW / ALD): a
      // register spill would add scratch loads and stores to that count and let a barrier pass before a tile has
      // landed.  A build whose GEMM kernels use scratch memory is refused here instead of computing wrong results.
      hipFuncAttributes fa{};
      e = hipFuncGetAttributes(&fa, k);
      if (e != hipSuccess) return e;
      if (fa.localSizeBytes != 0) return hipErrorInvalidDeviceFunction;
    }
    return hipSuccess;
  }();
  return st;
}

hipError_t launch_prefill_gateup(const uint16_t* x, int M, const Plan& plan, int expert_sel, int x2_only,
                                 int n_row_tiles, const WeightView& wv, uint16_t* hact, int ldh,
                                 hipStream_t stream) {
  if (wv.n_chunks <= 0 || n_row_tiles <= 0) return hipSuccess;
  hipError_t e = ensure_lds_attr();
  if (e != hipSuccess) return e;
  const int n_ctiles = (wv.n_chunks + 1) / 2;
  const int total = grid_blocks(n_row_tiles * n_ctiles);
  if (wv.q4)
    hipLaunchKernelGGL(k_prefill_gateup_q4, dim3(total), dim3(THREADS), KERNEL_LDS, stream, x, M, plan, expert_sel, x2_only,
                       cu_count(), n_ctiles, wv, hact, ldh);
  else
    hipLaunchKernelGGL(k_prefill_gateup, dim3(total), dim3(THREADS), KERNEL_LDS, stream, x, M, plan, expert_sel, x2_only,
                       cu_count(), n_ctiles, wv, hact, ldh);
  return hipGetLastError();
}

hipError_t launch_prefill_down(const uint16_t* hact, int ldh, int M, const Plan& plan, int expert_sel,
                               int x2_only, int n_row_tiles, const WeightView& wv, float* yp, size_t slab_stride,
                               int n_split, int accumulate, hipStream_t stream) {
  if (wv.n_chunks <= 0 || n_row_tiles <= 0) return hipSuccess;
  hipError_t e = ensure_lds_attr();
  if (e != hipSuccess) return e;
  const int n_ntiles = (M + BN - 1) / BN;
  const int total = grid_blocks(n_row_tiles * n_ntiles * n_split);
  if (wv.q4)
    hipLaunchKernelGGL(k_prefill_down_q4, dim3(total), dim3(THREADS), KERNEL_LDS, stream, hact, ldh, M, plan, expert_sel,
                       x2_only, cu_count(), n_ntiles, n_split, wv, yp, slab_stride, accumulate);
  else
    hipLaunchKernelGGL(k_prefill_down, dim3(total), dim3(THREADS), KERNEL_LDS, stream, hact, ldh, M, plan, expert_sel,
                       x2_only, cu_count(), n_ntiles, n_split, wv, yp, slab_stride, accumulate);
  return hipGetLastError();
}

hipError_t launch_prefill_combine(const float* yp, size_t slab_stride, int n_split, const float* ycc, int T, int k, int M,
                                  int n_x1, int has_shared, const Plan& plan, float* y, hipStream_t stream) {
  if (T <= 0) return hipSuccess;
  dim3 grid((M / 4 + 255) / 256, T);
  hipLaunchKernelGGL(k_prefill_combine, grid, dim3(256), 0, stream, yp, slab_stride, n_split, ycc, T, k, M, n_x1,
                     has_shared, plan, y);
  return hipGetLastError();
}

hipError_t launch_fill_zero(float* p, size_t n, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  int blocks = (int)std::min<size_t>((n + 255) / 256, 4096);
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

}  // namespace si
