// Internal declarations shared by the translation units of libscheinfer (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "scheinfer.h"
#include "cc_worker.h"

namespace si {

// Weight storage: see cc_worker.h (chunk-major; gate/up in 512-wide k panels, down in 256-column
// tiles with the contraction index grouped by 8).  A part (CC, CG or GG) of an expert is a contiguous
// range of chunks, so a CG copy is one memcpy and CG' is simply the CC chunk range of the same pinned
// buffer (Section III-B: same addresses).
inline size_t chunk_elems(int M) { return (size_t)3 * CHUNK_J * M; }
inline size_t chunk_bytes(int M) { return chunk_elems(M) * 2; }

constexpr int MAX_EXPERTS = 256;      // routed experts (a shared expert adds one more table entry)
constexpr int ROUTE_THREADS = 1024;   // block size of the assignment kernel
constexpr int TILE_ROWS = 256;        // rows per row tile of the prefill GEMMs (the last tile of an expert: see n_row_tiles)
constexpr int MAX_KSPLIT = 4;         // k-splits (output slabs) of the prefill down projection
constexpr int DECODE_TB = 4;          // most tokens handled per weight pass in the GEMV kernels
constexpr int DOWN_SLOTS = 32;        // j-splits of the decode down projection per part

// Row tiles of an expert (or of its X2 rows) with `rows` rows.  The GEMM kernels run, per tile, the body
// instantiated for the rows the tile really has (64, 128, 192, 256 or 320): a block streams its weight tile whatever
// the number of rows, so an expert with 140 rows gets one 192-row block, not two blocks of 128.
// A tile costs nearly the same whether it holds 10 rows or 256 (it streams the same weights, and its ring of LDS
// stages is latency bound when the rows are few: measured, 128 extra tiles of 5 rows cost a 2048-tile GEMM as much
// as 128 extra tiles of 256), so a remainder of at most TILE_ROWS_SPILL rows rides with the last full tile instead
// of becoming a tile of its own.  With a balanced router and a batch that gives each expert a multiple of 256 rows
// on average, about half the experts end a few rows past such a multiple.
constexpr int TILE_ROWS_SPILL = 64;  // the last tile of an expert also takes up to this many rows beyond TILE_ROWS
inline SI_HD int n_row_tiles(int rows) {
  return rows <= 0 ? 0 : rows <= TILE_ROWS ? 1 : (rows - TILE_ROWS_SPILL + TILE_ROWS - 1) / TILE_ROWS;
}

// Device-side result of the token assignment plus the launch tables derived from it.
// Expert tables have EX = E + (shared ? 1 : 0) entries; the shared expert is entry E and owns the
// rows [T*k, T*k + T) (row T*k + t belongs to token t, weight 1).
struct Plan {
  int32_t* idx;        // [T*k]
  float* w;            // [T*k]
  int32_t* count;      // [EX]
  int32_t* off;        // [EX+1]
  int32_t* count1;     // [EX]  pairs of the expert that belong to X1 tokens (t < T - n_g)
  int32_t* perm;       // [T*k]
  int32_t* inv;        // [T*k]
  int32_t* row_token;  // [T*k + T] token of each expert-sorted row
  int32_t* touched;    // [EX] experts with count > 0, ascending
  int32_t* n_touched;  // [1]
  int32_t* tile_e;     // [max_tiles] expert of each row tile (all rows)
  int32_t* tile_r;     // [max_tiles] index of the tile inside its expert
  int32_t* n_tiles;    // [1] row tiles of the routed experts (the shared expert's follow in the table)
  int32_t* tile_e_x2;  // the same for the X2 rows only (CG')
  int32_t* tile_r_x2;
  int32_t* n_tiles_x2;  // [1]
  int32_t* tile_flags;  // [1] bit 0: no routed expert has more than one row tile; bit 1: the same for the X2 rows
  int32_t n_routed;    // E: launches over "all experts" cover entries < n_routed only (the shared
                       // expert's weights live in their own buffer and get their own launch)
};

// user-visible copies (first E entries), any pointer may be null
struct RouteOut {
  int32_t* idx; float* w; int32_t* count; int32_t* off; int32_t* perm; int32_t* inv;
};

// route.hip
hipError_t launch_route(const float* logits, int T, int E, int k, int has_shared, int n_g,
                        const Plan& plan, const RouteOut& user, hipStream_t stream);

// Description of the weights one kernel launch works on.
struct WeightView {
  const uint16_t* base;   // chunk-major storage
  size_t expert_stride;   // elements between experts (0 when `base` already points at the expert)
  int chunk0;             // first chunk (relative to base / expert) to process
  int n_chunks;           // number of chunks to process
  int col0;               // hidden column (within the expert) of chunk0: indexes h / Hact columns
  int q4;                 // chunks are in the 4-bit storage form (cc_worker.h); strides still in uint16 units
  const int32_t* e_map;   // device [experts] or null: storage index of expert e inside `base` (-1: the expert has
                          // no weights in this storage and the launch skips it); null = expert e is at index e
};

#if defined(__HIPCC__)
// storage index of expert e for this launch; false when the launch has nothing for the expert
__device__ inline bool storage_index(const WeightView& wv, int e, int& se) {
  se = wv.e_map ? wv.e_map[e] : e;
  return se >= 0;
}
#endif

// decode.hip ---------------------------------------------------------------------------------
// h[row][j] = SiLU(x_row . Wg[j]) * (x_row . Wu[j]) for the rows of the selected experts.
//  expert_sel < 0: all touched experts (table lookup);  >= 0: only that expert.
//  x2_only: restrict to rows of X2 tokens (CG').
//  tb_hint: upper bound on the rows of one expert (T); picks the tokens-per-pass instantiation (1, 2 or 4).
// Token assignment folded into the first gate/up launch of a generation-phase call with few tokens (the launch of a
// separate assignment kernel costs as much as reading tens of megabytes): every block derives the assignment of
// the <= FUSED_ROUTE_MAX_T tokens itself and finds its expert from it; block (0, 0) also writes the tables that the
// later launches of the call and the caller read.  logits == nullptr: dense layer (one expert, weight 1).
constexpr int FUSED_ROUTE_MAX_T = 4;
constexpr int FUSED_ROUTE_MAX_PAIRS = 8;
struct FusedRoute {
  const float* logits;
  int T, E, k, has_shared, n_x1;
  RouteOut user;
};
hipError_t launch_decode_gateup(const uint16_t* x, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                int max_touched, const WeightView& wv, float* h, int ldh, hipStream_t stream,
                                const FusedRoute* fused_route = nullptr);
// part[slot][row][m] = sum over the j of the slot of h[row][j] * Wd[j][m]
// y[t][m] = sum_s w[t][s] * sum_slots part[slot][inv[t*k+s]][m] + shared rows + ycc[t][m]
struct DecodeCombineArgs {
  const float* part; size_t slot_stride;
  int n_slots_gg, n_slots_cg, n_slots_cc;   // valid slots per part (routed experts); slot ids: part*DOWN_SLOTS + s
  int s_slots_gg, s_slots_cg, s_slots_cc;   // the same for the rows of the shared expert
  const float* ycc;                         // [T1][M] or null
  int T, k, M, n_x1, has_shared;
};
// part[slot][row][m] = sum over the j of the slot of h[row][j] * Wd[j][m]
hipError_t launch_decode_down(const float* h, int ldh, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                              int max_touched, const WeightView& wv, int slot0, int chunks_per_slot,
                              float* part, size_t slot_stride, hipStream_t stream);
hipError_t launch_decode_combine(const DecodeCombineArgs& a, const Plan& plan, float* y, hipStream_t stream);

// prefill.hip --------------------------------------------------------------------------------
// Hact[row][c] (bf16) for c in [0, 64*n_chunks): SwiGLU of the gate/up products (MFMA, fp32 acc).
// n_row_tiles: (an upper bound on) the row tiles of the launch, for the grid; the kernels find the real ones
hipError_t launch_prefill_gateup(const uint16_t* x, int M, const Plan& plan, int expert_sel, int x2_only,
                                 int n_row_tiles, const WeightView& wv, uint16_t* hact, int ldh,
                                 hipStream_t stream);
// Yp[split][row][m] (fp32) (+)= Hact[row][chunks of the split] . Wd[chunks][m]; the chunk range of the launch is
// cut into n_split equal parts, each with its own output slab (summed by the combine kernel)
hipError_t launch_prefill_down(const uint16_t* hact, int ldh, int M, const Plan& plan, int expert_sel,
                               int x2_only, int n_row_tiles, const WeightView& wv, float* yp, size_t slab_stride,
                               int n_split, int accumulate, hipStream_t stream);
// y[t][m] = sum_s w[t][s]*Yp[inv[t*k+s]][m] + Yp[T*k+t][m] (shared) + ycc[t][m] (X1 rows)
hipError_t launch_prefill_combine(const float* yp, size_t slab_stride, int n_split, const float* ycc, int T, int k,
                                  int M, int n_x1, int has_shared, const Plan& plan, float* y, hipStream_t stream);
hipError_t launch_fill_zero(float* p, size_t n, hipStream_t stream);

// q4.hip -------------------------------------------------------------------------------------
// the GEMV launchers of decode.hip hand over to these when wv.q4 is set
hipError_t launch_decode_gateup_q4(const uint16_t* x, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                   int max_touched, const WeightView& wv, float* h, int ldh, hipStream_t stream);
hipError_t launch_decode_down_q4(const float* h, int ldh, int M, const Plan& plan, int tb_hint, int expert_sel, int x2_only,
                                 int max_touched, const WeightView& wv, int slot0, int chunks_per_slot, float* part,
                                 size_t slot_stride, hipStream_t stream);
// 4-bit chunks [wv.chunk0, +wv.n_chunks) of one expert (expert_sel >= 0) or of every routed expert that has rows
// -> bf16 chunks 0..n_chunks at dst (+ e * dst_estride)
hipError_t launch_dequant_q4(const WeightView& wv, int M, const Plan& plan, int expert_sel, int x2_only, int n_experts,
                             uint16_t* dst, size_t dst_estride, hipStream_t stream);

}  // namespace si
