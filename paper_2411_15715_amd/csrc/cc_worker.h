// Host-only declarations of the CC worker pool (no HIP types), shared with the GPU-side scheduler.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace si {

constexpr int CHUNK_J = 64;  // hidden columns per weight chunk

#if defined(__HIPCC__)
#define SI_HD __host__ __device__
#else
#define SI_HD
#endif

// Weight storage.  One chunk holds CHUNK_J = 64 consecutive hidden columns j of one expert in three
// blocks of 64*M bf16 each: [gate | up | down].
//  gate / up block: [M/PW panels][64 j][PW m], PW = panel_width(M) (512 for the model shapes).  A row
//    segment of a panel is PW contiguous contraction elements of FC1: one 1 KB wave load of the GEMV,
//    and the 16 rows of a GEMV block are 16 KB contiguous; the MFMA kernels fetch 128-byte pieces at a
//    1 KB stride, which spreads over the memory channels (a plain [j][m] layout puts the 256 rows of a
//    tile 8 KB apart, all on the same channels).
//  down block: [M/NW tiles][8 q][NW m][8 i] holding Wd[j0 + 8q + i][m], NW = ntile_width(M) (256): the
//    contraction index of FC2 is contiguous in groups of 8 (one 128-bit load per lane of the GEMV, one
//    8-element MFMA operand fragment), and everything a 256-column GEMV block or MFMA tile needs from a
//    chunk is one contiguous 32 KB run.
inline SI_HD int panel_width(int M) { int p = 512; while (M % p) p >>= 1; return p; }
inline SI_HD int ntile_width(int M) { int p = 256; while (M % p) p >>= 1; return p; }
// element offset inside a gate (or up) block of (j in chunk, m)
inline SI_HD size_t gu_off(int j, int m, int PW) { return ((size_t)(m / PW) * CHUNK_J + j) * PW + (m % PW); }
// element offset inside a down block of (j in chunk, m)
inline SI_HD size_t dn_off(int j, int m, int NW) {
  return (((size_t)(m / NW) * 8 + (j >> 3)) * NW + (m % NW)) * 8 + (j & 7);
}

// 4-bit storage of a chunk (weights given as codes 0..15 standing for (code - 8) * scale, with bf16 group
// scales): 102*M bytes = 51*M uint16 units, in six sections at these byte offsets
//   0     gate codes  [64 j][M/2 bytes]      32M   up codes (same)      64M   down codes
//   96M   gate scales [64 j][M/64] bf16      98M   up scales (same)     100M  down scales [M] bf16
// Gate / up codes are plain rows (a GEMV wave reads 1 KB = 2048 elements of a row per instruction).  Inside
// every 32-bit word (8 consecutive m) element e = 2p + h sits at nibble p + 4h, so that
// (word >> 4p) & 0x000F000F holds the pair (e = 2p, e = 2p + 1) in the two halves of a register, ready to be
// turned into two bf16 values and multiplied with the bf16 pair of x by one dot-product instruction.
// Down codes: [M/NW tiles][2 halves][NW m][16 bytes], the 16 bytes holding j = 32*half .. 32*half + 31 of
// column m (one 128-bit load per GEMV thread and half); inside every word (8 consecutive j) element e sits at
// nibble 2e for e < 4 and 2(e-4)+1 for e >= 4, so that word & 0x0F0F0F0F and (word >> 4) & 0x0F0F0F0F hold
// elements 0..3 and 4..7 as bytes (one byte-to-float conversion each).
inline SI_HD size_t q4_chunk_u16(int M) { return (size_t)51 * M; }
inline SI_HD size_t q4_off_codes(int which, int M) { return (size_t)32 * M * which; }        // which: 0 gate, 1 up, 2 down
inline SI_HD size_t q4_off_scales(int which, int M) { return (size_t)96 * M + (size_t)2 * M * which; }
inline SI_HD int q4_fc1_nibble(int m) { return ((m & 7) >> 1) + 4 * (m & 1); }
inline SI_HD size_t q4_fc1_word(int j, int m, int M) { return (size_t)j * (M / 8) + m / 8; }  // 32-bit word index in the block
inline SI_HD int q4_fc2_nibble(int j) { const int e = j & 7; return e < 4 ? 2 * e : 2 * (e - 4) + 1; }
inline SI_HD size_t q4_fc2_word(int j, int m, int NW) {
  return (((size_t)(m / NW) * 2 + (j >> 5)) * NW + (m % NW)) * 4 + ((j & 31) >> 3);
}

// cc_worker.cpp ------------------------------------------------------------------------------
class CcPool;
CcPool* cc_pool_create(int n_threads);
void cc_pool_destroy(CcPool*);
struct CcJob {
  const uint16_t* x;      // host [T1][M] bf16
  const int32_t* idx;     // host [T*k]
  const float* w;         // host [T*k]
  int T1, k, M, E;
  const uint16_t* routed; // host chunk-major, expert stride below; CC chunks are the first n_cc_chunks
  size_t expert_stride;   // elements
  int n_cc_chunks;
  const uint16_t* shared; // host chunk-major or null
  int s_cc_chunks;
  float* ycc;             // host [T1][M] fp32, overwritten
  int q4;                 // chunks are in the 4-bit storage form (expert_stride still in uint16 units)
  // per-expert storage (whole-expert placement), both null or both set: expert e starts at routed + e_off[e]
  // (uint16 units) and has e_cc_chunks[e] CC chunks; they replace expert_stride / n_cc_chunks
  const uint64_t* e_off;
  const int32_t* e_cc_chunks;
};
void cc_pool_run(CcPool*, const CcJob& job);   // blocks until done
void cc_pool_start(CcPool*, const CcJob& job); // asynchronous
void cc_pool_wait(CcPool*);

}  // namespace si
