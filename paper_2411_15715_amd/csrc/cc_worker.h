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
};
void cc_pool_run(CcPool*, const CcJob& job);   // blocks until done
void cc_pool_start(CcPool*, const CcJob& job); // asynchronous
void cc_pool_wait(CcPool*);

}  // namespace si
