// Host-only declarations of the CC worker pool (no HIP types), shared with the GPU-side scheduler.
#pragma once
#include <stddef.h>
#include <stdint.h>

namespace si {

constexpr int CHUNK_J = 64;  // hidden columns per weight chunk (see si_internal.h for the layout)

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
