// Host side of the layer: the CC part (Section III-B: parameters stored and executed on the CPU;
// Stream-A of Section III-C).  A persistent pool of threads computes, for the X1 tokens,
//   Y^CC[t] = sum_s w[t][s] * ( SiLU(x_t Wg^CC) * (x_t Wu^CC) ) Wd^CC   (+ the shared expert's CC part)
// from the chunk-major bf16 weights in pinned host memory, in fp32.
//
// Work items are (expert, block of up to 8 rows of that expert, slice of its CC chunks); each item
// owns its output rows in a scratch array, so no two threads ever add into the same memory and the
// result does not depend on scheduling.  A second pass sums slices and slots per token.
#include <atomic>
#include <condition_variable>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <thread>
#include <vector>

#include <algorithm>
#include <cmath>
#include <immintrin.h>

#include "cc_worker.h"

namespace si {

namespace {

typedef float v8f __attribute__((vector_size(32)));
typedef uint16_t v8u16 __attribute__((vector_size(16)));
typedef uint32_t v8u32 __attribute__((vector_size(32)));

constexpr int RB = 8;  // rows per item

inline v8f bf16x8_to_f32(const uint16_t* p) {
  v8u16 raw;
  std::memcpy(&raw, p, sizeof raw);
  v8u32 wide = __builtin_convertvector(raw, v8u32) << 16;
  v8f out;
  std::memcpy(&out, &wide, sizeof out);
  return out;
}

// the 8 codes of a 32-bit word as floats (code - 8), element order 0..7, for the two nibble orders of the
// 4-bit storage (cc_worker.h)
inline v8f q4_word(uint32_t w, const v8u32& shifts) {
  v8u32 v = {w, w, w, w, w, w, w, w};
  v = (v >> shifts) & 15u;
  typedef int32_t v8i32 __attribute__((vector_size(32)));
  return __builtin_convertvector((v8i32)v, v8f) - 8.f;
}
const v8u32 Q4_FC1_SHIFTS = {0, 16, 4, 20, 8, 24, 12, 28};
const v8u32 Q4_FC2_SHIFTS = {0, 8, 16, 24, 4, 12, 20, 28};

inline float bf16_to_f32(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  std::memcpy(&f, &u, sizeof f);
  return f;
}

inline float hsum(v8f v) { return ((v[0] + v[4]) + (v[2] + v[6])) + ((v[1] + v[5]) + (v[3] + v[7])); }

inline float silu_f(float z) { return z / (1.f + std::exp(-z)); }

// ---- AVX-512 (with BF16 dot products) versions of the two steps on the bf16 storage form, chosen at run time.
// FC1: x and the weights are both bf16, so vdpbf16ps forms the products exactly and accumulates them in fp32,
// 32 weights per instruction and no conversions.  FC2: h stays fp32; weights are widened 16 at a time.
#define SI_AVX512 __attribute__((target("avx512f,avx512bw,avx512vl,avx512dq,avx512bf16")))

bool cpu_has_avx512_bf16() {
  static const bool ok = __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
                         __builtin_cpu_supports("avx512vl") && __builtin_cpu_supports("avx512dq") &&
                         __builtin_cpu_supports("avx512bf16");
  return ok;
}

// h[r][jj] for the 64 hidden columns of one chunk; xrow[r] points at the bf16 token (M elements)
SI_AVX512 void fc1_chunk_avx512(const uint16_t* gblk, const uint16_t* ublk, const uint16_t* const* xrow, int nrows, int M,
                                int PW, float* hbuf, int rb) {
  for (int jj = 0; jj < CHUNK_J; ++jj) {
    __m512 ag[8], au[8];
    for (int r = 0; r < rb; ++r) { ag[r] = _mm512_setzero_ps(); au[r] = _mm512_setzero_ps(); }
    for (int p0 = 0; p0 < M; p0 += PW) {
      const uint16_t* grow = gblk + ((size_t)(p0 / PW) * CHUNK_J + jj) * PW;
      const uint16_t* urow = ublk + ((size_t)(p0 / PW) * CHUNK_J + jj) * PW;
      for (int m = 0; m < PW; m += 32) {
        const __m512bh wg = (__m512bh)_mm512_loadu_si512(grow + m), wu = (__m512bh)_mm512_loadu_si512(urow + m);
        for (int r = 0; r < nrows; ++r) {
          const __m512bh xv = (__m512bh)_mm512_loadu_si512(xrow[r] + p0 + m);
          ag[r] = _mm512_dpbf16_ps(ag[r], wg, xv);
          au[r] = _mm512_dpbf16_ps(au[r], wu, xv);
        }
      }
    }
    for (int r = 0; r < nrows; ++r) {
      const float g = _mm512_reduce_add_ps(ag[r]), u = _mm512_reduce_add_ps(au[r]);
      hbuf[(size_t)r * CHUNK_J + jj] = g / (1.f + std::exp(-g)) * u;
    }
  }
}

// out[r][m] += sum_j h[r][j] Wd[j][m] over the 64 j of one chunk; down block [M/NW][8 q][NW m][8 i]
SI_AVX512 void fc2_chunk_avx512(const uint16_t* db, const float* hbuf, int nrows, int M, int NW, float* const* out) {
  for (int m = 0; m < M; m += 2) {
    __m512 acc[8];
    for (int r = 0; r < nrows; ++r) acc[r] = _mm512_setzero_ps();
    for (int q = 0; q < 8; ++q) {
      // 16 bf16: columns m and m+1, rows 8q..8q+7 each (m is even and NW is even, so both lie in one tile)
      const __m256i raw = _mm256_loadu_si256(reinterpret_cast<const __m256i*>(db + dn_off(q * 8, m, NW)));
      const __m512 w = _mm512_castsi512_ps(_mm512_slli_epi32(_mm512_cvtepu16_epi32(raw), 16));
      for (int r = 0; r < nrows; ++r) {
        const __m512 hv = _mm512_broadcast_f32x8(_mm256_loadu_ps(hbuf + (size_t)r * CHUNK_J + q * 8));
        acc[r] = _mm512_fmadd_ps(hv, w, acc[r]);
      }
    }
    for (int r = 0; r < nrows; ++r) {
      const __m256 lo = _mm512_castps512_ps256(acc[r]), hi = _mm512_extractf32x8_ps(acc[r], 1);
      // sum of the 8 lanes of each half
      __m256 t = _mm256_hadd_ps(lo, hi);          // (l0+l1, l2+l3, h0+h1, h2+h3 | l4+l5, l6+l7, h4+h5, h6+h7)
      t = _mm256_hadd_ps(t, t);                   // (l0..3, h0..3, .. | l4..7, h4..7, ..)
      const __m128 s = _mm_add_ps(_mm256_castps256_ps128(t), _mm256_extractf128_ps(t, 1));
      out[r][m] += _mm_cvtss_f32(s);
      out[r][m + 1] += _mm_cvtss_f32(_mm_shuffle_ps(s, s, 1));
    }
  }
}

struct Item {
  int expert;      // E = shared
  int row0, nrows; // range in the expert's row list
  int c0, c1;      // CC chunk range
  int slice;
};

}  // namespace

class CcPool {
 public:
  explicit CcPool(int n) : n_threads_(n < 1 ? 1 : n) {
    for (int i = 0; i < n_threads_; ++i) threads_.emplace_back([this, i] { worker(i); });
  }
  ~CcPool() {
    {
      std::lock_guard<std::mutex> lk(mu_);
      stop_ = true;
      ++generation_;
    }
    cv_.notify_all();
    for (auto& t : threads_) t.join();
  }

  void start(const CcJob& job) {
    wait();
    job_ = job;
    plan();
    {
      std::lock_guard<std::mutex> lk(mu_);
      next_item_.store(0);
      next_token_.store(0);
      items_done_.store(0);
      running_ = n_threads_;
      ++generation_;
    }
    cv_.notify_all();
  }

  void wait() {
    std::unique_lock<std::mutex> lk(mu_);
    done_cv_.wait(lk, [this] { return running_ == 0; });
  }

 private:
  int cc_chunks(int e) const {
    const CcJob& j = job_;
    return e >= j.E ? j.s_cc_chunks : j.e_cc_chunks ? j.e_cc_chunks[e] : j.n_cc_chunks;
  }

  // expert-sorted row lists of the X1 tokens (built on the host from idx; order as the GPU's)
  void plan() {
    const CcJob& j = job_;
    const int EX = j.E + (j.shared ? 1 : 0);
    row_begin_.assign(EX + 1, 0);
    for (int t = 0; t < j.T1; ++t)
      for (int s = 0; s < j.k; ++s) row_begin_[j.idx[(size_t)t * j.k + s] + 1]++;
    if (j.shared) row_begin_[j.E + 1] = j.T1;
    for (int e = 0; e < EX; ++e) row_begin_[e + 1] += row_begin_[e];
    const int n_rows = row_begin_[EX];
    row_pair_.resize(n_rows);  // pair id t*k+s, or -(t+1) for a shared row
    std::vector<int> fill(row_begin_.begin(), row_begin_.end() - 1);
    for (int t = 0; t < j.T1; ++t)
      for (int s = 0; s < j.k; ++s) row_pair_[fill[j.idx[(size_t)t * j.k + s]]++] = t * j.k + s;
    if (j.shared)
      for (int t = 0; t < j.T1; ++t) row_pair_[fill[j.E]++] = -(t + 1);
    // number of row blocks, then how finely to slice the chunk range
    int n_blocks = 0;
    for (int e = 0; e < EX; ++e) n_blocks += (row_begin_[e + 1] - row_begin_[e] + RB - 1) / RB;
    int want = 4 * n_threads_;
    n_slices_ = n_blocks >= want ? 1 : (want + (n_blocks > 0 ? n_blocks : 1) - 1) / (n_blocks > 0 ? n_blocks : 1);
    int max_chunks = j.shared ? j.s_cc_chunks : 0;
    for (int e = 0; e < j.E; ++e) max_chunks = std::max(max_chunks, cc_chunks(e));
    if (n_slices_ > max_chunks) n_slices_ = max_chunks > 0 ? max_chunks : 1;
    items_.clear();
    for (int e = 0; e < EX; ++e) {
      const int nch = cc_chunks(e);
      if (nch == 0) continue;
      for (int r = row_begin_[e]; r < row_begin_[e + 1]; r += RB)
        for (int z = 0; z < n_slices_; ++z) {
          int c0 = (int)((long)nch * z / n_slices_), c1 = (int)((long)nch * (z + 1) / n_slices_);
          if (c1 > c0) items_.push_back({e, r, std::min(RB, row_begin_[e + 1] - r), c0, c1, z});
        }
    }
    scratch_.assign((size_t)n_slices_ * n_rows * j.M, 0.f);
    n_rows_ = n_rows;
  }

  void run_item(const Item& it, std::vector<float>& xf, std::vector<float>& hbuf) {
    const CcJob& j = job_;
    const int M = j.M;
    const int PW = panel_width(M), NW = ntile_width(M);
    const uint16_t* ebase = it.expert >= j.E ? j.shared
                            : j.e_off ? j.routed + j.e_off[it.expert] : j.routed + (size_t)it.expert * j.expert_stride;
    xf.resize((size_t)RB * M);
    for (int r = 0; r < it.nrows; ++r) {
      int pr = row_pair_[it.row0 + r];
      int t = pr >= 0 ? pr / j.k : -pr - 1;
      const uint16_t* xr = j.x + (size_t)t * M;
      for (int m = 0; m < M; m += 8) {
        v8f v = bf16x8_to_f32(xr + m);
        std::memcpy(&xf[(size_t)r * M + m], &v, sizeof v);
      }
    }
    hbuf.resize((size_t)RB * CHUNK_J);
    if (j.q4) {
      run_chunks_q4(it, ebase, xf, hbuf);
      return;
    }
    if (cpu_has_avx512_bf16() && !force_generic_) {
      const uint16_t* xrow[RB];
      float* orow[RB];
      for (int r = 0; r < it.nrows; ++r) {
        const int pr = row_pair_[it.row0 + r];
        xrow[r] = j.x + (size_t)(pr >= 0 ? pr / j.k : -pr - 1) * M;
        orow[r] = &scratch_[((size_t)it.slice * n_rows_ + it.row0 + r) * M];
      }
      for (int c = it.c0; c < it.c1; ++c) {
        const uint16_t* cb = ebase + (size_t)c * 3 * CHUNK_J * M;
        fc1_chunk_avx512(cb, cb + (size_t)CHUNK_J * M, xrow, it.nrows, M, PW, hbuf.data(), RB);
        fc2_chunk_avx512(cb + (size_t)2 * CHUNK_J * M, hbuf.data(), it.nrows, M, NW, orow);
      }
      return;
    }
    for (int c = it.c0; c < it.c1; ++c) {
      const uint16_t* cb = ebase + (size_t)c * 3 * CHUNK_J * M;
      // FC1 + activation (gate / up blocks: [M/PW panels][64 j][PW m])
      for (int jj = 0; jj < CHUNK_J; ++jj) {
        const uint16_t* gblk = cb;
        const uint16_t* ublk = cb + (size_t)CHUNK_J * M;
        v8f ag[RB], au[RB];
        for (int r = 0; r < RB; ++r) { ag[r] = v8f{0, 0, 0, 0, 0, 0, 0, 0}; au[r] = ag[r]; }
        for (int m = 0; m < M; m += 8) {
          const size_t wo = gu_off(jj, m, PW);
          v8f wg = bf16x8_to_f32(gblk + wo), wu = bf16x8_to_f32(ublk + wo);
          for (int r = 0; r < it.nrows; ++r) {
            v8f xv;
            std::memcpy(&xv, &xf[(size_t)r * M + m], sizeof xv);
            ag[r] += xv * wg;
            au[r] += xv * wu;
          }
        }
        for (int r = 0; r < it.nrows; ++r) hbuf[(size_t)r * CHUNK_J + jj] = silu_f(hsum(ag[r])) * hsum(au[r]);
      }
      // FC2: down block [M/NW tiles][8 q][NW m][8 i]
      const uint16_t* db = cb + (size_t)2 * CHUNK_J * M;
      for (int m = 0; m < M; ++m) {
        v8f wd[8];
        for (int q = 0; q < 8; ++q) wd[q] = bf16x8_to_f32(db + dn_off(q * 8, m, NW));
        for (int r = 0; r < it.nrows; ++r) {
          v8f a = v8f{0, 0, 0, 0, 0, 0, 0, 0};
          for (int q = 0; q < 8; ++q) {
            v8f hv;
            std::memcpy(&hv, &hbuf[(size_t)r * CHUNK_J + q * 8], sizeof hv);
            a += hv * wd[q];
          }
          scratch_[((size_t)it.slice * n_rows_ + it.row0 + r) * M + m] += hsum(a);
        }
      }
    }
  }

  // the same two steps on the 4-bit storage form: codes are widened to (code - 8) and multiplied by their group
  // scale in fp32 (exact: at most 12 significant bits)
  void run_chunks_q4(const Item& it, const uint16_t* ebase, const std::vector<float>& xf, std::vector<float>& hbuf) {
    const CcJob& j = job_;
    const int M = j.M, NW = ntile_width(M);
    for (int c = it.c0; c < it.c1; ++c) {
      const unsigned char* cb = reinterpret_cast<const unsigned char*>(ebase + (size_t)c * q4_chunk_u16(M));
      const uint32_t* gq = reinterpret_cast<const uint32_t*>(cb + q4_off_codes(0, M));
      const uint32_t* uq = reinterpret_cast<const uint32_t*>(cb + q4_off_codes(1, M));
      const uint32_t* dq = reinterpret_cast<const uint32_t*>(cb + q4_off_codes(2, M));
      const uint16_t* gs = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(0, M));
      const uint16_t* us = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(1, M));
      const uint16_t* ds = reinterpret_cast<const uint16_t*>(cb + q4_off_scales(2, M));
      for (int jj = 0; jj < CHUNK_J; ++jj) {
        v8f ag[RB], au[RB];
        for (int r = 0; r < RB; ++r) { ag[r] = v8f{0, 0, 0, 0, 0, 0, 0, 0}; au[r] = ag[r]; }
        for (int m = 0; m < M; m += 8) {
          const float sg = bf16_to_f32(gs[(size_t)jj * (M / 64) + m / 64]), su = bf16_to_f32(us[(size_t)jj * (M / 64) + m / 64]);
          const v8f wg = q4_word(gq[q4_fc1_word(jj, m, M)], Q4_FC1_SHIFTS) * sg;
          const v8f wu = q4_word(uq[q4_fc1_word(jj, m, M)], Q4_FC1_SHIFTS) * su;
          for (int r = 0; r < it.nrows; ++r) {
            v8f xv;
            std::memcpy(&xv, &xf[(size_t)r * M + m], sizeof xv);
            ag[r] += xv * wg;
            au[r] += xv * wu;
          }
        }
        for (int r = 0; r < it.nrows; ++r) hbuf[(size_t)r * CHUNK_J + jj] = silu_f(hsum(ag[r])) * hsum(au[r]);
      }
      for (int m = 0; m < M; ++m) {
        v8f wd[8];
        for (int q = 0; q < 8; ++q) wd[q] = q4_word(dq[q4_fc2_word(q * 8, m, NW)], Q4_FC2_SHIFTS);
        const float sd = bf16_to_f32(ds[m]);
        for (int r = 0; r < it.nrows; ++r) {
          v8f a = v8f{0, 0, 0, 0, 0, 0, 0, 0};
          for (int q = 0; q < 8; ++q) {
            v8f hv;
            std::memcpy(&hv, &hbuf[(size_t)r * CHUNK_J + q * 8], sizeof hv);
            a += hv * wd[q];
          }
          scratch_[((size_t)it.slice * n_rows_ + it.row0 + r) * M + m] += sd * hsum(a);
        }
      }
    }
  }

  void reduce_token(int t) {
    const CcJob& j = job_;
    const int M = j.M;
    float* out = j.ycc + (size_t)t * M;
    for (int m = 0; m < M; ++m) out[m] = 0.f;
    // rows of token t: find them through a per-token inverse built lazily
    for (int s = 0; s < j.k + (j.shared ? 1 : 0); ++s) {
      int row;
      float wgt;
      if (s < j.k) { row = inv_[(size_t)t * j.k + s]; wgt = j.w[(size_t)t * j.k + s]; }
      else { row = row_begin_[j.E] + t; wgt = 1.f; }
      const int e = s < j.k ? j.idx[(size_t)t * j.k + s] : j.E;
      if (cc_chunks(e) == 0) continue;
      for (int z = 0; z < n_slices_; ++z) {
        const float* src = &scratch_[((size_t)z * n_rows_ + row) * M];
        for (int m = 0; m < M; ++m) out[m] += wgt * src[m];
      }
    }
  }

  void worker(int) {
    unsigned long seen = 0;
    std::vector<float> xf, hbuf;
    for (;;) {
      {
        std::unique_lock<std::mutex> lk(mu_);
        cv_.wait(lk, [&] { return generation_ != seen; });
        seen = generation_;
        if (stop_) return;
      }
      const int n_items = (int)items_.size();
      for (;;) {
        int i = next_item_.fetch_add(1);
        if (i >= n_items) break;
        run_item(items_[i], xf, hbuf);
        items_done_.fetch_add(1);
      }
      // barrier: the inverse map is built by whoever finishes first; wait until all items are done
      while (items_done_.load(std::memory_order_acquire) < n_items) std::this_thread::yield();
      {
        std::lock_guard<std::mutex> lk(inv_mu_);
        if (inv_gen_ != seen) {
          inv_.assign((size_t)job_.T1 * job_.k, 0);
          for (int e = 0; e < job_.E; ++e)
            for (int r = row_begin_[e]; r < row_begin_[e + 1]; ++r) inv_[row_pair_[r]] = r;
          inv_gen_ = seen;
        }
      }
      for (;;) {
        int t = next_token_.fetch_add(1);
        if (t >= job_.T1) break;
        reduce_token(t);
      }
      {
        std::lock_guard<std::mutex> lk(mu_);
        if (--running_ == 0) done_cv_.notify_all();
      }
    }
  }

  bool force_generic_ = std::getenv("SI_CC_GENERIC") != nullptr;  // run the portable loops even where AVX-512 exists (tests)
  int n_threads_;
  std::vector<std::thread> threads_;
  std::mutex mu_, inv_mu_;
  std::condition_variable cv_, done_cv_;
  unsigned long generation_ = 0, inv_gen_ = 0;
  bool stop_ = false;
  int running_ = 0;
  CcJob job_{};
  std::vector<int> row_begin_, row_pair_, inv_;
  std::vector<Item> items_;
  std::vector<float> scratch_;
  int n_slices_ = 1, n_rows_ = 0;
  std::atomic<int> next_item_{0}, next_token_{0}, items_done_{0};
};

CcPool* cc_pool_create(int n_threads) { return new CcPool(n_threads); }
void cc_pool_destroy(CcPool* p) { delete p; }
void cc_pool_start(CcPool* p, const CcJob& job) { p->start(job); }
void cc_pool_wait(CcPool* p) { p->wait(); }
void cc_pool_run(CcPool* p, const CcJob& job) {
  p->start(job);
  p->wait();
}

}  // namespace si
