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


// ---- AVX-512 versions for the 4-bit storage form.  Codes become bf16 pairs without any widening: for a 32-bit
// word w of gate / up codes, ((w >> 4p) & 0x000F000F) | 0x43004300 holds the bf16 values 128 + code of elements
// 2p and 2p+1 of the word (exact), and vdpbf16ps multiplies them with the matching bf16 pair of x.  Per group of
// 64 weights: x.W = scale * (sum x (128 + code) - 136 sum x).  The pairs of x (and of h for FC2, split into a
// bf16 head and a bf16 remainder so that h keeps ~16 significant bits) are laid out once per token in the order
// the shifted words deliver the codes.
struct Q4X {                      // per token: M/128 blocks of 128 elements = 16 code words
  std::vector<uint32_t> pairs;    // [block][p][16]  lane i = x pair (elements 8i+2p, 8i+2p+1 of the block)
  std::vector<float> wsum;        // [block][16]     lane i = sum of the 8 x values of word i
};

SI_AVX512 void q4_prepare_x(const uint16_t* x, int M, Q4X* o) {
  const int nb = M / 128;
  o->pairs.resize((size_t)nb * 64);
  o->wsum.resize((size_t)nb * 16);
  const uint32_t* xp = reinterpret_cast<const uint32_t*>(x);
  for (int b = 0; b < nb; ++b) {
    uint32_t(*lane)[16] = reinterpret_cast<uint32_t(*)[16]>(&o->pairs[(size_t)b * 64]);
    float* sum = &o->wsum[(size_t)b * 16];
    for (int i = 0; i < 16; ++i) {
      float s = 0.f;
      for (int pp = 0; pp < 4; ++pp) {
        const uint32_t u = xp[64 * b + 4 * i + pp];
        lane[pp][i] = u;
        s += bf16_to_f32((uint16_t)(u & 0xffffu)) + bf16_to_f32((uint16_t)(u >> 16));
      }
      sum[i] = s;
    }
  }
}

SI_AVX512 inline __m512i q4_pairs(__m512i w, int shift, __m512i mask, __m512i magic) {
  // (w >> shift) & mask | magic in two instructions (shift, ternary logic 0xEA = (a & b) | c)
  return _mm512_ternarylogic_epi32(_mm512_srli_epi32(w, shift), mask, magic, 0xEA);
}

// h[r][jj] for the 64 hidden columns of one chunk (M a multiple of 128)
SI_AVX512 void fc1_chunk_q4_avx512(const uint32_t* gq, const uint32_t* uq, const uint16_t* gs, const uint16_t* us,
                                   const Q4X* xs, int nrows, int M, float* hbuf) {
  const __m512i mask = _mm512_set1_epi32(0x000F000F), magic = _mm512_set1_epi32(0x43004300);
  const __m512 off = _mm512_set1_ps(136.f);
  const int nb = M / 128, MG = M / 64;
  for (int jj = 0; jj < CHUNK_J; ++jj) {
    __m512 ag[8], au[8];
    for (int r = 0; r < nrows; ++r) { ag[r] = _mm512_setzero_ps(); au[r] = _mm512_setzero_ps(); }
    const uint32_t* grow = gq + (size_t)jj * (M / 8);
    const uint32_t* urow = uq + (size_t)jj * (M / 8);
    for (int b = 0; b < nb; ++b) {
      const __m512i wg = _mm512_loadu_si512(grow + 16 * b), wu = _mm512_loadu_si512(urow + 16 * b);
      __m512i pg[4], pu[4];
      for (int pp = 0; pp < 4; ++pp) { pg[pp] = q4_pairs(wg, 4 * pp, mask, magic); pu[pp] = q4_pairs(wu, 4 * pp, mask, magic); }
      // words 0..7 of the block belong to scale group 2b, words 8..15 to group 2b+1
      const __m512 sg = _mm512_mask_blend_ps(0xFF00, _mm512_set1_ps(bf16_to_f32(gs[(size_t)jj * MG + 2 * b])),
                                             _mm512_set1_ps(bf16_to_f32(gs[(size_t)jj * MG + 2 * b + 1])));
      const __m512 su = _mm512_mask_blend_ps(0xFF00, _mm512_set1_ps(bf16_to_f32(us[(size_t)jj * MG + 2 * b])),
                                             _mm512_set1_ps(bf16_to_f32(us[(size_t)jj * MG + 2 * b + 1])));
      for (int r = 0; r < nrows; ++r) {
        const uint32_t* xp = &xs[r].pairs[(size_t)b * 64];
        __m512 dg = _mm512_setzero_ps(), du = _mm512_setzero_ps();
        for (int pp = 0; pp < 4; ++pp) {
          const __m512bh xv = (__m512bh)_mm512_loadu_si512(xp + 16 * pp);
          dg = _mm512_dpbf16_ps(dg, (__m512bh)pg[pp], xv);
          du = _mm512_dpbf16_ps(du, (__m512bh)pu[pp], xv);
        }
        const __m512 corr = _mm512_mul_ps(off, _mm512_loadu_ps(&xs[r].wsum[(size_t)b * 16]));
        ag[r] = _mm512_fmadd_ps(sg, _mm512_sub_ps(dg, corr), ag[r]);
        au[r] = _mm512_fmadd_ps(su, _mm512_sub_ps(du, corr), au[r]);
      }
    }
    for (int r = 0; r < nrows; ++r) {
      const float g = _mm512_reduce_add_ps(ag[r]), u = _mm512_reduce_add_ps(au[r]);
      hbuf[(size_t)r * CHUNK_J + jj] = g / (1.f + std::exp(-g)) * u;
    }
  }
}

// out[r][m] += scale[m] * (sum_j h[r][j] code[j][m] - 8 sum_j h[r][j]) over the 64 j of one chunk.
// Down codes: [M/NW][2 halves][NW m][16 bytes]; inside a word element e sits at nibble 2e (e < 4) or 2(e-4)+1, so
// the shift by 4q pairs up elements (0,2), (4,6), (1,3), (5,7) for q = 0..3.
SI_AVX512 void fc2_chunk_q4_avx512(const uint32_t* dq, const uint16_t* ds, const float* hbuf, int nrows, int M, int NW,
                                   float* const* out) {
  static const int EA[4] = {0, 4, 1, 5}, EB[4] = {2, 6, 3, 7};
  const __m512i mask = _mm512_set1_epi32(0x000F000F), magic = _mm512_set1_epi32(0x43004300);
  // per row: pairs of h in the order above, as bf16 head and bf16 remainder; lane = (m_local 0..3, word k 0..3)
  alignas(64) uint32_t hh[8][2][4][16], hl[8][2][4][16];
  float hsum[8];
  for (int r = 0; r < nrows; ++r) {
    const float* h = hbuf + (size_t)r * CHUNK_J;
    auto head = [](float v) { uint32_t u; std::memcpy(&u, &v, 4); return u & 0xffff0000u; };
    auto as_f = [](uint32_t u) { float v; std::memcpy(&v, &u, 4); return v; };
    auto tail = [&](float v) { return head(v - as_f(head(v))); };
    // the offset term uses the sum of exactly the values the dot products see (head + remainder), so that the
    // 128 * sum h parts cancel to rounding
    float s = 0.f;
    for (int jx = 0; jx < CHUNK_J; ++jx) s += as_f(head(h[jx])) + as_f(tail(h[jx]));
    hsum[r] = s;
    for (int half = 0; half < 2; ++half)
      for (int q = 0; q < 4; ++q)
        for (int k = 0; k < 4; ++k) {
          const float a = h[32 * half + 8 * k + EA[q]], b = h[32 * half + 8 * k + EB[q]];
          const uint32_t ph = (head(a) >> 16) | head(b), pl = (tail(a) >> 16) | tail(b);
          for (int ml = 0; ml < 4; ++ml) { hh[r][half][q][ml * 4 + k] = ph; hl[r][half][q][ml * 4 + k] = pl; }
        }
  }
  for (int m = 0; m < M; m += 4) {
    const size_t i0 = (((size_t)(m / NW) * 2) * NW + (m % NW)) * 4;  // word index of (half 0, column m)
    const __m512i w0 = _mm512_loadu_si512(dq + i0), w1 = _mm512_loadu_si512(dq + i0 + (size_t)NW * 4);
    __m512i p0[4], p1[4];
    for (int q = 0; q < 4; ++q) { p0[q] = q4_pairs(w0, 4 * q, mask, magic); p1[q] = q4_pairs(w1, 4 * q, mask, magic); }
    for (int r = 0; r < nrows; ++r) {
      __m512 acc = _mm512_setzero_ps();
      for (int q = 0; q < 4; ++q) {
        acc = _mm512_dpbf16_ps(acc, (__m512bh)p0[q], (__m512bh)_mm512_load_si512(hh[r][0][q]));
        acc = _mm512_dpbf16_ps(acc, (__m512bh)p0[q], (__m512bh)_mm512_load_si512(hl[r][0][q]));
        acc = _mm512_dpbf16_ps(acc, (__m512bh)p1[q], (__m512bh)_mm512_load_si512(hh[r][1][q]));
        acc = _mm512_dpbf16_ps(acc, (__m512bh)p1[q], (__m512bh)_mm512_load_si512(hl[r][1][q]));
      }
      alignas(64) float lanes[16];
      _mm512_store_ps(lanes, acc);
      for (int ml = 0; ml < 4; ++ml) {
        const float dot = (lanes[4 * ml] + lanes[4 * ml + 1]) + (lanes[4 * ml + 2] + lanes[4 * ml + 3]);
        out[r][m + ml] += bf16_to_f32(ds[m + ml]) * (dot - 136.f * hsum[r]);
      }
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
    if (j.q4 && cpu_has_avx512_bf16() && !force_generic_ && M % 128 == 0) {
      Q4X xq[RB];
      float* orow[RB];
      for (int r = 0; r < it.nrows; ++r) {
        const int pr = row_pair_[it.row0 + r];
        q4_prepare_x(j.x + (size_t)(pr >= 0 ? pr / j.k : -pr - 1) * M, M, &xq[r]);
        orow[r] = &scratch_[((size_t)it.slice * n_rows_ + it.row0 + r) * M];
      }
      for (int c = it.c0; c < it.c1; ++c) {
        const unsigned char* cb = reinterpret_cast<const unsigned char*>(ebase + (size_t)c * q4_chunk_u16(M));
        fc1_chunk_q4_avx512(reinterpret_cast<const uint32_t*>(cb + q4_off_codes(0, M)), reinterpret_cast<const uint32_t*>(cb + q4_off_codes(1, M)),
                            reinterpret_cast<const uint16_t*>(cb + q4_off_scales(0, M)), reinterpret_cast<const uint16_t*>(cb + q4_off_scales(1, M)),
                            xq, it.nrows, M, hbuf.data());
        fc2_chunk_q4_avx512(reinterpret_cast<const uint32_t*>(cb + q4_off_codes(2, M)), reinterpret_cast<const uint16_t*>(cb + q4_off_scales(2, M)),
                            hbuf.data(), it.nrows, M, NW, orow);
      }
      return;
    }
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
