// C ABI of the library: Memory Manager (slice + place, Section III-B) and Task Scheduler (one
// layer forward over the CPU / copy / GPU resources, Section III-C) for one MI355X.
//
//   Stream-A  CPU computation  -> CcPool worker threads
//   Stream-B  kernel launches  -> the calling host thread
//   Stream-C  CPU->GPU copies  -> copy_stream (hipMemcpyAsync from pinned memory into a staging ring)
//   Stream-D  GPU computation  -> the caller's stream
// Dependencies: a CG kernel waits for the event recorded after its copy; a copy into a staging
// slot waits for the event recorded after the kernels that last read the slot.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <functional>
#include <string>
#include <thread>
#include <vector>

#include "si_internal.h"
#include "si_error.h"

using namespace si;

namespace {

thread_local std::string g_err;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

}  // namespace

int si::set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_err = buf;
  return code;
}

namespace {

#define HIP_TRY(expr)                                                                           \
  do {                                                                                          \
    hipError_t _e = (expr);                                                                     \
    if (_e != hipSuccess) return fail(SI_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e));  \
  } while (0)

struct Seg { hipEvent_t a, b; int kind; int staged; };  // kind: SI_K_* kernel class, or SEG_COPY
constexpr int SEG_COPY = SI_K_COUNT;

int split_counts(int H, int g, float r_gg, float r_cg, int* n_gg, int* n_cg, int* n_cc) {
  if (H <= 0 || g <= 0 || H % g != 0) return -1;
  const double a = (double)r_gg, b = (double)r_gg + (double)r_cg;
  if (a < 0.0 || (double)r_cg < 0.0 || b > 1.0 + 1e-4) return -1;
  const int units = H / g;
  int ia = (int)std::floor(a * units + 0.5), ib = (int)std::floor(b * units + 0.5);
  ia = std::min(ia, units);
  ib = std::max(std::min(ib, units), ia);
  *n_gg = ia * g;
  *n_cg = (ib - ia) * g;
  *n_cc = H - ib * g;
  return 0;
}

// one expert [H][M] x3 -> chunk-major chunks [c0, c1) written at dst (layout: cc_worker.h)
void repack_chunks(const uint16_t* wg, const uint16_t* wu, const uint16_t* wd, int M, int c0, int c1, uint16_t* dst) {
  const int PW = panel_width(M), NW = ntile_width(M);
  for (int c = c0; c < c1; ++c) {
    uint16_t* o = dst + (size_t)(c - c0) * 3 * CHUNK_J * M;
    for (int f = 0; f < 2; ++f) {
      const uint16_t* src = (f ? wu : wg) + (size_t)c * CHUNK_J * M;
      uint16_t* blk = o + (size_t)f * CHUNK_J * M;
      for (int j = 0; j < CHUNK_J; ++j)
        for (int m = 0; m < M; m += PW) std::memcpy(blk + gu_off(j, m, PW), src + (size_t)j * M + m, (size_t)PW * 2);
    }
    uint16_t* d = o + (size_t)2 * CHUNK_J * M;
    const uint16_t* src = wd + (size_t)c * CHUNK_J * M;
    for (int j = 0; j < CHUNK_J; ++j) {
      const uint16_t* row = src + (size_t)j * M;
      for (int m = 0; m < M; ++m) d[dn_off(j, m, NW)] = row[m];
    }
  }
}

// 4-bit storage form of chunks [c0, c1) of one expert (layout: cc_worker.h).  Sources are the caller's plain
// arrays: codes [H][M/2] (element m in byte m/2, low nibble for even m), scales zg / zu [H][M/64], zd [H/64][M].
void repack_chunks_q4(const uint8_t* qg, const uint8_t* qu, const uint8_t* qd, const uint16_t* zg, const uint16_t* zu,
                      const uint16_t* zd, int M, int c0, int c1, uint16_t* dst16) {
  const int NW = ntile_width(M);
  for (int c = c0; c < c1; ++c) {
    unsigned char* cb = reinterpret_cast<unsigned char*>(dst16 + (size_t)(c - c0) * q4_chunk_u16(M));
    for (int f = 0; f < 2; ++f) {
      const uint8_t* src = (f ? qu : qg) + (size_t)c * CHUNK_J * (M / 2);
      uint32_t* out = reinterpret_cast<uint32_t*>(cb + q4_off_codes(f, M));
      for (size_t wi = 0; wi < (size_t)CHUNK_J * (M / 8); ++wi) {  // rows are contiguous in both layouts
        const uint8_t* b = src + wi * 4;
        out[wi] = (uint32_t)(b[0] & 15) | (uint32_t)(b[1] & 15) << 4 | (uint32_t)(b[2] & 15) << 8 | (uint32_t)(b[3] & 15) << 12 |
                  (uint32_t)(b[0] >> 4) << 16 | (uint32_t)(b[1] >> 4) << 20 | (uint32_t)(b[2] >> 4) << 24 | (uint32_t)(b[3] >> 4) << 28;
      }
      std::memcpy(cb + q4_off_scales(f, M), (f ? zu : zg) + (size_t)c * CHUNK_J * (M / 64), (size_t)CHUNK_J * (M / 64) * 2);
    }
    uint32_t* dout = reinterpret_cast<uint32_t*>(cb + q4_off_codes(2, M));
    std::memset(dout, 0, (size_t)32 * M);
    for (int j = 0; j < CHUNK_J; ++j) {
      const uint8_t* row = qd + ((size_t)c * CHUNK_J + j) * (M / 2);
      const int sh = 4 * q4_fc2_nibble(j);
      for (int m = 0; m < M; ++m) {
        const uint32_t code = (m & 1) ? (row[m >> 1] >> 4) : (row[m >> 1] & 15);
        dout[q4_fc2_word(j, m, NW)] |= code << sh;
      }
    }
    std::memcpy(cb + q4_off_scales(2, M), zd + (size_t)c * M, (size_t)M * 2);
  }
}

// Where the weights of a layer come from: bf16 arrays, or 4-bit codes with scales.
struct WeightSource {
  bool q4 = false;
  const uint16_t *g = nullptr, *u = nullptr, *d = nullptr, *sg = nullptr, *su = nullptr, *sd = nullptr;     // bf16
  const uint8_t *qg = nullptr, *qu = nullptr, *qd = nullptr, *sqg = nullptr, *squ = nullptr, *sqd = nullptr;  // codes
  const uint16_t *zg = nullptr, *zu = nullptr, *zd = nullptr, *szg = nullptr, *szu = nullptr, *szd = nullptr;  // scales
  // library storage of chunks [c, c+1) of routed expert e (e >= 0, hidden size H) or of the shared expert (e < 0)
  void repack(int e, int c, int H, int M, uint16_t* dst) const {
    if (!q4) {
      if (e < 0) repack_chunks(sg, su, sd, M, c, c + 1, dst);
      else repack_chunks(g + (size_t)e * H * M, u + (size_t)e * H * M, d + (size_t)e * H * M, M, c, c + 1, dst);
    } else if (e < 0) {
      repack_chunks_q4(sqg, squ, sqd, szg, szu, szd, M, c, c + 1, dst);
    } else {
      const size_t qo = (size_t)e * H * (M / 2), zo = (size_t)e * H * (M / 64), zdo = (size_t)e * (H / 64) * M;
      repack_chunks_q4(qg + qo, qu + qo, qd + qo, zg + zo, zu + zo, zd + zdo, M, c, c + 1, dst);
    }
  }
};

void parallel_for(int n, int n_threads, const std::function<void(int)>& fn) {
  if (n <= 0) return;
  n_threads = std::max(1, std::min(n_threads, n));
  std::atomic<int> next{0};
  std::vector<std::thread> th;
  for (int i = 0; i < n_threads; ++i)
    th.emplace_back([&] {
      for (;;) {
        int j = next.fetch_add(1);
        if (j >= n) break;
        fn(j);
      }
    });
  for (auto& t : th) t.join();
}

}  // namespace

struct si_layer {
  si_layer_desc_t desc{};
  int M = 0, H = 0, E = 0, k = 0, Hs = 0, EX = 0, has_shared = 0, max_T = 0, device = 0;
  int n_gg = 0, n_cg = 0, n_cc = 0, s_gg = 0, s_cg = 0, s_cc = 0;          // columns
  int ch_gg = 0, ch_cg = 0, ch_cc = 0, sch_gg = 0, sch_cg = 0, sch_cc = 0;  // chunks
  size_t ce = 0;                                                            // uint16 units per chunk
  int q4 = 0;                                                               // 4-bit storage form
  // whole-expert placement: place[e] in {0 GG, 1 CG, 2 CC}; every routed expert keeps all its H/64 chunks in one
  // place.  ch_gg / ch_cg / ch_cc then hold H/64 when any expert is placed there (else 0), so that everything
  // sized from them (staging, slots, workers) stays valid; per-expert counts come from e_chunks().
  int placed = 0;
  std::vector<uint8_t> place;
  std::vector<int32_t> gg_map;   // index of expert e in d_gg (-1: not resident); shared expert entry: 0
  std::vector<uint64_t> h_off;   // uint16 offset of expert e in h_routed
  std::vector<int32_t> e_cc;     // CC chunks per routed expert (for the workers)
  int32_t* d_emap = nullptr;     // device copy of gg_map
  uint16_t* d_gg = nullptr;     // device [E][ch_gg] chunks
  uint16_t* d_sgg = nullptr;    // device [sch_gg] chunks
  uint16_t* h_routed = nullptr; // pinned [E][ch_cc + ch_cg] chunks (CC first, then CG)
  uint16_t* h_shared = nullptr; // pinned [sch_cc + sch_cg] chunks
  int n_stage = 0, stage_chunks = 0;
  std::vector<uint16_t*> d_stage;
  std::vector<hipEvent_t> ev_ready, ev_free;
  std::vector<char> slot_used;
  long piece_counter = 0;
  // CG pieces copied ahead of the forward call that will use them (cross-layer prefetch in a stack):
  // the first pre_n pieces of the CG part, cut for path pre_path, sit in slots pre_slot[0..pre_n)
  int pre_n = 0, pre_path = 0;
  bool pre_shared = false;       // the pieces belong to the shared expert (MoE layer), else to expert 0 of a dense layer
  std::vector<int> pre_slot;
  // timing events of the copies issued ahead of a call live in two pools of their own, used alternately: the call
  // that consumes the pieces merges pre_segs into its own list and flips the pool, so the events its statistics
  // refer to stay untouched until the prefetch after the next one (the layer's own list and pool are never
  // touched from another layer's call)
  std::vector<hipEvent_t> pre_ev_pool[2];
  size_t pre_ev_used = 0;
  int pre_cur = 0;
  std::vector<Seg> pre_segs;
  bool cc_inflight = false;      // the host workers were started and not yet waited for
  si_layer* chain_next = nullptr;  // layer whose CG copies are issued once this call's own are (set by the stack)
  hipStream_t copy_stream = nullptr;      // Stream-C in use: the layer's own, or its stack's
  hipStream_t own_copy_stream = nullptr;  // the one this layer created and destroys
  hipEvent_t ev_host = nullptr;
  // device workspaces
  char* d_plan = nullptr;
  Plan plan{};
  int max_tiles = 0;
  float* d_h = nullptr;       // decode activations [rows_dec][ldh]
  int ldh_dec = 0, rows_dec = 0;
  float* d_part = nullptr;    // decode partials [3*DOWN_SLOTS][rows_dec][M]
  uint16_t* d_deq = nullptr;  // 4-bit layers: bf16 copies of the chunks a prompt-phase GEMM is about to read
  int deq_chunks = 0;         // capacity of d_deq in bf16 chunks
  uint16_t* d_hact = nullptr; // prefill activations
  size_t hact_elems = 0;
  float* d_yp = nullptr;      // prefill per-row outputs [MAX_KSPLIT][max_T*(k+shared)][M]
  size_t yp_slab = 0;         // elements per slab
  float* d_ycc = nullptr;     // [max_T][M]
  // pinned host mirrors
  uint16_t* hx = nullptr;
  int32_t* hidx = nullptr;
  float* hw = nullptr;
  int32_t* hcount = nullptr;  // [EX] count then [EX] count1
  float* hycc = nullptr;
  CcPool* pool = nullptr;
  // stats
  int profiling = 0;
  int in_staged = 0;  // the launches being enqueued read a staged piece
  std::vector<hipEvent_t> ev_pool;
  size_t ev_used = 0;
  std::vector<Seg> segs;
  hipEvent_t ev_t0 = nullptr, ev_t1 = nullptr;
  si_stats_t last{};

  // chunks of part (0 GG, 1 CG, 2 CC) that expert e holds (e == E: the shared expert)
  int e_chunks(int e, int part) const {
    if (e >= E) return part == 0 ? sch_gg : part == 1 ? sch_cg : sch_cc;
    if (placed) return place[e] == part ? H / CHUNK_J : 0;
    return part == 0 ? ch_gg : part == 1 ? ch_cg : ch_cc;
  }
  const uint16_t* host_base(int e) const { return e >= E ? h_shared : h_routed + h_off[e]; }
};

namespace {

template <class T>
int dev_alloc(T** p, size_t n) {
  *p = nullptr;
  if (n == 0) return SI_OK;
  hipError_t e = hipMalloc((void**)p, n * sizeof(T));
  if (e != hipSuccess) { (void)hipGetLastError(); return fail(SI_ENOMEM, "hipMalloc of %zu bytes failed: %s", n * sizeof(T), hipGetErrorString(e)); }
  return SI_OK;
}

template <class T>
int pin_alloc(T** p, size_t n) {
  *p = nullptr;
  if (n == 0) return SI_OK;
  hipError_t e = hipHostMalloc((void**)p, n * sizeof(T), hipHostMallocDefault);
  if (e != hipSuccess) { (void)hipGetLastError(); return fail(SI_ENOMEM, "hipHostMalloc of %zu bytes failed: %s", n * sizeof(T), hipGetErrorString(e)); }
  return SI_OK;
}

hipEvent_t next_event(si_layer* L) {
  if (L->ev_used == L->ev_pool.size()) {
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    L->ev_pool.push_back(e);
  }
  return L->ev_pool[L->ev_used++];
}

struct SegScope {
  si_layer* L; hipStream_t s; int kind; hipEvent_t a = nullptr;
  SegScope(si_layer* l, hipStream_t st, int k) : L(l), s(st), kind(k) {
    if (L->profiling) { a = next_event(L); if (a) (void)hipEventRecord(a, s); }
  }
  ~SegScope() {
    if (L->profiling && a) { hipEvent_t b = next_event(L); if (b) { (void)hipEventRecord(b, s); L->segs.push_back({a, b, kind, L->in_staged}); } }
  }
};

int validate_desc(const si_layer_desc_t* d, int* g_out) {
  if (!d) return fail(SI_EINVAL, "desc is NULL");
  if (d->d_model <= 0 || d->d_model % 64 != 0 || d->d_model > 8192)
    return fail(SI_EINVAL, "d_model=%d must be a positive multiple of 64 (<= 8192)", d->d_model);
  int g = d->granule == 0 ? 64 : d->granule;
  if (g <= 0 || g % 64 != 0) return fail(SI_EINVAL, "granule=%d must be a positive multiple of 64", d->granule);
  if (d->d_ff > 65536 || d->d_ff_shared > 65536) return fail(SI_EINVAL, "d_ff / d_ff_shared must be <= 65536");
  if (d->d_ff <= 0 || d->d_ff % g != 0) return fail(SI_EINVAL, "d_ff=%d must be a positive multiple of granule=%d", d->d_ff, g);
  if (d->d_ff_shared < 0 || d->d_ff_shared % g != 0)
    return fail(SI_EINVAL, "d_ff_shared=%d must be 0 or a multiple of granule=%d", d->d_ff_shared, g);
  if (d->n_experts < 1 || d->n_experts > MAX_EXPERTS) return fail(SI_EINVAL, "n_experts=%d out of range [1,%d]", d->n_experts, MAX_EXPERTS);
  if (d->top_k < 1 || d->top_k > d->n_experts) return fail(SI_EINVAL, "top_k=%d must be in [1, n_experts=%d]", d->top_k, d->n_experts);
  if (!(d->r_gg >= 0.f && d->r_gg <= 1.f && d->r_cg >= 0.f && d->r_cg <= 1.f && d->r_cc >= 0.f && d->r_cc <= 1.f))
    return fail(SI_EINVAL, "rates must each lie in [0,1] (got %g %g %g)", d->r_gg, d->r_cg, d->r_cc);
  if (std::fabs((double)d->r_gg + d->r_cg + d->r_cc - 1.0) > 1e-4)
    return fail(SI_EINVAL, "rates must sum to 1 (got %g)", (double)d->r_gg + d->r_cg + d->r_cc);
  if (d->max_tokens < 1) return fail(SI_EINVAL, "max_tokens=%d must be >= 1", d->max_tokens);
  if (d->cc_threads < 0 || d->cc_threads > 1024) return fail(SI_EINVAL, "cc_threads=%d out of range", d->cc_threads);
  if (d->stage_mib < 0 || d->n_stage < 0 || d->n_stage == 1 || d->n_stage > 16)
    return fail(SI_EINVAL, "stage_mib=%d / n_stage=%d invalid (n_stage must be 0 or in [2,16])", d->stage_mib, d->n_stage);
  if (d->deq_mib < 0 || d->deq_mib > (64 << 10)) return fail(SI_EINVAL, "deq_mib=%d out of range [0, 65536]", d->deq_mib);
  *g_out = g;
  return SI_OK;
}

int ceil_div(int a, int b) { return (a + b - 1) / b; }

}  // namespace

extern "C" {

const char* si_last_error(void) { return g_err.c_str(); }
const char* si_version(void) { return "scheinfer-mi355x 0.1 (gfx950)"; }

int si_split_counts(int32_t d_ff, int32_t granule, float r_gg, float r_cg, int32_t* n_gg, int32_t* n_cg, int32_t* n_cc) {
  int g = granule == 0 ? 64 : granule;
  int a, b, c;
  if (!n_gg || !n_cg || !n_cc) return fail(SI_EINVAL, "output pointer is NULL");
  if (split_counts(d_ff, g, r_gg, r_cg, &a, &b, &c)) return fail(SI_EINVAL, "invalid d_ff/granule/rates");
  *n_gg = a; *n_cg = b; *n_cc = c;
  return SI_OK;
}

int si_repack_chunks(const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down, int32_t d_ff, int32_t d_model,
                     int32_t chunk0, int32_t n_chunks, uint16_t* out) {
  if (!w_gate || !w_up || !w_down || !out) return fail(SI_EINVAL, "NULL pointer");
  if (d_model <= 0 || d_model % 8 != 0 || d_ff <= 0 || d_ff % CHUNK_J != 0) return fail(SI_EINVAL, "bad d_ff=%d / d_model=%d", d_ff, d_model);
  if (chunk0 < 0 || n_chunks < 0 || (chunk0 + n_chunks) * CHUNK_J > d_ff) return fail(SI_EINVAL, "chunk range [%d,+%d) outside d_ff=%d", chunk0, n_chunks, d_ff);
  repack_chunks(w_gate, w_up, w_down, d_model, chunk0, chunk0 + n_chunks, out);
  return SI_OK;
}

static int cc_compute_impl(const uint16_t* x, const int32_t* idx, const float* w, int32_t T1, int32_t k, int32_t d_model,
                           int32_t n_experts, const uint16_t* routed, uint64_t expert_stride, int32_t n_cc_chunks,
                           const uint16_t* shared, int32_t s_cc_chunks, int32_t threads, float* ycc, int q4) {
  if (!x || !idx || !w || !ycc || (!routed && n_cc_chunks > 0)) return fail(SI_EINVAL, "NULL pointer");
  if (T1 < 0 || k < 1 || d_model <= 0 || d_model % 8 != 0 || n_experts < 1 || n_cc_chunks < 0 || s_cc_chunks < 0 || threads < 1)
    return fail(SI_EINVAL, "bad argument");
  for (long q = 0; q < (long)T1 * k; ++q)
    if (idx[q] < 0 || idx[q] >= n_experts) return fail(SI_EINVAL, "idx[%ld]=%d outside [0,%d)", q, idx[q], n_experts);
  if (T1 == 0) return SI_OK;
  CcJob job{};
  job.x = x; job.idx = idx; job.w = w; job.T1 = T1; job.k = k; job.M = d_model; job.E = n_experts;
  job.routed = routed; job.expert_stride = (size_t)expert_stride; job.n_cc_chunks = n_cc_chunks;
  job.shared = s_cc_chunks > 0 ? shared : nullptr; job.s_cc_chunks = shared ? s_cc_chunks : 0; job.ycc = ycc;
  job.q4 = q4;
  if (n_cc_chunks == 0 && !job.shared) { std::memset(ycc, 0, (size_t)T1 * d_model * 4); return SI_OK; }
  CcPool* pool = cc_pool_create(threads);
  cc_pool_run(pool, job);
  cc_pool_destroy(pool);
  return SI_OK;
}

int si_cc_compute(const uint16_t* x, const int32_t* idx, const float* w, int32_t T1, int32_t k, int32_t d_model,
                  int32_t n_experts, const uint16_t* routed, uint64_t expert_stride, int32_t n_cc_chunks,
                  const uint16_t* shared, int32_t s_cc_chunks, int32_t threads, float* ycc) {
  return cc_compute_impl(x, idx, w, T1, k, d_model, n_experts, routed, expert_stride, n_cc_chunks, shared, s_cc_chunks, threads, ycc, 0);
}

int si_repack_chunks_q4(const si_q4_weights_t* w, int32_t d_ff, int32_t d_model, int32_t chunk0, int32_t n_chunks, uint16_t* out) {
  if (!w || !w->q_gate || !w->q_up || !w->q_down || !w->z_gate || !w->z_up || !w->z_down || !out) return fail(SI_EINVAL, "NULL pointer");
  if (d_model <= 0 || d_model % 64 != 0 || d_ff <= 0 || d_ff % CHUNK_J != 0) return fail(SI_EINVAL, "bad d_ff=%d / d_model=%d", d_ff, d_model);
  if (chunk0 < 0 || n_chunks < 0 || (chunk0 + n_chunks) * CHUNK_J > d_ff) return fail(SI_EINVAL, "chunk range [%d,+%d) outside d_ff=%d", chunk0, n_chunks, d_ff);
  repack_chunks_q4(w->q_gate, w->q_up, w->q_down, w->z_gate, w->z_up, w->z_down, d_model, chunk0, chunk0 + n_chunks, out);
  return SI_OK;
}

int si_cc_compute_q4(const uint16_t* x, const int32_t* idx, const float* w, int32_t T1, int32_t k, int32_t d_model,
                     int32_t n_experts, const uint16_t* routed, uint64_t expert_stride, int32_t n_cc_chunks,
                     const uint16_t* shared, int32_t s_cc_chunks, int32_t threads, float* ycc) {
  if (d_model % 64 != 0) return fail(SI_EINVAL, "d_model=%d must be a multiple of 64", d_model);
  return cc_compute_impl(x, idx, w, T1, k, d_model, n_experts, routed, expert_stride, n_cc_chunks, shared, s_cc_chunks, threads, ycc, 1);
}

void si_layer_destroy(si_layer_t* L) {
  if (!L) return;
  (void)hipSetDevice(L->device);
  if (L->pool) cc_pool_destroy(L->pool);
  if (L->copy_stream) { (void)hipStreamSynchronize(L->copy_stream); }
  (void)hipDeviceSynchronize();
  L->copy_stream = L->own_copy_stream;
  for (auto p : L->d_stage) if (p) (void)hipFree(p);
  for (auto e : L->ev_ready) if (e) (void)hipEventDestroy(e);
  for (auto e : L->ev_free) if (e) (void)hipEventDestroy(e);
  for (auto e : L->ev_pool) if (e) (void)hipEventDestroy(e);
  for (auto& pool : L->pre_ev_pool) for (auto e : pool) if (e) (void)hipEventDestroy(e);
  if (L->ev_host) (void)hipEventDestroy(L->ev_host);
  if (L->ev_t0) (void)hipEventDestroy(L->ev_t0);
  if (L->ev_t1) (void)hipEventDestroy(L->ev_t1);
  if (L->copy_stream) (void)hipStreamDestroy(L->copy_stream);
  void* dev[] = {L->d_gg, L->d_sgg, L->d_plan, L->d_h, L->d_part, L->d_hact, L->d_yp, L->d_ycc, L->d_deq, L->d_emap};
  for (void* p : dev) if (p) (void)hipFree(p);
  void* pin[] = {L->h_routed, L->h_shared, L->hx, L->hidx, L->hw, L->hcount, L->hycc};
  for (void* p : pin) if (p) (void)hipHostFree(p);
  delete L;
}

}  // extern "C"

namespace {

// Staging ring (Stream-C) and host workers, sized independently of the slicing rates so that a layer can be
// re-sliced without touching them: a decode piece must hold whole down-projection slots of the largest part an
// expert could have (all of its chunks).
int setup_staging(si_layer* L) {
  if (L->d_stage.empty()) {
    const size_t stage_bytes = (size_t)(L->desc.stage_mib == 0 ? 256 : L->desc.stage_mib) << 20;
    const int sc = (int)std::max<size_t>(1, stage_bytes / (L->ce * 2));
    const int cps_max = std::max({ceil_div(L->H / CHUNK_J, 16), ceil_div(L->Hs / CHUNK_J, 16), 8});  // the largest cps_of() can return
    L->stage_chunks = std::max(sc, cps_max);
    L->d_stage.assign(L->n_stage, nullptr);
    L->ev_ready.assign(L->n_stage, nullptr);
    L->ev_free.assign(L->n_stage, nullptr);
    L->slot_used.assign(L->n_stage, 0);
    for (int i = 0; i < L->n_stage; ++i) {
      int rc = dev_alloc(&L->d_stage[i], (size_t)L->stage_chunks * L->ce);
      if (rc) return rc;
      HIP_TRY(hipEventCreateWithFlags(&L->ev_ready[i], hipEventDisableTiming));
      HIP_TRY(hipEventCreateWithFlags(&L->ev_free[i], hipEventDisableTiming));
    }
  }
  return SI_OK;
}

int setup_pool(si_layer* L) {
  if (!L->pool && L->ch_cc + L->sch_cc > 0) {
    const int hw_threads = (int)std::max(1u, std::thread::hardware_concurrency());
    L->pool = cc_pool_create(L->desc.cc_threads == 0 ? std::min(16, hw_threads) : L->desc.cc_threads);
  }
  return SI_OK;
}

int create_impl(const si_layer_desc_t* desc, const WeightSource& src, const uint8_t* placement, si_layer_t** out) {
  int g = 64;
  if (!out) return fail(SI_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = validate_desc(desc, &g);
  if (rc) return rc;
  if (!src.q4) {
    if (!src.g || !src.u || !src.d) return fail(SI_EINVAL, "expert weight pointer is NULL");
    if (desc->d_ff_shared > 0 && (!src.sg || !src.su || !src.sd))
      return fail(SI_EINVAL, "d_ff_shared > 0 but a shared weight pointer is NULL");
  } else {
    if (!src.qg || !src.qu || !src.qd || !src.zg || !src.zu || !src.zd) return fail(SI_EINVAL, "expert code or scale pointer is NULL");
    if (desc->d_ff_shared > 0 && (!src.sqg || !src.squ || !src.sqd || !src.szg || !src.szu || !src.szd))
      return fail(SI_EINVAL, "d_ff_shared > 0 but a shared code or scale pointer is NULL");
  }
  int n_dev = 0;
  if (hipGetDeviceCount(&n_dev) != hipSuccess || desc->device < 0 || desc->device >= n_dev) {
    (void)hipGetLastError();
    return fail(SI_EHIP, "HIP device %d not available (%d devices visible)", desc->device, n_dev);
  }
  HIP_TRY(hipSetDevice(desc->device));

  si_layer* L = new si_layer();
  L->desc = *desc;
  L->M = desc->d_model; L->H = desc->d_ff; L->E = desc->n_experts; L->k = desc->top_k; L->Hs = desc->d_ff_shared;
  L->has_shared = L->Hs > 0; L->EX = L->E + L->has_shared; L->max_T = desc->max_tokens; L->device = desc->device;
  split_counts(L->H, g, desc->r_gg, desc->r_cg, &L->n_gg, &L->n_cg, &L->n_cc);
  if (L->has_shared) split_counts(L->Hs, g, desc->r_gg, desc->r_cg, &L->s_gg, &L->s_cg, &L->s_cc);
  L->ch_gg = L->n_gg / CHUNK_J; L->ch_cg = L->n_cg / CHUNK_J; L->ch_cc = L->n_cc / CHUNK_J;
  L->sch_gg = L->s_gg / CHUNK_J; L->sch_cg = L->s_cg / CHUNK_J; L->sch_cc = L->s_cc / CHUNK_J;
  int n_place[3] = {0, 0, 0};
  if (placement) {
    L->placed = 1;
    L->place.assign(placement, placement + L->E);
    for (int e = 0; e < L->E; ++e) {
      if (placement[e] > 2) { const int v = placement[e]; delete L; return fail(SI_EINVAL, "placement[%d]=%d must be 0 (GG), 1 (CG) or 2 (CC)", e, v); }
      n_place[placement[e]]++;
    }
    const int Hch = L->H / CHUNK_J;
    L->ch_gg = n_place[0] ? Hch : 0; L->ch_cg = n_place[1] ? Hch : 0; L->ch_cc = n_place[2] ? Hch : 0;
    L->n_gg = L->ch_gg * CHUNK_J; L->n_cg = L->ch_cg * CHUNK_J; L->n_cc = L->ch_cc * CHUNK_J;
  }
  L->q4 = src.q4 ? 1 : 0;
  L->ce = src.q4 ? q4_chunk_u16(L->M) : chunk_elems(L->M);
  const int M = L->M, E = L->E, k = L->k, T = L->max_T;
  const size_t ce = L->ce;
  const int hch = L->ch_cc + L->ch_cg, shch = L->sch_cc + L->sch_cg;
  // per-expert storage: index in d_gg, offset in h_routed, CC chunks
  L->gg_map.assign(L->EX, 0);
  L->h_off.assign(L->E, 0);
  L->e_cc.assign(L->E, 0);
  size_t gg_experts = 0, host_units = 0;
  for (int e = 0; e < L->E; ++e) {
    const int g_e = L->e_chunks(e, 0), h_e = L->e_chunks(e, 1) + L->e_chunks(e, 2);
    L->gg_map[e] = g_e > 0 || !L->placed ? (int32_t)gg_experts : -1;
    if (g_e > 0 || !L->placed) ++gg_experts;
    L->h_off[e] = host_units;
    host_units += (size_t)h_e * L->ce;
    L->e_cc[e] = L->e_chunks(e, 2);
  }

#define TRY_OR_DESTROY(expr) do { int _rc = (expr); if (_rc) { si_layer_destroy(L); return _rc; } } while (0)
#define HIP_OR_DESTROY(expr) do { hipError_t _e = (expr); if (_e != hipSuccess) { fail(SI_EHIP, "%s failed: %s", #expr, hipGetErrorString(_e)); si_layer_destroy(L); return SI_EHIP; } } while (0)

  // ---- placement: GG -> device, CC | CG -> pinned host (CG' aliases the CC range)
  TRY_OR_DESTROY(dev_alloc(&L->d_gg, gg_experts * L->ch_gg * ce));
  TRY_OR_DESTROY(dev_alloc(&L->d_sgg, (size_t)L->sch_gg * ce));
  TRY_OR_DESTROY(pin_alloc(&L->h_routed, host_units));
  if (L->placed) {
    TRY_OR_DESTROY(dev_alloc(&L->d_emap, (size_t)L->EX));
    HIP_OR_DESTROY(hipMemcpy(L->d_emap, L->gg_map.data(), (size_t)L->EX * 4, hipMemcpyHostToDevice));
  }
  TRY_OR_DESTROY(pin_alloc(&L->h_shared, (size_t)shch * ce));
  const int hw_threads = (int)std::max(1u, std::thread::hardware_concurrency());
  const int rp_threads = std::min(16, hw_threads);
  {
    // host parts: repack straight into the pinned buffers
    // host chunks of expert e: its CC range then its CG range = source chunks [0, CC + CG) in both modes (a placed
    // expert has all its chunks in one of the two)
    std::vector<std::pair<int, int>> host_items;
    for (int e = 0; e < E; ++e)
      for (int c = 0; c < L->e_chunks(e, 1) + L->e_chunks(e, 2); ++c) host_items.push_back({e, c});
    parallel_for((int)host_items.size(), rp_threads, [&](int i) {
      const int e = host_items[i].first, c = host_items[i].second;
      src.repack(e, c, L->H, M, L->h_routed + L->h_off[e] + (size_t)c * ce);
    });
    parallel_for(shch, rp_threads, [&](int c) { src.repack(-1, c, L->Hs, M, L->h_shared + (size_t)c * ce); });
    // GG parts: repack through a pinned bounce buffer, a group of chunks at a time
    const int bounce_chunks = std::max(1, (int)std::min<size_t>(256, ((size_t)256 << 20) / (ce * 2)));
    uint16_t* bounce = nullptr;
    if ((size_t)E * L->ch_gg + L->sch_gg > 0) TRY_OR_DESTROY(pin_alloc(&bounce, (size_t)bounce_chunks * ce));
    auto upload = [&](int e, int Hx, int c_first, int n, uint16_t* dst) -> hipError_t {
      for (int c0 = 0; c0 < n; c0 += bounce_chunks) {
        int nb = std::min(bounce_chunks, n - c0);
        parallel_for(nb, rp_threads, [&](int i) { src.repack(e, c_first + c0 + i, Hx, M, bounce + (size_t)i * ce); });
        hipError_t e2 = hipMemcpy(dst + (size_t)c0 * ce, bounce, (size_t)nb * ce * 2, hipMemcpyHostToDevice);
        if (e2 != hipSuccess) return e2;
      }
      return hipSuccess;
    };
    hipError_t ue = hipSuccess;
    for (int e = 0; e < E && ue == hipSuccess; ++e)
      if (L->e_chunks(e, 0) > 0)
        ue = upload(e, L->H, L->placed ? 0 : hch, L->ch_gg, L->d_gg + (size_t)L->gg_map[e] * L->ch_gg * ce);
    if (ue == hipSuccess && L->has_shared) ue = upload(-1, L->Hs, shch, L->sch_gg, L->d_sgg);
    if (bounce) (void)hipHostFree(bounce);
    HIP_OR_DESTROY(ue);
  }

  // ---- staging ring for CG / CG' copies (Stream-C)
  L->n_stage = desc->n_stage == 0 ? 2 : desc->n_stage;
  const bool any_host = hch + shch > 0;
  if (any_host) TRY_OR_DESTROY(setup_staging(L));
  HIP_OR_DESTROY(hipStreamCreateWithFlags(&L->copy_stream, hipStreamNonBlocking));
  L->own_copy_stream = L->copy_stream;
  HIP_OR_DESTROY(hipEventCreateWithFlags(&L->ev_host, hipEventDisableTiming));
  HIP_OR_DESTROY(hipEventCreate(&L->ev_t0));
  HIP_OR_DESTROY(hipEventCreate(&L->ev_t1));

  // ---- workspaces
  const size_t n_pairs = (size_t)T * k, n_rows = n_pairs + (L->has_shared ? T : 0);
  L->max_tiles = (int)(n_rows / 64) + L->EX + 2;  // row-tile tables for the smallest tile (64 rows)
  {
    size_t ints = 0;
    auto take = [&](size_t n) { size_t o = ints; ints += (n + 3) / 4 * 4; return o; };
    size_t o_idx = take(n_pairs), o_w = take(n_pairs), o_count = take(L->EX), o_off = take(L->EX + 1), o_count1 = take(L->EX),
           o_perm = take(n_pairs), o_inv = take(n_pairs), o_rt = take(n_rows), o_touched = take(L->EX), o_nt = take(4),
           o_te = take(L->max_tiles), o_tr = take(L->max_tiles), o_te2 = take(L->max_tiles), o_tr2 = take(L->max_tiles);
    TRY_OR_DESTROY(dev_alloc(&L->d_plan, ints * 4));
    int32_t* b = reinterpret_cast<int32_t*>(L->d_plan);
    L->plan.idx = b + o_idx; L->plan.w = reinterpret_cast<float*>(b + o_w); L->plan.count = b + o_count;
    L->plan.off = b + o_off; L->plan.count1 = b + o_count1; L->plan.perm = b + o_perm; L->plan.inv = b + o_inv;
    L->plan.row_token = b + o_rt; L->plan.touched = b + o_touched; L->plan.n_touched = b + o_nt;
    L->plan.n_tiles = b + o_nt + 1; L->plan.n_tiles_x2 = b + o_nt + 2; L->plan.tile_flags = b + o_nt + 3;
    L->plan.n_routed = E;
    L->plan.tile_e = b + o_te; L->plan.tile_r = b + o_tr; L->plan.tile_e_x2 = b + o_te2; L->plan.tile_r_x2 = b + o_tr2;
  }
  const int T_dec = std::min(T, SI_DECODE_MAX_T);
  L->rows_dec = T_dec * (k + L->has_shared);
  L->ldh_dec = std::max(L->H, L->Hs);
  TRY_OR_DESTROY(dev_alloc(&L->d_h, (size_t)L->rows_dec * L->ldh_dec));
  TRY_OR_DESTROY(dev_alloc(&L->d_part, (size_t)3 * DOWN_SLOTS * L->rows_dec * M));
  {
    // widest launch whatever the slicing rates: a part never has more columns than its expert
    int cols = std::max(L->H, L->Hs);
    if (L->q4 && desc->deq_mib > 0) {
      // two-pass prompt phase on request: bf16 scratch that a dequantisation kernel fills and the bf16 GEMMs read
      // (the fewer sub-pieces, the fewer short launches), at least one chunk per routed expert, never more than
      // the largest part needs.  By default (deq_mib = 0) the GEMMs convert the codes on their way into LDS.
      const size_t cb16 = chunk_elems(M) * 2;
      L->deq_chunks = (int)std::max<size_t>((size_t)E, ((size_t)desc->deq_mib << 20) / cb16);
      L->deq_chunks = std::min(L->deq_chunks, std::max(E, E * std::max({L->H / CHUNK_J, L->Hs / CHUNK_J, 1})));
      TRY_OR_DESTROY(dev_alloc(&L->d_deq, (size_t)L->deq_chunks * chunk_elems(M)));
      cols = std::max(cols, L->deq_chunks * CHUNK_J);
    }
    L->hact_elems = n_rows * (size_t)cols;
    // the prompt-phase GEMMs address the rows of their A operands (x, then the activations) with 32-bit element offsets
    if (L->hact_elems >= ((size_t)1 << 31) || (size_t)T * M >= ((size_t)1 << 31)) {
      fail(SI_EINVAL, "max_tokens = %d too large: an operand of the prompt-phase GEMMs would exceed 2^31 elements", T);
      si_layer_destroy(L);
      return SI_EINVAL;
    }
    TRY_OR_DESTROY(dev_alloc(&L->d_hact, L->hact_elems));
    L->yp_slab = n_rows * (size_t)M;
    TRY_OR_DESTROY(dev_alloc(&L->d_yp, (size_t)MAX_KSPLIT * L->yp_slab));
  }
  TRY_OR_DESTROY(dev_alloc(&L->d_ycc, (size_t)T * M));
  TRY_OR_DESTROY(pin_alloc(&L->hx, (size_t)T * M));
  TRY_OR_DESTROY(pin_alloc(&L->hidx, n_pairs));
  TRY_OR_DESTROY(pin_alloc(&L->hw, n_pairs));
  TRY_OR_DESTROY(pin_alloc(&L->hcount, (size_t)2 * L->EX));
  TRY_OR_DESTROY(pin_alloc(&L->hycc, (size_t)T * M));
  TRY_OR_DESTROY(setup_pool(L));
  HIP_OR_DESTROY(hipDeviceSynchronize());
  *out = L;
  return SI_OK;
}

}  // namespace

extern "C" {

int si_layer_create(const si_layer_desc_t* desc, const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down,
                    const uint16_t* shared_gate, const uint16_t* shared_up, const uint16_t* shared_down,
                    si_layer_t** out) {
  WeightSource src;
  src.g = w_gate; src.u = w_up; src.d = w_down; src.sg = shared_gate; src.su = shared_up; src.sd = shared_down;
  return create_impl(desc, src, nullptr, out);
}

int si_layer_create_placed(const si_layer_desc_t* desc, const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down,
                           const uint16_t* shared_gate, const uint16_t* shared_up, const uint16_t* shared_down,
                           const uint8_t* placement, si_layer_t** out) {
  if (!placement) return fail(SI_EINVAL, "placement is NULL");
  WeightSource src;
  src.g = w_gate; src.u = w_up; src.d = w_down; src.sg = shared_gate; src.su = shared_up; src.sd = shared_down;
  return create_impl(desc, src, placement, out);
}

int si_layer_create_q4(const si_layer_desc_t* desc, const si_q4_weights_t* routed, const si_q4_weights_t* shared,
                       const uint8_t* placement, si_layer_t** out) {
  if (!routed) return fail(SI_EINVAL, "routed is NULL");
  if (desc && desc->d_ff_shared > 0 && !shared) return fail(SI_EINVAL, "d_ff_shared > 0 but shared is NULL");
  WeightSource src;
  src.q4 = true;
  src.qg = routed->q_gate; src.qu = routed->q_up; src.qd = routed->q_down;
  src.zg = routed->z_gate; src.zu = routed->z_up; src.zd = routed->z_down;
  if (shared) {
    src.sqg = shared->q_gate; src.squ = shared->q_up; src.sqd = shared->q_down;
    src.szg = shared->z_gate; src.szu = shared->z_up; src.szd = shared->z_down;
  }
  return create_impl(desc, src, placement, out);
}

int si_layer_resplit(si_layer_t* L, float r_gg, float r_cg, float r_cc) {
  if (!L) return fail(SI_EINVAL, "layer is NULL");
  if (L->placed) return fail(SI_ESTATE, "a layer with whole-expert placement has no slicing rates to change");
  si_layer_desc_t d = L->desc;
  d.r_gg = r_gg; d.r_cg = r_cg; d.r_cc = r_cc;
  int g = 64;
  if (int rc = validate_desc(&d, &g)) return rc;
  HIP_TRY(hipSetDevice(L->device));
  int n_gg, n_cg, n_cc, s_gg = 0, s_cg = 0, s_cc = 0;
  split_counts(L->H, g, r_gg, r_cg, &n_gg, &n_cg, &n_cc);
  if (L->has_shared) split_counts(L->Hs, g, r_gg, r_cg, &s_gg, &s_cg, &s_cc);
  // nothing may be in flight on the old buffers (a forward call that failed half-way may have left the host workers running)
  if (L->pool) cc_pool_wait(L->pool);
  HIP_TRY(hipStreamSynchronize(L->copy_stream));
  HIP_TRY(hipDeviceSynchronize());
  const size_t ce = L->ce;

  // Move the chunks of one expert set (n_exp experts of `total` chunks each) from the old boundary between host
  // and device (host_old chunks on the host, the rest resident) to the new one.  Chunk c of expert e sits at
  // host[e*host_n + c] for c < host_n, else at dev[e*(total - host_n) + c - host_n].
  auto move = [&](int n_exp, int total, int host_old, int host_new, uint16_t** host, uint16_t** dev) -> int {
    if (host_old == host_new) return SI_OK;
    uint16_t *nh = nullptr, *nd = nullptr;
    int rc = pin_alloc(&nh, (size_t)n_exp * host_new * ce);
    if (rc == SI_OK) rc = dev_alloc(&nd, (size_t)n_exp * (total - host_new) * ce);
    const int keep_h = std::min(host_old, host_new), keep_d0 = std::max(host_old, host_new);
    const int gg_old = total - host_old, gg_new = total - host_new;
    for (int e = 0; e < n_exp && rc == SI_OK; ++e) {
      hipError_t he = hipSuccess;
      if (keep_h > 0) std::memcpy(nh + (size_t)e * host_new * ce, *host + (size_t)e * host_old * ce, (size_t)keep_h * ce * 2);
      if (host_new > host_old)  // chunks [host_old, host_new) leave the GPU
        he = hipMemcpy(nh + ((size_t)e * host_new + host_old) * ce, *dev + (size_t)e * gg_old * ce,
                       (size_t)(host_new - host_old) * ce * 2, hipMemcpyDeviceToHost);
      else                      // chunks [host_new, host_old) become resident
        he = hipMemcpy(nd + (size_t)e * gg_new * ce, *host + ((size_t)e * host_old + host_new) * ce,
                       (size_t)(host_old - host_new) * ce * 2, hipMemcpyHostToDevice);
      if (he == hipSuccess && total > keep_d0)  // chunks [keep_d0, total) stay resident
        he = hipMemcpy(nd + ((size_t)e * gg_new + (keep_d0 - host_new)) * ce, *dev + ((size_t)e * gg_old + (keep_d0 - host_old)) * ce,
                       (size_t)(total - keep_d0) * ce * 2, hipMemcpyDeviceToDevice);
      if (he != hipSuccess) rc = fail(SI_EHIP, "copy while re-slicing failed: %s", hipGetErrorString(he));
    }
    if (rc != SI_OK) {
      if (nh) (void)hipHostFree(nh);
      if (nd) (void)hipFree(nd);
      return rc;
    }
    if (*host) (void)hipHostFree(*host);
    if (*dev) (void)hipFree(*dev);
    *host = nh;
    *dev = nd;
    return SI_OK;
  };
  const int Hch = L->H / CHUNK_J, sHch = L->Hs / CHUNK_J;
  // Routed experts first, then the shared expert; each set either moves completely or keeps its old buffers, and
  // the counts of a set change with its buffers, so the layer stays usable if the second move runs out of memory.
  int rc = move(L->E, Hch, L->ch_cc + L->ch_cg, (n_cc + n_cg) / CHUNK_J, &L->h_routed, &L->d_gg);
  if (rc == SI_OK) {
    L->n_gg = n_gg; L->n_cg = n_cg; L->n_cc = n_cc;
    L->ch_gg = n_gg / CHUNK_J; L->ch_cg = n_cg / CHUNK_J; L->ch_cc = n_cc / CHUNK_J;
    for (int e = 0; e < L->E; ++e) { L->h_off[e] = (uint64_t)e * (L->ch_cc + L->ch_cg) * ce; L->e_cc[e] = L->ch_cc; }
    if (L->has_shared) rc = move(1, sHch, L->sch_cc + L->sch_cg, (s_cc + s_cg) / CHUNK_J, &L->h_shared, &L->d_sgg);
    if (rc == SI_OK) {
      L->s_gg = s_gg; L->s_cg = s_cg; L->s_cc = s_cc;
      L->sch_gg = s_gg / CHUNK_J; L->sch_cg = s_cg / CHUNK_J; L->sch_cc = s_cc / CHUNK_J;
      L->desc.r_gg = r_gg; L->desc.r_cg = r_cg; L->desc.r_cc = r_cc;
    }
  }
  L->pre_n = 0;
  L->pre_slot.clear();
  if (L->ch_cc + L->ch_cg + L->sch_cc + L->sch_cg > 0) {
    const int rc2 = setup_staging(L);
    if (rc2) return rc2;
  }
  const int rc3 = setup_pool(L);
  return rc ? rc : rc3;
}

int si_layer_split_info(const si_layer_t* L, int32_t* n_gg, int32_t* n_cg, int32_t* n_cc, int32_t* s_gg, int32_t* s_cg, int32_t* s_cc) {
  if (!L) return fail(SI_EINVAL, "layer is NULL");
  if (n_gg) *n_gg = L->n_gg;
  if (n_cg) *n_cg = L->n_cg;
  if (n_cc) *n_cc = L->n_cc;
  if (s_gg) *s_gg = L->s_gg;
  if (s_cg) *s_cg = L->s_cg;
  if (s_cc) *s_cc = L->s_cc;
  return SI_OK;
}

int si_layer_set_profiling(si_layer_t* L, int32_t on) {
  if (!L) return fail(SI_EINVAL, "layer is NULL");
  L->profiling = on ? 1 : 0;
  return SI_OK;
}

int si_route(const float* logits_dev, int32_t T, int32_t E, int32_t k, const si_routing_out_t* out, void* stream) {
  if (!logits_dev || !out) return fail(SI_EINVAL, "logits_dev or out is NULL");
  if (T < 0 || E < 1 || E > MAX_EXPERTS || k < 1 || k > E) return fail(SI_EINVAL, "bad T=%d E=%d k=%d", T, E, k);
  if (T == 0) return SI_OK;
  // scratch for idx / w when the caller does not ask for them
  int32_t* tmp = nullptr;
  const size_t n = (size_t)T * k;
  Plan p{};
  RouteOut u{nullptr, nullptr, out->count, out->off, out->perm, out->inv};
  hipStream_t s = (hipStream_t)stream;
  if (!out->idx || !out->w) {
    HIP_TRY(hipMallocAsync((void**)&tmp, 2 * n * 4, s));
  }
  p.idx = out->idx ? out->idx : tmp;
  p.w = out->w ? out->w : reinterpret_cast<float*>(tmp + n);
  hipError_t e = launch_route(logits_dev, T, E, k, 0, 0, p, u, s);
  if (tmp) (void)hipFreeAsync(tmp, s);
  if (e != hipSuccess) return fail(SI_EHIP, "route launch failed: %s", hipGetErrorString(e));
  return SI_OK;
}

}  // extern "C"

namespace {

// chunks per j-slot of the decode down projection: at most DOWN_SLOTS slots per part, and at least 8 chunks
// (256 KB of weights per block) so that small experts do not shatter into tiny blocks
// A launch over many experts gets at most 16 slots per expert; a launch over one large expert (a dense layer, a shared
// expert) up to DOWN_SLOTS when 16 slots would leave fewer than two blocks per compute unit (each block walks its
// chunks one after the other with eight loads per lane in flight, so few long blocks leave the memory system idle:
// the shared expert of the Qwen-shaped layer went from 2.5 to 5 TB/s).
int cps_of(int ch, bool single_expert, int M) {
  const int slots = single_expert && ceil_div(M, 256) * 16 < 512 ? DOWN_SLOTS : 16;
  return std::max(1, std::max(ceil_div(ch, slots), std::min(8, ch)));
}

// chunks per staged piece of a part with `cps` chunks per j-slot
int piece_chunks(const si_layer* L, int path, int cps) {
  return path == SI_DECODE ? std::max(cps, L->stage_chunks / cps * cps) : L->stage_chunks;
}

// Copy the first CG pieces of a layer into its staging ring ahead of its forward call (as many as the ring has
// slots): what can travel before the layer's own token assignment is known.  A dense layer: its one expert.  An MoE
// layer: its shared expert, which every token uses (which routed experts are streamed is known only after the
// assignment); the forward call then takes the shared expert first, while the ring still holds the pieces.
int prefetch_cg(si_layer* N, int path) {
  if (N->pre_n > 0) return SI_OK;
  const bool dense = N->E == 1 && !N->has_shared && N->ch_cg > 0;
  const bool shared = N->E > 1 && N->has_shared && N->sch_cg > 0 && !N->placed;
  if (!dense && !shared) return SI_OK;
  HIP_TRY(hipSetDevice(N->device));
  const int n_cg = dense ? N->ch_cg : N->sch_cg, n_cc = dense ? N->ch_cc : N->sch_cc;
  const int piece_max = piece_chunks(N, path, cps_of(n_cg, true, N->M));
  const uint16_t* hbase = dense ? N->h_routed : N->h_shared;
  N->pre_segs.clear();
  N->pre_ev_used = 0;
  auto pre_event = [&]() -> hipEvent_t {
    auto& pool = N->pre_ev_pool[N->pre_cur];
    if (N->pre_ev_used == pool.size()) {
      hipEvent_t e = nullptr;
      if (hipEventCreate(&e) != hipSuccess) return nullptr;
      pool.push_back(e);
    }
    return pool[N->pre_ev_used++];
  };
  N->pre_slot.clear();
  for (int c = 0; c < n_cg && (int)N->pre_slot.size() < N->n_stage; c += piece_max) {
    const int n = std::min(piece_max, n_cg - c);
    const int slot = (int)(N->piece_counter++ % N->n_stage);
    if (N->slot_used[slot]) HIP_TRY(hipStreamWaitEvent(N->copy_stream, N->ev_free[slot], 0));
    hipEvent_t ea = N->profiling ? pre_event() : nullptr, eb = ea ? pre_event() : nullptr;
    if (eb) HIP_TRY(hipEventRecord(ea, N->copy_stream));
    HIP_TRY(hipMemcpyAsync(N->d_stage[slot], hbase + (size_t)(n_cc + c) * N->ce, (size_t)n * N->ce * 2, hipMemcpyHostToDevice, N->copy_stream));
    if (eb) { HIP_TRY(hipEventRecord(eb, N->copy_stream)); N->pre_segs.push_back({ea, eb, SEG_COPY, 0}); }
    HIP_TRY(hipEventRecord(N->ev_ready[slot], N->copy_stream));
    N->pre_slot.push_back(slot);
  }
  N->pre_n = (int)N->pre_slot.size();
  N->pre_path = path;
  N->pre_shared = shared;
  return SI_OK;
}

}  // namespace

extern "C" {


int si_layer_forward(si_layer_t* L, const void* x_dev, const float* logits_dev, int32_t T, int32_t n_g, int32_t mode,
                     float* y_dev, const si_routing_out_t* rout, void* stream_v) {
  if (!L) return fail(SI_EINVAL, "layer is NULL");
  if (T < 0 || n_g < 0 || n_g > T) return fail(SI_EINVAL, "need 0 <= n_g <= T (T=%d n_g=%d)", T, n_g);
  if (mode != SI_AUTO && mode != SI_DECODE && mode != SI_PREFILL) return fail(SI_EINVAL, "bad mode %d", mode);
  if (T > L->max_T) return fail(SI_ESTATE, "T=%d exceeds max_tokens=%d", T, L->max_T);
  if (T == 0) return SI_OK;
  if (!x_dev || !y_dev) return fail(SI_EINVAL, "x_dev or y_dev is NULL");
  if (L->E > 1 && !logits_dev) return fail(SI_EINVAL, "logits_dev is NULL for a layer with %d experts", L->E);
  const bool few_rows = T <= SI_DECODE_AUTO_T && ceil_div(T * L->k, L->E) <= SI_DECODE_AUTO_ROWS;
  const int path = mode == SI_AUTO ? (few_rows ? SI_DECODE : SI_PREFILL) : mode;
  if (path == SI_DECODE && T > SI_DECODE_MAX_T) return fail(SI_ESTATE, "SI_DECODE needs T <= %d (T=%d)", SI_DECODE_MAX_T, T);
  HIP_TRY(hipSetDevice(L->device));
  hipStream_t stream = (hipStream_t)stream_v;
  const uint16_t* x = static_cast<const uint16_t*>(x_dev);
  const int M = L->M, E = L->E, k = L->k, EX = L->EX;
  const size_t ce = L->ce;
  const int n_x1 = T - n_g;
  const int hch = L->ch_cc + L->ch_cg;
  const bool any_cc = L->ch_cc + L->sch_cc > 0, any_cg = L->ch_cg + L->sch_cg > 0;
  const bool need_cc = any_cc && n_x1 > 0;   // Stream-A work
  const bool need_cgp = any_cc && n_g > 0;   // CG': CC weights on the GPU for X2
  const bool need_counts = (any_cg || need_cgp) && E > 1;  // which experts to stream
  const bool need_sync = need_cc || need_counts;
  const auto wall0 = std::chrono::steady_clock::now();

  // Whatever way the call ends, nothing of it may outlive it on the host: on an error return the host workers are
  // waited for (they read hx / hidx / hw, which the next call overwrites) and the prefetch state is dropped.
  struct ExitGuard {
    si_layer* L; bool ok = false;
    ~ExitGuard() {
      if (ok) return;
      if (L->cc_inflight) { cc_pool_wait(L->pool); L->cc_inflight = false; }
      L->pre_n = 0;
      L->in_staged = 0;
    }
  } guard{L};
  L->ev_used = 0;
  L->segs.clear();
  L->in_staged = 0;
  if (L->pre_n > 0 && L->pre_path != path) L->pre_n = 0;  // cut for the other path: copy again
  if (L->pre_n > 0 && !L->pre_segs.empty()) {
    // the copies issued ahead of this call belong to its statistics; their events stay valid until the prefetch
    // after the next one (prefetch_cg records into the other pool from now on)
    L->segs.insert(L->segs.end(), L->pre_segs.begin(), L->pre_segs.end());
    L->pre_cur ^= 1;
  }
  L->pre_segs.clear();
  si_stats_t st{};
  st.path = path;
  st.n_touched = -1;
  if (L->profiling) HIP_TRY(hipEventRecord(L->ev_t0, stream));

  // ---- token assignment (Section II-A)
  RouteOut u{};
  if (rout) u = RouteOut{rout->idx, rout->w, rout->count, rout->off, rout->perm, rout->inv};
  // Generation phase of a fully resident bf16 layer with very few (token, expert) pairs: a launch costs as much as
  // reading tens of megabytes of weights (Section III-C: with few tokens the launch time rivals the compute time),
  // so the assignment is derived inside the first gate/up launch instead of by a kernel of its own.
  const bool resident_only = !any_cg && !need_cgp && !need_cc && !L->placed && !L->q4 && L->ch_gg > 0;
  bool fuse_route = path == SI_DECODE && resident_only && T <= FUSED_ROUTE_MAX_T && T * k <= FUSED_ROUTE_MAX_PAIRS;
  FusedRoute fr{E > 1 ? logits_dev : nullptr, T, E, k, L->has_shared, n_x1, u};
  if (!fuse_route) {
    SegScope sc(L, stream, 0);
    hipError_t e = launch_route(E > 1 ? logits_dev : nullptr, T, E, k, L->has_shared, n_g, L->plan, u, stream);
    if (e != hipSuccess) return fail(SI_EHIP, "route launch failed: %s", hipGetErrorString(e));
  }
  // ---- hand-off to the host: the rows of X1 and the assignment go to the CPU for the CC part (Section III-B),
  //      and with them the per-expert counts the copy scheduler needs
  if (need_sync) {
    if (need_cc) {
      HIP_TRY(hipMemcpyAsync(L->hx, x, (size_t)n_x1 * M * 2, hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipMemcpyAsync(L->hidx, L->plan.idx, (size_t)T * k * 4, hipMemcpyDeviceToHost, stream));
      HIP_TRY(hipMemcpyAsync(L->hw, L->plan.w, (size_t)T * k * 4, hipMemcpyDeviceToHost, stream));
    }
    HIP_TRY(hipMemcpyAsync(L->hcount, L->plan.count, (size_t)EX * 4, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipMemcpyAsync(L->hcount + EX, L->plan.count1, (size_t)EX * 4, hipMemcpyDeviceToHost, stream));
    HIP_TRY(hipEventRecord(L->ev_host, stream));
    const auto h0 = std::chrono::steady_clock::now();
    HIP_TRY(hipEventSynchronize(L->ev_host));
    st.handoff_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - h0).count();
    int nt = 0;
    for (int e = 0; e < EX; ++e) nt += L->hcount[e] > 0;
    st.n_touched = nt;
  } else if (E == 1) {
    st.n_touched = EX;
  }
  std::chrono::steady_clock::time_point cc0;
  if (need_cc) {
    CcJob job{};
    job.x = L->hx; job.idx = L->hidx; job.w = L->hw; job.T1 = n_x1; job.k = k; job.M = M; job.E = E;
    job.routed = L->h_routed; job.expert_stride = (size_t)hch * ce; job.n_cc_chunks = L->ch_cc;
    if (L->placed) { job.e_off = L->h_off.data(); job.e_cc_chunks = L->e_cc.data(); }
    job.shared = (L->has_shared && L->sch_cc > 0) ? L->h_shared : nullptr; job.s_cc_chunks = L->sch_cc;
    job.ycc = L->hycc;
    job.q4 = L->q4;
    if (L->ch_cc == 0 && !job.shared) {
      std::memset(L->hycc, 0, (size_t)n_x1 * M * 4);
    } else {
      cc0 = std::chrono::steady_clock::now();
      cc_pool_start(L->pool, job);
      L->cc_inflight = true;
    }
  }

  // counts per expert as known on the host (dense layers need no copy)
  auto rows_all = [&](int e) { return need_sync ? L->hcount[e] : T; };
  auto rows_x2 = [&](int e) { return need_sync ? L->hcount[e] - L->hcount[EX + e] : n_g; };
  const int max_touched = std::min(EX, T * k + L->has_shared);
  const int tiles_upper = (T * k) / TILE_ROWS + std::min(E, T * k);  // bound on the routed row tiles
  // (whole-expert placement: every routed expert has H/64 chunks wherever it lives)
  const bool one = E == 1;
  const int cps_gg = cps_of(L->placed ? L->H / CHUNK_J : L->ch_gg, one, M), cps_cg = cps_of(L->placed ? L->H / CHUNK_J : L->ch_cg, one, M),
            cps_cc = cps_of(L->placed ? L->H / CHUNK_J : L->ch_cc, one, M);
  const int scps_gg = cps_of(L->sch_gg, true, M), scps_cg = cps_of(L->sch_cg, true, M), scps_cc = cps_of(L->sch_cc, true, M);
  const size_t slot_stride = (size_t)L->rows_dec * M;
  // k-splits of the prefill down projection: enough blocks to fill 256 CUs when there are few row tiles
  const int n_ntiles = ceil_div(M, 256);
  const int rt_guess = std::max(ceil_div(T * k, TILE_ROWS), std::min(E, T * k));  // row tiles if the rows spread evenly
  const int split_call = std::min(MAX_KSPLIT, std::max(1, 256 / (std::max(1, rt_guess) * n_ntiles)));
  hipError_t ke = hipSuccess;
#define K_TRY(expr) do { ke = (expr); if (ke != hipSuccess) return fail(SI_EHIP, "%s failed: %s", #expr, hipGetErrorString(ke)); } while (0)

  // process chunks [c0, c0+n) (relative to `base`) of a part on the GPU.
  //   expert_sel < 0: all routed experts from their resident GG storage
  //   col_base: hidden column of chunk c0 within the expert;  part: 0 GG, 1 CG, 2 CC(CG')
  auto run_part = [&](const uint16_t* base, size_t estride, int expert_sel, int is_shared, int c0, int n, int col_base,
                      int part, int part_chunk0, int x2_only, bool first_for_rows) -> int {
    if (n <= 0) return SI_OK;
    WeightView wv{base, estride, c0, n, 0, L->q4, nullptr};
    if (L->placed && !is_shared) {
      // every expert has all its chunks in one place: one slot range and one column range serve all parts, and
      // the launch over all resident experts finds each expert's storage through the map
      part = 0;
      col_base = (part_chunk0 + 0) * CHUNK_J;
      if (expert_sel < 0) wv.e_map = L->d_emap;
    }
    const int esel = is_shared ? E : expert_sel;
    if (path == SI_DECODE) {
      wv.col0 = col_base;
      const int cps = is_shared ? (part == 0 ? scps_gg : part == 1 ? scps_cg : scps_cc) : (part == 0 ? cps_gg : part == 1 ? cps_cg : cps_cc);
      {
        SegScope sc(L, stream, SI_K_DECODE_GATEUP);
        K_TRY(launch_decode_gateup(x, M, L->plan, T, esel, x2_only, max_touched, wv, L->d_h, L->ldh_dec, stream,
                                   fuse_route ? &fr : nullptr));
        fuse_route = false;  // the tables exist from here on
      }
      SegScope sc(L, stream, SI_K_DECODE_DOWN);
      K_TRY(launch_decode_down(L->d_h, L->ldh_dec, M, L->plan, T, esel, x2_only, max_touched, wv,
                               part * DOWN_SLOTS + part_chunk0 / cps, cps, L->d_part, slot_stride, stream));
    } else {
      const int n_rt = esel >= 0 ? n_row_tiles(x2_only ? rows_x2(esel) : rows_all(esel)) : tiles_upper;
      // bf16 layers: one pass over the chunk range.  4-bit layers: the range goes through the bf16 scratch in
      // sub-pieces (dequantise, FC1, FC2 accumulating), as many chunks per expert as the scratch holds.
      const bool two_pass = L->q4 && L->d_deq;
      const int cap = !two_pass ? n : std::max(1, esel >= 0 ? L->deq_chunks : L->deq_chunks / E);
      for (int s0 = 0; s0 < n; s0 += cap) {
        const int ns = std::min(cap, n - s0);
        const bool first = first_for_rows && s0 == 0;
        WeightView wg = wv;
        if (two_pass) {
          WeightView src{base, estride, c0 + s0, ns, 0, 1, wv.e_map};
          const size_t dst_stride = esel >= 0 ? 0 : (size_t)ns * chunk_elems(M);
          {
            SegScope sc(L, stream, SI_K_FILL);
            K_TRY(launch_dequant_q4(src, M, L->plan, esel, x2_only, E, L->d_deq, dst_stride, stream));
          }
          wg = WeightView{L->d_deq, dst_stride, 0, ns, 0, 0, nullptr};
        }
        const int ldh = ns * CHUNK_J;
        {
          SegScope sc(L, stream, SI_K_PREFILL_GATEUP);
          K_TRY(launch_prefill_gateup(x, M, L->plan, esel, x2_only, n_rt, wg, L->d_hact, ldh, stream));
        }
        SegScope sc(L, stream, SI_K_PREFILL_DOWN);
        const int split = first ? split_call : std::min(split_call, std::max(1, ns / 8));
        K_TRY(launch_prefill_down(L->d_hact, ldh, M, L->plan, esel, x2_only, n_rt, wg, L->d_yp, L->yp_slab, split,
                                  first ? 0 : 1, stream));
      }
    }
    return SI_OK;
  };

  // ---- GG part (Stream-D), enqueued first so that it runs under the first copies.
  // In the prefill path the GG launch overwrites the per-row outputs and every staged piece adds to
  // them; rows without a GG part start from zero.
  {
    int rc;
    if (path == SI_PREFILL) {
      SegScope sc(L, stream, SI_K_FILL);
      for (int q = 0; q < split_call; ++q) {
        if (L->ch_gg == 0 || L->placed) K_TRY(launch_fill_zero(L->d_yp + q * L->yp_slab, (size_t)T * k * M, stream));
        if (L->has_shared && L->sch_gg == 0) K_TRY(launch_fill_zero(L->d_yp + q * L->yp_slab + (size_t)T * k * M, (size_t)T * M, stream));
      }
    }
    if (path == SI_DECODE && L->placed) {
      // rows of experts that no launch of this call writes (CC experts of X1 tokens) must read as zero in the merge
      SegScope sc(L, stream, SI_K_FILL);
      const int n_slots = ceil_div(L->H / CHUNK_J, cps_of(L->H / CHUNK_J, one, M));
      for (int q = 0; q < n_slots; ++q) K_TRY(launch_fill_zero(L->d_part + (size_t)q * slot_stride, (size_t)T * k * M, stream));
    }
    if (E == 1) rc = run_part(L->d_gg, 0, 0, 0, 0, L->ch_gg, hch * CHUNK_J, 0, 0, 0, true);
    else rc = run_part(L->d_gg, (size_t)L->ch_gg * ce, -1, 0, 0, L->ch_gg, hch * CHUNK_J, 0, 0, 0, true);
    if (rc) return rc;
    if (L->has_shared) {
      rc = run_part(L->d_sgg, 0, 0, 1, 0, L->sch_gg, (L->sch_cc + L->sch_cg) * CHUNK_J, 0, 0, 0, true);
      if (rc) return rc;
    }
    st.bytes_gg = 0;
    for (int e = 0; e < EX; ++e) {
      const bool touched = need_sync ? L->hcount[e] > 0 : true;
      if (touched) st.bytes_gg += (double)L->e_chunks(e, 0) * ce * 2;
    }
    if (!need_sync && E > 1) st.bytes_gg = -1;  // not known on the host without the counts
  }

  // ---- CG and CG' parts: copy (Stream-C) double-buffered against compute (Stream-D)
  if (any_cg || need_cgp) {
    const bool shared_first = L->pre_n > 0 && L->pre_shared;  // its first pieces are already in the ring
    for (int ei = 0; ei < EX; ++ei) {
      const int e = !shared_first ? ei : ei == 0 ? E : ei - 1;
      if (rows_all(e) <= 0) continue;
      const bool sh = e >= E;
      const int n_cc_e = L->e_chunks(e, 2), n_cg_e = L->e_chunks(e, 1);
      if (n_cc_e + n_cg_e == 0) continue;
      const uint16_t* hbase = L->host_base(e);
      for (int part = 1; part <= 2; ++part) {  // CG on all rows, then CG' (the CC range) on the X2 rows
        const int x2_only = part == 2;
        if (part == 2 && (!need_cgp || rows_x2(e) <= 0)) continue;
        const int pc0 = part == 2 ? 0 : n_cc_e, pn = part == 2 ? n_cc_e : n_cg_e;
        const int cps = sh ? (part == 2 ? scps_cc : scps_cg) : (part == 2 ? cps_cc : cps_cg);
        const int piece_max = piece_chunks(L, path, cps);
        for (int c = 0; c < pn; c += piece_max) {
          const int n = std::min(piece_max, pn - c);
          int slot;
          if (part == 1 && sh == L->pre_shared && c / piece_max < L->pre_n) {
            slot = L->pre_slot[c / piece_max];  // already on its way (prefetched after the previous layer's copies)
          } else {
            slot = (int)(L->piece_counter++ % L->n_stage);
            if (L->slot_used[slot]) HIP_TRY(hipStreamWaitEvent(L->copy_stream, L->ev_free[slot], 0));
            {
              SegScope sc(L, L->copy_stream, SEG_COPY);
              HIP_TRY(hipMemcpyAsync(L->d_stage[slot], hbase + (size_t)(pc0 + c) * ce, (size_t)n * ce * 2, hipMemcpyHostToDevice, L->copy_stream));
            }
            HIP_TRY(hipEventRecord(L->ev_ready[slot], L->copy_stream));
          }
          HIP_TRY(hipStreamWaitEvent(stream, L->ev_ready[slot], 0));
          {
            L->in_staged = 1;
            int rc = run_part(L->d_stage[slot], 0, sh ? 0 : e, sh, 0, n, (pc0 + c) * CHUNK_J, part, c, x2_only, false);
            L->in_staged = 0;
            if (rc) return rc;
          }
          HIP_TRY(hipEventRecord(L->ev_free[slot], stream));
          L->slot_used[slot] = 1;
          st.bytes_streamed += (double)n * ce * 2;
          st.n_copies++;
        }
      }
    }
  }

  L->pre_n = 0;
  // ---- cross-layer prefetch: this call's copies are all enqueued; before blocking on the CC workers put the
  //      next layer's first CG pieces on the link so that it never idles between layers
  if (L->chain_next) {
    int rc = prefetch_cg(L->chain_next, path);
    if (rc) return rc;
  }

  // ---- CC result: wait for Stream-A, send Y^CC to the GPU
  const float* ycc_dev = nullptr;
  if (need_cc) {
    if (L->ch_cc > 0 || (L->has_shared && L->sch_cc > 0)) {
      cc_pool_wait(L->pool);
      L->cc_inflight = false;
      st.cc_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - cc0).count();
      double b = 0;
      for (int e = 0; e < EX; ++e) if (L->hcount[EX + e] > 0) b += (double)L->e_chunks(e, 2) * ce * 2;
      st.bytes_cc = b;
    }
    HIP_TRY(hipMemcpyAsync(L->d_ycc, L->hycc, (size_t)n_x1 * M * 4, hipMemcpyHostToDevice, stream));
    ycc_dev = L->d_ycc;
  }

  // ---- merge: Y = Y^CC (or Y^CG') + Y^CG + Y^GG (Eq. 2) and the weighted sum over experts
  {
    SegScope sc(L, stream, path == SI_DECODE ? SI_K_DECODE_COMBINE : SI_K_PREFILL_COMBINE);
    if (path == SI_DECODE) {
      DecodeCombineArgs a{};
      a.part = L->d_part; a.slot_stride = slot_stride;
      a.n_slots_gg = ceil_div(L->ch_gg, cps_gg); a.n_slots_cg = ceil_div(L->ch_cg, cps_cg); a.n_slots_cc = need_cgp ? ceil_div(L->ch_cc, cps_cc) : 0;
      if (L->placed) {  // all parts of the routed experts share the first slot range
        a.n_slots_gg = ceil_div(L->H / CHUNK_J, cps_of(L->H / CHUNK_J, one, M));
        a.n_slots_cg = a.n_slots_cc = 0;
      }
      a.s_slots_gg = ceil_div(L->sch_gg, scps_gg); a.s_slots_cg = ceil_div(L->sch_cg, scps_cg); a.s_slots_cc = need_cgp ? ceil_div(L->sch_cc, scps_cc) : 0;
      a.ycc = ycc_dev; a.T = T; a.k = k; a.M = M; a.n_x1 = n_x1; a.has_shared = L->has_shared;
      K_TRY(launch_decode_combine(a, L->plan, y_dev, stream));
    } else {
      K_TRY(launch_prefill_combine(L->d_yp, L->yp_slab, split_call, ycc_dev, T, k, M, n_x1, L->has_shared, L->plan, y_dev, stream));
    }
  }
  if (L->profiling) HIP_TRY(hipEventRecord(L->ev_t1, stream));
  st.enqueue_ms = std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - wall0).count();
  st.total_ms = st.enqueue_ms;  // replaced by event time in si_layer_stats when profiling is on
  L->last = st;
  guard.ok = true;
  return SI_OK;
}

int si_layer_stats(si_layer_t* L, si_stats_t* out) {
  if (!L || !out) return fail(SI_EINVAL, "layer or out is NULL");
  si_stats_t st = L->last;
  if (L->profiling && L->ev_used > 0) {
    HIP_TRY(hipSetDevice(L->device));
    HIP_TRY(hipEventSynchronize(L->ev_t1));
    HIP_TRY(hipStreamSynchronize(L->copy_stream));
    float ms = 0.f;
    HIP_TRY(hipEventElapsedTime(&ms, L->ev_t0, L->ev_t1));
    st.total_ms = ms;
    st.copy_ms = st.gpu_ms = st.route_ms = st.staged_ms = 0.f;
    for (int i = 0; i < SI_K_COUNT; ++i) { st.kernel_ms[i] = 0.f; st.kernel_launches[i] = 0; }
    for (const Seg& s : L->segs) {
      float d = 0.f;
      HIP_TRY(hipEventElapsedTime(&d, s.a, s.b));
      if (s.kind == SEG_COPY) { st.copy_ms += d; continue; }
      st.gpu_ms += d;
      st.kernel_ms[s.kind] += d;
      st.kernel_launches[s.kind] += 1;
      if (s.staged) st.staged_ms += d;
      if (s.kind == SI_K_ROUTE) st.route_ms += d;
    }
    float mx = std::max(st.copy_ms, std::max(st.gpu_ms, st.cc_ms));
    st.overlap = st.total_ms > 0.f ? mx / st.total_ms : 0.f;
    // share of the resident-part (GG) kernel time that ran while a weight copy was in flight
    std::vector<std::pair<float, float>> copies;
    auto offset = [&](hipEvent_t e, float* o) { return hipEventElapsedTime(o, L->ev_t0, e); };
    for (const Seg& s : L->segs)
      if (s.kind == SEG_COPY) {
        float a = 0.f, b = 0.f;
        if (offset(s.a, &a) == hipSuccess && offset(s.b, &b) == hipSuccess) copies.push_back({a, b});
        else (void)hipGetLastError();  // a prefetched copy may have been recorded before this call's first event
      }
    float gg_ms = 0.f, gg_cov = 0.f;
    for (const Seg& s : L->segs) {
      const bool weight_kernel = s.kind == SI_K_DECODE_GATEUP || s.kind == SI_K_DECODE_DOWN || s.kind == SI_K_PREFILL_GATEUP || s.kind == SI_K_PREFILL_DOWN;
      if (!weight_kernel || s.staged) continue;
      float a = 0.f, b = 0.f;
      HIP_TRY(offset(s.a, &a));
      HIP_TRY(offset(s.b, &b));
      gg_ms += b - a;
      for (const auto& c : copies) gg_cov += std::max(0.f, std::min(b, c.second) - std::max(a, c.first));  // copies do not overlap each other
    }
    st.gg_in_copy = gg_ms > 0.f && !copies.empty() ? std::min(1.f, gg_cov / gg_ms) : 0.f;
  }
  *out = st;
  return SI_OK;
}

// ------------------------------------------------------------------------------------------------
// A stack of layers run back to back (the MLP / MoE blocks of consecutive Transformer layers with the
// residual connection around each; attention is outside this library): x_{l+1} = bf16(x_l + y_l).
// ------------------------------------------------------------------------------------------------
}  // extern "C"

struct si_stack {
  std::vector<si_layer*> layers;
  int M = 0, max_T = 0, device = 0;
  uint16_t* d_x[2] = {nullptr, nullptr};  // hidden state between layers, bf16 [max_T][M]
  float* d_y = nullptr;                   // layer output, f32 [max_T][M]
  // One Stream-C for the whole stack: copies run in the order they are enqueued, so the pieces prefetched for
  // layer l+1 queue up behind layer l's own instead of sharing the link with them (which would hold back
  // layer l, and with it the start of layer l+1's CPU part).
  hipStream_t copy_stream = nullptr;
};

namespace {

// out_bf16 (if not null) = bf16(x + y), out_f32 (if not null) = x + y; 8 elements per thread
__global__ __launch_bounds__(256) void k_residual(const uint16_t* __restrict__ x, const float* __restrict__ y, size_t n8,
                                                   uint16_t* __restrict__ out_bf16, float* __restrict__ out_f32) {
  const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n8) return;
  const uint4 xv = reinterpret_cast<const uint4*>(x)[i];
  const float4 y0 = reinterpret_cast<const float4*>(y)[2 * i], y1 = reinterpret_cast<const float4*>(y)[2 * i + 1];
  const uint32_t xw[4] = {xv.x, xv.y, xv.z, xv.w};
  const float yv[8] = {y0.x, y0.y, y0.z, y0.w, y1.x, y1.y, y1.z, y1.w};
  float r[8];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    r[2 * q] = __uint_as_float(xw[q] << 16) + yv[2 * q];
    r[2 * q + 1] = __uint_as_float(xw[q] & 0xffff0000u) + yv[2 * q + 1];
  }
  if (out_f32) {
    reinterpret_cast<float4*>(out_f32)[2 * i] = make_float4(r[0], r[1], r[2], r[3]);
    reinterpret_cast<float4*>(out_f32)[2 * i + 1] = make_float4(r[4], r[5], r[6], r[7]);
  }
  if (out_bf16) {
    uint32_t o[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      uint32_t a = __float_as_uint(r[2 * q]), b = __float_as_uint(r[2 * q + 1]);
      a += 0x7fffu + ((a >> 16) & 1u);  // round to nearest even
      b += 0x7fffu + ((b >> 16) & 1u);
      o[q] = (a >> 16) | (b & 0xffff0000u);
    }
    reinterpret_cast<uint4*>(out_bf16)[i] = make_uint4(o[0], o[1], o[2], o[3]);
  }
}

}  // namespace

extern "C" {

int si_stack_create(si_layer_t* const* layers, int32_t n_layers, si_stack_t** out) {
  if (!layers || !out || n_layers < 1) return fail(SI_EINVAL, "si_stack_create: need layers, out and n_layers >= 1");
  for (int i = 0; i < n_layers; ++i) {
    if (!layers[i]) return fail(SI_EINVAL, "si_stack_create: layer %d is NULL", i);
    if (layers[i]->M != layers[0]->M || layers[i]->device != layers[0]->device)
      return fail(SI_EINVAL, "si_stack_create: layer %d differs from layer 0 in d_model or device", i);
    for (int j = 0; j < i; ++j)
      if (layers[j] == layers[i]) return fail(SI_EINVAL, "si_stack_create: layer %d appears twice", i);
  }
  si_stack* S = new (std::nothrow) si_stack();
  if (!S) return fail(SI_ENOMEM, "si_stack_create: out of host memory");
  S->layers.assign(layers, layers + n_layers);
  S->M = layers[0]->M;
  S->device = layers[0]->device;
  S->max_T = layers[0]->max_T;
  for (int i = 1; i < n_layers; ++i) S->max_T = std::min(S->max_T, layers[i]->max_T);
  hipError_t e = hipSetDevice(S->device);
  int rc = e == hipSuccess ? SI_OK : fail(SI_EHIP, "hipSetDevice failed: %s", hipGetErrorString(e));
  const size_t n = (size_t)S->max_T * S->M;
  if (rc == SI_OK) rc = dev_alloc(&S->d_x[0], n);
  if (rc == SI_OK) rc = dev_alloc(&S->d_x[1], n);
  if (rc == SI_OK) rc = dev_alloc(&S->d_y, n);
  if (rc == SI_OK && (e = hipStreamCreateWithFlags(&S->copy_stream, hipStreamNonBlocking)) != hipSuccess)
    rc = fail(SI_EHIP, "hipStreamCreateWithFlags failed: %s", hipGetErrorString(e));
  if (rc != SI_OK) { S->layers.clear(); si_stack_destroy(S); return rc; }
  for (si_layer* L : S->layers) {
    (void)hipStreamSynchronize(L->copy_stream);
    L->copy_stream = S->copy_stream;
  }
  *out = S;
  return SI_OK;
}

void si_stack_destroy(si_stack_t* S) {
  if (!S) return;
  (void)hipSetDevice(S->device);
  if (S->copy_stream) (void)hipStreamSynchronize(S->copy_stream);
  for (si_layer* L : S->layers) { L->copy_stream = L->own_copy_stream; L->pre_n = 0; }
  if (S->copy_stream) (void)hipStreamDestroy(S->copy_stream);
  for (auto* p : S->d_x) if (p) (void)hipFree(p);
  if (S->d_y) (void)hipFree(S->d_y);
  delete S;
}

int si_stack_forward(si_stack_t* S, const void* x_dev, const float* const* logits_dev, int32_t T, int32_t n_g, int32_t mode,
                     float* h_out_dev, int32_t prefetch, void* stream_v) {
  if (!S) return fail(SI_EINVAL, "stack is NULL");
  if (T < 0 || T > S->max_T) return fail(SI_ESTATE, "T=%d outside [0, %d]", T, S->max_T);
  if (T == 0) return SI_OK;
  if (!x_dev || !h_out_dev) return fail(SI_EINVAL, "x_dev or h_out_dev is NULL");
  HIP_TRY(hipSetDevice(S->device));
  hipStream_t stream = (hipStream_t)stream_v;
  const int nl = (int)S->layers.size();
  const size_t n8 = (size_t)T * S->M / 8;
  const uint16_t* x = static_cast<const uint16_t*>(x_dev);
  for (int l = 0; l < nl; ++l) {
    si_layer* L = S->layers[l];
    const float* lg = logits_dev ? logits_dev[l] : nullptr;
    // bit 0: layer l+1 after layer l; bit 1: layer 0 (for the next call) after the last layer
    L->chain_next = ((prefetch & 1) && l + 1 < nl) ? S->layers[l + 1] : ((prefetch & 2) && l + 1 == nl) ? S->layers[0] : nullptr;
    const int rc = si_layer_forward(L, x, lg, T, n_g, mode, S->d_y, nullptr, stream_v);
    L->chain_next = nullptr;
    if (rc != SI_OK) return rc;
    const bool last = l + 1 == nl;
    uint16_t* xn = last ? nullptr : S->d_x[l & 1];
    hipLaunchKernelGGL(k_residual, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream, x, S->d_y, n8, xn,
                       last ? h_out_dev : nullptr);
    HIP_TRY(hipGetLastError());
    x = xn;
  }
  return SI_OK;
}

}  // extern "C"
