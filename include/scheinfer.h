/*
 * scheinfer.h - C ABI of the partitioned feed-forward layer for one MI355X (gfx950).
 *
 * The layer is a dense SwiGLU MLP or the routed experts of a sparse MoE block whose weights are
 * sliced along the hidden dimension into three parts (Section III-B, "Memory Manager"):
 *   GG  stored in GPU memory, run on the GPU
 *   CG  stored in pinned host memory, copied to the GPU for every call, run on the GPU
 *   CC  stored in host memory, run on host threads; its result is sent to the GPU and added
 * and whose output is the sum of the three partial products (Eq. 1-2), identical to the unsliced
 * layer.  In the prompt phase the last n_g tokens (X2) run their CC share on the GPU from the same
 * host addresses (CG', Section IV-B); in the generation phase n_g = 0.
 *
 * Conventions
 *  - Every function returns SI_OK (0) or a negative SI_E* code; the text of the last error of the
 *    calling thread is available from si_last_error().  Nothing throws, aborts or prints.
 *  - "host" / "device" on a pointer says where the memory lives.  Device pointers are plain HIP
 *    device addresses (e.g. torch.Tensor.data_ptr()); `stream` is a hipStream_t passed as void*.
 *  - bf16 values travel as their 16-bit patterns (uint16_t).
 *  - The library owns what it allocates (GG buffers, pinned CG/CC buffers, staging ring,
 *    workspaces, worker threads) and frees it in si_layer_destroy().  The caller owns x, logits, y
 *    and the stream.
 *  - A layer handle is not thread-safe: one forward at a time per layer.
 */
#ifndef SCHEINFER_H
#define SCHEINFER_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define SI_OK 0
#define SI_EINVAL (-1) /* bad shape, rate, pointer or argument combination */
#define SI_ENOMEM (-2) /* a device or pinned-host allocation failed */
#define SI_EHIP (-3)   /* a HIP runtime call failed (text in si_last_error) */
#define SI_ESTATE (-4) /* call not valid for this layer, e.g. T > max_tokens */

#define SI_AUTO 0    /* decode path when T <= SI_DECODE_AUTO_T and an expert receives on average at most
                        SI_DECODE_AUTO_ROWS rows (ceil(T*top_k/n_experts)), else prefill path: the GEMV kernels pass
                        over an expert's weights once per 4 of its rows, the GEMM kernels once per 64..256 */
#define SI_DECODE 1  /* expert GEMV path (bandwidth bound), T <= SI_DECODE_MAX_T */
#define SI_PREFILL 2 /* grouped MFMA GEMM path */
#define SI_DECODE_AUTO_T 8
#define SI_DECODE_AUTO_ROWS 4
#define SI_DECODE_MAX_T 16

typedef struct si_layer si_layer_t; /* opaque */

/*
 * Shape and placement of one layer.  Symbols as in Section IV-A.2: M = d_model, H = d_ff.
 * Rates r_gg, r_cg, r_cc are the slicing rates of Section IV-A (each in [0,1], sum 1 within 1e-4).
 * They are turned into hidden-column counts by cumulative rounding to `granule` columns:
 *   n_GG = g*floor(r_GG*H/g + 1/2),  n_GG + n_CG = g*floor((r_GG+r_CG)*H/g + 1/2),  n_CC = rest,
 * computed in double from the float rates.  Columns are ordered [CC | CG | GG] as in Section III-B.
 * Every routed expert is sliced with the same rates along its own d_ff; the shared expert (if any)
 * likewise along d_ff_shared.
 */
typedef struct {
  int32_t d_model;     /* M, multiple of 64 */
  int32_t d_ff;        /* H per routed expert, multiple of granule */
  int32_t n_experts;   /* E; a dense MLP is E = 1, top_k = 1, logits = NULL */
  int32_t top_k;       /* 1 <= top_k <= E */
  int32_t d_ff_shared; /* 0 = no shared expert; else multiple of granule */
  float r_gg, r_cg, r_cc;
  int32_t granule;     /* hidden columns per slicing unit; 0 -> 64; must be a multiple of 64 */
  int32_t max_tokens;  /* largest T a forward call may pass; sizes the workspaces.  max_tokens * d_model and
                          max_tokens * (top_k + 1 if shared) * max(d_ff, d_ff_shared) must stay below 2^31
                          (the prompt-phase GEMMs address operand rows with 32-bit element offsets) */
  int32_t cc_threads;  /* host threads for the CC part; 0 -> min(16, hardware threads) */
  int32_t device;      /* HIP device ordinal */
  int32_t stage_mib;   /* size of one staging buffer for CG copies in MiB; 0 -> 256 */
  int32_t n_stage;     /* number of staging buffers (>= 2); 0 -> 2 (double buffering) */
  int32_t deq_mib;     /* 4-bit layers only.  0: the prompt-phase GEMMs read the 4-bit chunks and convert them on
                          their way into LDS (no scratch).  > 0: two passes instead, a dequantisation kernel writing
                          bf16 copies into a device scratch of this many MiB (never more than the largest part
                          needs) that the bf16 GEMMs then read, piece by piece */
} si_layer_desc_t;

/* Optional device outputs of the token-assignment step; any pointer may be NULL.
 *   idx[T*k] i32   experts of each token, slots ordered by (logit descending, index ascending)
 *   w[T*k]  f32    softmax over the k selected logits
 *   count[E] i32   pairs per expert;  off[E+1] i32 exclusive prefix sum
 *   perm[T*k] i32  pair id t*k+s at each expert-sorted position (ascending (t,s) inside an expert)
 *   inv[T*k] i32   inverse of perm                                                              */
typedef struct {
  int32_t* idx;
  float* w;
  int32_t* count;
  int32_t* off;
  int32_t* perm;
  int32_t* inv;
} si_routing_out_t;

/* Timings of the most recent forward call of a layer (milliseconds, from HIP events and the host
 * clock) and the bytes it moved.  overlap = max(copy_ms, gpu_ms, cc_ms) / total_ms: 1.0 means the
 * layer took as long as its slowest resource, the objective t_fin = max(tau_G, tau_C) of Section
 * IV-A.2. */
#define SI_K_ROUTE 0           /* token-assignment kernels */
#define SI_K_DECODE_GATEUP 1   /* GEMV FC1 + SwiGLU */
#define SI_K_DECODE_DOWN 2     /* GEMV FC2 */
#define SI_K_DECODE_COMBINE 3
#define SI_K_PREFILL_GATEUP 4  /* MFMA FC1 + SwiGLU */
#define SI_K_PREFILL_DOWN 5    /* MFMA FC2 */
#define SI_K_PREFILL_COMBINE 6
#define SI_K_FILL 7
#define SI_K_COUNT 8

typedef struct {
  float total_ms;     /* first enqueue to last kernel, on the caller's stream */
  float copy_ms;      /* busy time of the host->device weight copies (Stream-C) */
  float gpu_ms;       /* sum of kernel time on the compute stream (Stream-D), incl. waits on copies excluded */
  float cc_ms;        /* host wall time of the CC workers (Stream-A) */
  float route_ms;     /* token-assignment kernels */
  double bytes_streamed;  /* CG (+CG') weight bytes copied host->device */
  double bytes_gg;        /* GG weight bytes read by the kernels (algorithmic) */
  double bytes_cc;        /* CC weight bytes read by the host workers (algorithmic) */
  float overlap;
  int32_t n_copies;   /* number of staged pieces */
  int32_t n_touched;  /* experts with at least one token (-1 if not known on the host) */
  int32_t path;       /* SI_DECODE or SI_PREFILL actually taken */
  float kernel_ms[SI_K_COUNT];         /* summed HIP-event time of each kernel class (SI_K_*) */
  int32_t kernel_launches[SI_K_COUNT]; /* launches of each class */
  float staged_ms;    /* part of gpu_ms spent in kernels that read a staged (CG / CG') piece */
  float handoff_ms;   /* host wait for the token assignment to reach the host (0 if not needed) */
  float enqueue_ms;   /* host wall time spent inside the forward call (Stream-B) */
  float gg_in_copy;   /* share of the resident-part (GG) kernel time that ran while a weight copy was in flight
                         (1.0 = the GG compute is completely hidden under the copies; 0 when nothing is copied) */
} si_stats_t;

/*
 * Create a layer: slice the weights by the rates in `desc` and place the parts (Section III-B).
 * w_gate, w_up, w_down: HOST, bf16, each [n_experts][d_ff][d_model] (index j of d_ff, m of
 * d_model); gate and up are the two halves of FC1 (sliced by columns j), down is FC2 (sliced by
 * rows j).  shared_*: HOST, bf16 [d_ff_shared][d_model], or NULL when d_ff_shared == 0.
 * The caller keeps ownership; the library repacks during the call and never reads them again.
 * Errors: SI_EINVAL (null pointer, bad shape/rate/granule, max_tokens beyond the limit above), SI_ENOMEM, SI_EHIP.
 */
int si_layer_create(const si_layer_desc_t* desc, const uint16_t* w_gate, const uint16_t* w_up,
                    const uint16_t* w_down, const uint16_t* shared_gate, const uint16_t* shared_up,
                    const uint16_t* shared_down, si_layer_t** out);

/*
 * Whole-expert placement: instead of slicing every routed expert by the three rates, each expert lives entirely
 * in one place, placement[e] = 0 (GG: resident in GPU memory), 1 (CG: pinned host memory, streamed when the
 * expert receives tokens) or 2 (CC: computed by the host workers; on the GPU through CG' for the X2 tokens).
 * The output is the same as for any slicing (Section III-B: the partition changes where a product is formed, not
 * its value); what changes is which bytes cross the host link for a given routing, e.g. keeping the most
 * frequently chosen experts resident.  placement: HOST [n_experts].  The rates of `desc` still slice the shared
 * expert, if any.  Otherwise as si_layer_create.
 */
int si_layer_create_placed(const si_layer_desc_t* desc, const uint16_t* w_gate, const uint16_t* w_up,
                           const uint16_t* w_down, const uint16_t* shared_gate, const uint16_t* shared_up,
                           const uint16_t* shared_down, const uint8_t* placement, si_layer_t** out);

/*
 * A placement from expert frequencies (a heuristic of this library, not of the paper): the n_gg experts with the
 * largest freq[e] become GG; the others are taken in descending frequency and given to CG while CG's share of
 * the frequency mass handed out so far stays at or below cg_share, else to CC (cg_share = the r_CG / (r_CG +
 * r_CC) that the slicing-rate solver balances link and host with).  Ties: lower expert index first.
 * freq HOST [n_experts] >= 0; placement HOST [n_experts], written.
 */
int si_place_experts(const double* freq, int32_t n_experts, int32_t n_gg, double cg_share, uint8_t* placement);

/*
 * The same layer from 4-bit weights (the paper evaluates INT4 models, Section V-A, without naming a format;
 * this one is the library's own): a weight is a code c in 0..15 standing for (c - 8) * scale.
 *   q_gate, q_up, q_down  HOST uint8 [n_experts][d_ff][d_model/2]: element m of row j is the low nibble of byte
 *                         m/2 for even m, the high nibble for odd m
 *   z_gate, z_up          HOST bf16 [n_experts][d_ff][d_model/64]: one scale per 64 consecutive m of a row (the
 *                         contraction index of FC1)
 *   z_down                HOST bf16 [n_experts][d_ff/64][d_model]: one scale per 64 consecutive j of a column (the
 *                         contraction index of FC2)
 * `shared`: the shared expert's arrays without the leading [n_experts], or NULL when d_ff_shared == 0.
 * `placement`: NULL (slice by the rates) or HOST [n_experts] as for si_layer_create_placed.
 * Everything else (slicing, placement, forward, stats) is as for si_layer_create; the parts keep the 4-bit
 * form in HBM, in pinned memory and on the host link (102*d_model bytes per 64 hidden columns instead of
 * 384*d_model).  Generation-phase kernels and the host workers multiply codes and scales in fp32 (exact); the
 * prompt-phase GEMMs read the same chunks and feed the matrix cores (c - 8) * scale rounded to bf16, converted
 * on the way into LDS (or, with desc->deq_mib > 0, by a separate pass into a bf16 scratch).
 */
typedef struct {
  const uint8_t* q_gate;
  const uint8_t* q_up;
  const uint8_t* q_down;
  const uint16_t* z_gate;
  const uint16_t* z_up;
  const uint16_t* z_down;
} si_q4_weights_t;
int si_layer_create_q4(const si_layer_desc_t* desc, const si_q4_weights_t* routed, const si_q4_weights_t* shared,
                       const uint8_t* placement, si_layer_t** out);

/*
 * Change the slicing rates of an existing layer (e.g. to the r_CG* that si_solve_split returned for measurements
 * taken on this very layer).  The library holds every chunk exactly once, either resident or in pinned memory, in
 * a form that does not depend on the rates; re-slicing moves the chunks whose place changes across the host link
 * and reallocates the two buffers (both old and new exist during the call).  Synchronises the device; not meant
 * for the hot path (Section III-B: the paper slices once and keeps the rates of the generation phase).
 * Errors: SI_EINVAL (rates), SI_ESTATE (layer created with whole-expert placement), SI_ENOMEM, SI_EHIP; on
 * SI_ENOMEM / SI_EHIP the layer keeps working with the rates si_layer_split_info reports.
 */
int si_layer_resplit(si_layer_t* layer, float r_gg, float r_cg, float r_cc);

/* Hidden-column counts actually used (routed expert n_*, shared expert s_*; any pointer may be
 * NULL).  Tests read the counts from here instead of re-deriving the rounding. */
int si_layer_split_info(const si_layer_t* layer, int32_t* n_gg, int32_t* n_cg, int32_t* n_cc,
                        int32_t* s_gg, int32_t* s_cg, int32_t* s_cc);

/* The same rounding as a pure function (no GPU needed): rates -> column counts. */
int si_split_counts(int32_t d_ff, int32_t granule, float r_gg, float r_cg, int32_t* n_gg,
                    int32_t* n_cg, int32_t* n_cc);

/*
 * One layer forward (the Task Scheduler of Section III-C for one MLP / MoE block).
 *  x_dev      DEVICE bf16 [T][d_model]
 *  logits_dev DEVICE f32 [T][n_experts] router logits; NULL for a dense layer (n_experts == 1)
 *  T          0 <= T <= max_tokens (T == 0 is a no-op)
 *  n_g        number of trailing tokens (X2 = last n_g rows) whose CC share runs on the GPU via CG'
 *             (Section IV-B); 0 in the generation phase; n_g == T means the host computes nothing
 *  mode       SI_AUTO | SI_DECODE | SI_PREFILL
 *  y_dev      DEVICE f32 [T][d_model], overwritten with the layer output
 *  routing_out optional device outputs of the token assignment (NULL, or any member NULL)
 *  stream     hipStream_t (as void*) the call is ordered on
 * Ordering: all GPU work is enqueued on `stream` or joined into it by events; y_dev is valid once
 * `stream` reaches the point after the call.  The call returns without a full device
 * synchronisation, but the host thread blocks (a) until the token assignment has reached the host
 * when the layer has a CG part with more than one expert or a CC part, and (b) until the CC
 * workers have finished.
 * Errors: SI_EINVAL (null pointers, n_g > T, bad mode), SI_ESTATE (T > max_tokens, or SI_DECODE
 * with T > SI_DECODE_MAX_T), SI_EHIP.
 */
int si_layer_forward(si_layer_t* layer, const void* x_dev, const float* logits_dev, int32_t T,
                     int32_t n_g, int32_t mode, float* y_dev, const si_routing_out_t* routing_out,
                     void* stream);

/*
 * Token assignment alone (Section II-A: the gating function assigns tokens to experts): top-k on
 * the raw logits (ties -> lower expert index), softmax over the k selected logits, per-expert
 * histogram, exclusive prefix sum and the stable expert-sorted permutation.
 * logits_dev DEVICE f32 [T][E]; out: device pointers (any may be NULL); 1 <= k <= E <= 256.
 */
int si_route(const float* logits_dev, int32_t T, int32_t E, int32_t k, const si_routing_out_t* out,
             void* stream);

/*
 * si_route for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results.  Where si_route takes a stream-ordered
 * temporary for the idx / w tables that the caller does not ask for, this call uses a fixed array that lives in
 * the library's device image (2 * 4 * SI_ROUTE_NOALLOC_MAX_PAIRS bytes = 1 MiB on every GPU the library runs on,
 * held until the process ends) and calls no allocating routine.
 * Limits: T * k <= SI_ROUTE_NOALLOC_MAX_PAIRS, else SI_EINVAL.  Runs on the current HIP device.
 * All calls on one GPU share that GPU's array: two calls that overlap on one GPU (different streams, or threads)
 * race unless both pass idx and w themselves; calls ordered on one stream are safe.  The array keeps the previous
 * call's contents; every entry a call reads was written by that call first.
 */
#define SI_ROUTE_NOALLOC_MAX_PAIRS 131072
int si_route_noalloc(const float* logits_dev, int32_t T, int32_t E, int32_t k, const si_routing_out_t* out,
                     void* stream);

/* Timings and byte counts of the last forward call; synchronises the layer's events. */
int si_layer_stats(si_layer_t* layer, si_stats_t* out);

/* Turn per-call event timing on (1) or off (0, default).  Off removes all event records that
 * exist only for si_layer_stats. */
int si_layer_set_profiling(si_layer_t* layer, int32_t on);

/*
 * Host-only pieces of the layer, usable without a GPU (the CPU test-suite drives them directly).
 *
 * si_repack_chunks: the storage transform of the Memory Manager for one expert.  Source HOST bf16
 * w_gate/w_up/w_down [d_ff][d_model]; writes chunks [chunk0, chunk0+n_chunks) (64 hidden columns
 * each) to `out` (HOST, n_chunks * 3*64*d_model elements).  One chunk is [ gate | up | down ] with
 *   gate / up block [M/PW][64 j][PW m]   (PW = largest power of two <= 512 dividing d_model)
 *   down block      [M/NW][8 q][NW m][8 i] = Wd[j0 + 8q + i][m]   (NW likewise, <= 256)
 * i.e. FC1 rows cut into panels along the contraction index m, and the contraction index j of FC2
 * made contiguous in groups of 8 inside tiles of NW output columns.
 *
 * si_cc_compute: what the CC workers do (Stream-A, Section III-C): for tokens t < T1
 *   ycc[t] = sum_s w[t][s] * MLP^CC_{idx[t][s]}(x[t])  (+ the shared expert's CC columns),
 * over the first n_cc_chunks chunks of every expert's host storage.  All pointers HOST.
 *   x [T1][M] bf16; idx, w [T1][k]; routed: chunk-major, expert e at routed + e*expert_stride
 *   (elements); shared: chunk-major or NULL; ycc [T1][M] f32, overwritten.  threads >= 1.
 */
int si_repack_chunks(const uint16_t* w_gate, const uint16_t* w_up, const uint16_t* w_down, int32_t d_ff,
                     int32_t d_model, int32_t chunk0, int32_t n_chunks, uint16_t* out);
int si_cc_compute(const uint16_t* x, const int32_t* idx, const float* w, int32_t T1, int32_t k, int32_t d_model,
                  int32_t n_experts, const uint16_t* routed, uint64_t expert_stride, int32_t n_cc_chunks,
                  const uint16_t* shared, int32_t s_cc_chunks, int32_t threads, float* ycc);

/* The host-only pieces for the 4-bit storage form: one expert's arrays (w: [d_ff][d_model/2] codes,
 * [d_ff][d_model/64] and [d_ff/64][d_model] scales) -> n_chunks * 51*d_model uint16 units of library storage
 * (per chunk: gate, up, down codes, then gate, up, down scales), and the CC workers on such storage
 * (expert_stride in uint16 units).  d_model must be a multiple of 64. */
int si_repack_chunks_q4(const si_q4_weights_t* w, int32_t d_ff, int32_t d_model, int32_t chunk0, int32_t n_chunks,
                        uint16_t* out);
int si_cc_compute_q4(const uint16_t* x, const int32_t* idx, const float* w, int32_t T1, int32_t k, int32_t d_model,
                     int32_t n_experts, const uint16_t* routed, uint64_t expert_stride, int32_t n_cc_chunks,
                     const uint16_t* shared, int32_t s_cc_chunks, int32_t threads, float* ycc);

/* Free everything the layer owns.  NULL is allowed. */
void si_layer_destroy(si_layer_t* layer);

/*
 * A stack of layers run back to back: the MLP / MoE blocks of consecutive Transformer layers with the
 * residual connection around each (attention lies outside this library),
 *   x_0 = x,   x_{l+1} = bf16(x_l + Layer_l(x_l)),   h_out = x_{n-1} + Layer_{n-1}(x_{n-1})   (fp32, not rounded).
 * Each layer keeps its own slicing rates, e.g. the r_GG that si_assign_gpu_memory gave it (Section IV-A.4).
 * prefetch bit 0: the first CG pieces of layer l+1 are put on the host link as soon as the copies of layer l are
 * enqueued, before the host waits for layer l's CC workers, so that the link does not idle between layers.  What
 * travels ahead is what does not depend on layer l+1's own token assignment: the one expert of a dense layer, or
 * the shared expert of an MoE layer (which that layer's call then takes first); routed experts never do.
 * prefetch bit 1: likewise layer 0's pieces after the last layer, for the next call on this stack (token by
 * token generation); they are used if that call takes the same path (decode / prefill) and copied again if not.
 *
 * si_stack_create: `layers` HOST array of n_layers >= 1 distinct layer handles with equal d_model on one
 *   device.  The stack borrows the layers (the caller destroys them after the stack; a layer belongs to at
 *   most one stack at a time) and owns two bf16 hidden-state buffers, one fp32 output buffer of max_tokens x
 *   d_model (the smallest max_tokens) and one copy stream that all its layers use while the stack exists, so
 *   that weight copies cross the host link in the order they were enqueued.
 * si_stack_forward: x_dev DEVICE bf16 [T][d_model]; logits_dev HOST array of n_layers DEVICE pointers
 *   (f32 [T][n_experts] of each layer; entries of dense layers and the array itself may be NULL when every
 *   layer is dense); n_g, mode, stream as in si_layer_forward, applied to every layer; h_out_dev DEVICE
 *   f32 [T][d_model].  Errors as si_layer_forward.
 */
typedef struct si_stack si_stack_t;
int si_stack_create(si_layer_t* const* layers, int32_t n_layers, si_stack_t** out);
int si_stack_forward(si_stack_t* stack, const void* x_dev, const float* const* logits_dev, int32_t T, int32_t n_g,
                     int32_t mode, float* h_out_dev, int32_t prefetch, void* stream);
void si_stack_destroy(si_stack_t* stack);

/* Text of the last error raised on the calling thread ("" if none). */
const char* si_last_error(void);

/* Library version string. */
const char* si_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SCHEINFER_H */
