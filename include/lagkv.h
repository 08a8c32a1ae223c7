/*
 * lagkv.h - C ABI of the LagKV KV-cache compression pass for AMD MI355X (gfx950).
 *
 * The pass is the one defined in "LagKV: Lag-Relative Information of the KV
 * Cache Tells Which Tokens Are Important" (arXiv 2504.04704), Methodology,
 * subsection "LagKV": the cache of every KV head is split into S attention
 * sink rows, chunks of L rows ("lag size") and a trailing sliding window; a
 * chunk is scored against the NEXT chunk (Eq. 7-11), the k = floor(r*L) best
 * rows of each chunk are kept and everything is compacted into a dense cache
 * whose length is given by Eq. 12.
 *
 * General conventions
 *   - Every K/V/score/index pointer is a DEVICE pointer owned by the caller.
 *     The parameter, plan and cache structs are HOST memory.
 *   - Tensors are [B, H, T, D]; the channel axis D is contiguous, the other
 *     strides are given in ELEMENTS in lagkv_params (0 = dense default).
 *     Layers may be folded into B: streams never interact.
 *   - All (b, h) streams have the same length, because every head keeps
 *     exactly k rows per chunk.
 *   - Calls validate on the host, enqueue on the given HIP stream
 *     (hipStream_t passed as void*, NULL = default stream) and return without
 *     synchronising.  Output sizes are pure functions of (T, S, L, k), see
 *     lagkv_plan.  Nothing is enqueued when validation fails.
 *   - The library allocates no device memory and keeps no state between calls: every
 *     call is a function of its arguments (launch overrides travel in lagkv_params).
 *   - Return value: a lagkv_status.  Inputs must be finite; NaN/Inf give
 *     unspecified scores (never out-of-bounds accesses).
 *   - Arithmetic: inputs as stored (fp32, bf16 or fp16), all scoring math in fp32,
 *     scores fp32, kept rows copied bit for bit.
 */
#ifndef LAGKV_H
#define LAGKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LAGKV_OK = 0,
  LAGKV_EINVAL = 1,     /* null pointer, r outside (0,1], k = floor(r*L) < 1, S < 0, L < 1 ... */
  LAGKV_ESHAPE = 2,     /* B/H/D/T/strides inconsistent or beyond the supported limits          */
  LAGKV_EDTYPE = 3,     /* unknown dtype or variant                                              */
  LAGKV_ECAPACITY = 4,  /* lagkv_cache too small for the rows to be appended                     */
  LAGKV_EWORKSPACE = 5, /* workspace pointer missing or shorter than lagkv_workspace_bytes()     */
  LAGKV_EHIP = 6        /* a HIP runtime call or kernel launch failed                            */
} lagkv_status;

typedef enum { LAGKV_F32 = 0, LAGKV_BF16 = 1, LAGKV_F16 = 2 /* IEEE binary16 */ } lagkv_dtype;

typedef enum {
  LAGKV_SCORE_LAG = 0,   /* Eq. 7-11: min/max from the next chunk                       */
  LAGKV_SCORE_LOCAL = 1, /* Eq. 14-15 (Scoring Methods ablation): min/max from the chunk */
  LAGKV_SCORE_L2 = 2     /* Eq. 16: score = -||K_t||_2, V unused                         */
} lagkv_variant;

/* Statement of the problem: shape of the cache and the three knobs of the method. */
typedef struct {
  int32_t B, H, D;     /* batch (x layers), KV heads, head dimension (D >= 1; D >= 2 if std_ddof=1) */
  int32_t S, L;        /* sink size S >= 0 and lag size L >= 1 (bullets 2-4 of subsection LagKV)     */
  double r;            /* retention ratio in (0, 1]; k = floor(r*L) rows kept per chunk, must be >= 1   */
  int32_t dtype;       /* lagkv_dtype of K and V                                                     */
  int32_t variant;     /* lagkv_variant                                                              */
  int32_t std_ddof;    /* divisor of the channel-wise std is D - std_ddof; 1 (default reading) or 0  */
  int32_t launch;      /* 0 = automatic launch choice, else a value returned by lagkv_launch_hint()   */
  int64_t stride_b, stride_h, stride_t; /* INPUT strides in elements; 0 = dense [B,H,T,D]           */
} lagkv_params;

/* Partition of a cache of T rows whose first n_static rows are final. */
typedef struct {
  int64_t n_chunks; /* full L-chunks after the static part                                  */
  int64_t n_scored; /* chunks that have a reference chunk = n_chunks - 1, or 0 if T-n_static < 2L */
  int64_t rem;      /* (T - n_static) mod L; these rows join the sliding window             */
  int64_t k;        /* rows kept per scored chunk                                           */
  int64_t T_out;    /* length after compression (Eq. 12 when n_static == S); T if no-op     */
} lagkv_plan_t;

/*
 * Host-only arithmetic of the partition bullets and Eq. 12-13.  n_static < 0
 * means "fresh cache" (n_static = S).  When T - n_static < 2L the pass is a
 * no-op (nothing is compressed below S + 2L): n_scored = 0 and T_out = T; not an error.
 */
int lagkv_plan(const lagkv_params* p, int64_t T, int64_t n_static, lagkv_plan_t* out);

/*
 * Inverse of Eq. 12-13 (host only): the retention that reaches a wanted compression
 * ratio C = 1 - L_R / T at fixed sink S and lag L, as the Experiments section does when
 * it adapts r per target ratio.  *k_out receives the LARGEST k in [1, L] whose
 * compression ratio (Eq. 13 with rL = k) is >= C, i.e. the most rows that may be kept
 * per chunk while still compressing at least that much; *r_out a ratio with
 * floor(r * L) == k exactly (the midpoint (k + 0.5) / L, or 1 when k == L).
 * LAGKV_EINVAL: null pointers, S < 0, L < 1, T < S + 2L (nothing is compressed, C = 0
 * whatever r), C outside [0, 1), or C not reachable even with k = 1.
 */
int lagkv_keep_for_compression(int64_t T, int32_t S, int32_t L, double C, int64_t* k_out,
                               double* r_out);

/*
 * Device workspace, in bytes, that lagkv_compress / lagkv_append_and_compress need for
 * these parameters (p->launch included) and T rows (for append: T = cache capacity, the
 * bound that holds for any single append).  0 when the fused kernels serve the shape: rows
 * of 48 to 512 bytes that are a multiple of 16 bytes, strides that are multiples of 16
 * bytes, a lag that fits the LDS budget.  The three-kernel path used for every other shape stages scores and kept
 * positions there.  The answer assumes 16-byte aligned K / V / output / cache pointers (any
 * hipMalloc'ed buffer is); a caller whose pointers are only element-aligned must ask, and
 * call, with a launch hint of LAGKV_PATH_STAGED.  Returns 0 on invalid parameters as well.
 */
size_t lagkv_workspace_bytes(const lagkv_params* p, int64_t T);

/*
 * Eq. 7-11: scores of every scored chunk.
 *   K, V    [B,H,T,D] device, dtype p->dtype (V may be NULL for LAGKV_SCORE_L2)
 *   scores  [B,H,n_scored*L] device fp32, dense; entry j of a stream belongs to
 *           row S + j.  Within a chunk the scores are softmax(std(Kbar)) +
 *           softmax(std(Vbar)) and sum to 2 (LAG, LOCAL); for LAGKV_SCORE_L2
 *           they are -||K_t||_2.
 * A reference channel with max == min contributes 0 to every token.
 * n_scored == 0: returns LAGKV_OK and writes nothing.
 * ws / ws_bytes: unused (every path writes the scores straight to `scores`); kept so
 * that the three device calls share one argument pattern.  May be NULL / 0.
 */
int lagkv_score(const lagkv_params* p, const void* K, const void* V, int64_t T,
                float* scores, void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Per-chunk, per-head top-k (the selection step after Eq. 11: every head keeps its own
 * k best rows of every chunk).
 *   scores  [B,H,n_scored*L] device fp32 as written by lagkv_score
 *   kept    [B,H,n_scored,k] device int32: absolute row positions (S + p*L + t)
 *           of the k highest scores of chunk p, ASCENDING.  Equal scores: the
 *           lower position wins.
 */
int lagkv_select(const lagkv_params* p, const float* scores, int64_t T, int32_t* kept,
                 void* hip_stream);

/*
 * The whole pass: score, select, compact.
 *   K_out, V_out  [B,H,T_out,D] device, dense, same dtype; row order: the S sink
 *                 rows, the kept rows of chunk 0, 1, ... (ascending position),
 *                 then the window rows S + n_scored*L .. T-1.  Bit copies.
 *   idx_out       [B,H,T_out] device int32 source row of every output row, or NULL
 *   scores_out    [B,H,n_scored*L] device fp32 as lagkv_score, or NULL
 * Inputs and outputs must not overlap.  No-op case (T - S < 2L): copies the
 * input (T_out = T).
 */
int lagkv_compress(const lagkv_params* p, const void* K, const void* V, int64_t T,
                   void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                   void* ws, size_t ws_bytes, void* hip_stream);

/*
 * Decode-time cache under recursive compression (Methodology: the same pass is applied
 * again whenever the uncompressed tail has grown by one lag, in prefill and in decode).  All buffers are caller-owned device
 * memory, dense [B,H,capacity,D] (p->stride_* describe K_new/V_new only).
 * The four counters are host integers, identical for every stream, and are
 * updated by lagkv_append_and_compress before it returns (the device work is
 * only enqueued).  A zero-initialised struct with buffers set is an empty cache.
 */
typedef struct {
  void* K;          /* [B,H,capacity,D]                                              */
  void* V;          /* [B,H,capacity,D]                                              */
  int32_t* pos;     /* [B,H,capacity] original position of every row held, or NULL   */
  int64_t capacity; /* rows per stream                                               */
  int64_t n_static; /* rows that are final: min(n_seen,S) + k * (chunks compressed)  */
  int64_t n_tail;   /* uncompressed rows after them; < 2L between calls              */
  int64_t n_seen;   /* tokens appended so far                                        */
} lagkv_cache;

/*
 * lagkv_compress for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments and results as lagkv_compress without ws / ws_bytes: when the three-kernel path
 * is taken, its scores and kept positions are staged in a fixed device array inside the
 * library (LAGKV_STATIC_SCRATCH_BYTES per GPU, held from the first call on that GPU until
 * the process ends) instead.  The call allocates and frees nothing.
 *   - LAGKV_EWORKSPACE when the pass would need more than LAGKV_STATIC_SCRATCH_BYTES
 *     (use lagkv_compress with a workspace then); nothing is enqueued.
 *   - The device that is current when the call is made must be the stream's device.
 *   - All calls on one GPU share that GPU's array: two calls that may run at the same time
 *     (different streams, different threads) race on it and must be serialised by the
 *     caller.  Nothing in the array has to be cleared between calls: every word a kernel
 *     reads is written earlier in the same call.
 */
#define LAGKV_STATIC_SCRATCH_BYTES (16u << 20)
int lagkv_compress_static(const lagkv_params* p, const void* K, const void* V, int64_t T,
                          void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                          void* hip_stream);

/*
 * Host only: set the counters of `cache` to the state of a cache that holds the output of
 * lagkv_compress on T rows (Eq. 12: n_static = S + k*n_scored, n_tail = L + rem,
 * n_seen = T; when T - S < 2L nothing was compressed: n_static = min(T, S),
 * n_tail = T - n_static).  Buffers and capacity are left as they are.
 * LAGKV_ECAPACITY if capacity < T_out, LAGKV_EINVAL on null pointers.
 */
int lagkv_cache_after_compress(const lagkv_params* p, int64_t T, lagkv_cache* cache);

/*
 * Host only: rows to hand to the next lagkv_append_and_compress call when a prompt is
 * compressed chunk by chunk during prefill (Ablation, prefill-stage compression): the
 * first call of an empty cache takes S + 2L rows (the shortest prefix that compresses
 * anything), every later call one lag L, both capped by rows_left.  Returns 0 when
 * rows_left <= 0 or on invalid arguments.
 */
int64_t lagkv_prefill_rows(const lagkv_params* p, const lagkv_cache* cache, int64_t rows_left);

/*
 * Append n_new rows per stream (K_new, V_new: [B,H,n_new,D] with p->stride_*,
 * 0 = dense), then, while the tail holds at least 2L rows, score its oldest L
 * rows against the next L, keep k of them right after the static part and
 * slide the remaining tail down.  Equivalent to lagkv_compress on the whole
 * history.  n_new = 0 is allowed.  Needs capacity >= n_static + n_tail + n_new.
 * All three scoring variants run in one fused kernel per call when the shape allows
 * (see lagkv_workspace_bytes); ws is used by the three-kernel path only.
 */
int lagkv_append_and_compress(const lagkv_params* p, lagkv_cache* cache, const void* K_new,
                              const void* V_new, int64_t n_new, void* ws, size_t ws_bytes,
                              void* hip_stream);

/*
 * Launch override for benchmarks, tests and sweeps.  A pure function: it packs its
 * arguments into the value lagkv_params.launch carries for ONE call; the library keeps
 * nothing.  0 in any argument means "choose automatically" (and launch = 0 is the same as
 * lagkv_launch_hint(0, 0, 0)).
 *   path      LAGKV_PATH_AUTO (the register-resident kernel where it applies, else the
 *             streaming fused kernel, else the three-kernel path); LAGKV_PATH_FUSED (the
 *             streaming fused kernel; error LAGKV_ESHAPE when the fused kernels do not
 *             cover the shape); LAGKV_PATH_STAGED (three-kernel path); or
 *             LAGKV_PATH_RESIDENT (the one-shot kernel that keeps a batch of rows in
 *             registers and reads every row once: 256-byte rows, L of 128, 256 or 512,
 *             not Eq. 16; LAGKV_ESHAPE otherwise; append calls treat it as FUSED)
 *   waves     wavefronts per workgroup of the fused kernels: 1 (append only), 2, 4 or 8
 *   segments  pieces each stream is cut into by the one-shot kernel, 1 .. 2^20
 * Returns -1 for a value the kernels do not support.  lagkv_workspace_bytes must be
 * asked with the same launch value as the call it sizes the workspace for.
 */
enum { LAGKV_PATH_AUTO = 0, LAGKV_PATH_FUSED = 1, LAGKV_PATH_STAGED = 2, LAGKV_PATH_RESIDENT = 3 };
int32_t lagkv_launch_hint(int path, int waves, int segments);

/*
 * lagkv_launch_hint with two further overrides (0 = automatic), for sweeps:
 *   order   which stream the i-th workgroup takes: LAGKV_ORDER_LINEAR (stream i),
 *           LAGKV_ORDER_EVEN_ODD (even streams first: the workgroups resident at one
 *           time span the whole tensor), LAGKV_ORDER_XCD (i mod 8 picks one eighth of
 *           the streams, so each of the eight L2 slices sees a contiguous eighth) or
 *           LAGKV_ORDER_BITREV (bit-reversed i).  Orders whose precondition fails
 *           (stream count not a multiple of 8 / not a power of two) fall back to LINEAR.
 *   select  how a chunk's top-k is taken: LAGKV_SELECT_WAVE (one wavefront, a different
 *           one for each chunk; bisection over the key bits with ballots) or
 *           LAGKV_SELECT_GROUP (all wavefronts; four 8-bit digit histograms in LDS; needs
 *           L <= threads of the workgroup, else WAVE).  The kept set is the same.
 * Returns -1 for an unknown value.
 */
enum { LAGKV_ORDER_LINEAR = 0, LAGKV_ORDER_EVEN_ODD = 1, LAGKV_ORDER_XCD = 2, LAGKV_ORDER_BITREV = 3 };
enum { LAGKV_SELECT_AUTO = 0, LAGKV_SELECT_WAVE = 1, LAGKV_SELECT_GROUP = 2 };
int32_t lagkv_launch_hint_ex(int path, int waves, int segments, int order, int select);

/*
 * Which kernels lagkv_compress runs for these parameters (launch override included) on a
 * cache of T rows held in 16-byte aligned buffers: LAGKV_PATH_RESIDENT, LAGKV_PATH_FUSED
 * (the streaming one-shot kernel) or LAGKV_PATH_STAGED (the three-kernel path, which needs
 * the workspace); for benchmarks and profiles that have to name the kernel they time.
 * Host only.  Returns minus the lagkv_status the call itself would return for parameters
 * it rejects.
 */
int lagkv_path_for(const lagkv_params* p, int64_t T);

/* Static, human readable text for a lagkv_status. */
const char* lagkv_strerror(int status);

/* Library version, major*10000 + minor*100 + patch. */
int lagkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LAGKV_H */
