// C ABI of the LagKV compression pass (see include/lagkv.h): host-side validation,
// the partition arithmetic of Eq. 12-13, path choice and kernel launches.
#include "lagkv.h"

#include <cmath>
#include <cstring>

#include "lagkv_internal.hpp"

using namespace lagkv;

namespace {

// Launch override carried by lagkv_params.launch (see lagkv_launch_hint):
//   bits 0-1 path, bits 2-5 wavefronts, bits 6-26 segments, bits 27-28 stream order,
//   bits 29-30 selection mode; 0 everywhere = automatic.
struct Hint {
  int path, waves, nseg, order, sel;
};
constexpr int kHintWavesShift = 2, kHintSegShift = 6, kHintOrderShift = 27, kHintSelShift = 29;
constexpr int kMaxSegments = 1 << 20;

bool parse_hint(int32_t v, Hint* h) {
  if (v < 0) return false;
  h->path = v & 3;
  h->waves = (v >> kHintWavesShift) & 15;
  h->nseg = (v >> kHintSegShift) & ((1 << 21) - 1);
  h->order = (v >> kHintOrderShift) & 3;
  h->sel = (v >> kHintSelShift) & 3;
  if (h->waves != 0 && h->waves != 1 && h->waves != 2 && h->waves != 4 && h->waves != 8) return false;
  return h->nseg <= kMaxSegments && h->sel <= LAGKV_SELECT_GROUP;
}

constexpr int64_t kMaxRows = 0x7fffffffLL;  // positions are int32
constexpr size_t kAlign = 256;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Norm {  // validated, normalised parameters
  int B, H, D, S, L, k, esize, f16, ddof, variant;
  int64_t streams;
  int64_t rowbytes;
  Hint hint;
};

int validate(const lagkv_params* p, Norm* n) {
  if (!p) return LAGKV_EINVAL;
  if (p->dtype != LAGKV_F32 && p->dtype != LAGKV_BF16 && p->dtype != LAGKV_F16) return LAGKV_EDTYPE;
  if (p->variant < LAGKV_SCORE_LAG || p->variant > LAGKV_SCORE_L2) return LAGKV_EDTYPE;
  if (!parse_hint(p->launch, &n->hint)) return LAGKV_EINVAL;
  if (p->std_ddof != 0 && p->std_ddof != 1) return LAGKV_EINVAL;
  if (p->B < 1 || p->H < 1 || p->D < 1) return LAGKV_ESHAPE;
  if (p->std_ddof == 1 && p->D < 2 && p->variant != LAGKV_SCORE_L2) return LAGKV_ESHAPE;
  if (p->S < 0 || p->L < 1) return LAGKV_EINVAL;
  if (!(p->r > 0.0) || !(p->r <= 1.0)) return LAGKV_EINVAL;  // also rejects NaN
  const double kd = std::floor(p->r * (double)p->L);
  if (kd < 1.0) return LAGKV_EINVAL;
  if (p->stride_b < 0 || p->stride_h < 0 || p->stride_t < 0) return LAGKV_ESHAPE;
  n->B = p->B;
  n->H = p->H;
  n->D = p->D;
  n->S = p->S;
  n->L = p->L;
  n->k = (int)kd;
  n->esize = p->dtype == LAGKV_F32 ? 4 : 2;
  n->f16 = p->dtype == LAGKV_F16 ? 1 : 0;
  n->ddof = p->std_ddof;
  n->variant = p->variant;
  n->streams = (int64_t)p->B * p->H;
  n->rowbytes = (int64_t)p->D * n->esize;
  if (n->streams > (1 << 24)) return LAGKV_ESHAPE;
  return LAGKV_OK;
}

void plan_of(const Norm& n, int64_t T, int64_t n_static, lagkv_plan_t* out) {
  const int64_t rest = T - n_static;
  out->k = n.k;
  if (rest < 2 * (int64_t)n.L) {  // below 2L rows after the static part nothing is compressed
    const int64_t r = rest > 0 ? rest : 0;
    out->n_chunks = r / n.L;
    out->rem = r % n.L;
    out->n_scored = 0;
    out->T_out = T;
    return;
  }
  out->n_chunks = rest / n.L;
  out->rem = rest % n.L;
  out->n_scored = out->n_chunks - 1;  // the last chunk has no reference
  out->T_out = n_static + (int64_t)n.k * out->n_scored + n.L + out->rem;  // Eq. 12
}

// Input strides in bytes; 0 means dense [B,H,T,D].
int strides_of(const lagkv_params* p, const Norm& n, int64_t T, int64_t* sb, int64_t* sh,
               int64_t* st) {
  const int64_t t = p->stride_t ? p->stride_t : n.D;
  const int64_t h = p->stride_h ? p->stride_h : t * T;
  const int64_t b = p->stride_b ? p->stride_b : h * n.H;
  if (t < n.D) return LAGKV_ESHAPE;
  *st = t * n.esize;
  *sh = h * n.esize;
  *sb = b * n.esize;
  return LAGKV_OK;
}

bool shape_fused(const Norm& n, int64_t sb, int64_t sh, int64_t st) {
  if (n.rowbytes % 16 != 0 || n.rowbytes < 48 || n.rowbytes > 512) return false;  // whole 16-byte slices
  return ((sb | sh | st) & 15) == 0;
}

int pick_waves(const Norm& n) {
  int nw = n.hint.waves ? n.hint.waves : 4;
  while (nw > 1 && fused_lds_bytes(n.D, n.L, n.k, nw) > (size_t)kMaxLdsBytes) nw >>= 1;
  return nw;
}

bool fused_fits(const Norm& n) {
  return split_lds_bytes(n.D, n.esize, n.L, n.k, 2) <= (size_t)80 * 1024 &&
         fused_lds_bytes(n.D, n.L, n.k, 1) <= (size_t)kMaxLdsBytes;
}

bool staged_fits(const Norm& n) {
  return staged_score_lds_bytes(n.D, n.L) <= (size_t)kMaxLdsBytes &&
         ((size_t)n.L + n.k) * 4 <= (size_t)kMaxLdsBytes;
}

// Wavefronts per workgroup of the tensor-split kernel (0 = its LDS need does not fit).
// Long chunks keep eight wavefronts streaming; for short chunks the per-chunk serial part
// (fold, selection by one wavefront, barriers) weighs more, and smaller workgroups - more of
// them per CU, each with its own selection - overlap it better (measured: L=128 0.59 ms with 2
// against 0.80 ms with 8 wavefronts on 256 streams of 16K rows).
int split_nw(const Norm& n) {
  int nw = n.L >= 512 ? 8 : n.L >= 256 ? 4 : 2;
  const int t = n.hint.waves;
  if (t == 2 || t == 4 || t == 8) nw = t;
  while (nw >= 2 && split_lds_bytes(n.D, n.esize, n.L, n.k, nw) > (size_t)80 * 1024) nw >>= 1;
  return nw >= 2 ? nw : 0;
}

// Streams are cut into segments only when there are too few of them to fill the chip: the
// target is 2 workgroups per CU (256 CUs) of 8 wavefronts, 3 of 4, 6 of 2 (measured optima;
// every segment reads one extra chunk for its first reference), and segments keep >= 4 chunks.
int pick_segments_split(const Norm& n, int64_t n_s, int nw) {
  int64_t nseg;
  if (n.hint.nseg) {
    nseg = n.hint.nseg;
  } else {
    const int64_t capacity = 256 * (nw >= 8 ? 2 : nw >= 4 ? 3 : 6);
    nseg = n.streams >= capacity ? 1 : (capacity + n.streams - 1) / n.streams;
    const int64_t cap = n_s / 4 > 1 ? n_s / 4 : 1;
    if (nseg > cap) nseg = cap;
  }
  if (nseg > n_s) nseg = n_s;
  if (nseg < 1) nseg = 1;
  return (int)nseg;
}

// Segments of the register-resident kernel: one workgroup per CU is resident, so streams are
// cut only until every CU has a workgroup (measured from 8 to 1024 streams: more segments
// never pay - every segment reads one extra chunk and runs a short last batch).
int pick_segments_hold(const Norm& n, int64_t n_s) {
  int64_t nseg = n.hint.nseg;
  if (!nseg) {
    nseg = n.streams >= 256 ? 1 : (256 + n.streams - 1) / n.streams;
    const int64_t cap = n_s / 4 > 1 ? n_s / 4 : 1;
    if (nseg > cap) nseg = cap;
  }
  if (nseg > n_s) nseg = n_s;
  return (int)(nseg < 1 ? 1 : nseg);
}

// The register-resident kernel is the default wherever it applies (rows of 256 bytes, lags
// of 128, 256 or 512 rows, Eq. 7-11 or Eq. 14-15): it reads every row once, where the
// streaming kernel reads the kept rows a second time for the compaction (and, for
// Eq. 14-15, every row a second time for the scoring); measured faster or equal from 8 to
// 1024 streams.
bool use_resident(const Norm& n) {
  if (n.variant == LAGKV_SCORE_L2 || !hold_supported(n.D, n.esize, n.L, n.k)) return false;
  return n.hint.path == LAGKV_PATH_RESIDENT || n.hint.path == LAGKV_PATH_AUTO;
}

// Launch the one-shot fused kernel.
int launch_fused_any(PassArgs& a, const Norm& n, hipStream_t s) {
  a.order = n.hint.order;
  a.sel = n.hint.sel;
  if (use_resident(n)) {
    a.nwaves = 8;
    a.nseg = pick_segments_hold(n, a.n_s);
    return launch_hold_pass(a, s) == hipSuccess ? LAGKV_OK : LAGKV_EHIP;
  }
  if (n.hint.path == LAGKV_PATH_RESIDENT) return LAGKV_ESHAPE;
  a.nwaves = split_nw(n);
  a.nseg = pick_segments_split(n, a.n_s, a.nwaves);
  return launch_split_pass(a, s) == hipSuccess ? LAGKV_OK : LAGKV_EHIP;
}

// Workspace of the three-kernel path for one pass: [scores][kept]
struct StagedWs {
  size_t off_scores, off_kept, total;
};
StagedWs staged_ws(const Norm& n, int64_t n_s, bool need_scores) {
  StagedWs w;
  w.off_scores = 0;
  const size_t sc = need_scores ? align_up((size_t)n.streams * n_s * n.L * 4) : 0;
  w.off_kept = sc;
  w.total = sc + align_up((size_t)n.streams * n_s * n.k * 4);
  return w;
}

// Workspace of the three-kernel append: [scores][kept][stage K][stage V][stage pos]
struct AppendWs {
  size_t off_scores, off_kept, off_k, off_v, off_pos, total;
};
AppendWs append_ws(const Norm& n, int64_t q, int64_t rows_staged) {
  AppendWs w;
  size_t o = 0;
  w.off_scores = o;
  o += align_up((size_t)n.streams * q * n.L * 4);
  w.off_kept = o;
  o += align_up((size_t)n.streams * q * n.k * 4);
  w.off_k = o;
  o += align_up((size_t)n.streams * rows_staged * n.rowbytes);
  w.off_v = o;
  o += align_up((size_t)n.streams * rows_staged * n.rowbytes);
  w.off_pos = o;
  o += align_up((size_t)n.streams * rows_staged * 4);
  w.total = o;
  return w;
}

int hip_status(hipError_t e) { return e == hipSuccess ? LAGKV_OK : LAGKV_EHIP; }

bool aligned_to(const void* p, uintptr_t a) { return ((uintptr_t)p & (a - 1)) == 0; }

void fill_pass(PassArgs* a, const Norm& n, const void* K, const void* V, int64_t T,
               const lagkv_plan_t& pl, int64_t sb, int64_t sh, int64_t st) {
  std::memset(a, 0, sizeof(*a));
  a->K = (const char*)K;
  a->V = (const char*)V;
  a->sb = sb;
  a->sh = sh;
  a->st = st;
  a->T = T;
  a->T_out = pl.T_out;
  a->n_s = pl.n_scored;
  a->B = n.B;
  a->H = n.H;
  a->D = n.D;
  a->S = n.S;
  a->L = n.L;
  a->k = n.k;
  a->esize = n.esize;
  a->f16 = n.f16;
  a->ddof = n.ddof;
  a->variant = n.variant;
  a->nseg = 1;
  a->nwaves = 4;
}

}  // namespace

extern "C" {

int lagkv_plan(const lagkv_params* p, int64_t T, int64_t n_static, lagkv_plan_t* out) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (!out) return LAGKV_EINVAL;
  if (T < 0 || T > kMaxRows) return LAGKV_ESHAPE;
  if (n_static < 0) n_static = n.S;
  if (n_static > T && T >= n.S) return LAGKV_EINVAL;
  plan_of(n, T, n_static, out);
  return LAGKV_OK;
}

int lagkv_keep_for_compression(int64_t T, int32_t S, int32_t L, double C, int64_t* k_out,
                               double* r_out) {
  if (!k_out || !r_out || S < 0 || L < 1 || !(C >= 0.0) || !(C < 1.0)) return LAGKV_EINVAL;
  if (T < (int64_t)S + 2 * (int64_t)L) return LAGKV_EINVAL;
  const int64_t n_s = (T - S) / L - 1, m = (T - S) % L;
  // Eq. 12-13 with rL = k: C(k) = 1 - (S + k*n_s + L + m) / T, decreasing in k.  Start from the
  // closed form and settle the boundary with the exact comparison the definition uses.
  auto ratio = [&](int64_t k) { return 1.0 - (double)(S + k * n_s + L + m) / (double)T; };
  int64_t k = (int64_t)std::floor(((1.0 - C) * (double)T - (double)(S + L + m)) / (double)n_s);
  if (k > L) k = L;
  if (k < 1) k = 1;
  while (k < L && ratio(k + 1) >= C) ++k;
  while (k >= 1 && ratio(k) < C) --k;
  if (k < 1) return LAGKV_EINVAL;
  *k_out = k;
  *r_out = k == L ? 1.0 : ((double)k + 0.5) / (double)L;
  return LAGKV_OK;
}

size_t lagkv_workspace_bytes(const lagkv_params* p, int64_t T) {
  Norm n;
  if (validate(p, &n) != LAGKV_OK || T < 1 || T > kMaxRows) return 0;
  int64_t sb, sh, st;
  if (strides_of(p, n, T, &sb, &sh, &st) != LAGKV_OK) return 0;
  const bool fused = n.hint.path != LAGKV_PATH_STAGED && shape_fused(n, sb, sh, st) && fused_fits(n);
  if (fused) return 0;
  // one pass over T rows, and an append into a cache of capacity T
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  const size_t pass = staged_ws(n, pl.n_scored > 0 ? pl.n_scored : 1, true).total;
  const size_t app = append_ws(n, T / n.L + 1, T).total;
  return pass > app ? pass : app;
}

int lagkv_score(const lagkv_params* p, const void* K, const void* V, int64_t T, float* scores,
                void* ws, size_t ws_bytes, void* hip_stream) {
  (void)ws;  // no path stages anything for the scores alone
  (void)ws_bytes;
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (T < 1 || T > kMaxRows) return LAGKV_ESHAPE;
  if (!K || (!V && n.variant != LAGKV_SCORE_L2)) return LAGKV_EINVAL;
  if (!aligned_to(K, n.esize) || !aligned_to(V, n.esize)) return LAGKV_EINVAL;
  int64_t sb, sh, st;
  rc = strides_of(p, n, T, &sb, &sh, &st);
  if (rc != LAGKV_OK) return rc;
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  if (pl.n_scored == 0) return LAGKV_OK;
  if (!scores) return LAGKV_EINVAL;
  hipStream_t s = (hipStream_t)hip_stream;
  PassArgs a;
  fill_pass(&a, n, K, V, T, pl, sb, sh, st);
  a.scores = scores;
  const int force = n.hint.path;
  const bool fused_ok = shape_fused(n, sb, sh, st) && fused_fits(n) &&
                        fused_supported(n.D, n.esize, sb, sh, st, K, V, nullptr, nullptr);
  if ((force == LAGKV_PATH_FUSED || force == LAGKV_PATH_RESIDENT) && !fused_ok) return LAGKV_ESHAPE;
  if (fused_ok && force != LAGKV_PATH_STAGED) return launch_fused_any(a, n, s);
  if (!staged_fits(n)) return LAGKV_ESHAPE;
  return hip_status(launch_staged_score(a, n.S, scores, s));
}

int lagkv_select(const lagkv_params* p, const float* scores, int64_t T, int32_t* kept,
                 void* hip_stream) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (T < 1 || T > kMaxRows) return LAGKV_ESHAPE;
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  if (pl.n_scored == 0) return LAGKV_OK;
  if (!scores || !kept) return LAGKV_EINVAL;
  if (((size_t)n.L + n.k) * 4 > (size_t)kMaxLdsBytes) return LAGKV_ESHAPE;
  return hip_status(launch_select(scores, n.streams, pl.n_scored, n.L, n.k, n.S, kept,
                                  (hipStream_t)hip_stream));
}

int lagkv_compress(const lagkv_params* p, const void* K, const void* V, int64_t T, void* K_out,
                   void* V_out, int32_t* idx_out, float* scores_out, void* ws, size_t ws_bytes,
                   void* hip_stream) {
  return lagkv::compress_with_workspace(p, K, V, T, K_out, V_out, idx_out, scores_out, ws, ws_bytes,
                                        hip_stream);
}

}  // extern "C"

// Workspace one lagkv_compress call needs (0: the fused kernels serve it, or the parameters
// are invalid and the call itself will say so).
size_t lagkv::compress_workspace_need(const lagkv_params* p, int64_t T) {
  Norm n;
  if (validate(p, &n) != LAGKV_OK || T < 1 || T > kMaxRows) return 0;
  int64_t sb, sh, st;
  if (strides_of(p, n, T, &sb, &sh, &st) != LAGKV_OK) return 0;
  if (n.hint.path != LAGKV_PATH_STAGED && shape_fused(n, sb, sh, st) && fused_fits(n)) return 0;
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  return pl.n_scored > 0 ? staged_ws(n, pl.n_scored, true).total : 0;
}

// The whole pass with the workspace given by the caller (lagkv_compress) or taken from the
// library's static scratch (lagkv_compress_static).
int lagkv::compress_with_workspace(const lagkv_params* p, const void* K, const void* V, int64_t T,
                                   void* K_out, void* V_out, int32_t* idx_out, float* scores_out,
                                   void* ws, size_t ws_bytes, void* hip_stream) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (T < 1 || T > kMaxRows) return LAGKV_ESHAPE;
  if (!K || !V || !K_out || !V_out) return LAGKV_EINVAL;
  if (!aligned_to(K, n.esize) || !aligned_to(V, n.esize) || !aligned_to(K_out, n.esize) ||
      !aligned_to(V_out, n.esize))
    return LAGKV_EINVAL;
  int64_t sb, sh, st;
  rc = strides_of(p, n, T, &sb, &sh, &st);
  if (rc != LAGKV_OK) return rc;
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  hipStream_t s = (hipStream_t)hip_stream;
  if (pl.n_scored == 0) {  // nothing to compress: the output is the input
    const int64_t osh = T * n.rowbytes, osb = osh * n.H;
    hipError_t e = launch_copy_rows((const char*)K, sb, sh, st, (char*)K_out, osb, osh, n.rowbytes,
                                    n.B, n.H, T, n.rowbytes, s);
    if (e == hipSuccess)
      e = launch_copy_rows((const char*)V, sb, sh, st, (char*)V_out, osb, osh, n.rowbytes, n.B, n.H,
                           T, n.rowbytes, s);
    if (e == hipSuccess && idx_out) e = launch_iota_rows(idx_out, n.streams, T, 0, T, 0, s);
    return hip_status(e);
  }
  PassArgs a;
  fill_pass(&a, n, K, V, T, pl, sb, sh, st);
  a.K_out = (char*)K_out;
  a.V_out = (char*)V_out;
  a.idx_out = idx_out;
  a.scores = scores_out;
  const int force = n.hint.path;
  const bool fused_ok = shape_fused(n, sb, sh, st) && fused_fits(n) &&
                        fused_supported(n.D, n.esize, sb, sh, st, K, V, K_out, V_out);
  if ((force == LAGKV_PATH_FUSED || force == LAGKV_PATH_RESIDENT) && !fused_ok) return LAGKV_ESHAPE;
  if (fused_ok && force != LAGKV_PATH_STAGED) return launch_fused_any(a, n, s);
  if (!staged_fits(n)) return LAGKV_ESHAPE;
  const StagedWs w = staged_ws(n, pl.n_scored, scores_out == nullptr);
  if (!ws || ws_bytes < w.total || !aligned_to(ws, 16)) return LAGKV_EWORKSPACE;
  float* sc = scores_out ? scores_out : (float*)((char*)ws + w.off_scores);
  int32_t* kept = (int32_t*)((char*)ws + w.off_kept);
  hipError_t e = launch_staged_score(a, n.S, sc, s);
  if (e == hipSuccess) e = launch_select(sc, n.streams, pl.n_scored, n.L, n.k, n.S, kept, s);
  if (e == hipSuccess) e = launch_staged_gather(a, kept, s);
  return hip_status(e);
}

extern "C" {

int lagkv_cache_after_compress(const lagkv_params* p, int64_t T, lagkv_cache* c) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (!c) return LAGKV_EINVAL;
  if (T < 0 || T > kMaxRows) return LAGKV_ESHAPE;
  lagkv_plan_t pl;
  plan_of(n, T, n.S, &pl);
  if (c->capacity < pl.T_out) return LAGKV_ECAPACITY;
  // Eq. 12: the output is [sink | k rows per scored chunk | last chunk + remainder]
  c->n_static = pl.n_scored > 0 ? n.S + (int64_t)n.k * pl.n_scored : (T < n.S ? T : n.S);
  c->n_tail = pl.T_out - c->n_static;
  c->n_seen = T;
  return LAGKV_OK;
}

int64_t lagkv_prefill_rows(const lagkv_params* p, const lagkv_cache* c, int64_t rows_left) {
  Norm n;
  if (validate(p, &n) != LAGKV_OK || !c || rows_left <= 0) return 0;
  const int64_t want = c->n_seen == 0 ? (int64_t)n.S + 2 * (int64_t)n.L : (int64_t)n.L;
  return rows_left < want ? rows_left : want;
}

int lagkv_append_and_compress(const lagkv_params* p, lagkv_cache* c, const void* K_new,
                              const void* V_new, int64_t n_new, void* ws, size_t ws_bytes,
                              void* hip_stream) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return rc;
  if (!c || !c->K || !c->V) return LAGKV_EINVAL;
  if (n_new < 0 || c->capacity < 1 || c->n_static < 0 || c->n_tail < 0 || c->n_seen < 0)
    return LAGKV_EINVAL;
  if (n_new > 0 && (!K_new || !V_new)) return LAGKV_EINVAL;
  if (c->capacity > kMaxRows || c->n_seen + n_new > kMaxRows) return LAGKV_ESHAPE;
  if (!aligned_to(c->K, n.esize) || !aligned_to(c->V, n.esize) || !aligned_to(K_new, n.esize) ||
      !aligned_to(V_new, n.esize))
    return LAGKV_EINVAL;
  const int64_t held = c->n_static + c->n_tail;
  if (held + n_new > c->capacity) return LAGKV_ECAPACITY;
  int64_t sb = 0, sh = 0, st = 0;
  if (n_new > 0) {
    rc = strides_of(p, n, n_new, &sb, &sh, &st);
    if (rc != LAGKV_OK) return rc;
  }
  // host arithmetic of the recursion: the sink fills first, then the tail is cut
  // into L-chunks and all but the last full one are compressed
  const int64_t total = held + n_new;
  int64_t base = c->n_static;
  if (c->n_seen < n.S) {
    const int64_t seen = c->n_seen + n_new;
    base = seen < n.S ? seen : n.S;
  }
  const int64_t tail = total - base;
  const int64_t q = tail >= 2 * (int64_t)n.L ? tail / n.L - 1 : 0;
  hipStream_t s = (hipStream_t)hip_stream;
  const int force = n.hint.path;
  const bool fused_ok = shape_fused(n, sb, sh, st) && fused_fits(n) &&
                        fused_supported(n.D, n.esize, sb, sh, st, c->K, c->V, K_new, V_new);
  if ((force == LAGKV_PATH_FUSED || force == LAGKV_PATH_RESIDENT) && !fused_ok) return LAGKV_ESHAPE;
  hipError_t e = hipSuccess;
  if (fused_ok && force != LAGKV_PATH_STAGED) {
    if (n_new > 0 || q > 0) {
      AppendArgs a;
      std::memset(&a, 0, sizeof(a));
      a.K = (char*)c->K;
      a.V = (char*)c->V;
      a.pos = c->pos;
      a.K_new = (const char*)K_new;
      a.V_new = (const char*)V_new;
      a.nsb = sb;
      a.nsh = sh;
      a.nst = st;
      a.capacity = c->capacity;
      a.n_static = c->n_static;
      a.n_tail = c->n_tail;
      a.n_seen = c->n_seen;
      a.n_new = n_new;
      a.rounds = q;
      a.B = n.B;
      a.H = n.H;
      a.D = n.D;
      a.S = n.S;
      a.L = n.L;
      a.k = n.k;
      a.esize = n.esize;
      a.f16 = n.f16;
      a.ddof = n.ddof;
      a.variant = n.variant;
      a.sel = n.hint.sel;
      a.nwaves = pick_waves(n);
      // the single-round kernel serves the steady decode step unless a launch shape is forced
      if (n.hint.waves == 0 && decode_step_supported(a)) e = launch_decode_step(a, s);
      else e = launch_fused_append(a, s);
    }
  } else {
    if (!staged_fits(n)) return LAGKV_ESHAPE;
    const int64_t rows_staged = q > 0 ? q * n.k + (tail - q * n.L) : 0;
    const AppendWs w = append_ws(n, q, rows_staged);
    if (q > 0 && (!ws || ws_bytes < w.total || !aligned_to(ws, 16))) return LAGKV_EWORKSPACE;
    const int64_t csh = c->capacity * n.rowbytes, csb = csh * n.H;
    if (n_new > 0) {
      e = launch_copy_rows((const char*)K_new, sb, sh, st, (char*)c->K + held * n.rowbytes, csb, csh,
                           n.rowbytes, n.B, n.H, n_new, n.rowbytes, s);
      if (e == hipSuccess)
        e = launch_copy_rows((const char*)V_new, sb, sh, st, (char*)c->V + held * n.rowbytes, csb,
                             csh, n.rowbytes, n.B, n.H, n_new, n.rowbytes, s);
      if (e == hipSuccess && c->pos)
        e = launch_iota_rows(c->pos, n.streams, c->capacity, held, n_new, (int32_t)c->n_seen, s);
    }
    if (e == hipSuccess && q > 0) {
      char* wsb = (char*)ws;
      float* sc = (float*)(wsb + w.off_scores);
      int32_t* kept = (int32_t*)(wsb + w.off_kept);
      PassArgs a;
      lagkv_plan_t pl;
      pl.n_chunks = q + 1;
      pl.n_scored = q;
      pl.rem = 0;
      pl.k = n.k;
      pl.T_out = rows_staged;
      fill_pass(&a, n, c->K, c->V, total, pl, csb, csh, n.rowbytes);
      e = launch_staged_score(a, base, sc, s);
      if (e == hipSuccess) e = launch_select(sc, n.streams, q, n.L, n.k, base, kept, s);
      GatherMap m;
      m.n_pre = 0;
      m.pre0 = 0;
      m.n_kept = q * n.k;
      m.post0 = base + q * n.L;
      m.n_out = rows_staged;
      const int64_t ssh = rows_staged * n.rowbytes, ssb = ssh * n.H;
      if (e == hipSuccess)
        e = launch_gather_rows((const char*)c->K, csb, csh, n.rowbytes, n.B, n.H, wsb + w.off_k,
                               n.rowbytes, n.esize, kept, nullptr, m, s);
      if (e == hipSuccess)
        e = launch_gather_rows((const char*)c->V, csb, csh, n.rowbytes, n.B, n.H, wsb + w.off_v,
                               n.rowbytes, n.esize, kept, nullptr, m, s);
      if (e == hipSuccess)
        e = launch_copy_rows(wsb + w.off_k, ssb, ssh, n.rowbytes, (char*)c->K + base * n.rowbytes,
                             csb, csh, n.rowbytes, n.B, n.H, rows_staged, n.rowbytes, s);
      if (e == hipSuccess)
        e = launch_copy_rows(wsb + w.off_v, ssb, ssh, n.rowbytes, (char*)c->V + base * n.rowbytes,
                             csb, csh, n.rowbytes, n.B, n.H, rows_staged, n.rowbytes, s);
      if (e == hipSuccess && c->pos) {
        // positions are a [streams, capacity] tensor of one 4-byte channel
        e = launch_gather_rows((const char*)c->pos, c->capacity * 4 * n.H, c->capacity * 4, 4, n.B,
                               n.H, wsb + w.off_pos, 4, 4, kept, nullptr, m, s);
        if (e == hipSuccess)
          e = launch_copy_rows(wsb + w.off_pos, rows_staged * 4 * n.H, rows_staged * 4, 4,
                               (char*)c->pos + base * 4, c->capacity * 4 * n.H, c->capacity * 4, 4,
                               n.B, n.H, rows_staged, 4, s);
      }
    }
  }
  if (e != hipSuccess) return LAGKV_EHIP;
  c->n_seen += n_new;
  c->n_static = base + q * n.k;
  c->n_tail = tail - q * n.L;
  return LAGKV_OK;
}

int32_t lagkv_launch_hint(int path, int waves, int segments) {
  if (path < 0 || path > LAGKV_PATH_RESIDENT || segments < 0 || segments > kMaxSegments) return -1;
  if (waves != 0 && waves != 1 && waves != 2 && waves != 4 && waves != 8) return -1;
  return (int32_t)(path | (waves << kHintWavesShift) | (segments << kHintSegShift));
}

int32_t lagkv_launch_hint_ex(int path, int waves, int segments, int order, int select) {
  const int32_t base = lagkv_launch_hint(path, waves, segments);
  if (base < 0 || order < 0 || order > LAGKV_ORDER_BITREV || select < 0 || select > LAGKV_SELECT_GROUP)
    return -1;
  return base | (order << kHintOrderShift) | (select << kHintSelShift);
}

int lagkv_path_for(const lagkv_params* p, int64_t T) {
  Norm n;
  int rc = validate(p, &n);
  if (rc != LAGKV_OK) return -rc;
  if (T < 1 || T > kMaxRows) return -LAGKV_ESHAPE;
  int64_t sb, sh, st;
  rc = strides_of(p, n, T, &sb, &sh, &st);
  if (rc != LAGKV_OK) return -rc;
  const int force = n.hint.path;
  const bool fused_ok = shape_fused(n, sb, sh, st) && fused_fits(n);
  if ((force == LAGKV_PATH_FUSED || force == LAGKV_PATH_RESIDENT) && !fused_ok) return -LAGKV_ESHAPE;
  if (fused_ok && force != LAGKV_PATH_STAGED) {
    if (use_resident(n)) return LAGKV_PATH_RESIDENT;
    return force == LAGKV_PATH_RESIDENT ? -LAGKV_ESHAPE : LAGKV_PATH_FUSED;
  }
  return staged_fits(n) ? LAGKV_PATH_STAGED : -LAGKV_ESHAPE;
}

const char* lagkv_strerror(int status) {
  switch (status) {
    case LAGKV_OK: return "ok";
    case LAGKV_EINVAL: return "invalid argument (null pointer, r outside (0,1], floor(r*L) < 1, S < 0, L < 1, misaligned pointer)";
    case LAGKV_ESHAPE: return "unsupported or inconsistent shape, stride or size";
    case LAGKV_EDTYPE: return "unknown dtype or scoring variant";
    case LAGKV_ECAPACITY: return "cache capacity too small for the appended rows";
    case LAGKV_EWORKSPACE: return "workspace missing, misaligned or smaller than lagkv_workspace_bytes()";
    case LAGKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int lagkv_version(void) { return 200; }

}  // extern "C"
