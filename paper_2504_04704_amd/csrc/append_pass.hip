// Decode-time LagKV kernel for gfx950: append rows to a dense cache and compress, in
// place, every chunk of the tail that has a reference chunk.
//
// Row layout (shared with the one-shot kernel): a token row (D channels) is up to 16*LPR
// bytes and is held by LPR consecutive lanes, 16 bytes each (lanes beyond a shorter row's
// slices repeat its last one, see row_ops.hpp), so one wave64 load instruction
// fetches 64/LPR whole rows and the per-token channel reductions of Eq. 10 are DPP
// reductions over LPR lanes.  The per-channel min/max of Eq. 7-8 accumulate in
// registers down the rows a lane visits and are folded across row groups and
// wavefronts once per chunk.
#include "lagkv_internal.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"
#include "wg_select.hpp"
#include "lds_dma.hpp"

namespace lagkv {

// K and V statistics side by side for the kernel whose lanes handle both tensors: the running
// per-channel min/max (Eq. 7-8) and the form Eq. 9 consumes, one TStats / TRef per tensor.
template <int VEC>
struct ChanStats {
  TStats<VEC> K, V;
  __device__ __forceinline__ void reset() {
    K.reset();
    V.reset();
  }
};
template <int VEC>
struct RefStats {
  TRef<VEC> K, V;
  __device__ __forceinline__ void from(const ChanStats<VEC>& s, bool live) {
    K.from(s.K, live);
    V.from(s.V, live);
  }
};

struct Geometry {
  int lane, wave, nw;  // lane in wave, wave in workgroup, waves per workgroup
  int rl, cl;          // row within a wave step, lane within the row
  int clc;             // 16-byte column slice of the lane (the last one again beyond the row's slices)
  bool live;           // the lane holds channels of its own
  int rowbytes;        // bytes of a dense row
  int rps;             // rows per workgroup step
  int row0;            // first row this lane visits
};

template <int LPR>
__device__ __forceinline__ Geometry make_geometry(int units) {
  Geometry g;
  g.lane = threadIdx.x & 63;
  g.wave = threadIdx.x >> 6;
  g.nw = blockDim.x >> 6;
  g.rl = g.lane / LPR;
  g.cl = g.lane % LPR;
  g.live = g.cl < units;
  g.clc = g.live ? g.cl : units - 1;
  g.rowbytes = units * 16;
  g.rps = g.nw * (kWave / LPR);
  g.row0 = g.wave * (kWave / LPR) + g.rl;
  return g;
}

// One pass over the L rows of a chunk.  STATS: fold the rows into `acc`.  SCORE:
// write the channel variance of every token, normalised with `ref`, to sK/sV (LDS).
// Rows past L are clamped to the last row (duplicates do not change min/max).
template <typename ET, int LPR, bool STATS, bool SCORE>
__device__ __forceinline__ void scan_chunk(const char* __restrict__ kp, const char* __restrict__ vp,
                                           int64_t st, int L, const Geometry& g,
                                           ChanStats<ET::VEC>& acc, const RefStats<ET::VEC>& ref,
                                           float inv_D, float inv_dof, float* sK, float* sV) {
  constexpr int VEC = ET::VEC;
  constexpr int U = 4;
  const int n_iter = (L + g.rps - 1) / g.rps;
  const int64_t coff = (int64_t)g.clc * 16;
  for (int it = 0; it < n_iter; it += U) {
    uint4 kq[U], vq[U];
    int r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      r[u] = g.row0 + (it + u) * g.rps;
      const int rr = r[u] < L ? r[u] : L - 1;
      kq[u] = ld16(kp + (int64_t)rr * st + coff);
      vq[u] = ld16(vp + (int64_t)rr * st + coff);
    }
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      float x0[VEC], x1[VEC];
      float sgK0 = 0.f, sgK1 = 0.f, sgV0 = 0.f, sgV1 = 0.f;
      unpack<ET>(kq[u], x0);
      unpack<ET>(kq[u + 1], x1);
      if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          acc.K.mn[j] = fminf(fminf(acc.K.mn[j], x0[j]), x1[j]);
          acc.K.mx[j] = fmaxf(fmaxf(acc.K.mx[j], x0[j]), x1[j]);
        }
      }
      if constexpr (SCORE) {
        sgK0 = token_var<LPR, VEC>(x0, ref.K.mn, ref.K.iv, ref.K.bias, inv_D, inv_dof, g.live);
        sgK1 = token_var<LPR, VEC>(x1, ref.K.mn, ref.K.iv, ref.K.bias, inv_D, inv_dof, g.live);
      }
      unpack<ET>(vq[u], x0);
      unpack<ET>(vq[u + 1], x1);
      if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          acc.V.mn[j] = fminf(fminf(acc.V.mn[j], x0[j]), x1[j]);
          acc.V.mx[j] = fmaxf(fmaxf(acc.V.mx[j], x0[j]), x1[j]);
        }
      }
      if constexpr (SCORE) {
        sgV0 = token_var<LPR, VEC>(x0, ref.V.mn, ref.V.iv, ref.V.bias, inv_D, inv_dof, g.live);
        sgV1 = token_var<LPR, VEC>(x1, ref.V.mn, ref.V.iv, ref.V.bias, inv_D, inv_dof, g.live);
        if (g.cl == 0) {
          if (r[u] < L) {
            sK[r[u]] = sgK0;
            sV[r[u]] = sgV0;
          }
          if (r[u + 1] < L) {
            sK[r[u + 1]] = sgK1;
            sV[r[u + 1]] = sgV1;
          }
        }
      }
    }
  }
}

// Fold the per-lane partial min/max across the row groups of a wave and across the
// wavefronts of the workgroup; every lane ends with the statistics of its own VEC
// channels over the whole chunk.  Contains one __syncthreads(), which also publishes
// the spreads written by scan_chunk.  statbuf: [nw][4][D] floats of LDS.
template <int LPR, int VEC>
__device__ __forceinline__ void fold_stats(ChanStats<VEC>& acc, const Geometry& g, float* statbuf,
                                           int D) {
#pragma unroll
  for (int m = LPR; m < kWave; m <<= 1) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      acc.K.mn[j] = fminf(acc.K.mn[j], __shfl_xor(acc.K.mn[j], m));
      acc.K.mx[j] = fmaxf(acc.K.mx[j], __shfl_xor(acc.K.mx[j], m));
      acc.V.mn[j] = fminf(acc.V.mn[j], __shfl_xor(acc.V.mn[j], m));
      acc.V.mx[j] = fmaxf(acc.V.mx[j], __shfl_xor(acc.V.mx[j], m));
    }
  }
  if (g.nw > 1) {
    if (g.rl == 0) {
      float* w = statbuf + (size_t)g.wave * 4 * D + g.clc * VEC;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        w[j] = acc.K.mn[j];
        w[D + j] = acc.K.mx[j];
        w[2 * D + j] = acc.V.mn[j];
        w[3 * D + j] = acc.V.mx[j];
      }
    }
    __syncthreads();
    for (int w = 0; w < g.nw; ++w) {
      const float* rd = statbuf + (size_t)w * 4 * D + g.clc * VEC;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        acc.K.mn[j] = fminf(acc.K.mn[j], rd[j]);
        acc.K.mx[j] = fmaxf(acc.K.mx[j], rd[j + D]);
        acc.V.mn[j] = fminf(acc.V.mn[j], rd[j + 2 * D]);
        acc.V.mx[j] = fmaxf(acc.V.mx[j], rd[j + 3 * D]);
      }
    }
  } else {
    __syncthreads();
  }
}

struct LdsLayout {
  int off_sK, off_sV, off_list, off_stat, total;  // in bytes
};
__host__ __device__ inline LdsLayout lds_layout(int D, int L, int k, int nw) {
  LdsLayout l;
  const int lp = (L + 3) & ~3;
  const int kp = (k + 3) & ~3;
  l.off_sK = 0;
  l.off_sV = lp * 4;
  l.off_list = 2 * lp * 4;
  l.off_stat = l.off_list + kp * 4;
  l.total = l.off_stat + (nw > 1 ? nw * 4 * D * 4 : 0);
  return l;
}

// ---------------------------------------------------------------------------------
// Decode-time variant: one workgroup per stream, in place.  Appends the new rows,
// then compresses `rounds` chunks of the tail front to back (each against the raw
// next chunk) and finally slides what is left of the tail down behind the kept rows.
// Every in-place move goes destination <= source in ascending order, one register
// staged batch at a time: a batch is loaded, the workgroup synchronises, the batch is
// stored; the rows a later batch reads lie above everything stored so far.
// ---------------------------------------------------------------------------------
template <int LPR>
__device__ __forceinline__ void move_rows_down(char* kc, char* vc, int32_t* pc, int64_t src0,
                                               int64_t dst0, int64_t nrows, const Geometry& g,
                                               int tid, int nthreads) {
  const int64_t rowbytes = g.rowbytes, coff = (int64_t)g.clc * 16;
  constexpr int UB = 4;
  const int64_t batch = (int64_t)UB * g.rps;
  for (int64_t r0 = 0; r0 < nrows; r0 += batch) {
    uint4 kq[UB], vq[UB];
    int32_t pv[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int64_t r = r0 + u * g.rps + g.row0;
      if (r < nrows) {
        kq[u] = ld16(kc + (src0 + r) * rowbytes + coff);
        vq[u] = ld16(vc + (src0 + r) * rowbytes + coff);
        if (pc && g.cl == 0) pv[u] = pc[src0 + r];
      }
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int64_t r = r0 + u * g.rps + g.row0;
      if (r < nrows) {
        st16(kc + (dst0 + r) * rowbytes + coff, kq[u]);
        st16(vc + (dst0 + r) * rowbytes + coff, vq[u]);
        if (pc && g.cl == 0) pc[dst0 + r] = pv[u];
      }
    }
  }
  (void)tid;
  (void)nthreads;
}

template <typename ET, int LPR>
__global__ void __launch_bounds__(512) fused_append_kernel(const AppendArgs a) {
  constexpr int VEC = ET::VEC;
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int units = (a.D * a.esize) >> 4;
  const Geometry g = make_geometry<LPR>(units);
  const LdsLayout lay = lds_layout(a.D, a.L, a.k, g.nw);
  float* sK = reinterpret_cast<float*>(lds + lay.off_sK);
  float* sV = reinterpret_cast<float*>(lds + lay.off_sV);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);

  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int64_t stream = blockIdx.x;
  const int64_t b = stream / a.H, h = stream % a.H;
  const int64_t rowbytes = g.rowbytes;
  char* kc = a.K + stream * a.capacity * rowbytes;
  char* vc = a.V + stream * a.capacity * rowbytes;
  int32_t* pc = a.pos ? a.pos + stream * a.capacity : nullptr;
  const int L = a.L, k = a.k;
  const float inv_D = 1.0f / (float)a.D;
  const float inv_dof = 1.0f / (float)(a.D - a.ddof);

  for (int i = tid; i < k; i += nthreads) list[i] = 0;

  // 1. append
  const int64_t end0 = a.n_static + a.n_tail;
  if (a.n_new > 0) {
    const char* kn = a.K_new + b * a.nsb + h * a.nsh;
    const char* vn = a.V_new + b * a.nsb + h * a.nsh;
    copy_rows_kv<LPR>(kn, vn, a.nst, kc + end0 * rowbytes, vc + end0 * rowbytes, rowbytes, a.n_new,
                      units, tid, nthreads);
    if (pc)
      for (int64_t i = tid; i < a.n_new; i += nthreads) pc[end0 + i] = (int32_t)(a.n_seen + i);
  }
  if (a.rounds <= 0) return;
  __syncthreads();

  // static boundary after the append (the sink fills up first)
  const int64_t total = end0 + a.n_new;
  int64_t base = a.n_static;
  if (a.n_seen < a.S) {
    const int64_t seen = a.n_seen + a.n_new;
    base = seen < a.S ? seen : a.S;
  }

  ChanStats<VEC> acc;
  RefStats<VEC> ref;
  const int64_t coff = (int64_t)g.clc * 16;
  for (int64_t j = 0; j < a.rounds; ++j) {
    const int64_t cur = base + j * L;      // rows of the chunk (not yet moved)
    const int64_t dst = base + j * k;      // where its kept rows go
    if (a.variant == 2) {
      // Eq. 16: score = -||K_t||_2 from the chunk's keys alone; V is read only where it is kept
      const int n_iter = (L + g.rps - 1) / g.rps;
      for (int it = 0; it < n_iter; ++it) {
        const int r = g.row0 + it * g.rps;
        float x[VEC];
        unpack<ET>(ld16(kc + (cur + (r < L ? r : L - 1)) * rowbytes + coff), x);
        float ss = 0.f;
#pragma unroll
        for (int i = 0; i < VEC; ++i) ss = fmaf(x[i], x[i], ss);
        if (!g.live) ss = 0.f;
        ss = group_sum<LPR>(ss);
        if (g.cl == 0 && r < L) sK[r] = -sqrtf(ss);
      }
      __syncthreads();
      if (g.wave == 0) wave_topk_scores(sK, L, k, list, g.lane);
    } else {
      acc.reset();
      const int64_t refc = (a.variant == 1) ? cur : cur + L;  // Eq. 14-15 vs Eq. 7-8
      scan_chunk<ET, LPR, true, false>(kc + refc * rowbytes, vc + refc * rowbytes, rowbytes, L, g, acc,
                                       ref, inv_D, inv_dof, sK, sV);
      fold_stats<LPR, VEC>(acc, g, statbuf, a.D);
      ref.from(acc, g.live);
      scan_chunk<ET, LPR, false, true>(kc + cur * rowbytes, vc + cur * rowbytes, rowbytes, L, g, acc,
                                       ref, inv_D, inv_dof, sK, sV);
      __syncthreads();
      if (g.wave == 0) wave_score_select_any(sK, sV, L, k, true, nullptr, list, nullptr, g.lane);
    }
    __syncthreads();
    // staged in-place gather of the kept rows
    constexpr int UB = 4;
    for (int s0 = 0; s0 < k; s0 += UB * g.rps) {
      uint4 kq[UB], vq[UB];
      int32_t pv[UB];
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const int sl = s0 + u * g.rps + g.row0;
        if (sl < k) {
          const int64_t src = cur + list[sl];
          kq[u] = ld16(kc + src * rowbytes + coff);
          vq[u] = ld16(vc + src * rowbytes + coff);
          if (pc && g.cl == 0) pv[u] = pc[src];
        }
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
#pragma unroll
      for (int u = 0; u < UB; ++u) {
        const int sl = s0 + u * g.rps + g.row0;
        if (sl < k) {
          st16(kc + (dst + sl) * rowbytes + coff, kq[u]);
          st16(vc + (dst + sl) * rowbytes + coff, vq[u]);
          if (pc && g.cl == 0) pc[dst + sl] = pv[u];
        }
      }
    }
    __syncthreads();  // list and statbuf are rewritten by the next round
  }
  // 3. slide the rest of the tail behind the kept rows
  const int64_t src0 = base + a.rounds * L, dst0 = base + a.rounds * k;
  if (src0 != dst0)
    move_rows_down<LPR>(kc, vc, pc, src0, dst0, total - src0, g, tid, nthreads);
}

// ---------------------------------------------------------------------------------
// Single-round decode step: the common call, in which the appended rows complete
// exactly one more chunk (2L <= tail + new < 3L, sink already full; Eq. 7-11 scoring, or
// Eq. 16 with the reference steps reduced to the row moves).
// The new rows are never stored at the end of the tail first: the tail is addressed
// "virtually" (row v lives in the cache when v < n_tail, else in K_new/V_new), every
// row is read from memory once and written once at its final place:
//   rows [L,2L)  reference chunk: min/max (Eq. 7-8), parked in LDS, stored at [k, k+L)
//   rows [0,L)   scored (Eq. 9-11); the k kept rows are read again (L2) -> [0,k)
//   rows [2L,..) -> [k+L, ..)
// Half of the wavefronts handle K rows, half V rows (as in the one-shot kernel).  Rows that
// are read for the last time and all stores use the streaming cache policy: the pass over 8192
// streams does not fit any cache, and the hints are worth 2.8 % (0.570 -> 0.554 ms per call).
// ---------------------------------------------------------------------------------
struct StepLds {
  int off_vK, off_vV, off_list, off_sel, off_pos, off_stat, off_stash, total;  // bytes
};
__host__ __device__ inline StepLds step_lds(int D, int L, int k, int nw, int rowbytes) {
  StepLds l;
  const int lp = (L + 3) & ~3, kp = (k + 3) & ~3;
  l.off_vK = 0;
  l.off_vV = lp * 4;
  l.off_list = 2 * lp * 4;
  l.off_sel = l.off_list + kp * 4;               // scratch of the workgroup-wide selection
  l.off_pos = l.off_sel + group_sel_bytes();     // positions of the (< 3L) tail rows
  l.off_stat = l.off_pos + 3 * lp * 4;           // [wave][mn|mx][D]
  l.off_stash = (l.off_stat + nw * 2 * D * 4 + 15) & ~15;  // [K|V][L][rowbytes]
  l.total = l.off_stash + 2 * L * rowbytes;
  return l;
}

// RAG: rows of fewer than LPR 16-byte slices (their size is then a run-time value).
template <typename ET, int LPR, bool RAG>
__global__ void __launch_bounds__(512, 4) decode_step_kernel(const AppendArgs a) {
  constexpr int VEC = ET::VEC, RPW = kWave / LPR, U = 4;
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int tid = threadIdx.x, nthreads = blockDim.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nw = nthreads >> 6, G = nw >> 1;
  const int units = RAG ? (a.D * a.esize) >> 4 : LPR;
  const int rowbytes = units * 16;
  const int L = a.L, k = a.k;
  const StepLds lay = step_lds(a.D, L, k, nw, rowbytes);
  float* vK = reinterpret_cast<float*>(lds + lay.off_vK);
  float* vV = reinterpret_cast<float*>(lds + lay.off_vV);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  uint32_t* selbuf = reinterpret_cast<uint32_t*>(lds + lay.off_sel);
  int32_t* ptail = reinterpret_cast<int32_t*>(lds + lay.off_pos);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);
  const bool l2 = a.variant == 2;        // Eq. 16: keys only, no reference statistics
  const bool group_sel = a.sel == kSelGroup && L <= nthreads;

  const int tensor = wave >= G ? 1 : 0;  // 0: K rows, 1: V rows
  const int gslot = wave - tensor * G;
  const int rl = lane / LPR, cl = lane % LPR;
  const bool live = !RAG || cl < units;
  const int clc = live ? cl : units - 1;  // a lane beyond the row's slices repeats the last one
  const int R = G * RPW, row0 = gslot * RPW + rl;
  const int n_iter = (L + R - 1) / R;
  const int64_t stream = blockIdx.x;
  const int64_t b = stream / a.H, h = stream % a.H;
  // tail row 0 of this wavefront's tensor, at this lane's 16-byte slice
  char* ct = (tensor ? a.V : a.K) + (stream * a.capacity + a.n_static) * rowbytes + clc * 16;
  const char* fresh = a.n_new > 0 ? (tensor ? a.V_new : a.K_new) + b * a.nsb + h * a.nsh + clc * 16 : ct;
  const int n_tail = (int)a.n_tail, n_all = (int)(a.n_tail + a.n_new);
  auto src = [&](int v) -> const char* {
    return v < n_tail ? ct + (int64_t)v * rowbytes : fresh + (int64_t)(v - n_tail) * a.nst;
  };
  float* myvar = tensor ? vV : vK;
  char* mystash = lds + lay.off_stash + (size_t)tensor * L * rowbytes + clc * 16;
  int32_t* pc = a.pos ? a.pos + stream * a.capacity + a.n_static : nullptr;
  const float inv_D = 1.0f / (float)a.D;
  const float inv_dof = 1.0f / (float)(a.D - a.ddof);

  for (int i = tid; i < k; i += nthreads) list[i] = 0;
  if (pc)
    for (int v = tid; v < n_all; v += nthreads)
      ptail[v] = v < n_tail ? pc[v] : (int32_t)(a.n_seen + (v - n_tail));

  // 0. the first PF steps of the chunk (all of it for L <= PF * R) are requested right away,
  // so that they travel together with the reference rows instead of after the first barrier
  constexpr int PF = 8;
  uint4 cq[PF];
  const bool scores_rows = !l2 || tensor == 0;   // Eq. 16 reads only the keys of the chunk
  if (scores_rows) {
#pragma unroll
    for (int u = 0; u < PF; ++u) {
      const int r = row0 + u * R;
      if (u < n_iter) cq[u] = ld16(src(r < L ? r : L - 1));
    }
  }

  // 1. reference chunk (tail rows [L,2L)): statistics, rows parked in LDS
  TStats<VEC> acc;
  acc.reset();
  for (int it = 0; it < n_iter; it += U) {
    uint4 q[U];
    int r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      r[u] = row0 + (it + u) * R;
      q[u] = ld16_last(src(L + (r[u] < L ? r[u] : L - 1)));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!l2) {
        float x[VEC];
        unpack<ET>(q[u], x);
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          acc.mn[j] = fminf(acc.mn[j], x[j]);
          acc.mx[j] = fmaxf(acc.mx[j], x[j]);
        }
      }
      if (r[u] < L) *reinterpret_cast<uint4*>(mystash + (size_t)r[u] * rowbytes) = q[u];
    }
  }
#pragma unroll
  for (int m = LPR; m < kWave; m <<= 1) {
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      acc.mn[j] = fminf(acc.mn[j], __shfl_xor(acc.mn[j], m));
      acc.mx[j] = fmaxf(acc.mx[j], __shfl_xor(acc.mx[j], m));
    }
  }
  if (rl == 0) {
    float* w = statbuf + (size_t)wave * 2 * a.D + clc * VEC;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      w[j] = acc.mn[j];
      w[a.D + j] = acc.mx[j];
    }
  }
  __syncthreads();
  for (int g = 0; g < G; ++g) {
    const float* rd = statbuf + (size_t)(tensor * G + g) * 2 * a.D + clc * VEC;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      acc.mn[j] = fminf(acc.mn[j], rd[j]);
      acc.mx[j] = fmaxf(acc.mx[j], rd[j + a.D]);
    }
  }
  TRef<VEC> ref;
  ref.from(acc, live);

  // 2. the chunk (tail rows [0,L)): channel variance of every token (Eq. 9-10), or, for
  // Eq. 16, minus the key norm (the V wavefronts then read nothing here)
  auto score_row = [&](const uint4& q, int r) __attribute__((always_inline)) {
    float x[VEC];
    unpack<ET>(q, x);
    float v;
    if (l2) {
      float ss = 0.f;
#pragma unroll
      for (int j = 0; j < VEC; ++j) ss = fmaf(x[j], x[j], ss);
      if (!live) ss = 0.f;
      v = -sqrtf(group_sum<LPR>(ss));
    } else {
      v = token_var<LPR, VEC>(x, ref.mn, ref.iv, ref.bias, inv_D, inv_dof, live);
    }
    if (cl == 0 && r < L) myvar[r] = v;
  };
  if (scores_rows) {
#pragma unroll
    for (int u = 0; u < PF; ++u)
      if (u < n_iter) score_row(cq[u], row0 + u * R);
    for (int it = PF; it < n_iter; it += U) {
      uint4 q[U];
      int r[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        r[u] = row0 + (it + u) * R;
        q[u] = ld16(src(r[u] < L ? r[u] : L - 1));
      }
#pragma unroll
      for (int u = 0; u < U; ++u) score_row(q[u], r[u]);
    }
  }
  // 2b. the rows behind the reference chunk (tail rows [2L, n_all)) are requested now and stored
  // at the end: their flight overlaps the selection.  (Reads of this stream's rows all precede
  // its first store except the kept rows, which are read before the barrier of step 3.)
  const int nrem = n_all - 2 * L;
  uint4 rq[PF];
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int r = u * R + row0;
    if (r < nrem) rq[u] = ld16_last(src(2 * L + r));
  }
  if (group_sel && l2) group_sel_clear(selbuf, tid, nthreads);
  __syncthreads();
  if (group_sel) {
    if (l2) group_topk(tid < L ? ordered_key(vK[tid]) : 0u, L, k, selbuf, list, nullptr, tid, nw);
    else group_score_select(vK, vV, L, k, true, nullptr, selbuf, list, nullptr, tid, nthreads);
  } else if (wave == 0) {
    if (l2) wave_topk_scores(vK, L, k, list, lane);
    else wave_score_select_lean(vK, vV, L, k, true, nullptr, list, nullptr, lane);
  }
  __syncthreads();

  // 3. kept rows -> [0,k).  A batch is loaded, the workgroup synchronises, the batch is
  // stored: destination <= source and later batches read rows above everything stored.
  constexpr int UB = 4;
  for (int s0 = 0; s0 < k; s0 += UB * R) {
    uint4 g[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int s = s0 + u * R + row0;
      if (s < k) g[u] = ld16_last(src((int)list[s]));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int s = s0 + u * R + row0;
      if (s < k) st16_out(ct + (int64_t)s * rowbytes, g[u]);
    }
  }
  // 4. the parked reference rows -> [k, k+L): they cover dead rows of the chunk and their own
  // old place only
  for (int r = row0; r < L; r += R)
    st16_out(ct + (int64_t)(k + r) * rowbytes, *reinterpret_cast<const uint4*>(mystash + (size_t)r * rowbytes));
  // 5. the rest of the tail, rows [2L, n_all) -> [k+L, ..): the first PF steps from the registers
  // (requested in 2b; their destinations lie below every row still to be read), what is left
  // batch by batch as in 3.
#pragma unroll
  for (int u = 0; u < PF; ++u) {
    const int r = u * R + row0;
    if (r < nrem) st16_out(ct + (int64_t)(k + L + r) * rowbytes, rq[u]);
  }
  for (int r0 = PF * R; r0 < nrem; r0 += UB * R) {
    uint4 g[UB];
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int r = r0 + u * R + row0;
      if (r < nrem) g[u] = ld16_last(src(2 * L + r));
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
#pragma unroll
    for (int u = 0; u < UB; ++u) {
      const int r = r0 + u * R + row0;
      if (r < nrem) st16_out(ct + (int64_t)(k + L + r) * rowbytes, g[u]);
    }
  }
  if (pc) {  // every position was read into LDS before the first barrier
    for (int s = tid; s < k; s += nthreads) pc[s] = ptail[list[s]];
    for (int i = tid; i < n_all - L; i += nthreads) pc[k + i] = ptail[L + i];
  }
}

// ---------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------
static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

bool fused_supported(int D, int esize, int64_t sb, int64_t sh, int64_t st, const void* K,
                     const void* V, const void* Ko, const void* Vo) {
  if (lanes_per_row(D, esize) == 0) return false;
  if ((sb | sh | st) & 15) return false;
  return aligned16(K) && aligned16(V) && aligned16(Ko) && aligned16(Vo);
}

size_t fused_lds_bytes(int D, int L, int k, int nwaves) {
  return (size_t)lds_layout(D, L, k, nwaves).total;
}

template <typename ET>
static hipError_t launch_append_t(const AppendArgs& a, int lpr, dim3 grid, dim3 block, size_t lds,
                                  hipStream_t s) {
  switch (lpr) {
    case 4: fused_append_kernel<ET, 4><<<grid, block, lds, s>>>(a); break;
    case 8: fused_append_kernel<ET, 8><<<grid, block, lds, s>>>(a); break;
    case 16: fused_append_kernel<ET, 16><<<grid, block, lds, s>>>(a); break;
    case 32: fused_append_kernel<ET, 32><<<grid, block, lds, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

// Largest LDS footprint of the single-round kernel: two workgroups share a CU.
constexpr size_t kStepMaxLds = 80 * 1024;

bool decode_step_supported(const AppendArgs& a) {
  const int lpr = lanes_per_row(a.D, a.esize);
  if (lpr == 0 || a.variant == 1 || a.rounds != 1 || a.n_seen < a.S) return false;
  return (size_t)step_lds(a.D, a.L, a.k, 8, row_units(a.D, a.esize) * 16).total <= kStepMaxLds;
}

template <typename KF>
static hipError_t launch_step_one(KF kernel, const AppendArgs& a, dim3 grid, dim3 block, size_t lds,
                                  hipStream_t s) {
  if (lds > 64 * 1024) {  // beyond the default dynamic LDS limit: opt in (idempotent)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  kernel<<<grid, block, lds, s>>>(a);
  return hipGetLastError();
}

template <typename ET>
static hipError_t launch_step_t(const AppendArgs& a, int lpr, dim3 grid, dim3 block, size_t lds,
                                hipStream_t s) {
  const bool rag = row_units(a.D, a.esize) != lpr;
  switch (lpr * 2 + (rag ? 1 : 0)) {
    case 8: return launch_step_one(decode_step_kernel<ET, 4, false>, a, grid, block, lds, s);
    case 9: return launch_step_one(decode_step_kernel<ET, 4, true>, a, grid, block, lds, s);
    case 16: return launch_step_one(decode_step_kernel<ET, 8, false>, a, grid, block, lds, s);
    case 17: return launch_step_one(decode_step_kernel<ET, 8, true>, a, grid, block, lds, s);
    case 32: return launch_step_one(decode_step_kernel<ET, 16, false>, a, grid, block, lds, s);
    case 33: return launch_step_one(decode_step_kernel<ET, 16, true>, a, grid, block, lds, s);
    case 64: return launch_step_one(decode_step_kernel<ET, 32, false>, a, grid, block, lds, s);
    case 65: return launch_step_one(decode_step_kernel<ET, 32, true>, a, grid, block, lds, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_decode_step(const AppendArgs& a, hipStream_t s) {
  const int lpr = lanes_per_row(a.D, a.esize);
  const int64_t streams = (int64_t)a.B * a.H;
  if (!decode_step_supported(a) || streams <= 0 || streams > 0x7fffffffLL) return hipErrorInvalidValue;
  if (a.n_tail + a.n_new < 2 * (int64_t)a.L || a.n_tail + a.n_new >= 3 * (int64_t)a.L)
    return hipErrorInvalidValue;
  const size_t lds = (size_t)step_lds(a.D, a.L, a.k, 8, row_units(a.D, a.esize) * 16).total;
  const dim3 grid((unsigned)streams), block(8 * kWave);
  if (a.esize == 4) return launch_step_t<F32>(a, lpr, grid, block, lds, s);
  return a.f16 ? launch_step_t<F16>(a, lpr, grid, block, lds, s)
               : launch_step_t<BF16>(a, lpr, grid, block, lds, s);
}

hipError_t launch_fused_append(const AppendArgs& a, hipStream_t s) {
  const int lpr = lanes_per_row(a.D, a.esize);
  const int64_t streams = (int64_t)a.B * a.H;
  if (lpr == 0 || streams <= 0 || streams > 0x7fffffffLL) return hipErrorInvalidValue;
  const size_t lds = fused_lds_bytes(a.D, a.L, a.k, a.nwaves);
  if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;
  const dim3 grid((unsigned)streams), block(a.nwaves * kWave);
  if (a.esize == 4) return launch_append_t<F32>(a, lpr, grid, block, lds, s);
  return a.f16 ? launch_append_t<F16>(a, lpr, grid, block, lds, s)
               : launch_append_t<BF16>(a, lpr, grid, block, lds, s);
}

}  // namespace lagkv
