// Tensor-split streaming LagKV kernel for gfx950: the one-shot pass for everything the
// register-resident kernel does not take (Eq. 16 scoring, lags other than 128, 256 or 512 rows,
// rows other than 256 bytes), and for any shape on request.
//
// A workgroup walks a segment of one stream backwards and scores chunk p with the
// statistics of chunk p+1 while folding chunk p's own min/max for chunk p-1, so every
// input byte is streamed once.  The first half of the wavefronts handles only K rows and
// the second half only V rows:
// a lane carries the statistics of ONE tensor, which halves the register footprint and
// lets 16 wavefronts share a CU (4 per SIMD) with eight 16-byte loads in flight each.
// The kept rows are re-read for the compaction right after the selection (measured: 1.24 to
// 1.29 times the algorithmic bytes cross the L2; the 256 MiB memory-side cache serves part of
// that second read of the chunks in flight, 2 workgroups per CU x 2 x L rows).
#include "lagkv_internal.hpp"
#include "lds_dma.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"
#include "wg_select.hpp"

#ifndef LAGKV_SPLIT_U
#define LAGKV_SPLIT_U 4      // rows in flight per lane
#endif
#ifndef LAGKV_SPLIT_UG
#define LAGKV_SPLIT_UG 8     // kept rows in flight per lane in the compaction
#endif
#ifndef LAGKV_SPLIT_DMA
#define LAGKV_SPLIT_DMA 1    // 1: asynchronous global->LDS row loads when the rows of a chunk divide evenly
#endif
#ifndef LAGKV_LOCAL_REV
#define LAGKV_LOCAL_REV 1     // LocalKV: second pass over a chunk in reverse row order
#endif
#ifndef LAGKV_SPLIT_WPE
#define LAGKV_SPLIT_WPE 4    // wavefronts per SIMD the register budget is set for
#endif

namespace lagkv {

struct SplitLds {
  int off_vK, off_vV, off_list, off_sel, off_stat, off_ring, total;  // bytes
};
__host__ __device__ inline SplitLds split_lds(int D, int L, int k, int nw, bool ring) {
  SplitLds l;
  const int lp = (L + 3) & ~3, kp = (k + 3) & ~3;
  l.off_vK = 0;
  l.off_vV = lp * 4;
  l.off_list = 2 * lp * 4;
  l.off_sel = l.off_list + kp * 4;              // scratch of the workgroup-wide selection
  l.off_stat = (l.off_sel + group_sel_bytes() + 15) & ~15;
  l.off_ring = (l.off_stat + nw * 2 * D * 4 + 1023) & ~1023;  // [wave][mn|mx][D], then the rings
  l.total = ring ? l.off_ring + nw * kRing * 1024 : l.off_stat + nw * 2 * D * 4;
  return l;
}

// EXACT: L is a multiple of the rows one step covers and the LDS ring fits: uniform row
// addressing and asynchronous loads.  EXACT=false serves any L through registers.
template <typename ET, int LPR, bool EXACT>
__global__ void __launch_bounds__(512, LAGKV_SPLIT_WPE) split_pass_kernel(const PassArgs a) {
  constexpr int VEC = ET::VEC;
  constexpr int RPW = kWave / LPR;
  constexpr int U = LAGKV_SPLIT_U;
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int nw = nthreads >> 6, G = nw >> 1;
  constexpr bool use_dma = EXACT && LAGKV_SPLIT_DMA;
  const SplitLds lay = split_lds(a.D, a.L, a.k, nw, use_dma);
  float* vK = reinterpret_cast<float*>(lds + lay.off_vK);
  float* vV = reinterpret_cast<float*>(lds + lay.off_vV);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  uint32_t* selbuf = reinterpret_cast<uint32_t*>(lds + lay.off_sel);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);

  const int tensor = wave >= G ? 1 : 0;  // 0: this wavefront handles K rows, 1: V rows
  const int gslot = wave - tensor * G;
  const int rl = lane / LPR, cl = lane % LPR;
  // rows of `units` 16-byte slices: a lane beyond them repeats the last slice (row_ops.hpp)
  const int units = (a.D * a.esize) >> 4;
  const bool live = cl < units;
  const int clc = live ? cl : units - 1;
  const int R = G * RPW;                  // rows of one tensor covered per step
  const int row0 = gslot * RPW + rl;
  const int L = a.L, k = a.k, S = a.S;
  const int n_iter = (L + R - 1) / R;
  const int64_t rowbytes = (int64_t)units * 16;
  const int64_t coff = (int64_t)clc * 16;

  const int64_t stream = stream_of(blockIdx.x / a.nseg, (int64_t)a.B * a.H, a.order);
  const int seg = blockIdx.x % a.nseg;
  const int64_t b = stream / a.H, h = stream % a.H;
  const char* kin = a.K + b * a.sb + h * a.sh;
  const char* vin = a.V + b * a.sb + h * a.sh;
  const char* tin = tensor ? vin : kin;
  const bool gather = a.K_out != nullptr;
  char* kout = gather ? a.K_out + stream * a.T_out * rowbytes : nullptr;
  char* vout = gather ? a.V_out + stream * a.T_out * rowbytes : nullptr;
  char* tout = tensor ? vout : kout;
  int32_t* iout = (gather && a.idx_out) ? a.idx_out + stream * a.T_out : nullptr;
  float* sout = a.scores ? a.scores + stream * a.n_s * L : nullptr;
  float* myvar = tensor ? vV : vK;
  const float inv_D = 1.0f / (float)a.D;
  const float inv_dof = 1.0f / (float)(a.D - a.ddof);
  const bool local = a.variant == 1;  // Eq. 14-15: statistics from the chunk itself

  for (int i = tid; i < k; i += nthreads) list[i] = 0;

  // sink rows and the sliding window (last full chunk + remainder) are plain copies
  if (gather && seg == 0 && S > 0) {
    copy_rows_kv<LPR>(kin, vin, a.st, kout, vout, rowbytes, S, units, tid, nthreads);
    if (iout)
      for (int i = tid; i < S; i += nthreads) iout[i] = i;
  }
  if (gather && seg == a.nseg - 1) {
    const int64_t w0 = S + a.n_s * L, o0 = S + a.n_s * k, nwin = a.T - w0;
    copy_rows_kv<LPR>(kin + w0 * a.st, vin + w0 * a.st, a.st, kout + o0 * rowbytes,
                      vout + o0 * rowbytes, rowbytes, nwin, units, tid, nthreads);
    if (iout)
      for (int64_t i = tid; i < nwin; i += nthreads) iout[o0 + i] = (int32_t)(w0 + i);
  }

  const int64_t p0 = (int64_t)seg * a.n_s / a.nseg;
  const int64_t p1 = (int64_t)(seg + 1) * a.n_s / a.nseg;

  TStats<VEC> acc;
  TRef<VEC> ref;

  // One pass over the L rows of this wavefront's tensor.  When L is a multiple of the
  // rows one step covers (the usual case) a row address is a wave-uniform base plus one
  // 32-bit lane offset, so no per-lane address arithmetic is needed; steps past the end
  // repeat the last step.  Otherwise rows past L repeat the last row, lane by lane.
  constexpr bool exact = EXACT;
  const uint32_t lane_off = (uint32_t)(row0 * a.st) + (uint32_t)clc * 16u;
  // consume U loaded rows whose first step is `it` (rows of steps past the end are skipped)
  auto consume = [&](const uint4 (&q)[U], const int (&r)[U], auto stats_tag, auto score_tag)
                     __attribute__((always_inline)) {
    constexpr bool STATS = decltype(stats_tag)::value, SCORE = decltype(score_tag)::value;
#pragma unroll
    for (int u = 0; u < U; u += 2) {
      float x0[VEC], x1[VEC];
      unpack<ET>(q[u], x0);
      unpack<ET>(q[u + 1], x1);
      if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          acc.mn[j] = fminf(fminf(acc.mn[j], x0[j]), x1[j]);
          acc.mx[j] = fmaxf(fmaxf(acc.mx[j], x0[j]), x1[j]);
        }
      }
      if constexpr (SCORE) {
        const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof, live);
        const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof, live);
        if (cl == 0) {
          if (r[u] < L) myvar[r[u]] = v0;
          if (r[u + 1] < L) myvar[r[u + 1]] = v1;
        }
      }
    }
  };
  // issue the loads of the U steps that start at step `it` of the chunk whose first row
  // is `row`
  auto issue = [&](uint4 (&q)[U], int (&r)[U], int64_t row, int it) __attribute__((always_inline)) {
    const char* ubase = tin + row * a.st;  // wave-uniform
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if constexpr (exact) {
        const int step = it + u < n_iter ? it + u : n_iter - 1;
        r[u] = it + u < n_iter ? row0 + step * R : L;  // L: nothing to store
        q[u] = ld16(ubase + (int64_t)step * R * a.st + lane_off);
      } else {
        r[u] = row0 + (it + u) * R;
        q[u] = ld16(ubase + coff + (int64_t)(r[u] < L ? r[u] : L - 1) * a.st);
      }
    }
  };
  // one pass over the L rows of this wavefront's tensor in the chunk whose first row is `row`
  auto scan_regs = [&](int64_t row, auto stats_tag, auto score_tag) __attribute__((always_inline)) {
    for (int it = 0; it < n_iter; it += U) {
      uint4 q[U];
      int r[U];
      issue(q, r, row, it);
      consume(q, r, stats_tag, score_tag);
    }
  };
  // The same pass with asynchronous loads: steps land in this wavefront's LDS ring and
  // are consumed two at a time, kRing-2 steps behind the loads.
  const uint32_t ring_lds = lds_offset(lds + lay.off_ring) + (uint32_t)wave * (kRing * 1024u);
  const uint32_t ring_lane = ring_lds + (uint32_t)lane * 16u;
  const uint32_t var_lds = lds_offset(myvar) + (uint32_t)row0 * 4u;
  // rev: walk the steps of the chunk from the last to the first (used for a second pass over a chunk,
  // whose most recently read rows are the ones still in the L2)
  auto scan_dma = [&](int64_t row, bool rev, auto stats_tag, auto score_tag) __attribute__((always_inline)) {
    constexpr bool STATS = decltype(stats_tag)::value, SCORE = decltype(score_tag)::value;
    const char* ubase = tin + row * a.st;  // wave-uniform
    auto phys = [&](int step) __attribute__((always_inline)) { return rev ? n_iter - 1 - step : step; };
    auto dma = [&](int step) __attribute__((always_inline)) {
      __builtin_amdgcn_global_load_lds((gptr_t)(ubase + (int64_t)phys(step) * R * a.st + lane_off),
                                       (lptr_t)(lds + lay.off_ring + (wave * kRing + step % kRing) * 1024),
                                       16, 0, 0);
    };
    auto pair = [&](int s, const u32x4& qa, const u32x4& qb) __attribute__((always_inline)) {
      float x0[VEC], x1[VEC];
      unpack<ET>(make_uint4(qa.x, qa.y, qa.z, qa.w), x0);
      unpack<ET>(make_uint4(qb.x, qb.y, qb.z, qb.w), x1);
      if constexpr (STATS) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          acc.mn[j] = fminf(fminf(acc.mn[j], x0[j]), x1[j]);
          acc.mx[j] = fmaxf(fmaxf(acc.mx[j], x0[j]), x1[j]);
        }
      }
      if constexpr (SCORE) {
        const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof, live);
        const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof, live);
        if (cl == 0) {
          lds_store_f32(var_lds + (uint32_t)(phys(s) * R) * 4u, v0);
          if (s + 1 < n_iter) lds_store_f32(var_lds + (uint32_t)(phys(s + 1) * R) * 4u, v1);
        }
      }
    };
    const int ahead = n_iter < kRing ? n_iter : kRing;
    for (int s = 0; s < ahead; ++s) dma(s);
    int s = 0;
    // steady state: steps s and s+1 have landed once at most kRing-2 loads are pending
    for (; s + kRing + 1 < n_iter; s += 2) {
      u32x4 qa, qb;
      lds_read_pair_after<kRing - 2>(qa, qb, ring_lane + (uint32_t)(s % kRing) * 1024u,
                                     ring_lane + (uint32_t)((s + 1) % kRing) * 1024u);
      dma(s + kRing);      // the two slots just read are free again
      dma(s + kRing + 1);
      pair(s, qa, qb);
    }
    // tail: everything has been issued; wait for all of it once
    for (; s < n_iter; s += 2) {
      u32x4 qa, qb;
      const int s1 = s + 1 < n_iter ? s + 1 : s;  // odd step count: the last step twice
      lds_read_pair_after<0>(qa, qb, ring_lane + (uint32_t)(s % kRing) * 1024u,
                             ring_lane + (uint32_t)(s1 % kRing) * 1024u);
      if (s + kRing < n_iter) dma(s + kRing);
      pair(s, qa, qb);
    }
    lds_drain();
  };
  auto scan = [&](int64_t row, bool rev, auto stats_tag, auto score_tag) __attribute__((always_inline)) {
    if constexpr (use_dma) scan_dma(row, rev, stats_tag, score_tag);
    else scan_regs(row, stats_tag, score_tag);
  };
  // combine acc over the row groups of a wavefront and the wavefronts of the tensor
  // group; one __syncthreads inside (it also publishes the variances)
  auto fold = [&]() __attribute__((always_inline)) {
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        acc.mn[j] = fminf(acc.mn[j], __shfl_xor(acc.mn[j], m));
        acc.mx[j] = fmaxf(acc.mx[j], __shfl_xor(acc.mx[j], m));
      }
    }
    if (G > 1) {
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
    } else {
      __syncthreads();
    }
  };
  using T_ = std::true_type;
  using F_ = std::false_type;

  auto compact = [&](int64_t p) __attribute__((always_inline)) {
    const char* src = tin + (S + p * L) * a.st + coff;
    char* dst = tout + (S + p * k) * rowbytes + coff;
    constexpr int UG = LAGKV_SPLIT_UG;
    for (int s0 = row0; s0 < k; s0 += UG * R) {
      uint4 g[UG];
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const int s = s0 + u * R;
        g[u] = ld16_last(src + (int64_t)list[s < k ? s : s0] * a.st);
      }
#pragma unroll
      for (int u = 0; u < UG; ++u) {
        const int s = s0 + u * R;
        if (s < k) st16_out(dst + (int64_t)s * rowbytes, g[u]);
      }
    }
    if (iout)
      for (int i = tid; i < k; i += nthreads)
        iout[S + p * k + i] = (int32_t)(S + p * L + list[i]);
  };

  // Eq. 10-11 and the top-k of chunk p from the variances in vK / vV (visible to all).
  // Selection by all wavefronts needs one token per thread; otherwise one wavefront does
  // it, a different one for every chunk so that the work is spread over the SIMDs.
  // Chunks longer than 512 tokens go to all wavefronts by default (several tokens per thread):
  // one wavefront would need the chunk's keys in LDS and a pass over them per key bit.
  const int eg = (L + nthreads - 1) / nthreads;  // tokens per thread
  const bool group_sel = (a.sel == kSelGroup || (a.sel == kSelAuto && L > 512)) && eg <= kGroupSelMaxKeys;
  auto select = [&](int64_t p) __attribute__((always_inline)) {
    float* g = sout ? sout + p * L : nullptr;
    if (group_sel) {
      if (eg == 1) group_score_select(vK, vV, L, k, gather, g, selbuf, list, nullptr, tid, nthreads);
      else if (eg == 2) group_score_select_multi<2>(vK, vV, L, k, gather, g, selbuf, list, tid, nthreads);
      else group_score_select_multi<4>(vK, vV, L, k, gather, g, selbuf, list, tid, nthreads);
    } else if (wave == (a.sel == kSelWave ? (int)(p % nw) : 0)) {
      wave_score_select_lean(vK, vV, L, k, gather, g, list, nullptr, lane);
    }
  };

  if (a.variant == 2) {
    // Eq. 16: score = -||K_t||_2.  No reference and no softmax; V is read only where it is kept.
    // All wavefronts share the K rows of the chunk.
    const int R2 = nw * RPW, r2 = wave * RPW + rl;
    const int n_iter2 = (L + R2 - 1) / R2;
    for (int64_t p = p1 - 1; p >= p0; --p) {
      const char* cb = kin + (S + p * L) * a.st + coff;
      for (int it = 0; it < n_iter2; it += U) {
        uint4 q[U];
        int r[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          r[u] = r2 + (it + u) * R2;
          q[u] = ld16(cb + (int64_t)(r[u] < L ? r[u] : L - 1) * a.st);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
          float x[VEC];
          unpack<ET>(q[u], x);
          float ss = 0.f;
#pragma unroll
          for (int j = 0; j < VEC; ++j) ss = fmaf(x[j], x[j], ss);
          if (!live) ss = 0.f;
          ss = group_sum<LPR>(ss);
          if (cl == 0 && r[u] < L) vK[r[u]] = -sqrtf(ss);
        }
      }
      if (group_sel) group_sel_clear(selbuf, tid, nthreads);
      __syncthreads();
      if (sout)
        for (int i = tid; i < L; i += nthreads) sout[p * L + i] = vK[i];
      if (group_sel) {
        if (eg == 1) {
          group_topk(tid < L ? ordered_key(vK[tid]) : 0u, L, k, selbuf, list, nullptr, tid, nw);
        } else {
          uint32_t keys[kGroupSelMaxKeys];
#pragma unroll
          for (int e = 0; e < kGroupSelMaxKeys; ++e) {
            const int t = e * nthreads + tid;
            keys[e] = t < L ? ordered_key(vK[t]) : 0u;
          }
          group_topk_multi<kGroupSelMaxKeys>(keys, L, k, selbuf, list, tid, nthreads);
        }
      } else if (wave == (a.sel == kSelWave ? (int)(p % nw) : 0)) {
        wave_topk_scores(vK, L, k, list, lane);
      }
      __syncthreads();
      if (gather) compact(p);
    }
    return;
  }

  if (local) {
    for (int64_t p = p1 - 1; p >= p0; --p) {
      const int64_t crow = S + p * L;
      acc.reset();
      scan(crow, false, T_{}, F_{});
      fold();
      ref.from(acc, live);
      scan(crow, LAGKV_LOCAL_REV != 0, F_{}, T_{});
      __syncthreads();
      select(p);
      __syncthreads();
      if (gather) compact(p);
    }
    return;
  }

  // statistics of the chunk after the segment: the first reference
  acc.reset();
  scan(S + p1 * L, false, T_{}, F_{});
  fold();
  ref.from(acc, live);
  __syncthreads();  // statbuf is rewritten by the next fold
  for (int64_t p = p1 - 1; p >= p0; --p) {
    acc.reset();
    scan(S + p * L, false, T_{}, T_{});
    fold();  // barrier inside: the variances are visible
    ref.from(acc, live);  // chunk p is the reference of chunk p-1 (done before the selection so
                    // that the running statistics are dead across it: fewer live registers)
    select(p);
    __syncthreads();
    if (gather) compact(p);
  }
}

// ------------------------------------------------------------------------ host side
// A workgroup may use up to 80 KiB of LDS so that two of them share the 160 KiB of a CU.
constexpr size_t kSplitMaxLds = 80 * 1024;

static bool split_exact(int lpr, int L, int nwaves) {
  return L % ((nwaves / 2) * (kWave / lpr)) == 0;
}
// The asynchronous-load variant needs the ring as well; if that does not fit, the
// register variant (which serves any L) is used.
static bool split_uses_ring(int D, int L, int k, int nwaves, int lpr) {
  return LAGKV_SPLIT_DMA && split_exact(lpr, L, nwaves) &&
         (size_t)split_lds(D, L, k, nwaves, true).total <= kSplitMaxLds;
}

size_t split_lds_bytes(int D, int esize, int L, int k, int nwaves) {
  const int lpr = lanes_per_row(D, esize);
  if (lpr == 0) return (size_t)-1;
  return (size_t)split_lds(D, L, k, nwaves, split_uses_ring(D, L, k, nwaves, lpr)).total;
}

template <typename K>
static hipError_t launch_one(K kernel, const PassArgs& a, dim3 grid, dim3 block, size_t lds,
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
static hipError_t launch_split_t(const PassArgs& a, int lpr, bool ring, dim3 grid, dim3 block,
                                 size_t lds, hipStream_t s) {
  switch (lpr * 2 + (ring ? 1 : 0)) {
    case 8: return launch_one(split_pass_kernel<ET, 4, false>, a, grid, block, lds, s);
    case 9: return launch_one(split_pass_kernel<ET, 4, true>, a, grid, block, lds, s);
    case 16: return launch_one(split_pass_kernel<ET, 8, false>, a, grid, block, lds, s);
    case 17: return launch_one(split_pass_kernel<ET, 8, true>, a, grid, block, lds, s);
    case 32: return launch_one(split_pass_kernel<ET, 16, false>, a, grid, block, lds, s);
    case 33: return launch_one(split_pass_kernel<ET, 16, true>, a, grid, block, lds, s);
    case 64: return launch_one(split_pass_kernel<ET, 32, false>, a, grid, block, lds, s);
    case 65: return launch_one(split_pass_kernel<ET, 32, true>, a, grid, block, lds, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_split_pass(const PassArgs& a, hipStream_t s) {
  const int lpr = lanes_per_row(a.D, a.esize);
  const int64_t nblocks = (int64_t)a.B * a.H * a.nseg;
  if (lpr == 0 || nblocks <= 0 || nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  if (a.nwaves != 2 && a.nwaves != 4 && a.nwaves != 8) return hipErrorInvalidValue;
  // per-lane input offsets are 32 bit: the rows of one step must lie within 2 GiB
  if (a.st * (int64_t)((a.nwaves / 2) * (kWave / lpr)) >= (1LL << 31)) return hipErrorInvalidValue;
  const bool ring = split_uses_ring(a.D, a.L, a.k, a.nwaves, lpr);
  const size_t lds = (size_t)split_lds(a.D, a.L, a.k, a.nwaves, ring).total;
  if (lds > kSplitMaxLds) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblocks), block(a.nwaves * kWave);
  if (a.esize == 4) return launch_split_t<F32>(a, lpr, ring, grid, block, lds, s);
  return a.f16 ? launch_split_t<F16>(a, lpr, ring, grid, block, lds, s)
               : launch_split_t<BF16>(a, lpr, ring, grid, block, lds, s);
}

}  // namespace lagkv
