// Workgroup-wide chunk softmax (Eq. 10-11) and top-k for the LagKV kernels (gfx950): every
// wavefront of the workgroup takes part, one token per thread.  The single-wavefront
// form in wave_ops.hpp leaves the other wavefronts of the workgroup waiting for up to a
// quarter of a chunk's time; here the k-th largest score is found with four 8-bit digit
// histograms in LDS (one barrier per digit) instead of one ballot round per key bit.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lds_dma.hpp"
#include "wave_ops.hpp"

namespace lagkv {

// How the per-chunk selection is carried out (PassArgs::sel / AppendArgs::sel; the values
// of LAGKV_SELECT_* in the public header):
//   kSelAuto   the kernel's default
//   kSelWave   one wavefront (wave_ops.hpp); the wavefront rotates from chunk to chunk so
//              that the work does not always land on the same SIMD
//   kSelGroup  all wavefronts (this file) when the chunk has at most one token per thread
enum { kSelAuto = 0, kSelWave = 1, kSelGroup = 2 };

// LDS words: 4 histograms of 256 16-bit bins (a bin counts at most 512 keys), partial
// reductions, counts
constexpr int kGroupSelHist = 4 * 128;
constexpr int kGroupSelWords = kGroupSelHist + 64;

__host__ __device__ inline int group_sel_bytes() { return kGroupSelWords * 4; }

// Sum over lanes >= the calling lane (inclusive), all 64 lanes active.
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    const uint32_t o = (uint32_t)__shfl_down((int)v, d);
    if (lane + d < kWave) v += o;
  }
  return v;
}

__device__ __forceinline__ uint32_t rl_u(uint32_t v, int l) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}

// Top-k of one key per thread (0 = no token), by all threads of the workgroup.
//   key      ordered key of token `tid` (0 when tid >= L)
//   scratch  kGroupSelWords words of LDS; the histograms must be ZERO on entry and are
//            left dirty (the caller zeroes them before the next use, behind a barrier)
//   list     receives the k kept positions, ascending; slotmap (optional) [L]: output slot
//            of a kept token, -1 otherwise.  Visible to other wavefronts after the
//            caller's next barrier.
// Order: key descending, position ascending (ties go to the lower position).
// Contains five barriers; every thread of the workgroup must call it.
__device__ __forceinline__ void group_topk(uint32_t key, int L, int k, uint32_t* scratch,
                                           uint32_t* list, int32_t* slotmap, int tid, int nw) {
  const int lane = tid & 63, wave = tid >> 6;
  const bool live = tid < L;
  uint32_t* cnt = scratch + kGroupSelHist + 32;
  uint32_t prefix = 0;
  int need = k;
#pragma unroll
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    uint32_t* h = scratch + round * 128;  // bin d: half (d & 1) of word d >> 1
    const bool in = live && (round == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)));
    // wavefront-aggregated count when a whole wavefront shares the digit (the usual case
    // for the leading digits of scores that all lie within a few binades)
    const uint32_t digit = (key >> shift) & 255u;
    const uint64_t inm = __ballot(in);
    if (inm) {
      const int first = __builtin_ctzll(inm);
      const uint32_t d0 = rl_u(digit, first);
      const uint64_t same = __ballot(in && digit == d0);
      if (same == inm) {
        if (lane == first) atomicAdd(&h[d0 >> 1], (uint32_t)__popcll(inm) << ((d0 & 1u) * 16u));
      } else if (in) {
        atomicAdd(&h[digit >> 1], 1u << ((digit & 1u) * 16u));
      }
    }
    __syncthreads();
    // every wavefront scans the 256 bins: lane l owns bins 4l .. 4l+3
    const uint2 cw = *reinterpret_cast<const uint2*>(&h[lane * 2]);
    const uint4 c = make_uint4(cw.x & 0xffffu, cw.x >> 16, cw.y & 0xffffu, cw.y >> 16);
    const uint32_t tot = c.x + c.y + c.z + c.w;
    const uint32_t suf = wave_suffix_sum(tot, lane);
    const uint64_t reach = __ballot(suf >= (uint32_t)need);  // not empty: the bins hold >= need keys
    const int ls = 63 - __builtin_clzll(reach);              // highest lane whose suffix reaches need
    const uint32_t c0 = rl_u(c.x, ls), c1 = rl_u(c.y, ls), c2 = rl_u(c.z, ls), c3 = rl_u(c.w, ls);
    uint32_t above = rl_u(suf, ls) - (c0 + c1 + c2 + c3);    // keys in the bins of higher lanes
    int d;
    if (above + c3 >= (uint32_t)need) {
      d = 3;
    } else if (above + c3 + c2 >= (uint32_t)need) {
      d = 2;
      above += c3;
    } else if (above + c3 + c2 + c1 >= (uint32_t)need) {
      d = 1;
      above += c3 + c2;
    } else {
      d = 0;
      above += c3 + c2 + c1;
    }
    prefix |= (uint32_t)(ls * 4 + d) << shift;
    need -= (int)above;  // keys strictly above the chosen bin are all kept
  }
  // prefix is the k-th largest key; `need` of the keys equal to it are admitted, lowest positions first
  const bool gt = live && key > prefix, eq = live && key == prefix;
  const uint64_t mg = __ballot(gt), me = __ballot(eq);
  if (lane == 0) {
    cnt[wave * 2] = (uint32_t)__popcll(mg);
    cnt[wave * 2 + 1] = (uint32_t)__popcll(me);
  }
  __syncthreads();
  int base = 0, eq_before = 0;
  for (int w = 0; w < wave; ++w) {
    const int g = (int)cnt[w * 2], e = (int)cnt[w * 2 + 1];
    const int room = need - eq_before;
    base += g + (e < room ? e : (room > 0 ? room : 0));
    eq_before += e;
  }
  const bool keep = gt || (eq && (eq_before + prefix_popc(me) < need));
  const uint64_t mk = __ballot(keep);
  const int slot = base + prefix_popc(mk);
  if (keep) list[slot] = (uint32_t)tid;
  if (slotmap && live) slotmap[tid] = keep ? slot : -1;
  (void)nw;
}

// Zero the histograms of `scratch`; a barrier must follow before group_topk adds to them.
__device__ __forceinline__ void group_sel_clear(uint32_t* scratch, int tid, int nthreads) {
  for (int i = tid; i < kGroupSelHist; i += nthreads) scratch[i] = 0u;
}

// Chunk softmax of K and V, their sum (Eq. 10-11) and, if asked, the top-k, by ALL
// wavefronts of the workgroup; needs L <= blockDim.x.  On entry vK[t], vV[t] (LDS) hold the
// channel VARIANCE of token t, visible to every thread; on return vK[t] holds the final
// score (written by thread t).  Every thread of the workgroup must call it; it contains
// seven barriers (two for the softmax, five in group_topk) and the list is visible after
// the caller's next one.
__device__ __forceinline__ void group_score_select(float* vK, const float* vV, int L, int k,
                                                   bool do_select, float* gout, uint32_t* scratch,
                                                   uint32_t* list, int32_t* slotmap, int tid,
                                                   int nthreads) {
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const bool live = tid < L;
  float* red = reinterpret_cast<float*>(scratch + kGroupSelHist);  // [nw][2] maxima, then [nw][2] sums
  group_sel_clear(scratch, tid, nthreads);
  const float sK = live ? std_of_var(vK[tid]) : -INFINITY;
  const float sV = live ? std_of_var(vV[tid]) : -INFINITY;
  float mK = wave_max(sK), mV = wave_max(sV);
  if (lane == 0) {
    red[wave * 2] = mK;
    red[wave * 2 + 1] = mV;
  }
  __syncthreads();
  for (int w = 0; w < nw; ++w) {
    mK = fmaxf(mK, red[w * 2]);
    mV = fmaxf(mV, red[w * 2 + 1]);
  }
  const float eK = live ? __expf(sK - mK) : 0.f;
  const float eV = live ? __expf(sV - mV) : 0.f;
  const float aK = wave_sum(eK), aV = wave_sum(eV);
  if (lane == 0) {
    red[16 + wave * 2] = aK;
    red[16 + wave * 2 + 1] = aV;
  }
  __syncthreads();
  float tK = 0.f, tV = 0.f;
  for (int w = 0; w < nw; ++w) {  // the same order in every thread: one value for the whole chunk
    tK += red[16 + w * 2];
    tV += red[16 + w * 2 + 1];
  }
  const float s = eK * (1.0f / tK) + eV * (1.0f / tV);
  if (live) {
    vK[tid] = s;
    // (a store the compiler does not know of, hence does not wait for at the barriers below)
    if (gout) st4_out_at(gout, (uint32_t)tid * 4u, __float_as_uint(s));
  }
  if (do_select) group_topk(live ? ordered_key(s) : 0u, L, k, scratch, list, slotmap, tid, nw);
}

}  // namespace lagkv
