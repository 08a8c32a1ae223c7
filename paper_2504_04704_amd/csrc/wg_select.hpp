// Workgroup-wide chunk softmax (Eq. 10-11) and top-k for the LagKV kernels (gfx950): every
// wavefront of the workgroup takes part, one token per thread.  The single-wavefront
// form in wave_ops.hpp leaves the other wavefronts of the workgroup waiting for up to a
// quarter of a chunk's time; here the k-th largest score is found with up to four 8-bit
// digit histograms in LDS (one barrier per digit) instead of one ballot round per key bit.
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
constexpr int kGroupSelMaxKeys = 4;   // keys per thread of the multi-key forms (chunks of up to 4 x threads)
constexpr int kGroupSelWords = kGroupSelHist + 64 + kGroupSelMaxKeys * 8 * 2;
// word offset of the multi-key forms' counts: [key slab][wavefront][greater | equal]
constexpr int kGroupSelCountsMulti = kGroupSelHist + 64;
// word offset (in the scratch) of the per-wavefront maxima a caller may supply, see
// group_score_select<true>
constexpr int kGroupSelPremax = kGroupSelHist + 48;

__host__ __device__ inline int group_sel_bytes() { return kGroupSelWords * 4; }

// Sum over lanes >= the calling lane (inclusive), all 64 lanes active: four shifted adds
// inside each row of 16 lanes (row_shl:n gives lane i the value of lane i + n, zero past
// the end of the row), then the totals of the rows above through scalar registers.
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shl0(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xf, 0xf, true);
}
__device__ __forceinline__ uint32_t rl_u(uint32_t v, int l) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, l);
}
__device__ __forceinline__ uint32_t wave_suffix_sum(uint32_t v, int lane) {
  v += dpp_shl0<0x101>(v);
  v += dpp_shl0<0x102>(v);
  v += dpp_shl0<0x104>(v);
  v += dpp_shl0<0x108>(v);
  const uint32_t t1 = rl_u(v, 16), t2 = rl_u(v, 32), t3 = rl_u(v, 48);
  const uint32_t up = lane < 16 ? t1 + t2 + t3 : lane < 32 ? t2 + t3 : lane < 48 ? t3 : 0u;
  return v + up;
}

constexpr int kGroupSelMaxWaves = 8;

// Top-k of one key per thread (0 = no token), by all threads of the workgroup (at most
// kGroupSelMaxWaves wavefronts).
//   key      ordered key of token `tid` (0 when tid >= L)
//   scratch  kGroupSelWords words of LDS; the histograms must be ZERO on entry and are
//            left dirty (the caller zeroes them before the next use, behind a barrier)
//   list     receives the k kept positions, ascending; slotmap (optional) [L]: output slot
//            of a kept token, -1 otherwise.  Visible to other wavefronts after the
//            caller's next barrier.
//   pos_out  (optional, global memory) [k]: receives pos0 + position of the kept tokens,
//            ascending, stored from assembly like the kernels' other outputs
// Order: key descending, position ascending (ties go to the lower position).
// One barrier per digit (the digits stop as soon as the bin of the k-th key is taken
// whole, which every wavefront sees alike) and one for the counts; every thread of the
// workgroup must call it.
__device__ __forceinline__ void group_topk(uint32_t key, int L, int k, uint32_t* scratch,
                                           uint32_t* list, int32_t* slotmap, int tid, int nw,
                                           int32_t* pos_out = nullptr, uint32_t pos0 = 0) {
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const bool live = tid < L;
  uint32_t* cnt = scratch + kGroupSelHist + 32;  // [kGroupSelMaxWaves][2], 16-byte aligned
  uint32_t prefix = 0;
  int need = k;
  bool whole = false;  // the chosen bin is kept whole: keys >= prefix are the answer
#pragma unroll
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    uint32_t* h = scratch + round * 128;  // bin d: half (d & 1) of word d >> 1
    const bool in = live && (round == 0 || (key >> (shift + 8)) == (prefix >> (shift + 8)));
    const uint32_t digit = (key >> shift) & 255u;
    if (round == 0) {
      // wavefront-aggregated count when a whole wavefront shares the leading digit (the
      // usual case for scores that all lie within a few binades)
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
    } else if (in) {
      atomicAdd(&h[digit >> 1], 1u << ((digit & 1u) * 16u));
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
    uint32_t cd;
    if (above + c3 >= (uint32_t)need) {
      d = 3;
      cd = c3;
    } else if (above + c3 + c2 >= (uint32_t)need) {
      d = 2;
      cd = c2;
      above += c3;
    } else if (above + c3 + c2 + c1 >= (uint32_t)need) {
      d = 1;
      cd = c1;
      above += c3 + c2;
    } else {
      d = 0;
      cd = c0;
      above += c3 + c2 + c1;
    }
    prefix |= (uint32_t)(ls * 4 + d) << shift;
    need -= (int)above;  // keys strictly above the chosen bin are all kept
    if ((int)cd == need) {  // ... and so is the whole bin: no key below `prefix` is needed
      whole = true;
      break;
    }
  }
  // Otherwise prefix is the k-th largest key; `need` of the keys equal to it are admitted,
  // lowest positions first.
  const bool gt = live && (whole ? key >= prefix : key > prefix);
  const bool eq = live && !whole && key == prefix;
  const uint64_t mg = __ballot(gt), me = __ballot(eq);
  if (lane == 0) {
    cnt[wave * 2] = (uint32_t)__popcll(mg);
    cnt[wave * 2 + 1] = (uint32_t)__popcll(me);
  }
  __syncthreads();
  uint4 cq[kGroupSelMaxWaves / 2];  // all counts at once (entries of absent wavefronts are not used)
#pragma unroll
  for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) cq[i] = reinterpret_cast<const uint4*>(cnt)[i];
  int base = 0, eq_before = 0;
#pragma unroll
  for (int w = 0; w < kGroupSelMaxWaves - 1; ++w) {
    if (w < wave) {
      const int g = (int)((w & 1) ? cq[w >> 1].z : cq[w >> 1].x);
      const int e = (int)((w & 1) ? cq[w >> 1].w : cq[w >> 1].y);
      const int room = need - eq_before;
      base += g + (e < room ? e : (room > 0 ? room : 0));
      eq_before += e;
    }
  }
  const bool keep = gt || (eq && (eq_before + prefix_popc(me) < need));
  const uint64_t mk = __ballot(keep);
  const int slot = base + prefix_popc(mk);
  if (keep) {
    list[slot] = (uint32_t)tid;
    if (pos_out) st4_out_at(pos_out, (uint32_t)slot * 4u, pos0 + (uint32_t)tid);
  }
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
// two barriers for the softmax (one with PREMAX) and those of group_topk; the list is
// visible after the caller's next one.
// PREMAX: the caller has already left upper bounds of the variances in the scratch, words
// kGroupSelPremax + w for w < nw, visible to every thread: the first nw/2 bound the K
// variances, the others the V variances (any bound at least as large as every variance
// serves: the softmax does not depend on the shift, which is only there against overflow).
template <bool PREMAX = false>
__device__ __forceinline__ void group_score_select(float* vK, const float* vV, int L, int k,
                                                   bool do_select, float* gout, uint32_t* scratch,
                                                   uint32_t* list, int32_t* slotmap, int tid,
                                                   int nthreads, int32_t* pos_out = nullptr,
                                                   uint32_t pos0 = 0) {
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  const bool live = tid < L;
  float* red = reinterpret_cast<float*>(scratch + kGroupSelHist);  // [nw][2] maxima, then [nw][2] sums
  group_sel_clear(scratch, tid, nthreads);
  const float sK = live ? std_of_var(vK[tid]) : -INFINITY;
  const float sV = live ? std_of_var(vV[tid]) : -INFINITY;
  float mK, mV;
  if constexpr (PREMAX) {
    const float* pm = reinterpret_cast<const float*>(scratch + kGroupSelPremax);
    float4 r[kGroupSelMaxWaves / 4];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 4; ++i) r[i] = reinterpret_cast<const float4*>(pm)[i];
    const float* rf = reinterpret_cast<const float*>(r);
    float bK = 0.f, bV = 0.f;  // variances are >= 0
#pragma unroll
    for (int w = 0; w < kGroupSelMaxWaves; ++w) {
      if (w < nw / 2) bK = fmaxf(bK, rf[w]);
      else if (w < nw) bV = fmaxf(bV, rf[w]);
    }
    mK = std_of_var(bK);
    mV = std_of_var(bV);
  } else {
    mK = wave_max(sK);
    mV = wave_max(sV);
    if (lane == 0) {
      red[wave * 2] = mK;
      red[wave * 2 + 1] = mV;
    }
    __syncthreads();
    float4 r[kGroupSelMaxWaves / 2];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) r[i] = reinterpret_cast<const float4*>(red)[i];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) {
      if (2 * i < nw) {
        mK = fmaxf(mK, r[i].x);
        mV = fmaxf(mV, r[i].y);
      }
      if (2 * i + 1 < nw) {
        mK = fmaxf(mK, r[i].z);
        mV = fmaxf(mV, r[i].w);
      }
    }
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
  {
    float4 r[kGroupSelMaxWaves / 2];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) r[i] = reinterpret_cast<const float4*>(red + 16)[i];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) {  // the same order in every thread: one value for the whole chunk
      if (2 * i < nw) {
        tK += r[i].x;
        tV += r[i].y;
      }
      if (2 * i + 1 < nw) {
        tK += r[i].z;
        tV += r[i].w;
      }
    }
  }
  const float s = eK * fast_rcp(tK) + eV * fast_rcp(tV);
  if (live) {
    vK[tid] = s;
    // (a store the compiler does not know of, hence does not wait for at the barriers below)
    if (gout) st4_out_at(gout, (uint32_t)tid * 4u, __float_as_uint(s));
  }
  if (do_select) group_topk(live ? ordered_key(s) : 0u, L, k, scratch, list, slotmap, tid, nw, pos_out, pos0);
}

// ---- chunks longer than the workgroup: EG tokens per thread ----------------------------
// Token e * nthreads + tid is key e of thread tid (so that position order is (e, wavefront,
// lane) order).  Same algorithm, same scratch (histograms ZERO on entry), same barriers.
template <int EG>
__device__ __forceinline__ void group_topk_multi(const uint32_t (&key)[EG], int L, int k, uint32_t* scratch,
                                                 uint32_t* list, int tid, int nthreads,
                                                 int32_t* pos_out = nullptr, uint32_t pos0 = 0) {
  static_assert(EG >= 1 && EG <= kGroupSelMaxKeys, "keys per thread");
  const int lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), nw = nthreads >> 6;
  uint32_t* cnt = scratch + kGroupSelCountsMulti;
  bool live[EG];
#pragma unroll
  for (int e = 0; e < EG; ++e) live[e] = e * nthreads + tid < L;
  uint32_t prefix = 0;
  int need = k;
  bool whole = false;
#pragma unroll
  for (int round = 0; round < 4; ++round) {
    const int shift = 24 - 8 * round;
    uint32_t* h = scratch + round * 128;
#pragma unroll
    for (int e = 0; e < EG; ++e) {
      const bool in = live[e] && (round == 0 || (key[e] >> (shift + 8)) == (prefix >> (shift + 8)));
      const uint32_t digit = (key[e] >> shift) & 255u;
      if (round == 0) {
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
      } else if (in) {
        atomicAdd(&h[digit >> 1], 1u << ((digit & 1u) * 16u));
      }
    }
    __syncthreads();
    const uint2 cw = *reinterpret_cast<const uint2*>(&h[lane * 2]);
    const uint4 c = make_uint4(cw.x & 0xffffu, cw.x >> 16, cw.y & 0xffffu, cw.y >> 16);
    const uint32_t tot = c.x + c.y + c.z + c.w;
    const uint32_t suf = wave_suffix_sum(tot, lane);
    const uint64_t reach = __ballot(suf >= (uint32_t)need);
    const int ls = 63 - __builtin_clzll(reach);
    const uint32_t c0 = rl_u(c.x, ls), c1 = rl_u(c.y, ls), c2 = rl_u(c.z, ls), c3 = rl_u(c.w, ls);
    uint32_t above = rl_u(suf, ls) - (c0 + c1 + c2 + c3);
    int d;
    uint32_t cd;
    if (above + c3 >= (uint32_t)need) {
      d = 3;
      cd = c3;
    } else if (above + c3 + c2 >= (uint32_t)need) {
      d = 2;
      cd = c2;
      above += c3;
    } else if (above + c3 + c2 + c1 >= (uint32_t)need) {
      d = 1;
      cd = c1;
      above += c3 + c2;
    } else {
      d = 0;
      cd = c0;
      above += c3 + c2 + c1;
    }
    prefix |= (uint32_t)(ls * 4 + d) << shift;
    need -= (int)above;
    if ((int)cd == need) {
      whole = true;
      break;
    }
  }
  bool gt[EG], eq[EG];
  uint64_t me[EG];
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    gt[e] = live[e] && (whole ? key[e] >= prefix : key[e] > prefix);
    eq[e] = live[e] && !whole && key[e] == prefix;
    const uint64_t mg = __ballot(gt[e]);
    me[e] = __ballot(eq[e]);
    if (lane == 0) {
      cnt[(e * kGroupSelMaxWaves + wave) * 2] = (uint32_t)__popcll(mg);
      cnt[(e * kGroupSelMaxWaves + wave) * 2 + 1] = (uint32_t)__popcll(me[e]);
    }
  }
  __syncthreads();
  // kept tokens before each of this thread's keys, in position order (slab, wavefront, lane)
  int base = 0, eq_before = 0;
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    uint4 cq[kGroupSelMaxWaves / 2];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i)
      cq[i] = reinterpret_cast<const uint4*>(cnt + e * kGroupSelMaxWaves * 2)[i];
    int base_e = base, eqb_e = eq_before;  // ... before this wavefront's part of slab e
#pragma unroll
    for (int w = 0; w < kGroupSelMaxWaves; ++w) {
      if (w < nw) {
        const int g = (int)((w & 1) ? cq[w >> 1].z : cq[w >> 1].x);
        const int q = (int)((w & 1) ? cq[w >> 1].w : cq[w >> 1].y);
        const int room = need - eq_before;
        const int add = g + (q < room ? q : (room > 0 ? room : 0));
        base += add;
        eq_before += q;
        if (w < wave) {
          base_e = base;
          eqb_e = eq_before;
        }
      }
    }
    const bool keep = gt[e] || (eq[e] && (eqb_e + prefix_popc(me[e]) < need));
    const uint64_t mk = __ballot(keep);
    const int slot = base_e + prefix_popc(mk);
    if (keep) {
      const uint32_t t = (uint32_t)(e * nthreads + tid);
      list[slot] = t;
      if (pos_out) st4_out_at(pos_out, (uint32_t)slot * 4u, pos0 + t);
    }
  }
}

// Chunk softmax of K and V, their sum and, if asked, the top-k for a chunk of up to
// EG * blockDim.x tokens; otherwise as group_score_select.
template <int EG>
__device__ __forceinline__ void group_score_select_multi(float* vK, const float* vV, int L, int k,
                                                         bool do_select, float* gout, uint32_t* scratch,
                                                         uint32_t* list, int tid, int nthreads) {
  const int lane = tid & 63, wave = tid >> 6, nw = nthreads >> 6;
  float* red = reinterpret_cast<float*>(scratch + kGroupSelHist);
  group_sel_clear(scratch, tid, nthreads);
  float sK[EG], sV[EG];
  float mK = -INFINITY, mV = -INFINITY;
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    const int t = e * nthreads + tid;
    sK[e] = t < L ? std_of_var(vK[t]) : -INFINITY;
    sV[e] = t < L ? std_of_var(vV[t]) : -INFINITY;
    mK = fmaxf(mK, sK[e]);
    mV = fmaxf(mV, sV[e]);
  }
  mK = wave_max(mK);
  mV = wave_max(mV);
  if (lane == 0) {
    red[wave * 2] = mK;
    red[wave * 2 + 1] = mV;
  }
  __syncthreads();
  {
    float4 r[kGroupSelMaxWaves / 2];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) r[i] = reinterpret_cast<const float4*>(red)[i];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) {
      if (2 * i < nw) {
        mK = fmaxf(mK, r[i].x);
        mV = fmaxf(mV, r[i].y);
      }
      if (2 * i + 1 < nw) {
        mK = fmaxf(mK, r[i].z);
        mV = fmaxf(mV, r[i].w);
      }
    }
  }
  float eK[EG], eV[EG];
  float aK = 0.f, aV = 0.f;
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    const bool live = e * nthreads + tid < L;
    eK[e] = live ? __expf(sK[e] - mK) : 0.f;
    eV[e] = live ? __expf(sV[e] - mV) : 0.f;
    aK += eK[e];
    aV += eV[e];
  }
  aK = wave_sum(aK);
  aV = wave_sum(aV);
  if (lane == 0) {
    red[16 + wave * 2] = aK;
    red[16 + wave * 2 + 1] = aV;
  }
  __syncthreads();
  float tK = 0.f, tV = 0.f;
  {
    float4 r[kGroupSelMaxWaves / 2];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) r[i] = reinterpret_cast<const float4*>(red + 16)[i];
#pragma unroll
    for (int i = 0; i < kGroupSelMaxWaves / 2; ++i) {
      if (2 * i < nw) {
        tK += r[i].x;
        tV += r[i].y;
      }
      if (2 * i + 1 < nw) {
        tK += r[i].z;
        tV += r[i].w;
      }
    }
  }
  const float rK = fast_rcp(tK), rV = fast_rcp(tV);
  uint32_t keys[EG];
#pragma unroll
  for (int e = 0; e < EG; ++e) {
    const int t = e * nthreads + tid;
    const float sc = eK[e] * rK + eV[e] * rV;
    keys[e] = t < L ? ordered_key(sc) : 0u;
    if (t < L) {
      vK[t] = sc;
      if (gout) st4_out_at(gout, (uint32_t)t * 4u, __float_as_uint(sc));
    }
  }
  if (do_select) group_topk_multi<EG>(keys, L, k, scratch, list, tid, nthreads);
}

}  // namespace lagkv
