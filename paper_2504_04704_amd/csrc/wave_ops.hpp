// Wave64 building blocks for the LagKV kernels (gfx950): DPP row reductions,
// whole-wave reductions, ordered float keys, the chunk softmax (Eq. 10-11) and the
// wave-level top-k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace lagkv {

constexpr int kWave = 64;

#ifndef LAGKV_FAST_SQRT
#define LAGKV_FAST_SQRT 1
#endif
// Square root of a token's channel variance (Eq. 10).  The hardware square root
// (1 ulp) is an order of magnitude shorter than the correctly rounded sequence and
// well inside the 1e-5 score tolerance; every kernel goes through this one function.
__device__ __forceinline__ float std_of_var(float v) {
#if LAGKV_FAST_SQRT
  return __builtin_amdgcn_sqrtf(v);
#else
  return sqrtf(v);
#endif
}

// Reciprocal of a softmax denominator: the hardware reciprocal (1 ulp), as for the channel
// ranges; the full division sequence is a dozen instructions longer.
__device__ __forceinline__ float fast_rcp(float v) { return __builtin_amdgcn_rcpf(v); }

// ---- DPP moves inside a row of 16 lanes ------------------------------------------
// quad_perm(1,0,3,2)=0xB1 (xor 1), quad_perm(2,3,0,1)=0x4E (xor 2),
// row_half_mirror=0x141 (i <-> 7-i), row_mirror=0x140 (i <-> 15-i).
template <int CTRL>
__device__ __forceinline__ int dpp_mov_i(int v) {
  return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, false);
}
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(float, dpp_mov_i<CTRL>(__builtin_bit_cast(int, v)));
}

// Sum over groups of LPR consecutive lanes (LPR a power of two <= 64); every lane of
// a group receives the total.  All 64 lanes must be active.
template <int LPR>
__device__ __forceinline__ float group_sum(float v) {
  if constexpr (LPR >= 2) v += dpp_mov<0xB1>(v);
  if constexpr (LPR >= 4) v += dpp_mov<0x4E>(v);
  if constexpr (LPR >= 8) v += dpp_mov<0x141>(v);
  if constexpr (LPR >= 16) v += dpp_mov<0x140>(v);
  if constexpr (LPR >= 32) v += __shfl_xor(v, 16);
  if constexpr (LPR >= 64) v += __shfl_xor(v, 32);
  return v;
}

// Whole-wave reductions: DPP inside each row of 16 lanes, then the four row results
// are read through scalar registers.  The result is wave-uniform; all lanes active.
__device__ __forceinline__ float rl_f(float v, int l) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
}
__device__ __forceinline__ float wave_sum(float v) {
  v = group_sum<16>(v);
  return (rl_f(v, 0) + rl_f(v, 16)) + (rl_f(v, 32) + rl_f(v, 48));
}
__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  return fmaxf(fmaxf(rl_f(v, 0), rl_f(v, 16)), fmaxf(rl_f(v, 32), rl_f(v, 48)));
}
__device__ __forceinline__ uint32_t umax_(uint32_t a, uint32_t b) { return a > b ? a : b; }
__device__ __forceinline__ uint32_t umin_(uint32_t a, uint32_t b) { return a < b ? a : b; }
__device__ __forceinline__ uint32_t wave_umax(uint32_t v) {
  v = umax_(v, (uint32_t)dpp_mov_i<0xB1>((int)v));
  v = umax_(v, (uint32_t)dpp_mov_i<0x4E>((int)v));
  v = umax_(v, (uint32_t)dpp_mov_i<0x141>((int)v));
  v = umax_(v, (uint32_t)dpp_mov_i<0x140>((int)v));
  return umax_(umax_((uint32_t)__builtin_amdgcn_readlane((int)v, 0),
                     (uint32_t)__builtin_amdgcn_readlane((int)v, 16)),
               umax_((uint32_t)__builtin_amdgcn_readlane((int)v, 32),
                     (uint32_t)__builtin_amdgcn_readlane((int)v, 48)));
}
__device__ __forceinline__ uint32_t wave_umin(uint32_t v) { return ~wave_umax(~v); }

// Number of set bits of `mask` strictly below the calling lane.
__device__ __forceinline__ int prefix_popc(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Monotone map from float to uint32: a < b  <=>  key(a) < key(b) for finite values;
// -0 and +0 get the same key.  No finite value maps to key 0.
__device__ __forceinline__ uint32_t ordered_key(float s) {
  uint32_t b = __float_as_uint(s + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Wave-level top-k.  key(e) is the ordered key of token t = e*64 + lane (0 for t >= L).
//   list     receives the k kept token positions, ascending (LDS)
//   slotmap  optional [L]: output slot of a kept token, -1 otherwise (LDS)
// Order: score descending, position ascending.  The k-th largest key is found bit by
// bit with ballots, starting below the bits all keys share; all larger keys are kept
// and ties with it are admitted from the lowest position up.  A prefix count over
// (element, lane) is position order.
template <int E, typename F>
__device__ __forceinline__ void for_each_slab(int ne, F f) {
  if constexpr (E > 0) {
#pragma unroll
    for (int e = 0; e < E; ++e) f(e);
  } else {
    for (int e = 0; e < ne; ++e) f(e);
  }
}

template <int E, typename KeyFn>
__device__ __forceinline__ void wave_topk(KeyFn key, int L, int k, uint32_t* list, int32_t* slotmap,
                                          int lane) {
  const int ne = (L + kWave - 1) / kWave;
  uint32_t hi = 0, lo = 0xffffffffu;
  for_each_slab<E>(ne, [&](int e) {
    const uint32_t u = key(e);
    hi = umax_(hi, u);
    lo = umin_(lo, u ? u : 0xffffffffu);
  });
  hi = wave_umax(hi);
  lo = wave_umin(lo);
  uint32_t theta = hi;  // all real keys equal: the threshold is that key
  if (hi != lo) {
    const int top = 31 - __builtin_clz(hi ^ lo);  // highest bit in which two keys differ
    theta = hi & ~((2u << top) - 1u);             // the shared prefix
    for (int bit = top; bit >= 0; --bit) {
      const uint32_t cand = theta | (1u << bit);
      int cnt = 0;
      for_each_slab<E>(ne, [&](int e) { cnt += __popcll(__ballot(key(e) >= cand)); });
      if (cnt >= k) theta = cand;
    }
  }
  int n_gt = 0;
  for_each_slab<E>(ne, [&](int e) { n_gt += __popcll(__ballot(key(e) > theta)); });
  const int need_eq = k - n_gt;
  int base = 0, eq_seen = 0;
  for_each_slab<E>(ne, [&](int e) {
    const uint32_t u = key(e);
    const int t = e * kWave + lane;
    const bool eq = (u == theta) && (t < L);
    const uint64_t eqm = __ballot(eq);
    const bool keep = ((u > theta) && (t < L)) || (eq && (eq_seen + prefix_popc(eqm) < need_eq));
    const uint64_t km = __ballot(keep);
    const int slot = base + prefix_popc(km);
    if (keep) list[slot] = (uint32_t)t;
    if (slotmap && t < L) slotmap[t] = keep ? slot : -1;
    base += __popcll(km);
    eq_seen += __popcll(eqm);
  });
}

// Chunk softmax of K and V, their sum (Eq. 10-11) and, if asked, the top-k, by ONE
// wavefront.  On entry vK[t], vV[t] (LDS) hold the channel VARIANCE of token t (the
// square root of Eq. 10's "Std." is taken here, once per token).  On return vK[t]
// holds the final score.  gout: optional global destination of the L scores.
//   score = exp(sK - max sK) * (1 / sum) + exp(sV - max sV) * (1 / sum)
// E > 0: the chunk's L <= 64*E tokens live in registers; E == 0: any L, through LDS.
template <int E>
__device__ __forceinline__ void wave_score_select(float* vK, const float* vV, int L, int k,
                                                  bool do_select, float* gout, uint32_t* list,
                                                  int32_t* slotmap, int lane) {
  if constexpr (E > 0) {
    float eK[E], eV[E];
    float mK = -INFINITY, mV = -INFINITY;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int t = e * kWave + lane;
      eK[e] = t < L ? std_of_var(vK[t]) : -INFINITY;
      eV[e] = t < L ? std_of_var(vV[t]) : -INFINITY;
      mK = fmaxf(mK, eK[e]);
      mV = fmaxf(mV, eV[e]);
    }
    mK = wave_max(mK);
    mV = wave_max(mV);
    float aK = 0.f, aV = 0.f;
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int t = e * kWave + lane;
      eK[e] = t < L ? __expf(eK[e] - mK) : 0.f;
      eV[e] = t < L ? __expf(eV[e] - mV) : 0.f;
      aK += eK[e];
      aV += eV[e];
    }
    const float rK = 1.0f / wave_sum(aK), rV = 1.0f / wave_sum(aV);
    uint32_t keys[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int t = e * kWave + lane;
      const float s = eK[e] * rK + eV[e] * rV;
      keys[e] = t < L ? ordered_key(s) : 0u;
      if (t < L) {
        vK[t] = s;
        if (gout) gout[t] = s;
      }
    }
    if (do_select) wave_topk<E>([&](int e) { return keys[e]; }, L, k, list, slotmap, lane);
  } else {
    float mK = -INFINITY, mV = -INFINITY;
    for (int t = lane; t < L; t += kWave) {
      mK = fmaxf(mK, std_of_var(vK[t]));
      mV = fmaxf(mV, std_of_var(vV[t]));
    }
    mK = wave_max(mK);
    mV = wave_max(mV);
    float aK = 0.f, aV = 0.f;
    for (int t = lane; t < L; t += kWave) {
      aK += __expf(std_of_var(vK[t]) - mK);
      aV += __expf(std_of_var(vV[t]) - mV);
    }
    const float rK = 1.0f / wave_sum(aK), rV = 1.0f / wave_sum(aV);
    for (int t = lane; t < L; t += kWave) {
      const float s = __expf(std_of_var(vK[t]) - mK) * rK + __expf(std_of_var(vV[t]) - mV) * rV;
      vK[t] = s;
      if (gout) gout[t] = s;
    }
    if (do_select)
      wave_topk<0>(
          [&](int e) {
            const int t = e * kWave + lane;
            return t < L ? ordered_key(vK[t]) : 0u;
          },
          L, k, list, slotmap, lane);
  }
}

// Dispatch on the number of 64-token slabs of a chunk.
__device__ __forceinline__ void wave_score_select_any(float* vK, const float* vV, int L, int k,
                                                      bool do_select, float* gout, uint32_t* list,
                                                      int32_t* slotmap, int lane) {
  if (L <= 64) wave_score_select<1>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 128) wave_score_select<2>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 256) wave_score_select<4>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 512) wave_score_select<8>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 1024) wave_score_select<16>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else wave_score_select<0>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
}

// Register-lean dispatch for callers that hold other state in registers: chunks of
// up to 512 tokens in registers, longer ones through LDS.  Deliberately NOT inlined:
// it runs once per chunk on one wavefront, and keeping it out of line keeps its
// temporaries out of the caller's register allocation.
__device__ __attribute__((noinline)) void wave_score_select_lean(float* vK, const float* vV, int L, int k,
                                                       bool do_select, float* gout, uint32_t* list,
                                                       int32_t* slotmap, int lane) {
  if (L <= 128) wave_score_select<2>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 256) wave_score_select<4>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else if (L <= 512) wave_score_select<8>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
  else wave_score_select<0>(vK, vV, L, k, do_select, gout, list, slotmap, lane);
}

// Top-k of L given scores (LDS), any L.
__device__ __forceinline__ void wave_topk_scores(const float* sc, int L, int k, uint32_t* list,
                                                 int lane) {
  auto run = [&](auto e_tag) {
    constexpr int E = decltype(e_tag)::value;
    if constexpr (E > 0) {
      uint32_t keys[E];
#pragma unroll
      for (int e = 0; e < E; ++e) {
        const int t = e * kWave + lane;
        keys[e] = t < L ? ordered_key(sc[t]) : 0u;
      }
      wave_topk<E>([&](int e) { return keys[e]; }, L, k, list, nullptr, lane);
    } else {
      wave_topk<0>(
          [&](int e) {
            const int t = e * kWave + lane;
            return t < L ? ordered_key(sc[t]) : 0u;
          },
          L, k, list, nullptr, lane);
    }
  };
  if (L <= 128) run(std::integral_constant<int, 2>{});
  else if (L <= 512) run(std::integral_constant<int, 8>{});
  else if (L <= 1024) run(std::integral_constant<int, 16>{});
  else run(std::integral_constant<int, 0>{});
}

}  // namespace lagkv
