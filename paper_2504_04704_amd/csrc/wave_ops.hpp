// Wave64 building blocks for the LagKV kernels (gfx950): DPP row reductions,
// whole-wave reductions, ordered float keys and the wave-level top-k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lagkv {

constexpr int kWave = 64;

// ---- DPP moves inside a row of 16 lanes ------------------------------------------
// quad_perm(1,0,3,2)=0xB1 (xor 1), quad_perm(2,3,0,1)=0x4E (xor 2),
// row_half_mirror=0x141 (i <-> 7-i), row_mirror=0x140 (i <-> 15-i).
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
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

__device__ __forceinline__ float wave_sum(float v) { return group_sum<64>(v); }

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_mov<0xB1>(v));
  v = fmaxf(v, dpp_mov<0x4E>(v));
  v = fmaxf(v, dpp_mov<0x141>(v));
  v = fmaxf(v, dpp_mov<0x140>(v));
  v = fmaxf(v, __shfl_xor(v, 16));
  v = fmaxf(v, __shfl_xor(v, 32));
  return v;
}

// Number of set bits of `mask` strictly below the calling lane.
__device__ __forceinline__ int prefix_popc(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0));
}

// Monotone map from float to uint32: a < b  <=>  key(a) < key(b) for finite values;
// -0 and +0 get the same key.
__device__ __forceinline__ uint32_t ordered_key(float s) {
  uint32_t b = __float_as_uint(s + 0.0f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Wave-level top-k over L scores held in LDS.
//   sc    L fp32 scores (LDS), token t at sc[t]
//   list  receives the k kept token positions, ascending (LDS)
// Order: score descending, position ascending.  Method: the k-th largest key is
// found bit by bit (32 counting rounds with ballots), all larger keys are kept and
// ties with it are admitted from the lowest position up.  Token t lives in lane
// t % 64, element t / 64, so a prefix count over (element, lane) is position order.
// E > 0: keys are kept in E registers per lane (L <= 64*E); E == 0: re-read from LDS.
template <int E>
__device__ __forceinline__ void wave_select(const float* sc, int L, int k, uint32_t* list,
                                            int lane) {
  const int ne = (L + kWave - 1) / kWave;
  uint32_t key[E > 0 ? E : 1];
  if constexpr (E > 0) {
#pragma unroll
    for (int e = 0; e < E; ++e) {
      const int t = e * kWave + lane;
      key[e] = (t < L) ? ordered_key(sc[t]) : 0u;
    }
  }
  auto get = [&](int e) -> uint32_t {
    if constexpr (E > 0) {
      return key[e];
    } else {
      const int t = e * kWave + lane;
      return (t < L) ? ordered_key(sc[t]) : 0u;
    }
  };
  uint32_t theta = 0;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = theta | (1u << bit);
    int cnt = 0;
    if constexpr (E > 0) {
#pragma unroll
      for (int e = 0; e < E; ++e) cnt += __popcll(__ballot(get(e) >= cand));
    } else {
      for (int e = 0; e < ne; ++e) cnt += __popcll(__ballot(get(e) >= cand));
    }
    if (cnt >= k) theta = cand;
  }
  int n_gt = 0;
  if constexpr (E > 0) {
#pragma unroll
    for (int e = 0; e < E; ++e) n_gt += __popcll(__ballot(get(e) > theta));
  } else {
    for (int e = 0; e < ne; ++e) n_gt += __popcll(__ballot(get(e) > theta));
  }
  const int need_eq = k - n_gt;
  int base = 0, eq_seen = 0;
  auto emit = [&](int e) {
    const uint32_t u = get(e);
    const int t = e * kWave + lane;
    const bool eq = (u == theta) && (t < L);
    const uint64_t eqm = __ballot(eq);
    const bool keep = ((u > theta) && (t < L)) || (eq && (eq_seen + prefix_popc(eqm) < need_eq));
    const uint64_t km = __ballot(keep);
    if (keep) list[base + prefix_popc(km)] = (uint32_t)t;
    base += __popcll(km);
    eq_seen += __popcll(eqm);
  };
  if constexpr (E > 0) {
#pragma unroll
    for (int e = 0; e < E; ++e) emit(e);
  } else {
    for (int e = 0; e < ne; ++e) emit(e);
  }
}

// Dispatch on the number of 64-token slabs of a chunk.
__device__ __forceinline__ void wave_select_any(const float* sc, int L, int k, uint32_t* list,
                                                int lane) {
  if (L <= 64) wave_select<1>(sc, L, k, list, lane);
  else if (L <= 128) wave_select<2>(sc, L, k, list, lane);
  else if (L <= 256) wave_select<4>(sc, L, k, list, lane);
  else if (L <= 512) wave_select<8>(sc, L, k, list, lane);
  else if (L <= 1024) wave_select<16>(sc, L, k, list, lane);
  else wave_select<0>(sc, L, k, list, lane);
}

// Softmax over the chunk for K and V and their sum (Eq. 10-11), by one wave.
//   sK, sV  per-token spreads (LDS); on return sK[t] holds the final score
//   gout    optional global destination of the L scores
__device__ __forceinline__ void wave_chunk_softmax(float* sK, const float* sV, int L, float* gout,
                                                   int lane) {
  float mK = -INFINITY, mV = -INFINITY;
  for (int t = lane; t < L; t += kWave) {
    mK = fmaxf(mK, sK[t]);
    mV = fmaxf(mV, sV[t]);
  }
  mK = wave_max(mK);
  mV = wave_max(mV);
  float aK = 0.f, aV = 0.f;
  for (int t = lane; t < L; t += kWave) {
    aK += expf(sK[t] - mK);
    aV += expf(sV[t] - mV);
  }
  aK = wave_sum(aK);
  aV = wave_sum(aV);
  for (int t = lane; t < L; t += kWave) {
    const float s = expf(sK[t] - mK) / aK + expf(sV[t] - mV) / aV;
    sK[t] = s;
    if (gout) gout[t] = s;
  }
}

}  // namespace lagkv
