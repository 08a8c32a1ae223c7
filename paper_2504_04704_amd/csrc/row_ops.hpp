// Per-row arithmetic shared by the fused LagKV kernels: element unpacking, 16-byte
// accesses and the two-pass channel variance of a normalised token (Eq. 9-10).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "wave_ops.hpp"

namespace lagkv {

// Element types: VEC = elements in 16 bytes.
struct F32 {
  static constexpr int VEC = 4;
  static constexpr int KIND = 0;
};
struct BF16 {
  static constexpr int VEC = 8;
  static constexpr int KIND = 1;
};
struct F16 {
  static constexpr int VEC = 8;
  static constexpr int KIND = 2;
};
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));

template <typename ET>
__device__ __forceinline__ void unpack(const uint4& q, float (&x)[ET::VEC]) {
  if constexpr (ET::KIND == 0) {
    x[0] = __uint_as_float(q.x);
    x[1] = __uint_as_float(q.y);
    x[2] = __uint_as_float(q.z);
    x[3] = __uint_as_float(q.w);
  } else if constexpr (ET::KIND == 2) {  // binary16 -> fp32 is exact (hardware conversion)
    const uint32_t w[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const half2_t h = __builtin_bit_cast(half2_t, w[i]);
      x[2 * i] = (float)h.x;
      x[2 * i + 1] = (float)h.y;
    }
  } else {  // bf16 -> fp32 is a 16-bit shift; element 2i is the low half of word i
    x[0] = __uint_as_float(q.x << 16);
    x[1] = __uint_as_float(q.x & 0xffff0000u);
    x[2] = __uint_as_float(q.y << 16);
    x[3] = __uint_as_float(q.y & 0xffff0000u);
    x[4] = __uint_as_float(q.z << 16);
    x[5] = __uint_as_float(q.z & 0xffff0000u);
    x[6] = __uint_as_float(q.w << 16);
    x[7] = __uint_as_float(q.w & 0xffff0000u);
  }
}

__device__ __forceinline__ uint4 ld16(const char* p) {
  return *reinterpret_cast<const uint4*>(p);
}
__device__ __forceinline__ void st16(char* p, const uint4& v) {
  *reinterpret_cast<uint4*>(p) = v;
}

#ifndef LAGKV_FAST_RCP
#define LAGKV_FAST_RCP 1
#endif
// 1 / (max - min) of a reference channel (Eq. 9), or 0 for a constant channel so that
// it contributes nothing.  The hardware reciprocal (1 ulp) is used by every kernel.
__device__ __forceinline__ float inv_range(float mn, float mx) {
#if LAGKV_FAST_RCP
  return mx > mn ? __builtin_amdgcn_rcpf(mx - mn) : 0.f;
#else
  return mx > mn ? 1.0f / (mx - mn) : 0.f;
#endif
}

// Variance over the D channels of one normalised token (Eq. 9-10; the square root is
// taken later, once per token).  zbar = (x - mn) * iv.  Two passes: the mean first
// (any error in it only enters the variance to second order, so the cheap fma form
// seeded with bias = sum_j -(mn_j*iv_j) is used), then the centred sum of squares
// from the exactly subtracted (x - mn).  The row is spread over LPR lanes.
// `live`: false in a lane that holds no channels of its own (rows that do not fill LPR lanes,
// see lanes_per_row: such a lane repeats the row's last 16 bytes and its statistics carry
// iv = 0, so only its centred squares have to be dropped).
template <int LPR, int VEC>
__device__ __forceinline__ float token_var(const float (&x)[VEC], const float (&mn)[VEC],
                                           const float (&iv)[VEC], float bias, float inv_D,
                                           float inv_dof, bool live = true) {
  float s = bias;
#pragma unroll
  for (int j = 0; j < VEC; ++j) s = fmaf(x[j], iv[j], s);
  s = group_sum<LPR>(s);
  const float mean = s * inv_D;
  float ss = 0.f;
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    const float d = fmaf(x[j] - mn[j], iv[j], -mean);
    ss = fmaf(d, d, ss);
  }
  if (!live) ss = 0.f;
  ss = group_sum<LPR>(ss);
  return ss * inv_dof;
}

template <int VEC>
struct TStats {  // running per-channel min/max of the lane's VEC channels (Eq. 7-8)
  float mn[VEC], mx[VEC];
  __device__ __forceinline__ void reset() {
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      mn[j] = INFINITY;
      mx[j] = -INFINITY;
    }
  }
};

// Makes the running statistics materialise where this is called.  Without it the compiler
// is free to postpone the whole min/max chain of an unrolled sweep to the point where its
// result is used, which keeps the unpacked rows of the entire sweep alive in registers.
template <int VEC>
__device__ __forceinline__ void pin(TStats<VEC>& s) {
#pragma unroll
  for (int j = 0; j < VEC; ++j) asm volatile("" : "+v"(s.mn[j]), "+v"(s.mx[j]));
}

template <int VEC>
struct TRef {  // reference statistics as Eq. 9 consumes them: zbar = (x - mn) * iv
  float mn[VEC], iv[VEC];
  float bias;
  // live = false: a lane without channels of its own (see token_var) contributes nothing
  __device__ __forceinline__ void from(const TStats<VEC>& s, bool live = true) {
    bias = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      mn[j] = s.mn[j];
      iv[j] = live ? inv_range(s.mn[j], s.mx[j]) : 0.f;
      bias -= mn[j] * iv[j];
    }
  }
};

// Reference statistics for the one-sweep variance below: zbar - 1/2 = x * iv + sh with
// sh = -(mn * iv) - 1/2 rounded once.
// `wide` (the same in every lane that built it from the same statistics): some channel's
// offset is so large against its range that the rounding of sh alone could move a score by
// more than 2e-6 relative (|sh| > 64: the error of a token's standard deviation from this
// source is at most 2^-25 times the r.m.s. of sh over the channels).
template <int VEC>
struct TRefFast {
  float iv[VEC], sh[VEC];
  bool wide;
  // iv and sh of the lane's VEC consecutive channels, as one thread per channel computed them
  // (iv = inv_range(mn, mx), sh = fma(-mn, iv, -1/2))
  __device__ __forceinline__ void load(const float* ivp, const float* shp) {
    float big = 0.f;
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      iv[j] = ivp[j];
      sh[j] = shp[j];
      big = fmaxf(big, fabsf(sh[j]));
    }
    wide = __any(big > 64.f);
  }
};

// Variance over the D channels of one normalised token in ONE sweep over its channels: sum
// and sum of squares of zbar - 1/2 (normalised values lie around [0,1], so the shift keeps
// the two sums from cancelling), 8 instructions per row slice shorter than token_var.
// `sumsq` receives the sum of squares.  A caller must redo with token_var every token with
// sumsq^2 > 256 * D^2 * variance (a nearly constant token: mean square^2 > 256 * variance,
// where the subtraction of the two sums loses more than the score tolerance allows; inside
// the bound the error of the standard deviation stays under 2e-6), and everything built on
// `wide` statistics.
template <int LPR, int VEC>
__device__ __forceinline__ float token_var_fast(const float (&x)[VEC], const float (&iv)[VEC],
                                                const float (&sh)[VEC], float inv_D, float inv_dof,
                                                float& sumsq) {
  float s1 = 0.f, s2 = 0.f;
#pragma unroll
  for (int j = 0; j < VEC; ++j) {
    const float y = fmaf(x[j], iv[j], sh[j]);
    s1 += y;
    s2 = fmaf(y, y, s2);
  }
  s1 = group_sum<LPR>(s1);
  s2 = group_sum<LPR>(s2);
  sumsq = s2;
  return fmaf(-s1 * inv_D, s1, s2) * inv_dof;
}

// dst row r <- src row r for r < nrows, K and V together, 16 bytes per lane; rows of `units`
// 16-byte slices (lanes beyond a row's slices repeat its last one).
template <int LPR>
__device__ __forceinline__ void copy_rows_kv(const char* __restrict__ ks, const char* __restrict__ vs,
                                             int64_t sst, char* __restrict__ kd,
                                             char* __restrict__ vd, int64_t dst_st, int64_t nrows,
                                             int units, int tid, int nthreads) {
  const int cl = tid % LPR < units ? tid % LPR : units - 1;
  const int64_t ng = nthreads / LPR;
  for (int64_t r = tid / LPR; r < nrows; r += ng) {
    const uint4 a = ld16(ks + r * sst + cl * 16);
    const uint4 b = ld16(vs + r * sst + cl * 16);
    st16(kd + r * dst_st + cl * 16, a);
    st16(vd + r * dst_st + cl * 16, b);
  }
}

// Rows the fused kernels take: whole 16-byte slices, 48 to 512 bytes.  A row is held by
// LPR = 4, 8, 16 or 32 consecutive lanes, 16 bytes each; when its `units` slices do not fill
// them, the lanes left over repeat the last slice (loads and stores of the same bytes twice are
// harmless, min/max do not change) and are left out of the sums over the channels.
inline int row_units(int D, int esize) {
  const int64_t bytes = (int64_t)D * esize;
  return (bytes % 16 == 0 && bytes >= 48 && bytes <= 512) ? (int)(bytes / 16) : 0;
}
inline int lanes_per_row(int D, int esize) {
  const int u = row_units(D, esize);
  return u == 0 ? 0 : u <= 4 ? 4 : u <= 8 ? 8 : u <= 16 ? 16 : 32;
}

}  // namespace lagkv
