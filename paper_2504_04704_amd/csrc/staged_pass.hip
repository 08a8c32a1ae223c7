// Three-kernel LagKV path for gfx950: score -> select -> gather.  It accepts any head
// dimension, element alignment and stride, reads every chunk twice (once as the
// reference of its predecessor) and stages scores and kept positions in global
// memory.  lagkv_select is always served from here; lagkv_score / lagkv_compress /
// lagkv_append_and_compress use it for shapes the fused kernels do not cover.
#include "lagkv_internal.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"

namespace lagkv {

// ekind: 4 = fp32, 2 = bf16, 3 = fp16
__device__ __forceinline__ float load_elem(const char* row, int c, int ekind) {
  if (ekind == 4) return reinterpret_cast<const float*>(row)[c];
  if (ekind == 3) return (float)reinterpret_cast<const _Float16*>(row)[c];
  return __uint_as_float((uint32_t) reinterpret_cast<const uint16_t*>(row)[c] << 16);
}

// One workgroup per (stream, scored chunk).  LDS: mn/iv of K and V [4][D], spreads
// [2][L], partial min/max [4][256].  Phase 1: per-channel min/max of the NEXT chunk
// (Eq. 7-8), all threads (row groups x channels).  Phase 2: one wavefront per token: normalise (Eq. 9), mean and centred sum
// of squares over the channels (Eq. 10).  Phase 3: chunk softmax and K+V sum
// (Eq. 10-11) by wavefront 0.
__global__ void __launch_bounds__(256) staged_score_kernel(const PassArgs a, int64_t row0,
                                                           float* __restrict__ scores) {
  extern __shared__ float4 lds_raw[];
  float* lds = reinterpret_cast<float*>(lds_raw);
  const int D = a.D, L = a.L, esize = a.esize == 4 ? 4 : (a.f16 ? 3 : 2);
  float* mnK = lds;
  float* ivK = mnK + D;
  float* mnV = ivK + D;
  float* ivV = mnV + D;
  float* sK = ivV + D;
  float* sV = sK + L;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
  const int64_t stream = blockIdx.x / a.n_s, p = blockIdx.x % a.n_s;
  const int64_t b = stream / a.H, h = stream % a.H;
  const char* kin = a.K + b * a.sb + h * a.sh + (row0 + p * L) * a.st;
  if (a.variant == 2) {  // Eq. 16: score = -||K_t||_2; no reference, no softmax, V unused
    float* out = scores + (stream * a.n_s + p) * L;
    for (int r = wave; r < L; r += nw) {
      const char* kr = kin + (int64_t)r * a.st;
      float s = 0.f;
      for (int c = lane; c < D; c += kWave) {
        const float x = load_elem(kr, c, esize);
        s = fmaf(x, x, s);
      }
      s = wave_sum(s);
      if (lane == 0) out[r] = -sqrtf(s);
    }
    return;
  }
  const char* vin = a.V + b * a.sb + h * a.sh + (row0 + p * L) * a.st;
  // Eq. 7-8 take the reference from the next chunk, Eq. 14-15 from the chunk itself
  const int64_t ref_off = (a.variant == 1) ? 0 : (int64_t)L * a.st;
  const char* kref = kin + ref_off;
  const char* vref = vin + ref_off;

  // Phase 1 with every thread at work: the threads form G row groups of Dc channels; group g
  // folds rows g, g+G, ... of the reference chunk, and the G partial results per channel are
  // combined through LDS.
  const int nthr = blockDim.x;
  const int Dc = D < nthr ? D : nthr, G = nthr / Dc;
  float* red = sV + L;                       // [4][G][Dc]
  for (int c0 = 0; c0 < D; c0 += Dc) {
    const int g = tid / Dc, c = c0 + tid % Dc;
    if (g < G && c < D) {
      float lo = INFINITY, hi = -INFINITY, lov = INFINITY, hiv = -INFINITY;
      for (int r = g; r < L; r += G) {
        const float x = load_elem(kref + (int64_t)r * a.st, c, esize);
        const float y = load_elem(vref + (int64_t)r * a.st, c, esize);
        lo = fminf(lo, x);
        hi = fmaxf(hi, x);
        lov = fminf(lov, y);
        hiv = fmaxf(hiv, y);
      }
      float* w = red + g * Dc + (c - c0);
      w[0] = lo;
      w[G * Dc] = hi;
      w[2 * G * Dc] = lov;
      w[3 * G * Dc] = hiv;
    }
    __syncthreads();
    if (tid < Dc && c0 + tid < D) {
      float lo = INFINITY, hi = -INFINITY, lov = INFINITY, hiv = -INFINITY;
      for (int g2 = 0; g2 < G; ++g2) {
        const float* rd = red + g2 * Dc + tid;
        lo = fminf(lo, rd[0]);
        hi = fmaxf(hi, rd[G * Dc]);
        lov = fminf(lov, rd[2 * G * Dc]);
        hiv = fmaxf(hiv, rd[3 * G * Dc]);
      }
      mnK[c0 + tid] = lo;
      ivK[c0 + tid] = inv_range(lo, hi);
      mnV[c0 + tid] = lov;
      ivV[c0 + tid] = inv_range(lov, hiv);
    }
    __syncthreads();
  }

  const float inv_D = 1.0f / (float)D, inv_dof = 1.0f / (float)(D - a.ddof);
  for (int r = wave; r < L; r += nw) {
    const char* kr = kin + (int64_t)r * a.st;
    const char* vr = vin + (int64_t)r * a.st;
    float s = 0.f, t = 0.f;
    for (int c = lane; c < D; c += kWave) {
      s += (load_elem(kr, c, esize) - mnK[c]) * ivK[c];
      t += (load_elem(vr, c, esize) - mnV[c]) * ivV[c];
    }
    const float muK = wave_sum(s) * inv_D, muV = wave_sum(t) * inv_D;
    s = 0.f;
    t = 0.f;
    for (int c = lane; c < D; c += kWave) {
      const float dk = (load_elem(kr, c, esize) - mnK[c]) * ivK[c] - muK;
      const float dv = (load_elem(vr, c, esize) - mnV[c]) * ivV[c] - muV;
      s = fmaf(dk, dk, s);
      t = fmaf(dv, dv, t);
    }
    s = wave_sum(s);
    t = wave_sum(t);
    if (lane == 0) {
      sK[r] = s * inv_dof;  // variance; the square root is taken with the softmax
      sV[r] = t * inv_dof;
    }
  }
  __syncthreads();
  if (wave == 0)
    wave_score_select_any(sK, sV, L, 0, false, scores + (stream * a.n_s + p) * L, nullptr, nullptr, lane);
}

// One wavefront per (stream, chunk): top-k of L scores, ascending absolute positions.
__global__ void __launch_bounds__(64) select_kernel(const float* __restrict__ scores, int64_t n_s,
                                                    int L, int k, int64_t row0,
                                                    int32_t* __restrict__ kept) {
  extern __shared__ float4 lds_raw[];
  float* sc = reinterpret_cast<float*>(lds_raw);
  uint32_t* list = reinterpret_cast<uint32_t*>(sc + L);
  const int lane = threadIdx.x;
  const int64_t chunk = blockIdx.x, p = chunk % n_s;
  const float* src = scores + chunk * L;
  for (int t = lane; t < L; t += kWave) sc[t] = src[t];
  for (int i = lane; i < k; i += kWave) list[i] = 0;
  __syncthreads();
  wave_topk_scores(sc, L, k, list, lane);
  __syncthreads();
  for (int i = lane; i < k; i += kWave)
    kept[chunk * k + i] = (int32_t)(row0 + p * L + list[i]);
}

template <typename UT>
__global__ void __launch_bounds__(256) gather_rows_kernel(const char* __restrict__ src, int64_t sb,
                                                          int64_t sh, int64_t st, int H,
                                                          char* __restrict__ dst, int64_t units,
                                                          const int32_t* __restrict__ kept,
                                                          int32_t* __restrict__ idx_out,
                                                          GatherMap m, int rows_per_block) {
  const int64_t blocks_per_stream = (m.n_out + rows_per_block - 1) / rows_per_block;
  const int64_t stream = blockIdx.x / blocks_per_stream;
  const int64_t r0 = (blockIdx.x % blocks_per_stream) * rows_per_block;
  const int64_t b = stream / H, h = stream % H;
  const char* sbase = src + b * sb + h * sh;
  char* dbase = dst + stream * m.n_out * units * (int64_t)sizeof(UT);
  const int64_t nrows = (m.n_out - r0) < rows_per_block ? (m.n_out - r0) : rows_per_block;
  for (int64_t i = threadIdx.x; i < nrows * units; i += blockDim.x) {
    const int64_t slot = r0 + i / units, u = i % units;
    int64_t srow;
    if (slot < m.n_pre) srow = m.pre0 + slot;
    else if (slot < m.n_pre + m.n_kept) srow = kept[stream * m.n_kept + (slot - m.n_pre)];
    else srow = m.post0 + (slot - m.n_pre - m.n_kept);
    reinterpret_cast<UT*>(dbase + slot * units * (int64_t)sizeof(UT))[u] =
        reinterpret_cast<const UT*>(sbase + srow * st)[u];
    if (idx_out && u == 0) idx_out[stream * m.n_out + slot] = (int32_t)srow;
  }
}

template <typename UT>
__global__ void __launch_bounds__(256) copy_rows_kernel(const char* __restrict__ src, int64_t ssb,
                                                        int64_t ssh, int64_t sst,
                                                        char* __restrict__ dst, int64_t dsb,
                                                        int64_t dsh, int64_t dst_st, int H,
                                                        int64_t rows, int64_t units,
                                                        int rows_per_block) {
  const int64_t blocks_per_stream = (rows + rows_per_block - 1) / rows_per_block;
  const int64_t stream = blockIdx.x / blocks_per_stream;
  const int64_t r0 = (blockIdx.x % blocks_per_stream) * rows_per_block;
  const int64_t b = stream / H, h = stream % H;
  const char* sbase = src + b * ssb + h * ssh;
  char* dbase = dst + b * dsb + h * dsh;
  const int64_t nrows = (rows - r0) < rows_per_block ? (rows - r0) : rows_per_block;
  for (int64_t i = threadIdx.x; i < nrows * units; i += blockDim.x) {
    const int64_t r = r0 + i / units, u = i % units;
    reinterpret_cast<UT*>(dbase + r * dst_st)[u] = reinterpret_cast<const UT*>(sbase + r * sst)[u];
  }
}

__global__ void __launch_bounds__(256) iota_rows_kernel(int32_t* __restrict__ pos, int64_t capacity,
                                                        int64_t at, int64_t n, int32_t first) {
  const int64_t nb = (n + blockDim.x - 1) / blockDim.x;
  const int64_t stream = blockIdx.x / nb;
  const int64_t i = (blockIdx.x % nb) * blockDim.x + threadIdx.x;
  if (i < n) pos[stream * capacity + at + i] = first + (int32_t)i;
}

// ------------------------------------------------------------------------ host side
// mn/iv of K and V [4][D], variances [2][L], partial min/max of the row groups [4][256]
size_t staged_score_lds_bytes(int D, int L) { return ((size_t)4 * D + 2 * (size_t)L + 4 * 256) * 4; }

hipError_t launch_staged_score(const PassArgs& a, int64_t row0, float* scores, hipStream_t s) {
  const int64_t nblocks = (int64_t)a.B * a.H * a.n_s;
  if (nblocks <= 0 || nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const size_t lds = staged_score_lds_bytes(a.D, a.L);
  if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;
  staged_score_kernel<<<dim3((unsigned)nblocks), dim3(256), lds, s>>>(a, row0, scores);
  return hipGetLastError();
}

hipError_t launch_select(const float* scores, int64_t streams, int64_t n_s, int L, int k,
                         int64_t row0, int32_t* kept, hipStream_t s) {
  const int64_t nblocks = streams * n_s;
  if (nblocks <= 0 || nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const size_t lds = ((size_t)L + (size_t)k) * 4;
  if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;
  select_kernel<<<dim3((unsigned)nblocks), dim3(kWave), lds, s>>>(scores, n_s, L, k, row0, kept);
  return hipGetLastError();
}

static bool all_aligned(int unit, const void* a, const void* b, int64_t s0, int64_t s1, int64_t s2,
                        int64_t s3, int64_t s4, int64_t s5, int64_t rowbytes) {
  const uintptr_t m = (uintptr_t)unit - 1;
  return !(((uintptr_t)a | (uintptr_t)b | (uintptr_t)s0 | (uintptr_t)s1 | (uintptr_t)s2 |
            (uintptr_t)s3 | (uintptr_t)s4 | (uintptr_t)s5 | (uintptr_t)rowbytes) & m);
}

hipError_t launch_gather_rows(const char* src, int64_t sb, int64_t sh, int64_t st, int B, int H,
                              char* dst, int64_t rowbytes, int esize, const int32_t* kept,
                              int32_t* idx_out, const GatherMap& m, hipStream_t s) {
  if (m.n_out <= 0) return hipSuccess;
  const int rpb = 8;
  const int64_t nblocks = (int64_t)B * H * ((m.n_out + rpb - 1) / rpb);
  if (nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblocks), block(256);
  if (all_aligned(16, src, dst, sb, sh, st, 0, 0, 0, rowbytes))
    gather_rows_kernel<uint4><<<grid, block, 0, s>>>(src, sb, sh, st, H, dst, rowbytes / 16, kept,
                                                     idx_out, m, rpb);
  else if (esize == 4)
    gather_rows_kernel<uint32_t><<<grid, block, 0, s>>>(src, sb, sh, st, H, dst, rowbytes / 4, kept,
                                                        idx_out, m, rpb);
  else
    gather_rows_kernel<uint16_t><<<grid, block, 0, s>>>(src, sb, sh, st, H, dst, rowbytes / 2, kept,
                                                        idx_out, m, rpb);
  return hipGetLastError();
}

hipError_t launch_staged_gather(const PassArgs& a, const int32_t* kept, hipStream_t s) {
  GatherMap m;
  m.n_pre = a.S;
  m.pre0 = 0;
  m.n_kept = a.n_s * a.k;
  m.post0 = a.S + a.n_s * a.L;
  m.n_out = a.T_out;
  const int64_t rowbytes = (int64_t)a.D * a.esize;
  hipError_t e = launch_gather_rows(a.K, a.sb, a.sh, a.st, a.B, a.H, a.K_out, rowbytes, a.esize,
                                    kept, a.idx_out, m, s);
  if (e != hipSuccess) return e;
  return launch_gather_rows(a.V, a.sb, a.sh, a.st, a.B, a.H, a.V_out, rowbytes, a.esize, kept,
                            nullptr, m, s);
}

hipError_t launch_copy_rows(const char* src, int64_t ssb, int64_t ssh, int64_t sst, char* dst,
                            int64_t dsb, int64_t dsh, int64_t dst_st, int B, int H, int64_t rows,
                            int64_t rowbytes, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int rpb = 8;
  const int64_t nblocks = (int64_t)B * H * ((rows + rpb - 1) / rpb);
  if (nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblocks), block(256);
  if (all_aligned(16, src, dst, ssb, ssh, sst, dsb, dsh, dst_st, rowbytes))
    copy_rows_kernel<uint4><<<grid, block, 0, s>>>(src, ssb, ssh, sst, dst, dsb, dsh, dst_st, H, rows,
                                                   rowbytes / 16, rpb);
  else if (all_aligned(4, src, dst, ssb, ssh, sst, dsb, dsh, dst_st, rowbytes))
    copy_rows_kernel<uint32_t><<<grid, block, 0, s>>>(src, ssb, ssh, sst, dst, dsb, dsh, dst_st, H,
                                                      rows, rowbytes / 4, rpb);
  else
    copy_rows_kernel<uint16_t><<<grid, block, 0, s>>>(src, ssb, ssh, sst, dst, dsb, dsh, dst_st, H,
                                                      rows, rowbytes / 2, rpb);
  return hipGetLastError();
}

hipError_t launch_iota_rows(int32_t* pos, int64_t streams, int64_t capacity, int64_t at, int64_t n,
                            int32_t first, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  const int64_t nblocks = streams * ((n + 255) / 256);
  if (nblocks > 0x7fffffffLL) return hipErrorInvalidValue;
  iota_rows_kernel<<<dim3((unsigned)nblocks), dim3(256), 0, s>>>(pos, capacity, at, n, first);
  return hipGetLastError();
}

}  // namespace lagkv
