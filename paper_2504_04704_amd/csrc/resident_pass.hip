// Chunk-resident LagKV kernel for gfx950: every input byte is fetched once and the
// kept rows are written straight from registers, so nothing is re-read.
//
// A workgroup walks a segment of one stream backwards like the streaming kernel, but
// holds the WHOLE current chunk in VGPRs: the first half of its wavefronts owns the K
// rows, the second half the V rows; a lane keeps 16 bytes of each of up to RS rows.
// All loads of a chunk are issued up front (maximum memory-level parallelism), the
// rows are folded into the per-channel min/max (Eq. 7-8) and scored against the
// previous chunk's statistics (Eq. 9-10) as they arrive, one wavefront runs the chunk
// softmax (Eq. 10-11) and the top-k, and every lane then stores those of its rows that
// were kept.  Serves chunks of up to min(512, RS * (64/LPR) * 4) rows; longer chunks use
// the streaming kernel.
#include "lagkv_internal.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"

namespace lagkv {

constexpr int kResidentRows = 32;  // RS: rows a lane holds per chunk

struct ResidentLds {
  int off_vK, off_vV, off_slot, off_list, off_stat, total;  // bytes
};
__host__ __device__ inline ResidentLds resident_lds(int D, int L, int k, int nw) {
  ResidentLds l;
  const int lp = (L + 3) & ~3, kp = (k + 3) & ~3;
  l.off_vK = 0;
  l.off_vV = lp * 4;
  l.off_slot = 2 * lp * 4;
  l.off_list = 3 * lp * 4;
  l.off_stat = l.off_list + kp * 4;
  l.total = l.off_stat + nw * 2 * D * 4;  // [wave][mn|mx][D]
  return l;
}

// FULL: the chunk fills all RS steps (L == RS * R), which makes the code branch-free so
// that the hardware load counter can be waited on row by row.
template <typename ET, int LPR, int G, bool FULL>
__global__ void __launch_bounds__(512) resident_pass_kernel(const PassArgs a) {
  constexpr int VEC = ET::VEC;
  constexpr int RPW = kWave / LPR;
  constexpr int RS = kResidentRows;
  constexpr int R = G * RPW;  // rows of one tensor covered per step
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int tid = threadIdx.x, nthreads = 2 * G * kWave;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform by construction
  const ResidentLds lay = resident_lds(a.D, a.L, a.k, 2 * G);
  float* vK = reinterpret_cast<float*>(lds + lay.off_vK);
  float* vV = reinterpret_cast<float*>(lds + lay.off_vV);
  int32_t* slotmap = reinterpret_cast<int32_t*>(lds + lay.off_slot);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);

  const int tensor = wave >= G ? 1 : 0;     // 0: this wavefront owns K rows, 1: V rows
  const int gslot = wave - tensor * G;      // wavefront index inside its tensor group
  const int rl = lane / LPR, cl = lane % LPR;
  const int row_first = gslot * RPW + rl;   // row of step 0; step i holds row_first + i*R
  const int L = a.L, k = a.k, S = a.S;
  const int nsteps = FULL ? RS : L / R;     // exact and <= RS (checked on the host)
  const int64_t rowbytes = (int64_t)LPR * 16;
  // per-lane byte offsets (32 bit); everything else in an address is wave-uniform
  const uint32_t lane_in = (uint32_t)(row_first * a.st) + (uint32_t)cl * 16u;
  const uint32_t lane_col = (uint32_t)cl * 16u;

  const int64_t stream = blockIdx.x / a.nseg;
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
  float* myvar = (tensor ? vV : vK) + row_first;   // + i*R is an immediate offset
  const int32_t* myslot = slotmap + row_first;
  const float inv_D = 1.0f / (float)a.D;
  const float inv_dof = 1.0f / (float)(a.D - a.ddof);
  const bool local = a.variant == 1;  // Eq. 14-15: statistics from the chunk itself

  for (int i = tid; i < k; i += nthreads) list[i] = 0;
  for (int i = tid; i < L; i += nthreads) slotmap[i] = -1;

  // sink rows and the sliding window (last full chunk + remainder) are plain copies
  if (gather && seg == 0 && S > 0) {
    copy_rows_kv<LPR>(kin, vin, a.st, kout, vout, rowbytes, S, tid, nthreads);
    if (iout)
      for (int i = tid; i < S; i += nthreads) iout[i] = i;
  }
  if (gather && seg == a.nseg - 1) {
    const int64_t w0 = S + a.n_s * L, o0 = S + a.n_s * k, nwin = a.T - w0;
    copy_rows_kv<LPR>(kin + w0 * a.st, vin + w0 * a.st, a.st, kout + o0 * rowbytes,
                      vout + o0 * rowbytes, rowbytes, nwin, tid, nthreads);
    if (iout)
      for (int64_t i = tid; i < nwin; i += nthreads) iout[o0 + i] = (int32_t)(w0 + i);
  }

  const int64_t p0 = (int64_t)seg * a.n_s / a.nseg;
  const int64_t p1 = (int64_t)(seg + 1) * a.n_s / a.nseg;

  uint4 q[RS];
  TStats<VEC> acc;
  TRef<VEC> ref;

  // issue every load of the chunk whose first row is `row`: a uniform base per step plus
  // one per-lane offset.  With an odd step count the last row is loaded twice so that the
  // rows can be consumed in pairs.
  auto load_chunk = [&](int64_t row) __attribute__((always_inline)) {
    const char* base = tin + row * a.st;
#pragma unroll
    for (int i = 0; i < RS; ++i) {
      if (i < nsteps) {
        q[i] = ld16(base + (int64_t)i * R * a.st + lane_in);
      } else if (i == nsteps && (nsteps & 1)) {
        q[i] = ld16(base + (int64_t)(i - 1) * R * a.st + lane_in);
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // keep every load ahead of the arithmetic below
  };
  // fold the resident rows into acc (STATS) and/or write their variances (SCORE)
  auto scan = [&](auto stats_tag, auto score_tag) __attribute__((always_inline)) {
    constexpr bool STATS = decltype(stats_tag)::value, SCORE = decltype(score_tag)::value;
#pragma unroll
    for (int i = 0; i < RS; i += 2) {
      if (i < nsteps) {
        float x0[VEC], x1[VEC];
        unpack<ET>(q[i], x0);
        unpack<ET>(q[i + 1], x1);
        if constexpr (STATS) {
#pragma unroll
          for (int j = 0; j < VEC; ++j) {
            acc.mn[j] = fminf(fminf(acc.mn[j], x0[j]), x1[j]);
            acc.mx[j] = fmaxf(fmaxf(acc.mx[j], x0[j]), x1[j]);
          }
        }
        if constexpr (SCORE) {
          const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
          const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
          if (cl == 0) {
            myvar[i * R] = v0;
            if (i + 1 < nsteps) myvar[(i + 1) * R] = v1;
          }
        }
        __builtin_amdgcn_sched_barrier(0);  // one row pair at a time: bounded live ranges
      }
    }
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
    if constexpr (G > 1) {
      if (rl == 0) {
        float* w = statbuf + (size_t)wave * 2 * a.D + cl * VEC;
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
          w[j] = acc.mn[j];
          w[a.D + j] = acc.mx[j];
        }
      }
      __syncthreads();
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float* rd = statbuf + (size_t)(tensor * G + g) * 2 * a.D + cl * VEC;
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

  if (!local) {  // statistics of the chunk after the segment: the first reference
    acc.reset();
    load_chunk(S + p1 * L);
    scan(T_{}, F_{});
    fold();
    ref.from(acc);
    __syncthreads();  // statbuf is rewritten by the next fold
  }

  for (int64_t p = p1 - 1; p >= p0; --p) {
    acc.reset();
    load_chunk(S + p * L);
    if (local) {
      scan(T_{}, F_{});
      fold();
      ref.from(acc);
      scan(F_{}, T_{});
      __syncthreads();
    } else {
      scan(T_{}, T_{});
      fold();
    }
    if (wave == 0) {
      wave_score_select_lean(vK, vV, L, k, gather, sout ? sout + p * L : nullptr, list, slotmap, lane);
    } else if (!local) {
      ref.from(acc);  // chunk p is the reference of chunk p-1
    }
    __syncthreads();
    if (gather) {
      char* dst = tout + (S + p * k) * rowbytes;
#pragma unroll
      for (int i = 0; i < RS; ++i) {
        if (i < nsteps) {
          const int s = myslot[i * R];
          if (s >= 0) st16(dst + ((uint32_t)s * (uint32_t)rowbytes + lane_col), q[i]);
        }
      }
      if (iout)
        for (int i = tid; i < k; i += nthreads)
          iout[S + p * k + i] = (int32_t)(S + p * L + list[i]);
    }
    if (wave == 0 && !local) ref.from(acc);
  }
}

// ------------------------------------------------------------------------ host side
// Wavefronts per tensor group (1, 2 or 4) for this row size and lag, or 0 when the
// kernel does not serve it: L must be an exact multiple of the rows one step covers and
// fit kResidentRows steps.
static int resident_group(int D, int esize, int L) {
  const int lpr = lanes_per_row(D, esize);
  if (lpr == 0 || L > 512) return 0;
  const int rpw = kWave / lpr;
  for (int g = 1; g <= 4; g *= 2) {
    const int r = g * rpw;
    if (L % r == 0 && L / r <= kResidentRows) return g;
  }
  return 0;
}

int resident_waves(int D, int esize, int L) { return 2 * resident_group(D, esize, L); }

size_t resident_lds_bytes(int D, int L, int k, int nwaves) {
  return (size_t)resident_lds(D, L, k, nwaves).total;
}

template <typename ET, int LPR>
static hipError_t launch_resident_g(const PassArgs& a, int g, dim3 grid, dim3 block, size_t lds,
                                    hipStream_t s) {
  const bool full = false && a.L == kResidentRows * g * (kWave / LPR);  // FULL variant disabled: spills
  switch (g * 2 + (full ? 1 : 0)) {
    case 2: resident_pass_kernel<ET, LPR, 1, false><<<grid, block, lds, s>>>(a); break;
    case 3: resident_pass_kernel<ET, LPR, 1, true><<<grid, block, lds, s>>>(a); break;
    case 4: resident_pass_kernel<ET, LPR, 2, false><<<grid, block, lds, s>>>(a); break;
    case 5: resident_pass_kernel<ET, LPR, 2, true><<<grid, block, lds, s>>>(a); break;
    case 8: resident_pass_kernel<ET, LPR, 4, false><<<grid, block, lds, s>>>(a); break;
    case 9: resident_pass_kernel<ET, LPR, 4, true><<<grid, block, lds, s>>>(a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <typename ET>
static hipError_t launch_resident_t(const PassArgs& a, int lpr, int g, dim3 grid, dim3 block,
                                    size_t lds, hipStream_t s) {
  switch (lpr) {
    case 4: return launch_resident_g<ET, 4>(a, g, grid, block, lds, s);
    case 8: return launch_resident_g<ET, 8>(a, g, grid, block, lds, s);
    case 16: return launch_resident_g<ET, 16>(a, g, grid, block, lds, s);
    case 32: return launch_resident_g<ET, 32>(a, g, grid, block, lds, s);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_resident_pass(const PassArgs& a, hipStream_t s) {
  const int lpr = lanes_per_row(a.D, a.esize);
  const int g = resident_group(a.D, a.esize, a.L);
  const int64_t nblocks = (int64_t)a.B * a.H * a.nseg;
  if (lpr == 0 || g == 0 || 2 * g != a.nwaves || nblocks <= 0 || nblocks > 0x7fffffffLL)
    return hipErrorInvalidValue;
  // per-lane input offsets are 32 bit: rows of one step must lie within 2 GiB
  if (a.st * (int64_t)(g * (kWave / lpr)) >= (1LL << 31)) return hipErrorInvalidValue;
  const size_t lds = resident_lds_bytes(a.D, a.L, a.k, 2 * g);
  if (lds > (size_t)kMaxLdsBytes) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nblocks), block(2 * g * kWave);
  return a.esize == 4 ? launch_resident_t<F32>(a, lpr, g, grid, block, lds, s)
                      : launch_resident_t<BF16>(a, lpr, g, grid, block, lds, s);
}

}  // namespace lagkv
