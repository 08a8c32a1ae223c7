// Register-resident LagKV kernel for gfx950: the one-shot pass for rows of 256 bytes and
// lags of 128, 256 or 512 rows, in which every input row is read from memory exactly ONCE.
//
// A workgroup of eight wavefronts (four on K rows, four on V rows) walks a segment of one
// stream backwards, one BATCH of 512 rows at a time (1, 2 or 4 chunks).  The 32 row
// slices a lane loads for a batch stay in 128 of its registers until the selection is
// known; the kept rows are then stored from those registers, so the compaction reads
// nothing.  (A chunk of K and V is up to 256 KiB, more than the LDS of a CU but half of
// its register file: one workgroup per CU, two wavefronts per SIMD, 256 registers each.)
// Per batch:
//   1. issue all 32 loads of the lane (32 KiB in flight per wavefront);
//   2. per chunk, fold the rows into per-channel min/max (Eq. 7-8) as they arrive, reduce
//      over the wavefront and park the partial result in LDS;            -- barrier --
//   3. per chunk, take the reference statistics (the next chunk's, Eq. 7-8, or the
//      chunk's own, Eq. 14-15) and compute every token's channel variance from the
//      registers (Eq. 9-10).  A batch of ONE chunk whose reference is the previous
//      batch's chunk does 2 and 3 in a single sweep;                     -- barrier --
//   4. chunk softmax, K+V sum and top-k (Eq. 10-11): all wavefronts together for a
//      512-row chunk, one wavefront per chunk otherwise;                 -- barrier --
//   5. store the kept rows from the registers, and their original positions.
#include "lagkv_internal.hpp"
#include "lds_dma.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"
#include "wg_select.hpp"

namespace lagkv {

constexpr int kHoldSteps = 32;   // row slices a lane keeps per batch
constexpr int kHoldWaves = 8;

// Row loads go through a raw buffer descriptor: the batch's first row is the (scalar) base,
// the lane's place in a step one 32-bit vector offset shared by all 32 loads, the step a
// scalar offset - no per-load 64-bit vector address, which is what lets 128 registers of
// row data and the arithmetic state fit a 256-register wavefront.
typedef uint32_t buf_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ __amdgpu_buffer_rsrc_t row_buffer(const char* base) {
  // untyped 32-bit data format, no stride, range = the whole 32-bit offset space
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, 0xffffffff, 0x00020000);
}
__device__ __forceinline__ uint4 buf_ld16(__amdgpu_buffer_rsrc_t r, uint32_t lane_off, uint32_t step_off) {
  const buf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, step_off, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

struct HoldLds {
  int off_vK, off_vV, off_slot, off_list, off_sel, off_stat, total;  // bytes
};
// rows: rows per batch; C: chunks per batch
__host__ __device__ inline HoldLds hold_lds(int D, int rows, int k, int C) {
  HoldLds l;
  const int kp = (k + 3) & ~3;
  l.off_vK = 0;
  l.off_vV = rows * 4;
  l.off_slot = 2 * rows * 4;                 // int32 [rows]: output slot within the chunk, or -1
  l.off_list = 3 * rows * 4;                 // uint32 [C][kp]
  l.off_sel = l.off_list + C * kp * 4;
  l.off_stat = (l.off_sel + group_sel_bytes() + 15) & ~15;   // float [2][C][wave][mn|mx][D]
  l.total = l.off_stat + 2 * C * kHoldWaves * 2 * D * 4;
  return l;
}

// NSC: steps (of R = 4 * 64/LPR rows) per chunk: L = NSC * R; C = 32 / NSC chunks per batch.
// LOCAL: Eq. 14-15 (a chunk is its own reference) instead of Eq. 7-8.
template <typename ET, int LPR, int NSC, bool LOCAL>
__global__ void __launch_bounds__(512, 2) hold_pass_kernel(const PassArgs a) {
  constexpr int VEC = ET::VEC;
  constexpr int RPW = kWave / LPR;
  constexpr int G = kHoldWaves / 2;
  constexpr int R = G * RPW;
  constexpr int C = kHoldSteps / NSC;
  constexpr int L = NSC * R;
  constexpr int E = (L + kWave - 1) / kWave;
  // one chunk per batch whose reference is the previous batch's chunk: a single sweep
  constexpr bool single = C == 1 && !LOCAL;
  constexpr bool local = LOCAL;
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = a.k, S = a.S;
  const int kp = (k + 3) & ~3;
  const HoldLds lay = hold_lds(a.D, kHoldSteps * R, k, C);
  float* vK = reinterpret_cast<float*>(lds + lay.off_vK);
  float* vV = reinterpret_cast<float*>(lds + lay.off_vV);
  int32_t* slotmap = reinterpret_cast<int32_t*>(lds + lay.off_slot);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  uint32_t* selbuf = reinterpret_cast<uint32_t*>(lds + lay.off_sel);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);

  const int tensor = wave >= G ? 1 : 0;  // 0: this wavefront handles K rows, 1: V rows
  const int gslot = wave - tensor * G;
  const int rl = lane / LPR, cl = lane % LPR;
  const int row0 = gslot * RPW + rl;
  constexpr int64_t rowbytes = (int64_t)LPR * 16;
  const int64_t coff = (int64_t)cl * 16;

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
  const uint32_t lane_off = (uint32_t)(row0 * a.st) + (uint32_t)cl * 16u;
  const uint32_t step_bytes = (uint32_t)(R * a.st);

  uint4 hold[kHoldSteps];
  TStats<VEC> acc;
  TRef<VEC> ref;
  // The partial statistics are double-buffered by batch parity: slot (q, c) holds chunk c of
  // the batches with parity q, so that chunk 0 of the previous batch - the reference of
  // this batch's top chunk - is still there while this batch parks its own.
  int q = 0;

  // reduce acc over the row groups of the wavefront and park it as chunk c's partial result
  auto park = [&](int c) __attribute__((always_inline)) {
#pragma unroll
    for (int m = LPR; m < kWave; m <<= 1) {
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        acc.mn[j] = fminf(acc.mn[j], __shfl_xor(acc.mn[j], m));
        acc.mx[j] = fmaxf(acc.mx[j], __shfl_xor(acc.mx[j], m));
      }
    }
    if (rl == 0) {
      float* w = statbuf + ((size_t)(q * C + c) * kHoldWaves + wave) * 2 * a.D + cl * VEC;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        w[j] = acc.mn[j];
        w[a.D + j] = acc.mx[j];
      }
    }
  };
  // statistics of chunk c of the batch of parity qq, folded over the wavefronts of this tensor
  auto folded = [&](int qq, int c, TRef<VEC>& out) __attribute__((always_inline)) {
    TStats<VEC> f;
    f.reset();
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float* rd = statbuf + ((size_t)(qq * C + c) * kHoldWaves + tensor * G + g) * 2 * a.D + cl * VEC;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        f.mn[j] = fminf(f.mn[j], rd[j]);
        f.mx[j] = fmaxf(f.mx[j], rd[j + a.D]);
      }
    }
    out.from(f);
  };

  if constexpr (!local) {
    // statistics of the chunk after the segment: the first reference
    const __amdgpu_buffer_rsrc_t rows = row_buffer(tin + (S + p1 * L) * a.st);
#pragma unroll
    for (int j = 0; j < NSC; ++j) hold[j] = buf_ld16(rows, lane_off, (uint32_t)j * step_bytes);
    acc.reset();
#pragma unroll
    for (int j = 0; j < NSC; ++j) {
      float x[VEC];
      unpack<ET>(hold[j], x);
#pragma unroll
      for (int i = 0; i < VEC; ++i) {
        acc.mn[i] = fminf(acc.mn[i], x[i]);
        acc.mx[i] = fmaxf(acc.mx[i], x[i]);
      }
    }
    q = 1;     // parked as chunk 0 of the batch "before" the first one
    park(0);
    q = 0;
    __syncthreads();
  }

  for (int64_t pe = p1; pe > p0;) {
    const int64_t pb = pe - C > p0 ? pe - C : p0;
    const int cb = (int)(pe - pb);  // chunks of this batch (the last batch of a segment may be short)
    const __amdgpu_buffer_rsrc_t rows = row_buffer(tin + (S + pb * L) * a.st);
    if constexpr (single) folded(q ^ 1, 0, ref);

    // 1. all loads of the batch
#pragma unroll
    for (int c = 0; c < C; ++c) {
      if (c < cb) {
#pragma unroll
        for (int j = 0; j < NSC; ++j) {
          const int s = c * NSC + j;
          hold[s] = buf_ld16(rows, lane_off, (uint32_t)s * step_bytes);
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);  // every load is issued before the first row is waited for
    // 2. per-channel min/max of every chunk (and, for a single chunk with a known
    // reference, the variances in the same sweep)
#pragma unroll
    for (int c = 0; c < C; ++c) {
      if (c < cb) {
        acc.reset();
#pragma unroll
        for (int j = 0; j < NSC; j += 2) {
          const int s = c * NSC + j;
          float x0[VEC], x1[VEC];
          unpack<ET>(hold[s], x0);
          unpack<ET>(hold[s + 1], x1);
#pragma unroll
          for (int i = 0; i < VEC; ++i) {
            acc.mn[i] = fminf(fminf(acc.mn[i], x0[i]), x1[i]);
            acc.mx[i] = fmaxf(fmaxf(acc.mx[i], x0[i]), x1[i]);
          }
          pin(acc);
          if constexpr (single) {
            const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
            const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
            if (cl == 0) {
              myvar[s * R + row0] = v0;
              myvar[(s + 1) * R + row0] = v1;
            }
          }
          __builtin_amdgcn_sched_barrier(0);  // keep the pairs in order: interleaving them costs registers
        }
        park(c);
      }
    }
    __syncthreads();
    // 3. variances of every chunk against its reference
    if constexpr (!single) {
#pragma unroll
      for (int c = 0; c < C; ++c) {
        if (c < cb) {
          if constexpr (local) folded(q, c, ref);
          else if (c + 1 < cb) folded(q, c + 1, ref);
          else folded(q ^ 1, 0, ref);
#pragma unroll
          for (int j = 0; j < NSC; j += 2) {
            const int s = c * NSC + j;
            float x0[VEC], x1[VEC];
            // (opaque to the compiler, so that it unpacks again here instead of keeping the
            // first sweep's unpacked rows alive in registers)
            asm volatile("" : "+v"(hold[s].x), "+v"(hold[s].y), "+v"(hold[s].z), "+v"(hold[s].w));
            asm volatile("" : "+v"(hold[s + 1].x), "+v"(hold[s + 1].y), "+v"(hold[s + 1].z), "+v"(hold[s + 1].w));
            unpack<ET>(hold[s], x0);
            unpack<ET>(hold[s + 1], x1);
            const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
            const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
            if (cl == 0) {
              myvar[s * R + row0] = v0;
              myvar[(s + 1) * R + row0] = v1;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
        }
      }
    }
    if constexpr (!single) __syncthreads();
    // 4. scores and selection
    if constexpr (C == 1) {
      group_score_select(vK, vV, L, k, gather, sout ? sout + pb * L : nullptr, selbuf, list, slotmap, tid,
                         nthreads);
    } else {
      if (wave < cb)
        wave_score_select<E>(vK + wave * L, vV + wave * L, L, k, gather, sout ? sout + (pb + wave) * L : nullptr,
                             list + wave * kp, slotmap + wave * L, lane);
    }
    __syncthreads();
    // 5. kept rows from the registers
    if (gather) {
#pragma unroll
      for (int c = 0; c < C; ++c) {
        if (c < cb) {
          char* dst = tout + (S + (pb + c) * k) * rowbytes + coff;
#pragma unroll
          for (int j = 0; j < NSC; ++j) {
            const int s = c * NSC + j;
            const int sl = slotmap[s * R + row0];
            if (sl >= 0) st16_out(dst + (int64_t)sl * rowbytes, hold[s]);
          }
        }
      }
      if (iout)
        for (int i = tid; i < cb * k; i += nthreads) {
          const int c = i / k, j = i - c * k;
          iout[S + (pb + c) * k + j] = (int32_t)(S + (pb + c) * L + list[c * kp + j]);
        }
    }
    pe = pb;
    q ^= 1;
    // no barrier here: the next batch writes the statistics and variances (last read before
    // the barrier above) before its first barrier, the slot map and the lists after it
  }
}

// ------------------------------------------------------------------------ host side
constexpr size_t kHoldMaxLds = 160 * 1024;

static int hold_nsc(int L, int lpr) {
  const int R = (kHoldWaves / 2) * (kWave / lpr);
  if (L % R) return 0;
  const int nsc = L / R;
  return (nsc == 8 || nsc == 16 || nsc == 32) ? nsc : 0;
}

bool hold_supported(int D, int esize, int L, int k) {
  const int lpr = lanes_per_row(D, esize);
  if (lpr != 16) return false;
  const int nsc = hold_nsc(L, lpr);
  if (!nsc) return false;
  const int R = (kHoldWaves / 2) * (kWave / lpr);
  return (size_t)hold_lds(D, kHoldSteps * R, k, kHoldSteps / nsc).total <= kHoldMaxLds;
}

template <typename K>
static hipError_t launch_hold_one(K kernel, const PassArgs& a, dim3 grid, size_t lds, hipStream_t s) {
  if (lds > 64 * 1024) {  // beyond the default dynamic LDS limit: opt in (idempotent)
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
  }
  kernel<<<grid, dim3(kHoldWaves * kWave), lds, s>>>(a);
  return hipGetLastError();
}

template <typename ET, bool LOCAL>
static hipError_t launch_hold_v(const PassArgs& a, int nsc, dim3 grid, size_t lds, hipStream_t s) {
  switch (nsc) {
    case 8: return launch_hold_one(hold_pass_kernel<ET, 16, 8, LOCAL>, a, grid, lds, s);
    case 16: return launch_hold_one(hold_pass_kernel<ET, 16, 16, LOCAL>, a, grid, lds, s);
    case 32: return launch_hold_one(hold_pass_kernel<ET, 16, 32, LOCAL>, a, grid, lds, s);
    default: return hipErrorInvalidValue;
  }
}
template <typename ET>
static hipError_t launch_hold_t(const PassArgs& a, int nsc, dim3 grid, size_t lds, hipStream_t s) {
  return a.variant == 1 ? launch_hold_v<ET, true>(a, nsc, grid, lds, s)
                        : launch_hold_v<ET, false>(a, nsc, grid, lds, s);
}

hipError_t launch_hold_pass(const PassArgs& a, hipStream_t s) {
  if (!hold_supported(a.D, a.esize, a.L, a.k) || a.variant == 2) return hipErrorInvalidValue;
  const int lpr = 16, nsc = hold_nsc(a.L, lpr), R = (kHoldWaves / 2) * (kWave / lpr);
  const int64_t nblocks = (int64_t)a.B * a.H * a.nseg;
  if (nblocks <= 0 || nblocks > 0x7fffffffLL || a.nseg < 1 || a.nseg > a.n_s) return hipErrorInvalidValue;
  // offsets inside a batch are 32 bit: its rows must lie within 2 GiB
  if (a.st * (int64_t)R * kHoldSteps >= (1LL << 31)) return hipErrorInvalidValue;
  const size_t lds = (size_t)hold_lds(a.D, kHoldSteps * R, a.k, kHoldSteps / nsc).total;
  const dim3 grid((unsigned)nblocks);
  if (a.esize == 4) return launch_hold_t<F32>(a, nsc, grid, lds, s);
  return a.f16 ? launch_hold_t<F16>(a, nsc, grid, lds, s) : launch_hold_t<BF16>(a, nsc, grid, lds, s);
}

}  // namespace lagkv
