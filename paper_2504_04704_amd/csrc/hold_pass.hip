// Register-resident LagKV kernel for gfx950: the one-shot pass for rows of 256 bytes and
// lags of 128, 256 or 512 rows, in which every input row is read from memory exactly ONCE.
//
// A workgroup of eight wavefronts (four on K rows, four on V rows) walks a segment of one
// stream backwards, one BATCH of 512 rows at a time (1, 2 or 4 chunks).  The 32 row
// slices a lane handles in a batch stay in 128 of its registers until the selection is
// known; the kept rows are then stored from those registers, so the compaction reads
// nothing.  (A chunk of K and V is up to 256 KiB, more than the LDS of a CU but half of
// its register file: one workgroup per CU, two wavefronts per SIMD, 256 registers each.)
//
// With a single workgroup on a CU nothing else hides its selection, so the memory stream
// is kept going from inside:
//   * rows arrive through a per-wavefront LDS ring filled by asynchronous global->LDS loads
//     that run a fixed number of steps AHEAD of the arithmetic, across batch borders: while
//     a batch is selected, the first steps of the next batch are in flight;
//   * the stores of a batch's kept rows are deferred into the next batch's sweep: slice s
//     of the old batch is stored right before slice s of the new batch replaces it.
// Per batch:
//   1. sweep, the batch's chunks from the LAST one down to the first (the order of the whole
//      walk): per slice, store the previous batch's slice if kept, take the new slice from
//      the ring, fold it into the per-channel min/max of its chunk (Eq. 7-8) and - the
//      reference of a chunk being the chunk swept just before it - compute the token's
//      variance (Eq. 9-10) right away, in one sweep over its channels (token_var_fast; a
//      chunk outside that form's error bound is redone in two passes from the registers).
//      At the end of a chunk the wavefront parks its partial statistics in LDS; behind a
//      barrier one thread per channel combines them and publishes what the variance of the
//      next chunk needs, which every lane then only reads;
//                                                                        -- barrier --
//   2. only for Eq. 14-15, where a chunk is its own reference: a second sweep over the
//      registers computes the variances once the chunk's statistics are complete;
//                                                                        -- barrier --
//   3. chunk softmax, K+V sum and top-k (Eq. 10-11): all wavefronts together for a
//      512-row chunk, one wavefront per chunk otherwise; original positions are written.
//                                                                        -- barrier --
// All vector-memory traffic of the loop is issued from assembly with explicit counter
// waits (the compiler sees none of it and therefore never drains it at a barrier).
#include "lagkv_internal.hpp"
#include "lds_dma.hpp"
#include "row_ops.hpp"
#include "wave_ops.hpp"
#include "wg_select.hpp"

namespace lagkv {

constexpr int kHoldSteps = 32;   // row slices a lane keeps per batch
constexpr int kHoldWaves = 8;

// Ring slots (1 KiB steps) per wavefront: as many as the LDS holds beside the statistics.
__host__ __device__ constexpr int hold_ring(int C, bool local) { return local && C > 2 ? 8 : 16; }
// Parked statistics: one slot per chunk of a batch for Eq. 14-15 (read after the sweep), two
// that alternate from chunk to chunk for Eq. 7-8 (a chunk reads the one before it).
__host__ __device__ constexpr int hold_stat_slots(int C, bool local) { return local ? C : 2; }

struct HoldLds {
  int off_vK, off_vV, off_slot, off_list, off_sel, off_stat, off_ref, off_ring, total;  // bytes
};
// rows: rows per batch; C: chunks per batch
__host__ __device__ inline HoldLds hold_lds(int D, int rows, int k, int C, bool local) {
  HoldLds l;
  const int kp = (k + 3) & ~3;
  l.off_vK = 0;
  l.off_vV = rows * 4;
  l.off_slot = 2 * rows * 4;                 // int32 [rows]: output slot within the chunk, or -1
  l.off_list = 3 * rows * 4;                 // uint32 [C][kp]
  l.off_sel = l.off_list + C * kp * 4;
  l.off_stat = (l.off_sel + group_sel_bytes() + 15) & ~15;   // float [slot][wave][mn|mx][D]
  // float [chunk of the batch (Eq. 14-15) | 1][K|V][iv|sh][D]
  l.off_ref = l.off_stat + hold_stat_slots(C, local) * kHoldWaves * 2 * D * 4;
  l.off_ring = (l.off_ref + (local ? C : 1) * 4 * D * 4 + 1023) & ~1023;
  l.total = l.off_ring + kHoldWaves * hold_ring(C, local) * 1024;
  return l;
}

// One-off 16-byte row loads before the loop, through a raw buffer descriptor (untyped
// 32-bit data format, no stride, range = the whole 32-bit offset space): scalar base, one
// 32-bit lane offset, scalar step offset.
typedef uint32_t buf_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 buf_ld16(const char* base, uint32_t lane_off, uint32_t step_off) {
  const __amdgpu_buffer_rsrc_t r =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<char*>(base), 0, 0xffffffff, 0x00020000);
  const buf_u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(r, lane_off, step_off, 0);
  return make_uint4(v.x, v.y, v.z, v.w);
}

// Workgroup barrier for LDS traffic only: waits for this wavefront's LDS operations, not for
// its vector-memory operations (a __syncthreads() carries a fence that may wait for those).
__device__ __forceinline__ void lds_barrier() {
  asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// f(integral_constant<int, I>) for I = BEGIN, BEGIN + STEP, ... < END
template <int BEGIN, int END, int STEP, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>{});
    static_for<BEGIN + STEP, END, STEP>(f);
  }
}

// NSC: steps (of R = 16 rows) per chunk: L = NSC * R; C = 32 / NSC chunks per batch.
// LOCAL: Eq. 14-15 (a chunk is its own reference) instead of Eq. 7-8.
template <typename ET, int NSC, bool LOCAL>
__global__ void __launch_bounds__(512, 2) hold_pass_kernel(const PassArgs a) {
  constexpr int LPR = 16;
  constexpr int VEC = ET::VEC;
  constexpr int RPW = kWave / LPR;
  constexpr int G = kHoldWaves / 2;
  constexpr int R = G * RPW;
  constexpr int C = kHoldSteps / NSC;
  constexpr int L = NSC * R;
  constexpr int E = (L + kWave - 1) / kWave;
  constexpr int NR = hold_ring(C, LOCAL);
  constexpr bool local = LOCAL;
  static_assert(kHoldSteps % NR == 0 && NR % 2 == 0, "a batch starts at ring slot 0");
  extern __shared__ float4 lds_raw[];
  char* lds = reinterpret_cast<char*>(lds_raw);
  const int tid = threadIdx.x, nthreads = blockDim.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k = a.k, S = a.S;
  const int kp = (k + 3) & ~3;
  const HoldLds lay = hold_lds(a.D, kHoldSteps * R, k, C, LOCAL);
  float* vK = reinterpret_cast<float*>(lds + lay.off_vK);
  float* vV = reinterpret_cast<float*>(lds + lay.off_vV);
  int32_t* slotmap = reinterpret_cast<int32_t*>(lds + lay.off_slot);
  uint32_t* list = reinterpret_cast<uint32_t*>(lds + lay.off_list);
  uint32_t* selbuf = reinterpret_cast<uint32_t*>(lds + lay.off_sel);
  float* statbuf = reinterpret_cast<float*>(lds + lay.off_stat);
  float* refbuf = reinterpret_cast<float*>(lds + lay.off_ref);

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
    copy_rows_kv<LPR>(kin, vin, a.st, kout, vout, rowbytes, S, LPR, tid, nthreads);
    if (iout)
      for (int i = tid; i < S; i += nthreads) iout[i] = i;
  }
  if (gather && seg == a.nseg - 1) {
    const int64_t w0 = S + a.n_s * L, o0 = S + a.n_s * k, nwin = a.T - w0;
    copy_rows_kv<LPR>(kin + w0 * a.st, vin + w0 * a.st, a.st, kout + o0 * rowbytes,
                      vout + o0 * rowbytes, rowbytes, nwin, LPR, tid, nthreads);
    if (iout)
      for (int64_t i = tid; i < nwin; i += nthreads) iout[o0 + i] = (int32_t)(w0 + i);
  }

  const int64_t p0 = (int64_t)seg * a.n_s / a.nseg;
  const int64_t p1 = (int64_t)(seg + 1) * a.n_s / a.nseg;
  const uint32_t lane_off = (uint32_t)(row0 * a.st) + (uint32_t)cl * 16u;
  const int64_t step_bytes = (int64_t)R * a.st;
  // this wavefront's ring (wave-uniform LDS byte address) and the lane's 16 bytes in a slot
  const uint32_t ring_base =
      __builtin_amdgcn_readfirstlane(lds_offset(lds + lay.off_ring) + (uint32_t)wave * (NR * 1024u));
  const uint32_t ring_lane = ring_base + (uint32_t)lane * 16u;

  uint4 hold[kHoldSteps];
  TStats<VEC> acc;
  // The variances are computed in one sweep over a token's channels (token_var_fast) from
  // these statistics; where that is not accurate enough (see its bound) the whole chunk's
  // are computed again from the rows in the registers, in two passes.
  TRefFast<VEC> rf;
  float vmin = 0.f, qmax = 0.f;  // smallest variance, largest sum of squares of a chunk's tokens
  // Eq. 7-8: the two statistics slots alternate; `qc` is the slot that holds the statistics
  // of the chunk swept last, the reference of the next one.  (A wavefront parks into the
  // other slot only after it has read this one, and nobody reads that other slot again
  // before the barrier that follows the park.)
  int qc = 0;

  // reduce acc over the four row groups of the wavefront and park it in statistics slot
  // `slot`.  The reduction scatters: in the exchange across 16 lanes one side keeps the
  // minima and the other the (negated) maxima, in the exchange across 32 lanes each side
  // keeps half of the channels, so that 12 (not 32) values cross lanes and every lane ends
  // up storing VEC/2 finished values.
  auto park = [&](int slot) __attribute__((always_inline)) {
    constexpr int H = VEC / 2;
    const bool hi16 = (lane & 16) != 0, hi32 = (lane & 32) != 0;
    float keep[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
      const float lo = acc.mn[j], nhi = -acc.mx[j];
      keep[j] = fminf(hi16 ? nhi : lo, __shfl_xor(hi16 ? lo : nhi, 16));
    }
    float fin[H];
#pragma unroll
    for (int i = 0; i < H; ++i)
      fin[i] = fminf(hi32 ? keep[H + i] : keep[i], __shfl_xor(hi32 ? keep[i] : keep[H + i], 32));
    float* w = statbuf + ((size_t)slot * kHoldWaves + wave) * 2 * a.D + (hi16 ? a.D : 0) + cl * VEC + (hi32 ? H : 0);
#pragma unroll
    for (int i = 0; i < H; ++i) w[i] = hi16 ? -fin[i] : fin[i];
  };
  // statistics in slot `slot`, folded over the wavefronts of this tensor
  auto folded_stats = [&](int slot, TStats<VEC>& f) __attribute__((always_inline)) {
    f.reset();
#pragma unroll
    for (int g = 0; g < G; ++g) {
      const float* rd = statbuf + ((size_t)slot * kHoldWaves + tensor * G + g) * 2 * a.D + cl * VEC;
#pragma unroll
      for (int j = 0; j < VEC; ++j) {
        f.mn[j] = fminf(f.mn[j], rd[j]);
        f.mx[j] = fmaxf(f.mx[j], rd[j + a.D]);
      }
    }
  };
  auto folded = [&](int slot, TRef<VEC>& out) __attribute__((always_inline)) {
    TStats<VEC> f;
    folded_stats(slot, f);
    out.from(f);
  };

  // The statistics every wavefront has parked in `slot` are combined and turned into the form
  // token_var_fast takes ONCE, by one thread per channel, instead of by every lane where it
  // needs them (which then only reads its 16 values from `out`).  To be called by all
  // threads behind the barrier that follows the park; the result is read behind a later
  // barrier.
  auto publish_ref = [&](int slot, float* out) __attribute__((always_inline)) {
    int t = tid;
    asm volatile("" : "+v"(t));  // (addresses worked out here, not kept in registers across the sweep)
    if (t < 2 * a.D) {
      const int tn = t >= a.D ? 1 : 0, ch = t - tn * a.D;
      float mn = INFINITY, mx = -INFINITY;
#pragma unroll
      for (int g = 0; g < G; ++g) {
        const float* rd = statbuf + ((size_t)slot * kHoldWaves + tn * G + g) * 2 * a.D + ch;
        mn = fminf(mn, rd[0]);
        mx = fmaxf(mx, rd[a.D]);
      }
      const float iv = inv_range(mn, mx);
      out[(tn * 2) * a.D + ch] = iv;
      out[(tn * 2 + 1) * a.D + ch] = fmaf(-mn, iv, -0.5f);
    }
  };

  if constexpr (!local) {
    // statistics of the chunk after the segment: the first reference
    const char* first = tin + (S + p1 * L) * a.st;
#pragma unroll
    for (int j = 0; j < NSC; ++j) hold[j] = buf_ld16(first, lane_off, (uint32_t)(j * step_bytes));
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
    park(qc);
  }
  // Everything the compiler knows to be in flight (the copies and loads above) is drained
  // here, once; inside the loop it sees no vector-memory operation at all.
  __syncthreads();
  if constexpr (!local) {
    publish_ref(qc, refbuf);
    __syncthreads();
  }

  // A batch is consumed in the order u = 0, 2, ... of "consumption indices": index u is step
  // u % NSC of chunk C - 1 - u / NSC of the batch, i.e. step s_of(u) in position order.  The
  // FIRST batch of a segment takes the chunks that do not fill a batch (its lowest chunk
  // numbers; its first live index is kHoldSteps - nsb), all later ones are full.  The ring
  // slot of index u is u % NR.
  int nsb = (int)((p1 - p0 - 1) % C + 1) * NSC;         // steps of the current batch
  int64_t pb = p1 - nsb / NSC;                          // its first chunk
  int seg_left = (int)(p1 - p0) * NSC;                  // steps of the segment not yet swept ...
  int dma_left = seg_left;                              // ... and not yet asked for
  // The loads follow the consumption order with one running address: a step further after
  // every load and, after the last step of a chunk, back to the first step of the chunk
  // before it - which is the next one to sweep, in this batch or in the one after it.
  const char* dma_ptr = tin + (S + (p1 - 1) * L) * a.st;
  const int64_t chunk_back = 2 * (int64_t)NSC * step_bytes;
  // load of the next index, which sits `pos` steps into its chunk, into ring slot `slot`
  auto dma_next = [&](int pos, int slot) __attribute__((always_inline)) {
    if (dma_left > 0) {
      dma_rows16(lane_off, dma_ptr, ring_base + (uint32_t)slot * 1024u);
      dma_ptr += step_bytes;
      if (pos == NSC - 1) dma_ptr -= chunk_back;
      --dma_left;
    }
  };
  {
    const int u0 = kHoldSteps - nsb;
#pragma unroll
    for (int j = 0; j < NR; ++j) dma_next(j % NSC, (u0 + j) % NR);
  }

  char* prev_dst = tout;                                // output of the previous batch's first chunk
  const int64_t kbytes = (int64_t)k * rowbytes;
  int prev_nsb = 0;                                     // steps of the previous batch still to be stored

  // kept slices s, s+1 of the previous batch -> output (chunk c of that batch)
  auto store_prev = [&](int s, int c) __attribute__((always_inline)) {
    char* dst = prev_dst + (int64_t)c * kbytes;  // wave-uniform
    const int sl0 = slotmap[s * R + row0], sl1 = slotmap[(s + 1) * R + row0];
    if (sl0 >= 0) st16_out_at(dst, (uint32_t)sl0 * (uint32_t)rowbytes + (uint32_t)coff, hold[s]);
    if (sl1 >= 0) st16_out_at(dst, (uint32_t)sl1 * (uint32_t)rowbytes + (uint32_t)coff, hold[s + 1]);
  };

  const float guard_scale = 256.f * (float)a.D * (float)a.D;
  // variances of this wavefront's rows of chunk c of the batch in the registers, two passes
  // over the channels, against the statistics in slot `slot` (the rare case, see above)
  auto redo_chunk = [&](auto c_tag, int slot, float& vmax) __attribute__((always_inline)) {
    constexpr int c = decltype(c_tag)::value;
    TRef<VEC> ref;
    folded(slot, ref);
#pragma unroll
    for (int j = 0; j < NSC; j += 2) {
      const int s = c * NSC + j;
      float x0[VEC], x1[VEC];
      // (copies made opaque to the compiler, so that it unpacks again here instead of keeping
      // the sweep's unpacked rows alive in registers)
      uint4 t0 = hold[s], t1 = hold[s + 1];
      asm volatile("" : "+v"(t0.x), "+v"(t0.y), "+v"(t0.z), "+v"(t0.w));
      asm volatile("" : "+v"(t1.x), "+v"(t1.y), "+v"(t1.z), "+v"(t1.w));
      unpack<ET>(t0, x0);
      unpack<ET>(t1, x1);
      const float v0 = token_var<LPR, VEC>(x0, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
      const float v1 = token_var<LPR, VEC>(x1, ref.mn, ref.iv, ref.bias, inv_D, inv_dof);
      vmax = fmaxf(fmaxf(vmax, v0), v1);
      if (cl == 0) {
        myvar[s * R + row0] = v0;
        myvar[(s + 1) * R + row0] = v1;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  while (seg_left > 0) {
    const int cb = nsb / NSC;  // chunks of this batch (the first batch of a segment may be short)
    float vmax = 0.f;  // largest variance this wavefront has computed in this batch
    // (every lane of a row holds the row's variance: the four rows through scalar registers)
    auto post_vmax = [&]() __attribute__((always_inline)) {
      const float m = fmaxf(fmaxf(rl_f(vmax, 0), rl_f(vmax, 16)), fmaxf(rl_f(vmax, 32), rl_f(vmax, 48)));
      if (lane == 0) reinterpret_cast<float*>(selbuf)[kGroupSelPremax + wave] = m;
    };

    // 1. sweep (unrolled over the pairs of steps; u, c and s are compile-time constants)
    static_for<0, kHoldSteps, 2>([&](auto step_tag) __attribute__((always_inline)) {
      constexpr int u = decltype(step_tag)::value;
      constexpr int c = C - 1 - u / NSC;
      constexpr int s = c * NSC + u % NSC;
      if constexpr (u % NSC == 0) {
        acc.reset();
        if constexpr (!local) {
          if (c < cb) {  // reference: the chunk swept last (by now parked by every wavefront)
            rf.load(refbuf + (tensor * 2) * a.D + cl * VEC, refbuf + (tensor * 2 + 1) * a.D + cl * VEC);
            vmin = rf.wide ? -1.f : INFINITY;
            qmax = 0.f;
          }
        }
      }
      // The two wavefronts of a SIMD (w and w + G) compete for its issue slots and the
      // older one wins every tie, which lets it finish its sweep a quarter earlier and then
      // wait at the barrier.  Giving the younger one the higher priority on every other
      // pair of steps evens the two out.
      if (wave >= G) __builtin_amdgcn_s_setprio((u / 2) % 2 == 0 ? 1 : 0);
      if (gather && s < prev_nsb) store_prev(s, c);
      if (c < cb) {
        // Indices u and u+1 have landed once at most NR-2 younger loads are pending (the
        // stores issued in between only make this wait stricter: operations complete in
        // order, and how many stores there were depends on the data); for the last steps of
        // the segment fewer loads were issued, so everything is waited for.
        u32x4 qa, qb;
        constexpr int oa = (u % NR) * 1024, ob = ((u + 1) % NR) * 1024;
        if (seg_left >= NR) lds_read_pair_after_at<NR - 2, oa, ob>(qa, qb, ring_lane);
        else lds_read_pair_after_at<0, oa, ob>(qa, qb, ring_lane);
        seg_left -= 2;
        // the two slots are free again: the loads NR indices ahead, into the next batch if need be
        constexpr int t = u + NR;
        dma_next(t % NSC, t % NR);
        dma_next((t + 1) % NSC, (t + 1) % NR);
        hold[s] = make_uint4(qa.x, qa.y, qa.z, qa.w);
        hold[s + 1] = make_uint4(qb.x, qb.y, qb.z, qb.w);
        float x0[VEC], x1[VEC];
        unpack<ET>(hold[s], x0);
        unpack<ET>(hold[s + 1], x1);
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
          acc.mn[i] = fminf(fminf(acc.mn[i], x0[i]), x1[i]);
          acc.mx[i] = fmaxf(fmaxf(acc.mx[i], x0[i]), x1[i]);
        }
        pin(acc);
        if constexpr (!local) {
          float q0, q1;
          const float v0 = token_var_fast<LPR, VEC>(x0, rf.iv, rf.sh, inv_D, inv_dof, q0);
          const float v1 = token_var_fast<LPR, VEC>(x1, rf.iv, rf.sh, inv_D, inv_dof, q1);
          vmax = fmaxf(fmaxf(vmax, v0), v1);
          vmin = fminf(fminf(vmin, v0), v1);
          qmax = fmaxf(fmaxf(qmax, q0), q1);
          asm volatile("" : "+v"(vmin), "+v"(qmax), "+v"(vmax));  // evaluated here, not collected at the end
          if (cl == 0) {
            myvar[s * R + row0] = v0;
            myvar[(s + 1) * R + row0] = v1;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);  // keep the pairs in order: interleaving them costs registers
      if constexpr ((u + 2) % NSC == 0) {
        if (c < cb) {
          if constexpr (local) {
            park(c);
          } else {
            const bool redo = __any(!(guard_scale * vmin >= qmax * qmax));
            park(qc ^ 1);
            qc ^= 1;
            if (redo) {  // (after the park: the running statistics are out of the registers)
              if constexpr (C == 1) vmax = 0.f;
              redo_chunk(std::integral_constant<int, c>{}, qc ^ 1, vmax);
            }
            // the next chunk of the batch takes these statistics at its first step
            if constexpr (c > 0) {
              lds_barrier();
              publish_ref(qc, refbuf);
              lds_barrier();
            }
          }
        }
      }
    });
    if constexpr (!local && C == 1) post_vmax();
    lds_barrier();
    if constexpr (!local) publish_ref(qc, refbuf);  // read by the next sweep, behind the barriers of the selection
    // 2. Eq. 14-15: variances of every chunk against its own statistics.  Nothing overlaps
    // this sweep (the ring is full long before it ends), so it uses the short one-sweep
    // variance and falls back on the two-pass form where that one is not accurate enough.
    if constexpr (local) {
#pragma unroll
      for (int c = 0; c < C; ++c)
        if (c < cb) publish_ref(c, refbuf + c * 4 * a.D);
      lds_barrier();
      static_for<0, C, 1>([&](auto c_tag) __attribute__((always_inline)) {
        constexpr int c = decltype(c_tag)::value;
        if (c < cb) {
          const float* rb = refbuf + c * 4 * a.D;
          rf.load(rb + (tensor * 2) * a.D + cl * VEC, rb + (tensor * 2 + 1) * a.D + cl * VEC);
          // smallest variance and largest sum of squares of this wavefront's tokens
          vmin = rf.wide ? -1.f : INFINITY;
          qmax = 0.f;
#pragma unroll
          for (int j = 0; j < NSC; j += 2) {
            const int s = c * NSC + j;
            float x0[VEC], x1[VEC];
            // (copies made opaque to the compiler, so that it unpacks again here instead of
            // keeping the first sweep's unpacked rows alive in registers)
            uint4 t0 = hold[s], t1 = hold[s + 1];
            asm volatile("" : "+v"(t0.x), "+v"(t0.y), "+v"(t0.z), "+v"(t0.w));
            asm volatile("" : "+v"(t1.x), "+v"(t1.y), "+v"(t1.z), "+v"(t1.w));
            unpack<ET>(t0, x0);
            unpack<ET>(t1, x1);
            float q0, q1;
            const float v0 = token_var_fast<LPR, VEC>(x0, rf.iv, rf.sh, inv_D, inv_dof, q0);
            const float v1 = token_var_fast<LPR, VEC>(x1, rf.iv, rf.sh, inv_D, inv_dof, q1);
            vmax = fmaxf(fmaxf(vmax, v0), v1);
            vmin = fminf(fminf(vmin, v0), v1);
            qmax = fmaxf(fmaxf(qmax, q0), q1);
            asm volatile("" : "+v"(vmin), "+v"(qmax), "+v"(vmax));  // evaluated here, not collected at the end
            if (cl == 0) {
              myvar[s * R + row0] = v0;
              myvar[(s + 1) * R + row0] = v1;
            }
            __builtin_amdgcn_sched_barrier(0);
          }
          // the rare chunk with a token outside the bound: all of this wavefront's rows again,
          // two passes over the channels
          if (__any(!(guard_scale * vmin >= qmax * qmax))) {
            if constexpr (C == 1) vmax = 0.f;
            redo_chunk(c_tag, c, vmax);
          }
        }
      });
      if constexpr (C == 1) post_vmax();
      lds_barrier();
    }
    // 3. scores and selection
    if constexpr (C == 1) {
      // (the kept tokens' original positions go out from the selection itself)
      group_score_select<true>(vK, vV, L, k, gather, sout ? sout + pb * L : nullptr, selbuf, list, slotmap, tid,
                               nthreads, iout ? iout + S + pb * k : nullptr, (uint32_t)(S + pb * L));
    } else {
      if (wave < cb)
        wave_score_select<E>(vK + wave * L, vV + wave * L, L, k, gather, sout ? sout + (pb + wave) * L : nullptr,
                             list + wave * kp, slotmap + wave * L, lane);
    }
    lds_barrier();
    if (C > 1 && iout)
      for (int i = tid; i < cb * k; i += nthreads) {
        const int c = i / k, j = i - c * k;  // (positions of a batch's chunks are contiguous in the output)
        st4_out_at(iout + S + pb * k, (uint32_t)i * 4u, (uint32_t)(S + (pb + c) * L + list[c * kp + j]));
      }
    // The kept rows stay in the registers; the next sweep (or the flush below) stores them.
    // The next batch rewrites the statistics and variances (last read before the barrier
    // above) during its sweep, the slot map and the lists only after its own first barrier.
    prev_dst = tout + (S + pb * k) * rowbytes;
    prev_nsb = nsb;
    pb -= C;
    nsb = kHoldSteps;
  }
  static_for<0, kHoldSteps, 2>([&](auto step_tag) __attribute__((always_inline)) {
    constexpr int s = decltype(step_tag)::value;
    if (gather && s < prev_nsb) store_prev(s, s / NSC);
  });
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
  if (lpr != 16 || row_units(D, esize) != 16) return false;  // rows of exactly 256 bytes
  const int nsc = hold_nsc(L, lpr);
  if (!nsc) return false;
  const int R = (kHoldWaves / 2) * (kWave / lpr);
  return (size_t)hold_lds(D, kHoldSteps * R, k, kHoldSteps / nsc, true).total <= kHoldMaxLds &&
         (size_t)hold_lds(D, kHoldSteps * R, k, kHoldSteps / nsc, false).total <= kHoldMaxLds;
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
    case 8: return launch_hold_one(hold_pass_kernel<ET, 8, LOCAL>, a, grid, lds, s);
    case 16: return launch_hold_one(hold_pass_kernel<ET, 16, LOCAL>, a, grid, lds, s);
    case 32: return launch_hold_one(hold_pass_kernel<ET, 32, LOCAL>, a, grid, lds, s);
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
  // per-lane offsets inside a step are 32 bit, and so are the step offsets of the first loads
  if (a.st * (int64_t)R * kHoldSteps >= (1LL << 31)) return hipErrorInvalidValue;
  const size_t lds = (size_t)hold_lds(a.D, kHoldSteps * R, a.k, kHoldSteps / nsc, a.variant == 1).total;
  const dim3 grid((unsigned)nblocks);
  if (a.esize == 4) return launch_hold_t<F32>(a, nsc, grid, lds, s);
  return a.f16 ? launch_hold_t<F16>(a, nsc, grid, lds, s) : launch_hold_t<BF16>(a, nsc, grid, lds, s);
}

}  // namespace lagkv
