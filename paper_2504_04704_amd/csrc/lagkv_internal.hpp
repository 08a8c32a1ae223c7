// Internal interface between the C-ABI host layer (lagkv_api.hip) and the kernel
// launchers (split_pass.hip, append_pass.hip, staged_pass.hip).  Not part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lagkv.h"

namespace lagkv {

// Workspace bytes of one lagkv_compress call, and lagkv_compress with an explicit workspace
// (both defined in lagkv_api.hip).
size_t compress_workspace_need(const lagkv_params* p, int64_t T);
int compress_with_workspace(const lagkv_params* p, const void* K, const void* V, int64_t T,
                            void* K_out, void* V_out, int32_t* idx_out, float* scores_out, void* ws,
                            size_t ws_bytes, void* hip_stream);

// One compression pass over [streams] caches.  Strides are in BYTES here.
struct PassArgs {
  const char* K;
  const char* V;
  char* K_out;      // dense [streams, T_out, D] or nullptr (score only)
  char* V_out;
  int32_t* idx_out; // dense [streams, T_out] or nullptr
  float* scores;    // dense [streams, n_s*L] or nullptr
  int64_t sb, sh, st;  // input strides (bytes) of batch, head, row
  int64_t T;           // input rows per stream
  int64_t T_out;       // output rows per stream
  int64_t n_s;         // scored chunks per stream (>= 1)
  int32_t B, H, D;
  int32_t S, L, k;
  int32_t esize;       // bytes per element (4 = fp32, 2 = bf16 or fp16)
  int32_t f16;         // 2-byte elements are IEEE binary16 (else bfloat16)
  int32_t ddof;
  int32_t variant;
  int32_t nseg;        // segments each stream is cut into (one-shot kernels)
  int32_t nwaves;      // wavefronts per workgroup (one-shot kernels)
  int32_t order;       // workgroup -> stream order (see stream_of)
  int32_t sel;         // selection mode (see wg_select.hpp)
};

// Which of n streams the i-th workgroup (or group of segment workgroups) takes.
//   0  i                               consecutive workgroups take consecutive streams
//   1  even streams first, then odd    the workgroups resident at one time span the whole tensor
//   2  i % 8 picks one eighth of the streams (n divisible by 8): workgroups are dealt to the
//      eight XCDs round-robin, so every XCD's L2 then sees one contiguous eighth
//   3  bit reversal of i (n a power of two): neighbours in time are far apart in memory
// Every order is a permutation of [0, n); orders whose precondition fails fall back to 0.
__host__ __device__ inline int64_t stream_of(int64_t i, int64_t n, int order) {
  if (order == 1) {
    const int64_t half = (n + 1) / 2;
    return i < half ? 2 * i : 2 * (i - half) + 1;
  }
  if (order == 2 && n % 8 == 0) return (i % 8) * (n / 8) + i / 8;
  if (order == 3 && n > 1 && (n & (n - 1)) == 0) {
    int bits = 0;
    while ((int64_t(1) << bits) < n) ++bits;
    int64_t r = 0;
    for (int b = 0; b < bits; ++b) r |= ((i >> b) & 1) << (bits - 1 - b);
    return r;
  }
  return i;
}

// In-place append + recursive compression of [streams] dense caches.
struct AppendArgs {
  char* K;             // [streams, capacity, D]
  char* V;
  int32_t* pos;        // [streams, capacity] or nullptr
  const char* K_new;   // [B,H,n_new,D] with strides below, or nullptr when n_new == 0
  const char* V_new;
  int64_t nsb, nsh, nst;  // strides (bytes) of K_new / V_new
  int64_t capacity;
  int64_t n_static;    // before the call
  int64_t n_tail;      // before the call (without the new rows)
  int64_t n_seen;      // before the call
  int64_t n_new;
  int64_t rounds;      // chunks to compress after the append (host arithmetic)
  int32_t B, H, D;
  int32_t S, L, k;
  int32_t esize, f16, ddof, variant;
  int32_t nwaves;
  int32_t sel;         // selection mode (see wg_select.hpp)
};

// True when the fused kernels can serve this row size / alignment.
bool fused_supported(int D, int esize, int64_t sb, int64_t sh, int64_t st, const void* K,
                     const void* V, const void* Ko, const void* Vo);
size_t fused_lds_bytes(int D, int L, int k, int nwaves);

// One-shot fused kernel (tensor-split streaming): nwaves in {2,4,8}.
size_t split_lds_bytes(int D, int esize, int L, int k, int nwaves);
hipError_t launch_split_pass(const PassArgs& a, hipStream_t s);

// One-shot register-resident kernel (every row read once): 256-byte rows, L in {128, 256, 512}.
bool hold_supported(int D, int esize, int L, int k);
hipError_t launch_hold_pass(const PassArgs& a, hipStream_t s);

hipError_t launch_fused_append(const AppendArgs& a, hipStream_t s);
// Single-round decode step (exactly one chunk completes; no intermediate append copy).
bool decode_step_supported(const AppendArgs& a);
hipError_t launch_decode_step(const AppendArgs& a, hipStream_t s);

// Three-kernel path (any D, any alignment).
hipError_t launch_staged_score(const PassArgs& a, int64_t row0, float* scores, hipStream_t s);
hipError_t launch_select(const float* scores, int64_t streams, int64_t n_s, int L, int k,
                         int64_t row0, int32_t* kept, hipStream_t s);
hipError_t launch_staged_gather(const PassArgs& a, const int32_t* kept, hipStream_t s);
size_t staged_score_lds_bytes(int D, int L);

// Dense output row `slot` of a stream <- input row src(slot):
//   slot <  n_pre            : pre0 + slot
//   slot <  n_pre + n_kept   : kept[stream][slot - n_pre]
//   else                     : post0 + (slot - n_pre - n_kept)
struct GatherMap {
  int64_t n_pre, pre0, n_kept, post0, n_out;
};
hipError_t launch_gather_rows(const char* src, int64_t sb, int64_t sh, int64_t st, int B, int H,
                              char* dst, int64_t rowbytes, int esize, const int32_t* kept,
                              int32_t* idx_out, const GatherMap& m, hipStream_t s);
// pos[stream][at + i] = first + i for i < n
hipError_t launch_iota_rows(int32_t* pos, int64_t streams, int64_t capacity, int64_t at, int64_t n,
                            int32_t first, hipStream_t s);

// dst[b,h,r,:] = src[b,h,r,:] for r < rows; strides in bytes, rowbytes contiguous.
hipError_t launch_copy_rows(const char* src, int64_t ssb, int64_t ssh, int64_t sst, char* dst,
                            int64_t dsb, int64_t dsh, int64_t dst_st, int B, int H, int64_t rows,
                            int64_t rowbytes, hipStream_t s);

constexpr int kMaxLdsBytes = 64 * 1024;

}  // namespace lagkv
