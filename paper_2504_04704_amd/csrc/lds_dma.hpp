// Asynchronous global -> LDS row loads (gfx950 global_load_lds_dwordx4), the assembly
// LDS accessors that go with them, and the streaming store used for output rows.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "row_ops.hpp"

#ifndef LAGKV_NT_STORE
#define LAGKV_NT_STORE 2     // output-row stores: 0 plain, 1 non-temporal, 2 non-temporal at workgroup scope
#endif
#ifndef LAGKV_SPLIT_RING
#define LAGKV_SPLIT_RING 8   // 1 KiB LDS slots per wavefront for the asynchronous row loads
#endif

namespace lagkv {

// 16-byte store of an output row slice.  The compacted cache is written once and not read
// again by this pass: non-temporal, workgroup scope ("sc0 nt").  Measured on the 128K
// workload: plain 17.4x ms, nt 17.35 ms, sc0 nt 17.26 ms, any sc1 form 17.4-17.9 ms.  The
// builtin offers nt only, hence the instruction is written out; the compiler does not count
// it in vmcnt, which can only make its later waits stricter, never weaker.
__device__ __forceinline__ void st16_out(char* p, const uint4& v) {
#if LAGKV_NT_STORE == 2
  typedef uint32_t vec4_t __attribute__((ext_vector_type(4)));
  const vec4_t q = {v.x, v.y, v.z, v.w};
  asm volatile("global_store_dwordx4 %0, %1, off sc0 nt" ::"v"(p), "v"(q) : "memory");
#elif LAGKV_NT_STORE == 1
  __builtin_nontemporal_store(v.x, reinterpret_cast<uint32_t*>(p));
  __builtin_nontemporal_store(v.y, reinterpret_cast<uint32_t*>(p) + 1);
  __builtin_nontemporal_store(v.z, reinterpret_cast<uint32_t*>(p) + 2);
  __builtin_nontemporal_store(v.w, reinterpret_cast<uint32_t*>(p) + 3);
#else
  st16(p, v);
#endif
}

// 16-byte load of a row slice that is read for the last time (the second read of a kept
// row): non-temporal, so that it does not displace lines other workgroups still need
// (17.30 -> 17.16 ms on the 128K workload).  The four loads merge into one dwordx4.
__device__ __forceinline__ uint4 ld16_last(const char* p) {
  const uint32_t* q = reinterpret_cast<const uint32_t*>(p);
  return make_uint4(__builtin_nontemporal_load(q), __builtin_nontemporal_load(q + 1),
                    __builtin_nontemporal_load(q + 2), __builtin_nontemporal_load(q + 3));
}

// ---- asynchronous global -> LDS row loads (gfx950 global_load_lds_dwordx4) -----------
// A wave-wide load writes lane l's 16 bytes to LDS at base + 16*l without passing
// through VGPRs and is tracked by the vector-memory counter (vmcnt, in order).  Each
// wavefront owns a ring of kRing slots of 1 KiB; a slot receives one step (64/LPR rows).
// The loads are issued kRing-2 steps ahead of the arithmetic.  The LDS reads of landed
// slots and the variance stores are written in assembly with explicit counter waits so
// that they are not serialised behind the loads still in flight.
constexpr int kRing = LAGKV_SPLIT_RING;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

__device__ __forceinline__ uint32_t lds_offset(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}
// wait until at most PENDING vector-memory operations are outstanding, then read two
// landed 16-byte entries
template <int PENDING>
__device__ __forceinline__ void lds_read_pair_after(u32x4& a, u32x4& b, uint32_t la, uint32_t lb) {
  asm volatile(
      "s_waitcnt vmcnt(%4)\n\t"
      "ds_read_b128 %0, %2\n\t"
      "ds_read_b128 %1, %3\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a), "=&v"(b)
      : "v"(la), "v"(lb), "n"(PENDING)
      : "memory");
}
// The same with one base address and two immediate byte offsets (below 64 KiB): a kernel
// whose slots are compile-time constants then keeps one address register, not one per slot.
template <int PENDING, int OFFA, int OFFB>
__device__ __forceinline__ void lds_read_pair_after_at(u32x4& a, u32x4& b, uint32_t base) {
  static_assert(OFFA >= 0 && OFFA < 65536 && OFFB >= 0 && OFFB < 65536, "ds_read offset field");
  asm volatile(
      "s_waitcnt vmcnt(%3)\n\t"
      "ds_read_b128 %0, %2 offset:%4\n\t"
      "ds_read_b128 %1, %2 offset:%5\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(a), "=&v"(b)
      : "v"(base), "n"(PENDING), "n"(OFFA), "n"(OFFB)
      : "memory");
}
__device__ __forceinline__ void lds_store_f32(uint32_t addr, float v) {
  asm volatile("ds_write_b32 %0, %1" ::"v"(addr), "v"(v) : "memory");
}
__device__ __forceinline__ void lds_drain() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// The same asynchronous row load written out, for kernels that keep loads in flight across
// barriers: the compiler does not know of it and so never waits for it on its own (a load it
// knows of is drained at the next fence).  Lane l's 16 bytes at sbase + lane_off are written
// to LDS at lds_addr + 16*l; sbase and lds_addr are wave-uniform.  M0 carries the LDS address
// (M0 is a reserved register to the compiler: it holds nothing there across a statement and
// loads it again before each of its own uses, so the block need not - and cannot - name it as
// clobbered; the scalar copy of the base stands between the write of M0 and the load that
// reads it, which needs one wait state).
// The rows it loads are read exactly once by the kernel that uses it (the register-resident
// one), hence non-temporal: measured 14.39 against 14.64 ms on the 128K workload ("sc0 nt"
// the same, "sc1" no gain).
#ifndef LAGKV_DMA16_FLAGS
#define LAGKV_DMA16_FLAGS "nt"
#endif
__device__ __forceinline__ void dma_rows16(uint32_t lane_off, const char* sbase, uint32_t lds_addr) {
  uint64_t base;  // (see sgpr_base_note below; the copy is also the wait state after the write of M0)
  asm volatile(
      "s_mov_b32 m0, %3\n\t"
      "s_mov_b64 %0, %2\n\t"
      "global_load_lds_dwordx4 %1, %0 " LAGKV_DMA16_FLAGS
      : "=&s"(base)
      : "v"(lane_off), "s"(sbase), "s"(lds_addr)
      : "memory");
}

// Stores like st16_out (not known to the compiler) with a wave-uniform base and a 32-bit lane
// offset (one address register instead of two), 16 and 4 bytes.
// sgpr_base_note: a vector-memory instruction must not read a scalar register within five wait
// states of a VECTOR instruction that wrote it (v_readlane / v_readfirstlane - which is how the
// compiler brings back a base address it had to park in a vector register).  The compiler
// inserts those wait states for its own instructions but cannot see into an asm block, so a
// base handed to these blocks is first copied by a SCALAR move (interlocked in hardware on its
// read side, and a scalar write needs no wait before a vector-memory read): without the copy
// the store could go out with a stale half of its address.
__device__ __forceinline__ void st16_out_at(char* sbase, uint32_t voff, const uint4& v) {
  typedef uint32_t vec4_t __attribute__((ext_vector_type(4)));
  const vec4_t q = {v.x, v.y, v.z, v.w};
#ifndef LAGKV_STORE_AT_FLAGS
#define LAGKV_STORE_AT_FLAGS "sc0 nt"
#endif
  uint64_t base;
  asm volatile("s_mov_b64 %0, %3\n\tglobal_store_dwordx4 %1, %2, %0 " LAGKV_STORE_AT_FLAGS
               : "=&s"(base)
               : "v"(voff), "v"(q), "s"(sbase)
               : "memory");
}
// (Scores and positions: once per token, not per row slice - here the five wait states are
// simply spent, which holds whatever wrote the registers before.)
__device__ __forceinline__ void st4_out_at(void* sbase, uint32_t voff, uint32_t v) {
  asm volatile("s_nop 4\n\tglobal_store_dword %0, %1, %2" ::"v"(voff), "v"(v), "s"(sbase) : "memory");
}


}  // namespace lagkv
