// Device-side helpers shared by the kernels that stage operands HBM/L2 -> LDS with
// global_load_lds_dwordx4 and count their transfers by hand (gfx950).  Not installed.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace jk {
namespace dev {

// 16 bytes per lane straight from global memory into LDS (global_load_lds_dwordx4): lane l
// of the wave lands at lds_base + 16*l and fetches base + voff (a wave-uniform 64-bit base
// in scalar registers plus the lane's unsigned 32-bit byte offset).  Written as inline
// assembly so that the compiler does not know about the transfer: its own bookkeeping
// would make every later LDS read wait for ALL outstanding transfers, which would
// serialise a multi-stage ring.  The kernels order transfers and reads themselves
// (vmcnt waits + barriers).
__device__ __forceinline__ void dma16(const uint16_t* base, unsigned voff, unsigned lds_base) {
  const unsigned m = __builtin_amdgcn_readfirstlane(lds_base);  // wave-uniform by construction
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(m), "v"(voff), "s"(base)
               : "memory", "m0");
}

// A wave-uniform pointer, made so for the compiler (scalar registers)
__device__ __forceinline__ const uint16_t* uniform_ptr(const uint16_t* p) {
  const unsigned long long v = reinterpret_cast<unsigned long long>(p);
  const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
  const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
  return reinterpret_cast<const uint16_t*>(((unsigned long long)hi << 32) | lo);
}

// s_waitcnt immediate on gfx9 that waits for vmcnt <= n only: vmcnt sits in bits [3:0] and
// [15:14]; expcnt and lgkmcnt are left at their maxima
constexpr int vmcnt_imm(int n) { return ((n & 0xF) | ((n >> 4) << 14)) | 0x0F70; }

// wait until at most N of this wave's transfers are outstanding (they complete in issue order)
template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
  __builtin_amdgcn_s_waitcnt(vmcnt_imm(N));
  asm volatile("" ::: "memory");
}

// Stores that go through to memory at once (system scope: sc0 sc1), for results that
// nothing in the same kernel reads again.  An ordinary store leaves its line dirty in the
// XCD's L2, and the write-back of all such lines is part of the kernel's end: megabytes of
// results written in the last microsecond of a short kernel then lengthen it measurably.
typedef unsigned int store_u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int store_u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_through(void* dst, store_u32x4 v) {
  // (the wait state behind it: a vector instruction that overwrites the data registers of a store of more than
  // 64 bits must not be the very next one, and the compiler does not look for that hazard behind an asm statement)
  asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 0" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(void* dst, store_u32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1" ::"v"(dst), "v"(v) : "memory");
}
__device__ __forceinline__ void store_through(void* dst, unsigned int v) {
  asm volatile("global_store_dword %0, %1, off sc0 sc1" ::"v"(dst), "v"(v) : "memory");
}

}  // namespace dev
}  // namespace jk
