// Vector-memory requests whose completion the kernel tracks by hand (gfx950 only).
//
// The compiler's own wait insertion is exact only for requests it can see and, for direct
// global->LDS loads, falls back to waiting for everything.  Kernels that keep several requests
// in flight across loop iterations therefore issue them through inline assembly and wait with
// explicit counts.  Requests of a wave complete in the order they were issued, so "at most N
// outstanding" (s_waitcnt vmcnt(N)) means that all but the N youngest have completed; a wait with
// too small an N only waits longer, one with too large an N reads data that has not arrived.
// Every use of a register loaded this way must come after a tie() that follows the wait: the
// empty volatile asm makes the value depend on that point of the instruction stream.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace qasr {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));

// 64 lanes x 16 bytes from per-lane global addresses to LDS at lds_wave_base + 16 * lane
// (lds_wave_base must be wave-uniform).  Completion is counted by vmcnt.
// (m0 is written here and cannot be named as clobbered: to the compiler it is a reserved register,
// it refuses to honour such a clobber.  The kernels that use these loads index no register
// dynamically and send no messages, the compiler's own uses of m0; every such load sets m0 itself.)
__device__ __forceinline__ void direct_load16(const void* gptr, const unsigned char* lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(gptr), "s"(m0v) : "memory");
}
// The same load at device scope (sc1): it never hits in the vector cache of the compute unit, so it
// sees what other workgroups of the same XCD have stored (and the XCD's L2 has acknowledged) earlier
// in the same kernel.  A vector-cache invalidate that spares the L2 does not exist on this chip:
// `buffer_inv sc0` leaves stale lines in place and `buffer_inv sc1` also drops the L2's contents (15 us).
__device__ __forceinline__ void direct_load16_dev(const void* gptr, const unsigned char* lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off sc1"
               :: "v"(gptr), "s"(m0v) : "memory");
}
template <bool DEV>
__device__ __forceinline__ void direct_load16_scope(const void* gptr, const unsigned char* lds_wave_base) {
  if constexpr (DEV) direct_load16_dev(gptr, lds_wave_base);
  else direct_load16(gptr, lds_wave_base);
}

// One dword per active lane from per-lane global addresses to LDS at lds_wave_base + 4 * lane.
__device__ __forceinline__ void direct_load4(const void* gptr, const unsigned char* lds_wave_base) {
  const uint32_t m0v = __builtin_amdgcn_readfirstlane(
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)lds_wave_base);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :: "v"(gptr), "s"(m0v) : "memory");
}

// Global loads whose completion the kernel waits for by hand (wait_vm / tie below).  The
// compiler does not know that the result is still in flight, so every use has to come after a
// tie() that follows the wait.
__device__ __forceinline__ v4i gload16(const void* p) {
  v4i r;
  asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
// same, through a raw buffer resource: address = base + voff (per lane) + soff (wave-uniform)
__device__ __forceinline__ v4i bload16(v4i rsrc, uint32_t voff, uint32_t soff) {
  v4i r;
  asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(r) : "v"(voff), "s"(rsrc), "s"(soff) : "memory");
  return r;
}
__device__ __forceinline__ v4i make_rsrc(const void* base, uint32_t bytes) {
  const uint64_t a = (uint64_t)(uintptr_t)base;
  return (v4i){(int)(uint32_t)a, (int)(uint32_t)((a >> 32) & 0xffffu), (int)bytes, 0x00027000};
}
__device__ __forceinline__ int32_t gload4(const void* p) {
  int32_t r;
  asm volatile("global_load_dword %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
__device__ __forceinline__ int32_t gload_i8(const void* p) {   // one sign-extended byte
  int32_t r;
  asm volatile("global_load_sbyte %0, %1, off" : "=v"(r) : "v"(p) : "memory");
  return r;
}
template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}
// at most n vector-memory operations outstanding (n wave-uniform).  `s_waitcnt` takes its count as
// an immediate, so a run-time count selects among 33 instructions: a balanced tree of scalar
// comparisons, five on any path (a 33-way switch compiles to a long chain of branches and mask
// bookkeeping that the pipelined kernels would pay at every chunk).  Exact up to 32; above that,
// 32 (which is within the bound asked for).
template <int LO, int HI>
__device__ __forceinline__ void wait_vm_between(int n) {      // LO <= n < HI
  if constexpr (HI - LO == 1) {
    wait_vm<LO>();
  } else {
    constexpr int MID = (LO + HI) / 2;
    if (n < MID) wait_vm_between<LO, MID>(n);
    else wait_vm_between<MID, HI>(n);
  }
}
__device__ __forceinline__ void wait_vm_dyn(int n) {
  n = __builtin_amdgcn_readfirstlane(n);
  if (n >= 32) wait_vm<32>();
  else wait_vm_between<0, 32>(n < 0 ? 0 : n);
}
// makes every later use of v depend on this point of the (volatile-ordered) instruction stream
__device__ __forceinline__ void tie(v4i& v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void tie(int32_t& v) { asm volatile("" : "+v"(v)); }

}  // namespace qasr
