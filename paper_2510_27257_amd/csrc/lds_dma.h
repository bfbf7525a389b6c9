// Direct-to-LDS loads and explicitly waited LDS reads for gfx950 (shared by the GEMM and attention kernels).
//
// The compiler neither tracks the completion of direct-to-LDS loads nor may it order LDS reads behind
// them (through builtins it would wait for vmcnt(0) before every transposing read), so kernels that
// pipeline such loads issue their LDS reads as inline assembly and place the waits themselves:
//   v = lds_read_*(addr);  ...  lds_wait<N>();  lds_tie(v);  use(v);
#pragma once
#include "common.h"

namespace {

typedef unsigned u32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));
typedef void __attribute__((address_space(3))) * lptr_t;

// The result of these reads is valid only after lds_wait<N>() + lds_tie() on the destination.
template <int OFF>
__device__ __forceinline__ u32x4_t lds_read_b128(unsigned addr) {
  u32x4_t v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF, int HI>
__device__ __forceinline__ u32x4_t lds_read_tr16(unsigned addr) {
  u32x2_t lo, hi;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(lo) : "v"(addr), "n"(OFF));
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(hi) : "v"(addr), "n"(OFF + HI));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
}
// Waits until at most N LDS operations of this wave are outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void lds_wait() {
  asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N));
}
// Pins the fragments behind the preceding lds_wait: no use of them can be scheduled above it.
template <int NF>
__device__ __forceinline__ void lds_tie(u32x4_t (&f)[NF]) {
#pragma unroll
  for (int i = 0; i < NF; i++) asm volatile("" : "+v"(f[i]));
}

// One wave instruction: lane i copies 16 bytes from base + voff(lane) + soff to lds + 16*i (lds is wave-uniform).
// (Kept in a device function: the builtin is not callable where the host pass parses a kernel body.)
__device__ __forceinline__ void dma_load16(__amdgpu_buffer_rsrc_t rsrc, char *lds, unsigned voff, unsigned soff) {
  __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lptr_t)lds, 16, voff, soff, 0, 0);
}

}  // namespace
