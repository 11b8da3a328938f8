// Asynchronous HBM -> LDS tile copies and transposing LDS reads shared by the GEMM and attention kernels (gfx950).
#pragma once
#include "common.h"

namespace mlm {

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) void glb_void_t;
typedef short v4s_t __attribute__((ext_vector_type(4)));
typedef short v8s_t __attribute__((ext_vector_type(8)));

// One wave-wide 16-byte-per-lane copy HBM -> LDS: lane t's 16 bytes land at lds_addr + 16 t (lds_addr is the
// wave-uniform LDS byte address, passed in M0).  Written as inline assembly so that the compiler's conservative
// "LDS DMA may alias any LDS read" rule does not turn every fragment read into s_waitcnt vmcnt(0); completion is
// tracked by hand with wait_vmcnt<> below.
__device__ __forceinline__ void dma16(const bf16* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
// Same with 4 bytes per lane: lane t's dword lands at lds_addr + 4 t (one 256-byte vector per wave instruction).
__device__ __forceinline__ void dma4(const float* g, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_addr), "v"(g) : "memory");
}
__device__ __forceinline__ uint32_t lds_offset_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const unsigned char*)p;
}

// s_waitcnt vmcnt(N) only (lgkmcnt / expcnt left at "no wait"): gfx9 encoding vmcnt[3:0] | expcnt<<4 | lgkm<<8 | vmcnt[5:4]<<14
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | (7 << 4) | (15 << 8) | ((N >> 4) << 14));
}

// ds_read_b64_tr_b16: within each group of 16 lanes, lane j supplies the address of 4 consecutive bf16 of row j/4
// (columns 4 (j%4) .. +3 of a 4 x 16 block) and lane i receives the 4 rows of column i of that block.
__device__ __forceinline__ v4s_t lds_read_tr16(const unsigned char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_t*)p);
}

}  // namespace mlm
