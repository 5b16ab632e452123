// Pieces shared by the kernels that feed the bf16 matrix cores through direct global-to-LDS
// loads (syrk_bf16.h, gemm_f16x2.h).
//
// global_load_lds_dwordx4 writes the 16 bytes of lane i at LDS address M0 + 16 i: a wavefront
// fills 1 KiB of consecutive LDS, each lane choosing its own global address.  The compiler
// cannot tell the LDS stages of a software pipeline apart and waits for every outstanding
// load before the first LDS read it sees, so the LDS reads of the main loops are issued as
// inline assembly and every wait is written out: LDS_DMA_WAIT_VM(n) lets n vector-memory
// operations stay outstanding (they complete in order), and each read group carries its own
// s_waitcnt lgkmcnt, with the registers it makes valid as operands so that no use can be
// scheduled ahead of it.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace shampoo {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;
typedef const __attribute__((address_space(1))) void glb_void;

// a wave-uniform pointer, held in scalar registers
__device__ __forceinline__ const char *uniform_ptr(const void *p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return reinterpret_cast<const char *>(((uint64_t)hi << 32) | lo);
}

// 16 bytes from LDS byte address `addr` + imm (imm: compile-time, below 65536)
#define LDS_DS_READ_B128(dst, addr, imm) asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(imm) : "memory")
// s_waitcnt vmcnt(n) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the other counters at their maxima)
#define LDS_DMA_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (((n) >> 4) << 14) | (7 << 4) | (15 << 8))
#define LDS_SCHED_BARRIER() __builtin_amdgcn_sched_barrier(0)

}  // namespace shampoo
