// Direct global -> LDS copies (buffer_load ... lds, gfx950) and the small vector
// types the bf16 Stage-2 kernels share.
#pragma once
#include "common.h"

namespace dash {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Buffer resource (raw, no stride) over `bytes` bytes at p: loads past the end
// return zero instead of touching memory.
__device__ __forceinline__ u32x4 make_rsrc(const void* p, int64_t bytes) {
  const uint64_t base = (uint64_t)p;
  u32x4 rs;
  rs[0] = __builtin_amdgcn_readfirstlane((uint32_t)base);
  rs[1] = __builtin_amdgcn_readfirstlane((uint32_t)(base >> 32) & 0xffffu);
  rs[2] = __builtin_amdgcn_readfirstlane((uint32_t)bytes);
  rs[3] = 0x00020000u;
  return rs;
}

// One wave copies 64 x 16 bytes from global memory straight into LDS: lane l
// fetches 16 bytes at resource base + voff (per lane) + soff (uniform) and they
// land at LDS byte address lds_addr (uniform) + 16 l.  The copy is counted by
// vmcnt; it is issued from assembly so that the compiler does not order later
// LDS reads of other slots behind it, and the caller waits with s_waitcnt vmcnt
// before the barrier that publishes the slot.
__device__ __forceinline__ void copy16_to_lds(u32x4 rsrc, uint32_t lds_addr, uint32_t voff, uint32_t soff) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :: "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// LDS byte address of a pointer into the workgroup's dynamic shared memory
__device__ __forceinline__ uint32_t lds_addr_of(const void* p) {
  return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const char*)p;
}

// Transposing LDS read (ds_read_b64_tr_b16): within each group of 16 lanes, lane
// s points at four consecutive 16-bit elements; lane i of the group receives
// element i % 4 of the four source lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.
// Two reads give one 8-element MFMA operand.
__device__ __forceinline__ bf16x8 lds_read_tr_pair(const char* lo_addr, const char* hi_addr) {
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(lo_addr));
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)(hi_addr));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

}  // namespace dash
