// Device-side helpers shared by the gfx950 kernels of the DashAttention library:
// bf16 <-> fp32 bit conversions, wave64 cross-lane reductions (DPP + bpermute),
// MFMA operand vector types.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dash {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;

constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (inputs are finite here; NaN kept NaN).
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16_bits(lo) | (f32_to_bf16_bits(hi) << 16);
}

template <typename T> struct elem;   // element loads that widen to fp32
template <> struct elem<float> {
  static constexpr int kVec = 4;     // elements per 16 bytes
  __device__ static __forceinline__ float ld(const float* p) { return *p; }
  __device__ static __forceinline__ void st(float* p, float v) { *p = v; }
};
template <> struct elem<uint16_t> {
  static constexpr int kVec = 8;
  __device__ static __forceinline__ float ld(const uint16_t* p) { return bf16_bits_to_f32(*p); }
  __device__ static __forceinline__ void st(uint16_t* p, float v) { *p = (uint16_t)f32_to_bf16_bits(v); }
};

// ---- DPP moves (wave64, rows of 16 lanes) ---------------------------------
template <int CTRL> __device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xF, 0xF, true));
}
struct OpAdd { __device__ __forceinline__ float operator()(float a, float b) const { return a + b; } };
struct OpMax { __device__ __forceinline__ float operator()(float a, float b) const { return fmaxf(a, b); } };
// combine over the 16 lanes of a DPP row; every lane of the row gets the result
template <typename Op> __device__ __forceinline__ float row16_reduce(float v, Op op) {
  v = op(v, dpp_f<0xB1>(v));   // quad_perm [1,0,3,2]
  v = op(v, dpp_f<0x4E>(v));   // quad_perm [2,3,0,1]
  v = op(v, dpp_f<0x141>(v));  // row_half_mirror
  v = op(v, dpp_f<0x140>(v));  // row_mirror
  return v;
}
// Whole-wave combine: DPP inside each 16-lane row, then the four row results are
// read as scalars (no LDS round trip).  The result is wave-uniform by
// construction, so every decision derived from it is identical in all lanes.
template <typename Op> __device__ __forceinline__ float wave_reduce(float v, Op op) {
  v = row16_reduce(v, op);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
  const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
  const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
  return op(op(r0, r1), op(r2, r3));
}
__device__ __forceinline__ float wave_sum(float v) {
  // materialise v first: a multiply contracted into the first DPP add would make
  // lane 0 of each row see a differently rounded partial sum than its partner
  asm volatile("" : "+v"(v));
  return wave_reduce(v, OpAdd());
}
__device__ __forceinline__ float wave_max(float v) { return wave_reduce(v, OpMax()); }
__device__ __forceinline__ float row16_sum(float v) { return row16_reduce(v, OpAdd()); }

__device__ __forceinline__ uint32_t lane_id() { return threadIdx.x & 63u; }

}  // namespace dash
