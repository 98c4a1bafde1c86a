// Block-mean summary of one chunk (Eq. 3 at the zero summary query; Alg. 1) by the first
// 256 threads of a workgroup: shared by the Stage-0 kernel and by the decode step's
// Stage-1 kernel, which summarises the chunk the current token completes.
#pragma once
#include "common.h"

namespace dash {

// sm: 2048 doubles of LDS.  Thread (r0, cg) sums the 16-byte column group cg of rows r0,
// r0 + rp, ... in fp64 (exact for 64..128 inputs of comparable magnitude), the partial sums
// are added per column in a fixed order and the mean is rounded once to fp32.  Ends with the
// store; contains one workgroup barrier, so all threads of the workgroup must call it (those
// from 256 up only take part in the barrier).
template <typename T>
__device__ __forceinline__ void kbar_block_mean(const T* __restrict__ k, float* __restrict__ kbar, double* sm,
                                                int block, int d, int t_c, int c, int r, int b, int h_kv,
                                                int64_t ks_b, int64_t ks_h, int64_t ks_t) {
  constexpr int VEC = elem<T>::kVec;
  const int cg_n = d / VEC;              // 16-byte column groups per row
  const int rp = 256 / cg_n;             // rows covered per pass
  if (threadIdx.x < 256) {
    const int cg = threadIdx.x % cg_n, r0 = threadIdx.x / cg_n;
    const T* base = k + b * ks_b + r * ks_h + (int64_t)c * block * ks_t + cg * VEC;
    double acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; e++) acc[e] = 0.0;
    for (int row = r0; row < block; row += rp) {
      const u32x4 raw = *reinterpret_cast<const u32x4*>(base + (int64_t)row * ks_t);
      if constexpr (VEC == 8) {
#pragma unroll
        for (int e = 0; e < 4; e++) {
          acc[2 * e] += (double)bf16_lo(raw[e]);
          acc[2 * e + 1] += (double)bf16_hi(raw[e]);
        }
      } else {
#pragma unroll
        for (int e = 0; e < 4; e++) acc[e] += (double)__uint_as_float(raw[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < VEC; e++) sm[r0 * d + cg * VEC + e] = acc[e];
  }
  __syncthreads();
  const int col = threadIdx.x;
  if (col < d) {
    double s = 0.0;
    for (int rr = 0; rr < rp; rr++) s += sm[rr * d + col];
    kbar[(((int64_t)b * h_kv + r) * t_c + c) * d + col] = (float)(s * (1.0 / (double)block));
  }
}

}  // namespace dash
