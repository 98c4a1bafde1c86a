// Stage 0: block-mean key summaries (Sec. 3.1, Eq. 3 with the summary query at
// its zero initial value, i.e. uniform pooling; Alg. 1).
//
// One workgroup per (chunk, kv-head, batch).  The chunk (block x d elements) is
// streamed once with 16-byte loads; sums are accumulated in fp64, which is exact
// for 64..128 bf16/fp32 inputs of comparable magnitude, so the fp32 result is
// the correctly rounded mean independent of summation order.
#include "common.h"
#include "dash_internal.h"

namespace dash {

template <typename T>
__global__ __launch_bounds__(256) void kbar_compress_kernel(
    const T* __restrict__ k, float* __restrict__ kbar, int block,
    int d, int t_c, int first_chunk, int64_t ks_b, int64_t ks_h, int64_t ks_t) {
  constexpr int VEC = elem<T>::kVec;
  __shared__ double sm[2048];
  const int c = first_chunk + blockIdx.x;
  const int r = blockIdx.y, b = blockIdx.z, h_kv = gridDim.y;
  const int cg_n = d / VEC;              // 16-byte column groups per row
  const int rp = 256 / cg_n;             // rows covered per pass
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
  __syncthreads();
  const int col = threadIdx.x;
  if (col < d) {
    double s = 0.0;
    for (int rr = 0; rr < rp; rr++) s += sm[rr * d + col];
    const float mean = (float)(s * (1.0 / (double)block));
    const int64_t o = (((int64_t)b * h_kv + r) * t_c + c) * d + col;
    kbar[o] = mean;
  }
}

hipError_t launch_kbar_compress(const dash_params& p, const Layout& L, const void* k, float* kbar,
                                int first_chunk, int n_chunks, hipStream_t st) {
  if (n_chunks <= 0) return hipSuccess;
  dim3 grid(n_chunks, p.h_kv, p.batch), blk(256);
  if (p.dtype == DASH_BF16)
    hipLaunchKernelGGL(kbar_compress_kernel<uint16_t>, grid, blk, 0, st, (const uint16_t*)k, kbar,
                       p.block_size, p.head_dim, L.t_c, first_chunk, p.k_stride[0],
                       p.k_stride[1], p.k_stride[2]);
  else
    hipLaunchKernelGGL(kbar_compress_kernel<float>, grid, blk, 0, st, (const float*)k, kbar,
                       p.block_size, p.head_dim, L.t_c, first_chunk, p.k_stride[0], p.k_stride[1],
                       p.k_stride[2]);
  return hipGetLastError();
}

}  // namespace dash
