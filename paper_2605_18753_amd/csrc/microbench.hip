// Two yardstick kernels for bench.py (not part of the DashAttention ABI; built into
// their own library): what this GPU sustains on a plain streaming read of HBM and on a
// register-fed loop of bf16 matrix-core instructions.  The roofline fractions of the
// attention kernels are quoted against the datasheet peaks; these figures say how much
// of those peaks is reachable at all on the same box, clocks and power limit.
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace {

typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

// grid-stride read of n 16-byte words, four loads in flight per thread
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4* __restrict__ p, size_t n, uint32_t* sink) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  u32x4 acc = {0, 0, 0, 0};
  for (; i + 3 * stride < n; i += 4 * stride) {
    const u32x4 a = p[i], b = p[i + stride], c = p[i + 2 * stride], d = p[i + 3 * stride];
    acc ^= a ^ b ^ c ^ d;
  }
  for (; i < n; i += stride) acc ^= p[i];
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345u) sink[0] = 1u;   // never true for the fill bench.py uses
}

// Every wave issues `iters` rounds of 8 independent v_mfma_f32_32x32x16_bf16 on operands it
// keeps in registers (no memory traffic inside the loop).  random_operands: pseudo-random
// bf16 values in [-2, 2) (the data toggles, as real activations do); else all ones.
__global__ __launch_bounds__(256) void mfma_loop_kernel(float* sink, int iters, int random_operands) {
  const uint32_t t = blockIdx.x * 256u + threadIdx.x;
  bf16x8 a[4], b[2];
  uint32_t s = t * 2654435761u + 12345u;
  for (int i = 0; i < 4; i++)
    for (int j = 0; j < 8; j++) {
      s = s * 1664525u + 1013904223u;
      a[i][j] = random_operands ? (__bf16)((float)(int)(s >> 20) * (1.f / 1024.f) - 2.f) : (__bf16)1.f;
    }
  for (int i = 0; i < 2; i++)
    for (int j = 0; j < 8; j++) {
      s = s * 1664525u + 1013904223u;
      b[i][j] = random_operands ? (__bf16)((float)(int)(s >> 20) * (1.f / 1024.f) - 2.f) : (__bf16)1.f;
    }
  f32x16 c[8];
  for (int i = 0; i < 8; i++)
    for (int j = 0; j < 16; j++) c[i][j] = 0.f;
  for (int it = 0; it < iters; it++) {
#pragma unroll
    for (int i = 0; i < 8; i++) c[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i & 3], b[i >> 2], c[i], 0, 0, 0);
  }
  float r = 0.f;
  for (int i = 0; i < 8; i++)
    for (int j = 0; j < 16; j++) r += c[i][j];
  if (r == 0.123f) sink[0] = r;
}

}  // namespace

extern "C" {

// Reads `bytes` bytes (a multiple of 16) at device pointer src once.  sink: 4 device bytes.
int dash_mb_stream_read(const void* src, size_t bytes, void* sink, void* stream) {
  if (!src || !sink || (bytes & 15) != 0) return -1;
  hipLaunchKernelGGL(stream_read_kernel, dim3(8192), dim3(256), 0, (hipStream_t)stream,
                     (const u32x4*)src, bytes / 16, (uint32_t*)sink);
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

// Launches n_blocks workgroups of four waves, each wave issuing 8 * iters matrix-core
// instructions of 32768 flops.  Returns the flops of the launch through *flops.
int dash_mb_mfma_loop(void* sink, int n_blocks, int iters, int random_operands, double* flops, void* stream) {
  if (!sink || n_blocks < 1 || iters < 1) return -1;
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(n_blocks), dim3(256), 0, (hipStream_t)stream, (float*)sink, iters,
                     random_operands);
  if (flops) *flops = (double)n_blocks * 4.0 * iters * 8.0 * 32768.0;
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
