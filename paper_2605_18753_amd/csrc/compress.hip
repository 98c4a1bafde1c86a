// Stage 0: key summaries of every complete chunk (Sec. 3.1; Alg. 1): the block mean
// (Eq. 3 with the summary query at its zero initial value, i.e. uniform pooling)
// and the learned form (Eq. 3: one softmax attention of a summary query over the
// chunk's own keys, the keys serving as values).
//
// One workgroup per (chunk, kv-head, batch).  The chunk (block x d elements) is
// streamed once with 16-byte loads; sums are accumulated in fp64, which is exact
// for 64..128 bf16/fp32 inputs of comparable magnitude, so the fp32 result is
// the correctly rounded mean independent of summation order.
#include "common.h"
#include "compress_body.h"
#include "dash_internal.h"

namespace dash {

template <typename T>
__global__ __launch_bounds__(256) void kbar_compress_kernel(
    const T* __restrict__ k, float* __restrict__ kbar, int block,
    int d, int t_c, int first_chunk, int64_t ks_b, int64_t ks_h, int64_t ks_t) {
  __shared__ double sm[2048];
  const int c = first_chunk + blockIdx.x;
  const int r = blockIdx.y, b = blockIdx.z, h_kv = gridDim.y;
  kbar_block_mean<T>(k, kbar, sm, block, d, t_c, c, r, b, h_kv, ks_b, ks_h, ks_t);
}


// Learned summary (Eq. 3; Alg. 1): kbar_c = softmax(K_c qbar / sqrt(d))^T K_c.
// Same decomposition as the mean kernel: thread (r0, cg) owns the 16-byte column
// group cg of rows r0, r0 + rp, ...; it keeps those rows in registers, so the
// chunk is read once.  Scores, softmax and the weighted sum are fp64, so the
// fp32 result is the correctly rounded value except in the rare case that the
// exact one lies within ~1e-15 of a rounding boundary.
template <typename T>
__global__ __launch_bounds__(256) void kbar_summarize_kernel(
    const T* __restrict__ k, const float* __restrict__ qbar, float* __restrict__ kbar, int block,
    int d, int t_c, int first_chunk, int64_t ks_b, int64_t ks_h, int64_t ks_t, int64_t qs_b,
    int64_t qs_h, int64_t qs_c, double scale) {
  constexpr int VEC = elem<T>::kVec;
  constexpr int MAXR = 16;                // rows per thread: block / rp <= 128 / 8
  __shared__ double sm[2048];
  __shared__ double sc[128], ew[128];
  const int c = first_chunk + blockIdx.x;
  const int r = blockIdx.y, b = blockIdx.z, h_kv = gridDim.y;
  const int cg_n = d / VEC;              // 16-byte column groups per row (a power of two <= 32)
  const int rp = 256 / cg_n;             // rows covered per pass
  const int cg = threadIdx.x % cg_n, r0 = threadIdx.x / cg_n;
  const int nrow = block / rp;
  const T* base = k + b * ks_b + r * ks_h + (int64_t)c * block * ks_t + cg * VEC;
  const float* qp = qbar + b * qs_b + r * qs_h + (int64_t)c * qs_c + cg * VEC;
  double qv[VEC];
#pragma unroll
  for (int e = 0; e < VEC; e++) qv[e] = (double)qp[e];
  u32x4 raw[MAXR];
  auto key = [&](const u32x4& w, int e) -> double {
    if constexpr (VEC == 8) return (double)((e & 1) ? bf16_hi(w[e >> 1]) : bf16_lo(w[e >> 1]));
    else return (double)__uint_as_float(w[e]);
  };
  // all loads first, so that they are in flight together
#pragma unroll
  for (int i = 0; i < MAXR; i++)
    if (i < nrow) raw[i] = *reinterpret_cast<const u32x4*>(base + (int64_t)(r0 + i * rp) * ks_t);
  // scores s_t = <qbar, k_t> * scale: per-thread partial over its column group, then
  // a butterfly over the cg_n lanes that share the row
#pragma unroll
  for (int i = 0; i < MAXR; i++) {
    if (i < nrow) {
      double part = 0.0;
#pragma unroll
      for (int e = 0; e < VEC; e++) part += qv[e] * key(raw[i], e);
      for (int m = 1; m < cg_n; m <<= 1) part += __shfl_xor(part, m);
      if (cg == 0) sc[r0 + i * rp] = part * scale;
    }
  }
  __syncthreads();
  // softmax weights: thread t < block owns score t; maximum and sum by wave
  // reductions plus one exchange through LDS (every thread ends up with the same
  // values: the combination order is fixed)
  __shared__ double red[8];
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nw = (block + 63) >> 6;            // waves that own scores (1 or 2)
  double mine = threadIdx.x < block ? sc[threadIdx.x] : -INFINITY;
  double wm = mine;
  for (int m = 32; m >= 1; m >>= 1) wm = fmax(wm, __shfl_xor(wm, m));
  if (lane == 0) red[wv] = wm;
  __syncthreads();
  double mx = red[0];
  for (int i = 1; i < nw; i++) mx = fmax(mx, red[i]);
  const double ex = threadIdx.x < block ? exp(mine - mx) : 0.0;
  if (threadIdx.x < block) ew[threadIdx.x] = ex;
  double ws = ex;
  for (int m = 32; m >= 1; m >>= 1) ws += __shfl_xor(ws, m);
  if (lane == 0) red[4 + wv] = ws;
  __syncthreads();
  double den = red[4];
  for (int i = 1; i < nw; i++) den += red[4 + i];
  double acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; e++) acc[e] = 0.0;
#pragma unroll
  for (int i = 0; i < MAXR; i++) {
    if (i < nrow) {
      const double w = ew[r0 + i * rp];
#pragma unroll
      for (int e = 0; e < VEC; e++) acc[e] += w * key(raw[i], e);
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; e++) sm[r0 * d + cg * VEC + e] = acc[e];
  __syncthreads();
  const int col = threadIdx.x;
  if (col < d) {
    double s = 0.0;
    for (int rr = 0; rr < rp; rr++) s += sm[rr * d + col];
    const int64_t o = (((int64_t)b * h_kv + r) * t_c + c) * d + col;
    kbar[o] = (float)(s / den);
  }
}

// Backward of the learned summary (Eq. 3): with a = softmax(K_c qbar scale) and a given
// dkbar_c:  da = K_c dkbar_c,  ds = a (da - <a, da>),
//   dK_c += a dkbar_c^T + scale ds qbar^T,   dqbar_c = scale K_c^T ds.
// Same decomposition as the forward kernel (one workgroup per chunk, thread = a
// 16-byte column group of rows r0, r0 + rp, ...); fp32 arithmetic (the result is
// compared at gradient tolerance, not bit for bit).  dk is read, incremented and
// written back in the run dtype; dqbar is written per chunk.
template <typename T>
__global__ __launch_bounds__(256) void kbar_summarize_bwd_kernel(
    const T* __restrict__ k, const float* __restrict__ qbar, const float* __restrict__ dkbar,
    T* __restrict__ dk, float* __restrict__ dqbar, int block, int d, int t_c, int64_t ks_b, int64_t ks_h,
    int64_t ks_t, int64_t qs_b, int64_t qs_h, int64_t qs_c, float scale) {
  constexpr int VEC = elem<T>::kVec;
  constexpr int MAXR = 16;
  __shared__ float sm[2048];
  __shared__ float sc[128], da_s[128], a_s[128], ds_s[128];
  __shared__ float red[12];
  const int c = blockIdx.x, r = blockIdx.y, b = blockIdx.z, h_kv = gridDim.y;
  const int cg_n = d / VEC, rp = 256 / cg_n;
  const int cg = threadIdx.x % cg_n, r0 = threadIdx.x / cg_n;
  const int nrow = block / rp;
  const int64_t koff = b * ks_b + r * ks_h + (int64_t)c * block * ks_t + cg * VEC;
  const float* qp = qbar + b * qs_b + r * qs_h + (int64_t)c * qs_c + cg * VEC;
  const float* gp = dkbar + (((int64_t)b * h_kv + r) * t_c + c) * d + cg * VEC;
  float qv[VEC], gv[VEC];
#pragma unroll
  for (int e = 0; e < VEC; e++) { qv[e] = qp[e]; gv[e] = gp[e]; }
  u32x4 raw[MAXR];
  auto key = [&](const u32x4& w, int e) -> float {
    if constexpr (VEC == 8) return (e & 1) ? bf16_hi(w[e >> 1]) : bf16_lo(w[e >> 1]);
    else return __uint_as_float(w[e]);
  };
#pragma unroll
  for (int i = 0; i < MAXR; i++)
    if (i < nrow) raw[i] = *reinterpret_cast<const u32x4*>(k + koff + (int64_t)(r0 + i * rp) * ks_t);
  // per row: s = <qbar, k> scale and da = <dkbar, k>
#pragma unroll
  for (int i = 0; i < MAXR; i++) {
    if (i < nrow) {
      float ps = 0.f, pa = 0.f;
#pragma unroll
      for (int e = 0; e < VEC; e++) { ps = fmaf(qv[e], key(raw[i], e), ps); pa = fmaf(gv[e], key(raw[i], e), pa); }
      for (int m = 1; m < cg_n; m <<= 1) { ps += __shfl_xor(ps, m); pa += __shfl_xor(pa, m); }
      if (cg == 0) { sc[r0 + i * rp] = ps * scale; da_s[r0 + i * rp] = pa; }
    }
  }
  __syncthreads();
  // softmax over the chunk's rows and <a, da>: thread t < block owns row t
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int nw = (block + 63) >> 6;
  const float mine = threadIdx.x < block ? sc[threadIdx.x] : -INFINITY;
  float wm = mine;
  for (int m = 32; m >= 1; m >>= 1) wm = fmaxf(wm, __shfl_xor(wm, m));
  if (lane == 0) red[wv] = wm;
  __syncthreads();
  float mx = red[0];
  for (int i = 1; i < nw; i++) mx = fmaxf(mx, red[i]);
  const float ex = threadIdx.x < block ? expf(mine - mx) : 0.f;
  const float myda = threadIdx.x < block ? da_s[threadIdx.x] : 0.f;
  float ws = ex, wd = ex * myda;
  for (int m = 32; m >= 1; m >>= 1) { ws += __shfl_xor(ws, m); wd += __shfl_xor(wd, m); }
  if (lane == 0) { red[4 + wv] = ws; red[8 + wv] = wd; }
  __syncthreads();
  float den = red[4], dot = red[8];
  for (int i = 1; i < nw; i++) { den += red[4 + i]; dot += red[8 + i]; }
  if (threadIdx.x < block) {
    const float aw = ex / den;
    a_s[threadIdx.x] = aw;
    ds_s[threadIdx.x] = aw * (myda - dot / den);
  }
  __syncthreads();
  // dK rows and the partial sums of dqbar
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; e++) acc[e] = 0.f;
#pragma unroll
  for (int i = 0; i < MAXR; i++) {
    if (i < nrow) {
      const int row = r0 + i * rp;
      const float aw = a_s[row], dsw = ds_s[row] * scale;
      T* dkp = dk + koff + (int64_t)row * ks_t;
#pragma unroll
      for (int e = 0; e < VEC; e++) {
        acc[e] = fmaf(dsw, key(raw[i], e), acc[e]);
        elem<T>::st(dkp + e, elem<T>::ld(dkp + e) + aw * gv[e] + dsw * qv[e]);
      }
    }
  }
#pragma unroll
  for (int e = 0; e < VEC; e++) sm[r0 * d + cg * VEC + e] = acc[e];
  __syncthreads();
  const int col = threadIdx.x;
  if (col < d) {
    float t = 0.f;
    for (int rr = 0; rr < rp; rr++) t += sm[rr * d + col];
    dqbar[(((int64_t)b * h_kv + r) * t_c + c) * d + col] = t;
  }
}

hipError_t launch_kbar_summarize_bwd(const dash_params& p, const Layout& L, const void* k, const float* qbar,
                                     const int64_t* qs, const float* dkbar, void* dk, float* dqbar,
                                     hipStream_t st) {
  if (L.t_c <= 0) return hipSuccess;
  dim3 grid(L.t_c, p.h_kv, p.batch), blk(256);
  if (p.dtype == DASH_BF16)
    hipLaunchKernelGGL(kbar_summarize_bwd_kernel<uint16_t>, grid, blk, 0, st, (const uint16_t*)k, qbar, dkbar,
                       (uint16_t*)dk, dqbar, p.block_size, p.head_dim, L.t_c, p.k_stride[0], p.k_stride[1],
                       p.k_stride[2], qs[0], qs[1], qs[2], L.scale);
  else
    hipLaunchKernelGGL(kbar_summarize_bwd_kernel<float>, grid, blk, 0, st, (const float*)k, qbar, dkbar,
                       (float*)dk, dqbar, p.block_size, p.head_dim, L.t_c, p.k_stride[0], p.k_stride[1],
                       p.k_stride[2], qs[0], qs[1], qs[2], L.scale);
  return hipGetLastError();
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

hipError_t launch_kbar_summarize(const dash_params& p, const Layout& L, const void* k, const float* qbar,
                                 const int64_t* qs, float* kbar, int first_chunk, int n_chunks,
                                 hipStream_t st) {
  if (n_chunks <= 0) return hipSuccess;
  dim3 grid(n_chunks, p.h_kv, p.batch), blk(256);
  // the logit scale in double: the default 1/sqrt(d) is not rounded through fp32
  const double scale = p.scale > 0.f ? (double)p.scale : 1.0 / sqrt((double)p.head_dim);
  if (p.dtype == DASH_BF16)
    hipLaunchKernelGGL(kbar_summarize_kernel<uint16_t>, grid, blk, 0, st, (const uint16_t*)k, qbar, kbar,
                       p.block_size, p.head_dim, L.t_c, first_chunk, p.k_stride[0], p.k_stride[1],
                       p.k_stride[2], qs[0], qs[1], qs[2], scale);
  else
    hipLaunchKernelGGL(kbar_summarize_kernel<float>, grid, blk, 0, st, (const float*)k, qbar, kbar,
                       p.block_size, p.head_dim, L.t_c, first_chunk, p.k_stride[0], p.k_stride[1],
                       p.k_stride[2], qs[0], qs[1], qs[2], scale);
  return hipGetLastError();
}

}  // namespace dash
