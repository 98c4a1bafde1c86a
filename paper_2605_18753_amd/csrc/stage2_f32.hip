// Stage 2 and dense attention for fp32 tensors: a plain fp32 VALU kernel (one
// workgroup per query token and kv-head, one wave per query head, lanes over the
// 64 keys of a tile for the logits and over the head dimension for P.V).  It is
// the correctness vehicle of the fp32 configuration, not a tuned path; the
// arithmetic follows Alg. 3 / Proposition 1 with fp32 accumulation and expf.
#include <math.h>

#include "common.h"
#include "dash_internal.h"

namespace dash {

struct S2FArgs {
  const float* q; const float* k; const float* v; float* o;
  const uint32_t* mask; const float* bias;
  int h_kv, g_q, n_q, n_kv, block, t_all, words, pos0, causal, d;
  int64_t qs_b, qs_h, qs_t, ks_b, ks_h, ks_t, vs_b, vs_h, vs_t, os_b, os_h, os_t;
  float scale;
};

template <bool DENSE>
__global__ __launch_bounds__(256) void s2_f32_kernel(S2FArgs a) {
  __shared__ float qs[4][128];
  __shared__ float ps[4][64];
  const int tok = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int pos = a.pos0 + tok;
  const int cw = pos / a.block;
  const int nsub = a.block >> 6;
  const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + tok;
  const uint32_t* mrow = DENSE ? nullptr : a.mask + base * a.words;
  const float* brow = DENSE ? nullptr : a.bias + base * a.t_all;
  const float* kb = a.k + b * a.ks_b + r * a.ks_h;
  const float* vb = a.v + b * a.vs_b + r * a.vs_h;
  const int last = a.causal ? cw : a.t_all - 1;   // DENSE: last chunk to visit

  for (int hl = wave; hl < a.g_q; hl += 4) {
    const int head = r * a.g_q + hl;
    const float* qp = a.q + b * a.qs_b + head * a.qs_h + (int64_t)tok * a.qs_t;
    for (int e = lane; e < a.d; e += 64) qs[wave][e] = qp[e];
    __builtin_amdgcn_wave_barrier();
    float m = -INFINITY, l = 0.f, o0 = 0.f, o1 = 0.f;
    int rank = 0;
    const int n_iter = DENSE ? last + 1 : a.words * 32;
    for (int u = 0; u < n_iter; u++) {
      if (!DENSE) {
        const uint32_t w = mrow[u >> 5];
        if (w == 0u) { u |= 31; continue; }
        if (!((w >> (u & 31)) & 1u)) continue;
      }
      const bool diag = a.causal && u == cw;
      float bias = 0.f;
      if (!DENSE && !diag) bias = brow[rank++];
      for (int sub = 0; sub < nsub; sub++) {
        const int kpos0 = u * a.block + sub * 64;
        const int key = kpos0 + lane;
        const bool valid = key < a.n_kv && (!diag || key <= pos);
        float z = -INFINITY;
        if (valid) {
          const float* kr = kb + (int64_t)key * a.ks_t;
          float acc = 0.f;
          for (int e = 0; e < a.d; e += 4) {
            const f32x4 kk = *reinterpret_cast<const f32x4*>(kr + e);
            acc = fmaf(qs[wave][e], kk[0], acc);
            acc = fmaf(qs[wave][e + 1], kk[1], acc);
            acc = fmaf(qs[wave][e + 2], kk[2], acc);
            acc = fmaf(qs[wave][e + 3], kk[3], acc);
          }
          z = fmaf(acc, a.scale, bias);
        }
        const float m_new = fmaxf(m, wave_max(z));
        if (m_new == -INFINITY) continue;
        const float p = valid ? expf(z - m_new) : 0.f;
        const float corr = expf(m - m_new);
        l = l * corr + wave_sum(p);
        o0 *= corr; o1 *= corr;
        m = m_new;
        ps[wave][lane] = p;
        __builtin_amdgcn_wave_barrier();
        const int kmax = min(64, a.n_kv - kpos0);
        for (int kk = 0; kk < kmax; kk++) {
          const float pk = ps[wave][kk];
          const float* vr = vb + (int64_t)(kpos0 + kk) * a.vs_t;
          o0 = fmaf(pk, vr[lane], o0);
          if (a.d > 64) o1 = fmaf(pk, vr[lane + 64], o1);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
    float* op = a.o + b * a.os_b + head * a.os_h + (int64_t)tok * a.os_t;
    const float inv = 1.f / l;
    if (lane < a.d) op[lane] = o0 * inv;
    if (a.d > 64) op[lane + 64] = o1 * inv;
    __builtin_amdgcn_wave_barrier();
  }
}

hipError_t launch_s2_f32(const dash_params& p, const Layout& L, const void* q, const void* k,
                         const void* v, void* o, const uint32_t* mask, const float* bias,
                         bool dense, hipStream_t st) {
  S2FArgs a;
  a.q = (const float*)q; a.k = (const float*)k; a.v = (const float*)v; a.o = (float*)o;
  a.mask = mask; a.bias = bias;
  a.h_kv = p.h_kv; a.g_q = L.g_q; a.n_q = p.n_q; a.n_kv = p.n_kv; a.block = p.block_size;
  a.t_all = L.t_all; a.words = L.words; a.pos0 = L.pos0; a.causal = p.causal; a.d = p.head_dim;
  a.qs_b = p.q_stride[0]; a.qs_h = p.q_stride[1]; a.qs_t = p.q_stride[2];
  a.ks_b = p.k_stride[0]; a.ks_h = p.k_stride[1]; a.ks_t = p.k_stride[2];
  a.vs_b = p.v_stride[0]; a.vs_h = p.v_stride[1]; a.vs_t = p.v_stride[2];
  a.os_b = p.o_stride[0]; a.os_h = p.o_stride[1]; a.os_t = p.o_stride[2];
  a.scale = L.scale;
  dim3 grid(p.n_q, p.h_kv, p.batch);
  if (dense) hipLaunchKernelGGL(s2_f32_kernel<true>, grid, dim3(256), 0, st, a);
  else hipLaunchKernelGGL(s2_f32_kernel<false>, grid, dim3(256), 0, st, a);
  return hipGetLastError();
}

}  // namespace dash
