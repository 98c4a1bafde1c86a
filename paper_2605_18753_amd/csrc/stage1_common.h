// Shared by the Stage-1 kernels (stage1.hip, stage1_regs.hip): kernel arguments, the
// entmax exponent modes and the power terms of the threshold equation (Eq. 2; Alg. 2).
#pragma once
#include "common.h"

namespace dash {

struct S1Args {
  const void* q;
  const uint16_t* ksplit;
  const float* scores;
  const float* kbar;         // fp32 summaries (the decode kernel scores against them itself)
  // decode: the cache update folded into the Stage-1 launch (extra workgroups), or k_upd == null
  const void* k_upd; float* kbar_upd; int64_t ks_b, ks_h, ks_t;
  uint32_t* mask;
  int32_t* cnt;
  int32_t* idx;
  float* bias;
  float* tau;
  int batch, h_q, h_kv, g_q, n_q, n_kv, block, t_c, t_all, words, pos0, causal, window, ld;
  const int32_t* seq_lens;   // decode with per-sequence lengths (device, [batch]) or null
  int tok_base, tok_end;     // this launch covers query tokens [tok_base, tok_end) of every sequence
  int64_t qs_b, qs_h, qs_t;
  float xscale, pexp, alpha, inv_sigma;
};

enum { MODE_P1 = 0, MODE_P2 = 1, MODE_P4 = 2, MODE_GEN = 3, MODE_BISECT = 4 };

// u^p and u^(p-1) for u >= 0 (0 -> 0, and 0 for the derivative term as well)
template <int MODE>
__device__ __forceinline__ void pow_terms(float u, float p, float& f, float& g) {
  if constexpr (MODE == MODE_P1) {
    f = u; g = u > 0.f ? 1.f : 0.f;
  } else if constexpr (MODE == MODE_P2) {
    f = u * u; g = u;
  } else if constexpr (MODE == MODE_P4) {
    const float u2 = u * u; g = u2 * u; f = u2 * u2;
  } else {
    g = u > 0.f ? exp2f((p - 1.f) * log2f(u)) : 0.f;
    f = g * u;
  }
}
template <int MODE> __device__ __forceinline__ float pow_p(float u, float p) {
  float f, g; pow_terms<MODE>(u, p, f, g); return f;
}

// The register-resident Stage 1 (stage1_regs.hip), one object file per GQA group size.
hipError_t launch_s1_regs_g1(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st);
hipError_t launch_s1_regs_g2(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st);
hipError_t launch_s1_regs_g4(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st);
hipError_t launch_s1_regs_g8(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st);
hipError_t launch_s1_regs_g16(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st);

}  // namespace dash
