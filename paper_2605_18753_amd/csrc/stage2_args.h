// Kernel arguments shared by the bf16 Stage-2 kernels (prefill / dense in
// stage2.hip, split-KV decode in stage2_decode.hip).
#pragma once
#include "common.h"
#include "dash_internal.h"

namespace dash {

struct S2Args {
  const uint16_t* q; const uint16_t* k; const uint16_t* v; uint16_t* o;
  const uint32_t* mask; const float* bias;
  int h_q, h_kv, g_q, n_q, n_kv, block, t_all, words, pos0, causal, n_tiles, hb;
  int64_t qs_b, qs_h, qs_t, ks_b, ks_h, ks_t, vs_b, vs_h, vs_t, os_b, os_h, os_t;
  float c1;      // scale * log2(e)
  float* part;   // decode partials
  const int32_t* seq_lens;   // decode: per-sequence cache lengths (device, [batch]) or null
};

constexpr float kLazy = 8.f;   // lazy-rescale slack, in base-2 logit units

inline void fill_s2_args(S2Args& a, const dash_params& p, const Layout& L, const void* q, const void* k,
                         const void* v, void* o, const uint32_t* mask, const float* bias) {
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v; a.o = (uint16_t*)o;
  a.mask = mask; a.bias = bias; a.part = nullptr; a.seq_lens = L.seq_lens;
  a.h_q = p.h_q; a.h_kv = p.h_kv; a.g_q = L.g_q; a.n_q = p.n_q; a.n_kv = p.n_kv;
  a.block = p.block_size; a.t_all = L.t_all; a.words = L.words; a.pos0 = L.pos0;
  a.causal = p.causal;
  a.hb = p.h_kv * p.batch;
  a.n_tiles = 1;
  a.qs_b = p.q_stride[0]; a.qs_h = p.q_stride[1]; a.qs_t = p.q_stride[2];
  a.ks_b = p.k_stride[0]; a.ks_h = p.k_stride[1]; a.ks_t = p.k_stride[2];
  a.vs_b = p.v_stride[0]; a.vs_h = p.v_stride[1]; a.vs_t = p.v_stride[2];
  a.os_b = p.o_stride[0]; a.os_h = p.o_stride[1]; a.os_t = p.o_stride[2];
  a.c1 = L.scale * kLog2e;
}

}  // namespace dash
