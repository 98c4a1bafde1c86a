// C ABI of the DashAttention library: argument validation, workspace carving and
// kernel sequencing.  Host code only; every kernel lives in its own file.
#include <math.h>
#include <stdlib.h>
#include <string.h>

#include "dash_internal.h"

// Scratch for dash_attn_decode_static, the entry point for callers that cannot allocate: one
// array per GPU the library's code is loaded on, held until the process ends.  In host code the
// name stands for the symbol, not for a device address: the address is asked for once per device
// (static_scratch below) and only that pointer is handed to kernels.
constexpr size_t kStaticScratchBytes = (size_t)8 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace dash {

static std::atomic<void*> g_scratch_ptr[64];   // per device ordinal; nullptr = not asked for yet

// The current device's copy of `scratch`.  Thread-safe (two threads that race both look the
// address up and store the same value).
static int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return DASH_ELAUNCH;
  if (dev < 0 || dev >= 64) return DASH_EUNSUPPORTED;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return DASH_ELAUNCH;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);
  }
  *out = ptr;
  return DASH_OK;
}

static size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

static bool strides_ok(const int64_t s[3], int d, int vec) {
  return s[2] >= d && s[0] % vec == 0 && s[1] % vec == 0 && s[2] % vec == 0 && s[0] >= 0 && s[1] >= 0;
}

int make_layout(const dash_params* p, Layout* L, bool routing) {
  if (!p || !L) return DASH_EINVAL;
  if (p->batch < 1 || p->h_q < 1 || p->h_kv < 1 || p->n_q < 1 || p->n_kv < 1) return DASH_EINVAL;
  if (p->h_q % p->h_kv != 0 || p->n_q > p->n_kv) return DASH_EINVAL;
  if (!(p->alpha > 1.f) || !(p->gamma > 0.f) || !(p->sigma > 0.f)) return DASH_EINVAL;
  if (!isfinite(p->alpha) || !isfinite(p->gamma) || !isfinite(p->scale)) return DASH_EINVAL;
  if (p->causal != 0 && p->causal != 1) return DASH_EINVAL;
  if (p->window < 0 || p->window > 8 || (p->window > 0 && !p->causal)) return DASH_EINVAL;
  if (p->dtype != DASH_F32 && p->dtype != DASH_BF16) return DASH_EINVAL;
  if (p->head_dim < 1 || p->block_size < 1) return DASH_EINVAL;
  if (routing && !p->causal && p->n_kv % p->block_size != 0) return DASH_EINVAL;
  const int vec = p->dtype == DASH_BF16 ? 8 : 4;
  if (p->head_dim % vec == 0) {
    if (!strides_ok(p->q_stride, p->head_dim, vec) || !strides_ok(p->k_stride, p->head_dim, vec) ||
        !strides_ok(p->v_stride, p->head_dim, vec) || !strides_ok(p->o_stride, p->head_dim, vec))
      return DASH_EINVAL;
  }
  if (p->head_dim != 64 && p->head_dim != 128) return DASH_EUNSUPPORTED;
  if (p->block_size != 64 && p->block_size != 128) return DASH_EUNSUPPORTED;
  const int g = p->h_q / p->h_kv;
  if (g != 1 && g != 2 && g != 4 && g != 8 && g != 16) return DASH_EUNSUPPORTED;
  // tokens of one row tile must share their candidate set
  if (p->n_q > 1 && (p->n_kv - p->n_q) % 64 != 0) return DASH_EUNSUPPORTED;
  memset(L, 0, sizeof(*L));
  L->g_q = g;
  L->t_c = p->n_kv / p->block_size;
  L->t_all = (p->n_kv + p->block_size - 1) / p->block_size;
  if (L->t_all > 2048) return DASH_EUNSUPPORTED;
  L->words = (L->t_all + 31) / 32;
  L->pos0 = p->n_kv - p->n_q;
  L->scale = p->scale > 0.f ? p->scale : (float)(1.0 / sqrt((double)p->head_dim));
  L->xscale = (float)((double)p->gamma * ((double)p->alpha - 1.0) * (double)L->scale);
  L->pexp = (float)(1.0 / ((double)p->alpha - 1.0));
  L->use_mfma = p->dtype == DASH_BF16 && p->n_q > 1;
  const bool decode_mfma = p->dtype == DASH_BF16 && p->n_q == 1;
  int splits = 1;
  if (decode_mfma) {
    const int pairs = p->batch * p->h_kv;
    const int target = 512;   // workgroups per launch: two per CU
    splits = (target + pairs - 1) / pairs;
    if (splits > 64) splits = 64;
    if (splits > L->t_all) splits = L->t_all;
    if (splits < 1) splits = 1;
  }
  L->splits = splits;
  const size_t rows = (size_t)p->batch * p->h_kv * p->n_q;
  size_t off = 0;
  L->off_ksplit = off;
  if (L->use_mfma) off += align256((size_t)p->batch * p->h_kv * L->t_c * 3 * p->head_dim * 2);
  L->off_mask = off;  off += align256(rows * L->words * 4);
  L->off_bias = off;  off += align256(rows * L->t_all * 4);
  L->off_scores = off;
  // fp32 score rows: fp32 prefill only (a decode step keeps its scores in LDS)
  if (!L->use_mfma && !(p->n_q == 1 && p->causal))
    off += align256((size_t)p->batch * p->h_q * p->n_q * (L->t_c > 0 ? L->t_c : 1) * 4);
  L->off_part = off;
  if (decode_mfma) off += align256((size_t)p->batch * p->h_kv * splits * g * (p->head_dim + 2) * 4);
  L->total = off > 0 ? off : 256;
  if (p->dtype == DASH_BF16) {
    // the bf16 kernels address one (batch, kv-head) slice of every tensor with 32-bit byte
    // offsets and a 32-bit buffer size: a slice must span less than 2 GiB
    const int64_t lim = (int64_t)1 << 31;
    const int64_t nq = p->n_q, nk = p->n_kv, d = p->head_dim;
    if (((g - 1) * p->q_stride[1] + (nq - 1) * p->q_stride[2] + d) * 2 >= lim ||
        ((g - 1) * p->o_stride[1] + (nq - 1) * p->o_stride[2] + d) * 2 >= lim ||
        ((nk - 1) * p->k_stride[2] + d) * 2 >= lim || ((nk - 1) * p->v_stride[2] + d) * 2 >= lim)
      return DASH_EUNSUPPORTED;
  }
  return DASH_OK;
}

static int check_ws(const Layout& L, void* ws, size_t bytes) {
  if (!ws || ((uintptr_t)ws & 255) != 0 || bytes < L.total) return DASH_EWORKSPACE;
  return DASH_OK;
}

static int run_stage1(const dash_params* p, const Layout& L, const void* q, const float* kbar,
                      uint32_t* mask, int32_t* cnt, int32_t* idx, float* bias, float* tau,
                      char* ws, hipStream_t st, const void* k_upd = nullptr, float* kbar_upd = nullptr) {
  S1Out out;
  out.mask = mask ? mask : reinterpret_cast<uint32_t*>(ws + L.off_mask);
  out.bias = bias ? bias : reinterpret_cast<float*>(ws + L.off_bias);
  out.cnt = cnt; out.idx = idx; out.tau = tau;
  hipError_t e;
  if (L.use_mfma) {
    e = launch_s1_route(*p, L, q, kbar, reinterpret_cast<uint16_t*>(ws + L.off_ksplit), nullptr, out, st);
  } else if (p->n_q == 1 && p->causal) {
    e = launch_s1_decode(*p, L, q, kbar, out, k_upd, kbar_upd, st);   // scores, threshold and lists in one launch
  } else {
    float* scores = reinterpret_cast<float*>(ws + L.off_scores);
    e = launch_s1_scores_f32(*p, L, q, kbar, scores, st);
    if (e != hipSuccess) return DASH_ELAUNCH;
    e = launch_s1_route(*p, L, q, kbar, nullptr, scores, out, st);
  }
  return e == hipSuccess ? DASH_OK : DASH_ELAUNCH;
}

static int run_stage2(const dash_params* p, const Layout& L, const void* q, const void* k,
                      const void* v, void* o, const uint32_t* mask, const float* bias, char* ws,
                      bool dense, hipStream_t st) {
  const uint32_t* m = mask ? mask : reinterpret_cast<const uint32_t*>(ws + L.off_mask);
  const float* bb = bias ? bias : reinterpret_cast<const float*>(ws + L.off_bias);
  hipError_t e;
  if (p->dtype == DASH_F32) e = launch_s2_f32(*p, L, q, k, v, o, m, bb, dense, st);
  else if (p->n_q == 1)
    e = launch_decode_s2(*p, L, q, k, v, o, m, bb, reinterpret_cast<float*>(ws + L.off_part), dense, st);
  else e = launch_s2_mfma(*p, L, q, k, v, o, m, bb, dense, st);
  return e == hipSuccess ? DASH_OK : DASH_ELAUNCH;
}

}  // namespace dash

using namespace dash;

extern "C" {

int32_t dash_list_stride(const dash_params* p) {
  Layout L;
  return make_layout(p, &L) == DASH_OK ? L.t_all : -1;
}

int32_t dash_mask_words(const dash_params* p) {
  Layout L;
  return make_layout(p, &L) == DASH_OK ? L.words : -1;
}

int dash_attn_workspace_bytes(const dash_params* p, size_t* out_bytes) {
  if (!out_bytes) return DASH_EINVAL;
  Layout L;
  const int rc = make_layout(p, &L, false);
  if (rc != DASH_OK) return rc;
  *out_bytes = L.total;
  return DASH_OK;
}

int dash_kbar_compress(const dash_params* p, const void* k, float* kbar, int32_t first_chunk,
                       int32_t n_chunks, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!k || (!kbar && L.t_c > 0)) return DASH_EINVAL;
  if (n_chunks < 0) { first_chunk = 0; n_chunks = L.t_c; }
  if (first_chunk < 0 || first_chunk + n_chunks > L.t_c) return DASH_EINVAL;
  return launch_kbar_compress(*p, L, k, kbar, first_chunk, n_chunks, (hipStream_t)stream) == hipSuccess
             ? DASH_OK : DASH_ELAUNCH;
}

int dash_kbar_summarize(const dash_params* p, const void* k, const float* qbar,
                        const int64_t* qbar_stride, float* kbar, int32_t first_chunk,
                        int32_t n_chunks, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!k || !qbar || !qbar_stride || (!kbar && L.t_c > 0)) return DASH_EINVAL;
  const int vec = p->dtype == DASH_BF16 ? 8 : 4;
  for (int i = 0; i < 3; i++)
    if (qbar_stride[i] < 0 || qbar_stride[i] % vec != 0) return DASH_EINVAL;
  if (((uintptr_t)qbar & 15) != 0) return DASH_EINVAL;
  if (n_chunks < 0) { first_chunk = 0; n_chunks = L.t_c; }
  if (first_chunk < 0 || first_chunk + n_chunks > L.t_c) return DASH_EINVAL;
  return launch_kbar_summarize(*p, L, k, qbar, qbar_stride, kbar, first_chunk, n_chunks,
                               (hipStream_t)stream) == hipSuccess ? DASH_OK : DASH_ELAUNCH;
}

int dash_stage1_route(const dash_params* p, const void* q, const float* kbar, uint32_t* mask,
                      int32_t* blk_cnt, int32_t* blk_idx, float* blk_bias, float* tau,
                      void* workspace, size_t workspace_bytes, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!q || (!kbar && L.t_c > 0)) return DASH_EINVAL;
  if ((rc = check_ws(L, workspace, workspace_bytes)) != DASH_OK) return rc;
  return run_stage1(p, L, q, kbar, mask, blk_cnt, blk_idx, blk_bias, tau, (char*)workspace,
                    (hipStream_t)stream);
}

int dash_stage2_attend(const dash_params* p, const void* q, const void* k, const void* v, void* o,
                       const uint32_t* mask, const float* blk_bias, void* workspace,
                       size_t workspace_bytes, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!q || !k || !v || !o) return DASH_EINVAL;
  if ((rc = check_ws(L, workspace, workspace_bytes)) != DASH_OK) return rc;
  return run_stage2(p, L, q, k, v, o, mask, blk_bias, (char*)workspace, false, (hipStream_t)stream);
}

int dash_attn_prefill(const dash_params* p, const void* q, const void* k, const void* v, void* o,
                      float* kbar, uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                      float* blk_bias, float* tau, void* workspace, size_t workspace_bytes,
                      void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!q || !k || !v || !o || (!kbar && L.t_c > 0)) return DASH_EINVAL;
  if ((rc = check_ws(L, workspace, workspace_bytes)) != DASH_OK) return rc;
  hipStream_t st = (hipStream_t)stream;
  if (launch_kbar_compress(*p, L, k, kbar, 0, L.t_c, st) != hipSuccess) return DASH_ELAUNCH;
  rc = run_stage1(p, L, q, kbar, mask, blk_cnt, blk_idx, blk_bias, tau, (char*)workspace, st);
  if (rc != DASH_OK) return rc;
  return run_stage2(p, L, q, k, v, o, mask, blk_bias, (char*)workspace, false, st);
}

static int decode_impl(const dash_params* p, const void* q, const void* k_cache, const void* v_cache,
                       float* kbar_cache, const int32_t* seq_lens, bool update_cache, void* o,
                       uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx, float* blk_bias, float* tau,
                       void* workspace, size_t workspace_bytes, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (p->n_q != 1 || !p->causal) return DASH_EINVAL;
  if (!q || !k_cache || !v_cache || (!kbar_cache && L.t_c > 0) || !o) return DASH_EINVAL;
  if (seq_lens && p->dtype != DASH_BF16) return DASH_EUNSUPPORTED;
  if ((rc = check_ws(L, workspace, workspace_bytes)) != DASH_OK) return rc;
  L.seq_lens = seq_lens;
  hipStream_t st = (hipStream_t)stream;
  // a current token that completes a chunk: that chunk is summarised now, by extra workgroups
  // of the Stage-1 launch; it becomes a candidate only for later positions
  rc = run_stage1(p, L, q, kbar_cache, mask, blk_cnt, blk_idx, blk_bias, tau, (char*)workspace, st,
                  update_cache ? k_cache : nullptr, update_cache ? kbar_cache : nullptr);
  if (rc != DASH_OK) return rc;
  return run_stage2(p, L, q, k_cache, v_cache, o, mask, blk_bias, (char*)workspace, false, st);
}

int dash_attn_decode(const dash_params* p, const void* q, const void* k_cache, const void* v_cache,
                     float* kbar_cache, void* o, uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                     float* blk_bias, float* tau, void* workspace, size_t workspace_bytes,
                     void* stream) {
  return decode_impl(p, q, k_cache, v_cache, kbar_cache, nullptr, true, o, mask, blk_cnt, blk_idx,
                     blk_bias, tau, workspace, workspace_bytes, stream);
}

int dash_attn_decode_static(const dash_params* p, const void* q, const void* k_cache, const void* v_cache,
                            float* kbar_cache, void* o, uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                            float* blk_bias, float* tau, void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (L.total > kStaticScratchBytes) return DASH_EWORKSPACE;   // larger than the built-in scratch
  void* ws = nullptr;
  if ((rc = static_scratch(&ws)) != DASH_OK) return rc;
  return decode_impl(p, q, k_cache, v_cache, kbar_cache, nullptr, true, o, mask, blk_cnt, blk_idx,
                     blk_bias, tau, ws, kStaticScratchBytes, stream);
}

int dash_attn_decode_ragged(const dash_params* p, const void* q, const void* k_cache,
                            const void* v_cache, float* kbar_cache, const int32_t* seq_lens,
                            int32_t update_cache, void* o, uint32_t* mask, int32_t* blk_cnt,
                            int32_t* blk_idx, float* blk_bias, float* tau, void* workspace,
                            size_t workspace_bytes, void* stream) {
  if (!seq_lens) return DASH_EINVAL;
  return decode_impl(p, q, k_cache, v_cache, kbar_cache, seq_lens, update_cache != 0, o, mask, blk_cnt,
                     blk_idx, blk_bias, tau, workspace, workspace_bytes, stream);
}

int dense_attn(const dash_params* p, const void* q, const void* k, const void* v, void* o,
               void* workspace, size_t workspace_bytes, void* stream) {
  Layout L;
  int rc = make_layout(p, &L, false);
  if (rc != DASH_OK) return rc;
  if (!q || !k || !v || !o) return DASH_EINVAL;
  if ((rc = check_ws(L, workspace, workspace_bytes)) != DASH_OK) return rc;
  return run_stage2(p, L, q, k, v, o, nullptr, nullptr, (char*)workspace, true, (hipStream_t)stream);
}

static int backward_layout(const dash_params* p, Layout* L) {
  int rc = make_layout(p, L);
  if (rc != DASH_OK) return rc;
  if (p->n_q != p->n_kv) return DASH_EUNSUPPORTED;
  // p = 1/(alpha-1) < 1/2: the entmax slope is unbounded at the edge of the support and the
  // fp32 scores no longer carry the gradient of rows with a chunk near its threshold
  if (p->alpha > 3.f) return DASH_EUNSUPPORTED;
  return DASH_OK;
}

int dash_attn_backward_workspace_bytes(const dash_params* p, size_t* out_bytes) {
  if (!out_bytes) return DASH_EINVAL;
  Layout L;
  const int rc = backward_layout(p, &L);
  if (rc != DASH_OK) return rc;
  *out_bytes = backward_workspace_bytes(*p, L);
  return DASH_OK;
}

int dash_attn_backward(const dash_params* p, const void* q, const void* k, const void* v,
                       const void* d_o, const float* kbar, const uint32_t* mask, const float* blk_bias,
                       const float* tau, void* dq, void* dk, void* dv, float* dkbar, void* workspace,
                       size_t workspace_bytes, void* stream) {
  Layout L;
  const int rc = backward_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!q || !k || !v || !d_o || !mask || !blk_bias || !tau || !dq || !dk || !dv ||
      (!kbar && L.t_c > 0))
    return DASH_EINVAL;
  if (!workspace || ((uintptr_t)workspace & 255) != 0 || workspace_bytes < backward_workspace_bytes(*p, L))
    return DASH_EWORKSPACE;
  return launch_backward(*p, L, q, k, v, d_o, kbar, mask, blk_bias, tau, dq, dk, dv, dkbar, (char*)workspace,
                         (hipStream_t)stream) == hipSuccess ? DASH_OK : DASH_ELAUNCH;
}

int dash_kbar_summarize_backward(const dash_params* p, const void* k, const float* qbar,
                                 const int64_t* qbar_stride, const float* dkbar, void* dk, float* dqbar,
                                 void* stream) {
  Layout L;
  int rc = make_layout(p, &L);
  if (rc != DASH_OK) return rc;
  if (!k || !qbar || !qbar_stride || !dk || ((!dkbar || !dqbar) && L.t_c > 0)) return DASH_EINVAL;
  const int vec = p->dtype == DASH_BF16 ? 8 : 4;
  for (int i = 0; i < 3; i++)
    if (qbar_stride[i] < 0 || qbar_stride[i] % vec != 0) return DASH_EINVAL;
  if (((uintptr_t)qbar & 15) != 0) return DASH_EINVAL;
  return launch_kbar_summarize_bwd(*p, L, k, qbar, qbar_stride, dkbar, dk, dqbar, (hipStream_t)stream) == hipSuccess
             ? DASH_OK : DASH_ELAUNCH;
}

const char* dash_strerror(int code) {
  switch (code) {
    case DASH_OK: return "ok";
    case DASH_EINVAL: return "invalid argument";
    case DASH_EUNSUPPORTED: return "unsupported configuration";
    case DASH_EWORKSPACE: return "workspace missing, misaligned or too small";
    case DASH_ELAUNCH: return "HIP launch error";
    default: return "unknown status";
  }
}

}  // extern "C"
