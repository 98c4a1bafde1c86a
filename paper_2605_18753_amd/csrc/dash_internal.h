// Host-side internals of the DashAttention library: derived sizes, the layout
// of the caller-provided workspace, and the launchers each kernel file exports.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "../../include/dash_attn.h"

namespace dash {

struct Layout {
  int g_q;          // query heads per kv head
  int t_c;          // complete chunks: floor(n_kv / block)  (have a summary)
  int t_all;        // ceil(n_kv / block) = list stride (candidates + diagonal)
  int words;        // mask words per query
  int pos0;         // sequence position of query 0: n_kv - n_q
  int splits;       // decode: KV splits per (batch, kv head)
  float scale;      // logit scale
  float xscale;     // gamma * (alpha-1) * scale: Stage-1 score factor
  float pexp;       // 1/(alpha-1)
  bool use_mfma;    // bf16 prefill path (split summaries + MFMA Stage 1/2)
  const int32_t* seq_lens;   // decode with per-sequence lengths: device array [batch], else null
  // workspace offsets in bytes (256-aligned); 0-sized regions share offsets
  size_t off_ksplit, off_mask, off_bias, off_scores, off_part, total;
};

// Validates p and fills L.  Returns a dash_status.  routing = false skips the
// checks that only the Stage-1 router needs (dense attention, size queries).
int make_layout(const dash_params* p, Layout* L, bool routing = true);

// A kernel that uses a large amount of dynamic LDS (up to the 160 KB of a compute unit) has to opt in, per device, to the size
// it is launched with.  The opt-in is a property of the loaded kernel on that device, not a
// stream operation, so it is made when a launch first needs that much there and the size
// granted is recorded (per device ordinal; two threads that race both make the call, and
// the larger size wins).  Nothing else in the library outlives a call.
struct LdsOptIn { std::atomic<uint32_t> granted[64] = {}; };
inline hipError_t allow_dyn_lds(const void* kern, size_t bytes, LdsOptIn& rec) {
  if (bytes <= 48 * 1024) return hipSuccess;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const bool tracked = dev >= 0 && dev < 64;
  if (tracked && rec.granted[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
  e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
  if (e == hipSuccess && tracked) {
    uint32_t cur = rec.granted[dev].load(std::memory_order_relaxed);
    while (cur < bytes && !rec.granted[dev].compare_exchange_weak(cur, (uint32_t)bytes, std::memory_order_release)) {}
  }
  return e;
}

struct S1Out {
  uint32_t* mask; int32_t* cnt; int32_t* idx; float* bias; float* tau;
};

hipError_t launch_kbar_compress(const dash_params& p, const Layout& L, const void* k, float* kbar,
                                int first_chunk, int n_chunks, hipStream_t st);
hipError_t launch_kbar_summarize(const dash_params& p, const Layout& L, const void* k, const float* qbar,
                                 const int64_t* qs, float* kbar, int first_chunk, int n_chunks,
                                 hipStream_t st);
hipError_t launch_s1_scores_f32(const dash_params& p, const Layout& L, const void* q,
                                const float* kbar, float* scores, hipStream_t st);
// ksplit != NULL: bf16 MFMA scorer (the split of kbar is written to ksplit first);
// otherwise the scores are read from `scores` (written by launch_s1_scores_f32).
hipError_t launch_s1_route(const dash_params& p, const Layout& L, const void* q, const float* kbar,
                           uint16_t* ksplit, const float* scores, const S1Out& out, hipStream_t st);
hipError_t launch_s1_decode(const dash_params& p, const Layout& L, const void* q, const float* kbar,
                            const S1Out& out, const void* k_upd, float* kbar_upd, hipStream_t st);
hipError_t launch_s2_mfma(const dash_params& p, const Layout& L, const void* q, const void* k,
                          const void* v, void* o, const uint32_t* mask, const float* bias,
                          bool dense, hipStream_t st);
hipError_t launch_s2_f32(const dash_params& p, const Layout& L, const void* q, const void* k,
                         const void* v, void* o, const uint32_t* mask, const float* bias,
                         bool dense, hipStream_t st);
// Backward of the bf16 prefill path (block-mean summaries): scratch size and the
// kernel sequence; ws must hold backward_workspace_bytes() bytes.
size_t backward_workspace_bytes(const dash_params& p, const Layout& L);
hipError_t launch_backward(const dash_params& p, const Layout& L, const void* q, const void* k, const void* v,
                           const void* d_o, const float* kbar, const uint32_t* mask,
                           const float* bias, const float* tau, void* dq, void* dk, void* dv, float* dkbar_out,
                           char* ws, hipStream_t st);
hipError_t launch_kbar_summarize_bwd(const dash_params& p, const Layout& L, const void* k, const float* qbar,
                                     const int64_t* qs, const float* dkbar, void* dk, float* dqbar,
                                     hipStream_t st);
hipError_t launch_decode_s2(const dash_params& p, const Layout& L, const void* q, const void* k,
                            const void* v, void* o, const uint32_t* mask, const float* bias,
                            float* partials, bool dense, hipStream_t st);

}  // namespace dash
