/*
 * dash_attn.h -- C ABI of the MI355X (gfx950) DashAttention library.
 *
 * The library implements the forward hot path of DashAttention (and the backward
 * pass of its prefill path, dash_attn_backward):
 *   Stage 0  block-mean key summaries                     (Sec. 3.1, Eq. 3 at a zero
 *                                                          summary query; Alg. 1)
 *   Stage 1  entmax chunk routing per query, GQA averaged  (Sec. 3.2, Eq. 4; Alg. 2)
 *            + the routing bias of the prior               (Sec. 3.4, Proposition 1)
 *   Stage 2  block-sparse softmax attention over the kept  (Sec. 3.3, Eq. 5-6 in the
 *            chunks with the bias added to the logits       bias form of Prop. 1; Alg. 3)
 *   plus a split-KV decode variant of Stage 2 (Sec. 3.5) and a dense reference
 *   attention (Eq. 1).
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates no device memory, never synchronises, reads no environment
 *     variable, and enqueues all work on `stream` (a hipStream_t passed as void*;
 *     NULL = the default stream).  Nothing a call computes depends on an earlier
 *     call: the only thing the library remembers is, per device, that a kernel's
 *     one-time opt-in to a large dynamic LDS size has been made (thread-safe), and the
 *     address of the scratch array of dash_attn_decode_static.
 *     Entry points may be called from several threads.
 *   - Tensors are [batch, head, token, head_dim] with head_dim contiguous; the
 *     other three strides are given in ELEMENTS in dash_params.  Rows must be
 *     16-byte aligned (base pointers 16-byte aligned, strides multiples of 8
 *     elements for bf16 / 4 for fp32).  bf16 tensors: one (batch, kv-head) slice
 *     of q, k, v, o (for q and o: the g_q heads of a kv-head) must span less than
 *     2 GiB, as the kernels address it with 32-bit byte offsets
 *     (DASH_EUNSUPPORTED otherwise).
 *   - Return value: DASH_OK (0) or a negative dash_status.  On a non-zero return
 *     nothing was enqueued (validation errors) or the outputs are undefined
 *     (DASH_ELAUNCH).  No exceptions or aborts cross this boundary.
 *   - Query index t of the n_q queries sits at sequence position
 *     n_kv - n_q + t.  Prefill passes n_q == n_kv; decode passes n_q == 1 and a
 *     KV cache that already contains the current token.
 *   - Causal: the routing candidates of a query are the complete chunks strictly
 *     before its own chunk (Alg. 2, "c < c_i"); its own chunk is always attended,
 *     causally masked, with bias 0 (the diagonal branch).  Non-causal: every
 *     chunk is a candidate, there is no diagonal branch, and n_kv must be a
 *     multiple of block_size (dense_attn and the size queries accept any n_kv).
 *   - kbar pointers may be NULL when n_kv < block_size (no complete chunk).
 *   - Limits of this build (DASH_EUNSUPPORTED beyond them): at most 2048 chunks per
 *     sequence, ceil(n_kv / block_size) <= 2048 (131072 tokens at chunks of 64, 262144 at
 *     128); a call with several queries (n_q > 1) that continues a longer cache must start
 *     at a multiple of 64 tokens, (n_kv - n_q) % 64 == 0; head_dim 64 or 128; block_size
 *     64 or 128; h_q / h_kv in {1, 2, 4, 8, 16}; window <= 8.
 */
#ifndef DASH_ATTN_H_
#define DASH_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum dash_status {
  DASH_OK = 0,
  DASH_EINVAL = -1,       /* NULL pointer, non-positive size, h_q % h_kv != 0, alpha <= 1, ...   */
  DASH_EUNSUPPORTED = -2, /* a combination this build has no kernel for (see dash_params)         */
  DASH_EWORKSPACE = -3,   /* workspace NULL / misaligned / smaller than dash_attn_workspace_bytes */
  DASH_ELAUNCH = -4       /* the HIP runtime reported an error at launch                          */
} dash_status;

enum { DASH_F32 = 0, DASH_BF16 = 1 };

typedef struct dash_params {
  int32_t batch;       /* >= 1                                                        */
  int32_t h_q;         /* query heads                                                 */
  int32_t h_kv;        /* key/value heads; g_q = h_q / h_kv in {1,2,4,8,16}           */
  int32_t n_q;         /* queries per sequence                                        */
  int32_t n_kv;        /* keys per sequence, n_kv >= n_q                              */
  int32_t head_dim;    /* 64 or 128                                                   */
  int32_t block_size;  /* chunk size B: 64 or 128                                     */
  int32_t causal;      /* 0 / 1                                                       */
  int32_t dtype;       /* DASH_F32 or DASH_BF16: element type of q, k, v, o           */
  float alpha;         /* entmax alpha, > 1                                           */
  float gamma;         /* Stage-1 temperature (Eq. 4), > 0                            */
  float sigma;         /* prior strength (Sec. 3.4), > 0; large => pure block mask    */
  float scale;         /* logit scale; <= 0 selects 1/sqrt(head_dim)                  */
  int32_t window;      /* causal only: complete chunks just before the query's own
                          that are always attended with bias 0 and leave the
                          candidate set (0: Alg. 2; 1: the diagonal block and the
                          last block, the local window of App. B.1); 0..8            */
  int64_t q_stride[3]; /* batch, head, token strides of q, in elements               */
  int64_t k_stride[3];
  int64_t v_stride[3];
  int64_t o_stride[3];
} dash_params;

/* Number of chunk slots per query in the list outputs below:
 * ceil(n_kv / block_size) (candidates plus the diagonal chunk). */
int32_t dash_list_stride(const dash_params* p);

/* Number of 32-bit words per query in the bit-packed chunk mask (Alg. 2's M,
 * 32 chunks per word, bit c%32 of word c/32): ceil(dash_list_stride / 32). */
int32_t dash_mask_words(const dash_params* p);

/* Bytes of device scratch the calls below need for these parameters (host
 * computation only).  The workspace must be 256-byte aligned.  One query serves every
 * call, dense_attn included, so it accepts what any of them accepts: a non-causal n_kv
 * that is not a multiple of block_size gets a size here and DASH_EINVAL from the
 * routing calls (a tail chunk has no summary), which dense_attn does not need. */
int dash_attn_workspace_bytes(const dash_params* p, size_t* out_bytes);

/* Stage 0 (Eq. 3 at zero summary query = uniform mean; Alg. 1).
 *   k     in  [batch,h_kv,n_kv,d] run dtype, strides k_stride
 *   kbar  out [batch,h_kv,T_c,d] fp32 contiguous, T_c = floor(n_kv/block_size):
 *         the mean of each complete chunk, accumulated exactly and rounded once
 *         to fp32.  This is the persistent chunk-summary cache of Sec. 3.5.
 *   first_chunk, n_chunks: the chunk range to (re)compute, e.g. only a chunk
 *         that was just completed during decoding; n_chunks < 0 means all. */
int dash_kbar_compress(const dash_params* p, const void* k, float* kbar,
                       int32_t first_chunk, int32_t n_chunks, void* stream);

/* Stage 0 with a learned summary query (Sec. 3.1 Eq. 3; Alg. 1): the summary of a
 * chunk is one softmax attention of the query over the chunk's own keys, with
 * the keys as values: kbar_c = softmax(K_c qbar scale)^T K_c (scale as in
 * dash_params, default 1/sqrt(d)).  A zero query gives dash_kbar_compress' result.
 *   k           in  as for dash_kbar_compress
 *   qbar        in  fp32 device pointer, 16-byte aligned, d contiguous; element
 *               (b, r, c) starts at b*qbar_stride[0] + r*qbar_stride[1] +
 *               c*qbar_stride[2] (elements; multiples of 4 for fp32 keys and of 8
 *               for bf16 keys; 0 broadcasts): one vector per kv-head (Sec. 3.1:
 *               strides {0, d, 0}) or one per chunk with the rotary embedding
 *               already applied (Alg. 1: strides {h_kv*T_c*d or 0, T_c*d, d})
 *   qbar_stride in  host pointer to 3 strides
 *   kbar        out as for dash_kbar_compress (fp32; scores, softmax and the
 *               weighted sum are evaluated in fp64 and rounded once)
 *   first_chunk, n_chunks: as for dash_kbar_compress.
 * Errors: DASH_EINVAL for null pointers, negative or misaligned strides or a chunk
 * range outside [0, T_c). */
int dash_kbar_summarize(const dash_params* p, const void* k, const float* qbar,
                        const int64_t* qbar_stride, float* kbar, int32_t first_chunk,
                        int32_t n_chunks, void* stream);

/* Stage 1 (Eq. 4, GQA averaging, Prop. 1 bias; Alg. 2).
 *   q     in  [batch,h_q,n_q,d]
 *   kbar  in  fp32 summaries from dash_kbar_compress
 * Outputs, each [batch,h_kv,n_q,...] contiguous; any of blk_cnt/blk_idx/tau may
 * be NULL (not produced); mask and blk_bias may be NULL, in which case they are
 * kept inside the workspace for dash_stage2_attend:
 *   mask     uint32 [.., dash_mask_words]   bit c set iff chunk c is attended
 *            (routed chunks, plus, when causal, the window chunks and the
 *            diagonal chunk)
 *   blk_cnt  int32  [..]                    number of attended chunks
 *   blk_idx  int32  [.., dash_list_stride]  their ids, ascending (diagonal last)
 *   blk_bias fp32   [.., dash_list_stride]  d_{i,c} in the same order (0 for the
 *            window and diagonal chunks); entries past blk_cnt are unspecified
 *   tau      fp32   [batch,h_q,n_q]         entmax threshold of every query head
 *            in the domain x = gamma (alpha-1) <q,kbar> scale (0 if no candidate) */
int dash_stage1_route(const dash_params* p, const void* q, const float* kbar,
                      uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                      float* blk_bias, float* tau,
                      void* workspace, size_t workspace_bytes, void* stream);

/* Stage 2 (Eq. 6 in the bias form of Prop. 1; Alg. 3): for every query,
 * softmax over the tokens of its attended chunks of (q.k*scale + d), times v.
 *   mask, blk_bias: as produced by dash_stage1_route (NULL = read them from the
 *   same workspace the Stage-1 call used).  o out [batch,h_q,n_q,d]. */
int dash_stage2_attend(const dash_params* p, const void* q, const void* k,
                       const void* v, void* o, const uint32_t* mask,
                       const float* blk_bias,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Whole prefill path: Stage 0 (all chunks) -> Stage 1 -> Stage 2.
 * kbar is an output (the caller keeps it as the summary cache); the list
 * outputs are optional as in dash_stage1_route. */
int dash_attn_prefill(const dash_params* p, const void* q, const void* k,
                      const void* v, void* o, float* kbar, uint32_t* mask,
                      int32_t* blk_cnt, int32_t* blk_idx, float* blk_bias,
                      float* tau, void* workspace, size_t workspace_bytes,
                      void* stream);

/* One decode step (n_q must be 1; always causal): Stage 1 on the cached
 * summaries, then split-KV Stage 2 and the log-sum-exp merge of the partial
 * results (Sec. 3.5).  kbar_cache is in/out: if the current token completes a
 * chunk (n_kv % block_size == 0) that chunk's summary is written by the same
 * launch that routes (it is the query's own chunk, not a candidate of this
 * step); the other entries are read only.  List outputs optional as above. */
int dash_attn_decode(const dash_params* p, const void* q, const void* k_cache,
                     const void* v_cache, float* kbar_cache, void* o,
                     uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                     float* blk_bias, float* tau,
                     void* workspace, size_t workspace_bytes, void* stream);

/* dash_attn_decode for callers that cannot allocate device memory or carry a workspace
 * (code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc):
 * the same step with the same kernels and the same results, except that the scratch
 * (attended-chunk lists when not asked for, split-KV partial results)
 * lives in an 8 MiB array inside the library, one per GPU, held until the process ends.
 * The call allocates nothing.  DASH_EWORKSPACE if dash_attn_workspace_bytes(p) exceeds
 * 8 MiB (the 128k-token decode step of 16 sequences x 8 kv-heads needs 2.1 MiB).
 * Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (different
 * streams or threads) race; nothing in it has to survive from one call to the next. */
int dash_attn_decode_static(const dash_params* p, const void* q, const void* k_cache,
                            const void* v_cache, float* kbar_cache, void* o,
                            uint32_t* mask, int32_t* blk_cnt, int32_t* blk_idx,
                            float* blk_bias, float* tau, void* stream);

/* One decode step for a batch of sequences of different lengths sharing one cache
 * allocation (Sec. 3.5, the decoding regime of a serving loop): as
 * dash_attn_decode, except that sequence b holds seq_lens[b] tokens (its current
 * token included) in rows 0 .. seq_lens[b]-1 of its k_cache / v_cache slice and
 * its query sits at position seq_lens[b]-1; p->n_kv is the capacity (row count)
 * of the cache and sizes the strides, lists and workspace.
 *   seq_lens      in  int32 device pointer [batch]; values outside [1, n_kv] are
 *                 clamped into that range by the kernels (never read out of bounds)
 *   update_cache  != 0: the block-mean summary of a chunk that a sequence's current
 *                 token completes (seq_lens[b] % block_size == 0) is written into
 *                 kbar_cache, per sequence; 0: kbar_cache is read only (the
 *                 caller maintains it, e.g. with dash_kbar_summarize)
 * kbar_cache [batch,h_kv,floor(n_kv/block),d]; only the summaries of a sequence's
 * complete chunks before its current one are read.  bf16 only (DASH_EUNSUPPORTED
 * otherwise); DASH_EINVAL for a NULL seq_lens. */
int dash_attn_decode_ragged(const dash_params* p, const void* q, const void* k_cache,
                            const void* v_cache, float* kbar_cache, const int32_t* seq_lens,
                            int32_t update_cache, void* o, uint32_t* mask, int32_t* blk_cnt,
                            int32_t* blk_idx, float* blk_bias, float* tau, void* workspace,
                            size_t workspace_bytes, void* stream);

/* Dense reference attention (Eq. 1), same tensors and layouts, no routing.
 * The denominator of every speed-up figure.  alpha/gamma/sigma/block_size are
 * ignored except for validation. */
int dense_attn(const dash_params* p, const void* q, const void* k, const void* v,
               void* o, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of dash_attn_prefill (end of Sec. 3.3: the output is differentiable in
 * q, k, v and the prior, and the gradient reaches the Stage-1 weights and the
 * Stage-0 summaries; Sec. 3.5: the backward pass reuses the forward's chunk mask,
 * the entmax Jacobian being zero outside the support).  Within the forward's
 * support the gradient is exact; at a support change the map is only piecewise
 * differentiable and the Jacobian of the current support is used.
 *   q, k, v        in  the forward's inputs (same dash_params)
 *   d_o            in  gradient of the loss with respect to the forward's output o,
 *                  layout and strides of o (o itself is not needed: <dO, o> is
 *                  recomputed in fp32)
 *   kbar           in  the summaries Stage 1 routed on (fp32): the block means the
 *                  forward wrote, or the learned ones of dash_kbar_summarize
 *   mask, blk_bias, tau  in  the forward's Stage-1 outputs (all three required)
 *   dq, dk, dv     out gradients in the run dtype with the strides of q, k, v;
 *                  every element is written
 *   dkbar          out, optional, fp32 [batch,h_kv,T_c,d] contiguous.  NULL: the
 *                  summaries are block means and dk includes the path through the
 *                  routing scores into them (each key of a complete chunk receives
 *                  1/B of its summary's gradient).  Otherwise the summaries are an
 *                  input of their own (e.g. from dash_kbar_summarize): their
 *                  gradient is written here and dk holds the attention part only;
 *                  dash_kbar_summarize_backward then carries it on to the keys and
 *                  the summary query
 *   workspace      device scratch of dash_attn_backward_workspace_bytes bytes,
 *                  256-byte aligned (separate from, or reusing, the forward's; two
 *                  calls in flight must not share it)
 * For alpha > 2 the entmax slope is unbounded at the edge of the support, so rows
 * with a chunk close to its threshold have gradients only as accurate as the fp32
 * scores allow; alpha <= 3 only (checked against the oracle up to there;
 * DASH_EUNSUPPORTED above).  n_q == n_kv only (DASH_EUNSUPPORTED otherwise).  bf16 tensors take the matrix-core
 * kernels; fp32 tensors take plain fp32 kernels that accumulate dk and dv with
 * atomics (a correctness vehicle like the fp32 forward, sums in no fixed order);
 * DASH_EINVAL for a NULL pointer. */
int dash_attn_backward_workspace_bytes(const dash_params* p, size_t* out_bytes);
int dash_attn_backward(const dash_params* p, const void* q, const void* k, const void* v,
                       const void* d_o, const float* kbar,
                       const uint32_t* mask, const float* blk_bias, const float* tau,
                       void* dq, void* dk, void* dv, float* dkbar,
                       void* workspace, size_t workspace_bytes, void* stream);

/* Backward of dash_kbar_summarize (Eq. 3; the trainable Stage 0 of Sec. 3.3's last
 * paragraph): with a = softmax(K_c qbar scale) per chunk and the summaries'
 * gradient dkbar, adds a dkbar_c^T + scale ds qbar^T (ds = a (K_c dkbar_c - <a, K_c dkbar_c>))
 * to the keys' gradient and writes the summary query's gradient per chunk.
 *   k, qbar, qbar_stride  in   as for dash_kbar_summarize
 *   dkbar   in      fp32 [batch,h_kv,T_c,d] (dash_attn_backward's dkbar output)
 *   dk      in/out  run dtype, strides of k: rows of complete chunks are read,
 *                   incremented and written back
 *   dqbar   out     fp32 [batch,h_kv,T_c,d]: the gradient of the query of every
 *                   chunk; a query shared by several chunks (stride 0) has their sum
 *                   as its gradient, which is left to the caller
 * Errors as for dash_kbar_summarize. */
int dash_kbar_summarize_backward(const dash_params* p, const void* k, const float* qbar,
                                 const int64_t* qbar_stride, const float* dkbar, void* dk,
                                 float* dqbar, void* stream);

/* Static, NUL-terminated description of a dash_status. */
const char* dash_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif /* DASH_ATTN_H_ */
