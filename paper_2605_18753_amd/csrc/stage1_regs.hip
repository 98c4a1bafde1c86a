// Stage 1 with the score rows held in registers (bf16 prefill, rows of up to 1536
// candidate chunks): the same routing as stage1.hip (Sec. 3.2, Eq. 4; Alg. 2; the bias of
// Proposition 1), the scores going from the matrix cores to the lists without being
// written to LDS or HBM.
//
// Why a second kernel.  stage1.hip keeps the score rows of a workgroup in LDS, which
// limits a workgroup to 16-64 rows, and every workgroup reads the split summaries of all
// its candidate chunks (768 bytes per chunk at d = 128): that traffic, not arithmetic,
// is what its time goes to.  Here the accumulator layout of v_mfma_f32_16x16x32_bf16 is
// used as the solver's layout: with A = 16 query rows and B = 16 chunk summaries, lane
// (m = lane % 16, kq = lane / 16) receives the scores of rows 4 kq .. 4 kq + 3 at chunk
// 16 ct + m, so after all chunk tiles the 16 lanes of a DPP row hold four complete score
// rows (chunk c in lane c % 16), which is what the 16-lane threshold solver wants.  Rows
// are ordered token-major (row = token * g_q + head), so those four rows are 4 / g_q
// tokens (g_q <= 4) or a quarter or half of one token's heads (g_q = 16, 8: the group
// weight is then completed across DPP rows).  A wave owns 16 rows and walks all chunk
// tiles; the waves of a workgroup share every tile of split summaries through LDS
// (buffer_load ... lds, a ring of three or five stages), so a tile is fetched once per workgroup:
//   rows of up to 256 chunks:  8 waves x 16 rows = 128 rows, at most 64 score registers
//                              per lane: two workgroups per CU (four waves per SIMD);
//   rows of up to 512 chunks:  the same with up to 128 score registers, one workgroup
//                              per CU;
//   rows of up to 1536 chunks: the 8 waves form 4 pairs (64 rows); the waves of a pair
//                              hold the first and the second half of the same 16 rows
//                              (up to 192 score registers per lane) and combine their
//                              partial sums through LDS, one barrier per solver step
//                              (d = 128 only).
//
// Arithmetic is that of stage1.hip step by step (scores: the same three MFMAs per d
// slice into the same two accumulators; threshold: the same bracketed Newton iteration
// with the same in-lane and DPP-row summation order), so for rows of up to 512 chunks
// masks, counts, ids and thresholds are bit-identical to that kernel's; the group weight
// of g_q = 8, 16, mu = mean ln w, and the sums of a row split over two waves are added in
// another order and may differ in the last place.
//
// This file is compiled once per GQA group size (-DDASH_S1R_G=1, 2, 4, 8, 16), each
// object providing launch_s1_regs_g<G>.
#include <math.h>

#include <type_traits>

#include "common.h"
#include "dash_internal.h"
#include "lds_copy.h"
#include "stage1_common.h"

namespace dash {

#ifndef DASH_S1R_G
#error "compile with -DDASH_S1R_G=<GQA group size: 1, 2, 4, 8 or 16>"
#endif

template <int D, int STAGES_> struct RegsCfg {
  static constexpr int NW = 8;                               // waves per workgroup
  static constexpr int KS = D / 32;                          // contraction steps per product
  static constexpr int PART_BYTES = D * 2;                   // one bf16 piece of a summary
  static constexpr int ROW_BYTES = 3 * PART_BYTES;           // the three pieces of one chunk
  static constexpr int SPP = D / 8;                          // 16-byte slots per piece
  static constexpr int SPR = 3 * SPP;                        // ... per chunk
  static constexpr int TILE_BYTES = 16 * ROW_BYTES;          // 16 chunks
  static constexpr int IPW = (TILE_BYTES / 1024 + NW - 1) / NW;   // copy instructions per wave and tile
  static constexpr int STAGE_BYTES = IPW * NW * 1024;        // tile + room for the surplus instructions' zeros
  static constexpr int STAGES = STAGES_;                     // ring depth: 3 where two workgroups share a CU, 5 where one has it
  static_assert(STAGES >= 2 && STAGES <= 5, "the counted waits below cover up to three newer tiles in flight");
  static constexpr int RING_BYTES = STAGES * STAGE_BYTES;
  static constexpr int XCH_FLOATS = 2 * NW * 4 * 12;         // exchange area of the wave pairs (see PairX)
  static constexpr int LDS_BYTES = RING_BYTES + XCH_FLOATS * 4;
};

// Exchange between the two waves that share 16 rows (waves w and w ^ 4): DPP row kq of a
// wave hands up to 8 floats to DPP row kq of its partner (swap), or every wave a flag to
// the whole workgroup (any_flag).  One barrier per call, two alternating buffers: every
// wave of the workgroup makes the same sequence of calls.
struct PairX {
  float* area;   // LDS: [2 buffers][8 waves][4 DPP rows][12]: 8 values, 1 flag, 3 unused
  int wave, kq, m, buf;
  template <int K>
  __device__ __forceinline__ bool swap(const float (&mine)[K], float (&other)[K]) {
    static_assert(K <= 8, "at most 8 values per exchange");
    float* slot = area + ((buf * 8 + wave) * 4 + kq) * 12;
    if (m == 0) {
#pragma unroll
      for (int k = 0; k < K; k++) slot[k] = mine[k];
    }
    __syncthreads();
    const float* o = area + ((buf * 8 + (wave ^ 4)) * 4 + kq) * 12;
#pragma unroll
    for (int k = 0; k < K; k++) other[k] = o[k];
    buf ^= 1;
    return false;
  }
  // whether any wave of the workgroup raises its flag
  __device__ __forceinline__ bool any_flag(bool flag) {
    float* slot = area + ((buf * 8 + wave) * 4) * 12 + 8;
    if (m == 0 && kq == 0) *slot = flag ? 1.f : 0.f;
    __syncthreads();
    bool any = false;
#pragma unroll
    for (int w = 0; w < 8; w++) any = any || area[((buf * 8 + w) * 4) * 12 + 8] != 0.f;
    buf ^= 1;
    return any;
  }
};

// [x - tau]_+ for a threshold inside the solver's bracket: tau >= max - 1, so x - tau <= 1
// and the clamp of the subtraction to [0, 1] (one instruction) is the positive part;
// x = -inf (an absent chunk) and -inf - -inf give 0.
__device__ __forceinline__ float excess(float x, float tau) { return __builtin_amdgcn_fmed3f(x - tau, 0.f, 1.f); }

// One bracketed Newton step of row state (tau, lo, hi, done) from the sums F = sum u^p,
// G = sum u^(p-1) at tau: the update of stage1.hip's 16-lane solver.
template <int MODE>
__device__ __forceinline__ void newton_step(float F, float G, float p, int n_cand, float& tau, float& lo, float& hi,
                                            bool& done) {
  if (done) return;
  const float f = F - 1.f;
  if (f == 0.f) { done = true; return; }
  if (f > 0.f) lo = tau; else hi = tau;
  const float mid = 0.5f * (lo + hi);
  float cand = (MODE == MODE_BISECT || !(G > 0.f)) ? mid : tau + f / (p * G);
  if (MODE != MODE_BISECT && cand == tau) { done = true; return; }   // Newton step below the fp32 spacing of tau
  if (!(cand > lo && cand < hi)) cand = mid;
  if (!(cand > lo && cand < hi)) { done = true; tau = lo; return; }  // bracket closed
  // alpha = 1.5: a Newton step s from the left leaves an error of about (n / 2G) s^2;
  // once that is below 2e-8 the step is final
  if (MODE == MODE_P2 && f > 0.f && cand != mid) {
    const float st = cand - tau;
    if ((float)n_cand * st * st < 4e-8f * G) done = true;
  }
  tau = cand;
}

// Threshold of four score rows per lane at once (rows j = 0..3; row j of DPP row kq is
// spread over the row's 16 lanes, NT values per lane; with SPLIT = 2 over the 16 lanes
// of this wave and of its partner): the iteration of stage1.hip's 16-lane solver, row by
// row the same operations in the same order.
template <int NT, int MODE, int SPLIT>
__device__ __forceinline__ void solve4(const f32x4 (&v)[NT], int n_cand, float alpha, float p, float (&tau)[4],
                                       PairX& px, int half) {
  float mloc[4], lo[4], hi[4], mx[4];
  bool done[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < NT; t++) m = fmaxf(m, v[t][j]);
    mloc[j] = m;
    mx[j] = row16_reduce(m, OpMax());
  }
  if constexpr (SPLIT == 2) {
    float other[4];
    px.swap(mx, other);
#pragma unroll
    for (int j = 0; j < 4; j++) mx[j] = fmaxf(mx[j], other[j]);
  }
#pragma unroll
  for (int j = 0; j < 4; j++) {
    lo[j] = mx[j] - 1.f;
    hi[j] = mx[j] - exp2f(-(alpha - 1.f) * log2f((float)n_cand));
    tau[j] = lo[j];
    done[j] = false;
  }
  if constexpr (MODE != MODE_BISECT) {
    // warm start on the 16 lane maxima (a subset: its root and every Newton iterate from
    // the left on it are lower bounds of tau)
#pragma unroll
    for (int j = 0; j < 4; j++) {
#pragma unroll
      for (int it = 0; it < 5; it++) {
        float f, g;
        pow_terms<MODE>(excess(mloc[j], tau[j]), p, f, g);
        asm volatile("" : "+v"(f), "+v"(g));
        const float F = row16_reduce(f, OpAdd()), G = row16_reduce(g, OpAdd());
        if (F > 1.f && G > 0.f) tau[j] += (F - 1.f) / (p * G);
      }
    }
    if constexpr (SPLIT == 2) {   // each wave started on its own half: the larger lower bound serves both
      float other[4];
      px.swap(tau, other);
#pragma unroll
      for (int j = 0; j < 4; j++) tau[j] = fmaxf(tau[j], other[j]);
    }
#pragma unroll
    for (int j = 0; j < 4; j++) {
      tau[j] = fmaxf(tau[j], lo[j]);
      if (!(tau[j] < hi[j])) tau[j] = lo[j];
    }
  }
  for (int it = 0; it < 64; it++) {
    float FG[8];
#pragma unroll
    for (int j = 0; j < 4; j++) {
      float F = 0.f, G = 0.f;
#pragma unroll
      for (int t = 0; t < NT; t++) {
        float f, g;
        pow_terms<MODE>(excess(v[t][j], tau[j]), p, f, g);
        F += f; G += g;
      }
      // keep the partial sums as rounded values: a multiply contracted into the first
      // cross-lane add would make the lanes of a row disagree by an ulp
      asm volatile("" : "+v"(F), "+v"(G));
      FG[j] = row16_reduce(F, OpAdd());
      FG[4 + j] = row16_reduce(G, OpAdd());
    }
    if constexpr (SPLIT == 2) {
      // both waves add first half + second half in that order, so they take the same step
      float other[8];
      px.swap(FG, other);
#pragma unroll
      for (int k = 0; k < 8; k++) FG[k] = half == 0 ? FG[k] + other[k] : other[k] + FG[k];
    }
    bool all_done = true;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      newton_step<MODE>(FG[j], FG[4 + j], p, n_cand, tau[j], lo[j], hi[j], done[j]);
      all_done = all_done && done[j];
    }
    bool busy = __any(!all_done);
    if constexpr (SPLIT == 2) busy = px.any_flag(busy);   // the loop ends for the whole workgroup at once
    if (!busy) break;
  }
}

// One workgroup's rows with NT chunk tiles of 16 per wave.  SPLIT = 1: every wave holds
// whole rows (n_cand <= 16 NT).  SPLIT = 2: waves w and w + 4 hold chunk tiles
// [0, NT) and [NT, 2 NT) of the same 16 rows (n_cand <= 32 NT).
template <int D, int G, int MODE, int SPLIT, int NT, int STAGES>
__device__ __forceinline__ void regs_tile(const S1Args& a, char* lds, int b, int r, int tok0, int ntile) {
  using C = RegsCfg<D, STAGES>;
  constexpr int TPL = G >= 4 ? 1 : 4 / G;     // tokens per lane (its four rows are TPL tokens x HPL heads)
  constexpr int HPL = G >= 4 ? 4 : G;         // heads of one token held by a lane
  constexpr int KQT = G > 4 ? G / 4 : 1;      // DPP rows that share one token (g_q = 8: 2, g_q = 16: 4)
  constexpr int TPW = 16 / G;                 // tokens per wave
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int half = SPLIT == 2 ? wave >> 2 : 0;
  const int m = lane & 15, kq = lane >> 4;
  const int tok_w0 = tok0 + (SPLIT == 2 ? wave & 3 : wave) * TPW;
  // The wave's tokens share one candidate set (they lie in one chunk); the workgroup's may
  // span two chunks, so all waves walk the tiles of the longest set (ntile) and a wave
  // treats the chunks past its own set as absent.
  int n_cand = a.causal ? max((a.pos0 + min(tok_w0, a.tok_end - 1)) / a.block - a.window, 0) : a.t_c;
  if (n_cand > a.t_c) n_cand = a.t_c;
  PairX px{reinterpret_cast<float*>(lds + C::RING_BYTES), wave, kq, m, 0};

  f32x4 v[NT];   // scores, then probabilities: v[t][j] = row 4 kq + j at chunk 16 (half NT + t) + m
#pragma unroll
  for (int t = 0; t < NT; t++) v[t] = f32x4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  float tau[4] = {0.f, 0.f, 0.f, 0.f};

  if (ntile > 0) {
    // ---- Q fragments (operand A): row m of the wave, d 32 ks + 8 kq .. + 7 ----------
    bf16x8 qf[C::KS];
    {
      const int tok = tok_w0 + m / G, head = r * G + m % G;
      const uint16_t* qp = (const uint16_t*)a.q + b * a.qs_b + head * a.qs_h +
                           (int64_t)(tok < a.n_q ? tok : a.n_q - 1) * a.qs_t + kq * 8;
#pragma unroll
      for (int ks = 0; ks < C::KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
#pragma unroll
      for (int ks = 0; ks < C::KS; ks++) asm volatile("" : "+v"(qf[ks]));   // landed before the counted waits
    }
    // ---- tiles of split summaries: global -> LDS --------------------------------------
    // A tile is 16 chunks x 3 pieces x d bf16, contiguous in memory.  Copy instruction i
    // of the workgroup fills LDS slots 64 i .. 64 i + 63 (16 bytes each); slot s holds, of
    // chunk s / SPR, piece (s % SPR) / SPP, the 16-byte unit (s % SPP) ^ (chunk % SPP): the
    // XOR spreads the 16 chunks a B-operand read touches over all banks.  Wave w issues
    // instructions w and w + 8; those past the end of the tile (and chunks past the last
    // summary) read zeros through the bounded resource.
    const u32x4 ks_rs = make_rsrc(a.ksplit + ((int64_t)b * a.h_kv + r) * a.t_c * 3 * D, (int64_t)a.t_c * C::ROW_BYTES);
    uint32_t src_off[C::IPW];
#pragma unroll
    for (int i = 0; i < C::IPW; i++) {
      const int s = (wave + C::NW * i) * 64 + lane;
      const int c = s / C::SPR, piece = (s % C::SPR) / C::SPP, unit = (s % C::SPP) ^ (c & (C::SPP - 1));
      src_off[i] = s < 16 * C::SPR ? (uint32_t)(c * C::ROW_BYTES + piece * C::PART_BYTES + unit * 16) : 0xfffffff0u;
    }
    const uint32_t lds0 = lds_addr_of(lds);
    auto issue_tile = [&](int gt) __attribute__((always_inline)) {
      const uint32_t dst = lds0 + (uint32_t)(gt % C::STAGES) * C::STAGE_BYTES + (uint32_t)wave * 1024u;
#pragma unroll
      for (int i = 0; i < C::IPW; i++)
        copy16_to_lds(ks_rs, dst + i * C::NW * 1024, src_off[i], (uint32_t)gt * C::TILE_BYTES);
    };
    // operand B read address inside a stage: chunk m, unit (4 ks + kq) ^ (m % SPP) of a piece
    const uint32_t b_rd = (uint32_t)(m * C::ROW_BYTES);
#pragma unroll
    for (int gt = 0; gt < C::STAGES - 1; gt++)
      if (gt < ntile) issue_tile(gt);
    // all waves take part in the copy of, and the barrier for, every tile; a wave runs the
    // matrix cores on the tiles of its own half only
#pragma nounroll
    for (int h = 0; h < SPLIT; h++) {
#pragma unroll
      for (int t = 0; t < NT; t++) {
        const int gt = h * NT + t;
        if (gt < ntile) {
          // this wave's copies of tile gt have landed (newer tiles may stay in flight); the
          // barrier publishes everybody's and retires the reads of tile gt - 1, whose stage
          // the next copy overwrites
          const int newer = min(ntile - 1 - gt, C::STAGES - 2);
          if (newer <= 0) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(0) : "memory");
          else if (newer == 1) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(C::IPW) : "memory");
          else if (newer == 2) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(2 * C::IPW) : "memory");
          else asm volatile("s_waitcnt vmcnt(%0)" :: "n"(3 * C::IPW) : "memory");
          __syncthreads();
          if (gt + C::STAGES - 1 < ntile) issue_tile(gt + C::STAGES - 1);
          if (h == half) {
            const char* sb = lds + (gt % C::STAGES) * C::STAGE_BYTES + b_rd;
            f32x4 acc_hi = {0.f, 0.f, 0.f, 0.f}, acc_lo = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < C::KS; ks++) {
              const int unit = ((4 * ks + kq) ^ (m & (C::SPP - 1))) * 16;
              const bf16x8 s0 = *reinterpret_cast<const bf16x8*>(sb + unit);
              const bf16x8 s1 = *reinterpret_cast<const bf16x8*>(sb + C::PART_BYTES + unit);
              const bf16x8 s2 = *reinterpret_cast<const bf16x8*>(sb + 2 * C::PART_BYTES + unit);
              acc_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], s0, acc_hi, 0, 0, 0);
              acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], s1, acc_lo, 0, 0, 0);
              acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], s2, acc_lo, 0, 0, 0);
            }
            if (gt * 16 + m < n_cand) {
#pragma unroll
              for (int j = 0; j < 4; j++) v[t][j] = (acc_hi[j] + acc_lo[j]) * a.xscale;
            }
          }
        }
      }
    }
  }
  // With SPLIT = 2 the solver exchanges through LDS behind barriers, so every wave of the
  // workgroup enters it (ntile > 0 there; a wave with no candidate of its own still
  // serves its partner and keeps the barrier count).
  if (SPLIT == 2 || n_cand > 0) {
    // ---- thresholds, then probabilities in place ---------------------------------------
    solve4<NT, MODE, SPLIT>(v, max(n_cand, 1), a.alpha, a.pexp, tau, px, half);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int j = 0; j < 4; j++) v[t][j] = pow_p<MODE>(excess(v[t][j], tau[j]), a.pexp);
  }
  if (a.tau && m == 0 && half == 0) {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int row = 4 * kq + j;
      const int tok = tok_w0 + row / G, head = r * G + row % G;
      if (tok < a.tok_end) a.tau[((int64_t)b * a.h_q + head) * a.n_q + tok] = n_cand > 0 ? tau[j] : 0.f;
    }
  }

  // ---- group weights, bias, lists: one token per DPP row (or per KQT rows) at a time ------
  const float inv_g = 1.f / (float)G;
#pragma unroll
  for (int tt = 0; tt < TPL; tt++) {
    const int tok = tok_w0 + (KQT > 1 ? kq / KQT : kq * TPL + tt);
    const bool tok_ok = tok < a.tok_end && (kq % KQT) == 0;   // of the rows sharing a token the first one writes
    float slog = 0.f, nsup = 0.f;
#pragma unroll
    for (int t = 0; t < NT; t++) {
      float s = 0.f;
      if ((half * NT + t) * 16 + m < n_cand) {
#pragma unroll
        for (int h = 0; h < HPL; h++) s += v[t][tt * HPL + h];
      }
      if constexpr (KQT >= 2) s += __shfl_xor(s, 16);
      if constexpr (KQT == 4) s += __shfl_xor(s, 32);
      s *= inv_g;
      // ln via the hardware log2 (about 1 ulp): ample for a bias that is divided by sigma
      const float lw = s > 0.f ? __builtin_amdgcn_logf(s) * 0.6931471805599453f : INFINITY;   // +inf: not routed
      if (s > 0.f) { slog += lw; nsup += 1.f; }
      v[t][tt * HPL] = lw;   // the token's probabilities are not needed any more
    }
    asm volatile("" : "+v"(slog));
    slog = row16_reduce(slog, OpAdd());
    nsup = row16_reduce(nsup, OpAdd());
    int running = 0;   // list position of this wave's first routed chunk
    if constexpr (SPLIT == 2) {
      const float mine[2] = {slog, nsup};
      float other[2];
      px.swap(mine, other);
      if (half == 1) running = (int)other[1];   // the first half's routed chunks come first
      slog = half == 0 ? slog + other[0] : other[0] + slog;
      nsup = half == 0 ? nsup + other[1] : other[1] + nsup;
    }
    const int total = (int)nsup;   // routed chunks of the token
    const float mu = nsup > 0.f ? slog / nsup : 0.f;
    const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + (tok_ok ? tok : 0);
    int32_t* oidx = a.idx ? a.idx + base * a.t_all : nullptr;
    float* obias = a.bias + base * a.t_all;
    // mask word w of the token is kept by lane w % 16 of its DPP row, in slot w / 16
    uint32_t word[4] = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int t = 0; t < NT; t++) {
      const bool member = v[t][tt * HPL] != INFINITY;
      const uint64_t bal = __ballot(member);
      const uint32_t field = (uint32_t)(bal >> (16 * kq)) & 0xffffu;
      const int gt = half * NT + t;   // NT is even: a mask word lies in one half
      if (m == ((gt >> 1) & 15)) {
#pragma unroll
        for (int i = 0; i < 4; i++)
          if ((gt >> 5) == i) word[i] |= field << (16 * (t & 1));
      }
      if (member && tok_ok) {
        const int pos = running + __popc(field & ((1u << m) - 1u));
        if (oidx) oidx[pos] = gt * 16 + m;
        obias[pos] = (v[t][tt * HPL] - mu) * a.inv_sigma;
      }
      running += __popc(field);
    }
    // words [w_lo, w_hi) are this wave's to write: those of its tiles, and for the last
    // half every word behind them (local chunks, zeros)
    const int w_lo = half * (NT / 2);
    const int w_hi = half == SPLIT - 1 ? a.words : (half + 1) * (NT / 2);
    if (a.causal) {
      // the always-attended local set, bias 0: the chunks of the window, then the query's own
      const int cd = (a.pos0 + min(tok, a.n_q - 1)) / a.block;
      const int c0 = max(cd - a.window, 0);
      for (int c = c0; c <= cd; c++) {
        if (m == 0 && tok_ok && half == 0) {
          if (oidx) oidx[total + c - c0] = c;
          obias[total + c - c0] = 0.f;
        }
        if (((c >> 5) & 15) == m) {
#pragma unroll
          for (int i = 0; i < 4; i++)
            if ((c >> 9) == i) word[i] |= 1u << (c & 31);
        }
      }
      if (tok_ok && half == 0 && a.cnt && m == 0) a.cnt[base] = total + cd - c0 + 1;
    } else if (tok_ok && half == 0 && a.cnt && m == 0) {
      a.cnt[base] = total;
    }
    if (tok_ok) {
      uint32_t* om = a.mask + base * a.words;
#pragma unroll
      for (int i = 0; i < 4; i++) {   // at most 2048 chunks: 64 words
        const int w = 16 * i + m;
        if (w >= w_lo && w < w_hi) om[w] = word[i];
      }
    }
  }
}

// the longest candidate set among the workgroup's tokens: that of its last token
__device__ __forceinline__ int regs_ntile(const S1Args& a, int tok0, int tokt) {
  int n_max = a.causal ? max((a.pos0 + min(tok0 + tokt - 1, a.tok_end - 1)) / a.block - a.window, 0) : a.t_c;
  if (n_max > a.t_c) n_max = a.t_c;
  return (n_max + 15) >> 4;
}

// The three kernels.  VAR 0: rows of up to 256 chunks, whole rows per wave, at most 64 score
// registers per lane, so two workgroups (four waves per SIMD) share a CU, three-stage ring.
// VAR 1: rows of up to 512 chunks, whole rows per wave, one workgroup per CU, five-stage ring.
// VAR 2: rows of up to 1536 chunks split over wave pairs, 64 rows per workgroup.
template <int VAR> struct RegsVar {
  static constexpr int SPLIT = VAR == 2 ? 2 : 1;
  static constexpr int STAGES = VAR == 0 ? 3 : 5;
  static constexpr int MIN_WG = VAR == 0 ? 2 : 1;   // workgroups per CU the register budget is set for
};

template <int D, int G, int MODE, int VAR>
__global__ __launch_bounds__(512, RegsVar<VAR>::MIN_WG) void s1_regs_kernel(S1Args a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr int SPLIT = RegsVar<VAR>::SPLIT, ST = RegsVar<VAR>::STAGES;
  constexpr int TOKT = (8 / SPLIT) * 16 / G;   // tokens per workgroup
  const int hb = a.h_kv * a.batch;
  const int hbi = blockIdx.x % hb;
  const int tile = (int)(gridDim.x / hb) - 1 - (int)(blockIdx.x / hb);   // longest rows first
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int tok0 = a.tok_base + tile * TOKT;
  const int ntile = regs_ntile(a, tok0, TOKT);
  if constexpr (VAR == 0) {
    if (ntile <= 4) regs_tile<D, G, MODE, 1, 4, ST>(a, lds, b, r, tok0, ntile);
    else if (ntile <= 8) regs_tile<D, G, MODE, 1, 8, ST>(a, lds, b, r, tok0, ntile);
    else regs_tile<D, G, MODE, 1, 16, ST>(a, lds, b, r, tok0, ntile);
  } else if constexpr (VAR == 1) {
    regs_tile<D, G, MODE, 1, 32, ST>(a, lds, b, r, tok0, ntile);
  } else {
    if (ntile <= 64) regs_tile<D, G, MODE, 2, 32, ST>(a, lds, b, r, tok0, ntile);
    else regs_tile<D, G, MODE, 2, 48, ST>(a, lds, b, r, tok0, ntile);
  }
}

template <auto kern>
static hipError_t launch_regs_k(const S1Args& a, dim3 grid, size_t lds, hipStream_t st) {
  static LdsOptIn opt_in;   // one per kernel (kern is a template argument)
  if (hipError_t e = allow_dyn_lds((const void*)kern, lds, opt_in); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(512), lds, st, a);
  return hipGetLastError();
}

template <int D, int G, int VAR>
static hipError_t launch_regs(const S1Args& a, int mode, hipStream_t st) {
  constexpr size_t lds = RegsCfg<D, RegsVar<VAR>::STAGES>::LDS_BYTES;
  constexpr int tokt = (8 / RegsVar<VAR>::SPLIT) * 16 / G;
  const dim3 grid((unsigned)(((a.tok_end - a.tok_base + tokt - 1) / tokt) * a.h_kv * a.batch), 1, 1);
  switch (mode) {
    case MODE_P1: return launch_regs_k<s1_regs_kernel<D, G, MODE_P1, VAR>>(a, grid, lds, st);
    case MODE_P2: return launch_regs_k<s1_regs_kernel<D, G, MODE_P2, VAR>>(a, grid, lds, st);
    case MODE_P4: return launch_regs_k<s1_regs_kernel<D, G, MODE_P4, VAR>>(a, grid, lds, st);
    case MODE_GEN: return launch_regs_k<s1_regs_kernel<D, G, MODE_GEN, VAR>>(a, grid, lds, st);
    default: return launch_regs_k<s1_regs_kernel<D, G, MODE_BISECT, VAR>>(a, grid, lds, st);
  }
}

#define DASH_CAT2(a_, b_) a_##b_
#define DASH_CAT(a_, b_) DASH_CAT2(a_, b_)

// The launch for GQA group size DASH_S1R_G.  The caller has checked that the longest row
// has max_cand <= 512 candidates, or max_cand <= 1536 with head_dim 128.
hipError_t DASH_CAT(launch_s1_regs_g, DASH_S1R_G)(const S1Args& a, int head_dim, int mode, int max_cand, hipStream_t st) {
  constexpr int G = DASH_S1R_G;
  if (max_cand <= 256)
    return head_dim == 128 ? launch_regs<128, G, 0>(a, mode, st) : launch_regs<64, G, 0>(a, mode, st);
  if (max_cand <= 512)
    return head_dim == 128 ? launch_regs<128, G, 1>(a, mode, st) : launch_regs<64, G, 1>(a, mode, st);
  return launch_regs<128, G, 2>(a, mode, st);
}

}  // namespace dash
