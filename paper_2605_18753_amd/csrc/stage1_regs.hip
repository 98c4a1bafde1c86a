// Stage 1 for score rows of up to 512 candidates and GQA groups of 1, 2 or 4 (bf16
// prefill): the same routing as stage1.hip (Sec. 3.2, Eq. 4; Alg. 2; the bias of
// Proposition 1) with the score rows held in registers from the matrix cores to the
// lists, never written to LDS or HBM.
//
// Why a second kernel.  stage1.hip keeps the score rows of a workgroup in LDS, which
// limits a workgroup to 16-64 rows, and every workgroup reads the split summaries of all
// its candidate chunks (768 bytes per chunk at d = 128): that traffic, not arithmetic,
// is what its time goes to.  Here the accumulator layout of v_mfma_f32_16x16x32_bf16 is
// used as the solver's layout: with A = 16 query rows and B = 16 chunk summaries, lane
// (m = lane % 16, kq = lane / 16) receives the scores of rows 4 kq .. 4 kq + 3 at chunk
// 16 ct + m, so after all chunk tiles the 16 lanes of a DPP row hold four complete score
// rows (chunk c in lane c % 16), which is what the 16-lane threshold solver wants, and
// (rows being ordered token-major) the 4 / g_q tokens those rows belong to.  A wave owns
// 16 rows and walks all chunk tiles; the 8 waves of a workgroup (128 rows) share every
// tile of split summaries through LDS (buffer_load ... lds, three stages), so a tile is
// fetched once per 128 rows.
//
// Arithmetic is that of stage1.hip step by step (scores: the same three MFMAs per d
// slice into the same two accumulators; threshold: the same bracketed Newton iteration
// with the same in-lane and DPP-row summation order), so masks, counts, ids and
// thresholds are bit-identical to that kernel's; mu = mean ln w is summed over 16 lanes
// instead of 64 and may differ in the last place.
#include <math.h>

#include <type_traits>

#include "common.h"
#include "dash_internal.h"
#include "lds_copy.h"
#include "stage1_common.h"

namespace dash {

template <int D> struct RegsCfg {
  static constexpr int NW = 8;                               // waves per workgroup
  static constexpr int KS = D / 32;                          // contraction steps per product
  static constexpr int PART_BYTES = D * 2;                   // one bf16 piece of a summary
  static constexpr int ROW_BYTES = 3 * PART_BYTES;           // the three pieces of one chunk
  static constexpr int SPP = D / 8;                          // 16-byte slots per piece
  static constexpr int SPR = 3 * SPP;                        // ... per chunk
  static constexpr int TILE_BYTES = 16 * ROW_BYTES;          // 16 chunks
  static constexpr int IPW = (TILE_BYTES / 1024 + NW - 1) / NW;   // copy instructions per wave and tile
  static constexpr int STAGE_BYTES = IPW * NW * 1024;        // tile + room for the surplus instructions' zeros
  static constexpr int STAGES = 3;
  static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
};

// Threshold of four score rows per lane at once (rows j = 0..3; row j of DPP row kq is
// spread over the row's 16 lanes, NT values per lane): the iteration of stage1.hip's
// 16-lane solver, row by row the same operations in the same order.
template <int NT, int MODE>
__device__ __forceinline__ void solve4(const f32x4 (&v)[NT], int n_cand, float alpha, float p, float (&tau)[4]) {
  float mloc[4], lo[4], hi[4];
  bool done[4];
#pragma unroll
  for (int j = 0; j < 4; j++) {
    float m = -INFINITY;
#pragma unroll
    for (int t = 0; t < NT; t++) m = fmaxf(m, v[t][j]);
    mloc[j] = m;
    const float mx = row16_reduce(m, OpMax());
    lo[j] = mx - 1.f;
    hi[j] = mx - exp2f(-(alpha - 1.f) * log2f((float)n_cand));
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
        pow_terms<MODE>(fmaxf(mloc[j] - tau[j], 0.f), p, f, g);
        asm volatile("" : "+v"(f), "+v"(g));
        const float F = row16_reduce(f, OpAdd()), G = row16_reduce(g, OpAdd());
        if (F > 1.f && G > 0.f) tau[j] += (F - 1.f) / (p * G);
      }
      tau[j] = fmaxf(tau[j], lo[j]);
      if (!(tau[j] < hi[j])) tau[j] = lo[j];
    }
  }
  for (int it = 0; it < 64; it++) {
    bool all_done = true;
#pragma unroll
    for (int j = 0; j < 4; j++) {
      float F = 0.f, G = 0.f;
#pragma unroll
      for (int t = 0; t < NT; t++) {
        float f, g;
        pow_terms<MODE>(fmaxf(v[t][j] - tau[j], 0.f), p, f, g);
        F += f; G += g;
      }
      // keep the partial sums as rounded values: a multiply contracted into the first
      // cross-lane add would make the lanes of a row disagree by an ulp
      asm volatile("" : "+v"(F), "+v"(G));
      F = row16_reduce(F, OpAdd());
      G = row16_reduce(G, OpAdd());
      if (!done[j]) {
        const float f = F - 1.f;
        if (f == 0.f) {
          done[j] = true;
        } else {
          if (f > 0.f) lo[j] = tau[j]; else hi[j] = tau[j];
          const float mid = 0.5f * (lo[j] + hi[j]);
          float cand = (MODE == MODE_BISECT || !(G > 0.f)) ? mid : tau[j] + f / (p * G);
          if (MODE != MODE_BISECT && cand == tau[j]) {
            done[j] = true;                        // Newton step below the fp32 spacing of tau
          } else {
            if (!(cand > lo[j] && cand < hi[j])) cand = mid;
            if (!(cand > lo[j] && cand < hi[j])) { done[j] = true; tau[j] = lo[j]; }   // bracket closed
            else {
              // alpha = 1.5: a Newton step s from the left leaves an error of about
              // (n / 2G) s^2; once that is below 2e-8 the step is final
              if (MODE == MODE_P2 && f > 0.f && cand != mid) {
                const float st = cand - tau[j];
                if ((float)n_cand * st * st < 4e-8f * G) done[j] = true;
              }
              tau[j] = cand;
            }
          }
        }
      }
      all_done = all_done && done[j];
    }
    if (!__any(!all_done)) break;
  }
}

// One workgroup's tile with NT chunk tiles of 16 (NT = 4, 8, 16 or 32 covers n_cand <= 512).
template <int D, int G, int MODE, int NT>
__device__ __forceinline__ void regs_tile(const S1Args& a, char* lds, int b, int r, int tok0, int ntile) {
  using C = RegsCfg<D>;
  constexpr int TPL = 4 / G;                  // tokens per lane (its four rows are TPL tokens x G heads)
  constexpr int TPW = 16 / G;                 // tokens per wave
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int m = lane & 15, kq = lane >> 4;
  const int tok_w0 = tok0 + wave * TPW;
  // The wave's tokens share one candidate set (they lie in one chunk); the workgroup's may
  // span two chunks, so all waves walk the tiles of the longest set (ntile) and a wave
  // treats the chunks past its own set as absent.
  int n_cand = a.causal ? max((a.pos0 + min(tok_w0, a.tok_end - 1)) / a.block - a.window, 0) : a.t_c;
  if (n_cand > a.t_c) n_cand = a.t_c;

  f32x4 v[NT];   // scores, then probabilities: v[t][j] = row 4 kq + j at chunk 16 t + m
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
    auto issue_tile = [&](int t) __attribute__((always_inline)) {
      const uint32_t dst = lds0 + (uint32_t)(t % C::STAGES) * C::STAGE_BYTES + (uint32_t)wave * 1024u;
#pragma unroll
      for (int i = 0; i < C::IPW; i++)
        copy16_to_lds(ks_rs, dst + i * C::NW * 1024, src_off[i], (uint32_t)t * C::TILE_BYTES);
    };
    // operand B read address inside a stage: chunk m, unit (4 ks + kq) ^ (m % SPP) of a piece
    const uint32_t b_rd = (uint32_t)(m * C::ROW_BYTES);
    issue_tile(0);
    if (ntile > 1) issue_tile(1);
#pragma unroll
    for (int t = 0; t < NT; t++) {
      if (t < ntile) {
        // this wave's copies of tile t have landed (newer tiles may stay in flight); the
        // barrier publishes everybody's and retires the reads of tile t - 1
        const int newer = min(ntile - 1 - t, C::STAGES - 2);
        if (newer <= 0) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(0) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" :: "n"(C::IPW) : "memory");
        __syncthreads();
        if (t + 2 < ntile) issue_tile(t + 2);
        const char* sb = lds + (t % C::STAGES) * C::STAGE_BYTES + b_rd;
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
        if (t * 16 + m < n_cand) {
#pragma unroll
          for (int j = 0; j < 4; j++) v[t][j] = (acc_hi[j] + acc_lo[j]) * a.xscale;
        }
      }
    }
  }
  if (n_cand > 0) {
    // ---- thresholds, then probabilities in place ---------------------------------------
    solve4<NT, MODE>(v, n_cand, a.alpha, a.pexp, tau);
#pragma unroll
    for (int t = 0; t < NT; t++)
#pragma unroll
      for (int j = 0; j < 4; j++) v[t][j] = pow_p<MODE>(fmaxf(v[t][j] - tau[j], 0.f), a.pexp);
  }
  if (a.tau && m == 0) {
#pragma unroll
    for (int j = 0; j < 4; j++) {
      const int row = 4 * kq + j;
      const int tok = tok_w0 + row / G, head = r * G + row % G;
      if (tok < a.tok_end) a.tau[((int64_t)b * a.h_q + head) * a.n_q + tok] = n_cand > 0 ? tau[j] : 0.f;
    }
  }

  // ---- group weights, bias, lists: token kq * TPL + tt of the wave, one per DPP row at a time ----
  const float inv_g = 1.f / (float)G;
#pragma unroll
  for (int tt = 0; tt < TPL; tt++) {
    const int tok = tok_w0 + kq * TPL + tt;
    const bool tok_ok = tok < a.tok_end;
    float slog = 0.f, nsup = 0.f;
#pragma unroll
    for (int t = 0; t < NT; t++) {
      float s = 0.f;
      if (t * 16 + m < n_cand) {
#pragma unroll
        for (int h = 0; h < G; h++) s += v[t][tt * G + h];
      }
      s *= inv_g;
      // ln via the hardware log2 (about 1 ulp): ample for a bias that is divided by sigma
      const float lw = s > 0.f ? __builtin_amdgcn_logf(s) * 0.6931471805599453f : INFINITY;   // +inf: not routed
      if (s > 0.f) { slog += lw; nsup += 1.f; }
      v[t][tt * G] = lw;   // the token's probabilities are not needed any more
    }
    asm volatile("" : "+v"(slog));
    slog = row16_reduce(slog, OpAdd());
    nsup = row16_reduce(nsup, OpAdd());
    const float mu = nsup > 0.f ? slog / nsup : 0.f;
    const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + (tok_ok ? tok : 0);
    int32_t* oidx = a.idx ? a.idx + base * a.t_all : nullptr;
    float* obias = a.bias + base * a.t_all;
    // mask word w of the token is kept by lane w of its DPP row (a word past the 16th, which
    // only the local chunks can reach, by lane 0 as well)
    uint32_t word = 0u, word_hi = 0u;
    int running = 0;
#pragma unroll
    for (int t = 0; t < NT; t++) {
      const bool member = v[t][tt * G] != INFINITY;
      const uint64_t bal = __ballot(member);
      const uint32_t field = (uint32_t)(bal >> (16 * kq)) & 0xffffu;
      if (m == (t >> 1)) word |= field << (16 * (t & 1));
      if (member && tok_ok) {
        const int pos = running + __popc(field & ((1u << m) - 1u));
        if (oidx) oidx[pos] = t * 16 + m;
        obias[pos] = (v[t][tt * G] - mu) * a.inv_sigma;
      }
      running += __popc(field);
    }
    if (a.causal) {
      // the always-attended local set, bias 0: the chunks of the window, then the query's own
      const int cd = (a.pos0 + (tok_ok ? tok : 0)) / a.block;
      const int c0 = max(cd - a.window, 0);
      for (int c = c0; c <= cd; c++) {
        if (m == 0 && tok_ok) {
          if (oidx) oidx[running + c - c0] = c;
          obias[running + c - c0] = 0.f;
        }
        if ((c >> 5) == m) word |= 1u << (c & 31);
        if ((c >> 5) == 16 + m) word_hi |= 1u << (c & 31);
      }
      running += cd - c0 + 1;
    }
    if (tok_ok) {
      if (a.cnt && m == 0) a.cnt[base] = running;
      uint32_t* om = a.mask + base * a.words;
      if (m < a.words) om[m] = word;
      if (16 + m < a.words) om[16 + m] = word_hi;
    }
  }
}

template <int D, int G, int MODE>
__global__ __launch_bounds__(512) void s1_regs_kernel(S1Args a) {
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  constexpr int TOKT = RegsCfg<D>::NW * 16 / G;   // tokens per workgroup
  const int hb = a.h_kv * a.batch;
  const int hbi = blockIdx.x % hb;
  const int tile = (int)(gridDim.x / hb) - 1 - (int)(blockIdx.x / hb);   // longest rows first
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int tok0 = a.tok_base + tile * TOKT;
  // the longest candidate set among the workgroup's tokens: that of its last token
  int n_max = a.causal ? max((a.pos0 + min(tok0 + TOKT - 1, a.tok_end - 1)) / a.block - a.window, 0) : a.t_c;
  if (n_max > a.t_c) n_max = a.t_c;
  const int ntile = (n_max + 15) >> 4;
  if (ntile <= 4) regs_tile<D, G, MODE, 4>(a, lds, b, r, tok0, ntile);
  else if (ntile <= 8) regs_tile<D, G, MODE, 8>(a, lds, b, r, tok0, ntile);
  else if (ntile <= 16) regs_tile<D, G, MODE, 16>(a, lds, b, r, tok0, ntile);
  else regs_tile<D, G, MODE, 32>(a, lds, b, r, tok0, ntile);
}

template <int D, int G>
static hipError_t launch_regs_g(const S1Args& a, int mode, dim3 grid, hipStream_t st) {
  constexpr size_t lds = RegsCfg<D>::LDS_BYTES;
#define DASH_RG(MODE_) hipLaunchKernelGGL((s1_regs_kernel<D, G, MODE_>), grid, dim3(512), lds, st, a)
  switch (mode) {
    case MODE_P1: DASH_RG(MODE_P1); break;
    case MODE_P2: DASH_RG(MODE_P2); break;
    case MODE_P4: DASH_RG(MODE_P4); break;
    case MODE_GEN: DASH_RG(MODE_GEN); break;
    default: DASH_RG(MODE_BISECT); break;
  }
#undef DASH_RG
  return hipGetLastError();
}

bool s1_regs_applicable(const dash_params& p, const Layout& L, int max_cand) {
  return L.use_mfma && (L.g_q == 1 || L.g_q == 2 || L.g_q == 4) && max_cand <= 512 && L.words <= 32 &&
         !L.seq_lens;
}

hipError_t launch_s1_regs(const dash_params& p, const Layout& L, const S1Args& a, hipStream_t st) {
  int mode;
  if (a.pexp < 1.f) mode = MODE_BISECT;
  else if (a.pexp == 1.f) mode = MODE_P1;
  else if (a.pexp == 2.f) mode = MODE_P2;
  else if (a.pexp == 4.f) mode = MODE_P4;
  else mode = MODE_GEN;
  const int tokt = 8 * 16 / L.g_q;
  dim3 grid((unsigned)(((a.tok_end - a.tok_base + tokt - 1) / tokt) * p.h_kv * p.batch), 1, 1);
  if (p.head_dim == 128) {
    if (L.g_q == 4) return launch_regs_g<128, 4>(a, mode, grid, st);
    if (L.g_q == 2) return launch_regs_g<128, 2>(a, mode, grid, st);
    return launch_regs_g<128, 1>(a, mode, grid, st);
  }
  if (L.g_q == 4) return launch_regs_g<64, 4>(a, mode, grid, st);
  if (L.g_q == 2) return launch_regs_g<64, 2>(a, mode, grid, st);
  return launch_regs_g<64, 1>(a, mode, grid, st);
}

}  // namespace dash
