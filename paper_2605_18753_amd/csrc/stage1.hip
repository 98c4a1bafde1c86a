// Stage 1: entmax chunk routing (Sec. 3.2, Eq. 4; Alg. 2) and the routing bias
// of the prior in the form of Proposition 1.
//
// A workgroup owns a tile of 16*MT (token, head) rows of one kv-head: all g_q
// heads of 16*MT/g_q consecutive tokens, which share one candidate set (the
// complete chunks before the tokens' own chunk).  It
//   1. fills an LDS score matrix x[row][chunk] = gamma (alpha-1) <q, kbar> scale,
//      either with bf16 MFMAs against the exact 3-way bf16 split of the fp32
//      summaries (products exact, fp32 accumulation: fp32-accurate scores), or by
//      copying fp32 scores a separate kernel wrote (fp32 inputs, decode);
//   2. solves sum_c [x_c - tau]_+^(1/(alpha-1)) = 1 per row: one wave per row,
//      the row spread over the 64 lanes in registers, wave reductions per step;
//      bracketed Newton from the left end of [max-1, max-n^-(alpha-1)] (the
//      residual is convex for alpha <= 2) with bisection as the safeguard and as
//      the only step for alpha > 2;
//   3. averages the per-head probabilities over the GQA group, takes
//      mu = mean ln w over the support, d = (ln w - mu)/sigma, and emits the
//      bit-packed mask plus the compacted (index, bias) list via wave ballots,
//      appending, when causal, the always-attended local chunks with bias 0: the
//      `window` complete chunks before the query's own (they are not candidates)
//      and the query's own (diagonal) chunk.
// Nothing of the score matrix ever goes to HBM on the MFMA path.
#include <math.h>
#include <stdlib.h>

#include "common.h"
#include "compress_body.h"
#include "dash_internal.h"
#include "stage1_common.h"

namespace dash {

// Whether a token range whose longest row has max_cand candidates goes to the
// register-resident kernels (stage1_regs.hip): bf16 prefill, rows of up to 512 chunks, or
// up to 1536 at head dimension 128.
static bool s1_regs_applicable(const dash_params& p, const Layout& L, int max_cand) {
  if (!L.use_mfma || L.seq_lens) return false;
  return max_cand <= 512 || (max_cand <= 1536 && p.head_dim == 128);
}

static hipError_t launch_s1_regs(const dash_params& p, const Layout& L, const S1Args& a, int max_cand, hipStream_t st) {
  int mode;
  if (a.pexp < 1.f) mode = MODE_BISECT;
  else if (a.pexp == 1.f) mode = MODE_P1;
  else if (a.pexp == 2.f) mode = MODE_P2;
  else if (a.pexp == 4.f) mode = MODE_P4;
  else mode = MODE_GEN;
  switch (L.g_q) {
    case 1: return launch_s1_regs_g1(a, p.head_dim, mode, max_cand, st);
    case 2: return launch_s1_regs_g2(a, p.head_dim, mode, max_cand, st);
    case 4: return launch_s1_regs_g4(a, p.head_dim, mode, max_cand, st);
    case 8: return launch_s1_regs_g8(a, p.head_dim, mode, max_cand, st);
    default: return launch_s1_regs_g16(a, p.head_dim, mode, max_cand, st);
  }
}

// Solve RB rows at once (interleaved for ILP).  Row values live in registers:
// lane l holds chunks l, l+64, ...  On exit the rows of S hold the per-head
// entmax probabilities.
template <int NJ, int RB, int MODE>
__device__ __forceinline__ void solve_rows(float* S, int ld, int row0, int n_cand, float alpha,
                                           float p, int lane, float* tau_out /*[RB]*/) {
  float v[RB][NJ], mx[RB], lo[RB], hi[RB], tau[RB];
  bool done[RB];
#pragma unroll
  for (int rb = 0; rb < RB; rb++) {
    float m = -INFINITY;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int c = lane + 64 * j;
      v[rb][j] = c < n_cand ? S[(row0 + 4 * rb) * ld + c] : -INFINITY;
      m = fmaxf(m, v[rb][j]);
    }
    mx[rb] = wave_max(m);
    lo[rb] = mx[rb] - 1.f;
    hi[rb] = mx[rb] - exp2f(-(alpha - 1.f) * log2f((float)n_cand));
    tau[rb] = lo[rb];
    done[rb] = false;
  }
  if constexpr (MODE != MODE_BISECT) {
    // warm start on the 64 lane maxima (a subset: its root and every Newton
    // iterate from the left on it are lower bounds of tau)
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
      float ml = -INFINITY;
#pragma unroll
      for (int j = 0; j < NJ; j++) ml = fmaxf(ml, v[rb][j]);
      for (int it = 0; it < 5; it++) {
        float f, g;
        pow_terms<MODE>(fmaxf(ml - tau[rb], 0.f), p, f, g);
        const float F = wave_sum(f), G = wave_sum(g);
        if (F > 1.f && G > 0.f) tau[rb] += (F - 1.f) / (p * G);
      }
      tau[rb] = fmaxf(tau[rb], lo[rb]);
      if (!(tau[rb] < hi[rb])) tau[rb] = lo[rb];
    }
  }
  for (int it = 0; it < 64; it++) {
    bool all_done = true;
#pragma unroll
    for (int rb = 0; rb < RB; rb++) {
      float F = 0.f, G = 0.f;
#pragma unroll
      for (int j = 0; j < NJ; j++) {
        float f, g;
        pow_terms<MODE>(fmaxf(v[rb][j] - tau[rb], 0.f), p, f, g);
        F += f; G += g;
      }
      F = wave_sum(F);
      G = wave_sum(G);
      if (!done[rb]) {
        const float f = F - 1.f;
        if (f == 0.f) {
          done[rb] = true;
        } else {
          if (f > 0.f) lo[rb] = tau[rb]; else hi[rb] = tau[rb];
          const float mid = 0.5f * (lo[rb] + hi[rb]);
          float cand = (MODE == MODE_BISECT || !(G > 0.f)) ? mid : tau[rb] + f / (p * G);
          if (MODE != MODE_BISECT && cand == tau[rb]) {
            done[rb] = true;                       // Newton step below the fp32 spacing of tau
          } else {
            if (!(cand > lo[rb] && cand < hi[rb])) cand = mid;
            if (!(cand > lo[rb] && cand < hi[rb])) {
              done[rb] = true;                     // bracket closed: adjacent floats
              tau[rb] = lo[rb];
            } else {
              if (MODE == MODE_P2 && f > 0.f && cand != mid) {   // see solve_rows16
                const float st = cand - tau[rb];
                if ((float)n_cand * st * st < 4e-8f * G) done[rb] = true;
              }
              tau[rb] = cand;
            }
          }
        }
      }
      all_done = all_done && done[rb];
    }
    if (all_done) break;
  }
#pragma unroll
  for (int rb = 0; rb < RB; rb++) {
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      const int c = lane + 64 * j;
      if (c < n_cand) S[(row0 + 4 * rb) * ld + c] = pow_p<MODE>(fmaxf(v[rb][j] - tau[rb], 0.f), p);
    }
    tau_out[rb] = tau[rb];
  }
}

// Rows are dealt to the four waves round robin (wave w: rows w, w+4, ...), so a
// decode tile with only g_q valid rows still uses all waves; rows of tokens past
// the end of the sequence are skipped.
template <int NJ, int MODE>
__device__ __forceinline__ void solve_wave_rows(float* S, const S1Args& a, int wave, int nrows,
                                                int n_cand, int lane, int b, int r, int tok0) {
  constexpr int RB = NJ <= 8 ? 4 : (NJ == 16 ? 2 : 1);
  for (int rr = wave; rr < nrows; rr += 4 * RB) {
    if (tok0 + rr / a.g_q >= a.tok_end) break;  // this and all later rows are padding
    float t[RB];
    solve_rows<NJ, RB, MODE>(S, a.ld, rr, n_cand, a.alpha, a.pexp, lane, t);
    if (a.tau && lane == 0) {
#pragma unroll
      for (int rb = 0; rb < RB; rb++) {
        const int row = rr + 4 * rb;
        const int tok = tok0 + row / a.g_q, head = r * a.g_q + row % a.g_q;
        if (row < nrows && tok < a.tok_end) a.tau[((int64_t)b * a.h_q + head) * a.n_q + tok] = t[rb];
      }
    }
  }
}

// Same solve with one row per 16-lane DPP row: a wave works on four rows at once
// (rows row0 + 4q for DPP row q, which keeps the LDS reads conflict-free), lane
// l of a DPP row holds chunks l, l+16, ...  All per-row quantities are per-lane
// values that are equal inside a DPP row, the reductions stay inside the row (no
// LDS round trip), and finished rows simply stop updating.  Used while a row
// fits 32 registers per lane (n_cand <= 512).
template <int NJ, int MODE>
__device__ __forceinline__ void solve_rows16(float* S, int ld, int row0, int n_cand, float alpha,
                                             float p, int lane, float& tau_out) {
  const int l16 = lane & 15, row = row0 + 4 * (lane >> 4);
  float v[NJ];
  float m = -INFINITY;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int c = l16 + 16 * j;
    v[j] = c < n_cand ? S[row * ld + c] : -INFINITY;
    m = fmaxf(m, v[j]);
  }
  const float mx = row16_reduce(m, OpMax());
  float lo = mx - 1.f;
  float hi = mx - exp2f(-(alpha - 1.f) * log2f((float)n_cand));
  float tau = lo;
  if constexpr (MODE != MODE_BISECT) {
    // Warm start: the root of the same equation restricted to the 16 lane maxima
    // is a lower bound of tau (dropping terms lowers the residual), and so is
    // every Newton iterate from the left on it.  A few cheap steps on one value
    // per lane land close to tau; the bracket below still covers any overshoot.
#pragma unroll
    for (int it = 0; it < 5; it++) {
      float f, g;
      pow_terms<MODE>(fmaxf(m - tau, 0.f), p, f, g);
      asm volatile("" : "+v"(f), "+v"(g));
      const float F = row16_reduce(f, OpAdd()), G = row16_reduce(g, OpAdd());
      if (F > 1.f && G > 0.f) tau += (F - 1.f) / (p * G);
    }
    tau = fmaxf(tau, lo);
    if (!(tau < hi)) tau = lo;
  }
  bool done = false;
  for (int it = 0; it < 64; it++) {
    float F = 0.f, G = 0.f;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
      float f, g;
      pow_terms<MODE>(fmaxf(v[j] - tau, 0.f), p, f, g);
      F += f; G += g;
    }
    // keep the partial sums as rounded values: a multiply contracted into the
    // first cross-lane add would make the lanes of a row disagree by an ulp
    asm volatile("" : "+v"(F), "+v"(G));
    F = row16_reduce(F, OpAdd());
    G = row16_reduce(G, OpAdd());
    if (!done) {
      const float f = F - 1.f;
      if (f == 0.f) {
        done = true;
      } else {
        if (f > 0.f) lo = tau; else hi = tau;
        const float mid = 0.5f * (lo + hi);
        float cand = (MODE == MODE_BISECT || !(G > 0.f)) ? mid : tau + f / (p * G);
        if (MODE != MODE_BISECT && cand == tau) {
          done = true;
        } else {
          if (!(cand > lo && cand < hi)) cand = mid;
          if (!(cand > lo && cand < hi)) { done = true; tau = lo; }
          else {
            // alpha = 1.5: a Newton step s from the left leaves an error of about
            // (k / 2G) s^2 <= (n / 2G) s^2 (f'' = 2k, f' = -2G); once that is below
            // 2e-8 the step is final and the confirming evaluation is skipped
            if (MODE == MODE_P2 && f > 0.f && cand != mid) {
              const float st = cand - tau;
              if ((float)n_cand * st * st < 4e-8f * G) done = true;
            }
            tau = cand;
          }
        }
      }
    }
    if (!__any(!done)) break;
  }
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int c = l16 + 16 * j;
    if (c < n_cand) S[row * ld + c] = pow_p<MODE>(fmaxf(v[j] - tau, 0.f), p);
  }
  tau_out = tau;
}

template <int NJ, int MODE>
__device__ __forceinline__ void solve_wave_rows16(float* S, const S1Args& a, int wave, int passes,
                                                  int n_cand, int lane, int b, int r, int tok0) {
  for (int ps = 0; ps < passes; ps++) {
    const int row0 = ps * 16 + wave;
    float t;
    solve_rows16<NJ, MODE>(S, a.ld, row0, n_cand, a.alpha, a.pexp, lane, t);
    if (a.tau && (lane & 15) == 0) {
      const int row = row0 + 4 * (lane >> 4);
      const int tok = tok0 + row / a.g_q, head = r * a.g_q + row % a.g_q;
      if (tok < a.tok_end) a.tau[((int64_t)b * a.h_q + head) * a.n_q + tok] = t;
    }
  }
}

template <int NJ>
__device__ __forceinline__ void emit_token(const float* S, const S1Args& a, uint32_t* mw, int tl,
                                           int tok, int n_cand, int lane, int b, int r) {
  const float inv_g = 1.f / (float)a.g_q;
  float lw[NJ];
  float slog = 0.f, nsup = 0.f;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int c = lane + 64 * j;
    float s = 0.f;
    if (c < n_cand)
      for (int h = 0; h < a.g_q; h++) s += S[(tl * a.g_q + h) * a.ld + c];
    s *= inv_g;
    // ln via the hardware log2 (about 1 ulp): ample for a bias that is divided by sigma
    lw[j] = s > 0.f ? __builtin_amdgcn_logf(s) * 0.6931471805599453f : INFINITY;   // +inf marks "not routed"
    if (s > 0.f) { slog += lw[j]; nsup += 1.f; }
  }
  slog = wave_sum(slog);
  nsup = wave_sum(nsup);
  const float mu = nsup > 0.f ? slog / nsup : 0.f;
  const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + tok;
  int32_t* oidx = a.idx ? a.idx + base * a.t_all : nullptr;
  float* obias = a.bias + base * a.t_all;
  for (int wi = lane; wi < a.words; wi += 64) mw[wi] = 0u;
  __builtin_amdgcn_wave_barrier();
  int running = 0;
#pragma unroll
  for (int j = 0; j < NJ; j++) {
    const int c = lane + 64 * j;
    const bool member = lw[j] != INFINITY;
    const uint64_t bal = __ballot(member);
    if (lane == 0 && 2 * j < a.words) {
      mw[2 * j] = (uint32_t)bal;
      if (2 * j + 1 < a.words) mw[2 * j + 1] = (uint32_t)(bal >> 32);
    }
    if (member) {
      const int pos = running + __popcll(bal & ((1ull << lane) - 1ull));
      if (oidx) oidx[pos] = c;
      obias[pos] = (lw[j] - mu) * a.inv_sigma;
    }
    running += __popcll(bal);
  }
  __builtin_amdgcn_wave_barrier();
  if (a.causal) {
    // the always-attended local set, bias 0: the chunks of the window, then the
    // query's own chunk
    const int cd = (a.pos0 + tok) / a.block;
    const int c0 = max(cd - a.window, 0);
    if (lane == 0) {
      for (int c = c0; c <= cd; c++) {
        if (oidx) oidx[running + c - c0] = c;
        obias[running + c - c0] = 0.f;
        mw[c >> 5] |= 1u << (c & 31);
      }
    }
    running += cd - c0 + 1;
  }
  __builtin_amdgcn_wave_barrier();
  if (a.cnt && lane == 0) a.cnt[base] = running;
  uint32_t* om = a.mask + base * a.words;
  for (int wi = lane; wi < a.words; wi += 64) om[wi] = mw[wi];
  __builtin_amdgcn_wave_barrier();
}

// The same emission by all four waves of the workgroup, for tiles that hold a single
// token (decode; prefill at a GQA group of 16): wave w takes the 64-chunk slots
// j = w, w + 4, ...; the ranks of a slot's members start at the number of members in
// the slots below it, exchanged through LDS, as are the partial sums of ln w.  Same
// arithmetic per chunk as emit_token; the sums are combined wave by wave, so mu may
// differ from the single-wave order in the last place.
template <int NJ, int NWV = 4>
__device__ __forceinline__ void emit_token_wg(const float* S, const S1Args& a, uint32_t* mw, int* xcnt,
                                              float* xsum, int tok, int n_cand, int lane, int wave,
                                              int b, int r) {
  constexpr int NW = (NJ + NWV - 1) / NWV;   // slots per wave (NWV waves in the workgroup)
  const float inv_g = 1.f / (float)a.g_q;
  float lw[NW];
  float slog = 0.f, nsup = 0.f;
#pragma unroll
  for (int jj = 0; jj < NW; jj++) {
    const int c = lane + 64 * (wave + NWV * jj);
    float s = 0.f;
    if (wave + NWV * jj < NJ && c < n_cand)
      for (int h = 0; h < a.g_q; h++) s += S[h * a.ld + c];
    s *= inv_g;
    lw[jj] = s > 0.f ? __builtin_amdgcn_logf(s) * 0.6931471805599453f : INFINITY;   // +inf marks "not routed"
    if (s > 0.f) { slog += lw[jj]; nsup += 1.f; }
  }
  slog = wave_sum(slog);
  nsup = wave_sum(nsup);
  uint64_t bal[NW];
#pragma unroll
  for (int jj = 0; jj < NW; jj++) {
    bal[jj] = __ballot(lw[jj] != INFINITY);
    if (lane == 0 && wave + NWV * jj < NJ) xcnt[wave + NWV * jj] = __popcll(bal[jj]);
  }
  if (lane == 0) { xsum[wave] = slog; xsum[NWV + wave] = nsup; }
  for (int wi = threadIdx.x; wi < a.words; wi += 64 * NWV) mw[wi] = 0u;
  __syncthreads();
  float slog_t, nsup_t;
  if constexpr (NWV == 4) {
    slog_t = (xsum[0] + xsum[1]) + (xsum[2] + xsum[3]);
    nsup_t = (xsum[4] + xsum[5]) + (xsum[6] + xsum[7]);
  } else {
    slog_t = 0.f; nsup_t = 0.f;
#pragma unroll
    for (int w = 0; w < NWV; w += 4) {
      slog_t += (xsum[w] + xsum[w + 1]) + (xsum[w + 2] + xsum[w + 3]);
      nsup_t += (xsum[NWV + w] + xsum[NWV + w + 1]) + (xsum[NWV + w + 2] + xsum[NWV + w + 3]);
    }
  }
  const float mu = nsup_t > 0.f ? slog_t / nsup_t : 0.f;
  // members below each of this wave's slots: lane l holds the count of slot l
  const int mine = lane < NJ ? xcnt[lane] : 0;
  int incl = mine;
#pragma unroll
  for (int off = 1; off < 32; off <<= 1) {
    const int t = __shfl_up(incl, off);
    if (lane >= off) incl += t;
  }
  const int total = __shfl(incl, NJ - 1);
  const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + tok;
  int32_t* oidx = a.idx ? a.idx + base * a.t_all : nullptr;
  float* obias = a.bias + base * a.t_all;
#pragma unroll
  for (int jj = 0; jj < NW; jj++) {
    const int j = wave + NWV * jj;
    if (j >= NJ) break;
    const int start = __shfl(incl - mine, j);
    const int c = lane + 64 * j;
    if (lane == 0 && 2 * j < a.words) {
      mw[2 * j] = (uint32_t)bal[jj];
      if (2 * j + 1 < a.words) mw[2 * j + 1] = (uint32_t)(bal[jj] >> 32);
    }
    if (lw[jj] != INFINITY) {
      const int pos = start + __popcll(bal[jj] & ((1ull << lane) - 1ull));
      if (oidx) oidx[pos] = c;
      obias[pos] = (lw[jj] - mu) * a.inv_sigma;
    }
  }
  __syncthreads();
  int running = total;
  if (a.causal) {
    // the always-attended local set, bias 0: the chunks of the window, then the
    // query's own chunk
    const int cd = (a.pos0 + tok) / a.block;
    const int c0 = max(cd - a.window, 0);
    if (threadIdx.x == 0) {
      for (int c = c0; c <= cd; c++) {
        if (oidx) oidx[running + c - c0] = c;
        obias[running + c - c0] = 0.f;
        mw[c >> 5] |= 1u << (c & 31);
      }
    }
    running += cd - c0 + 1;
  }
  __syncthreads();
  if (a.cnt && threadIdx.x == 0) a.cnt[base] = running;
  uint32_t* om = a.mask + base * a.words;
  for (int wi = threadIdx.x; wi < a.words; wi += 64 * NWV) om[wi] = mw[wi];
}

template <int MT, int D, bool FROM_MFMA>
__global__ __launch_bounds__(256) void s1_route_kernel(S1Args a) {
  extern __shared__ float S[];   // [16*MT][ld] scores, then per-head probabilities
  __shared__ uint32_t mwords[4][64];
  __shared__ int xcnt[32];
  __shared__ float xsum[8];
  constexpr int ROWS = 16 * MT;
  const int tokt = ROWS / a.g_q;
  // workgroup id -> (tile, kv-head, batch), the (head, batch) pair fastest: the 8
  // XCDs are fed round robin, so each one keeps few heads' summaries in its L2
  const int hb = a.h_kv * a.batch;
  const int hbi = blockIdx.x % hb;
  const int tile = (int)(gridDim.x / hb) - 1 - (int)(blockIdx.x / hb);   // longest rows first
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int tok0 = a.tok_base + tile * tokt;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  // per-sequence cache length (decode): query 0 of sequence b sits at len_b - n_q
  if (a.seq_lens) a.pos0 = min(max(a.seq_lens[b], a.n_q), a.n_kv) - a.n_q;
  int n_cand = a.causal ? max((a.pos0 + tok0) / a.block - a.window, 0) : a.t_c;
  if (n_cand > a.t_c) n_cand = a.t_c;

  if (n_cand > 0) {
    if constexpr (FROM_MFMA) {
      const int m = lane & 15, kq = lane >> 4;
      bf16x8 qf[MT][D / 32];
#pragma unroll
      for (int mt = 0; mt < MT; mt++) {
        const int row = mt * 16 + m;
        const int tok = tok0 + row / a.g_q, head = r * a.g_q + row % a.g_q;
        const uint16_t* qp = (const uint16_t*)a.q + b * a.qs_b + head * a.qs_h +
                             (int64_t)(tok < a.n_q ? tok : a.n_q - 1) * a.qs_t + kq * 8;
#pragma unroll
        for (int ks = 0; ks < D / 32; ks++)
          qf[mt][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
      }
      const int ntile_c = (n_cand + 15) >> 4;
      const uint16_t* kb = a.ksplit + ((int64_t)b * a.h_kv + r) * a.t_c * 3 * D + kq * 8;
      // Operand registers are double buffered: the loads of this wave's next chunk
      // tile are in flight while the current one goes through the MFMAs.  The loads
      // are issued from assembly and waited for by count (the newest tile's loads may
      // stay outstanding): left to the compiler, the schedule ends up waiting for the
      // loads it has just issued, which exposes the L2 latency once per tile.
      constexpr int KS = D / 32;
      bf16x8 kf[2][3][KS];
      auto load_tile = [&](int ct, bf16x8 (&dst)[3][KS]) {
        const int c = ct * 16 + m;
        const uint16_t* kp = kb + (int64_t)(c < n_cand ? c : n_cand - 1) * 3 * D;
#pragma unroll
        for (int sp = 0; sp < 3; sp++)
#pragma unroll
          for (int ks = 0; ks < KS; ks++)
            asm volatile("global_load_dwordx4 %0, %1, off offset:%2"
                         : "=v"(dst[sp][ks]) : "v"(kp), "n"((sp * D + ks * 32) * 2) : "memory");
      };
      // wait until at most `newer` loads are outstanding; the fragments are passed
      // through so that their consumers cannot be scheduled above the wait
      auto wait_tile = [&](bf16x8 (&t)[3][KS], bool next_in_flight) {
        if (next_in_flight) {
          if constexpr (KS == 4)
            asm volatile("s_waitcnt vmcnt(12)" : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[0][2]), "+v"(t[0][3]),
                         "+v"(t[1][0]), "+v"(t[1][1]), "+v"(t[1][2]), "+v"(t[1][3]),
                         "+v"(t[2][0]), "+v"(t[2][1]), "+v"(t[2][2]), "+v"(t[2][3]));
          else
            asm volatile("s_waitcnt vmcnt(6)" : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[1][0]), "+v"(t[1][1]),
                         "+v"(t[2][0]), "+v"(t[2][1]));
        } else {
          if constexpr (KS == 4)
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[0][2]), "+v"(t[0][3]),
                         "+v"(t[1][0]), "+v"(t[1][1]), "+v"(t[1][2]), "+v"(t[1][3]),
                         "+v"(t[2][0]), "+v"(t[2][1]), "+v"(t[2][2]), "+v"(t[2][3]));
          else
            asm volatile("s_waitcnt vmcnt(0)" : "+v"(t[0][0]), "+v"(t[0][1]), "+v"(t[1][0]), "+v"(t[1][1]),
                         "+v"(t[2][0]), "+v"(t[2][1]));
        }
      };
      auto mma_tile = [&](int ct, const bf16x8 (&src)[3][D / 32]) {
        f32x4 acc_hi[MT], acc_lo[MT];
#pragma unroll
        for (int mt = 0; mt < MT; mt++) { acc_hi[mt] = f32x4{0, 0, 0, 0}; acc_lo[mt] = f32x4{0, 0, 0, 0}; }
#pragma unroll
        for (int ks = 0; ks < D / 32; ks++)
#pragma unroll
          for (int mt = 0; mt < MT; mt++) {
            acc_hi[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[mt][ks], src[0][ks], acc_hi[mt], 0, 0, 0);
            acc_lo[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[mt][ks], src[1][ks], acc_lo[mt], 0, 0, 0);
            acc_lo[mt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[mt][ks], src[2][ks], acc_lo[mt], 0, 0, 0);
          }
        const int c = ct * 16 + m;
        if (c < n_cand) {
#pragma unroll
          for (int mt = 0; mt < MT; mt++)
#pragma unroll
            for (int j = 0; j < 4; j++)
              S[(mt * 16 + 4 * kq + j) * a.ld + c] = (acc_hi[mt][j] + acc_lo[mt][j]) * a.xscale;
        }
      };
      // the Q fragments must have landed (and be known to) before the counted waits
#pragma unroll
      for (int mt = 0; mt < MT; mt++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++) asm volatile("" : "+v"(qf[mt][ks]));
      if (wave < ntile_c) load_tile(wave, kf[0]);
      for (int ct = wave; ct < ntile_c; ct += 8) {
        const bool more1 = ct + 4 < ntile_c;
        if (more1) load_tile(ct + 4, kf[1]);
        wait_tile(kf[0], more1);
        mma_tile(ct, kf[0]);
        if (more1) {
          const bool more2 = ct + 8 < ntile_c;
          if (more2) load_tile(ct + 8, kf[0]);
          wait_tile(kf[1], more2);
          mma_tile(ct + 4, kf[1]);
        }
      }
    } else {
      for (int row = wave; row < ROWS; row += 4) {
        const int tok = tok0 + row / a.g_q, head = r * a.g_q + row % a.g_q;
        const float* src = a.scores + (((int64_t)b * a.h_q + head) * a.n_q + (tok < a.n_q ? tok : 0)) * a.t_c;
        const bool ok = tok < a.tok_end;
        // padding rows are zero-filled only where the solver reads them (the 16-lane-row
        // solver takes four rows at a time; the wave-per-row solver stops at the first)
        if (!ok && n_cand > 512) break;
        for (int c = lane; c < n_cand; c += 64) S[row * a.ld + c] = ok ? src[c] : 0.f;
      }
    }
  }
  __syncthreads();

  const int nj = (n_cand + 63) >> 6;
  if (n_cand > 0) {
    int mode;
    if (a.pexp < 1.f) mode = MODE_BISECT;
    else if (a.pexp == 1.f) mode = MODE_P1;
    else if (a.pexp == 2.f) mode = MODE_P2;
    else if (a.pexp == 4.f) mode = MODE_P4;
    else mode = MODE_GEN;
#define DASH_SOLVE(NJ_)                                                                          \
  switch (mode) {                                                                                \
    case MODE_P1: solve_wave_rows<NJ_, MODE_P1>(S, a, wave, ROWS, n_cand, lane, b, r, tok0); break; \
    case MODE_P2: solve_wave_rows<NJ_, MODE_P2>(S, a, wave, ROWS, n_cand, lane, b, r, tok0); break; \
    case MODE_P4: solve_wave_rows<NJ_, MODE_P4>(S, a, wave, ROWS, n_cand, lane, b, r, tok0); break; \
    case MODE_GEN: solve_wave_rows<NJ_, MODE_GEN>(S, a, wave, ROWS, n_cand, lane, b, r, tok0); break; \
    default: solve_wave_rows<NJ_, MODE_BISECT>(S, a, wave, ROWS, n_cand, lane, b, r, tok0); break; \
  }
#define DASH_SOLVE16(NJ_)                                                                        \
  switch (mode) {                                                                                \
    case MODE_P1: solve_wave_rows16<NJ_, MODE_P1>(S, a, wave, MT, n_cand, lane, b, r, tok0); break; \
    case MODE_P2: solve_wave_rows16<NJ_, MODE_P2>(S, a, wave, MT, n_cand, lane, b, r, tok0); break; \
    case MODE_P4: solve_wave_rows16<NJ_, MODE_P4>(S, a, wave, MT, n_cand, lane, b, r, tok0); break; \
    case MODE_GEN: solve_wave_rows16<NJ_, MODE_GEN>(S, a, wave, MT, n_cand, lane, b, r, tok0); break; \
    default: solve_wave_rows16<NJ_, MODE_BISECT>(S, a, wave, MT, n_cand, lane, b, r, tok0); break; \
  }
    if (n_cand <= 64) { DASH_SOLVE16(4) }
    else if (n_cand <= 128) { DASH_SOLVE16(8) }
    else if (n_cand <= 256) { DASH_SOLVE16(16) }
    else if (n_cand <= 512) { DASH_SOLVE16(32) }
    else if (nj <= 16) { DASH_SOLVE(16) }
    else { DASH_SOLVE(32) }
#undef DASH_SOLVE16
#undef DASH_SOLVE
  } else if (a.tau) {
    for (int row = threadIdx.x; row < ROWS; row += 256) {
      const int tok = tok0 + row / a.g_q, head = r * a.g_q + row % a.g_q;
      if (tok < a.tok_end) a.tau[((int64_t)b * a.h_q + head) * a.n_q + tok] = 0.f;
    }
  }
  __syncthreads();

  if (tokt == 1 || a.tok_end - tok0 <= 1) {
    // one token in the tile (GQA group of 16, or a decode step): all four waves share
    // its emission
    if (tok0 >= a.tok_end) return;
    if (nj <= 4) emit_token_wg<4>(S, a, mwords[0], xcnt, xsum, tok0, n_cand, lane, wave, b, r);
    else if (nj <= 8) emit_token_wg<8>(S, a, mwords[0], xcnt, xsum, tok0, n_cand, lane, wave, b, r);
    else if (nj <= 16) emit_token_wg<16>(S, a, mwords[0], xcnt, xsum, tok0, n_cand, lane, wave, b, r);
    else emit_token_wg<32>(S, a, mwords[0], xcnt, xsum, tok0, n_cand, lane, wave, b, r);
    return;
  }
  for (int tl = wave; tl < tokt; tl += 4) {
    const int tok = tok0 + tl;
    if (tok >= a.tok_end) break;
    uint32_t* mw = mwords[wave];
    if (nj <= 1) emit_token<1>(S, a, mw, tl, tok, n_cand, lane, b, r);
    else if (nj <= 2) emit_token<2>(S, a, mw, tl, tok, n_cand, lane, b, r);
    else if (nj <= 4) emit_token<4>(S, a, mw, tl, tok, n_cand, lane, b, r);
    else if (nj <= 8) emit_token<8>(S, a, mw, tl, tok, n_cand, lane, b, r);
    else if (nj <= 16) emit_token<16>(S, a, mw, tl, tok, n_cand, lane, b, r);
    else emit_token<32>(S, a, mw, tl, tok, n_cand, lane, b, r);
  }
}

// Stage 1 of a decode step in one launch: one workgroup of 16 waves per (sequence,
// kv-head) computes the scores of the pair's g_q query rows against all candidate
// summaries (the arithmetic of s1_scores_f32_kernel: a 16-lane DPP row per chunk, fp32
// FMA in the same order, row reduction), keeps them in LDS, and goes on to the threshold
// and the lists with the same solvers and the same emission as s1_route_kernel: no score
// row goes through HBM and the step has one dependent launch less.  The summaries are
// streamed with eight 16-byte loads in flight per lane and the next batch of 256 chunks
// requested before the current one is used.
template <typename T, int D>
__global__ __launch_bounds__(1024) void s1_decode_kernel(S1Args a) {
  extern __shared__ float S[];   // [16][ld] score rows (g_q of them used), then the query rows [g_q][D] in fp32
  __shared__ uint32_t mwords[64];
  __shared__ int xcnt[32];
  __shared__ float xsum[32];
  constexpr int CPG = 4;         // chunks per 16-lane group and batch
  constexpr int NV = D / 64;     // 16-byte loads per chunk and lane
  const int pairs = a.h_kv * a.batch;
  const int r = blockIdx.x % a.h_kv, b = (blockIdx.x % pairs) / a.h_kv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  if ((int)blockIdx.x >= pairs) {
    // The second half of the grid (launched only with a.k_upd): a current token that completes
    // a chunk has that chunk summarised now.  The chunk is the query's own, not a candidate of
    // this step, so nothing in the other workgroups reads what is written here.
    const int len = a.seq_lens ? min(max(a.seq_lens[b], 1), a.n_kv) : a.n_kv;
    if (len % a.block != 0) return;
    kbar_block_mean<T>((const T*)a.k_upd, a.kbar_upd, reinterpret_cast<double*>(S), a.block, D, a.t_c,
                       len / a.block - 1, r, b, a.h_kv, a.ks_b, a.ks_h, a.ks_t);
    return;
  }
  if (a.seq_lens) a.pos0 = min(max(a.seq_lens[b], 1), a.n_kv) - 1;   // per-sequence cache length
  int n_cand = max(a.pos0 / a.block - a.window, 0);
  if (n_cand > a.t_c) n_cand = a.t_c;
  float* qs = S + 16 * a.ld;

  if (n_cand > 0) {
    const T* qg = (const T*)a.q + b * a.qs_b + (int64_t)r * a.g_q * a.qs_h;
    for (int i = threadIdx.x; i < a.g_q * D; i += 1024) qs[i] = elem<T>::ld(qg + (i / D) * a.qs_h + (i % D));
    // the 16-lane-row solver (rows of up to 512 chunks) reads four rows at a time: zero the unused ones
    if (n_cand <= 512)
      for (int i = threadIdx.x; i < (16 - a.g_q) * n_cand; i += 1024) S[(a.g_q + i / n_cand) * a.ld + i % n_cand] = 0.f;
    __syncthreads();
    const int cl = threadIdx.x >> 4, l16 = threadIdx.x & 15;
    bool on_mfma = false;
    if constexpr (sizeof(T) == 2) {
      if (a.g_q >= 8) {
        // GQA groups of 8 and 16 fill a 16-row matrix-core tile: the scores of 16 chunks at a
        // time from v_mfma_f32_16x16x32_bf16, A = the group's query rows (exact in bf16), B =
        // the fp32 summaries split on the fly into three bf16 pieces by truncation (exact:
        // x = hi + mid + lo), three products per d slice into two accumulators as in the
        // prefill kernels, so a decode step and a prefill see the same scores.  Lane
        // (n = lane % 16, kq = lane / 16) supplies d 32 ks + 8 kq .. + 7 of chunk 16 ct + n and
        // receives the scores of heads 4 kq .. 4 kq + 3 at that chunk.  Wave w takes the chunk
        // tiles w, w + 16, ...; the loads of its next tile are in flight during the current one.
        on_mfma = true;
        constexpr int KS = D / 32;
        const int n16 = lane & 15, kq = lane >> 4;
        bf16x8 qf[KS];
        {
          const uint16_t* qp = (const uint16_t*)a.q + b * a.qs_b + (int64_t)(r * a.g_q + (n16 < a.g_q ? n16 : 0)) * a.qs_h + kq * 8;
#pragma unroll
          for (int ks = 0; ks < KS; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 32);
        }
        const float* kt0 = a.kbar + ((int64_t)b * a.h_kv + r) * a.t_c * D + kq * 8;
        const int ntile_c = (n_cand + 15) >> 4;
        f32x4 kv[2][KS][2];
        auto load_tile = [&](int ct, f32x4 (&dst)[KS][2]) {
          const int c = ct * 16 + n16;
          const float* kp = kt0 + (int64_t)(c < n_cand ? c : n_cand - 1) * D;
#pragma unroll
          for (int ks = 0; ks < KS; ks++) {
            dst[ks][0] = *reinterpret_cast<const f32x4*>(kp + ks * 32);
            dst[ks][1] = *reinterpret_cast<const f32x4*>(kp + ks * 32 + 4);
          }
        };
        auto use_tile = [&](int ct, const f32x4 (&src)[KS][2]) {
          f32x4 acc_hi = {0.f, 0.f, 0.f, 0.f}, acc_lo = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
          for (int ks = 0; ks < KS; ks++) {
            u32x4 p_hi, p_mid, p_lo;
#pragma unroll
            for (int e2 = 0; e2 < 4; e2++) {   // elements 2 e2, 2 e2 + 1 of the lane's eight
              uint32_t h2[2], m2[2], l2[2];
#pragma unroll
              for (int t = 0; t < 2; t++) {
                const float x = src[ks][e2 >> 1][2 * (e2 & 1) + t];
                const uint32_t hb = __float_as_uint(x) & 0xffff0000u;
                const float r1 = x - __uint_as_float(hb);
                const uint32_t mb = __float_as_uint(r1) & 0xffff0000u;
                const float r2 = r1 - __uint_as_float(mb);
                h2[t] = hb; m2[t] = mb; l2[t] = __float_as_uint(r2);
              }
              // the upper halves of two words side by side (element 2 e2 in the low half)
              p_hi[e2] = __builtin_amdgcn_perm(h2[1], h2[0], 0x07060302u);
              p_mid[e2] = __builtin_amdgcn_perm(m2[1], m2[0], 0x07060302u);
              p_lo[e2] = __builtin_amdgcn_perm(l2[1], l2[0], 0x07060302u);
            }
            acc_hi = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], __builtin_bit_cast(bf16x8, p_hi), acc_hi, 0, 0, 0);
            acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], __builtin_bit_cast(bf16x8, p_mid), acc_lo, 0, 0, 0);
            acc_lo = __builtin_amdgcn_mfma_f32_16x16x32_bf16(qf[ks], __builtin_bit_cast(bf16x8, p_lo), acc_lo, 0, 0, 0);
          }
          const int c = ct * 16 + n16;
          if (c < n_cand) {
#pragma unroll
            for (int j = 0; j < 4; j++)
              if (4 * kq + j < a.g_q) S[(4 * kq + j) * a.ld + c] = (acc_hi[j] + acc_lo[j]) * a.xscale;
          }
        };
        if (wave < ntile_c) load_tile(wave, kv[0]);
        for (int ct = wave; ct < ntile_c; ct += 32) {
          if (ct + 16 < ntile_c) load_tile(ct + 16, kv[1]);
          use_tile(ct, kv[0]);
          if (ct + 16 < ntile_c) {
            if (ct + 32 < ntile_c) load_tile(ct + 32, kv[0]);
            use_tile(ct + 16, kv[1]);
          }
        }
      }
    }
    const float* kbase = a.kbar + ((int64_t)b * a.h_kv + r) * a.t_c * D + 4 * l16;
    f32x4 kk[2][CPG][NV];
    auto load_batch = [&](int c0, f32x4 (&dst)[CPG][NV]) {
#pragma unroll
      for (int u = 0; u < CPG; u++) {
        const int c = c0 + u * 64 + cl;
        const float* kp = kbase + (int64_t)(c < n_cand ? c : n_cand - 1) * D;
#pragma unroll
        for (int i = 0; i < NV; i++) dst[u][i] = *reinterpret_cast<const f32x4*>(kp + 64 * i);
      }
    };
    auto use_batch = [&](int c0, const f32x4 (&src)[CPG][NV]) {
      for (int h = 0; h < a.g_q; h++) {
        f32x4 qv[NV];
#pragma unroll
        for (int i = 0; i < NV; i++) qv[i] = *reinterpret_cast<const f32x4*>(qs + h * D + 4 * l16 + 64 * i);
#pragma unroll
        for (int u = 0; u < CPG; u++) {
          float acc = 0.f;
#pragma unroll
          for (int i = 0; i < NV; i++)
#pragma unroll
            for (int e = 0; e < 4; e++) acc = fmaf(qv[i][e], src[u][i][e], acc);
          acc = row16_sum(acc);
          const int c = c0 + u * 64 + cl;
          if (l16 == 0 && c < n_cand) S[h * a.ld + c] = acc * a.xscale;
        }
      }
    };
    constexpr int STEP = 64 * CPG;
    if (!on_mfma) load_batch(0, kk[0]);
    for (int c0 = 0; !on_mfma && c0 < n_cand; c0 += 2 * STEP) {
      if (c0 + STEP < n_cand) load_batch(c0 + STEP, kk[1]);
      use_batch(c0, kk[0]);
      if (c0 + STEP < n_cand) {
        if (c0 + 2 * STEP < n_cand) load_batch(c0 + 2 * STEP, kk[0]);
        use_batch(c0 + STEP, kk[1]);
      }
    }
  }
  __syncthreads();

  const int nj = (n_cand + 63) >> 6;
  if (n_cand > 0) {
    int mode;
    if (a.pexp < 1.f) mode = MODE_BISECT;
    else if (a.pexp == 1.f) mode = MODE_P1;
    else if (a.pexp == 2.f) mode = MODE_P2;
    else if (a.pexp == 4.f) mode = MODE_P4;
    else mode = MODE_GEN;
    if (n_cand <= 512) {
      // four rows per wave, one per DPP row: waves 0..3 cover the 16 rows
      if (wave < 4) {
#define DASH_SOLVE16(NJ_)                                                                           \
  switch (mode) {                                                                                   \
    case MODE_P1: solve_wave_rows16<NJ_, MODE_P1>(S, a, wave, 1, n_cand, lane, b, r, 0); break;     \
    case MODE_P2: solve_wave_rows16<NJ_, MODE_P2>(S, a, wave, 1, n_cand, lane, b, r, 0); break;     \
    case MODE_P4: solve_wave_rows16<NJ_, MODE_P4>(S, a, wave, 1, n_cand, lane, b, r, 0); break;     \
    case MODE_GEN: solve_wave_rows16<NJ_, MODE_GEN>(S, a, wave, 1, n_cand, lane, b, r, 0); break;   \
    default: solve_wave_rows16<NJ_, MODE_BISECT>(S, a, wave, 1, n_cand, lane, b, r, 0); break;      \
  }
        if (n_cand <= 64) { DASH_SOLVE16(4) }
        else if (n_cand <= 128) { DASH_SOLVE16(8) }
        else if (n_cand <= 256) { DASH_SOLVE16(16) }
        else { DASH_SOLVE16(32) }
#undef DASH_SOLVE16
      }
    } else if (wave < a.g_q) {
      // one row per wave, all rows at once
      float t;
#define DASH_SOLVE(NJ_)                                                                             \
  switch (mode) {                                                                                   \
    case MODE_P1: solve_rows<NJ_, 1, MODE_P1>(S, a.ld, wave, n_cand, a.alpha, a.pexp, lane, &t); break;   \
    case MODE_P2: solve_rows<NJ_, 1, MODE_P2>(S, a.ld, wave, n_cand, a.alpha, a.pexp, lane, &t); break;   \
    case MODE_P4: solve_rows<NJ_, 1, MODE_P4>(S, a.ld, wave, n_cand, a.alpha, a.pexp, lane, &t); break;   \
    case MODE_GEN: solve_rows<NJ_, 1, MODE_GEN>(S, a.ld, wave, n_cand, a.alpha, a.pexp, lane, &t); break; \
    default: solve_rows<NJ_, 1, MODE_BISECT>(S, a.ld, wave, n_cand, a.alpha, a.pexp, lane, &t); break;    \
  }
      if (nj <= 16) { DASH_SOLVE(16) } else { DASH_SOLVE(32) }
#undef DASH_SOLVE
      if (a.tau && lane == 0) a.tau[((int64_t)b * a.h_q + r * a.g_q + wave) * a.n_q] = t;
    }
  } else if (a.tau) {
    if (threadIdx.x < a.g_q) a.tau[((int64_t)b * a.h_q + r * a.g_q + threadIdx.x) * a.n_q] = 0.f;
  }
  __syncthreads();

  if (nj <= 4) emit_token_wg<4, 16>(S, a, mwords, xcnt, xsum, 0, n_cand, lane, wave, b, r);
  else if (nj <= 8) emit_token_wg<8, 16>(S, a, mwords, xcnt, xsum, 0, n_cand, lane, wave, b, r);
  else if (nj <= 16) emit_token_wg<16, 16>(S, a, mwords, xcnt, xsum, 0, n_cand, lane, wave, b, r);
  else emit_token_wg<32, 16>(S, a, mwords, xcnt, xsum, 0, n_cand, lane, wave, b, r);
}

// fp32 scores for fp32 inputs and for decode: one 16-lane DPP row per chunk,
// coalesced float4 reads of the fp32 summaries, fp32 FMA, row reduction.  A
// workgroup covers 64 chunks (four per DPP row) and issues all its summary loads
// before the first use, so enough bytes are in flight to stream the cache.
template <typename T, int D>
__global__ __launch_bounds__(256) void s1_scores_f32_kernel(
    const T* __restrict__ q, const float* __restrict__ kbar, float* __restrict__ scores, int h_q,
    int h_kv, int g_q, int n_q, int block, int t_c, int pos0, int causal, int64_t qs_b,
    int64_t qs_h, int64_t qs_t, float xscale, const int32_t* __restrict__ seq_lens, int n_kv) {
  constexpr int CPG = 4;                      // chunks per 16-lane group
  const int tok = blockIdx.y;
  const int b = blockIdx.z / h_kv, r = blockIdx.z % h_kv;
  if (seq_lens) pos0 = min(max(seq_lens[b], n_q), n_kv) - n_q;   // per-sequence cache length (decode)
  int n_cand = causal ? (pos0 + tok) / block : t_c;
  if (n_cand > t_c) n_cand = t_c;
  const int c0 = blockIdx.x * 16 * CPG;
  if (c0 >= n_cand) return;
  const int cl = threadIdx.x >> 4, l16 = threadIdx.x & 15;
  const float* kbase = kbar + ((int64_t)b * h_kv + r) * t_c * D + 4 * l16;
  float kk[CPG][D / 64][4];
#pragma unroll
  for (int u = 0; u < CPG; u++) {
    const int c = c0 + u * 16 + cl;
    const float* kp = kbase + (int64_t)(c < n_cand ? c : n_cand - 1) * D;
#pragma unroll
    for (int i = 0; i < D / 64; i++) {
      const f32x4 t = *reinterpret_cast<const f32x4*>(kp + 64 * i);
      kk[u][i][0] = t[0]; kk[u][i][1] = t[1]; kk[u][i][2] = t[2]; kk[u][i][3] = t[3];
    }
  }
  for (int h = 0; h < g_q; h++) {
    const int head = r * g_q + h;
    const T* qp = q + b * qs_b + head * qs_h + (int64_t)tok * qs_t + 4 * l16;
    float qv[D / 64][4];
#pragma unroll
    for (int i = 0; i < D / 64; i++)
#pragma unroll
      for (int e = 0; e < 4; e++) qv[i][e] = elem<T>::ld(qp + 64 * i + e);
    float* srow = scores + (((int64_t)b * h_q + head) * n_q + tok) * t_c;
#pragma unroll
    for (int u = 0; u < CPG; u++) {
      float acc = 0.f;
#pragma unroll
      for (int i = 0; i < D / 64; i++)
#pragma unroll
        for (int e = 0; e < 4; e++) acc = fmaf(qv[i][e], kk[u][i][e], acc);
      acc = row16_sum(acc);
      const int c = c0 + u * 16 + cl;
      if (l16 == 0 && c < n_cand) srow[c] = acc * xscale;
    }
  }
}

hipError_t launch_s1_scores_f32(const dash_params& p, const Layout& L, const void* q,
                                const float* kbar, float* scores, hipStream_t st) {
  if (L.t_c == 0) return hipSuccess;
  dim3 grid((L.t_c + 63) / 64, p.n_q, p.batch * p.h_kv), blk(256);
#define DASH_SC(T_, D_)                                                                           \
  hipLaunchKernelGGL((s1_scores_f32_kernel<T_, D_>), grid, blk, 0, st, (const T_*)q, kbar, scores, \
                     p.h_q, p.h_kv, L.g_q, p.n_q, p.block_size, L.t_c, L.pos0, p.causal,          \
                     p.q_stride[0], p.q_stride[1], p.q_stride[2], L.xscale, L.seq_lens, p.n_kv)
  if (p.dtype == DASH_BF16) {
    if (p.head_dim == 128) DASH_SC(uint16_t, 128); else DASH_SC(uint16_t, 64);
  } else {
    if (p.head_dim == 128) DASH_SC(float, 128); else DASH_SC(float, 64);
  }
#undef DASH_SC
  return hipGetLastError();
}

template <auto kern>
static hipError_t launch_route_k(const S1Args& a, dim3 grid, size_t lds, hipStream_t st) {
  static LdsOptIn opt_in;   // one per kernel (kern is a template argument)
  if (hipError_t e = allow_dyn_lds((const void*)kern, lds, opt_in); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, a);
  return hipGetLastError();
}

// Exact 3-way bf16 split of the fp32 summaries: x = hi + mid + lo with every piece
// obtained by truncation (same sign, no rounding), laid out [chunk][3][d].
__global__ __launch_bounds__(256) void ksplit_kernel(const float* __restrict__ kbar,
                                                     uint16_t* __restrict__ ksplit, int64_t n_rows,
                                                     int d) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= n_rows * d) return;
  const int64_t row = i / d;
  const int col = (int)(i % d);
  const float x = kbar[i];
  const uint32_t hi = __float_as_uint(x) & 0xffff0000u;
  const float r1 = x - __uint_as_float(hi);
  const uint32_t mid = __float_as_uint(r1) & 0xffff0000u;
  const float r2 = r1 - __uint_as_float(mid);
  uint16_t* o = ksplit + row * 3 * d + col;
  o[0] = (uint16_t)(hi >> 16);
  o[d] = (uint16_t)(mid >> 16);
  o[2 * d] = (uint16_t)(__float_as_uint(r2) >> 16);
}

static S1Args make_s1_args(const dash_params& p, const Layout& L, const void* q, const float* kbar, const S1Out& out) {
  S1Args a;
  a.q = q; a.ksplit = nullptr; a.scores = nullptr; a.kbar = kbar; a.k_upd = nullptr; a.kbar_upd = nullptr; a.ks_b = a.ks_h = a.ks_t = 0;
  a.mask = out.mask; a.cnt = out.cnt; a.idx = out.idx; a.bias = out.bias; a.tau = out.tau;
  a.batch = p.batch; a.h_q = p.h_q; a.h_kv = p.h_kv; a.g_q = L.g_q; a.n_q = p.n_q; a.n_kv = p.n_kv;
  a.block = p.block_size; a.seq_lens = L.seq_lens;
  a.t_c = L.t_c; a.t_all = L.t_all; a.words = L.words; a.pos0 = L.pos0; a.causal = p.causal; a.window = p.window;
  a.qs_b = p.q_stride[0]; a.qs_h = p.q_stride[1]; a.qs_t = p.q_stride[2];
  a.xscale = L.xscale; a.pexp = L.pexp; a.alpha = p.alpha; a.inv_sigma = 1.f / p.sigma;
  a.ld = 0; a.tok_base = 0; a.tok_end = p.n_q;
  return a;
}

// Stage 1 of a decode step (n_q = 1, causal): one launch, one workgroup per (sequence, kv-head).
hipError_t launch_s1_decode(const dash_params& p, const Layout& L, const void* q, const float* kbar,
                            const S1Out& out, const void* k_upd, float* kbar_upd, hipStream_t st) {
  S1Args a = make_s1_args(p, L, q, kbar, out);
  // k_upd: also summarise the chunk the current token completes, in a second set of workgroups
  // (uniform lengths: only if n_kv is a multiple of the chunk size; per-sequence lengths: decided per sequence)
  const bool upd = k_upd && kbar_upd && L.t_c > 0 && (L.seq_lens || p.n_kv % p.block_size == 0);
  if (upd) { a.k_upd = k_upd; a.kbar_upd = kbar_upd; a.ks_b = p.k_stride[0]; a.ks_h = p.k_stride[1]; a.ks_t = p.k_stride[2]; }
  int max_cand = L.t_c;
  if (!L.seq_lens) {
    max_cand = L.pos0 / p.block_size - p.window;
    if (max_cand > L.t_c) max_cand = L.t_c;
    if (max_cand < 0) max_cand = 0;
  }
  a.ld = ((max_cand + 15) / 16) * 16 + 4;
  size_t lds = ((size_t)16 * a.ld + (size_t)L.g_q * p.head_dim) * 4;
  if (upd && lds < 2048 * sizeof(double)) lds = 2048 * sizeof(double);   // the block mean's partial sums
  const dim3 grid((unsigned)(p.batch * p.h_kv * (upd ? 2 : 1)), 1, 1);
  static LdsOptIn opt_in[4];   // one per kernel below
  const void* kern;
  int which;
  if (p.dtype == DASH_BF16) {
    which = p.head_dim == 128 ? 0 : 1;
    kern = p.head_dim == 128 ? (const void*)s1_decode_kernel<uint16_t, 128> : (const void*)s1_decode_kernel<uint16_t, 64>;
  } else {
    which = p.head_dim == 128 ? 2 : 3;
    kern = p.head_dim == 128 ? (const void*)s1_decode_kernel<float, 128> : (const void*)s1_decode_kernel<float, 64>;
  }
  if (hipError_t e = allow_dyn_lds(kern, lds, opt_in[which]); e != hipSuccess) return e;
  switch (which) {
    case 0: hipLaunchKernelGGL((s1_decode_kernel<uint16_t, 128>), grid, dim3(1024), lds, st, a); break;
    case 1: hipLaunchKernelGGL((s1_decode_kernel<uint16_t, 64>), grid, dim3(1024), lds, st, a); break;
    case 2: hipLaunchKernelGGL((s1_decode_kernel<float, 128>), grid, dim3(1024), lds, st, a); break;
    default: hipLaunchKernelGGL((s1_decode_kernel<float, 64>), grid, dim3(1024), lds, st, a); break;
  }
  return hipGetLastError();
}

hipError_t launch_s1_route(const dash_params& p, const Layout& L, const void* q, const float* kbar,
                           uint16_t* ksplit, const float* scores, const S1Out& out, hipStream_t st) {
  if (ksplit != nullptr && L.t_c > 0) {
    const int64_t n_rows = (int64_t)p.batch * p.h_kv * L.t_c;
    const int64_t n = n_rows * p.head_dim;
    hipLaunchKernelGGL(ksplit_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, kbar,
                       ksplit, n_rows, p.head_dim);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  S1Args a = make_s1_args(p, L, q, kbar, out);
  a.ksplit = ksplit; a.scores = scores;
  const bool mfma = L.use_mfma && ksplit != nullptr;
  // Token ranges, each launched with the kernel and the sizes that fit its longest row
  // (causal rows grow with the position; boundaries at multiples of 64 tokens, longest
  // range first).  The register-resident kernels take the tokens whose rows have up to
  // 256, up to 512, and up to 1536 candidates (the last at head dimension 128), one range each.
  // What is left goes to the kernel below, which keeps the score rows of a workgroup in
  // LDS, sized for the longest row of its launch: there a long prefill is cut into four
  // ranges, so that the early ones get more rows per workgroup (fewer re-reads of the
  // summaries) and more workgroups per CU.  Measured with that kernel alone: 96k tokens,
  // GQA group 16: 25.9 -> 17.9 ms; 128k tokens, chunk 128: 12.5 -> 11.0 ms.
  int bounds[9];
  int nb = 0;
  bounds[nb++] = 0;
  if (p.causal && p.n_q > 1 && !L.seq_lens) {
    // the first token whose row has more than `cap` candidates
    auto first_beyond = [&](int cap) {
      const int64_t t = (int64_t)(cap + 1 + p.window) * p.block_size - L.pos0;
      return (int)(t < 0 ? 0 : (t > p.n_q ? p.n_q : t));
    };
    int lds_from = 0;   // tokens from here on go to the LDS-row kernel
    if (mfma) {
      const int t256 = first_beyond(256);
      if (t256 > 0 && t256 < p.n_q) bounds[nb++] = t256;
      const int t512 = first_beyond(512);
      const int t1536 = p.head_dim == 128 ? first_beyond(1536) : t512;
      if (t512 > t256 && t512 < p.n_q) bounds[nb++] = t512;
      if (t1536 > t512 && t1536 < p.n_q) bounds[nb++] = t1536;
      lds_from = t1536;
    }
    if (L.t_c >= 1024 && lds_from < p.n_q) {
      for (int sg = 1; sg < 4; sg++) {
        const int t = (int)((lds_from + (int64_t)(p.n_q - lds_from) * sg / 4 + 63) / 64 * 64);
        if (t > bounds[nb - 1] && t < p.n_q) bounds[nb++] = t;
      }
    }
  }
  bounds[nb] = p.n_q;
  for (int sg = nb - 1; sg >= 0; sg--) {
    const int t0 = bounds[sg], t1 = bounds[sg + 1];
    if (t1 <= t0) continue;
    int max_cand = L.t_c;
    if (p.causal && !L.seq_lens) {
      max_cand = (L.pos0 + t1 - 1) / p.block_size - p.window;
      if (max_cand > L.t_c) max_cand = L.t_c;
      if (max_cand < 0) max_cand = 0;
    }
    a.ld = ((max_cand + 15) / 16) * 16 + 4;
    a.tok_base = t0; a.tok_end = t1;
    if (mfma && s1_regs_applicable(p, L, max_cand)) {
      // the score rows stay in registers (stage1_regs.hip)
      if (hipError_t e = launch_s1_regs(p, L, a, max_cand, st); e != hipSuccess) return e;
      continue;
    }
    int mt = 1;
    if (mfma) {
      if ((size_t)64 * a.ld * 4 <= 65536) mt = 4;
      else if ((size_t)32 * a.ld * 4 <= 81920) mt = 2;
    }
    const int tokt = 16 * mt / L.g_q;
    // x = tiles * kv-heads * batch, decoded in the kernel
    dim3 grid((unsigned)(((t1 - t0 + tokt - 1) / tokt) * p.h_kv * p.batch), 1, 1);
    const size_t lds = (size_t)16 * mt * a.ld * 4;
    hipError_t e;
    if (!mfma) {
      e = p.head_dim == 128 ? launch_route_k<s1_route_kernel<1, 128, false>>(a, grid, lds, st)
                            : launch_route_k<s1_route_kernel<1, 64, false>>(a, grid, lds, st);
    } else {
#define DASH_RT(MT_)                                                                     \
  (p.head_dim == 128 ? launch_route_k<s1_route_kernel<MT_, 128, true>>(a, grid, lds, st) \
                     : launch_route_k<s1_route_kernel<MT_, 64, true>>(a, grid, lds, st))
      e = mt == 4 ? DASH_RT(4) : (mt == 2 ? DASH_RT(2) : DASH_RT(1));
#undef DASH_RT
    }
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace dash
