// Split-KV decode of Stage 2 (bf16): one query token per sequence attends its
// routed chunks with the Stage-1 bias added to the logits (Sec. 3.3 Eq. 6 in the
// bias form of Proposition 1; Alg. 3), the attended list cut into splits whose
// partial results a merge kernel combines (Sec. 3.5); the dense decode reference
// (Eq. 1) comes from the same template.
//
// Tiling.  A workgroup (4 waves) owns 128 (token, head) rows of one kv-head:
// wave w owns 32 rows = all g_q heads of 32/g_q consecutive tokens (its
// "granule").  The workgroup walks the union of its tokens' chunk masks in
// ascending order; every 64-key tile of K and V is staged once in LDS (double
// buffered: the global loads of tile j+1 are in flight while tile j is
// computed) and a wave skips the MFMA work of a chunk none of its tokens kept.
// Rows of a granule that did not keep a chunk get bias -inf for it, which keeps
// the per-token result exact.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16, wave64).  Both products are
// computed transposed so that no register shuffle is needed between them:
//   S^T[key,row]  = K[key,:] . Q[row,:]      A = K tile (LDS), B = Q (registers)
//   O^T[d,row]   += V^T[d,key] . P^T[key,row] A = V^T tile (LDS), B = P (registers)
// In the 32x32 accumulator layout lane (n = lane%32, h = lane/32) holds, for
// row n, the 16 keys {8q + 4h + i}: exactly the operand-B slots of lane (n, h)
// once the contraction index of the second product is permuted accordingly.
// That permutation is applied for free when V is transposed into LDS (an 8x8
// bf16 register transpose per thread).  Row max / row sum are in-lane plus one
// cross-half exchange, and the O rescale is a per-lane scalar.
#include <math.h>
#include <stdlib.h>

#include <type_traits>

#include "common.h"
#include "dash_internal.h"
#include "stage2_args.h"

// Two workgroups (8 waves) per CU: with <= 256 VGPRs per wave a second wave per
// SIMD overlaps its softmax VALU work with the other wave's MFMAs.
#ifndef DASH_S2_MIN_WG
#define DASH_S2_MIN_WG 2
#endif

namespace dash {


template <int D> struct S2Cfg {
  static constexpr int KLD = D + 8;          // bf16 elements per K row in LDS
  static constexpr int VLD = 64 + 8;         // bf16 elements per V^T row in LDS
  static constexpr int K_ELEMS = 64 * KLD;
  static constexpr int V_ELEMS = D * VLD;
  static constexpr int K_LOADS = (64 * D * 2 / 16) / 128;   // 16-byte loads per K-staging thread
  static constexpr size_t LDS_BYTES = (size_t)2 * (K_ELEMS + V_ELEMS) * 2 + 5 * 64 * 4;
};

// slot (position along the contraction index as stored in LDS) -> key offset
// inside a 64-key tile: slot bits [g:2 | h:1 | i_hi:1 | i_lo:2] <-> key bits
// [g:2 | i_hi:1 | h:1 | i_lo:2]
__device__ __forceinline__ int slot_group_key(int sg, int i) {
  return (sg >> 1) * 16 + (i >> 2) * 8 + (sg & 1) * 4 + (i & 3);
}

// RT: 32-row tiles per wave (1 or 2).  A wave owns 32*RT (token, head) rows; the
// K / V^T fragments it reads from LDS are reused for its RT row tiles, so RT = 2
// halves the LDS traffic per MFMA flop.
//
// DECODE: one query token per sequence (n_q == 1).  All four waves hold the same
// g_q rows and compute the same S^T; wave w accumulates only the d-tile w of
// O^T.  The workgroup handles the `split`-th share of the token's attended
// chunks and writes an unnormalised partial (O, running max, running sum) that
// a merge kernel combines (split-KV decoding, Sec. 3.5).
template <int D, int RT, bool DENSE, bool DECODE>
__global__ __launch_bounds__(256, DASH_S2_MIN_WG) void s2_decode_kernel(S2Args a) {
  using C = S2Cfg<D>;
  static_assert(!DECODE || RT == 1, "decode uses one row tile");
  extern __shared__ __attribute__((aligned(16))) uint16_t lds[];
  uint16_t* Ks = lds;                               // [2][64][KLD]
  uint16_t* Vt = lds + 2 * C::K_ELEMS;              // [2][D][VLD]
  uint32_t* wgmask = reinterpret_cast<uint32_t*>(lds + 2 * (C::K_ELEMS + C::V_ELEMS));  // [64]
  uint32_t* wvmask = wgmask + 64;                   // [4][64]

  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int n = lane & 31, h = lane >> 5;
  // workgroup id -> (tile, kv-head, batch): consecutive ids walk the (head, batch)
  // pairs so that the 8 XCDs (round-robin dispatch) each see few distinct KV streams
  const int hbi = blockIdx.x % a.hb;
  const int tile = a.n_tiles - 1 - blockIdx.x / a.hb;   // longest rows first; DECODE: split id
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  constexpr int WROWS = 32 * RT;                    // rows per wave
  const int tokw = DECODE ? 1 : WROWS / a.g_q;      // tokens per wave
  const int tok_w0 = DECODE ? 0 : tile * 4 * tokw + wave * tokw;   // first token of this wave
  const int nsub = a.block >> 6;

  // ---- per-row constants (row tile rt, row n of it) -----------------------
  int my_tok[RT], my_head[RT], row_pos[RT];
  bool row_ok[RT];
#pragma unroll
  for (int rt = 0; rt < RT; rt++) {
    const int row = rt * 32 + n;
    my_tok[rt] = DECODE ? 0 : tok_w0 + row / a.g_q;
    my_head[rt] = r * a.g_q + row % a.g_q;
    row_ok[rt] = DECODE ? row < a.g_q : my_tok[rt] < a.n_q;
    row_pos[rt] = a.pos0 + (row_ok[rt] ? my_tok[rt] : a.n_q - 1);
  }
  // chunk of the wave's tokens (all tokens of a wave share it)
  const int cw = (a.pos0 + (tok_w0 < a.n_q ? tok_w0 : a.n_q - 1)) / a.block;
  const bool wave_ok = tok_w0 < a.n_q;

  // ---- Q fragments (operand B of S^T = K Q^T) ----------------------------
  bf16x8 qf[RT][D / 16];
#pragma unroll
  for (int rt = 0; rt < RT; rt++) {
    const uint16_t* qp = a.q + b * a.qs_b + my_head[rt] * a.qs_h +
                         (int64_t)(row_ok[rt] ? my_tok[rt] : a.n_q - 1) * a.qs_t + h * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) qf[rt][ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }

  // ---- chunk bitmaps -------------------------------------------------------
  // lane t < tokw tracks token tok_w0 + t: its mask row, its rank in the compact
  // bias list, and the next bias value (prefetched).
  const int trk_tok = tok_w0 + lane;
  const bool trk_ok = lane < tokw && trk_tok < a.n_q;
  const int64_t trk_base = ((int64_t)b * a.h_kv + r) * a.n_q + (trk_ok ? trk_tok : 0);
  const uint32_t* trk_mask = DENSE ? nullptr : a.mask + trk_base * a.words;
  const float* trk_bias = DENSE ? nullptr : a.bias + trk_base * a.t_all;
  int trk_rank = 0, trk_wi = -1;
  uint32_t trk_word = 0;
  float trk_next = 0.f;

  for (int i = tid; i < 5 * 64; i += 256) wgmask[i] = 0u;
  __syncthreads();
  if (DENSE) {
    // every chunk up to the wave's own (causal) / every chunk (non-causal)
    const int last = a.causal ? cw : a.t_all - 1;
    if (wave_ok)
      for (int wi = lane; wi < a.words; wi += 64) {
        const int lo = wi * 32;
        uint32_t m = 0u;
        if (last >= lo) m = (last - lo >= 31) ? 0xffffffffu : ((2u << (last - lo)) - 1u);
        wvmask[wave * 64 + wi] = m;
        if (m) atomicOr(&wgmask[wi], m);
      }
  } else {
    if (wave_ok)
      for (int wi = lane; wi < a.words; wi += 64) {
        uint32_t m = 0u;
        for (int t = 0; t < tokw; t++)
          if (tok_w0 + t < a.n_q)
            m |= a.mask[(((int64_t)b * a.h_kv + r) * a.n_q + tok_w0 + t) * a.words + wi];
        wvmask[wave * 64 + wi] = m;
        if (m) atomicOr(&wgmask[wi], m);
      }
  }
  __syncthreads();
  if (DECODE) {
    // keep only this split's share of the attended chunks: entries
    // [e0, e1) of the ascending list.  Wave 0: lane wi owns mask word wi.
    if (wave == 0) {
      const uint32_t w0 = wgmask[lane];
      const int pc = __popc(w0);
      int incl = pc;                               // inclusive prefix sum over lanes
#pragma unroll
      for (int off = 1; off < 64; off <<= 1) {
        const int t = __shfl_up(incl, off);
        if (lane >= off) incl += t;
      }
      const int total = __shfl(incl, 63);
      const int per = (total + a.n_tiles - 1) / a.n_tiles;
      const int e0 = tile * per, e1 = min(total, e0 + per);
      const int start = incl - pc;                 // rank of this word's first set bit
      uint32_t w = w0;
      int drop = e0 - start;                       // set bits to clear from the bottom
      for (int i = 0; i < drop && w; i++) w &= w - 1u;
      int keep = e1 - max(start, e0);              // set bits to keep after that
      uint32_t kept = 0u;
      for (int i = 0; i < keep && w; i++) { kept |= w & (0u - w); w &= w - 1u; }
      wgmask[lane] = kept;
      if (lane == 0) wvmask[0] = (uint32_t)min(e0, total);   // rank of the split's first entry
    }
    __syncthreads();
    trk_rank = (int)wvmask[0];
    __syncthreads();
    // every wave participates in every kept chunk
    for (int i = tid; i < 64; i += 256) { const uint32_t w = wgmask[i]; wvmask[i] = w; wvmask[64 + i] = w; wvmask[128 + i] = w; wvmask[192 + i] = w; }
    __syncthreads();
  }
  if (!DENSE && !DECODE && trk_ok && trk_rank < a.t_all) trk_next = trk_bias[trk_rank];

  // ---- tile iterator (workgroup-uniform) ---------------------------------
  int it_wi = -1, it_sub = nsub - 1, it_u = -1;
  uint32_t it_bits = 0u;
  auto advance = [&]() -> bool {   // moves (it_u, it_sub) to the next 64-key tile
    if (it_u >= 0 && it_sub + 1 < nsub) { it_sub++; return true; }
    while (it_bits == 0u) {
      if (++it_wi >= a.words) return false;
      it_bits = __builtin_amdgcn_readfirstlane(wgmask[it_wi]);
    }
    it_u = it_wi * 32 + __builtin_ctz(it_bits);
    it_bits &= it_bits - 1u;
    it_sub = 0;
    return true;
  };

  // ---- staging -------------------------------------------------------------
  // Threads 0..127 stage K (row-major copy), threads 128..255 stage V (8x8 bf16
  // register transpose into the permuted V^T layout).  Every load address is
  // "uniform tile base + uniform per-load stride + per-thread byte offset", so the
  // per-tile address arithmetic is scalar.
  const bool stage_k = tid < 128;
  const int st = tid & 127;
  const char* kbase = reinterpret_cast<const char*>(a.k + b * a.ks_b + r * a.ks_h);
  const char* vbase = reinterpret_cast<const char*>(a.v + b * a.vs_b + r * a.vs_h);
  u32x4 sreg[8];
  u32x4 sreg2[DECODE ? 8 : 1];   // decode: second set, tiles are fetched two ahead
  const int v_sg = st & 7, v_dg = st >> 3;          // V: slot group, 8-column group
  constexpr int KROWS = 128 / (D / 8);              // K rows covered by one load of the 128 threads
  const int k_row0 = st / (D / 8), k_col = (st % (D / 8)) * 8;
  const int v_row0 = (v_sg >> 1) * 16 + (v_sg & 1) * 4;
  const uint32_t k_toff = (uint32_t)(k_row0 * a.ks_t + k_col) * 2u;     // bytes
  const uint32_t v_toff = (uint32_t)(v_row0 * a.vs_t + v_dg * 8) * 2u;
  const bool v_active = v_dg < D / 8;
  auto stage_load = [&](int u, int sub, u32x4 (&sreg)[8]) {
    const int kpos0 = u * a.block + sub * 64;
    if (kpos0 + 64 <= a.n_kv) {
      if (stage_k) {
        const char* tb = kbase + (int64_t)kpos0 * a.ks_t * 2;
#pragma unroll
        for (int i = 0; i < C::K_LOADS; i++)
          sreg[i] = *reinterpret_cast<const u32x4*>(tb + (int64_t)i * KROWS * a.ks_t * 2 + k_toff);
      } else if (v_active) {
        const char* tb = vbase + (int64_t)kpos0 * a.vs_t * 2;
#pragma unroll
        for (int i = 0; i < 8; i++)
          sreg[i] = *reinterpret_cast<const u32x4*>(tb + (int64_t)((i >> 2) * 8 + (i & 3)) * a.vs_t * 2 + v_toff);
      }
    } else {
      // ragged last tile: clamp the row index (those keys are masked later)
      if (stage_k) {
#pragma unroll
        for (int i = 0; i < C::K_LOADS; i++) {
          int key = kpos0 + i * KROWS + k_row0;
          key = key < a.n_kv ? key : a.n_kv - 1;
          sreg[i] = *reinterpret_cast<const u32x4*>(kbase + ((int64_t)key * a.ks_t + k_col) * 2);
        }
      } else if (v_active) {
#pragma unroll
        for (int i = 0; i < 8; i++) {
          int key = kpos0 + slot_group_key(v_sg, i);
          key = key < a.n_kv ? key : a.n_kv - 1;
          sreg[i] = *reinterpret_cast<const u32x4*>(vbase + ((int64_t)key * a.vs_t + v_dg * 8) * 2);
        }
      }
    }
  };
  uint16_t* const k_dst0 = Ks + k_row0 * C::KLD + k_col;
  uint16_t* const v_dst0 = Vt + (v_dg * 8) * C::VLD + v_sg * 8;
  auto stage_store = [&](int buf, const u32x4 (&sreg)[8]) {
    if (stage_k) {
      uint16_t* dst = k_dst0 + buf * C::K_ELEMS;
#pragma unroll
      for (int i = 0; i < C::K_LOADS; i++)
        *reinterpret_cast<u32x4*>(dst + i * KROWS * C::KLD) = sreg[i];
    } else if (v_active) {
      uint16_t* dst = v_dst0 + buf * C::V_ELEMS;
      // 8x8 bf16 transpose: column e of the 8 loaded rows becomes one 16-byte row
#pragma unroll
      for (int e = 0; e < 8; e++) {
        u32x4 o;
#pragma unroll
        for (int i2 = 0; i2 < 4; i2++) {
          const uint32_t lo = sreg[2 * i2][e >> 1], hi = sreg[2 * i2 + 1][e >> 1];
          // byte select: low halves {hi[1:0], lo[1:0]} or high halves {hi[3:2], lo[3:2]}
          o[i2] = __builtin_amdgcn_perm(hi, lo, (e & 1) ? 0x07060302u : 0x05040100u);
        }
        *reinterpret_cast<u32x4*>(dst + e * C::VLD) = o;
      }
    }
  };

  // ---- online-softmax state (base-2 logits) -------------------------------
  float m_run[RT], l_run[RT];
  constexpr int NDT = DECODE ? 1 : D / 32;
  f32x16 oacc[RT][NDT];
#pragma unroll
  for (int rt = 0; rt < RT; rt++) {
    m_run[rt] = -INFINITY; l_run[rt] = 0.f;
#pragma unroll
    for (int dt = 0; dt < NDT; dt++)
#pragma unroll
      for (int j = 0; j < 16; j++) oacc[rt][dt][j] = 0.f;
  }

  float bias_row[RT];   // bias * log2e of this lane's rows for the current chunk
#pragma unroll
  for (int rt = 0; rt < RT; rt++) bias_row[rt] = 0.f;
  bool wave_on = false, diag = false;

  // DECODE: one token per workgroup, so the bias list is walked with wave-uniform
  // (scalar) loads; they do not queue behind the vector loads of the tile prefetch.
  const float* dec_bias = DENSE ? nullptr : a.bias + (((int64_t)b * a.h_kv + r) * a.n_q) * a.t_all;
  int dec_rank = DECODE ? __builtin_amdgcn_readfirstlane(trk_rank) : 0;

  auto begin_chunk = [&](int u) {
    // decides participation and fetches the per-token bias of chunk u
    wave_on = wave_ok && ((__builtin_amdgcn_readfirstlane(wvmask[wave * 64 + (u >> 5)]) >> (u & 31)) & 1u);
    diag = a.causal && u == cw;
    if (!wave_on) return;
    if constexpr (DECODE) {
      // every chunk this workgroup visits is one of the token's attended chunks,
      // in list order; padded rows simply share the bias
      float bt = 0.f;
      if (!DENSE && !diag) { bt = dec_bias[dec_rank] * kLog2e; dec_rank++; }
      bias_row[0] = bt;
      return;
    }
    float bt = 0.f;
    if (!DENSE && !diag) {
      bt = -INFINITY;
      if (trk_ok) {
        if ((u >> 5) != trk_wi) { trk_wi = u >> 5; trk_word = trk_mask[trk_wi]; }
        if ((trk_word >> (u & 31)) & 1u) {
          bt = trk_next * kLog2e;
          trk_rank++;
          if (trk_rank < a.t_all) trk_next = trk_bias[trk_rank];
        }
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; rt++) bias_row[rt] = __shfl(bt, (rt * 32 + n) / a.g_q);
  };

  // One 64-key tile: S^T = K Q^T, online softmax, O^T += V^T P^T.  MASKED adds
  // the causal / sequence-end key mask (diagonal chunk and ragged tail only).
  auto compute = [&](int buf, int kpos0, auto masked_tag) {
    constexpr bool MASKED = decltype(masked_tag)::value;
    const uint16_t* Kb = Ks + buf * C::K_ELEMS + n * C::KLD + h * 8;
    const uint16_t* Vb = Vt + buf * C::V_ELEMS + n * C::VLD + h * 8;
    f32x16 s[RT][2];
#pragma unroll
    for (int rt = 0; rt < RT; rt++)
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int j = 0; j < 16; j++) s[rt][kt][j] = 0.f;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++)
#pragma unroll
      for (int kt = 0; kt < 2; kt++) {
        const bf16x8 ka = *reinterpret_cast<const bf16x8*>(Kb + kt * 32 * C::KLD + ks * 16);
#pragma unroll
        for (int rt = 0; rt < RT; rt++)
          s[rt][kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka, qf[rt][ks], s[rt][kt], 0, 0, 0);
      }
    bf16x8 pb[RT][4];
    bool grow = false;
    float tmax[RT];
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
      float mloc = -INFINITY;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int j = 0; j < 16; j++) {
          if constexpr (MASKED) {
            const int kp = kpos0 + kt * 32 + (j >> 2) * 8 + h * 4 + (j & 3);
            const bool dead = (diag && kp > row_pos[rt]) || kp >= a.n_kv;
            s[rt][kt][j] = dead ? -INFINITY : s[rt][kt][j];
          }
          mloc = fmaxf(mloc, s[rt][kt][j]);
        }
      mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
      // max of the base-2 logits s*c1 + bias over the tile (c1 > 0)
      tmax[rt] = fmaf(mloc, a.c1, bias_row[rt]);
      grow = grow || (tmax[rt] > m_run[rt] + kLazy);
    }
    // Lazy rescaling: the reference max m_run of a row is only raised when the
    // tile's max exceeds it by more than 2^kLazy; until then p = 2^(t - m_run)
    // may reach 2^kLazy, which fp32 / bf16 hold without loss, and the final
    // division by the row sum is unaffected.  Raising it is rare after the
    // first tiles, so the O rescale below is almost never executed.
    if (__any(grow)) {
#pragma unroll
      for (int rt = 0; rt < RT; rt++) {
        const float m_new = fmaxf(m_run[rt], tmax[rt]);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float corr = __builtin_amdgcn_exp2f(m_run[rt] - m_use);   // m_run = -inf -> 0
        m_run[rt] = m_new;
        l_run[rt] *= corr;
#pragma unroll
        for (int dt = 0; dt < NDT; dt++)
#pragma unroll
          for (int j = 0; j < 16; j++) oacc[rt][dt][j] *= corr;
      }
    }
#pragma unroll
    for (int rt = 0; rt < RT; rt++) {
      const float off = bias_row[rt] - (m_run[rt] == -INFINITY ? 0.f : m_run[rt]);
      float lsum = 0.f;
#pragma unroll
      for (int kt = 0; kt < 2; kt++)
#pragma unroll
        for (int j = 0; j < 16; j++) {
          const float pj = __builtin_amdgcn_exp2f(fmaf(s[rt][kt][j], a.c1, off));
          lsum += pj;
          pb[rt][kt * 2 + (j >> 3)][j & 7] = (__bf16)pj;
        }
      l_run[rt] += lsum;
    }
    if constexpr (DECODE) {
      if (wave < D / 32) {
#pragma unroll
        for (int g = 0; g < 4; g++) {
          const bf16x8 va = *reinterpret_cast<const bf16x8*>(Vb + wave * 32 * C::VLD + g * 16);
          oacc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[0][g], oacc[0][0], 0, 0, 0);
        }
      }
    } else {
#pragma unroll
      for (int g = 0; g < 4; g++)
#pragma unroll
        for (int dt = 0; dt < D / 32; dt++) {
          const bf16x8 va = *reinterpret_cast<const bf16x8*>(Vb + dt * 32 * C::VLD + g * 16);
#pragma unroll
          for (int rt = 0; rt < RT; rt++)
            oacc[rt][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va, pb[rt][g], oacc[rt][dt], 0, 0, 0);
        }
    }
  };

  // ---- main loop -----------------------------------------------------------
  auto run_tile = [&](int cu, int csub, int buf) {
    if (wave_on) {
      const int kpos0 = cu * a.block + csub * 64;
      if (diag || kpos0 + 64 > a.n_kv) compute(buf, kpos0, std::true_type{});
      else compute(buf, kpos0, std::false_type{});
    }
  };
  int buf = 0;
  if constexpr (!DECODE) {
    bool have = advance();
    if (have) {
      stage_load(it_u, it_sub, sreg);
      stage_store(0, sreg);
    }
    __syncthreads();
    while (have) {
      const int cu = it_u, csub = it_sub;
      const bool more = advance();
      // bias bookkeeping first: its wait on the previously prefetched bias must not
      // also wait for the tile loads issued next
      if (csub == 0) begin_chunk(cu);
      if (more) stage_load(it_u, it_sub, sreg);
      run_tile(cu, csub, buf);
      if (more) stage_store(buf ^ 1, sreg);
      __syncthreads();
      buf ^= 1;
      have = more;
    }
  } else {
    // Decode is bound by HBM latency x bandwidth, not by compute: keep two tiles
    // (64 KB per workgroup) in flight.  While tile j is computed from LDS, tile
    // j+1 and tile j+2 are on their way into the two register sets, which swap
    // roles every iteration (the loop body is written out twice).
    bool have0 = advance();
    int u0 = it_u, s0 = it_sub;
    if (have0) { stage_load(u0, s0, sreg); stage_store(0, sreg); }
    bool have1 = have0 && advance();
    int u1 = it_u, s1 = it_sub;
    if (have1) stage_load(u1, s1, sreg);
    bool have2 = have1 && advance();
    int u2 = it_u, s2 = it_sub;
    if (have2) stage_load(u2, s2, sreg2);
    __syncthreads();
    auto step = [&](u32x4 (&pr)[8]) {
      // pr holds tile j+1 (if any); after it is stored it receives tile j+3
      if (s0 == 0) begin_chunk(u0);
      run_tile(u0, s0, buf);
      if (have1) stage_store(buf ^ 1, pr);
      const bool have3 = have2 && advance();
      if (have3) stage_load(it_u, it_sub, pr);
      __syncthreads();
      buf ^= 1;
      have0 = have1; u0 = u1; s0 = s1;
      have1 = have2; u1 = u2; s1 = s2;
      have2 = have3; u2 = it_u; s2 = it_sub;
    };
    while (have0) {
      step(sreg);
      if (!have0) break;
      step(sreg2);
    }
  }

  // ---- finalise ------------------------------------------------------------
#pragma unroll
  for (int rt = 0; rt < RT; rt++) {
    const float l_tot = l_run[rt] + __shfl_xor(l_run[rt], 32);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if constexpr (DECODE) {
      // partial record per (batch, kv-head, split, head-in-group): D floats of
      // unnormalised O, then the running max (base-2 logits) and the running sum
      if (row_ok[0] && wave < D / 32) {
        float* pp = a.part + ((((int64_t)b * a.h_kv + r) * a.n_tiles + tile) * a.g_q + n) * (D + 2);
#pragma unroll
        for (int j = 0; j < 16; j++)
          pp[wave * 32 + (j >> 2) * 8 + h * 4 + (j & 3)] = oacc[0][0][j];
        if (wave == 0 && h == 0) { pp[D] = m_run[0]; pp[D + 1] = l_tot; }
      }
    } else if (row_ok[rt]) {
      uint16_t* op = a.o + b * a.os_b + my_head[rt] * a.os_h + (int64_t)my_tok[rt] * a.os_t;
#pragma unroll
      for (int dt = 0; dt < NDT; dt++)
#pragma unroll
        for (int q4 = 0; q4 < 4; q4++) {
          const int d0 = dt * 32 + q4 * 8 + h * 4;
          uint2 w;
          w.x = pack_bf16x2(oacc[rt][dt][q4 * 4 + 0] * inv, oacc[rt][dt][q4 * 4 + 1] * inv);
          w.y = pack_bf16x2(oacc[rt][dt][q4 * 4 + 2] * inv, oacc[rt][dt][q4 * 4 + 3] * inv);
          *reinterpret_cast<uint2*>(op + d0) = w;
        }
    }
  }
}

template <int D, int RT, bool DENSE, bool DECODE>
static hipError_t launch_s2_t(const S2Args& a, hipStream_t st) {
  using C = S2Cfg<D>;
  auto kern = s2_decode_kernel<D, RT, DENSE, DECODE>;
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       (int)C::LDS_BYTES);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.hb), dim3(256), C::LDS_BYTES, st, a);
  return hipGetLastError();
}

// Merge of the split-KV partials: o = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s.
template <typename T>
__global__ __launch_bounds__(128) void decode_merge_kernel(const float* __restrict__ part,
                                                           T* __restrict__ o, int h_q, int h_kv,
                                                           int g_q, int splits, int d,
                                                           int64_t os_b, int64_t os_h) {
  const int head = blockIdx.x, b = blockIdx.y;
  const int r = head / g_q, hl = head % g_q;
  const int col = threadIdx.x;
  const int rec = d + 2;
  const float* base = part + (((int64_t)b * h_kv + r) * splits * g_q + hl) * rec;
  float M = -INFINITY;
  for (int s = 0; s < splits; s++) M = fmaxf(M, base[(int64_t)s * g_q * rec + d]);
  float num = 0.f, den = 0.f;
  for (int s = 0; s < splits; s++) {
    const float* ps = base + (int64_t)s * g_q * rec;
    const float m = ps[d];
    const float w = m == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m - M);
    den += w * ps[d + 1];
    if (col < d && w > 0.f) num += w * ps[col];
  }
  if (col < d) elem<T>::st(o + b * os_b + head * os_h + col, num / den);
}

hipError_t launch_decode_s2(const dash_params& p, const Layout& L, const void* q, const void* k,
                            const void* v, void* o, const uint32_t* mask, const float* bias,
                            float* partials, bool dense, hipStream_t st) {
  S2Args a;
  fill_s2_args(a, p, L, q, k, v, o, mask, bias);
  a.n_tiles = L.splits;
  a.part = partials;
  hipError_t e;
  if (p.head_dim == 128)
    e = dense ? launch_s2_t<128, 1, true, true>(a, st) : launch_s2_t<128, 1, false, true>(a, st);
  else
    e = dense ? launch_s2_t<64, 1, true, true>(a, st) : launch_s2_t<64, 1, false, true>(a, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_merge_kernel<uint16_t>, dim3(p.h_q, p.batch), dim3(128), 0, st, partials,
                     (uint16_t*)o, p.h_q, p.h_kv, L.g_q, L.splits, p.head_dim, p.o_stride[0],
                     p.o_stride[1]);
  return hipGetLastError();
}

}  // namespace dash
