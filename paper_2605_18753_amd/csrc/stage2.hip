// Stage 2 (bf16 prefill): block-sparse softmax attention over the routed chunks
// with the Stage-1 bias added to the logits (Sec. 3.3 Eq. 6 in the bias form of
// Proposition 1; Alg. 3), and the dense reference attention (Eq. 1) from the
// same template.
//
// Tiling.  A workgroup (4 waves) owns 128 (token, head) rows of one kv-head:
// wave w owns 32 rows = all g_q heads of 32/g_q consecutive tokens.  The
// workgroup walks the union of its tokens' chunk masks in ascending order.
// Every 64-key tile of K and V is copied once from global memory straight into
// LDS (buffer_load_dwordx4 ... lds, no staging registers), two stages deep: the copy
// of tile j+1 is in flight while tile j is computed.  A wave skips the MFMA work
// of a chunk none of its tokens kept; rows of a wave that did not keep a chunk
// get bias -inf for it, which keeps the per-token result exact.
//
// LDS layout.  Tiles are row major ([key][d], no padding: the direct copy writes
// 1 KB contiguous per wave instruction) with the 16-byte chunks of every row
// permuted by an XOR pattern chosen per tensor so that the operand reads below
// are free of bank conflicts; the permutation is applied on the global side
// (which chunk a lane fetches), so it costs nothing.
//
// MFMA formulation (v_mfma_f32_32x32x16_bf16, wave64).  Both products are
// computed transposed so that no register shuffle is needed between them:
//   S^T[key,row]  = K[key,:] . Q[row,:]      A = K tile (LDS), B = Q (registers)
//   O^T[d,row]   += V^T[d,key] . P^T[key,row] A = V^T (LDS, transposing read), B = P
// In the 32x32 accumulator layout lane (n = lane%32, h = lane/32) holds, for
// row n, the 16 keys {8q + 4h + i}: exactly the operand-B slots of lane (n, h)
// once the contraction index of the second product is ordered accordingly.  The
// V^T operand is read from the row-major V tile with ds_read_b64_tr_b16, which
// hands each lane four consecutive keys of one d column.  Row max / row sum are
// in-lane plus one cross-half exchange, and the O rescale is a per-lane scalar.
#include <math.h>
#include <stdlib.h>

#include <type_traits>

#include "common.h"
#include "dash_internal.h"
#include "lds_copy.h"
#include "stage2_args.h"

namespace dash {


template <int D> struct S2Cfg {
  static constexpr int NCH = D / 8;                       // 16-byte chunks per row
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int TILE_BYTES = 64 * ROW_BYTES;       // one K or V tile
  static constexpr int COPIES = TILE_BYTES / 16 / 256;    // copy instructions per thread, tile and tensor
  static constexpr int ROWS_PER_COPY = 256 / NCH;         // rows one copy instruction of the workgroup covers
  static constexpr int MASK_OFF = 4 * TILE_BYTES;            // after the K ring [2] and the V ring [2]
  static constexpr size_t LDS_BYTES = (size_t)MASK_OFF + 5 * 64 * 4;
};

// Chunk permutations (position of logical 16-byte chunk c of tile row `row`).
// K: the A-operand read has lanes n = 0..15 on 16 consecutive rows at the same
// logical chunk, so those rows must spread over all 16 chunk slots of a 256-byte
// bank window.  V: the transposing read has 16 lanes on 4 consecutive rows x 4
// consecutive chunks, so rows r..r+3 must land in different 64-byte groups.
template <int D> __device__ __forceinline__ int k_swz(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int v_swz(int row) {
  return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

template <int D, bool DENSE>
__global__ __launch_bounds__(256, 2) void s2_attend_kernel(S2Args a) {
  using C = S2Cfg<D>;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  uint32_t* wgmask = reinterpret_cast<uint32_t*>(lds + C::MASK_OFF);   // [64]
  uint32_t* wvmask = wgmask + 64;                                      // [4][64]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  // workgroup id -> (tile, kv-head, batch): consecutive ids walk the (head, batch)
  // pairs so that the 8 XCDs (round-robin dispatch) each see few distinct KV streams
  const int hbi = blockIdx.x % a.hb;
  const int tile = a.n_tiles - 1 - blockIdx.x / a.hb;   // longest rows first
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int tokw = 32 / a.g_q;                          // tokens per wave
  const int tok_w0 = tile * 4 * tokw + wave * tokw;     // first token of this wave
  const int nsub = a.block >> 6;

  // ---- per-row constants ---------------------------------------------------
  const int my_tok = tok_w0 + n / a.g_q;
  const int my_head = r * a.g_q + n % a.g_q;
  const bool row_ok = my_tok < a.n_q;
  const int row_pos = a.pos0 + (row_ok ? my_tok : a.n_q - 1);
  // chunk of the wave's tokens (all tokens of a wave share it)
  const int cw = (a.pos0 + (tok_w0 < a.n_q ? tok_w0 : a.n_q - 1)) / a.block;
  const bool wave_ok = tok_w0 < a.n_q;

  // ---- Q fragments (operand B of S^T = K Q^T) ------------------------------
  bf16x8 qf[D / 16];
  {
    const uint16_t* qp = a.q + b * a.qs_b + my_head * a.qs_h +
                         (int64_t)(row_ok ? my_tok : a.n_q - 1) * a.qs_t + h * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
    // the loads must be complete (and known to be) before the tile loop: a wait for
    // them inside the loop would also wait for the tile copies in flight
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) asm volatile("" : "+v"(qf[ks]));
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
  if (!DENSE && trk_ok && trk_rank < a.t_all) trk_next = trk_bias[trk_rank];

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

  // ---- global -> LDS tile copies -------------------------------------------
  // Copy instruction i of wave w fills the 1 KB LDS segment (4i + w): slot
  // s = (4i + w) * 64 + lane, tile row s / NCH, chunk position s % NCH, which
  // receives logical chunk pos ^ swz(row) of that row.  The swizzle depends only
  // on (w, lane), so each thread keeps one byte offset per tensor; the tile and
  // instruction offsets are scalar (buffer addressing: resource + lane offset +
  // scalar offset).  The resource ends with the last key, so the rows a ragged
  // last tile has beyond n_kv read as zeros instead of touching memory.
  const u32x4 k_rs = make_rsrc(a.k + b * a.ks_b + r * a.ks_h, (((int64_t)a.n_kv - 1) * a.ks_t + D) * 2);
  const u32x4 v_rs = make_rsrc(a.v + b * a.vs_b + r * a.vs_h, (((int64_t)a.n_kv - 1) * a.vs_t + D) * 2);
  const uint32_t lds0 = lds_addr_of(lds);
  const int c_row = (wave * 64 + lane) / C::NCH, c_pos = lane % C::NCH;
  const uint32_t k_off = (uint32_t)(c_row * (int)a.ks_t * 2 + ((c_pos ^ k_swz<D>(c_row)) << 4));
  const uint32_t v_off = (uint32_t)(c_row * (int)a.vs_t * 2 + ((c_pos ^ v_swz<D>(c_row)) << 4));
  const uint32_t k_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.ks_t * 2);
  const uint32_t v_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.vs_t * 2);
  // copy instruction c of a tile: c < COPIES moves K rows, the rest V rows
  uint32_t cp_k = 0, cp_v = 0;   // scalar byte offsets of the tile being copied
  auto copy_begin = [&](int u, int sub) {
    cp_k = (uint32_t)(u * a.block + sub * 64) * (uint32_t)a.ks_t * 2u;
    cp_v = (uint32_t)(u * a.block + sub * 64) * (uint32_t)a.vs_t * 2u;
  };
  auto copy_one = [&](int c, int slot) {
    if (c < C::COPIES)
      copy16_to_lds(k_rs, lds0 + slot * C::TILE_BYTES + wave * 1024 + c * 4096, k_off, cp_k + c * k_step);
    else
      copy16_to_lds(v_rs, lds0 + (2 + slot) * C::TILE_BYTES + wave * 1024 + (c - C::COPIES) * 4096, v_off,
                    cp_v + (c - C::COPIES) * v_step);
  };

  // ---- operand read addresses (bytes inside a stage) -------------------------
  // K, A operand of S^T: lane (n, h) reads logical chunk 2 ks + h of rows n, 32 + n
  uint32_t k_rd[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++)
    k_rd[ks] = (uint32_t)(n * C::ROW_BYTES + (((2 * ks + h) ^ k_swz<D>(n)) << 4));
  // V, A operand of O^T (transposing read): lanes 16 g .. 16 g + 15 serve d
  // columns 16 (g & 1) .. + 15 of a d-tile and contraction half h = g >> 1; lane
  // s of the group points at key row 4 h + s / 4, d offset 16 (g & 1) + 4 (s % 4)
  // of d-tile t, which the row's swizzle moved to 64-byte group t ^ swz(row).
  const int s16 = lane & 15, a16 = (lane >> 4) & 1;
  uint32_t v_rd[D / 32];
#pragma unroll
  for (int t = 0; t < D / 32; t++)
    v_rd[t] = (uint32_t)((4 * h + (s16 >> 2)) * C::ROW_BYTES +
                         ((((4 * t) ^ v_swz<D>(s16 >> 2)) + 2 * a16 + ((s16 & 3) >> 1)) << 4) + ((s16 & 1) << 3));

  // ---- online-softmax state (base-2 logits) -------------------------------
  float m_run = -INFINITY, l_run = 0.f;
  constexpr int NDT = D / 32;
  f32x16 oacc[NDT];
#pragma unroll
  for (int dt = 0; dt < NDT; dt++)
#pragma unroll
    for (int j = 0; j < 16; j++) oacc[dt][j] = 0.f;

  float bias_row = 0.f;   // bias * log2e of this lane's row for the current chunk
  bool wave_on = false, diag = false;

  auto begin_chunk = [&](int u) {
    // decides participation and fetches the per-token bias of chunk u
    wave_on = wave_ok && ((__builtin_amdgcn_readfirstlane(wvmask[wave * 64 + (u >> 5)]) >> (u & 31)) & 1u);
    diag = a.causal && u == cw;
    if (!wave_on) return;
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
    bias_row = __shfl(bt, n / a.g_q);
  };

  // ---- one 64-key tile -------------------------------------------------------
  // S^T = K Q^T, online softmax, O^T += V^T P^T.  The source is written slot by
  // slot (one MFMA per slot, its operand reads a few slots ahead, a share of the
  // softmax VALU work behind it) in the order the instructions should issue, and
  // the scheduler may not move code across slots.  VALU budget: an MFMA 32x32x16
  // leaves about 24 issue cycles of its 32, an exponential takes 8 and a plain
  // VALU op 4.  P = LDS slot of the tile (compile time: every LDS offset is an
  // immediate).  MASKED adds the causal / sequence-end key mask (diagonal chunk
  // and ragged tail only).
  auto tile_math = [&](auto p_tag, auto m_tag, int kpos0, bool more) {
    constexpr int P = decltype(p_tag)::value;
    constexpr bool MASKED = decltype(m_tag)::value;
    constexpr int NS = D / 8;                                 // MFMAs per product and tile
    const char* kb = lds + P * C::TILE_BYTES;                  // K ring
    const char* vb = lds + (2 + P) * C::TILE_BYTES;            // V ring
    auto k_read = [&](int i) -> bf16x8 {   // slot i: d slice i / 2, key half i % 2
      return *reinterpret_cast<const bf16x8*>(kb + k_rd[i >> 1] + (i & 1) * 32 * C::ROW_BYTES);
    };
    auto v_read = [&](int i) -> bf16x8 {   // slot i: contraction step g = i / NDT, d-tile t = i % NDT
      const int g = i / NDT, t = i % NDT;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vb + v_rd[t] + (16 * g) * C::ROW_BYTES));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
          (__attribute__((address_space(3))) s16x4*)(vb + v_rd[t] + (16 * g + 8) * C::ROW_BYTES));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    };
    constexpr int KAHEAD = 4, VAHEAD = 2;
    f32x16 s[2];
    {
      bf16x8 kf[NS];
#pragma unroll
      for (int i = 0; i < KAHEAD; i++) kf[i] = k_read(i);
#pragma unroll
      for (int i = 0; i < NS; i++) {
        if (i + KAHEAD < NS) kf[i + KAHEAD] = k_read(i + KAHEAD);
        // the copies of the next tile are issued one at a time between the MFMAs: a
        // burst right after the barrier would queue all waves behind the 64 B/clk
        // global -> LDS path
        if ((i & 1) == 0 && (i >> 1) < 2 * C::COPIES) {
          if (more) copy_one(i >> 1, P ^ 1);
        }
        const int ks = i >> 1, kt = i & 1;
        if (ks == 0) {
          const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[ks], z, 0, 0, 0);
        } else {
          s[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[ks], s[kt], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    float mloc = -INFINITY;
    // MASKED: key kpos0 + 4 h + c (c = the compile-time part of the key index of
    // an accumulator register) is dead if it lies after the row's position in the
    // diagonal chunk or past the end of the sequence, i.e. if c > lim
    int lim = 0;
    if constexpr (MASKED) {
      const int k0 = kpos0 + 4 * h;
      lim = min(diag ? row_pos - k0 : 0x7fffffff, a.n_kv - 1 - k0);
      asm volatile("" : "+v"(lim));   // keep the per-register comparisons against immediates
    }
#pragma unroll
    for (int kt = 0; kt < 2; kt++)
#pragma unroll
      for (int j = 0; j < 16; j += 2) {
        if constexpr (MASKED) {
#pragma unroll
          for (int jj = j; jj < j + 2; jj++) {
            const int c = kt * 32 + (jj >> 2) * 8 + (jj & 3);
            s[kt][jj] = c > lim ? -INFINITY : s[kt][jj];
          }
        }
        mloc = fmaxf(fmaxf(mloc, s[kt][j]), s[kt][j + 1]);
      }
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    // max of the base-2 logits s*c1 + bias over the tile (c1 > 0)
    const float tmax = fmaf(mloc, a.c1, bias_row);
    // Lazy rescaling: the reference max m_run of a row is only raised when the
    // tile's max exceeds it by more than 2^kLazy; until then p = 2^(t - m_run)
    // may reach 2^kLazy, which fp32 / bf16 hold without loss, and the final
    // division by the row sum is unaffected.  Raising it is rare after the
    // first tiles, so the O rescale below is almost never executed.
    // The two outcomes rejoin only after the second product, so the accumulators
    // never have to be copied between registers on the common path.
    auto second_product = [&]() {
      const float off = bias_row - (m_run == -INFINITY ? 0.f : m_run);
      u32x4 pb[4];
      float lsum = 0.f;
      // exponential pair k: P^T slots 2 (k % 4), + 1 of contraction step g = k / 4
      auto e_pair = [&](int k) {
        const int g = k >> 2, kt = g >> 1, j = 8 * (g & 1) + 2 * (k & 3);
        const float p0 = __builtin_amdgcn_exp2f(fmaf(s[kt][j], a.c1, off));
        const float p1 = __builtin_amdgcn_exp2f(fmaf(s[kt][j + 1], a.c1, off));
        lsum += p0 + p1;
        asm volatile("" : "+v"(lsum));   // keeps the row-sum update in its slot
        const bf16x2 w = {(__bf16)p0, (__bf16)p1};
        pb[g][k & 3] = __builtin_bit_cast(uint32_t, w);
      };
      {
        bf16x8 vf[NS];
#pragma unroll
        for (int i = 0; i < VAHEAD; i++) vf[i] = v_read(i);
#pragma unroll
        for (int k = 0; k < 4; k++) e_pair(k);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int i = 0; i < NS; i++) {
          if (i + VAHEAD < NS) vf[i + VAHEAD] = v_read(i + VAHEAD);
          const int g = i / NDT, t = i % NDT;
          oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i], __builtin_bit_cast(bf16x8, pb[g]), oacc[t], 0, 0, 0);
          // the remaining 12 pairs go behind the first MFMAs: pairs of step g + 1
          // must be complete before slot NDT * (g + 1)
          constexpr int PPS = D == 128 ? 1 : 2;
#pragma unroll
          for (int kk = 0; kk < PPS; kk++)
            if (4 + i * PPS + kk < 16) e_pair(4 + i * PPS + kk);
          __builtin_amdgcn_sched_barrier(0);
        }
      }
      l_run += lsum;
    };
    if (__builtin_expect(__any(tmax > m_run + kLazy), 0)) {
      const float m_new = fmaxf(m_run, tmax);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m_run - m_use);   // m_run = -inf -> 0
      m_run = m_new;
      l_run *= corr;
#pragma unroll
      for (int dt = 0; dt < NDT; dt++)
#pragma unroll
        for (int j = 0; j < 16; j++) oacc[dt][j] *= corr;
      second_product();
    } else {
      second_product();
    }
  };

  // ---- main loop -----------------------------------------------------------
  // LDS: K ring [2] then V ring [2]; tile j lives in slot j & 1 of both.  At the
  // top of iteration j the wave waits for its own copies of tile j, the barrier
  // makes everybody's copies visible and guarantees that tile j - 1 (the other
  // slot) is no longer read; then the copies of tile j + 1 are issued between the
  // MFMAs of the first product of tile j and run during the rest of it.  The loop body is written out twice so that the
  // slot is a compile-time constant.
  bool have = advance();
  if (have) {
    copy_begin(it_u, it_sub);
#pragma unroll
    for (int c = 0; c < 2 * C::COPIES; c++) copy_one(c, 0);
  }
  auto iteration = [&](auto p_tag) {
    constexpr int P = decltype(p_tag)::value;
    const int cu = it_u, csub = it_sub;
    const bool more = advance();
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's copies of tile j have landed
    __syncthreads();
    if (csub == 0) begin_chunk(cu);
    if (more) copy_begin(it_u, it_sub);
    if (wave_on) {
      const int kpos0 = cu * a.block + csub * 64;
      if (diag || kpos0 + 64 > a.n_kv) tile_math(p_tag, std::true_type{}, kpos0, more);
      else tile_math(p_tag, std::false_type{}, kpos0, more);
    } else if (more) {
#pragma unroll
      for (int c = 0; c < 2 * C::COPIES; c++) copy_one(c, P ^ 1);
    }
    have = more;
  };
  while (have) {
    iteration(std::integral_constant<int, 0>{});
    if (!have) break;
    iteration(std::integral_constant<int, 1>{});
  }

  // ---- finalise ------------------------------------------------------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
  if (row_ok) {
    uint16_t* op = a.o + b * a.os_b + my_head * a.os_h + (int64_t)my_tok * a.os_t;
#pragma unroll
    for (int t = 0; t < NDT; t++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        // accumulator t, registers 4 q4 .. + 3: O^T rows 8 q4 + 4 h + i of d-tile t
        const int m0 = q4 * 8 + h * 4;
        uint2 w;
        w.x = pack_bf16x2(oacc[t][q4 * 4 + 0] * inv, oacc[t][q4 * 4 + 1] * inv);
        w.y = pack_bf16x2(oacc[t][q4 * 4 + 2] * inv, oacc[t][q4 * 4 + 3] * inv);
        *reinterpret_cast<uint2*>(op + t * 32 + m0) = w;
      }
  }
}

template <int D, bool DENSE>
static hipError_t launch_s2_t(const S2Args& a, hipStream_t st) {
  using C = S2Cfg<D>;
  auto kern = s2_attend_kernel<D, DENSE>;
  static LdsOptIn opt_in;
  if (hipError_t e = allow_dyn_lds((const void*)kern, C::LDS_BYTES, opt_in); e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.hb), dim3(256), C::LDS_BYTES, st, a);
  return hipGetLastError();
}

hipError_t launch_s2_mfma(const dash_params& p, const Layout& L, const void* q, const void* k,
                          const void* v, void* o, const uint32_t* mask, const float* bias,
                          bool dense, hipStream_t st) {
  S2Args a;
  fill_s2_args(a, p, L, q, k, v, o, mask, bias);
  const int tok_tile = 4 * (32 / L.g_q);
  a.n_tiles = (p.n_q + tok_tile - 1) / tok_tile;
  if (p.head_dim == 128) return dense ? launch_s2_t<128, true>(a, st) : launch_s2_t<128, false>(a, st);
  return dense ? launch_s2_t<64, true>(a, st) : launch_s2_t<64, false>(a, st);
}

}  // namespace dash
