// Backward pass of the prefill path (bf16 on the matrix cores; fp32 tensors on
// plain kernels at the end of the file): gradients of the block-sparse
// attention with the routing prior with respect to q, k and v, including the
// path through the bias into the Stage-1 entmax weights and from there into the
// block-mean summaries (end of Sec. 3.3: the output is differentiable in q, k, v
// and the prior, so the gradient reaches Stage 1 and Stage 0; Sec. 3.5: the
// backward pass reuses the forward's chunk mask because the entmax Jacobian is
// zero outside the support).
//
// With P = softmax(z + d) over the attended tokens (z = q.k scale, d the bias
// of the token's chunk, 0 on the local chunks), o = P V and upstream dO:
//   dP = V dO,  D = <P, dP> (= <dO, o>),  dz = P (dP - D)
//   dq = scale K^T dz,  dK = scale dz q^T,  dV = P dO^T
//   dd_c = sum over the group's heads and the chunk's tokens of dz
//   dlnw_c = (dd_c - mean_R dd) / sigma,  dw_c = dlnw_c / w_c,  dw_hat = dw / g_q
//   dx_{h,c} = g_{h,c} (dw_hat_c - sum_j g_{h,j} dw_hat_j / sum_j g_{h,j}),
//       g_{h,c} = p u^(p-1) on the head's support, u = x - tau, p = 1/(alpha-1)
//   dq_h += c sum_c dx_{h,c} kbar_c,  dkbar_c = c sum_{rows} dx q,  c = gamma (alpha-1) scale
//   dK_j += dkbar_c / B for the keys of a complete chunk c (block mean).
//
// Kernels:
//   bwd_q_kernel   owns 128 (token, head) rows like the forward kernel and walks the
//                  union of their chunks; launched twice: <GRAD = false> for the row
//                  log-sum-exp and D, <GRAD = true> for dq (attention part, fp32), dd
//                  and a dense copy of the bias; the latter also marks, per chunk,
//                  which row tiles attend it.
//   bwd_route_kernel  one wave per (kv-head, token): prior and entmax Jacobian,
//                  dx per head and chunk, the routing part of dq, final dq.
//   bwd_kv_kernel  owns a 64-key tile, walks the row tiles that attend its chunk and
//                  accumulates dK, dV and the chunk's dkbar without atomics.
//   bwd_f32_*      the same chain for fp32 tensors on the VALU (row kernel with atomics,
//                  the routing kernel above, a per-chunk dkbar kernel).
// MFMA operand layouts are those of the forward kernel: every product is
// arranged so that the accumulator of the first product is directly the
// B operand of the second; the transposed operand comes from LDS through the
// transposing read.
#include <math.h>
#include <stdlib.h>

#include "common.h"
#include "dash_internal.h"
#include "lds_copy.h"

namespace dash {

struct BwdArgs {
  const uint16_t *q, *k, *v, *d_o;
  uint16_t *dq, *dk, *dv;
  const float* kbar; const uint32_t* mask; const float* bias; const float* tau;
  float *lse, *dsum;       // [batch, h_q, n_q]: base-2 log-sum-exp of the logits, <dO, o>
  float *biasd, *dbd;      // [batch, h_kv, n_q, t_all]: bias and its gradient by chunk id
  float* dxd;              // [batch, h_q, n_q, t_all]: entmax-score gradient by chunk id
  float* dq32;             // [batch, h_q, n_q, D]: attention part of dq
  uint32_t* colmask;       // [batch*h_kv, t_all, cwords]: bit T set iff row tile T attends the chunk
  float* dkbar_out;        // optional [batch, h_kv, t_c, D]: gradient of the summaries (then not folded into dk)
  int h_q, h_kv, g_q, n_q, n_kv, block, t_c, t_all, words, causal, window, n_tiles, hb, cwords;
  int64_t qs_b, qs_h, qs_t, ks_b, ks_h, ks_t, vs_b, vs_h, vs_t, os_b, os_h, os_t;
  float c1, scale, xscale, pexp, sigma;
};

template <int D> struct BCfg {
  static constexpr int NCH = D / 8;
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int TILE_BYTES = 64 * ROW_BYTES;
  static constexpr int COPIES = TILE_BYTES / 16 / 256;
  static constexpr int ROWS_PER_COPY = 256 / NCH;
  static constexpr int NDT = D / 32;
  static constexpr int NS = D / 8;
};

// Chunk permutation of a 64-row tile (position of logical 16-byte chunk c of row
// `row` is c ^ swz(row)), chosen so that both kinds of operand reads are free of
// bank conflicts: the A-operand read has 16 lanes on 16 consecutive rows at one
// logical chunk (they must land in 16 different slots of a 256-byte bank window),
// the transposing read has 16 lanes on 4 consecutive rows x 2 consecutive chunks
// (rows r..r+3 must land in different 64-byte groups).
template <int D> __device__ __forceinline__ int swz(int row) {
  return D == 128 ? (((row & 3) << 2) | ((row >> 2) & 3)) : ((((row >> 1) & 1) << 2) | ((row >> 2) & 3));
}
// byte offset of element (row, d0) of a tile, d0 a multiple of 4
template <int D> __device__ __forceinline__ uint32_t tile_off(int row, int d0) {
  return (uint32_t)(row * BCfg<D>::ROW_BYTES + (((d0 >> 3) ^ swz<D>(row)) << 4) + ((d0 & 7) << 1));
}

// Operand addresses.  Because the chunk permutation is an XOR, the offsets of the
// d slices of one row differ from the first one by an XOR with a constant, so a
// lane keeps one base offset per kind of read instead of one register per slice.
// A operand slice `i` (d slice ks = i / 2, 32-row half i % 2) of a row-major tile;
// base = tile_off(row, 8 h): the slice starts at d = 16 ks + 8 h, chunk 2 ks + h
template <int D> __device__ __forceinline__ bf16x8 read_a(const char* tile, uint32_t base, int i) {
  return *reinterpret_cast<const bf16x8*>(tile + (base ^ (uint32_t)((i >> 1) << 5)) + (i & 1) * 32 * BCfg<D>::ROW_BYTES);
}
// transposed A operand: contraction step g (16 tile rows), d-tile t; lo / hi address the
// two 8-row halves of step 0 at d-tile 0 (d-tile t starts 4 t chunks further)
template <int D> __device__ __forceinline__ bf16x8 read_t(const char* tile, uint32_t lo, uint32_t hi, int g, int t) {
  return lds_read_tr_pair(tile + (lo ^ (uint32_t)(t << 6)) + (16 * g) * BCfg<D>::ROW_BYTES,
                          tile + (hi ^ (uint32_t)(t << 6)) + (16 * g) * BCfg<D>::ROW_BYTES);
}

// two fp32 -> packed bf16 (round to nearest even) with the hardware conversion
__device__ __forceinline__ uint32_t cvt_bf16x2(float lo, float hi) {
  const bf16x2 w = {(__bf16)lo, (__bf16)hi};
  return __builtin_bit_cast(uint32_t, w);
}

__device__ __forceinline__ f32x16 zero16() {
  const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  return z;
}

__global__ void bwd_fill_zero_kernel(uint32_t* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    p[i] = 0u;
}

// ---------------------------------------------------------------------------
// Row-owner kernel.
// ---------------------------------------------------------------------------
// GRAD = false: the first walk (row log-sum-exp and D into the workspace; few registers, dO
// fragments in registers, three workgroups per CU).  GRAD = true: the second walk (dq, bias
// gradient, column masks; dO rows as an LDS operand, two workgroups per CU).
template <int D, bool GRAD>
__global__ __launch_bounds__(256, GRAD ? 2 : 3) void bwd_q_kernel(BwdArgs a) {
  using C = BCfg<D>;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* k_t = lds;                            // K tile
  char* v_t = lds + C::TILE_BYTES;            // V tile
  char* do_t = lds + 2 * C::TILE_BYTES;       // GRAD: dO rows of the workgroup's 128 rows (stationary)
  uint32_t* wgmask = reinterpret_cast<uint32_t*>(lds + (GRAD ? 4 : 2) * C::TILE_BYTES);   // [64]
  uint32_t* wvmask = wgmask + 64;                                            // [4][64]

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int hbi = blockIdx.x % a.hb;
  const int tile = a.n_tiles - 1 - blockIdx.x / a.hb;
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int tokw = 32 / a.g_q;
  const int tok_w0 = tile * 4 * tokw + wave * tokw;
  const int nsub = a.block >> 6;

  const int my_tok = tok_w0 + n / a.g_q;
  const int my_head = r * a.g_q + n % a.g_q;
  const bool row_ok = my_tok < a.n_q;
  const int row_tok = row_ok ? my_tok : a.n_q - 1;
  const int row_pos = row_tok;                                   // n_q == n_kv
  const int cw = (tok_w0 < a.n_q ? tok_w0 : a.n_q - 1) / a.block;
  const bool wave_ok = tok_w0 < a.n_q;

  // ---- row fragments as B operands: q in registers; dO in registers (first walk) or in LDS
  // (second walk, each wave its own 32 rows)
  bf16x8 qf[D / 16], dof[GRAD ? 1 : D / 16];
  {
    const uint16_t* qp = a.q + b * a.qs_b + my_head * a.qs_h + (int64_t)row_tok * a.qs_t + h * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
  }
  if constexpr (!GRAD) {
    const uint16_t* dop = a.d_o + b * a.os_b + my_head * a.os_h + (int64_t)row_tok * a.os_t + h * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) dof[ks] = *reinterpret_cast<const bf16x8*>(dop + ks * 16);
  } else {
    const u32x4 o_rs = make_rsrc(a.d_o + b * a.os_b + (int64_t)r * a.g_q * a.os_h,
                                 ((int64_t)(a.g_q - 1) * a.os_h + ((int64_t)a.n_q - 1) * a.os_t + D) * 2);
    constexpr int RPI = 64 / C::NCH;             // rows one copy instruction covers
#pragma unroll
    for (int i = 0; i < 32 / RPI; i++) {
      const int rw = i * RPI + lane / C::NCH;    // row of this wave
      const int tk = min(tok_w0 + rw / a.g_q, a.n_q - 1);
      const uint32_t voff = (uint32_t)((tk * (int)a.os_t + (rw % a.g_q) * (int)a.os_h) * 2) +
                            (uint32_t)(((lane % C::NCH) ^ swz<D>(wave * 32 + rw)) << 4);
      copy16_to_lds(o_rs, lds_addr_of(do_t) + (wave * 32 + i * RPI) * C::ROW_BYTES, voff, 0u);
    }
  }
  const uint32_t do_rd = tile_off<D>(wave * 32 + n, 8 * h);

  // ---- chunk bitmaps ---------------------------------------------------------
  const int trk_tok = tok_w0 + lane;
  const bool trk_ok = lane < tokw && trk_tok < a.n_q;
  const int64_t trk_base = ((int64_t)b * a.h_kv + r) * a.n_q + (trk_ok ? trk_tok : 0);
  const uint32_t* trk_mask = a.mask + trk_base * a.words;
  const float* trk_bias = a.bias + trk_base * a.t_all;
  int trk_rank = 0, trk_wi = -1;
  uint32_t trk_word = 0;
  bool trk_has = false;

  for (int i = tid; i < 5 * 64; i += 256) wgmask[i] = 0u;
  __syncthreads();
  if (wave_ok)
    for (int wi = lane; wi < a.words; wi += 64) {
      uint32_t m = 0u;
      for (int t = 0; t < tokw; t++)
        if (tok_w0 + t < a.n_q)
          m |= a.mask[(((int64_t)b * a.h_kv + r) * a.n_q + tok_w0 + t) * a.words + wi];
      wvmask[wave * 64 + wi] = m;
      if (m) atomicOr(&wgmask[wi], m);
    }
  __syncthreads();
  // tell the key-owner kernel which chunks this row tile attends
  if constexpr (GRAD)
  for (int wi = tid; wi < a.words; wi += 256) {
    uint32_t m = wgmask[wi];
    while (m) {
      const int c = wi * 32 + __builtin_ctz(m);
      m &= m - 1u;
      if (c < a.t_all)
        atomicOr(&a.colmask[((int64_t)hbi * a.t_all + c) * a.cwords + (tile >> 5)], 1u << (tile & 31));
    }
  }

  // ---- tile iterator ---------------------------------------------------------
  int it_wi = -1, it_sub = nsub - 1, it_u = -1;
  uint32_t it_bits = 0u;
  auto advance = [&]() -> bool {
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

  // ---- tile copies -------------------------------------------------------------
  const u32x4 k_rs = make_rsrc(a.k + b * a.ks_b + r * a.ks_h, (((int64_t)a.n_kv - 1) * a.ks_t + D) * 2);
  const u32x4 v_rs = make_rsrc(a.v + b * a.vs_b + r * a.vs_h, (((int64_t)a.n_kv - 1) * a.vs_t + D) * 2);
  const uint32_t lds0 = lds_addr_of(lds);
  const int c_row = (wave * 64 + lane) / C::NCH, c_pos = lane % C::NCH;
  const uint32_t k_off = (uint32_t)(c_row * (int)a.ks_t * 2 + ((c_pos ^ swz<D>(c_row)) << 4));
  const uint32_t v_off = (uint32_t)(c_row * (int)a.vs_t * 2 + ((c_pos ^ swz<D>(c_row)) << 4));
  const uint32_t k_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.ks_t * 2);
  const uint32_t v_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.vs_t * 2);

  // ---- operand read offsets ------------------------------------------------------
  // A operand: lane (n, h) reads logical chunk 2 ks + h of rows n, 32 + n.
  // Transposing read: lanes 16 g' .. 16 g' + 15 serve d columns 16 (g' & 1) .. + 15
  // of a d-tile and contraction half h = g' >> 1; lane s of the group points at
  // tile row 4 h + s / 4 (+ 8 for the second read), d offset 16 (g' & 1) + 4 (s % 4).
  const uint32_t a_rd = tile_off<D>(n, 8 * h);
  const int s16 = lane & 15, a16 = (lane >> 4) & 1;
  const uint32_t t_lo = tile_off<D>(4 * h + (s16 >> 2), 16 * a16 + 4 * (s16 & 3));
  const uint32_t t_hi = tile_off<D>(8 + 4 * h + (s16 >> 2), 16 * a16 + 4 * (s16 & 3));

  // first walk (GRAD = false): running max, sum of exponentials and sum of exponentials
  // times dP; D = <P, dP> = <dO, o> is taken from the latter two in fp32 (the stored bf16
  // output would put its rounding error into every dz of the row).  Second walk: both
  // come from the workspace.
  float m_run = -INFINITY, l_run = 0.f, dn_run = 0.f, lse2 = 0.f, dsum = 0.f;
  f32x16 dqacc[GRAD ? C::NDT : 1];
#pragma unroll
  for (int t = 0; t < (GRAD ? C::NDT : 1); t++) dqacc[t] = zero16();
  float db_acc = 0.f;
  if constexpr (GRAD) {
    const int64_t row = ((int64_t)b * a.h_q + my_head) * a.n_q + row_tok;
    lse2 = a.lse[row];
    dsum = a.dsum[row];
  }

  {
    constexpr bool grad = GRAD;
    float trk_next = (trk_ok && a.t_all > 0) ? trk_bias[0] : 0.f;
    float bias_row = 0.f;
    bool wave_on = false, diag = false;
    while (advance()) {
      const int cu = it_u, csub = it_sub;
      const uint32_t soff_k = (uint32_t)(cu * a.block + csub * 64) * (uint32_t)a.ks_t * 2u;
      const uint32_t soff_v = (uint32_t)(cu * a.block + csub * 64) * (uint32_t)a.vs_t * 2u;
      __syncthreads();                      // the previous tile is no longer read
#pragma unroll
      for (int c = 0; c < C::COPIES; c++) {
        copy16_to_lds(k_rs, lds0 + wave * 1024 + c * 4096, k_off, soff_k + c * k_step);
        copy16_to_lds(v_rs, lds0 + C::TILE_BYTES + wave * 1024 + c * 4096, v_off, soff_v + c * v_step);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();

      if (csub == 0) {
        wave_on = wave_ok && ((__builtin_amdgcn_readfirstlane(wvmask[wave * 64 + (cu >> 5)]) >> (cu & 31)) & 1u);
        diag = a.causal && cu == cw;
        if (wave_on) {
          float bt = 0.f;
          trk_has = false;
          if (!diag) {
            bt = -INFINITY;
            if (trk_ok) {
              if ((cu >> 5) != trk_wi) { trk_wi = cu >> 5; trk_word = trk_mask[trk_wi]; }
              if ((trk_word >> (cu & 31)) & 1u) {
                trk_has = true;
                bt = trk_next * kLog2e;
                if (grad) a.biasd[trk_base * a.t_all + cu] = trk_next;
                trk_rank++;
                if (trk_rank < a.t_all) trk_next = trk_bias[trk_rank];
              }
            }
          }
          bias_row = __shfl(bt, n / a.g_q);
        }
      }
      if (!wave_on) continue;
      const int kpos0 = cu * a.block + csub * 64;

      // the tile in two halves of 32 keys (keeps one S^T and one dP^T accumulator live)
      u32x4 pb[4];
      float dssum = 0.f;
      const float off = bias_row - lse2;
#pragma unroll
      for (int kt = 0; kt < 2; kt++) {
        // S^T = K Q^T, dP^T = V dO^T
        f32x16 s = zero16(), dp = zero16();
#pragma unroll
        for (int ks = 0; ks < D / 16; ks++) {
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_a<D>(k_t, a_rd, 2 * ks + kt), qf[ks], s, 0, 0, 0);
          if constexpr (GRAD)
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_a<D>(v_t, a_rd, 2 * ks + kt),
                                                         read_a<D>(do_t, do_rd, 2 * ks), dp, 0, 0, 0);
          else
            dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_a<D>(v_t, a_rd, 2 * ks + kt), dof[ks], dp, 0, 0, 0);
        }
        // key mask: causal inside the diagonal chunk, and the end of the sequence
        if (diag || kpos0 + 64 > a.n_kv) {
          const int k0 = kpos0 + 32 * kt + 4 * h;
          const int lim = min(diag ? row_pos - k0 : 0x7fffffff, a.n_kv - 1 - k0);
#pragma unroll
          for (int j = 0; j < 16; j++) {
            const int c = (j >> 2) * 8 + (j & 3);
            s[j] = c > lim ? -INFINITY : s[j];
          }
        }
        if (!grad) {
          float mloc = -INFINITY;
#pragma unroll
          for (int j = 0; j < 16; j++) mloc = fmaxf(mloc, s[j]);
          mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
          const float tmax = fmaf(mloc, a.c1, bias_row);
          const float m_new = fmaxf(m_run, tmax);
          const float m_use = m_new == -INFINITY ? 0.f : m_new;
          float lsum = 0.f, dnsum = 0.f;
#pragma unroll
          for (int j = 0; j < 16; j++) {
            const float e = __builtin_amdgcn_exp2f(fmaf(s[j], a.c1, bias_row - m_use));
            lsum += e;
            dnsum = fmaf(e, dp[j], dnsum);
          }
          const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
          l_run = l_run * corr + lsum;
          dn_run = dn_run * corr + dnsum;
          m_run = m_new;
        } else {
          // dS^T = P^T (dP^T - D), packed as the B operand of the second product
#pragma unroll
          for (int k = 0; k < 8; k++) {
            const int g = 2 * kt + (k >> 2), j = 8 * (k >> 2) + 2 * (k & 3);
            const float p0 = __builtin_amdgcn_exp2f(fmaf(s[j], a.c1, off));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(s[j + 1], a.c1, off));
            const float d0 = p0 * (dp[j] - dsum);
            const float d1 = p1 * (dp[j + 1] - dsum);
            dssum += d0 + d1;
            pb[g][k & 3] = cvt_bf16x2(d0, d1);
          }
        }
      }
      if constexpr (GRAD) {
      db_acc += dssum;
      // dQ^T += K^T dS^T
#pragma unroll
      for (int i = 0; i < C::NS; i++) {
        const int g = i / C::NDT, t = i % C::NDT;
        dqacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t<D>(k_t, t_lo, t_hi, g, t),
                                                           __builtin_bit_cast(bf16x8, pb[g]), dqacc[t], 0, 0, 0);
      }
      if (csub == nsub - 1) {
        // bias gradient of chunk cu: sum over the keys (both lane halves) and the
        // token's heads (adjacent lanes), written by the lane that tracks the token
        float tot = db_acc + __shfl_xor(db_acc, 32);
        for (int o = 1; o < a.g_q; o <<= 1) tot += __shfl_xor(tot, o);
        const float mine = __shfl(tot, (lane * a.g_q) & 31);
        if (!diag && trk_ok && trk_has) a.dbd[trk_base * a.t_all + cu] = mine;
        db_acc = 0.f;
      }
      }
    }
    if constexpr (!GRAD) {
      const float l_tot = l_run + __shfl_xor(l_run, 32);
      const float dn_tot = dn_run + __shfl_xor(dn_run, 32);
      lse2 = (m_run == -INFINITY ? 0.f : m_run) + __builtin_amdgcn_logf(l_tot);   // v_log_f32: log2
      dsum = l_tot > 0.f ? dn_tot / l_tot : 0.f;
    }
  }

  // ---- outputs -----------------------------------------------------------------
  if (row_ok) {
    const int64_t row = ((int64_t)b * a.h_q + my_head) * a.n_q + my_tok;
    if constexpr (!GRAD) {
      if (h == 0) { a.lse[row] = lse2; a.dsum[row] = dsum; }
    }
    float* dq = a.dq32 + row * D;
    if constexpr (GRAD)
#pragma unroll
    for (int t = 0; t < C::NDT; t++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const int m0 = q4 * 8 + h * 4;
        float4 w;
        w.x = dqacc[t][q4 * 4 + 0] * a.scale; w.y = dqacc[t][q4 * 4 + 1] * a.scale;
        w.z = dqacc[t][q4 * 4 + 2] * a.scale; w.w = dqacc[t][q4 * 4 + 3] * a.scale;
        *reinterpret_cast<float4*>(dq + t * 32 + m0) = w;
      }
  }
}

// ---------------------------------------------------------------------------
// Routing backward: one wave per (batch, kv-head, token).
// ---------------------------------------------------------------------------
// u^p and p u^(p-1) for u > 0
__device__ __forceinline__ void pow_and_slope(float u, float p, float& w, float& g) {
  if (p == 2.f) { w = u * u; g = 2.f * u; }
  else if (p == 1.f) { w = u; g = 1.f; }
  else { w = __builtin_amdgcn_exp2f(p * __builtin_amdgcn_logf(u)); g = p * w / u; }
}

template <int D, int G, typename T>
__global__ __launch_bounds__(64) void bwd_route_kernel(BwdArgs a) {
  constexpr int SEG = 64;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  float* qs = reinterpret_cast<float*>(lds);                 // [G][D]
  int* cidx = reinterpret_cast<int*>(qs + G * D);            // [t_c]
  float* dwl = reinterpret_cast<float*>(cidx + a.t_c);       // [t_c]
  float* dxs = dwl + a.t_c;                                  // [G][SEG]

  const int lane = threadIdx.x;
  const int tok = blockIdx.x % a.n_q;
  const int hbi = blockIdx.x / a.n_q;
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int n_cand = a.causal ? max(tok / a.block - a.window, 0) : a.t_c;
  const int64_t trow = ((int64_t)b * a.h_kv + r) * a.n_q + tok;
  const uint32_t* mrow = a.mask + trow * a.words;
  const float* dbrow = a.dbd + trow * a.t_all;
  const float* kb = a.kbar + ((int64_t)b * a.h_kv + r) * a.t_c * D;

  for (int i = lane; i < G * D; i += 64) {
    const int hh = i / D, d = i % D;
    qs[i] = elem<T>::ld(reinterpret_cast<const T*>(a.q) + b * a.qs_b + (r * G + hh) * a.qs_h + (int64_t)tok * a.qs_t + d);
  }
  // routed candidates, ascending
  int n_r = 0;
  for (int base = 0; base < n_cand; base += 64) {
    const int c = base + lane;
    const bool bit = c < n_cand && ((mrow[c >> 5] >> (c & 31)) & 1u);
    const uint64_t bal = __ballot(bit);
    if (bit) cidx[n_r + __popcll(bal & ((1ull << lane) - 1ull))] = c;
    n_r += __popcll(bal);
  }
  __syncthreads();

  float acc_q[G][2];            // routing part of dq: this lane's d pair (D = 128) or single d (D = 64)
#pragma unroll
  for (int hh = 0; hh < G; hh++) acc_q[hh][0] = acc_q[hh][1] = 0.f;

  if (n_r > 0) {
    float tauh[G];
#pragma unroll
    for (int hh = 0; hh < G; hh++) tauh[hh] = a.tau[((int64_t)b * a.h_q + r * G + hh) * a.n_q + tok];
    float dsum = 0.f;
    for (int e = lane; e < n_r; e += 64) dsum += dbrow[cidx[e]];
    const float dmean = wave_sum(dsum) / (float)n_r;

    // sweep A: scores, weights, slopes; S0 = sum g, S1 = sum g dw_hat per head.
    // Eight lanes share a routed chunk (lane = 8 cs + dp): lane dp reads the dp-th
    // eighth of the summary row, so a wave instruction covers 8 whole rows, and the
    // partial dot products are combined over the 8 lanes by DPP.  Every lane of the
    // group then holds all scores; lane dp keeps the per-head results of the heads
    // hh = dp (mod 8) (slopes to memory, their sums in registers).
    constexpr int DP = D / 8;                      // d range of one lane
    // With few heads the routing part of dq is accumulated in the same sweep:
    // sum_c dx_c kbar_c = sum_c (g_c dw_hat_c) kbar_c - ratio sum_c g_c kbar_c, two sums whose
    // weights are known chunk by chunk, so the summary rows are read once.
    constexpr bool FUSE = 2 * G * DP <= 64;
    const int cs = lane >> 3, dp = lane & 7;
    float s0[G], s1[G];
#pragma unroll
    for (int hh = 0; hh < G; hh++) s0[hh] = s1[hh] = 0.f;
    float a1[FUSE ? G : 1][DP], a2[FUSE ? G : 1][DP];
    if constexpr (FUSE) {
#pragma unroll
      for (int hh = 0; hh < G; hh++)
#pragma unroll
        for (int j = 0; j < DP; j++) a1[hh][j] = a2[hh][j] = 0.f;
    }
    for (int e0 = 0; e0 < n_r; e0 += 8) {
      const int e = e0 + cs;
      const bool live = e < n_r;
      const int c = cidx[live ? e : n_r - 1];
      const float4* krow = reinterpret_cast<const float4*>(kb + (int64_t)c * D + dp * DP);
      float x[G];
#pragma unroll
      for (int hh = 0; hh < G; hh++) x[hh] = 0.f;
      float kvr[DP];
#pragma unroll
      for (int d4 = 0; d4 < DP / 4; d4++) {
        const float4 kv = krow[d4];
        kvr[4 * d4] = kv.x; kvr[4 * d4 + 1] = kv.y; kvr[4 * d4 + 2] = kv.z; kvr[4 * d4 + 3] = kv.w;
#pragma unroll
        for (int hh = 0; hh < G; hh++) {
          const float4 qv = *reinterpret_cast<const float4*>(qs + hh * D + dp * DP + d4 * 4);
          x[hh] = fmaf(qv.x, kv.x, fmaf(qv.y, kv.y, fmaf(qv.z, kv.z, fmaf(qv.w, kv.w, x[hh]))));
        }
      }
      float gd[G], wsum = 0.f;
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        float xs = x[hh];
        asm volatile("" : "+v"(xs));
        xs += dpp_f<0xB1>(xs);     // lane ^ 1
        xs += dpp_f<0x4E>(xs);     // lane ^ 2
        xs += dpp_f<0x141>(xs);    // the other quad of the 8 lanes
        const float u = xs * a.xscale - tauh[hh];
        float wv = 0.f;
        gd[hh] = 0.f;
        if (u > 0.f) pow_and_slope(u, a.pexp, wv, gd[hh]);
        wsum += wv;
      }
      // dw_hat = dlnw / w / g_q with w = wsum / g_q
      const float dwh = wsum > 0.f ? (dbrow[c] - dmean) / (a.sigma * wsum) : 0.f;
      if (live) {
        if (dp == 0) dwl[e] = dwh;
#pragma unroll
        for (int hh = 0; hh < G; hh++)
          if ((hh & 7) == dp) {
            s0[hh] += gd[hh];
            s1[hh] += gd[hh] * dwh;
            a.dxd[(((int64_t)b * a.h_q + r * G + hh) * a.n_q + tok) * a.t_all + c] = gd[hh];
          }
        if constexpr (FUSE) {
#pragma unroll
          for (int hh = 0; hh < G; hh++) {
            const float w1 = gd[hh] * dwh, w2 = gd[hh];
#pragma unroll
            for (int j = 0; j < DP; j++) {
              a1[hh][j] = fmaf(w1, kvr[j], a1[hh][j]);
              a2[hh][j] = fmaf(w2, kvr[j], a2[hh][j]);
            }
          }
        }
      }
    }
    float ratio[G];
#pragma unroll
    for (int hh = 0; hh < G; hh++) {
      const float t0 = wave_sum(s0[hh]), t1 = wave_sum(s1[hh]);
      ratio[hh] = t0 > 0.f ? t1 / t0 : 0.f;
    }
    if constexpr (FUSE) {
      // dx for the key-owner kernel (each lane turns the slopes it wrote itself into dx)
      for (int e0 = 0; e0 < n_r; e0 += 8) {
        const int e = e0 + cs;
        if (e < n_r) {
          const int c = cidx[e];
          const float dwh = dwl[e];
#pragma unroll
          for (int hh = 0; hh < G; hh++)
            if ((hh & 7) == dp) {
              float* px = a.dxd + (((int64_t)b * a.h_q + r * G + hh) * a.n_q + tok) * a.t_all + c;
              *px = *px * (dwh - ratio[hh]);
            }
        }
      }
      // routing part of dq: combine the two sums, add up the 8 chunk slots (lanes that differ
      // in cs), and hand lane (cs, dp) the d = dp DP + cs DP/8 .. of its output pair
#pragma unroll
      for (int hh = 0; hh < G; hh++) {
        float v0 = 0.f, v1 = 0.f;
#pragma unroll
        for (int j = 0; j < DP; j++) {
          float t = a1[hh][j] - ratio[hh] * a2[hh][j];
          t += __shfl_xor(t, 8);
          t += __shfl_xor(t, 16);
          t += __shfl_xor(t, 32);
          if (D == 128) {
            if ((j >> 1) == cs) { if (j & 1) v1 = t; else v0 = t; }
          } else {
            if (j == cs) v0 = t;
          }
        }
        acc_q[hh][0] = v0;
        acc_q[hh][1] = v1;
      }
    } else
    // sweep B, one segment of SEG routed chunks at a time: dx (each lane turns the slopes
    // it wrote itself into dx), then dq += dx kbar with the lanes over d
    for (int e0 = 0; e0 < n_r; e0 += SEG) {
      __syncthreads();
#pragma unroll
      for (int it = 0; it < SEG / 8; it++) {
        const int j = it * 8 + cs, e = e0 + j;
        if (e < n_r) {
          const int c = cidx[e];
          const float dwh = dwl[e];
#pragma unroll
          for (int hh = 0; hh < G; hh++)
            if ((hh & 7) == dp) {
              float* px = a.dxd + (((int64_t)b * a.h_q + r * G + hh) * a.n_q + tok) * a.t_all + c;
              const float dx = *px * (dwh - ratio[hh]);
              *px = dx;
              dxs[hh * SEG + j] = dx;
            }
        }
      }
      __syncthreads();
      const int cnt = min(SEG, n_r - e0);
      for (int j = 0; j < cnt; j++) {
        const int c = cidx[e0 + j];
        float k0, k1 = 0.f;
        if (D == 128) {
          const float2 kv = *reinterpret_cast<const float2*>(kb + (int64_t)c * D + 2 * lane);
          k0 = kv.x; k1 = kv.y;
        } else {
          k0 = kb[(int64_t)c * D + lane];
        }
#pragma unroll
        for (int hh = 0; hh < G; hh++) {
          const float dx = dxs[hh * SEG + j];
          acc_q[hh][0] = fmaf(dx, k0, acc_q[hh][0]);
          acc_q[hh][1] = fmaf(dx, k1, acc_q[hh][1]);
        }
      }
    }
  }
  // final dq = attention part + routing part; a lane owns the d pair 2 lane .. (D = 128) or the
  // single d = lane (D = 64) in the two-sweep variant, d = 16 dp + 2 cs .. or 8 dp + cs in the fused one
  constexpr bool FUSED = 2 * G * (D / 8) <= 64;
  const int d_own = FUSED ? (D == 128 ? 16 * (lane & 7) + 2 * (lane >> 3) : 8 * (lane & 7) + (lane >> 3))
                          : (D == 128 ? 2 * lane : lane);
#pragma unroll
  for (int hh = 0; hh < G; hh++) {
    const int64_t row = ((int64_t)b * a.h_q + r * G + hh) * a.n_q + tok;
    T* out = reinterpret_cast<T*>(a.dq) + b * a.qs_b + (r * G + hh) * a.qs_h + (int64_t)tok * a.qs_t;
    if (D == 128) {
      const float2 base = *reinterpret_cast<const float2*>(a.dq32 + row * D + d_own);
      const float v0 = fmaf(a.xscale, acc_q[hh][0], base.x), v1 = fmaf(a.xscale, acc_q[hh][1], base.y);
      if constexpr (sizeof(T) == 2) *reinterpret_cast<uint32_t*>(out + d_own) = cvt_bf16x2(v0, v1);
      else *reinterpret_cast<float2*>(out + d_own) = make_float2(v0, v1);
    } else {
      elem<T>::st(out + d_own, fmaf(a.xscale, acc_q[hh][0], a.dq32[row * D + d_own]));
    }
  }
}

// ---------------------------------------------------------------------------
// Key-owner kernel: one 64-key tile per workgroup.
// ---------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256, 2) void bwd_kv_kernel(BwdArgs a) {
  using C = BCfg<D>;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  char* k_t = lds;                             // this workgroup's 64 keys (stationary)
  char* v_t = lds + C::TILE_BYTES;             // and values
  char* q_t = lds + 2 * C::TILE_BYTES;         // 64 query rows of the current step
  char* d_t = lds + 3 * C::TILE_BYTES;         // and their dO rows
  float* cmb_s = reinterpret_cast<float*>(lds + 4 * C::TILE_BYTES);   // [64] per-row scalars
  float* dsum_s = cmb_s + 64;
  float* dx_s = dsum_s + 64;
  int* pos_s = reinterpret_cast<int*>(dx_s + 64);
  float* redf = reinterpret_cast<float*>(pos_s + 64);                 // [D] dkbar of the chunk
  float* red = redf + D;                                              // [RG][D] dkbar partials
  constexpr int RG = 256 / C::NCH, RPG = 64 / RG;   // dkbar: row groups per workgroup, rows per group

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int kh = wave & 1, rh = wave >> 1;
  const int hbi = blockIdx.x % a.hb;
  const int ktile = blockIdx.x / a.hb;          // early key tiles (the most rows) first
  const int r = hbi % a.h_kv, b = hbi / a.h_kv;
  const int kpos0 = ktile * 64;
  const int c = kpos0 / a.block;
  const int tok_step = 64 / a.g_q;              // tokens per 64-row step
  const int my_key = kpos0 + kh * 32 + n;

  const u32x4 k_rs = make_rsrc(a.k + b * a.ks_b + r * a.ks_h, (((int64_t)a.n_kv - 1) * a.ks_t + D) * 2);
  const u32x4 v_rs = make_rsrc(a.v + b * a.vs_b + r * a.vs_h, (((int64_t)a.n_kv - 1) * a.vs_t + D) * 2);
  const u32x4 q_rs = make_rsrc(a.q + b * a.qs_b + (int64_t)r * a.g_q * a.qs_h,
                               ((int64_t)(a.g_q - 1) * a.qs_h + ((int64_t)a.n_q - 1) * a.qs_t + D) * 2);
  const u32x4 o_rs = make_rsrc(a.d_o + b * a.os_b + (int64_t)r * a.g_q * a.os_h,
                               ((int64_t)(a.g_q - 1) * a.os_h + ((int64_t)a.n_q - 1) * a.os_t + D) * 2);
  const uint32_t lds0 = lds_addr_of(lds);
  const int c_row = (wave * 64 + lane) / C::NCH, c_pos = lane % C::NCH;
  const uint32_t c_chunk = (uint32_t)((c_pos ^ swz<D>(c_row)) << 4);
  const int c_tok = c_row / a.g_q, c_head = c_row % a.g_q;
  const uint32_t q_off = (uint32_t)((c_tok * (int)a.qs_t + c_head * (int)a.qs_h) * 2) + c_chunk;
  const uint32_t o_off = (uint32_t)((c_tok * (int)a.os_t + c_head * (int)a.os_h) * 2) + c_chunk;
  const uint32_t q_step = (uint32_t)((C::ROWS_PER_COPY / a.g_q) * (int)a.qs_t * 2);
  const uint32_t o_step = (uint32_t)((C::ROWS_PER_COPY / a.g_q) * (int)a.os_t * 2);
  // the key and value tiles, once (rows past the end of the sequence read as zeros)
  {
    const uint32_t k_off = (uint32_t)(c_row * (int)a.ks_t * 2) + c_chunk;
    const uint32_t v_off = (uint32_t)(c_row * (int)a.vs_t * 2) + c_chunk;
#pragma unroll
    for (int i = 0; i < C::COPIES; i++) {
      const uint32_t la = lds0 + wave * 1024 + i * 4096;
      copy16_to_lds(k_rs, la, k_off, (uint32_t)(kpos0 + i * C::ROWS_PER_COPY) * (uint32_t)a.ks_t * 2u);
      copy16_to_lds(v_rs, la + C::TILE_BYTES, v_off, (uint32_t)(kpos0 + i * C::ROWS_PER_COPY) * (uint32_t)a.vs_t * 2u);
    }
  }

  // operand read offsets: B operands (keys kh*32 + n) and A operands (rows rh*32 + n)
  // share the row-major pattern; the transposing reads walk this wave's 32 rows
  const uint32_t b_rd = tile_off<D>(kh * 32 + n, 8 * h), a_rd = tile_off<D>(rh * 32 + n, 8 * h);
  const int s16 = lane & 15, a16 = (lane >> 4) & 1;
  const uint32_t t_lo = tile_off<D>(rh * 32 + 4 * h + (s16 >> 2), 16 * a16 + 4 * (s16 & 3));
  const uint32_t t_hi = tile_off<D>(rh * 32 + 8 + 4 * h + (s16 >> 2), 16 * a16 + 4 * (s16 & 3));

  f32x16 dkacc[C::NDT], dvacc[C::NDT];
#pragma unroll
  for (int t = 0; t < C::NDT; t++) { dkacc[t] = zero16(); dvacc[t] = zero16(); }
  float kbv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};   // dkbar partial: 8 d of this thread's rows

  // Steps: the 64-row halves of the row tiles whose bit is set in this chunk's column
  // mask, ascending.  The per-row scalars of a step (mask bit, bias, dx, log-sum-exp,
  // D) are fetched one step ahead into registers, all addresses known up front, so
  // that their latency overlaps the previous step instead of preceding the tile copies.
  const uint32_t* cm = a.colmask + ((int64_t)hbi * a.t_all + c) * a.cwords;
  int st_wi = -1, st_half = 1, st_T = 0;
  uint32_t st_bits = 0u;
  auto next_step = [&]() -> int {        // first token of the next step, or -1
    for (;;) {
      if (st_half == 0) { st_half = 1; }
      else {
        while (st_bits == 0u) {
          if (++st_wi >= a.cwords) return -1;
          st_bits = __builtin_amdgcn_readfirstlane(cm[st_wi]);
        }
        st_T = st_wi * 32 + __builtin_ctz(st_bits);
        st_bits &= st_bits - 1u;
        st_half = 0;
      }
      const int t0 = st_T * 2 * tok_step + st_half * tok_step;
      if (t0 < a.n_q) return t0;
    }
  };
  // this lane's row of a step (lanes 0..15 of each wave: row 16 wave + lane)
  const int s_row = wave * 16 + (lane & 15);
  const int s_head = r * a.g_q + s_row % a.g_q;
  uint32_t f_mask = 0u;
  float f_bias = 0.f, f_dx = 0.f, f_lse = 0.f, f_dsum = 0.f;
  int f_tok = 0;
  bool f_ok = false;
  auto fetch = [&](int t0) {
    const int tk = t0 + s_row / a.g_q;
    f_ok = tk < a.n_q;
    f_tok = f_ok ? tk : a.n_q - 1;
    const int64_t trow = ((int64_t)b * a.h_kv + r) * a.n_q + f_tok;
    const int64_t hrow = ((int64_t)b * a.h_q + s_head) * a.n_q + f_tok;
    f_mask = a.mask[trow * a.words + (c >> 5)];
    f_bias = a.biasd[trow * a.t_all + c];      // meaningful only where the mask bit is set
    f_dx = a.dxd[hrow * a.t_all + c];          // and, for dx, where the chunk is a candidate
    f_lse = a.lse[hrow];
    f_dsum = a.dsum[hrow];
  };
  int tok0 = next_step();
  if (tok0 >= 0 && lane < 16) fetch(tok0);
  while (tok0 >= 0) {
    __syncthreads();                    // the previous step is no longer read
    int have = 0;
    if (lane < 16) {
      const bool bit = f_ok && ((f_mask >> (c & 31)) & 1u);
      const int cdiag = f_tok / a.block;
      const bool isdiag = a.causal && c == cdiag;
      const int n_cand = a.causal ? max(cdiag - a.window, 0) : a.t_c;
      // bias - log-sum-exp in base-2 units (-inf: the row does not attend the chunk)
      cmb_s[s_row] = bit ? (isdiag ? 0.f : f_bias * kLog2e) - f_lse : -INFINITY;
      dx_s[s_row] = (bit && c < n_cand) ? f_dx : 0.f;
      dsum_s[s_row] = f_dsum;
      pos_s[s_row] = a.causal ? f_tok : 0x7fffffff;
      have = bit ? 1 : 0;
    }
    const int cur_tok0 = tok0;
    tok0 = next_step();
    if (tok0 >= 0 && lane < 16) fetch(tok0);
    if (!__syncthreads_or(have)) continue;
    // is the chunk a routing candidate of any row of this step?  (the candidate count
    // grows with the position, so the step's last token decides)
    const bool any_cand = c < (a.causal ? max(min(cur_tok0 + tok_step - 1, a.n_q - 1) / a.block - a.window, 0)
                                        : a.t_c);
    // the key mask matters only where the rows' own chunk is this one, or at the end of the sequence
    const bool masked = (a.causal && (cur_tok0 + tok_step - 1) / a.block >= c && cur_tok0 / a.block <= c) ||
                        kpos0 + 64 > a.n_kv;
    const uint32_t soff_q = (uint32_t)cur_tok0 * (uint32_t)a.qs_t * 2u;
    const uint32_t soff_o = (uint32_t)cur_tok0 * (uint32_t)a.os_t * 2u;
#pragma unroll
    for (int i = 0; i < C::COPIES; i++) {
      const uint32_t la = lds0 + 2 * C::TILE_BYTES + wave * 1024 + i * 4096;
      copy16_to_lds(q_rs, la, q_off, soff_q + i * q_step);
      copy16_to_lds(o_rs, la + C::TILE_BYTES, o_off, soff_o + i * o_step);
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    // S = Q K^T and dP = dO V^T for this wave's 32 rows x 32 keys
    // (the base offsets are made opaque here so that the per-slice offsets derived from
    // them are formed next to their use instead of being kept in registers across steps)
    uint32_t a_b = a_rd, b_b = b_rd, tl = t_lo, th = t_hi;
    asm volatile("" : "+v"(a_b), "+v"(b_b), "+v"(tl), "+v"(th));
    f32x16 s = zero16(), dp = zero16();
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) {
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_a<D>(q_t, a_b, 2 * ks), read_a<D>(k_t, b_b, 2 * ks), s, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_a<D>(d_t, a_b, 2 * ks), read_a<D>(v_t, b_b, 2 * ks), dp, 0, 0, 0);
    }
    u32x4 pp[2], pd[2];
#pragma unroll
    for (int q4 = 0; q4 < 4; q4++) {
      const int row0 = rh * 32 + 8 * q4 + 4 * h;
      const float4 d4 = *reinterpret_cast<const float4*>(dsum_s + row0);
      const float4 b4 = *reinterpret_cast<const float4*>(cmb_s + row0);
      int4 p4 = {0x7fffffff, 0x7fffffff, 0x7fffffff, 0x7fffffff};
      if (masked) p4 = *reinterpret_cast<const int4*>(pos_s + row0);
      const float ds[4] = {d4.x, d4.y, d4.z, d4.w};
      const float bs[4] = {b4.x, b4.y, b4.z, b4.w};
      const int ps[4] = {p4.x, p4.y, p4.z, p4.w};
      float pv[4], dv[4];
#pragma unroll
      for (int i = 0; i < 4; i++) {
        const int j = q4 * 4 + i;
        const bool dead = masked && (my_key > ps[i] || my_key >= a.n_kv);
        const float p = dead ? 0.f : __builtin_amdgcn_exp2f(fmaf(s[j], a.c1, bs[i]));
        pv[i] = p;
        dv[i] = p * (dp[j] - ds[i]);
      }
      pp[q4 >> 1][(q4 & 1) * 2 + 0] = cvt_bf16x2(pv[0], pv[1]);
      pp[q4 >> 1][(q4 & 1) * 2 + 1] = cvt_bf16x2(pv[2], pv[3]);
      pd[q4 >> 1][(q4 & 1) * 2 + 0] = cvt_bf16x2(dv[0], dv[1]);
      pd[q4 >> 1][(q4 & 1) * 2 + 1] = cvt_bf16x2(dv[2], dv[3]);
    }
    // dV^T += dO^T P,  dK^T += Q^T dS  (contraction over this wave's 32 rows)
#pragma unroll
    for (int g = 0; g < 2; g++)
#pragma unroll
      for (int t = 0; t < C::NDT; t++) {
        dvacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t<D>(d_t, tl, th, g, t),
                                                           __builtin_bit_cast(bf16x8, pp[g]), dvacc[t], 0, 0, 0);
        dkacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_t<D>(q_t, tl, th, g, t),
                                                           __builtin_bit_cast(bf16x8, pd[g]), dkacc[t], 0, 0, 0);
      }
    // dkbar += sum_rows dx q: thread tid takes the 8 d of chunk tid % NCH and the RPG rows of group tid / NCH
    if (any_cand) {
      const int cs = tid % C::NCH, rg = tid / C::NCH;
#pragma unroll
      for (int rr = 0; rr < RPG; rr++) {
        const int row = rg * RPG + rr;
        const float dx = dx_s[row];
        const bf16x8 qv = *reinterpret_cast<const bf16x8*>(q_t + tile_off<D>(row, 8 * cs));
#pragma unroll
        for (int e = 0; e < 8; e++) kbv[e] = fmaf(dx, (float)qv[e], kbv[e]);
      }
    }
  }

  // ---- combine the two row halves and write ------------------------------------
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // a workgroup without any step: its K / V copies
  __syncthreads();
  {
    const int cs = tid % C::NCH, rg = tid / C::NCH;
#pragma unroll
    for (int e = 0; e < 8; e++) red[rg * D + 8 * cs + e] = kbv[e];
  }
  float* xch = reinterpret_cast<float*>(lds);          // [2 kh][2 tensors][NDT*16][64 lanes]
  if (rh == 1) {
#pragma unroll
    for (int t = 0; t < C::NDT; t++)
#pragma unroll
      for (int j = 0; j < 16; j++) {
        xch[((kh * 2 + 0) * C::NDT * 16 + t * 16 + j) * 64 + lane] = dkacc[t][j];
        xch[((kh * 2 + 1) * C::NDT * 16 + t * 16 + j) * 64 + lane] = dvacc[t][j];
      }
  }
  __syncthreads();
  if (tid < D) {
    float t = 0.f;
    for (int g = 0; g < RG; g++) t += red[g * D + tid];
    redf[tid] = t;
  }
  __syncthreads();
  if (a.dkbar_out && tid < D && c < a.t_c && kpos0 % a.block == 0)
    a.dkbar_out[(((int64_t)b * a.h_kv + r) * a.t_c + c) * D + tid] = redf[tid] * a.xscale;
  if (rh == 0 && my_key < a.n_kv) {
    // block-mean summaries: every key of a complete chunk receives 1/B of the chunk's dkbar
    const float kscale = (c < a.t_c && !a.dkbar_out) ? a.xscale / (float)a.block : 0.f;
    uint16_t* dkp = a.dk + b * a.ks_b + r * a.ks_h + (int64_t)my_key * a.ks_t;
    uint16_t* dvp = a.dv + b * a.vs_b + r * a.vs_h + (int64_t)my_key * a.vs_t;
#pragma unroll
    for (int t = 0; t < C::NDT; t++)
#pragma unroll
      for (int q4 = 0; q4 < 4; q4++) {
        const int d0 = t * 32 + q4 * 8 + h * 4;
        float kv[4], vv[4];
#pragma unroll
        for (int i = 0; i < 4; i++) {
          const int j = q4 * 4 + i;
          const float kbar_g = redf[d0 + i];
          kv[i] = (dkacc[t][j] + xch[((kh * 2 + 0) * C::NDT * 16 + t * 16 + j) * 64 + lane]) * a.scale +
                  kbar_g * kscale;
          vv[i] = dvacc[t][j] + xch[((kh * 2 + 1) * C::NDT * 16 + t * 16 + j) * 64 + lane];
        }
        uint2 w;
        w.x = cvt_bf16x2(kv[0], kv[1]); w.y = cvt_bf16x2(kv[2], kv[3]);
        *reinterpret_cast<uint2*>(dkp + d0) = w;
        w.x = cvt_bf16x2(vv[0], vv[1]); w.y = cvt_bf16x2(vv[2], vv[3]);
        *reinterpret_cast<uint2*>(dvp + d0) = w;
      }
  }
}

// ---------------------------------------------------------------------------
// fp32 tensors: plain VALU kernels (the correctness vehicle of the fp32
// configuration, like the fp32 forward; not a tuned path).  One workgroup per
// (token, kv-head), one wave per query head, lanes over the 64 keys of a tile
// for the logits and over the head dimension for the sums; dK, dV and the bias
// gradient are accumulated with fp32 atomics into zeroed outputs.  The routing
// kernel above is shared with the bf16 path.
// ---------------------------------------------------------------------------
__global__ void bwd_f32_zero_kernel(BwdArgs a, int d, int batch) {
  const int64_t rows = (int64_t)batch * a.h_kv * a.n_kv;
  float* dk = reinterpret_cast<float*>(a.dk);
  float* dv = reinterpret_cast<float*>(a.dv);
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < rows * d; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t row = i / d;
    const int e = (int)(i % d);
    const int key = (int)(row % a.n_kv);
    const int64_t hb = row / a.n_kv;
    const int r = (int)(hb % a.h_kv), b = (int)(hb / a.h_kv);
    dk[b * a.ks_b + r * a.ks_h + (int64_t)key * a.ks_t + e] = 0.f;
    dv[b * a.vs_b + r * a.vs_h + (int64_t)key * a.vs_t + e] = 0.f;
  }
}

__global__ __launch_bounds__(256) void bwd_f32_row_kernel(BwdArgs a, int d) {
  __shared__ float qs[4][128], dos[4][128], ps[4][64], zs[4][64];
  const int tok = blockIdx.x, r = blockIdx.y, b = blockIdx.z;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int pos = tok;                                   // n_q == n_kv
  const int cw = pos / a.block;
  const int nsub = a.block >> 6;
  const int64_t base = ((int64_t)b * a.h_kv + r) * a.n_q + tok;
  const uint32_t* mrow = a.mask + base * a.words;
  const float* brow = a.bias + base * a.t_all;
  const float* kb = reinterpret_cast<const float*>(a.k) + b * a.ks_b + r * a.ks_h;
  const float* vb = reinterpret_cast<const float*>(a.v) + b * a.vs_b + r * a.vs_h;
  float* dkb = reinterpret_cast<float*>(a.dk) + b * a.ks_b + r * a.ks_h;
  float* dvb = reinterpret_cast<float*>(a.dv) + b * a.vs_b + r * a.vs_h;

  for (int hl = wave; hl < a.g_q; hl += 4) {
    const int head = r * a.g_q + hl;
    const float* qp = reinterpret_cast<const float*>(a.q) + b * a.qs_b + head * a.qs_h + (int64_t)tok * a.qs_t;
    const float* dop = reinterpret_cast<const float*>(a.d_o) + b * a.os_b + head * a.os_h + (int64_t)tok * a.os_t;
    for (int e = lane; e < d; e += 64) { qs[wave][e] = qp[e]; dos[wave][e] = dop[e]; }
    __builtin_amdgcn_wave_barrier();
    // logit and dP = <dO, v> of this lane's key of a 64-key tile
    auto key_terms = [&](int kpos0, bool diag, float bias, float& z, float& dp) -> bool {
      const int key = kpos0 + lane;
      const bool valid = key < a.n_kv && (!diag || key <= pos);
      z = -INFINITY;
      dp = 0.f;
      if (valid) {
        const float* kr = kb + (int64_t)key * a.ks_t;
        const float* vr = vb + (int64_t)key * a.vs_t;
        float acc = 0.f, acd = 0.f;
        for (int e = 0; e < d; e += 4) {
          const f32x4 kk = *reinterpret_cast<const f32x4*>(kr + e);
          const f32x4 vv = *reinterpret_cast<const f32x4*>(vr + e);
#pragma unroll
          for (int i = 0; i < 4; i++) {
            acc = fmaf(qs[wave][e + i], kk[i], acc);
            acd = fmaf(dos[wave][e + i], vv[i], acd);
          }
        }
        z = fmaf(acc, a.scale, bias);
        dp = acd;
      }
      return valid;
    };
    float lse = 0.f, dsum = 0.f, dq0 = 0.f, dq1 = 0.f;
    for (int pass = 0; pass < 2; pass++) {
      float m = -INFINITY, l = 0.f, dn = 0.f;
      int rank = 0;
      for (int u = 0; u < a.words * 32; u++) {
        const uint32_t w = mrow[u >> 5];
        if (w == 0u) { u |= 31; continue; }
        if (!((w >> (u & 31)) & 1u)) continue;
        const bool diag = a.causal && u == cw;
        float bias = 0.f;
        if (!diag) bias = brow[rank++];
        float chunk_dz = 0.f;
        for (int sub = 0; sub < nsub; sub++) {
          const int kpos0 = u * a.block + sub * 64;
          float z, dp;
          const bool valid = key_terms(kpos0, diag, bias, z, dp);
          if (pass == 0) {
            const float m_new = fmaxf(m, wave_max(z));
            if (m_new == -INFINITY) continue;
            const float p = valid ? expf(z - m_new) : 0.f;
            const float corr = expf(m - m_new);
            l = l * corr + wave_sum(p);
            dn = dn * corr + wave_sum(p * dp);
            m = m_new;
            continue;
          }
          const float p = valid ? expf(z - lse) : 0.f;
          const float dz = p * (dp - dsum);
          chunk_dz += wave_sum(dz);
          ps[wave][lane] = dz;
          zs[wave][lane] = p;
          __builtin_amdgcn_wave_barrier();
          const int kmax = min(64, a.n_kv - kpos0);
          for (int kk = 0; kk < kmax; kk++) {
            const float dzk = ps[wave][kk], pk = zs[wave][kk];
            if (pk == 0.f && dzk == 0.f) continue;
            const int64_t key = kpos0 + kk;
            const float* kr = kb + key * a.ks_t;
            dq0 = fmaf(dzk, kr[lane], dq0);
            atomicAdd(dkb + key * a.ks_t + lane, a.scale * dzk * qs[wave][lane]);
            atomicAdd(dvb + key * a.vs_t + lane, pk * dos[wave][lane]);
            if (d > 64) {
              dq1 = fmaf(dzk, kr[lane + 64], dq1);
              atomicAdd(dkb + key * a.ks_t + lane + 64, a.scale * dzk * qs[wave][lane + 64]);
              atomicAdd(dvb + key * a.vs_t + lane + 64, pk * dos[wave][lane + 64]);
            }
          }
          __builtin_amdgcn_wave_barrier();
        }
        if (pass == 1 && !diag && lane == 0) atomicAdd(a.dbd + base * a.t_all + u, chunk_dz);
      }
      if (pass == 0) {
        lse = m + logf(l);
        dsum = dn / l;
      }
    }
    const int64_t row = ((int64_t)b * a.h_q + head) * a.n_q + tok;
    a.dq32[row * d + lane] = a.scale * dq0;
    if (d > 64) a.dq32[row * d + lane + 64] = a.scale * dq1;
    __builtin_amdgcn_wave_barrier();
  }
}

// dkbar_c = xscale sum over the tokens that route to chunk c and their heads of dx q; folded
// into the chunk's keys (block mean) or written out.  One workgroup per (chunk, kv-head, batch),
// thread = head-dimension index.
__global__ __launch_bounds__(128) void bwd_f32_kbar_kernel(BwdArgs a, int d) {
  const int c = blockIdx.x, r = blockIdx.y, b = blockIdx.z, t = threadIdx.x;
  const int i0 = a.causal ? (c + 1 + a.window) * a.block : 0;       // first token with c among its candidates
  float acc = 0.f;
  for (int i = i0; i < a.n_q; i++) {
    const int64_t trow = ((int64_t)b * a.h_kv + r) * a.n_q + i;
    if (!((a.mask[trow * a.words + (c >> 5)] >> (c & 31)) & 1u)) continue;
    for (int hl = 0; hl < a.g_q; hl++) {
      const int head = r * a.g_q + hl;
      const float dx = a.dxd[(((int64_t)b * a.h_q + head) * a.n_q + i) * a.t_all + c];
      if (t < d)
        acc = fmaf(dx, reinterpret_cast<const float*>(a.q)[b * a.qs_b + head * a.qs_h + (int64_t)i * a.qs_t + t], acc);
    }
  }
  if (t >= d) return;
  const float g = acc * a.xscale;
  if (a.dkbar_out) {
    a.dkbar_out[(((int64_t)b * a.h_kv + r) * a.t_c + c) * d + t] = g;
  } else {
    float* dk = reinterpret_cast<float*>(a.dk) + b * a.ks_b + r * a.ks_h;
    for (int j = 0; j < a.block; j++) dk[(int64_t)(c * a.block + j) * a.ks_t + t] += g / (float)a.block;
  }
}

template <int D> static hipError_t launch_bwd_f32(const BwdArgs& a, int batch, hipStream_t st) {
  hipError_t e;
  hipLaunchKernelGGL(bwd_f32_zero_kernel, dim3(1024), dim3(256), 0, st, a, D, batch);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  const size_t nwords = (size_t)batch * a.h_kv * a.n_q * a.t_all;         // the bias gradient, by chunk id
  hipLaunchKernelGGL(bwd_fill_zero_kernel, dim3(1024), dim3(256), 0, st, reinterpret_cast<uint32_t*>(a.dbd), nwords);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  hipLaunchKernelGGL(bwd_f32_row_kernel, dim3(a.n_q, a.h_kv, batch), dim3(256), 0, st, a, D);
  if ((e = hipGetLastError()) != hipSuccess) return e;
  if ((e = launch_route_g<D, float>(a, batch, st)) != hipSuccess) return e;
  if (a.t_c > 0) {
    hipLaunchKernelGGL(bwd_f32_kbar_kernel, dim3(a.t_c, a.h_kv, batch), dim3(128), 0, st, a, D);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

// ---------------------------------------------------------------------------
// Host side
// ---------------------------------------------------------------------------
static size_t al256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t backward_workspace_bytes(const dash_params& p, const Layout& L) {
  const size_t rows_q = (size_t)p.batch * p.h_q * p.n_q, rows_kv = (size_t)p.batch * p.h_kv * p.n_q;
  const int tok_tile = 4 * (32 / L.g_q);
  const int n_tiles = (p.n_q + tok_tile - 1) / tok_tile;
  const int cwords = (n_tiles + 31) / 32;
  return 2 * al256(rows_q * 4) + 2 * al256(rows_kv * L.t_all * 4) + al256(rows_q * L.t_all * 4) +
         al256(rows_q * p.head_dim * 4) + al256((size_t)p.batch * p.h_kv * L.t_all * cwords * 4);
}

template <int D, int G, typename T> static hipError_t launch_route(const BwdArgs& a, int batch, hipStream_t st) {
  const size_t lds = (size_t)G * D * 4 + (size_t)a.t_c * 8 + (size_t)G * 64 * 4 + 64;
  auto kern = bwd_route_kernel<D, G, T>;     // at most 29 KB of LDS (t_c <= 2048): no opt-in needed
  hipLaunchKernelGGL(kern, dim3((unsigned)((size_t)batch * a.h_kv * a.n_q)), dim3(64), lds, st, a);
  return hipGetLastError();
}

template <int D, typename T> static hipError_t launch_route_g(const BwdArgs& a, int batch, hipStream_t st) {
  switch (a.g_q) {
    case 1: return launch_route<D, 1, T>(a, batch, st);
    case 2: return launch_route<D, 2, T>(a, batch, st);
    case 4: return launch_route<D, 4, T>(a, batch, st);
    case 8: return launch_route<D, 8, T>(a, batch, st);
    default: return launch_route<D, 16, T>(a, batch, st);
  }
}

template <int D> static hipError_t launch_bwd_t(const BwdArgs& a, int batch, hipStream_t st) {
  using C = BCfg<D>;
  static LdsOptIn done_lse, done_grad, done_kv;
  hipError_t e;
  {
    const size_t nwords = (size_t)a.hb * a.t_all * a.cwords;
    hipLaunchKernelGGL(bwd_fill_zero_kernel, dim3((unsigned)((nwords + 255) / 256 < 1024 ? (nwords + 255) / 256 : 1024)),
                       dim3(256), 0, st, a.colmask, nwords);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    const size_t lds = 2 * C::TILE_BYTES + 5 * 64 * 4;
    auto kern = bwd_q_kernel<D, false>;
    if ((e = allow_dyn_lds((const void*)kern, lds, done_lse)) != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.hb), dim3(256), lds, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  {
    const size_t lds = 4 * C::TILE_BYTES + 5 * 64 * 4;
    auto kern = bwd_q_kernel<D, true>;
    if ((e = allow_dyn_lds((const void*)kern, lds, done_grad)) != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(a.n_tiles * a.hb), dim3(256), lds, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  if ((e = launch_route_g<D, uint16_t>(a, batch, st)) != hipSuccess) return e;
  {
    const size_t xch = (size_t)2 * 2 * C::NDT * 16 * 64 * 4;
    const size_t tiles = 4 * C::TILE_BYTES;
    // tiles (reused for the end-of-kernel exchange), 4 per-row scalar arrays, dkbar and its partials
    const size_t lds = (xch > tiles ? xch : tiles) + 4 * 64 * 4 + D * 4 + (size_t)(256 / C::NCH) * D * 4;
    auto kern = bwd_kv_kernel<D>;
    if ((e = allow_dyn_lds((const void*)kern, lds, done_kv)) != hipSuccess) return e;
    const int ktiles = (a.n_kv + 63) / 64;
    hipLaunchKernelGGL(kern, dim3(ktiles * a.hb), dim3(256), lds, st, a);
    if ((e = hipGetLastError()) != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_backward(const dash_params& p, const Layout& L, const void* q, const void* k, const void* v,
                           const void* d_o, const float* kbar, const uint32_t* mask,
                           const float* bias, const float* tau, void* dq, void* dk, void* dv, float* dkbar_out,
                           char* ws, hipStream_t st) {
  BwdArgs a;
  a.dkbar_out = dkbar_out;
  a.q = (const uint16_t*)q; a.k = (const uint16_t*)k; a.v = (const uint16_t*)v;
  a.d_o = (const uint16_t*)d_o;
  a.dq = (uint16_t*)dq; a.dk = (uint16_t*)dk; a.dv = (uint16_t*)dv;
  a.kbar = kbar; a.mask = mask; a.bias = bias; a.tau = tau;
  a.h_q = p.h_q; a.h_kv = p.h_kv; a.g_q = L.g_q; a.n_q = p.n_q; a.n_kv = p.n_kv; a.block = p.block_size;
  a.t_c = L.t_c; a.t_all = L.t_all; a.words = L.words; a.causal = p.causal; a.window = p.window;
  a.hb = p.h_kv * p.batch;
  const int tok_tile = 4 * (32 / L.g_q);
  a.n_tiles = (p.n_q + tok_tile - 1) / tok_tile;
  a.cwords = (a.n_tiles + 31) / 32;
  a.qs_b = p.q_stride[0]; a.qs_h = p.q_stride[1]; a.qs_t = p.q_stride[2];
  a.ks_b = p.k_stride[0]; a.ks_h = p.k_stride[1]; a.ks_t = p.k_stride[2];
  a.vs_b = p.v_stride[0]; a.vs_h = p.v_stride[1]; a.vs_t = p.v_stride[2];
  a.os_b = p.o_stride[0]; a.os_h = p.o_stride[1]; a.os_t = p.o_stride[2];
  a.c1 = L.scale * kLog2e; a.scale = L.scale; a.xscale = L.xscale; a.pexp = L.pexp; a.sigma = p.sigma;
  const size_t rows_q = (size_t)p.batch * p.h_q * p.n_q, rows_kv = (size_t)p.batch * p.h_kv * p.n_q;
  size_t off = 0;
  a.lse = (float*)(ws + off);    off += al256(rows_q * 4);
  a.dsum = (float*)(ws + off);   off += al256(rows_q * 4);
  a.biasd = (float*)(ws + off);  off += al256(rows_kv * L.t_all * 4);
  a.dbd = (float*)(ws + off);    off += al256(rows_kv * L.t_all * 4);
  a.dxd = (float*)(ws + off);    off += al256(rows_q * L.t_all * 4);
  a.dq32 = (float*)(ws + off);   off += al256(rows_q * p.head_dim * 4);
  a.colmask = (uint32_t*)(ws + off);
  if (p.dtype == DASH_F32)
    return p.head_dim == 128 ? launch_bwd_f32<128>(a, p.batch, st) : launch_bwd_f32<64>(a, p.batch, st);
  return p.head_dim == 128 ? launch_bwd_t<128>(a, p.batch, st) : launch_bwd_t<64>(a, p.batch, st);
}

}  // namespace dash
