// Split-KV decode of Stage 2 (bf16): one query token per sequence attends its
// routed chunks with the Stage-1 bias added to the logits (Sec. 3.3 Eq. 6 in the
// bias form of Proposition 1; Alg. 3), the attended list cut into splits whose
// partial results a merge kernel combines (Sec. 3.5); the dense decode reference
// (Eq. 1) comes from the same template.
//
// The step is bound by HBM: every attended chunk is read once (K and V rows,
// 2 * block * d * 2 bytes) and used for 4 * g_q flops per byte.  A workgroup
// (4 waves) owns entries [e0, e1) of one (batch, kv-head) pair's ascending list
// and streams them as 32-key sub-tiles copied from global memory straight into an
// LDS ring (buffer_load ... lds, no staging registers): NST - 1 sub-tiles are in
// flight while one is computed, and three workgroups share a CU, so a workgroup
// that is starting up or draining does not leave the memory pipe idle.
//
// Work per sub-tile: all four waves compute the same S^T = K Q^T (32 keys x 32
// rows, the g_q query heads padded to 32) and the same softmax statistics; wave
// w accumulates only d-tile w of O^T += V^T P^T.  The MFMA formulation, the
// swizzled row-major LDS tiles and the transposing V reads are those of the
// prefill kernel.  The attended chunk ids are decoded from the bit mask held in
// one VGPR (lane i = mask word i); the bias list is read with scalar loads.
#include <math.h>
#include <stdlib.h>

#include <type_traits>

#include "common.h"
#include "dash_internal.h"
#include "lds_copy.h"
#include "stage2_args.h"

namespace dash {


constexpr int kDecStages = 3;   // LDS ring depth (sub-tiles)

template <int D> struct DecCfg {
  static constexpr int NCH = D / 8;                        // 16-byte chunks per row
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int SUB_BYTES = 32 * ROW_BYTES;         // one 32-key K or V sub-tile
  static constexpr int STAGE_BYTES = 2 * SUB_BYTES;        // K then V
  static constexpr int COPIES = SUB_BYTES / 16 / 256;      // copy instructions per thread, sub-tile and tensor
  static constexpr int ROWS_PER_COPY = 256 / NCH;
  static constexpr size_t LDS_BYTES = (size_t)kDecStages * STAGE_BYTES;
};

// same chunk permutations as the prefill tiles (see stage2.hip)
template <int D> __device__ __forceinline__ int dk_swz(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int dv_swz(int row) {
  return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

template <int D, bool DENSE>
__global__ __launch_bounds__(256, 3) void s2_decode_kernel(S2Args a) {
  using C = DecCfg<D>;
  constexpr int NST = kDecStages;
  extern __shared__ __attribute__((aligned(1024))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n = lane & 31, h = lane >> 5;
  const int pairs = a.hb, splits = a.n_tiles;
  const int pair = blockIdx.x % pairs, split = blockIdx.x / pairs;
  const int r = pair % a.h_kv, b = pair / a.h_kv;
  // length of this sequence's cache (the current token included): the capacity
  // n_kv, or the caller's per-sequence value, clamped to [1, n_kv]
  const int len = a.seq_lens ? min(max(__builtin_amdgcn_readfirstlane(a.seq_lens[b]), 1), a.n_kv) : a.n_kv;
  const int pos = len - 1;                    // the query's sequence position
  const int cw = pos / a.block;               // its (diagonal) chunk
  const int nsub = a.block >> 5;              // 32-key sub-tiles per chunk

  // ---- this workgroup's share of the attended list -------------------------
  // lane i holds mask word i; `total` entries in ascending order, the diagonal
  // chunk last.  Entries [e0, e1) are ours.
  uint32_t word = 0u;
  if (!DENSE && lane < a.words) word = a.mask[(int64_t)pair * a.words + lane];
  int total;
  int incl = 0;
  if (DENSE) {
    total = (a.causal ? cw : a.t_all - 1) + 1;
  } else {
    incl = __popc(word);
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
      const int t = __shfl_up(incl, off);
      if (lane >= off) incl += t;
    }
    total = __builtin_amdgcn_readlane(incl, 63);
  }
  const int per = (total + splits - 1) / splits;
  const int e0 = split * per, e1 = min(total, e0 + per);
  float* part = a.part + (((int64_t)pair * splits + split) * a.g_q) * (D + 2);
  if (e0 >= e1) {
    // empty split: weight zero in the merge
    if (wave == 0 && lane < a.g_q) { part[lane * (D + 2) + D] = -INFINITY; part[lane * (D + 2) + D + 1] = 0.f; }
    return;
  }
  // chunk-id iterator over the mask, positioned at entry e0 (wave-uniform scalars)
  int it_wi = 0;
  uint32_t it_bits = 0u;
  if (!DENSE) {
    // first word whose inclusive count exceeds e0
    const uint64_t ball = __ballot(incl > e0);
    it_wi = __builtin_ctzll(ball);
    const int before = __builtin_amdgcn_readlane(incl, it_wi) - __popc(__builtin_amdgcn_readlane(word, it_wi));
    it_bits = __builtin_amdgcn_readlane(word, it_wi);
    for (int i = before; i < e0; i++) it_bits &= it_bits - 1u;   // drop the entries below e0
  }
  int it_e = e0;   // entry the iterator points at
  auto next_id = [&]() -> int {   // id of entry it_e, then advance
    int id;
    if (DENSE) {
      id = it_e;
    } else {
      while (it_bits == 0u) { it_wi++; it_bits = __builtin_amdgcn_readlane(word, it_wi); }
      id = it_wi * 32 + __builtin_ctz(it_bits);
      it_bits &= it_bits - 1u;
    }
    it_e++;
    return id;
  };

  // ---- Q fragments: rows >= g_q repeat valid heads (their results are dropped) --
  const int my_head = r * a.g_q + n % a.g_q;
  bf16x8 qf[D / 16];
  {
    const uint16_t* qp = a.q + b * a.qs_b + my_head * a.qs_h + h * 8;
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) qf[ks] = *reinterpret_cast<const bf16x8*>(qp + ks * 16);
#pragma unroll
    for (int ks = 0; ks < D / 16; ks++) asm volatile("" : "+v"(qf[ks]));   // loads done before the loop
  }

  // ---- global -> LDS sub-tile copies (layout as in the prefill kernel) -------
  const u32x4 k_rs = make_rsrc(a.k + b * a.ks_b + r * a.ks_h, (((int64_t)len - 1) * a.ks_t + D) * 2);
  const u32x4 v_rs = make_rsrc(a.v + b * a.vs_b + r * a.vs_h, (((int64_t)len - 1) * a.vs_t + D) * 2);
  const uint32_t lds0 = lds_addr_of(lds);
  const int c_row = (wave * 64 + lane) / C::NCH, c_pos = lane % C::NCH;
  const uint32_t k_off = (uint32_t)(c_row * (int)a.ks_t * 2 + ((c_pos ^ dk_swz<D>(c_row)) << 4));
  const uint32_t v_off = (uint32_t)(c_row * (int)a.vs_t * 2 + ((c_pos ^ dv_swz<D>(c_row)) << 4));
  const uint32_t k_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.ks_t * 2);
  const uint32_t v_step = (uint32_t)(C::ROWS_PER_COPY * (int)a.vs_t * 2);
  const int n_sub = (e1 - e0) * nsub;   // sub-tiles this workgroup streams
  int cp_t = 0, cp_sub = 0, cp_id = next_id();
  auto copy_next = [&]() {   // sub-tile cp_t -> ring slot cp_t % NST
    const uint32_t dst = lds0 + (cp_t % NST) * C::STAGE_BYTES + wave * 1024;
    const uint32_t key0 = (uint32_t)(cp_id * a.block + cp_sub * 32);
    const uint32_t tk = key0 * (uint32_t)a.ks_t * 2u, tv = key0 * (uint32_t)a.vs_t * 2u;
#pragma unroll
    for (int i = 0; i < C::COPIES; i++) copy16_to_lds(k_rs, dst + i * 4096, k_off, tk + i * k_step);
#pragma unroll
    for (int i = 0; i < C::COPIES; i++) copy16_to_lds(v_rs, dst + C::SUB_BYTES + i * 4096, v_off, tv + i * v_step);
    cp_t++;
    if (++cp_sub == nsub) { cp_sub = 0; if (it_e < e1) cp_id = next_id(); }
  };
  // ---- operand read addresses (bytes inside a ring slot) -----------------------
  uint32_t k_rd[D / 16];
#pragma unroll
  for (int ks = 0; ks < D / 16; ks++)
    k_rd[ks] = (uint32_t)(n * C::ROW_BYTES + (((2 * ks + h) ^ dk_swz<D>(n)) << 4));
  const int s16 = lane & 15, a16 = (lane >> 4) & 1;
  const int dtile = wave < D / 32 ? wave : 0;   // the d-tile this wave accumulates
  const uint32_t v_rd = (uint32_t)(C::SUB_BYTES + (4 * h + (s16 >> 2)) * C::ROW_BYTES +
                                   ((((4 * dtile) ^ dv_swz<D>(s16 >> 2)) + 2 * a16 + ((s16 & 3) >> 1)) << 4) +
                                   ((s16 & 1) << 3));

  // ---- online-softmax state (base-2 logits) -------------------------------
  float m_run = -INFINITY, l_run = 0.f;
  f32x16 oacc;
#pragma unroll
  for (int j = 0; j < 16; j++) oacc[j] = 0.f;
  // the bias list is read with explicit scalar loads: a vector load in the loop
  // would be waited for with vmcnt(0), i.e. together with every copy in flight
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  u32x2 bias_base;
  {
    const uint64_t bp = (uint64_t)(DENSE ? nullptr : a.bias + (int64_t)pair * a.t_all);
    bias_base[0] = __builtin_amdgcn_readfirstlane((uint32_t)bp);
    bias_base[1] = __builtin_amdgcn_readfirstlane((uint32_t)(bp >> 32));
  }
  auto load_bias = [&](int e) -> float {
    float v;
    asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)"
                 : "=s"(v) : "s"(bias_base), "s"(__builtin_amdgcn_readfirstlane(e * 4)) : "memory");
    return v;
  };

  // ---- prologue: NST - 1 sub-tiles in flight ---------------------------------
#pragma unroll
  for (int i = 0; i < NST - 1; i++)
    if (i < n_sub) copy_next();

  // ---- main loop ---------------------------------------------------------------
  // Iteration t: wait until this wave's copies of sub-tile t have landed (all but
  // the newest NST - 2 sub-tiles' worth of copies; everything once the last
  // sub-tile has been issued), barrier (everybody's copies visible; sub-tile
  // t - 1 no longer read), start the copy of sub-tile t + NST - 1 into the slot
  // of sub-tile t - 1, compute sub-tile t.
  int e_c = e0, sub_c = 0;
  float bias_c = 0.f;
  for (int t = 0; t < n_sub; t++) {
    if (sub_c == 0) {
      // the diagonal chunk (last entry of a causal list) carries bias 0
      const bool is_diag = a.causal && e_c == total - 1;
      bias_c = (DENSE || is_diag) ? 0.f : load_bias(e_c) * kLog2e;
    }
    if (cp_t - t - 1 >= NST - 2) {
      static_assert(NST == 3, "the wait below counts one sub-tile's copies");
      if constexpr (C::COPIES == 2) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
      else asm volatile("s_waitcnt vmcnt(2)" ::: "memory");
    } else {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    }
    __syncthreads();
    if (cp_t < n_sub) copy_next();

    const char* sb = lds + (t % NST) * C::STAGE_BYTES;
    f32x16 s;
    {
      bf16x8 kf[D / 16];
#pragma unroll
      for (int ks = 0; ks < D / 16; ks++) kf[ks] = *reinterpret_cast<const bf16x8*>(sb + k_rd[ks]);
      const f32x16 z = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[0], z, 0, 0, 0);
#pragma unroll
      for (int ks = 1; ks < D / 16; ks++) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[ks], qf[ks], s, 0, 0, 0);
    }
    // V^T fragments of this wave's d-tile (contraction steps g = 0, 1)
    bf16x8 vf[2];
    if (wave < D / 32) {
#pragma unroll
      for (int g = 0; g < 2; g++) {
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(sb + v_rd + (16 * g) * C::ROW_BYTES));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
            (__attribute__((address_space(3))) s16x4*)(sb + v_rd + (16 * g + 8) * C::ROW_BYTES));
        vf[g] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
      }
    }
    // keys after the query's position (diagonal chunk only) are dead
    if (a.causal && e_c == total - 1) {
      const int lim = pos - (cw * a.block + sub_c * 32 + 4 * h);   // dead if c > lim
#pragma unroll
      for (int j = 0; j < 16; j++) {
        const int c = (j >> 2) * 8 + (j & 3);
        s[j] = c > lim ? -INFINITY : s[j];
      }
    }
    float mloc = -INFINITY;
#pragma unroll
    for (int j = 0; j < 16; j += 2) mloc = fmaxf(fmaxf(mloc, s[j]), s[j + 1]);
    mloc = fmaxf(mloc, __shfl_xor(mloc, 32));
    const float tmax = fmaf(mloc, a.c1, bias_c);
    // lazy rescaling: see the prefill kernel
    if (__any(tmax > m_run + kLazy)) {
      const float m_new = fmaxf(m_run, tmax);
      const float m_use = m_new == -INFINITY ? 0.f : m_new;
      const float corr = __builtin_amdgcn_exp2f(m_run - m_use);
      m_run = m_new;
      l_run *= corr;
#pragma unroll
      for (int j = 0; j < 16; j++) oacc[j] *= corr;
    }
    const float off = bias_c - (m_run == -INFINITY ? 0.f : m_run);
    u32x4 pb[2];
    float lsum = 0.f;
#pragma unroll
    for (int j = 0; j < 16; j += 2) {
      const float p0 = __builtin_amdgcn_exp2f(fmaf(s[j], a.c1, off));
      const float p1 = __builtin_amdgcn_exp2f(fmaf(s[j + 1], a.c1, off));
      lsum += p0 + p1;
      const bf16x2 w2 = {(__bf16)p0, (__bf16)p1};
      pb[j >> 3][(j & 7) >> 1] = __builtin_bit_cast(uint32_t, w2);
    }
    l_run += lsum;
    if (wave < D / 32) {
#pragma unroll
      for (int g = 0; g < 2; g++)
        oacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[g], __builtin_bit_cast(bf16x8, pb[g]), oacc, 0, 0, 0);
    }
    if (++sub_c == nsub) { sub_c = 0; e_c++; }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // no copy may outlive the workgroup's LDS

  // ---- partial record per (pair, split, head-in-group): D floats of unnormalised
  // O, then the running max (base-2 logits) and the running sum ----------------
  const float l_tot = l_run + __shfl_xor(l_run, 32);
  if (n < a.g_q) {
    float* pp = part + n * (D + 2);
    if (wave < D / 32) {
#pragma unroll
      for (int j = 0; j < 16; j++) pp[wave * 32 + (j >> 2) * 8 + h * 4 + (j & 3)] = oacc[j];
    }
    if (wave == 0 && h == 0) { pp[D] = m_run; pp[D + 1] = l_tot; }
  }
}

template <int D, bool DENSE>
static hipError_t launch_decode_t(const S2Args& a, hipStream_t st) {
  using C = DecCfg<D>;
  auto kern = s2_decode_kernel<D, DENSE>;
  static LdsOptIn opt_in;
  if (hipError_t e = allow_dyn_lds((const void*)kern, C::LDS_BYTES, opt_in); e != hipSuccess) return e;
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
  if (p.head_dim == 128) e = dense ? launch_decode_t<128, true>(a, st) : launch_decode_t<128, false>(a, st);
  else e = dense ? launch_decode_t<64, true>(a, st) : launch_decode_t<64, false>(a, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(decode_merge_kernel<uint16_t>, dim3(p.h_q, p.batch), dim3(128), 0, st, partials,
                     (uint16_t*)o, p.h_q, p.h_kv, L.g_q, L.splits, p.head_dim, p.o_stride[0],
                     p.o_stride[1]);
  return hipGetLastError();
}

}  // namespace dash
