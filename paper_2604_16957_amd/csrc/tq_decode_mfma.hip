// Matrix-core fused int4 decode attention for gfx950 (phase 1 of Sec. 3.2: per-chunk partials).
//
// Why matrix cores: with a GQA group of G query heads every stored element is used by G heads;
// at G=8 and d=128 that is 25.6 flop per HBM byte, above the vector-ALU ridge of the chip, so the
// two contractions (Alg. 1 lines 5 and 9) run on v_mfma_f32_16x16x32_f16 and the vector ALU only
// unpacks nibbles, applies the per-group scale/zero-point and does the softmax.
//
// Exactness: codes 0..15 enter the MFMA as fp16 SUBNORMALS (the nibble sits in the low mantissa
// bits, value c*2^-24, or c*2^-20 for a nibble at bit 4) so unpacking is one AND per pair of
// elements; products and sums are exact in the fp32 accumulator.  Scale and zero-point are applied
// outside the contraction in fp32:  q.k^ = sum_g s_g (q_g.c_g - z_g sum(q_g))  and
// sum_t p_t v^_t = sum_t (p_t s_t) c_t - sum_t (p_t s_t) z_t, where the product p_t s_t is rounded
// to fp16 once and the SAME rounded value is used in both terms.
// The matrix core truncates when it adds into the fp32 accumulator (measured: about -0.3 ulp per
// step), and sum_t (p_t s_t) c_t is a sum of positive terms ~200x larger than the result, so the
// codes are centred inside the accumulator: every P V step is followed by a second MFMA of the same
// A operand against the constant -8 (the matrix pipe is otherwise ~15% busy), and the zero-point
// term uses z - 8.  The running sum then stays at the size of the result.
//
// Mapping (one 64-lane wave; lane = 16*kq + c):
//   QK^T is computed transposed, S^T = K Q^T: A = codes (row = token, 8 k-slots per lane = one packed
//   word), B = query.  The 16 B-columns hold G (padded to GP) heads x 16/GP group replicas: column
//   (h, r) only has non-zero query entries on the k-slots of "its" groups, so one accumulator holds
//   the per-group partial dot products of several groups side by side and the per-group scale is
//   applied to NA = (d/32)/(16/GP) accumulators instead of d/32.  Replicas are summed with DPP
//   row rotations.  The S^T accumulator layout (lane = head column, 4 token rows per lane block) is
//   the A-operand layout of P V when P V is computed as rows (h, r) x columns (dims): lane (h, r) of
//   block kq already holds the probabilities of its 8 tokens, so they never move between lanes.
//   For P V the contraction runs over tokens, so each lane needs 8 tokens of one dim in its k-slots:
//   it loads the same packed word of 8 tokens and transposes 8x8 nibbles with two v_perm_b32 stages;
//   the nibble-level stage is free because the unpack masks already separate even and odd nibbles.
//
// Work split: grid (n_splits, H_kv, B), 4 waves per block; the waves of a block interleave
// 32-token supertiles of the chunk, keep private online-softmax state, and are merged through LDS
// so that the block writes one partial (o_c, m_c, l_c) per query head.
#include <type_traits>

#include "tq_internal.h"

namespace tq {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half4v __attribute__((ext_vector_type(4)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

constexpr float kNegBig = -1.0e30f;
constexpr float kSlack = 2.0f;              // log2 units: exp2(score - reference) <= 4
constexpr uint32_t kMaskLo = 0x000F000Fu;   // nibbles 0 and 4 of a word -> fp16 subnormals c * 2^-24
constexpr uint32_t kMaskHi = 0x00F000F0u;   // nibbles 1 and 5           -> c * 2^-20
constexpr uint32_t kNeg8Lo = 0x80088008u;   // two fp16 of value -8 * 2^-24
constexpr uint32_t kNeg8Hi = 0x80808080u;   // two fp16 of value -8 * 2^-20

template <int D, int GP>
struct Cfg {
  static constexpr int NG = D / kGroup;          // quantisation groups per token
  static constexpr int GR = 16 / GP;             // group replicas among the 16 columns / rows
  static constexpr int NA = NG / GR;             // groups handled per lane (accumulators per K tile)
  static constexpr int NJ = NG;                  // K MFMAs per 16-token tile (= packed words per lane)
  static constexpr int NCS = D / 128;            // V column sets (16 packed words each)
  static constexpr bool SWAP = (D == 128 && GP == 8);
  static_assert(NG % GR == 0 && NA >= 1, "unsupported (head_dim, padded GQA) pair");
  // K MFMA j takes, from lane block kq, packed word a_word(j,kq) of group a_group(j,kq) and adds
  // into accumulator acc(j); column replica r of that accumulator stands for group r*NA + acc(j).
  static __device__ constexpr int a_group(int j, int kq) {
    return SWAP ? 2 * (kq >> 1) + (j & 1) : (D == 128 ? kq : 2 * kq + (j >> 2));
  }
  static __device__ constexpr int a_word(int j, int kq) {
    return SWAP ? 2 * (j >> 1) + (kq & 1) : (D == 128 ? j : (j & 3));
  }
  static __device__ constexpr int acc(int j) { return SWAP ? (j & 1) : (D == 128 ? 0 : (NA == 2 ? (j >> 2) : 0)); }
};

// token held by row r of a 16-token K tile (and by the matching k-slots of the P V contraction);
// chosen so that one V load instruction of the wave covers 4 consecutive tokens
__device__ __forceinline__ constexpr int tok_of_row(int r) { return 4 * (r & 3) + (r >> 2); }
__device__ __forceinline__ constexpr int row_of_tok(int t) { return 4 * (t & 3) + (t >> 2); }

__device__ __forceinline__ half8v as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_bit_cast(half8v, uint4v{a, b, c, d});
}
__device__ __forceinline__ half8v unpack_word(uint32_t w) {   // 8 nibbles -> 8 fp16 subnormals
  const uint32_t s = w >> 8;
  return as_half8(w & kMaskLo, w & kMaskHi, s & kMaskLo, s & kMaskHi);
}
__device__ __forceinline__ float4v mfma16(half8v a, half8v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
// reductions over the four 16-lane blocks (lanes l, l^16, l^32, l^48).  The swap builtins return a
// 2-vector; its elements are copied to scalars before any bit_cast (a bit_cast applied directly to
// a vector-element expression reads element 0).
__device__ __forceinline__ void swap32(float x, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ void swap16(float x, float& lo, float& hi) {
  const uint32_t u = __builtin_bit_cast(uint32_t, x);
  const auto r = __builtin_amdgcn_permlane16_swap(u, u, false, false);
  const uint32_t r0 = r[0], r1 = r[1];
  lo = __builtin_bit_cast(float, r0);
  hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float blocks_max(float x) {
  float a, b;
  swap32(x, a, b);
  x = fmaxf(a, b);
  swap16(x, a, b);
  return fmaxf(a, b);
}
__device__ __forceinline__ float blocks_sum(float x) {
  float a, b;
  swap32(x, a, b);
  x = a + b;
  swap16(x, a, b);
  return a + b;
}
template <int ROT>
__device__ __forceinline__ float row_ror_add(float x) {      // x + (x rotated by ROT inside its 16-lane row)
  const int y = __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x120 + ROT, 0xF, 0xF, false);
  return x + __builtin_bit_cast(float, y);
}

// one 32-token supertile of raw loads, kept in registers while in flight
template <int D>
struct Stage {
  uint4v k[2][D / 128];        // K codes: tile, 16-byte chunk
  uint32_t v[D / 128][8];      // V codes: column set, token slot
  uint32_t ksz[D / 64];        // K scale (lanes 0-31) or zero-point (lanes 32-63) of one token
  uint32_t vsz[D / 64];
};

template <int D, int GP>
__global__ __launch_bounds__(256, 2) void decode_partial_mfma_kernel(DecodeParams p) {
  using C = Cfg<D, GP>;
  constexpr int NG = C::NG, NA = C::NA, NJ = C::NJ, NCS = C::NCS;
  constexpr int TB = D / 2;                       // bytes of codes per token
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, kq = lane >> 4;
  const int hl = c % GP, rep = c / GP;            // head and group replica of this lane's column / row
  const int split = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
  const int G = p.gqa;

  // wave-private LDS: scales / zero-points of one supertile as [tile][group][row]; K as fp16,
  // V as fp32 with the zero-point already shifted by -8.  Then the block-shared merge area.
  __shared__ __attribute__((aligned(16))) _Float16 lds_ks[4][2][NG][16];
  __shared__ __attribute__((aligned(16))) _Float16 lds_kz[4][2][NG][16];
  __shared__ __attribute__((aligned(16))) float lds_vs[4][2][NG][16];
  __shared__ __attribute__((aligned(16))) float lds_vz[4][2][NG][16];
  __shared__ float lds_f[4][16];
  __shared__ float lds_o[4][GP][D];
  __shared__ float lds_zc[4][GP][NG];
  __shared__ float lds_m[4][GP], lds_l[4][GP];

  // ---- addressing: wave-uniform bases (scalar registers) + per-lane 32-bit byte offsets
  const int64_t row0 = (int64_t)(b * p.n_kv_heads + kv) * p.row_stride;
  const int begin = split * p.tokens_per_split;
  const int end = min(p.seq_len, begin + p.tokens_per_split);
  const int n_full = (end - begin) >> 5;          // whole 32-token supertiles of this chunk
  const bool has_tail = ((end - begin) & 31) != 0;  // only the sequence's last supertile can be ragged
  const int last_tok = p.seq_len - 1;
  const char* kc_row = reinterpret_cast<const char*>(p.k_codes) + row0 * TB;
  const char* vc_row = reinterpret_cast<const char*>(p.v_codes) + row0 * TB;
  const uint32_t koff = tok_of_row(c) * TB + kq * (D / 8);
  const uint32_t voff = kq * TB + c * 4 * NCS;
  const int sz_tok = lane & 31;                   // token (within the supertile) whose scales this lane fetches
  const int which = lane >> 5;                    // 0: this lane fetches scales, 1: zero-points
  const char* ksz_row = reinterpret_cast<const char*>(which ? p.k_zero : p.k_scale) + row0 * (NG * 2);
  const char* vsz_row = reinterpret_cast<const char*>(which ? p.v_zero : p.v_scale) + row0 * (NG * 2);

  auto load_stage = [&](Stage<D>& st, int sidx, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    const int base = begin + sidx * 32;
    if constexpr (!TAIL) {
      const char* kb = kc_row + (int64_t)base * TB;
      const char* vb = vc_row + (int64_t)base * TB;
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int ch = 0; ch < D / 128; ++ch)
          st.k[t][ch] = *reinterpret_cast<const uint4v*>(kb + koff + t * 16 * TB + ch * 16);
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int cs = 0; cs < NCS; ++cs)
          st.v[cs][i] = *reinterpret_cast<const uint32_t*>(vb + voff + (16 * (i >> 2) + 4 * (i & 3)) * TB + cs * 4);
      const int64_t so = (int64_t)(base + sz_tok) * (NG * 2);
#pragma unroll
      for (int i = 0; i < D / 64; ++i) {
        st.ksz[i] = *reinterpret_cast<const uint32_t*>(ksz_row + so + i * 4);
        st.vsz[i] = *reinterpret_cast<const uint32_t*>(vsz_row + so + i * 4);
      }
    } else {                                      // ragged tail: clamp every token to the last valid one
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int tok = min(base + 16 * t + tok_of_row(c), last_tok);
#pragma unroll
        for (int ch = 0; ch < D / 128; ++ch)
          st.k[t][ch] = *reinterpret_cast<const uint4v*>(kc_row + (int64_t)tok * TB + kq * (D / 8) + ch * 16);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int tok = min(base + 16 * (i >> 2) + 4 * (i & 3) + kq, last_tok);
#pragma unroll
        for (int cs = 0; cs < NCS; ++cs)
          st.v[cs][i] = *reinterpret_cast<const uint32_t*>(vc_row + (int64_t)tok * TB + c * 4 * NCS + cs * 4);
      }
      const int64_t so = (int64_t)min(base + sz_tok, last_tok) * (NG * 2);
#pragma unroll
      for (int i = 0; i < D / 64; ++i) {
        st.ksz[i] = *reinterpret_cast<const uint32_t*>(ksz_row + so + i * 4);
        st.vsz[i] = *reinterpret_cast<const uint32_t*>(vsz_row + so + i * 4);
      }
    }
  };

  // first loads go out before the query set-up so that their latency overlaps it
  Stage<D> stA, stB;
  if (wave < n_full) load_stage(stA, wave, std::false_type{});

  // ---- query operands (Alg. 1 line 1 is folded into the exp2 argument instead of the query)
  const _Float16* qh = p.q + (int64_t)(b * p.n_q_heads + kv * G + (hl < G ? hl : 0)) * D;
  half8v qb[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int g = C::a_group(j, kq), w = C::a_word(j, kq);
    const bool mine = (g == rep * NA + C::acc(j)) && hl < G;
    half8v x = *reinterpret_cast<const half8v*>(qh + g * kGroup + w * 8);
    // k-slot order of unpack_word: nibbles 0,4,1,5,2,6,3,7; the "hi" slots carry c*2^-20, so pre-divide by 16
    half8v y = {x[0], x[4], x[1] * (_Float16)0.0625f, x[5] * (_Float16)0.0625f,
                x[2], x[6], x[3] * (_Float16)0.0625f, x[7] * (_Float16)0.0625f};
    if (!mine) y = half8v{0, 0, 0, 0, 0, 0, 0, 0};
    qb[j] = y;
  }
  float qsum[NA];                                 // 2^-24 * sum of q over each of this lane's groups
#pragma unroll
  for (int a = 0; a < NA; ++a) {
    float s = 0.0f;
    const half8v* qg = reinterpret_cast<const half8v*>(qh + (rep * NA + a) * kGroup);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const half8v x = qg[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (float)x[e];
    }
    qsum[a] = (hl < G) ? s * 0x1p-24f : 0.0f;
  }
  const float kappa = p.scale_log2 * 0x1p24f;     // raw accumulator units -> log2 units
  const float slack = kSlack / kappa;             // the rescale slack in raw units

  // ---- running state
  float m_run = kNegBig;                          // running max of this lane's head, raw units
  float l_run = 0.0f;                             // this lane's share of sum(exp)
  float zacc[NA];
#pragma unroll
  for (int a = 0; a < NA; ++a) zacc[a] = 0.0f;
  float4v oacc[NCS][8][NA];
#pragma unroll
  for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int a = 0; a < NA; ++a) oacc[cs][m][a] = float4v{0, 0, 0, 0};

  const half8v neg8_lo = as_half8(kNeg8Lo, kNeg8Lo, kNeg8Lo, kNeg8Lo);
  const half8v neg8_hi = as_half8(kNeg8Hi, kNeg8Hi, kNeg8Hi, kNeg8Hi);

  // LDS destinations of this lane's scale / zero-point token (constant over the loop)
  const int sz_slot = (sz_tok >> 4) * (NG * 16) + row_of_tok(sz_tok & 15);
  _Float16* const k_dst = (which ? &lds_kz[wave][0][0][0] : &lds_ks[wave][0][0][0]) + sz_slot;
  float* const v_dst = (which ? &lds_vz[wave][0][0][0] : &lds_vs[wave][0][0][0]) + sz_slot;
  const float v_shift = which ? -8.0f : 0.0f;

  auto process = [&](const Stage<D>& cur, int sidx, auto tail_tag) {
    constexpr bool TAIL = decltype(tail_tag)::value;
    // -- scales and zero-points: one token per lane -> LDS, transposed to [group][row]
#pragma unroll
    for (int i = 0; i < D / 64; ++i) {
      const half2v ks = __builtin_bit_cast(half2v, cur.ksz[i]);
      const half2v vs = __builtin_bit_cast(half2v, cur.vsz[i]);
      k_dst[(2 * i) * 16] = ks[0];
      k_dst[(2 * i + 1) * 16] = ks[1];
      v_dst[(2 * i) * 16] = (float)vs[0] + v_shift;
      v_dst[(2 * i + 1) * 16] = (float)vs[1] + v_shift;
    }
    __builtin_amdgcn_wave_barrier();   // LDS is in order per wave; only the compiler must not reorder

    // -- scores, S^T = K Q^T, per-group scale and zero-point applied in fp32 (raw units: 2^-24)
    float sc[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      uint32_t w[NJ];
      if constexpr (C::SWAP) {
        auto s01 = __builtin_amdgcn_permlane16_swap(cur.k[t][0][0], cur.k[t][0][1], false, false);
        auto s23 = __builtin_amdgcn_permlane16_swap(cur.k[t][0][2], cur.k[t][0][3], false, false);
        w[0] = s01[0]; w[1] = s01[1]; w[2] = s23[0]; w[3] = s23[1];
      } else {
#pragma unroll
        for (int j = 0; j < NJ; ++j) w[j] = cur.k[t][j >> 2][j & 3];
      }
      float4v acc[NA];
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[a] = float4v{0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[C::acc(j)] = mfma16(unpack_word(w[j]), qb[j], acc[C::acc(j)]);
      float part[4] = {0, 0, 0, 0};
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        const int g = rep * NA + a;
        const half4v s4 = *reinterpret_cast<const half4v*>(&lds_ks[wave][t][g][4 * kq]);
        const half4v z4 = *reinterpret_cast<const half4v*>(&lds_kz[wave][t][g][4 * kq]);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const float e = fmaf(-(float)z4[i], qsum[a], acc[a][i]);
          part[i] = fmaf((float)s4[i], e, part[i]);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        float x = part[i];
        if constexpr (C::GR >= 2) x = row_ror_add<8>(x);
        if constexpr (C::GR >= 4) x = row_ror_add<4>(x);
        if constexpr (C::GR >= 8) x = row_ror_add<2>(x);
        if constexpr (TAIL) {
          const int tok = begin + sidx * 32 + 16 * t + tok_of_row(4 * kq + i);
          x = (tok < end) ? x : -INFINITY;
        }
        sc[t][i] = x;
      }
    }

    // -- online softmax over the 32 tokens (Alg. 1 lines 6-7, 10), block-wise.  m_run is a per-head
    //    REFERENCE, not the exact running max: it only moves when some score exceeds it by more than
    //    kSlack (log2 units), so exp2(score - m_run) <= 2^kSlack = 4 and p * s_v stays inside fp16 for
    //    every representable scale, while the accumulator rescale (Alg. 1 lines 7, 9) becomes rare.
    //    Any reference gives the same o / l, and the chunk merge (Eq. 6) accepts any m_c.
    const float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                           fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    if (__builtin_amdgcn_ballot_w64(mx > m_run + slack) != 0) {   // wave-uniform, rare
      const float m_new = fmaxf(m_run, blocks_max(mx));
      const float f = __builtin_amdgcn_exp2f((m_run - m_new) * kappa);
      m_run = m_new;
      l_run *= f;
#pragma unroll
      for (int a = 0; a < NA; ++a) zacc[a] *= f;
      if (kq == 0) lds_f[wave][c] = f;                       // c = (head, replica): same f for all replicas
      __builtin_amdgcn_wave_barrier();
      float fr[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) fr[i] = lds_f[wave][(4 * kq + i) % GP];
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
          for (int a = 0; a < NA; ++a)
#pragma unroll
            for (int i = 0; i < 4; ++i) oacc[cs][m][a][i] *= fr[i];
    }
    const float mk = m_run * kappa;
    float pr[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pr[t][i] = __builtin_amdgcn_exp2f(fmaf(sc[t][i], kappa, -mk));
        l_run += pr[t][i];
      }

    // -- P V with rows (head, replica): A = fp16(p * s_v) for the lane's group of each pass
    half8v pa[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a) {
      const int g = rep * NA + a;
      const float4v s0 = *reinterpret_cast<const float4v*>(&lds_vs[wave][0][g][4 * kq]);
      const float4v s1 = *reinterpret_cast<const float4v*>(&lds_vs[wave][1][g][4 * kq]);
      const float4v z0 = *reinterpret_cast<const float4v*>(&lds_vz[wave][0][g][4 * kq]);
      const float4v z1 = *reinterpret_cast<const float4v*>(&lds_vz[wave][1][g][4 * kq]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {             // fma(p, s, 0) rounded once to fp16 (v_fma_mixlo/hi_f16)
        pa[a][2 * i] = (_Float16)__builtin_fmaf(pr[0][i], s0[i], 0.0f);
        pa[a][2 * i + 1] = (_Float16)__builtin_fmaf(pr[1][i], s1[i], 0.0f);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {             // zero-point term from the SAME rounded operand
        zacc[a] = fmaf((float)pa[a][2 * i], z0[i], zacc[a]);
        zacc[a] = fmaf((float)pa[a][2 * i + 1], z1[i], zacc[a]);
      }
    }

    // -- V codes: 8 tokens x 8 nibbles per lane -> 8 dims x 8 tokens (two byte-permute stages),
    //    consumed two dims at a time so that few unpacked operands are live
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs) {
      uint32_t x[8], y[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[i] = __builtin_amdgcn_perm(cur.v[cs][i + 4], cur.v[cs][i], 0x05040100u);
        x[i + 4] = __builtin_amdgcn_perm(cur.v[cs][i + 4], cur.v[cs][i], 0x07060302u);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        if ((i & 2) == 0) {
          y[i] = __builtin_amdgcn_perm(x[i + 2], x[i], 0x06020400u);
          y[i + 2] = __builtin_amdgcn_perm(x[i + 2], x[i], 0x07030501u);
        }
      }
      // y[2I+a], nibble 2M+cc = token slot (2M+a), dim (2I+cc) of the packed word
#pragma unroll
      for (int I = 0; I < 4; ++I) {
        const uint32_t r0 = y[2 * I], r1 = y[2 * I + 1], s0 = r0 >> 8, s1 = r1 >> 8;
        const half8v v_even = as_half8(r0 & kMaskLo, r1 & kMaskLo, s0 & kMaskLo, s1 & kMaskLo);
        const half8v v_odd = as_half8(r0 & kMaskHi, r1 & kMaskHi, s0 & kMaskHi, s1 & kMaskHi);
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          oacc[cs][2 * I][a] = mfma16(pa[a], v_even, oacc[cs][2 * I][a]);
          oacc[cs][2 * I + 1][a] = mfma16(pa[a], v_odd, oacc[cs][2 * I + 1][a]);
        }
#pragma unroll
        for (int a = 0; a < NA; ++a) {
          oacc[cs][2 * I][a] = mfma16(pa[a], neg8_lo, oacc[cs][2 * I][a]);
          oacc[cs][2 * I + 1][a] = mfma16(pa[a], neg8_hi, oacc[cs][2 * I + 1][a]);
        }
      }
    }
  };

  // ---- main loop over this wave's whole supertiles (wave, wave+4, ...), two register stages in ping-pong
  for (int sidx = wave; sidx < n_full; sidx += 8) {
    if (sidx + 4 < n_full) load_stage(stB, sidx + 4, std::false_type{});
    process(stA, sidx, std::false_type{});
    if (sidx + 4 >= n_full) break;
    if (sidx + 8 < n_full) load_stage(stA, sidx + 8, std::false_type{});
    process(stB, sidx + 4, std::false_type{});
  }
  if (has_tail && (n_full & 3) == wave) {                    // the ragged last supertile of the sequence
    load_stage(stA, n_full, std::true_type{});
    process(stA, n_full, std::true_type{});
  }

  // ---- wave result -> LDS
  const bool active = wave < n_full + (has_tail ? 1 : 0);
  const float l_tot = blocks_sum(l_run);
#pragma unroll
  for (int a = 0; a < NA; ++a) zacc[a] = blocks_sum(zacc[a]);
  if (kq == 0 && hl < GP) {
    if (rep == 0) {
      lds_m[wave][hl] = active ? m_run * kappa : kNegBig;
      lds_l[wave][hl] = active ? l_tot : 0.0f;
    }
#pragma unroll
    for (int a = 0; a < NA; ++a) lds_zc[wave][hl][rep * NA + a] = zacc[a];
  }
#pragma unroll
  for (int cs = 0; cs < NCS; ++cs) {
    const int word = c * NCS + cs;                // packed word (8 dims) this lane's column stands for
    const int g = word >> 2;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = 4 * kq + i, h = r % GP, a_mine = g - (r / GP) * NA;
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        if (a == a_mine) {
#pragma unroll
          for (int m = 0; m < 8; ++m)
            lds_o[wave][h][word * 8 + m] = oacc[cs][m][a][i] * ((m & 1) ? 0x1p20f : 0x1p24f);
        }
      }
    }
  }
  __syncthreads();

  // ---- merge the four waves, write one partial per query head (Sec. 3.2)
  for (int idx = threadIdx.x; idx < G * D; idx += 256) {
    const int h = idx / D, j = idx % D;
    float mg = lds_m[0][h];
#pragma unroll
    for (int w = 1; w < 4; ++w) mg = fmaxf(mg, lds_m[w][h]);
    float num = 0.0f, den = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float e = __builtin_amdgcn_exp2f(lds_m[w][h] - mg);
      num = fmaf(lds_o[w][h][j] - lds_zc[w][h][j >> 5], e, num);
      den = fmaf(lds_l[w][h], e, den);
    }
    const int64_t ph = (int64_t)(b * p.n_q_heads + kv * G + h) * p.n_splits + split;
    p.part_o[ph * D + j] = num;
    if (j == 0) { p.part_ml[ph * 2] = mg; p.part_ml[ph * 2 + 1] = den; }
  }
}

int padded_gqa(int head_dim, int gqa) {
  if (head_dim == 128) return gqa <= 4 ? 4 : (gqa <= 8 ? 8 : 0);
  return gqa <= 2 ? 2 : (gqa <= 4 ? 4 : 0);
}

}  // namespace

bool mfma_supported(int head_dim, int gqa) {
  return (head_dim == 128 || head_dim == 256) && gqa >= 1 && padded_gqa(head_dim, gqa) != 0;
}

hipError_t launch_partial_mfma(const DecodeParams& p, int batch, int head_dim, hipStream_t s) {
  const dim3 grid(p.n_splits, p.n_kv_heads, batch), block(256);
  const int gp = padded_gqa(head_dim, p.gqa);
  if (head_dim == 128 && gp == 8) hipLaunchKernelGGL((decode_partial_mfma_kernel<128, 8>), grid, block, 0, s, p);
  else if (head_dim == 128 && gp == 4) hipLaunchKernelGGL((decode_partial_mfma_kernel<128, 4>), grid, block, 0, s, p);
  else if (head_dim == 256 && gp == 4) hipLaunchKernelGGL((decode_partial_mfma_kernel<256, 4>), grid, block, 0, s, p);
  else if (head_dim == 256 && gp == 2) hipLaunchKernelGGL((decode_partial_mfma_kernel<256, 2>), grid, block, 0, s, p);
  else return hipErrorNotSupported;
  return hipGetLastError();
}

}  // namespace tq
