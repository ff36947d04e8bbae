// Generic vector-ALU decode attention: the fused int4 kernel for any GQA ratio, and (same
// template, fp16 loader) the attention phase of the dequantize-then-attend comparator.
// Also the chunk merge of Sec. 3.2, Eq. 6.
//
// Work split: grid (n_splits, H_kv * head_tiles, B); a block of four 64-wide waves owns one
// chunk of one KV head.  D/8 lanes cooperate on a token (each lane holds 8 consecutive
// head_dim elements: one 32-bit word of codes, or 16 B of fp16), so a wave walks 64/(D/8)
// tokens at a time and every token-slot keeps its own online-softmax state (m, l, o) for up to
// 8 query heads of the GQA group in registers (Alg. 1, the loop over the tokens).  Slots are merged with
// wave shuffles, waves through LDS, and the block writes ONE un-normalised partial
// (o_c, m_c, l_c) per query head (Sec. 3.2).  Scores live in log2 units so exp is exp2.
#include <algorithm>
#include <type_traits>

#include "tq_internal.h"

namespace tq {
namespace {

// query heads per block pass: 8, or 4 at d=512 (the block merge keeps 4 waves x heads x d floats in LDS)
constexpr int head_tile(int d) { return d <= 256 ? 8 : 4; }
constexpr float kNegBig = -1.0e30f;  // "no token seen yet" running max (finite: no inf-inf)

union Pack16 { uint4 v; half_t h[8]; };

template <int D, bool DENSE>
__global__ __launch_bounds__(256) void decode_partial_valu_kernel(DecodeParams p) {
  constexpr int LPT = D / 8;           // lanes per token
  constexpr int TPW = 64 / LPT;        // token slots per wave
  constexpr int SPB = 4 * TPW;         // token slots per block
  constexpr int kHeadTile = head_tile(D);

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int sub = lane % LPT;          // which 8-element piece of the head vector
  const int slot = wave * TPW + lane / LPT;
  const int NG = D / p.group;          // groups per token (the group size is a launch parameter: 32, 64 or 128)
  const int grp = sub * 8 / p.group;   // quantisation group of that piece

  int split = blockIdx.x, b = blockIdx.z, tokens_per_split = p.tokens_per_split, part_stride = p.n_splits;
  if (p.var_chunks > 0) {                         // per-sequence lengths: which (sequence, chunk) is this block's
    VarPlan vp;
    if (!var_plan(p, blockIdx.x, vp)) return;
    split = vp.chunk;
    b = vp.b;
    tokens_per_split = vp.chunk_tokens;
    part_stride = kMaxSplits;
  }
  const int head_tiles = (p.gqa + kHeadTile - 1) / kHeadTile;
  const int kv = blockIdx.y / head_tiles;
  const int tile = blockIdx.y % head_tiles;
  const int h0 = kv * p.gqa + tile * kHeadTile;          // first query head of this pass
  const int nh = min(kHeadTile, p.gqa - tile * kHeadTile);

  // query piece for each head, pre-multiplied by attn_scale * log2(e) (Alg. 1, the query pre-scaling)
  float qf[kHeadTile][8];
#pragma unroll
  for (int h = 0; h < kHeadTile; ++h) {
    if (h < nh) {
      Pack16 u;
      u.v = *reinterpret_cast<const uint4*>(p.q + ((int64_t)(b * p.n_q_heads + h0 + h) * D + sub * 8));
#pragma unroll
      for (int j = 0; j < 8; ++j) qf[h][j] = (float)u.h[j] * p.scale_log2;
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) qf[h][j] = 0.0f;
    }
  }

  float m[kHeadTile], l[kHeadTile], o[kHeadTile][8];
#pragma unroll
  for (int h = 0; h < kHeadTile; ++h) {
    m[h] = kNegBig;
    l[h] = 0.0f;
#pragma unroll
    for (int j = 0; j < 8; ++j) o[h][j] = 0.0f;
  }

  const int begin = split * tokens_per_split;
  const int seq = p.seq_lens ? var_len(p, b) : p.seq_len;
  if (begin >= seq) return;                              // chunk past the end of its sequence: nothing to emit
  const int end = min(seq, begin + tokens_per_split);
  const int start = p.seq_lens ? var_start(p, b) : p.start;
  // paged cache under a window: the chunks count from a supertile boundary up to 31 tokens before the window
  const int lead = (p.block_table && p.seq_lens) ? var_first(p, b) - start : 0;
  const int64_t row0 = (int64_t)(b * p.n_kv_heads + kv) * p.row_stride + start;

  // row of the arrays that holds token t of this sequence (clamped to the chunk: always a written token)
  auto row_of = [&](int t) -> int64_t {
    const int tc = t < end ? t : end - 1;
    if (p.block_table) {                                 // paged cache: the page the block table names for this token
      const int ta = start + tc;
      const int page = p.block_table[(int64_t)b * p.max_blocks + (ta >> p.page_shift)];
      return ((int64_t)page * p.n_kv_heads + kv) * p.row_stride + (ta & ((1 << p.page_shift) - 1));
    }
    return row0 + tc;
  };
  // Dense fp16 rows (the comparator): 32 bytes per lane and token are all a pass asks of the memory system, far
  // too little in flight to keep it busy, so the loads run kAhead passes ahead of the arithmetic in a small
  // register ring (a pass past the end of the chunk re-reads its last row).
  constexpr int kAhead = DENSE ? 3 : 0;
  uint4 k_raw[kAhead + 1], v_raw[kAhead + 1];
  if constexpr (DENSE) {
#pragma unroll
    for (int s = 0; s < kAhead; ++s) {
      const int64_t row = row_of(begin + s * SPB + slot);
      k_raw[s] = *reinterpret_cast<const uint4*>(p.k_dense + row * D + sub * 8);
      v_raw[s] = *reinterpret_cast<const uint4*>(p.v_dense + row * D + sub * 8);
    }
  }

  for (int t0 = begin; t0 < end; t0 += SPB) {
    const int t = t0 + slot;
    const bool valid = t < end && t >= lead;
    const int64_t row = row_of(t);

    float kf[8], vf[8];
    if constexpr (DENSE) {
      {
        const int64_t ahead = row_of(t + kAhead * SPB);
        k_raw[kAhead] = *reinterpret_cast<const uint4*>(p.k_dense + ahead * D + sub * 8);
        v_raw[kAhead] = *reinterpret_cast<const uint4*>(p.v_dense + ahead * D + sub * 8);
      }
      Pack16 ku, vu;
      ku.v = k_raw[0];
      vu.v = v_raw[0];
#pragma unroll
      for (int s = 0; s < kAhead; ++s) { k_raw[s] = k_raw[s + 1]; v_raw[s] = v_raw[s + 1]; }
#pragma unroll
      for (int j = 0; j < 8; ++j) { kf[j] = (float)ku.h[j]; vf[j] = (float)vu.h[j]; }
    } else {
      const uint32_t kw = *reinterpret_cast<const uint32_t*>(p.k_codes + row * (D / 2) + sub * 4);
      const uint32_t vw = *reinterpret_cast<const uint32_t*>(p.v_codes + row * (D / 2) + sub * 4);
      const float ks = (float)p.k_scale[row * NG + grp], kz = (float)p.k_zero[row * NG + grp];
      const float vs = (float)p.v_scale[row * NG + grp], vz = (float)p.v_zero[row * NG + grp];
#pragma unroll
      for (int j = 0; j < 8; ++j) {                      // dequant4: nibble j, then (q - z) s
        kf[j] = ((float)((kw >> (4 * j)) & 0xFu) - kz) * ks;
        vf[j] = ((float)((vw >> (4 * j)) & 0xFu) - vz) * vs;
      }
    }

#pragma unroll
    for (int h = 0; h < kHeadTile; ++h) {
      float a = 0.0f;
#pragma unroll
      for (int j = 0; j < 8; ++j) a = fmaf(qf[h][j], kf[j], a);
#pragma unroll
      for (int off = 1; off < LPT; off <<= 1) a += __shfl_xor(a, off);   // Alg. 1, the score
      const float m_new = valid ? fmaxf(m[h], a) : m[h];
      // Alg. 1's correction factor is 1 unless this token raises the running maximum of some slot of the wave,
      // which soon becomes rare: the accumulator is only rescaled then
      if (__builtin_amdgcn_ballot_w64(m_new > m[h]) != 0) {
        const float corr = __builtin_amdgcn_exp2f(m[h] - m_new);
        l[h] *= corr;
#pragma unroll
        for (int j = 0; j < 8; ++j) o[h][j] *= corr;
        m[h] = m_new;
      }
      const float pr = valid ? __builtin_amdgcn_exp2f(a - m_new) : 0.0f;
      l[h] += pr;
#pragma unroll
      for (int j = 0; j < 8; ++j) o[h][j] = fmaf(pr, vf[j], o[h][j]);
    }
  }

  // merge the token slots of this wave (same head, same dims, different tokens)
#pragma unroll
  for (int off = LPT; off < 64; off <<= 1) {
#pragma unroll
    for (int h = 0; h < kHeadTile; ++h) {
      const float m_o = __shfl_xor(m[h], off);
      const float m_n = fmaxf(m[h], m_o);
      const float wa = exp2f(m[h] - m_n), wb = exp2f(m_o - m_n);
      l[h] = l[h] * wa + __shfl_xor(l[h], off) * wb;
#pragma unroll
      for (int j = 0; j < 8; ++j) o[h][j] = o[h][j] * wa + __shfl_xor(o[h][j], off) * wb;
      m[h] = m_n;
    }
  }

  __shared__ float lds_o[4][kHeadTile][D];
  __shared__ float lds_m[4][kHeadTile], lds_l[4][kHeadTile];
  if (lane < LPT) {
#pragma unroll
    for (int h = 0; h < kHeadTile; ++h) {
#pragma unroll
      for (int j = 0; j < 8; ++j) lds_o[wave][h][sub * 8 + j] = o[h][j];
      if (lane == 0) { lds_m[wave][h] = m[h]; lds_l[wave][h] = l[h]; }
    }
  }
  __syncthreads();

  for (int idx = threadIdx.x; idx < nh * D; idx += 256) {
    const int h = idx / D, j = idx % D;
    float mg = lds_m[0][h];
#pragma unroll
    for (int w = 1; w < 4; ++w) mg = fmaxf(mg, lds_m[w][h]);
    float num = 0.0f, den = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float e = exp2f(lds_m[w][h] - mg);
      num = fmaf(lds_o[w][h][j], e, num);
      den = fmaf(lds_l[w][h], e, den);
    }
    const int64_t ph = ((int64_t)(b * p.n_q_heads + h0 + h) * part_stride + split);
    p.part_o[ph * D + j] = num;
    if (j == 0) { p.part_ml[ph * 2] = mg; p.part_ml[ph * 2 + 1] = den; }
  }
}

// Append-and-attend in a merge kernel: the step's new token of (row b, KV head kv), quantised with the device
// function the append kernel uses (same bits; Sec. 2.1) by the block's first 8 * D / 32 threads (four lanes per
// group of 32 elements, eight elements each, K and V), stored at `append_pos` if `store`, and left dequantised
// (Eq. 3) in hat[0] (K) and hat[1] (V).  The caller synchronises the block before reading hat.
template <int D>
__device__ inline void quantize_new_token(const DecodeParams& p, int b, int kv, int append_pos, int tid, bool store,
                                          float (*hat)[D]) {
  constexpr int NG = D / kGroup;
  if (tid < 8 * NG) {
    const int which = tid / (4 * NG), g = (tid >> 2) % NG, part4 = tid & 3;   // 0 = K, 1 = V
    const half_t* src = (which ? p.v_new : p.k_new) + (int64_t)(b * p.n_kv_heads + kv) * D + g * kGroup + part4 * 8;
    Pack16 u;
    u.v = *reinterpret_cast<const uint4*>(src);
    float x[8];
#pragma unroll
    for (int jj = 0; jj < 8; ++jj) x[jj] = (float)u.h[jj];
    float mn = x[0], mx = x[0];
#pragma unroll
    for (int jj = 1; jj < 8; ++jj) { mn = fminf(mn, x[jj]); mx = fmaxf(mx, x[jj]); }
    // the group's min and max: over the four lanes (exact in any order)
    mn = fminf(mn, __shfl_xor(mn, 1)); mx = fmaxf(mx, __shfl_xor(mx, 1));
    mn = fminf(mn, __shfl_xor(mn, 2)); mx = fmaxf(mx, __shfl_xor(mx, 2));
    half_t s16, z16;
    quantize_scale_zero(mn, mx, s16, z16);
    const float sf = (float)s16, zf = (float)z16;
    // Eq. 3 by the shortcut of the append kernel, redone with correctly rounded divides where it could matter
    // (same bits either way; the divides are most of this function's time, which the merge kernel waits for)
    const QuantFast fast = quantize_fast_setup(sf, zf, fmaxf(fabsf(mn), fabsf(mx)));
    float far = 0.0f;
    uint32_t w = quantize_word_fast(u.h, fast, far);
    if (quantize_fast_in_doubt(far, fast)) w = quantize_word(x, sf, zf);
    if (store) {
      int64_t row = (int64_t)(b * p.n_kv_heads + kv) * p.row_stride + append_pos;
      if (p.block_table) {                         // paged cache: the page the block table names for that position
        const int page = p.block_table[(int64_t)b * p.max_blocks + (append_pos >> p.page_shift)];
        row = ((int64_t)page * p.n_kv_heads + kv) * p.row_stride + (append_pos & ((1 << p.page_shift) - 1));
      }
      uint8_t* codes = const_cast<uint8_t*>(which ? p.v_codes : p.k_codes) + row * (D / 2) + g * (kGroup / 2);
      reinterpret_cast<uint32_t*>(codes)[part4] = w;
      if (part4 == 0) const_cast<half_t*>(which ? p.v_scale : p.k_scale)[row * NG + g] = s16;
      if (part4 == 1) const_cast<half_t*>(which ? p.v_zero : p.k_zero)[row * NG + g] = z16;
    }
#pragma unroll
    for (int jj = 0; jj < 8; ++jj)
      hat[which][g * kGroup + part4 * 8 + jj] = ((float)((w >> (4 * jj)) & 0xFu) - zf) * sf;   // Eq. 3
  }
}

// Eq. 6 with un-normalised chunk outputs: o = sum_c e^{m_c-m_g} o_c / sum_c e^{m_c-m_g} l_c.
// One block per query head.  The chunk weights are computed once (one chunk per thread) and kept
// in LDS; the weighted sum over chunks is split over 256/D thread groups with independent,
// unrolled loads, so the kernel is a handful of memory round trips long.
// THREADS: 256 (d = 512: 1024, two threads per output element, so that 128 chunks are four rounds of loads per
// thread, not eight); for launches of thousands of blocks with few chunks each, D threads: twice as many blocks
// fit a compute unit, and such a launch is as long as its rounds of blocks.
// SLICES: blocks that share a query head, each with D / SLICES of its output elements (d = 512 with at most 64
// outputs: four or eight blocks of 512 threads per head: with few heads the partials, 256 KB a head at 128 chunks,
// are otherwise pulled in by as many compute units as there are heads).  Every slice works out the chunk weights and,
// when appending, the new token's score for itself; slice 0 stores the token.
template <int D, int THREADS, int SLICES = 1>
__global__ __launch_bounds__(THREADS) void reduce_kernel(DecodeParams p) {
  constexpr int WAVES = THREADS / 64;
  constexpr int DS = D / SLICES;                  // output elements of this block
  static_assert(D % SLICES == 0 && THREADS % DS == 0 && THREADS >= kMaxSplits && THREADS >= 8 * (D / kGroup),
                "one thread per chunk, per lane of the appender");
  constexpr int PARTS = THREADS / DS;
  // b: row of the [B * n_queries][H_q] outputs (one per query token of every sequence)
  const int h = blockIdx.x / SLICES, slice = blockIdx.x % SLICES, b = blockIdx.y, tid = threadIdx.x;
  const int part_stride = p.var_chunks > 0 ? kMaxSplits : p.n_splits;   // chunk slots a row has in the workspace
  const int64_t ph0 = (int64_t)(b * p.n_q_heads + h) * part_stride;
  __shared__ float w_c[kMaxSplits];
  __shared__ float red_m[WAVES], red_l[WAVES];
  __shared__ float acc_part[PARTS][DS];

  // chunks that exist for this sequence: all of them, or those that start before its own end (with a plan made
  // on the device: its chunk length, which the decode kernel left in the workspace)
  int n = p.n_splits;
  int append_pos = p.append_pos;
  if (p.seq_lens) {
    const int sequence = p.n_queries > 1 ? b / p.n_queries : b;
    const int c = p.var_chunks > 0 ? *p.plan : p.tokens_per_split;
    n = min(n, (var_len(p, sequence) + c - 1) / c);
    // append-and-attend: the sequence's length counts the new token, which goes to its last position; a
    // sequence with no cached token has no chunk (the one the decode kernel made up is ignored)
    const int total = max(1, min(p.seq_lens[sequence], p.seq_len));
    append_pos = total - 1;
    if (total + p.len_bias < 1) n = 0;
  }
  // The first chunks of this thread's output element, and the chunks' (m, l), are asked for before anything
  // else: they do not depend on the weights, so the kernel is about one memory round trip long (two with
  // per-sequence lengths, which have to arrive first).
  constexpr int FIRST = 16;
  const int jl = tid % DS, j = slice * DS + jl, part = tid / DS;
  const float* src = p.part_o + ph0 * D + j;
  float pre[FIRST];
#pragma unroll
  for (int u = 0; u < FIRST; ++u) pre[u] = src[(int64_t)min(part + u * PARTS, max(n, 1) - 1) * D];
  float2 ml = {kNegBig, 0.0f};
  if (tid < n) ml = *reinterpret_cast<const float2*>(p.part_ml + (ph0 + tid) * 2);
  const float m = tid < n ? ml.x : kNegBig, l = tid < n ? ml.y : 0.0f;

  // Append-and-attend in the merge (p.k_new set; one query token, common length): the step's new token is not in
  // the chunks.  Every block quantises it for its KV head with the device function the append kernel uses (same
  // bits; Sec. 2.1), the block of the group's first query head stores it, and its attention term enters Eq. 6
  // as one more chunk: m = its score, l = 1, o = its dequantised V.
  __shared__ float hat[2][D];
  __shared__ float red_a[WAVES];
  const bool appending = p.k_new != nullptr;
  float a_new = kNegBig;
  // (the chunk maxima of each wave go to LDS ahead of the barriers below, which then serve them as well)
  float mw = m;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) mw = fmaxf(mw, __shfl_xor(mw, off));
  if ((tid & 63) == 0) red_m[tid >> 6] = mw;
  if (!appending) __syncthreads();
  if (appending) {
    static_assert(THREADS >= D, "one query element per thread");
    // (asked for with everything else above, not behind the block barrier below: one memory round trip less)
    const float q_e = tid < D ? (float)p.q[(int64_t)(b * p.n_q_heads + h) * D + tid] : 0.0f;
    const int kv = h / p.gqa;
    quantize_new_token<D>(p, b, kv, append_pos, tid, h % p.gqa == 0 && slice == 0, hat);
    __syncthreads();
    float prod = tid < D ? q_e * hat[0][tid] : 0.0f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) prod += __shfl_xor(prod, off);
    if ((tid & 63) == 0) red_a[tid >> 6] = prod;
    __syncthreads();
    float dot = 0.0f;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) dot += red_a[w];
    a_new = dot * p.scale_log2;
  }
  float mg = fmaxf(red_m[0], a_new);
#pragma unroll
  for (int w = 1; w < WAVES; ++w) mg = fmaxf(mg, red_m[w]);
  const float w = exp2f(m - mg);
  if (tid < n) w_c[tid] = w;
  float lw = l * w;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) lw += __shfl_xor(lw, off);
  if ((tid & 63) == 0) red_l[tid >> 6] = lw;
  __syncthreads();
  float den = red_l[0] + red_l[1];
  if constexpr (WAVES >= 4) den += red_l[2] + red_l[3];
#pragma unroll
  for (int w = 4; w < WAVES; w += 4) den += (red_l[w] + red_l[w + 1]) + (red_l[w + 2] + red_l[w + 3]);

  float num = 0.0f;
  if (appending) {
    const float w_new = exp2f(a_new - mg);
    den += w_new;
    if (part == 0) num = w_new * hat[1][j];
  }
#pragma unroll
  for (int u = 0; u < FIRST; ++u) {
    const int c = part + u * PARTS;
    num = c < n ? fmaf(pre[u], w_c[c], num) : num;
  }
  int c = part + FIRST * PARTS;
  for (; c + 7 * PARTS < n; c += 8 * PARTS) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[(int64_t)(c + u * PARTS) * D];
#pragma unroll
    for (int u = 0; u < 8; ++u) num = fmaf(v[u], w_c[c + u * PARTS], num);
  }
  for (; c < n; c += PARTS) num = fmaf(src[(int64_t)c * D], w_c[c], num);
  if constexpr (PARTS > 1) {
    acc_part[part][jl] = num;
    __syncthreads();
    if (part == 0) {
#pragma unroll
      for (int q = 1; q < PARTS; ++q) num += acc_part[q][jl];
    }
  }
  if (part == 0) p.out[(int64_t)(b * p.n_q_heads + h) * D + j] = (half_t)(num / den);
}

// Folds the n chunks of HPT output rows into their running (maximum, numerator, denominator), CW chunks at a
// time, all of a round's loads in flight together (Eq. 6 with Alg. 1's rescaling applied to chunks).
template <int D, int HPT, int CW>
__device__ __forceinline__ void fold_chunks(const float* __restrict__ part_ml, const float* __restrict__ part_o,
                                            const int64_t (&row)[HPT], int part_stride, int n, int j,
                                            float (&m_run)[HPT], float (&num)[HPT], float (&den)[HPT]) {
  for (int c0 = 0; c0 < n; c0 += CW) {
    float2 ml[HPT][CW];
    float o[HPT][CW];
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
#pragma unroll
      for (int u = 0; u < CW; ++u) {
        const int64_t ph = row[i] * part_stride + min(c0 + u, n - 1);
        ml[i][u] = *reinterpret_cast<const float2*>(part_ml + ph * 2);
        o[i][u] = part_o[ph * D + j];
      }
    }
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
      float mx = m_run[i];
#pragma unroll
      for (int u = 0; u < CW; ++u) mx = c0 + u < n ? fmaxf(mx, ml[i][u].x) : mx;
      const float keep = exp2f(m_run[i] - mx);
      num[i] *= keep;
      den[i] *= keep;
#pragma unroll
      for (int u = 0; u < CW; ++u) {
        const float e = c0 + u < n ? exp2f(ml[i][u].x - mx) : 0.0f;
        num[i] = fmaf(o[i][u], e, num[i]);
        den[i] = fmaf(ml[i][u].y, e, den[i]);
      }
      m_run[i] = mx;
    }
  }
}

// Eq. 6 for launches of many hundreds of outputs and more (a dozen sequences and up): one block per (output row,
// 2 * HPT query heads of a KV head's group), a thread per output element and HPT heads.  The chunks are folded in
// four at a time (sequences of up to four chunks: one round of loads) or 32 / HPT at a time, all their loads in
// flight together, with a running maximum (Alg. 1's rescaling applied to chunks): no LDS, no barrier, and a
// launch of a quarter of the blocks that one block per query head needs.
// Append-and-attend (p.k_new set; one query token): every block quantises its KV head's new token, the group's
// first block stores it, every head's score of it is a sum over the D threads that hold the head, and it enters
// the fold as the last chunk (m = the score, l = 1, o = the dequantised V), as in reduce_kernel.
template <int D, int HPT>
// (at least five waves per SIMD for the four-heads instance: at 97 registers the compiler left it at four, and the
// launch of eight blocks per compute unit a third longer)
__global__ __launch_bounds__(2 * D, HPT == 4 ? 5 : 4) void reduce_group_kernel(DecodeParams p) {
  static_assert(D % 64 == 0 && 2 * D >= 8 * (D / kGroup), "whole waves per head; one thread per lane of the appender");
  // HPT heads per thread, 2 * HPT per block: a KV head's group takes `subs` blocks
  const int subs = (p.gqa + 2 * HPT - 1) / (2 * HPT);
  const int kv = blockIdx.x / subs, h0 = (blockIdx.x - kv * subs) * (2 * HPT);
  // (part: the same in all lanes of a wave, D being a multiple of 64: said so, the rows' addresses are scalar,
  // which saves the four-chunk fold some 30 vector registers; the wide fold would need more scalar registers than
  // there are and keeps its addresses in vector registers, part_v)
  const int b = blockIdx.y, tid = threadIdx.x, j = tid % D, part_v = tid / D, part = __builtin_amdgcn_readfirstlane(part_v);
  const int part_stride = p.var_chunks > 0 ? kMaxSplits : p.n_splits;
  int n = p.n_splits;
  int append_pos = p.append_pos;
  if (p.seq_lens) {
    const int sequence = p.n_queries > 1 ? b / p.n_queries : b;
    const int c = p.var_chunks > 0 ? *p.plan : p.tokens_per_split;
    n = min(n, (var_len(p, sequence) + c - 1) / c);
    // (append-and-attend: the length counts the new token, which goes to the last position; a sequence with no
    // cached token has no chunk)
    const int total = max(1, min(p.seq_lens[sequence], p.seq_len));
    append_pos = total - 1;
    if (total + p.len_bias < 1) n = 0;
  }
  const bool appending = p.k_new != nullptr;
  __shared__ float hat[2][D];
  __shared__ float red_a[2 * D / 64][HPT];
  if (appending) {
    quantize_new_token<D>(p, b, kv, append_pos, tid, h0 == 0, hat);
    __syncthreads();
  }
  int64_t row[HPT];
#pragma unroll
  for (int i = 0; i < HPT; ++i) row[i] = (int64_t)b * p.n_q_heads + kv * p.gqa + min(h0 + part * HPT + i, p.gqa - 1);
  float m_run[HPT], num[HPT], den[HPT];
#pragma unroll
  for (int i = 0; i < HPT; ++i) { m_run[i] = kNegBig; num[i] = 0.0f; den[i] = 0.0f; }
  // (up to four chunks: one round of loads; more: 32 / HPT at a time, so that a sequence of many chunks among
  // short ones, up to 128, stays a few rounds.  HPT = 4 is launched only where a sequence has at most 16 chunks:
  // four at a time, and 50 registers fewer)
  if (HPT == 4 || n <= 4) {
    fold_chunks<D, HPT, 4>(p.part_ml, p.part_o, row, part_stride, n, j, m_run, num, den);
  } else {
    int64_t row_v[HPT];
#pragma unroll
    for (int i = 0; i < HPT; ++i) row_v[i] = (int64_t)b * p.n_q_heads + kv * p.gqa + min(h0 + part_v * HPT + i, p.gqa - 1);
    fold_chunks<D, HPT, 32 / HPT>(p.part_ml, p.part_o, row_v, part_stride, n, j, m_run, num, den);
  }
  if (appending) {                                // (block-uniform)
    float prod[HPT];
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
      prod[i] = (float)p.q[row[i] * D + j] * hat[0][j];
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) prod[i] += __shfl_xor(prod[i], off);
    }
    if ((tid & 63) == 0) {
#pragma unroll
      for (int i = 0; i < HPT; ++i) red_a[tid >> 6][i] = prod[i];
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < HPT; ++i) {
      float dot = 0.0f;
#pragma unroll
      for (int w = 0; w < D / 64; ++w) dot += red_a[part * (D / 64) + w][i];
      const float a_new = dot * p.scale_log2;
      const float mx = fmaxf(m_run[i], a_new);
      const float keep = exp2f(m_run[i] - mx), e = exp2f(a_new - mx);
      num[i] = fmaf(hat[1][j], e, num[i] * keep);
      den[i] = fmaf(den[i], keep, e);
    }
  }
#pragma unroll
  for (int i = 0; i < HPT; ++i)
    if (h0 + part * HPT + i < p.gqa) p.out[row[i] * D + j] = (half_t)(num[i] / den[i]);
}

}  // namespace

hipError_t launch_partial_valu(const DecodeParams& p, int batch, int head_dim, bool dense, hipStream_t s) {
  const int head_tiles = (p.gqa + head_tile(head_dim) - 1) / head_tile(head_dim);
  const dim3 grid = p.var_chunks > 0 ? dim3(p.var_chunks, p.n_kv_heads * head_tiles, 1)
                                     : dim3(p.n_splits, p.n_kv_heads * head_tiles, batch);
  const dim3 block(256);
  if (head_dim == 128) {
    if (dense) hipLaunchKernelGGL((decode_partial_valu_kernel<128, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((decode_partial_valu_kernel<128, false>), grid, block, 0, s, p);
  } else if (head_dim == 256) {
    if (dense) hipLaunchKernelGGL((decode_partial_valu_kernel<256, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((decode_partial_valu_kernel<256, false>), grid, block, 0, s, p);
  } else {
    if (dense) hipLaunchKernelGGL((decode_partial_valu_kernel<512, true>), grid, block, 0, s, p);
    else hipLaunchKernelGGL((decode_partial_valu_kernel<512, false>), grid, block, 0, s, p);
  }
  return hipGetLastError();
}

// (measured on 64 query heads over 8 KV heads, sequences with their own lengths: no difference at 8 sequences,
// 2 % per decode at 12, 8-10 % at 32 and 48, 6-8 % at 128 and 256)
// Query heads per thread of reduce_group_kernel (a block: twice as many).  Measured against 4 and 1 on 64 query
// heads over 8 KV heads: 4 is as good where every sequence has a few chunks but a block then pulls in eight heads'
// partials, which for a sequence of 128 chunks among short ones is 512 KB through one compute unit (64 sequences,
// one of 65536 tokens: 55 µs per decode against 40 with one block per head, 45 with 2); 1 is no faster than one block
// per head.  (Where the host can rule such sequences out, launch_reduce takes 4.)
constexpr int kGroupHeads = 2;
bool reduce_is_grouped(int head_dim, int64_t out_rows, int n_q_heads, int gqa) {
  return head_dim == 128 && out_rows * n_q_heads >= 768 && gqa >= 4;
}

hipError_t launch_reduce(const DecodeParams& p, int batch, int head_dim, hipStream_t s) {
  const dim3 grid(p.n_q_heads, batch * std::max(1, p.n_queries));
  const bool many = (int64_t)grid.x * grid.y >= 4096;      // several rounds of blocks: smaller blocks, more at once
  if (reduce_is_grouped(head_dim, grid.y, p.n_q_heads, p.gqa)) {
    // Heads per thread: two; four (one block per KV head of eight query heads) where there are thousands of
    // outputs and no sequence can have more than 16 chunks, which the host can tell from the longest length
    // allowed and the planner's shortest chunk, or from the chunk count asked for.
    const int most_chunks = p.var_chunks > 0 ? (p.seq_len + p.var_min_chunk - 1) / std::max(1, p.var_min_chunk) : p.n_splits;
    if (many && most_chunks <= 16)
      hipLaunchKernelGGL((reduce_group_kernel<128, 4>), dim3(p.n_kv_heads * ((p.gqa + 7) / 8), grid.y), dim3(256), 0, s, p);
    else
      hipLaunchKernelGGL((reduce_group_kernel<128, kGroupHeads>),
                         dim3(p.n_kv_heads * ((p.gqa + 2 * kGroupHeads - 1) / (2 * kGroupHeads)), grid.y), dim3(256), 0, s, p);
  }
  else if (head_dim == 128 && many) hipLaunchKernelGGL((reduce_kernel<128, 128>), grid, dim3(128), 0, s, p);
  else if (head_dim == 128) hipLaunchKernelGGL((reduce_kernel<128, 256>), grid, dim3(256), 0, s, p);
  else if (head_dim == 256) hipLaunchKernelGGL((reduce_kernel<256, 256>), grid, dim3(256), 0, s, p);
  // d = 512: with few outputs, several blocks per query head (measured: 32 outputs 8 slices, 64 outputs 4; from
  // 128 outputs on slicing no longer pays and one block of 1024 threads per head is the shortest)
  else if ((int64_t)grid.x * grid.y <= 32) hipLaunchKernelGGL((reduce_kernel<512, 512, 8>), dim3(8 * grid.x, grid.y), dim3(512), 0, s, p);
  else if ((int64_t)grid.x * grid.y <= 64) hipLaunchKernelGGL((reduce_kernel<512, 512, 4>), dim3(4 * grid.x, grid.y), dim3(512), 0, s, p);
  else hipLaunchKernelGGL((reduce_kernel<512, 1024>), grid, dim3(1024), 0, s, p);
  return hipGetLastError();
}

}  // namespace tq
