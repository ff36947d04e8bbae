// Matrix-core fused int4 decode attention for head_dim 512 (the global-attention column of the kernel
// configuration table, Appendix A: 32 query heads on one KV head), phase 1 of Sec. 3.2.
//
// At d = 512 a KV head's query group is a tile of 16 or 32 rows, every fetched byte is used by all of them,
// and the work is arithmetic, not traffic: both contractions of Alg. 1 (the score and the update of the output accumulator) run on
// v_mfma_f32_16x16x32_f16 for all rows of the tile at once, and the vector ALU prepares each operand once
// per block, whatever the number of rows.
//
// One block = one chunk of one KV head x one tile of query rows; 4 waves that split the HEAD DIMENSION:
// wave w owns dims 128w .. 128w+127, i.e. quantisation groups 4w .. 4w+3.
//   scores  S^T = K Q^T (rows = 16 tokens, columns = 16 query rows), one MFMA per group: lane (kq, c) feeds
//           packed word kq of the group of token c, its codes as fp16 SUBNORMALS (value c 2^-24, or c 2^-20
//           for a nibble at bit 4: two ANDs per word pair, and the products and their sum are exact in the
//           fp32 accumulator).  Scale and zero-point are applied to the accumulator in fp32,
//             q.k^ = sum_g s_g (q_g.c_g - z_g sum(q_g)),
//           so the scores carry no fp16 rounding of K (they are exponentiated: an error there is an error of
//           the same relative size in a weight).  The four waves exchange their partial scores through LDS
//           (one barrier per 32 tokens, two buffers) and every wave adds them up in the same order, so all
//           four hold the same scores, bit for bit, and run the same online softmax.
//   P V     rows = query rows, columns = dims: the accumulator layout of S^T (lane = query row, four
//           tokens per lane and 16-token tile) IS the A-operand layout of P, so probabilities never move
//           between lanes.  Lane (kq, c) reads packed word 16w + c of its 8 tokens, transposes 8 x 8
//           nibbles with two byte-permute stages and DEQUANTISES them into fp16 operands ((c - z) s of Eq. 3:
//           1024 + c built by OR-ing the nibble into the mantissa of fp16 1024, then one mixed-precision FMA
//           per element, (1024 + c) s - (1024 + z) s in fp32, rounded once to fp16; scale and zero-point
//           differ per token), one B operand per dim of the word; the wave accumulates its 128 output
//           dims for every row of the tile, and no merge between the waves is needed.  (V enters the output
//           linearly, so its fp16 rounding stays at the size of the fp16 rounding of the output itself.)
// Data path: the packed stream goes from global memory straight into LDS (global_load_lds_dwordx4, no
// registers in between), a ring of NSTG stages of one 32-token step each, filled NSTG - 1 steps ahead of the
// arithmetic by all four waves together.  The source address of such a load is free per lane while its
// LDS destination is linear, so K codes land as [group][token] (the order the A operands are read in:
// no bank conflicts) and the rest lands as it lies in HBM, V codes with 64 B of padding per four tokens.
// A wave waits for its own loads of the next stage before the step's one barrier, so behind the barrier
// the whole stage is there for everybody, and the stage read two steps ago is free to be refilled.
//
// Query rows: n_queries * G rows (t, g) per KV head (several query tokens: the sequence's last n_queries
// tokens, causal among themselves), cut into tiles of 16 * RT rows; each row has its own [first, end) of
// visible tokens, applied to the scores of every step.
#include <algorithm>
#include <type_traits>

#include "tq_internal.h"

namespace tq {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr int D = 512;
constexpr int NG = D / kGroup;        // 16 groups per token
constexpr int TB = D / 2;             // bytes of codes per token
constexpr float kNegBig = -1.0e30f;   // "no token seen yet" (finite: no inf - inf)
constexpr uint32_t kNib = 0x000F000Fu;     // one nibble in each half of a dword
constexpr uint32_t kMagic = 0x64006400u;   // fp16 pair (1024, 1024): OR-ing a nibble into the mantissa gives 1024 + c

// Scale and offset of one token's group for dequant2: (1024 + c) s + t with t = -(1024 + z) s  =  (c - z) s.
// z s and 1024 s are exact in fp32, their sum is rounded at 2^-24 of 1024 s: far below an fp16 ulp of the result.
struct ScaleOffset { float s, t; };
__device__ __forceinline__ ScaleOffset scale_offset(half_t s16, half_t z16) {
  const float s = (float)s16;
  return {s, -fmaf(1024.0f, s, (float)z16 * s)};
}
// two codes (bits 0-3 and 16-19 of `bits`) -> the fp16 pair of their values (c - z) s (Eq. 3), each computed in
// fp32 and rounded ONCE (fp16 sources, fp32 arithmetic, fp16 result: one mixed-precision FMA per element)
__device__ __forceinline__ uint32_t dequant2(uint32_t bits, ScaleOffset lo, ScaleOffset hi) {
  uint32_t u;                                                   // (bits & kNib) | kMagic in one instruction
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(u) : "v"(bits), "v"(kNib), "v"(kMagic));
  const half2v x = __builtin_bit_cast(half2v, u);               // (1024 + c_lo, 1024 + c_hi), exact
  const half2v r = {(half_t)fmaf((float)x[0], lo.s, lo.t), (half_t)fmaf((float)x[1], hi.s, hi.t)};
  return __builtin_bit_cast(uint32_t, r);
}
__device__ __forceinline__ half8v as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_bit_cast(half8v, uint4v{a, b, c, d});
}
__device__ __forceinline__ float4v mfma16(half8v a, half8v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}

// What one 32-token step needs from its stage, per lane (kq, c) of wave w.
// Token slot i of a lane: token 4kq + i of the step's first 16-token tile (i < 4), of its second (i >= 4).
struct StepK {
  uint32_t kw[2][4];     // K codes of token 16t + c: packed word kq of groups 4w .. 4w+3
  uint2 ks[2][4], kz[2][4];   // scales and zero-points of those four groups (fp16 x 4), token 16t + 4kq + i
};
struct StepV {
  uint32_t vw[8];        // V codes of token slot i: packed word 16w + c (group 4w + c/4)
  half_t vs[8], vz[8];
};

// One stage of the ring: a 32-token step of one KV head.
constexpr int kStageK = 0;                        // K codes, 16-byte pieces [group 16][token 32]
constexpr int kStageV = 32 * TB;                  // V codes, as in HBM, eight loads of 4 tokens, 64 B apart
constexpr int kVChunk = 4 * TB + 64;
constexpr int kStageS = kStageV + 8 * kVChunk;    // k_scale, k_zero, v_scale, v_zero: [token 32][group 16] fp16 each
constexpr int kStageBytes = kStageS + 4 * 32 * NG * 2;
constexpr int kLoadsPerStage = 5;                 // per lane: 2 K, 2 V, 1 scale array (wave w: array w)

// direct global -> LDS load of 16 B per lane: lane l's bytes land at lds_base + 16 l (M0 carries the base)
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :: "v"(voff), "s"(sbase), "s"(lds_base) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() {    // until at most N vector-memory loads of this wave are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// RT: 16-row tiles per block.  NSTG: stages of the ring (3 with 16 rows: two blocks fit a compute unit's LDS and
// registers and cover each other's waits; more where a compute unit gets one block anyway).
template <int RT, int NSTG>
__global__ __launch_bounds__(256, NSTG == 3 ? 2 : 1) void decode_partial_wide_kernel(DecodeParams p) {
  static_assert(NSTG >= 3 && NSTG <= 6, "ring depth");
  // partial scores of the four waves, [buffer][wave][row tile, token tile][lane]: two buffers and one barrier per
  // step with 16 rows; with 32 rows one buffer and a second barrier (before it is written again), which keeps
  // the block at half a compute unit's LDS
  constexpr int SB = RT == 1 ? 2 : 1;
  __shared__ float4v s_part[SB][4][RT * 2][64];
  __shared__ __attribute__((aligned(16))) char ring[NSTG * kStageBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, kq = lane >> 4;

  int split = blockIdx.x, b = blockIdx.z, tokens_per_split = p.tokens_per_split, part_stride = p.n_splits;
  if (p.var_chunks > 0) {                         // per-sequence lengths: which (sequence, chunk) is this block's
    VarPlan vp;
    if (!var_plan(p, blockIdx.x, vp)) return;
    split = __builtin_amdgcn_readfirstlane(vp.chunk);           // (wave-uniform by construction: tell the compiler)
    b = __builtin_amdgcn_readfirstlane(vp.b);
    tokens_per_split = __builtin_amdgcn_readfirstlane(vp.chunk_tokens);
    part_stride = kMaxSplits;
  }
  const int tiles = p.kv_share;                   // row tiles per KV head
  const int kv = blockIdx.y / tiles, tile = blockIdx.y - kv * tiles;
  const int NQ = p.n_queries, GF = p.gqa, rows_total = NQ * GF;

  const int seq = p.seq_lens ? var_len(p, b) : p.seq_len;       // tokens the LAST query token attends, from `start`
  const int start = p.seq_lens ? var_start(p, b) : p.start;
  const bool paged = p.block_table != nullptr;
  // paged cache under a window: the chunks count from a 32-token boundary up to 31 tokens before the window
  const int lead = (paged && p.seq_lens) ? var_first(p, b) - start : 0;
  const int begin = split * tokens_per_split;
  if (begin >= seq) return;                       // chunk past the end of its sequence: nothing to emit
  const int end = min(seq, begin + tokens_per_split);
  const int64_t row0 = (int64_t)(b * p.n_kv_heads + kv) * p.row_stride + start;

  // ---- this lane's column of each row tile: which (query token, head) it is and which tokens it sees
  int64_t qrow[RT];
  bool rvalid[RT];
  int lo_col[RT], end_col[RT];
  auto row_of = [&](int r, int64_t& out_row, int& t_q) {        // tile row -> row of q / out / the partials
    t_q = r / GF;
    out_row = (int64_t)(b * NQ + t_q) * p.n_q_heads + kv * GF + (r - t_q * GF);
  };
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    const int r = (tile * RT + rt) * 16 + c;
    rvalid[rt] = r < rows_total;
    int t_q;
    row_of(min(r, rows_total - 1), qrow[rt], t_q);
    // query token t attends NQ - 1 - t tokens fewer than the last one; under a window its own last `row_window`
    const int own_end = seq - (NQ - 1 - t_q);
    end_col[rt] = rvalid[rt] ? min(end, own_end) : begin;
    lo_col[rt] = (NQ > 1 && p.row_window > 0) ? max(0, start + own_end - p.row_window) - start : lead;
  }
  // the tokens that every row of the tile sees: [lo_all, end_all) (columns past the last row do not count)
  int lo_all = 0, end_all = end;
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    lo_all = max(lo_all, rvalid[rt] ? lo_col[rt] : 0);
    end_all = min(end_all, rvalid[rt] ? end_col[rt] : end);
  }
#pragma unroll
  for (int off = 1; off < 16; off <<= 1) {
    lo_all = max(lo_all, __shfl_xor(lo_all, off));
    end_all = min(end_all, __shfl_xor(end_all, off));
  }
  lo_all = __builtin_amdgcn_readfirstlane(lo_all);
  end_all = __builtin_amdgcn_readfirstlane(end_all);

  // ---- one step of the chunk -> its stage of the ring: kLoadsPerStage loads per lane, all 256 lanes.
  //      Step j starts 32 j tokens past `begin`; tokens at or past `end` are clamped to the last one (their
  //      scores are masked).  Paged cache: start + the step's first token is a multiple of 32 and a page a
  //      multiple of 32 tokens, so a step lies in one page.
  const int page_mask = paged ? (1 << p.page_shift) - 1 : 0;
  const int32_t* const tbl = paged ? p.block_table + (int64_t)b * p.max_blocks : nullptr;
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)ring;
  const char* const sz_array = reinterpret_cast<const char*>(wave == 0 ? p.k_scale : wave == 1 ? p.k_zero
                                                             : wave == 2 ? p.v_scale : p.v_zero);
  auto issue_step = [&](int j) {
    const int tok0 = begin + 32 * j;
    int64_t base = row0 + tok0;                   // wave-uniform
    if (paged) {
      // the page of this step: a scalar load (a vector load here would make the compiler wait for every
      // outstanding load of the ring)
      const int ta = start + tok0;
      const uint32_t byte = (uint32_t)min(ta >> p.page_shift, p.max_blocks - 1) * 4;
      int page;
      asm volatile("s_load_dword %0, %1, %2\n\ts_waitcnt lgkmcnt(0)" : "=s"(page) : "s"(tbl), "s"(byte) : "memory");
      base = ((int64_t)page * p.n_kv_heads + kv) * p.row_stride + (ta & page_mask);
    }
    const int last = end - 1 - tok0;              // >= 0: the step's last valid token
    const uint32_t l = ring_lds + (j % NSTG) * kStageBytes;
    const char* const kc = reinterpret_cast<const char*>(p.k_codes) + base * TB;
    const char* const vc = reinterpret_cast<const char*>(p.v_codes) + base * TB;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      // K: piece (group g, token t) goes to position 32 g + t; this lane fills position 256 u + threadIdx.x
      const int g = 8 * u + 2 * wave + (lane >> 5), t = min(lane & 31, last);
      dma16(kc, (uint32_t)(t * TB + g * 16), l + kStageK + (256 * u + 64 * wave) * 16);
      // V: load r = 4u + wave brings tokens 4r .. 4r+3 whole; this lane's piece: token 4r + lane/16, bytes 16 (lane%16)
      const int r = 4 * u + wave, tv = min(4 * r + (lane >> 4), last);
      dma16(vc, (uint32_t)(tv * TB + (lane & 15) * 16), l + kStageV + r * kVChunk);
    }
    // scale / zero-point array `wave`: token lane/2, half lane%2 of its 32 bytes
    dma16(sz_array + base * (NG * 2), (uint32_t)(min(lane >> 1, last) * (NG * 2) + (lane & 1) * 16),
          l + kStageS + wave * (32 * NG * 2));
  };
  auto read_k = [&](int j, StepK& st) {
    const char* const stg = ring + (j % NSTG) * kStageBytes;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
#pragma unroll
      for (int m = 0; m < 4; ++m)
        st.kw[t][m] = *reinterpret_cast<const uint32_t*>(stg + kStageK + ((4 * wave + m) * 32 + 16 * t + c) * 16 + 4 * kq);
#pragma unroll
      for (int i = 0; i < 4; ++i) {               // the accumulator rows of this lane: tokens 16t + 4kq + i
        const int tok = 16 * t + 4 * kq + i;
        st.ks[t][i] = *reinterpret_cast<const uint2*>(stg + kStageS + tok * (NG * 2) + 8 * wave);
        st.kz[t][i] = *reinterpret_cast<const uint2*>(stg + kStageS + 32 * NG * 2 + tok * (NG * 2) + 8 * wave);
      }
    }
  };
  auto read_v = [&](int j, StepV& st) {
    const char* const stg = ring + (j % NSTG) * kStageBytes;
#pragma unroll
    for (int i = 0; i < 8; ++i) {                 // token 16 (i/4) + 4 kq + i%4: load 4 (i/4) + kq, its token i%4
      const int tok = 16 * (i >> 2) + 4 * kq + (i & 3);
      st.vw[i] = *reinterpret_cast<const uint32_t*>(stg + kStageV + (4 * (i >> 2) + kq) * kVChunk + (i & 3) * TB +
                                                    4 * (16 * wave + c));
      st.vs[i] = *reinterpret_cast<const half_t*>(stg + kStageS + 2 * 32 * NG * 2 + tok * (NG * 2) + 2 * (4 * wave + (c >> 2)));
      st.vz[i] = *reinterpret_cast<const half_t*>(stg + kStageS + 3 * 32 * NG * 2 + tok * (NG * 2) + 2 * (4 * wave + (c >> 2)));
    }
  };

  // ---- running state (Alg. 1, the initialisation), scores in log2 units
  float m_run[RT], l_run[RT];                     // per column (query row); l: this lane's share of the sum
  float4v oacc[RT][8];                            // rows 4kq+i of the tile, dim 8(16w+c) + index
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    m_run[rt] = kNegBig;
    l_run[rt] = 0.0f;
#pragma unroll
    for (int mm = 0; mm < 8; ++mm) oacc[rt][mm] = float4v{0, 0, 0, 0};
  }

  // ---- prologue: the first NSTG - 1 steps are on their way while the query operands are built
  const int n_steps = (end - begin + 31) >> 5;
#pragma unroll
  for (int j = 0; j < NSTG - 1; ++j)
    if (j < n_steps) issue_step(j);

  // ---- query operands: B of S^T = K Q^T, MFMA m = group 4w + m, this lane's k-slots = its dims 8kq .. 8kq+7.
  //      k-slot order of an unpacked word: dims 0,4,1,5,2,6,3,7; the nibbles at bit 4 carry c 2^-20, so their
  //      query entries are pre-divided by 16.  qsum: 2^-24 sum of q over the group (for the zero-point term).
  half8v qb[RT][4];
  float qsum[RT][4];
#pragma unroll
  for (int rt = 0; rt < RT; ++rt)
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      const half8v x = *reinterpret_cast<const half8v*>(p.q + qrow[rt] * D + 32 * (4 * wave + m) + 8 * kq);
      const half_t sixteenth = (half_t)0.0625f;
      half8v y = {x[0], x[4], x[1] * sixteenth, x[5] * sixteenth, x[2], x[6], x[3] * sixteenth, x[7] * sixteenth};
      float sum = 0.0f;
#pragma unroll
      for (int e = 0; e < 8; ++e) sum += (float)x[e];
      sum += __shfl_xor(sum, 16);                 // the other three words of the group (same value in all four lanes)
      sum += __shfl_xor(sum, 32);
      if (!rvalid[rt]) { y = half8v{0, 0, 0, 0, 0, 0, 0, 0}; sum = 0.0f; }
      qb[rt][m] = y;
      qsum[rt][m] = sum * 0x1p-24f;
    }
  const float raw_to_log2 = p.scale_log2 * 0x1p24f;              // accumulator units -> log2 units

  wait_loads<0>();
  __syncthreads();                                // the prologue's stages have landed, everybody's part of them

  for (int it = 0; it < n_steps; ++it) {
    const int tok0 = begin + 32 * it;
    StepK cur;
    read_k(it, cur);

    // -- this wave's share of the scores (Alg. 1, the score step): its four groups of K against the query rows,
    //    per-group scale and zero-point applied in fp32 (accumulator units: 2^-24)
    float4v sacc[RT][2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float4v acc[RT][4];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const uint32_t w = cur.kw[t][m], w8 = w >> 8;
        const half8v a = as_half8(w & kNib, w & (kNib << 4), w8 & kNib, w8 & (kNib << 4));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt][m] = mfma16(a, qb[rt][m], float4v{0, 0, 0, 0});
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint32_t sw[2] = {cur.ks[t][i].x, cur.ks[t][i].y}, zw[2] = {cur.kz[t][i].x, cur.kz[t][i].y};
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          float x = 0.0f;
#pragma unroll
          for (int m = 0; m < 4; ++m) {
            const float sg = (float)__builtin_bit_cast(half_t, (uint16_t)(sw[m >> 1] >> (16 * (m & 1))));
            const float zg = (float)__builtin_bit_cast(half_t, (uint16_t)(zw[m >> 1] >> (16 * (m & 1))));
            x = fmaf(sg, fmaf(-zg, qsum[rt][m], acc[rt][m][i]), x);
          }
          sacc[rt][t][i] = x;
        }
      }
    }
    const int buf = SB == 2 ? (it & 1) : 0;
    if (SB == 1) __syncthreads();                 // everybody has read the previous step's partial scores
#pragma unroll
    for (int rt = 0; rt < RT; ++rt)
#pragma unroll
      for (int t = 0; t < 2; ++t) s_part[buf][wave][rt * 2 + t][lane] = sacc[rt][t];
    // The step's one barrier.  Before it every wave makes sure that its own loads of stage it + 1 have landed
    // (loads complete in order; only the stages issued after that one may still be out), so behind it the
    // whole of stage it + 1 is there for everybody; and everybody is done with stage it - 1, which is refilled.
    switch (min(NSTG - 3, max(0, n_steps - it - 2))) {           // stages issued after stage it + 1
      case 3: wait_loads<3 * kLoadsPerStage>(); break;
      case 2: wait_loads<2 * kLoadsPerStage>(); break;
      case 1: wait_loads<1 * kLoadsPerStage>(); break;
      default: wait_loads<0>(); break;
    }
    __syncthreads();
    if (it + NSTG - 1 < n_steps) issue_step(it + NSTG - 1);

    // -- online softmax (Alg. 1: the maximum, the weights and the running sum), the same in all four waves.  A step that every row of the
    //    tile sees in full needs no masks: all steps but the few that hold a row's first or last token.
    half8v pa[RT];
    float corr[RT];
    bool moved = false;
    auto softmax = [&](auto masked_tag) {
      constexpr bool MASKED = decltype(masked_tag)::value;
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float sc[2][4];
        bool ok[2][4];
        float mx = kNegBig;
#pragma unroll
        for (int t = 0; t < 2; ++t) {
          const float4v x = (s_part[buf][0][rt * 2 + t][lane] + s_part[buf][1][rt * 2 + t][lane]) +
                            (s_part[buf][2][rt * 2 + t][lane] + s_part[buf][3][rt * 2 + t][lane]);
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const int tok = tok0 + 16 * t + 4 * kq + i;
            ok[t][i] = !MASKED || (tok >= lo_col[rt] && tok < end_col[rt]);
            sc[t][i] = x[i] * raw_to_log2;
            mx = ok[t][i] ? fmaxf(mx, sc[t][i]) : mx;
          }
        }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run[rt], mx);
        moved = moved || m_new > m_run[rt];
        corr[rt] = __builtin_amdgcn_exp2f(m_run[rt] - m_new);
        m_run[rt] = m_new;
        float sum = 0.0f;
        float pr[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            pr[t][i] = ok[t][i] ? __builtin_amdgcn_exp2f(sc[t][i] - m_new) : 0.0f;
            sum += pr[t][i];
          }
        l_run[rt] = fmaf(l_run[rt], corr[rt], sum);
        // k-slots 2i, 2i+1: token slots i and 4+i
        pa[rt] = half8v{(half_t)pr[0][0], (half_t)pr[1][0], (half_t)pr[0][1], (half_t)pr[1][1],
                        (half_t)pr[0][2], (half_t)pr[1][2], (half_t)pr[0][3], (half_t)pr[1][3]};
      }
    };
    if (tok0 >= lo_all && tok0 + 32 <= end_all) softmax(std::false_type{});
    else softmax(std::true_type{});
    if (__builtin_amdgcn_ballot_w64(moved) != 0) {               // some row's maximum moved: rescale (Alg. 1, the correction of the accumulator)
#pragma unroll
      for (int rt = 0; rt < RT; ++rt) {
        float fr[4];                                             // accumulator row 4kq+i is the column of lane 4kq+i
#pragma unroll
        for (int i = 0; i < 4; ++i) fr[i] = __shfl(corr[rt], 4 * kq + i);
#pragma unroll
        for (int mm = 0; mm < 8; ++mm)
#pragma unroll
          for (int i = 0; i < 4; ++i) oacc[rt][mm][i] *= fr[i];
      }
    }

    // -- P V (Alg. 1, the accumulator update): 8 tokens x 8 nibbles per lane -> 8 dims x 8 tokens, dequantised per token pair
    {
      StepV curv;
      read_v(it, curv);
      uint32_t x[8], y[8];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        x[i] = __builtin_amdgcn_perm(curv.vw[i + 4], curv.vw[i], 0x05040100u);
        x[i + 4] = __builtin_amdgcn_perm(curv.vw[i + 4], curv.vw[i], 0x07060302u);
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if ((i & 2) == 0) {
          y[i] = __builtin_amdgcn_perm(x[i + 2], x[i], 0x06020400u);
          y[i + 2] = __builtin_amdgcn_perm(x[i + 2], x[i], 0x07030501u);
        }
      // y[2I+a]: byte M = token slot 2M+a, low nibble dim 2I, high nibble dim 2I+1 of the packed word
      ScaleOffset so[8];                                         // per token slot; k-slot pair i: token slots i and 4+i
#pragma unroll
      for (int i = 0; i < 8; ++i) so[i] = scale_offset(curv.vs[i], curv.vz[i]);
#pragma unroll
      for (int I = 0; I < 4; ++I) {
        const uint32_t r0 = y[2 * I], r1 = y[2 * I + 1];
        const half8v v_even = as_half8(dequant2(r0, so[0], so[4]), dequant2(r1, so[1], so[5]),
                                       dequant2(r0 >> 8, so[2], so[6]), dequant2(r1 >> 8, so[3], so[7]));
        const half8v v_odd = as_half8(dequant2(r0 >> 4, so[0], so[4]), dequant2(r1 >> 4, so[1], so[5]),
                                      dequant2(r0 >> 12, so[2], so[6]), dequant2(r1 >> 12, so[3], so[7]));
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) {
          oacc[rt][2 * I] = mfma16(pa[rt], v_even, oacc[rt][2 * I]);
          oacc[rt][2 * I + 1] = mfma16(pa[rt], v_odd, oacc[rt][2 * I + 1]);
        }
      }
    }
  }

  // ---- the chunk's partial (o_c, m_c, l_c) per query row (Sec. 3.2), un-normalised
#pragma unroll
  for (int rt = 0; rt < RT; ++rt) {
    float l_tot = l_run[rt] + __shfl_xor(l_run[rt], 16);
    l_tot += __shfl_xor(l_tot, 32);
    if (wave == 0 && kq == 0 && rvalid[rt]) {
      const int64_t ph = qrow[rt] * part_stride + split;
      p.part_ml[ph * 2] = m_run[rt];
      p.part_ml[ph * 2 + 1] = l_tot;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int r = (tile * RT + rt) * 16 + 4 * kq + i;
      if (r >= rows_total) continue;
      int64_t orow;
      int t_q;
      row_of(r, orow, t_q);
      float4v* dst = reinterpret_cast<float4v*>(p.part_o + (orow * part_stride + split) * D + 8 * (16 * wave + c));
      dst[0] = float4v{oacc[rt][0][i], oacc[rt][1][i], oacc[rt][2][i], oacc[rt][3][i]};
      dst[1] = float4v{oacc[rt][4][i], oacc[rt][5][i], oacc[rt][6][i], oacc[rt][7][i]};
    }
  }
}

}  // namespace

bool wide_supported(int head_dim) { return head_dim == D; }

// Row tiles per KV head for `rows` query rows: tiles of 32 rows (the stream is dequantised once for twice the
// rows) where that still gives every compute unit two blocks (`units` = batch x KV heads, `tokens` = the longest
// sequence), else tiles of 16.
int wide_row_tiles(int rows, int64_t units, int tokens) {
  const int t16 = (rows + 15) / 16, t32 = (rows + 31) / 32;
  const int64_t max_splits = std::max(1, std::min(kMaxSplits, tokens / 64));
  return (rows > 16 && units * t32 * max_splits >= 512) ? t32 : t16;
}

hipError_t launch_partial_wide(const DecodeParams& p_in, int batch, int head_dim, hipStream_t s) {
  DecodeParams p = p_in;
  if (head_dim != D || p.gqa < 1 || p.kv_share < 1) return hipErrorInvalidValue;
  if (p.n_queries < 1) p.n_queries = 1;
  if (p.n_queries > kMaxQueries) return hipErrorInvalidValue;
  const int rows = p.n_queries * p.gqa;
  const int per_tile = (rows + p.kv_share - 1) / p.kv_share;
  if (per_tile > 32) return hipErrorInvalidValue;
  const int rt = per_tile > 16 ? 2 : 1;
  if ((int64_t)p.kv_share * 16 * rt < rows) return hipErrorInvalidValue;
  if (p.block_table && (p.page_shift < 5 || !p.seq_lens)) return hipErrorInvalidValue;   // a step must not straddle pages
  const dim3 grid = p.var_chunks > 0 ? dim3(p.var_chunks, p.n_kv_heads * p.kv_share, 1)
                                     : dim3(p.n_splits, p.n_kv_heads * p.kv_share, batch);
  // more blocks than compute units: shallow rings, two blocks per unit (16-row tiles); else one block with a deep ring
  const bool crowded = (int64_t)grid.x * grid.y * grid.z > 256;
  if (rt == 2) hipLaunchKernelGGL((decode_partial_wide_kernel<2, 3>), grid, dim3(256), 0, s, p);
  else if (crowded) hipLaunchKernelGGL((decode_partial_wide_kernel<1, 3>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((decode_partial_wide_kernel<1, 6>), grid, dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace tq
