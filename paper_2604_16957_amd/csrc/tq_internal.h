// Internal declarations shared by the library's translation units (host launchers and
// the parameter blocks their kernels take).  Not part of the public ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tq.h"

namespace tq {

constexpr int kGroup = 32;        // elements per quantisation group (Sec. 2.1): the paper's configuration and the one the
                                  // matrix-core kernels are built for; also the piece of a vector one thread of the
                                  // quantiser handles.  Groups of 64 and 128 (DecodeParams::group) take the generic kernels.
constexpr int kMaxSplits = 128;   // upper bound on sequence chunks (Sec. 3.2); sizes the workspace
constexpr int kTile = 32;         // chunk boundaries are multiples of this many tokens
constexpr int kMaxQueries = 8;    // query tokens per sequence in one call (the masked path covers two supertiles)

typedef _Float16 half_t;

// Arguments of the decode kernels (fused int4, dense fp16 comparator, merge).
struct DecodeParams {
  const uint8_t* k_codes;   // [B][H_kv][row_stride][D/2]
  const uint8_t* v_codes;
  const half_t* k_scale;    // [B][H_kv][row_stride][D/32]
  const half_t* k_zero;
  const half_t* v_scale;
  const half_t* v_zero;
  const half_t* k_dense;    // comparator only: [B][H_kv][row_stride][D]
  const half_t* v_dense;
  const half_t* q;          // [B][n_queries][H_q][D]
  const int32_t* seq_lens;  // device, [B], or null: tokens each sequence attends (clamped to [1, seq_len])
  float* part_o;            // [B][n_queries][H_q][n_splits][D]   un-normalised chunk outputs
  float* part_ml;           // [B][n_queries][H_q][n_splits][2]   (running max in log2 units, sum of exp)
  half_t* out;              // [B][n_queries][H_q][D]
  int32_t* plan;            // one int behind part_ml: the chunk length of a device-planned launch, for the merge kernel
  int32_t n_q_heads, n_kv_heads, gqa;
  int32_t group;            // elements per quantisation group: 32, 64 or 128 (scale / zero-point arrays: D / group per token)
  // Query tokens per sequence (>= 1): the sequence's last n_queries tokens, query t attending all tokens up
  // to its own (n_queries - 1 - t fewer than the sequence holds).  Matrix-core kernel only.
  int32_t n_queries;
  // Matrix-core kernel: a KV head has n_queries * gqa_full query rows (gqa_full = H_q / H_kv).  Where that is
  // more than its tile takes, kv_share blocks (blockIdx.y = kv * kv_share + part) stream the same KV head,
  // each for gqa consecutive rows (gqa then counts one block's rows).
  int32_t kv_share, gqa_full;
  int32_t row_stride;       // tokens between consecutive (b, kv head) rows
  int32_t seq_len, n_splits, tokens_per_split;   // seq_len: every sequence's length, or the bound of seq_lens
  float scale_log2;         // attn_scale * log2(e)
  // Per-sequence lengths: the chunking is worked out ON THE DEVICE from seq_lens (see var_plan), so that
  // every block gets about the same number of tokens whatever the mix of lengths.  var_chunks > 0 turns
  // it on: blockIdx.x is then a slot in the list of all (sequence, chunk) pairs of one KV head, the
  // partials are strided by kMaxSplits, and n_splits / tokens_per_split are not used.
  int32_t batch, var_chunks, var_min_chunk;
  // Sliding window: a sequence attends tokens [start, start + its length).  Common length: `start` (host)
  // and seq_len already the windowed length.  Per-sequence lengths: window > 0 and the kernels derive
  // both from seq_lens (var_len / var_start below).
  int32_t start, window;
  // Several query tokens under a window: `window` above (and `start` / seq_len) describe the span all rows
  // together attend, window + n_queries - 1 tokens; row_window is the window of one row (0 = none).
  int32_t row_window;
  // Paged cache: block_table non-null = the six arrays are a POOL of pages, [n_pages][H_kv][row_stride] rows
  // with row_stride = 2^page_shift tokens per page, and token t of sequence b lives in page
  // block_table[b * max_blocks + (t >> page_shift)] at row t & (row_stride - 1).
  const int32_t* block_table;
  int32_t max_blocks, page_shift;
  // Append-and-attend (merge kernel, one query token, common length): k_new / v_new non-null = one new token per
  // sequence, fp16 [B][H_kv][1][D], not among the tokens the chunks cover; the merge kernel quantises it, writes it
  // at token append_pos of its row and adds its attention term to Eq. 6.
  // With per-sequence lengths the lengths COUNT the new token (len_bias = -1: the chunks cover one token fewer)
  // and it is written at each sequence's own last position.
  const half_t* k_new;
  const half_t* v_new;
  int32_t append_pos;
  int32_t len_bias;
  // Matrix-core kernel, many single-chunk rows: 1, 2 or 4 = a block takes 8 / waves_per_row (sequence, KV head)
  // rows with that many waves each (grid.y counts groups of rows); anything else = one row per block.
  int32_t waves_per_row;
  int32_t merge_slot;       // matrix-core kernel: >= 0 selects a set of arrival counters and makes the last
                            // block of every (b, kv head) merge the chunks and write `out`; < 0: partials only
};

#ifdef __HIPCC__
// Sec. 2.1, Eq. 2-3.  Every fp32 step is a separately rounded operation (no contraction, correctly rounded
// divides), so the bits are the same wherever this runs.
// Eq. 2 from a group's min and max: s = (max - min) / 15 stored as fp16 (a scale that rounds to zero becomes
// 1.0), z = -min / s from the STORED scale (saturated, never -0).
__device__ inline void quantize_scale_zero(float mn, float mx, half_t& s16, half_t& z16) {
#pragma clang fp contract(off)
  const float s32 = __fdiv_rn(__fsub_rn(mx, mn), 15.0f);
  s16 = (half_t)s32;
  if ((__builtin_bit_cast(uint16_t, s16) & 0x7FFFu) == 0) s16 = (half_t)1.0f;
  const float z32 = __fdiv_rn(__fsub_rn(0.0f, mn), (float)s16);
  z16 = (half_t)z32;
  uint16_t zb = __builtin_bit_cast(uint16_t, z16);
  if ((zb & 0x7FFFu) == 0x7C00u) zb = (uint16_t)((zb & 0x8000u) | 0x7BFFu);
  if (zb == 0x8000u) zb = 0;
  z16 = __builtin_bit_cast(half_t, zb);
}
// Eq. 3 for 8 consecutive elements: q = clamp(round_half_even(x / s + z), 0, 15), element j in bits 4j..4j+3
__device__ inline uint32_t quantize_word(const float* x, float sf, float zf) {
#pragma clang fp contract(off)
  uint32_t acc = 0;
#pragma unroll
  for (int j = 0; j < 8; ++j) {
    const float v = __fadd_rn(__fdiv_rn(x[j], sf), zf);
    const float r = fminf(fmaxf(rintf(v), 0.0f), 15.0f);
    acc |= (uint32_t)r << (4 * j);
  }
  return acc;
}
// The same codes, bit for bit, without a correctly rounded divide per element.  x / s + z is formed as one fused
// multiply-add with a reciprocal of s refined once per group (the scale is shared), which lands within a few units
// in the last place of what quantize_word rounds.  The two can pick different codes only where the value sits that
// close to a rounding boundary k + 1/2: those elements push `far` (the largest distance of a value from its rounded
// integer) up to 1/2 - tol, and the caller then redoes its words with quantize_word, so that the result never
// depends on the shortcut.  On zero-mean data about one group in a thousand is redone.
struct QuantFast { float zf, rcp, tol; };
__device__ inline QuantFast quantize_fast_setup(float sf, float zf, float abs_max) {
#pragma clang fp contract(off)
  QuantFast f;
  f.zf = zf;
  const float r0 = __builtin_amdgcn_rcpf(sf);              // 1 ulp; one Newton step brings it to about half an ulp
  f.rcp = __builtin_fmaf(__builtin_fmaf(-sf, r0, 1.0f), r0, r0);
  // with Q = abs_max / s >= |x/s| and V = Q + |z| >= |x/s + z|: the reciprocal moves the quotient by at most
  // 2^-23 Q, quantize_word's own two roundings by 2^-24 (Q + V), the fused one by 2^-24 V: below 2^-21 V together,
  // doubled for margin
  f.tol = (abs_max * f.rcp * 1.0001f + fabsf(zf)) * 0x1p-20f;
  return f;
}
__device__ inline bool quantize_fast_in_doubt(float far, const QuantFast& f) { return !(far < 0.5f - f.tol); }
__device__ inline uint32_t quantize_word_fast(const half_t* x, const QuantFast& f, float& far) {
#pragma clang fp contract(off)
  // Adding 1.5 * 2^23 rounds a value of [0, 15] to an integer, half to even, and leaves that integer in the low
  // bits of the sum's encoding; eight encodings summed at 4-bit offsets carry the same known excess.
  constexpr float kMagic = 12582912.0f;
  constexpr uint32_t kExcess = 0x4B400000u * 0x11111111u;
  uint32_t acc = 0;
#pragma unroll
  for (int j = 7; j >= 0; --j) {
    const float v = __builtin_amdgcn_fmed3f(__builtin_fmaf((float)x[j], f.rcp, f.zf), 0.0f, 15.0f);
    const float t = v + kMagic;
    far = fmaxf(far, fabsf(v - (t - kMagic)));
    acc = (acc << 4) + __float_as_uint(t);
  }
  return acc - kExcess;
}
// Device-side chunk plan for per-sequence lengths.  One chunk length C for all sequences (var_chunk_tokens
// below), so that the list "all chunks of sequence 0, then of sequence 1, ..." has at most p.var_chunks
// entries: the grid.  Slot s of that list -> (b, chunk); returns false past the end of the list.
// Everything here is wave-uniform.
struct VarPlan { int chunk_tokens, b, chunk; };
__device__ inline int var_full_len(const DecodeParams& p, int b) {
  return max(1, min(p.seq_lens[b], p.seq_len) + p.len_bias);
}
// The first token sequence b attends; the token its chunks are counted from (the same, except in a paged
// cache, where it is rounded down to a supertile boundary so that no supertile straddles two pages: the
// kernels mask the tokens in between); and the tokens from there to the sequence's end.
__device__ inline int var_first(const DecodeParams& p, int b) {
  const int n = var_full_len(p, b);
  return p.window > 0 ? n - min(n, p.window) : 0;
}
__device__ inline int var_start(const DecodeParams& p, int b) {
  const int f = var_first(p, b);
  return p.block_table ? f & ~(kTile - 1) : f;
}
__device__ inline int var_len(const DecodeParams& p, int b) { return var_full_len(p, b) - var_start(p, b); }
// sum of x over the 64 lanes of the wave (the same value in every lane; all lanes must be active)
__device__ inline int wave_sum(int x) {
  x += __builtin_amdgcn_update_dpp(0, x, 0x128, 0xF, 0xF, false);   // row_ror:8, 4, 2, 1: sum of each row of 16
  x += __builtin_amdgcn_update_dpp(0, x, 0x124, 0xF, 0xF, false);
  x += __builtin_amdgcn_update_dpp(0, x, 0x122, 0xF, 0xF, false);
  x += __builtin_amdgcn_update_dpp(0, x, 0x121, 0xF, 0xF, false);
  return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) + __builtin_amdgcn_readlane(x, 32) +
         __builtin_amdgcn_readlane(x, 48);
}
// Tokens sequence (64 tile + lane) attends, 0 past the batch: the planner below keeps one sequence per lane.
__device__ inline int var_len_of_lane(const DecodeParams& p, int tile) {
  const int b = tile * 64 + (int)(threadIdx.x & 63);
  return b < p.batch ? var_len(p, b) : 0;
}
// The planner keeps one sequence per lane: the lengths of the first 64 * kPlanTiles sequences stay in registers
// (batches up to 256), those of larger batches are re-read where needed.
constexpr int kPlanTiles = 4;
struct VarLens { int len[kPlanTiles]; };
__device__ inline void var_lens_load(const DecodeParams& p, VarLens& L) {
#pragma unroll
  for (int t = 0; t < kPlanTiles; ++t) L.len[t] = t * 64 < p.batch ? var_len_of_lane(p, t) : 0;
}
// ceil(len / c), the chunks of a sequence, without the integer division (some forty instructions, and the planner
// below does dozens per wave before its first load): the quotient is estimated with the float reciprocal of c,
// handed in as rc, and put right by one step either way.  Exact for 0 <= len, c < 2^23 with c >= 32: len + c - 1
// is then exact as a float, the estimate is off by less than 2^-21 of a quotient below 2^19, i.e. by less than one.
// Longer caches take the division.
__device__ inline int var_chunks_of(int len, int c, float rc, bool exact_floats) {
  const int x = len + c - 1;
  if (!exact_floats) return x / c;
  int q = (int)((float)x * rc);
  const int r = x - q * c;
  q += r >= c ? 1 : 0;
  q -= r < 0 ? 1 : 0;
  return q;
}
__device__ inline bool var_exact_floats(const DecodeParams& p) { return p.seq_len < (1 << 23); }

// The chunk length: the smallest multiple of 32 tokens for which all sequences together need at most
// p.var_chunks chunks (the grid), not below p.var_min_chunk and long enough that no sequence needs more than
// kMaxSplits.  The count for a candidate length is a wave-wide sum, and the candidates are bisected between
// total / var_chunks (too short unless every sequence ends on a chunk boundary) and
// total / (var_chunks - batch) (always enough: a sequence wastes less than one chunk).  Called by whole waves
// at the start of a kernel; every wave of a launch gets the same answer.
__device__ inline int var_chunk_tokens(const DecodeParams& p, const VarLens& L) {
  const int tiles = (p.batch + 63) >> 6;
  long long mine = 0;
#pragma unroll
  for (int t = 0; t < kPlanTiles; ++t) mine += L.len[t];
  for (int t = kPlanTiles; t < tiles; ++t) mine += var_len_of_lane(p, t);
  const long long total = ((long long)wave_sum((int)(mine >> 24)) << 24) + wave_sum((int)(mine & 0xFFFFFF));
  const int floor_c = max(p.var_min_chunk, (p.seq_len + kMaxSplits - 1) / kMaxSplits);
  auto round_up = [](long long c) { return (int)((c + kTile - 1) / kTile * kTile); };
  const int budget = p.var_chunks - p.batch;      // >= var_chunks / 2 by the host's choice of var_chunks
  // (the two bounds: 32-bit divisions where the total allows, which is nearly always; a 64-bit one is some
  // hundred and fifty instructions)
  const bool narrow = total < (1ll << 31) - (1 << 24) && p.var_chunks < (1 << 24);
  const long long need_hi = narrow ? (long long)(((uint32_t)total + (uint32_t)budget - 1) / (uint32_t)budget)
                                   : (total + budget - 1) / budget;
  const long long need_lo = narrow ? (long long)(((uint32_t)total + (uint32_t)p.var_chunks - 1) / (uint32_t)p.var_chunks)
                                   : (total + p.var_chunks - 1) / p.var_chunks;
  int hi = round_up(max((long long)floor_c, need_hi));
  int lo = round_up(max((long long)floor_c, need_lo));
  const bool fl = var_exact_floats(p);
  while (lo < hi) {
    const int mid = (lo + (hi - lo) / 2) / kTile * kTile;        // lo <= mid < hi, a multiple of 32
    const float rmid = 1.0f / (float)mid;
    int n = 0;
#pragma unroll
    for (int t = 0; t < kPlanTiles; ++t)
      if (t < tiles) n += var_chunks_of(L.len[t], mid, rmid, fl);
    for (int t = kPlanTiles; t < tiles; ++t) n += var_chunks_of(var_len_of_lane(p, t), mid, rmid, fl);
    if (wave_sum(n) <= p.var_chunks) hi = mid;
    else lo = mid + kTile;
  }
  return hi;
}
// Slot of the chunk list -> (sequence, chunk of it); false past the end of the list.  The chunk counts sit one
// sequence per lane; the tile of 64 sequences that holds the slot is found with wave-wide sums, the sequence
// inside it with a prefix sum over the lanes.  The chunk length goes to p.plan for the merge kernel.
__device__ inline bool var_plan(const DecodeParams& p, int slot, VarPlan& out) {
  VarLens L;
  var_lens_load(p, L);
  const int c = var_chunk_tokens(p, L);
  out.chunk_tokens = c;
  if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *p.plan = c;
  const int tiles = (p.batch + 63) >> 6, lane = threadIdx.x & 63;
  int first = 0;
  bool found = false;
  const float rc = 1.0f / (float)c;
  const bool fl = var_exact_floats(p);
  auto visit = [&](int t, int len) {              // tile t: does it hold the slot?  (wave-uniform)
    const int n = var_chunks_of(len, c, rc, fl);  // this lane's sequence: its chunks
    const int in_tile = wave_sum(n);
    if (slot < first + in_tile) {
      int incl = n;                               // inclusive prefix sum over the lanes
      for (int d = 1; d < 64; d <<= 1) {
        const int y = __shfl_up(incl, d);
        if (lane >= d) incl += y;
      }
      const int i = __ffsll((unsigned long long)__ballot(slot < first + incl)) - 1;   // first lane past the slot
      out.b = t * 64 + i;
      out.chunk = slot - first - (__builtin_amdgcn_readlane(incl, i) - __builtin_amdgcn_readlane(n, i));
      found = true;
    }
    first += in_tile;
  };
#pragma unroll
  for (int t = 0; t < kPlanTiles; ++t)
    if (t < tiles && !found) visit(t, L.len[t]);
  for (int t = kPlanTiles; t < tiles && !found; ++t) visit(t, var_len_of_lane(p, t));
  return found;
}
#endif

// Workspace carving: part_o first, then part_ml, both sized for kMaxSplits.
inline size_t workspace_o_floats(int batch, int n_q_heads, int head_dim) {
  return (size_t)batch * n_q_heads * kMaxSplits * head_dim;
}
inline size_t workspace_ml_floats(int batch, int n_q_heads) {
  return (size_t)batch * n_q_heads * kMaxSplits * 2;
}

// Launchers (each returns a hipError_t from hipGetLastError after the launch).
// A paged view of a pool: sequence b's token t lives in page block_table[b * max_blocks + (t >> page_shift)].
struct PagedView { const int32_t* block_table; int32_t max_blocks, page_shift, batch; };

// pos_dev (device, [B]) non-null: sequence b is written at pos_dev[b] + pos; a sequence whose tokens would not
// fit into [0, capacity) (paged: into its max_blocks pages) is skipped.  pv non-null: c is a pool of pages.
hipError_t launch_quantize(const tq_kv_cache& c, const void* k_new, const void* v_new, int pos,
                           const int32_t* pos_dev, int n_new, hipStream_t s, const PagedView* pv = nullptr);
hipError_t launch_dequant_dense(const tq_kv_cache& c, int seq_len, half_t* k_dense, half_t* v_dense,
                                hipStream_t s);
hipError_t launch_partial_valu(const DecodeParams& p, int batch, int head_dim, bool dense, hipStream_t s);
// Attention phase of the unfused comparator on the matrix cores (dense fp16 K^ / V^ in p.k_dense / p.v_dense,
// p.row_stride rows apart per (sequence, KV head)): head_dim 128 or 256, up to 16 query heads per KV head, one
// common length.  Chunks of whole 32-token tiles; writes the partials the merge kernel reads.
bool dense_mfma_supported(int head_dim, int gqa);
int dense_mfma_waves(int head_dim);
hipError_t launch_partial_dense_mfma(const DecodeParams& p, int batch, int head_dim, hipStream_t s);
bool mfma_supported(int head_dim, int gqa);
bool mfma_supports_group(int head_dim, int group_size, int capacity);   // groups of 32 always; 64 / 128: see there
// How many blocks share the stream of one KV head for this many query rows per KV head (1 where they fit one
// tile, 0 = unsupported): the planner counts batch * n_kv_heads * share rows, and the launch is given the same
// number in DecodeParams::kv_share.
int mfma_kv_share(int head_dim, int gqa);
// With merge_slot >= 0 the kernel also does the chunk merge (Eq. 6) and writes p.out: one launch per decode.
// The slot names the set of arrival counters the launch uses; mfma_merge_slot_of hands every workspace a set of
// its own, for the life of the process, or -1 once all sets are taken (the caller then runs the merge kernel).
// A launch whose rows are single chunks counts nothing and takes any slot >= 0.
bool mfma_can_merge(int batch, int n_kv_heads);
int mfma_merge_slot_of(const void* workspace);
hipError_t launch_partial_mfma(const DecodeParams& p, int batch, int head_dim, int merge_slot, hipStream_t s);
// head_dim 512: matrix-core kernel whose blocks take a tile of 16 or 32 query rows of one KV head
// (p.kv_share = row tiles per KV head, from wide_row_tiles; p.gqa = H_q / H_kv; p.n_queries query tokens).
bool wide_supported(int head_dim);
int wide_row_tiles(int rows, int64_t units, int tokens);
hipError_t launch_partial_wide(const DecodeParams& p, int batch, int head_dim, hipStream_t s);
hipError_t launch_reduce(const DecodeParams& p, int batch, int head_dim, hipStream_t s);
// Whether the merge of that many outputs runs as one block per (output row, KV head).
bool reduce_is_grouped(int head_dim, int64_t out_rows, int n_q_heads, int gqa);

}  // namespace tq
