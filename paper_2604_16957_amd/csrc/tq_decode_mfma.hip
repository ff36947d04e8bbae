// Matrix-core fused int4 decode attention for gfx950 (phase 1 of Sec. 3.2: per-chunk partials; for
// short sequences also phase 2, the chunk merge of Eq. 6, done by the block that finishes last).
//
// Why matrix cores: with a GQA group of G query heads every stored element is used by G heads;
// at G=8 and d=128 that is 25.6 flop per HBM byte, above the vector-ALU ridge of the chip, so the
// two contractions (the score step and the accumulator update of Alg. 1) run on v_mfma_f32_16x16x32_f16 and the vector ALU only
// unpacks nibbles, applies the per-group scale/zero-point of K and does the softmax.
//
// Data path: the packed stream never passes through vector registers on its way in.  Each wave owns
// a ring of LDS stages and fills them with direct global->LDS loads (global_load_lds_dwordx4: 64
// lanes x 16 B = 1 KB per instruction, tracked by vmcnt), one 32-token supertile ahead of the one
// being consumed, with no register cost; the per-lane source address of such a load is free, so K
// codes and the fp16 scale / zero-point arrays are gathered into the order the lanes read them back
// in.  What a supertile needs from LDS is copied into registers ahead of use (its V part at the start
// of its K phase, the next supertile's K part during the current softmax / P V phase).  The ring is
// only two stages deep on purpose: once the last byte has landed every wave still has `ring depth`
// supertiles to compute, and at 16 supertiles per wave that drain outweighs a deeper prefetch.
// The stream is read once, and its loads say so (non-temporal cache policy, template parameter NT).
//
// Exactness: codes 0..15 enter the MFMA as fp16 SUBNORMALS (the nibble sits in the low mantissa
// bits, value c*2^-24, or c*2^-20 for a nibble at bit 4) so unpacking is one AND per pair of
// elements; products and sums are exact in the fp32 accumulator.  Scale and zero-point are applied
// outside the contraction:  q.k^ = sum_g s_g (q_g.c_g - z_g sum(q_g))  in fp32 on the vector ALU, and
// sum_t p_t v^_t = sum_t (p_t s_t) c_t - sum_t (p_t s_t) z_t, where the product p_t s_t is rounded
// to fp16 once and the SAME rounded operand multiplies the codes and (in a small extra MFMA whose
// B operand is the stored fp16 zero-point itself) the zero-points.
// The matrix core aligns the 32 products of an MFMA to its fp32 accumulator and TRUNCATES each of
// them, so an accumulator that grows (a sum of positive terms, ~200x larger than the result it is
// later differenced into) costs accuracy in proportion to the tokens it has taken in.  Both sums are
// therefore kept balanced around zero, at no cost in matrix instructions: a supertile is two 16-token
// tiles, and the weights of the SECOND tile enter the A operand negated.  For the codes the second
// tile's nibbles are complemented (15 - c, one NOT per packed word):
//   sum_t0 w c - sum_t1 w (15 - c)  =  sum_t w c  - 15 sum_t1 w ,
// for the zero-points the second tile's B entries get their sign flipped and a constant B operand
// (0 on first-tile slots, 15 on second-tile slots) follows:
//   sum_t w z - 15 sum_t1 w .
// The two 15 sum_t1 w terms cancel in the difference, exactly (same A operand), and each running sum
// stays at the size of the result.
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
//   it reads the same packed word of 8 tokens and regroups it with one v_perm_b32 per (token pair, byte);
//   a byte's two nibbles go through the matrix core mixed (n_even + 16 n_odd, still an exact subnormal)
//   next to n_even alone, and the odd dim is recovered from the two sums at the end (see `pv`).
//
// Work split: grid (n_splits, H_kv * kv_share, B), 8 waves per block, one block per compute unit; the
// waves of a block share the chunk's 32-token supertiles in a fixed pattern (17:15 or 9:7 between the older
// and the younger wave of a SIMD, see the kernel), keep private online-softmax state, and are merged through
// LDS so that the block writes one partial (o_c, m_c, l_c) per query row.
//
// Query rows: the tile's GP columns take the G heads of the GQA group (Sec. 3.1), or, with several query
// tokens per sequence (the sequence's last n_queries tokens, causal among themselves), the n_queries * G
// rows (token, head) of one KV head; rows beyond one tile go to further blocks on the same KV head
// (kv_share of them).  Per-row limits (causal end, window start) only exist in the masked path that the
// ragged last supertile takes anyway.
#include <mutex>
#include <type_traits>
#include <unordered_map>

#include "tq_internal.h"

namespace tq {
namespace {

typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;
constexpr int kMaxDevices = 64;

// Arrival counters of the in-kernel chunk merge: one per (b, kv head), in kCounterSlots independent sets.  A set
// belongs to ONE WORKSPACE (the host keeps the table, see merge_slot_of): calls that may be in flight at the same
// time have different workspaces by the contract of the decode calls (they would overwrite each other's partials
// otherwise), hence different sets, whether they are issued eagerly or replayed from a captured graph, which
// keeps the set it was captured with.  Zero when the module is loaded; the block that arrives last wraps its
// counter back to zero, so every launch leaves them zero again.  A workspace that finds all sets taken gets the
// merge kernel instead (two launches: always correct).
constexpr int kCounterSlots = 256;
constexpr int kCountersPerSlot = 2048;
// Within a set, the counters of neighbouring (b, KV head) rows lie 128 bytes apart (row r at (r % 64) * 32 + r / 64):
// the blocks of a launch finish at about the same time, and their atomics on counters that share a cache line
// queue up behind one another at that line's channel (8 KV heads x 32 chunks on one line: 1.4 us of a 13 us call).
__device__ __attribute__((aligned(256))) unsigned int g_arrivals[kCounterSlots * kCountersPerSlot];
static_assert(kCountersPerSlot == 64 * 32, "the spreading below");
__device__ __forceinline__ int arrival_counter(int row) { return (row & 63) * 32 + (row >> 6); }
constexpr float kSlack = 2.0f;              // log2 units: exp2(score - reference) <= 4
constexpr uint32_t kMaskLo = 0x000F000Fu;   // nibbles 0 and 4 of a word -> fp16 subnormals c * 2^-24
constexpr uint32_t kMaskHi = 0x00F000F0u;   // nibbles 1 and 5           -> c * 2^-20
constexpr uint32_t kPos15Odd = 0x4B800000u; // fp16 pair (0, 15): k-slots alternate first tile, second tile

template <int D, int GP, int NW>
struct Cfg {
  static constexpr int NG = D / kGroup;          // quantisation groups per token
  static constexpr int GR = 16 / GP;             // group replicas among the 16 columns / rows
  static constexpr int NA = NG / GR;             // groups handled per lane (accumulators per K tile)
  static constexpr int NJ = NG;                  // K MFMAs per 16-token tile (= packed words per lane)
  static constexpr int NCS = D / 128;            // V column sets (16 packed words each)
  static constexpr bool SWAP = (D == 128 && GP == 8);
  // WIDE: every column of the tile is a query row of its own (no group replicas), so each of the four groups of
  // a token has its own score accumulator, and the P V columns are regrouped so that the 16 columns of one
  // matrix instruction lie in ONE group (see `pv`): its A operand p * s_v is then right for all of them.
  static constexpr bool WIDE = (GR == 1);
  static constexpr int NDW = (NA + 1) / 2;       // dwords of fp16 scales (or zero-points) a lane needs per token
  static_assert(NG % GR == 0 && NA >= 1 && (NA <= 2 || (WIDE && D == 128)), "unsupported (head_dim, padded GQA) pair");
  // K MFMA j takes, from lane block kq, packed word a_word(j,kq) of group a_group(j,kq) and adds
  // into accumulator acc(j); column replica r of that accumulator stands for group r*NA + acc(j).
  static __device__ constexpr int a_group(int j, int kq) {
    return WIDE ? j : SWAP ? 2 * (kq >> 1) + (j & 1) : (D == 128 ? kq : 2 * kq + (j >> 2));
  }
  static __device__ constexpr int a_word(int j, int kq) {
    return WIDE ? kq : SWAP ? 2 * (j >> 1) + (kq & 1) : (D == 128 ? j : (j & 3));
  }
  static __device__ constexpr int acc(int j) {
    return WIDE ? j : SWAP ? (j & 1) : (D == 128 ? 0 : (NA == 2 ? (j >> 2) : 0));
  }

  // LDS stage of one 32-token supertile, in the order the stream is laid out in HBM
  static constexpr int TB = D / 2;               // bytes of codes per token
  static constexpr int KT = 16 * TB;             // one 16-token K tile
  static constexpr int VB = 32 * TB;             // V codes of the supertile
  static constexpr int SZ = 32 * NG * 2;         // one fp16 scale (or zero-point) array of the supertile
  static constexpr int OFF_V = 2 * KT, OFF_KS = OFF_V + VB, OFF_KZ = OFF_KS + SZ, OFF_VS = OFF_KZ + SZ,
                       OFF_VZ = OFF_VS + SZ, STAGE = OFF_VZ + SZ;
  static constexpr int NS = 2;                  // ring depth per wave (LDS: 160 KB per CU)
  // The two waves of a SIMD split its supertiles (PER / 2 + 1) : (PER / 2 - 1), the older wave the larger share:
  // 17 : 15 where the loop is leanest (measured: the older wave of the d = 128, 8-row kernel takes 1.32 us per
  // supertile, the younger 1.45 us), 9 : 7 elsewhere
  static constexpr int PER = (D == 128 && GP == 8) ? 32 : 16;
  static constexpr int LPS = 2 * (KT / 1024) + VB / 1024 + 4 * (SZ / 256);   // load instructions per stage
  static constexpr int RING = NW * NS * STAGE;
  static constexpr int MERGE = (NW * GP * D + 2 * NW * GP) * 4;  // o, m, l
  // the block-merge area sits behind the rings where both fit into the 160 KB of a compute unit, else on top of them
  static constexpr bool ALIAS = RING + MERGE > 160 * 1024;
  static constexpr int OFF_MERGE = ALIAS ? 0 : RING;
  // Where the query block of a wave lands before it is turned into operands: in an area of its own if
  // there is room, so that the whole ring can be filled at once; else in the last ring slot.
  static constexpr int QBLK = GP * D * 2;
  static_assert(QBLK <= STAGE, "the query block borrows one ring slot");
  static constexpr bool QSEP = !ALIAS && RING + MERGE + NW * QBLK <= 160 * 1024;
  static constexpr int OFF_QBLK = RING + MERGE;
  static constexpr int SMEM = ALIAS ? (RING > MERGE ? RING : MERGE) : RING + MERGE + (QSEP ? NW * QBLK : 0);
  // The fp16 scale and zero-point arrays are fetched dword by dword (two groups of one token), and the
  // direct loads may gather: with NA == 2 a lane needs exactly one dword per token, so the dwords are
  // laid out in LDS as [kq][replica][tile][i] and a lane reads its eight tokens with two 16-byte reads; with
  // NA == 4 (WIDE) it needs both dwords of a token: [kq][dword][tile][i], four 16-byte reads.
  static constexpr bool PERM = (NA == 2);
  // Whether the K part of the next supertile is fetched into registers during the current one (it is
  // not where the accumulators alone take half of the register file).
  static constexpr bool PFK = !(D == 256 && NA == 2);
  static __device__ constexpr int sz_token(int P) {       // token (0..31) whose dword sits at stage dword P
    return WIDE ? 16 * ((P >> 2) & 1) + 4 * (P & 3) + (P >> 4)
                : PERM ? 16 * ((P >> 2) & 1) + 4 * (P & 3) + (P >> 3) / GR : P / (NG / 2);
  }
  static __device__ constexpr int sz_column(int P) {      // which dword of that token's NG/2
    return WIDE ? (P >> 3) & 1 : PERM ? (P >> 3) % GR : P % (NG / 2);
  }
};

// token held by row r of a 16-token K tile (and by the matching k-slots of the P V contraction):
// lane block kq then owns tokens kq, kq+4, kq+8, kq+12 of each tile, which keeps the four blocks'
// LDS reads of the V codes on different banks
__device__ __forceinline__ constexpr int tok_of_row(int r) { return 4 * (r & 3) + (r >> 2); }

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

// ---- direct global -> LDS loads.  Written as asm so that the compiler does not serialise them
// against later LDS reads: each wave tracks its own ring with explicit vmcnt waits instead.
// Lane l's bytes land at lds_base + l * (16 | 4).  M0 carries the LDS base of the instruction.
// (M0 cannot be named as a clobber: the compiler reserves it and rejects that.  It keeps no value live in M0
// across other instructions either: each of its own uses, such as an indexed register move, writes M0 right
// before.  The kernels in this file and in tq_decode_wide.hip contain no such use at all: in their assembly M0
// appears inside these blocks only.)
// NT = the non-temporal cache policy: the packed stream is read once, and telling the caches so is worth
// 6-9 % of the kernel's time (plain loads of the same 168 MB: 28 us per launch, non-temporal: 25 us).
// Where several blocks stream the same KV head the later readers live on what the first left in the
// caches, and the loads stay plain.
#define TQ_LDS_LOAD(NT_, TEXT_PLAIN, TEXT_NT, ...)                     \
  do {                                                                 \
    if constexpr (NT_) asm volatile(TEXT_NT :: __VA_ARGS__ : "memory"); \
    else asm volatile(TEXT_PLAIN :: __VA_ARGS__ : "memory");           \
  } while (0)
template <bool NT>
__device__ __forceinline__ void dma4(const void* sbase, uint32_t voff, uint32_t lds_base) {
  TQ_LDS_LOAD(NT, "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1",
              "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1 nt",
              "v"(voff), "s"(sbase), "s"(lds_base));
}
__device__ __forceinline__ void dma16_lane(const void* addr, uint32_t lds_base) {   // per-lane 64-bit address
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
               :: "v"(addr), "s"(lds_base) : "memory");
}
__device__ __forceinline__ void dma4_lane(const void* addr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off"
               :: "v"(addr), "s"(lds_base) : "memory");
}
// Several loads of one array behind a single M0: the instruction's immediate offset moves the global
// and the LDS address alike, so pieces that are equally far apart on both sides share the base.
template <bool NT, int O1>
__device__ __forceinline__ void dma16_x2(const void* sbase, uint32_t voff, uint32_t lds_base) {
  TQ_LDS_LOAD(NT, "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\t"
                  "global_load_lds_dwordx4 %0, %1 offset:%3",
              "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\t"
              "global_load_lds_dwordx4 %0, %1 offset:%3 nt",
              "v"(voff), "s"(sbase), "s"(lds_base), "n"(O1));
}
template <bool NT, int O0, int O1>
__device__ __forceinline__ void dma16_x2o(const void* sbase, uint32_t voff, uint32_t lds_base) {
  TQ_LDS_LOAD(NT, "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3\n\t"
                  "global_load_lds_dwordx4 %0, %1 offset:%4",
              "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3 nt\n\t"
              "global_load_lds_dwordx4 %0, %1 offset:%4 nt",
              "v"(voff), "s"(sbase), "s"(lds_base), "n"(O0), "n"(O1));
}
template <bool NT>
__device__ __forceinline__ void dma16_x4(const void* sbase, uint32_t voff, uint32_t lds_base) {
  TQ_LDS_LOAD(NT, "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\t"
                  "global_load_lds_dwordx4 %0, %1 offset:1024\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048\n\t"
                  "global_load_lds_dwordx4 %0, %1 offset:3072",
              "s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 nt\n\t"
              "global_load_lds_dwordx4 %0, %1 offset:1024 nt\n\tglobal_load_lds_dwordx4 %0, %1 offset:2048 nt\n\t"
              "global_load_lds_dwordx4 %0, %1 offset:3072 nt",
              "v"(voff), "s"(sbase), "s"(lds_base));
}
// device-scope (all compute dies) store and load of one float, without any cache-wide maintenance
__device__ __forceinline__ void st_dev2(float* p, float a, float b) {      // two floats, 8-byte aligned
  const uint64_t bits = (uint64_t)__builtin_bit_cast(uint32_t, a) | ((uint64_t)__builtin_bit_cast(uint32_t, b) << 32);
  __hip_atomic_store(reinterpret_cast<uint64_t*>(p), bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
template <int N>
__device__ __forceinline__ void wait_loads() {               // until at most N loads are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

// PLAIN = the launch has none of the per-sequence machinery: one common length, a contiguous cache, one query
// token, one block per (chunk, KV head, sequence).  Everything below that serves the other shapes then folds
// away at compile time; what is left is a short prologue (the first loads leave sooner) and a loop without the
// scalar bookkeeping of pages and packed rows.
//
// GS = log2(group size / 32).  Groups of 64 or 128 elements (Sec. 2.1) change what the stored scales and zero-points
// MEAN, not what the kernel does with them: the direct loads fetch, for every 32-dim block of a token, the dword
// that holds its group's value (one dword of two groups per token at 64, one dword of two TOKENS at 128), and the
// lane copies the half it needs into both halves of the register, after which everything is as with groups of 32.
// Instantiated for the layouts whose metadata is gathered dword by dword (d = 128 with 8 or 16 rows).
template <int D, int GP, int NW, bool NT, bool PLAIN, int GS = 0>
__global__ __launch_bounds__(NW * 64, (NW + 3) / 4) void decode_partial_mfma_kernel(DecodeParams p) {
  using C = Cfg<D, GP, NW>;
  static_assert(GS == 0 || ((C::PERM || C::WIDE) && !PLAIN), "larger groups: the gathered metadata layouts only");
  constexpr int SZB = (D / kGroup * 2) >> GS;     // bytes of one metadata array per token
  constexpr int NG = C::NG, NA = C::NA, NJ = C::NJ, NCS = C::NCS, TB = C::TB, NS = C::NS, LPS = C::LPS, GR = C::GR;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  if constexpr (PLAIN) {
    // every kernel argument the prologue needs, asked for at once: one round trip to the scalar cache before the
    // first stream loads leave instead of two (the compiler otherwise fetches q and start behind a branch)
    asm volatile("" :: "s"(p.q), "s"(p.start), "s"(p.k_codes), "s"(p.v_codes), "s"(p.k_scale), "s"(p.k_zero),
                 "s"(p.v_scale), "s"(p.v_zero), "s"(p.seq_len), "s"(p.tokens_per_split), "s"(p.row_stride),
                 "s"(p.n_kv_heads), "s"(p.n_q_heads), "s"(p.gqa));
  }
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, kq = lane >> 4;
  const int hl = c % GP, rep = c / GP;            // head and group replica of this lane's column / row
  int split = blockIdx.x, b = blockIdx.z, tokens_per_split = p.tokens_per_split, part_stride = p.n_splits;
  int kvv = blockIdx.y;                           // KV head x part of its query group (see kv_share)
  // Many short sequences (more units of work than the chip holds blocks): a block takes NW / W of them, W waves
  // each, instead of one.  With a common length a unit is a (sequence, KV head) row of a single chunk, and
  // blockIdx.y counts groups of rows of the list [batch][KV head x part]; with per-sequence lengths a unit is a
  // slot of the chunk list, and blockIdx.x counts groups of slots.  A wave past the end of its list has no tokens
  // and only keeps the barriers company.
  const int W = PLAIN ? NW : p.waves_per_row;     // NW: the whole block on one unit
  const bool whole = W == NW;
  bool row_valid = true;
  if (!PLAIN && !whole && p.var_chunks == 0) {
    const int rows_y = p.n_kv_heads * p.kv_share, total = p.batch * rows_y;
    // One wave per row and per-sequence lengths: in list order a block's eight waves would all get rows of ONE
    // sequence, and the launch would last as long as the longest sequence.  The two waves of a SIMD share its
    // vector ALU, so what has to be even is the sum of their two rows: every block orders the sequences by length
    // (a stable counting sort on the supertile count, in the idle block-merge area of LDS: the same order in every
    // block) and pairs the i-th shortest with the i-th longest, the older wave of the SIMD taking the longer.
    bool paired = false;
    if constexpr (!C::ALIAS) {
      constexpr int kPairMaxBatch = NW * 64;                 // one sequence per thread
      static_assert(C::MERGE >= (NW * 64 + 128 + kPairMaxBatch) * 4, "the ordering uses the block-merge area");
      paired = W == 1 && p.seq_lens != nullptr && (p.batch & 1) == 0 && p.batch <= kPairMaxBatch;
      if (paired) {
        int* const cnt = reinterpret_cast<int*>(smem + C::OFF_MERGE);      // [wave][64]: sequences of the wave per supertile count
        int* const tot = cnt + NW * 64;                                     // [64]: sequences per count, then where each count starts
        int* const order = tot + 128;                                       // [batch]: sequences, shortest first
        const int t = threadIdx.x;                                          // this thread's sequence
        const bool have = t < p.batch;
        const int bk = have ? min(63, (var_len(p, t) + 31) >> 5) : 64;
        cnt[t] = 0;
        __syncthreads();
        // place among the wave's sequences of the same count, by index
        int ahead = 0;
        for (uint64_t todo = __builtin_amdgcn_ballot_w64(have); todo != 0;) {
          const int lead = __builtin_ctzll(todo);
          const int bv = __shfl(bk, lead);
          const uint64_t same = __builtin_amdgcn_ballot_w64(bk == bv);
          if (bk == bv) ahead = __builtin_popcountll(same & ((1ull << lane) - 1));
          if (lane == lead) cnt[wave * 64 + bv] = __builtin_popcountll(same);
          todo &= ~same;
        }
        __syncthreads();
        if (t < 64) {                                        // count t: where each wave's share starts inside it
          int acc = 0;
          for (int wv = 0; wv < NW; ++wv) { const int n_w = cnt[wv * 64 + t]; cnt[wv * 64 + t] = acc; acc += n_w; }
          tot[t] = acc;
        }
        __syncthreads();
        if (t == 0) {
          int acc = 0;
          for (int k = 0; k < 64; ++k) { const int n_k = tot[k]; tot[k] = acc; acc += n_k; }
        }
        __syncthreads();
        if (have) order[tot[bk] + cnt[wave * 64 + bk] + ahead] = t;
        __syncthreads();
        const int half = p.batch >> 1;
        const int pair = blockIdx.y * 4 + (wave & 3);        // waves w and w + 4 sit on one SIMD
        row_valid = pair < half * rows_y;
        const int pc = min(pair, half * rows_y - 1);
        const int i = pc % half;
        kvv = __builtin_amdgcn_readfirstlane(pc / half);
        b = __builtin_amdgcn_readfirstlane(min(max(order[(wave >> 2) ? i : p.batch - 1 - i], 0), p.batch - 1));
      }
    }
    if (!paired) {
      const int row = blockIdx.y * (NW / W) + wave / W;
      row_valid = row < total;
      const int r = min(row, total - 1);
      b = __builtin_amdgcn_readfirstlane(r / rows_y);
      kvv = __builtin_amdgcn_readfirstlane(r - (r / rows_y) * rows_y);
    }
  }
  const int kv_share = PLAIN ? 1 : p.kv_share;
  const int kv = PLAIN ? kvv : kvv / kv_share;    // the KV head whose rows are read
  if (!PLAIN && p.var_chunks > 0) {                         // per-sequence lengths: which (sequence, chunk) is this block's
    VarPlan vp;
    vp.b = 0;
    vp.chunk = 0;
    const bool listed = var_plan(p, whole ? blockIdx.x : blockIdx.x * (NW / W) + wave / W, vp);
    if (whole && !listed) return;                 // (with several units per block nobody leaves before the barriers)
    row_valid = listed;
    split = __builtin_amdgcn_readfirstlane(vp.chunk);     // (wave-uniform by construction: tell the compiler)
    b = __builtin_amdgcn_readfirstlane(vp.b);
    tokens_per_split = __builtin_amdgcn_readfirstlane(vp.chunk_tokens);
    part_stride = kMaxSplits;
  }
  const int G = p.gqa;
  // Several query tokens per sequence (they are the sequence's last NQ tokens and causal among themselves):
  // a KV head then has NQ * GF query rows, row r = t * GF + g for query token t and head g of the group,
  // cut into kv_share parts of G rows; this block holds rows part * G .. part * G + G - 1.
  const int NQ = PLAIN ? 1 : p.n_queries, GF = PLAIN ? G : p.gqa_full;
  const int part = kvv - kv * kv_share;
  auto query_token = [&](int h) { return NQ > 1 ? min(part * G + h, NQ * GF - 1) / GF : 0; };
  auto query_row = [&](int h) -> int64_t {        // row of q / out / the partials that tile row h stands for
    const int r = part * G + h, t = query_token(h);
    return (int64_t)(b * NQ + t) * p.n_q_heads + kv * GF + (r - t * GF);
  };

  char* const ring = smem + wave * (NS * C::STAGE);
  const uint32_t ring_lds =
      (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * (NS * C::STAGE);

  // ---- addressing: wave-uniform bases (scalar registers) + per-lane 32-bit byte offsets
  // tokens this sequence attends: the common length, or its own (a chunk past its end is empty); with a
  // sliding window the row simply starts `start` tokens later
  const bool var_lens = !PLAIN && p.seq_lens != nullptr;
  const int seq = !row_valid ? 0 : var_lens ? var_len(p, b) : p.seq_len;
  const int start = var_lens ? var_start(p, b) : p.start;
  // first row of the six arrays this block reads from: the sequence's own row (contiguous cache), or the
  // pool's row 0 (paged cache: the page's rows are added supertile by supertile)
  const bool paged = !PLAIN && p.block_table != nullptr;
  // paged cache: token indices below count from `start` as well, but the rows are found page by page; the
  // window's first token may lie up to 31 tokens after `start` (see var_start)
  const int lead = (paged && var_lens) ? var_first(p, b) - start : 0;
  const int pstart = paged ? start : 0;           // added to a token index where a page is looked up
  const int64_t row0 = paged ? 0 : (int64_t)(b * p.n_kv_heads + kv) * p.row_stride + start;
  const int begin0 = split * tokens_per_split;    // first token of the chunk
  // A chunk past the end of its sequence has nothing to emit: the merge kernel works out from the same
  // lengths which chunks exist.  (With the in-kernel merge the block still has to be counted in, so it
  // goes through and publishes an empty partial.)
  if (!PLAIN && whole && begin0 >= seq && p.merge_slot < 0) return;
  const int end = max(begin0, min(seq, begin0 + tokens_per_split));
  // Several query tokens under a sliding window: the rows start at different tokens (row t one token after
  // row t - 1); the supertile that holds those starts takes the masked path too (wave 0, after its other work)
  // and the fast path starts behind it.  The same goes for a paged cache under a window, whose first supertile
  // holds `lead` tokens before the window.  With both, the rows start at tokens lead .. lead + NQ - 1, which may
  // straddle the sequence's first two supertiles: then the second is masked as well, in whichever chunk it lies.
  const bool rows_windowed = !PLAIN && NQ > 1 && p.row_window > 0;
  const bool straddle = rows_windowed && lead + NQ - 1 >= 32;
  const bool head = (rows_windowed || lead > 0) && end > begin0 && (begin0 == 0 || (begin0 == 32 && straddle));
  const bool head2 = head && begin0 == 0 && straddle && end > 32;
  const int begin = begin0 + (head2 ? 64 : head ? 32 : 0);   // origin of the supertile indices below
  // `seq` is what the last query token attends; query token t attends NQ - 1 - t tokens fewer.  Supertiles
  // that every row attends in full take the fast path; the sequence's last one or two (ragged, or holding
  // tokens some rows must not see) take the masked path.
  const int n_full = max(0, min(end, seq - (NQ - 1)) - begin) >> 5;
  const int n_tail = ((end - begin + 31) >> 5) - n_full;   // 0, 1 or 2 (NQ <= 8)
  const int last_tok = pstart + seq - 1;
  const int end_col = min(end, seq - (NQ - 1 - query_token(hl)));   // first token this lane's column must not see
  // ... and, under a window, the first one it sees: its own length less the window, relative to the row start
  const int lo_col = !head ? 0 : rows_windowed
                                     ? max(0, start + seq - (NQ - 1 - query_token(hl)) - p.row_window) - start : lead;
  const char* kc_row = reinterpret_cast<const char*>(p.k_codes) + row0 * TB;
  const char* vc_row = reinterpret_cast<const char*>(p.v_codes) + row0 * TB;
  const char* sz_row[4] = {reinterpret_cast<const char*>(p.k_scale) + row0 * SZB,
                           reinterpret_cast<const char*>(p.k_zero) + row0 * SZB,
                           reinterpret_cast<const char*>(p.v_scale) + row0 * SZB,
                           reinterpret_cast<const char*>(p.v_zero) + row0 * SZB};
  // Where a supertile starts: in a contiguous cache, `tok0` tokens into the sequence's own row; in a paged
  // one, in the page the block table names, at the token's offset inside the page (supertiles never
  // straddle pages: a page is a multiple of 32 tokens and paged sequences start at token 0).
  struct Bases { const char* k; const char* v; const char* s[4]; };
  const Bases row_bases = {kc_row, vc_row, {sz_row[0], sz_row[1], sz_row[2], sz_row[3]}};
  const int32_t* const tbl = paged ? p.block_table + (int64_t)b * p.max_blocks : nullptr;
  const int page_mask = (1 << p.page_shift) - 1;
  auto page_of = [&](int tok0) { return tbl[min(tok0 >> p.page_shift, p.max_blocks - 1)]; };
  auto bases_of_page = [&](int page) -> Bases {   // row 0 of `page` for this KV head (a page is 2^page_shift rows)
    const int64_t r = (int64_t)(page * p.n_kv_heads + kv) << p.page_shift;
    const int64_t rc = r * TB, rs = r * SZB;
    return {row_bases.k + rc, row_bases.v + rc, {row_bases.s[0] + rs, row_bases.s[1] + rs, row_bases.s[2] + rs,
                                                 row_bases.s[3] + rs}};
  };
  const uint32_t koff = tok_of_row(c) * TB + kq * (D / 8);   // this lane's 16 B (x D/128) of a K tile
  // scale / zero-point arrays: destination dword u*64+lane of the stage comes from (token, dword) of the supertile
  uint32_t sz_tok[C::SZ / 256], sz_col[C::SZ / 256];
#pragma unroll
  for (int u = 0; u < C::SZ / 256; ++u) {
    sz_tok[u] = C::sz_token(u * 64 + lane);
    sz_col[u] = C::sz_column(u * 64 + lane);
  }

  // Fills the ring slot at LDS address l with the supertile whose codes start off_c bytes into the row:
  // LPS load instructions, all 64 lanes each.  vk, vv, vs are the per-lane byte offsets inside the
  // supertile (K tile, V block, scale array).
  const uint32_t lane16 = lane * 16;
  uint32_t szoff[C::SZ / 256];
#pragma unroll
  for (int u = 0; u < C::SZ / 256; ++u)           // (larger groups: the token's only dword, or the dword it shares)
    szoff[u] = GS == 0 ? (sz_tok[u] * (NG / 2) + sz_col[u]) * 4 : GS == 1 ? sz_tok[u] * 4 : (sz_tok[u] >> 1) * 4;
  auto issue_at = [&](uint32_t l, const Bases& B, uint32_t off_c, uint32_t vk, uint32_t vv,
                      const uint32_t (&vs)[C::SZ / 256]) {
    const uint32_t off_s = off_c >> (3 + GS);     // SZB / TB: metadata bytes per code byte
    // the supertile's offset goes into the (scalar) base, not into the per-lane offsets: scalar adds are free
    // next to a vector ALU that is the kernel's bottleneck
    const char* const bk = B.k + off_c;
    const char* const bv = B.v + off_c;
    if constexpr (D == 128) {
      dma16_x2<NT, 1024>(bk, vk, l);                                   // two K tiles: 1 KB apart on both sides
      dma16_x2<NT, 1024>(bv, vv, l + C::OFF_V);
    } else {
      dma16_x2<NT, 2048>(bk, vk, l);                                   // first 16 B of each lane, tiles 0 and 1
      dma16_x2o<NT, 16, 2064>(bk, vk, l + 1024 - 16);                  // second 16 B: +16 in HBM, +1024 in LDS
      dma16_x4<NT>(bv, vv, l + C::OFF_V);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int u = 0; u < C::SZ / 256; ++u) dma4<NT>(B.s[a] + off_s, vs[u], l + C::OFF_KS + a * C::SZ + u * 256);
  };
  // supertile starting tok0 tokens into the sequence (page known in the paged case) -> ring slot at l
  auto issue_tok = [&](uint32_t l, int tok0, int page, uint32_t vk, uint32_t vv, const uint32_t (&vs)[C::SZ / 256]) {
    if (paged) issue_at(l, bases_of_page(page), (uint32_t)(tok0 & page_mask) * TB, vk, vv, vs);
    else issue_at(l, row_bases, (uint32_t)tok0 * TB, vk, vv, vs);
  };
  auto issue_tail = [&](int slot, int sidx) {     // ragged last supertile: clamp every token to the last valid one
    const int base = pstart + begin + sidx * 32;
    const uint32_t l = ring_lds + slot * C::STAGE;
    // token index -> row of the arrays below: the sequence's row, or the page that holds this supertile
    const Bases B = paged ? bases_of_page(page_of(base)) : row_bases;
    const int row_first = paged ? (base & ~page_mask) : 0;
    const char* const kc_row = B.k - (int64_t)row_first * TB;
    const char* const vc_row = B.v - (int64_t)row_first * TB;
    const char* const sz_row[4] = {B.s[0] - (int64_t)row_first * SZB, B.s[1] - (int64_t)row_first * SZB,
                                   B.s[2] - (int64_t)row_first * SZB, B.s[3] - (int64_t)row_first * SZB};
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int tok = min(base + 16 * t + tok_of_row(c), last_tok);
#pragma unroll
      for (int ch = 0; ch < D / 128; ++ch)
        dma16_lane(kc_row + (int64_t)tok * TB + kq * (D / 8) + ch * 16, l + t * C::KT + ch * 1024);
    }
#pragma unroll
    for (int u = 0; u < C::VB / 1024; ++u) {
      const int chunk = u * 64 + lane;            // 16-byte chunk of the supertile's V codes
      const int tok = min(base + chunk / (TB / 16), last_tok);
      dma16_lane(vc_row + (int64_t)tok * TB + (chunk % (TB / 16)) * 16, l + C::OFF_V + u * 1024);
    }
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
      for (int u = 0; u < C::SZ / 256; ++u) {
        const int tok = min(base + (int)sz_tok[u], last_tok);
        const int64_t src = GS == 0 ? (int64_t)tok * (NG * 2) + sz_col[u] * 4 : GS == 1 ? (int64_t)tok * 4 : (int64_t)(tok >> 1) * 4;
        dma4_lane(sz_row[a] + src, l + C::OFF_KS + a * C::SZ + u * 256);
      }
  };
  auto tok_of = [&](int sidx) { return pstart + begin + sidx * 32; };
  auto issue = [&](int slot, int sidx) {
    const int tok0 = tok_of(sidx);
    issue_tok(ring_lds + slot * C::STAGE, tok0, paged ? page_of(tok0) : 0, koff, lane16, szoff);
  };
  // ---- work distribution.  The block's 8 waves sit two to a SIMD (waves w and w+4), and the SIMD
  //      issues from its older wave first, so wave w gets through a supertile in less time than wave w+4
  //      (about 7/9 of it in the heavier instances, 10/11 in the leanest).  The chunk's supertiles are
  //      therefore dealt round-robin to the four SIMDs, and of every PERIOD that a SIMD gets, its older wave
  //      takes PERIOD/2 + 1 and the younger PERIOD/2 - 1, in a fixed pattern.
  //      The split is static: the summation order, and with it every output bit, is the same on every
  //      launch.  The ragged last supertile, if any, goes to the wave whose turn it would be and takes
  //      the clamped path.
  static_assert(NW == 8, "the work split assumes two waves per SIMD");
  const int simd = wave & 3, young = wave >> 2;
  constexpr int PERIOD = C::PER, OLD = PERIOD / 2 + 1, YNG = PERIOD / 2 - 1;   // of every PER supertiles of a SIMD: older wave, younger wave
  const int sub = wave % W;                       // (several rows per block: the W waves of a row take its supertiles in turn)
  auto sidx_of = [&](int i) {                     // i-th supertile of this wave -> supertile of the chunk
    if (!whole) return W * i + sub;
    const int blk = young ? i / YNG : i / OLD, j = i - blk * (young ? YNG : OLD);
    const int k = PERIOD * blk + (young ? 2 * j + 1 : (j < PERIOD / 2 ? 2 * j : PERIOD - 1));
    return 4 * k + simd;
  };
  auto count_of = [&](int n) {                    // how many of the chunk's first n supertiles are this wave's
    if (!whole) return n > sub ? (n - sub + W - 1) / W : 0;
    const int K = n > simd ? (n - simd + 3) >> 2 : 0, r = K % PERIOD;
    return young ? YNG * (K / PERIOD) + (r >> 1) : OLD * (K / PERIOD) + ((r + 1) >> 1);
  };
  const int n_mine = count_of(n_full);
  // ---- prologue: the query rows of this KV head's group come in by direct load as well (so that every
  //      vector-memory operation of the kernel is one of the counted loads), then the ring is filled.
  //      Where the query block has to borrow the last ring slot, that slot is filled once the query
  //      operands sit in registers.
  // One stage is issued before the query operands are built.  The second follows once those operands sit in
  // registers (d = 256) or, at d = 128, only when the first has landed and its K part has been read: with every
  // wave's first stage requested alone, the first stages arrive within a short span of each other instead of
  // queueing behind other waves' second stages, and the waves start (and end) closer together (0.1 - 0.3 us of
  // the 128K launch; at d = 256 the later point costs 0.3 us).
  constexpr int NPRE = NS - 1;
  const bool kSecondAfterFirstLanded = D == 128 && whole;   // (rows packed several to a block: 256 x 512 tokens 39.2 -> 40.0 us with it)
  // (a borrowed slot: behind its K tiles where the block fits there, else from the slot's start)
  constexpr int Q_IN_SLOT = C::QBLK <= C::STAGE - C::OFF_V ? C::OFF_V : 0;
  char* const q_area = C::QSEP ? smem + C::OFF_QBLK + wave * C::QBLK : ring + (NS - 1) * C::STAGE + Q_IN_SLOT;
  {
    const uint32_t l = C::QSEP ? (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + C::OFF_QBLK +
                                     wave * C::QBLK
                               : ring_lds + (NS - 1) * C::STAGE + Q_IN_SLOT;
#pragma unroll
    for (int u = 0; u < GP * D * 2 / 1024; ++u) {
      const int chunk = u * 64 + lane;            // 16-byte chunk of the [GP][D] fp16 query block
      const int h = min(chunk / (D / 8), G - 1);
      dma16_lane(p.q + query_row(h) * D + (chunk % (D / 8)) * 8, l + u * 1024);
    }
  }
  // A wave has up to NS stages out before its loop and issues one per supertile while it has supertiles left.
  // (Stand-in loads that kept the count of outstanding loads the same to the end were taken out: the one issued in
  // a wave's last iteration made it wait a whole memory round trip for bytes nobody reads, 0.3 us per launch at
  // llama128k and 0.8 us at gemma32k; the waits below count what is really out instead.)
  if (n_mine > 0) {
#pragma unroll
    for (int s = 0; s < NPRE; ++s) {
      if (s < n_mine) issue(s, sidx_of(s));
    }
  }
  // (the first loads are on their way: whatever they do not need is worked out behind them)
  __builtin_amdgcn_sched_barrier(0);
  bool tail_mine[4];                              // [2], [3]: the masked FIRST supertile(s) (see `head`), the one just
                                                  // before `begin` and the one before that
#pragma unroll
  for (int u = 0; u < 2; ++u) tail_mine[u] = u < n_tail && count_of(n_full + u + 1) != count_of(n_full + u);
  tail_mine[2] = head && (whole ? wave == 0 : sub == 0);
  tail_mine[3] = head2 && (whole ? wave == 0 : sub == 0);
  static_assert(NPRE == 1, "one stage follows the query block");
  if (n_mine > 0) wait_loads<LPS>();                         // (the stage issued after the query block may still be out)
  else wait_loads<0>();

  // ---- query operands (the query pre-scaling of Alg. 1 is folded into the exp2 argument instead of the query)
  const _Float16* qh = reinterpret_cast<const _Float16*>(q_area) + hl * D;
  half8v qraw[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j)
    qraw[j] = *reinterpret_cast<const half8v*>(qh + C::a_group(j, kq) * kGroup + C::a_word(j, kq) * 8);
  half8v qgrp[NA][4];
#pragma unroll
  for (int a = 0; a < NA; ++a)
#pragma unroll
    for (int i = 0; i < 4; ++i) qgrp[a][i] = *reinterpret_cast<const half8v*>(qh + (rep * NA + a) * kGroup + i * 8);

  half8v qb[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const bool mine = (C::a_group(j, kq) == rep * NA + C::acc(j)) && hl < G;
    const half8v x = qraw[j];
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
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (float)qgrp[a][i][e];
    qsum[a] = (hl < G) ? s * 0x1p-24f : 0.0f;
  }
  const float kappa = p.scale_log2 * 0x1p24f;     // raw accumulator units -> log2 units
  const float slack = kSlack / kappa;             // the rescale slack in raw units
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the query block has been read: its slot may be refilled
  if (!kSecondAfterFirstLanded && NS - 1 < n_mine) issue(NS - 1, sidx_of(NS - 1));
  // supertile NS, the first one issued inside the loop, and how to step from one supertile to the next:
  // position j in the wave's pattern of 9 (or 7) out of 16
  int nx_j = young ? NS % YNG : NS % OLD;
  int nx_tok = tok_of(sidx_of(NS));
  // The page of the next supertile is looked up one supertile ahead of its use, by a scalar load the
  // compiler does not wait for: the wait is the lgkmcnt(0) that precedes every issue in the loop (the
  // value is threaded through that statement so that nothing reads it earlier).
  auto page_ahead = [&](int tok0) {
    int page;
    const uint32_t byte = (uint32_t)min(tok0 >> p.page_shift, p.max_blocks - 1) * 4;
    asm volatile("s_load_dword %0, %1, %2" : "=&s"(page) : "s"(tbl), "s"(byte) : "memory");
    return page;
  };
  int nx_page = paged ? __builtin_amdgcn_readfirstlane(page_of(nx_tok)) : 0;

  // ---- running state
  float m_run = kNegBig;                          // per-head reference for exp2 (raw units)
  float l_run = 0.0f;                             // this lane's share of sum(exp)
  float4v zacc[NA];                               // sum_t w z - 15 sum_t1 w (w = p s_v), rows (head, replica), col = group
  // rows (head, replica), col = packed word; [2j]: sum_t w c - 15 sum_t1 w for dim 2j of the word, [2j+1]: the same
  // for c(2j) + 16 c(2j+1), less 255 sum_t1 w.  WIDE: [2g], [2g+1] are the even and the mixed sum of group g, whose
  // column c stands for byte c / 4 of the group's word c % 4; one accumulator each.
  constexpr int NAO = C::WIDE ? 1 : NA;
  float4v oacc[NCS][8][NAO];
#pragma unroll
  for (int a = 0; a < NA; ++a) zacc[a] = float4v{0, 0, 0, 0};
#pragma unroll
  for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
    for (int m = 0; m < 8; ++m)
#pragma unroll
      for (int a = 0; a < NAO; ++a) oacc[cs][m][a] = float4v{0, 0, 0, 0};

  const half8v pos15_odd = as_half8(kPos15Odd, kPos15Odd, kPos15Odd, kPos15Odd);

  // per-lane LDS byte offsets inside a stage
  // K codes: the 16 B this lane asked for; where the query operand is block-diagonal over pairs of
  // groups (SWAP), words w and w+2 of groups 2(kq/2) and 2(kq/2)+1 of token row c instead
  // (WIDE: word kq of every group of token row c, one dword each, 256 B apart)
  const uint32_t k_rd = C::WIDE ? c * 16 + 4 * kq : C::SWAP ? (32 * (kq >> 1) + c) * 16 + 4 * (kq & 1) : lane * 16;
  // packed word(s) c of token kq (+4i); WIDE: word c % 4 of every group, 16 B apart
  const uint32_t v_rd = C::WIDE ? kq * TB + (c & 3) * 4 : kq * TB + c * 4 * NCS;
  const uint32_t v_sel = 0x0C000C00u | ((4u + (c >> 2)) << 16) | (uint32_t)(c >> 2);   // WIDE: this column's byte of a word
  // scales of this lane's groups / zero-point of the group this lane's P V column (packed word c) lies in,
  // tokens kq (+4i): eight consecutive dwords in the permuted layout, else one halfword per token at the
  // array's own stride
  // (WIDE: the zero-point operand's column c stands for group c % 4)
  const int gz = C::WIDE ? (c & 3) : (c * NCS) >> 2;
  const uint32_t sz_rd = C::WIDE ? kq * 64 : C::PERM ? (kq * GR + rep) * 32 : (kq * NG + rep * NA) * 2;
  const uint32_t zb_rd = C::WIDE ? kq * 64 + (gz >> 1) * 32 : C::PERM ? (kq * GR + (gz >> 1)) * 32 : (kq * NG + gz) * 2;
  // which half of a zero-point dword: the group's place in its pair; with larger groups the pair's place among the
  // token's two groups, or the token's place in its pair of tokens (this lane's tokens are kq, kq + 4, ...)
  const bool zb_hi = GS == 0 ? (gz & 1) : GS == 1 ? ((gz >> 1) & 1) : (kq & 1);
  const uint32_t zb_sel = zb_hi ? 0x07060302u : 0x05040100u;
  // larger groups: the half of a fetched scale / zero-point dword that this lane's 32-dim blocks share.  With 8 rows
  // the lane's two blocks are 2 rep and 2 rep + 1 (group rep of the token's two); with 16 rows register dw holds
  // blocks 2 dw and 2 dw + 1 (group dw); with groups of 128 it is the token's parity either way.
  const uint32_t dup_lo = 0x01000100u, dup_hi = 0x03020302u;
  const uint32_t dup_lane = (GS == 2 ? (kq & 1) : rep) ? dup_hi : dup_lo;

  // Everything a supertile needs from LDS is fetched into registers well before it is used: the K part
  // while the previous supertile is still in its P V phase, the V part at the start of the K phase.
  constexpr int NDW = C::NDW, NVW = C::WIDE ? NG : NCS;
  struct KRegs { uint32_t kw[2][NJ]; uint32_t ks[NDW][2][4], kz[NDW][2][4]; };   // kw[t][j]: A operand of K MFMA j, tile t
  struct VRegs { uint32_t v[NVW][8]; uint32_t vs[NDW][2][4]; uint32_t zb[8]; };
  auto load_sz1 = [&](const char* arr, uint32_t rd, uint32_t (&dst)[2][4]) {
    if constexpr (C::PERM || C::WIDE) {
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const uint4v x = *reinterpret_cast<const uint4v*>(arr + rd + t * 16);
        dst[t][0] = x[0]; dst[t][1] = x[1]; dst[t][2] = x[2]; dst[t][3] = x[3];
      }
    } else {
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          dst[t][i] = *reinterpret_cast<const uint16_t*>(arr + (t * 16 + i * 4) * NG * 2 + rd);
    }
  };
  auto load_sz = [&](const char* arr, uint32_t rd, uint32_t (&dst)[NDW][2][4]) {
#pragma unroll
    for (int dw = 0; dw < NDW; ++dw) {
      load_sz1(arr + dw * 32, rd, dst[dw]);
      if constexpr (GS > 0) {
        const uint32_t sel = (GS == 1 && C::WIDE) ? (dw ? dup_hi : dup_lo) : dup_lane;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
          for (int i = 0; i < 4; ++i) dst[dw][t][i] = __builtin_amdgcn_perm(dst[dw][t][i], dst[dw][t][i], sel);
      }
    }
  };
  auto load_k = [&](int slot, KRegs& r) {
    const char* st = ring + slot * C::STAGE;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      if constexpr (C::WIDE) {
#pragma unroll
        for (int j = 0; j < NJ; ++j) r.kw[t][j] = *reinterpret_cast<const uint32_t*>(st + t * C::KT + j * 256 + k_rd);
      } else if constexpr (C::SWAP) {
        // the lane wants words w, w+2 of two neighbouring groups, 256 B apart in the tile: two 2-dword reads
        const uint32_t* g0 = reinterpret_cast<const uint32_t*>(st + t * C::KT + k_rd);
        r.kw[t][0] = g0[0]; r.kw[t][2] = g0[2]; r.kw[t][1] = g0[64]; r.kw[t][3] = g0[66];
      } else {
#pragma unroll
        for (int ch = 0; ch < D / 128; ++ch) {
          const uint4v x = *reinterpret_cast<const uint4v*>(st + t * C::KT + ch * 1024 + k_rd);
          r.kw[t][ch * 4 + 0] = x[0]; r.kw[t][ch * 4 + 1] = x[1]; r.kw[t][ch * 4 + 2] = x[2]; r.kw[t][ch * 4 + 3] = x[3];
        }
      }
    }
    load_sz(st + C::OFF_KS, sz_rd, r.ks);
    load_sz(st + C::OFF_KZ, sz_rd, r.kz);
    __builtin_amdgcn_sched_barrier(0);
  };
  auto load_v = [&](int slot, VRegs& r) {
    const char* st = ring + slot * C::STAGE;
#pragma unroll
    for (int cs = 0; cs < NVW; ++cs)
#pragma unroll
      for (int i = 0; i < 8; ++i)                 // token slot i: token 16*(i/4) + 4*(i%4) + kq
        r.v[cs][i] = *reinterpret_cast<const uint32_t*>(st + C::OFF_V + (16 * (i >> 2) + 4 * (i & 3)) * TB + v_rd +
                                                        cs * (C::WIDE ? 16 : 4));
    load_sz(st + C::OFF_VS, sz_rd, r.vs);
    uint32_t zr[2][4];
    load_sz1(st + C::OFF_VZ, zb_rd, zr);
#pragma unroll
    for (int i = 0; i < 8; ++i) r.zb[i] = zr[i >> 2][i & 3];
    __builtin_amdgcn_sched_barrier(0);
  };
  // fp16 scale / zero-point number a (of this lane's NA) out of a fetched register
  auto sz_half = [&](uint32_t w, int a) -> _Float16 {
    const uint16_t h = (uint16_t)(a == 0 ? w : w >> 16);
    return __builtin_bit_cast(_Float16, h);
  };

  // -- scores, S^T = K Q^T, per-group scale and zero-point applied in fp32 (raw units: 2^-24)
  auto scores = [&](const KRegs& r, int sidx, auto tail_tag, float (&sc)[2][4]) {
    constexpr bool TAIL = decltype(tail_tag)::value;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float4v acc[NA];
#pragma unroll
      for (int a = 0; a < NA; ++a) acc[a] = float4v{0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc[C::acc(j)] = mfma16(unpack_word(r.kw[t][j]), qb[j], acc[C::acc(j)]);
#pragma unroll
      for (int i = 0; i < 4; ++i) {               // token 16t + 4i + kq
        float x = 0.0f;
#pragma unroll
        for (int a = 0; a < NA; ++a)
          x = __builtin_fmaf((float)sz_half(r.ks[a >> 1][t][i], a & 1),
                             __builtin_fmaf(-(float)sz_half(r.kz[a >> 1][t][i], a & 1), qsum[a], acc[a][i]), x);
        if constexpr (GR >= 2) x = row_ror_add<8>(x);
        if constexpr (GR >= 4) x = row_ror_add<4>(x);
        if constexpr (GR >= 8) x = row_ror_add<2>(x);
        if constexpr (TAIL) {
          const int tok = begin + sidx * 32 + 16 * t + tok_of_row(4 * kq + i);
          x = (tok >= lo_col && tok < end_col) ? x : -INFINITY;
        }
        sc[t][i] = x;
      }
    }
  };

  // -- online softmax over the 32 tokens (Alg. 1: the maximum, the weights and the running sum), block-wise.  m_run is a per-head
  //    REFERENCE, not the exact running max: it only moves when some score exceeds it by more than
  //    kSlack (log2 units), so exp2(score - m_run) <= 2^kSlack = 4 and p * s_v stays inside fp16 for
  //    every representable scale, while the accumulator rescale (Alg. 1, the correction factor) becomes rare.
  //    When it moves it is set kSlack ABOVE the new maximum, so the next move needs a score 2*kSlack
  //    higher than any seen so far; the weights then start at 2^-kSlack, far inside fp16's normal range.
  //    Any reference gives the same o / l, and the chunk merge (Eq. 6) accepts any m_c.
  //    Then A = fp16(+-p * s_v) (minus on the second tile's k-slots), rows (head, replica), one operand
  //    per group of the lane; the zero-point term goes through the matrix core with the stored fp16
  //    zero-points (sign flipped on the second tile's k-slots) as B operand.
  auto softmax = [&](const float (&sc)[2][4], const VRegs& r, half8v (&pa)[NA]) {
    const float mx = fmaxf(fmaxf(fmaxf(sc[0][0], sc[0][1]), fmaxf(sc[0][2], sc[0][3])),
                           fmaxf(fmaxf(sc[1][0], sc[1][1]), fmaxf(sc[1][2], sc[1][3])));
    if (__builtin_amdgcn_ballot_w64(mx > m_run + slack) != 0) {   // wave-uniform, rare
      // Every head's reference becomes at least its own current maximum plus kSlack (for the heads that outgrew
      // theirs the next move is then 2*kSlack away; the others get their headroom back while the rescale is being
      // paid for anyway).  A reference is thus never more than kSlack above its head's running maximum: one that
      // followed every move of a neighbour instead would creep up and push the head's own weights p * s_v down
      // into fp16's subnormals on a sharp softmax.
      const float m_new = fmaxf(m_run, blocks_max(mx) + slack);
      const float f = __builtin_amdgcn_exp2f((m_run - m_new) * kappa);
      m_run = m_new;
      l_run *= f;
      float fr[4];                                           // accumulator row 4kq+i belongs to head (4kq+i) % GP
#pragma unroll
      for (int i = 0; i < 4; ++i) fr[i] = __shfl(f, (4 * kq + i) % GP);
#pragma unroll
      for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int i = 0; i < 4; ++i) zacc[a][i] *= fr[i];
#pragma unroll
      for (int cs = 0; cs < NCS; ++cs)
#pragma unroll
        for (int m = 0; m < 8; ++m)
#pragma unroll
          for (int a = 0; a < NAO; ++a)
#pragma unroll
            for (int i = 0; i < 4; ++i) oacc[cs][m][a][i] *= fr[i];
    }
    const float mk = fmaxf(m_run * kappa, -3.0e38f);         // (finite also for a column that has seen no token yet)
    float pr[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        pr[t][i] = __builtin_amdgcn_exp2f(fmaf(sc[t][i], kappa, -mk));
        l_run += pr[t][i];
      }
    half8v zb;
#pragma unroll
    for (int i = 0; i < 4; ++i) {                 // k-slots 2i, 2i+1: tokens 4i + kq of tile 0 and of tile 1
#pragma unroll
      for (int a = 0; a < NA; ++a) {
        pa[a][2 * i] = (_Float16)__builtin_fmaf(pr[0][i], (float)sz_half(r.vs[a >> 1][0][i], a & 1), 0.0f);
        pa[a][2 * i + 1] = (_Float16)__builtin_fmaf(-pr[1][i], (float)sz_half(r.vs[a >> 1][1][i], a & 1), 0.0f);
      }
    }
    if constexpr (C::PERM || C::WIDE) {
      uint32_t zw[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) zw[i] = __builtin_amdgcn_perm(r.zb[4 + i], r.zb[i], zb_sel) ^ 0x80000000u;
      zb = as_half8(zw[0], zw[1], zw[2], zw[3]);
    } else {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        zb[2 * i] = sz_half(r.zb[i], 0);
        zb[2 * i + 1] = -sz_half(r.zb[4 + i], 0);
      }
    }
#pragma unroll
    for (int a = 0; a < NA; ++a) zacc[a] = mfma16(pa[a], zb, zacc[a]);
#pragma unroll
    for (int a = 0; a < NA; ++a) zacc[a] = mfma16(pa[a], pos15_odd, zacc[a]);
  };

  // -- V codes: each lane holds the same packed word (8 dims) of 8 tokens and needs, per dim, the 8 tokens in
  //    the k-slots of a B operand.  One byte-permute per (token pair, byte of the word) puts the pair's bytes
  //    into the low byte of the two halves of a register: as fp16 subnormals that is n_even + 16 n_odd of the
  //    byte's two nibbles, and one AND leaves n_even alone.  P V is linear in V, so the MIXED operand goes
  //    through the matrix core as it is (its accumulator holds  sum w (n_even + 16 n_odd) ) and the odd dim is
  //    recovered at the very end as (mixed - even) / 16: two vector instructions per pair of B registers instead
  //    of the four that separating every nibble takes.  (The mixed sum is 17 times larger and is divided by 16
  //    again: the odd dims carry about 1.5 times the accumulation noise of the even ones, a small part of the
  //    error budget.)  The complement of the second tile (15 - n in every nibble, i.e. 255 - byte) keeps both
  //    accumulators balanced around zero as before:  even: -15 sum_t1 w,  mixed: -255 sum_t1 w,  so that
  //    (mixed - even) / 16 carries the same -15 sum_t1 w that the zero-point sum cancels.
  //    WIDE: the 16 columns of a matrix instruction are the 4 words x 4 bytes of ONE group (column c = byte c / 4
  //    of word c % 4), so the lane holds that word of every group and picks its byte with a selector of its own.
  auto pv = [&](const VRegs& r, const half8v (&pa)[NA]) {
    if constexpr (C::WIDE) {
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        uint32_t mix[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) mix[i] = __builtin_amdgcn_perm(~r.v[g][i + 4], r.v[g][i], v_sel);
        const half8v v_mixed = as_half8(mix[0], mix[1], mix[2], mix[3]);
        const half8v v_even = as_half8(mix[0] & kMaskLo, mix[1] & kMaskLo, mix[2] & kMaskLo, mix[3] & kMaskLo);
        oacc[0][2 * g][0] = mfma16(pa[g], v_even, oacc[0][2 * g][0]);
        oacc[0][2 * g + 1][0] = mfma16(pa[g], v_mixed, oacc[0][2 * g + 1][0]);
      }
      return;
    }
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs) {
      uint32_t v1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) v1[i] = ~r.v[cs][i + 4];   // second tile: 15 - code in every nibble
#pragma unroll
      for (int j = 0; j < 4; ++j) {               // byte j of the word: dims 2j and 2j + 1
        const uint32_t sel = 0x0C000C00u | ((4u + j) << 16) | (uint32_t)j;   // [tile 0 byte j, 0, tile 1 byte j, 0]
        uint32_t mix[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) mix[i] = __builtin_amdgcn_perm(v1[i], r.v[cs][i], sel);
        const half8v v_mixed = as_half8(mix[0], mix[1], mix[2], mix[3]);
        const half8v v_even = as_half8(mix[0] & kMaskLo, mix[1] & kMaskLo, mix[2] & kMaskLo, mix[3] & kMaskLo);
#pragma unroll
        for (int a = 0; a < NAO; ++a) {
          oacc[cs][2 * j][a] = mfma16(pa[a], v_even, oacc[cs][2 * j][a]);
          oacc[cs][2 * j + 1][a] = mfma16(pa[a], v_mixed, oacc[cs][2 * j + 1][a]);
        }
      }
    }
  };

  // ---- main loop.  Supertile i: its K part already sits in registers; fetch its V part, compute the
  //      scores, fetch the K part of supertile i+1 (whose stage has to have landed by then), softmax,
  //      refill the ring slot of supertile i with supertile i+NS, P V.
  KRegs kr;
  VRegs vr;
  static_assert(C::PFK && NS == 2, "the waits below count one or two stages");
  if (n_mine > 0) {
    if (!kSecondAfterFirstLanded && n_mine > 1) wait_loads<LPS>();   // (loads land in order: stage 0 is in)
    else wait_loads<0>();
    load_k(0, kr);
    if (kSecondAfterFirstLanded && NS - 1 < n_mine) issue(NS - 1, sidx_of(NS - 1));
  }
  int slot = 0;
  for (int i = 0; i < n_mine; ++i) {
    const int next = (slot + 1 == NS) ? 0 : slot + 1;
    load_v(slot, vr);
    // The slot's bytes all sit in registers from here on; its refill with supertile i + NS is issued after the
    // softmax all the same.  (Measured at 128K / at the d = 256 instance: issued here, +0.4 / +0.6 us; issued after
    // the P V phase, +0.4 / +0.3 us; a ring of three stages, +1.0 us: the memory system is at its limit, and
    // requests queued earlier than needed only delay the ones a wave is waiting for.  Issued here AND waited for
    // stage by stage, so that two stages are in flight: the kernel alone unchanged, the decode call 1 us slower.)
    auto refill = [&] {
      asm volatile("s_waitcnt lgkmcnt(0)" : "+s"(nx_page) :: "memory");   // every LDS read of this slot has returned
      if (i + NS < n_mine) {
        issue_tok(ring_lds + slot * C::STAGE, nx_tok, nx_page, koff, lane16, szoff);
        // next supertile of the pattern: of every PERIOD the older wave holds k = 0, 2, .., PERIOD-2 and PERIOD-1,
        // the younger k = 1, 3, .., PERIOD-3
        const int step = young ? (nx_j < YNG - 1 ? 2 : 4) : (nx_j < PERIOD / 2 - 1 ? 2 : 1);
        nx_j = (nx_j == (young ? YNG - 1 : OLD - 1)) ? 0 : nx_j + 1;
        nx_tok += whole ? step * (4 * 32) : W * 32;
        if (paged) nx_page = page_ahead(nx_tok);
      }
    };
    float sc[2][4];
    // (the wave asks for issue priority while it unpacks K, feeds the matrix cores and scales the scores: the two
    //  waves of a SIMD then take turns phase by phase rather than instruction by instruction, 0 - 1 % faster at
    //  128K from box to box, 0.4 % at the d = 256 instance)
    __builtin_amdgcn_s_setprio(1);
    scores(kr, 0, std::false_type{}, sc);
    __builtin_amdgcn_s_setprio(0);
    // The only stage out is the next supertile's.  Past the last supertile there is nothing to wait for and the
    // fetch reads unused bytes; skipping it there takes a branch in the loop, which the d = 128 instances pay for in
    // registers and schedule (16-row tile 33.3 -> 35.4 us, 8-row 28.7 -> 28.95) and the d = 256 instance gains by.
    if (D == 128 || i + 1 < n_mine) {
      wait_loads<0>();
      load_k(next, kr);
    }
    half8v pa[NA];
    softmax(sc, vr, pa);
    refill();
    pv(vr, pa);
    slot = next;
  }
  wait_loads<0>();                                           // (nothing is out any more: the rings are quiet)
#pragma unroll 1
  for (int u = 0; u < (PLAIN ? 1 : 4); ++u) {                // the masked supertiles: the sequence's last one or two,
    if (!tail_mine[u]) continue;                             // and under a window its first (or first two)
    const int sidx = u < 2 ? n_full + u : 1 - u;
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    issue_tail(0, sidx);
    wait_loads<0>();
    load_k(0, kr);
    load_v(0, vr);
    if constexpr (GS == 2) {
      // a token pair's dword may reach one token past the sequence's last: whatever lies there must not meet the
      // (zero) weights of the masked tokens as an Inf or NaN (the scores of such tokens are replaced, not scaled)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i)
          if (begin + sidx * 32 + 16 * t + 4 * i + kq >= seq) {
#pragma unroll
            for (int dw = 0; dw < NDW; ++dw) vr.vs[dw][t][i] = 0;
            vr.zb[4 * t + i] = 0;
          }
    }
    float sc[2][4];
    scores(kr, sidx, std::true_type{}, sc);
    half8v pa[NA];
    softmax(sc, vr, pa);
    pv(vr, pa);
  }

  // ---- wave result -> LDS.  Of a lane's NA accumulators per row only the one whose group the lane's packed
  //      word belongs to is meaningful (and, the zero-point operand being laid out to match, the same one of its
  //      NA zero-point sums): it is selected, brought to common units (the 2^24 / 2^20 of the two nibble
  //      positions), the zero-point sum is taken off, and the eight dims of the word leave as two 16-byte writes.
  float* const lds_o = reinterpret_cast<float*>(smem + C::OFF_MERGE);  // [NW][GP][D]   sum_t p_t v^_t
  float* const lds_m = lds_o + NW * GP * D;                            // [GP][NW]
  float* const lds_l = lds_m + NW * GP;                                // [GP][NW]
  if constexpr (C::ALIAS) __syncthreads();                   // everybody is done reading the rings
  const bool active = n_mine > 0 || tail_mine[0] || tail_mine[1] || tail_mine[2] || tail_mine[3];
  const float l_tot = blocks_sum(l_run);
  if (kq == 0 && rep == 0) {
    // (a row whose tokens were all masked still has the initial reference: it counts as empty)
    lds_m[hl * NW + wave] = (active && m_run > kNegBig) ? m_run * kappa : kNegBig;
    lds_l[hl * NW + wave] = active ? l_tot : 0.0f;
  }
  if constexpr (C::WIDE) {
    // row 4 kq + i = head; group g's zero-point sum of that head sits in column g (any column c with c % 4 == g)
    // of zacc[g]; this lane's column is byte c / 4 of word c % 4 of every group: two neighbouring dims per group
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const float zc = __shfl(zacc[g][i], (lane & 48) | g);
        const float even = oacc[0][2 * g][0][i], mixed = oacc[0][2 * g + 1][0][i];
        float2 o2;
        o2.x = fmaf(even, 0x1p24f, -zc);
        o2.y = fmaf(mixed - even, 0x1p20f, -zc);
        *reinterpret_cast<float2*>(lds_o + (wave * GP + 4 * kq + i) * D + (4 * g + (c & 3)) * 8 + 2 * (c >> 2)) = o2;
      }
  }
#pragma unroll
  for (int i = 0; i < (C::WIDE ? 0 : 4); ++i) {
    const int r = 4 * kq + i, h = r % GP, rp = r / GP;       // accumulator row -> (head, replica)
#pragma unroll
    for (int cs = 0; cs < NCS; ++cs) {
      const int word = c * NCS + cs;              // packed word (8 dims) this lane's column stands for
      const int a_mine = (word >> 2) - rp * NA;
      const bool second = NA == 2 && a_mine == 1;
      const float zc = second ? zacc[NA - 1][i] : zacc[0][i];
      float4v lo, hi;
      float acc[8];
#pragma unroll
      for (int m = 0; m < 8; ++m) acc[m] = second ? oacc[cs][m][NAO - 1][i] : oacc[cs][m][0][i];
#pragma unroll
      for (int m = 0; m < 4; ++m) {               // dim m: the even sum, or (mixed - even) / 16, in units of 2^-24
        lo[m] = fmaf((m & 1) ? acc[m] - acc[m - (m & 1)] : acc[m], (m & 1) ? 0x1p20f : 0x1p24f, -zc);
        hi[m] = fmaf((m & 1) ? acc[m + 4] - acc[m + 4 - (m & 1)] : acc[m + 4], (m & 1) ? 0x1p20f : 0x1p24f, -zc);
      }
      if (a_mine >= 0 && a_mine < NA) {
        float4v* dst = reinterpret_cast<float4v*>(lds_o + (wave * GP + h) * D + word * 8);
        dst[0] = lo;
        dst[1] = hi;
      }
    }
  }
  __syncthreads();

  // ---- merge the waves, write one partial per query head (Sec. 3.2); where the sequence is a single
  //      chunk and the kernel is to produce the output, that partial, normalised, IS the output.
  //      A thread takes two neighbouring dims of one head: the waves' maxima and sums of that head arrive as
  //      16-byte reads (the same for the whole wave at d = 128, where wave h merges head h).
  const bool direct = p.merge_slot >= 0 && p.n_splits == 1;
  // `first` .. `first + count - 1`: the waves to merge; `stride`, `lane0`: this thread's place among the threads that do it
  auto merge_waves = [&](int first, int count, int lane0, int stride) {
    for (int idx = lane0; idx < G * (D / 2); idx += stride) {
      const int h = idx / (D / 2), j = (idx % (D / 2)) * 2;
      float2 ow[NW];                              // (asked for first: their latency hides behind the weights' arithmetic)
#pragma unroll
      for (int w = 0; w < NW; ++w) ow[w] = *reinterpret_cast<const float2*>(lds_o + (w * GP + h) * D + j);
      float mw[NW], lw[NW];
#pragma unroll
      for (int w4 = 0; w4 < NW; w4 += 4) {
        const float4v a = *reinterpret_cast<const float4v*>(lds_m + h * NW + w4);
        const float4v bb = *reinterpret_cast<const float4v*>(lds_l + h * NW + w4);
#pragma unroll
        for (int u = 0; u < 4; ++u) { mw[w4 + u] = a[u]; lw[w4 + u] = bb[u]; }
      }
      float mg = kNegBig;
#pragma unroll
      for (int w = 0; w < NW; ++w) mg = (w >= first && w < first + count) ? fmaxf(mg, mw[w]) : mg;
      float n0 = 0.0f, n1 = 0.0f, den = 0.0f;
#pragma unroll
      for (int w = 0; w < NW; ++w) {
        if (w < first || w >= first + count) continue;       // (wave-uniform)
        const float e = __builtin_amdgcn_exp2f(mw[w] - mg);
        n0 = fmaf(ow[w].x, e, n0);
        n1 = fmaf(ow[w].y, e, n1);
        den = fmaf(lw[w], e, den);
      }
      if (direct) {
        half2v r;
        r[0] = (_Float16)(n0 / den);
        r[1] = (_Float16)(n1 / den);
        *reinterpret_cast<half2v*>(p.out + query_row(h) * D + j) = r;
      } else {
        // device-scope stores: they go through to where every compute die sees them (the L2 caches of
        // different dies are not coherent with each other), so no cache-wide write-back is needed later
        const int64_t ph = query_row(h) * part_stride + split;
        st_dev2(p.part_o + ph * D + j, n0, n1);
        if (j == 0) st_dev2(p.part_ml + ph * 2, mg, den);
      }
    }
  };
  if (!whole) {                                   // several units per block: the W waves of one merge among themselves
    // (a single-chunk row: the output; a slot of the chunk list: its partial)
    if (row_valid) merge_waves(wave - sub, W, sub * 64 + lane, W * 64);
    return;
  }
  merge_waves(0, NW, threadIdx.x, NW * 64);
  if (p.merge_slot < 0 || direct) return;

  // ---- chunk merge (Eq. 6) by whichever block of this (b, kv head) finishes last.  A block publishes
  //      its partial (device-scope stores, waited for), then counts itself in; the one that sees all
  //      others counted re-reads all partials, with device-scope loads and in chunk order, so the
  //      result does not depend on which block that is.
  const int n = p.n_splits;
  int* const is_last = reinterpret_cast<int*>(smem);
  wait_loads<0>();                                // vmcnt counts stores too: this wave's partial has landed
  __syncthreads();                                // every wave's has; and nobody reads the block-merge area any more
  if (threadIdx.x == 0) {
    unsigned int* ctr = &g_arrivals[p.merge_slot * kCountersPerSlot + arrival_counter(b * (p.n_kv_heads * kv_share) + kvv)];
    *is_last = atomicInc(ctr, (unsigned int)(n - 1)) == (unsigned int)(n - 1);   // wraps to 0 on the last arrival
  }
  __syncthreads();
  if (*is_last == 0) return;
  // What orders the partials before their readers is the machine's memory model for device-scope ATOMIC accesses,
  // not a pair of fences: every partial is written with device-scope atomic stores (write-through: complete, as
  // counted by vmcnt, once the data sits where every compute die reads it), the wave waits for vmcnt(0) and the
  // block for its barrier before one thread counts the block in with a device-scope atomic, and the last block
  // issues its device-scope atomic loads (which do not hit lines a die cached earlier) only after that atomic has
  // returned.  A release fence before the count and an acquire fence after it (agent scope) were measured instead:
  // each block then writes its die's whole L2 back and invalidates it, and a decode of 256 blocks over 8K tokens
  // goes from 11.0 to 13.5 us (release alone +1.2 us, acquire alone +0.9 us), more than the separate merge kernel
  // costs (13.1 us), for no access that the atomics do not already cover.
  float* const c_m = reinterpret_cast<float*>(smem) + 64;     // [G][n] chunk maxima, then chunk weights
  float* const c_l = c_m + GP * kMaxSplits;                    // [G][n] chunk sums
  float* const h_den = c_l + GP * kMaxSplits;                  // [G]
  // Everything is asked for at once, so the merge is about one memory round trip long: the first 32
  // chunks of this thread's output elements (which do not need the weights yet) and the chunk maxima
  // and sums; the weights are worked out while the loads are in flight.
  constexpr int PER = GP * D / (NW * 64);         // output elements per thread (padded group)
  constexpr int FIRST = 32;
  float pre[PER][FIRST];
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int idx = threadIdx.x + e * NW * 64, h = idx / D, j = idx % D;
    const float* src = p.part_o + query_row(h < G ? h : 0) * n * D + j;
#pragma unroll
    for (int u = 0; u < FIRST; ++u) pre[e][u] = ld_dev(src + (int64_t)(u < n ? u : n - 1) * D);
  }
  for (int idx = threadIdx.x; idx < G * n; idx += NW * 64) {
    const float* ml = p.part_ml + (query_row(idx / n) * n + idx % n) * 2;
    c_m[(idx / n) * kMaxSplits + idx % n] = ld_dev(ml);
    c_l[(idx / n) * kMaxSplits + idx % n] = ld_dev(ml + 1);
  }
  __syncthreads();
  for (int h = wave; h < G; h += NW) {            // a wave per head: its chunk weights and its denominator
    float mx = kNegBig;
    for (int cc = lane; cc < n; cc += 64) mx = fmaxf(mx, c_m[h * kMaxSplits + cc]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    float dsum = 0.0f;
    for (int cc = lane; cc < n; cc += 64) {
      const float w = __builtin_amdgcn_exp2f(c_m[h * kMaxSplits + cc] - mx);
      c_m[h * kMaxSplits + cc] = w;
      dsum = fmaf(c_l[h * kMaxSplits + cc], w, dsum);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) dsum += __shfl_xor(dsum, off);
    if (lane == 0) h_den[h] = dsum;
  }
  __syncthreads();
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int idx = threadIdx.x + e * NW * 64, h = idx / D, j = idx % D;
    if (h >= G) continue;
    const int64_t row = query_row(h);
    const float* src = p.part_o + row * n * D + j;
    const float* w = c_m + h * kMaxSplits;
    float num = 0.0f;
#pragma unroll
    for (int u = 0; u < FIRST; ++u) num = fmaf(pre[e][u], u < n ? w[u] : 0.0f, num);
    int cc = FIRST;
    for (; cc + 8 <= n; cc += 8) {
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = ld_dev(src + (int64_t)(cc + u) * D);
#pragma unroll
      for (int u = 0; u < 8; ++u) num = fmaf(v[u], w[cc + u], num);
    }
    for (; cc < n; ++cc) num = fmaf(ld_dev(src + (int64_t)cc * D), w[cc], num);
    p.out[row * D + j] = (half_t)(num / h_den[h]);
  }
}

int padded_gqa(int head_dim, int gqa) {           // columns a group of `gqa` heads takes in the tile; 0 = too many
  if (head_dim == 128) return gqa <= 4 ? 4 : (gqa <= 8 ? 8 : (gqa <= 16 ? 16 : 0));
  return gqa <= 2 ? 2 : 0;
}
// At d = 128 a tile holds up to 16 query rows (at about 1.25 times the 8-row tile's time per token), at d = 256 two.
// A group with more rows is cut into the fewest equal parts that fit, one block each on the same KV head.
// (16 heads per KV head, one sequence, one 16-row block against two 8-row blocks: 8K tokens 14.4 against 15.5 us,
// 32K 18.8 against 19.7, 128K 39.8 against 52.1; 8 sequences of 32K 64.3 against 102.8 us.)
int kv_share_of(int head_dim, int gqa) {
  if (gqa < 1 || (head_dim != 128 && head_dim != 256)) return 0;
  // d=256: a tile of 4 rows needs more registers than a lane has (its loop spills), and two blocks of 2 rows
  // that stream the same KV head are faster than one of 4 (measured: 52.9 us against 69.0 us at 64/16 heads, 32K)
  const int cap = head_dim == 128 ? 16 : 2;
  for (int share = (gqa + cap - 1) / cap; share <= gqa; ++share)
    if (gqa % share == 0) return share;
  return 0;
}

template <int D, int GP, bool NT, bool PLAIN, int GS = 0>
hipError_t launch_as(const DecodeParams& p, dim3 grid, hipStream_t s) {
  static_assert((64 + (2 * GP * kMaxSplits + GP) ) * 4 <= Cfg<D, GP, 8>::SMEM, "the chunk merge reuses the block's LDS");
  // one block of 8 waves per compute unit: 8 rings of 2 x 5 KB (d=128) or 2 x 10 KB (d=256, all 160 KB of LDS)
  constexpr int NW = 8;
  constexpr int smem = Cfg<D, GP, NW>::SMEM;
  static_assert(smem <= 160 * 1024, "LDS budget of one compute unit");
  // dynamic LDS above 64 KB has to be opted into, once per device and kernel instance (any thread may get here first)
  static std::once_flag configured[kMaxDevices];
  static hipError_t outcome[kMaxDevices];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::call_once(configured[dev], [&] {
    outcome[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(&decode_partial_mfma_kernel<D, GP, NW, NT, PLAIN, GS>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
  });
  if (outcome[dev] != hipSuccess) return outcome[dev];
  hipLaunchKernelGGL((decode_partial_mfma_kernel<D, GP, NW, NT, PLAIN, GS>), grid, dim3(NW * 64), smem, s, p);
  return hipGetLastError();
}
// the stream is read once (non-temporal loads) unless several blocks share a KV head
template <int D, int GP>
hipError_t launch(const DecodeParams& p, dim3 grid, hipStream_t s) {
  if constexpr (D == 128 && GP >= 8) {            // groups of 64 / 128 elements
    if (p.group == 2 * kGroup)
      return p.kv_share == 1 ? launch_as<D, GP, true, false, 1>(p, grid, s) : launch_as<D, GP, false, false, 1>(p, grid, s);
    if (p.group == 4 * kGroup)
      return p.kv_share == 1 ? launch_as<D, GP, true, false, 2>(p, grid, s) : launch_as<D, GP, false, false, 2>(p, grid, s);
  }
  if (p.group != kGroup) return hipErrorNotSupported;
  const bool plain = p.kv_share == 1 && p.n_queries == 1 && p.waves_per_row == 8 && p.var_chunks == 0 &&
                     p.seq_lens == nullptr && p.block_table == nullptr;
  if (plain) return launch_as<D, GP, true, true>(p, grid, s);
  return p.kv_share == 1 ? launch_as<D, GP, true, false>(p, grid, s) : launch_as<D, GP, false, false>(p, grid, s);
}

}  // namespace

int mfma_kv_share(int head_dim, int gqa) { return kv_share_of(head_dim, gqa); }

bool mfma_supported(int head_dim, int gqa) { return kv_share_of(head_dim, gqa) > 0; }

// Groups of 64 or 128 elements: head_dim 128 only; at 128 two tokens share a dword of every metadata array, which
// has to be aligned and must not straddle two (sequence, KV head) rows: an even number of tokens per row.
bool mfma_supports_group(int head_dim, int group, int capacity) {
  if (group == kGroup) return true;
  return head_dim == 128 && (group == 2 * kGroup || (group == 4 * kGroup && capacity % 2 == 0));
}

bool mfma_can_merge(int batch, int n_kv_heads) { return (int64_t)batch * n_kv_heads <= kCountersPerSlot; }

int mfma_merge_slot_of(const void* workspace) {
  static std::mutex guard;
  static std::unordered_map<const void*, int> slots;
  std::lock_guard<std::mutex> lock(guard);
  const auto it = slots.find(workspace);
  if (it != slots.end()) return it->second;
  if ((int)slots.size() >= kCounterSlots) return -1;
  const int slot = (int)slots.size();
  slots.emplace(workspace, slot);
  return slot;
}

hipError_t launch_partial_mfma(const DecodeParams& p_in, int batch, int head_dim, int merge_slot, hipStream_t s) {
  DecodeParams p = p_in;
  if (p.n_queries < 1) p.n_queries = 1;
  if (p.n_queries > kMaxQueries) return hipErrorNotSupported;
  p.gqa_full = p.gqa;
  // blocks per KV head: the caller's choice (it sized the chunk plan by it), checked against the tiles there are
  const int rows = p.gqa * p.n_queries;
  if (p.kv_share < 1 || rows % p.kv_share != 0 || padded_gqa(head_dim, rows / p.kv_share) == 0) return hipErrorNotSupported;
  p.gqa = rows / p.kv_share;
  const int rows_y = p.n_kv_heads * p.kv_share;
  p.merge_slot = -1;
  if (merge_slot >= 0) {
    if ((p.n_splits > 1 && !mfma_can_merge(batch, rows_y)) || p.out == nullptr || merge_slot >= kCounterSlots)
      return hipErrorInvalidValue;
    p.merge_slot = merge_slot;
  }
  if (p.waves_per_row != 1 && p.waves_per_row != 2 && p.waves_per_row != 4) p.waves_per_row = 8;
  // several units per block: single-chunk rows whose output the kernel writes itself, or the slots of a chunk list
  if (p.waves_per_row != 8 && p.var_chunks == 0 && (p.merge_slot < 0 || p.n_splits != 1 || p.block_table))
    return hipErrorInvalidValue;
  const int per_block = 8 / p.waves_per_row;
  const dim3 grid = p.var_chunks > 0 ? dim3((p.var_chunks + per_block - 1) / per_block, rows_y, 1)
                    : per_block > 1  ? dim3(1, (batch * rows_y + per_block - 1) / per_block, 1)
                                     : dim3(p.n_splits, rows_y, batch);
  int gp = padded_gqa(head_dim, p.gqa);
  if (p.group != kGroup && gp == 4) gp = 8;       // (larger groups: the 8- and 16-row layouts only)
  if (head_dim == 128 && gp == 16) return launch<128, 16>(p, grid, s);
  if (head_dim == 128 && gp == 8) return launch<128, 8>(p, grid, s);
  if (head_dim == 128 && gp == 4) return launch<128, 4>(p, grid, s);
  if (head_dim == 256 && gp == 2) return launch<256, 2>(p, grid, s);
  return hipErrorNotSupported;
}

}  // namespace tq
