// Attention phase of the unfused comparator (Sec. 3.1: dequantise to dense fp16, then attend) on the matrix
// cores: phase 1 of Sec. 3.2 over dense fp16 K^ and V^ [B][H_kv][S][d], for up to 16 query heads per KV head.
// A comparator is only worth comparing against if it runs at the speed its bytes allow; with the arithmetic on
// the vector ALU (the generic kernel's dense instance) it reaches about a third of that.
//
// One block = one chunk of one KV head; its waves take the chunk's 32-token supertiles in turn, each with a ring
// of two LDS stages filled by direct global->LDS loads one supertile ahead, private online-softmax state (Alg. 1),
// and a merge through LDS at the end (one partial per query head and block, the format of the fused kernels, so
// that the same merge kernel finishes the job).
//
// Scores are computed transposed, S^T = K Q^T (A = 16 tokens x 32 dims of K^, B = the query heads), so that the
// accumulator layout (lane = head, 4 tokens per 16-lane block) is the A-operand layout of P V.  K^ needs no
// preparation: the direct loads gather each lane's 16 bytes (8 dims of one token) into lane order.
// For P V the contraction runs over tokens, so a lane needs 8 tokens of ONE dim in its k-slots while a dense row
// holds the dims of one token: the lane reads the dword (two neighbouring dims) of two neighbouring token rows
// and one byte-permute each pairs the even dims and the odd dims of the two tokens; the even and the odd dims go
// through separate matrix instructions (column c = dim 2c, or 2c + 1, of a 32-dim block).
#include <mutex>

#include "tq_internal.h"

namespace tq {
namespace {

typedef _Float16 half8v __attribute__((ext_vector_type(8)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));

constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float4v mfma16(half8v a, half8v b, float4v c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
}
__device__ __forceinline__ half8v as_half8(uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  return __builtin_bit_cast(half8v, uint4v{a, b, c, d});
}
// reductions over the four 16-lane blocks (lanes l, l^16, l^32, l^48)
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

// Direct global -> LDS load of 16 bytes per lane (non-temporal: the dense tensors are read once).  Lane l's bytes
// land at m0 + OFF + 16 l; the immediate offset moves the global and the LDS address alike, so the caller
// passes the LDS address less OFF.  Written as asm so that the compiler does not serialise the loads against
// later LDS reads: each wave tracks its ring with explicit vmcnt waits.  (M0 cannot be named as a clobber; the
// compiler keeps no value live in it across other instructions.)
template <int OFF>
__device__ __forceinline__ void dma16(const void* sbase, uint32_t voff, uint32_t m0) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1 offset:%3 nt"
               :: "v"(voff), "s"(sbase), "s"(m0), "n"(OFF) : "memory");
}
__device__ __forceinline__ void dma16_lane(const void* addr, uint32_t m0) {   // per-lane 64-bit address
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" :: "v"(addr), "s"(m0) : "memory");
}
template <int N>
__device__ __forceinline__ void wait_loads() {               // until at most N vector-memory operations are outstanding
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

template <int D>
struct DenseCfg {
  static constexpr int NW = 512 / D;                 // waves per block: 4 at d = 128, 2 at d = 256
  static constexpr int NJ = D / 32;                  // 32-dim blocks: K matrix instructions per 16-token tile
  static constexpr int ROWB = D * 2;                 // bytes of one dense row
  static constexpr int RPI = 1024 / ROWB;            // V rows per 1 KB load instruction
  static constexpr int KPART = 32 * ROWB;            // K^ of a supertile, [tile][dim block][lane] x 16 B
  static constexpr int VINS = 32 * ROWB / 1024;      // load instructions for V^ of a supertile
  // V^ rows keep their order; a gap after every 1 KB piece moves the four rows that the four 16-lane blocks read at
  // the same time (4 rows apart) into different banks: 16 dwords from one such row to the next
  static constexpr int VGAP = 16 * RPI;
  static __host__ __device__ constexpr int v_piece(int u) { return u * (1024 + VGAP); }
  static constexpr int VPART = VINS * (1024 + VGAP);
  static constexpr int STAGE = KPART + VPART;
  static constexpr int LPS = 2 * NJ + VINS;          // load instructions per stage
  static constexpr int RING = NW * 2 * STAGE;
  static constexpr int MERGE = (NW * 16 * D + 2 * NW * 16) * 4;   // o, m, l of every wave; it takes the rings' place
  static constexpr int SMEM = RING > MERGE ? RING : MERGE;
};

template <int D>
__global__ __launch_bounds__(DenseCfg<D>::NW * 64, 1) void dense_partial_mfma_kernel(DecodeParams p) {
  using C = DenseCfg<D>;
  constexpr int NW = C::NW, NJ = C::NJ, ROWB = C::ROWB, LPS = C::LPS;
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int c = lane & 15, kq = lane >> 4;
  const int split = blockIdx.x, kv = blockIdx.y, b = blockIdx.z;
  const int G = p.gqa, h0 = kv * G;
  const int begin = split * p.tokens_per_split;
  if (begin >= p.seq_len) return;                            // (the whole block: nothing to emit)
  const int end = min(p.seq_len, begin + p.tokens_per_split);
  const int n_full = (end - begin) >> 5;                     // supertiles every token of which exists
  const bool ragged = ((end - begin) & 31) != 0;

  const int64_t row0 = (int64_t)(b * p.n_kv_heads + kv) * p.row_stride;
  const char* const k_chunk = reinterpret_cast<const char*>(p.k_dense) + (row0 + begin) * ROWB;
  const char* const v_chunk = reinterpret_cast<const char*>(p.v_dense) + (row0 + begin) * ROWB;
  char* const ring = smem + wave * (2 * C::STAGE);
  const uint32_t ring_lds = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem + wave * (2 * C::STAGE);

  // K^: lane (c, kq) of the load for (tile t, dim block j) fetches dims 32 j + 8 kq .. + 7 of token 16 t + c
  const uint32_t k_off = c * ROWB + kq * 16;
  const uint32_t lane16 = lane * 16;
  auto issue = [&](int slot, int sidx) {                     // supertile sidx of the chunk -> ring slot
    const uint32_t l = ring_lds + slot * C::STAGE;
    const char* const kb = k_chunk + (int64_t)sidx * (32 * ROWB);
    const char* const vb = v_chunk + (int64_t)sidx * (32 * ROWB);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const char* const kt = kb + t * 16 * ROWB;
      dma16<0>(kt, k_off, l + (t * NJ + 0) * 1024);
      dma16<64>(kt, k_off, l + (t * NJ + 1) * 1024 - 64);
      dma16<128>(kt, k_off, l + (t * NJ + 2) * 1024 - 128);
      dma16<192>(kt, k_off, l + (t * NJ + 3) * 1024 - 192);
      if constexpr (NJ == 8) {
        dma16<256>(kt, k_off, l + (t * NJ + 4) * 1024 - 256);
        dma16<320>(kt, k_off, l + (t * NJ + 5) * 1024 - 320);
        dma16<384>(kt, k_off, l + (t * NJ + 6) * 1024 - 384);
        dma16<448>(kt, k_off, l + (t * NJ + 7) * 1024 - 448);
      }
    }
#pragma unroll
    for (int u = 0; u < C::VINS; u += 4) {
      const char* const vq = vb + u * 1024;
      dma16<0>(vq, lane16, l + C::KPART + C::v_piece(u));
      dma16<1024>(vq, lane16, l + C::KPART + C::v_piece(u + 1) - 1024);
      dma16<2048>(vq, lane16, l + C::KPART + C::v_piece(u + 2) - 2048);
      dma16<3072>(vq, lane16, l + C::KPART + C::v_piece(u + 3) - 3072);
    }
  };
  // the chunk's ragged last supertile: every token index clamped to the chunk's last token (finite values that
  // the masked weights then multiply by zero)
  auto issue_ragged = [&](int slot, int sidx) {
    const uint32_t l = ring_lds + slot * C::STAGE;
    const int last = end - 1 - begin;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      const int tok = min(sidx * 32 + 16 * t + c, last);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
        dma16_lane(k_chunk + (int64_t)tok * ROWB + j * 64 + kq * 16, l + (t * NJ + j) * 1024);
    }
#pragma unroll
    for (int u = 0; u < C::VINS; ++u) {
      const int tok = min(sidx * 32 + u * C::RPI + lane / (ROWB / 16), last);
      dma16_lane(v_chunk + (int64_t)tok * ROWB + (lane % (ROWB / 16)) * 16, l + C::KPART + C::v_piece(u));
    }
  };

  // the block's waves take the chunk's supertiles in turn
  const int n_mine = n_full > wave ? (n_full - wave + NW - 1) / NW : 0;
  if (n_mine > 0) issue(0, wave);
  if (n_mine > 1) issue(1, wave + NW);

  // query operands: column c = head c of the group; dim block j, k-slots = dims 32 j + 8 kq .. + 7
  half8v qb[NJ];
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    qb[j] = half8v{0, 0, 0, 0, 0, 0, 0, 0};
    if (c < G) qb[j] = *reinterpret_cast<const half8v*>(p.q + (int64_t)(b * p.n_q_heads + h0 + c) * D + 32 * j + 8 * kq);
  }

  float m_run = kNegBig;                                     // running maximum of this lane's head (log2 units)
  float l_run = 0.0f;                                        // this lane's share of the running sum
  float4v oacc[NJ][2];                                       // rows = heads, column c = dim 32 j + 2 c (+ 1)
#pragma unroll
  for (int j = 0; j < NJ; ++j) oacc[j][0] = oacc[j][1] = float4v{0, 0, 0, 0};

  // V^ rows this lane's k-slots stand for: k-slot pair m holds tokens (4 kq + 2 m, + 1) of the first tile for
  // m = 0, 1 and of the second for m = 2, 3, which is where the score accumulators leave the weights
  uint32_t v_rd[4];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int r = (m < 2 ? 0 : 16) + 4 * kq + 2 * (m & 1);
    v_rd[m] = C::KPART + C::v_piece(r / C::RPI) + (r % C::RPI) * ROWB + c * 4;
  }

  auto process = [&](int slot, int sidx, bool masked, auto&& after_reads) {
    const char* st = ring + slot * C::STAGE;
    uint4v kr[2][NJ];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int j = 0; j < NJ; ++j) kr[t][j] = *reinterpret_cast<const uint4v*>(st + (t * NJ + j) * 1024 + lane16);
    uint32_t va[NJ][4], vb[NJ][4];                           // the two token rows of k-slot pair m, dims 32 j + 2 c, + 1
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        va[j][m] = *reinterpret_cast<const uint32_t*>(st + v_rd[m] + j * 64);
        vb[j][m] = *reinterpret_cast<const uint32_t*>(st + v_rd[m] + j * 64 + ROWB);
      }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");       // the slot's bytes sit in registers: it may be refilled
    after_reads();

    float x[2][4];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float4v acc = float4v{0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < NJ; ++j) acc = mfma16(__builtin_bit_cast(half8v, kr[t][j]), qb[j], acc);
#pragma unroll
      for (int i = 0; i < 4; ++i) {                          // token 16 t + 4 kq + i, head c
        x[t][i] = acc[i] * p.scale_log2;
        if (masked && begin + sidx * 32 + 16 * t + 4 * kq + i >= end) x[t][i] = -INFINITY;
      }
    }
    // Alg. 1: running maximum, correction of what has been accumulated, weights, running sum
    const float mx = fmaxf(fmaxf(fmaxf(x[0][0], x[0][1]), fmaxf(x[0][2], x[0][3])),
                           fmaxf(fmaxf(x[1][0], x[1][1]), fmaxf(x[1][2], x[1][3])));
    const float m_new = fmaxf(m_run, blocks_max(mx));
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {
      const float f = __builtin_amdgcn_exp2f(m_run - m_new);
      m_run = m_new;
      l_run *= f;
      float fr[4];                                           // accumulator row 4 kq + i belongs to head 4 kq + i
#pragma unroll
      for (int i = 0; i < 4; ++i) fr[i] = __shfl(f, 4 * kq + i);
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 2; ++e)
#pragma unroll
          for (int i = 0; i < 4; ++i) oacc[j][e][i] *= fr[i];
    }
    half8v pa;
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float pr = __builtin_amdgcn_exp2f(x[t][i] - m_run);
        l_run += pr;
        pa[4 * t + i] = (_Float16)pr;
      }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      uint32_t ev[4], od[4];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        ev[m] = __builtin_amdgcn_perm(vb[j][m], va[j][m], 0x05040100u);   // dim 2c of the two tokens
        od[m] = __builtin_amdgcn_perm(vb[j][m], va[j][m], 0x07060302u);   // dim 2c + 1
      }
      oacc[j][0] = mfma16(pa, as_half8(ev[0], ev[1], ev[2], ev[3]), oacc[j][0]);
      oacc[j][1] = mfma16(pa, as_half8(od[0], od[1], od[2], od[3]), oacc[j][1]);
    }
  };

  for (int i = 0; i < n_mine; ++i) {
    const int slot = i & 1;
    if (i + 1 < n_mine) wait_loads<LPS>();                   // (loads complete in order: the older stage has landed)
    else wait_loads<0>();
    process(slot, wave + NW * i, false, [&] {
      if (i + 2 < n_mine) issue(slot, wave + NW * (i + 2));
    });
  }
  if (ragged && wave == n_full % NW) {                       // the wave whose turn the last supertile is
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    issue_ragged(0, n_full);
    wait_loads<0>();
    process(0, n_full, true, [] {});
  }

  // ---- wave result -> LDS (over the rings, once every wave has left its own), merge of the waves, one partial per head
  const float l_tot = blocks_sum(l_run);
  __syncthreads();
  float* const lds_o = reinterpret_cast<float*>(smem);      // [NW][16][D]
  float* const lds_m = lds_o + NW * 16 * D;                  // [16][NW]
  float* const lds_l = lds_m + NW * 16;
  if (kq == 0) {
    lds_m[c * NW + wave] = m_run;
    lds_l[c * NW + wave] = l_tot;
  }
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      float2 o2;
      o2.x = oacc[j][0][i];
      o2.y = oacc[j][1][i];
      *reinterpret_cast<float2*>(lds_o + (wave * 16 + 4 * kq + i) * D + 32 * j + 2 * c) = o2;
    }
  __syncthreads();
  for (int idx = threadIdx.x; idx < G * (D / 2); idx += NW * 64) {
    const int h = idx / (D / 2), j = (idx % (D / 2)) * 2;
    float mg = kNegBig;
#pragma unroll
    for (int w = 0; w < NW; ++w) mg = fmaxf(mg, lds_m[h * NW + w]);
    float n0 = 0.0f, n1 = 0.0f, den = 0.0f;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
      const float e = __builtin_amdgcn_exp2f(lds_m[h * NW + w] - mg);
      const float2 o2 = *reinterpret_cast<const float2*>(lds_o + (w * 16 + h) * D + j);
      n0 = fmaf(o2.x, e, n0);
      n1 = fmaf(o2.y, e, n1);
      den = fmaf(lds_l[h * NW + w], e, den);
    }
    const int64_t ph = (int64_t)(b * p.n_q_heads + h0 + h) * p.n_splits + split;
    *reinterpret_cast<float2*>(p.part_o + ph * D + j) = make_float2(n0, n1);
    if (j == 0) *reinterpret_cast<float2*>(p.part_ml + ph * 2) = make_float2(mg, den);
  }
}

template <int D>
hipError_t launch_dense(const DecodeParams& p, int batch, hipStream_t s) {
  using C = DenseCfg<D>;
  static_assert(C::SMEM <= 160 * 1024, "LDS budget of one compute unit");
  // dynamic LDS above 64 KB has to be opted into, once per device and kernel instance (any thread may get here first)
  static std::once_flag configured[64];
  static hipError_t outcome[64];
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  std::call_once(configured[dev], [&] {
    outcome[dev] = hipFuncSetAttribute(reinterpret_cast<const void*>(&dense_partial_mfma_kernel<D>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, C::SMEM);
  });
  if (outcome[dev] != hipSuccess) return outcome[dev];
  hipLaunchKernelGGL((dense_partial_mfma_kernel<D>), dim3(p.n_splits, p.n_kv_heads, batch), dim3(C::NW * 64), C::SMEM, s, p);
  return hipGetLastError();
}

}  // namespace

bool dense_mfma_supported(int head_dim, int gqa) { return (head_dim == 128 || head_dim == 256) && gqa >= 1 && gqa <= 16; }

int dense_mfma_waves(int head_dim) { return 512 / head_dim; }

hipError_t launch_partial_dense_mfma(const DecodeParams& p, int batch, int head_dim, hipStream_t s) {
  if (!dense_mfma_supported(head_dim, p.gqa) || !p.k_dense || !p.v_dense || p.tokens_per_split % kTile != 0 ||
      p.start != 0 || p.seq_lens || p.block_table || (int64_t)p.tokens_per_split * head_dim * 2 >= (1ll << 31))
    return hipErrorNotSupported;
  return head_dim == 128 ? launch_dense<128>(p, batch, s) : launch_dense<256>(p, batch, s);
}

}  // namespace tq
