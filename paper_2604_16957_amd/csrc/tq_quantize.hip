// Quantise-and-append (Sec. 2.1, Eq. 2-3) and the comparator's dense dequantisation
// (the materialising step of the dequantize-then-attend baseline, Sec. 3.1).
//
// One thread owns 32 consecutive head_dim elements of one token: it reads 64 B of fp16 (four 128-bit loads),
// finds min/max in registers, and writes 16 B of codes; with groups of 32 that is a whole group, and the
// thread also writes its fp16 scale and zero-point; a group of 64 or 128 elements is 2 or 4 neighbouring
// lanes, which exchange their minima and maxima (exact in any order) before the scale is worked out, and the
// first of them writes it.  No LDS.  The arithmetic must give the
// same bits on every IEEE machine, so each fp32 step is a separately rounded operation:
// contraction is off for this file and the correctly rounded divide is used.
#include <algorithm>

#include "tq_internal.h"

#pragma clang fp contract(off)

namespace tq {
namespace {

struct QuantParams {
  const half_t* src[2];   // k_new, v_new: [B*H_kv][n_new][D]
  uint8_t* codes[2];      // [B*H_kv][capacity][D/2]
  half_t* scale[2];       // [B*H_kv][capacity][D/32]
  half_t* zero[2];
  int32_t n_new, capacity, pos, head_dim, n_kv_heads;
  int32_t group;              // elements per quantisation group: 32, 64 or 128
  const int32_t* pos_dev;     // per-sequence positions (device, [B]) or null
  const int32_t* block_table; // paged cache (see DecodeParams): [B][max_blocks] page numbers, or null
  int32_t max_blocks, page_shift;
  int64_t groups_per_tensor;  // B*H_kv*n_new*(D/32): 32-element pieces, one per thread
};

typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
union Pack16 { uint4 v; half_t h[8]; };

// 16-byte store with the non-temporal hint: bulk output that the writing kernel never reads again (a 128K layer's
// bulk quantise 124.4 -> 119.9 us with it, the comparator's dequantise-then-attend 240.8 -> 225.2 us)
__device__ __forceinline__ void store_stream16(void* dst, uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
  typedef uint32_t u4v __attribute__((ext_vector_type(4)));
  const u4v x = {a, b, c, d};
  __builtin_nontemporal_store(x, reinterpret_cast<u4v*>(dst));
}

__global__ __launch_bounds__(256) void quantize_append_kernel(QuantParams p) {
  const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= p.groups_per_tensor) return;
  const int which = blockIdx.y;                       // 0 = K, 1 = V
  // The source is one contiguous run of 64-byte pieces in thread order, so its loads do not wait for the index
  // arithmetic below.  Four 16-byte loads at a 64-byte stride across the wave: the wave's 4 KB is contiguous and
  // the lines are reused out of the cache between the four loads.  Both a non-temporal hint and an exchange through
  // LDS that makes every load fully coalesced were measured slower (by 11 and 13 %).
  const uint4* src = reinterpret_cast<const uint4*>(p.src[which] + idx * kGroup);
  Pack16 u[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) u[i].v = src[i];
  const int ng = p.head_dim / kGroup;                 // 32-element pieces per token
  const int g = (int)(idx % ng);
  const int64_t vec = idx / ng;                       // (b*H_kv + h) * n_new + t
  const int64_t bh = vec / p.n_new;
  const int t = (int)(vec % p.n_new);
  int pos = p.pos;
  if (p.pos_dev) {
    pos = p.pos_dev[bh / p.n_kv_heads] + p.pos;
    const int64_t room = p.block_table ? ((int64_t)p.max_blocks << p.page_shift) : p.capacity;
    if (pos < 0 || pos > room - p.n_new) return;          // this sequence's tokens do not fit: nothing is written
  }

  half2_t mn2, mx2;                                    // running min / max of the even and the odd elements
#pragma unroll
  for (int i = 0; i < 4; ++i) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const half2_t e = {u[i].h[2 * j], u[i].h[2 * j + 1]};
      mn2 = (i | j) ? __builtin_elementwise_min(mn2, e) : e;
      mx2 = (i | j) ? __builtin_elementwise_max(mx2, e) : e;
    }
  }
  // Eq. 2 over the whole group: this thread's 32 elements, and with larger groups its 1 or 3 neighbours'
  // (pieces of a group are consecutive lanes of one wave, and they leave or stay together above)
  float mn = fminf((float)mn2[0], (float)mn2[1]), mx = fmaxf((float)mx2[0], (float)mx2[1]);
  const int pieces = p.group / kGroup;                 // 1, 2 or 4
  for (int off = 1; off < pieces; off <<= 1) {
    mn = fminf(mn, __shfl_xor(mn, off));
    mx = fmaxf(mx, __shfl_xor(mx, off));
  }
  half_t s16, z16;
  quantize_scale_zero(mn, mx, s16, z16);
  const float sf = (float)s16, zf = (float)z16;
  uint32_t w[4];
  // Eq. 3: by the shortcut, and again by correctly rounded divides where the shortcut could matter
  const QuantFast fast = quantize_fast_setup(sf, zf, fmaxf(fabsf(mn), fabsf(mx)));
  float far = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) w[i] = quantize_word_fast(u[i].h, fast, far);
  if (quantize_fast_in_doubt(far, fast)) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      float x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) x[j] = (float)u[i].h[j];
      w[i] = quantize_word(x, sf, zf);
    }
  }
  int64_t row = bh * p.capacity + pos + t;
  if (p.block_table) {                                 // paged cache: capacity is the page length
    const int tok = pos + t;
    const int page = p.block_table[(bh / p.n_kv_heads) * p.max_blocks + (tok >> p.page_shift)];
    row = ((int64_t)page * p.n_kv_heads + bh % p.n_kv_heads) * p.capacity + (tok & ((1 << p.page_shift) - 1));
  }
  store_stream16(p.codes[which] + row * (p.head_dim / 2) + g * (kGroup / 2), w[0], w[1], w[2], w[3]);
  if (g % pieces == 0) {
    p.scale[which][row * (ng / pieces) + g / pieces] = s16;
    p.zero[which][row * (ng / pieces) + g / pieces] = z16;
  }
}

struct DequantParams {
  const uint8_t* codes[2];
  const half_t* scale[2];
  const half_t* zero[2];
  half_t* dense[2];           // [B*H_kv][seq_len][D]
  int32_t seq_len, capacity, head_dim, group, rows;   // rows = B * H_kv
};

// x^ = (q - z) * s (Eq. 3) rounded to fp16: what "dequantize, then attend" materialises.
// One thread per packed word (8 elements): a wave reads 256 contiguous bytes of codes and writes 1 KB of
// contiguous fp16 with one 16-byte store per lane.  (One thread per 32 elements, four 16-byte stores at a 64-byte
// stride across the wave, was measured at 176 us for a 128K layer against this kernel's time: the partial lines
// of every store went to the L2 one by one.)  grid: (pieces of a row's seq_len * D / 8 words, row or rows, K | V).
__global__ __launch_bounds__(256) void dequant_dense_kernel(DequantParams p) {
  const int which = blockIdx.z;
  const int wpt = p.head_dim / 8;                     // packed words per token
  const uint32_t idx = blockIdx.x * blockDim.x + threadIdx.x;   // word of the (sequence, KV head) row's seq_len tokens
  if (idx >= (uint32_t)p.seq_len * wpt) return;
  const uint32_t t = idx / wpt, wd = idx - t * wpt;   // (head_dim is a power of two: shifts)
  const int gpt = p.head_dim / p.group;               // groups per token
  const int g = wd * 8 / p.group;
  for (int bh = blockIdx.y; bh < p.rows; bh += gridDim.y) {
    const int64_t row = (int64_t)bh * p.capacity + t;
    const uint32_t w = *reinterpret_cast<const uint32_t*>(p.codes[which] + row * (p.head_dim / 2) + wd * 4);
    const float sf = (float)p.scale[which][row * gpt + g];
    const float zf = (float)p.zero[which][row * gpt + g];
    Pack16 u;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float q = (float)((w >> (4 * j)) & 0xFu);
      u.h[j] = (half_t)((q - zf) * sf);
    }
    store_stream16(p.dense[which] + ((int64_t)bh * p.seq_len + t) * p.head_dim + wd * 8, u.v.x, u.v.y, u.v.z, u.v.w);
  }
}

}  // namespace

hipError_t launch_quantize(const tq_kv_cache& c, const void* k_new, const void* v_new, int pos,
                           const int32_t* pos_dev, int n_new, hipStream_t s, const PagedView* pv) {
  QuantParams p;
  p.src[0] = static_cast<const half_t*>(k_new);
  p.src[1] = static_cast<const half_t*>(v_new);
  p.codes[0] = static_cast<uint8_t*>(c.k_codes);
  p.codes[1] = static_cast<uint8_t*>(c.v_codes);
  p.scale[0] = static_cast<half_t*>(c.k_scale);
  p.scale[1] = static_cast<half_t*>(c.v_scale);
  p.zero[0] = static_cast<half_t*>(c.k_zero);
  p.zero[1] = static_cast<half_t*>(c.v_zero);
  p.n_new = n_new;
  p.group = c.group_size;
  p.capacity = c.capacity;
  p.pos = pos;
  p.pos_dev = pos_dev;
  p.block_table = pv ? pv->block_table : nullptr;
  p.max_blocks = pv ? pv->max_blocks : 0;
  p.page_shift = pv ? pv->page_shift : 0;
  p.n_kv_heads = c.n_kv_heads;
  p.head_dim = c.head_dim;
  const int batch = pv ? pv->batch : c.batch;            // in a paged pool c.batch counts pages, not sequences
  p.groups_per_tensor = (int64_t)batch * c.n_kv_heads * n_new * (c.head_dim / kGroup);
  const unsigned blocks = (unsigned)((p.groups_per_tensor + 255) / 256);
  hipLaunchKernelGGL(quantize_append_kernel, dim3(blocks, 2), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_dequant_dense(const tq_kv_cache& c, int seq_len, half_t* k_dense, half_t* v_dense,
                                hipStream_t s) {
  DequantParams p;
  p.codes[0] = static_cast<const uint8_t*>(c.k_codes);
  p.codes[1] = static_cast<const uint8_t*>(c.v_codes);
  p.scale[0] = static_cast<const half_t*>(c.k_scale);
  p.scale[1] = static_cast<const half_t*>(c.v_scale);
  p.zero[0] = static_cast<const half_t*>(c.k_zero);
  p.zero[1] = static_cast<const half_t*>(c.v_zero);
  p.dense[0] = k_dense;
  p.dense[1] = v_dense;
  p.seq_len = seq_len;
  p.capacity = c.capacity;
  p.head_dim = c.head_dim;
  p.group = c.group_size;
  p.rows = c.batch * c.n_kv_heads;
  if ((int64_t)seq_len * (c.head_dim / 8) >= (1ll << 32)) return hipErrorNotSupported;   // a row's words are counted in 32 bits
  const unsigned blocks = (unsigned)(((int64_t)seq_len * (c.head_dim / 8) + 255) / 256);
  hipLaunchKernelGGL(dequant_dense_kernel, dim3(blocks, (unsigned)std::min(p.rows, 65535), 2), dim3(256), 0, s, p);
  return hipGetLastError();
}

}  // namespace tq
