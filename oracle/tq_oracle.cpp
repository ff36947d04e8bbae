// CPU oracle for compressed-domain int4 decode attention.
//
// TEST INFRASTRUCTURE ONLY.  Plain, slow, obviously-correct reference used by tests/, by the
// smoke check and by the benchmark's cpu_baseline leg.  The product (the HIP library) never
// links, loads or calls anything here, and this file shares no code, header, table or helper
// with it.
//
// What it computes, and from where:
//   * per-group asymmetric int4 quantisation and its inverse        (Sec. 2.1, Eq. 2-3)
//   * two codes per byte, element j of a packed word in bits 4j..4j+3 (Sec. 2.1; nibble order
//     as implied by the masks/pre-division of Eq. 5)
//   * decode attention as its plain definition: softmax(alpha q.k^)v^ over the dequantised
//     cache, in fp64, one query row per head, kv_head = head / gqa   (Sec. 3.1; GQA rule at
//     the end of Sec. 3.1).  Online softmax (Alg. 1) and the split-K merge (Eq. 6) are
//     algebraic identities of this definition, so the definition is the oracle; a literal
//     Alg. 1 + Eq. 6 version is also here so tests can show the two agree.
//
// Readings where the paper is silent (all listed in the design notes):
//   scale and zero-point are computed in fp32 and stored as fp16; codes are computed from the
//   STORED values; ties round half-to-even; a constant (or fp16-underflowing) group gets
//   scale 1.0 and zero-point -min; zero-point saturates at +-65504 and -0 is stored as +0.
//
// Group size g: 32 (the paper's configuration), 64 or 128 (Sec. 2.1 states the scheme for any g).
//
// Pins (tests/test_oracle_*.py): closed-form groups, half-even ties, |x^-x| <= s/2, nibble
// order, 4 + 32/g bits/element and the memory table (Table 4 / Eq. 1), exhaustive fp16 conversion
// against an independent converter, S=1, identical keys, score-shift invariance, argmax limit,
// brute force on tiny inputs with exact rationals, Alg. 1 + Eq. 6 == definition, GQA mapping,
// token-permutation invariance.  No function here is "parity unpinned".

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <thread>
#include <vector>

namespace {

constexpr int kMaxGroup = 128;                     // group sizes offered: 32 (the paper's), 64, 128

inline bool group_ok(int d, int g) { return (g == 32 || g == 64 || g == 128) && d > 0 && d % g == 0; }

// ---- fp16 <-> fp32, bit level (IEEE binary16, round-to-nearest-even) -------------------

float half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  const uint32_t exp = (h >> 10) & 0x1Fu;
  const uint32_t man = h & 0x3FFu;
  uint32_t out;
  if (exp == 0) {
    if (man == 0) {
      out = sign;
    } else {  // subnormal: value = man * 2^-24; normalise
      int e = -1;
      uint32_t m = man;
      do { ++e; m <<= 1; } while ((m & 0x400u) == 0);
      out = sign | ((uint32_t)(127 - 15 - e) << 23) | ((m & 0x3FFu) << 13);
    }
  } else if (exp == 31) {
    out = sign | 0x7F800000u | (man << 13);
  } else {
    out = sign | ((exp + (127 - 15)) << 23) | (man << 13);
  }
  float f;
  std::memcpy(&f, &out, 4);
  return f;
}

uint16_t float_to_half_bits_rne(float f) {
  uint32_t x;
  std::memcpy(&x, &f, 4);
  const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
  const uint32_t absx = x & 0x7FFFFFFFu;
  if (absx >= 0x7F800000u) {                 // inf / nan
    return (uint16_t)(sign | 0x7C00u | (absx > 0x7F800000u ? 0x200u | ((absx >> 13) & 0x3FFu) : 0u));
  }
  const int32_t e = (int32_t)(absx >> 23) - 127;   // unbiased exponent
  uint32_t man = (absx & 0x7FFFFFu) | 0x800000u;   // 24-bit significand with hidden bit
  if (e >= 16) return (uint16_t)(sign | 0x7C00u);  // certainly overflows (>= 65536)
  if (e >= -14) {                                  // normal half (before rounding)
    uint32_t half_man = man >> 13;                 // 11 bits incl. hidden
    const uint32_t rem = man & 0x1FFFu;
    if (rem > 0x1000u || (rem == 0x1000u && (half_man & 1u))) ++half_man;
    uint32_t he = (uint32_t)(e + 15);
    if (half_man == 0x800u) { half_man = 0x400u; ++he; }  // significand carried out
    if (he >= 31) return (uint16_t)(sign | 0x7C00u);
    return (uint16_t)(sign | (he << 10) | (half_man & 0x3FFu));
  }
  if (e < -25) return sign;                        // < 2^-25: rounds to zero
  // subnormal half: value = man * 2^(e-23); target unit 2^-24  => shift right by (-e - 1)
  const int shift = -e - 1;                        // 14..24
  const uint32_t q = man >> shift;
  const uint32_t rem = man & ((1u << shift) - 1u);
  const uint32_t halfway = 1u << (shift - 1);
  uint32_t r = q;
  if (rem > halfway || (rem == halfway && (q & 1u))) ++r;
  return (uint16_t)(sign | r);                     // r == 0x400 becomes the smallest normal
}

// ---- quantiser (Sec. 2.1, Eq. 2-3) ------------------------------------------------------

// One group of g consecutive elements: g/2 bytes of codes, one scale, one zero-point.
void quantize_group(const uint16_t* x16, int g, uint8_t* codes_out, uint16_t* s_out, uint16_t* z_out) {
  float x[kMaxGroup] = {};                          // (callers pass g >= 32; zeroed only to say so to the compiler)
  for (int j = 0; j < g; ++j) x[j] = half_bits_to_float(x16[j]);
  float mn = x[0], mx = x[0];
  for (int j = 1; j < g; ++j) { mn = std::min(mn, x[j]); mx = std::max(mx, x[j]); }
  volatile float range = mx - mn;                  // volatile: keep each fp32 step separate
  volatile float s32 = range / 15.0f;              // Eq. 2, scale
  uint16_t s16 = float_to_half_bits_rne(s32);
  if ((s16 & 0x7FFFu) == 0) s16 = 0x3C00u;         // constant / underflowing group -> scale 1
  const float sf = half_bits_to_float(s16);
  volatile float negmin = 0.0f - mn;
  volatile float z32 = negmin / sf;                // Eq. 2, zero-point, from the stored scale
  uint16_t z16 = float_to_half_bits_rne(z32);
  if ((z16 & 0x7FFFu) == 0x7C00u) z16 = (uint16_t)((z16 & 0x8000u) | 0x7BFFu);  // saturate
  if (z16 == 0x8000u) z16 = 0;
  const float zf = half_bits_to_float(z16);
  uint8_t c[kMaxGroup];
  for (int j = 0; j < g; ++j) {
    volatile float t = x[j] / sf;                  // Eq. 3: x/s ...
    volatile float u = t + zf;                     // ... + z, as a separate fp32 add
    float r = std::nearbyintf(u);                  // half-to-even in the default rounding mode
    r = std::min(15.0f, std::max(0.0f, r));
    c[j] = (uint8_t)r;
  }
  for (int b = 0; b < g / 2; ++b) codes_out[b] = (uint8_t)(c[2 * b] | (c[2 * b + 1] << 4));
  *s_out = s16;
  *z_out = z16;
}

inline int code_at(const uint8_t* codes, int j) {  // element j of a packed vector
  const uint8_t byte = codes[j >> 1];
  return (j & 1) ? (byte >> 4) : (byte & 0xF);
}

inline double dequant_elem(const uint8_t* codes, const uint16_t* s, const uint16_t* z, int j, int g) {
  const double sf = (double)half_bits_to_float(s[j / g]);
  const double zf = (double)half_bits_to_float(z[j / g]);
  return ((double)code_at(codes, j) - zf) * sf;    // Eq. 3, x^ = (q - z) s, in fp64
}

struct CacheView {
  const uint8_t* codes; const uint16_t* scale; const uint16_t* zero;
  int64_t capacity; int d; int g;
  const uint8_t* tok_codes(int64_t bh, int64_t t) const { return codes + (bh * capacity + t) * (d / 2); }
  const uint16_t* tok_scale(int64_t bh, int64_t t) const { return scale + (bh * capacity + t) * (d / g); }
  const uint16_t* tok_zero(int64_t bh, int64_t t) const { return zero + (bh * capacity + t) * (d / g); }
};

void dequant_head(const CacheView& c, int64_t bh, int64_t S, std::vector<double>& out) {
  out.resize((size_t)S * c.d);
  for (int64_t t = 0; t < S; ++t)
    for (int j = 0; j < c.d; ++j)
      out[(size_t)t * c.d + j] = dequant_elem(c.tok_codes(bh, t), c.tok_scale(bh, t), c.tok_zero(bh, t), j, c.g);
}

// softmax(alpha * q.K^ + bias) V^ for one query row, by definition (max-subtracted).
void attend_row_naive(const double* q, const double* K, const double* V, int64_t S, int d,
                      double alpha, double bias, double* out) {
  std::vector<double> a((size_t)S);
  double m = -std::numeric_limits<double>::infinity();
  for (int64_t i = 0; i < S; ++i) {
    double dot = 0.0;
    for (int j = 0; j < d; ++j) dot += q[j] * K[(size_t)i * d + j];
    a[(size_t)i] = alpha * dot + bias;
    m = std::max(m, a[(size_t)i]);
  }
  double denom = 0.0;
  for (int64_t i = 0; i < S; ++i) { a[(size_t)i] = std::exp(a[(size_t)i] - m); denom += a[(size_t)i]; }
  for (int j = 0; j < d; ++j) out[j] = 0.0;
  for (int64_t i = 0; i < S; ++i) {
    const double p = a[(size_t)i] / denom;
    for (int j = 0; j < d; ++j) out[j] += p * V[(size_t)i * d + j];
  }
}

// Alg. 1 on tokens [lo, hi): returns the NORMALISED chunk output o/l plus (m, l).
void alg1_chunk(const double* q_scaled, const double* K, const double* V, int64_t lo, int64_t hi,
                int d, double* o_c, double* m_c, double* l_c) {
  double m = -std::numeric_limits<double>::infinity(), l = 0.0;
  std::vector<double> o((size_t)d, 0.0);
  for (int64_t i = lo; i < hi; ++i) {
    double a = 0.0;
    for (int j = 0; j < d; ++j) a += q_scaled[j] * K[(size_t)i * d + j];
    const double m_new = std::max(m, a);
    const double corr = std::exp(m - m_new);       // exp(-inf) = 0 on the first token
    const double p = std::exp(a - m_new);
    l = l * corr + p;
    for (int j = 0; j < d; ++j) o[(size_t)j] = o[(size_t)j] * corr + p * V[(size_t)i * d + j];
    m = m_new;
  }
  for (int j = 0; j < d; ++j) o_c[j] = o[(size_t)j] / l;
  *m_c = m; *l_c = l;
}

template <class F>
void parallel_for(int64_t n, int nthreads, F f) {
  nthreads = (int)std::max<int64_t>(1, std::min<int64_t>(nthreads, n));
  if (nthreads == 1) { for (int64_t i = 0; i < n; ++i) f(i); return; }
  std::vector<std::thread> th;
  for (int t = 0; t < nthreads; ++t)
    th.emplace_back([=]() { for (int64_t i = t; i < n; i += nthreads) f(i); });
  for (auto& x : th) x.join();
}

}  // namespace

extern "C" {

float orc_half_to_float(uint16_t h) { return half_bits_to_float(h); }
uint16_t orc_float_to_half(float f) { return float_to_half_bits_rne(f); }

// x: fp16 bits [n_vec][d]; codes [n_vec][d/2]; scale, zero: fp16 bits [n_vec][d/g], g = the group size.
int orc_quantize(const uint16_t* x, int64_t n_vec, int d, int g, uint8_t* codes, uint16_t* scale,
                 uint16_t* zero, int nthreads) {
  if (!group_ok(d, g)) return -1;
  const int ng = d / g;
  parallel_for(n_vec, nthreads, [=](int64_t v) {
    for (int i = 0; i < ng; ++i)
      quantize_group(x + v * d + i * g, g, codes + v * (d / 2) + i * (g / 2), scale + v * ng + i, zero + v * ng + i);
  });
  return 0;
}

// fp64 value of every stored element: out [n_vec][d].
int orc_dequantize_f64(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                       int64_t n_vec, int d, int g, double* out) {
  if (!group_ok(d, g)) return -1;
  const int ng = d / g;
  for (int64_t v = 0; v < n_vec; ++v)
    for (int j = 0; j < d; ++j)
      out[v * d + j] = dequant_elem(codes + v * (d / 2), scale + v * ng, zero + v * ng, j, g);
  return 0;
}

// What the unfused comparator's dense buffer must hold: fp16_rne of the fp64 value.
int orc_dequantize_f16(const uint8_t* codes, const uint16_t* scale, const uint16_t* zero,
                       int64_t n_vec, int d, int g, uint16_t* out) {
  if (!group_ok(d, g)) return -1;
  const int ng = d / g;
  for (int64_t v = 0; v < n_vec; ++v)
    for (int j = 0; j < d; ++j) {
      // (c - z) s has at most 4+11+11 significant bits: exact in fp64, and its fp32 rounding
      // followed by fp16 rounding could double-round, so round once from fp64 by hand.
      const double x = dequant_elem(codes + v * (d / 2), scale + v * ng, zero + v * ng, j, g);
      float f = (float)x;
      if ((double)f != x) {  // make the fp32 intermediate "sticky" so the fp16 rounding is single
        uint32_t u; std::memcpy(&u, &f, 4);
        const bool f_mag_bigger = std::fabs((double)f) > std::fabs(x);
        if (!(u & 1u)) { u = f_mag_bigger ? u - 1 : u + 1; }  // move to the odd neighbour toward x
        std::memcpy(&f, &u, 4);
      }
      out[v * d + j] = float_to_half_bits_rne(f);
    }
  return 0;
}

// Decode attention by definition over DENSE fp64 K^, V^ [B][H_kv][S][d]; q fp16 bits [B][H_q][d];
// out fp64 [B][H_q][d].  score_bias is added to every score (test hook: the result must not move).
int orc_attend_dense_f64(const uint16_t* q, const double* K, const double* V, int B, int Hq, int Hkv,
                         int64_t S, int d, double alpha, double score_bias, double* out, int nthreads) {
  if (Hkv <= 0 || Hq % Hkv != 0 || S < 1) return -1;
  const int G = Hq / Hkv;
  parallel_for((int64_t)B * Hq, nthreads, [=](int64_t bh) {
    const int b = (int)(bh / Hq), h = (int)(bh % Hq);
    const int kv = h / G;                                  // GQA rule, Sec. 3.1
    std::vector<double> qd((size_t)d);
    for (int j = 0; j < d; ++j) qd[(size_t)j] = (double)half_bits_to_float(q[bh * d + j]);
    const size_t off = ((size_t)b * Hkv + kv) * (size_t)S * d;
    attend_row_naive(qd.data(), K + off, V + off, S, d, alpha, score_bias, out + bh * d);
  });
  return 0;
}

// Decode attention by definition over the PACKED cache (canonical layout, row stride `capacity`).
int orc_attend_packed_f64(const uint16_t* q,
                          const uint8_t* k_codes, const uint16_t* k_scale, const uint16_t* k_zero,
                          const uint8_t* v_codes, const uint16_t* v_scale, const uint16_t* v_zero,
                          int B, int Hq, int Hkv, int64_t capacity, int64_t S, int d, int g, double alpha,
                          double* out, int nthreads) {
  if (Hkv <= 0 || Hq % Hkv != 0 || S < 1 || S > capacity || !group_ok(d, g)) return -1;
  const int G = Hq / Hkv;
  const CacheView kc{k_codes, k_scale, k_zero, capacity, d, g}, vc{v_codes, v_scale, v_zero, capacity, d, g};
  parallel_for((int64_t)B * Hkv, nthreads, [=](int64_t bkv) {
    std::vector<double> K, V, qd((size_t)d);
    dequant_head(kc, bkv, S, K);
    dequant_head(vc, bkv, S, V);
    const int b = (int)(bkv / Hkv), kv = (int)(bkv % Hkv);
    for (int h = kv * G; h < (kv + 1) * G; ++h) {          // heads with h / G == kv
      const int64_t bh = (int64_t)b * Hq + h;
      for (int j = 0; j < d; ++j) qd[(size_t)j] = (double)half_bits_to_float(q[bh * d + j]);
      attend_row_naive(qd.data(), K.data(), V.data(), S, d, alpha, 0.0, out + bh * d);
    }
  });
  return 0;
}

// Literal Alg. 1 per chunk followed by the Eq. 6 merge, fp64, over dense K^, V^.
// bounds: n_chunks+1 increasing token indices, bounds[0]=0, bounds[n_chunks]=S.
int orc_attend_alg1_eq6_f64(const uint16_t* q, const double* K, const double* V, int B, int Hq, int Hkv,
                            int64_t S, int d, double alpha, const int64_t* bounds, int n_chunks,
                            double* out) {
  if (Hkv <= 0 || Hq % Hkv != 0 || S < 1 || n_chunks < 1) return -1;
  if (bounds[0] != 0 || bounds[n_chunks] != S) return -2;
  for (int c = 0; c < n_chunks; ++c) if (bounds[c + 1] <= bounds[c]) return -2;
  const int G = Hq / Hkv;
  std::vector<double> qs((size_t)d), oc((size_t)n_chunks * d), mc((size_t)n_chunks), lc((size_t)n_chunks);
  for (int64_t bh = 0; bh < (int64_t)B * Hq; ++bh) {
    const int b = (int)(bh / Hq), h = (int)(bh % Hq), kv = h / G;
    for (int j = 0; j < d; ++j)                            // Alg. 1 starts by pre-scaling the query
      qs[(size_t)j] = (double)half_bits_to_float(q[bh * d + j]) * alpha;
    const size_t off = ((size_t)b * Hkv + kv) * (size_t)S * d;
    for (int c = 0; c < n_chunks; ++c)
      alg1_chunk(qs.data(), K + off, V + off, bounds[c], bounds[c + 1], d,
                 &oc[(size_t)c * d], &mc[(size_t)c], &lc[(size_t)c]);
    double mg = -std::numeric_limits<double>::infinity();
    for (int c = 0; c < n_chunks; ++c) mg = std::max(mg, mc[(size_t)c]);
    double den = 0.0;
    for (int c = 0; c < n_chunks; ++c) den += lc[(size_t)c] * std::exp(mc[(size_t)c] - mg);
    for (int j = 0; j < d; ++j) {
      double num = 0.0;                                    // Eq. 6
      for (int c = 0; c < n_chunks; ++c)
        num += lc[(size_t)c] * std::exp(mc[(size_t)c] - mg) * oc[(size_t)c * d + j];
      out[bh * d + j] = num / den;
    }
  }
  return 0;
}

// Bytes of a KV cache (K and V) for n_layers x n_kv_heads x seq_len tokens of dim d at int4 with one fp16 scale
// and one fp16 zero-point per group of g elements (Sec. 2.1: 4 + 32/g bits per element), and the same at fp16 (Eq. 1).
int64_t orc_kv_bytes_int4(int64_t n_layers, int64_t n_kv_heads, int64_t seq_len, int64_t d, int64_t g) {
  return 2 * n_layers * n_kv_heads * seq_len * (d / 2 + 2 * 2 * (d / g));
}
int64_t orc_kv_bytes_fp16(int64_t n_layers, int64_t n_kv_heads, int64_t seq_len, int64_t d) {
  return 2 * n_layers * n_kv_heads * seq_len * d * 2;
}

}  // extern "C"
