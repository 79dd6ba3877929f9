// NQKV CPU oracle -- TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, single-purpose CPU statement of what the NQKV hot path computes:
// per-block normal-quantile quantization of a KV cache (paper Sec. 3.2, Fig. 5) and
// softmax attention of one query row over the dequantized cache (paper Sec. 3.2,
// decoding-phase equations).  It exists so that tests, the smoke check and the
// benchmark's cpu_baseline leg can compare the GPU library against it.  Nothing in
// the product path may call it, and it shares no code, header, table or constant
// with the GPU library.
//
// Conventions (each is a reading of the paper where the paper itself is silent):
//   * codebook, variant 0: 2^k levels = medians of 2^k equal-probability bins of
//     N(0,1), divided by the largest one, built for the positive half and mirrored
//     (Sec. 1: the data points are normal-distribution quantiles; Sec. 3.2);
//     variant 1: zero-preserving asymmetric table in the Normal-Float style the
//     paper cites for its 4-bit experiments (Sec. 3.2), with this build's own
//     tail offset delta = 2^-(k+1);
//   * block = `blk` consecutive head_dim elements of one token of one head
//     (Fig. 5 caption); scale = max |x| of the block, kept as the fp16 it is;
//   * nearest level decided as  code = #{ j : float(x) > fl32(t_j * float(s)) }
//     with fp32 mid-point thresholds t_j, ties to the lower level;
//   * codes packed LSB-first: element i of a token-head row owns bits [k*i, k*i+k);
//   * dequantized value = fp16_rne( fl32( level[code] * float(s) ) ) (Fig. 5 caption:
//     indices are looked up and restored to FP16);
//   * attention in fp64 over the exact products level*scale, one (batch, head) at a
//     time, the token appended this step included (Sec. 3.2 decoding phase).
//
// Floating point: everything that decides a code or a stored bit is written in fp32
// with one rounding per operation (compile with -ffp-contract=off, no fast-math);
// attention is fp64.  fp16 <-> fp32 conversion is done in software below.

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <functional>
#include <thread>
#include <vector>

namespace {

// ---------------------------------------------------------------- fp16 helpers
// IEEE binary16 -> binary32, exact (subnormals, infinities and NaN included).
float half_bits_to_float(uint16_t h) {
  const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
  const uint32_t exp = (h >> 10) & 0x1fu;
  const uint32_t man = h & 0x3ffu;
  uint32_t out;
  if (exp == 0) {
    if (man == 0) {
      out = sign;
    } else {
      // subnormal: value = man * 2^-24; normalise
      int e = -1;
      uint32_t m = man;
      do { m <<= 1; ++e; } while ((m & 0x400u) == 0);
      out = sign | (uint32_t)(127 - 15 - e) << 23 | (m & 0x3ffu) << 13;
    }
  } else if (exp == 31) {
    out = sign | 0x7f800000u | man << 13;
  } else {
    out = sign | (exp + 127 - 15) << 23 | man << 13;
  }
  float f;
  std::memcpy(&f, &out, 4);
  return f;
}

// binary32 -> binary16, round to nearest even, subnormal results kept.
uint16_t float_to_half_bits_rne(float f) {
  uint32_t x;
  std::memcpy(&x, &f, 4);
  const uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
  const uint32_t absx = x & 0x7fffffffu;
  if (absx >= 0x7f800000u) {                       // inf / nan
    return (uint16_t)(sign | 0x7c00u | ((absx > 0x7f800000u) ? 0x200u : 0u));
  }
  if (absx >= 0x477ff000u) {                       // >= 65520 rounds to inf
    return (uint16_t)(sign | 0x7c00u);
  }
  const int e = (int)(absx >> 23) - 127;           // unbiased exponent
  if (e >= -14) {                                  // normal half range
    const uint32_t man = absx & 0x7fffffu;
    uint32_t h = (uint32_t)(e + 15) << 10 | man >> 13;
    const uint32_t rest = man & 0x1fffu;
    if (rest > 0x1000u || (rest == 0x1000u && (h & 1u))) ++h;   // may carry into exponent: correct
    return (uint16_t)(sign | h);
  }
  if (e < -25) return sign;                        // below half of the smallest subnormal
  // subnormal half: value = m * 2^-24 with m in [0, 1023]
  const uint32_t man = (absx & 0x7fffffu) | 0x800000u;  // 24-bit significand, value = man * 2^(e-23)
  const int shift = -e - 1;                        // m = man * 2^(e-23+24) = man >> (-e-1)
  uint32_t m = man >> shift;
  const uint32_t rest = man & ((1u << shift) - 1u);
  const uint32_t half = 1u << (shift - 1);
  if (rest > half || (rest == half && (m & 1u))) ++m;
  return (uint16_t)(sign | m);
}

// ---------------------------------------------------------------- normal quantile
// Upper-tail quantile: the x >= 0 with  P(Z > x) = tail,  0 < tail <= 1/2, found by
// bisection on  P(Z > x) = erfc(x / sqrt 2) / 2  (monotone decreasing in x).
double upper_tail_quantile(double tail) {
  double lo = 0.0, hi = 40.0;
  for (int it = 0; it < 200; ++it) {
    const double mid = 0.5 * (lo + hi);
    const double p = 0.5 * std::erfc(mid / std::sqrt(2.0));
    if (p > tail) lo = mid; else hi = mid;
  }
  return 0.5 * (lo + hi);
}

// Independent (batch, head) slices handed round-robin to n_threads host threads.
void run_parallel(int64_t n_items, int n_threads, const std::function<void(int64_t)>& body) {
  if (n_threads <= 1 || n_items <= 1) {
    for (int64_t i = 0; i < n_items; ++i) body(i);
    return;
  }
  const int nt = (int)std::min<int64_t>(n_threads, n_items);
  std::vector<std::thread> pool;
  pool.reserve(nt);
  for (int w = 0; w < nt; ++w) {
    pool.emplace_back([=, &body]() {
      for (int64_t i = w; i < n_items; i += nt) body(i);
    });
  }
  for (auto& t : pool) t.join();
}
}  // namespace

extern "C" {

// Number of host threads the oracle would use for "all cores".
int oracle_hardware_threads() {
  const unsigned n = std::thread::hardware_concurrency();
  return n ? (int)n : 1;
}

// fp16 helpers exported so that tests can pin them against numpy.float16.
float oracle_half_to_float(uint16_t h) { return half_bits_to_float(h); }
uint16_t oracle_float_to_half(float f) { return float_to_half_bits_rne(f); }

// Codebook (Sec. 1 / Sec. 3.2: data points are quantile points of N(0,1)).
//   k in [1, 8], L = 2^k.
//   levels64[L]  : normalised levels in fp64, ascending, levels64[0] = -1, levels64[L-1] = 1
//   levels32[L]  : the same rounded once to fp32
//   thresh32[L-1]: fp32 mid-points  t_j = (levels32[j-1] + levels32[j]) * 0.5f,  j = 1..L-1,
//                  stored at thresh32[j-1]
// Returns 0, or -1 on a bad argument.
int oracle_codebook(int k, int variant, double* levels64, float* levels32, float* thresh32) {
  if (k < 1 || k > 8 || (variant != 0 && variant != 1)) return -1;
  const int L = 1 << k;
  std::vector<double> lev(L);
  if (variant == 0) {
    // Median of bin i of L equal-probability bins: Phi^-1((i + 1/2) / L).
    // Positive half: i = L/2 .. L-1, upper tail = (L - 1 - i + 1/2) / L.
    const double top = upper_tail_quantile(0.5 / L);
    for (int i = L / 2; i < L; ++i) {
      const double tail = ((double)(L - 1 - i) + 0.5) / (double)L;
      const double c = upper_tail_quantile(tail) / top;
      lev[i] = (i == L - 1) ? 1.0 : c;
      lev[L - 1 - i] = -lev[i];
    }
  } else {
    // Zero-preserving table: L/2 strictly positive levels, one exact zero and
    // L/2 - 1 strictly negative ones.  Each side is a set of evenly spaced
    // probabilities between 1/2 and 1 - delta pushed through Phi^-1, then divided by
    // the largest, so both ends are exactly +-1.   delta = 2^-(k+1).
    if (k < 2) return -1;
    const double delta = std::ldexp(1.0, -(k + 1));
    const int n_pos = L / 2;          // positive side gets the extra level
    const int n_neg = L / 2 - 1;
    const double top = upper_tail_quantile(delta);
    // positive: probabilities p_m = 1/2 + m * (1/2 - delta) / n_pos, m = 1..n_pos
    for (int m = 1; m <= n_pos; ++m) {
      const double p = 0.5 + (double)m * (0.5 - delta) / (double)n_pos;
      const double c = upper_tail_quantile(1.0 - p) / top;
      lev[n_neg + m] = (m == n_pos) ? 1.0 : c;
    }
    lev[n_neg] = 0.0;
    // negative: p_m = 1/2 + m * (1/2 - delta) / n_neg, m = 1..n_neg, mirrored
    for (int m = 1; m <= n_neg; ++m) {
      const double p = 0.5 + (double)m * (0.5 - delta) / (double)n_neg;
      const double c = upper_tail_quantile(1.0 - p) / top;
      lev[n_neg - m] = (m == n_neg) ? -1.0 : -c;
    }
  }
  for (int i = 0; i < L; ++i) {
    if (levels64) levels64[i] = lev[i];
    if (levels32) levels32[i] = (float)lev[i];
  }
  if (thresh32) {
    for (int j = 1; j < L; ++j) {
      const float a = (float)lev[j - 1];
      const float b = (float)lev[j];
      const float sum = a + b;          // one fp32 rounding
      thresh32[j - 1] = sum * 0.5f;     // exact
    }
  }
  return 0;
}

// Quantize ONE block (Fig. 5: each block is quantized on its own).
//   x[blk]      fp16 bit patterns (finite)
//   levels32[L] the codebook
//   codes[blk]  out: one code per element (not packed)
//   scale       out: fp16 bit pattern of max |x|
void oracle_quantize_block(const uint16_t* x, int blk, int k, const float* levels32,
                           uint8_t* codes, uint16_t* scale) {
  const int L = 1 << k;
  // scale: the largest magnitude, compared as real numbers (fp16 -> fp32 is exact)
  uint16_t s_bits = 0;
  float s32 = 0.0f;
  for (int i = 0; i < blk; ++i) {
    const float a = std::fabs(half_bits_to_float(x[i]));
    if (a > s32) { s32 = a; s_bits = (uint16_t)(x[i] & 0x7fffu); }
  }
  *scale = s_bits;
  for (int i = 0; i < blk; ++i) {
    const float x32 = half_bits_to_float(x[i]);
    int code = 0;
    for (int j = 1; j < L; ++j) {
      const float sum = levels32[j - 1] + levels32[j];
      const float t = sum * 0.5f;
      const float T = t * s32;            // one fp32 rounding (built with -ffp-contract=off)
      if (x32 > T) ++code;
    }
    codes[i] = (uint8_t)code;
  }
}

// Pack `n` codes of k bits LSB-first into ceil(n*k/8) bytes: code i owns bits
// [k*i, k*i+k) of the stream, bit b of the stream is bit (b & 7) of byte (b >> 3).
void oracle_pack_bits(const uint8_t* codes, int64_t n, int k, uint8_t* bytes) {
  const int64_t n_bytes = (n * k + 7) / 8;
  std::memset(bytes, 0, (size_t)n_bytes);
  for (int64_t i = 0; i < n; ++i) {
    for (int b = 0; b < k; ++b) {
      if ((codes[i] >> b) & 1u) {
        const int64_t pos = i * k + b;
        bytes[pos >> 3] = (uint8_t)(bytes[pos >> 3] | (1u << (pos & 7)));
      }
    }
  }
}

void oracle_unpack_bits(const uint8_t* bytes, int64_t n, int k, uint8_t* codes) {
  for (int64_t i = 0; i < n; ++i) {
    unsigned c = 0;
    for (int b = 0; b < k; ++b) {
      const int64_t pos = i * k + b;
      c |= (unsigned)((bytes[pos >> 3] >> (pos & 7)) & 1u) << b;
    }
    codes[i] = (uint8_t)c;
  }
}

// Quantize a tensor into a cache (prefill and append are the same operation, Sec. 3.2:
// new keys/values are quantized and placed at the end; older entries never change).
//   src      fp16 bits, logical [B, H, n_tokens, D], element strides sb, sh, ss, D contiguous
//   codes    uint8 [B, H, cap_tokens, D*k/8]   (rows [dst_off, dst_off+n_tokens) written)
//   scales   fp16 bits [B, H, cap_tokens, D/blk]
// Returns 0, or -1 on a bad argument.
int oracle_quantize_kv(const uint16_t* src, int64_t sb, int64_t sh, int64_t ss,
                       int B, int H, int D, int64_t n_tokens,
                       int k, int blk, const float* levels32,
                       int64_t cap_tokens, int64_t dst_off,
                       uint8_t* codes, uint16_t* scales, int n_threads) {
  if (k < 1 || k > 8 || blk < 1 || D % blk != 0 || (D * k) % 8 != 0) return -1;
  if (dst_off < 0 || n_tokens < 0 || dst_off + n_tokens > cap_tokens) return -1;
  const int nb = D / blk;
  const int64_t row_bytes = (int64_t)D * k / 8;
  run_parallel((int64_t)B * H, n_threads, [&](int64_t bh) {
    const int b = (int)(bh / H), h = (int)(bh % H);
    std::vector<uint8_t> row_codes(D);
    for (int64_t t = 0; t < n_tokens; ++t) {
      const uint16_t* x = src + b * sb + h * sh + t * ss;
      const int64_t row = (bh * cap_tokens + dst_off + t);
      for (int j = 0; j < nb; ++j) {
        oracle_quantize_block(x + (int64_t)j * blk, blk, k, levels32,
                              row_codes.data() + (int64_t)j * blk, scales + row * nb + j);
      }
      oracle_pack_bits(row_codes.data(), D, k, codes + row * row_bytes);
    }
  });
  return 0;
}

// Blocks over the token's hidden vector (Fig. 5: every token is cut into blocks of a fixed
// size; Sec. 4.1: block size 256).  The hidden vector of one token is its H heads of D elements
// side by side, h-major; a block is `blk_hidden` consecutive elements of it, a multiple of D, so
// it covers blk_hidden / D whole heads.  Each block is quantized on its own exactly like any
// other block (oracle_quantize_block).  The cache keeps its per-head layout: codes uint8
// [B, H, cap_tokens, D*k/8] and ONE scale per token-head, fp16 bits [B, H, cap_tokens, 1] -- the
// block's scale written once for every head the block covers -- so that dequantization and
// attention read it as a cache of block size D.
//   src  fp16 bits, element (b,h,t,d) at b*sb + h*sh + t*ss + d  (token-major [B,S,H*D]: sh = D, ss = H*D)
// Returns 0, or -1 on a bad argument.
int oracle_quantize_kv_hidden(const uint16_t* src, int64_t sb, int64_t sh, int64_t ss,
                              int B, int H, int D, int64_t n_tokens,
                              int k, int blk_hidden, const float* levels32,
                              int64_t cap_tokens, int64_t dst_off,
                              uint8_t* codes, uint16_t* scales, int n_threads) {
  if (k < 1 || k > 8 || (D * k) % 8 != 0) return -1;
  if (blk_hidden < D || blk_hidden % D != 0 || ((int64_t)H * D) % blk_hidden != 0) return -1;
  if (dst_off < 0 || n_tokens < 0 || dst_off + n_tokens > cap_tokens) return -1;
  const int heads_per_block = blk_hidden / D;
  const int blocks_per_token = H / heads_per_block;
  const int64_t row_bytes = (int64_t)D * k / 8;
  run_parallel((int64_t)B * n_tokens, n_threads, [&](int64_t bt) {
    const int64_t b = bt / n_tokens, t = bt % n_tokens;
    std::vector<uint16_t> x((size_t)blk_hidden);
    std::vector<uint8_t> c((size_t)blk_hidden);
    for (int j = 0; j < blocks_per_token; ++j) {
      // gather the block: heads j*heads_per_block .. +heads_per_block-1 of this token
      for (int g = 0; g < heads_per_block; ++g) {
        const int h = j * heads_per_block + g;
        const uint16_t* row = src + b * sb + (int64_t)h * sh + t * ss;
        for (int d = 0; d < D; ++d) x[(size_t)g * D + d] = row[d];
      }
      uint16_t scale = 0;
      oracle_quantize_block(x.data(), blk_hidden, k, levels32, c.data(), &scale);
      for (int g = 0; g < heads_per_block; ++g) {
        const int h = j * heads_per_block + g;
        const int64_t row = ((int64_t)b * H + h) * cap_tokens + dst_off + t;
        oracle_pack_bits(c.data() + (size_t)g * D, D, k, codes + row * row_bytes);
        scales[row] = scale;
      }
    }
  });
  return 0;
}

// Dequantize tokens [off, off+n_tokens) of a cache to fp16 (Fig. 5 caption; Sec. 3.2
// X' = dequantize(I)):  out = fp16_rne( fl32( level[code] * float(scale) ) ).
//   dst fp16 bits, logical [B, H, n_tokens, D], strides sb, sh, ss.
int oracle_dequantize_kv(const uint8_t* codes, const uint16_t* scales,
                         int B, int H, int D, int k, int blk, const float* levels32,
                         int64_t cap_tokens, int64_t off, int64_t n_tokens,
                         uint16_t* dst, int64_t sb, int64_t sh, int64_t ss, int n_threads) {
  if (k < 1 || k > 8 || blk < 1 || D % blk != 0 || (D * k) % 8 != 0) return -1;
  if (off < 0 || n_tokens < 0 || off + n_tokens > cap_tokens) return -1;
  const int nb = D / blk;
  const int64_t row_bytes = (int64_t)D * k / 8;
  run_parallel((int64_t)B * H, n_threads, [&](int64_t bh) {
    const int b = (int)(bh / H), h = (int)(bh % H);
    std::vector<uint8_t> row_codes(D);
    for (int64_t t = 0; t < n_tokens; ++t) {
      const int64_t row = bh * cap_tokens + off + t;
      oracle_unpack_bits(codes + row * row_bytes, D, k, row_codes.data());
      uint16_t* y = dst + b * sb + h * sh + t * ss;
      for (int d = 0; d < D; ++d) {
        const float s32 = half_bits_to_float(scales[row * nb + d / blk]);
        const float prod = levels32[row_codes[d]] * s32;   // one fp32 rounding
        y[d] = float_to_half_bits_rne(prod);
      }
    }
  });
  return 0;
}

// Plain softmax attention of one query row in fp64 (Sec. 3.2 decoding phase:
// A = Softmax(t_Q X_K'^T), t_O = A X_V'), with an explicit score factor sigma:
//   z_t = sigma * sum_d q_d K[t,d];  out_d = sum_t exp(z_t - max z) V[t,d] / sum_t exp(z_t - max z)
//   q [D], K [S, D], V [S, D], out [D]
void oracle_attention_f64(const double* q, const double* K, const double* V,
                          int64_t S, int D, double sigma, double* out) {
  std::vector<double> z((size_t)S);
  double zmax = -INFINITY;
  for (int64_t t = 0; t < S; ++t) {
    double dot = 0.0;
    for (int d = 0; d < D; ++d) dot += q[d] * K[t * D + d];
    z[(size_t)t] = sigma * dot;
    if (z[(size_t)t] > zmax) zmax = z[(size_t)t];
  }
  double denom = 0.0;
  for (int d = 0; d < D; ++d) out[d] = 0.0;
  for (int64_t t = 0; t < S; ++t) {
    const double p = std::exp(z[(size_t)t] - zmax);
    denom += p;
    for (int d = 0; d < D; ++d) out[d] += p * V[t * D + d];
  }
  for (int d = 0; d < D; ++d) out[d] /= denom;
}

// Exact (unrounded) dequantized values of one (batch, head) slab in fp64:
//   X[t, d] = double(level32[code]) * double(scale)   -- a 24-bit by 11-bit product, exact.
void oracle_dequantize_slab_f64(const uint8_t* codes, const uint16_t* scales,
                                int D, int k, int blk, const float* levels32,
                                int64_t n_tokens, double* X) {
  const int nb = D / blk;
  const int64_t row_bytes = (int64_t)D * k / 8;
  std::vector<uint8_t> row_codes(D);
  for (int64_t t = 0; t < n_tokens; ++t) {
    oracle_unpack_bits(codes + t * row_bytes, D, k, row_codes.data());
    for (int d = 0; d < D; ++d) {
      const double s = (double)half_bits_to_float(scales[t * nb + d / blk]);
      X[t * D + d] = (double)levels32[row_codes[d]] * s;
    }
  }
}

// Decode attention for one new query per (batch, head) over the first seq_len cached
// tokens, the token appended this step included (Sec. 3.2: append, then dequantize the
// whole cache, then attend).  fp64 attention over the exact dequantized values.
//   q        fp16 bits [B, H, D] contiguous
//   k_codes, v_codes uint8 [B, H, cap_tokens, D*k/8];  k_scales, v_scales fp16 [B, H, cap_tokens, D/blk]
//   out      double [B, H, D]
int oracle_decode_attention(const uint16_t* q,
                            const uint8_t* k_codes, const uint16_t* k_scales,
                            const uint8_t* v_codes, const uint16_t* v_scales,
                            int B, int H, int D, int k, int blk, const float* levels32,
                            int64_t cap_tokens, int64_t seq_len, float softmax_scale,
                            double* out, int n_threads) {
  if (k < 1 || k > 8 || blk < 1 || D % blk != 0 || (D * k) % 8 != 0) return -1;
  if (seq_len < 1 || seq_len > cap_tokens) return -1;
  const int nb = D / blk;
  const int64_t row_bytes = (int64_t)D * k / 8;
  run_parallel((int64_t)B * H, n_threads, [&](int64_t bh) {
    std::vector<double> qd(D), Kx((size_t)seq_len * D), Vx((size_t)seq_len * D);
    for (int d = 0; d < D; ++d) qd[d] = (double)half_bits_to_float(q[bh * D + d]);
    oracle_dequantize_slab_f64(k_codes + bh * cap_tokens * row_bytes, k_scales + bh * cap_tokens * nb,
                               D, k, blk, levels32, seq_len, Kx.data());
    oracle_dequantize_slab_f64(v_codes + bh * cap_tokens * row_bytes, v_scales + bh * cap_tokens * nb,
                               D, k, blk, levels32, seq_len, Vx.data());
    oracle_attention_f64(qd.data(), Kx.data(), Vx.data(), seq_len, D, (double)softmax_scale,
                         out + bh * D);
  });
  return 0;
}

// Decode attention for q_len new queries per (batch, head) (several tokens appended in one step:
// Sec. 1, the cache is append-only and new keys/values go to its end; Sec. 3.2 decoding-phase
// equations applied to each new token in turn).  The queries belong to the LAST q_len tokens of
// the first seq_len cached tokens, so query i sees what a one-token step at that position would:
// tokens [0, seq_len - q_len + 1 + i).  fp64 attention over the exact dequantized values.
//   q    fp16 bits [B, H, q_len, D] contiguous;  out double [B, H, q_len, D];  caches as above
int oracle_decode_attention_multi(const uint16_t* q,
                                  const uint8_t* k_codes, const uint16_t* k_scales,
                                  const uint8_t* v_codes, const uint16_t* v_scales,
                                  int B, int H, int D, int k, int blk, const float* levels32,
                                  int64_t cap_tokens, int64_t seq_len, int q_len, float softmax_scale,
                                  double* out, int n_threads) {
  if (k < 1 || k > 8 || blk < 1 || D % blk != 0 || (D * k) % 8 != 0) return -1;
  if (q_len < 1 || seq_len < q_len || seq_len > cap_tokens) return -1;
  const int nb = D / blk;
  const int64_t row_bytes = (int64_t)D * k / 8;
  run_parallel((int64_t)B * H, n_threads, [&](int64_t bh) {
    std::vector<double> qd(D), Kx((size_t)seq_len * D), Vx((size_t)seq_len * D);
    oracle_dequantize_slab_f64(k_codes + bh * cap_tokens * row_bytes, k_scales + bh * cap_tokens * nb,
                               D, k, blk, levels32, seq_len, Kx.data());
    oracle_dequantize_slab_f64(v_codes + bh * cap_tokens * row_bytes, v_scales + bh * cap_tokens * nb,
                               D, k, blk, levels32, seq_len, Vx.data());
    for (int i = 0; i < q_len; ++i) {
      const int64_t visible = seq_len - q_len + 1 + i;
      for (int d = 0; d < D; ++d) qd[d] = (double)half_bits_to_float(q[(bh * q_len + i) * D + d]);
      oracle_attention_f64(qd.data(), Kx.data(), Vx.data(), visible, D, (double)softmax_scale,
                           out + (bh * q_len + i) * D);
    }
  });
  return 0;
}

}  // extern "C"
