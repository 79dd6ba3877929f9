// Host side of libnqkv: the C ABI declared in include/nqkv.h -- argument validation, the
// quantile table, split planning and kernel dispatch.  Every check runs before any HIP call,
// so error paths are testable on a machine without a GPU.
#include "../../include/nqkv.h"
#include "nqkv_internal.h"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <vector>

namespace nqkv {

// Entry c = { the one threshold that may lie in cell c widened by the margin (2.0 when there is
// none: never exceeded, since |x| <= s), number of thresholds certainly below the cell }.
// Returns false when some widened cell would hold two thresholds or the table leaves [-1, 1]:
// such tables take the threshold scan.
bool build_cell_table(const float* levels, int k, uint32_t* thr_bits, uint32_t* below) {
  const int L = 1 << k;
  if (!(levels[0] >= -1.0f && levels[L - 1] <= 1.0f)) return false;
  for (int c = 0; c < code_search::kCells; ++c) {
    const float lo = (float)c - code_search::kCellMargin;
    const float hi = (float)c + 1.0f + code_search::kCellMargin;
    int inside = 0;
    uint32_t n_below = 0;
    float cand = 2.0f;
    for (int j = 1; j < L; ++j) {
      const float t = (levels[j - 1] + levels[j]) * 0.5f;
      const float tau = t * code_search::kCellScale + code_search::kCellBias;
      if (tau < lo) ++n_below;
      if (tau >= lo && tau <= hi) { cand = t; ++inside; }
    }
    if (inside > 1) return false;
    std::memcpy(&thr_bits[c], &cand, 4);
    below[c] = n_below;
  }
  return true;
}

}  // namespace nqkv

namespace {

using namespace nqkv;

constexpr int64_t kLongItemTokens = 4096;   // see fill_decode_common
constexpr int64_t kMaxSequences = (int64_t)1 << 24;      // (batch row, head) pairs of one cache
constexpr int64_t kMaxCutSequences = 65535;              // ... of a cache whose sequences are cut: one ticket counter each

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const nqkv_cache_desc* d) {
  if (!d) return NQKV_EINVAL;
  if (d->B < 1 || d->H < 1 || d->cap_tokens < 1) return NQKV_EINVAL;
  if (d->flags & ~(int32_t)(NQKV_FLAG_SCAN_QUANTIZER | NQKV_FLAG_WORKGROUP_PER_ITEM)) return NQKV_EINVAL;
  if (d->D < 1 || d->k < 1 || d->block < 1) return NQKV_EINVAL;
  if (d->k != 2 && d->k != 3 && d->k != 4) return NQKV_EUNSUPPORTED;
  if (d->D != 64 && d->D != 128) return NQKV_EUNSUPPORTED;
  if (d->block != 64 && d->block != 128) return NQKV_EUNSUPPORTED;
  if (d->D % d->block != 0) return NQKV_EINVAL;
  // 16-bit grid dimensions (heads in y, batch rows of one or two tensors in z) and 32-bit item counts
  if (d->H > 65535 || d->B > 32767 || (int64_t)d->B * d->H > kMaxSequences) return NQKV_EUNSUPPORTED;
  if (d->cap_tokens > ((int64_t)1 << 31) - 1) return NQKV_EUNSUPPORTED;
  return NQKV_OK;
}

int check_levels(const float* levels, int k, LevelTable* out) {
  if (!levels) return NQKV_EINVAL;
  const int L = 1 << k;
  for (int i = 0; i < L; ++i) {
    if (!std::isfinite(levels[i])) return NQKV_EINVAL;
    if (i > 0 && !(levels[i] > levels[i - 1])) return NQKV_EINVAL;
  }
  std::memset(out, 0, sizeof(*out));
  for (int i = 0; i < L; ++i) out->v[i] = levels[i];
  return NQKV_OK;
}

int check_strided(const nqkv_cache_desc* d, int64_t sb, int64_t sh, int64_t st, int64_t n_tokens) {
  if (sb < 0 || sh < 0 || st < 0) return NQKV_EINVAL;
  if ((sb % 8) || (sh % 8) || (st % 8)) return NQKV_EINVAL;   // every row 16-byte aligned
  if (n_tokens > 1 && st < d->D) return NQKV_EINVAL;
  // offsets inside one (b,h) slab are formed in 32 bits (chunk index, byte offset)
  if (n_tokens * (d->D / 8) >= ((int64_t)1 << 31) - 4096) return NQKV_EUNSUPPORTED;
  if (n_tokens > 0 && ((n_tokens - 1) * st + d->D) * 2 >= ((int64_t)1 << 31)) return NQKV_EUNSUPPORTED;
  return NQKV_OK;
}

int check_range(const nqkv_cache_desc* d, int64_t off, int64_t n) {
  if (n < 0 || off < 0 || off > d->cap_tokens || n > d->cap_tokens - off) return NQKV_EINVAL;
  return NQKV_OK;
}

// Upper-tail normal quantile by Newton's method on Q(x) = erfc(x / sqrt 2) / 2, started at 0.
// Q is convex and decreasing on x >= 0, so the iterates climb monotonically to the root.
double normal_upper_quantile(double tail) {
  const double inv_sqrt2 = 0.70710678118654752440;
  const double inv_sqrt_2pi = 0.39894228040143267794;
  double x = 0.0;
  for (int it = 0; it < 200; ++it) {
    const double q = 0.5 * std::erfc(x * inv_sqrt2);
    const double pdf = inv_sqrt_2pi * std::exp(-0.5 * x * x);
    const double step = (q - tail) / pdf;
    x += step;
    if (std::fabs(step) <= 1e-17 * (1.0 + x)) break;
  }
  return x;
}

// ---- fp16 look-up table for the attention kernel ---------------------------------------
// binary32 -> binary16 bits, round to nearest even (host rounding mode is the default one).
uint16_t f32_to_f16_bits(float x) {
  const uint16_t sign = std::signbit(x) ? 0x8000u : 0u;
  const double a = std::fabs((double)x);
  if (a == 0.0) return sign;
  int e2;
  const double m = std::frexp(a, &e2);      // a = m * 2^e2, m in [0.5, 1)
  int E = e2 - 1;                           // a = (2m) * 2^E, 2m in [1, 2)
  if (E < -14) {                            // subnormal half: units of 2^-24
    const double qd = std::nearbyint(std::ldexp(a, 24));
    return (uint16_t)(sign | (uint16_t)qd); // 1024 encodes the smallest normal, as it should
  }
  double qd = std::nearbyint(std::ldexp(m, 11));   // 2m * 1024 in [1024, 2048]
  if (qd >= 2048.0) { qd = 1024.0; ++E; }
  if (E > 15) return (uint16_t)(sign | 0x7c00u);
  return (uint16_t)(sign | ((uint32_t)(E + 15) << 10) | ((uint32_t)qd - 1024u));
}

double f16_bits_to_f64(uint16_t h) {
  const int e = (h >> 10) & 31, m = h & 1023;
  const double v = e ? std::ldexp(1024.0 + m, e - 25) : std::ldexp((double)m, -24);
  return (h & 0x8000u) ? -v : v;
}

// Picks gamma (itself an fp16 number in [1/4, 8)) minimising the worst relative error of
// fp16(gamma * level[i]) over the table, and returns those fp16 entries.  The last result is
// remembered per thread, so repeated calls with one table cost a 64-byte compare.
struct LutChoice {
  int L = 0;
  float levels[kMaxLevels];
  uint16_t bits[kMaxLevels];
  float gamma = 1.0f;
};

const LutChoice& choose_lut_scale(const float* levels, int L) {
  static thread_local LutChoice memo;
  if (memo.L == L && std::memcmp(memo.levels, levels, sizeof(float) * L) == 0) return memo;
  double best_err = 1e30, best_gamma = 1.0;
  for (int E = -2; E <= 2; ++E) {
    for (int m = 0; m < 1024; ++m) {
      const double gamma = std::ldexp(1024.0 + m, E - 10);
      double worst = 0.0;
      for (int i = 0; i < L && worst < best_err; ++i) {
        const double exact = gamma * (double)levels[i];
        if (exact == 0.0) continue;
        const double got = f16_bits_to_f64(f32_to_f16_bits((float)exact));
        worst = std::fmax(worst, std::fabs(got - exact) / std::fabs(exact));
      }
      if (worst < best_err || (worst == best_err && std::fabs(gamma - 1.0) < std::fabs(best_gamma - 1.0))) {
        best_err = worst;
        best_gamma = gamma;
      }
    }
  }
  memo.L = L;
  std::memcpy(memo.levels, levels, sizeof(float) * L);
  memo.gamma = (float)best_gamma;
  for (int i = 0; i < L; ++i) memo.bits[i] = f32_to_f16_bits((float)(best_gamma * (double)levels[i]));
  return memo;
}

size_t workspace_need(const nqkv_cache_desc* d, int splits) {
  if (splits <= 1) return 0;
  return kTicketBytes + (size_t)d->B * d->H * splits * (d->D + 2) * sizeof(float);
}

// Persistent grid size: two eight-wave workgroups fit on a compute unit (64 KiB table each).
// The compute-unit count is asked of the current device once and remembered per device index
// (a constant of the hardware, not a setting: racing first calls store the same number).
int max_decode_workgroups() {
  constexpr int kMaxDevices = 64;
  static std::atomic<int> cus_of_device[kMaxDevices];
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 2 * 256;
  cus = cus_of_device[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cus_of_device[dev].store(cus, std::memory_order_relaxed);
  }
  return 2 * cus;
}

int plan_splits(const nqkv_cache_desc* d, int64_t seq_len, int num_splits, int* splits) {
  if (seq_len < 1 || seq_len > d->cap_tokens) return NQKV_EINVAL;
  if (num_splits < 0 || num_splits > 1024) return NQKV_EINVAL;
  if (num_splits > 0) {
    if ((int64_t)num_splits > seq_len) return NQKV_EINVAL;
    if (num_splits > 1 && (int64_t)d->B * d->H > kMaxCutSequences) return NQKV_EUNSUPPORTED;
    *splits = num_splits;
    return NQKV_OK;
  }
  // Every item (one piece of one (b,h) sequence) costs a few microseconds of set-up, merge and,
  // when a sequence is cut, publishing a partial result; measured on MI355X the best cut gives
  // about one item per compute unit when B*H alone does not, and no cut otherwise.  Never cut
  // below one trip of one wave.
  const int64_t bh = (int64_t)d->B * d->H;
  const int64_t target = 256;
  const int64_t trip = (int64_t)decode_chunk_tokens(d->D);
  int64_t want = target / bh;
  int64_t longest = seq_len / trip;
  if (want > longest) want = longest;
  if (want > 1024) want = 1024;
  if (want < 1) want = 1;
  *splits = (int)want;
  return NQKV_OK;
}

// Cut of a sequence for the several-queries kernel, in whole 32-token pieces.  One workgroup per
// piece, each building its own look-up table, so pieces are kept at one sweep of the eight waves
// or longer; measured on MI355X, one workgroup per compute unit is as fast as two (13.7 vs 14.5 us
// at B8 H32 D64 S2048, 39.5 vs 39.0 us at B1 H32 D128 S32768) and costs half the partial results.
int plan_multi(const nqkv_cache_desc* d, int64_t seq_len, int64_t max_tokens, int q_len, int num_splits, int* splits) {
  if (q_len < 1 || q_len > 16) return q_len < 1 ? NQKV_EINVAL : NQKV_EUNSUPPORTED;
  if (seq_len < q_len || seq_len > max_tokens || seq_len >= ((int64_t)1 << 31) - 64) return NQKV_EINVAL;
  if (num_splits < 0 || num_splits > 1024) return NQKV_EINVAL;
  const int64_t trips = (seq_len + decode_multi_trip_tokens() - 1) / decode_multi_trip_tokens();
  if (num_splits > 0) {
    if ((int64_t)num_splits > trips) return NQKV_EINVAL;
    if (num_splits > 1 && (int64_t)d->B * d->H > kMaxCutSequences) return NQKV_EUNSUPPORTED;
    *splits = num_splits;
    return NQKV_OK;
  }
  const int64_t bh = (int64_t)d->B * d->H;
  const int64_t target = (int64_t)max_decode_workgroups() / 2;
  int64_t want = target / bh;
  const int64_t longest = seq_len / decode_multi_item_tokens();
  if (want > longest) want = longest;
  if (want > 1024) want = 1024;
  if (want < 1) want = 1;
  *splits = (int)want;
  return NQKV_OK;
}

size_t multi_workspace_need(const nqkv_cache_desc* d, int q_len, int splits) {
  if (splits <= 1) return 0;
  return (size_t)d->B * d->H * splits * q_len * (d->D + 2) * sizeof(float);
}

}  // namespace

extern "C" {

const char* nqkv_strerror(int status) {
  switch (status) {
    case NQKV_OK: return "ok";
    case NQKV_EINVAL: return "invalid argument (null or misaligned pointer, size or range out of bounds)";
    case NQKV_EUNSUPPORTED: return "configuration not supported by the gfx950 kernels";
    case NQKV_EWORKSPACE: return "workspace too small";
    case NQKV_EHIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int nqkv_version(void) { return 100; }

int nqkv_build_codebook(int k, int variant, float* levels_out) {
  if (k < 1 || k > 8 || !levels_out) return NQKV_EINVAL;
  if (variant != 0 && variant != 1) return NQKV_EINVAL;
  const int L = 1 << k;
  double lev[256];
  if (variant == 0) {
    // level i = median of the i-th of L equal-probability slices of N(0,1), over the largest
    const double top = normal_upper_quantile(1.0 / (2.0 * L));
    const int half = L / 2;
    for (int m = 0; m < half; ++m) {          // m-th positive level, counted from the centre
      const double tail = (2.0 * (half - 1 - m) + 1.0) / (2.0 * L);
      const double v = (m == half - 1) ? 1.0 : normal_upper_quantile(tail) / top;
      lev[half + m] = v;
      lev[half - 1 - m] = -v;
    }
  } else {
    if (k < 2) return NQKV_EINVAL;
    const double delta = std::ldexp(1.0, -(k + 1));
    const int n_pos = L / 2, n_neg = L / 2 - 1;
    const double top = normal_upper_quantile(delta);
    lev[n_neg] = 0.0;
    for (int m = 1; m <= n_pos; ++m) {
      const double tail = 0.5 - m * (0.5 - delta) / n_pos;
      lev[n_neg + m] = (m == n_pos) ? 1.0 : normal_upper_quantile(tail) / top;
    }
    for (int m = 1; m <= n_neg; ++m) {
      const double tail = 0.5 - m * (0.5 - delta) / n_neg;
      lev[n_neg - m] = (m == n_neg) ? -1.0 : -normal_upper_quantile(tail) / top;
    }
  }
  for (int i = 0; i < L; ++i) levels_out[i] = (float)lev[i];
  return NQKV_OK;
}

// Shared by nqkv_quantize_kv_pair (offsets == nullptr) and its per-sequence-offset form, where
// dst_token_offset is the largest offset the array may hold.
static int quantize_pair_impl(const nqkv_cache_desc* desc, const float* levels,
                              const void* k_src, const void* v_src,
                              int64_t stride_b, int64_t stride_h, int64_t stride_t,
                              int64_t n_tokens, const int32_t* offsets, int64_t dst_token_offset,
                              void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                              void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  QuantParams p;
  std::memset(&p, 0, sizeof(p));
  if ((rc = check_levels(levels, desc->k, &p.levels))) return rc;
  if ((rc = check_range(desc, dst_token_offset, n_tokens))) return rc;
  if ((rc = check_strided(desc, stride_b, stride_h, stride_t, n_tokens))) return rc;
  if (n_tokens == 0) return NQKV_OK;           // nothing to do: pointers are not looked at
  const bool pair = v_src || v_codes || v_scales;
  if (!k_src || !k_codes || !k_scales || !aligned16(k_src) || !aligned16(k_codes) || !aligned16(k_scales))
    return NQKV_EINVAL;
  if (pair && (!v_src || !v_codes || !v_scales || !aligned16(v_src) || !aligned16(v_codes) || !aligned16(v_scales)))
    return NQKV_EINVAL;
  if (pair && (int64_t)desc->B * 2 > 65535) return NQKV_EUNSUPPORTED;
  p.t[0].src = static_cast<const uint16_t*>(k_src);
  p.t[0].codes = static_cast<uint8_t*>(k_codes);
  p.t[0].scales = static_cast<uint16_t*>(k_scales);
  p.t[1].src = static_cast<const uint16_t*>(v_src);
  p.t[1].codes = static_cast<uint8_t*>(v_codes);
  p.t[1].scales = static_cast<uint16_t*>(v_scales);
  p.n_tensors = pair ? 2 : 1;
  p.B = desc->B;
  p.H = desc->H;
  p.stride_b = stride_b;
  p.stride_h = stride_h;
  p.stride_t = stride_t;
  p.n_tokens = n_tokens;
  p.tok_off = dst_token_offset;
  p.tok_offs = offsets;
  p.max_off = (int)std::min<int64_t>(dst_token_offset, ((int64_t)1 << 31) - 1);
  p.cap_tokens = desc->cap_tokens;
  p.impl = (!(desc->flags & NQKV_FLAG_SCAN_QUANTIZER) && build_cell_table(levels, desc->k, p.cell_thr, p.cell_below)) ? 0 : 1;
  const hipError_t e = launch_quantize(p, desc->D, desc->k, desc->block, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_quantize_kv_pair(const nqkv_cache_desc* desc, const float* levels,
                          const void* k_src, const void* v_src,
                          int64_t stride_b, int64_t stride_h, int64_t stride_t,
                          int64_t n_tokens, int64_t dst_token_offset,
                          void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                          void* hip_stream) {
  return quantize_pair_impl(desc, levels, k_src, v_src, stride_b, stride_h, stride_t, n_tokens, nullptr, dst_token_offset,
                            k_codes, k_scales, v_codes, v_scales, hip_stream);
}

int nqkv_quantize_kv_pair_varlen(const nqkv_cache_desc* desc, const float* levels,
                                 const void* k_src, const void* v_src,
                                 int64_t stride_b, int64_t stride_h, int64_t stride_t,
                                 int64_t n_tokens, const int32_t* dst_token_offsets, int64_t max_offset,
                                 void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                                 void* hip_stream) {
  if (!dst_token_offsets || (reinterpret_cast<uintptr_t>(dst_token_offsets) & 3u)) return NQKV_EINVAL;
  if (max_offset > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
  return quantize_pair_impl(desc, levels, k_src, v_src, stride_b, stride_h, stride_t, n_tokens, dst_token_offsets, max_offset,
                            k_codes, k_scales, v_codes, v_scales, hip_stream);
}

int nqkv_quantize_kv(const nqkv_cache_desc* desc, const float* levels,
                     const void* src, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                     int64_t n_tokens, int64_t dst_token_offset,
                     void* codes, void* scales, void* hip_stream) {
  return nqkv_quantize_kv_pair(desc, levels, src, nullptr, stride_b, stride_h, stride_t, n_tokens,
                               dst_token_offset, codes, scales, nullptr, nullptr, hip_stream);
}

int nqkv_quantize_kv_hidden(const nqkv_cache_desc* desc, const float* levels,
                            const void* k_src, const void* v_src,
                            int64_t stride_b, int64_t stride_h, int64_t stride_t,
                            int64_t n_tokens, int64_t dst_token_offset, int block_hidden,
                            void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                            void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (desc->block != desc->D) return NQKV_EINVAL;                 // the cache holds one scale per token-head
  if (block_hidden == desc->D)                                      // a block is one head: the ordinary quantizer
    return nqkv_quantize_kv_pair(desc, levels, k_src, v_src, stride_b, stride_h, stride_t, n_tokens,
                                 dst_token_offset, k_codes, k_scales, v_codes, v_scales, hip_stream);
  if (block_hidden != 128 && block_hidden != 256) return NQKV_EUNSUPPORTED;
  if (block_hidden % desc->D != 0 || ((int64_t)desc->H * desc->D) % block_hidden != 0) return NQKV_EINVAL;
  QuantParams p;
  std::memset(&p, 0, sizeof(p));
  if ((rc = check_levels(levels, desc->k, &p.levels))) return rc;
  if ((rc = check_range(desc, dst_token_offset, n_tokens))) return rc;
  if ((rc = check_strided(desc, stride_b, stride_h, stride_t, n_tokens))) return rc;
  if (desc->H > 1 && stride_h < desc->D) return NQKV_EINVAL;
  if (n_tokens == 0) return NQKV_OK;
  // offsets inside one batch row are formed in 32 bits: source extent, cache extent, chunk count
  const int64_t src_extent = (((int64_t)desc->H - 1) * stride_h + (n_tokens - 1) * stride_t + desc->D) * 2;
  const int64_t cache_extent = (int64_t)desc->H * desc->cap_tokens * (desc->D * desc->k / 8);
  const int64_t chunks = n_tokens * desc->H * (desc->D / 8);
  if (src_extent >= ((int64_t)1 << 31) || cache_extent >= ((int64_t)1 << 31) || chunks >= ((int64_t)1 << 31) - 8192)
    return NQKV_EUNSUPPORTED;
  const bool pair = v_src || v_codes || v_scales;
  if (!k_src || !k_codes || !k_scales || !aligned16(k_src) || !aligned16(k_codes) || !aligned16(k_scales))
    return NQKV_EINVAL;
  if (pair && (!v_src || !v_codes || !v_scales || !aligned16(v_src) || !aligned16(v_codes) || !aligned16(v_scales)))
    return NQKV_EINVAL;
  if ((n_tokens + 31) / 32 > 65535 || (int64_t)desc->B * 2 > 65535) return NQKV_EUNSUPPORTED;   // 16-bit grid dimensions
  p.t[0].src = static_cast<const uint16_t*>(k_src);
  p.t[0].codes = static_cast<uint8_t*>(k_codes);
  p.t[0].scales = static_cast<uint16_t*>(k_scales);
  p.t[1].src = static_cast<const uint16_t*>(v_src);
  p.t[1].codes = static_cast<uint8_t*>(v_codes);
  p.t[1].scales = static_cast<uint16_t*>(v_scales);
  p.n_tensors = pair ? 2 : 1;
  p.B = desc->B;
  p.H = desc->H;
  p.stride_b = stride_b;
  p.stride_h = stride_h;
  p.stride_t = stride_t;
  p.n_tokens = n_tokens;
  p.tok_off = dst_token_offset;
  p.cap_tokens = desc->cap_tokens;
  p.impl = (!(desc->flags & NQKV_FLAG_SCAN_QUANTIZER) && build_cell_table(levels, desc->k, p.cell_thr, p.cell_below)) ? 0 : 1;
  const hipError_t e = launch_quantize_hidden(p, desc->D, desc->k, block_hidden, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_dequantize_kv(const nqkv_cache_desc* desc, const float* levels,
                       const void* codes, const void* scales,
                       int64_t token_offset, int64_t n_tokens,
                       void* dst, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                       void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  QuantParams p;
  std::memset(&p, 0, sizeof(p));
  if ((rc = check_levels(levels, desc->k, &p.levels))) return rc;
  if ((rc = check_range(desc, token_offset, n_tokens))) return rc;
  if ((rc = check_strided(desc, stride_b, stride_h, stride_t, n_tokens))) return rc;
  if (n_tokens == 0) return NQKV_OK;           // nothing to do: pointers are not looked at
  if (!codes || !scales || !dst || !aligned16(codes) || !aligned16(scales) || !aligned16(dst)) return NQKV_EINVAL;
  p.t[0].codes = const_cast<uint8_t*>(static_cast<const uint8_t*>(codes));
  p.t[0].scales = const_cast<uint16_t*>(static_cast<const uint16_t*>(scales));
  p.t[0].dst = static_cast<uint16_t*>(dst);
  p.n_tensors = 1;
  p.B = desc->B;
  p.H = desc->H;
  p.stride_b = stride_b;
  p.stride_h = stride_h;
  p.stride_t = stride_t;
  p.n_tokens = n_tokens;
  p.tok_off = token_offset;
  p.cap_tokens = desc->cap_tokens;
  const hipError_t e = launch_dequantize(p, desc->D, desc->k, desc->block, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_decode_workspace_bytes(const nqkv_cache_desc* desc, int64_t seq_len, int num_splits,
                                size_t* bytes_out, int* splits_out) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!bytes_out) return NQKV_EINVAL;
  int splits = 1;
  if ((rc = plan_splits(desc, seq_len, num_splits, &splits))) return rc;
  *bytes_out = workspace_need(desc, splits);
  if (splits_out) *splits_out = splits;
  return NQKV_OK;
}

int nqkv_decode_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
  if (workspace_bytes < kTicketBytes) return NQKV_EWORKSPACE;
  const hipError_t e = launch_clear_words(static_cast<uint32_t*>(workspace), (int)(kTicketBytes / sizeof(uint32_t)),
                                          static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_decode_workspace_check(const void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
  if (workspace_bytes < kTicketBytes) return NQKV_EWORKSPACE;
  std::vector<uint32_t> words(kTicketBytes / sizeof(uint32_t));
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (hipMemcpyAsync(words.data(), workspace, kTicketBytes, hipMemcpyDeviceToHost, stream) != hipSuccess) return NQKV_EHIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return NQKV_EHIP;
  for (uint32_t w : words) {
    if (w != 0) return NQKV_EWORKSPACE;       // a counter left armed, or the status word a kernel set
  }
  return NQKV_OK;
}

// Ragged batch on a grid of one workgroup per item, more items than can be resident: dispatch
// the long sequences first (the kernel ranks the lengths itself; it handles up to 64 of them).
// Measured at B16 H56 S<=16384, lengths spread over [S/8, S] in random batch order: 211 -> 175 us.
static int longest_first_pays(const DecodeParams& p, const int32_t* lens, int B) {
  return lens && B >= 2 && B <= 64 && p.max_workgroups >= p.n_items && p.n_items > max_decode_workgroups();
}

// The part of DecodeParams every decode entry point fills the same way.
static void fill_decode_common(DecodeParams* p, const nqkv_cache_desc* desc, const LevelTable& checked,
                               const void* q, const void* k_new, const void* v_new,
                               int64_t new_stride_b, int64_t new_stride_h,
                               const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                               float softmax_scale, void* out, void* workspace, int items_per_sequence,
                               int64_t item_tokens) {
  p->q = static_cast<const uint16_t*>(q);
  p->k_codes = static_cast<const uint8_t*>(k_codes);
  p->k_scales = static_cast<const uint16_t*>(k_scales);
  p->v_codes = static_cast<const uint8_t*>(v_codes);
  p->v_scales = static_cast<const uint16_t*>(v_scales);
  p->out = static_cast<uint16_t*>(out);
  p->tickets = static_cast<uint32_t*>(workspace);
  p->partials = reinterpret_cast<float*>(static_cast<char*>(workspace) + kTicketBytes);
  p->n_items = desc->B * desc->H * items_per_sequence;
  p->splits = items_per_sequence;
  // Grid: short items share a persistent grid of two workgroups per compute unit (one table build
  // serves several items); long items get a workgroup each, which the dispatcher hands out as
  // earlier ones finish -- with more items than resident workgroups that balances better than a
  // fixed deal (measured: 896 items of 16384 tokens 332 -> 319 us; 8192 items of 128 tokens 52 -> 65 us).
  p->max_workgroups = ((desc->flags & NQKV_FLAG_WORKGROUP_PER_ITEM) || item_tokens >= kLongItemTokens)
                          ? p->n_items : max_decode_workgroups();
  p->n_seqs = desc->B;
  p->cap_tokens = desc->cap_tokens;
  const LutChoice& lut = choose_lut_scale(checked.v, 1 << desc->k);
  std::memcpy(p->lut_levels, lut.bits, sizeof(uint16_t) * (1 << desc->k));
  p->inv_gamma = 1.0f / lut.gamma;
  p->scale_log2e = (float)((double)softmax_scale * 1.44269504088896340736 / (double)lut.gamma);
  p->k_new = static_cast<const uint16_t*>(k_new);
  p->v_new = static_cast<const uint16_t*>(v_new);
  p->new_stride_b = new_stride_b;
  p->new_stride_h = new_stride_h;
  p->H = desc->H;
}

// Shared by nqkv_decode_attention (k_new == nullptr) and nqkv_decode_step.
static int decode_impl(const nqkv_cache_desc* desc, const float* levels, const void* q,
                       const void* k_new, const void* v_new, int64_t new_stride_b, int64_t new_stride_h,
                       const int32_t* lens,
                       const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                       int64_t seq_len, float softmax_scale, void* out,
                       void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream,
                       bool static_workspace = false) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const bool fuse = k_new != nullptr;
  DecodeParams p;
  std::memset(&p, 0, sizeof(p));
  LevelTable checked;
  if ((rc = check_levels(levels, desc->k, &checked))) return rc;
  if (seq_len < 1 || seq_len > desc->cap_tokens) return NQKV_EINVAL;
  // the fused step streams the seq_len - 1 tokens already cached and takes the last one from
  // k_new / v_new
  const int64_t n_cached = fuse ? seq_len - 1 : seq_len;
  int splits = 1;
  if (n_cached >= 1) {
    if ((rc = plan_splits(desc, n_cached, num_splits, &splits))) return rc;
  } else if (num_splits < 0 || num_splits > 1) {
    return NQKV_EINVAL;
  }
  if (!std::isfinite(softmax_scale)) return NQKV_EINVAL;
  const void* ptrs[] = {q, k_codes, k_scales, v_codes, v_scales, out};
  for (const void* ptr : ptrs) {
    if (!ptr || !aligned16(ptr)) return NQKV_EINVAL;
  }
  if (fuse) {
    if (!v_new || !aligned16(k_new) || !aligned16(v_new)) return NQKV_EINVAL;
    if (new_stride_b < 0 || new_stride_h < 0 || (new_stride_b % 8) || (new_stride_h % 8)) return NQKV_EINVAL;
  }
  const size_t need = workspace_need(desc, splits);
  if (static_workspace) {
    if (need > kStaticScratchBytes) return NQKV_EWORKSPACE;       // refused before anything touches the GPU
  } else if (need > 0) {
    if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
    if (workspace_bytes < need) return NQKV_EWORKSPACE;
  }
  // one item's byte range is addressed with 32-bit offsets
  if ((n_cached / splits + 1) * (int64_t)(desc->D * desc->k / 8) >= ((int64_t)1 << 31)) return NQKV_EUNSUPPORTED;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (static_workspace && need > 0) {
    // the library's own array on the current device, by its device address
    if (static_scratch(&workspace) != hipSuccess) return NQKV_EHIP;
  }
  if (fuse && !build_cell_table(levels, desc->k, p.cell_thr, p.cell_below)) {
    // a table the in-kernel code search cannot take: append with the quantizer, then attend
    if (lens) return NQKV_EUNSUPPORTED;        // (the quantizer appends at one row for the whole batch)
    // That attention runs over seq_len tokens, one more than the step was planned for above, and
    // may cut the sequence into one more piece: everything that call checks is checked here
    // first, so that an error still means nothing was launched and the cache is untouched.
    int splits_att = 1;
    if ((rc = plan_splits(desc, seq_len, num_splits, &splits_att))) return rc;
    const size_t need_att = workspace_need(desc, splits_att);
    if (need_att > 0) {
      if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
      if (workspace_bytes < need_att) return NQKV_EWORKSPACE;
    }
    if ((seq_len / splits_att + 1) * (int64_t)(desc->D * desc->k / 8) >= ((int64_t)1 << 31)) return NQKV_EUNSUPPORTED;
    rc = nqkv_quantize_kv_pair(desc, levels, k_new, v_new, new_stride_b, new_stride_h, desc->D, 1, seq_len - 1,
                               const_cast<void*>(k_codes), const_cast<void*>(k_scales),
                               const_cast<void*>(v_codes), const_cast<void*>(v_scales), hip_stream);
    if (rc) return rc;
    return decode_impl(desc, levels, q, nullptr, nullptr, 0, 0, nullptr, k_codes, k_scales, v_codes, v_scales, seq_len,
                       softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
  }
  fill_decode_common(&p, desc, checked, q, k_new, v_new, new_stride_b, new_stride_h, k_codes, k_scales, v_codes, v_scales,
                     softmax_scale, out, workspace, splits, n_cached / splits);
  p.split_base = (int)(n_cached / splits);
  p.split_rem = (int)(n_cached % splits);
  p.pos = seq_len - 1;
  p.seq_lens = lens;                                    // fused: lens[b] = cached rows = the new token's row
  p.max_len = (int)n_cached;
  p.longest_first = longest_first_pays(p, lens, desc->B);
  // The array keeps whatever the last call on this GPU left in it: clear the counters this call uses.
  if (static_workspace && splits > 1 && launch_clear_words(p.tickets, desc->B * desc->H, stream) != hipSuccess) return NQKV_EHIP;
  const hipError_t e = launch_decode_attention(p, desc->D, desc->k, desc->block, fuse, stream);
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_decode_attention(const nqkv_cache_desc* desc, const float* levels,
                          const void* q,
                          const void* k_codes, const void* k_scales,
                          const void* v_codes, const void* v_scales,
                          int64_t seq_len, float softmax_scale, void* out,
                          void* workspace, size_t workspace_bytes, int num_splits,
                          void* hip_stream) {
  return decode_impl(desc, levels, q, nullptr, nullptr, 0, 0, nullptr, k_codes, k_scales, v_codes, v_scales, seq_len,
                     softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
}

int nqkv_decode_attention_static(const nqkv_cache_desc* desc, const float* levels,
                                 const void* q,
                                 const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales,
                                 int64_t seq_len, float softmax_scale, void* out,
                                 int num_splits, void* hip_stream) {
  static_assert(NQKV_STATIC_SCRATCH_BYTES == kStaticScratchBytes, "header and library disagree on the array size");
  return decode_impl(desc, levels, q, nullptr, nullptr, 0, 0, nullptr, k_codes, k_scales, v_codes, v_scales, seq_len,
                     softmax_scale, out, nullptr, 0, num_splits, hip_stream, true);
}

int nqkv_decode_step(const nqkv_cache_desc* desc, const float* levels,
                     const void* q, const void* k_new, const void* v_new,
                     int64_t new_stride_b, int64_t new_stride_h,
                     void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                     int64_t pos, float softmax_scale, void* out,
                     void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  if (!k_new) return NQKV_EINVAL;
  if (pos < 0 || (desc && pos >= desc->cap_tokens)) return NQKV_EINVAL;
  return decode_impl(desc, levels, q, k_new, v_new, new_stride_b, new_stride_h, nullptr, k_codes, k_scales, v_codes,
                     v_scales, pos + 1, softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
}

int nqkv_decode_attention_varlen(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                 const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales,
                                 const int32_t* seq_lens, int64_t max_seq_len, float softmax_scale, void* out,
                                 void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  if (!seq_lens || (reinterpret_cast<uintptr_t>(seq_lens) & 3u)) return NQKV_EINVAL;
  return decode_impl(desc, levels, q, nullptr, nullptr, 0, 0, seq_lens, k_codes, k_scales, v_codes, v_scales,
                     max_seq_len, softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
}

int nqkv_decode_step_varlen(const nqkv_cache_desc* desc, const float* levels,
                            const void* q, const void* k_new, const void* v_new,
                            int64_t new_stride_b, int64_t new_stride_h,
                            void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                            const int32_t* pos, int64_t max_pos, float softmax_scale, void* out,
                            void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  if (!k_new) return NQKV_EINVAL;
  if (!pos || (reinterpret_cast<uintptr_t>(pos) & 3u)) return NQKV_EINVAL;
  if (max_pos < 0 || (desc && max_pos >= desc->cap_tokens)) return NQKV_EINVAL;
  return decode_impl(desc, levels, q, k_new, v_new, new_stride_b, new_stride_h, pos, k_codes, k_scales, v_codes,
                     v_scales, max_pos + 1, softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
}

// Paged cache: the pool holds num_pages pages of [H][P] rows (P = desc->cap_tokens tokens per
// page, a power of two >= 128 so that no wave trip straddles two pages); logical page j of
// sequence b is page block_table[b * table_stride + j].  A sequence is cut into work items of
// whole pages, as many items as the contiguous calls would use splits.
struct PagedPlan {
  int page_shift;
  int items;             // work items per sequence
  int64_t item_tokens;   // tokens per item: a multiple of the page size
};

static int plan_paged(const nqkv_cache_desc* desc, int64_t n_cached, PagedPlan* plan) {
  const int64_t P = desc->cap_tokens;
  if (P < 128 || (P & (P - 1)) != 0 || P > ((int64_t)1 << 24)) return NQKV_EUNSUPPORTED;
  int shift = 0;
  while (((int64_t)1 << shift) < P) ++shift;
  const int64_t pages = n_cached <= 0 ? 1 : (n_cached + P - 1) / P;
  const int64_t bh = (int64_t)desc->B * desc->H;
  const int64_t target = 256;
  int64_t want = target / bh;
  if (want > pages) want = pages;
  if (want > 1024) want = 1024;
  if (want < 1) want = 1;
  const int64_t pages_per_item = (pages + want - 1) / want;
  plan->page_shift = shift;
  plan->items = (int)((pages + pages_per_item - 1) / pages_per_item);
  plan->item_tokens = pages_per_item * P;
  return NQKV_OK;
}

int nqkv_decode_paged_workspace_bytes(const nqkv_cache_desc* desc, int64_t max_tokens, size_t* bytes_out, int* items_out) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!bytes_out || max_tokens < 1) return NQKV_EINVAL;
  PagedPlan plan;
  if ((rc = plan_paged(desc, max_tokens, &plan))) return rc;
  *bytes_out = workspace_need(desc, plan.items);
  if (items_out) *items_out = plan.items;
  return NQKV_OK;
}

static int decode_paged_impl(const nqkv_cache_desc* desc, const float* levels, const void* q,
                             const void* k_new, const void* v_new, int64_t new_stride_b, int64_t new_stride_h,
                             const int32_t* lens, const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                             const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                             int64_t n_cached, float softmax_scale, void* out,
                             void* workspace, size_t workspace_bytes, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const bool fuse = k_new != nullptr;
  DecodeParams p;
  std::memset(&p, 0, sizeof(p));
  LevelTable checked;
  if ((rc = check_levels(levels, desc->k, &checked))) return rc;
  const int64_t P = desc->cap_tokens;
  if (n_cached < (fuse ? 0 : 1)) return NQKV_EINVAL;
  if (!lens || (reinterpret_cast<uintptr_t>(lens) & 3u) || !block_table || (reinterpret_cast<uintptr_t>(block_table) & 3u))
    return NQKV_EINVAL;
  if (num_pages < 1 || num_pages > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
  PagedPlan plan;
  if ((rc = plan_paged(desc, n_cached, &plan))) return rc;
  // table columns the kernel may look at: the pages of the cached tokens, and the page of the new row
  const int64_t cached_pages = n_cached <= 0 ? 0 : (n_cached + P - 1) / P;
  const int64_t cols = std::max<int64_t>(1, fuse ? std::max<int64_t>(cached_pages, n_cached / P + 1) : cached_pages);
  if (table_stride < cols || table_stride > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
  if (n_cached + plan.item_tokens > ((int64_t)1 << 31) - 1) return NQKV_EUNSUPPORTED;
  if (!std::isfinite(softmax_scale)) return NQKV_EINVAL;
  const void* ptrs[] = {q, k_codes, k_scales, v_codes, v_scales, out};
  for (const void* ptr : ptrs) {
    if (!ptr || !aligned16(ptr)) return NQKV_EINVAL;
  }
  if (fuse) {
    if (!v_new || !aligned16(k_new) || !aligned16(v_new)) return NQKV_EINVAL;
    if (new_stride_b < 0 || new_stride_h < 0 || (new_stride_b % 8) || (new_stride_h % 8)) return NQKV_EINVAL;
    if (!build_cell_table(levels, desc->k, p.cell_thr, p.cell_below)) return NQKV_EUNSUPPORTED;
  }
  const size_t need = workspace_need(desc, plan.items);
  if (need > 0) {
    if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
    if (workspace_bytes < need) return NQKV_EWORKSPACE;
  }
  fill_decode_common(&p, desc, checked, q, k_new, v_new, new_stride_b, new_stride_h, k_codes, k_scales, v_codes, v_scales,
                     softmax_scale, out, workspace, plan.items, plan.item_tokens);
  p.split_base = (int)plan.item_tokens;                // items are runs of whole pages
  p.split_rem = 0;
  p.seq_lens = lens;
  p.max_len = (int)n_cached;
  p.longest_first = longest_first_pays(p, lens, desc->B);
  p.block_table = block_table;
  p.table_stride = (int)table_stride;
  p.num_pages = (int)num_pages;
  p.page_shift = plan.page_shift;
  const hipError_t e = launch_decode_attention(p, desc->D, desc->k, desc->block, fuse, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

static int quantize_paged_impl(const nqkv_cache_desc* desc, const float* levels,
                               const void* k_src, const void* v_src,
                               int64_t stride_b, int64_t stride_h, int64_t stride_t,
                               int64_t n_tokens, const int32_t* offsets, int64_t dst_token_offset,
                               const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                               void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                               void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  QuantParams p;
  std::memset(&p, 0, sizeof(p));
  if ((rc = check_levels(levels, desc->k, &p.levels))) return rc;
  PagedPlan plan;
  if ((rc = plan_paged(desc, 1, &plan))) return rc;                // page size check
  const int64_t P = desc->cap_tokens;
  if (n_tokens < 0 || dst_token_offset < 0) return NQKV_EINVAL;
  if (!block_table || (reinterpret_cast<uintptr_t>(block_table) & 3u)) return NQKV_EINVAL;
  if (num_pages < 1 || num_pages > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
  if (table_stride < 1 || table_stride > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
  if (dst_token_offset + n_tokens > table_stride * P) return NQKV_EINVAL;        // rows beyond the table
  if ((rc = check_strided(desc, stride_b, stride_h, stride_t, n_tokens))) return rc;
  if (dst_token_offset + n_tokens >= ((int64_t)1 << 31) / (desc->D / 8)) return NQKV_EUNSUPPORTED;   // 32-bit chunk indices
  if (n_tokens == 0) return NQKV_OK;
  const bool pair = v_src || v_codes || v_scales;
  if (!k_src || !k_codes || !k_scales || !aligned16(k_src) || !aligned16(k_codes) || !aligned16(k_scales))
    return NQKV_EINVAL;
  if (pair && (!v_src || !v_codes || !v_scales || !aligned16(v_src) || !aligned16(v_codes) || !aligned16(v_scales)))
    return NQKV_EINVAL;
  if ((int64_t)desc->B * 2 > 65535) return NQKV_EUNSUPPORTED;
  p.t[0].src = static_cast<const uint16_t*>(k_src);
  p.t[0].codes = static_cast<uint8_t*>(k_codes);
  p.t[0].scales = static_cast<uint16_t*>(k_scales);
  p.t[1].src = static_cast<const uint16_t*>(v_src);
  p.t[1].codes = static_cast<uint8_t*>(v_codes);
  p.t[1].scales = static_cast<uint16_t*>(v_scales);
  p.n_tensors = pair ? 2 : 1;
  p.B = desc->B;
  p.H = desc->H;
  p.stride_b = stride_b;
  p.stride_h = stride_h;
  p.stride_t = stride_t;
  p.n_tokens = n_tokens;
  p.tok_off = dst_token_offset;
  p.tok_offs = offsets;
  p.max_off = (int)dst_token_offset;                   // (< 2^31 by the check above)
  p.cap_tokens = P;
  p.impl = (!(desc->flags & NQKV_FLAG_SCAN_QUANTIZER) && build_cell_table(levels, desc->k, p.cell_thr, p.cell_below)) ? 0 : 1;
  p.block_table = block_table;
  p.table_stride = (int)table_stride;
  p.num_pages = (int)num_pages;
  p.page_shift = plan.page_shift;
  const hipError_t e = launch_quantize_paged(p, desc->D, desc->k, desc->block, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_quantize_kv_paged(const nqkv_cache_desc* desc, const float* levels,
                           const void* k_src, const void* v_src,
                           int64_t stride_b, int64_t stride_h, int64_t stride_t,
                           int64_t n_tokens, int64_t dst_token_offset,
                           const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                           void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                           void* hip_stream) {
  return quantize_paged_impl(desc, levels, k_src, v_src, stride_b, stride_h, stride_t, n_tokens, nullptr, dst_token_offset,
                             block_table, table_stride, num_pages, k_codes, k_scales, v_codes, v_scales, hip_stream);
}

int nqkv_quantize_kv_paged_varlen(const nqkv_cache_desc* desc, const float* levels,
                                  const void* k_src, const void* v_src,
                                  int64_t stride_b, int64_t stride_h, int64_t stride_t,
                                  int64_t n_tokens, const int32_t* dst_token_offsets, int64_t max_offset,
                                  const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                  void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                                  void* hip_stream) {
  if (!dst_token_offsets || (reinterpret_cast<uintptr_t>(dst_token_offsets) & 3u)) return NQKV_EINVAL;
  return quantize_paged_impl(desc, levels, k_src, v_src, stride_b, stride_h, stride_t, n_tokens, dst_token_offsets, max_offset,
                             block_table, table_stride, num_pages, k_codes, k_scales, v_codes, v_scales, hip_stream);
}

int nqkv_decode_attention_paged(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                const int32_t* seq_lens, int64_t max_seq_len, float softmax_scale, void* out,
                                void* workspace, size_t workspace_bytes, void* hip_stream) {
  return decode_paged_impl(desc, levels, q, nullptr, nullptr, 0, 0, seq_lens, block_table, table_stride, num_pages,
                           k_codes, k_scales, v_codes, v_scales, max_seq_len, softmax_scale, out, workspace,
                           workspace_bytes, hip_stream);
}

int nqkv_decode_step_paged(const nqkv_cache_desc* desc, const float* levels,
                           const void* q, const void* k_new, const void* v_new,
                           int64_t new_stride_b, int64_t new_stride_h,
                           void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                           const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                           const int32_t* pos, int64_t max_pos, float softmax_scale, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!k_new) return NQKV_EINVAL;
  return decode_paged_impl(desc, levels, q, k_new, v_new, new_stride_b, new_stride_h, pos, block_table, table_stride,
                           num_pages, k_codes, k_scales, v_codes, v_scales, max_pos, softmax_scale, out, workspace,
                           workspace_bytes, hip_stream);
}

int nqkv_decode_multi_workspace_bytes(const nqkv_cache_desc* desc, int64_t seq_len, int q_len, int num_splits,
                                      size_t* bytes_out, int* splits_out) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!bytes_out) return NQKV_EINVAL;
  int splits = 1;
  if ((rc = plan_multi(desc, seq_len, desc->cap_tokens, q_len, num_splits, &splits))) return rc;
  *bytes_out = multi_workspace_need(desc, q_len, splits);
  if (splits_out) *splits_out = splits;
  return NQKV_OK;
}

// Shared by nqkv_decode_attention_multi (lens == nullptr) and its per-sequence-length form.
static int decode_multi_impl(const nqkv_cache_desc* desc, const float* levels, const void* q,
                             const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                             const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                             const int32_t* lens, int64_t seq_len, int q_len, float softmax_scale, void* out,
                             void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  LevelTable checked;
  if ((rc = check_levels(levels, desc->k, &checked))) return rc;
  int64_t max_tokens = desc->cap_tokens;
  int page_shift = 0;
  if (block_table) {
    // desc->cap_tokens is the page size; a sequence may hold as many tokens as its table row has pages
    PagedPlan pages;
    if ((rc = plan_paged(desc, 1, &pages))) return rc;
    if (reinterpret_cast<uintptr_t>(block_table) & 3u) return NQKV_EINVAL;
    if (num_pages < 1 || num_pages > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
    if (table_stride < 1 || table_stride > ((int64_t)1 << 31) - 1) return NQKV_EINVAL;
    page_shift = pages.page_shift;
    max_tokens = table_stride * desc->cap_tokens;
  }
  int splits = 1;
  if ((rc = plan_multi(desc, seq_len, max_tokens, q_len, num_splits, &splits))) return rc;
  if (!std::isfinite(softmax_scale)) return NQKV_EINVAL;
  const void* ptrs[] = {q, k_codes, k_scales, v_codes, v_scales, out};
  for (const void* ptr : ptrs) {
    if (!ptr || !aligned16(ptr)) return NQKV_EINVAL;
  }
  const size_t need = multi_workspace_need(desc, q_len, splits);
  if (need > 0) {
    if (!workspace || !aligned16(workspace)) return NQKV_EINVAL;
    if (workspace_bytes < need) return NQKV_EWORKSPACE;
  }
  const int64_t trip = decode_multi_trip_tokens();
  const int64_t trips = (seq_len + trip - 1) / trip;
  // one piece's byte range is addressed with 32-bit offsets
  if ((trips / splits + 1) * trip * (int64_t)(desc->D * desc->k / 8) >= ((int64_t)1 << 31)) return NQKV_EUNSUPPORTED;
  MultiParams p;
  std::memset(&p, 0, sizeof(p));
  p.q = static_cast<const uint16_t*>(q);
  p.k_codes = static_cast<const uint8_t*>(k_codes);
  p.k_scales = static_cast<const uint16_t*>(k_scales);
  p.v_codes = static_cast<const uint8_t*>(v_codes);
  p.v_scales = static_cast<const uint16_t*>(v_scales);
  p.out = static_cast<uint16_t*>(out);
  p.partials = static_cast<float*>(workspace);
  p.n_items = desc->B * desc->H * splits;
  p.splits = splits;
  p.split_base = (int)(trips / splits);
  p.split_rem = (int)(trips % splits);
  p.seq_len = (int)seq_len;
  p.q_len = q_len;
  p.cap_tokens = desc->cap_tokens;
  p.seq_lens = lens;
  p.H = desc->H;
  p.block_table = block_table;
  p.table_stride = (int)table_stride;
  p.num_pages = (int)num_pages;
  p.page_shift = page_shift;
  // (one workgroup per item always; the order matters once they cannot all be resident)
  p.n_seqs = desc->B;
  p.longest_first = lens && desc->B >= 2 && desc->B <= 64 && p.n_items > max_decode_workgroups() &&
                    trips / splits >= kLongItemTokens / trip;
  const LutChoice& lut = choose_lut_scale(checked.v, 1 << desc->k);
  std::memcpy(p.lut_levels, lut.bits, sizeof(uint16_t) * (1 << desc->k));
  p.inv_gamma = 1.0f / lut.gamma;
  p.scale_log2e = (float)((double)softmax_scale * 1.44269504088896340736 / (double)lut.gamma);
  const hipError_t e = launch_decode_attention_multi(p, desc->D, desc->k, desc->block, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? NQKV_OK : NQKV_EHIP;
}

int nqkv_decode_attention_multi(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                int64_t seq_len, int q_len, float softmax_scale, void* out,
                                void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  return decode_multi_impl(desc, levels, q, k_codes, k_scales, v_codes, v_scales, nullptr, 0, 0, nullptr, seq_len, q_len, softmax_scale, out,
                           workspace, workspace_bytes, num_splits, hip_stream);
}

int nqkv_decode_attention_multi_varlen(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                       const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                       const int32_t* seq_lens, int64_t max_seq_len, int q_len, float softmax_scale, void* out,
                                       void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  if (!seq_lens || (reinterpret_cast<uintptr_t>(seq_lens) & 3u)) return NQKV_EINVAL;
  return decode_multi_impl(desc, levels, q, k_codes, k_scales, v_codes, v_scales, nullptr, 0, 0, seq_lens, max_seq_len, q_len, softmax_scale, out,
                           workspace, workspace_bytes, num_splits, hip_stream);
}

int nqkv_decode_multi_paged_workspace_bytes(const nqkv_cache_desc* desc, int64_t max_seq_len, int q_len, int num_splits,
                                            size_t* bytes_out, int* splits_out) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!bytes_out) return NQKV_EINVAL;
  PagedPlan pages;
  if ((rc = plan_paged(desc, 1, &pages))) return rc;
  int splits = 1;
  if ((rc = plan_multi(desc, max_seq_len, ((int64_t)1 << 31) - 65, q_len, num_splits, &splits))) return rc;
  *bytes_out = multi_workspace_need(desc, q_len, splits);
  if (splits_out) *splits_out = splits;
  return NQKV_OK;
}

int nqkv_decode_attention_multi_paged(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                      const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                      const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                      const int32_t* seq_lens, int64_t max_seq_len, int q_len, float softmax_scale, void* out,
                                      void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream) {
  if (!seq_lens || (reinterpret_cast<uintptr_t>(seq_lens) & 3u) || !block_table) return NQKV_EINVAL;
  return decode_multi_impl(desc, levels, q, k_codes, k_scales, v_codes, v_scales, block_table, table_stride, num_pages,
                           seq_lens, max_seq_len, q_len, softmax_scale, out, workspace, workspace_bytes, num_splits, hip_stream);
}

}  // extern "C"
