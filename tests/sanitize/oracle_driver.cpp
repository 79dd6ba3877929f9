// Runs every entry point of the CPU oracle on small inputs in a build under AddressSanitizer /
// UndefinedBehaviorSanitizer (the oracle's source is compiled into this program), with a few
// self-checks -- packing round trip, the quantizer's round-trip bound, attention over one token --
// so that the calls are not optimised away.  Exits 0 and prints "oracle sanitizer run: ok".
#include "../../oracle/nqkv_oracle.cpp"

#include <cstdio>
#include <random>

#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

int main() {
  std::mt19937 rng(7);
  std::normal_distribution<float> gauss(0.0f, 1.0f);
  CHECK(oracle_hardware_threads() >= 1);
  for (uint32_t h = 0; h < 65536; h += 7) {                      // fp16 round trip of finite patterns
    if ((h & 0x7c00u) == 0x7c00u) continue;
    CHECK(oracle_float_to_half(oracle_half_to_float((uint16_t)h)) == (uint16_t)h);
  }
  CHECK(oracle_float_to_half(1e9f) == 0x7c00u && oracle_float_to_half(-1e-9f) == 0x8000u);
  for (int variant = 0; variant < 2; ++variant) {
    for (int k = (variant ? 2 : 1); k <= 8; ++k) {
      const int L = 1 << k;
      std::vector<double> l64(L);
      std::vector<float> l32(L), thr(L - 1);
      CHECK(oracle_codebook(k, variant, l64.data(), l32.data(), thr.data()) == 0);
      for (int i = 1; i < L; ++i) CHECK(l32[i] > l32[i - 1]);
    }
  }
  CHECK(oracle_codebook(0, 0, nullptr, nullptr, nullptr) != 0);
  const int B = 2, H = 3;
  for (int D : {64, 128}) for (int k : {2, 3, 4}) for (int blk : {64, 128}) {
    if (blk > D) continue;
    const int L = 1 << k, n = 37, cap = 41, off = 3, nb = D / blk;
    std::vector<double> l64(L);
    std::vector<float> lv(L), thr(L - 1);
    CHECK(oracle_codebook(k, 0, l64.data(), lv.data(), thr.data()) == 0);
    std::vector<uint16_t> X((size_t)B * H * n * D), Y((size_t)B * H * n * D);
    for (auto& x : X) x = oracle_float_to_half(gauss(rng));
    for (int d = 0; d < D; ++d) X[d] = 0;                                         // an all-zero row
    const int64_t row_bytes = (int64_t)D * k / 8;
    std::vector<uint8_t> codes((size_t)B * H * cap * row_bytes, 0xAA), vcodes(codes);
    std::vector<uint16_t> scales((size_t)B * H * cap * nb, 0x1234), vscales(scales);
    for (int threads : {1, 5}) {
      CHECK(oracle_quantize_kv(X.data(), (int64_t)H * n * D, (int64_t)n * D, D, B, H, D, n, k, blk, lv.data(), cap, off,
                               codes.data(), scales.data(), threads) == 0);
    }
    CHECK(oracle_quantize_kv(X.data(), (int64_t)H * n * D, (int64_t)n * D, D, B, H, D, n, k, blk, lv.data(), cap, off + 2,
                             codes.data(), scales.data(), 1) != 0);                // past the capacity
    CHECK(codes[0] == 0xAA && scales[0] == 0x1234);                                // rows outside the range untouched
    CHECK(oracle_dequantize_kv(codes.data(), scales.data(), B, H, D, k, blk, lv.data(), cap, off, n,
                               Y.data(), (int64_t)H * n * D, (int64_t)n * D, D, 3) == 0);
    double gap = 0.0;
    for (int i = 1; i < L; ++i) gap = std::max(gap, (double)lv[i] - (double)lv[i - 1]);
    for (size_t b0 = 0; b0 < X.size(); b0 += blk) {                                // round-trip bound per block
      double s = 0.0;
      for (int i = 0; i < blk; ++i) s = std::max(s, std::fabs((double)oracle_half_to_float(X[b0 + i])));
      for (int i = 0; i < blk; ++i) {
        const double err = std::fabs((double)oracle_half_to_float(X[b0 + i]) - (double)oracle_half_to_float(Y[b0 + i]));
        CHECK(err <= s * (gap / 2 + 1.0 / 1024) + 1e-12);
      }
    }
    // pack / unpack round trip on a ragged length
    std::vector<uint8_t> c(45), back(45), bytes((45 * k + 7) / 8 + 1, 0xEE);
    for (auto& v : c) v = (uint8_t)(rng() % L);
    oracle_pack_bits(c.data(), 45, k, bytes.data());
    oracle_unpack_bits(bytes.data(), 45, k, back.data());
    CHECK(c == back && bytes.back() == 0xEE);
    // attention: V cache from the same data; one token -> its dequantized value row
    CHECK(oracle_quantize_kv(X.data(), (int64_t)H * n * D, (int64_t)n * D, D, B, H, D, n, k, blk, lv.data(), cap, 0,
                             vcodes.data(), vscales.data(), 2) == 0);
    std::vector<uint8_t> kc0(vcodes);
    std::vector<uint16_t> ks0(vscales), q((size_t)B * H * 4 * D);
    for (auto& x : q) x = oracle_float_to_half(gauss(rng) * 0.1f);
    std::vector<double> out((size_t)B * H * D), outm((size_t)B * H * 4 * D), row(D);
    CHECK(oracle_decode_attention(q.data(), kc0.data(), ks0.data(), vcodes.data(), vscales.data(), B, H, D, k, blk, lv.data(),
                                  cap, 1, 0.5f, out.data(), 2) == 0);
    oracle_dequantize_slab_f64(vcodes.data() + 1 * cap * row_bytes, vscales.data() + 1 * cap * nb, D, k, blk, lv.data(), 1, row.data());
    for (int d = 0; d < D; ++d) CHECK(out[1 * D + d] == row[d]);
    CHECK(oracle_decode_attention(q.data(), kc0.data(), ks0.data(), vcodes.data(), vscales.data(), B, H, D, k, blk, lv.data(),
                                  cap, n, 0.5f, out.data(), 4) == 0);
    CHECK(oracle_decode_attention(q.data(), kc0.data(), ks0.data(), vcodes.data(), vscales.data(), B, H, D, k, blk, lv.data(),
                                  cap, cap + 1, 0.5f, out.data(), 4) != 0);
    CHECK(oracle_decode_attention_multi(q.data(), kc0.data(), ks0.data(), vcodes.data(), vscales.data(), B, H, D, k, blk,
                                        lv.data(), cap, n, 4, 0.5f, outm.data(), 3) == 0);
    for (double v : outm) CHECK(std::isfinite(v));
    // blocks over the hidden vector (token-major source), block = 2 heads or the whole vector where it fits
    if (blk == D && (H * D) % (2 * D) != 0) {
      const int H2 = 4;
      std::vector<uint16_t> T((size_t)B * n * H2 * D);
      for (auto& x : T) x = oracle_float_to_half(gauss(rng));
      std::vector<uint8_t> hc((size_t)B * H2 * cap * row_bytes);
      std::vector<uint16_t> hs((size_t)B * H2 * cap);
      CHECK(oracle_quantize_kv_hidden(T.data(), (int64_t)n * H2 * D, D, (int64_t)H2 * D, B, H2, D, n, k, 2 * D, lv.data(), cap, 1,
                                      hc.data(), hs.data(), 2) == 0);
      CHECK(hs[((0 * H2 + 0) * cap + 1)] == hs[((0 * H2 + 1) * cap + 1)]);         // one scale for both heads of a block
    }
  }
  std::printf("oracle sanitizer run: ok\n");
  return 0;
}
