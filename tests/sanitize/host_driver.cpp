// Drives the host layer of libnqkv (argument validation, the quantile table, split and page
// planning, the look-up-table scaling, the quantizer's cell table) through the public C ABI in a
// CPU-only build under AddressSanitizer / UndefinedBehaviorSanitizer.  Kernel launchers are
// stubs (launch_stubs.cpp), so "device" pointers are never dereferenced: any aligned non-null
// address will do.  Exits 0 and prints "host-layer sanitizer run: ok" when nothing trips.
#include "../../include/nqkv.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <vector>

extern int g_stub_launches;

#define CHECK(cond)                                                              \
  do {                                                                           \
    if (!(cond)) {                                                               \
      std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
      return 1;                                                                  \
    }                                                                            \
  } while (0)

int main() {
  void* const P = reinterpret_cast<void*>(0x10000);         // an aligned "device" address
  // ---- quantile tables, every width and both variants
  for (int variant = 0; variant < 2; ++variant) {
    for (int k = 1; k <= 8; ++k) {
      std::vector<float> lv(1u << k, 0.0f);
      const int rc = nqkv_build_codebook(k, variant, lv.data());
      if (variant == 1 && k < 2) { CHECK(rc == NQKV_EINVAL); continue; }
      CHECK(rc == NQKV_OK);
      CHECK(lv.front() == -1.0f && lv.back() == 1.0f);
      for (size_t i = 1; i < lv.size(); ++i) CHECK(lv[i] > lv[i - 1]);
    }
  }
  float lv[16];
  CHECK(nqkv_build_codebook(0, 0, lv) == NQKV_EINVAL && nqkv_build_codebook(9, 0, lv) == NQKV_EINVAL);
  CHECK(nqkv_build_codebook(4, 2, lv) == NQKV_EINVAL && nqkv_build_codebook(4, 0, nullptr) == NQKV_EINVAL);

  // ---- every kernel geometry through every entry point (launches are counted by the stubs)
  const int Ds[] = {64, 128}, ks[] = {2, 3, 4}, blks[] = {64, 128};
  for (int D : Ds) for (int k : ks) for (int blk : blks) {
    if (blk > D) continue;
    nqkv_cache_desc d = {3, 5, D, k, blk, 0, 4096};
    CHECK(nqkv_build_codebook(k, 0, lv) == NQKV_OK);
    const int before = g_stub_launches;
    CHECK(nqkv_quantize_kv(&d, lv, P, 5 * 4096 * D, 4096 * D, D, 4096, 0, P, P, nullptr) == NQKV_OK);
    CHECK(nqkv_quantize_kv_pair(&d, lv, P, P, 5 * 64 * D, 64 * D, D, 7, 100, P, P, P, P, nullptr) == NQKV_OK);
    CHECK(nqkv_quantize_kv_pair_varlen(&d, lv, P, P, 5 * 64 * D, 64 * D, D, 7, static_cast<const int32_t*>(P), 4000, P, P, P, P, nullptr) == NQKV_OK);
    CHECK(nqkv_dequantize_kv(&d, lv, P, P, 10, 1000, P, 5 * 1000 * D, 1000 * D, D, nullptr) == NQKV_OK);
    for (int ns : {0, 1, 2, 7, 64, 1024}) {
      size_t bytes = 0; int splits = 0;
      CHECK(nqkv_decode_workspace_bytes(&d, 4096, ns, &bytes, &splits) == NQKV_OK);
      CHECK(splits >= 1 && (ns == 0 || splits == ns) && (splits == 1) == (bytes == 0));
      CHECK(nqkv_decode_attention(&d, lv, P, P, P, P, P, 4096, 0.7f, P, P, bytes, ns, nullptr) == NQKV_OK);
      CHECK(nqkv_decode_attention_varlen(&d, lv, P, P, P, P, P, static_cast<const int32_t*>(P), 4096, 0.7f, P, P, bytes, ns, nullptr) == NQKV_OK);
      if (bytes > 16) CHECK(nqkv_decode_attention(&d, lv, P, P, P, P, P, 4096, 0.7f, P, P, bytes - 1, ns, nullptr) == NQKV_EWORKSPACE);
      CHECK(nqkv_decode_workspace_bytes(&d, 4095, ns, &bytes, &splits) == NQKV_OK);
      CHECK(nqkv_decode_step(&d, lv, P, P, P, 5 * D, D, P, P, P, P, 4095, 1.0f, P, P, bytes, ns, nullptr) == NQKV_OK);
      CHECK(nqkv_decode_step_varlen(&d, lv, P, P, P, 5 * D, D, P, P, P, P, static_cast<const int32_t*>(P), 4095, 1.0f, P, P, bytes, ns, nullptr) == NQKV_OK);
      if (bytes <= NQKV_STATIC_SCRATCH_BYTES)
        CHECK(nqkv_decode_attention_static(&d, lv, P, P, P, P, P, 4095, 1.0f, P, ns, nullptr) == NQKV_OK);
    }
    CHECK(nqkv_decode_step(&d, lv, P, P, P, 5 * D, D, P, P, P, P, 0, 1.0f, P, nullptr, 0, 0, nullptr) == NQKV_OK);   // first token of an empty cache
    for (int q_len : {1, 4, 16}) for (int ns : {0, 1, 3}) {
      size_t bytes = 0; int splits = 0;
      CHECK(nqkv_decode_multi_workspace_bytes(&d, 4000, q_len, ns, &bytes, &splits) == NQKV_OK);
      CHECK(nqkv_decode_attention_multi(&d, lv, P, P, P, P, P, 4000, q_len, 1.0f, P, P, bytes, ns, nullptr) == NQKV_OK);
      CHECK(nqkv_decode_attention_multi_varlen(&d, lv, P, P, P, P, P, static_cast<const int32_t*>(P), 4000, q_len, 1.0f, P, P, bytes, ns, nullptr) == NQKV_OK);
    }
    // paged: pages of 256 tokens, 16 per sequence
    nqkv_cache_desc pd = {3, 5, D, k, blk, 0, 256};
    size_t pbytes = 0; int items = 0;
    CHECK(nqkv_decode_paged_workspace_bytes(&pd, 4096, &pbytes, &items) == NQKV_OK && items >= 1);
    CHECK(nqkv_decode_attention_paged(&pd, lv, P, P, P, P, P, static_cast<const int32_t*>(P), 16, 48, static_cast<const int32_t*>(P), 4096, 1.0f, P, P, pbytes, nullptr) == NQKV_OK);
    CHECK(nqkv_decode_paged_workspace_bytes(&pd, 4095, &pbytes, &items) == NQKV_OK);
    CHECK(nqkv_decode_step_paged(&pd, lv, P, P, P, 5 * D, D, P, P, P, P, static_cast<const int32_t*>(P), 16, 48, static_cast<const int32_t*>(P), 4095, 1.0f, P, P, pbytes, nullptr) == NQKV_OK);
    CHECK(nqkv_quantize_kv_paged(&pd, lv, P, P, 5 * 4096 * D, 4096 * D, D, 4096, 0, static_cast<const int32_t*>(P), 16, 48, P, P, P, P, nullptr) == NQKV_OK);
    CHECK(nqkv_quantize_kv_paged_varlen(&pd, lv, P, P, 5 * 8 * D, 8 * D, D, 8, static_cast<const int32_t*>(P), 4000, static_cast<const int32_t*>(P), 16, 48, P, P, P, P, nullptr) == NQKV_OK);
    size_t mb = 0; int ms = 0;
    CHECK(nqkv_decode_multi_paged_workspace_bytes(&pd, 4096, 4, 0, &mb, &ms) == NQKV_OK);
    CHECK(nqkv_decode_attention_multi_paged(&pd, lv, P, P, P, P, P, static_cast<const int32_t*>(P), 16, 48, static_cast<const int32_t*>(P), 4096, 4, 1.0f, P, P, mb, 0, nullptr) == NQKV_OK);
    CHECK(g_stub_launches > before + 40);
  }
  // hidden-vector blocks
  {
    nqkv_cache_desc d = {2, 8, 64, 4, 64, 0, 512};
    CHECK(nqkv_build_codebook(4, 1, lv) == NQKV_OK);
    CHECK(nqkv_quantize_kv_hidden(&d, lv, P, P, 512 * 512, 64, 512, 512, 0, 256, P, P, P, P, nullptr) == NQKV_OK);
    CHECK(nqkv_quantize_kv_hidden(&d, lv, P, P, 512 * 512, 64, 512, 512, 0, 192, P, P, P, P, nullptr) == NQKV_EUNSUPPORTED);
    CHECK(nqkv_quantize_kv_hidden(&d, lv, P, nullptr, 512 * 512, 64, 512, 0, 0, 256, nullptr, nullptr, nullptr, nullptr, nullptr) == NQKV_OK);
  }
  // ---- a table the cell search cannot take (crowded mid-points), one it can, and bad ones
  {
    nqkv_cache_desc d = {1, 6, 128, 4, 64, 0, 300};
    float crowded[16];
    for (int i = 0; i < 16; ++i) crowded[i] = -1.0f + 2.0f * (float)i / 15.0f;
    crowded[7] = -0.004f; crowded[8] = 0.004f; crowded[9] = 0.012f;
    size_t need_cached = 0, need_all = 0; int s1 = 0, s2 = 0;
    CHECK(nqkv_decode_workspace_bytes(&d, 255, 0, &need_cached, &s1) == NQKV_OK);
    CHECK(nqkv_decode_workspace_bytes(&d, 256, 0, &need_all, &s2) == NQKV_OK && s2 == s1 + 1);
    const int before = g_stub_launches;
    CHECK(nqkv_decode_step(&d, crowded, P, P, P, 6 * 128, 128, P, P, P, P, 255, 1.0f, P, P, need_cached, 0, nullptr) == NQKV_EWORKSPACE);
    CHECK(g_stub_launches == before);                         // refused before the append was launched
    CHECK(nqkv_decode_step(&d, crowded, P, P, P, 6 * 128, 128, P, P, P, P, 255, 1.0f, P, P, need_all, 0, nullptr) == NQKV_OK);
    CHECK(g_stub_launches == before + 2);                     // append, then attention
    CHECK(nqkv_decode_step_varlen(&d, crowded, P, P, P, 6 * 128, 128, P, P, P, P, static_cast<const int32_t*>(P), 255, 1.0f, P, P, need_all, 0, nullptr) == NQKV_EUNSUPPORTED);
    float bad[16];
    for (int i = 0; i < 16; ++i) bad[i] = (float)i;
    bad[5] = bad[4];
    CHECK(nqkv_quantize_kv(&d, bad, P, 0, 300 * 128, 128, 10, 0, P, P, nullptr) == NQKV_EINVAL);
    bad[5] = NAN;
    CHECK(nqkv_quantize_kv(&d, bad, P, 0, 300 * 128, 128, 10, 0, P, P, nullptr) == NQKV_EINVAL);
    for (int i = 0; i < 16; ++i) bad[i] = 100.0f * (float)(i - 8);                     // leaves [-1, 1]: threshold scan
    CHECK(nqkv_quantize_kv(&d, bad, P, 0, 300 * 128, 128, 10, 0, P, P, nullptr) == NQKV_OK);
  }
  // ---- refusals
  {
    nqkv_build_codebook(4, 0, lv);
    nqkv_cache_desc d = {2, 4, 64, 4, 64, 0, 16};
    nqkv_cache_desc bad = d;
    bad.flags = 4;
    CHECK(nqkv_quantize_kv(&bad, lv, P, 0, 0, 64, 1, 0, P, P, nullptr) == NQKV_EINVAL);
    bad = d; bad.D = 96;
    CHECK(nqkv_quantize_kv(&bad, lv, P, 0, 0, 64, 1, 0, P, P, nullptr) == NQKV_EUNSUPPORTED);
    bad = d; bad.B = 4096; bad.H = 4097;
    CHECK(nqkv_quantize_kv(&bad, lv, P, 0, 0, 64, 1, 0, P, P, nullptr) == NQKV_EUNSUPPORTED);
    CHECK(nqkv_quantize_kv(nullptr, lv, P, 0, 0, 64, 1, 0, P, P, nullptr) == NQKV_EINVAL);
    CHECK(nqkv_quantize_kv(&d, lv, P, 0, 0, 64, 2, 15, P, P, nullptr) == NQKV_EINVAL);
    CHECK(nqkv_quantize_kv(&d, lv, reinterpret_cast<void*>(0x10004), 0, 0, 64, 1, 0, P, P, nullptr) == NQKV_EINVAL);
    CHECK(nqkv_quantize_kv(&d, lv, nullptr, 0, 0, 64, 0, 0, nullptr, nullptr, nullptr) == NQKV_OK);
    CHECK(nqkv_decode_workspace_init(nullptr, 1 << 20, nullptr) == NQKV_EINVAL);
    CHECK(nqkv_decode_workspace_init(P, 100, nullptr) == NQKV_EWORKSPACE);
    CHECK(nqkv_decode_workspace_init(P, 1 << 20, nullptr) == NQKV_OK);
    CHECK(nqkv_strerror(NQKV_EWORKSPACE) != nullptr && nqkv_strerror(12345) != nullptr && nqkv_version() == 100);
  }
  std::printf("host-layer sanitizer run: ok (%d stub launches)\n", g_stub_launches);
  return 0;
}
