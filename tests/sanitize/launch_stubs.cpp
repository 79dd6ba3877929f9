// Stand-ins for the kernel launchers of libnqkv, for a CPU-only build of its host layer under
// AddressSanitizer / UndefinedBehaviorSanitizer: no GPU is touched; each stub checks the launch
// parameters the host layer filled in (everything a kernel would rely on) and counts the launch.
#include "../../paper_2505_16210_amd/csrc/nqkv_internal.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>

int g_stub_launches = 0;

namespace {
void require(bool ok, const char* what) {
  if (!ok) {
    std::fprintf(stderr, "launch stub: bad parameters: %s\n", what);
    std::abort();
  }
}
void check_quant(const nqkv::QuantParams& p) {
  require(p.n_tensors == 1 || p.n_tensors == 2, "n_tensors");
  require(p.B >= 1 && p.H >= 1 && p.n_tokens >= 1, "geometry");
  require(p.tok_off >= 0 && p.tok_off + p.n_tokens <= (p.block_table ? (int64_t)p.table_stride << p.page_shift : p.cap_tokens), "rows");
  for (int i = 1; i < nqkv::kMaxLevels && p.levels.v[i] != 0.0f; ++i) require(std::isfinite(p.levels.v[i]), "levels");
  require(p.impl == 0 || p.impl == 1, "impl");
  if (p.impl == 0)
    for (int c = 0; c < nqkv::kQuantCells; ++c) require(p.cell_below[c] <= 15u, "cell table");
  ++g_stub_launches;
}
void check_decode_lut(const uint16_t* lut, float inv_gamma, float scale_log2e) {
  require(std::isfinite(inv_gamma) && inv_gamma > 0.0f && std::isfinite(scale_log2e), "table scale");
  for (int i = 0; i < 4; ++i) require((lut[i] & 0x7c00u) != 0x7c00u, "fp16 table entry");
}
}  // namespace

namespace nqkv {

hipError_t launch_quantize(const QuantParams& p, int, int, int, hipStream_t) { check_quant(p); return hipSuccess; }
hipError_t launch_quantize_paged(const QuantParams& p, int, int, int, hipStream_t) {
  require(p.block_table && p.table_stride >= 1 && p.num_pages >= 1 && (1 << p.page_shift) == p.cap_tokens, "paged plan");
  check_quant(p);
  return hipSuccess;
}
hipError_t launch_quantize_hidden(const QuantParams& p, int D, int, int blk_hidden, hipStream_t) {
  require(blk_hidden % D == 0 && (p.H * D) % blk_hidden == 0, "hidden blocks");
  check_quant(p);
  return hipSuccess;
}
hipError_t launch_dequantize(const QuantParams& p, int, int, int, hipStream_t) {
  require(p.t[0].dst && p.t[0].codes && p.t[0].scales && p.n_tokens >= 1, "dequantize");
  ++g_stub_launches;
  return hipSuccess;
}
hipError_t launch_decode_attention(const DecodeParams& p, int D, int, int, bool fuse, hipStream_t) {
  require(p.n_items >= 1 && p.splits >= 1 && p.n_items % p.splits == 0, "items");
  require(p.max_workgroups >= 1, "grid");
  require(p.split_base >= 0 && p.split_rem >= 0 && p.split_rem < p.splits, "split geometry");
  require((fuse ? p.k_new && p.v_new : true) && p.q && p.out, "pointers");
  if (p.splits > 1) require(p.tickets && reinterpret_cast<char*>(p.partials) - reinterpret_cast<char*>(p.tickets) == (ptrdiff_t)kTicketBytes, "workspace layout");
  if (p.block_table) require(p.seq_lens && (p.split_base & ((1 << p.page_shift) - 1)) == 0, "paged items are whole pages");
  check_decode_lut(p.lut_levels, p.inv_gamma, p.scale_log2e);
  (void)D;
  ++g_stub_launches;
  return hipSuccess;
}
hipError_t launch_decode_attention_multi(const MultiParams& p, int, int, int, hipStream_t) {
  require(p.n_items >= 1 && p.splits >= 1 && p.q_len >= 1 && p.q_len <= 16 && p.seq_len >= p.q_len, "multi");
  require((int64_t)p.splits * p.split_base + p.split_rem == ((int64_t)p.seq_len + decode_multi_trip_tokens() - 1) / decode_multi_trip_tokens(), "multi split geometry");
  check_decode_lut(p.lut_levels, p.inv_gamma, p.scale_log2e);
  ++g_stub_launches;
  return hipSuccess;
}
int decode_multi_trip_tokens() { return 32; }
int decode_multi_item_tokens() { return 256; }
int decode_chunk_tokens(int D) { return 4 * (64 / (D / 32)); }
int decode_waves_per_workgroup() { return 8; }

hipError_t static_scratch(void** ptr_out) {
  alignas(256) static unsigned char fake[kStaticScratchBytes];
  *ptr_out = fake;
  return hipSuccess;
}
hipError_t launch_clear_words(uint32_t* words, int n, hipStream_t) {
  require(words && n >= 0 && (size_t)n * 4 <= kTicketBytes, "clear");
  ++g_stub_launches;
  return hipSuccess;
}

}  // namespace nqkv
