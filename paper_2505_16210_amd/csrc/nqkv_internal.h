// Internal declarations shared by the host layer and the kernel translation units of
// libnqkv.  Nothing here is part of the public ABI (see include/nqkv.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace nqkv {

constexpr int kMaxLevels = 16;  // kernels take tables for k <= 4
constexpr int kQuantCells = 65;  // index cells of the quantizer's code search

namespace code_search {
// Cell grid of the quantizer's fast code search: u = 32 * x/s + 32.5 in [0.5, 64.5], cell = floor(u).
constexpr int kCells = kQuantCells;
constexpr float kCellScale = 32.0f;
constexpr float kCellBias = 32.5f;
// u is produced by an fma whose result is forced onto a 1/8 grid (error <= 1/16) from a
// reciprocal good to 1 ulp (error < 1e-5 in u); 0.08 leaves > 5e-4 of slack in x/s, far more
// than the 2^-24 relative rounding of fl32(t * s).
constexpr float kCellMargin = 0.08f;
}  // namespace code_search

// The quantile table travels to the kernels by value (64 bytes of kernel arguments).
struct LevelTable {
  float v[kMaxLevels];
};

// One tensor's worth of pointers for the quantizer / dequantizer.
struct TensorPtrs {
  const uint16_t* src;   // fp16 source (quantize) -- unused by dequantize
  uint16_t* dst;         // fp16 destination (dequantize) -- unused by quantize
  uint8_t* codes;
  uint16_t* scales;
};

struct QuantParams {
  TensorPtrs t[2];       // [0] = K (or the only tensor), [1] = V
  int n_tensors;         // 1 or 2
  int B, H;
  int64_t stride_b, stride_h, stride_t;  // fp16 tensor strides, in elements
  int64_t n_tokens;      // tokens to process
  int64_t tok_off;       // first cache row
  // per-sequence first rows (NULL: tok_off for every sequence): device int32 [B], clamped into
  // [0, max_off] by the kernels
  const int32_t* tok_offs;
  int max_off;
  int64_t cap_tokens;
  LevelTable levels;
  int impl;              // 0 = cell-table quantizer, 1 = plain threshold scan
  // paged destination (NULL: contiguous [B][H][cap_tokens] rows): page of logical page j of
  // sequence b at block_table[b * table_stride + j], pages of [H][1 << page_shift] rows
  const int32_t* block_table;
  int table_stride;
  int num_pages;
  int page_shift;
  uint32_t cell_thr[kQuantCells];    // impl 0: fp32 bits of the threshold that may lie in the cell
  uint32_t cell_below[kQuantCells];  //         thresholds certainly below the cell
};

struct DecodeParams {
  const uint16_t* q;         // [B*H][D] fp16
  const uint8_t* k_codes;
  const uint16_t* k_scales;
  const uint8_t* v_codes;
  const uint16_t* v_scales;
  uint16_t* out;             // [B*H][D] fp16
  uint32_t* tickets;         // split-K: one arrival counter per (b,h), zero between calls
  float* partials;           // split-K: [B*H][splits][D+2] fp32 (m, l, o[D])
  int n_items;               // B*H*splits
  int splits;
  int split_base, split_rem; // seq_len = splits * split_base + split_rem
  int max_workgroups;        // grid size limit (2 per compute unit, or the item count: see fill_decode_common)
  int64_t cap_tokens;
  float scale_log2e;         // softmax_scale * log2(e) / gamma
  float inv_gamma;           // 1 / gamma: undoes the table scaling on the value side
  uint16_t lut_levels[kMaxLevels];   // fp16 bits of gamma * level[i] (see choose_lut_scale)
  // fused decode step only: the new token's fp16 key / value rows, element (b,h,d) at
  // b * new_stride_b + h * new_stride_h + d; its cache row `pos`; the quantizer's cell table
  const uint16_t* k_new;
  const uint16_t* v_new;
  int64_t new_stride_b, new_stride_h;
  int64_t pos;
  int H;
  // per-sequence lengths (NULL: every sequence has the same): cached tokens of sequence b, and
  // the length the split geometry is laid out for
  const int32_t* seq_lens;
  int max_len;
  // longest first (one workgroup per item, at most 64 sequences): work item i goes to the
  // sequence whose length ranks i / (H * splits)-th, so that the long ones are dispatched first
  int longest_first;
  int n_seqs;                // B
  // paged cache (NULL: contiguous [B][H][cap_tokens] rows): physical page of logical page j of
  // sequence b at block_table[b * table_stride + j]; the pool holds num_pages pages of
  // [H][1 << page_shift] rows; items cover split_base tokens, a multiple of the page size
  const int32_t* block_table;
  int table_stride;
  int num_pages;
  int page_shift;
  uint32_t cell_thr[kQuantCells];
  uint32_t cell_below[kQuantCells];
};

// Attention of several new queries per sequence (the last q_len cached tokens' queries).
struct MultiParams {
  const uint16_t* q;         // [B*H][q_len][D] fp16
  const uint8_t* k_codes;
  const uint16_t* k_scales;
  const uint8_t* v_codes;
  const uint16_t* v_scales;
  uint16_t* out;             // [B*H][q_len][D] fp16
  float* partials;           // splits > 1: [B*H][splits][q_len][D+2] fp32 (m, l, o[D])
  int n_items;               // B*H*splits
  int splits;
  int split_base, split_rem; // in 32-token trips: ceil(seq_len / 32) = splits * split_base + split_rem
  int seq_len, q_len;        // seq_len: cached tokens (with seq_lens: the largest, which the splits are laid out for)
  int64_t cap_tokens;
  float scale_log2e;         // softmax_scale * log2(e) / gamma
  float inv_gamma;
  uint16_t lut_levels[kMaxLevels];
  // per-sequence lengths (NULL: every sequence has seq_len): cached tokens of sequence b
  const int32_t* seq_lens;
  int H;
  // paged cache (NULL: contiguous rows), as in DecodeParams; needs seq_lens
  const int32_t* block_table;
  int table_stride;
  int num_pages;
  int page_shift;
  // ragged batch, long sequences first: see decode_multi_kernel (seq_lens set, at most 64 sequences)
  int longest_first;
  int n_seqs;                // B
};

// Bytes at the start of the split-K workspace that hold the ticket counters (one uint32 per
// (b,h), room for the largest supported B*H), before the partial results.
constexpr size_t kTicketBytes = 65536 * sizeof(uint32_t);
// The last word of that area (B*H <= 65535, so never a counter) is a status word: a kernel that
// is handed a ticket its own call cannot have issued sets bit 0 there.
constexpr uint32_t kWorkspaceStatusWord = 65535;

// Size of the library-owned scratch array behind nqkv_decode_attention_static (per GPU, held until
// the process ends): the ticket counters plus room for 3528 partial results at head size 128.
constexpr size_t kStaticScratchBytes = 2u << 20;
// Device address of that array on the current device (looked up once per device).
hipError_t static_scratch(void** ptr_out);
// Zero-fills n 32-bit words with a small kernel (safe to record into a HIP graph).
hipError_t launch_clear_words(uint32_t* words, int n, hipStream_t stream);

// Each returns hipSuccess or the launch error.  D in {64,128}, k in {2,3,4}, blk in {64,128}.
hipError_t launch_quantize(const QuantParams& p, int D, int k, int blk, hipStream_t stream);
hipError_t launch_dequantize(const QuantParams& p, int D, int k, int blk, hipStream_t stream);
// blocks of blk_hidden (128 or 256) consecutive elements of the token's hidden vector; cache with one scale per token-head
// rows [tok_off, tok_off + n_tokens) of every sequence into the pages its block table names
hipError_t launch_quantize_paged(const QuantParams& p, int D, int k, int blk, hipStream_t stream);
hipError_t launch_quantize_hidden(const QuantParams& p, int D, int k, int blk_hidden, hipStream_t stream);
// fuse: also quantize and append the new token (p.k_new / p.v_new) and attend over it
hipError_t launch_decode_attention(const DecodeParams& p, int D, int k, int blk, bool fuse, hipStream_t stream);

// q_len in [1, 16]
hipError_t launch_decode_attention_multi(const MultiParams& p, int D, int k, int blk, hipStream_t stream);
int decode_multi_trip_tokens();    // split boundaries of that kernel are multiples of this
int decode_multi_item_tokens();    // tokens one workgroup of it consumes per sweep of its waves

// Tokens one wave of the attention kernel consumes per main-loop trip; split boundaries are
// multiples of this.
int decode_chunk_tokens(int D);
int decode_waves_per_workgroup();

// Fills the quantizer's cell table; false when the table does not admit one (then use impl 1).
bool build_cell_table(const float* levels, int k, uint32_t* thr_bits, uint32_t* below);

}  // namespace nqkv
