// Block-wise quantile quantization of a K or V tensor into the packed cache
// (paper Sec. 3.2: I = quantize(X); Fig. 5: every token is cut into blocks and each block
// is quantized on its own).  gfx950 only.
//
// Two grids: a whole-slab kernel for prefill-sized calls (scalar buffer descriptors, no
// predication) and a flat kernel over all rows for calls with a few tokens per (b,h) (append).
//
// Work decomposition: one lane owns one 16-byte chunk = 8 consecutive fp16 of a token row,
// so a 64-element block is shared by 8 neighbouring lanes (16 for a 128-element block) and
// the block's max |x| is an all-reduce over those lanes done with DPP lane permutes -- no
// LDS, no barrier.  Loads are 128-bit and fully coalesced (a wave reads 1 KiB contiguous);
// each lane stores the 8 codes it produced as one 32-bit word (k = 4), or lanes of a pair /
// quad merge their 16- / 24-bit pieces first (k = 2 / 3) so that stores are whole dwords.
//
// Deciding the code.  The contract is  code = #{ j : x > fl32(t_j * s) }  over the fp32
// mid-point thresholds t_j.  Scanning all 2^k - 1 thresholds costs about two VALU
// operations per threshold and element, which at k = 4 would make the kernel ALU-bound
// well below HBM speed.  The "cell table" path gets the same codes with about eight
// operations per element: u = x * (32 / s) + 32.5 lands in one of 65 unit cells; for each
// cell a table (built once per workgroup in LDS from the thresholds) holds how many
// thresholds lie safely below the cell and the single threshold that may fall inside it,
// so one exact comparison against fl32(t * s) finishes the count.  The index u is only
// approximate (reciprocal, rounding), therefore a threshold counts as "inside" a cell when
// it is within the cell widened by a margin larger than any error u can carry; a table for
// which some widened cell would hold two thresholds is routed to the plain scan instead.
#include "code_search.h"
#include "scalar_read.h"
#include "nqkv_internal.h"

#include <cstring>

namespace nqkv {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 4;       // chunks per lane, all loads issued before any use

using namespace code_search;

// grid: SLAB  x = chunk tiles of one (b,h) slab, y = h, z = b + B * tensor
//       FLAT  x = chunk tiles over all rows of a tensor,  z = tensor   (few tokens: append)
template <int KBITS, int D, int BLK, bool FAST, bool FLAT>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const QuantParams p) {
  constexpr int CPR = D / 8;      // chunks per token row
  constexpr int LPB = BLK / 8;    // lanes that share one block
  constexpr int NB = D / BLK;
  __shared__ uint2 cells[FAST ? 128 : 1];   // 128 >= kCells: any 7-bit index stays inside
  // The cell table comes from the kernel arguments by vector loads.  They are issued first and
  // consumed after the source loads have gone out, so that their latency overlaps the source's
  // (the memory counter is positional: waiting for an early load does not wait for later ones).
  const uint2 my_cell = FAST ? fetch_cell(p.cell_thr, p.cell_below) : make_uint2(0, 0);

  const int tensor = FLAT ? (int)blockIdx.z : (int)(blockIdx.z >= (unsigned)p.B);
  const TensorPtrs tp = p.t[tensor];
  const uint32_t n = (uint32_t)p.n_tokens;
  const uint32_t tile0 = blockIdx.x * (kThreads * kUnroll) + threadIdx.x;

  uint4 w[kUnroll];
  bool valid[kUnroll];
  uint32_t bh_[kUnroll], t_[kUnroll], part_[kUnroll];
  int32_t off_[kUnroll];          // first cache row of the lane's sequence
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t c = tile0 + u * kThreads;
    uint32_t bh, t, b, h;
    if (FLAT) {
      const uint32_t row = c / CPR;
      bh = row / n;
      t = row - bh * n;
      b = bh / (uint32_t)p.H;
      h = bh - b * (uint32_t)p.H;
      valid[u] = bh < (uint32_t)(p.B * p.H);
    } else {
      b = blockIdx.z - (tensor ? (uint32_t)p.B : 0u);
      h = blockIdx.y;
      bh = b * (uint32_t)p.H + h;
      t = c / CPR;
      valid[u] = t < n;
    }
    const uint32_t part = c % CPR;
    bh_[u] = bh; t_[u] = t; part_[u] = part;
    w[u] = make_uint4(0, 0, 0, 0);
    off_[u] = (int32_t)p.tok_off;
    if (valid[u]) {
      if (p.tok_offs) off_[u] = min(max(p.tok_offs[b], 0), p.max_off);      // whatever the array holds, stay inside the cache
      const uint16_t* src = tp.src + (int64_t)b * p.stride_b + (int64_t)h * p.stride_h +
                            (int64_t)t * p.stride_t + part * 8;
      w[u] = *reinterpret_cast<const uint4*>(src);
    }
  }

  if (FAST) {
    put_cell(my_cell, cells);
    __syncthreads();
  }

#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    // block scale: max |x| as fp16 bits (for non-negative finite fp16, value order == bit order)
    const uint32_t M = 0x7fff7fffu;
    const uint32_t a = pk_max_u16(pk_max_u16(w[u].x & M, w[u].y & M), pk_max_u16(w[u].z & M, w[u].w & M));
    uint32_t s_bits = max(a & 0xffffu, a >> 16);
    s_bits = max(s_bits, dpp<kQuadXor1>(s_bits));
    s_bits = max(s_bits, dpp<kQuadXor2>(s_bits));
    s_bits = max(s_bits, dpp<kRowHalfMirror>(s_bits));
    if (LPB == 16) s_bits = max(s_bits, dpp<kRowMirror>(s_bits));

    const uint32_t packed = encode_chunk<KBITS, FAST>(w[u], s_bits, p.levels, cells);

    // destination chunk index inside the (b,h) slab of the cache
    const int64_t slab_row0 = (int64_t)bh_[u] * p.cap_tokens + off_[u];
    const int64_t chunk = (slab_row0 + t_[u]) * CPR + part_[u];
    uint32_t* codes32 = reinterpret_cast<uint32_t*>(tp.codes);
    if (KBITS == 4) {
      if (valid[u]) codes32[chunk] = packed;
    } else if (KBITS == 2) {
      const uint32_t odd = dpp<kQuadOdd>(packed);
      if (valid[u] && !(threadIdx.x & 1)) codes32[chunk >> 1] = packed | (odd << 16);
    } else {  // KBITS == 3: four lanes hold 4 x 24 bits = three dwords
      const uint32_t next = dpp<kQuadNext>(packed);
      const uint32_t q = threadIdx.x & 3;
      const uint32_t word = (packed >> (8 * q)) | (next << (24 - 8 * q));
      if (valid[u] && q != 3) codes32[(chunk >> 2) * 3 + q] = word;
    }
    if (valid[u] && (part_[u] % LPB) == 0) {
      tp.scales[(slab_row0 + t_[u]) * NB + part_[u] / LPB] = (uint16_t)s_bits;
    }
  }
}

// Whole-slab variant (prefill): grid x = chunk tiles of one (b,h) slab, y = h, z = b + B * tensor.
// Every address is a scalar buffer descriptor (source slab, code rows, scale rows of this (b,h))
// plus a 32-bit per-lane byte offset, so no 64-bit address arithmetic runs in the vector ALU and
// the ragged last tile needs no predication: chunks past the end read zeros, and their stores
// -- like the stores of lanes that have nothing to write -- carry an offset beyond the
// descriptor's range and are dropped by the hardware range check.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
constexpr int kBufferFlags = 0x00020000;       // raw buffer, 32-bit data format (gfx9 family)
constexpr uint32_t kDropStore = 0xffffffffu;   // voffset outside every descriptor
// Cache-policy bits of the source loads and code stores: the non-temporal hint.  Both streams pass
// once, a whole cache line per instruction; with the hint the prefill quantizer measured 7-13 %
// faster (1.67 -> 1.52 ms on 3.8 G elements per tensor).
constexpr int kNonTemporal = 2;

template <int KBITS, int D, int BLK, bool FAST, bool CONTIG, bool PAGED, int THREADS, int UNROLL>
__global__ __launch_bounds__(THREADS) void quantize_slab_kernel(const QuantParams p) {
  // (the tile shape of this kernel: see launch_slab)
  constexpr int kThreads = THREADS, kUnroll = UNROLL;
  constexpr int CPR = D / 8;      // chunks per token row
  constexpr int LPB = BLK / 8;    // lanes that share one block
  constexpr int NB = D / BLK;
  constexpr int kRowBytes = D * KBITS / 8;
  __shared__ uint2 cells[FAST ? 128 : 1];   // 128 >= kCells: any 7-bit index stays inside
  // The cell table comes from the kernel arguments by vector loads.  They are issued first and
  // consumed after the source loads have gone out, so that their latency overlaps the source's
  // (the memory counter is positional: waiting for an early load does not wait for later ones).
  const uint2 my_cell = FAST ? fetch_cell(p.cell_thr, p.cell_below) : make_uint2(0, 0);

  const uint32_t tensor = blockIdx.z >= (unsigned)p.B ? 1u : 0u;
  const uint32_t b = blockIdx.z - (tensor ? (uint32_t)p.B : 0u), h = blockIdx.y;
  const TensorPtrs tp = p.t[tensor];
  const uint32_t n = (uint32_t)p.n_tokens;
  // PAGED: tiles are laid over ABSOLUTE token positions (tile T = tokens [T * kTileTok, ...)), so
  // that a tile -- 64 or 128 tokens, which divides the page size -- lies inside one page
  // whatever tok_off is; the tile's destination is that page's rows of head h.
  constexpr uint32_t kTileTok = kThreads * kUnroll / CPR;
  // the sequence's own first row when the batch is ragged (clamped: whatever the array holds, the
  // rows written stay inside the cache / the table)
  uint32_t tok_off = (uint32_t)p.tok_off;
  if (p.tok_offs) tok_off = (uint32_t)__builtin_amdgcn_readfirstlane(min(max(scalar_read(p.tok_offs + b), 0), p.max_off));
  const uint32_t abs_tok0 = PAGED ? (tok_off / kTileTok + blockIdx.x) * kTileTok : 0u;
  int64_t row0 = ((int64_t)b * p.H + h) * p.cap_tokens + tok_off;
  if (PAGED) {
    const int32_t lp = min((int32_t)(abs_tok0 >> p.page_shift), p.table_stride - 1);
    const int32_t phys = min(max(scalar_read(p.block_table + ((int64_t)b * p.table_stride + lp)), 0), p.num_pages - 1);
    row0 = ((((int64_t)phys * p.H + h)) << p.page_shift) + (abs_tok0 & ((1u << p.page_shift) - 1u));
  }
  const uint32_t dst_rows = PAGED ? kTileTok : n;
  const __amdgpu_buffer_rsrc_t src_r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(tp.src) + (int64_t)b * p.stride_b + (int64_t)h * p.stride_h, 0,
      (int)(((int64_t)(n - 1) * p.stride_t + D) * 2), kBufferFlags);
  const __amdgpu_buffer_rsrc_t code_r = __builtin_amdgcn_make_buffer_rsrc(
      tp.codes + row0 * kRowBytes, 0, (int)(dst_rows * kRowBytes), kBufferFlags);
  const __amdgpu_buffer_rsrc_t scale_r = __builtin_amdgcn_make_buffer_rsrc(
      tp.scales + row0 * NB, 0, (int)(dst_rows * NB * 2), kBufferFlags);
  // c0: this lane's first SOURCE chunk.  PAGED: absolute chunk minus the chunks before tok_off;
  // for lanes of the first tile that lie before tok_off this wraps to a huge number: past the
  // end, like the tail.  d0: the same lane's chunk inside the destination descriptor.
  const uint32_t c0 = PAGED ? abs_tok0 * CPR + threadIdx.x - tok_off * CPR
                            : blockIdx.x * (kThreads * kUnroll) + threadIdx.x;
  const uint32_t d0 = PAGED ? threadIdx.x : c0;
  const uint32_t total = n * CPR;

  uint4 w[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t c = c0 + u * kThreads;
    uint32_t voff;
    if (CONTIG) {
      voff = c * 16;                                           // rows back to back
    } else {
      voff = (c / CPR) * (uint32_t)(p.stride_t * 2) + (c % CPR) * 16;
    }
    if (c >= total) voff = kDropStore;                         // past the slab: reads zeros
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(src_r, voff, 0, kNonTemporal);
    w[u] = make_uint4(v.x, v.y, v.z, v.w);
  }

  if (FAST) {
    put_cell(my_cell, cells);
    __syncthreads();
  }

#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t c = c0 + u * kThreads;
    // block scale: max |x| as fp16 bits (for non-negative finite fp16, value order == bit order)
    const uint32_t M = 0x7fff7fffu;
    const uint32_t a = pk_max_u16(pk_max_u16(w[u].x & M, w[u].y & M), pk_max_u16(w[u].z & M, w[u].w & M));
    uint32_t s_bits = max(a & 0xffffu, a >> 16);
    s_bits = max(s_bits, dpp<kQuadXor1>(s_bits));
    s_bits = max(s_bits, dpp<kQuadXor2>(s_bits));
    s_bits = max(s_bits, dpp<kRowHalfMirror>(s_bits));
    if (LPB == 16) s_bits = max(s_bits, dpp<kRowMirror>(s_bits));

    const uint32_t packed = encode_chunk<KBITS, FAST>(w[u], s_bits, p.levels, cells);
    const bool live = c < total;
    const uint32_t dc = d0 + u * kThreads;               // chunk inside the destination descriptor
    if (KBITS == 4) {
      __builtin_amdgcn_raw_buffer_store_b32(packed, code_r, live ? dc * 4 : kDropStore, 0, kNonTemporal);
    } else if (KBITS == 2) {
      const uint32_t odd = dpp<kQuadOdd>(packed);
      const bool writer = live && !(threadIdx.x & 1);
      __builtin_amdgcn_raw_buffer_store_b32(packed | (odd << 16), code_r, writer ? dc * 2 : kDropStore, 0, kNonTemporal);
    } else {  // KBITS == 3: four lanes hold 4 x 24 bits = three dwords
      const uint32_t next = dpp<kQuadNext>(packed);
      const uint32_t q = threadIdx.x & 3;
      const uint32_t word = (packed >> (8 * q)) | (next << (24 - 8 * q));
      const bool writer = live && q != 3;
      __builtin_amdgcn_raw_buffer_store_b32(word, code_r, writer ? (dc >> 2) * 12 + q * 4 : kDropStore, 0, kNonTemporal);
    }
    const bool scale_writer = live && (dc % LPB) == 0;
    __builtin_amdgcn_raw_buffer_store_b16((unsigned short)s_bits, scale_r, scale_writer ? (dc / LPB) * 2 : kDropStore, 0, 0);
  }
}

// Blocks over the token's hidden vector (the paper's own geometry: a block is a fixed number of
// consecutive elements of the token's H*D hidden vector, 256 in its experiments), for caches
// that keep one scale per token-head.  grid: x = block position in the token, y = token tiles,
// z = b + B * tensor.  A workgroup takes ONE block position (LPB = 16 or 32 chunk lanes, i.e. 2 or 4
// heads of 64, 1 or 2 of 128) for a run of consecutive tokens: the half wave (or quarter) that
// holds a block reads its 256 or 512 contiguous source bytes, and for each head the code rows
// of consecutive tokens -- adjacent in the cache -- are written by the same workgroup in one
// run.  The block's max |x| is all-reduced with DPP inside 16-lane rows plus one ds_swizzle
// across the two rows of a half wave.  The source may be token-major ([B,S,H*D]: stride_h = D)
// or any other strided view; the block's scale goes to every head it covers.
template <int KBITS, int D, int LPB, bool FAST>
__global__ __launch_bounds__(kThreads) void quantize_hidden_kernel(const QuantParams p) {
  constexpr uint32_t CPH = D / 8;              // chunks per head row
  constexpr uint32_t HPB = LPB / CPH;          // heads per block
  constexpr uint32_t TOK = kThreads / LPB;     // tokens per pass of the workgroup
  constexpr uint32_t kRowBytes = D * KBITS / 8;
  __shared__ uint2 cells[FAST ? 128 : 1];
  const uint2 my_cell = FAST ? fetch_cell(p.cell_thr, p.cell_below) : make_uint2(0, 0);

  const uint32_t H = (uint32_t)p.H, n = (uint32_t)p.n_tokens;
  const uint32_t blk = blockIdx.x;
  const uint32_t tensor = blockIdx.z >= (unsigned)p.B ? 1u : 0u;
  const uint32_t b = blockIdx.z - (tensor ? (uint32_t)p.B : 0u);
  const TensorPtrs tp = p.t[tensor];
  const int64_t bh0 = (int64_t)b * H;
  const __amdgpu_buffer_rsrc_t src_r = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(tp.src) + (int64_t)b * p.stride_b, 0,
      (int)((((int64_t)H - 1) * p.stride_h + ((int64_t)n - 1) * p.stride_t + D) * 2), kBufferFlags);
  const __amdgpu_buffer_rsrc_t code_r = __builtin_amdgcn_make_buffer_rsrc(
      tp.codes + bh0 * p.cap_tokens * kRowBytes, 0, (int)((int64_t)H * p.cap_tokens * kRowBytes), kBufferFlags);
  const __amdgpu_buffer_rsrc_t scale_r = __builtin_amdgcn_make_buffer_rsrc(
      tp.scales + bh0 * p.cap_tokens, 0, (int)((int64_t)H * p.cap_tokens * 2), kBufferFlags);

  const uint32_t cib = threadIdx.x % LPB;                    // chunk inside the block
  const uint32_t head = blk * HPB + cib / CPH, part = cib % CPH;
  const uint32_t t_first = blockIdx.y * (TOK * kUnroll) + threadIdx.x / LPB;
  const uint32_t src_lane = head * (uint32_t)(p.stride_h * 2) + part * 16;

  uint4 w[kUnroll];
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t t = t_first + u * TOK;
    const uint32_t voff = t < n ? src_lane + t * (uint32_t)(p.stride_t * 2) : kDropStore;   // past the end: reads zeros
    const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(src_r, voff, 0, kNonTemporal);
    w[u] = make_uint4(v.x, v.y, v.z, v.w);
  }

  if (FAST) {
    put_cell(my_cell, cells);
    __syncthreads();
  }

  // Codes and scales are assembled in LDS as the tile's image of the cache -- per covered head,
  // the rows of the tile's consecutive tokens, which are contiguous in the cache -- and leave
  // from there as fully coalesced dword stores.  (Stored straight from the lanes that produce
  // them, every store instruction scatters eight pieces of 32-64 bytes.)
  constexpr uint32_t TILE_TOK = TOK * kUnroll;                // tokens per workgroup
  constexpr uint32_t kHeadDwords = TILE_TOK * kRowBytes / 4;   // one head's rows of the tile
  constexpr uint32_t kHeadPitch = kHeadDwords + 8;             // LDS pitch: heads land on different banks
  __shared__ uint32_t stage[HPB * kHeadPitch];
  __shared__ uint16_t stage_scale[HPB * TILE_TOK];
  const uint32_t h_local = cib / CPH, t_local0 = threadIdx.x / LPB;
#pragma unroll
  for (int u = 0; u < kUnroll; ++u) {
    const uint32_t M = 0x7fff7fffu;
    const uint32_t a = pk_max_u16(pk_max_u16(w[u].x & M, w[u].y & M), pk_max_u16(w[u].z & M, w[u].w & M));
    uint32_t s_bits = max(a & 0xffffu, a >> 16);
    s_bits = max(s_bits, dpp<kQuadXor1>(s_bits));
    s_bits = max(s_bits, dpp<kQuadXor2>(s_bits));
    s_bits = max(s_bits, dpp<kRowHalfMirror>(s_bits));
    s_bits = max(s_bits, dpp<kRowMirror>(s_bits));
    if (LPB == 32) s_bits = max(s_bits, (uint32_t)__builtin_amdgcn_ds_swizzle((int)s_bits, 0x401F));   // lane ^ 16

    const uint32_t packed = encode_chunk<KBITS, FAST>(w[u], s_bits, p.levels, cells);
    const uint32_t t_local = t_local0 + u * TOK;
    uint32_t* row = stage + h_local * kHeadPitch + t_local * (kRowBytes / 4);
    if (KBITS == 4) {
      row[part] = packed;
    } else if (KBITS == 2) {
      const uint32_t odd = dpp<kQuadOdd>(packed);
      if (!(threadIdx.x & 1)) row[part >> 1] = packed | (odd << 16);
    } else {  // KBITS == 3: four lanes hold 4 x 24 bits = three dwords
      const uint32_t next = dpp<kQuadNext>(packed);
      const uint32_t q4 = threadIdx.x & 3;
      const uint32_t word = (packed >> (8 * q4)) | (next << (24 - 8 * q4));
      if (q4 != 3) row[(part >> 2) * 3 + q4] = word;
    }
    if (part == 0) stage_scale[h_local * TILE_TOK + t_local] = (uint16_t)s_bits;   // once per covered head
  }
  __syncthreads();

  const uint32_t tile_t0 = blockIdx.y * TILE_TOK;
  const uint32_t row0 = (blk * HPB) * (uint32_t)p.cap_tokens + (uint32_t)p.tok_off + tile_t0;   // head 0 of the block, first token
#pragma unroll
  for (uint32_t i0 = 0; i0 < HPB * kHeadDwords; i0 += kThreads) {
    const uint32_t i = i0 + threadIdx.x;
    const uint32_t hl = i / kHeadDwords, off = i % kHeadDwords;          // head of the block, dword inside its rows
    const bool live = tile_t0 + off / (kRowBytes / 4) < n;
    const uint32_t voff = (row0 + hl * (uint32_t)p.cap_tokens) * kRowBytes + off * 4;
    __builtin_amdgcn_raw_buffer_store_b32(stage[hl * kHeadPitch + off], code_r, live ? voff : kDropStore, 0, kNonTemporal);
  }
  if (threadIdx.x < HPB * TILE_TOK) {
    const uint32_t hl = threadIdx.x / TILE_TOK, tl = threadIdx.x % TILE_TOK;
    const bool live = tile_t0 + tl < n;
    __builtin_amdgcn_raw_buffer_store_b16(stage_scale[threadIdx.x], scale_r,
                                          live ? (row0 + hl * (uint32_t)p.cap_tokens + tl) * 2 : kDropStore, 0, 0);
  }
}

template <int KBITS, int D>
hipError_t launch_hidden_one(const QuantParams& p, int lanes_per_block, hipStream_t stream) {
  const int heads_per_block = lanes_per_block / (D / 8);
  const int tokens_per_wg = (kThreads / lanes_per_block) * kUnroll;
  // x = block position (fastest), so that workgroups running side by side read one token row
  // end to end rather than one 256- or 512-byte stripe of many rows
  const dim3 grid((unsigned)(p.H / heads_per_block),
                  (unsigned)((p.n_tokens + tokens_per_wg - 1) / tokens_per_wg), (unsigned)(p.B * p.n_tensors));
  const bool fast = p.impl == 0;
  if (lanes_per_block == 32) {
    if (fast) hipLaunchKernelGGL((quantize_hidden_kernel<KBITS, D, 32, true>), grid, dim3(kThreads), 0, stream, p);
    else      hipLaunchKernelGGL((quantize_hidden_kernel<KBITS, D, 32, false>), grid, dim3(kThreads), 0, stream, p);
  } else {
    if constexpr (D == 64) {
      if (fast) hipLaunchKernelGGL((quantize_hidden_kernel<KBITS, D, 16, true>), grid, dim3(kThreads), 0, stream, p);
      else      hipLaunchKernelGGL((quantize_hidden_kernel<KBITS, D, 16, false>), grid, dim3(kThreads), 0, stream, p);
    } else {
      return hipErrorInvalidValue;      // a 128-element block is one head of 128: the ordinary quantizer
    }
  }
  return hipGetLastError();
}

// Tile shapes of the slab kernel: workgroups of 256 lanes taking 4 chunks each (64 tokens of a
// 128-wide head per workgroup), or of 128 lanes taking 2 (16 tokens).  Measured on MI355X, K and V
// in one launch, 4 bits (3 and 2 alike), large / small tile:
//   B16 H56 D128 S16384   1.48-1.51 ms / 1.41-1.42 ms     (block 128: 1.50-1.53 / 1.42)
//   B1  H32 D128 S32768   106.7 us     / 107.2 us
//   B32 H32 D128 S2048    213 us       / 220 us
//   B8  H32 D64  S2048    28.8 us      / 28.8 us
// The small tile interleaves the read and the write stream more finely, which the memory system
// rewards on long runs; short slabs prefer fewer, larger workgroups.  Long runs (8192 tokens per
// slab and more) take the small tile.  (Register counts -- 47 against 37 -- allow full occupancy
// either way; 128 lanes x 3 or 256 x 2 land in between, 512 x 1 and 256 x 1 are 10-20 % slower.)
constexpr int kLargeTileThreads = 256, kLargeTileUnroll = 4;
constexpr int kSmallTileThreads = 128, kSmallTileUnroll = 2;
constexpr int64_t kSmallTileFromTokens = 8192;

template <int KBITS, int D, int BLK, bool PAGED, int THREADS, int UNROLL>
void launch_slab(const QuantParams& p, dim3 grid, hipStream_t stream) {
  const bool fast = p.impl == 0, contig = p.stride_t == D;
  if (fast && contig)       hipLaunchKernelGGL((quantize_slab_kernel<KBITS, D, BLK, true, true, PAGED, THREADS, UNROLL>), grid, dim3(THREADS), 0, stream, p);
  else if (fast)            hipLaunchKernelGGL((quantize_slab_kernel<KBITS, D, BLK, true, false, PAGED, THREADS, UNROLL>), grid, dim3(THREADS), 0, stream, p);
  else if (contig)          hipLaunchKernelGGL((quantize_slab_kernel<KBITS, D, BLK, false, true, PAGED, THREADS, UNROLL>), grid, dim3(THREADS), 0, stream, p);
  else                      hipLaunchKernelGGL((quantize_slab_kernel<KBITS, D, BLK, false, false, PAGED, THREADS, UNROLL>), grid, dim3(THREADS), 0, stream, p);
}

template <int KBITS, int D, int BLK>
hipError_t launch_one(const QuantParams& p, hipStream_t stream) {
  constexpr int CPR = D / 8;
  const int64_t chunks_per_slab = p.n_tokens * CPR;
  // few tokens per (b,h): one flat grid over all rows (its chunk index is a 32-bit number)
  const bool flat = chunks_per_slab < 2 * kThreads && chunks_per_slab * p.B * p.H < ((int64_t)1 << 31);
  if (flat) {
    const int tile = kThreads * kUnroll;
    const int64_t total = chunks_per_slab * p.B * p.H;
    const dim3 grid((unsigned)((total + tile - 1) / tile), 1, (unsigned)p.n_tensors);
    if (p.impl == 0) hipLaunchKernelGGL((quantize_kernel<KBITS, D, BLK, true, true>), grid, dim3(kThreads), 0, stream, p);
    else             hipLaunchKernelGGL((quantize_kernel<KBITS, D, BLK, false, true>), grid, dim3(kThreads), 0, stream, p);
  } else if (p.n_tokens >= kSmallTileFromTokens) {
    constexpr int tile = kSmallTileThreads * kSmallTileUnroll;
    launch_slab<KBITS, D, BLK, false, kSmallTileThreads, kSmallTileUnroll>(
        p, dim3((unsigned)((chunks_per_slab + tile - 1) / tile), (unsigned)p.H, (unsigned)(p.B * p.n_tensors)), stream);
  } else {
    constexpr int tile = kLargeTileThreads * kLargeTileUnroll;
    launch_slab<KBITS, D, BLK, false, kLargeTileThreads, kLargeTileUnroll>(
        p, dim3((unsigned)((chunks_per_slab + tile - 1) / tile), (unsigned)p.H, (unsigned)(p.B * p.n_tensors)), stream);
  }
  return hipGetLastError();
}

template <int KBITS>
hipError_t launch_k(const QuantParams& p, int D, int blk, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_one<KBITS, 64, 64>(p, stream);
  if (D == 128 && blk == 64) return launch_one<KBITS, 128, 64>(p, stream);
  if (D == 128 && blk == 128) return launch_one<KBITS, 128, 128>(p, stream);
  return hipErrorInvalidValue;
}

}  // namespace

namespace {
template <int KBITS, int D, int BLK, int THREADS, int UNROLL>
hipError_t launch_paged_tile(const QuantParams& p, hipStream_t stream) {
  constexpr int kTileTok = THREADS * UNROLL / (D / 8);       // 16 .. 128: divides every page size
  // tiles lie over absolute token positions: the run [tok_off, tok_off + n) touches last - first + 1
  // of them; with per-sequence offsets, as many as a run of n tokens can touch at worst (workgroups
  // past a sequence's run find nothing to do)
  const int64_t first = p.tok_off / kTileTok, last = (p.tok_off + p.n_tokens - 1) / kTileTok;
  const int64_t tiles = p.tok_offs ? (p.n_tokens - 1 + kTileTok - 1) / kTileTok + 1 : last - first + 1;
  launch_slab<KBITS, D, BLK, true, THREADS, UNROLL>(p, dim3((unsigned)tiles, (unsigned)p.H, (unsigned)(p.B * p.n_tensors)), stream);
  return hipGetLastError();
}

template <int KBITS, int D, int BLK>
hipError_t launch_paged_one(const QuantParams& p, hipStream_t stream) {
  if (p.n_tokens >= kSmallTileFromTokens) return launch_paged_tile<KBITS, D, BLK, kSmallTileThreads, kSmallTileUnroll>(p, stream);
  return launch_paged_tile<KBITS, D, BLK, kLargeTileThreads, kLargeTileUnroll>(p, stream);
}

template <int KBITS>
hipError_t launch_paged_k(const QuantParams& p, int D, int blk, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_paged_one<KBITS, 64, 64>(p, stream);
  if (D == 128 && blk == 64) return launch_paged_one<KBITS, 128, 64>(p, stream);
  if (D == 128 && blk == 128) return launch_paged_one<KBITS, 128, 128>(p, stream);
  return hipErrorInvalidValue;
}
}  // namespace

hipError_t launch_quantize_paged(const QuantParams& p, int D, int k, int blk, hipStream_t stream) {
  switch (k) {
    case 2: return launch_paged_k<2>(p, D, blk, stream);
    case 3: return launch_paged_k<3>(p, D, blk, stream);
    case 4: return launch_paged_k<4>(p, D, blk, stream);
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_quantize_hidden(const QuantParams& p, int D, int k, int blk_hidden, hipStream_t stream) {
  const int lpb = blk_hidden / 8;
  if (lpb != 16 && lpb != 32) return hipErrorInvalidValue;
  if (D == 64) {
    switch (k) {
      case 2: return launch_hidden_one<2, 64>(p, lpb, stream);
      case 3: return launch_hidden_one<3, 64>(p, lpb, stream);
      case 4: return launch_hidden_one<4, 64>(p, lpb, stream);
    }
  } else if (D == 128) {
    switch (k) {
      case 2: return launch_hidden_one<2, 128>(p, lpb, stream);
      case 3: return launch_hidden_one<3, 128>(p, lpb, stream);
      case 4: return launch_hidden_one<4, 128>(p, lpb, stream);
    }
  }
  return hipErrorInvalidValue;
}

hipError_t launch_quantize(const QuantParams& p, int D, int k, int blk, hipStream_t stream) {
  switch (k) {
    case 2: return launch_k<2>(p, D, blk, stream);
    case 3: return launch_k<3>(p, D, blk, stream);
    case 4: return launch_k<4>(p, D, blk, stream);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace nqkv
