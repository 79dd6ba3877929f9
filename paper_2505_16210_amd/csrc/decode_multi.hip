// Dequantize-fused attention of SEVERAL new queries per sequence over the packed cache: the
// decoding-phase equations of paper Sec. 3.2 (A = Softmax(t_Q X_K'^T), t_O = A X_V') for the
// case where a step appends q_len > 1 tokens to the append-only cache (Sec. 1) and each of them
// needs its output -- query i sees the cache up to and including its own token.
//
// With up to 16 query rows per head the two products are real (if skinny) matrix products, so
// they run on the matrix cores, fp32 accumulate: v_mfma_f32_16x16x32_f16.  The table look-up that
// turns codes into fp16 levels is the same byte-indexed LDS table as in the one-query kernel and costs
// the same per cached element whatever q_len is; the arithmetic that the one-query kernel spends
// vector instructions on (dot products, weighted sums) moves to the matrix pipe.
//
// Operand layouts (lane l, i16 = l % 16, gq = l / 16):
//   A[row i16][k = 8 gq + 0..7],  B[k = 8 gq + 0..7][col i16],  C/D[row 4 gq + 0..3][col i16].
//
// Scores.   C1[token][query] = sum_d K[token][d] q[query][d]:  A = levels of a 16-token tile of
//   K (row = token i16), B = q^T.  One instruction contracts over 32 head-dim elements of one
//   64-element chunk, this lane's being  64 c + 16 a + 8 h + 0..7  for half h (a = gq, or a fixed
//   permutation of it, see load_k), so a lane needs 8 contiguous code bytes per chunk (dword h is
//   one operand) and the chunk lies inside one quantization block; the block scale of the token
//   multiplies C1 afterwards, in fp32 (a lane fetches the scales of one token of its quad of
//   rows, the quad shares them by DPP).
// Softmax.  A lane holds scores of tokens 4 gq + r (r = 0..3) of the tile for query i16: the
//   running maximum and sum are per lane (= per query), reduced over gq with lane swaps.
// Output.   O^T[d][query] = sum_token V[token][d] P[token][query]:  B = P^T is exactly the layout
//   C1 came out in (k = token 4 gq + r, col = query), converted to fp16 after multiplying in
//   the token's V block scale; one instruction contracts over the 32 tokens of two tiles (this
//   lane's eight: 4 gq + 0..3 of each).  A = V^T needs, per lane, one head-dim element of those
//   eight tokens; a look-up yields two adjacent elements of ONE token, so eight look-ups (the same
//   code byte of each token) are re-paired with v_perm_b32 into the operands of two instructions
//   (even and odd element).  Rows of one instruction are the 16 code bytes
//   4 (i16 % 8) + G + 2 (i16 / 8)  (G = 0, 1) of a 32-byte chunk, so that they too stay inside
//   one quantization block.
//
// 2-bit codes: a code byte holds four elements, so on the K side one look-up (two dwords) is a
// whole operand, and on the V side row i16 is code byte i16 of a 16-byte chunk: one look-up per
// token, re-paired into the operands of four instructions (element % 4).
//
// 3-bit codes: pairs of codes are 6-bit fields that do not align with bytes.  K side: the lane's
// 16 elements are 48 bits starting at byte 6 gq of the 24-byte chunk.  V side: row i16 is fields
// 2 i16 and 2 i16 + 1 (12 bits at bit 12 i16), which may straddle a dword: two staged dwords and a
// 64-bit shift per look-up pair.
//
// Work split: one workgroup of eight waves per (sequence, split); waves take 32-token trips
// round-robin; per-wave results (m, l per query, O) meet in LDS in the space of the look-up
// table, which is no longer needed then; with splits > 1 a second small kernel combines the
// partial results in split order.
#include <type_traits>

#include "decode_common.h"
#include "nqkv_internal.h"
#include "scalar_read.h"

namespace nqkv {
namespace {

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kTile = 16;                // tokens per matrix tile
constexpr int kTilesPerTrip = 2;
constexpr int kTrip = kTile * kTilesPerTrip;
constexpr int kSplitUnit = 32;           // split boundaries are multiples of this many tokens
constexpr int kMaxQ = 16;

typedef float float4_t __attribute__((ext_vector_type(4)));

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
// v_mfma_f32_16x16x32_f16: eight fp16 per lane and operand (four dwords)
__device__ __forceinline__ float4_t mfma32(const uint32_t (&a)[4], const uint32_t (&b)[4], float4_t c) {
  const u32x4_t av = {a[0], a[1], a[2], a[3]}, bv = {b[0], b[1], b[2], b[3]};
  return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(half8_t, av), __builtin_bit_cast(half8_t, bv), c, 0, 0, 0);
}

// All-reduce over the four 16-lane rows of a wave (lane bits 4 and 5): v_permlane32_swap exchanges
// lanes 32..63 of its first operand with lanes 0..31 of its second, v_permlane16_swap the odd rows
// of the first with the even rows of the second; fed two copies of x, the two results hold the
// two halves side by side.  (Inline assembly for the reason given in the one-query kernel; the
// s_nop covers the wait states after a VALU write of the operands.)
template <class Op>
__device__ __forceinline__ float allreduce_rows(float x, Op op) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  x = op(a, b);
  a = x; b = x;
  asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1" : "+v"(a), "+v"(b));
  return op(a, b);
}

__device__ __forceinline__ float half_lo(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w & 0xffffu)); }
__device__ __forceinline__ float half_hi(uint32_t w) { return (float)__builtin_bit_cast(_Float16, (unsigned short)(w >> 16)); }
__device__ __forceinline__ uint32_t pack_half2(float lo, float hi) {
  const half2_t h = {(_Float16)lo, (_Float16)hi};      // round to nearest even
  return __builtin_bit_cast(uint32_t, h);
}

template <int KBITS, int D, int BLK, bool PAGED>
__global__ __launch_bounds__(kThreads) __attribute__((amdgpu_waves_per_eu(4, 4)))     // 128 registers: two workgroups per CU
void decode_multi_kernel(const MultiParams p) {
  constexpr int KW = (KBITS == 2) ? 1 : 2;   // K side: dwords of codes per lane, chunk and token (16 elements)
  constexpr int TPT = kTilesPerTrip;
  static_assert(TPT % 2 == 0, "the value product contracts over two 16-token tiles");
  constexpr int TRIP = kTile * TPT;
  constexpr int NC = D / 64;                 // 64-element chunks of a row
  // Two chunks per row, whole bytes per lane: the lane's codes of BOTH chunks come with one load
  // (see load_k), so that a load instruction consumes whole rows.
  constexpr bool kWideK = D == 128 && KBITS != 3;
  constexpr int NB = D / BLK;                // quantization blocks of a row
  constexpr int CPB = BLK / 64;              // chunks per block
  constexpr uint32_t kRowBytes = D * KBITS / 8, kChunkBytes = 8 * KBITS, kScaleRowBytes = NB * 2;
  constexpr int XS = D + 1;                  // padded row of the merge buffer
  constexpr uint32_t kTileBytes = kTile * kRowBytes;          // one 16-token tile of value codes
  // Streaming phase: the table and, per wave, a staging area for the value tiles of a trip.
  // Merge phase (everything above is dead by then): the per-wave results.  80 KiB at D 128, 4 bits:
  // two workgroups fill the 160 KiB of a compute unit exactly.
  struct Lds {
    union {
      struct {
        __attribute__((aligned(256))) uint32_t lut[kLutWords];
        uint32_t stage[kWaves][TPT][kTileBytes / 4];
      };
      struct {
        float xo[kWaves][kMaxQ][XS];
        float wm[kWaves][kMaxQ], wl[kWaves][kMaxQ];
      };
    };
  };
  __shared__ Lds lds;
  const char* lut = reinterpret_cast<const char*>(lds.lut);

  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t i16 = lane & 15, gq = lane >> 4;
  const uint32_t lane_off = (KBITS == 4) ? (lane << 2) : (KBITS == 2) ? ((lane & 31) << 3) : ((lane & 31) << 2);
  // V side: the two code bytes of its dword this lane looks up (see the row mapping above)
  // (k = 2: a byte holds four elements, the lane looks up byte i16 % 4 of dword i16 / 4)
  const uint32_t vsel0 = 0x0c0c0000u | ((4u + (KBITS == 4 ? 2u * (i16 >> 3) : (i16 & 3u))) << 8);
  const uint32_t vsel1 = vsel0 + 0x100u;

  // ---- item geometry
  const uint32_t item = blockIdx.x;
  uint32_t bh = item / (uint32_t)p.splits;
  const uint32_t sp = item - bh * (uint32_t)p.splits;
  if (p.longest_first) {
    // Ragged batch, more workgroups than can be resident: item / (H * splits) is a RANK, and the
    // sequence is the one whose length has that rank (ties by index), so that the long sequences
    // are dispatched first and the short ones fill the tail of the grid.  Lane l holds the length
    // of sequence l (at most 64 of them); its rank is the number of sequences that come before it.
    const uint32_t nb = (uint32_t)p.n_seqs, rank = bh / (uint32_t)p.H, h = bh - rank * (uint32_t)p.H;
    int32_t len_l = -1;
    if (lane < nb) len_l = min(max(p.seq_lens[lane], p.q_len), p.seq_len);
    uint32_t before = 0;
    for (uint32_t s = 0; s < nb; ++s) {
      const int32_t len_s = __builtin_amdgcn_readlane(len_l, (int)s);
      before += (len_s > len_l || (len_s == len_l && s < lane)) ? 1u : 0u;
    }
    const uint64_t hit = __builtin_amdgcn_ballot_w64(lane < nb && before == rank);
    const uint32_t b = hit ? (uint32_t)__builtin_ctzll(hit) : rank;     // exactly one lane: the ranks are a permutation
    bh = b * (uint32_t)p.H + h;
  }
  // splits are whole 32-token pieces
  const int32_t u0 = (int32_t)sp * p.split_base + min((int32_t)sp, p.split_rem);
  const int32_t t0 = u0 * kSplitUnit;
  // the sequence's own length when the batch is ragged (whatever the array holds, stay inside
  // [q_len, the length the host planned for]); pieces past its end are empty
  int32_t seq_len = p.seq_len;
  if (p.seq_lens) seq_len = __builtin_amdgcn_readfirstlane(min(max(scalar_read(p.seq_lens + bh / (uint32_t)p.H), p.q_len), p.seq_len));
  const int32_t n_tok = max(min((p.split_base + ((int32_t)sp < p.split_rem ? 1 : 0)) * kSplitUnit, seq_len - t0), 0);
  // PAGED: the cache is a pool of pages behind a block table; descriptors are made per trip
  // (page_trip below) and this row is not used
  const int64_t row0 = PAGED ? 0 : (int64_t)bh * p.cap_tokens + t0;
  // item-relative token limit of this lane's query: query i sees tokens [0, seq_len - q_len + 1 + i)
  const int32_t qi = min((int32_t)i16, p.q_len - 1);
  const int32_t lim = min(n_tok, seq_len - p.q_len + 1 + qi - t0);
  const int32_t lim_first = seq_len - p.q_len + 1 - t0;             // query 0's, uniform

  const int scale_bytes = PAGED ? 0 : n_tok * (int)kScaleRowBytes;
  const __amdgpu_buffer_rsrc_t kc_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.k_codes) + row0 * kRowBytes, 0, PAGED ? 0 : n_tok * (int)kRowBytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t vc_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.v_codes) + row0 * kRowBytes, 0, PAGED ? 0 : n_tok * (int)kRowBytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t ks_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.k_scales) + row0 * NB, 0, scale_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t vs_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.v_scales) + row0 * NB, 0, scale_bytes, kBufferFlags);
  const __amdgpu_buffer_rsrc_t q_r = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.q) + (int64_t)bh * p.q_len * D, 0, p.q_len * D * 2, kBufferFlags);

  // per-lane byte offsets inside a tile (the trip and tile offsets are added to them: only the
  // vector offset takes part in the hardware range check, and rows past the item read zeros)
  // k = 3: the lane's 48 bits of a K row (16 elements) start at byte 6 gq of the chunk -- a 64-bit
  // load from the dword below it, shifted by 0 or 16; its 12 bits of a V row (fields 2 i16 and
  // 2 i16 + 1 of the chunk) start at bit 12 i16 -- a 64-bit load from dword min(12 i16 / 32, 4)
  const uint32_t v3_dw = min((12u * i16) >> 5, 4u);
  const uint32_t k3_shift = (gq & 1u) * 16u, v3_shift = 12u * i16 - 32u * v3_dw;
  const uint32_t k_voff = i16 * kRowBytes + (KBITS == 3 ? ((6u * gq) & ~3u) : gq * (4u * KW) * (kWideK ? 2u : 1u));      // + c * kChunkBytes
  // kWideK: lane group gq fetches bytes [8 KW gq, 8 KW (gq + 1)) of the row -- the 4 KW-byte units
  // 2 gq and 2 gq + 1 of the row's eight -- and v_permlane32_swap (lanes 32..63 of the first
  // operand <-> lanes 0..31 of the second) then leaves group gq with units a and a + 4, a = aq:
  // its 16 elements of chunk 0 and of chunk 1, as the operand layout wants, for the unit a below.
  const uint32_t aq = kWideK ? ((gq >> 1) | ((gq & 1u) << 1)) : gq;
  // Value codes go through LDS: a tile (16 consecutive rows, contiguous in the cache) is fetched
  // with ONE 128-bit load per lane -- lane L takes bytes [16 L, 16 L + 16) of the tile -- and
  // written to this wave's staging area, from which every lane reads the dwords the matrix-operand
  // layout wants (token 4 gq + e, dword v_dw of chunk c).  Fetching those dwords straight from
  // memory costs one load instruction per lane and token (2.4x the memory instructions of the
  // whole kernel, which is what bound it at 2 and 3 bits) and takes every cache line in pieces,
  // which rules out the non-temporal hint.  Inside each group of four rows the rows are stored
  // permuted (row e of group g at slot e ^ g), so that the four lane groups gq, which read rows
  // 64 or 32 bytes apart, spread over the banks; 3-bit rows (48 / 24 bytes) stay in place.
  constexpr bool kSwizzle = KBITS != 3;
  const uint32_t v_dw = (KBITS == 4) ? (i16 & 7u) : (KBITS == 2) ? (i16 >> 2) : v3_dw;
  const uint32_t st_byte = lane * 16u;                           // this lane's bytes of a tile
  const bool st_live = st_byte < kTileBytes;
  uint32_t st_addr = st_byte;
  if (kSwizzle) {
    const uint32_t t = st_byte / kRowBytes;
    st_addr = ((t & ~3u) | ((t & 3u) ^ ((t >> 2) & 3u))) * kRowBytes + st_byte % kRowBytes;
  }
  uint32_t* const st_wave = &lds.stage[wave][0][0];
  const char* rd_row[4];                                         // staged row of token 4 gq + e, at this lane's dword
#pragma unroll
  for (int e = 0; e < 4; ++e)
    rd_row[e] = reinterpret_cast<const char*>(st_wave) + (4u * gq + (kSwizzle ? (e ^ gq) : (uint32_t)e)) * kRowBytes + v_dw * 4u;
  // scales: lane (i16, gq) fetches those of token 4 gq + i16 % 4 only; the quad shares them by DPP
  const uint32_t s_voff = (4u * gq + (i16 & 3u)) * kScaleRowBytes;

  uint32_t kw[TPT][NC][KW];
  u32x4_t vst[TPT];                      // value tiles on their way to the staging area
  uint32_t ksr[TPT], vsr[TPT];

  auto load_scales = [&](__amdgpu_buffer_rsrc_t r, uint32_t voff) -> uint32_t {
    if constexpr (NB == 1) return __builtin_amdgcn_raw_buffer_load_b16(r, voff, 0, 0);
    else return __builtin_amdgcn_raw_buffer_load_b32(r, voff, 0, 0);
  };
  // PAGED: pool rows of the trip that starts at item-relative token tb.  Items and trips start at
  // multiples of 32 tokens and a page is a larger power of two, so a trip never straddles two
  // pages.  Table index and entry are clamped: nothing the table holds (and no trip past the end
  // of the sequence, whose row count is 0) can address memory outside the pool.
  int64_t trip_rows = 0;
  int32_t trip_left = 0;
  auto page_trip = [&](int32_t tb) {
    const uint32_t b = bh / (uint32_t)p.H, h = bh - b * (uint32_t)p.H;
    const int32_t tok = t0 + tb;
    const int32_t lp = min(tok >> p.page_shift, p.table_stride - 1);
    // (the clamps select as vector instructions: readfirstlane brings the results back to scalar
    // registers, so that the row arithmetic and the descriptors built from it stay scalar)
    const int32_t phys = __builtin_amdgcn_readfirstlane(min(max(scalar_read(p.block_table + ((int64_t)b * p.table_stride + lp)), 0), p.num_pages - 1));
    trip_rows = ((((int64_t)phys * p.H + h)) << p.page_shift) + (tok & ((1 << p.page_shift) - 1));
    trip_left = __builtin_amdgcn_readfirstlane(min(max(n_tok - tb, 0), TRIP));
  };
  auto load_k = [&](int32_t tb) {
    __amdgpu_buffer_rsrc_t cr = kc_r, sr = ks_r;
    if constexpr (PAGED) {
      page_trip(tb);
      cr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.k_codes) + trip_rows * kRowBytes, 0, trip_left * (int)kRowBytes, kBufferFlags);
      sr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.k_scales) + trip_rows * NB, 0, trip_left * (int)kScaleRowBytes, kBufferFlags);
      tb = 0;
    }
#pragma unroll
    for (int u = 0; u < TPT; ++u) {
      const uint32_t tok = (uint32_t)tb + u * kTile;
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        if constexpr (kWideK) {
          if (c == 0) {
            if constexpr (KBITS == 4) {
              const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(cr, k_voff + tok * kRowBytes, 0, kStreamOnce);
              kw[u][0][0] = v.x; kw[u][0][1] = v.y; kw[u][1][0] = v.z; kw[u][1][1] = v.w;
            } else {
              const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(cr, k_voff + tok * kRowBytes, 0, kStreamOnce);
              kw[u][0][0] = v.x; kw[u][1][0] = v.y;
            }
          }
        } else if constexpr (KBITS != 2) {
          const u32x2_t v = __builtin_amdgcn_raw_buffer_load_b64(cr, k_voff + tok * kRowBytes + c * kChunkBytes, 0, NC == 1 ? kStreamOnce : 0);
          kw[u][c][0] = v.x; kw[u][c][1] = v.y;
        } else {
          kw[u][c][0] = __builtin_amdgcn_raw_buffer_load_b32(cr, k_voff + tok * kRowBytes + c * kChunkBytes, 0, NC == 1 ? kStreamOnce : 0);
        }
      }
      ksr[u] = load_scales(sr, s_voff + tok * kScaleRowBytes);
    }
  };
  // (PAGED: the V rows of the trip whose K loads went out last -- load_k(tb) always precedes load_v(tb))
  auto load_v = [&](int32_t tb) {
    __amdgpu_buffer_rsrc_t cr = vc_r, sr = vs_r;
    if constexpr (PAGED) {
      cr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(p.v_codes) + trip_rows * kRowBytes, 0, trip_left * (int)kRowBytes, kBufferFlags);
      sr = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.v_scales) + trip_rows * NB, 0, trip_left * (int)kScaleRowBytes, kBufferFlags);
      tb = 0;
    }
#pragma unroll
    for (int u = 0; u < TPT; ++u) {
      const uint32_t tok = (uint32_t)tb + u * kTile;
      // (lanes past the tile, and rows past the item, read zeros: the offset is out of range)
      vst[u] = __builtin_amdgcn_raw_buffer_load_b128(cr, st_live ? tok * kRowBytes + st_byte : 0xffffffffu, 0, kStreamOnce);
      vsr[u] = load_scales(sr, s_voff + tok * kScaleRowBytes);
    }
  };
  // scale of token 4 gq + r, block b: held by lane r of this lane's quad (quad_perm broadcast)
  auto scale_of = [&](uint32_t s, auto r_tag, int b) {
    constexpr int R = decltype(r_tag)::value;
    const uint32_t w = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)s, R * 0x55, 0xf, 0xf, true);
    return b ? half_hi(w) : half_lo(w);
  };
  int32_t base = (int32_t)wave * TRIP;
  load_k(base);
  // the query operand: q[query i16][64 c + 16 aq + 8 h + 0..7] for chunk c, half h -- 32 bytes per chunk;
  // rows beyond q_len read zeros
  uint32_t qb[NC][2][4];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
#pragma unroll
    for (int hlf = 0; hlf < 2; ++hlf) {
      const u32x4_t v = __builtin_amdgcn_raw_buffer_load_b128(q_r, (i16 * D + 64u * c + 16u * aq + 8u * hlf) * 2u, 0, 0);
      qb[c][hlf][0] = v.x; qb[c][hlf][1] = v.y; qb[c][hlf][2] = v.z; qb[c][hlf][3] = v.w;
    }
  }
  build_lut<KBITS>(p, lds.lut);          // ends with a barrier

  float4_t acc[NC][4];                   // k = 4: [chunk][2 G + parity of the element]; k = 2, 3: [chunk][element % 4]
#pragma unroll
  for (int c = 0; c < NC; ++c)
#pragma unroll
    for (int v = 0; v < 4; ++v) acc[c][v] = float4_t{0, 0, 0, 0};
  float m_run = kNoScore;                // this lane's query, log2 domain; equal over gq
  float l_run = 0.0f;                    // over this lane's own tokens only

  constexpr int32_t stride = kWaves * TRIP;
  // One 32-token trip.  FULL: every token of it exists and is visible to every query (all trips but
  // the sequence's last few); the other copy masks per token and query.  Two copies of the whole
  // body rather than branches inside it, so that each is one straight-line scheduling region.
  auto trip_body = [&](auto full_tag) {
    constexpr bool FULL = decltype(full_tag)::value;
    load_v(base);

    // ---- scores of the trip's two tiles
    if constexpr (kWideK) {
      // (the s_nop covers the wait states between a write of the operands and the swap)
#pragma unroll
      for (int u = 0; u < TPT; ++u)
#pragma unroll
        for (int i = 0; i < KW; ++i) asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(kw[u][0][i]), "+v"(kw[u][1][i]));
    }
    float z[TPT][4];
#pragma unroll
    for (int u = 0; u < TPT; ++u) {
      float4_t c1[NB];
#pragma unroll
      for (int b = 0; b < NB; ++b) c1[b] = float4_t{0, 0, 0, 0};
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        if constexpr (KBITS == 4) {
          // dword h of the lane's eight code bytes: elements 8 h .. 8 h + 7 of its sixteen
#pragma unroll
          for (int hlf = 0; hlf < 2; ++hlf) {
            const uint32_t w = kw[u][c][hlf];
            const uint32_t x[4] = {*reinterpret_cast<const uint32_t*>(lut + row_addr<0>(w, lane_off)),
                                   *reinterpret_cast<const uint32_t*>(lut + row_addr<1>(w, lane_off)),
                                   *reinterpret_cast<const uint32_t*>(lut + row_addr<2>(w, lane_off)),
                                   *reinterpret_cast<const uint32_t*>(lut + row_addr<3>(w, lane_off))};
            c1[c / CPB] = mfma32(x, qb[c][hlf], c1[c / CPB]);
          }
        } else if constexpr (KBITS == 3) {
          // eight 6-bit pairs from the lane's 48 bits
          const uint64_t x64 = (((uint64_t)kw[u][c][1] << 32) | kw[u][c][0]) >> k3_shift;
          const uint32_t xw[2] = {(uint32_t)x64, (uint32_t)(x64 >> 32)};
#pragma unroll
          for (int hlf = 0; hlf < 2; ++hlf) {
            uint32_t x[4];
#pragma unroll
            for (int j = 0; j < 4; ++j)
              x[j] = *reinterpret_cast<const uint32_t*>(lut + ((field<2>(xw, 24 * hlf + 6 * j, 6) << 7) | lane_off));
            c1[c / CPB] = mfma32(x, qb[c][hlf], c1[c / CPB]);
          }
        } else {
          // a byte of 2-bit codes is four elements: two look-ups are one operand
          const uint32_t w0 = kw[u][c][0];
          const uint2 y0 = *reinterpret_cast<const uint2*>(lut + row_addr<0>(w0, lane_off));
          const uint2 y1 = *reinterpret_cast<const uint2*>(lut + row_addr<1>(w0, lane_off));
          const uint2 y2 = *reinterpret_cast<const uint2*>(lut + row_addr<2>(w0, lane_off));
          const uint2 y3 = *reinterpret_cast<const uint2*>(lut + row_addr<3>(w0, lane_off));
          const uint32_t xa[4] = {y0.x, y0.y, y1.x, y1.y}, xb[4] = {y2.x, y2.y, y3.x, y3.y};
          c1[c / CPB] = mfma32(xa, qb[c][0], c1[c / CPB]);
          c1[c / CPB] = mfma32(xb, qb[c][1], c1[c / CPB]);
        }
      }
      auto score = [&](auto r_tag) {
        constexpr int r = decltype(r_tag)::value;
        float v = 0.0f;
#pragma unroll
        for (int b = 0; b < NB; ++b) v = __builtin_fmaf(c1[b][r], scale_of(ksr[u], r_tag, b), v);
        v *= p.scale_log2e;
        // tokens past the item or not yet visible to this lane's query
        if (!FULL) v = (base + u * kTile + (int32_t)(4u * gq) + r < lim) ? v : -INFINITY;
        z[u][r] = v;
      };
      score(std::integral_constant<int, 0>{}); score(std::integral_constant<int, 1>{});
      score(std::integral_constant<int, 2>{}); score(std::integral_constant<int, 3>{});
    }
    float m_trip = fmaxf(fmaxf(z[0][0], z[0][1]), fmaxf(z[0][2], z[0][3]));
#pragma unroll
    for (int u = 1; u < TPT; ++u) m_trip = fmaxf(m_trip, fmaxf(fmaxf(z[u][0], z[u][1]), fmaxf(z[u][2], z[u][3])));
    m_trip = allreduce_rows(m_trip, [](float a, float b) { return fmaxf(a, b); });
    const float m_new = fmaxf(m_run, m_trip);
    if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0) {       // uniform: some query's maximum grew
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_new);
#pragma unroll
      for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int v = 0; v < 4; ++v) acc[c][v] *= alpha;
      l_run *= alpha;
      m_run = m_new;
    }
    float pw[TPT][4];
#pragma unroll
    for (int u = 0; u < TPT; ++u)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        pw[u][r] = __builtin_amdgcn_exp2f(z[u][r] - m_run);
        l_run += pw[u][r];
      }

    load_k(base + stride);      // past the end on the last trip: reads zeros

    // ---- the trip's value tiles: registers -> staging area.  Written and read by different lanes of
    // this one wave: LDS operations of a wave complete in order, the fences keep the compiler from
    // reordering them (and from moving the next trip's writes above this trip's reads).
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int u = 0; u < TPT; ++u)
      if (st_live) *reinterpret_cast<u32x4_t*>(reinterpret_cast<char*>(st_wave) + u * kTileBytes + st_addr) = vst[u];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    auto staged = [&](int u, int c, int e, int word) {
      return *reinterpret_cast<const uint32_t*>(rd_row[e] + u * kTileBytes + c * kChunkBytes + word * 4);
    };

    // ---- weighted values: one instruction contracts over the 32 tokens of two tiles (this lane's
    // eight: 4 gq + 0..3 of each)
    constexpr uint32_t kLo = 0x05040100u, kHi = 0x07060302u;     // v_perm_b32: low / high halves of two dwords
#pragma unroll
    for (int up = 0; up < TPT; up += 2) {
      uint32_t b2[NB][4];       // P^T of the two tiles times the V block scale, fp16
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        const int u = up + t;
        // weights to fp16 pairs first, then one packed multiply per pair and block with the scales
        // of the pair's two tokens (fetched from the quad by DPP, re-paired by v_perm_b32)
        const uint32_t p01 = pack_half2(pw[u][0], pw[u][1]), p23 = pack_half2(pw[u][2], pw[u][3]);
        const uint32_t w0 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)vsr[u], 0x00, 0xf, 0xf, true);
        const uint32_t w1 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)vsr[u], 0x55, 0xf, 0xf, true);
        const uint32_t w2 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)vsr[u], 0xaa, 0xf, 0xf, true);
        const uint32_t w3 = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)vsr[u], 0xff, 0xf, 0xf, true);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
          const uint32_t sel = b ? 0x07060302u : 0x05040100u;
          const uint32_t s01 = __builtin_amdgcn_perm(w1, w0, sel), s23 = __builtin_amdgcn_perm(w3, w2, sel);
          b2[b][2 * t] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, p01) * __builtin_bit_cast(half2_t, s01));
          b2[b][2 * t + 1] = __builtin_bit_cast(uint32_t, __builtin_bit_cast(half2_t, p23) * __builtin_bit_cast(half2_t, s23));
        }
      }
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const uint32_t (&bb)[4] = b2[c / CPB];
        if constexpr (KBITS == 4) {
#pragma unroll
          for (int G = 0; G < 2; ++G) {
            uint32_t h[8];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const uint32_t addr = __builtin_amdgcn_perm(staged(up + t, c, e, 0), lane_off, G ? vsel1 : vsel0);
                h[4 * t + e] = *reinterpret_cast<const uint32_t*>(lut + addr);
              }
            // {h.lo} over the eight tokens -> even element's operand, {h.hi} -> odd element's
            const uint32_t ev[4] = {__builtin_amdgcn_perm(h[1], h[0], kLo), __builtin_amdgcn_perm(h[3], h[2], kLo),
                                    __builtin_amdgcn_perm(h[5], h[4], kLo), __builtin_amdgcn_perm(h[7], h[6], kLo)};
            const uint32_t od[4] = {__builtin_amdgcn_perm(h[1], h[0], kHi), __builtin_amdgcn_perm(h[3], h[2], kHi),
                                    __builtin_amdgcn_perm(h[5], h[4], kHi), __builtin_amdgcn_perm(h[7], h[6], kHi)};
            acc[c][2 * G] = mfma32(ev, bb, acc[c][2 * G]);
            acc[c][2 * G + 1] = mfma32(od, bb, acc[c][2 * G + 1]);
          }
        } else {
          // elements 4 i16 + 0..3 of the chunk: hx = {0, 1}, hy = {2, 3} per token
          uint32_t hx[8], hy[8];
#pragma unroll
          for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              if constexpr (KBITS == 3) {
                // fields 2 i16 and 2 i16 + 1 of the chunk: 12 bits that may straddle a dword
                const uint32_t x = (uint32_t)(((((uint64_t)staged(up + t, c, e, 1)) << 32) | staged(up + t, c, e, 0)) >> v3_shift);
                hx[4 * t + e] = *reinterpret_cast<const uint32_t*>(lut + (((x & 63u) << 7) | lane_off));
                hy[4 * t + e] = *reinterpret_cast<const uint32_t*>(lut + ((((x >> 6) & 63u) << 7) | lane_off));
              } else {
                const uint32_t addr = __builtin_amdgcn_perm(staged(up + t, c, e, 0), lane_off, vsel0);
                const uint2 y = *reinterpret_cast<const uint2*>(lut + addr);
                hx[4 * t + e] = y.x; hy[4 * t + e] = y.y;
              }
            }
#pragma unroll
          for (int v = 0; v < 4; ++v) {
            const uint32_t (&hh)[8] = (v < 2) ? hx : hy;
            const uint32_t sel = (v & 1) ? kHi : kLo;
            const uint32_t a[4] = {__builtin_amdgcn_perm(hh[1], hh[0], sel), __builtin_amdgcn_perm(hh[3], hh[2], sel),
                                   __builtin_amdgcn_perm(hh[5], hh[4], sel), __builtin_amdgcn_perm(hh[7], hh[6], sel)};
            acc[c][v] = mfma32(a, bb, acc[c][v]);
          }
        }
      }
    }
  };
  const int32_t n_clear = min(n_tok, lim_first);          // tokens every query sees, uniform
  for (; base + TRIP <= n_clear; base += stride) trip_body(std::true_type{});
  for (; base < n_tok; base += stride) trip_body(std::false_type{});     // the sequence's ragged / causal end

  // ---- merge the eight waves.  The table is dead once every wave is here.
  const float l_wave = allreduce_rows(l_run, [](float a, float b) { return a + b; });
  __syncthreads();
  if ((int32_t)i16 < p.q_len) {
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
      for (int v = 0; v < 4; ++v)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const uint32_t row = 4u * gq + r;                       // the instruction's output row
          const uint32_t d = (KBITS == 4) ? 64u * c + 8u * (row & 7u) + 2u * ((v >> 1) + 2u * (row >> 3)) + (v & 1)
                                          : 64u * c + 4u * row + v;
          lds.xo[wave][i16][d] = acc[c][v][r];
        }
    if (gq == 0) { lds.wm[wave][i16] = m_run; lds.wl[wave][i16] = l_wave; }
  }
  __syncthreads();
  const int32_t n_out = p.q_len * D;
  for (int32_t idx = (int32_t)threadIdx.x; idx < n_out; idx += kThreads) {
    const int32_t qy = idx / D, d = idx % D;
    float m_all = lds.wm[0][qy];
#pragma unroll
    for (int w = 1; w < kWaves; ++w) m_all = fmaxf(m_all, lds.wm[w][qy]);
    float l_all = 0.0f, o = 0.0f;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const float f = __builtin_amdgcn_exp2f(lds.wm[w][qy] - m_all);     // 0 for a wave without visible tokens
      l_all += lds.wl[w][qy] * f;
      o += lds.xo[w][qy][d] * f;
    }
    if (p.splits == 1) {
      p.out[((int64_t)bh * p.q_len + qy) * D + d] = __builtin_bit_cast(unsigned short, (_Float16)(o * p.inv_gamma / l_all));
    } else {
      float* rec = p.partials + (((int64_t)bh * p.splits + sp) * p.q_len + qy) * (D + 2);
      rec[2 + d] = o;
      if (d == 0) { rec[0] = m_all; rec[1] = l_all; }
    }
  }
}

// splits > 1: fold the partial results of one (sequence, query) in split order; one thread per
// output element.  (A split whose tokens the query cannot see has l = 0 and the sentinel maximum.)
template <int D>
__global__ __launch_bounds__(D) void combine_multi_kernel(const MultiParams p) {
  const int64_t bq = blockIdx.x;                     // (b*H + h) * q_len + query
  const int64_t bh = bq / p.q_len, qy = bq % p.q_len;
  const int d = threadIdx.x;
  float mm = kNoScore, ll = 0.0f, oo = 0.0f;
  // eight splits per round, so that their loads are in flight together; a record past the last
  // split is a clamped duplicate that enters with weight 0
  constexpr int U = 8;
  for (int s0 = 0; s0 < p.splits; s0 += U) {
    float ms[U], ls[U], os[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int s = min(s0 + u, p.splits - 1);
      const float* rec = p.partials + ((bh * p.splits + s) * p.q_len + qy) * (D + 2);
      ms[u] = rec[0]; ls[u] = rec[1]; os[u] = rec[2 + d];
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float m_s = (s0 + u < p.splits) ? ms[u] : -INFINITY;
      const float m_new = fmaxf(mm, m_s);
      const float f_old = __builtin_amdgcn_exp2f(mm - m_new), f_s = __builtin_amdgcn_exp2f(m_s - m_new);
      ll = ll * f_old + ls[u] * f_s;
      oo = oo * f_old + os[u] * f_s;
      mm = m_new;
    }
  }
  p.out[bq * D + d] = __builtin_bit_cast(unsigned short, (_Float16)(oo * p.inv_gamma / ll));
}

template <int KBITS, int D, int BLK>
hipError_t launch_dims(const MultiParams& p, int B_H, hipStream_t stream) {
  if (p.block_table) hipLaunchKernelGGL((decode_multi_kernel<KBITS, D, BLK, true>), dim3((unsigned)p.n_items), dim3(kThreads), 0, stream, p);
  else hipLaunchKernelGGL((decode_multi_kernel<KBITS, D, BLK, false>), dim3((unsigned)p.n_items), dim3(kThreads), 0, stream, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || p.splits == 1) return e;
  hipLaunchKernelGGL((combine_multi_kernel<D>), dim3((unsigned)(B_H * p.q_len)), dim3(D), 0, stream, p);
  return hipGetLastError();
}

template <int KBITS>
hipError_t launch_k(const MultiParams& p, int bh, int D, int blk, hipStream_t stream) {
  if (D == 64 && blk == 64) return launch_dims<KBITS, 64, 64>(p, bh, stream);
  if (D == 128 && blk == 64) return launch_dims<KBITS, 128, 64>(p, bh, stream);
  if (D == 128 && blk == 128) return launch_dims<KBITS, 128, 128>(p, bh, stream);
  return hipErrorInvalidValue;
}

}  // namespace

int decode_multi_trip_tokens() { return kSplitUnit; }
int decode_multi_item_tokens() { return kWaves * kTrip; }

hipError_t launch_decode_attention_multi(const MultiParams& p, int D, int k, int blk, hipStream_t stream) {
  if (p.q_len < 1 || p.q_len > kMaxQ || p.splits < 1 || p.n_items % p.splits) return hipErrorInvalidValue;
  const int bh = p.n_items / p.splits;
  if (k == 4) return launch_k<4>(p, bh, D, blk, stream);
  if (k == 2) return launch_k<2>(p, bh, D, blk, stream);
  if (k == 3) return launch_k<3>(p, bh, D, blk, stream);
  return hipErrorInvalidValue;
}

}  // namespace nqkv
