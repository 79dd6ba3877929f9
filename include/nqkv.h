/*
 * nqkv.h -- C ABI of the NQKV hot path for AMD MI355X (gfx950).
 *
 * NQKV (arXiv 2505.16210) stores the key/value cache of a transformer decoder as k-bit
 * indices into a small table of normal-distribution quantile points, one table look-up
 * range ("block") at a time, and dequantizes the cache when attention needs it
 * (paper Sec. 3.2 and Fig. 5).  This library implements exactly that path for one GPU:
 *
 *   nqkv_build_codebook    the quantile table                        (Sec. 1, Sec. 3.2)
 *   nqkv_quantize_kv       fp16 K or V -> packed indices + scales    (Sec. 3.2 prefill eqs;
 *   nqkv_quantize_kv_pair  K and V in one launch                      decoding-phase append)
 *   nqkv_dequantize_kv     indices -> fp16                           (Sec. 3.2, X' = dequantize(I))
 *   nqkv_decode_attention  softmax(q K'^T) V' read straight from the packed cache
 *                                                                    (Sec. 3.2 decoding phase)
 *   nqkv_decode_step       append + attention of one decode step in one launch (Sec. 3.2)
 *   nqkv_decode_attention_varlen / nqkv_decode_step_varlen  the same for per-sequence lengths
 *   nqkv_decode_attention_paged / nqkv_decode_step_paged  the same over a paged cache
 *   nqkv_quantize_kv_hidden  blocks over the token's hidden vector, token-major source
 *                                                                    (Fig. 5, Sec. 4.1)
 *   nqkv_decode_attention_multi (_varlen, _paged)  several new tokens' queries in one step
 *                                                                    (Sec. 1, Sec. 3.2)
 *
 * General rules
 *   - Every function returns NQKV_OK (0) or a negative NQKV_E* code.  Nothing throws,
 *     prints or exits.  All argument checks happen on the host before any GPU work, so a
 *     call that returns an error other than NQKV_EHIP has launched nothing.
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary memory.  The library allocates no device memory and keeps no state between
 *     calls.  Device pointers must be 16-byte aligned.
 *   - `hip_stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream and return; they never synchronise (the one exception,
 *     nqkv_decode_workspace_check, says so).
 *   - fp16 means IEEE binary16.  Inputs must be finite (not checked).
 *   - Results are bitwise reproducible for equal arguments (no floating-point atomics).
 *
 * Cache layout (one tensor, K or V), for B batch rows, H heads, head dimension D, k bits,
 * block size `block`, capacity cap_tokens:
 *   codes  : uint8  [B][H][cap_tokens][D*k/8]   element i of a (b,h,token) row owns bits
 *                                               [k*i, k*i+k) of that row's little-endian
 *                                               bit stream (bit n = bit n&7 of byte n>>3)
 *   scales : fp16   [B][H][cap_tokens][D/block] max |x| over `block` consecutive head-dim
 *                                               elements of one token of one head
 * A block never spans tokens or heads (Fig. 5 caption: every token is cut into blocks).
 * Performance note: cap_tokens sets the distance between the (b,h) slabs of a tensor.  The
 * kernels are fastest when a slab of codes (cap_tokens * D*k/8 bytes) is a multiple of 1 KiB, so
 * that every wave load starts on a cache-line boundary (the one-query attention kernels start an
 * item on a line themselves when k is 2 or 4; otherwise a capacity of 16385 tokens measured 11 %
 * slower than 16400 or 16640), and distances of a power of two plus 8 KiB are worth avoiding
 * (slabs streamed together then share few memory channels).  Any capacity is correct.
 *
 * Quantization rule (the paper leaves rounding details open; this is the library's
 * contract): with s = the block's fp16 scale, t_j = (c[j-1] + c[j]) * 0.5f the fp32
 * mid-points of the ascending table c[0..2^k-1],
 *     code(x) = number of j in [1, 2^k - 1] with  (float)x > fl32(t_j * (float)s)
 * i.e. nearest table entry, ties to the lower index.  An all-zero block gets code 0
 * everywhere and scale 0.
 */
#ifndef NQKV_H_
#define NQKV_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  NQKV_OK = 0,
  NQKV_EINVAL = -1,        /* null / misaligned pointer, size or range out of bounds        */
  NQKV_EUNSUPPORTED = -2,  /* well-formed but outside what the kernels are built for        */
  NQKV_EWORKSPACE = -3,    /* workspace smaller than nqkv_decode_workspace_bytes reports    */
  NQKV_EHIP = -4           /* a HIP runtime call (kernel launch) failed                     */
};

/* Static, NUL-terminated description of a status code. */
const char* nqkv_strerror(int status);

/* Library ABI version (major * 100 + minor). */
int nqkv_version(void);

/*
 * Per-call options, OR-ed into nqkv_cache_desc.flags.  They never change results (codes stay
 * bit-identical, attention stays within its tolerance), only which kernel variant or launch
 * shape a call uses; they exist for A/B measurements and for tests that must reach both
 * variants.  The library itself holds no settings.
 */
enum {
  NQKV_FLAG_SCAN_QUANTIZER = 1,      /* quantizer: plain scan of all thresholds instead of the
                                        cell-table code search                                   */
  NQKV_FLAG_WORKGROUP_PER_ITEM = 2   /* decode attention: one workgroup per work item whatever
                                        its length, instead of a persistent grid for short items */
};

/*
 * Quantile table (Sec. 1: the table entries are quantile points of a normal distribution).
 * Host only; touches no GPU.
 *   k          bits per index, 1..8 (the kernels accept tables for k = 2, 3, 4)
 *   variant    0: symmetric table, level i = Phi^-1((i + 1/2) / 2^k) divided by the largest
 *                 level, i.e. the medians of 2^k equal-probability slices of N(0,1);
 *                 levels_out[i] == -levels_out[2^k-1-i] exactly
 *              1: zero-preserving table in the NormalFloat style the paper cites for its
 *                 4-bit runs: 2^(k-1) positive levels, an exact 0 and 2^(k-1)-1 negative
 *                 levels, each side from evenly spaced probabilities in (1/2, 1 - 2^-(k+1)]
 *                 pushed through Phi^-1 and divided by the largest (k >= 2)
 *   levels_out host float[2^k], ascending, levels_out[0] = -1, levels_out[2^k-1] = +1
 */
int nqkv_build_codebook(int k, int variant, float* levels_out);

/* Geometry of one cache tensor.  Plain data, read during the call only. */
typedef struct nqkv_cache_desc {
  int32_t B;           /* batch rows, >= 1                                                   */
  int32_t H;           /* heads, 1..65535; B <= 32767, B*H <= 2^24 (<= 65535 when a call   */
                       /* cuts sequences into pieces: num_splits > 1)                        */
  int32_t D;           /* head dimension: 64 or 128                                          */
  int32_t k;           /* bits per index: 2, 3 or 4                                          */
  int32_t block;       /* elements per scale: 64 or 128, must divide D                       */
  int32_t flags;       /* 0, or NQKV_FLAG_* values OR-ed together                            */
  int64_t cap_tokens;  /* token capacity of the codes / scales arrays, >= 1                  */
} nqkv_cache_desc;

/*
 * Quantize n_tokens tokens of one tensor into cache rows
 * [dst_token_offset, dst_token_offset + n_tokens)  (Sec. 3.2: I = quantize(X) at prefill;
 * at decode the new token's indices are appended and older entries never change -- prefill
 * and append are this same call with different offsets).
 *   levels  host float[2^k], ascending (from nqkv_build_codebook or the caller's own)
 *   src     device fp16, logical shape [B][H][n_tokens][D]; element (b,h,t,d) is at
 *           src + b*stride_b + h*stride_h + t*stride_t + d (strides in elements, D contiguous,
 *           stride_t a multiple of 8)
 *   codes, scales  device, layouts above; rows outside the written range are untouched
 * Errors: NQKV_EINVAL for null/misaligned pointers, n_tokens < 0, a range outside
 * [0, cap_tokens], a non-ascending table; NQKV_EUNSUPPORTED for D/k/block outside the lists
 * above.  n_tokens == 0 is a successful no-op whatever the data pointers are.
 */
int nqkv_quantize_kv(const nqkv_cache_desc* desc, const float* levels,
                     const void* src, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                     int64_t n_tokens, int64_t dst_token_offset,
                     void* codes, void* scales, void* hip_stream);

/*
 * The same for a key tensor and a value tensor of equal geometry and strides in ONE kernel
 * launch (the decode-step append of Sec. 3.2 quantizes t_K and t_V together).
 */
int nqkv_quantize_kv_pair(const nqkv_cache_desc* desc, const float* levels,
                          const void* k_src, const void* v_src,
                          int64_t stride_b, int64_t stride_h, int64_t stride_t,
                          int64_t n_tokens, int64_t dst_token_offset,
                          void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                          void* hip_stream);

/*
 * nqkv_quantize_kv_pair for a batch whose sequences stand at different positions (a step that
 * appends n_tokens tokens to every sequence of a ragged batch): sequence b's tokens go to cache
 * rows [dst_token_offsets[b], dst_token_offsets[b] + n_tokens).
 *   dst_token_offsets  device int32 [B], 4-byte aligned, read by the kernel only; values are
 *                      clamped into [0, max_offset] (no out-of-bounds write; the rows written for
 *                      a sequence whose entry was out of range are then unspecified)
 *   max_offset         host upper bound of the entries, max_offset + n_tokens <= cap_tokens
 * Errors: as nqkv_quantize_kv_pair, plus NQKV_EINVAL for a null / misaligned array.
 */
int nqkv_quantize_kv_pair_varlen(const nqkv_cache_desc* desc, const float* levels,
                                 const void* k_src, const void* v_src,
                                 int64_t stride_b, int64_t stride_h, int64_t stride_t,
                                 int64_t n_tokens, const int32_t* dst_token_offsets, int64_t max_offset,
                                 void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                                 void* hip_stream);

/*
 * Dequantize cache rows [token_offset, token_offset + n_tokens) to fp16
 * (Fig. 5 caption: indices are looked up in the table and restored to FP16):
 *     dst = fp16_round_to_nearest_even( fl32( levels[code] * (float)scale ) )
 *   dst  device fp16, logical [B][H][n_tokens][D], strides as for nqkv_quantize_kv.
 */
int nqkv_dequantize_kv(const nqkv_cache_desc* desc, const float* levels,
                       const void* codes, const void* scales,
                       int64_t token_offset, int64_t n_tokens,
                       void* dst, int64_t stride_b, int64_t stride_h, int64_t stride_t,
                       void* hip_stream);

/*
 * Workspace needed by nqkv_decode_attention for a given sequence length.
 *   num_splits  0: the library chooses how many pieces each (b,h) sequence is cut into;
 *               >0: use exactly this many (1..1024, at most seq_len)
 *   bytes_out   receives the workspace size in bytes (0 when one piece is used)
 *   splits_out  receives the number of pieces that will be used (may be NULL)
 * Host only.
 *
 * Workspace contract: the first 256 KiB hold arrival counters that must be ZERO when a call
 * starts.  Clear the workspace once after allocating it (nqkv_decode_workspace_init, or any
 * zero-fill); every call leaves the counters zero again, so the same workspace can be reused by
 * later calls on the same stream with any geometry.  Calls that share a workspace must not
 * overlap in time.  If the counters are NOT zero when a call starts (memory that was never
 * cleared, or written by something else since), that call's output is undefined; a kernel that
 * notices -- it is handed a ticket its own call cannot have issued -- marks the workspace, and
 * nqkv_decode_workspace_check reports it.
 */
int nqkv_decode_workspace_bytes(const nqkv_cache_desc* desc, int64_t seq_len, int num_splits,
                                size_t* bytes_out, int* splits_out);

/*
 * Clears the counters of a split-K workspace (its first 256 KiB) with a small kernel enqueued on
 * `hip_stream`: the once-after-allocation step of the contract above, and the way back from a
 * workspace that nqkv_decode_workspace_check found dirty.  A kernel, not a memset, so it may be
 * recorded into a HIP graph.
 * Errors: NQKV_EINVAL for a null / misaligned pointer, NQKV_EWORKSPACE for fewer than 256 KiB.
 */
int nqkv_decode_workspace_init(void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Host-visible check of that contract, for debugging and for callers that recycle memory: copies
 * the counters back and returns NQKV_OK when all are zero, NQKV_EWORKSPACE when any is not (a
 * counter left armed by a call that never finished, memory that was never cleared, or the mark
 * of a kernel that was handed an impossible ticket).  Unlike every other call this one WAITS for
 * `hip_stream` (it has to, to look at the memory); use it when no call on this workspace is in
 * flight on another stream.
 * Errors: NQKV_EINVAL for a null / misaligned pointer, NQKV_EWORKSPACE also for fewer than 256 KiB.
 */
int nqkv_decode_workspace_check(const void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Attention of one new query per (batch, head) over the first seq_len cached tokens
 * (Sec. 3.2 decoding phase: A = Softmax(t_Q X_K'^T), t_O = A X_V', with X' the dequantized
 * cache), computed without materialising X':
 *     z_t   = softmax_scale * sum_d q[d] * levels[Kcode[t,d]] * Kscale[t, d/block]
 *     out_d = sum_t exp(z_t - max z) * levels[Vcode[t,d]] * Vscale[t, d/block] / sum_t exp(z_t - max z)
 * The token appended in this decode step must already be in the cache (append first, then
 * attend, as in the paper).  K and V caches share `desc`.
 *   q, out        device fp16 [B][H][D] contiguous
 *   workspace     device memory of at least the size reported by nqkv_decode_workspace_bytes
 *                 for the same (desc, seq_len, num_splits), zero-filled before its first use
 *                 (see there); may be NULL when that size is 0
 * Arithmetic: table entries are rounded to fp16 for the look-up, products accumulate in
 * fp32, exp in fp32; the result is within 2e-3 (relative to the largest |out| of the row)
 * of the same formula evaluated in fp64.  At k = 4 and k = 2 the product softmax weight x
 * value scale is rounded to fp16 before it multiplies the levels (two tokens share one
 * instruction): value blocks whose scale is below 2^-14 lose precision, and single outputs
 * can be off by up to 1e-2 of max(|out|, 1 % of the row's largest |out|).  Different
 * num_splits give results that differ by rounding only; equal arguments give equal bits.
 * Errors: as above, plus NQKV_EINVAL for seq_len outside [1, cap_tokens] and
 * NQKV_EWORKSPACE for a short workspace.
 */
int nqkv_decode_attention(const nqkv_cache_desc* desc, const float* levels,
                          const void* q,
                          const void* k_codes, const void* k_scales,
                          const void* v_codes, const void* v_scales,
                          int64_t seq_len, float softmax_scale, void* out,
                          void* workspace, size_t workspace_bytes, int num_splits,
                          void* hip_stream);

/*
 * nqkv_decode_attention for callers that cannot allocate device memory or pass a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, results and errors as nqkv_decode_attention (equal bits for equal num_splits), but
 * the split-K workspace is a fixed array of NQKV_STATIC_SCRATCH_BYTES inside the library's code
 * object: every GPU the library is used on holds one such array until the process ends.  The call
 * allocates nothing and frees nothing; it enqueues a small clearing kernel (when the sequence is
 * cut) and the attention kernel on `hip_stream`.
 *   - A geometry whose workspace (nqkv_decode_workspace_bytes for the same arguments) exceeds
 *     NQKV_STATIC_SCRATCH_BYTES is refused with NQKV_EWORKSPACE before any GPU work.
 *   - All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (two
 *     streams, two threads) race on it and give undefined results; serialise them.
 *   - A failed address look-up of the array returns NQKV_EHIP.
 */
#define NQKV_STATIC_SCRATCH_BYTES (2u << 20)
int nqkv_decode_attention_static(const nqkv_cache_desc* desc, const float* levels,
                                 const void* q,
                                 const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales,
                                 int64_t seq_len, float softmax_scale, void* out,
                                 int num_splits, void* hip_stream);

/*
 * One whole decode step of Sec. 3.2 in a single launch: quantize the new token's key and value
 * (I_tK = quantize(t_K), I_tV = quantize(t_V)), append their indices at cache row `pos`
 * (I <- Concat(I, I_t)), and attend over rows [0, pos] -- the appended token included.
 * The cache afterwards holds exactly the bytes nqkv_quantize_kv_pair(n_tokens = 1,
 * dst_token_offset = pos) would have written, and `out` is what nqkv_decode_attention(seq_len =
 * pos + 1) would return up to rounding (the new token enters the softmax from registers).
 *   k_new, v_new  device fp16, one row per (b,h): element (b,h,d) at
 *                 b*new_stride_b + h*new_stride_h + d (strides in elements, multiples of 8)
 *   pos           0 .. cap_tokens-1; rows [0, pos) must already be valid
 *   workspace     as for nqkv_decode_attention, sized with
 *                 nqkv_decode_workspace_bytes(desc, max(pos, 1), num_splits)
 * A table whose neighbouring mid-points lie closer than about 1/32 of its range cannot be searched
 * by the kernel's own quantizer; for such a table the call runs as two launches (append with
 * nqkv_quantize_kv_pair's kernel, then nqkv_decode_attention over pos + 1 tokens) and the
 * workspace must satisfy nqkv_decode_workspace_bytes(desc, pos + 1, num_splits) as well.  All of
 * this is checked before the first launch.
 * Errors: as nqkv_decode_attention, plus NQKV_EINVAL for a null/misaligned k_new or v_new.
 */
int nqkv_decode_step(const nqkv_cache_desc* desc, const float* levels,
                     const void* q, const void* k_new, const void* v_new,
                     int64_t new_stride_b, int64_t new_stride_h,
                     void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                     int64_t pos, float softmax_scale, void* out,
                     void* workspace, size_t workspace_bytes, int num_splits,
                     void* hip_stream);

/*
 * The two decode calls for a batch whose sequences differ in length (continuous batching): the
 * number of cached tokens of sequence b comes from device memory instead of an argument.
 *   seq_lens  device int32 [B], 4-byte aligned: tokens of sequence b to attend over, 1..max_seq_len
 *   pos       device int32 [B]: cached rows of sequence b = the row its new token is appended at,
 *             0..max_pos
 *   max_seq_len / max_pos  host upper bound of the array's values (<= cap_tokens, < cap_tokens):
 *             the split count and the workspace are planned for it, as by
 *             nqkv_decode_workspace_bytes(desc, max_seq_len, ...) / (desc, max(max_pos, 1), ...)
 * The arrays are read by the kernel only; values outside the stated range are clamped into it
 * (no out-of-bounds access), the result for such a sequence is then unspecified.  Everything
 * else is as for nqkv_decode_attention / nqkv_decode_step, which these equal when all entries
 * are the same.  Errors: as those, plus NQKV_EINVAL for a null / misaligned array, and
 * NQKV_EUNSUPPORTED from nqkv_decode_step_varlen for a table the in-kernel quantizer cannot take.
 */
int nqkv_decode_attention_varlen(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                 const void* k_codes, const void* k_scales,
                                 const void* v_codes, const void* v_scales,
                                 const int32_t* seq_lens, int64_t max_seq_len, float softmax_scale, void* out,
                                 void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream);
int nqkv_decode_step_varlen(const nqkv_cache_desc* desc, const float* levels,
                            const void* q, const void* k_new, const void* v_new,
                            int64_t new_stride_b, int64_t new_stride_h,
                            void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                            const int32_t* pos, int64_t max_pos, float softmax_scale, void* out,
                            void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream);

/*
 * The decode calls, and the quantizer, over a PAGED cache.  The pool is num_pages pages; a page holds P =
 * desc->cap_tokens tokens (a power of two, at least 128) of all H heads in the layout of a
 * one-sequence cache -- codes uint8 [num_pages][H][P][D*k/8], scales fp16
 * [num_pages][H][P][D/block] (so a page can also be filled with nqkv_quantize_kv on a desc
 * with B = 1 and pointers offset to the page).  Logical page j of sequence b (its tokens j*P ..
 * j*P+P-1) is page block_table[b*table_stride + j].
 *   block_table  device int32, 4-byte aligned; entries of pages that hold tokens (and, for the
 *                step, the page of row pos[b]) must be valid page numbers; indices and entries
 *                are clamped into the table and the pool before use, so no value can cause an
 *                out-of-bounds access
 *   seq_lens / pos, max_seq_len / max_pos   as for the _varlen calls (max_* bound by
 *                table_stride * P instead of the capacity)
 *   workspace    sized with nqkv_decode_paged_workspace_bytes(desc, max_seq_len or
 *                max(max_pos, 1), ...), which also reports into how many work items (runs of
 *                whole pages) a sequence is cut; may be NULL when that size is 0
 * Results: as nqkv_decode_attention_varlen / nqkv_decode_step_varlen on the same tokens laid
 * out contiguously, up to the rounding of a different split.
 * Errors: as those, plus NQKV_EUNSUPPORTED for a page size that is not a power of two >= 128.
 */
/*
 * nqkv_quantize_kv_pair into a paged cache (layout and block table as described above): tokens
 * [dst_token_offset, dst_token_offset + n_tokens) of EVERY sequence of the batch go to the pages
 * its row of the block table names -- prefill (offset 0) or a multi-token append.  The pages
 * touched must be valid entries; n_tokens is the same for all sequences (call per sequence, with
 * B = 1 and the sequence's table row, for ragged prompts).  v_* may all be NULL.
 * Errors: as nqkv_quantize_kv, plus NQKV_EINVAL for a null / misaligned table or rows beyond
 * table_stride * P, NQKV_EUNSUPPORTED for a page size that is not a power of two >= 128.
 */
int nqkv_quantize_kv_paged(const nqkv_cache_desc* desc, const float* levels,
                           const void* k_src, const void* v_src,
                           int64_t stride_b, int64_t stride_h, int64_t stride_t,
                           int64_t n_tokens, int64_t dst_token_offset,
                           const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                           void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                           void* hip_stream);
/* The same with a first row per sequence (dst_token_offsets / max_offset as for
 * nqkv_quantize_kv_pair_varlen; max_offset + n_tokens <= table_stride * P). */
int nqkv_quantize_kv_paged_varlen(const nqkv_cache_desc* desc, const float* levels,
                                  const void* k_src, const void* v_src,
                                  int64_t stride_b, int64_t stride_h, int64_t stride_t,
                                  int64_t n_tokens, const int32_t* dst_token_offsets, int64_t max_offset,
                                  const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                  void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                                  void* hip_stream);
int nqkv_decode_paged_workspace_bytes(const nqkv_cache_desc* desc, int64_t max_tokens,
                                      size_t* bytes_out, int* items_out);
int nqkv_decode_attention_paged(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                const int32_t* seq_lens, int64_t max_seq_len, float softmax_scale, void* out,
                                void* workspace, size_t workspace_bytes, void* hip_stream);
int nqkv_decode_step_paged(const nqkv_cache_desc* desc, const float* levels,
                           const void* q, const void* k_new, const void* v_new,
                           int64_t new_stride_b, int64_t new_stride_h,
                           void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                           const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                           const int32_t* pos, int64_t max_pos, float softmax_scale, void* out,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Quantization with blocks over the token's hidden vector (Fig. 5: every token is cut into
 * blocks of a fixed size; Sec. 4.1: block size 256).  The hidden vector of a token is its H
 * heads of D elements side by side; a block is `block_hidden` consecutive elements of it and so
 * covers block_hidden / D whole heads.  Each block is quantized exactly like the blocks of
 * nqkv_quantize_kv (same scale, code and packing rules).  The cache keeps the per-head layout of
 * the other calls with ONE scale per token-head -- desc->block must equal desc->D -- and the
 * block's scale is stored once for every head the block covers, so nqkv_dequantize_kv,
 * nqkv_decode_attention and nqkv_decode_step read the result as it is.
 *   k_src, v_src  device fp16, element (b,h,t,d) at b*stride_b + h*stride_h + t*stride_t + d;
 *                 the projection's own token-major layout [B, S, H*D] is stride_h = D,
 *                 stride_t = H*D (strides in elements, multiples of 8).  v_* may all be NULL.
 *   block_hidden  128 or 256, a multiple of D that divides H*D; or D itself (then the same
 *                 as nqkv_quantize_kv_pair)
 * Errors: as nqkv_quantize_kv, plus NQKV_EINVAL for desc->block != desc->D or a block_hidden
 * that does not fit the head geometry, NQKV_EUNSUPPORTED for other block sizes, for a batch row
 * whose source or cache extent reaches 2 GiB, or for more than 2 097 120 tokens in one call.
 */
int nqkv_quantize_kv_hidden(const nqkv_cache_desc* desc, const float* levels,
                            const void* k_src, const void* v_src,
                            int64_t stride_b, int64_t stride_h, int64_t stride_t,
                            int64_t n_tokens, int64_t dst_token_offset, int block_hidden,
                            void* k_codes, void* k_scales, void* v_codes, void* v_scales,
                            void* hip_stream);

/*
 * Attention for a step that appended SEVERAL tokens (Sec. 1: new keys and values go to the end of
 * the append-only cache; Sec. 3.2 decoding-phase equations, once per new token): the q_len
 * queries of a (batch, head) belong to the LAST q_len of the first seq_len cached tokens, and
 * query i attends over tokens [0, seq_len - q_len + 1 + i) -- what nqkv_decode_attention would
 * give it at that sequence length.  The new tokens must already be in the cache
 * (nqkv_quantize_kv_pair with n_tokens = q_len appends them; nqkv_quantize_kv_pair_varlen when the
 * sequences stand at different positions).  The products run on the matrix
 * cores (fp16 inputs, fp32 accumulation); weights times the value scale are rounded to fp16, so
 * value scales below 2^-14 lose precision.  Tolerance as for nqkv_decode_attention.
 *   q, out     device fp16 [B][H][q_len][D] contiguous
 *   q_len      1..16
 *   workspace  nqkv_decode_multi_workspace_bytes(desc, seq_len, q_len, num_splits, ...) bytes
 *              (partial results only: no zero-fill needed); may be NULL when that is 0
 * Errors: NQKV_EINVAL for null / misaligned pointers, q_len < 1, seq_len outside
 * [q_len, cap_tokens], num_splits above the number of 32-token pieces of the sequence;
 * NQKV_EUNSUPPORTED for q_len > 16;
 * NQKV_EWORKSPACE for a short workspace.
 */
int nqkv_decode_multi_workspace_bytes(const nqkv_cache_desc* desc, int64_t seq_len, int q_len, int num_splits,
                                      size_t* bytes_out, int* splits_out);
int nqkv_decode_attention_multi(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                int64_t seq_len, int q_len, float softmax_scale, void* out,
                                void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream);

/*
 * The same for a batch whose sequences differ in length: sequence b holds seq_lens[b] cached
 * tokens (device int32 [B], 4-byte aligned, q_len..max_seq_len; values outside are clamped into
 * that range, the result for such a sequence is then unspecified), its q_len queries are those of
 * its own last q_len tokens.  Splits and workspace are planned for max_seq_len
 * (nqkv_decode_multi_workspace_bytes(desc, max_seq_len, q_len, ...)).  Equals
 * nqkv_decode_attention_multi when all entries are max_seq_len.
 * Errors: as there, plus NQKV_EINVAL for a null / misaligned array.
 */
int nqkv_decode_attention_multi_varlen(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                       const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                       const int32_t* seq_lens, int64_t max_seq_len, int q_len, float softmax_scale, void* out,
                                       void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream);

/*
 * And over a PAGED cache (pool layout, block table and page size as for
 * nqkv_decode_attention_paged; desc->cap_tokens is the page size P): the q_len queries of sequence
 * b are those of its last q_len tokens, seq_lens[b] of them cached in the pages its table row
 * names.  The new tokens are appended first with nqkv_quantize_kv_paged or, when the positions
 * differ, nqkv_quantize_kv_paged_varlen.  max_seq_len is bound by table_stride * P; the workspace comes from
 * nqkv_decode_multi_paged_workspace_bytes(desc, max_seq_len, q_len, num_splits, ...).
 * Errors: as nqkv_decode_attention_multi_varlen, plus NQKV_EINVAL for a null / misaligned table or
 * a bad table_stride / num_pages, NQKV_EUNSUPPORTED for a page size that is not a power of two
 * >= 128.
 */
int nqkv_decode_multi_paged_workspace_bytes(const nqkv_cache_desc* desc, int64_t max_seq_len, int q_len, int num_splits,
                                            size_t* bytes_out, int* splits_out);
int nqkv_decode_attention_multi_paged(const nqkv_cache_desc* desc, const float* levels, const void* q,
                                      const void* k_codes, const void* k_scales, const void* v_codes, const void* v_scales,
                                      const int32_t* block_table, int64_t table_stride, int64_t num_pages,
                                      const int32_t* seq_lens, int64_t max_seq_len, int q_len, float softmax_scale, void* out,
                                      void* workspace, size_t workspace_bytes, int num_splits, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* NQKV_H_ */
