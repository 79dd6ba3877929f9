/*
 * nqkv_benchaux.h -- C ABI of libnqkv_benchaux, the measurement helpers used by the benchmark.
 * None of this is part of the NQKV method (libnqkv, nqkv.h); it is kept in a library of its own
 * so that the product library exports nothing but the method.
 *
 * All functions enqueue one kernel on `hip_stream` (a hipStream_t as void*, NULL = the default
 * stream) and return 0, -1 for a null / misaligned pointer or a size that is not a multiple of
 * 16, -4 when the launch failed.  Pointers are device memory owned by the caller.
 */
#ifndef NQKV_BENCHAUX_H_
#define NQKV_BENCHAUX_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Reads `bytes` of device memory at `src` once, with 128-bit non-temporal loads, and writes one
 * 32-bit xor checksum per workgroup to `checksums` (NQKV_AUX_PROBE_WORKGROUPS uint32).  Timed, it
 * gives the read bandwidth this machine delivers to the simplest possible kernel; the xor of all
 * checksums equals the xor of all 32-bit words of the buffer.
 */
#define NQKV_AUX_PROBE_WORKGROUPS 4096
int nqkv_aux_read_stream(const void* src, size_t bytes, void* checksums, void* hip_stream);

/* Copies `bytes` from src to dst with a plain kernel: reads and writes exactly `bytes` each, the
 * known quantity that HBM byte counters of a profiler run are scaled by. */
int nqkv_aux_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/*
 * A plain kernel with a fixed read : write mix: per tile it reads `reads` x 4 KiB from src and
 * writes `writes` x 4 KiB to dst (contiguous, 128-bit, non-temporal), tile after tile, for as many
 * whole tiles as both buffers hold; *tiles_out (host) receives that count, so the bytes moved are
 * tiles * 4096 * (reads + writes).  (reads, writes) is (4, 1), (1, 4) or (1, 1); anything else
 * returns -1.  Timed, it is what the memory system gives the simplest kernel with the mix of the
 * quantizer (4 : 1) or of the dequantizer (1 : 4) -- the yardstick for those kernels.  dst
 * receives a function of src (tile-wise xor of the pieces read, plus the piece's index).
 */
int nqkv_aux_mix_stream(const void* src, size_t src_bytes, void* dst, size_t dst_bytes, int reads, int writes,
                        size_t* tiles_out, void* hip_stream);

/* Launches a kernel that does nothing: the fixed cost of one launch. */
int nqkv_aux_empty_launch(void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* NQKV_BENCHAUX_H_ */
