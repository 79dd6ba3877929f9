// One 32-bit word from a wave-uniform address of read-only device memory (sequence lengths, a
// block table), as a scalar load.  Left to the compiler such a read becomes a vector load whose
// result -- and every address and buffer descriptor derived from it -- lives in vector registers
// and has to be made uniform again before each use.
#pragma once

#include <stdint.h>

namespace nqkv {

__device__ __forceinline__ int32_t scalar_read(const int32_t* uniform_ptr) {
  int32_t v;
  asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(uniform_ptr) : "memory");
  return v;
}

}  // namespace nqkv
