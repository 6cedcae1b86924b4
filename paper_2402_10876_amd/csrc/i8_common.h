// Internal: device-side helpers shared by the int8 kernels.
#pragma once
#include "device_common.h"

namespace twg {

typedef int intx16 __attribute__((ext_vector_type(16)));

// int32 sum -> int8: fp32(sum) (nearest even), one fp32 product with the scale, round half
// to even, clamp to [-128, 127].
__device__ __forceinline__ int requantize(int sum, float scale) {
  float x = (float)sum * scale;            // int -> fp32 (nearest even), one fp32 product
  x = __builtin_rintf(x);                  // halves to even
  x = __builtin_fminf(__builtin_fmaxf(x, -128.f), 127.f);
  return (int)x;
}

// Extra workgroups of a launch write 0 into one pruned column of C each.
template <bool OUT8>
__device__ __forceinline__ void zero_fill_column8(const GemmI8Args& g, int which) {
  const int col = g.zero_cols[which];
  constexpr int ES = OUT8 ? 1 : 4;
  char* row = (char*)g.C + (size_t)col * g.ldc * ES;
  const size_t bytes = (size_t)g.M * ES;
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (size_t b = (size_t)threadIdx.x * 16; b < bytes; b += (size_t)blockDim.x * 16) {
    if (b + 16 <= bytes) __builtin_nontemporal_store(z, (u32x4*)(row + b));
    else for (size_t i = b; i < bytes; ++i) row[i] = 0;
  }
}

}  // namespace twg
