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

// Implicit img2col: which of the CH wide-grid positions m .. m+CH-1 are output pixels (x < W and
// y < H).  CH = 4: one all-ones dword per valid position (int32 output); CH = 16: one 0xff byte
// per valid position (int8 output).  One division per thread.
template <int CH>
__device__ __forceinline__ u32x4 conv_valid_mask_i8(const GemmI8Args& g, int m) {
  const uint32_t P = (uint32_t)g.conv_P, L = (uint32_t)g.conv_L;
  const uint32_t line = (uint32_t)m / P;
  uint32_t x = (uint32_t)m - line * P, y = line % L;
  u32x4 v = {0u, 0u, 0u, 0u};
#pragma unroll
  for (int e = 0; e < CH; ++e) {
    const bool ok = x < (uint32_t)g.conv_W && y < (uint32_t)g.conv_H;
    if constexpr (CH == 4) v[e] = ok ? ~0u : 0u;
    else v[e >> 2] |= ok ? (0xffu << (8 * (e & 3))) : 0u;
    if (++x == P) { x = 0; if (++y == L) y = 0; }
  }
  return v;
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
