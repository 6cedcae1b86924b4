// Internal: device-side helpers shared by the kernels of this library.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace twg {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef int int2v __attribute__((ext_vector_type(2)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))
#define GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

constexpr int KS = 32;        // condensed rows per main-loop stage
constexpr int NTHREADS = 256;

// XOR mask applied to the byte offset inside a row of a k-major LDS tile with
// RB bytes per row.  The LDS has 64 banks of 4 bytes; one half-wave of a
// transposing read touches 4 consecutive rows x 64 bytes, and the mask sends
// those four pieces to the four different quarters of the 256-byte bank period.
template <int RB>
__device__ __forceinline__ int swz_mask(int row) {
  if constexpr (RB % 256 == 0) return (row & 3) << 6;
  else if constexpr (RB == 128) return ((row >> 1) & 1) << 6;  // two rows per period
  else return 0;                                                // RB == 64: four rows = one period
}
template <int RB>
__device__ __forceinline__ int swz(int row, int xbytes) {
  return row * RB + (xbytes ^ swz_mask<RB>(row));
}

// Workgroup id -> logical id.  Consecutive workgroup ids are dealt round-robin
// to the 8 XCDs (each with its own L2); the remap hands every XCD a contiguous
// range of logical ids.
__device__ __forceinline__ int xcd_remap(int bid, int n) {
  const int xcd = bid & 7, slot = bid >> 3;
  const int per = n >> 3, rem = n & 7;
  return (xcd < rem) ? xcd * (per + 1) + slot : rem * (per + 1) + (xcd - rem) * per + slot;
}

// Workgroup id -> (M-tile, launch position of the N-tile).
// mode 1: the XCD's contiguous range of logical ids, M-tile major.
// mode 2 (when the M-tiles divide evenly among the 8 XCDs): inside the XCD the
// ids are tile major and dealt so that the workgroups that start together on
// one CU (an idle XCD places its workgroups round-robin over its 32 CUs, so
// these are XCD-local slots s, s+32, s+64, ..) are consecutive: they work on
// the same weight tile at the same pace, and its rows are fetched from L2 once
// per CU rather than once per workgroup.
template <class Args>
__device__ __forceinline__ void tile_of_workgroup(const Args& g, int bid, int n_gemm, int& mt, int& t) {
  if (g.xcd_map == 2 && (g.n_mtiles & 7) == 0) {
    const int xcd = bid & 7, slot = bid >> 3;
    const int mts = g.n_mtiles >> 3, cnt = mts * g.n_tiles;
    const int cu = slot & 31, round = slot >> 5;
    const int rf = cnt >> 5, rn = cnt & 31;
    const int L = cu * rf + (cu < rn ? cu : rn) + round;
    t = L / mts;
    mt = xcd * mts + (L - t * mts);
    return;
  }
  const int lid = g.xcd_map ? xcd_remap(bid, n_gemm) : bid;
  mt = lid / g.n_tiles;
  t = lid - mt * g.n_tiles;
}

// Implicit img2col: which of the 8 wide-grid positions m .. m+7 are output pixels (x < W and
// y < H); all-ones halves for those, zero for the padding lanes.  One division per thread.
__device__ __forceinline__ u32x4 conv_valid_mask(const GemmArgs& g, int m) {
  const uint32_t P = (uint32_t)g.conv_P, L = (uint32_t)g.conv_L;
  const uint32_t line = (uint32_t)m / P;
  uint32_t x = (uint32_t)m - line * P, y = line % L;
  uint32_t h[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    h[e] = (x < (uint32_t)g.conv_W && y < (uint32_t)g.conv_H) ? 0xffffu : 0u;
    if (++x == P) { x = 0; if (++y == L) y = 0; }
  }
  u32x4 v;
#pragma unroll
  for (int j = 0; j < 4; ++j) v[j] = h[2 * j] | (h[2 * j + 1] << 16);
  return v;
}

// Extra workgroups of a launch write +0 into one pruned column of C each.
__device__ __forceinline__ void zero_fill_column(const GemmArgs& g, int which) {
  const int col = g.zero_cols[which];
  _Float16* row = g.C + (size_t)col * g.ldc;
  const u32x4 z = {0u, 0u, 0u, 0u};
  for (int m = threadIdx.x * 8; m < g.M; m += (int)blockDim.x * 8) {
    if (m + 8 <= g.M) __builtin_nontemporal_store(z, (u32x4*)(row + m));
    else for (int i = m; i < g.M; ++i) row[i] = (_Float16)0.f;
  }
}

}  // namespace twg
