// Internal: stream compaction shared by the device pruner and the device packer.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace twg {

// Condense: positions of the kept entries of each segment, in ascending order.
// One workgroup per segment (blockIdx.x); pos[i] = index among the kept (or -1), list[pos] = i.
static __global__ void compact(const int32_t* keep, int len, int32_t* pos, int32_t* list) {
  __shared__ int part[1024];
  __shared__ int base;
  const int32_t* kp = keep + (size_t)blockIdx.x * len;
  int32_t* ps = pos + (size_t)blockIdx.x * len;
  int32_t* ls = list + (size_t)blockIdx.x * len;
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (int c0 = 0; c0 < len; c0 += (int)blockDim.x) {
    const int i = c0 + threadIdx.x;
    const int v = i < len ? (kp[i] != 0) : 0;
    part[threadIdx.x] = v;
    __syncthreads();
    for (int d = 1; d < (int)blockDim.x; d <<= 1) {          // inclusive scan
      const int add = (int)threadIdx.x >= d ? part[threadIdx.x - d] : 0;
      __syncthreads();
      part[threadIdx.x] += add;
      __syncthreads();
    }
    if (i < len) {
      const int p = base + part[threadIdx.x] - v;
      ps[i] = v ? p : -1;
      if (v) ls[p] = i;
    }
    __syncthreads();
    if (threadIdx.x == 0) base += part[blockDim.x - 1];
    __syncthreads();
  }
}

}  // namespace twg
