// One-shot magnitude pruning of a device-resident weight into a TW / TVW mask
// (Algorithm 3: TW-C on whole columns, Condense, TW-R on the (1,G) row pieces of
// every tile of kept columns; TVW: then 2 of every 4 consecutive kept rows per
// column, Algorithm 2's VW with vectors of 4 and 50 %).  The importance score
// is the sum of squares (Section IV names weight magnitude as the simplest score;
// the paper's Taylor score needs gradients).
//
// Scores are exact: an fp16 value is an integer multiple of 2^-24, its square
// an integer multiple of 2^-48 below 2^80, and the sums are kept in 128-bit
// integers, so the ranking does not depend on the order of summation and a
// host implementation with big integers takes the same decisions.  Ranking is
// by (score, index): the lowest n are pruned, equal scores lose the lower index
// first.  This runs once per weight; the kernels are simple on purpose.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "prune.h"
#include "scan.h"

namespace twg {

namespace {

typedef unsigned __int128 u128;

__device__ __forceinline__ uint64_t magnitude24(uint16_t h) {   // |value| in units of 2^-24
  const uint32_t e = (h >> 10) & 31u, m = h & 1023u;
  return e == 0 ? (uint64_t)m : (uint64_t)(m | 1024u) << (e - 1);
}
__device__ __forceinline__ u128 square48(uint16_t h) {
  const uint64_t a = magnitude24(h);
  return (u128)a * (u128)a;
}
__device__ __forceinline__ bool before(u128 sa, int ia, u128 sb, int ib) {   // (score, index) order
  return sa < sb || (sa == sb && ia < ib);
}

// TW-C scores in two steps, exact and independent of any order (integer sums): thread (column,
// slice y of the rows k = y, y + slices, ..) writes the slice's sum of squares; column_score_finish
// adds a column's slices and clears its rank counter for the counting that follows.
__global__ void column_partial(const uint16_t* B, int K, int N, int ldb, u128* partial) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  u128 s = 0;
  for (int k = blockIdx.y; k < K; k += gridDim.y) s += square48(B[(size_t)k * ldb + n]);
  partial[(size_t)blockIdx.y * N + n] = s;
}
__global__ void column_score_finish(const u128* partial, int slices, int N, u128* score, int32_t* rank) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  u128 s = 0;
  for (int y = 0; y < slices; ++y) s += partial[(size_t)y * N + n];
  score[n] = s;
  rank[n] = 0;
}

// Rank by counting, in parts: workgroup (x, y, z) compares entries [256 x, +256) of segment z
// with entries [256 y, +256) of the same segment (staged in LDS; all lanes read the same LDS
// address, a broadcast) and adds the number that come before in (score, index) order to
// rank[i].  grid.z = segment (one for the columns, one per tile for the rows).
__global__ void rank_partial(const u128* score, int len, int32_t* rank) {
  constexpr int CHUNK = 256;
  __shared__ u128 chunk[CHUNK];
  const u128* s = score + (size_t)blockIdx.z * len;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  const int c0 = blockIdx.y * CHUNK, cn = min(CHUNK, len - c0);
  if ((int)threadIdx.x < cn) chunk[threadIdx.x] = s[c0 + threadIdx.x];
  __syncthreads();
  if (i >= len) return;
  const u128 mine = s[i];
  int r = 0;
  for (int j = 0; j < cn; ++j) r += before(chunk[j], c0 + j, mine, i);
  if (r) atomicAdd(rank + (size_t)blockIdx.z * len + i, r);
}
// keep[i] = 1 unless i is among the `n_pruned` lowest of its segment (in place: rank -> keep).
__global__ void keep_from_rank(int32_t* rank_keep, size_t n, int n_pruned) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) rank_keep[i] = rank_keep[i] >= n_pruned;
}
// TW-R scores: tile t = kept columns [t*G, min((t+1)*G, n_kept)); one wave per (tile, row), its
// lanes over the tile's columns (neighbouring lanes read neighbouring kept columns of one row).
// The lanes' 128-bit sums meet as three 32-bit limbs, each in a 64-bit word (64 lanes cannot
// overflow it), added across the wave; lane 0 carries them into the score and clears the row's
// rank counter.
__global__ void tile_row_scores(const uint16_t* B, int K, int ldb, int G, int n_kept,
                                const int32_t* kept_cols, u128* score, int32_t* rank) {
  const int t = blockIdx.y, lane = threadIdx.x & 63;
  const int k = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (k >= K) return;                                   // whole waves leave together
  const int c0 = t * G, c1 = min(c0 + G, n_kept);
  u128 s = 0;
  for (int c = c0 + lane; c < c1; c += 64) s += square48(B[(size_t)k * ldb + kept_cols[c]]);
  unsigned long long l0 = (uint32_t)s, l1 = (uint32_t)(s >> 32), l2 = (unsigned long long)(s >> 64);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) {
    l0 += __shfl_xor(l0, d);
    l1 += __shfl_xor(l1, d);
    l2 += __shfl_xor(l2, d);
  }
  if (lane == 0) {
    score[(size_t)t * K + k] = (u128)l0 + ((u128)l1 << 32) + ((u128)l2 << 64);
    rank[(size_t)t * K + k] = 0;
  }
}

// tile_mask[k][n] = column n kept and row k kept in n's tile; `mask` (TVW) starts as zeros.
__global__ void emit_tile_mask(int K, int N, int G, const int32_t* col_pos, const int32_t* row_keep,
                               uint8_t* tile_mask, uint8_t* zeroed) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (size_t)K * N) return;
  const int k = (int)(i / N), n = (int)(i % N);
  const int p = col_pos[n];
  const uint8_t v = p >= 0 && row_keep[(size_t)(p / G) * K + k];
  if (tile_mask) tile_mask[i] = v;
  if (zeroed) zeroed[i] = 0;
}

// 2:4 along the condensed kept rows of a tile: in every group of 4 consecutive kept rows
// and every column keep the 2 largest |w|; equal magnitudes: the lower position stays.
__global__ void two_of_four(const uint16_t* B, int K, int N, int ldb, int G, int n_kept, int rows_kept,
                            const int32_t* kept_cols, const int32_t* row_list, uint8_t* mask) {
  const int t = blockIdx.z, g = blockIdx.y, c = t * G + blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= min((t + 1) * G, n_kept) || (int)(blockIdx.x * blockDim.x + threadIdx.x) >= G) return;
  const int n = kept_cols[c];
  const int32_t* rows = row_list + (size_t)t * K + 4 * g;
  const int cnt = min(4, rows_kept - 4 * g);
  uint64_t mag[4];
  for (int p = 0; p < cnt; ++p) mag[p] = magnitude24(B[(size_t)rows[p] * ldb + n]);
  for (int p = 0; p < cnt; ++p) {
    int larger = 0;     // positions that come first: larger magnitude, or equal and lower
    for (int q = 0; q < cnt; ++q) larger += q != p && (mag[q] > mag[p] || (mag[q] == mag[p] && q < p));
    if (larger < 2) mask[(size_t)rows[p] * N + n] = 1;
  }
}

size_t align_up(size_t x) { return (x + 255) / 256 * 256; }

}  // namespace

// Row slices of the column scores: about 512 workgroups of 256 columns in all, so at most
// 2 MiB of partial sums whatever the shape.
static int column_slices(int K, int N) {
  const int nbx = (N + 255) / 256;
  const int want = 512 / nbx > 1 ? 512 / nbx : 1;
  return K < want ? K : want;
}

size_t prune_workspace_bytes(int K, int N, int G) {
  const size_t nt = (size_t)(N + G - 1) / G;
  return align_up((size_t)N * 16) + 3 * align_up((size_t)N * 4) +          // column score, keep, pos, list
         align_up(nt * K * 16) + 3 * align_up(nt * K * 4) +                 // row score, keep, pos, list
         align_up((size_t)column_slices(K, N) * N * 16);                    // column scores per row slice
}

hipError_t prune_device(const uint16_t* B, int K, int N, int ldb, int G, bool tvw, int n_cols_pruned,
                        int rows_per_tile, uint8_t* mask, uint8_t* tile_mask, void* workspace,
                        hipStream_t stream) {
  const int n_kept = N - n_cols_pruned;
  const int nt = (n_kept + G - 1) / G;
  char* w = (char*)workspace;
  const size_t ntmax = (size_t)(N + G - 1) / G;
  u128* col_score = (u128*)w;            w += align_up((size_t)N * 16);
  int32_t* col_keep = (int32_t*)w;       w += align_up((size_t)N * 4);
  int32_t* col_pos = (int32_t*)w;        w += align_up((size_t)N * 4);
  int32_t* kept_cols = (int32_t*)w;      w += align_up((size_t)N * 4);
  u128* row_score = (u128*)w;            w += align_up(ntmax * K * 16);
  int32_t* row_keep = (int32_t*)w;       w += align_up(ntmax * K * 4);
  int32_t* row_pos = (int32_t*)w;        w += align_up(ntmax * K * 4);
  int32_t* row_list = (int32_t*)w;       w += align_up(ntmax * K * 4);
  u128* col_partial = (u128*)w;
  const int T = 256;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this call's
  // a failed launch ends the call: later kernels would read workspace nobody wrote
#define TWG_LAUNCH(kernel, grid, block, ...)                                  \
  do {                                                                        \
    hipLaunchKernelGGL(kernel, grid, block, 0, stream, __VA_ARGS__);          \
    const hipError_t e_ = hipGetLastError();                                  \
    if (e_ != hipSuccess) return e_;                                          \
  } while (0)
  // (counters are cleared by the kernels, not by memset nodes: the caller may be capturing a graph)
  const int ky = column_slices(K, N);
  const unsigned nb = (unsigned)((N + T - 1) / T);
  TWG_LAUNCH(column_partial, dim3(nb, ky), dim3(T), B, K, N, ldb, col_partial);
  TWG_LAUNCH(column_score_finish, dim3(nb), dim3(T), col_partial, ky, N, col_score, col_keep);
  TWG_LAUNCH(rank_partial, dim3(nb, nb, 1), dim3(T), col_score, N, col_keep);
  TWG_LAUNCH(keep_from_rank, dim3(nb), dim3(T), col_keep, (size_t)N, n_cols_pruned);
  TWG_LAUNCH(compact, dim3(1), dim3(1024), col_keep, N, col_pos, kept_cols);
  if (nt > 0) {
    TWG_LAUNCH(tile_row_scores, dim3((K + 3) / 4, nt), dim3(T), B, K, ldb, G, n_kept, kept_cols, row_score, row_keep);
    const unsigned kb = (unsigned)((K + T - 1) / T), all = (unsigned)(((size_t)nt * K + T - 1) / T);
    TWG_LAUNCH(rank_partial, dim3(kb, kb, nt), dim3(T), row_score, K, row_keep);
    TWG_LAUNCH(keep_from_rank, dim3(all), dim3(T), row_keep, (size_t)nt * K, K - rows_per_tile);
  }
  const size_t total = (size_t)K * N;
  const unsigned eb = (unsigned)((total + T - 1) / T);      // the caller keeps K * N / 256 inside the grid limit
  if (tvw) {      // tile mask (if asked for) and an all-zero element mask for the 2:4 step to fill
    TWG_LAUNCH(emit_tile_mask, dim3(eb), dim3(T), K, N, G, col_pos, row_keep, tile_mask, mask);
  } else {        // TW: the element mask is the tile mask
    TWG_LAUNCH(emit_tile_mask, dim3(eb), dim3(T), K, N, G, col_pos, row_keep, mask, (uint8_t*)nullptr);
    if (tile_mask)
      TWG_LAUNCH(emit_tile_mask, dim3(eb), dim3(T), K, N, G, col_pos, row_keep, tile_mask, (uint8_t*)nullptr);
  }
  if (tvw && nt > 0 && rows_per_tile > 0) {
    TWG_LAUNCH(compact, dim3(nt), dim3(1024), row_keep, K, row_pos, row_list);
    const int groups = (rows_per_tile + 3) / 4;
    TWG_LAUNCH(two_of_four, dim3((G + 63) / 64, groups, nt), dim3(64), B, K, N, ldb, G, n_kept, rows_per_tile,
               kept_cols, row_list, mask);
  }
#undef TWG_LAUNCH
  return hipSuccess;
}

// ---- scratch for callers that cannot allocate -------------------------------------------
// One array per GPU, held until the process ends.  In host code its name is only a stand-in:
// the device address comes from hipGetSymbolAddress, once per device, and that pointer is what
// the kernels receive.
static __device__ __align__(256) unsigned char scratch[PRUNE_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex scratch_mutex;
void* scratch_ptr[MAX_DEVICES];     // per device: address of that device's copy of `scratch`
}  // namespace

hipError_t prune_static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (!scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    scratch_ptr[dev] = p;
  }
  *out = scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace twg
