// Internal: kernel argument block and launchers (host side sees only this).
#pragma once
#include <hip/hip_runtime_api.h>
#include <stdint.h>

namespace twg {

struct GemmArgs {
  const _Float16* A;   // KM kernels: K x M, element (i,k) at A[k*lda + i]; MK: A[i*lda + k]
  _Float16* C;         // KM kernels: N x M, element (i,n) at C[n*ldc + i]; MK: C[i*ldc + n]
  int M, lda, ldc;
  // TW: condensed weight image [sum Kp_t][G]; dense: B, K x N row-major
  const _Float16* vals;
  int ldb;                       // dense only
  const int32_t* row_idx;        // TW: padded kept-row lists (CTO_k as indices)
  const int32_t* tile_kp_off;    // TW: n_tiles+1 offsets into row_idx
  const int32_t* col_idx;        // TW: n_tiles*G kept-column indices, -1 = none (CTO_n)
  const int32_t* tile_order;     // TW: launch order of tiles (longest first) or null
  const int32_t* tile_sched;     // TW: per launch position {tile, kp offset, Kp_t, width}, 16-byte records
  int uniform_kp;                // > 0: every tile has this padded K_t and launch position = tile, so the
                                 // record is (pos, pos * uniform_kp, uniform_kp) and need not be loaded
  const int32_t* zero_cols;      // pruned columns of C, written as +0
  const uint32_t* meta;          // TVW: 2:4 position words
  const int32_t* ew_ptr;         // TEW: N+1 offsets into ew_pairs by original column of C
  const uint32_t* ew_pairs;      // TEW: restored elements, K row << 16 | fp16 bits (at least one readable word)
  int ew_last;                   // TEW: index of the last pair (0 when there is none)
  int n_zero;
  int n_tiles, n_mtiles;
  int K, N;                      // dense only
  int xcd_map;
  // Implicit img2col (0 = off): the "rows" of A are window shifts into a wide input (row list =
  // element offsets, lda = 1) and M counts the positions of the wide grid, P per line, L lines
  // per image block; positions with x >= W or y >= H are written as +0.
  int conv_P, conv_L, conv_H, conv_W;
  // K split across workgroups (1 = off): wg_split workgroups share one (M-tile, N-tile) pair on
  // disjoint ranges of the kept rows; fp32 partial tiles go to ws_partials, the workgroup that
  // arrives last at ws_counters[pair] adds them up in split order and runs the epilogue.
  int tiles_per_wg;              // asynchronous TW kernel: jobs per workgroup (> 1: the instances that loop)
  int wg_split;
  float* ws_partials;            // [pair][split][tile] fp32
  int* ws_counters;              // one per pair; zero between launches (the last arriver resets it)
};

// Int8 operands, int32 sums (gemm_i8.hip); layouts as the KM kernels above.
struct GemmI8Args {
  const int8_t* A;               // K x M bytes, element (i,k) at A[k*lda + i]
  void* C;                       // N x M, int32 or (c_i8) requantised int8
  int M, lda, ldc;
  int c_i8;
  float scale;
  const int8_t* vals;            // TW: condensed image [sum Kp_t][G] bytes; dense: B, K x N row-major
  int ldb;                       // dense only
  const int32_t* row_idx;
  const int32_t* col_idx;
  const int32_t* tile_sched;
  int uniform_kp;                // as in GemmArgs
  const int32_t* zero_cols;
  const uint32_t* meta;          // TVW: 2:4 position words
  int n_zero;
  int n_tiles, n_mtiles;
  int K, N;                      // dense only
  int xcd_map;
  int conv_P, conv_L, conv_H, conv_W;   // implicit img2col, as in GemmArgs (0 = off)
};
// G / tn in {64, 128}, tm in {128, 256} (and 64 for G = 128); hipErrorInvalidValue when no instance exists.
// The dense variant needs K % 64 == 0.
// ksplit = 2: two groups of four waves split K inside the workgroup (G = 128 with tm 64 / 128, G = 64 with tm 128).
hipError_t launch_tw_i8(int G, int tm, int ksplit, GemmI8Args g, hipStream_t stream);
hipError_t launch_dense_i8(int tn, int tm, GemmI8Args g, hipStream_t stream);
// int8 TVW on the sparse matrix instruction (gemm_tvw_i8.hip): G = 128 with tm in {64, 128}, G = 64 with tm = 128.
hipError_t launch_tvw_i8(int G, int tm, GemmI8Args g, hipStream_t stream);

// G / tn: tile width (32, 64, 128); tm: M-tile (64, 128, 256).
// hipErrorInvalidValue when no instance exists for (G, tm).
hipError_t launch_tw_km(int G, int tm, GemmArgs g, hipStream_t stream);
hipError_t launch_dense_km(int tn, int tm, GemmArgs g, hipStream_t stream);
// Row-major A (M x K) and C (M x N): compatibility path on the register-staged kernel.
hipError_t launch_tw_mk(int G, GemmArgs g, hipStream_t stream);
hipError_t launch_dense_mk(int tn, GemmArgs g, hipStream_t stream);
// Asynchronous-copy pipeline (gemm_dma.hip): G / tn in {64, 128}, depth = stages
// in flight (3 or 4); the dense variant needs K % 32 == 0.
// variant: DMA_WAVES4 = 4 waves per workgroup; DMA_WAVES8 = 8 waves splitting the tile
// (tm in {128, 256}, G = 128); DMA_KSPLIT2 = two groups of 4 waves splitting K inside
// the workgroup (dense: K % 64 == 0).
enum { DMA_WAVES4 = 0, DMA_WAVES8 = 1, DMA_KSPLIT2 = 2 };
// lidx: kept-row list through LDS (true) or by scalar loads (false; 4-wave and 8-wave instances
// at depth 3 / 4 have both routes, the others ignore it).
hipError_t launch_tw_km_dma(int G, int tm, int depth, int variant, bool lidx, GemmArgs g, hipStream_t stream);
// The same with K split across g.wg_split workgroups per tile (4 waves, 3 stages): (G, tm) in
// {(128, 128), (128, 64), (64, 128)}.
hipError_t launch_tw_km_dma_split(int G, int tm, GemmArgs g, hipStream_t stream);
// The same with the restored elements of a TEW weight added in the epilogue (g.ew_*).
hipError_t launch_tew_km_dma(int G, int tm, int depth, int variant, bool lidx, GemmArgs g, hipStream_t stream);
hipError_t launch_dense_km_dma(int tn, int tm, int depth, int variant, GemmArgs g, hipStream_t stream);
// Zero fill of n 32-bit words (the counters of a workspace).
hipError_t launch_zero_words(uint32_t* p, int n, hipStream_t stream);
// TVW (2:4 inside the kept rows) on the sparse matrix instruction (gemm_tvw.hip).
hipError_t launch_tvw_km(int G, int tm, int depth, GemmArgs g, hipStream_t stream);

}  // namespace twg
