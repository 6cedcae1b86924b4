/*
 * twgemm.h - C ABI of the tile-wise (TW) / tile-vector-wise (TVW) sparse GEMM
 * library for AMD MI355X (gfx950).
 *
 * The operation (paper Section III-A): C = A x B with A (M x K) activations,
 * B (K x N) a pruned weight and C (M x N).  B is pruned tile-wise: whole
 * columns are dropped (TW-C), the kept columns are cut into tiles of G, and
 * every tile drops its own set of K-rows (TW-R).  TVW additionally keeps only
 * 2 of every 4 consecutive kept rows per column (Section III-A, "TVW";
 * Algorithm 3).  TEW puts single elements back on top of a TW mask (Section
 * III-A, "TEW"; Algorithm 3, TEW); they are kept in compressed sparse column
 * form next to the TW part and, by linearity, added to the same fp32 sums
 * before the one rounding.  The library keeps B condensed per tile together with the
 * indices of the unpruned rows / columns (Section V, "Tile Fusion and
 * Compressed Tile Offset"; Listing 1's CTO_k / CTO_n) and computes
 *
 *      C = A . (B (.) mask)          fp16 inputs, fp32 accumulation, one
 *                                    round-to-nearest-even to fp16
 *
 * in one kernel launch: gather of the kept rows of A, dense (or 2:4 sparse)
 * matrix-core contraction over the condensed K, scatter to the kept columns
 * of C.  alpha = 1 and beta = 0 (Listing 1's alpha/beta are not exposed).
 *
 * Conventions
 *  - "host" pointers are ordinary CPU memory, "dev" pointers are device
 *    memory of the current HIP device.  fp16 values travel as uint16_t bit
 *    patterns on the host side and as raw 2-byte elements on the device.
 *  - The caller owns every buffer it passes; tw_pack* copy what they need.
 *    The library owns everything behind a handle until tw_free.
 *  - All functions return a tw_status; nothing throws across the boundary.
 *  - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *    tw_gemm / tw_dense_gemm only enqueue work on it: they never synchronise
 *    and never allocate.
 *  - Inputs are assumed finite.
 */
#ifndef TWGEMM_H
#define TWGEMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tw_handle_s* tw_handle_t; /* opaque packed weight */

typedef enum {
  TW_OK = 0,
  TW_ERR_ARG = 1,         /* null pointer, non-positive size, bad enum, misaligned buffer */
  TW_ERR_MASK = 2,        /* mask does not have the TW / TVW structure                    */
  TW_ERR_UNSUPPORTED = 3, /* valid request this build has no kernel for                   */
  TW_ERR_ALLOC = 4,       /* host or device allocation failed                             */
  TW_ERR_HIP = 5,         /* a HIP runtime call failed (no device, launch error)          */
  TW_ERR_STATE = 6,       /* handle has no device copy yet / already freed                */
  TW_ERR_TOO_LARGE = 7    /* tw_prune_dev_static: the problem needs more scratch than the
                             library's fixed array holds                                  */
} tw_status;

typedef enum { TW_PATTERN_TW = 0, TW_PATTERN_TVW = 1, TW_PATTERN_TEW = 2 } tw_pattern;

/* Element type of a packed weight (and of the A it multiplies). */
typedef enum { TW_DTYPE_F16 = 0, TW_DTYPE_I8 = 1 } tw_dtype;

/*
 * Memory layout of A and C.  Section V ("Memory Accesses Coalesce") stores the
 * tiles transposed so that skipping a K-column of A / an N-column of C becomes
 * skipping a contiguous row; TW_LAYOUT_KM is that form and the fast path.
 *   TW_LAYOUT_KM: A is stored K x M (element (i,k) at A[k*lda + i]),
 *                 C is stored N x M (element (i,n) at C[n*ldc + i]).
 *   TW_LAYOUT_MK: A is M x K row-major (A[i*lda + k]), C is M x N row-major.
 */
typedef enum { TW_LAYOUT_KM = 0, TW_LAYOUT_MK = 1 } tw_layout;

/*
 * Logical (layout-independent) view of a packed weight; all pointers are host
 * memory owned by the handle and valid until tw_free.
 *
 *   col_idx[n_kept]       ascending original indices of kept columns   (CTO_n as indices)
 *   cto_n[n_kept]         col_idx[j] - j                                (offset form, Section V)
 *   tile_k_off[n_tiles+1] prefix sums of K_t, the kept-row count of tile t
 *   row_idx[sum K_t]      per tile, ascending original K indices        (CTO_k as indices)
 *   cto_k[sum K_t]        row_idx[tile t][j] - j
 *   tile_col_off[n_tiles+1]  tile t covers condensed columns [tile_col_off[t],
 *        tile_col_off[t+1]), width W_t <= G.  From tw_pack: tile_col_off[t] =
 *        min(t*G, n_kept); a handle from tw_concat keeps its members' tile bounds.
 *   TW : values at val_off[t]: K_t x W_t row-major,
 *        V[j][w] = B[row_idx[t][j]][col_idx[tile_col_off[t]+w]]
 *   TVW: groups of 4 consecutive entries of row_idx[t]; n_g = ceil(K_t/4).
 *        values at val_off[t]: n_g x 2 x W_t; meta/valid at meta_off[t]: n_g x W_t bytes.
 *        meta  = p0 | p1<<2 with p0 < p1 the two stored positions of the group,
 *        valid = v0 | v1<<1, v_i = 1 if stored value i is a kept element of the
 *        mask (else it is a +0 filler).
 *   TEW: the TW fields describe the TW-level tile mask; the restored elements
 *        (mask set, tile mask clear) follow in compressed sparse column form over
 *        the ORIGINAL columns, pruned ones included: ew_col_ptr[N+1],
 *        ew_row[ew_nnz] ascending inside a column, ew_val[ew_nnz] fp16 bits.
 */
typedef struct {
  int32_t K, N, G, pattern;
  int32_t n_kept, n_tiles;
  const int32_t* col_idx;
  const int32_t* cto_n;
  const int32_t* tile_k_off;
  const int32_t* row_idx;
  const int32_t* cto_k;
  const int64_t* val_off;   /* n_tiles+1, in fp16 elements */
  const uint16_t* values;
  const int64_t* meta_off;  /* n_tiles+1, in bytes; NULL for TW */
  const uint8_t* meta;      /* NULL for TW */
  const uint8_t* valid;     /* NULL for TW */
  const int32_t* tile_col_off;
  int64_t ew_nnz;              /* 0 unless TEW */
  const int32_t* ew_col_ptr;   /* NULL unless TEW */
  const int32_t* ew_row;
  const uint16_t* ew_val;
  int32_t dtype;               /* TW_DTYPE_I8: every entry of `values` is an int8 value,
                                  sign-extended to 16 bits; offsets count elements */
} tw_packed_view;

/*
 * tw_pack_host - condense a pruned weight on the host (Section V: the weight is
 * condensed once, ahead of inference, not per call; Algorithm 3's Condense).
 *   B_host     K x N row-major fp16 bit patterns (ldb = N)
 *   mask_host  K x N bytes, non-zero = kept
 *   tile_mask_host  TVW, may be NULL: the TW-level mask the 2:4 step was
 *              applied to.  When NULL the kept rows/columns are the ones with
 *              any mask bit.  TEW, required: the TW-level mask; mask_host must
 *              contain it, what it adds are the restored elements.  Ignored for TW.
 *   G          tile width along N: 32, 64 or 128
 * Errors: TW_ERR_ARG (null / K,N < 1 / bad G or pattern / TEW without tile mask),
 * TW_ERR_MASK (a kept row of a tile has a hole, the element mask leaves the
 * tile mask (TVW) or does not contain it (TEW), or a 2:4 group keeps more than
 * two), TW_ERR_UNSUPPORTED (TEW with K > 65536), TW_ERR_ALLOC.  Touches no GPU.
 */
tw_status tw_pack_host(const uint16_t* B_host, const uint8_t* mask_host,
                       const uint8_t* tile_mask_host, int K, int N, int G,
                       int pattern, tw_handle_t* out);

/* tw_upload - copy the device image of a packed weight to the current HIP
 * device (synchronous).  Idempotent.  Errors: TW_ERR_ARG, TW_ERR_ALLOC, TW_ERR_HIP. */
tw_status tw_upload(tw_handle_t h);

/* tw_pack - tw_pack_host followed by tw_upload ("tw_pack(B, mask, G, pattern) -> handle"). */
tw_status tw_pack(const uint16_t* B_host, const uint8_t* mask_host,
                  const uint8_t* tile_mask_host, int K, int N, int G,
                  int pattern, tw_handle_t* out);

/*
 * tw_prune_dev - one-shot pruning of a weight that lives on the device into a TW
 * or TVW mask, also on the device (Algorithm 3, TW and TVW, with the sum of
 * squares as importance score; the multi-stage schedule of Algorithm 1 and the
 * Taylor score of Section IV need training data and are not part of this).
 *   TW-C: the n_cols_pruned columns with the lowest scores are dropped.
 *   TW-R: the kept columns are cut into tiles of G; in every tile the
 *         rows_per_tile rows with the highest scores are kept.
 *   TVW : in every tile, every run of 4 consecutive kept rows keeps per column
 *         the 2 largest |w| (equal magnitudes: the lower position stays).
 * Scores are exact integers (squares in units of 2^-48, 128-bit sums), ranked by
 * (score, index): the result does not depend on summation order.
 *   B_dev       K x N fp16 row-major, ldb >= N, finite values
 *   mask_dev    K x N bytes, written 0/1;  tile_mask_dev  the TW-level mask, may be NULL
 *   workspace_dev, workspace_bytes   scratch of at least tw_prune_workspace_bytes(K, N, G),
 *               16-byte aligned, owned by the caller
 * Only enqueues kernels on `stream`; allocates nothing.  Errors: TW_ERR_ARG,
 * TW_ERR_UNSUPPORTED (TEW), TW_ERR_HIP.
 */
tw_status tw_prune_workspace_bytes(int K, int N, int G, size_t* bytes);
tw_status tw_prune_dev(const void* B_dev, int K, int N, int ldb, int G, int pattern,
                       int n_cols_pruned, int rows_per_tile, uint8_t* mask_dev,
                       uint8_t* tile_mask_dev, void* workspace_dev, size_t workspace_bytes,
                       void* stream);

/*
 * tw_prune_dev_static - tw_prune_dev for callers that cannot allocate or hand over device
 * memory beyond inputs and outputs: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments minus the workspace, same kernels, same
 * result; the scratch is a fixed array of 8 MiB inside the library's device code (one per
 * GPU, held until the process ends) instead of a caller buffer.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine).
 *   Limit: tw_prune_workspace_bytes(K, N, G) <= 8 MiB, i.e. ceil(N/G) * K * 28 + N * 28 bytes
 *   plus alignment (768 x 3072 at G = 128: 0.6 MiB; 4096 x 4096 at G = 128: 3.6 MiB); larger
 *   problems get TW_ERR_TOO_LARGE and nothing is enqueued.
 *   Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams,
 *   two threads) race; serialise them or use tw_prune_dev with separate workspaces.  Nothing
 *   in the array has to start at zero; it keeps the last call's contents.
 * Errors: as tw_prune_dev, plus TW_ERR_TOO_LARGE.
 */
tw_status tw_prune_dev_static(const void* B_dev, int K, int N, int ldb, int G, int pattern,
                              int n_cols_pruned, int rows_per_tile, uint8_t* mask_dev,
                              uint8_t* tile_mask_dev, void* stream);

/*
 * tw_pack_dev - tw_pack for a weight and masks in device memory (Algorithm 3's Condense and
 * Section V's offline condensing, run by kernels on `stream`).  TW and TVW: the kept-column
 * list, the per-tile kept-row lists, the condensed values, the 2:4 positions and the
 * kernel-facing image are all produced on the device; only the index lists (a few KB) visit
 * the host, which lays out offsets, padding and the launch order of the tiles exactly as for
 * tw_pack.  The result is the same handle bit for bit; its logical values are copied to the
 * host only when tw_export, tw_unpack or tw_concat ask for them.  TEW goes through the host
 * packer (the weight and masks are copied to the host).  Allocates device memory and waits
 * for `stream`: an offline step like tw_pack.  Arguments and errors as tw_pack_host, B with
 * leading dimension ldb >= N; TW_ERR_HIP for a failed runtime call.
 */
tw_status tw_pack_dev(const void* B_dev, int ldb, const uint8_t* mask_dev,
                      const uint8_t* tile_mask_dev, int K, int N, int G, int pattern,
                      void* stream, tw_handle_t* out);

/*
 * tw_concat - one handle for the weights parts[0..n) side by side along N:
 * B = [B_0 | B_1 | ...] (same K, G and pattern; N = sum of the members' N).
 * A tw_gemm on it computes the members' products from one read of A in one
 * launch, which is how independent GEMMs on the same input (the Q, K and V
 * projections of an attention layer) fill the device together; Section V
 * ("Tile Fusion") runs a weight's tiles concurrently for the same reason.
 * The members' tiles are kept as they are (no tile spans two members), so
 * rows [N_0 + .. + N_{i-1}, .. + N_i) of C (KM layout) are member i's C.
 * The members stay valid and independent.  upload != 0 also copies the device
 * image to the current device.  Errors: TW_ERR_ARG (null, n < 1, members
 * differ in K, G or pattern), TW_ERR_ALLOC, TW_ERR_HIP.
 */
tw_status tw_concat(const tw_handle_t* parts, int n, int upload, tw_handle_t* out);

/*
 * tw_gemm - C = A . (B (.) mask) for a packed weight (Listing 1 as one grouped
 * launch; every element of C is written, pruned columns as +0).
 *   A_dev, C_dev  device fp16; 16-byte aligned; lda, ldc in elements,
 *                 multiples of 8.  KM: lda >= M, ldc >= M.  MK: lda >= K, ldc >= N.
 *   M             >= 1
 * Asynchronous on `stream`; allocates nothing; concurrent calls must use
 * distinct C.  Errors: TW_ERR_ARG, TW_ERR_STATE (not uploaded),
 * TW_ERR_UNSUPPORTED (layout without a kernel: TVW and TEW exist for
 * TW_LAYOUT_KM only, TEW for G = 64 and 128), TW_ERR_HIP (launch failed).
 */
tw_status tw_gemm(const void* A_dev, int M, int lda, int layout, tw_handle_t h,
                  void* C_dev, int ldc, void* stream);

/*
 * tw_gemm_ex - tw_gemm with the launch options of THIS call (nothing process-wide is read when
 * `opts` is given, so threads may launch the same handle with different options at the same
 * time), and optionally a workspace that lets the library split long kept-row lists across
 * workgroups (Section V: few or uneven tiles leave the device under-used; one launch for all
 * tiles lets the scheduler even that out, and a weight with fewer (M-tile, N-tile) pairs than
 * the GPU has compute units needs its K loop shared out as well).
 *   opts          NULL = the defaults (tw_launch_opts_init's values); else every field as
 *                 described at tw_set_option, 0 = heuristic / default:
 *                   tile_m 0|64|128|256, kernel 0..2, depth 0|3..8, waves 0|4|8, ksplit 0..2,
 *                   xcd_map -1 (default) | 0 | 1 | 2,
 *                   wg_split 0 = automatic when a workspace is given, 1 = never,
 *                            2..8 = that many workgroups per (M-tile, N-tile) pair,
 *                   idx_route 0 = automatic, 1 = kept-row lists by scalar loads, 2 = through LDS,
 *                   tiles_per_wg 0 = automatic (one: more never measured faster), 1..8 = tiles a
 *                            workgroup of the asynchronous TW kernel computes one after the
 *                            other (same results bit for bit)
 *   workspace_dev device memory, 256-byte aligned, at least tw_gemm_workspace_bytes(h, M) bytes,
 *                 prepared ONCE with tw_workspace_init (its first 4 KiB are counters that every
 *                 launch leaves at zero again).  Launches that share a workspace must not
 *                 overlap (same stream, or ordered otherwise); after a failed launch call
 *                 tw_workspace_init again.  fp32 partial tiles are added in a fixed order before
 *                 the one rounding: results do not depend on timing.  TW pattern, TW_LAYOUT_KM,
 *                 G = 64 or 128; other launches ignore the workspace.
 * Asynchronous on `stream`; allocates nothing.  Errors: as tw_gemm; TW_ERR_ARG also for an
 * invalid option value, a misaligned workspace, or wg_split > 1 with a workspace too small.
 */
typedef struct {
  int32_t tile_m, kernel, depth, waves, ksplit, xcd_map, wg_split, idx_route, tiles_per_wg;
  void* workspace_dev;
  size_t workspace_bytes;
} tw_launch_opts;
tw_status tw_launch_opts_init(tw_launch_opts* opts);
tw_status tw_gemm_workspace_bytes(tw_handle_t h, int M, size_t* bytes);
tw_status tw_workspace_init(void* workspace_dev, size_t workspace_bytes, void* stream);
tw_status tw_gemm_ex(const void* A_dev, int M, int lda, int layout, tw_handle_t h,
                     void* C_dev, int ldc, const tw_launch_opts* opts, void* stream);

/*
 * tw_dense_gemm - the dense baseline C = A . B on the same matrix cores, same
 * layouts and precision (Section V: the dense tiled GEMM the method starts from).
 *   B_dev  device fp16, K x N row-major, ldb >= N, multiple of 8, 16-byte aligned.
 */
tw_status tw_dense_gemm(const void* A_dev, const void* B_dev, void* C_dev,
                        int M, int K, int N, int lda, int ldb, int ldc,
                        int layout, void* stream);

/*
 * Int8 (Section VI-B "Int8 Quantization": the pattern is independent of the
 * element type, the matrix cores run the same condensed product on int8
 * operands with int32 sums).  TW and TVW patterns, TW_LAYOUT_KM only.
 *
 * tw_pack_i8_host / tw_pack_i8 - as tw_pack_host / tw_pack for a K x N row-major
 *   int8 weight (ldb = N); pattern TW or TVW (TEW: TW_ERR_UNSUPPORTED), tile_mask as
 *   there.  Same errors.  The handle works with
 *   tw_upload, tw_concat (members of one dtype), tw_export (see `dtype`),
 *   tw_unpack (values sign-extended to 16 bits), tw_flop_counts and tw_free;
 *   tw_gemm refuses it (TW_ERR_ARG), as tw_gemm_i8 refuses an fp16 handle.
 * tw_gemm_i8 - C = A . (B (.) mask), exact in int32 (|sum| <= K * 2^14 < 2^31 for
 *   K <= 131071; larger K: TW_ERR_UNSUPPORTED).
 *   A_dev   device int8, K x M (element (i,k) at A[k*lda + i]), 16-byte aligned,
 *           lda >= M, multiple of 16, K * lda < 2^32
 *   C_dev   device, N x M (element (i,n) at C[n*ldc + i]), 16-byte aligned, ldc >= M,
 *           multiple of 16, in elements of:
 *             c_dtype = 0: int32 sums;
 *             c_dtype = 1: int8 = clamp(round-half-even(fp32(sum) * scale), -128, 127),
 *                          the product taken in fp32 with one rounding
 *           pruned columns are written as 0.
 *   Asynchronous on `stream`, allocates nothing.  Errors: TW_ERR_ARG, TW_ERR_STATE,
 *   TW_ERR_UNSUPPORTED (G = 32, K or A too large), TW_ERR_HIP.
 * tw_dense_gemm_i8 - the dense int8 baseline on the same matrix cores and layouts:
 *   B_dev K x N row-major int8, ldb >= N, multiple of 16, 16-byte aligned;
 *   K % 64 != 0 gives TW_ERR_UNSUPPORTED.
 */
tw_status tw_pack_i8_host(const int8_t* B_host, const uint8_t* mask_host,
                          const uint8_t* tile_mask_host, int K, int N, int G, int pattern,
                          tw_handle_t* out);
tw_status tw_pack_i8(const int8_t* B_host, const uint8_t* mask_host, const uint8_t* tile_mask_host,
                     int K, int N, int G, int pattern, tw_handle_t* out);
tw_status tw_gemm_i8(const void* A_dev, int M, int lda, tw_handle_t h, void* C_dev, int ldc,
                     int c_dtype, float scale, void* stream);
tw_status tw_dense_gemm_i8(const void* A_dev, const void* B_dev, void* C_dev, int M, int K, int N,
                           int lda, int ldb, int ldc, int c_dtype, float scale, void* stream);

/*
 * Convolution without a materialised img2col matrix (Section VI-A turns a convolution into
 * C = A x B by img2col; row m of A is the input window of output position m, row
 * k = (c*R + r)*S + s of the K x N weight is filter tap (r, s) of input channel c).
 * The input is stored "wide", channel-major, padding included:
 *     X[c*ldx + b*L*P + yy*P + xx],  c < C, b < B (images), yy < L (lines of an image
 *     block), xx < P (elements of a line),  L >= H+R-1,  P >= W+S-1.
 * Output position m = b*L*P + y*P + x is an output pixel iff y < H and x < W; its window is
 * X[c][m + r*P + s], so row k of A is the run of X that starts r*P + s elements into channel
 * c, and the kernel gathers it from there.  C is N x ldc with all B*L*P positions of the wide
 * grid: output pixels hold the convolution, the other positions +0 (where the zeros of a
 * zero-padded layout sit depends on the caller's (R-1)/2, (S-1)/2 shift; this call does not
 * care), pruned output channels +0.
 *
 * tw_conv_bind - bind a geometry to an uploaded TW or TVW handle (fp16 or int8) with
 *   K = C*R*S: *out receives a binding that owns the per-tile kept-row lists as element offsets
 *   on the device (allocates).  The handle is not changed: several bindings (geometries) of one
 *   handle may exist and launch at the same time; the handle must outlive them.  With c = 8
 *   (fp16) or 16 (int8) elements per 16-byte copy: ldx a multiple of c,
 *   ldx >= roundup_c(B*L*P) + (R-1)*P + S-1 so that the windows of the last positions stay
 *   inside channel rows of ldx elements; C*ldx < 2^31.
 *   Errors: TW_ERR_ARG, TW_ERR_STATE (not uploaded), TW_ERR_UNSUPPORTED (G = 32, TEW),
 *   TW_ERR_ALLOC, TW_ERR_HIP.
 * tw_conv_free - release a binding (NULL is a no-op).
 * tw_conv_gemm - the launch.  X_dev fp16, C rows of ldx elements, 16-byte aligned; C_dev fp16
 *   N x ldc, ldc >= B*L*P, multiple of 8, 16-byte aligned.  Asynchronous on `stream`,
 *   allocates nothing.  Errors: TW_ERR_ARG (also: a binding of an int8 handle), TW_ERR_HIP.
 * tw_conv_gemm_i8 - the same for an int8 handle: X_dev int8, C_dev int32 (c_dtype 0) or int8
 *   requantised with `scale` (c_dtype 1) as in tw_gemm_i8, ldc >= B*L*P, multiple of 16.
 */
typedef struct { int32_t C, R, S, B, H, W, P, L; } tw_conv_geom;
typedef struct tw_conv_s* tw_conv_t; /* opaque: a geometry bound to a packed weight */
tw_status tw_conv_bind(tw_handle_t h, const tw_conv_geom* geom, int64_t ldx, tw_conv_t* out);
tw_status tw_conv_free(tw_conv_t binding);
tw_status tw_conv_gemm(const void* X_dev, tw_conv_t binding, void* C_dev, int ldc, void* stream);
tw_status tw_conv_gemm_i8(const void* X_dev, tw_conv_t binding, void* C_dev, int ldc, int c_dtype,
                          float scale, void* stream);

/* tw_export - fill *out with the logical view (host pointers owned by h). */
tw_status tw_export(tw_handle_t h, tw_packed_view* out);

/* tw_unpack - inverse of packing: writes B (.) mask (fp16 bits, pruned = +0)
 * and the mask (0/1), both K x N row-major host buffers; either may be NULL. */
tw_status tw_unpack(tw_handle_t h, uint16_t* B_masked_host, uint8_t* mask_host);

/* tw_free - release host and device memory of a handle (NULL is a no-op). */
tw_status tw_free(tw_handle_t h);

/* tw_status_str - static string for a status code. */
const char* tw_status_str(int status);

/*
 * Tuning / introspection (not needed for correct use).
 * tw_set_option: process-wide DEFAULTS of the launch options, read once at the start of every
 * call that is not given options of its own (tw_gemm, tw_dense_gemm, the int8 and convolution
 * launches, tw_launch_opts_init); meant for tests and experiments: code that launches from
 * several threads passes tw_launch_opts to tw_gemm_ex instead.  Unknown names give TW_ERR_ARG.
 *   "tile_m"   0 = heuristic, else force the M-tile (64, 128 or 256)
 *   "xcd_map"  1 (default) = remap workgroup ids so that one XCD walks all
 *              N-tiles of an M-band; 0 = plain order; 2 = as 1, and the
 *              workgroups that start together on one CU share a weight tile
 *              (measured within 2 % of mode 1 either way)
 *   "kernel"   0 = automatic, 1 = register-staged pipeline, 2 = asynchronous
 *              global->LDS copy pipeline (TW_ERR_UNSUPPORTED where it has no instance)
 *   "waves"    4 (default) or 8 waves per workgroup in the asynchronous pipeline
 *   "ksplit"   0 = automatic, 1 = never, 2 = always split K between two wave groups
 *              of a workgroup (long K, few tiles)
 *   "depth"    stages in flight of the asynchronous pipeline: 3 (default) .. 8 (6 and 8 exist for
              4-wave tiles of 64 x 128, 128 x 128 and 128 x 64 only; TVW: 3 or 4)
   "idx_route" how the asynchronous TW kernel reads a tile's kept-row list: 0 = automatic
              (through LDS where at most one and a half 4-wave workgroups per CU run, scalar loads
              otherwise), 1 = scalar loads, 2 = through LDS
   "wg_split" K split across workgroups (tw_gemm_ex with a workspace): 0 / 1 = off,
              2..8 = workgroups per (M-tile, N-tile) pair
 *   "tiles_per_wg" tiles a workgroup of the asynchronous TW kernel computes one after the other
 *              (plain TW, 4 waves, G = 128, 64- or 128-row tiles, 3 stages; ignored elsewhere): the
 *              stores of a finished tile drain while the next one loads.  0 = automatic (one:
 *              with every tile resident at once the launches are faster than with tiles in
 *              sequence), 1..8 = that many; the results do not change
 *   "tile_order"  read by tw_pack / tw_concat: 1 (default) = tiles are launched longest
 *              kept-row list first (uneven tiles, Section V "load imbalance"); 0 = in
 *              column order
 * tw_flop_counts: condensed work of a handle (any pointer may be NULL):
 *   *sum_kw  = sum over tiles of K_t * W_t (kept-row x width products),
 *   *sum_k   = sum over tiles of K_t,
 *   *k_union = number of K rows kept by at least one tile (the rows of A a
 *              launch has to read).
 */
tw_status tw_set_option(const char* name, int value);
tw_status tw_flop_counts(tw_handle_t h, int64_t* sum_kw, int64_t* sum_k, int64_t* k_union);

/*
 * tw_calibrate - measurement aid, not part of the method: enqueues ONE kernel that does
 * nothing but stream memory or issue matrix-core instructions, so that a benchmark can time
 * what this GPU sustains and price the GEMM kernels against it as well as against the
 * published peaks.  *units receives the work of the launch: bytes moved (streams) or
 * dense-equivalent floating-point / integer operations (matrix loops).
 *   TW_CAL_COPY      dst[0..bytes) = src[0..bytes), 16 bytes per thread and step; units = 2 * bytes
 *   TW_CAL_READ      reads src[0..bytes) (dst: at least 16 bytes, normally untouched)
 *   TW_CAL_WRITE     zero-fills dst[0..bytes)
 *   TW_CAL_STORE_CT  zero-fills dst as an N x 4096 fp16 array in the GEMM epilogue's pattern
 *                    (128 rows x 256 bytes per workgroup), N = bytes / 8192 rounded down to 128
 *   TW_CAL_MFMA_F16 / TW_CAL_SMFMAC_F16 / TW_CAL_MFMA_I8   2048 workgroups x 4 waves, `iters`
 *                    rounds of 4 independent 32x32x16 f16 / 32x32x32 2:4-sparse f16 /
 *                    32x32x32 int8 instructions per wave, operands in registers; dst receives
 *                    one float per thread (bytes >= 2 MiB)
 * Buffers 16-byte aligned.  Asynchronous on `stream`, allocates nothing.
 * Errors: TW_ERR_ARG, TW_ERR_HIP.
 */
enum { TW_CAL_COPY = 0, TW_CAL_READ = 1, TW_CAL_WRITE = 2, TW_CAL_STORE_CT = 3,
       TW_CAL_MFMA_F16 = 10, TW_CAL_SMFMAC_F16 = 11, TW_CAL_MFMA_I8 = 12 };
tw_status tw_calibrate(int kind, void* dst_dev, const void* src_dev, size_t bytes, int iters,
                       void* stream, double* units);

#ifdef __cplusplus
}
#endif
#endif /* TWGEMM_H */
