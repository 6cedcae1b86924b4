// C ABI of the library (see include/twgemm.h): argument checks, upload of the
// packed image, kernel selection.  No torch types, no exceptions across.
#include <hip/hip_runtime_api.h>

#include <atomic>
#include <cstring>
#include <new>
#include <vector>

#include "kernels.h"
#include "packed.h"
#include "prune.h"

namespace {

std::atomic<int> opt_tile_m{0};
std::atomic<int> opt_xcd_map{1};
std::atomic<int> opt_kernel{0};   // 0 = automatic, 1 = register-staged, 2 = asynchronous copies
std::atomic<int> opt_depth{3};
std::atomic<int> opt_waves{4};
std::atomic<int> opt_ksplit{0};   // 0 = automatic, 1 = off, 2 = two K groups per workgroup
std::atomic<int> opt_wg_split{0}; // 0 / 1 = off, 2..8 = workgroups per tile (needs a workspace)
std::atomic<int> opt_tiles_per_wg{0};  // 0 = automatic, 1..8 = tiles a workgroup computes one after the other
std::atomic<int> opt_idx_route{0};// kept-row lists: 0 = automatic, 1 = scalar loads, 2 = through LDS

// What one launch runs with: the caller's tw_launch_opts, or the process defaults above
// (tw_set_option) when there is none.  Read once per call, never shared between calls.
struct Opts {
  int tile_m, xcd_map, kernel, depth, waves, ksplit, wg_split, idx_route, tiles_per_wg;
  void* ws;
  size_t ws_bytes;
};
Opts default_opts() {
  return Opts{opt_tile_m.load(), opt_xcd_map.load(), opt_kernel.load(), opt_depth.load(), opt_waves.load(),
              opt_ksplit.load(), opt_wg_split.load(), opt_idx_route.load(), opt_tiles_per_wg.load(), nullptr, 0};
}
bool opts_from(const tw_launch_opts* in, Opts* o) {
  *o = default_opts();
  if (!in) return true;
  if (in->tile_m != 0 && in->tile_m != 64 && in->tile_m != 128 && in->tile_m != 256) return false;
  if (in->kernel < 0 || in->kernel > 2 || in->ksplit < 0 || in->ksplit > 2) return false;
  if (in->depth != 0 && (in->depth < 3 || in->depth > 8)) return false;
  if (in->waves != 0 && in->waves != 4 && in->waves != 8) return false;
  if (in->xcd_map < -1 || in->xcd_map > 2 || in->wg_split < 0 || in->wg_split > 8) return false;
  if (in->idx_route < 0 || in->idx_route > 2) return false;
  if (in->tiles_per_wg < 0 || in->tiles_per_wg > 8) return false;
  if (in->workspace_dev && ((uintptr_t)in->workspace_dev & 255)) return false;
  o->tile_m = in->tile_m; o->kernel = in->kernel; o->ksplit = in->ksplit; o->wg_split = in->wg_split;
  o->idx_route = in->idx_route;
  o->tiles_per_wg = in->tiles_per_wg;
  o->depth = in->depth ? in->depth : 3;
  o->waves = in->waves ? in->waves : 4;
  o->xcd_map = in->xcd_map < 0 ? 1 : in->xcd_map;
  o->ws = in->workspace_dev; o->ws_bytes = in->workspace_dev ? in->workspace_bytes : 0;
  return true;
}

// Workspace of the K split across workgroups: 1024 counters, then the fp32 partial tiles.
constexpr size_t WS_COUNTER_BYTES = 4096;
constexpr int WS_MAX_PAIRS = (int)(WS_COUNTER_BYTES / 4);

bool valid_G(int G) { return G == 32 || G == 64 || G == 128; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// M-tile heuristic: the largest tile that still gives every CU (256 of them)
// about two workgroups; long K loops (matrix-core bound) accept fewer, larger
// workgroups, small problems fall back to smaller tiles.  Short K loops with one
// and a half workgroups per CU still take the larger tile (128 rows; 256 for G = 64):
// they are bound by the L2 -> LDS traffic, which is (tm + G) / (tm G) per product
// (measured on the 3 x 3 convolution 256 -> 256 at 56 x 56: 17.0 against 21.7 us).
// 256-row tiles of G = 128 (8 waves) need kept-row lists of at least 384 rows: with shorter
// ones they lose 3-6 % to 128-row tiles (1024 x 4096 at M = 8192 from HBM: 23.5 against 22.2 us
// at 87.5 %), with longer ones they win 10-25 % (44.5 against 49.1 us at 50 %).  `dense`: the
// dense kernel has no gather to hide and takes 256 rows from one workgroup per CU on when
// K >= 1024 (2304 x 256 at M = 25088: 41.3 against 48.5 us), 128 rows for shorter K
// (768 x 3072 at M = 4096: 23.8 against 25.5 us).
int pick_tile_m(const Opts& o, int M, int n_tiles, int G, int max_k, bool dense = false) {
  const int forced = o.tile_m;
  if (forced == 64 || forced == 128 || forced == 256) {
    if (!(G == 32 && forced == 64)) return forced;
  }
  const int cand[3] = {256, 128, 64};
  for (int tm : cand) {
    if (G == 32 && tm == 64) break;
    long need = max_k >= 768 ? 320 : 512;
    if (need == 512 && (tm == 128 || (tm == 256 && G == 64))) need = 384;
    if (tm == 256 && G == 128 && max_k < 384) continue;
    if (tm == 256 && dense) need = max_k >= 1024 ? 192 : 512;
    // one 256-row workgroup per CU with its kept-row lists through LDS: 3-9 % ahead of two
    // 128-row ones when the lists are long (4096 x 1024 at M = 8192: 46.9 against 49.5 us at
    // 50 %, 28.7 against 29.7 at 75 %; 2304 x 256 at M = 25088: 17.5 against 19.3 us)
    if (tm == 256 && G == 128 && !dense && max_k >= 640) need = 192;
    const long wgs = (long)((M + tm - 1) / tm) * n_tiles;
    if (wgs >= need) return tm;
  }
  return G == 32 ? 128 : 64;
}

// TVW tiles are 128 rows high, two workgroups per CU (76 KB of LDS each).  64-row tiles
// (three per CU) win where 128-row tiles would leave CUs idle or end in a thin last
// round: at most one workgroup per CU, or a remainder of at most half a round of 512.
// Measured on the configured shapes: 3-13 % on the BERT-base ones, while large grids and
// long K loops (the weight tile is re-read per workgroup) keep 128.  The 256-row instance
// (8 waves) is within 3 % of the 128-row one on those; it is taken where a few N-tiles with
// long kept-row lists meet many M-tiles (at most one round of 128-row workgroups, at least
// three quarters of a round of 256-row ones): every workgroup reads its whole weight tile, and
// 256 rows share it (from HBM, 4096 x 1024 at M = 8192: 36.6 / 23.0 / 16.4 against 38.9 / 25.9 /
// 17.3 us at 75 / 87.5 / 93.75 %; 2304 x 256 at M = 25088: 15.8 against 18.6 us).
int pick_tile_m_tvw(const Opts& o, int G, int M, int n_tiles, int max_k) {
  const int forced = o.tile_m;
  if (G != 128) return 128;
  if (forced == 64 || forced == 128 || forced == 256) return forced;
  const long wgs128 = (long)((M + 127) / 128) * n_tiles;
  if (wgs128 <= 256) return 64;
  if (wgs128 <= 512 && (long)((M + 255) / 256) * n_tiles >= 192 && max_k >= 512) return 256;
  const long tail = wgs128 % 512;
  return (wgs128 <= 1536 && tail != 0 && tail <= 256) ? 64 : 128;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// K-split inside the workgroup pays when 128-row tiles cannot give every CU a
// workgroup and the K loop is long enough to amortise the final reduction.  64-row tiles
// only where 128-row tiles would leave more than half of the CUs idle: they move half as much
// again from L2 into LDS per product and read A in 128-byte pieces (3072 x 768 at M = 4096 from
// cold HBM: 15.9 us with 64-row tiles, 13.7 with 128-row tiles; 4608 x 512 at M = 1568, 52
// tiles of 128 rows: 11.1 against 14.2 us the other way).
bool use_ksplit(int M, int n_tiles, int max_k, int* tm) {
  const long wgs128 = (long)((M + 127) / 128) * n_tiles;
  if (max_k < 12 * 32 || wgs128 > 320) return false;
  *tm = wgs128 < 128 ? 64 : 128;
  return true;
}

// K split across workgroups (needs a workspace).  *tm = M-tile, *S = workgroups per pair
// (1 = do not split).  Only on request: measured on the few-tile shapes it is built for
// (3072 x 768 at M = 4096; 4608 x 512 at M = 1568) it never beat the split inside the workgroup
// (two wave groups, partial sums through LDS): 18.7 against 11.9 us and 12.6 against 10.8 us at
// best.  The partial tiles have to pass through memory that is coherent across the XCDs' L2
// caches, and that traffic (4 bytes per output element and workgroup, written and read) costs
// more than the shorter K loops save.
void pick_wg_split(const Opts& o, int M, int n_tiles, int G, int max_k, int* tm, int* S) {
  *S = 1;
  if (o.wg_split < 2) return;
  const int forced_tm = (o.tile_m == 64 || o.tile_m == 128) ? o.tile_m : 0;
  int t = forced_tm ? forced_tm : 128;
  if (G == 64) t = 128;                       // the one split instance for G = 64
  const int stages = max_k / 32;
  int s = o.wg_split;
  if (s > stages) s = stages > 0 ? stages : 1;
  (void)M; (void)n_tiles;
  *tm = t;
  *S = s;
}

}  // namespace

// A convolution geometry bound to a packed weight: the kept-row lists of the handle's device
// image turned into element offsets for that geometry.  The handle itself is not changed.
struct tw_conv_s {
  tw_handle_t h = nullptr;
  tw_conv_geom geom{};
  int64_t ldx = 0;
  int32_t* d_off = nullptr;
};

extern "C" {

const char* tw_status_str(int s) {
  switch (s) {
    case TW_OK: return "ok";
    case TW_ERR_ARG: return "invalid argument";
    case TW_ERR_MASK: return "mask is not TW/TVW conformant";
    case TW_ERR_UNSUPPORTED: return "unsupported configuration";
    case TW_ERR_ALLOC: return "allocation failed";
    case TW_ERR_HIP: return "HIP runtime error";
    case TW_ERR_STATE: return "handle not uploaded";
    case TW_ERR_TOO_LARGE: return "problem larger than the library's static scratch (use the entry point that takes a workspace)";
    default: return "unknown status";
  }
}

tw_status tw_pack_host(const uint16_t* B, const uint8_t* mask, const uint8_t* tile_mask, int K,
                       int N, int G, int pattern, tw_handle_t* out) {
  if (!out) return TW_ERR_ARG;
  *out = nullptr;
  if (!B || !mask || K < 1 || N < 1 || !valid_G(G)) return TW_ERR_ARG;
  if (pattern != TW_PATTERN_TW && pattern != TW_PATTERN_TVW && pattern != TW_PATTERN_TEW) return TW_ERR_ARG;
  if (pattern == TW_PATTERN_TEW && !tile_mask) return TW_ERR_ARG;
  if (pattern == TW_PATTERN_TEW && K > 65536) return TW_ERR_UNSUPPORTED;   // restored rows travel as 16 bits
  tw_handle_s* h = new (std::nothrow) tw_handle_s();
  if (!h) return TW_ERR_ALLOC;
  tw_status st = twg::pack_host(B, mask, tile_mask, K, N, G, pattern, h);
  if (st != TW_OK) { delete h; return st; }
  *out = h;
  return TW_OK;
}

tw_status tw_upload(tw_handle_t h) {
  if (!h) return TW_ERR_ARG;
  twg::DeviceImage& d = h->img;
  if (d.blob) return TW_OK;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return TW_ERR_HIP;
  // one allocation, 256-byte aligned parts
  // (value parts are sized by n_vals / n_meta: a device-packed weight has no host copy of them)
  struct Part { const void* src; size_t bytes; size_t off; bool copy; };
  const bool i8 = h->dtype == TW_DTYPE_I8;
  const bool have_vals = i8 ? !d.vals8.empty() : !d.vals.empty();
  Part parts[10] = {
      {d.col_idx.data(), d.col_idx.size() * 4, 0, true},   {d.tile_kp_off.data(), d.tile_kp_off.size() * 4, 0, true},
      {d.row_idx.data(), d.row_idx.size() * 4, 0, true},   {d.zero_cols.data(), d.zero_cols.size() * 4, 0, true},
      {d.tile_order.data(), d.tile_order.size() * 4, 0, true},
      i8 ? Part{d.vals8.data(), d.n_vals, 0, have_vals} : Part{d.vals.data(), d.n_vals * 2, 0, have_vals},
      {d.meta.data(), d.n_meta * 4, 0, !d.meta.empty()}, {d.tile_sched.data(), d.tile_sched.size() * 4, 0, true},
      {d.ew_ptr.data(), d.ew_ptr.size() * 4, 0, true}, {d.ew_pairs.data(), d.ew_pairs.size() * 4, 0, true}};
  size_t total = 0;
  for (auto& p : parts) { p.off = total; total += align_up(p.bytes ? p.bytes : 1, 256); }
  void* blob = nullptr;
  if (hipMalloc(&blob, total) != hipSuccess) { (void)hipGetLastError(); return TW_ERR_ALLOC; }
  for (auto& p : parts) {
    if (!p.bytes || !p.copy) continue;
    if (hipMemcpy((char*)blob + p.off, p.src, p.bytes, hipMemcpyHostToDevice) != hipSuccess) {
      (void)hipFree(blob);
      return TW_ERR_HIP;
    }
  }
  char* b = (char*)blob;
  d.d_col_idx = (const int32_t*)(b + parts[0].off);
  d.d_tile_kp_off = (const int32_t*)(b + parts[1].off);
  d.d_row_idx = (const int32_t*)(b + parts[2].off);
  d.d_zero_cols = (const int32_t*)(b + parts[3].off);
  d.d_tile_order = (const int32_t*)(b + parts[4].off);
  d.d_vals = (const uint16_t*)(b + parts[5].off);
  d.d_meta = (const uint32_t*)(b + parts[6].off);
  d.d_tile_sched = (const int32_t*)(b + parts[7].off);
  d.d_ew_ptr = (const int32_t*)(b + parts[8].off);
  d.d_ew_pairs = (const uint32_t*)(b + parts[9].off);
  d.blob = blob; d.blob_bytes = total; d.device = dev;
  return TW_OK;
}

tw_status tw_pack(const uint16_t* B, const uint8_t* mask, const uint8_t* tile_mask, int K, int N,
                  int G, int pattern, tw_handle_t* out) {
  tw_status st = tw_pack_host(B, mask, tile_mask, K, N, G, pattern, out);
  if (st != TW_OK) return st;
  st = tw_upload(*out);
  if (st != TW_OK) { tw_free(*out); *out = nullptr; }
  return st;
}

tw_status tw_pack_i8_host(const int8_t* B, const uint8_t* mask, const uint8_t* tile_mask, int K, int N,
                          int G, int pattern, tw_handle_t* out) {
  if (!out) return TW_ERR_ARG;
  *out = nullptr;
  if (!B || !mask || K < 1 || N < 1 || !valid_G(G)) return TW_ERR_ARG;
  if (pattern == TW_PATTERN_TEW) return TW_ERR_UNSUPPORTED;
  if (pattern != TW_PATTERN_TW && pattern != TW_PATTERN_TVW) return TW_ERR_ARG;
  tw_handle_s* h = new (std::nothrow) tw_handle_s();
  if (!h) return TW_ERR_ALLOC;
  tw_status st;
  try {
    // the packer moves 16-bit patterns around without looking at them: int8 values
    // ride through it sign-extended
    std::vector<uint16_t> wide((size_t)K * N);
    for (size_t i = 0; i < wide.size(); ++i) wide[i] = (uint16_t)(int16_t)B[i];
    h->dtype = TW_DTYPE_I8;
    st = twg::pack_host(wide.data(), mask, tile_mask, K, N, G, pattern, h);
  } catch (const std::bad_alloc&) {
    st = TW_ERR_ALLOC;
  }
  if (st != TW_OK) { delete h; return st; }
  *out = h;
  return TW_OK;
}

tw_status tw_pack_i8(const int8_t* B, const uint8_t* mask, const uint8_t* tile_mask, int K, int N, int G,
                     int pattern, tw_handle_t* out) {
  tw_status st = tw_pack_i8_host(B, mask, tile_mask, K, N, G, pattern, out);
  if (st != TW_OK) return st;
  st = tw_upload(*out);
  if (st != TW_OK) { tw_free(*out); *out = nullptr; }
  return st;
}

tw_status tw_prune_workspace_bytes(int K, int N, int G, size_t* bytes) {
  if (!bytes || K < 1 || N < 1 || !valid_G(G)) return TW_ERR_ARG;
  *bytes = twg::prune_workspace_bytes(K, N, G);
  return TW_OK;
}

tw_status tw_prune_dev(const void* B_dev, int K, int N, int ldb, int G, int pattern, int n_cols_pruned,
                       int rows_per_tile, uint8_t* mask_dev, uint8_t* tile_mask_dev, void* workspace_dev,
                       size_t workspace_bytes, void* stream) {
  if (!B_dev || !mask_dev || !workspace_dev || K < 1 || N < 1 || ldb < N || !valid_G(G)) return TW_ERR_ARG;
  if (n_cols_pruned < 0 || n_cols_pruned > N || rows_per_tile < 0 || rows_per_tile > K) return TW_ERR_ARG;
  if (pattern == TW_PATTERN_TEW) return TW_ERR_UNSUPPORTED;
  if (pattern != TW_PATTERN_TW && pattern != TW_PATTERN_TVW) return TW_ERR_ARG;
  if (((uintptr_t)workspace_dev & 15) || workspace_bytes < twg::prune_workspace_bytes(K, N, G)) return TW_ERR_ARG;
  if (((size_t)K * N + 255) / 256 > 0x7fffffffu) return TW_ERR_UNSUPPORTED;   // one thread per element, grid limit
  if ((N + G - 1) / G > 65535 || (K + 255) / 256 > 65535 || (N + 255) / 256 > 65535) return TW_ERR_UNSUPPORTED;
  hipError_t e = twg::prune_device((const uint16_t*)B_dev, K, N, ldb, G, pattern == TW_PATTERN_TVW, n_cols_pruned,
                                   rows_per_tile, mask_dev, tile_mask_dev, workspace_dev, (hipStream_t)stream);
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

tw_status tw_prune_dev_static(const void* B_dev, int K, int N, int ldb, int G, int pattern, int n_cols_pruned,
                              int rows_per_tile, uint8_t* mask_dev, uint8_t* tile_mask_dev, void* stream) {
  if (!B_dev || !mask_dev || K < 1 || N < 1 || ldb < N || !valid_G(G)) return TW_ERR_ARG;
  if (n_cols_pruned < 0 || n_cols_pruned > N || rows_per_tile < 0 || rows_per_tile > K) return TW_ERR_ARG;
  if (pattern == TW_PATTERN_TEW) return TW_ERR_UNSUPPORTED;
  if (pattern != TW_PATTERN_TW && pattern != TW_PATTERN_TVW) return TW_ERR_ARG;
  if (twg::prune_workspace_bytes(K, N, G) > twg::PRUNE_STATIC_SCRATCH_BYTES) return TW_ERR_TOO_LARGE;
  if (((size_t)K * N + 255) / 256 > 0x7fffffffu) return TW_ERR_TOO_LARGE;
  if ((N + G - 1) / G > 65535 || (K + 255) / 256 > 65535 || (N + 255) / 256 > 65535) return TW_ERR_TOO_LARGE;
  void* ws = nullptr;
  if (twg::prune_static_scratch(&ws) != hipSuccess) { (void)hipGetLastError(); return TW_ERR_HIP; }
  hipError_t e = twg::prune_device((const uint16_t*)B_dev, K, N, ldb, G, pattern == TW_PATTERN_TVW, n_cols_pruned,
                                   rows_per_tile, mask_dev, tile_mask_dev, ws, (hipStream_t)stream);
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

tw_status tw_pack_dev(const void* B_dev, int ldb, const uint8_t* mask_dev, const uint8_t* tile_mask_dev, int K,
                      int N, int G, int pattern, void* stream, tw_handle_t* out) try {
  if (!out) return TW_ERR_ARG;
  *out = nullptr;
  if (!B_dev || !mask_dev || K < 1 || N < 1 || ldb < N || !valid_G(G)) return TW_ERR_ARG;
  if (pattern != TW_PATTERN_TW && pattern != TW_PATTERN_TVW && pattern != TW_PATTERN_TEW) return TW_ERR_ARG;
  hipStream_t s = (hipStream_t)stream;
  if (pattern != TW_PATTERN_TEW) {       // packed by kernels: only the index lists visit the host
    tw_handle_s* h = new (std::nothrow) tw_handle_s();
    if (!h) return TW_ERR_ALLOC;
    const tw_status st = twg::pack_device((const uint16_t*)B_dev, ldb, mask_dev, tile_mask_dev, K, N, G, pattern, s, h);
    if (st != TW_OK) { tw_free(h); return st; }
    *out = h;
    return TW_OK;
  }
  // TEW: through the host packer
  if (!tile_mask_dev) return TW_ERR_ARG;
  std::vector<uint16_t> B((size_t)K * N);
  std::vector<uint8_t> mask((size_t)K * N), tmask((size_t)K * N);
  if (hipMemcpy2DAsync(B.data(), (size_t)N * 2, B_dev, (size_t)ldb * 2, (size_t)N * 2, K, hipMemcpyDeviceToHost, s) !=
          hipSuccess ||
      hipMemcpyAsync(mask.data(), mask_dev, mask.size(), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipMemcpyAsync(tmask.data(), tile_mask_dev, tmask.size(), hipMemcpyDeviceToHost, s) != hipSuccess ||
      hipStreamSynchronize(s) != hipSuccess) {
    (void)hipGetLastError();
    return TW_ERR_HIP;
  }
  return tw_pack(B.data(), mask.data(), tmask.data(), K, N, G, pattern, out);
} catch (const std::bad_alloc&) {
  return TW_ERR_ALLOC;
}

tw_status tw_concat(const tw_handle_t* parts, int n, int upload, tw_handle_t* out) {
  if (!out) return TW_ERR_ARG;
  *out = nullptr;
  if (!parts || n < 1) return TW_ERR_ARG;
  for (int i = 0; i < n; ++i) {
    if (!parts[i]) return TW_ERR_ARG;
    const tw_status sf = twg::fetch_logical_values(parts[i]);   // a device-packed member
    if (sf != TW_OK) return sf;
  }
  tw_handle_s* h = new (std::nothrow) tw_handle_s();
  if (!h) return TW_ERR_ALLOC;
  tw_status st = twg::concat_host(parts, n, h);
  if (st == TW_OK && upload) st = tw_upload(h);
  if (st != TW_OK) { tw_free(h); return st; }
  *out = h;
  return TW_OK;
}

// The launch behind tw_gemm and tw_conv_gemm.  conv: A is the wide input, the row list holds
// window offsets (lda = 1) and M counts the wide grid.
static tw_status gemm_launch(const Opts& o, const void* A, int M, int lda, int layout, tw_handle_t h, void* C,
                             int ldc, void* stream, const tw_conv_s* conv) {
  twg::GemmArgs g{};
  g.A = (const _Float16*)A; g.C = (_Float16*)C; g.M = M; g.lda = lda; g.ldc = ldc;
  g.vals = (const _Float16*)h->img.d_vals;
  g.row_idx = h->img.d_row_idx; g.tile_kp_off = h->img.d_tile_kp_off;
  if (conv) {
    g.row_idx = conv->d_off;
    g.conv_P = conv->geom.P; g.conv_L = conv->geom.L; g.conv_H = conv->geom.H; g.conv_W = conv->geom.W;
  }
  g.col_idx = h->img.d_col_idx; g.tile_order = h->img.d_tile_order;
  g.tile_sched = h->img.d_tile_sched; g.uniform_kp = h->img.uniform_kp;
  g.zero_cols = h->img.d_zero_cols; g.n_zero = (int)h->img.zero_cols.size();
  g.meta = h->img.d_meta;
  g.ew_ptr = h->img.d_ew_ptr; g.ew_pairs = h->img.d_ew_pairs;
  g.ew_last = h->img.ew_pairs.empty() ? 0 : (int)h->img.ew_pairs.size() - 1;
  g.n_tiles = h->n_tiles; g.K = h->K; g.N = h->N; g.xcd_map = o.xcd_map;
  g.wg_split = 1;
  g.tiles_per_wg = 1;
  if (layout == TW_LAYOUT_MK) {
    hipError_t e = twg::launch_tw_mk(h->G, g, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
    return e == hipSuccess ? TW_OK : TW_ERR_HIP;
  }
  if (h->pattern == TW_PATTERN_TVW) {
    const int tvw_tm = pick_tile_m_tvw(o, h->G, M, h->n_tiles > 0 ? h->n_tiles : 1, h->max_kp);
    hipError_t e = twg::launch_tvw_km(h->G, tvw_tm, o.depth > 4 ? 4 : o.depth, g, (hipStream_t)stream);
    if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
    return e == hipSuccess ? TW_OK : TW_ERR_HIP;
  }
  int tm = pick_tile_m(o, M, h->n_tiles > 0 ? h->n_tiles : 1, h->G, h->max_kp);
  // no 64 x 64 instance of the asynchronous kernel (tried: one matrix instruction per wave and
  // k-step is too little work per barrier; plain TW falls back to the register-staged kernel)
  if ((h->pattern == TW_PATTERN_TEW || conv) && h->G == 64 && tm == 64) tm = 128;
  hipError_t e = hipErrorInvalidValue;
  // TEW: the same kernels with the restored elements added in the epilogue (3 stages only)
  const bool tew = h->pattern == TW_PATTERN_TEW;
  auto launch_dma = tew ? twg::launch_tew_km_dma : twg::launch_tw_km_dma;
  const int depth = tew ? 3 : o.depth;
  // the asynchronous kernel addresses A with 32-bit byte offsets
  const bool a_fits32 = conv || (unsigned long long)h->K * (unsigned long long)lda * 2ull < (1ull << 32);
  // K split across workgroups: few tiles, long kept-row lists, and a workspace to reduce through
  if (!tew && o.kernel != 1 && h->G != 32 && a_fits32 && o.ws && o.wg_split != 1 && h->n_tiles > 0) {
    int stm = 0, S = 0;
    pick_wg_split(o, M, h->n_tiles, h->G, h->max_kp, &stm, &S);
    if (S > 1) {
      const long pairs = (long)((M + stm - 1) / stm) * h->n_tiles;
      const size_t need = WS_COUNTER_BYTES + (size_t)pairs * S * stm * h->G * 4;
      if (pairs <= WS_MAX_PAIRS && need <= o.ws_bytes) {
        g.wg_split = S;
        g.ws_counters = (int*)o.ws;
        g.ws_partials = (float*)((char*)o.ws + WS_COUNTER_BYTES);
        hipError_t es = twg::launch_tw_km_dma_split(h->G, stm, g, (hipStream_t)stream);
        if (es != hipErrorInvalidValue) return es == hipSuccess ? TW_OK : TW_ERR_HIP;
        g.wg_split = 1;
      } else if (o.wg_split > 1) {
        return TW_ERR_ARG;          // a split was asked for and the workspace cannot hold it
      }
    }
  }
  if ((o.kernel != 1 || tew || conv) && h->G != 32 && a_fits32) {
    // long K with too few tiles to fill the chip: split K inside the workgroup
    // 256-row tiles run with 8 waves (64 x 64 per wave): half the registers per wave, two
    // workgroups per CU
    int variant = (o.waves == 8 || (tm == 256 && h->G == 128)) ? twg::DMA_WAVES8 : twg::DMA_WAVES4;
    int tmk = tm;
    const int ks = o.ksplit;
    if (ks == 2 || (ks == 0 && use_ksplit(M, h->n_tiles, h->max_kp, &tmk))) variant = twg::DMA_KSPLIT2;
    if (variant == twg::DMA_KSPLIT2 && ks == 2) tmk = tm == 256 ? 128 : tm;
    if (variant == twg::DMA_KSPLIT2 && h->G == 64) tmk = 128;   // the one K-split instance for G = 64
    // kept-row lists through LDS where at most one and a half 4-wave workgroups per CU run
    // (nothing else there hides the scalar loads' round trip: -6...-22 %) or one 8-wave
    // workgroup; by scalar loads for fuller CUs (two workgroups per CU: 3-7 % ahead of the LDS route, unless
    // the lists are long: 4096 x 1024 at M = 8192 and 50 %, 46.3 with LDS against 50.0 us)
    const int tmu = variant == twg::DMA_KSPLIT2 ? tmk : tm;
    auto lidx_for = [&](int v, int t) {
      if (o.idx_route) return o.idx_route == 2;
      const long wgs = (long)((M + t - 1) / t) * h->n_tiles;
      if (v == twg::DMA_WAVES8) return wgs <= 256;       // alone on its CU: nothing else hides the round trip
      return wgs <= 384 || (wgs <= 512 && h->max_kp >= 2048);
    };
    // several tiles per workgroup (plain TW, 4 waves, 64- or 128-row tiles of G = 128, 3 stages): on request
    if (!tew && variant == twg::DMA_WAVES4 && o.tiles_per_wg > 1) g.tiles_per_wg = o.tiles_per_wg;
    e = launch_dma(h->G, tmu, depth, variant, lidx_for(variant, tmu), g, (hipStream_t)stream);
    if (e == hipErrorInvalidValue && variant != twg::DMA_WAVES4)
      e = launch_dma(h->G, tm, depth, twg::DMA_WAVES4, lidx_for(twg::DMA_WAVES4, tm), g, (hipStream_t)stream);
  }
  if (e == hipErrorInvalidValue && o.kernel != 2 && !tew && !conv)
    e = twg::launch_tw_km(h->G, tm, g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

tw_status tw_launch_opts_init(tw_launch_opts* opts) {
  if (!opts) return TW_ERR_ARG;
  const Opts d = default_opts();
  opts->tile_m = d.tile_m; opts->kernel = d.kernel; opts->depth = d.depth; opts->waves = d.waves;
  opts->ksplit = d.ksplit; opts->xcd_map = d.xcd_map; opts->wg_split = d.wg_split; opts->idx_route = d.idx_route; opts->tiles_per_wg = d.tiles_per_wg;
  opts->workspace_dev = nullptr; opts->workspace_bytes = 0;
  return TW_OK;
}

tw_status tw_gemm_workspace_bytes(tw_handle_t h, int M, size_t* bytes) {
  if (!h || !bytes || M < 1) return TW_ERR_ARG;
  // enough for any split the library may choose at this M: 64-row tiles, 8 workgroups per pair,
  // as long as the pairs fit the counters (beyond that no split is used)
  const long pairs64 = (long)((M + 63) / 64) * (h->n_tiles > 0 ? h->n_tiles : 1);
  const long pairs = pairs64 < WS_MAX_PAIRS ? pairs64 : WS_MAX_PAIRS;
  *bytes = WS_COUNTER_BYTES + (size_t)pairs * 8 * 64 * 128 * 4;
  return TW_OK;
}

tw_status tw_workspace_init(void* workspace_dev, size_t workspace_bytes, void* stream) {
  if (!workspace_dev || ((uintptr_t)workspace_dev & 255) || workspace_bytes < WS_COUNTER_BYTES) return TW_ERR_ARG;
  return twg::launch_zero_words((uint32_t*)workspace_dev, WS_COUNTER_BYTES / 4, (hipStream_t)stream) == hipSuccess
             ? TW_OK : TW_ERR_HIP;
}

tw_status tw_gemm_ex(const void* A, int M, int lda, int layout, tw_handle_t h, void* C, int ldc,
                     const tw_launch_opts* opts, void* stream) {
  if (!A || !C || !h || M < 1) return TW_ERR_ARG;
  if (layout != TW_LAYOUT_KM && layout != TW_LAYOUT_MK) return TW_ERR_ARG;
  if (!aligned16(A) || !aligned16(C) || lda % 8 || ldc % 8) return TW_ERR_ARG;
  if (h->dtype != TW_DTYPE_F16) return TW_ERR_ARG;
  if (!h->img.blob) return TW_ERR_STATE;
  if (layout == TW_LAYOUT_MK) {
    if (lda < h->K || ldc < h->N) return TW_ERR_ARG;
    if (h->pattern != TW_PATTERN_TW) return TW_ERR_UNSUPPORTED;   // TVW and TEW exist for K x M only
  } else if (lda < M || ldc < M) {
    return TW_ERR_ARG;
  }
  Opts o;
  if (!opts_from(opts, &o)) return TW_ERR_ARG;
  return gemm_launch(o, A, M, lda, layout, h, C, ldc, stream, nullptr);
}

tw_status tw_gemm(const void* A, int M, int lda, int layout, tw_handle_t h, void* C, int ldc,
                  void* stream) {
  return tw_gemm_ex(A, M, lda, layout, h, C, ldc, nullptr, stream);
}

tw_status tw_conv_bind(tw_handle_t h, const tw_conv_geom* cg, int64_t ldx, tw_conv_t* out) {
  if (!out) return TW_ERR_ARG;
  *out = nullptr;
  if (!h || !cg) return TW_ERR_ARG;
  if (cg->C < 1 || cg->R < 1 || cg->S < 1 || cg->B < 1 || cg->H < 1 || cg->W < 1) return TW_ERR_ARG;
  if (cg->P < cg->W + cg->S - 1 || cg->L < cg->H + cg->R - 1) return TW_ERR_ARG;
  if ((int64_t)cg->C * cg->R * cg->S != h->K) return TW_ERR_ARG;
  const int64_t Mp = (int64_t)cg->B * cg->L * cg->P;
  if (Mp > INT32_MAX - 8) return TW_ERR_ARG;
  const int chunk = h->dtype == TW_DTYPE_I8 ? 16 : 8;          // elements per 16-byte copy
  const int64_t reach = (Mp + chunk - 1) / chunk * chunk + (int64_t)(cg->R - 1) * cg->P + cg->S - 1;
  if (ldx < reach || ldx % chunk || (int64_t)cg->C * ldx >= (1ll << 31)) return TW_ERR_ARG;
  if (h->pattern == TW_PATTERN_TEW || h->G == 32) return TW_ERR_UNSUPPORTED;
  if (!h->img.blob) return TW_ERR_STATE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return TW_ERR_HIP;
  if (dev != h->img.device) return TW_ERR_STATE;
  std::vector<int32_t> off;
  tw_conv_s* b = new (std::nothrow) tw_conv_s();
  if (!b) return TW_ERR_ALLOC;
  try {
    off.resize(h->img.row_idx.size());
  } catch (const std::bad_alloc&) {
    delete b;
    return TW_ERR_ALLOC;
  }
  const int RS = cg->R * cg->S;
  for (size_t i = 0; i < off.size(); ++i) {
    const int k = h->img.row_idx[i], c = k / RS, r = (k % RS) / cg->S, s = k % cg->S;
    off[i] = (int32_t)((int64_t)c * ldx + (int64_t)r * cg->P + s);
  }
  int32_t* d = nullptr;
  if (hipMalloc((void**)&d, off.size() * 4 + 4) != hipSuccess) { (void)hipGetLastError(); delete b; return TW_ERR_ALLOC; }
  if (hipMemcpy(d, off.data(), off.size() * 4, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(d);
    delete b;
    return TW_ERR_HIP;
  }
  b->h = h; b->geom = *cg; b->ldx = ldx; b->d_off = d;
  *out = b;
  return TW_OK;
}

tw_status tw_conv_free(tw_conv_t b) {
  if (!b) return TW_OK;
  const tw_status st = (b->d_off && hipFree(b->d_off) != hipSuccess) ? TW_ERR_HIP : TW_OK;
  delete b;
  return st;
}

tw_status tw_conv_gemm(const void* X, tw_conv_t b, void* C, int ldc, void* stream) {
  if (!X || !C || !b || !b->h) return TW_ERR_ARG;
  if (b->h->dtype != TW_DTYPE_F16) return TW_ERR_ARG;
  const int Mp = b->geom.B * b->geom.L * b->geom.P;
  if (!aligned16(X) || !aligned16(C) || ldc % 8 || ldc < Mp) return TW_ERR_ARG;
  return gemm_launch(default_opts(), X, Mp, 1, TW_LAYOUT_KM, b->h, C, ldc, stream, b);
}

tw_status tw_dense_gemm(const void* A, const void* B, void* C, int M, int K, int N, int lda,
                        int ldb, int ldc, int layout, void* stream) {
  if (!A || !B || !C || M < 1 || K < 1 || N < 1) return TW_ERR_ARG;
  if (layout != TW_LAYOUT_KM && layout != TW_LAYOUT_MK) return TW_ERR_ARG;
  if (!aligned16(A) || !aligned16(B) || !aligned16(C) || lda % 8 || ldb % 8 || ldc % 8)
    return TW_ERR_ARG;
  if (ldb < N) return TW_ERR_ARG;
  if (layout == TW_LAYOUT_MK) {
    if (lda < K || ldc < N) return TW_ERR_ARG;
  } else if (lda < M || ldc < M) {
    return TW_ERR_ARG;
  }
  twg::GemmArgs g{};
  g.A = (const _Float16*)A; g.C = (_Float16*)C; g.M = M; g.lda = lda; g.ldc = ldc;
  g.vals = (const _Float16*)B; g.ldb = ldb; g.K = K; g.N = N;
  const int tn = 128;
  g.n_tiles = (N + tn - 1) / tn;
  const Opts o = default_opts();
  g.xcd_map = o.xcd_map;
  g.wg_split = 1;
  if (layout == TW_LAYOUT_MK) {
    hipError_t em = twg::launch_dense_mk(tn, g, (hipStream_t)stream);
    return em == hipSuccess ? TW_OK : TW_ERR_HIP;
  }
  const int tm = pick_tile_m(o, M, g.n_tiles, tn, K, true);
  hipError_t e = hipErrorInvalidValue;
  const bool fits32 = (unsigned long long)K * (unsigned long long)lda * 2ull < (1ull << 32) &&
                      (unsigned long long)K * (unsigned long long)ldb * 2ull < (1ull << 32);
  if (o.kernel != 1 && K % 32 == 0 && fits32) {
    int variant = (o.waves == 8 || tm == 256) ? twg::DMA_WAVES8 : twg::DMA_WAVES4;
    int tmk = tm;
    const int ks = o.ksplit;
    if (K % 64 == 0 && (ks == 2 || (ks == 0 && use_ksplit(M, g.n_tiles, K, &tmk)))) variant = twg::DMA_KSPLIT2;
    if (variant == twg::DMA_KSPLIT2 && ks == 2) tmk = tm == 256 ? 128 : tm;
    e = twg::launch_dense_km_dma(tn, variant == twg::DMA_KSPLIT2 ? tmk : tm, o.depth, variant, g,
                                 (hipStream_t)stream);
    if (e == hipErrorInvalidValue && variant != twg::DMA_WAVES4)
      e = twg::launch_dense_km_dma(tn, tm, o.depth, twg::DMA_WAVES4, g, (hipStream_t)stream);
  }
  if (e == hipErrorInvalidValue && o.kernel != 2)
    e = twg::launch_dense_km(tn, tm, g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

// int8 M-tile: 256 rows while that still gives every CU two workgroups, else 128.  The 64-row
// instance (G = 128) is only used on request: it measured no better than 128 rows on the small
// BERT-base launches and worse on the dense baseline.  As for fp16, 256 rows need kept-row lists of
// at least 384 rows (1024 x 4096 at M = 8192 and 87.5 %, from HBM: 17.5 against 16.3 us).
static int pick_tile_m_i8(const Opts& o, int M, int n_tiles, int G, int max_k) {
  const int forced = o.tile_m;
  if (forced == 128 || forced == 256 || (forced == 64 && G == 128)) return forced;
  return (max_k >= 384 && (long)((M + 255) / 256) * n_tiles >= 512) ? 256 : 128;
}

// The launch behind tw_gemm_i8 and tw_conv_gemm_i8 (conv: see gemm_launch).
static tw_status gemm_i8_launch(const void* A, int M, int lda, tw_handle_t h, void* C, int ldc, int c_dtype,
                                float scale, void* stream, const tw_conv_s* conv) {
  const Opts o = default_opts();
  twg::GemmI8Args g{};
  g.A = (const int8_t*)A; g.C = C; g.M = M; g.lda = lda; g.ldc = ldc;
  g.c_i8 = c_dtype; g.scale = scale;
  g.vals = (const int8_t*)h->img.d_vals;
  g.row_idx = h->img.d_row_idx; g.col_idx = h->img.d_col_idx; g.tile_sched = h->img.d_tile_sched;
  g.uniform_kp = h->img.uniform_kp;
  if (conv) {
    g.row_idx = conv->d_off;
    g.conv_P = conv->geom.P; g.conv_L = conv->geom.L; g.conv_H = conv->geom.H; g.conv_W = conv->geom.W;
  }
  g.zero_cols = h->img.d_zero_cols; g.n_zero = (int)h->img.zero_cols.size();
  g.n_tiles = h->n_tiles; g.K = h->K; g.N = h->N; g.xcd_map = o.xcd_map ? 1 : 0;
  g.meta = h->img.d_meta;
  hipError_t e;
  if (h->pattern == TW_PATTERN_TVW) {
    // 64-row tiles where 128-row tiles would not give every CU a workgroup
    const int forced = o.tile_m;
    const long wgs128 = (long)((M + 127) / 128) * (h->n_tiles > 0 ? h->n_tiles : 1);
    const int tm = h->G != 128 ? 128 : (forced == 64 || forced == 128) ? forced : (wgs128 <= 256 ? 64 : 128);
    e = twg::launch_tvw_i8(h->G, tm, g, (hipStream_t)stream);
  } else {
    // long K with too few tiles to fill the chip: split K inside the workgroup (as the fp16 path)
    const int tm = pick_tile_m_i8(o, M, h->n_tiles > 0 ? h->n_tiles : 1, h->G, h->max_kp);
    const int ks = o.ksplit;
    int tmk = tm;
    e = hipErrorInvalidValue;
    // (from 12 stages of 64 rows on: below that the reduction through LDS costs more than it saves)
    if (ks == 2 || (ks == 0 && h->max_kp >= 768 && use_ksplit(M, h->n_tiles, h->max_kp, &tmk))) {
      if (ks == 2) tmk = tm == 256 ? 128 : tm;
      if (h->G == 64) tmk = 128;
      e = twg::launch_tw_i8(h->G, tmk, 2, g, (hipStream_t)stream);
    }
    if (e == hipErrorInvalidValue) e = twg::launch_tw_i8(h->G, tm, 1, g, (hipStream_t)stream);
  }
  if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

tw_status tw_gemm_i8(const void* A, int M, int lda, tw_handle_t h, void* C, int ldc, int c_dtype,
                     float scale, void* stream) {
  if (!A || !C || !h || M < 1 || (c_dtype != 0 && c_dtype != 1)) return TW_ERR_ARG;
  if (!aligned16(A) || !aligned16(C) || lda % 16 || ldc % 16 || lda < M || ldc < M) return TW_ERR_ARG;
  if (h->dtype != TW_DTYPE_I8) return TW_ERR_ARG;
  if (!h->img.blob) return TW_ERR_STATE;
  if (h->G == 32 || h->K > 131071) return TW_ERR_UNSUPPORTED;
  if ((unsigned long long)h->K * (unsigned long long)lda >= (1ull << 32)) return TW_ERR_UNSUPPORTED;
  return gemm_i8_launch(A, M, lda, h, C, ldc, c_dtype, scale, stream, nullptr);
}

tw_status tw_conv_gemm_i8(const void* X, tw_conv_t b, void* C, int ldc, int c_dtype, float scale,
                          void* stream) {
  if (!X || !C || !b || !b->h || (c_dtype != 0 && c_dtype != 1)) return TW_ERR_ARG;
  if (b->h->dtype != TW_DTYPE_I8) return TW_ERR_ARG;
  const int Mp = b->geom.B * b->geom.L * b->geom.P;
  if (!aligned16(X) || !aligned16(C) || ldc % 16 || ldc < Mp) return TW_ERR_ARG;
  if (b->h->K > 131071) return TW_ERR_UNSUPPORTED;
  return gemm_i8_launch(X, Mp, 1, b->h, C, ldc, c_dtype, scale, stream, b);
}

tw_status tw_dense_gemm_i8(const void* A, const void* B, void* C, int M, int K, int N, int lda, int ldb,
                           int ldc, int c_dtype, float scale, void* stream) {
  if (!A || !B || !C || M < 1 || K < 1 || N < 1 || (c_dtype != 0 && c_dtype != 1)) return TW_ERR_ARG;
  if (!aligned16(A) || !aligned16(B) || !aligned16(C) || lda % 16 || ldb % 16 || ldc % 16) return TW_ERR_ARG;
  if (ldb < N || lda < M || ldc < M) return TW_ERR_ARG;
  if (K % 64 || K > 131071) return TW_ERR_UNSUPPORTED;
  if ((unsigned long long)K * (unsigned long long)lda >= (1ull << 32) ||
      (unsigned long long)K * (unsigned long long)ldb >= (1ull << 32))
    return TW_ERR_UNSUPPORTED;
  twg::GemmI8Args g{};
  g.A = (const int8_t*)A; g.C = C; g.M = M; g.lda = lda; g.ldc = ldc;
  g.c_i8 = c_dtype; g.scale = scale;
  g.vals = (const int8_t*)B; g.ldb = ldb; g.K = K; g.N = N;
  const int tn = 128;
  g.n_tiles = (N + tn - 1) / tn;
  const Opts o = default_opts();
  g.xcd_map = o.xcd_map ? 1 : 0;
  hipError_t e = twg::launch_dense_i8(tn, pick_tile_m_i8(o, M, g.n_tiles, tn, K), g, (hipStream_t)stream);
  if (e == hipErrorInvalidValue) return TW_ERR_UNSUPPORTED;
  return e == hipSuccess ? TW_OK : TW_ERR_HIP;
}

tw_status tw_export(tw_handle_t h, tw_packed_view* out) {
  if (!h || !out) return TW_ERR_ARG;
  std::memset(out, 0, sizeof(*out));
  const tw_status sf = twg::fetch_logical_values(h);   // device-packed: the values come over now
  if (sf != TW_OK) return sf;
  out->K = h->K; out->N = h->N; out->G = h->G; out->pattern = h->pattern;
  out->n_kept = h->n_kept; out->n_tiles = h->n_tiles; out->dtype = h->dtype;
  out->col_idx = h->col_idx.data(); out->cto_n = h->cto_n.data();
  out->tile_k_off = h->tile_k_off.data(); out->row_idx = h->row_idx.data();
  out->cto_k = h->cto_k.data(); out->val_off = h->val_off.data(); out->values = h->values.data();
  out->tile_col_off = h->tile_col_off.data();
  if (h->pattern == TW_PATTERN_TEW) {
    out->ew_nnz = (int64_t)h->ew_row.size();
    out->ew_col_ptr = h->ew_col_ptr.data(); out->ew_row = h->ew_row.data(); out->ew_val = h->ew_val.data();
  }
  if (h->pattern == TW_PATTERN_TVW) {
    out->meta_off = h->meta_off.data(); out->meta = h->meta.data(); out->valid = h->valid.data();
  }
  return TW_OK;
}

tw_status tw_unpack(tw_handle_t h, uint16_t* Bm, uint8_t* mask) {
  if (!h) return TW_ERR_ARG;
  const tw_status sf = twg::fetch_logical_values(h);
  if (sf != TW_OK) return sf;
  return twg::unpack_host(h, Bm, mask);
}

tw_status tw_free(tw_handle_t h) {
  if (!h) return TW_OK;
  tw_status st = TW_OK;
  if (h->img.blob && hipFree(h->img.blob) != hipSuccess) st = TW_ERR_HIP;
  if (h->dev_logical && hipFree(h->dev_logical) != hipSuccess) st = TW_ERR_HIP;
  delete h;
  return st;
}

tw_status tw_set_option(const char* name, int value) {
  if (!name) return TW_ERR_ARG;
  if (!std::strcmp(name, "tile_m")) { opt_tile_m.store(value); return TW_OK; }
  if (!std::strcmp(name, "xcd_map")) { opt_xcd_map.store(value < 0 || value > 2 ? 1 : value); return TW_OK; }
  if (!std::strcmp(name, "kernel")) { opt_kernel.store(value); return TW_OK; }
  if (!std::strcmp(name, "waves")) { opt_waves.store(value == 8 ? 8 : 4); return TW_OK; }
  if (!std::strcmp(name, "ksplit")) { opt_ksplit.store(value); return TW_OK; }
  if (!std::strcmp(name, "tiles_per_wg")) { opt_tiles_per_wg.store(value < 0 || value > 8 ? 0 : value); return TW_OK; }
  if (!std::strcmp(name, "idx_route")) { opt_idx_route.store(value < 0 || value > 2 ? 0 : value); return TW_OK; }
  if (!std::strcmp(name, "wg_split")) { opt_wg_split.store(value < 0 || value > 8 ? 0 : value); return TW_OK; }
  if (!std::strcmp(name, "tile_order")) { twg::longest_first.store(value != 0); return TW_OK; }
  if (!std::strcmp(name, "depth")) { opt_depth.store(value >= 3 && value <= 8 ? value : 3); return TW_OK; }
  return TW_ERR_ARG;
}

tw_status tw_flop_counts(tw_handle_t h, int64_t* sum_kw, int64_t* sum_k, int64_t* k_union) {
  if (!h) return TW_ERR_ARG;
  if (sum_kw) *sum_kw = h->sum_kw;
  if (sum_k) *sum_k = h->sum_k;
  if (k_union) *k_union = h->k_union;
  return TW_OK;
}

}  // extern "C"
