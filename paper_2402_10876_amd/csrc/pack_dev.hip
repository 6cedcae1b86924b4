// Device-side packer: (B, mask[, tile mask]) in device memory -> packed handle, without moving
// the weight through the host.
//
// Paper: Section V condenses every B tile ahead of inference and replaces the tile masks by the
// indices of the unpruned rows / columns; Algorithm 3 condenses the kept columns before cutting
// tiles of G.  Here the same canonical form as the host packer's is produced by kernels:
//   structure  which columns keep anything, which rows keep anything in each tile of G kept
//              columns (one pass over the structure mask each), stream compaction into the
//              ascending index lists;
//   lists      only the index lists (a few KB) visit the host, where offsets, padding and the
//              launch order of the tiles are laid out exactly as for a host-packed weight;
//   values     one kernel gathers the kept values into the logical form (what tw_export
//              shows) and the kernel-facing image at once (TW), or forms the 2:4 positions
//              with the fill rule for short groups and then the register-order image (TVW).
// The logical values stay in device memory; they are copied to the host only if somebody asks
// for them (tw_export, tw_unpack, tw_concat).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <new>
#include <vector>

#include "packed.h"
#include "scan.h"

namespace twg {

namespace {

constexpr int T = 256;

// any[n] = 1 if column n of the K x N byte mask S has a non-zero entry
__global__ void column_any(const uint8_t* S, int K, int N, int32_t* any) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  int a = 0;
  for (int k = blockIdx.y; k < K; k += gridDim.y) a |= S[(size_t)k * N + n] != 0;
  if (a) any[n] = 1;                     // racing writers all store 1
}

// row_any[t][k] = 1 if row k has a non-zero entry among the columns of tile t; nnz counts S.
// blockIdx.y = row, threads over columns (no division per element); one atomic per workgroup.
__global__ void tile_row_any(const uint8_t* S, int K, int N, int G, const int32_t* col_pos, int32_t* row_any,
                             unsigned long long* nnz) {
  __shared__ int count;
  if (threadIdx.x == 0) count = 0;
  __syncthreads();
  int mine = 0;
  for (int k = blockIdx.y; k < K; k += gridDim.y)
    for (int n = blockIdx.x * blockDim.x + threadIdx.x; n < N; n += gridDim.x * blockDim.x)
      if (S[(size_t)k * N + n]) {
        row_any[(size_t)(col_pos[n] / G) * K + k] = 1;  // col_pos >= 0: the column has this entry; racing writers all store 1
        ++mine;
      }
  if (mine) atomicAdd(&count, mine);
  __syncthreads();
  if (threadIdx.x == 0 && count) atomicAdd(nnz, (unsigned long long)count);
}

// flag |= 1 where `inner` has an entry that `outer` lacks
__global__ void not_contained(const uint8_t* inner, const uint8_t* outer, size_t n, int32_t* flag) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n && inner[i] && !outer[i]) *flag = 1;
}

struct TileTables {           // device pointers, per tile t (n_tiles + 1 entries where offsets)
  const int32_t* tile_k_off;  // logical kept-row counts, prefix sums
  const int32_t* tile_kp_off; // padded, prefix sums (device image)
  const int32_t* tile_col_off;
  const int64_t* val_off;
  const int64_t* meta_off;
  const int32_t* row_idx;     // device image: padded lists at tile_kp_off
  const int32_t* col_idx;     // device image: [t * G + c], -1 = none
};

// TW: logical values V[t][j][c] and the image [kp0 + j][c] (zero padded), one thread per image element
__global__ void gather_tw(const uint16_t* B, int ldb, int G, TileTables tt, uint16_t* logical, uint16_t* image) {
  const int t = blockIdx.y;
  const int kp0 = tt.tile_kp_off[t], kp = tt.tile_kp_off[t + 1] - kp0;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kp * G) return;
  const int j = i / G, c = i - j * G;
  const int kt = tt.tile_k_off[t + 1] - tt.tile_k_off[t];
  const int w = tt.tile_col_off[t + 1] - tt.tile_col_off[t];
  uint16_t v = 0;
  if (j < kt && c < w) {
    v = B[(size_t)tt.row_idx[kp0 + j] * ldb + tt.col_idx[t * G + c]];
    logical[tt.val_off[t] + (size_t)j * w + c] = v;
  }
  image[(size_t)(kp0 + j) * G + c] = v;
}

// TVW, logical form: per (tile, group of 4 kept rows, column) the two stored positions, which
// of them are kept elements, and the two values (fillers are +0).  More than two kept elements
// in a group sets *bad.
__global__ void groups_tvw(const uint16_t* B, int ldb, const uint8_t* mask, int N, int G, TileTables tt,
                           uint16_t* values, uint8_t* meta, uint8_t* valid, int32_t* bad) {
  const int t = blockIdx.y;
  const int kp0 = tt.tile_kp_off[t];
  const int kt = tt.tile_k_off[t + 1] - tt.tile_k_off[t];
  const int w = tt.tile_col_off[t + 1] - tt.tile_col_off[t];
  const int ng = (kt + 3) / 4;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= ng * w) return;
  const int g = i / w, c = i - g * w;
  const int n = tt.col_idx[t * G + c];
  const int glen = min(4, kt - 4 * g);
  int rows[4], setbits = 0, nset = 0;
  for (int p = 0; p < glen; ++p) {
    rows[p] = tt.row_idx[kp0 + 4 * g + p];
    if (mask[(size_t)rows[p] * N + n]) { setbits |= 1 << p; ++nset; }
  }
  if (nset > 2) { *bad = 1; return; }
  int chosen = setbits;                  // top up with the lowest unset positions
  for (int p = 0; p < 4 && nset < 2; ++p)
    if (!(chosen >> p & 1)) { chosen |= 1 << p; ++nset; }
  int pos[2], q = 0;
  for (int p = 0; p < 4; ++p)
    if (chosen >> p & 1) pos[q++] = p;
  uint8_t vb = 0;
  uint16_t* v = values + tt.val_off[t];
  for (q = 0; q < 2; ++q) {
    uint16_t x = 0;
    if (setbits >> pos[q] & 1) { vb |= (uint8_t)(1 << q); x = B[(size_t)rows[pos[q]] * ldb + n]; }
    v[((size_t)g * 2 + q) * w + c] = x;
  }
  meta[tt.meta_off[t] + (size_t)g * w + c] = (uint8_t)(pos[0] | pos[1] << 2);
  valid[tt.meta_off[t] + (size_t)g * w + c] = vb;
}

// TVW, image: register order of the sparse matrix instruction's first operand (layout: see the
// host packer's build_device_values); one thread per (tile, 64-row stage, column block, lane)
__global__ void image_tvw(int G, TileTables tt, const uint16_t* values, const uint8_t* meta, uint16_t* img_vals,
                          uint32_t* img_meta) {
  const int t = blockIdx.y;
  const int nb_per_tile = G / 32;
  const int kp0 = tt.tile_kp_off[t], kp = tt.tile_kp_off[t + 1] - kp0;
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= kp / 64 * nb_per_tile * 64) return;
  const int l = i & 63, nb = (i >> 6) % nb_per_tile, s = (i >> 6) / nb_per_tile;
  const int kt = tt.tile_k_off[t + 1] - tt.tile_k_off[t];
  const int w = tt.tile_col_off[t + 1] - tt.tile_col_off[t];
  const int ng = (kt + 3) / 4;
  const uint16_t* v = values + tt.val_off[t];
  const uint8_t* me = meta + tt.meta_off[t];
  uint16_t* ov = img_vals + (size_t)kp0 / 2 * G;
  uint32_t* om = img_meta + (size_t)kp0 / 64 * nb_per_tile * 64;
  const int c = 32 * nb + l % 32;
  uint32_t word = 0;
  for (int u = 0; u < 2; ++u) {
    uint16_t* dst = ov + ((((size_t)s * 2 + u) * nb_per_tile + nb) * 64 + l) * 8;
    for (int j = 0; j < 4; ++j) {
      const int g = 16 * s + 8 * u + 4 * (l / 32) + j;
      uint32_t nib = 0x4;                               // positions (0,1), zero values
      uint16_t a = 0, b = 0;
      if (g < ng && c < w) {
        nib = me[(size_t)g * w + c];
        a = v[((size_t)g * 2 + 0) * w + c];
        b = v[((size_t)g * 2 + 1) * w + c];
      }
      dst[2 * j + 0] = a;
      dst[2 * j + 1] = b;
      word |= nib << (16 * u + 4 * j);
    }
  }
  om[((size_t)s * nb_per_tile + nb) * 64 + l] = word;
}

struct DevBuf {               // device allocation freed on scope exit
  void* p = nullptr;
  ~DevBuf() { if (p) (void)hipFree(p); }
  hipError_t alloc(size_t n) { return hipMalloc(&p, n ? n : 1); }
};

size_t up(size_t x) { return (x + 255) / 256 * 256; }

#define TWG_TRY(expr) do { if ((expr) != hipSuccess) { (void)hipGetLastError(); return TW_ERR_HIP; } } while (0)
#define TWG_LAUNCH(kernel, grid, block, ...)                                  \
  do {                                                                        \
    hipLaunchKernelGGL(kernel, grid, block, 0, s, __VA_ARGS__);               \
    if (hipGetLastError() != hipSuccess) return TW_ERR_HIP;                   \
  } while (0)

}  // namespace

tw_status pack_device(const uint16_t* B, int ldb, const uint8_t* mask, const uint8_t* tile_mask, int K, int N,
                      int G, int pattern, hipStream_t s, tw_handle_s* h) try {
  const bool tvw = pattern == TW_PATTERN_TVW;
  const uint8_t* S = (tvw && tile_mask) ? tile_mask : mask;
  h->K = K; h->N = N; h->G = G; h->pattern = pattern;
  if ((size_t)K * N / T + 1 > 0x7fffffffu) return TW_ERR_UNSUPPORTED;
  const size_t ntmax = (size_t)(N + G - 1) / G;
  (void)hipGetLastError();

  // ---- structure: kept columns, kept rows per tile --------------------------------------
  DevBuf ws;
  const size_t oN = up((size_t)N * 4), oR = up(ntmax * K * 4);
  if (ws.alloc(3 * oN + 3 * oR + 256) != hipSuccess) { (void)hipGetLastError(); return TW_ERR_ALLOC; }
  char* w = (char*)ws.p;
  int32_t* col_any = (int32_t*)w;        w += oN;
  int32_t* col_pos = (int32_t*)w;        w += oN;
  int32_t* col_list = (int32_t*)w;       w += oN;
  int32_t* row_any = (int32_t*)w;        w += oR;
  int32_t* row_pos = (int32_t*)w;        w += oR;
  int32_t* row_list = (int32_t*)w;       w += oR;
  unsigned long long* nnz = (unsigned long long*)w;
  int32_t* flags = (int32_t*)(w + 8);    // [0]: element mask leaves the tile mask, [1]: a 2:4 group keeps more than two
  TWG_TRY(hipMemsetAsync(col_any, 0, oN, s));
  TWG_TRY(hipMemsetAsync(row_any, 0, oR, s));
  TWG_TRY(hipMemsetAsync(nnz, 0, 256, s));
  const int ky = K < 64 ? K : 64;
  TWG_LAUNCH(column_any, dim3((N + T - 1) / T, ky), dim3(T), S, K, N, col_any);
  TWG_LAUNCH(compact, dim3(1), dim3(1024), col_any, N, col_pos, col_list);
  const unsigned eb = (unsigned)(((size_t)K * N + T - 1) / T);
  TWG_LAUNCH(tile_row_any, dim3((N + 4 * T - 1) / (4 * T), K < 65535 ? K : 65535), dim3(T), S, K, N, G, col_pos, row_any, nnz);
  TWG_LAUNCH(compact, dim3((unsigned)ntmax), dim3(1024), row_any, K, row_pos, row_list);
  if (tvw && tile_mask) TWG_LAUNCH(not_contained, dim3(eb), dim3(T), mask, tile_mask, (size_t)K * N, flags);

  // ---- the index lists visit the host -----------------------------------------------------
  std::vector<int32_t> cpos((size_t)N), rpos(ntmax * K);
  unsigned long long nnz_h = 0;
  int32_t flags_h[2] = {0, 0};
  TWG_TRY(hipMemcpyAsync(cpos.data(), col_pos, (size_t)N * 4, hipMemcpyDeviceToHost, s));
  TWG_TRY(hipMemcpyAsync(rpos.data(), row_pos, ntmax * K * 4, hipMemcpyDeviceToHost, s));
  TWG_TRY(hipMemcpyAsync(&nnz_h, nnz, 8, hipMemcpyDeviceToHost, s));
  TWG_TRY(hipMemcpyAsync(flags_h, flags, 8, hipMemcpyDeviceToHost, s));
  TWG_TRY(hipStreamSynchronize(s));
  if (flags_h[0]) return TW_ERR_MASK;
  for (int n = 0; n < N; ++n)
    if (cpos[n] >= 0) h->col_idx.push_back(n);
  const int n_tiles = ((int)h->col_idx.size() + G - 1) / G;
  h->tile_k_off.assign(n_tiles + 1, 0);
  for (int t = 0; t < n_tiles; ++t) {
    for (int k = 0; k < K; ++k)
      if (rpos[(size_t)t * K + k] >= 0) h->row_idx.push_back(k);
    h->tile_k_off[t + 1] = (int32_t)h->row_idx.size();
  }
  set_tiles_of_G(h);
  finish_lists(h);
  if (!tvw || tile_mask) {               // tile-wise: the structure mask is the union of its tiles' rows x columns
    if ((int64_t)nnz_h != h->sum_kw) return TW_ERR_MASK;
  }
  build_device_lists(h);

  // ---- device image and logical values ---------------------------------------------------------
  tw_status st = tw_upload(h);           // allocates all parts, copies the integer ones
  if (st != TW_OK) return st;
  twg::DeviceImage& d = h->img;
  const size_t n_log = (size_t)h->val_off[n_tiles], n_mb = (size_t)h->meta_off[n_tiles];
  const size_t o_val = 0, o_meta = up(n_log * 2), o_valid = o_meta + up(n_mb);
  const size_t o_tk = o_valid + up(n_mb), o_tc = o_tk + up((size_t)(n_tiles + 1) * 4);
  const size_t o_vo = o_tc + up((size_t)(n_tiles + 1) * 4), o_mo = o_vo + up((size_t)(n_tiles + 1) * 8);
  const size_t total = o_mo + up((size_t)(n_tiles + 1) * 8);
  void* lg = nullptr;
  if (hipMalloc(&lg, total) != hipSuccess) { (void)hipGetLastError(); return TW_ERR_ALLOC; }
  h->dev_logical = lg; h->dev_logical_meta_off = o_meta; h->dev_logical_valid_off = o_valid;
  h->host_values_ready = false;
  char* L = (char*)lg;
  TWG_TRY(hipMemcpyAsync(L + o_tk, h->tile_k_off.data(), (size_t)(n_tiles + 1) * 4, hipMemcpyHostToDevice, s));
  TWG_TRY(hipMemcpyAsync(L + o_tc, h->tile_col_off.data(), (size_t)(n_tiles + 1) * 4, hipMemcpyHostToDevice, s));
  TWG_TRY(hipMemcpyAsync(L + o_vo, h->val_off.data(), (size_t)(n_tiles + 1) * 8, hipMemcpyHostToDevice, s));
  TWG_TRY(hipMemcpyAsync(L + o_mo, h->meta_off.data(), (size_t)(n_tiles + 1) * 8, hipMemcpyHostToDevice, s));
  TWG_TRY(hipMemsetAsync((void*)d.d_vals, 0, d.n_vals * 2, s));
  TileTables tt{(const int32_t*)(L + o_tk), d.d_tile_kp_off, (const int32_t*)(L + o_tc), (const int64_t*)(L + o_vo),
                (const int64_t*)(L + o_mo), d.d_row_idx, d.d_col_idx};
  if (n_tiles > 0 && h->max_kp > 0) {
    if (!tvw) {
      TWG_LAUNCH(gather_tw, dim3((h->max_kp * G + T - 1) / T, n_tiles), dim3(T), B, ldb, G, tt,
                 (uint16_t*)(L + o_val), (uint16_t*)d.d_vals);
    } else {
      const int max_ng = (h->max_kp + 3) / 4;
      TWG_LAUNCH(groups_tvw, dim3((max_ng * G + T - 1) / T, n_tiles), dim3(T), B, ldb, mask, N, G, tt,
                 (uint16_t*)(L + o_val), (uint8_t*)(L + o_meta), (uint8_t*)(L + o_valid), flags + 1);
      TWG_LAUNCH(image_tvw, dim3((h->max_kp / 64 * (G / 32) * 64 + T - 1) / T, n_tiles), dim3(T), G, tt,
                 (const uint16_t*)(L + o_val), (const uint8_t*)(L + o_meta), (uint16_t*)d.d_vals,
                 (uint32_t*)d.d_meta);
    }
  }
  TWG_TRY(hipMemcpyAsync(flags_h, flags, 8, hipMemcpyDeviceToHost, s));
  TWG_TRY(hipStreamSynchronize(s));      // the workspace goes away when this returns
  if (flags_h[1]) return TW_ERR_MASK;
  return TW_OK;
} catch (const std::bad_alloc&) {
  return TW_ERR_ALLOC;
}

// Logical values of a device-packed handle, fetched on first use.
tw_status fetch_logical_values(tw_handle_s* h) try {
  if (!h->dev_logical || h->host_values_ready) return TW_OK;
  const int nt = h->n_tiles;
  const char* L = (const char*)h->dev_logical;
  h->values.resize((size_t)h->val_off[nt]);
  TWG_TRY(hipMemcpy(h->values.data(), L, h->values.size() * 2, hipMemcpyDeviceToHost));
  if (h->pattern == TW_PATTERN_TVW) {
    h->meta.resize((size_t)h->meta_off[nt]);
    h->valid.resize((size_t)h->meta_off[nt]);
    TWG_TRY(hipMemcpy(h->meta.data(), L + h->dev_logical_meta_off, h->meta.size(), hipMemcpyDeviceToHost));
    TWG_TRY(hipMemcpy(h->valid.data(), L + h->dev_logical_valid_off, h->valid.size(), hipMemcpyDeviceToHost));
  }
  h->host_values_ready = true;
  return TW_OK;
} catch (const std::bad_alloc&) {
  return TW_ERR_ALLOC;
}

}  // namespace twg
