// Internal: the object behind tw_handle_t.  Host-side logical form (what
// tw_export shows), the host staging copy of the device image, and the device
// pointers once uploaded.
#pragma once
#include <atomic>
#include <cstdint>
#include <vector>

#include "twgemm.h"

typedef struct ihipStream_t* hipStream_t;   // as the HIP runtime declares it (this header is also built without HIP)

namespace twg {

// K-step the device image is padded to.  One main-loop stage of the TW kernel
// consumes KSTEP_TW condensed rows, one stage of the TVW kernel KSTEP_TVW
// (two 2:4 sparse matrix-core instructions of 32 logical k each).
constexpr int KSTEP_TW = 32;
constexpr int KSTEP_TVW = 64;
constexpr int KSTEP_I8 = 64;     // int8 TW: one stage = two 32x32x32 matrix-core steps
constexpr int KSTEP_I8_TVW = 128; // int8 TVW: one stage = two 32x32x64 sparse steps
constexpr int ROW_IDX_SLACK = 1024 + KSTEP_I8_TVW;   // readable entries behind the last tile's list

struct DeviceImage {
  // host staging (filled by the packer)
  std::vector<int32_t> col_idx;      // n_tiles*G, -1 = no column (narrow last tile)
  std::vector<int32_t> tile_kp_off;  // n_tiles+1, prefix sums of padded K_t
  std::vector<int32_t> row_idx;      // sum Kp_t; pads repeat the tile's last kept row (0 if none)
  std::vector<int32_t> zero_cols;    // original indices of pruned columns
  std::vector<int32_t> tile_order;   // tiles by descending K_t (longest first)
  std::vector<int32_t> tile_sched;   // per launch position: {tile, kp offset, Kp_t, width}
  std::vector<uint16_t> vals;        // TW: [sum Kp_t][G]; TVW: swizzled compressed values
  std::vector<int8_t> vals8;         // int8: TW [sum Kp_t][G] bytes, TVW swizzled compressed bytes (vals is empty then)
  std::vector<uint32_t> meta;        // TVW: swizzled 2-bit position words
  std::vector<int32_t> ew_ptr;       // TEW: N+1 offsets into ew_pairs, by original column
  std::vector<uint32_t> ew_pairs;    // TEW: restored elements, row << 16 | fp16 bits
  int32_t uniform_kp = 0;            // > 0: all tiles have this padded K_t and are launched in column order
  size_t n_vals = 0, n_meta = 0;     // elements of the value / position-word parts (set with the lists)
  // device copies (one allocation, sub-pointers)
  void* blob = nullptr;
  size_t blob_bytes = 0;
  int device = -1;
  const int32_t* d_col_idx = nullptr;
  const int32_t* d_tile_kp_off = nullptr;
  const int32_t* d_row_idx = nullptr;
  const int32_t* d_zero_cols = nullptr;
  const int32_t* d_tile_order = nullptr;
  const int32_t* d_tile_sched = nullptr;
  const uint16_t* d_vals = nullptr;  // int8: the byte image, same slot
  const uint32_t* d_meta = nullptr;
  const int32_t* d_ew_ptr = nullptr;
  const uint32_t* d_ew_pairs = nullptr;
};

}  // namespace twg

struct tw_handle_s {
  int32_t K = 0, N = 0, G = 0, pattern = 0;
  int32_t dtype = TW_DTYPE_F16;      // int8 weights keep their bytes sign-extended in `values`
  int32_t n_kept = 0, n_tiles = 0;
  std::vector<int32_t> col_idx, cto_n, tile_col_off, tile_k_off, row_idx, cto_k;
  std::vector<int64_t> val_off, meta_off;
  std::vector<uint16_t> values;
  std::vector<uint8_t> meta, valid;
  std::vector<int32_t> ew_col_ptr, ew_row;   // TEW: restored elements, CSC over original columns
  std::vector<uint16_t> ew_val;
  int64_t sum_kw = 0, sum_k = 0;
  int32_t k_union = 0;  // K rows kept by at least one tile
  int32_t max_kp = 0;  // largest padded K_t
  twg::DeviceImage img;
  // device-side packing (tw_pack_dev): the logical values / 2:4 bytes live in this device
  // allocation (values first, then meta and valid at the offsets below) until somebody asks for
  // them on the host
  void* dev_logical = nullptr;
  size_t dev_logical_meta_off = 0, dev_logical_valid_off = 0;
  bool host_values_ready = true;     // false: `values` / `meta` / `valid` still have to be fetched
};

namespace twg {
// Fills *h from (B, mask[, tile_mask]).  Returns TW_OK / TW_ERR_MASK / TW_ERR_ALLOC.
tw_status pack_host(const uint16_t* B, const uint8_t* mask, const uint8_t* tile_mask,
                    int K, int N, int G, int pattern, tw_handle_s* h);
tw_status unpack_host(const tw_handle_s* h, uint16_t* Bm, uint8_t* mask);
// Fills *h with parts[0..n) side by side along N (same K, G and pattern).
tw_status concat_host(const tw_handle_s* const* parts, int n, tw_handle_s* h);
// Launch order of the tiles, read when a device image is built: 1 = longest K_t first.
extern std::atomic<int> longest_first;
// Builds h->img host staging from the logical form: the integer parts (from the lists alone),
// the value parts, or both.
void build_device_image(tw_handle_s* h);
void build_device_lists(tw_handle_s* h);
void build_device_values(tw_handle_s* h);
// From h->col_idx / tile_k_off / row_idx: tiles of G over the kept columns; then offsets,
// value offsets and the condensed work.
void set_tiles_of_G(tw_handle_s* h);
void finish_lists(tw_handle_s* h);
// Device-side packer (pack_dev.hip): fills *h from device buffers, image included (fp16, TW / TVW).
tw_status pack_device(const uint16_t* B, int ldb, const uint8_t* mask, const uint8_t* tile_mask, int K, int N,
                      int G, int pattern, hipStream_t stream, tw_handle_s* h);
// Copies the logical values of a device-packed handle to the host if they are not there yet.
tw_status fetch_logical_values(tw_handle_s* h);
}  // namespace twg
