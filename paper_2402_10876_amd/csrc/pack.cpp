// Host packer: pruned weight + mask -> condensed per-tile blocks, kept-row and
// kept-column index lists, compressed tile offsets and 2:4 positions.
//
// Paper: Section V removes the pruned rows and columns of every B tile offline
// and replaces the tile masks by the indices of the unpruned rows / columns
// ("Tile Fusion and Compressed Tile Offset"); Algorithm 3 condenses the kept
// columns before cutting tiles of G.  Integer work only; results are unique
// and compared bit for bit in the tests.
#include <algorithm>
#include <atomic>
#include <cstring>
#include <new>

#include "packed.h"

namespace twg {

std::atomic<int> longest_first{1};

namespace {

// kept-column list and per-tile kept-row lists of a structure mask S (K x N).
void structure_of(const uint8_t* S, int K, int N, int G, std::vector<int32_t>& cols,
                  std::vector<int32_t>& tile_k_off, std::vector<int32_t>& rows) {
  std::vector<uint8_t> col_any(N, 0);
  for (int k = 0; k < K; ++k) {
    const uint8_t* r = S + (size_t)k * N;
    for (int n = 0; n < N; ++n) col_any[n] |= (r[n] != 0);
  }
  cols.clear();
  for (int n = 0; n < N; ++n)
    if (col_any[n]) cols.push_back(n);
  const int n_kept = (int)cols.size();
  const int n_tiles = (n_kept + G - 1) / G;
  // tile id of every original column (-1 = pruned)
  std::vector<int32_t> tile_of(N, -1);
  for (int j = 0; j < n_kept; ++j) tile_of[cols[j]] = j / G;
  // row_any[t][k]
  std::vector<uint8_t> row_any((size_t)n_tiles * K, 0);
  for (int k = 0; k < K; ++k) {
    const uint8_t* r = S + (size_t)k * N;
    for (int j = 0; j < n_kept; ++j)
      if (r[cols[j]]) row_any[(size_t)(j / G) * K + k] = 1;
  }
  tile_k_off.assign(n_tiles + 1, 0);
  rows.clear();
  for (int t = 0; t < n_tiles; ++t) {
    for (int k = 0; k < K; ++k)
      if (row_any[(size_t)t * K + k]) rows.push_back(k);
    tile_k_off[t + 1] = (int32_t)rows.size();
  }
}

// true when S is exactly the union of (rows of tile t) x (columns of tile t)
bool is_tile_wise(const uint8_t* S, int K, int N, int G, const std::vector<int32_t>& cols,
                  const std::vector<int32_t>& tile_k_off) {
  // S is contained in that union by construction, so equality <=> equal counts
  int64_t nnz = 0;
  for (size_t i = 0, e = (size_t)K * N; i < e; ++i) nnz += (S[i] != 0);
  int64_t want = 0;
  const int n_kept = (int)cols.size();
  for (size_t t = 0; t + 1 < tile_k_off.size(); ++t) {
    int w = std::min(G, n_kept - (int)t * G);
    want += (int64_t)(tile_k_off[t + 1] - tile_k_off[t]) * w;
  }
  return nnz == want;
}

}  // namespace

// Tiles of G over the kept columns (Algorithm 3: Condense, then split by (1,G)).
void set_tiles_of_G(tw_handle_s* h) {
  h->n_kept = (int32_t)h->col_idx.size();
  h->n_tiles = (int32_t)h->tile_k_off.size() - 1;
  h->tile_col_off.resize(h->n_tiles + 1);
  for (int t = 0; t <= h->n_tiles; ++t) h->tile_col_off[t] = std::min(t * h->G, h->n_kept);
}

// Everything that follows from the index lists alone: offsets (index minus position, Section V),
// where each tile's values and 2:4 bytes start, the condensed work.
void finish_lists(tw_handle_s* h) {
  const bool tvw = h->pattern == TW_PATTERN_TVW;
  h->cto_n.resize(h->n_kept);
  for (int j = 0; j < h->n_kept; ++j) h->cto_n[j] = h->col_idx[j] - j;
  h->cto_k.resize(h->row_idx.size());
  h->val_off.assign(h->n_tiles + 1, 0);
  h->meta_off.assign(h->n_tiles + 1, 0);
  h->sum_kw = 0; h->sum_k = 0;
  for (int t = 0; t < h->n_tiles; ++t) {
    const int k0 = h->tile_k_off[t], kt = h->tile_k_off[t + 1] - k0;
    const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
    for (int j = 0; j < kt; ++j) h->cto_k[k0 + j] = h->row_idx[k0 + j] - j;
    h->sum_kw += (int64_t)kt * w;
    h->sum_k += kt;
    if (!tvw) {
      h->val_off[t + 1] = h->val_off[t] + (int64_t)kt * w;
    } else {
      const int ng = (kt + 3) / 4;
      h->val_off[t + 1] = h->val_off[t] + (int64_t)ng * 2 * w;
      h->meta_off[t + 1] = h->meta_off[t] + (int64_t)ng * w;
    }
  }
  std::vector<uint8_t> used(h->K, 0);
  for (int32_t r : h->row_idx) used[r] = 1;
  for (int32_t r : h->ew_row) used[r] = 1;
  h->k_union = 0;
  for (int k = 0; k < h->K; ++k) h->k_union += used[k];
}

tw_status pack_host(const uint16_t* B, const uint8_t* mask, const uint8_t* tile_mask, int K,
                    int N, int G, int pattern, tw_handle_s* h) try {
  h->K = K; h->N = N; h->G = G; h->pattern = pattern;
  const bool tvw = pattern == TW_PATTERN_TVW, tew = pattern == TW_PATTERN_TEW;
  const uint8_t* S = ((tvw || tew) && tile_mask) ? tile_mask : mask;
  structure_of(S, K, N, G, h->col_idx, h->tile_k_off, h->row_idx);
  set_tiles_of_G(h);
  if (!tvw || tile_mask) {
    if (!is_tile_wise(S, K, N, G, h->col_idx, h->tile_k_off)) return TW_ERR_MASK;
  }
  if (tvw && tile_mask) {
    for (size_t i = 0, e = (size_t)K * N; i < e; ++i)
      if (mask[i] && !tile_mask[i]) return TW_ERR_MASK;
  }
  if (tew) {   // the restored elements: in the mask, not in the tile mask; column by column
    for (size_t i = 0, e = (size_t)K * N; i < e; ++i)
      if (tile_mask[i] && !mask[i]) return TW_ERR_MASK;
    h->ew_col_ptr.assign(N + 1, 0);
    for (int n = 0; n < N; ++n) {
      for (int k = 0; k < K; ++k) {
        const size_t i = (size_t)k * N + n;
        if (mask[i] && !tile_mask[i]) { h->ew_row.push_back(k); h->ew_val.push_back(B[i]); }
      }
      h->ew_col_ptr[n + 1] = (int32_t)h->ew_row.size();
    }
  }
  finish_lists(h);
  h->values.assign((size_t)h->val_off[h->n_tiles], 0);
  if (!tvw) {
    for (int t = 0; t < h->n_tiles; ++t) {
      const int k0 = h->tile_k_off[t], kt = h->tile_k_off[t + 1] - k0;
      const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
      uint16_t* v = h->values.data() + h->val_off[t];
      const int32_t* cols = h->col_idx.data() + h->tile_col_off[t];
      for (int j = 0; j < kt; ++j) {
        const uint16_t* brow = B + (size_t)h->row_idx[k0 + j] * N;
        for (int c = 0; c < w; ++c) v[(size_t)j * w + c] = brow[cols[c]];
      }
    }
  } else {
    h->meta.assign((size_t)h->meta_off[h->n_tiles], 0);
    h->valid.assign((size_t)h->meta_off[h->n_tiles], 0);
    for (int t = 0; t < h->n_tiles; ++t) {
      const int k0 = h->tile_k_off[t], kt = h->tile_k_off[t + 1] - k0;
      const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
      const int ng = (kt + 3) / 4;
      uint16_t* v = h->values.data() + h->val_off[t];
      uint8_t* me = h->meta.data() + h->meta_off[t];
      uint8_t* va = h->valid.data() + h->meta_off[t];
      const int32_t* cols = h->col_idx.data() + h->tile_col_off[t];
      for (int g = 0; g < ng; ++g) {
        const int glen = std::min(4, kt - 4 * g);
        for (int c = 0; c < w; ++c) {
          const int n = cols[c];
          int setbits = 0, nset = 0;
          for (int p = 0; p < glen; ++p)
            if (mask[(size_t)h->row_idx[k0 + 4 * g + p] * N + n]) { setbits |= 1 << p; ++nset; }
          if (nset > 2) return TW_ERR_MASK;
          int chosen = setbits;  // top up with the lowest unset positions
          for (int p = 0; p < 4 && nset < 2; ++p)
            if (!(chosen >> p & 1)) { chosen |= 1 << p; ++nset; }
          int pos[2], i = 0;
          for (int p = 0; p < 4; ++p)
            if (chosen >> p & 1) pos[i++] = p;
          me[(size_t)g * w + c] = (uint8_t)(pos[0] | pos[1] << 2);
          uint8_t vb = 0;
          for (i = 0; i < 2; ++i) {
            if (setbits >> pos[i] & 1) {
              vb |= (uint8_t)(1 << i);
              v[((size_t)g * 2 + i) * w + c] = B[(size_t)h->row_idx[k0 + 4 * g + pos[i]] * N + n];
            }
          }
          va[(size_t)g * w + c] = vb;
        }
      }
    }
  }
  build_device_image(h);
  return TW_OK;
} catch (const std::bad_alloc&) {
  return TW_ERR_ALLOC;
}

tw_status unpack_host(const tw_handle_s* h, uint16_t* Bm, uint8_t* mask) {
  const size_t total = (size_t)h->K * h->N;
  if (Bm) std::memset(Bm, 0, total * sizeof(uint16_t));
  if (mask) std::memset(mask, 0, total);
  for (int t = 0; t < h->n_tiles; ++t) {
    const int k0 = h->tile_k_off[t], kt = h->tile_k_off[t + 1] - k0;
    const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
    const uint16_t* v = h->values.data() + h->val_off[t];
    const int32_t* cols = h->col_idx.data() + h->tile_col_off[t];
    if (h->pattern != TW_PATTERN_TVW) {
      for (int j = 0; j < kt; ++j) {
        const size_t row = (size_t)h->row_idx[k0 + j] * h->N;
        for (int c = 0; c < w; ++c) {
          if (Bm) Bm[row + cols[c]] = v[(size_t)j * w + c];
          if (mask) mask[row + cols[c]] = 1;
        }
      }
    } else {
      const uint8_t* me = h->meta.data() + h->meta_off[t];
      const uint8_t* va = h->valid.data() + h->meta_off[t];
      const int ng = (kt + 3) / 4;
      for (int g = 0; g < ng; ++g)
        for (int c = 0; c < w; ++c)
          for (int i = 0; i < 2; ++i) {
            if (!(va[(size_t)g * w + c] >> i & 1)) continue;
            const int p = me[(size_t)g * w + c] >> (2 * i) & 3;
            const size_t at = (size_t)h->row_idx[k0 + 4 * g + p] * h->N + cols[c];
            if (Bm) Bm[at] = v[((size_t)g * 2 + i) * w + c];
            if (mask) mask[at] = 1;
          }
    }
  }
  for (int n = 0; n + 1 < (int)h->ew_col_ptr.size(); ++n)
    for (int e = h->ew_col_ptr[n]; e < h->ew_col_ptr[n + 1]; ++e) {
      const size_t at = (size_t)h->ew_row[e] * h->N + n;
      if (Bm) Bm[at] = h->ew_val[e];
      if (mask) mask[at] = 1;
    }
  return TW_OK;
}

// Concatenation along N: the members' tiles, kept-row lists and condensed blocks
// follow one another unchanged; only the column indices move by the summed N of
// the members before.
tw_status concat_host(const tw_handle_s* const* parts, int n, tw_handle_s* h) try {
  const tw_handle_s* p0 = parts[0];
  h->K = p0->K; h->G = p0->G; h->pattern = p0->pattern; h->dtype = p0->dtype;
  h->N = 0; h->n_kept = 0; h->n_tiles = 0; h->sum_kw = 0; h->sum_k = 0;
  h->tile_col_off.assign(1, 0); h->tile_k_off.assign(1, 0);
  h->val_off.assign(1, 0); h->meta_off.assign(1, 0);
  if (h->pattern == TW_PATTERN_TEW) h->ew_col_ptr.assign(1, 0);
  for (int i = 0; i < n; ++i) {
    const tw_handle_s* p = parts[i];
    if (p->K != h->K || p->G != h->G || p->pattern != h->pattern || p->dtype != h->dtype) return TW_ERR_ARG;
    if ((int64_t)h->N + p->N > INT32_MAX) return TW_ERR_ARG;
    for (int32_t c : p->col_idx) h->col_idx.push_back(c + h->N);
    for (int t = 0; t < p->n_tiles; ++t) {
      h->tile_col_off.push_back(h->n_kept + p->tile_col_off[t + 1]);
      h->tile_k_off.push_back((int32_t)h->sum_k + p->tile_k_off[t + 1]);
      h->val_off.push_back((int64_t)h->values.size() + p->val_off[t + 1]);
      h->meta_off.push_back((int64_t)h->meta.size() + p->meta_off[t + 1]);
    }
    h->row_idx.insert(h->row_idx.end(), p->row_idx.begin(), p->row_idx.end());
    h->cto_k.insert(h->cto_k.end(), p->cto_k.begin(), p->cto_k.end());
    h->values.insert(h->values.end(), p->values.begin(), p->values.end());
    h->meta.insert(h->meta.end(), p->meta.begin(), p->meta.end());
    h->valid.insert(h->valid.end(), p->valid.begin(), p->valid.end());
    if (h->pattern == TW_PATTERN_TEW) {
      for (int c = 1; c <= p->N; ++c) h->ew_col_ptr.push_back((int32_t)h->ew_row.size() + p->ew_col_ptr[c]);
      h->ew_row.insert(h->ew_row.end(), p->ew_row.begin(), p->ew_row.end());
      h->ew_val.insert(h->ew_val.end(), p->ew_val.begin(), p->ew_val.end());
    }
    h->N += p->N; h->n_kept += p->n_kept; h->n_tiles += p->n_tiles;
    h->sum_kw += p->sum_kw; h->sum_k += p->sum_k;
  }
  h->cto_n.resize(h->n_kept);
  for (int j = 0; j < h->n_kept; ++j) h->cto_n[j] = h->col_idx[j] - j;
  std::vector<uint8_t> used(h->K, 0);
  for (int32_t r : h->row_idx) used[r] = 1;
  for (int32_t r : h->ew_row) used[r] = 1;
  h->k_union = 0;
  for (int k = 0; k < h->K; ++k) h->k_union += used[k];
  build_device_image(h);
  return TW_OK;
} catch (const std::bad_alloc&) {
  return TW_ERR_ALLOC;
}

// ---------------------------------------------------------------------------
// Device image.
//
// TW : per tile, Kp_t = K_t rounded up to KSTEP_TW rows of G halves, row-major,
//      zero filled (rows past K_t and columns past W_t).
// TVW: per tile, Kp_t = K_t rounded up to KSTEP_TVW.  The compressed tile is
//      stored in the register order of v_smfmac_f32_32x32x32_f16's sparse
//      operand: for K-stage s (64 rows), half u (32 rows), column block nb
//      (32 columns) and lane l:  column w = 32 nb + l%32, the 16 condensed rows
//      64 s + 32 u + 16 (l/32) .. +15, i.e. four groups of 4; element 2j+i is
//      stored value i of the lane's group j.  A lane's 8 halves are contiguous
//      (one 16-byte load), a wave's 64 lanes are contiguous (1 KiB).
//      Position words: one u32 per (s, nb, lane); bits [16u+4j+3 : 16u+4j] =
//      meta nibble of the lane's group j in half u (the instruction takes the
//      16-bit half selected by its ABID field, 2 bits per stored element).
// ---------------------------------------------------------------------------
void build_device_image(tw_handle_s* h) {
  build_device_lists(h);
  build_device_values(h);
}

// The integer parts of the device image: they follow from the logical lists alone.
void build_device_lists(tw_handle_s* h) {
  DeviceImage& d = h->img;
  const int G = h->G, nt = h->n_tiles;
  const bool tvw = h->pattern == TW_PATTERN_TVW;
  const bool i8 = h->dtype == TW_DTYPE_I8;
  const int kstep = i8 ? (tvw ? KSTEP_I8_TVW : KSTEP_I8) : tvw ? KSTEP_TVW : KSTEP_TW;
  d.col_idx.assign((size_t)nt * G, -1);
  for (int t = 0; t < nt; ++t)
    std::copy(h->col_idx.begin() + h->tile_col_off[t], h->col_idx.begin() + h->tile_col_off[t + 1],
              d.col_idx.begin() + (size_t)t * G);
  d.tile_kp_off.assign(nt + 1, 0);
  h->max_kp = 0;
  for (int t = 0; t < nt; ++t) {
    const int kt = h->tile_k_off[t + 1] - h->tile_k_off[t];
    const int kp = (kt + kstep - 1) / kstep * kstep;
    d.tile_kp_off[t + 1] = d.tile_kp_off[t] + kp;
    h->max_kp = std::max(h->max_kp, kp);
  }
  // slack behind the last tile (valid row 0): the K-split kernel copies stages of 64 rows and
  // may run one 32-row stage past a tile's end (it never multiplies it), and the TW kernel
  // stages the list through LDS in chunks of 8 stages, up to two chunks past a short tile
  d.row_idx.assign((size_t)d.tile_kp_off[nt] + ROW_IDX_SLACK, 0);
  for (int t = 0; t < nt; ++t) {
    const int k0 = h->tile_k_off[t], kt = h->tile_k_off[t + 1] - k0;
    const int kp0 = d.tile_kp_off[t], kp = d.tile_kp_off[t + 1] - kp0;
    for (int j = 0; j < kp; ++j)
      d.row_idx[kp0 + j] = kt ? h->row_idx[k0 + std::min(j, kt - 1)] : 0;
  }
  d.zero_cols.clear();
  {
    size_t j = 0;
    for (int n = 0; n < h->N; ++n) {
      if (j < h->col_idx.size() && h->col_idx[j] == n) { ++j; continue; }
      d.zero_cols.push_back(n);
    }
  }
  d.ew_ptr = h->ew_col_ptr;
  d.ew_pairs.resize(h->ew_row.size());
  for (size_t e = 0; e < h->ew_row.size(); ++e)
    d.ew_pairs[e] = (uint32_t)h->ew_row[e] << 16 | h->ew_val[e];
  d.tile_order.resize(nt);
  for (int t = 0; t < nt; ++t) d.tile_order[t] = t;
  if (longest_first.load())
    std::stable_sort(d.tile_order.begin(), d.tile_order.end(), [&](int a, int b) {
      return h->tile_k_off[a + 1] - h->tile_k_off[a] > h->tile_k_off[b + 1] - h->tile_k_off[b];
    });
  d.tile_sched.resize((size_t)nt * 4);
  for (int pos = 0; pos < nt; ++pos) {
    const int t = d.tile_order[pos];
    d.tile_sched[4 * pos + 0] = t;
    d.tile_sched[4 * pos + 1] = d.tile_kp_off[t];
    d.tile_sched[4 * pos + 2] = d.tile_kp_off[t + 1] - d.tile_kp_off[t];
    d.tile_sched[4 * pos + 3] = h->tile_col_off[t + 1] - h->tile_col_off[t];
  }
  // equal tiles launched in column order: the kernels can form the record from the position
  d.uniform_kp = nt > 0 ? d.tile_sched[2] : 0;
  for (int pos = 0; pos < nt && d.uniform_kp; ++pos)
    if (d.tile_sched[4 * pos] != pos || d.tile_sched[4 * pos + 2] != d.uniform_kp ||
        d.tile_sched[4 * pos + 1] != pos * d.uniform_kp)
      d.uniform_kp = 0;
  // sizes of the value parts (elements), so that a device image can be allocated before its
  // values exist (device-side packing)
  if (i8) { d.n_vals = tvw ? (size_t)d.tile_kp_off[nt] / 2 * G : ((size_t)d.tile_kp_off[nt] + KSTEP_I8) * G; }
  else d.n_vals = tvw ? (size_t)d.tile_kp_off[nt] / 2 * G : ((size_t)d.tile_kp_off[nt] + KSTEP_TW) * G;
  d.n_meta = !tvw ? 0 : i8 ? (size_t)d.tile_kp_off[nt] / 64 * (G / 32) * 64
                           : (size_t)d.tile_kp_off[nt] / KSTEP_TVW * (G / 32) * 64;
}

// The value parts of the device image, from the logical values (layouts above).
void build_device_values(tw_handle_s* h) {
  DeviceImage& d = h->img;
  const int G = h->G, nt = h->n_tiles;
  const bool tvw = h->pattern == TW_PATTERN_TVW;
  const bool i8 = h->dtype == TW_DTYPE_I8;
  if (i8 && tvw) {
    // int8 TVW, register order of v_smfmac_i32_32x32x64_i8's sparse operand: for K-stage s
    // (128 condensed rows), half u (64 rows = 16 groups of 4), column block nb and lane l:
    // column w = 32 nb + l%32; the lane's 16 bytes are stored values 0 and 1 of the groups
    // 8 (l/32) .. +7 of the half (byte 2j+i = value i of group j), its position word has the
    // meta nibble of group j at bits [4j+3 : 4j].  A lane's bytes are contiguous (one 16-byte
    // load), a wave's 64 lanes are contiguous (1 KiB); one word per (s, u, nb, lane).
    const int nbt = G / 32;
    d.vals.clear();
    d.vals8.assign((size_t)d.tile_kp_off[nt] / 2 * G, 0);
    d.meta.assign((size_t)d.tile_kp_off[nt] / 64 * nbt * 64, 0);
    for (int t = 0; t < nt; ++t) {
      const int kt = h->tile_k_off[t + 1] - h->tile_k_off[t];
      const int ng = (kt + 3) / 4;
      const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
      const int kp0 = d.tile_kp_off[t], kp = d.tile_kp_off[t + 1] - kp0;
      const uint16_t* v = h->values.data() + h->val_off[t];
      const uint8_t* me = h->meta.data() + h->meta_off[t];
      int8_t* ov = d.vals8.data() + (size_t)kp0 / 2 * G;
      uint32_t* om = d.meta.data() + (size_t)kp0 / 64 * nbt * 64;
      for (int su = 0; su < kp / 64; ++su)          // su = 2 s + u
        for (int nb = 0; nb < nbt; ++nb)
          for (int l = 0; l < 64; ++l) {
            const int c = 32 * nb + l % 32;
            int8_t* dst = ov + (((size_t)su * nbt + nb) * 64 + l) * 16;
            uint32_t word = 0;
            for (int j = 0; j < 8; ++j) {
              const int g = 16 * su + 8 * (l / 32) + j;   // logical group of 4 condensed rows
              uint32_t nib = 0x4;                         // positions (0,1), zero values
              if (g < ng && c < w) {
                nib = me[(size_t)g * w + c];
                dst[2 * j + 0] = (int8_t)(int16_t)v[((size_t)g * 2 + 0) * w + c];
                dst[2 * j + 1] = (int8_t)(int16_t)v[((size_t)g * 2 + 1) * w + c];
              }
              word |= nib << (4 * j);
            }
            om[((size_t)su * nbt + nb) * 64 + l] = word;
          }
    }
    return;
  }
  if (i8) {            // TW: the condensed rows as bytes
    d.vals.clear();
    d.meta.clear();
    d.vals8.assign(((size_t)d.tile_kp_off[nt] + KSTEP_I8) * G, 0);
    for (int t = 0; t < nt; ++t) {
      const int kt = h->tile_k_off[t + 1] - h->tile_k_off[t];
      const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
      const uint16_t* v = h->values.data() + h->val_off[t];
      int8_t* o = d.vals8.data() + (size_t)d.tile_kp_off[t] * G;
      for (int j = 0; j < kt; ++j)
        for (int c = 0; c < w; ++c) o[(size_t)j * G + c] = (int8_t)(int16_t)v[(size_t)j * w + c];
    }
    return;
  }
  if (!tvw) {
    d.vals.assign(((size_t)d.tile_kp_off[nt] + KSTEP_TW) * G, 0);
    for (int t = 0; t < nt; ++t) {
      const int kt = h->tile_k_off[t + 1] - h->tile_k_off[t];
      const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
      const uint16_t* v = h->values.data() + h->val_off[t];
      uint16_t* o = d.vals.data() + (size_t)d.tile_kp_off[t] * G;
      for (int j = 0; j < kt; ++j)
        std::copy(v + (size_t)j * w, v + (size_t)(j + 1) * w, o + (size_t)j * G);
    }
    d.meta.clear();
    return;
  }
  // TVW
  const int nb_per_tile = G / 32;
  d.vals.assign((size_t)d.tile_kp_off[nt] / 2 * G, 0);               // half the rows survive
  d.meta.assign((size_t)d.tile_kp_off[nt] / KSTEP_TVW * nb_per_tile * 64, 0);
  for (int t = 0; t < nt; ++t) {
    const int kt = h->tile_k_off[t + 1] - h->tile_k_off[t];
    const int ng = (kt + 3) / 4;
    const int w = h->tile_col_off[t + 1] - h->tile_col_off[t];
    const int kp0 = d.tile_kp_off[t], kp = d.tile_kp_off[t + 1] - kp0;
    const uint16_t* v = h->values.data() + h->val_off[t];
    const uint8_t* me = h->meta.data() + h->meta_off[t];
    uint16_t* ov = d.vals.data() + (size_t)kp0 / 2 * G;
    uint32_t* om = d.meta.data() + (size_t)kp0 / KSTEP_TVW * nb_per_tile * 64;
    for (int s = 0; s < kp / KSTEP_TVW; ++s)
      for (int nb = 0; nb < nb_per_tile; ++nb)
        for (int l = 0; l < 64; ++l) {
          const int c = 32 * nb + l % 32;
          uint32_t word = 0;
          for (int u = 0; u < 2; ++u) {
            uint16_t* dst = ov + ((((size_t)s * 2 + u) * nb_per_tile + nb) * 64 + l) * 8;
            for (int j = 0; j < 4; ++j) {
              const int g = 16 * s + 8 * u + 4 * (l / 32) + j;  // logical group of 4 rows
              uint32_t nib = 0x4;                               // positions (0,1), zero values
              if (g < ng && c < w) {
                nib = me[(size_t)g * w + c];
                dst[2 * j + 0] = v[((size_t)g * 2 + 0) * w + c];
                dst[2 * j + 1] = v[((size_t)g * 2 + 1) * w + c];
              }
              word |= nib << (16 * u + 4 * j);
            }
          }
          om[((size_t)s * nb_per_tile + nb) * 64 + l] = word;
        }
  }
}

}  // namespace twg
