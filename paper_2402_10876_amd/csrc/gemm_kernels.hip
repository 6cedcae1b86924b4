// HIP kernels for gfx950: the grouped TW kernel and the dense baseline.
//
// One workgroup owns one (M-tile, N-tile) pair (Listing 1's thread block; the
// paper's multi-stream / batched launches are replaced by this single grouped
// launch, Section V "Tile Fusion").  A and C are in the transposed form of
// Section V "Memory Accesses Coalesce": A is K x M and C is N x M with M
// contiguous, so a kept K-row of a tile is one contiguous run of A and a kept
// column of C is one contiguous run of C.
//
// Per K-stage of 32 condensed rows the workgroup
//   1. reads 32 entries of the tile's kept-row list (Listing 1: CTO_k),
//   2. copies those rows of A (TM halves each, 16 B per lane) and the next
//      32 x TN block of the condensed weight into LDS, both k-major,
//   3. feeds v_mfma_f32_32x32x16_f16 from LDS with ds_read_b64_tr_b16, the
//      transposing LDS read that turns a k-major tile into the 8-consecutive-k
//      per lane operand the matrix core wants.
// The epilogue rounds fp32 -> fp16 once, stages the tile in LDS and stores
// whole rows of C^T at the kept-column indices (Listing 1: CTO_n).  Extra
// workgroups of the same launch write +0 to the pruned columns of C.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace twg {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define LDS_PTR(T, p) ((T __attribute__((address_space(3)))*)(p))

constexpr int KS = 32;        // condensed rows per stage
constexpr int NTHREADS = 256;

// Byte offset of element (row, x) of a k-major LDS tile with RB bytes per row.
// 32-byte segments are XOR-swizzled so that the four rows touched by one
// 16-lane group of a transposing read fall into four different bank groups.
template <int RB>
__device__ __forceinline__ int swz(int row, int xbytes) {
  int a = row * RB + xbytes;
  if constexpr (RB % 128 == 0) return a ^ ((row & 3) << 5);
  else return a ^ (((row >> 1) & 1) << 5);  // RB == 64: two rows per 128 B
}

// MFMA operand for 32 consecutive x (rows of D for srcA, columns for srcB) and
// 16 consecutive k, from a k-major LDS tile.  Lane l gets x = x0 + l%32,
// k = k0 + 8*(l/32) .. +7.
template <int RB>
__device__ __forceinline__ half8 lds_operand(const char* tile, int x0, int k0, int lane) {
  const int p = lane & 15, q = lane >> 4;
  const int row = k0 + 8 * (q >> 1) + (p >> 2);
  const int xb = (x0 + 16 * (q & 1) + 4 * (p & 3)) * 2;
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, tile + swz<RB>(row, xb)));
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(short4v, tile + swz<RB>(row + 4, xb)));
  union { short4v s[2]; half8 h; } u;
  u.s[0] = lo; u.s[1] = hi;
  return u.h;
}

template <int TM, int TN, int WAVES_M, bool DENSE>
__global__ __launch_bounds__(NTHREADS) void tw_gemm_km_kernel(GemmArgs g) {
  constexpr int WAVES_N = 4 / WAVES_M;
  constexpr int WM = TM / WAVES_M, WN = TN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  static_assert(MB >= 1 && NB >= 1, "wave tile must hold a 32x32 block");
  constexpr int RBA = TM * 2, RBB = TN * 2;          // LDS row bytes
  constexpr int CA = TM / 8, CB = TN / 8;            // 16-byte chunks per row
  constexpr int NA = (KS * CA + NTHREADS - 1) / NTHREADS;  // chunks per thread and stage
  constexpr int NBK = (KS * CB + NTHREADS - 1) / NTHREADS;
  constexpr int STAGE_A = KS * RBA, STAGE_B = KS * RBB;
  constexpr int CS = (TM + 8) * 2;                   // epilogue row bytes
  constexpr int PIPE_BYTES = 2 * (STAGE_A + STAGE_B);
  constexpr int EPI_BYTES = TN * CS;
  constexpr int LDS_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_gemm = g.n_mtiles * g.n_tiles;

  // ---- extra workgroups: +0 into the pruned columns of C -----------------
  if ((int)blockIdx.x >= n_gemm) {
    const int col = g.zero_cols[blockIdx.x - n_gemm];
    _Float16* row = g.C + (size_t)col * g.ldc;
    const u32x4 z = {0u, 0u, 0u, 0u};
    for (int m = tid * 8; m < g.M; m += NTHREADS * 8) {
      if (m + 8 <= g.M) *(u32x4*)(row + m) = z;
      else for (int i = m; i < g.M; ++i) row[i] = (_Float16)0.f;
    }
    return;
  }

  // ---- workgroup -> (M-tile, N-tile).  Consecutive workgroup ids are dealt
  // round-robin to the 8 XCDs; remap so that each XCD gets a contiguous range
  // of logical ids, i.e. walks all N-tiles of an M-band out of its own L2.
  int lid = blockIdx.x;
  if (g.xcd_map) {
    const int xcd = lid & 7, slot = lid >> 3;
    const int per = n_gemm >> 3, rem = n_gemm & 7;
    lid = (xcd < rem) ? xcd * (per + 1) + slot : rem * (per + 1) + (xcd - rem) * per + slot;
  }
  const int mt = lid / g.n_tiles;
  int t = lid - mt * g.n_tiles;
  if (!DENSE && g.tile_order) t = g.tile_order[t];
  const int m0 = mt * TM;

  int kp0, ns;
  if constexpr (DENSE) { kp0 = 0; ns = (g.K + KS - 1) / KS; }
  else { kp0 = g.tile_kp_off[t]; ns = (g.tile_kp_off[t + 1] - kp0) / KS; }
  const _Float16* Bt = DENSE ? g.vals + (size_t)t * TN : g.vals + (size_t)kp0 * TN;

  // per-thread chunk coordinates
  int a_row[NA], a_c[NA], b_row[NBK], b_c[NBK];
  bool a_on[NA], b_on[NBK];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    int id = tid + i * NTHREADS;
    a_on[i] = id < KS * CA; a_row[i] = (id / CA) % KS; a_c[i] = id % CA;
    // chunks starting past M re-read chunk 0 of the row (their lanes are never stored)
    if (m0 + a_c[i] * 8 >= g.M) a_c[i] = 0;
  }
#pragma unroll
  for (int i = 0; i < NBK; ++i) {
    int id = tid + i * NTHREADS;
    b_on[i] = id < KS * CB; b_row[i] = (id / CB) % KS; b_c[i] = id % CB;
    if constexpr (DENSE) { if (t * TN + b_c[i] * 8 >= g.N) b_on[i] = false; }
  }
  // chunk slot in LDS keeps the logical position even when the source is clamped
  int a_slot[NA];
#pragma unroll
  for (int i = 0; i < NA; ++i) a_slot[i] = swz<RBA>(a_row[i], (((tid + i * NTHREADS) % CA) * 16));
  int b_slot[NBK];
#pragma unroll
  for (int i = 0; i < NBK; ++i) b_slot[i] = swz<RBB>(b_row[i], (((tid + i * NTHREADS) % CB) * 16));

  auto load_idx = [&](int s, int* out) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      if constexpr (DENSE) { int k = s * KS + a_row[i]; out[i] = k < g.K ? k : g.K - 1; }
      else out[i] = g.row_idx[kp0 + s * KS + a_row[i]];
    }
  };
  u32x4 ra[NA], rb[NBK];
  auto load_stage = [&](int s, const int* idx) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      ra[i] = *(const u32x4*)(g.A + (size_t)idx[i] * g.lda + m0 + a_c[i] * 8);
#pragma unroll
    for (int i = 0; i < NBK; ++i) {
      u32x4 v = {0u, 0u, 0u, 0u};
      if constexpr (DENSE) {
        int k = s * KS + b_row[i];
        if (b_on[i] && k < g.K) v = *(const u32x4*)(Bt + (size_t)k * g.ldb + b_c[i] * 8);
      } else {
        if (b_on[i]) v = *(const u32x4*)(Bt + (size_t)(s * KS + b_row[i]) * TN + b_c[i] * 8);
      }
      rb[i] = v;
    }
  };
  auto store_stage = [&](int buf) {
    char* As = lds + buf * (STAGE_A + STAGE_B);
    char* Bs = As + STAGE_A;
#pragma unroll
    for (int i = 0; i < NA; ++i) if (a_on[i]) *(u32x4*)(As + a_slot[i]) = ra[i];
#pragma unroll
    for (int i = 0; i < NBK; ++i) if ((tid + i * NTHREADS) < KS * CB) *(u32x4*)(Bs + b_slot[i]) = rb[i];
  };

  floatx16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  int idx[NA];
  if (ns > 0) {
    load_idx(0, idx);
    load_stage(0, idx);
    if (ns > 1) load_idx(1, idx);
  }
  for (int s = 0; s < ns; ++s) {
    store_stage(s & 1);
    __syncthreads();
    if (s + 1 < ns) {
      load_stage(s + 1, idx);
      if (s + 2 < ns) load_idx(s + 2, idx);
    }
    const char* As = lds + (s & 1) * (STAGE_A + STAGE_B);
    const char* Bs = As + STAGE_A;
#pragma unroll
    for (int kk = 0; kk < KS; kk += 16) {
      half8 a[MB], b[NB];
#pragma unroll
      for (int i = 0; i < MB; ++i) a[i] = lds_operand<RBA>(As, wm * WM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < NB; ++j) b[j] = lds_operand<RBB>(Bs, wn * WN + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue: fp32 -> fp16 (RNE), stage as [n][m], store rows of C^T ----
  __syncthreads();
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int n = wn * WN + j * 32 + (lane & 31);
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        const int m = wm * WM + i * 32 + 8 * rq + 4 * (lane >> 5);
        half4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = (_Float16)acc[i][j][rq * 4 + r];
        *(half4*)(lds + n * CS + m * 2) = v;
      }
    }
  __syncthreads();
  constexpr int ROWS_PER_PASS = NTHREADS / CA;
  const int c = tid % CA, r0 = tid / CA;
  const int m = m0 + c * 8;
#pragma unroll 4
  for (int n = r0; n < TN; n += ROWS_PER_PASS) {
    int col;
    if constexpr (DENSE) { col = t * TN + n; if (col >= g.N) col = -1; }
    else col = g.col_idx[t * TN + n];
    if (col < 0 || m >= g.M) continue;
    const u32x4 v = *(const u32x4*)(lds + n * CS + c * 16);
    _Float16* dst = g.C + (size_t)col * g.ldc + m;
    if (m + 8 <= g.M) *(u32x4*)dst = v;
    else {
      const _Float16* hv = (const _Float16*)&v;
      for (int i = 0; m + i < g.M; ++i) dst[i] = hv[i];
    }
  }
}

template <int TM, int TN, int WAVES_M, bool DENSE>
static hipError_t launch(const GemmArgs& g, hipStream_t stream) {
  const int grid = g.n_mtiles * g.n_tiles + g.n_zero;
  if (grid <= 0) return hipSuccess;
  hipLaunchKernelGGL((tw_gemm_km_kernel<TM, TN, WAVES_M, DENSE>), dim3(grid), dim3(NTHREADS), 0,
                     stream, g);
  return hipGetLastError();
}

template <bool DENSE>
static hipError_t dispatch(int G, int tm, GemmArgs& g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
#define TWG_CASE(TM_, TN_, WM_) \
  if (G == TN_ && tm == TM_) return launch<TM_, TN_, WM_, DENSE>(g, stream);
  TWG_CASE(64, 128, 1) TWG_CASE(128, 128, 2) TWG_CASE(256, 128, 2)
  TWG_CASE(64, 64, 2) TWG_CASE(128, 64, 2) TWG_CASE(256, 64, 4)
  TWG_CASE(128, 32, 4) TWG_CASE(256, 32, 4)
#undef TWG_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_tw_km(int G, int tm, GemmArgs g, hipStream_t stream) {
  return dispatch<false>(G, tm, g, stream);
}
hipError_t launch_dense_km(int tn, int tm, GemmArgs g, hipStream_t stream) {
  return dispatch<true>(tn, tm, g, stream);
}

}  // namespace twg
