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
#include <type_traits>

#include "device_common.h"

namespace twg {

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

// MK = true: A is M x K and C is M x N, both row-major (the layout Section V
// calls uncoalesced once rows are pruned).  Only the global accesses differ:
// the gather reads single halves A[m][row_idx[k]] and the scatter writes single
// halves C[m][col_idx[n]]; LDS tiles, MFMA feeding and staging are unchanged.
// It is a compatibility path and is not tuned.
template <int TM, int TN, int WAVES_M, bool DENSE, bool MK>
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
  constexpr int CS = (TM + 4) * 2;                   // epilogue row bytes: 66 dwords mod 64 banks = 2
  constexpr int PIPE_BYTES = 2 * (STAGE_A + STAGE_B);
  constexpr int EPI_BYTES = TN * CS;
  constexpr int LDS_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(16))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n_gemm = g.n_mtiles * g.n_tiles;

  // ---- extra workgroups: +0 into the pruned columns of C -----------------
  if ((int)blockIdx.x >= n_gemm) {
    if constexpr (MK) {
      const int col = g.zero_cols[blockIdx.x - n_gemm];
      for (int i = tid; i < g.M; i += NTHREADS) g.C[(size_t)i * g.ldc + col] = (_Float16)0.f;
    } else {
      zero_fill_column(g, blockIdx.x - n_gemm);
    }
    return;
  }

  // ---- workgroup -> (M-tile, N-tile): one XCD walks all N-tiles of an M-band
  // out of its own L2.
  int mt, t;
  tile_of_workgroup(g, blockIdx.x, n_gemm, mt, t);
  if (!DENSE && g.tile_order) t = g.tile_order[t];
  const int m0 = mt * TM;

  int kp0, ns;
  if constexpr (DENSE) { kp0 = 0; ns = (g.K + KS - 1) / KS; }
  else { kp0 = g.tile_kp_off[t]; ns = (g.tile_kp_off[t + 1] - kp0) / KS; }
  const _Float16* Bt = DENSE ? g.vals + (size_t)t * TN : g.vals + (size_t)kp0 * TN;

  // per-thread chunk coordinates.  Every thread moves NA chunks of A and NBK
  // chunks of B per stage, without branches: a tile with fewer chunks than
  // threads (TN = 32) is covered twice with identical data.
  int a_row[NA], a_c[NA], a_slot[NA], b_row[NBK], b_c[NBK], b_slot[NBK];
  bool b_live[NBK];
#pragma unroll
  for (int i = 0; i < NA; ++i) {
    const int id = (tid + i * NTHREADS) % (KS * CA);
    a_row[i] = id / CA; a_c[i] = id % CA;
    a_slot[i] = swz<RBA>(a_row[i], a_c[i] * 16);
    // chunks starting past M re-read chunk 0 of the row (their lanes are never stored)
    if (m0 + a_c[i] * 8 >= g.M) a_c[i] = 0;
  }
#pragma unroll
  for (int i = 0; i < NBK; ++i) {
    const int id = (tid + i * NTHREADS) % (KS * CB);
    b_row[i] = id / CB; b_c[i] = id % CB;
    b_slot[i] = swz<RBB>(b_row[i], b_c[i] * 16);
    b_live[i] = true;
    if constexpr (DENSE) {
      if (t * TN + b_c[i] * 8 >= g.N) { b_live[i] = false; b_c[i] = 0; }  // past the last column
    }
  }

  auto load_idx = [&](int s, int* out) {
#pragma unroll
    for (int i = 0; i < NA; ++i) {
      if constexpr (DENSE) { int k = s * KS + a_row[i]; out[i] = k < g.K ? k : g.K - 1; }
      else out[i] = g.row_idx[kp0 + s * KS + a_row[i]];
    }
  };
  // Two register sets: while stage s is consumed from LDS, the global loads of
  // stages s+1 and s+2 are in flight.
  u32x4 ra[2][NA], rb[2][NBK];
  auto load_stage = [&](int s, const int* idx, u32x4* pa, u32x4* pb) {
#pragma unroll
    for (int i = 0; i < NA; ++i)
      if constexpr (MK) {
        union { _Float16 e[8]; u32x4 v; } u;
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          int mm = m0 + a_c[i] * 8 + q;
          if (mm >= g.M) mm = g.M - 1;
          u.e[q] = g.A[(size_t)mm * g.lda + idx[i]];
        }
        pa[i] = u.v;
      } else {
        pa[i] = *(const u32x4*)(g.A + (size_t)idx[i] * g.lda + m0 + a_c[i] * 8);
      }
#pragma unroll
    for (int i = 0; i < NBK; ++i) {
      if constexpr (DENSE) {
        const int k = s * KS + b_row[i];
        const int kc = k < g.K ? k : g.K - 1;
        u32x4 v = *(const u32x4*)(Bt + (size_t)kc * g.ldb + b_c[i] * 8);
        const bool keep = b_live[i] && k < g.K;   // rows past K and columns past N count as zero
        pb[i] = keep ? v : u32x4{0u, 0u, 0u, 0u};
      } else {
        pb[i] = *(const u32x4*)(Bt + (size_t)(s * KS + b_row[i]) * TN + b_c[i] * 8);
      }
    }
  };
  auto store_stage = [&](int buf, const u32x4* pa, const u32x4* pb) {
    char* As = lds + buf * (STAGE_A + STAGE_B);
    char* Bs = As + STAGE_A;
#pragma unroll
    for (int i = 0; i < NA; ++i) *(u32x4*)(As + a_slot[i]) = pa[i];
#pragma unroll
    for (int i = 0; i < NBK; ++i) *(u32x4*)(Bs + b_slot[i]) = pb[i];
  };

  floatx16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // kept-column indices of the rows of C^T this thread will store (CTO_n)
  constexpr int ROWS_PER_PASS = NTHREADS / CA;
  constexpr int NPASS = TN / ROWS_PER_PASS;
  const int c = tid % CA, r0 = tid / CA;
  int cols[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    const int n = r0 + i * ROWS_PER_PASS;
    if constexpr (DENSE) { cols[i] = t * TN + n; if (cols[i] >= g.N) cols[i] = -1; }
    else cols[i] = g.col_idx[t * TN + n];
  }

  const int wm = wave % WAVES_M, wn = wave / WAVES_M;
  int idx[2][NA];
  if (ns > 0) {
    load_idx(0, idx[0]);
    load_idx(ns > 1 ? 1 : 0, idx[1]);
    load_stage(0, idx[0], ra[0], rb[0]);
    __builtin_amdgcn_sched_barrier(0);
    // same issue order as the steady state (index list of stage s+2 before the
    // data of stage s+1), so the loop's wait counts are exact from the start
    load_idx(ns > 2 ? 2 : 0, idx[0]);
    __builtin_amdgcn_sched_barrier(0);
    load_stage(ns > 1 ? 1 : 0, idx[1], ra[1], rb[1]);
    __builtin_amdgcn_sched_barrier(0);
  }

  // One main-loop iteration on register set P.  LOAD: also issue stage s+2.
  auto body = [&](int s, auto P_, auto LOAD_) {
    constexpr int P = decltype(P_)::value;
    constexpr bool LOAD = decltype(LOAD_)::value;
    store_stage(s & 1, ra[P], rb[P]);
    if constexpr (LOAD) {
      // issue order matters (loads retire in order): index list of stage s+3
      // first, then the data of stage s+2, so that waiting for an index list
      // never waits for data issued after it
      __builtin_amdgcn_sched_barrier(0);
      load_idx(s + 3 < ns ? s + 3 : ns - 1, idx[1 - P]);
      __builtin_amdgcn_sched_barrier(0);
      load_stage(s + 2, idx[P], ra[P], rb[P]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // LDS writes done, then workgroup barrier; outstanding global loads stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
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
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  {
    int s = 0;
    for (; s + 3 < ns; s += 2) {          // both iterations prefetch (s+1+2 < ns)
      body(s, I0{}, std::true_type{});
      body(s + 1, I1{}, std::true_type{});
    }
    // here s is even and ns - s is 0, 1, 2 or 3
    if (s + 2 < ns) {                      // three left: one more prefetching iteration
      body(s, I0{}, std::true_type{});
      body(s + 1, I1{}, std::false_type{});
      body(s + 2, I0{}, std::false_type{});
    } else if (s + 1 < ns) {
      body(s, I0{}, std::false_type{});
      body(s + 1, I1{}, std::false_type{});
    } else if (s < ns) {
      body(s, I0{}, std::false_type{});
    }
  }

  // ---- epilogue: fp32 -> fp16 (RNE), stage as [n][m], store rows of C^T ----
  // Destination offsets are formed here from the column indices loaded at kernel
  // start: loads and stores share one in-order counter, so no load may still be
  // pending once the stores begin, or every store would wait for its predecessor.
  const int m = m0 + c * 8;
  long long dst_off[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i)
    dst_off[i] = (cols[i] < 0 || m >= g.M) ? -1 : (long long)cols[i] * g.ldc + m;
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
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    const int n = r0 + i * ROWS_PER_PASS;
    if (dst_off[i] < 0) continue;
    // staging rows are 8-byte aligned only: two 8-byte reads per chunk
    union { uint2 h[2]; u32x4 v; } u;
    u.h[0] = *(const uint2*)(lds + n * CS + c * 16);
    u.h[1] = *(const uint2*)(lds + n * CS + c * 16 + 8);
    if constexpr (MK) {
      const _Float16* e = (const _Float16*)&u;
      for (int q = 0; q < 8 && m + q < g.M; ++q) g.C[(size_t)(m + q) * g.ldc + cols[i]] = e[q];
    } else {
      _Float16* dst = g.C + dst_off[i];
      if (m + 8 <= g.M) __builtin_nontemporal_store(u.v, (u32x4*)dst);
      else {
        const _Float16* e = (const _Float16*)(lds + n * CS + c * 16);
        for (int q = 0; m + q < g.M; ++q) dst[q] = e[q];
      }
    }
  }
}

template <int TM, int TN, int WAVES_M, bool DENSE, bool MK>
static hipError_t launch(const GemmArgs& g, hipStream_t stream) {
  const int grid = g.n_mtiles * g.n_tiles + g.n_zero;
  if (grid <= 0) return hipSuccess;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this launch's
  hipLaunchKernelGGL((tw_gemm_km_kernel<TM, TN, WAVES_M, DENSE, MK>), dim3(grid), dim3(NTHREADS),
                     0, stream, g);
  return hipGetLastError();
}

template <bool DENSE>
static hipError_t dispatch(int G, int tm, GemmArgs& g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
#define TWG_CASE(TM_, TN_, WM_) \
  if (G == TN_ && tm == TM_) return launch<TM_, TN_, WM_, DENSE, false>(g, stream);
  TWG_CASE(64, 128, 1) TWG_CASE(128, 128, 2) TWG_CASE(256, 128, 2)
  TWG_CASE(64, 64, 2) TWG_CASE(128, 64, 2) TWG_CASE(256, 64, 4)
  TWG_CASE(128, 32, 4) TWG_CASE(256, 32, 4)
#undef TWG_CASE
  return hipErrorInvalidValue;
}

template <bool DENSE>
static hipError_t dispatch_mk(int G, GemmArgs& g, hipStream_t stream) {
  g.n_mtiles = (g.M + 127) / 128;
  if (G == 128) return launch<128, 128, 2, DENSE, true>(g, stream);
  if (G == 64) return launch<128, 64, 2, DENSE, true>(g, stream);
  if (G == 32) return launch<128, 32, 4, DENSE, true>(g, stream);
  return hipErrorInvalidValue;
}


hipError_t launch_tw_km(int G, int tm, GemmArgs g, hipStream_t stream) {
  return dispatch<false>(G, tm, g, stream);
}
hipError_t launch_dense_km(int tn, int tm, GemmArgs g, hipStream_t stream) {
  return dispatch<true>(tn, tm, g, stream);
}
hipError_t launch_tw_mk(int G, GemmArgs g, hipStream_t stream) { return dispatch_mk<false>(G, g, stream); }
hipError_t launch_dense_mk(int tn, GemmArgs g, hipStream_t stream) { return dispatch_mk<true>(tn, g, stream); }

}  // namespace twg
