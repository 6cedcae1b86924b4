// Int8 TVW kernel: tile-wise condensation at the memory level, 2:4 along the condensed
// K inside the matrix core (Section III-A "TVW", Algorithm 3), on int8 operands with
// exact int32 sums (Section VI-B "Int8 Quantization").
//
// The structure is that of the fp16 TVW kernel with bytes for halves.  The sparse
// instruction v_smfmac_i32_32x32x64_i8 takes the 2:4 compressed matrix first, so the
// product is formed transposed:
//
//      C^T tile (n x m)  =  B^T tile (n x Kc, 2:4 along Kc)  .  A^T gathered (Kc x m)
//
// Per stage of 128 condensed rows (two sparse instructions deep) a workgroup copies, with
// global_load_lds_dwordx4 and three stages in flight, the 128 gathered rows of A, the
// tile's compressed values for those rows in the register order of the instruction (see
// the packer) and one position word per (half, column block, lane).
// Operand layouts (found with a one-wave probe against a CPU product, pinned by the parity
// tests): for one instruction = 64 condensed rows = 16 groups of 4,
//   sparse : lane l holds column n = l % 32 and, as its 16 bytes, the two stored values of
//            the groups 8 (l / 32) .. +7; its index word has 2 bits per stored value;
//   dense  : lane l holds m = l % 32 and 32 bytes: rows 16 (l/32) .. +15 and
//            32 + 16 (l/32) .. +15, i.e. four transposing byte reads at rows +0, +8, +32, +40.
#include <type_traits>

#include "device_common.h"
#include "i8_common.h"

namespace twg {

namespace {

typedef int int4v __attribute__((ext_vector_type(4)));
typedef int int8v __attribute__((ext_vector_type(8)));

template <int OFF>
__device__ __forceinline__ int2v tr8_read(uint32_t addr) {
  int2v v;
  asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ int4v lds_read128(uint32_t addr) {
  int4v v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ int lds_read32(uint32_t addr) {
  int v;
  asm volatile("ds_read_b32 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

struct DenseFrag8 { int2v q[4]; };     // 32 m x 64 k of A^T: 32 bytes per lane
__device__ __forceinline__ int8v as_int8v(const DenseFrag8& f) {
  int8v r;
#pragma unroll
  for (int i = 0; i < 4; ++i) { r[2 * i] = f.q[i][0]; r[2 * i + 1] = f.q[i][1]; }
  return r;
}

__device__ __forceinline__ int4v scalar_load4(const void* p) {
  int4v r;
  asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(r) : "s"(p));
  return r;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// XOR mask on the byte offset inside a k-major row of RB bytes: the 8 rows x 32 bytes a
// half-wave of the transposing read touches go to the 8 slots of the 256-byte bank period.
template <int RB>
__device__ __forceinline__ int swz8_mask(int row) {
  if constexpr (RB == 256) return (row & 7) << 5;
  else if constexpr (RB == 128) return ((row >> 1) & 3) << 5;
  else return ((row >> 2) & 1) << 5;
}

constexpr int KSV = 128;   // condensed rows per stage

}  // namespace

template <int TM, int TN, int WAVES_N, bool OUT8>
__global__ __launch_bounds__(256) void tvw_gemm_i8_kernel(GemmI8Args g) {
  constexpr int NW = 4, NT = 256, D = 3;
  constexpr int WAVES_M = NW / WAVES_N;
  constexpr int WN = TN / WAVES_N, WM = TM / WAVES_M;
  constexpr int NB = WN / 32, MB = WM / 32;
  static_assert(NB == 2 && (MB == 1 || MB == 2), "wave tiles are 64 columns by 32 or 64 rows of C^T");
  constexpr int NBT = TN / 32;                           // column blocks of the tile
  constexpr int RBA = TM;                                // LDS row bytes of the A tile
  constexpr int STAGE_A = KSV * RBA;                      // gathered A rows
  constexpr int STAGE_V = KSV / 2 * TN;                   // compressed values: 2 halves x NBT KiB
  constexpr int IB = 2 * NBT * 256;                      // position words: [half][block][lane]
  constexpr int STAGE_I = IB < 1024 ? 1024 : IB;
  constexpr int STAGE = STAGE_A + STAGE_V + STAGE_I;
  constexpr int NIA = STAGE_A / (1024 * NW), NIV = STAGE_V / (1024 * NW);   // copy instructions per wave and stage
  constexpr int RPIA = 1024 / RBA;                       // A rows per copy instruction
  static_assert(NIA == 2 || NIA == 4, "");
  static_assert(NIV >= 1 && (RPIA == 8 || RPIA == 16), "");
  constexpr int NPS = NIA + NIV + 1;
  constexpr int CS = (TM + 4) * 4;                       // epilogue: int32 tile staged as [n][m]
  constexpr int PIPE_BYTES = D * STAGE, EPI_BYTES = TN * CS;
  constexpr int LDS_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_gemm = g.n_mtiles * g.n_tiles;
  if ((int)blockIdx.x >= n_gemm) {
    zero_fill_column8<OUT8>(g, blockIdx.x - n_gemm);
    return;
  }
  int mt, pos;
  tile_of_workgroup(g, blockIdx.x, n_gemm, mt, pos);
  int t, kp0, ns;
  if (g.uniform_kp > 0) { t = pos; kp0 = pos * g.uniform_kp; ns = g.uniform_kp / KSV; }   // equal tiles in column order
  else {
    const int4v rec = scalar_load4(g.tile_sched + 4 * pos);
    t = rec[0]; kp0 = rec[1]; ns = rec[2] / KSV;
  }
  const int m0 = mt * TM;
  // this tile's compressed values (kp0/2 rows x TN bytes) and position words
  const char* Vt = (const char*)g.vals + (size_t)kp0 / 2 * TN;
  const char* It = (const char*)g.meta + (size_t)(kp0 / KSV) * IB;

  // ---- asynchronous copies -------------------------------------------------
  const int lb = lane * 16;
  const int a_rloc = lb / RBA;
  int a_el[NIA];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int row = (wave * NIA + j) * RPIA + a_rloc;
    a_el[j] = (lb % RBA) ^ swz8_mask<RBA>(row);
    if (m0 + a_el[j] >= g.M) a_el[j] = 0;       // past M: re-read chunk 0 (those lanes are never stored)
  }
  const char* Abase = (const char*)(g.A + m0);
  const uint32_t lda = (uint32_t)g.lda;         // the host checks that K * lda fits 32 bits
  typedef int sidx_t __attribute__((ext_vector_type(RPIA)));
  struct Rows { sidx_t r[NIA]; };
  auto fetch_rows = [&](int s, Rows& dst) {
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      const int* rp = g.row_idx + kp0 + s * KSV + (wave * NIA + j) * RPIA;
      if constexpr (RPIA == 8) asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
      else asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
    }
  };
  auto tie_rows = [&](Rows& x) {      // after a wait: no use of x may be moved above this point
    if constexpr (NIA == 2) asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]));
    else asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]), "+s"(x.r[2]), "+s"(x.r[3]));
  };
  auto issue = [&](int s, const Rows& rows) {     // copies of stage s; rows = its kept-row indices
    char* dstA = lds + (s % D) * STAGE;
    char* dstV = dstA + STAGE_A;
    char* dstI = dstV + STAGE_V;
#pragma unroll
    for (int j = 0; j < NIV; ++j) {       // compressed values: plain linear copy
      const int kb = wave * NIV + j;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Vt + (size_t)s * STAGE_V + kb * 1024 + lb),
                                       LDS_PTR(void, dstV + kb * 1024), 16, 0, 0);
    }
    // position words: every wave copies a quarter of the stage's IB bytes
    if (lane < IB / 64)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(It + (size_t)s * IB + wave * (IB / 4) + lb),
                                       LDS_PTR(void, dstI + wave * (IB / 4)), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int row = rows.r[j][0];
#pragma unroll
      for (int q = 1; q < RPIA; ++q) row = (a_rloc == q) ? rows.r[j][q] : row;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Abase + ((uint32_t)row * lda + (uint32_t)a_el[j])),
                                       LDS_PTR(void, dstA + (wave * NIA + j) * 1024), 16, 0, 0);
    }
  };

  intx16 acc[NB][MB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int wn = wave % WAVES_N, wm = wave / WAVES_N;
  const uint32_t lds0 = (uint32_t)(uintptr_t)LDS_PTR(char, lds);
  const int p = lane & 15, q4 = lane >> 4;
  const int frow = 16 * (q4 >> 1) + (p >> 1);
  uint32_t fa[MB];       // dense operand: A^T tile, block of 32 m
#pragma unroll
  for (int j = 0; j < MB; ++j) {
    const int xb = wm * WM + j * 32 + 16 * (q4 & 1) + 8 * (p & 1);
    fa[j] = lds0 + frow * RBA + (xb ^ swz8_mask<RBA>(frow));
  }
  uint32_t fv[NB], fi[NB];   // sparse operand and its position word, column block wn*NB + i
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    fv[i] = lds0 + STAGE_A + ((wn * NB + i) * 64 + lane) * 16;
    fi[i] = lds0 + STAGE_A + STAGE_V + ((wn * NB + i) * 64 + lane) * 4;
  }

  struct Step { DenseFrag8 d[MB]; int4v v[NB]; int idx[NB]; };
  Step f0, f1;
  auto read_step = [&](uint32_t boff, auto U_, Step& f) {
    constexpr int U = decltype(U_)::value;               // half-stage: rows 64U .. 64U+63
    // rows +8, +32, +40 and +64 leave the swizzle mask of a lane's row unchanged
#pragma unroll
    for (int j = 0; j < MB; ++j) {
      f.d[j].q[0] = tr8_read<(64 * U + 0) * RBA>(fa[j] + boff);
      f.d[j].q[1] = tr8_read<(64 * U + 8) * RBA>(fa[j] + boff);
      f.d[j].q[2] = tr8_read<(64 * U + 32) * RBA>(fa[j] + boff);
      f.d[j].q[3] = tr8_read<(64 * U + 40) * RBA>(fa[j] + boff);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      f.v[i] = lds_read128<U * NBT * 1024>(fv[i] + boff);
      f.idx[i] = lds_read32<U * NBT * 256>(fi[i] + boff);
    }
  };
  auto wait_step = [&](Step& f) {
    if constexpr (MB == 2)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f.d[0].q[0]), "+v"(f.d[0].q[1]), "+v"(f.d[0].q[2]), "+v"(f.d[0].q[3]),
                     "+v"(f.d[1].q[0]), "+v"(f.d[1].q[1]), "+v"(f.d[1].q[2]), "+v"(f.d[1].q[3]),
                     "+v"(f.v[0]), "+v"(f.v[1]), "+v"(f.idx[0]), "+v"(f.idx[1]));
    else
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f.d[0].q[0]), "+v"(f.d[0].q[1]), "+v"(f.d[0].q[2]), "+v"(f.d[0].q[3]),
                     "+v"(f.v[0]), "+v"(f.v[1]), "+v"(f.idx[0]), "+v"(f.idx[1]));
  };
  auto smfmac_step = [&](const Step& f) {
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < MB; ++j)
        acc[i][j] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(f.v[i], as_int8v(f.d[j]), acc[i][j], f.idx[i], 0, 0);
  };
  using U0 = std::integral_constant<int, 0>;
  using U1 = std::integral_constant<int, 1>;

  Rows rows_cur{}, rows_next{};
  if (ns > 0) {
    // kept-row lists of the first two stages in one round trip and their copies, then the
    // list of the third (a stage's list is 32 scalar registers per wave: three at once
    // would not fit the scalar register file)
    static_assert(D == 3, "");
    {
      Rows pro[2];
      fetch_rows(0, pro[0]);
      fetch_rows(ns > 1 ? 1 : 0, pro[1]);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      tie_rows(pro[0]);
      tie_rows(pro[1]);
      issue(0, pro[0]);
      if (ns > 1) issue(1, pro[1]);
    }
    fetch_rows(ns > 2 ? 2 : ns - 1, rows_cur);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    tie_rows(rows_cur);
  }
  for (int s = 0; s < ns; ++s) {
    if (s + 1 < ns) wait_vm<NPS>();      // own copies of stage s have landed
    else wait_vm<0>();
    asm volatile("s_barrier" ::: "memory");
    fetch_rows(s + D < ns ? s + D : ns - 1, rows_next);   // needed by the next iteration
    const uint32_t boff = (uint32_t)((s % D) * STAGE);
    read_step(boff, U0{}, f0);
    if (s > 0) smfmac_step(f1);          // second half of the previous stage
    wait_step(f0);                       // full wait: the scalar loads above are in as well
    tie_rows(rows_next);
    if (s + D - 1 < ns) issue(s + D - 1, rows_cur);
    read_step(boff, U1{}, f1);
    smfmac_step(f0);
    rows_cur = rows_next;
    wait_step(f1);
  }
  if (ns > 0) smfmac_step(f1);

  // ---- epilogue: acc[i][j][r] is C^T(n, m) with m = lane % 32 and
  // n = 8*(r/4) + 4*(lane/32) + r%4 inside the 32 x 32 block; staged as [n][m] (int32, or
  // int8 requantised in registers), then every thread finishes (column, CH x m) pieces with
  // one 16-byte streaming store each
  constexpr int CH = OUT8 ? 16 : 4;
  constexpr int ES = OUT8 ? 1 : 4;                        // bytes per staged element
  constexpr int CSE = OUT8 ? TM + 16 : CS;                // staged row bytes
  constexpr int CA = TM / CH;
  constexpr int RPP = NT / CA;
  static_assert(TN % RPP == 0, "");
  constexpr int NPASS = TN / RPP;
  const int c = tid % CA, r0 = tid / CA;
  const int m = m0 + c * CH;
  int cols[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) cols[i] = g.col_idx[t * TN + r0 + i * RPP];
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j) {
      const int mm = wm * WM + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = wn * WN + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if constexpr (OUT8) *(int8_t*)(lds + n * CSE + mm) = (int8_t)requantize(acc[i][j][r], g.scale);
        else *(int*)(lds + n * CSE + mm * 4) = acc[i][j][r];
      }
    }
  __syncthreads();
  int4v pc[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) pc[i] = *(const int4v*)(lds + (r0 + i * RPP) * CSE + c * CH * ES);
  if (g.conv_P) {                                // implicit img2col: padding lanes of the grid are 0
    const int4v vm = (int4v)conv_valid_mask_i8<CH>(g, m);
#pragma unroll
    for (int i = 0; i < NPASS; ++i) pc[i] &= vm;
  }
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    if (cols[i] < 0 || m >= g.M) continue;
    char* dst = (char*)g.C + ((size_t)cols[i] * g.ldc + m) * ES;
    if (m + CH <= g.M) __builtin_nontemporal_store(pc[i], (int4v*)dst);
    else {
#pragma unroll
      for (int e = 0; e < CH; ++e)
        if (m + e < g.M) {
          if constexpr (OUT8) dst[e] = (char)(pc[i][e >> 2] >> (8 * (e & 3)));
          else ((int*)dst)[e] = pc[i][e];
        }
    }
  }
}

template <int TM, int TN, int WAVES_N>
static hipError_t launch_tvw8(const GemmI8Args& g, hipStream_t stream) {
  const int grid = g.n_mtiles * g.n_tiles + g.n_zero;
  if (grid <= 0) return hipSuccess;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this launch's
  if (g.c_i8)
    hipLaunchKernelGGL((tvw_gemm_i8_kernel<TM, TN, WAVES_N, true>), dim3(grid), dim3(256), 0, stream, g);
  else
    hipLaunchKernelGGL((tvw_gemm_i8_kernel<TM, TN, WAVES_N, false>), dim3(grid), dim3(256), 0, stream, g);
  return hipGetLastError();
}

hipError_t launch_tvw_i8(int G, int tm, GemmI8Args g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (G == 128 && tm == 128) return launch_tvw8<128, 128, 2>(g, stream);
  if (G == 128 && tm == 64) return launch_tvw8<64, 128, 2>(g, stream);
  if (G == 64 && tm == 128) return launch_tvw8<128, 64, 1>(g, stream);
  return hipErrorInvalidValue;
}

}  // namespace twg
