// TVW kernel: tile-wise condensation at the memory level, 2:4 along the
// condensed K inside the matrix core (Section III-A "TVW"; Algorithm 3, TVW).
//
// gfx950's sparse matrix instruction v_smfmac_f32_32x32x32_f16 takes the 2:4
// compressed matrix as its FIRST operand, so the product is formed transposed:
//
//      C^T tile (n x m)  =  B^T tile (n x Kc, 2:4 along Kc)  .  A^T gathered (Kc x m)
//
// which is the layout the path uses anyway (A is K x M, C is N x M; Section V
// "Memory Accesses Coalesce").  Per stage of 64 condensed rows a workgroup
// copies, with global_load_lds_dwordx4 and D stages in flight,
//   - the 64 gathered rows of A (kept-row list = Listing 1's CTO_k),
//   - the tile's compressed values for those rows, already in the register
//     order of the instruction (see the packer), and
//   - one position word per (lane, column block): 2 bits per stored value.
// The dense operand is read from the k-major A tile with ds_read_b64_tr_b16;
// lane (m, g) of a 32-row half-stage needs rows 8g..8g+7 and 16+8g..16+8g+7.
// Synchronisation, scalar index loads and the inline-assembly LDS reads are
// those of the asynchronous TW kernel.
#include <type_traits>

#include "device_common.h"

namespace twg {

namespace {

typedef int int4v __attribute__((ext_vector_type(4)));
typedef _Float16 half16 __attribute__((ext_vector_type(16)));

template <int OFF>
__device__ __forceinline__ int2v tr_read(uint32_t addr) {
  int2v v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
template <int OFF>
__device__ __forceinline__ int4v lds_read128(uint32_t addr) {
  int4v v;
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}
__device__ __forceinline__ int lds_read32(uint32_t addr) {
  int v;
  asm volatile("ds_read_b32 %0, %1" : "=v"(v) : "v"(addr));
  return v;
}

struct DenseFrag { int2v q[4]; };     // 32 m x 32 k of A^T: 16 halves per lane
__device__ __forceinline__ half16 as_half16(const DenseFrag& f) {
  union { int2v s[4]; half16 h; } u;
  u.s[0] = f.q[0]; u.s[1] = f.q[1]; u.s[2] = f.q[2]; u.s[3] = f.q[3];
  return u.h;
}
__device__ __forceinline__ half8 as_half8(const int4v& v) {
  union { int4v i; half8 h; } u;
  u.i = v;
  return u.h;
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

}  // namespace

constexpr int KS2 = 64;   // condensed rows per stage (two sparse instructions deep)

template <int TM, int TN, int WAVES_N, int D, int NW = 4>
__global__ __launch_bounds__(NW * 64) void tvw_gemm_km_kernel(GemmArgs g) {
  constexpr int NT = NW * 64;                            // threads of the workgroup
  constexpr int WAVES_M = NW / WAVES_N;
  constexpr int WN = TN / WAVES_N, WM = TM / WAVES_M;
  constexpr int NB = WN / 32, MB = WM / 32;
  static_assert(NB == 2 && (MB == 1 || MB == 2), "wave tiles are 64 columns by 32 or 64 rows of C^T");
  constexpr int NBT = TN / 32;                           // column blocks of the tile
  constexpr int RBA = TM * 2;
  constexpr int STAGE_A = KS2 * RBA;                     // gathered A rows
  constexpr int STAGE_V = KS2 * TN;                      // compressed values: 2 halves x NBT KiB
  constexpr int STAGE_I = 1024;                          // position words (NBT x 256 B used)
  constexpr int STAGE = STAGE_A + STAGE_V + STAGE_I;
  constexpr int NIA = STAGE_A / (1024 * NW), NIV = STAGE_V / (1024 * NW);   // copy instructions per wave and stage
  constexpr int RPIA = 1024 / RBA;                       // A rows per copy instruction
  static_assert(NIA == 2 || NIA == 4, "");
  static_assert(NIV >= 1 && (RPIA == 2 || RPIA == 4 || RPIA == 8), "");
  static_assert(D == 3 || D == 4, "");
  constexpr int NPS = NIA + NIV + 1;
  constexpr int CA = TM / 8;
  constexpr int CS = (TM + 4) * 2;
  constexpr int PIPE_BYTES = D * STAGE, EPI_BYTES = TN * CS;
  constexpr int LDS_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_gemm = g.n_mtiles * g.n_tiles;
  if ((int)blockIdx.x >= n_gemm) {
    zero_fill_column(g, blockIdx.x - n_gemm);
    return;
  }
  int mt, pos;
  tile_of_workgroup(g, blockIdx.x, n_gemm, mt, pos);
  int t, kp0, ns;
  if (g.uniform_kp > 0) { t = pos; kp0 = pos * g.uniform_kp; ns = g.uniform_kp / KS2; }   // equal tiles in column order
  else {
    const int4v rec = scalar_load4(g.tile_sched + 4 * pos);
    t = rec[0]; kp0 = rec[1]; ns = rec[2] / KS2;
  }
  const int m0 = mt * TM;
  // this tile's compressed values and position words
  const char* Vt = (const char*)g.vals + (size_t)kp0 * TN;            // kp0/2 rows x TN x 2 B
  const char* It = (const char*)g.meta + (size_t)(kp0 / KS2) * (NBT * 256);

  constexpr int ROWS_PER_PASS = NT / CA;
  constexpr int NPASS = TN / ROWS_PER_PASS;
  const int c = tid % CA, r0 = tid / CA;
  int cols[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) cols[i] = g.col_idx[t * TN + r0 + i * ROWS_PER_PASS];

  // ---- asynchronous copies -------------------------------------------------
  const int lb = lane * 16;
  const int a_rloc = lb / RBA;
  int a_el[NIA];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int row = (wave * NIA + j) * RPIA + a_rloc;
    a_el[j] = ((lb % RBA) ^ swz_mask<RBA>(row)) / 2;
    if (m0 + a_el[j] >= g.M) a_el[j] = 0;
  }
  const _Float16* Abase = g.A + m0;
  typedef int sidx_t __attribute__((ext_vector_type(RPIA)));
  struct Rows { sidx_t r[NIA]; };
  auto fetch_rows = [&](int s, Rows& dst) {
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      const int* rp = g.row_idx + kp0 + s * KS2 + (wave * NIA + j) * RPIA;
      if constexpr (RPIA == 2) asm volatile("s_load_dwordx2 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
      else if constexpr (RPIA == 4) asm volatile("s_load_dwordx4 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
      else asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
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
    {                                     // position words of column block wave % NBT: 256 bytes
      // (every wave issues one, so that all waves have the same number of copies per
      // stage in flight; waves that share a block write the same bytes)
      const int nb = wave % NBT;
      if (lane < 16)
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR(It + (size_t)s * (NBT * 256) + nb * 256 + lb),
                                         LDS_PTR(void, dstI + nb * 256), 16, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int row = rows.r[j][0];
#pragma unroll
      for (int q = 1; q < RPIA; ++q) row = (a_rloc == q) ? rows.r[j][q] : row;
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Abase + (size_t)row * g.lda + a_el[j]),
                                       LDS_PTR(void, dstA + (wave * NIA + j) * 1024), 16, 0, 0);
    }
  };

  floatx16 acc[NB][MB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int wn = wave % WAVES_N, wm = wave / WAVES_N;
  const uint32_t lds0 = (uint32_t)(uintptr_t)LDS_PTR(char, lds);
  const int p = lane & 15, q4 = lane >> 4;
  const int frow = 8 * (q4 >> 1) + (p >> 2);
  uint32_t fa[MB];       // dense operand: A^T tile, block of 32 m
#pragma unroll
  for (int j = 0; j < MB; ++j)
    fa[j] = lds0 + swz<RBA>(frow, (wm * WM + j * 32 + 16 * (q4 & 1) + 4 * (p & 3)) * 2);
  uint32_t fv[NB], fi[NB];   // sparse operand and its position word, column block wn*NB + i
#pragma unroll
  for (int i = 0; i < NB; ++i) {
    fv[i] = lds0 + STAGE_A + ((wn * NB + i) * 64 + lane) * 16;
    fi[i] = lds0 + STAGE_A + STAGE_V + ((wn * NB + i) * 64 + lane) * 4;
  }

  struct Step { DenseFrag d[MB]; int4v v[NB]; };
  Step f0, f1;
  int idx[NB];
  auto read_step = [&](uint32_t boff, auto U_, Step& f) {
    constexpr int U = decltype(U_)::value;               // half-stage: rows 32U .. 32U+31
#pragma unroll
    for (int j = 0; j < MB; ++j) {
      f.d[j].q[0] = tr_read<(32 * U + 0) * RBA>(fa[j] + boff);
      f.d[j].q[1] = tr_read<(32 * U + 4) * RBA>(fa[j] + boff);
      f.d[j].q[2] = tr_read<(32 * U + 16) * RBA>(fa[j] + boff);
      f.d[j].q[3] = tr_read<(32 * U + 20) * RBA>(fa[j] + boff);
    }
#pragma unroll
    for (int i = 0; i < NB; ++i) f.v[i] = lds_read128<U * NBT * 1024>(fv[i] + boff);
  };
  auto wait_step = [&](Step& f) {
    if constexpr (MB == 2)
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f.d[0].q[0]), "+v"(f.d[0].q[1]), "+v"(f.d[0].q[2]), "+v"(f.d[0].q[3]),
                     "+v"(f.d[1].q[0]), "+v"(f.d[1].q[1]), "+v"(f.d[1].q[2]), "+v"(f.d[1].q[3]),
                     "+v"(f.v[0]), "+v"(f.v[1]), "+v"(idx[0]), "+v"(idx[1]));
    else
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(f.d[0].q[0]), "+v"(f.d[0].q[1]), "+v"(f.d[0].q[2]), "+v"(f.d[0].q[3]),
                     "+v"(f.v[0]), "+v"(f.v[1]), "+v"(idx[0]), "+v"(idx[1]));
  };
  auto smfmac_step = [&](auto U_, const Step& f, const int* ix) {
    constexpr int U = decltype(U_)::value;
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < MB; ++j)
        acc[i][j] = __builtin_amdgcn_smfmac_f32_32x32x32_f16(as_half8(f.v[i]), as_half16(f.d[j]),
                                                             acc[i][j], ix[i], 0, U);
  };
  using U0 = std::integral_constant<int, 0>;
  using U1 = std::integral_constant<int, 1>;

  Rows rows_cur{}, rows_next{};
  if (ns > 0) {
    // kept-row lists of the first D stages in one round trip, then D-1 stages of copies
    Rows pro[D];
#pragma unroll
    for (int d = 0; d < D; ++d) fetch_rows(d < ns ? d : ns - 1, pro[d]);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int d = 0; d < D; ++d) tie_rows(pro[d]);
#pragma unroll
    for (int d = 0; d < D - 1; ++d)
      if (d < ns) issue(d, pro[d]);
    rows_cur = pro[D - 1];
  }
  int idx_prev[NB] = {0, 0};
  for (int s = 0; s < ns; ++s) {
    int newer = ns - 1 - s;
    if (newer > D - 2) newer = D - 2;
    if (newer >= 2) wait_vm<2 * NPS>();
    else if (newer == 1) wait_vm<NPS>();
    else wait_vm<0>();
    asm volatile("s_barrier" ::: "memory");
    fetch_rows(s + D < ns ? s + D : ns - 1, rows_next);   // needed by the next iteration
    const uint32_t boff = (uint32_t)((s % D) * STAGE);
    read_step(boff, U0{}, f0);
#pragma unroll
    for (int i = 0; i < NB; ++i) idx[i] = lds_read32(fi[i] + boff);
    if (s > 0) smfmac_step(U1{}, f1, idx_prev);   // second half of the previous stage
    wait_step(f0);                       // full wait: the scalar loads above are in as well
    tie_rows(rows_next);
    if (s + D - 1 < ns) issue(s + D - 1, rows_cur);
    read_step(boff, U1{}, f1);
    smfmac_step(U0{}, f0, idx);
    // explicit moves behind the wait: a plain copy would make idx loop-carried, and
    // the compiler may then copy the read's destination before the wait
#pragma unroll
    for (int i = 0; i < NB; ++i) asm volatile("v_mov_b32 %0, %1" : "=v"(idx_prev[i]) : "v"(idx[i]));
    rows_cur = rows_next;
    wait_step(f1);
  }
  if (ns > 0) smfmac_step(U1{}, f1, idx_prev);

  // ---- epilogue: acc[i][j][r] is C^T(n, m) with m = lane % 32 and
  // n = 8*(r/4) + 4*(lane/32) + r%4 inside the 32 x 32 block -------------------
  const int m = m0 + c * 8;
  long long dst_off[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i)
    dst_off[i] = (cols[i] < 0 || m >= g.M) ? -1 : (long long)cols[i] * g.ldc + m;
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < MB; ++j) {
      const int mm = wm * WM + j * 32 + (lane & 31);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int n = wn * WN + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        *(_Float16*)(lds + n * CS + mm * 2) = (_Float16)acc[i][j][r];
      }
    }
  __syncthreads();
  union Chunk { uint2 h[2]; u32x4 v; };
  Chunk ck[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    const int n = r0 + i * ROWS_PER_PASS;
    ck[i].h[0] = *(const uint2*)(lds + n * CS + c * 16);
    ck[i].h[1] = *(const uint2*)(lds + n * CS + c * 16 + 8);
  }
  // implicit img2col: the padding lanes of the wide grid are written as +0 (uniform branch)
  u32x4 vm = {~0u, ~0u, ~0u, ~0u};
  if (g.conv_P) vm = conv_valid_mask(g, m);
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    if (dst_off[i] < 0) continue;
    _Float16* dst = g.C + dst_off[i];
    if (m + 8 <= g.M) __builtin_nontemporal_store(ck[i].v & vm, (u32x4*)dst);
    else {
      const int n = r0 + i * ROWS_PER_PASS;
      const uint16_t* e = (const uint16_t*)(lds + n * CS + c * 16);
#pragma unroll
      for (int qq = 0; qq < 8; ++qq)
        if (m + qq < g.M) ((uint16_t*)dst)[qq] = e[qq] & (uint16_t)(vm[qq >> 1] >> (16 * (qq & 1)));
    }
  }
}

template <int TM, int TN, int WAVES_N, int D, int NW = 4>
static hipError_t launch(const GemmArgs& g, hipStream_t stream) {
  const int grid = g.n_mtiles * g.n_tiles + g.n_zero;
  if (grid <= 0) return hipSuccess;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this launch's
  hipLaunchKernelGGL((tvw_gemm_km_kernel<TM, TN, WAVES_N, D, NW>), dim3(grid), dim3(NW * 64), 0,
                     stream, g);
  return hipGetLastError();
}

hipError_t launch_tvw_km(int G, int tm, int depth, GemmArgs g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (G == 128 && tm == 128 && depth == 3) return launch<128, 128, 2, 3>(g, stream);
  if (G == 128 && tm == 128 && depth == 4) return launch<128, 128, 2, 4>(g, stream);
  if (G == 128 && tm == 256) return launch<256, 128, 2, 3, 8>(g, stream);   // 8 waves, 64 x 64 per wave
  if (G == 128 && tm == 64 && depth == 3) return launch<64, 128, 2, 3>(g, stream);   // 64 x 32 per wave
  if (G == 128 && tm == 64 && depth == 4) return launch<64, 128, 2, 4>(g, stream);
  if (G == 64 && tm == 128 && depth == 3) return launch<128, 64, 1, 3>(g, stream);
  if (G == 64 && tm == 128 && depth == 4) return launch<128, 64, 1, 4>(g, stream);
  return hipErrorInvalidValue;
}

}  // namespace twg
