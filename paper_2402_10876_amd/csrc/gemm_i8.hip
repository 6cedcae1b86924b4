// Int8 TW kernel and dense int8 baseline for gfx950 (Section VI-B "Int8
// Quantization": the TW pattern does not depend on the element type; the matrix
// cores multiply int8 operands into int32 sums, which are exact).
//
// Same decomposition, layouts and pipeline as the fp16 asynchronous-copy kernel
// (one workgroup per (M-tile, N-tile) pair, Listing 1; A is K x M and C is N x M,
// Section V "Memory Accesses Coalesce"; global_load_lds_dwordx4 copies, three
// stages in flight, one vmcnt wait and one s_barrier per stage), with bytes
// instead of halves:
//
//   stage   : 64 condensed rows = two v_mfma_i32_32x32x32_i8 steps per block.
//   LDS     : k-major tiles, TM (TN) bytes per row.  One transposing read
//             (ds_read_b64_tr_b8) of a half-wave touches 8 consecutive rows x 32
//             bytes; the XOR mask below sends those eight pieces to the eight
//             32-byte slots of the 256-byte bank period.
//   operand : lane l of the matrix instruction holds m (or n) = l % 32 and the 16
//             bytes k = 16 (l / 32) .. +15 of the step: two transposing reads, 8 rows
//             apart, whose source lane p of a 16-lane group reads 8 bytes at row
//             k0 + p / 2, column x0 + 8 (p % 2).
//   output  : int32 sums, or int8 = clamp(rne(fp32(sum) * scale)) (one fp32 product).
#include <type_traits>

#include "device_common.h"
#include "i8_common.h"

namespace twg {

namespace {

typedef int int4v __attribute__((ext_vector_type(4)));

template <int OFF>
__device__ __forceinline__ int2v tr8_read(uint32_t addr) {
  int2v v;
  asm volatile("ds_read_b64_tr_b8 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

struct Frag8 { int2v lo, hi; };

__device__ __forceinline__ int4v as_int4(const Frag8& f) {
  int4v r;
  r[0] = f.lo[0]; r[1] = f.lo[1]; r[2] = f.hi[0]; r[3] = f.hi[1];
  return r;
}

template <int N>
__device__ __forceinline__ void wait_lds8(Frag8* f) {
  // s_waitcnt tied to the fragments so that no use can be moved above it
  if constexpr (N == 3)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi));
  else if constexpr (N == 4)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi), "+v"(f[3].lo), "+v"(f[3].hi));
  else if constexpr (N == 6)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi), "+v"(f[3].lo), "+v"(f[3].hi), "+v"(f[4].lo),
                 "+v"(f[4].hi), "+v"(f[5].lo), "+v"(f[5].hi));
  else static_assert(N == 3, "unsupported fragment count");
}

// Wave-uniform 16-byte record through the scalar cache, complete on return.
__device__ __forceinline__ int4v scalar_load4(const void* p) {
  int4v r;
  asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(r) : "s"(p));
  return r;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// XOR mask on the byte offset inside a row of RB bytes (a multiple of 32: the 16-byte
// chunks of the copies and the 8-byte pieces of the reads stay whole).
template <int RB>
__device__ __forceinline__ int swz8_mask(int row) {
  if constexpr (RB == 256) return (row & 7) << 5;
  else if constexpr (RB == 128) return ((row >> 1) & 3) << 5;   // two rows per bank period
  else return ((row >> 2) & 1) << 5;                           // RB == 64: four rows per period
}
template <int RB>
__device__ __forceinline__ int swz8(int row, int xbytes) {
  return row * RB + (xbytes ^ swz8_mask<RB>(row));
}

constexpr int KS8 = 64;      // condensed rows per stage
constexpr int D8 = 3;        // stages in flight

}  // namespace

// KSPLIT = 2: two groups of four waves own the same output tile; a stage then holds 128
// condensed rows, group g multiplies rows 64g..64g+63 of it and the partial sums are added
// through LDS before the epilogue (long K with too few tiles to fill the chip).
template <int TM, int TN, int WAVES_M, bool DENSE, bool OUT8, int NWAVES = 4, int KSPLIT = 1>
// (the 256 x 128 instance holds 128 accumulators per lane; its epilogue must not push the
// register count past two waves per SIMD, which the 72 KiB of LDS allow)
__global__ __launch_bounds__(NWAVES * 64, (TM * TN >= 256 * 128) ? 2 : 1) void tw_gemm_i8_kernel(GemmI8Args g) {
  constexpr int NT = NWAVES * 64, D = D8;
  constexpr int WPG = NWAVES / KSPLIT;       // waves per K group
  constexpr int KSS = KS8 * KSPLIT;          // condensed rows per pipeline stage
  static_assert(!(DENSE && KSPLIT > 1), "the dense baseline does not split K");
  constexpr int WAVES_N = WPG / WAVES_M;
  constexpr int WM = TM / WAVES_M, WN = TN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  static_assert(MB >= 1 && NB >= 1, "wave tile must hold a 32x32 block");
  constexpr int RBA = TM, RBB = TN;                    // LDS row bytes
  constexpr int STAGE_A = KSS * RBA, STAGE_B = KSS * RBB, STAGE = STAGE_A + STAGE_B;
  static_assert(STAGE_A % (1024 * NWAVES) == 0 && STAGE_B % (1024 * NWAVES) == 0,
                "a stage is a whole number of 1 KiB copies per wave");
  constexpr int NIA = STAGE_A / (1024 * NWAVES), NIB = STAGE_B / (1024 * NWAVES);
  constexpr int RPIA = 1024 / RBA, RPIB = 1024 / RBB;  // tile rows per copy instruction
  static_assert(RPIA == 4 || RPIA == 8 || RPIA == 16, "row lists are fetched 4, 8 or 16 entries at a time");
  constexpr int NPS = NIA + NIB;
  // epilogue: int32 tile staged as [n][m], half of the columns at a time
  constexpr int CS = (TM + 4) * 4;
  constexpr int HN = TN / 2;
  static_assert(HN % 32 == 0, "");
  constexpr int PIPE_BYTES = D * STAGE, EPI_BYTES = HN * CS;
  constexpr int RED_BYTES = KSPLIT > 1 ? TM * TN * 4 : 0;      // partial sums of group 1
  static_assert(RED_BYTES <= PIPE_BYTES, "the reduction reuses the pipeline buffers");
  constexpr int LDS_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int n_gemm = g.n_mtiles * g.n_tiles;
  if ((int)blockIdx.x >= n_gemm) {
    zero_fill_column8<OUT8>(g, blockIdx.x - n_gemm);
    return;
  }
  int mt, t;                             // t: launch position of the tile, then the tile itself
  tile_of_workgroup(g, blockIdx.x, n_gemm, mt, t);
  const int m0 = mt * TM;

  int kp0, ns64;                         // ns64: stages of 64 rows
  if constexpr (DENSE) { kp0 = 0; ns64 = g.K / KS8; }  // host guarantees K % 64 == 0
  else {
    if (g.uniform_kp > 0) { kp0 = t * g.uniform_kp; ns64 = g.uniform_kp / KS8; }   // equal tiles in column order
    else {
      const int4v rec = scalar_load4(g.tile_sched + 4 * t);
      t = rec[0]; kp0 = rec[1]; ns64 = rec[2] / KS8;
    }
  }
  const int ns = (ns64 + KSPLIT - 1) / KSPLIT;         // pipeline stages of KSS rows
  const int8_t* Bt = DENSE ? g.vals + (size_t)t * TN : g.vals + (size_t)kp0 * TN;
  const uint32_t ldb = DENSE ? (uint32_t)g.ldb : (uint32_t)TN;

  // ---- geometry of the asynchronous copies: instruction j of this wave fills LDS
  // bytes [(wave*NI + j) KiB, +1 KiB) of the stage; lane l owns the 16 bytes at l*16,
  // i.e. tile row (wave*NI + j)*RPI + l*16/RB at physical byte (l*16) % RB, which
  // holds the logical bytes physical ^ swz8_mask(row).
  const int lb = lane * 16;
  const int a_rloc = lb / RBA, b_rloc = lb / RBB;
  int a_el[NIA], b_el[NIB];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int row = (wave * NIA + j) * RPIA + a_rloc;
    a_el[j] = (lb % RBA) ^ swz8_mask<RBA>(row);
    if (m0 + a_el[j] >= g.M) a_el[j] = 0;   // past M: re-read chunk 0 (those lanes are never stored)
  }
#pragma unroll
  for (int j = 0; j < NIB; ++j) {
    const int row = (wave * NIB + j) * RPIB + b_rloc;
    b_el[j] = (lb % RBB) ^ swz8_mask<RBB>(row);
    if constexpr (DENSE) { if (t * TN + b_el[j] >= g.N) b_el[j] = 0; }
  }
  // wave-uniform base plus an unsigned 32-bit byte offset per lane (the host checks
  // that A and B fit)
  const char* Abase = (const char*)(g.A + m0);
  const char* Bbase = (const char*)Bt;
  const uint32_t lda = (uint32_t)g.lda;
  uint32_t b_off[NIB];
#pragma unroll
  for (int j = 0; j < NIB; ++j)
    b_off[j] = (uint32_t)((wave * NIB + j) * RPIB + b_rloc) * ldb + (uint32_t)b_el[j];

  // Kept-row indices of a stage for copy instruction j: RPIA consecutive entries of the
  // list at a wave-uniform address, through scalar loads written in assembly (a vector
  // load would share the in-order counter of the asynchronous copies).  Each fetch is
  // issued right after a stage barrier and waited for together with the first operand
  // reads of that stage, one iteration before its rows are needed.
  typedef int sidx_t __attribute__((ext_vector_type(RPIA)));
  struct Rows { sidx_t r[NIA]; };
  auto fetch_rows = [&](int s, Rows& dst) {
    if constexpr (!DENSE) {
#pragma unroll
      for (int j = 0; j < NIA; ++j) {
        const int* rp = g.row_idx + kp0 + s * KSS + (wave * NIA + j) * RPIA;
        if constexpr (RPIA == 4) asm volatile("s_load_dwordx4 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
        else if constexpr (RPIA == 8) asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
        else asm volatile("s_load_dwordx16 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
      }
    }
  };
  auto tie_rows = [&](Rows& x) {      // after a wait: no use of x may be moved above this point
    if constexpr (!DENSE) {
      if constexpr (NIA == 1) asm volatile("" : "+s"(x.r[0]));
      else if constexpr (NIA == 2) asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]));
      else asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]), "+s"(x.r[2]), "+s"(x.r[3]));
    }
  };
  static_assert(NIA == 1 || NIA == 2 || NIA == 4, "");
  auto issue = [&](int s, const Rows& rows) {     // copies of stage s; rows = its kept-row indices
    char* dstA = lds + (s % D) * STAGE;
    char* dstB = dstA + STAGE_A;
    const uint32_t bs = (uint32_t)s * (uint32_t)KSS * ldb;
#pragma unroll
    for (int j = 0; j < NIB; ++j)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Bbase + (bs + b_off[j])),
                                       LDS_PTR(void, dstB + (wave * NIB + j) * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int row;
      if constexpr (DENSE) row = s * KSS + (wave * NIA + j) * RPIA + a_rloc;
      else {
        row = rows.r[j][0];
#pragma unroll
        for (int q = 1; q < RPIA; ++q) row = (a_rloc == q) ? rows.r[j][q] : row;
      }
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Abase + ((uint32_t)row * lda + (uint32_t)a_el[j])),
                                       LDS_PTR(void, dstA + (wave * NIA + j) * 1024), 16, 0, 0);
    }
  };

  intx16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int grp = KSPLIT == 1 ? 0 : wave / WPG;        // K group
  const int wl = KSPLIT == 1 ? wave : wave % WPG;      // wave inside the group
  const int wm = wl % WAVES_M, wn = wl / WAVES_M;
  // per-lane LDS byte address of each operand block at stage buffer 0, k-step 0
  const uint32_t lds0 = (uint32_t)(uintptr_t)LDS_PTR(char, lds);
  const int p = lane & 15, q = lane >> 4;
  const int frow = 16 * (q >> 1) + (p >> 1);
  const int fcol = 16 * (q & 1) + 8 * (p & 1);
  uint32_t fa[MB], fb[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) fa[i] = lds0 + grp * (KS8 * RBA) + swz8<RBA>(frow, wm * WM + i * 32 + fcol);
#pragma unroll
  for (int j = 0; j < NB; ++j)
    fb[j] = lds0 + STAGE_A + grp * (KS8 * RBB) + swz8<RBB>(frow, wn * WN + j * 32 + fcol);

  constexpr int NF = MB + NB;
  Frag8 f0[NF], f1[NF];      // operands of k-steps 0 and 1 of a stage
  auto read_step = [&](uint32_t boff, auto KK_, Frag8* f) {
    constexpr int KK = decltype(KK_)::value;
    // rows +8 and +32 leave the swizzle mask of a lane's row unchanged
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      f[i].lo = tr8_read<KK * RBA>(fa[i] + boff);
      f[i].hi = tr8_read<(KK + 8) * RBA>(fa[i] + boff);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      f[MB + j].lo = tr8_read<KK * RBB>(fb[j] + boff);
      f[MB + j].hi = tr8_read<(KK + 8) * RBB>(fb[j] + boff);
    }
  };
  auto mfma_step = [&](const Frag8* f) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(as_int4(f[i]), as_int4(f[MB + j]), acc[i][j], 0, 0, 0);
  };
  using K0 = std::integral_constant<int, 0>;
  using K32 = std::integral_constant<int, 32>;

  Rows rows_cur, rows_next;
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
  bool live_prev = false;
  for (int s = 0; s < ns; ++s) {
    // own copies of stage s have landed: at most the copies of the one newer stage remain
    if (s + 1 < ns) wait_vm<NPS>();
    else wait_vm<0>();
    // everybody's copies of stage s have landed, everybody is done reading stage s-1
    asm volatile("s_barrier" ::: "memory");
    fetch_rows(s + D < ns ? s + D : ns - 1, rows_next);   // needed by the next iteration
    const uint32_t boff = (uint32_t)((s % D) * STAGE);
    read_step(boff, K0{}, f0);
    if (KSPLIT == 1 ? s > 0 : live_prev) mfma_step(f1);   // second k-step of the previous stage
    const bool live = KSPLIT == 1 || s * KSPLIT + grp < ns64;   // false only for group 1 on an odd tail
    wait_lds8<NF>(f0);                   // full wait: the scalar loads above are in as well
    tie_rows(rows_next);
    // the copies of stage s+D-1 go into the buffer of stage s-1, which every wave has
    // finished reading
    if (s + D - 1 < ns) issue(s + D - 1, rows_cur);
    read_step(boff, K32{}, f1);
    if (live) mfma_step(f0);
    live_prev = live;
    rows_cur = rows_next;
    wait_lds8<NF>(f1);
  }
  if (KSPLIT == 1 ? ns > 0 : live_prev) mfma_step(f1);

  if constexpr (KSPLIT > 1) {
    // group 1 hands its partial sums to group 0: [wave in group][register][lane]
    __syncthreads();
    int* red = (int*)lds + wl * (MB * NB * 16 * 64) + lane;
    if (grp == 1) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) red[((i * NB + j) * 16 + r) * 64] = acc[i][j][r];
    }
    __syncthreads();
    if (grp == 0) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] += red[((i * NB + j) * 16 + r) * 64];
    }
  }

  if constexpr (OUT8) {
    // ---- epilogue, int8 output: requantise in registers, stage the whole tile as bytes
    // [n][m] (rows of TM + 16 bytes), then one 16-byte streaming store of 16 m per thread
    constexpr int CS8 = TM + 16;
    static_assert(TN * CS8 <= LDS_BYTES, "");
    constexpr int CA = TM / 16;                  // pieces per column
    constexpr int RPP = NT / CA;                 // columns per pass
    static_assert(TN % RPP == 0, "");
    constexpr int NPASS = TN / RPP;
    const int c = tid % CA, r0 = tid / CA;
    const int m = m0 + c * 16;
    int cols[NPASS];                             // original column of C of every piece (CTO_n)
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      const int n = r0 + i * RPP;
      if constexpr (DENSE) { cols[i] = t * TN + n; if (cols[i] >= g.N) cols[i] = -1; }
      else cols[i] = g.col_idx[t * TN + n];
    }
    __syncthreads();                             // the pipeline buffers are free
    if (grp == 0) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int n = wn * WN + j * 32 + (lane & 31);
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int mm = wm * WM + i * 32 + 8 * rq + 4 * (lane >> 5);
          uint32_t pk = 0;
#pragma unroll
          for (int r = 0; r < 4; ++r)
            pk |= ((uint32_t)requantize(acc[i][j][rq * 4 + r], g.scale) & 0xffu) << (8 * r);
          *(uint32_t*)(lds + n * CS8 + mm) = pk;
        }
      }
    }
    __syncthreads();
    int4v pc[NPASS];
#pragma unroll
    for (int i = 0; i < NPASS; ++i) pc[i] = *(const int4v*)(lds + (r0 + i * RPP) * CS8 + c * 16);
    if constexpr (!DENSE) {
      if (g.conv_P) {                            // implicit img2col: padding lanes of the grid are 0
        const int4v vm = (int4v)conv_valid_mask_i8<16>(g, m);
#pragma unroll
        for (int i = 0; i < NPASS; ++i) pc[i] &= vm;
      }
    }
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      if (cols[i] < 0 || m >= g.M) continue;
      int8_t* dst = (int8_t*)g.C + (size_t)cols[i] * g.ldc + m;
      if (m + 16 <= g.M) __builtin_nontemporal_store(pc[i], (int4v*)dst);
      else {
#pragma unroll
        for (int e = 0; e < 16; ++e)
          if (m + e < g.M) dst[e] = (int8_t)(pc[i][e >> 2] >> (8 * (e & 3)));
      }
    }
  } else {
  // ---- epilogue, int32 output: stage as [n][m], half of the tile's columns at a time;
  // every thread then finishes (column, 4 x m) pieces with one 16-byte streaming store each
  constexpr int CH = 4;                        // m values per piece
  constexpr int CA = TM / CH;                  // pieces per column
  constexpr int RPP = NT / CA;                 // columns per pass
  static_assert(HN % RPP == 0, "");
  constexpr int NPASS = HN / RPP;
  const int c = tid % CA, r0 = tid / CA;
  const int m = m0 + c * CH;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    // original column of C of every piece (CTO_n); loaded before the barrier, used after
    int cols[NPASS];
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      const int n = h * HN + r0 + i * RPP;
      if constexpr (DENSE) { cols[i] = t * TN + n; if (cols[i] >= g.N) cols[i] = -1; }
      else cols[i] = g.col_idx[t * TN + n];
    }
    __syncthreads();                     // pipeline buffers / the previous half are free
    if (grp == 0) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) {
        const int nblk = wn * WN + j * 32;                 // wave-uniform
        if (nblk / HN != h) continue;
        const int n = nblk - h * HN + (lane & 31);
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const int mm = wm * WM + i * 32 + 8 * rq + 4 * (lane >> 5);
          int4v v;
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = acc[i][j][rq * 4 + r];
          *(int4v*)(lds + n * CS + mm * 4) = v;
        }
      }
    }
    __syncthreads();
    // all staged pieces into registers first (unconditional reads), then the stores
    int4v pc[NPASS];
#pragma unroll
    for (int i = 0; i < NPASS; ++i) pc[i] = *(const int4v*)(lds + (r0 + i * RPP) * CS + c * 16);
    if constexpr (!DENSE) {
      if (g.conv_P) {
        const int4v vm = (int4v)conv_valid_mask_i8<4>(g, m);
#pragma unroll
        for (int i = 0; i < NPASS; ++i) pc[i] &= vm;
      }
    }
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      if (cols[i] < 0 || m >= g.M) continue;
      int* dst = (int*)g.C + (size_t)cols[i] * g.ldc + m;
      if (m + 4 <= g.M) __builtin_nontemporal_store(pc[i], (int4v*)dst);
      else {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (m + e < g.M) dst[e] = pc[i][e];
      }
    }
  }
  }
}

template <int TM, int TN, int WAVES_M, bool DENSE, int NWAVES = 4, int KSPLIT = 1>
static hipError_t launch8(const GemmI8Args& g, hipStream_t stream) {
  const int grid = g.n_mtiles * g.n_tiles + g.n_zero;
  if (grid <= 0) return hipSuccess;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this launch's
  if (g.c_i8)
    hipLaunchKernelGGL((tw_gemm_i8_kernel<TM, TN, WAVES_M, DENSE, true, NWAVES, KSPLIT>), dim3(grid),
                       dim3(NWAVES * 64), 0, stream, g);
  else
    hipLaunchKernelGGL((tw_gemm_i8_kernel<TM, TN, WAVES_M, DENSE, false, NWAVES, KSPLIT>), dim3(grid),
                       dim3(NWAVES * 64), 0, stream, g);
  return hipGetLastError();
}

template <bool DENSE>
static hipError_t dispatch8(int G, int tm, GemmI8Args& g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (G == 128 && tm == 64) return launch8<64, 128, 1, DENSE>(g, stream);
  if (G == 128 && tm == 128) return launch8<128, 128, 2, DENSE>(g, stream);
  if (G == 128 && tm == 256) return launch8<256, 128, 2, DENSE>(g, stream);
  if (G == 64 && tm == 128) return launch8<128, 64, 2, DENSE>(g, stream);
  if (G == 64 && tm == 256) return launch8<256, 64, 4, DENSE>(g, stream);
  return hipErrorInvalidValue;
}

hipError_t launch_tw_i8(int G, int tm, int ksplit, GemmI8Args g, hipStream_t stream) {
  if (ksplit == 2) {          // two K groups of four waves
    g.n_mtiles = (g.M + tm - 1) / tm;
    if (G == 128 && tm == 64) return launch8<64, 128, 1, false, 8, 2>(g, stream);
    if (G == 128 && tm == 128) return launch8<128, 128, 2, false, 8, 2>(g, stream);
    if (G == 64 && tm == 128) return launch8<128, 64, 2, false, 8, 2>(g, stream);
    return hipErrorInvalidValue;
  }
  return dispatch8<false>(G, tm, g, stream);
}

hipError_t launch_dense_i8(int tn, int tm, GemmI8Args g, hipStream_t stream) {
  g.n_zero = 0;
  return dispatch8<true>(tn, tm, g, stream);
}

}  // namespace twg
