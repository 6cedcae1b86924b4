// Grouped TW kernel / dense baseline, asynchronous-copy pipeline for gfx950.
//
// Same decomposition and layouts as the register-staged kernel (one workgroup
// per (M-tile, N-tile) pair, Listing 1; A is K x M and C is N x M, Section V
// "Memory Accesses Coalesce"), but the stage copies never pass through
// registers: every wave issues global_load_lds_dwordx4, which moves 64 x 16
// bytes from per-lane global addresses straight into 1 KiB of LDS.  D stages
// of 32 condensed rows are in flight per workgroup; the only synchronisation
// per stage is one vmcnt wait and one s_barrier.
//
//   gather  : lane l of a copy instruction fetches one 16-byte chunk of row
//             row_idx[...] of A (Listing 1: CTO_k); the four (TM=128) rows an
//             instruction covers come from one scalar load of the index list.
//   LDS     : k-major tiles, 64-byte units XOR-swizzled (see swz_mask); the
//             swizzle is applied on the global side, the LDS side of a copy
//             instruction is always 1 KiB contiguous.
//   MFMA    : operands come from ds_read_b64_tr_b16 issued from inline
//             assembly.  The compiler orders every LDS read it knows about
//             behind all earlier asynchronous copies (vmcnt(0)), which would
//             serialise the pipeline; reads it cannot see are ordered by the
//             explicit waits written here instead.
//   overlap : the MFMAs of the second half of stage s are issued after the
//             barrier and the operand reads of stage s+1, so LDS latency is
//             hidden behind matrix-core work.
#include <type_traits>

#include "device_common.h"

namespace twg {

namespace {

template <int OFF>
__device__ __forceinline__ int2v tr_read(uint32_t addr) {
  int2v v;
  asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFF));
  return v;
}

// One matrix-core operand (32 x-values x 16 k) = two transposed 64-bit reads.
struct Frag { int2v lo, hi; };

__device__ __forceinline__ half8 as_half8(const Frag& f) {
  union { int2v s[2]; half8 h; } u;
  u.s[0] = f.lo; u.s[1] = f.hi;
  return u.h;
}

template <int N>
__device__ __forceinline__ void wait_lds(Frag* f) {
  // s_waitcnt tied to the fragments so that no use can be moved above it
  if constexpr (N == 2)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi));
  else if constexpr (N == 3)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi));
  else if constexpr (N == 4)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi), "+v"(f[3].lo), "+v"(f[3].hi));
  else if constexpr (N == 6)
    asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(f[0].lo), "+v"(f[0].hi), "+v"(f[1].lo), "+v"(f[1].hi),
                 "+v"(f[2].lo), "+v"(f[2].hi), "+v"(f[3].lo), "+v"(f[3].hi), "+v"(f[4].lo),
                 "+v"(f[4].hi), "+v"(f[5].lo), "+v"(f[5].hi));
  else static_assert(N == 2, "unsupported fragment count");
}

// Wave-uniform 16-byte record through the scalar cache, complete on return.
typedef int int4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ int4v scalar_load4(const void* p) {
  int4v r;
  asm volatile("s_load_dwordx4 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=s"(r) : "s"(p));
  return r;
}

template <int N>
__device__ __forceinline__ void wait_vm() {
  static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Waits until at most `newer` stages of NPS copies each are outstanding (newer <= MAXN; in the
// steady state newer == MAXN and the first comparison decides).
template <int NPS, int MAXN>
__device__ __forceinline__ void wait_stage(int newer) {
  if constexpr (MAXN == 0) wait_vm<0>();
  else {
    if (newer >= MAXN) wait_vm<MAXN * NPS>();
    else wait_stage<NPS, MAXN - 1>(newer);
  }
}

}  // namespace

// KSPLIT = 2: the workgroup has two groups of waves that own the same output
// tile; a pipeline stage then holds 64 condensed rows, group g multiplies rows
// 32g..32g+31 of it, and the two partial accumulators are added through LDS
// (in fp32, before the single rounding).  It gives a tile two waves per SIMD,
// which long-K problems with few tiles need to keep the matrix cores busy.

// ---- TEW: restored elements (Section III-A "TEW": the element-wise part is kept in
// compressed sparse column form and, the product being linear, computed apart from the
// TW part).  Here it is added to the fp32 sums of the thread that stores the 8 values
// C^T[col][m .. m+8): for every restored (k, v) of the column, s += v * A^T[k][m .. m+8).
// Pairs travel as k << 16 | fp16 bits; the list is padded in registers with
// (row 0, +0), which adds nothing.  Every load is unconditional (index clamped to the
// list, value selected afterwards): a load under a branch would be waited for on its own.  A rows are lda >= round-up-8(M) halves long, so the
// 16-byte read at m < M stays inside the row; lanes at or past M are not stored.
template <int P>      // P columns at a time: P times the loads in flight per round trip
__device__ __forceinline__ void ew_accumulate(const GemmArgs& g, const int (&lo)[P], const int (&hi)[P],
                                              const _Float16* A_m, float (&s)[P][8]) {
  constexpr int U = 8 / P;     // elements per column and round trip; the next ones are fetched meanwhile
  int e[P];
  uint32_t nx[P][U];
  bool more = false;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    e[p] = lo[p];
    more |= lo[p] < hi[p];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t w = g.ew_pairs[min(lo[p] + u, g.ew_last)];
      nx[p][u] = lo[p] + u < hi[p] ? w : 0u;
    }
  }
  while (more) {
    uint32_t pr[P][U];
    half8 a[P][U];
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        pr[p][u] = nx[p][u];
        a[p][u] = *(const half8*)(A_m + (size_t)(pr[p][u] >> 16) * g.lda);
      }
    more = false;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      e[p] += U;
      more |= e[p] < hi[p];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t w = g.ew_pairs[min(e[p] + u, g.ew_last)];
        nx[p][u] = e[p] + u < hi[p] ? w : 0u;
      }
    }
#pragma unroll
    for (int p = 0; p < P; ++p)
#pragma unroll
      for (int u = 0; u < U; ++u) {
        union { uint16_t b; _Float16 h; } cv;
        cv.b = (uint16_t)(pr[p][u] & 0xffffu);
        const float v = (float)cv.h;
#pragma unroll
        for (int q = 0; q < 8; ++q) s[p][q] = __builtin_fmaf(v, (float)a[p][u][q], s[p][q]);
      }
  }
}

__device__ __forceinline__ void store_row_chunk(const GemmArgs& g, _Float16* dst, int m, const float (&s)[8]) {
  half8 h;
#pragma unroll
  for (int q = 0; q < 8; ++q) h[q] = (_Float16)s[q];
  if (m + 8 <= g.M) __builtin_nontemporal_store(h, (half8*)dst);
  else for (int q = 0; m + q < g.M; ++q) dst[q] = h[q];
}

// A column the TW step dropped: nothing but its restored elements (usually none: +0).
__device__ __forceinline__ void ew_fill_column(const GemmArgs& g, int which) {
  const int col = g.zero_cols[which];
  const int lo = g.ew_ptr[col], hi = g.ew_ptr[col + 1];
  if (lo == hi) {                        // the usual case (uniform over the workgroup)
    zero_fill_column(g, which);
    return;
  }
  _Float16* row = g.C + (size_t)col * g.ldc;
  for (int m = threadIdx.x * 8; m < g.M; m += (int)blockDim.x * 8) {
    float s[1][8] = {{0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f}};
    const int lo1[1] = {lo}, hi1[1] = {hi};
    ew_accumulate<1>(g, lo1, hi1, g.A + m, s);
    store_row_chunk(g, row + m, m, s[0]);
  }
}

// SPLIT: K split across workgroups.  g.wg_split workgroups own the same (M-tile, N-tile) pair,
// each a contiguous share of the tile's stages; every one writes its fp32 partial tile to the
// workspace and takes a ticket at the pair's counter; the one that arrives last adds all partial
// tiles in split order (so the sum does not depend on who was last), runs the epilogue and puts
// the counter back to zero.  Nobody waits for anybody: a workgroup that is not last is done.
// LIDX: the kept-row list reaches the lanes through LDS (see fetch_rows) instead of scalar loads.
// MULTI: a workgroup computes g.tiles_per_wg jobs one after the other (job ids blockIdx.x,
// + gridDim.x, ..; gridDim.x is a multiple of 8, so every job keeps the workgroup's XCD).  The
// next job's first copies are issued as soon as every wave has read its staged chunks: the
// stores of the finished tile drain while the next one loads (the copies' waits count the
// stores as older operations, which only makes them wait longer).  Per job the kernel
// arguments are read again through a pointer the compiler cannot see through and the lane id is
// made opaque, so that nothing derived from them stays in registers across jobs.
template <int TM, int TN, int WAVES_M, int D, bool DENSE, int NWAVES = 4, int KSPLIT = 1, bool EW = false,
          bool SPLIT = false, bool LIDX = true, bool MULTI = false>
// (the TEW epilogue and the loop over jobs must not cost an instance a wave per SIMD: the second
// launch-bound asks the compiler to keep the register count within that occupancy)
__global__ __launch_bounds__(NWAVES * 64, (MULTI && TM * TN <= 64 * 128) ? 4 : ((EW || MULTI) && TM <= 128 && TN <= 128 && NWAVES == 4) ? 3 : 1)
void tw_gemm_km_dma_kernel(GemmArgs g_arg) {
  constexpr int NT = NWAVES * 64;          // threads of the workgroup
  constexpr int WPG = NWAVES / KSPLIT;     // waves per group
  constexpr int KSS = KS * KSPLIT;         // condensed rows per pipeline stage
  constexpr int WAVES_N = WPG / WAVES_M;
  constexpr int WM = TM / WAVES_M, WN = TN / WAVES_N;
  constexpr int MB = WM / 32, NB = WN / 32;
  static_assert(MB >= 1 && NB >= 1, "wave tile must hold a 32x32 block");
  constexpr int RBA = TM * 2, RBB = TN * 2;            // LDS row bytes
  constexpr int STAGE_A = KSS * RBA, STAGE_B = KSS * RBB, STAGE = STAGE_A + STAGE_B;
  static_assert(STAGE_A % 4096 == 0 && STAGE_B % 4096 == 0, "a stage is a whole number of 1 KiB copies per wave");
  static_assert(STAGE_A % (1024 * NWAVES) == 0 && STAGE_B % (1024 * NWAVES) == 0, "");
  constexpr int NIA = STAGE_A / (1024 * NWAVES), NIB = STAGE_B / (1024 * NWAVES);   // copy instructions per wave and stage
  constexpr int RPIA = 1024 / RBA, RPIB = 1024 / RBB;         // tile rows per copy instruction
  static_assert((RPIA == 2 || RPIA == 4 || RPIA == 8) && (NIA == 1 || NIA == 2 || NIA == 4), "");
  static_assert(D >= 3 && D <= 8, "stages in flight");
  constexpr int NPS = NIA + NIB;
  constexpr int CA = TM / 8;
  // epilogue row bytes: fp16, 66 dwords mod 64 banks = 2; with restored elements to add (EW) the
  // tile is staged in fp32 so that their products join the sum before the one rounding
  constexpr int CS = EW ? (TM + 4) * 4 : (TM + 4) * 2;
  static_assert(!(EW && DENSE), "");
  constexpr int PIPE_BYTES = D * STAGE, EPI_BYTES = (EW ? TN / 2 : TN) * CS;   // EW stages half a tile at a time
  constexpr int RED_BYTES = KSPLIT > 1 ? TM * TN * 4 : 0;      // partial accumulators of group 1
  static_assert(RED_BYTES <= PIPE_BYTES, "the reduction reuses the pipeline buffers");
  // kept-row lists travel through LDS as well: a ring of two chunks of 8 stages' indices behind
  // the pipeline buffers (the epilogue staging reuses the pipeline buffers only)
  constexpr int CH = 8 * KSS;                              // indices per chunk
  constexpr int NCI = CH * 4 / 1024;                       // 1 KiB copy instructions per chunk
  static_assert(NCI >= 1 && NCI <= NWAVES && CH * 4 % 1024 == 0, "");
  constexpr int MAIN_BYTES = PIPE_BYTES > EPI_BYTES ? PIPE_BYTES : EPI_BYTES;
  constexpr int IDX_OFF = (MAIN_BYTES + 1023) / 1024 * 1024;
  constexpr int LDS_BYTES = IDX_OFF + ((DENSE || !LIDX) ? 0 : 2 * CH * 4);
  __shared__ __attribute__((aligned(1024))) char lds[LDS_BYTES];

  static_assert(!SPLIT || (!DENSE && !EW && KSPLIT == 1), "the split across workgroups exists for plain TW");
  static_assert(!MULTI || (!DENSE && !EW && !SPLIT && KSPLIT == 1), "several jobs per workgroup exist for plain TW");
  auto job = [&](const GemmArgs& g, const int bid, const int tid) {
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int S = SPLIT ? g.wg_split : 1;
  const int n_gemm = g.n_mtiles * g.n_tiles * S;
  if (bid >= n_gemm) {
    if constexpr (EW) ew_fill_column(g, bid - n_gemm);
    else zero_fill_column(g, bid - n_gemm);
    return;
  }
  int mt, t;                             // t: launch position of the tile, then the tile itself
  int pair = 0, split = 0;
  if constexpr (SPLIT) {
    // the workgroups of a pair are neighbours in the XCD's contiguous range of logical ids:
    // they run on the same XCD at about the same time, and their partial tiles meet in its L2
    const int lid = g.xcd_map ? xcd_remap(bid, n_gemm) : bid;
    pair = lid / S;
    split = lid - pair * S;
    mt = pair / g.n_tiles;
    t = pair - mt * g.n_tiles;
  } else {
    tile_of_workgroup(g, bid, n_gemm, mt, t);
  }
  const int m0 = mt * TM;

  int kp0, ns32;                                       // ns32: stages of 32 rows
  if constexpr (DENSE) { kp0 = 0; ns32 = g.K / KS; }   // host guarantees K % (32 KSPLIT) == 0
  else {
    // equal tiles in column order (the usual per-tile pruning recipe): the record follows from
    // the launch position, which saves the first of the kernel's dependent round trips
    if (g.uniform_kp > 0) { kp0 = t * g.uniform_kp; ns32 = g.uniform_kp / KS; }
    else {
      const int4v rec = scalar_load4(g.tile_sched + 4 * t);
      t = rec[0]; kp0 = rec[1]; ns32 = rec[2] / KS;
    }
  }
  if constexpr (SPLIT) {                               // this workgroup's share of the stages
    const int first = ns32 * split / S, last = ns32 * (split + 1) / S;
    kp0 += first * KS;
    ns32 = last - first;
  }
  const int ns = (ns32 + KSPLIT - 1) / KSPLIT;         // pipeline stages of KSS rows
  const _Float16* Bt = DENSE ? g.vals + (size_t)t * TN : g.vals + (size_t)kp0 * TN;
  const int ldb = DENSE ? g.ldb : TN;

  // kept-column indices of the rows of C^T this thread will store (CTO_n)
  constexpr int ROWS_PER_PASS = NT / CA;
  constexpr int NPASS = TN / ROWS_PER_PASS;
  const int c = tid % CA, r0 = tid / CA;
  int cols[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i) {
    const int n = r0 + i * ROWS_PER_PASS;
    if constexpr (DENSE) { cols[i] = t * TN + n; if (cols[i] >= g.N) cols[i] = -1; }
    else cols[i] = g.col_idx[t * TN + n];
  }
  // ---- geometry of the asynchronous copies --------------------------------
  // Copy instruction j of this wave fills LDS bytes [(wave*NI + j) KiB, +1 KiB)
  // of the stage; lane l owns the 16 bytes at l*16, i.e. tile row
  // (wave*NI + j)*RPI + l*16/RB at physical byte (l*16) % RB, which holds the
  // logical bytes physical ^ swz_mask(row).
  const int lb = lane * 16;
  const int a_rloc = lb / RBA, b_rloc = lb / RBB;
  int a_el[NIA], b_el[NIB];
#pragma unroll
  for (int j = 0; j < NIA; ++j) {
    const int row = (wave * NIA + j) * RPIA + a_rloc;
    a_el[j] = ((lb % RBA) ^ swz_mask<RBA>(row)) / 2;
    if (m0 + a_el[j] >= g.M) a_el[j] = 0;   // past M: re-read chunk 0 (those lanes are never stored)
  }
#pragma unroll
  for (int j = 0; j < NIB; ++j) {
    const int row = (wave * NIB + j) * RPIB + b_rloc;
    b_el[j] = ((lb % RBB) ^ swz_mask<RBB>(row)) / 2;
    if constexpr (DENSE) { if (t * TN + b_el[j] >= g.N) b_el[j] = 0; }
  }
  // Addresses are a wave-uniform base plus an unsigned 32-bit byte offset per
  // lane (the host checks that A fits): one multiply-add per copy instruction.
  const char* Abase = (const char*)(g.A + m0);
  const char* Bbase = (const char*)Bt;
  const uint32_t lda2 = (uint32_t)g.lda * 2u, ldb2 = (uint32_t)ldb * 2u;
  uint32_t b_off[NIB];
#pragma unroll
  for (int j = 0; j < NIB; ++j)
    b_off[j] = (uint32_t)((wave * NIB + j) * RPIB + b_rloc) * ldb2 + (uint32_t)b_el[j] * 2u;

  // Row indices (Listing 1: CTO_k), two ways, both issued right after a stage barrier and
  // waited for with the first operand reads of that stage (one lgkmcnt(0) wait covers both).
  // LIDX: through LDS.  Chunk c of a tile's kept-row list (8 stages' worth) is copied into
  //   half c % 2 of a small ring by the same asynchronous copies as the operand tiles, so it
  //   is tracked by the same in-order counter and has landed, at no extra wait, long before
  //   its first stage is issued; every lane then picks the index of the row it copies with
  //   one ds_read_b32 per copy instruction.
  // else: scalar loads of the RPIA consecutive entries a copy instruction covers (wave-uniform
  //   address), the lane selects its own.  They miss the scalar cache on every stage and
  //   return out of order, so their whole round trip to L2 sits in the iteration.
  // Measured on the same box: with at most two 4-wave workgroups per CU (or the K-split
  // instances) the LDS route is 5-22 % faster, since nothing else on the CU hides that round
  // trip; with many workgroups per CU it is hidden anyway and the ring's extra barrier and
  // reads cost 3-5 %.  The host picks per launch.
  typedef int sidx_t __attribute__((ext_vector_type(RPIA)));
  struct Rows { std::conditional_t<LIDX, int, sidx_t> r[NIA]; };
  const uint32_t idx_lds0 = (uint32_t)(uintptr_t)LDS_PTR(char, lds) + IDX_OFF;
  auto issue_chunk = [&](int c) {        // waves 0 .. NCI-1: 1 KiB of the list each
    if constexpr (!DENSE && LIDX) {
      if (wave < NCI)
        __builtin_amdgcn_global_load_lds(GLOBAL_PTR((const char*)(g.row_idx + kp0) + ((size_t)c * CH * 4 + wave * 1024 + lb)),
                                         LDS_PTR(void, lds + IDX_OFF + (c & 1) * (CH * 4) + wave * 1024), 16, 0, 0);
    }
  };
  auto fetch_rows = [&](int s, Rows& dst) {      // rows of stage s; valid after the next lgkmcnt(0) wait
    if constexpr (!DENSE) {
#pragma unroll
      for (int j = 0; j < NIA; ++j) {
        if constexpr (LIDX) {
          const uint32_t pos = (uint32_t)(s * KSS + (wave * NIA + j) * RPIA + a_rloc) & (2 * CH - 1);
          asm volatile("ds_read_b32 %0, %1" : "=v"(dst.r[j]) : "v"(idx_lds0 + pos * 4));
        } else {
          const int* rp = g.row_idx + kp0 + s * KSS + (wave * NIA + j) * RPIA;
          if constexpr (RPIA == 2) asm volatile("s_load_dwordx2 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
          else if constexpr (RPIA == 4) asm volatile("s_load_dwordx4 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
          else asm volatile("s_load_dwordx8 %0, %1, 0x0" : "=s"(dst.r[j]) : "s"(rp));
        }
      }
    }
  };
  auto tie_rows = [&](Rows& x) {      // after a wait: no use of x may be moved above this point
    if constexpr (!DENSE && LIDX) {
      if constexpr (NIA == 1) asm volatile("" : "+v"(x.r[0]));
      else if constexpr (NIA == 2) asm volatile("" : "+v"(x.r[0]), "+v"(x.r[1]));
      else asm volatile("" : "+v"(x.r[0]), "+v"(x.r[1]), "+v"(x.r[2]), "+v"(x.r[3]));
    } else if constexpr (!DENSE) {
      if constexpr (NIA == 1) asm volatile("" : "+s"(x.r[0]));
      else if constexpr (NIA == 2) asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]));
      else asm volatile("" : "+s"(x.r[0]), "+s"(x.r[1]), "+s"(x.r[2]), "+s"(x.r[3]));
    }
  };
  auto issue = [&](int s, const Rows& rows) {     // copies of stage s; rows = its kept-row indices
    char* dstA = lds + (s % D) * STAGE;
    char* dstB = dstA + STAGE_A;
    const uint32_t bs = (uint32_t)s * (uint32_t)KSS * ldb2;
#pragma unroll
    for (int j = 0; j < NIB; ++j)
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Bbase + (bs + b_off[j])),
                                       LDS_PTR(void, dstB + (wave * NIB + j) * 1024), 16, 0, 0);
#pragma unroll
    for (int j = 0; j < NIA; ++j) {
      int row;
      if constexpr (DENSE) row = s * KSS + (wave * NIA + j) * RPIA + a_rloc;
      else if constexpr (LIDX) row = rows.r[j];
      else {
        row = rows.r[j][0];
#pragma unroll
        for (int q = 1; q < RPIA; ++q) row = (a_rloc == q) ? rows.r[j][q] : row;
      }
      __builtin_amdgcn_global_load_lds(GLOBAL_PTR(Abase + ((uint32_t)row * lda2 + (uint32_t)a_el[j] * 2u)),
                                       LDS_PTR(void, dstA + (wave * NIA + j) * 1024), 16, 0, 0);
    }
  };

  floatx16 acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int grp = wave / WPG, wl = wave % WPG;         // K-split group, wave inside the group
  const int wm = wl % WAVES_M, wn = wl / WAVES_M;
  // per-lane LDS byte address of each operand block at stage buffer 0, k-step 0
  const uint32_t lds0 = (uint32_t)(uintptr_t)LDS_PTR(char, lds);
  const int p = lane & 15, q = lane >> 4;
  const int frow = 8 * (q >> 1) + (p >> 2);
  uint32_t fa[MB], fb[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
    fa[i] = lds0 + grp * (KS * RBA) + swz<RBA>(frow, (wm * WM + i * 32 + 16 * (q & 1) + 4 * (p & 3)) * 2);
#pragma unroll
  for (int j = 0; j < NB; ++j)
    fb[j] = lds0 + STAGE_A + grp * (KS * RBB) + swz<RBB>(frow, (wn * WN + j * 32 + 16 * (q & 1) + 4 * (p & 3)) * 2);

  constexpr int NF = MB + NB;
  Frag f0[NF], f1[NF];       // operands of k-steps 0 and 1 of a stage
  auto read_step = [&](uint32_t boff, auto KK_, Frag* f) {
    constexpr int KK = decltype(KK_)::value;
#pragma unroll
    for (int i = 0; i < MB; ++i) {
      f[i].lo = tr_read<KK * RBA>(fa[i] + boff);
      f[i].hi = tr_read<(KK + 4) * RBA>(fa[i] + boff);
    }
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      f[MB + j].lo = tr_read<KK * RBB>(fb[j] + boff);
      f[MB + j].hi = tr_read<(KK + 4) * RBB>(fb[j] + boff);
    }
  };
  auto mfma_step = [&](const Frag* f) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(as_half8(f[i]), as_half8(f[MB + j]),
                                                           acc[i][j], 0, 0, 0);
  };
  using K0 = std::integral_constant<int, 0>;
  using K16 = std::integral_constant<int, 16>;

  Rows rows_cur, rows_next;
  if (ns > 0) {
    // (LIDX: the first two chunks of the kept-row list,) the indices of the first D stages in
    // one round trip, then the copies of D-1 stages
    issue_chunk(0);
    if (ns > 8) issue_chunk(1);
    Rows pro[D];
    if constexpr (!DENSE && LIDX) {
      wait_vm<0>();
      asm volatile("s_barrier" ::: "memory");
    }
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
    // own copies of stage s have landed: at most the copies of the newer stages remain
    // (a wave that also copies list chunks waits for one copy more at times: harmless)
    int newer = ns - 1 - s;
    if (newer > D - 2) newer = D - 2;
    wait_stage<NPS, D - 2>(newer);
    // everybody's copies of stage s have landed, everybody is done reading stage s-1
    asm volatile("s_barrier" ::: "memory");
    // rows of stage s+D: needed by the next iteration, so that the addresses of its copies
    // can be formed ahead of the wait that completes this fetch
    fetch_rows(s + D < ns ? s + D : ns - 1, rows_next);
    const uint32_t boff = (uint32_t)((s % D) * STAGE);
    read_step(boff, K0{}, f0);
    if (s > 0 && live_prev) mfma_step(f1);   // second k-step of the previous stage
    const bool live = s * KSPLIT + grp < ns32;   // false only for group 1 on an odd tail
    wait_lds<NF>(f0);                    // full wait: the index fetch above is in as well
    tie_rows(rows_next);
    // the copies of stage sn = s+D-1 go into the buffer of stage s-1, which every wave has
    // finished reading; when sn opens chunk c >= 1 of the list, chunk c+1 follows it into the
    // half of the ring whose last reader (stage 8c-1, two iterations ago) is behind this barrier
    const int sn = s + D - 1;
    if (sn < ns) {
      issue(sn, rows_cur);
      if ((sn & 7) == 0 && sn >= 8 && sn + 8 < ns) issue_chunk((sn >> 3) + 1);
    }
    read_step(boff, K16{}, f1);
    if (live) mfma_step(f0);
    live_prev = live;
    rows_cur = rows_next;
    wait_lds<NF>(f1);
  }
  if (ns > 0 && live_prev) mfma_step(f1);

  if constexpr (SPLIT) {
    if (S > 1) {
      __shared__ int ticket;
      constexpr int TILE = TM * TN;                       // floats per partial tile
      // partial tile as [wave][block][register][lane]: every store instruction of a wave is 256
      // contiguous bytes
      float* tile0 = g.ws_partials + (size_t)pair * S * TILE + wave * (MB * NB * 16 * 64) + lane;
      float* mine = tile0 + (size_t)split * TILE;
      // Partial tiles travel as device-scope relaxed atomic stores and loads: each access is
      // performed at the level that is coherent across the XCDs' L2 caches, so no cache-wide
      // write-back or invalidate is needed (a device-scope fence costs one of each per
      // workgroup and made the launch several times slower).  Order: own stores complete
      // (vmcnt), the workgroup's waves meet, then the ticket; the last arriver loads after it
      // has seen every ticket taken.
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r)
            __hip_atomic_store(mine + ((i * NB + j) * 16 + r) * 64, acc[i][j][r], __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
      wait_vm<0>();
      __syncthreads();
      if (tid == 0)
        ticket = __hip_atomic_fetch_add(g.ws_counters + pair, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __syncthreads();
      if (ticket != S - 1) return;                        // not the last one: done
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
      for (int q = 0; q < S; ++q) {                       // fixed order: the result does not depend on who is last
        const float* part = tile0 + (size_t)q * TILE;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r)
              acc[i][j][r] += __hip_atomic_load(part + ((i * NB + j) * 16 + r) * 64, __ATOMIC_RELAXED,
                                                __HIP_MEMORY_SCOPE_AGENT);
      }
      if (tid == 0)                                       // ready for the next launch
        __hip_atomic_store(g.ws_counters + pair, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }

  // ---- epilogue: fp32 -> fp16 (RNE), stage as [n][m], store rows of C^T ----
  const int m = m0 + c * 8;
  long long dst_off[NPASS];
#pragma unroll
  for (int i = 0; i < NPASS; ++i)
    dst_off[i] = (cols[i] < 0 || m >= g.M) ? -1 : (long long)cols[i] * g.ldc + m;
  __syncthreads();
  if constexpr (KSPLIT > 1) {
    // group 1 hands its fp32 partial sums to group 0: [wave in group][register][lane]
    float* red = (float*)lds + wl * (MB * NB * 16 * 64) + lane;
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
    __syncthreads();
  }
  if constexpr (EW) {
    // Restored elements of this thread's columns: [ew_lo, ew_hi) in the pair list.  Loaded here,
    // not at kernel start, where the dependent loads would hold up the first copies.
    int ew_lo[NPASS], ew_hi[NPASS];
#pragma unroll
    for (int i = 0; i < NPASS; ++i) {
      const int col = cols[i] < 0 ? 0 : cols[i];          // unconditional loads, selected afterwards
      const int p0 = g.ew_ptr[col], p1 = g.ew_ptr[col + 1];
      const bool live = dst_off[i] >= 0;
      ew_lo[i] = live ? p0 : 0;
      ew_hi[i] = live ? p1 : 0;
    }
    // fp32 staging, half of the tile's columns at a time (the staging area then fits the
    // pipeline buffers and does not cost occupancy); every thread finishes its
    // (column, 8 x m) pieces: restored elements added, one rounding, streaming store
    static_assert(NPASS % 2 == 0 && (TN / 2) % 32 == 0, "");
    constexpr int P = (NPASS / 2) % 2 == 0 ? 2 : 1;      // columns finished together
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      if (h) __syncthreads();
      if (grp == 0) {
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int j = 0; j < NB; ++j) {
            const int nblk = wn * WN + j * 32;                 // wave-uniform
            if (nblk / (TN / 2) != h) continue;
            const int n = nblk - h * (TN / 2) + (lane & 31);
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
              const int mm = wm * WM + i * 32 + 8 * rq + 4 * (lane >> 5);
              floatx4 v;
#pragma unroll
              for (int r = 0; r < 4; ++r) v[r] = acc[i][j][rq * 4 + r];
              *(floatx4*)(lds + n * CS + mm * 4) = v;
            }
          }
      }
      __syncthreads();
#pragma unroll
      for (int i = h * (NPASS / 2); i < (h + 1) * (NPASS / 2); i += P) {
        float sum[P][8];
        int lo2[P], hi2[P];
#pragma unroll
        for (int p = 0; p < P; ++p) {
          const int n = r0 + (i + p) * ROWS_PER_PASS - h * (TN / 2);
          const floatx4 lo4 = *(const floatx4*)(lds + n * CS + c * 32);
          const floatx4 hi4 = *(const floatx4*)(lds + n * CS + c * 32 + 16);
#pragma unroll
          for (int q = 0; q < 4; ++q) { sum[p][q] = lo4[q]; sum[p][4 + q] = hi4[q]; }
          lo2[p] = ew_lo[i + p];
          hi2[p] = ew_hi[i + p];
        }
        ew_accumulate<P>(g, lo2, hi2, g.A + (m < g.M ? m : 0), sum);
#pragma unroll
        for (int p = 0; p < P; ++p)
          if (dst_off[i + p] >= 0) store_row_chunk(g, g.C + dst_off[i + p], m, sum[p]);
      }
    }
  } else {
    if (grp == 0) {
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) {
          const int n = wn * WN + j * 32 + (lane & 31);
#pragma unroll
          for (int rq = 0; rq < 4; ++rq) {
            const int mm = wm * WM + i * 32 + 8 * rq + 4 * (lane >> 5);
            half4 v;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = (_Float16)acc[i][j][rq * 4 + r];
            *(half4*)(lds + n * CS + mm * 2) = v;
          }
        }
    }
    __syncthreads();
      // all staged chunks into registers first, then the stores back to back; C is
    // written once and not read again here: streaming (non-temporal) stores keep it
    // from lingering dirty in L2 until the end-of-kernel write-back
    union Chunk { uint2 h[2]; u32x4 v; };   // staging rows are 8-byte aligned only
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
  };   // job
  if constexpr (!MULTI) {
    job(g_arg, (int)blockIdx.x, (int)threadIdx.x);
  } else {
    typedef const GemmArgs __attribute__((address_space(4)))* karg_ptr;
    const int total_jobs = g_arg.n_mtiles * g_arg.n_tiles + g_arg.n_zero;
    for (int r = 0; r < g_arg.tiles_per_wg; ++r) {
      const int bid = (int)blockIdx.x + r * (int)gridDim.x;
      if (bid >= total_jobs) break;
      if (r) {                 // every wave has read its chunks of the staging area: it may be overwritten
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __syncthreads();
      }
      karg_ptr gp = (karg_ptr)__builtin_amdgcn_kernarg_segment_ptr();
      asm volatile("" : "+s"(gp));
      int tid = threadIdx.x;
      asm volatile("" : "+v"(tid));
      job(*(const GemmArgs*)gp, bid, tid);
    }
  }
}

template <int TM, int TN, int WAVES_M, int D, bool DENSE, int NWAVES = 4, int KSPLIT = 1, bool EW = false,
          bool SPLIT = false, bool LIDX = true, bool MULTI = false>
static hipError_t launch(const GemmArgs& g, hipStream_t stream) {
  const int jobs = g.n_mtiles * g.n_tiles * (SPLIT ? g.wg_split : 1) + g.n_zero;
  if (jobs <= 0) return hipSuccess;
  const int tpw = MULTI && g.tiles_per_wg > 1 ? g.tiles_per_wg : 1;
  const int grid = MULTI ? ((jobs + tpw - 1) / tpw + 7) / 8 * 8 : jobs;
  (void)hipGetLastError();   // an error left behind by an earlier call of this thread is not this launch's
  hipLaunchKernelGGL((tw_gemm_km_dma_kernel<TM, TN, WAVES_M, D, DENSE, NWAVES, KSPLIT, EW, SPLIT, LIDX, MULTI>), dim3(grid),
                     dim3(NWAVES * 64), 0, stream, g);
  return hipGetLastError();
}

// TEW instances: three stages in flight only.
static hipError_t dispatch_ew(int G, int tm, int variant, GemmArgs& g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (variant == DMA_KSPLIT2) {
    if (G == 128 && tm == 128) return launch<128, 128, 2, 3, false, 8, 2, true>(g, stream);
    if (G == 128 && tm == 64) return launch<64, 128, 1, 3, false, 8, 2, true>(g, stream);
    return hipErrorInvalidValue;
  }
  if (variant == DMA_WAVES8) {
    if (G == 128 && tm == 256) return launch<256, 128, 4, 3, false, 8, 1, true>(g, stream);
    return hipErrorInvalidValue;
  }
  if (G == 128 && tm == 64) return launch<64, 128, 1, 3, false, 4, 1, true>(g, stream);
  if (G == 128 && tm == 128) return launch<128, 128, 2, 3, false, 4, 1, true>(g, stream);
  if (G == 64 && tm == 128) return launch<128, 64, 2, 3, false, 4, 1, true>(g, stream);
  if (G == 64 && tm == 256) return launch<256, 64, 4, 3, false, 4, 1, true>(g, stream);
  return hipErrorInvalidValue;
}

// Both index routes of an instance (the dense baseline has no kept-row list: one instance).
template <int TM, int TN, int WAVES_M, int D, bool DENSE, int NWAVES = 4, bool MULTI_OK = false>
static hipError_t launch2(bool lidx, const GemmArgs& g, hipStream_t stream) {
  if constexpr (MULTI_OK && !DENSE) {
    if (g.tiles_per_wg > 1)
      return lidx ? launch<TM, TN, WAVES_M, D, false, NWAVES, 1, false, false, true, true>(g, stream)
                  : launch<TM, TN, WAVES_M, D, false, NWAVES, 1, false, false, false, true>(g, stream);
  }
  if constexpr (DENSE) return launch<TM, TN, WAVES_M, D, true, NWAVES>(g, stream);
  else if (lidx) return launch<TM, TN, WAVES_M, D, false, NWAVES, 1, false, false, true>(g, stream);
  else return launch<TM, TN, WAVES_M, D, false, NWAVES, 1, false, false, false>(g, stream);
}

template <bool DENSE>
static hipError_t dispatch(int G, int tm, int depth, int variant, bool lidx, GemmArgs& g, hipStream_t stream) {
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (variant == DMA_KSPLIT2) {   // two K-split groups of four waves (kept-row list through LDS)
    if (G == 128 && tm == 128 && depth == 3) return launch<128, 128, 2, 3, DENSE, 8, 2>(g, stream);
    if (G == 128 && tm == 64 && depth == 3) return launch<64, 128, 1, 3, DENSE, 8, 2>(g, stream);
    if (G == 128 && tm == 64 && depth == 4) return launch<64, 128, 1, 4, DENSE, 8, 2>(g, stream);
    if (G == 64 && tm == 128 && depth == 3) return launch<128, 64, 2, 3, DENSE, 8, 2>(g, stream);
    return hipErrorInvalidValue;
  }
  if (variant == DMA_WAVES8) {    // 512-thread workgroups: 64 x 32 (m x n) per wave
    if (G == 128 && tm == 128 && depth == 3) return launch2<128, 128, 2, 3, DENSE, 8>(lidx, g, stream);
    if (G == 128 && tm == 128 && depth == 4) return launch2<128, 128, 2, 4, DENSE, 8>(lidx, g, stream);
    if (G == 128 && tm == 256 && depth == 3) return launch2<256, 128, 4, 3, DENSE, 8>(lidx, g, stream);
    return hipErrorInvalidValue;
  }
#define TWG_CASE(TM_, TN_, WM_, D_) \
  if (G == TN_ && tm == TM_ && depth == D_) return launch2<TM_, TN_, WM_, D_, DENSE>(lidx, g, stream);
  if (G == 128 && tm == 64 && depth == 3) return launch2<64, 128, 1, 3, DENSE, 4, true>(lidx, g, stream);
  if (G == 128 && tm == 128 && depth == 3) return launch2<128, 128, 2, 3, DENSE, 4, true>(lidx, g, stream);
  TWG_CASE(256, 128, 2, 3)
  TWG_CASE(64, 128, 1, 4) TWG_CASE(128, 128, 2, 4) TWG_CASE(256, 128, 2, 4)
  TWG_CASE(128, 64, 2, 3) TWG_CASE(256, 64, 4, 3)
  TWG_CASE(128, 64, 2, 4) TWG_CASE(256, 64, 4, 4)
#undef TWG_CASE
  // deep pipelines for launches with about one workgroup per CU (kept-row list through LDS)
#define TWG_CASE(TM_, TN_, WM_, D_) \
  if (G == TN_ && tm == TM_ && depth == D_) return launch<TM_, TN_, WM_, D_, DENSE>(g, stream);
  TWG_CASE(64, 128, 1, 6) TWG_CASE(128, 128, 2, 6) TWG_CASE(128, 64, 2, 6)
  TWG_CASE(64, 128, 1, 8) TWG_CASE(128, 128, 2, 8) TWG_CASE(128, 64, 2, 8)
#undef TWG_CASE
  return hipErrorInvalidValue;
}

hipError_t launch_tw_km_dma(int G, int tm, int depth, int variant, bool lidx, GemmArgs g, hipStream_t stream) {
  return dispatch<false>(G, tm, depth, variant, lidx, g, stream);
}

static __global__ void zero_words(uint32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0u;
}
hipError_t launch_zero_words(uint32_t* p, int n, hipStream_t stream) {
  if (n <= 0) return hipSuccess;
  (void)hipGetLastError();
  hipLaunchKernelGGL(zero_words, dim3((n + 255) / 256), dim3(256), 0, stream, p, n);
  return hipGetLastError();
}

hipError_t launch_tw_km_dma_split(int G, int tm, GemmArgs g, hipStream_t stream) {
  if (g.wg_split < 1 || !g.ws_partials || !g.ws_counters) return hipErrorInvalidValue;
  g.n_mtiles = (g.M + tm - 1) / tm;
  if (G == 128 && tm == 128) return launch<128, 128, 2, 3, false, 4, 1, false, true>(g, stream);
  if (G == 128 && tm == 64) return launch<64, 128, 1, 3, false, 4, 1, false, true>(g, stream);
  if (G == 64 && tm == 128) return launch<128, 64, 2, 3, false, 4, 1, false, true>(g, stream);
  return hipErrorInvalidValue;
}
hipError_t launch_tew_km_dma(int G, int tm, int depth, int variant, bool, GemmArgs g, hipStream_t stream) {
  if (depth != 3) return hipErrorInvalidValue;
  return dispatch_ew(G, tm, variant, g, stream);
}
hipError_t launch_dense_km_dma(int tn, int tm, int depth, int variant, GemmArgs g, hipStream_t stream) {
  return dispatch<true>(tn, tm, depth, variant, true, g, stream);
}

}  // namespace twg
