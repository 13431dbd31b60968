// bf16 GEMMs C = A * B^T on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) with the epilogues of the PRISM polar iteration fused in (Table 1, rows
// "Newton-Schulz, U V^T": Gram/residual R = I - X^T X, Q = R/2 + alpha R^2, update X + X Q).
//
// Both operands are stored with K contiguous ([M][K] and [N][K]), which is the layout the
// instruction consumes: each lane feeds 8 consecutive k of one row.  The polar iteration is
// arranged so that every product has this form: the Gram matrix is taken from the [S][L] copy
// of the iterate, R and Q are symmetric, and the update reads the [L][S] copy.
//
// One workgroup = 4 wavefronts computes a T x T tile (T = 256 or 128) for one matrix; K runs in
// slabs of 32 moved straight from global memory into a four-deep LDS ring (no register staging;
// loads run three slabs ahead to cover the memory latency), in a swizzled layout that keeps the
// 16-byte fragment reads free of bank conflicts.  With a second A operand (the low half of a split-bf16 iterate) the K loop simply
// runs over both halves against the same B.
#include <type_traits>

#include "common.h"

namespace prism {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 32;
constexpr int NT = 256;

__device__ inline unsigned short f2bf(float x) {
  unsigned int u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even (inputs are finite here)
  return (unsigned short)(u >> 16);
}
__device__ inline float bf2f(unsigned short h) { return __uint_as_float(((unsigned int)h) << 16); }

typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

// LDS ring depth: loads run STAGES - 1 slabs ahead of the MFMAs.  T = 256: four (one workgroup per
// CU; a ring of five measured no faster).  T = 128: three, so that three workgroups fit a CU and
// overlap each other's prologue and epilogue (the 768-sized products are short: 24 slabs).
constexpr int stages_of(int T) { return T == 128 ? 3 : 4; }

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding)
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// DUAL (update GEMM with a split iterate): every K slab holds the high and the low half of A next
// to the one slab of B they both multiply, so B passes through the LDS once instead of twice.
template <int T, int EPI, bool SYM, bool DUAL>
__global__ __launch_bounds__(NT, T == 128 ? 3 : 1) void gemm_bf16_kernel(Bf16Desc g) {
  constexpr int STAGES = stages_of(T);
  constexpr int WT = T / 2;         // wave tile (2 x 2 waves)
  constexpr int NB = WT / 32;       // 32x32 blocks per wave and dimension
  constexpr int LDI = T / 64;       // direct-to-LDS load instructions per wave, operand and slab
  constexpr int OP_BYTES = T * 64;  // one operand slab in LDS: T rows x 32 bf16, unpadded
  constexpr int BUF_BYTES = 2 * OP_BYTES;
  // LDS: ring of STAGES buffers, each [A slab | B slab].  The LDS has 64 banks of 4 bytes and
  // serves a 16-byte read per lane in groups of 16 lanes, so 16 consecutive lanes must cover one
  // 256-byte bank line exactly once.  Four consecutive rows (64 bytes each) share a line; the
  // sixteen 16-byte chunks of line q sit at slot ((row & 3) * 4 + chunk) ^ (q & 15): the fragment
  // reads (16 consecutive rows, same chunk) then hit 16 different slots (measured: 116 B/clk/CU
  // against 82 for a swizzle over 128-byte lines and 63 unswizzled).
  extern __shared__ __align__(1024) unsigned char smem[];

  // SYM: A == B and the result is symmetric (Gram matrix, R^2): only the tiles on and above the
  // diagonal are computed, each off-diagonal tile is also written mirrored.
  const int tiles_m = g.M / T, tiles_n = g.N / T;
  const int per_mat = SYM ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  const int total = per_mat * g.batch;
  int wg = blockIdx.x;
  // Workgroup -> tile.  The hardware deals consecutive workgroups round-robin to the 8 XCDs, each
  // with its own L2.  g.xcd_private (set by the launcher for small matrices, or when all operands
  // of the launch fit the Infinity Cache together): every XCD gets a contiguous range of tiles, i.e. whole matrices, so
  // that the tiles sharing a panel share an L2 (without this the 768-sized Gram fetched 7x its
  // algorithmic bytes).  Otherwise workgroup i runs tile i: all XCDs sweep the same matrix and
  // share its panels through the Infinity Cache (private ranges measured 20 % slower at
  // 8 x 4096^2, where eight matrices at once overflow that cache).
  const bool xcd_private = g.xcd_private != 0;
  if ((total & 7) == 0 && xcd_private) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  const int b = wg / per_mat;
  int rem = wg - b * per_mat;
  int tm, tn;
  if (SYM) {       // row tm of the upper triangle holds tiles_m - tm tiles
    int left = rem;
    tm = 0;
    while (left >= tiles_m - tm) { left -= tiles_m - tm; ++tm; }
    tn = tm + left;
  } else if (g.xcd_blocks && !xcd_private) {
    // Every XCD sweeps blocks of 4 x 8 tiles of its own (its 32 CUs run one block at a time): the
    // tiles that meet in an L2 share 4 row panels and 8 column panels, where the plain order gives an
    // XCD two tile columns of every row, i.e. 16 row panels and 2 column panels per 32 tiles.
    const int x = rem & 7, q = rem >> 3;
    const int blk = (q >> 5) * 8 + x, w = q & 31, nbn = tiles_n >> 3;
    tm = (blk / nbn) * 4 + (w >> 3);
    tn = (blk % nbn) * 8 + (w & 7);
  } else {
    tm = rem / tiles_n;
    tn = rem - tm * tiles_n;
  }
  const int cb = g.ctrl_fixed ? 0 : b;   // split-K launches: every batch entry is a part of the same matrix
  if (g.ctrl && g.ctrl[cb].done) return;
  if (g.plain_filter && g.ctrl && ((g.ctrl[cb].plain != 0) != (g.plain_filter == 2))) return;
  const float alpha = g.ctrl ? g.ctrl[cb].alpha : 1.0f;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: LDS destinations stay scalar
  const int wm0 = (wave >> 1) * WT, wn0 = (wave & 1) * WT;
  const int m0 = tm * T, n0 = tn * T;
  const unsigned short* A1 = g.A + (long long)b * g.strideA + (long long)m0 * g.lda;
  const unsigned short* A2 = g.A2 ? g.A2 + (long long)b * g.strideA + (long long)m0 * g.lda : nullptr;
  const unsigned short* Bb = g.B + (long long)b * g.strideB + (long long)n0 * g.ldb;

  const int KT1 = g.K / BK;
  const int KT = (A2 && !DUAL) ? 2 * KT1 : KT1;

  // Global -> LDS without passing through registers (global_load_lds_dwordx4): one wave
  // instruction moves 64 lanes x 16 bytes into 1 KiB of consecutive LDS = 16 rows of a slab.
  // Lane l fills slot l & 15 of line l >> 4 of those 16 rows and fetches the chunk that belongs
  // there (the line index within the slab is (it * 4 + wave) * 4 + (l >> 4)).
  const int lq = lane >> 4, lu = (lane & 15) ^ ((wave * 4 + lq) & 15);
  unsigned aoff[LDI], boff[LDI];
#pragma unroll
  for (int it = 0; it < LDI; ++it) {
    const int row = (it * 4 + wave) * 16 + 4 * lq + (lu >> 2);
    aoff[it] = (unsigned)(row * g.lda + (lu & 3) * 8) * 2u;
    boff[it] = (unsigned)(row * g.ldb + (lu & 3) * 8) * 2u;
  }
  // one load instruction pair index u in [0, 2*LDI): even = A, odd = B
  auto issue_load = [&](int kt, int slot, int u) {
    const int it = u >> 1;
    const int kk0 = ((kt < KT1) ? kt : kt - KT1) * BK;
    unsigned char* dst = smem + slot * BUF_BYTES + wave * 1024 + it * 4096;
    if (u & 1) {
      __builtin_amdgcn_global_load_lds((gptr_t)((const char*)(Bb + kk0) + boff[it]), (lptr_t)(dst + OP_BYTES), 16, 0, 0);
    } else {
      const unsigned short* Ap = ((kt < KT1) ? A1 : A2) + kk0;
      __builtin_amdgcn_global_load_lds((gptr_t)((const char*)Ap + aoff[it]), (lptr_t)dst, 16, 0, 0);
    }
  };
  auto issue_loads = [&](int kt, int slot) {
#pragma unroll
    for (int u = 0; u < 2 * LDI; ++u) issue_load(kt, slot, u);
  };

  f32x16 acc[NB][NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragment addresses: row r = tile row, chunk cc = 2 * kk + (lane >> 5)
  const int lr = lane & 31, lh = lane >> 5;
  // (row block f starts 32 rows = 8 lines further on, which flips bit 3 of the line index)
  const unsigned char* Afr = smem + wm0 * 64 + (lr >> 2) * 256;
  const unsigned char* Bfr = smem + OP_BYTES + wn0 * 64 + (lr >> 2) * 256;
  int koff[2][2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int par = 0; par < 2; ++par)
      koff[kk][par] = ((((lr & 3) << 2) + kk * 2 + lh) ^ ((lr >> 2) + 8 * par)) << 4;
  bf16x8 fa[2][NB], fb[2][NB];
  // fragment f in [0, 2*NB) of sub-step kk: first the NB row blocks of A, then the NB of B
  auto load_frag = [&](int slot, int kk, int f) {
    const int o = slot * BUF_BYTES;
    if (f < NB) fa[kk][f] = *(const bf16x8*)(Afr + o + koff[kk][f & 1] + f * 2048);
    else fb[kk][f - NB] = *(const bf16x8*)(Bfr + o + koff[kk][(f - NB) & 1] + (f - NB) * 2048);
  };
  auto load_frags = [&](int slot, int kk) {
#pragma unroll
    for (int f = 0; f < 2 * NB; ++f) load_frag(slot, kk, f);
  };
  auto mfma_one = [&](int set, int m) {
    const int i = m / NB, j = m % NB;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
  };
  auto mfma_block = [&](int set) {
#pragma unroll
    for (int i = 0; i < NB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
  };
  // wait until the loads of slab `kt` have landed: up to STAGES - 2 younger slabs may still be in flight
  auto wait_slab = [&](int kt) {
    const int younger = KT - 1 - kt;
    if (younger >= 3 && STAGES >= 5) wait_vmcnt<6 * LDI>();
    else if (younger >= 2 && STAGES >= 4) wait_vmcnt<4 * LDI>();
    else if (younger >= 1) wait_vmcnt<2 * LDI>();
    else wait_vmcnt<0>();
  };

  // Workgroup barrier without the release fence of __syncthreads(): that fence would wait for
  // ALL outstanding loads (vmcnt(0)) and serialise the ring.  What must be complete is awaited
  // explicitly: this wave's share of the slab about to be consumed (wait_slab) and its own
  // fragment reads of the ring slot that is recycled after the barrier (lgkmcnt(0)).
  auto ring_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };

  if constexpr (DUAL) {
    // Ring of three buffers [A_hi slab | A_lo slab | B slab].  One slab = four sub-steps:
    //   0: hi(k 0..15) x B(k 0..15)   1: lo(k 0..15) x B(k 0..15)
    //   2: hi(k 16..31) x B(16..31)   3: lo(k 16..31) x B(16..31)
    // The fragments of a sub-step are read during the one before it; the single barrier of the
    // slab sits after sub-step 2 (all its fragments are in registers then), and sub-step 3
    // requests slab kt+3 into the buffer the barrier has just released.
    constexpr int DBUF = 3 * OP_BYTES;
    constexpr int NL = 3 * LDI;                 // load instructions per wave and slab
    constexpr int NM = NB * NB;                 // MFMAs per sub-step
    auto d_issue = [&](int kt_, int slot, int u) {
      const int op = u % 3, it = u / 3;
      const int kk0 = kt_ * BK;
      unsigned char* dst = smem + slot * DBUF + op * OP_BYTES + wave * 1024 + it * 4096;
      if (op == 2) __builtin_amdgcn_global_load_lds((gptr_t)((const char*)(Bb + kk0) + boff[it]), (lptr_t)dst, 16, 0, 0);
      else __builtin_amdgcn_global_load_lds((gptr_t)((const char*)((op ? A2 : A1) + kk0) + aoff[it]), (lptr_t)dst, 16, 0, 0);
    };
    const unsigned char* Ahi = smem + wm0 * 64 + (lr >> 2) * 256;
    const unsigned char* Alo = Ahi + OP_BYTES;
    const unsigned char* Bf = smem + 2 * OP_BYTES + wn0 * 64 + (lr >> 2) * 256;
    bf16x8 fA[NB], fB[NB], fb2[2][NB];          // fA: high half, fB: low half, fb2[kk]: B
    auto rd_hi = [&](int slot, int kk, int f) { fA[f] = *(const bf16x8*)(Ahi + slot * DBUF + koff[kk][f & 1] + f * 2048); };
    auto rd_lo = [&](int slot, int kk, int f) { fB[f] = *(const bf16x8*)(Alo + slot * DBUF + koff[kk][f & 1] + f * 2048); };
    auto rd_b = [&](int slot, int kk, int f) { fb2[kk][f] = *(const bf16x8*)(Bf + slot * DBUF + koff[kk][f & 1] + f * 2048); };
    auto mm_hi = [&](int kk, int m) { acc[m / NB][m % NB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fA[m / NB], fb2[kk][m % NB], acc[m / NB][m % NB], 0, 0, 0); };
    auto mm_lo = [&](int kk, int m) { acc[m / NB][m % NB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fB[m / NB], fb2[kk][m % NB], acc[m / NB][m % NB], 0, 0, 0); };
    // prologue: slabs 0, 1, 2
#pragma unroll
    for (int s0 = 0; s0 < 3; ++s0) {
#pragma unroll
      for (int u = 0; u < NL; ++u) d_issue(s0, s0, u);
    }
    wait_vmcnt<2 * NL>();
    ring_barrier();
#pragma unroll
    for (int f = 0; f < NB; ++f) { rd_hi(0, 0, f); rd_b(0, 0, f); }
    // MORE: slab kt+3 exists and is requested; NEXT: slab kt+1 exists; AHEAD: slab kt+2 exists
    // (its loads may still be in flight at the barrier)
    auto slab = [&](int kt, int slot, int nslot, auto more_c, auto next_c, auto ahead_c) {
      constexpr bool MORE = decltype(more_c)::value, NEXT = decltype(next_c)::value, AHEAD = decltype(ahead_c)::value;
      // sub-step 0: hi x B (first half of the slab); read lo (first half)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        if (m < NB) rd_lo(slot, 0, m);
        mm_hi(0, m);
        if ((m & 1) == 1) __builtin_amdgcn_sched_barrier(0);
      }
      // sub-step 1: lo x B (first half); read hi and B (second half)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        if (m < 2 * NB) { if (m & 1) rd_b(slot, 1, m >> 1); else rd_hi(slot, 1, m >> 1); }
        mm_lo(0, m);
        if ((m & 1) == 1) __builtin_amdgcn_sched_barrier(0);
      }
      // sub-step 2: hi x B (second half); read lo (second half)
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        if (m < NB) rd_lo(slot, 1, m);
        mm_hi(1, m);
        if ((m & 1) == 1) __builtin_amdgcn_sched_barrier(0);
      }
      // slab kt+1 must have landed; slab kt+2 (requested one slab ago) may still be in flight
      if (AHEAD) wait_vmcnt<NL>(); else wait_vmcnt<0>();
      ring_barrier();
      // sub-step 3: lo x B (second half); request slab kt+3; read hi and B of slab kt+1
#pragma unroll
      for (int m = 0; m < NM; ++m) {
        if (NEXT && m < 2 * NB) { if (m & 1) rd_b(nslot, 0, m >> 1); else rd_hi(nslot, 0, m >> 1); }
        if (MORE && m < NL) d_issue(kt + 3, slot, m);
        mm_lo(1, m);
        if ((m & 1) == 1) __builtin_amdgcn_sched_barrier(0);
      }
      if (MORE && NL > NM) {
#pragma unroll
        for (int u = NM; u < NL; ++u) d_issue(kt + 3, slot, u);
      }
    };
    typedef std::integral_constant<bool, true> yes;
    typedef std::integral_constant<bool, false> no;
    int slot = 0, kt = 0;
    for (; kt + 3 < KT; ++kt) {
      const int nslot = slot == 2 ? 0 : slot + 1;
      slab(kt, slot, nslot, yes(), yes(), yes());
      slot = nslot;
    }
    {  // the last three slabs (the launcher guarantees KT >= 3): nothing left to request
      const int s1 = slot == 2 ? 0 : slot + 1, s2 = s1 == 2 ? 0 : s1 + 1;
      slab(kt, slot, s1, no(), yes(), yes());
      slab(kt + 1, s1, s2, no(), yes(), no());
      slab(kt + 2, s2, slot, no(), no(), no());
    }
  } else {
  // Main loop.  Slab kt+STAGES-1 is requested at the top of slab kt (its ring slot was released
  // by the barrier that closed slab kt-1); the fragments of the second half of slab kt are read
  // while its first half computes, and after the single barrier of the slab the first fragments
  // of slab kt+1 are read while the second half computes.
  static_assert(BK == 32 && STAGES >= 3 && STAGES <= 5, "pipeline written for two sub-steps per slab");
#pragma unroll
  for (int s0 = 0; s0 < STAGES - 1; ++s0)
    if (s0 < KT) issue_loads(s0, s0);
  wait_slab(0);
  ring_barrier();
  load_frags(0, 0);
  int kt = 0, slot = 0;                 // slot = kt mod STAGES
  const int KT_main = KT - (STAGES - 1);
  constexpr int NF = 2 * NB;            // fragment reads per sub-step = interleave steps
  constexpr int MPS = NB * NB / NF;     // MFMAs per interleave step
  static_assert(2 * LDI == NF, "one load instruction per interleave step");
  for (; kt < KT_main; ++kt) {          // steady state: no conditions inside
    const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
    const int lslot = slot == 0 ? STAGES - 1 : slot - 1;   // slot of slab kt-1 = slot of slab kt+STAGES-1
    // sub-step 0 of slab kt: request slab kt+STAGES-1 and read the fragments of sub-step 1, one of
    // each between MFMAs so that they issue in the shadow of the matrix pipe
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      issue_load(kt + STAGES - 1, lslot, u);
      load_frag(slot, 1, u);
#pragma unroll
      for (int v = 0; v < MPS; ++v) mfma_one(0, u * MPS + v);
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<2 * (STAGES - 2) * LDI>();   // slab kt+1 has landed; the younger ones may be in flight
    ring_barrier();
#pragma unroll
    for (int u = 0; u < NF; ++u) {
      load_frag(nslot, 0, u);
#pragma unroll
      for (int v = 0; v < MPS; ++v) mfma_one(1, u * MPS + v);
      __builtin_amdgcn_sched_barrier(0);
    }
    slot = nslot;
  }
  for (; kt < KT; ++kt) {               // drain: nothing left to request
    const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
    load_frags(slot, 1);
    mfma_block(0);
    if (kt + 1 < KT) {
      wait_slab(kt + 1);
    }
    ring_barrier();
    if (kt + 1 < KT) load_frags(nslot, 0);
    mfma_block(1);
    slot = nslot;
  }

  }

  // epilogue: register r of lane l holds row (r/4)*8 + (l/32)*4 + r%4, column l%32 of a block
  float part = 0.0f;
  const float coef = g.coef_is_alpha ? alpha : 1.0f;
  const int rbase = (lane >> 5) * 4;
  if constexpr (SYM && (EPI == BEPI_GRAM || EPI == BEPI_POLYQ)) {
    // Each wave passes its tile through its own LDS strip of 32 rows (the ring is free after the
    // last barrier): row-wise for the tile itself, column-wise for its mirror image, so that both
    // are written with 16- and 32-byte vectors on contiguous runs.
    constexpr int SW = WT + 4;
    float* strip = (float*)smem + wave * 32 * SW;
    constexpr int LPR = WT / 8, RPI = 64 / LPR;
    const int rr = lane / LPR, cc = (lane % LPR) * 8;
    const int cq = lane >> 2, rq = lane & 3;
    const bool mirror = tm != tn;
    const long long b32 = (long long)b * g.strideC32, bb = (long long)b * g.strideCb;
    // R^2 epilogue: the entries of R of a row block are requested before its accumulators go
    // through LDS, those of the next block while the mirror image of this one is written.
    constexpr int ITS = 32 / RPI;
    f32x4 rin0[EPI == BEPI_POLYQ ? ITS : 1], rin1[EPI == BEPI_POLYQ ? ITS : 1];
    const bool lean = g.C32 == nullptr;   // GRAM: bf16 copy and diagonal only; POLYQ: R comes in bf16
    auto fetch_r = [&](int i) {
      if constexpr (EPI == BEPI_POLYQ) {
#pragma unroll
        for (int it = 0; it < ITS; ++it) {
          const int m = m0 + wm0 + i * 32 + it * RPI + rr, n = n0 + wn0 + cc;
          if (lean) {
            const u32x4 w = *(const u32x4*)(g.Cin16 + bb + (long long)m * g.ldcb + n);
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              rin0[it][2 * e] = __uint_as_float(w[e] << 16);
              rin0[it][2 * e + 1] = __uint_as_float(w[e] & 0xFFFF0000u);
              rin1[it][2 * e] = __uint_as_float(w[2 + e] << 16);
              rin1[it][2 * e + 1] = __uint_as_float(w[2 + e] & 0xFFFF0000u);
            }
          } else {
            const long long o32 = b32 + (long long)m * g.ldc32 + n;
            rin0[it] = *(const f32x4*)(g.C32 + o32);
            rin1[it] = *(const f32x4*)(g.C32 + o32 + 4);
          }
        }
      }
    };
    fetch_r(0);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          strip[((r >> 2) * 8 + rbase + (r & 3)) * SW + j * 32 + lr] = acc[i][j][r];
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const int row = it * RPI + rr;
        float* sp = strip + row * SW + cc;
        f32x4 v0 = *(const f32x4*)sp, v1 = *(const f32x4*)(sp + 4);
        const int m = m0 + wm0 + i * 32 + row, n = n0 + wn0 + cc;
        const long long o32 = b32 + (long long)m * g.ldc32 + n;
        if (EPI == BEPI_GRAM) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v0[e] = (m < g.n_true && n + e < g.n_true) ? ((m == n + e ? 1.0f : 0.0f) - v0[e]) : 0.0f;
            v1[e] = (m < g.n_true && n + 4 + e < g.n_true) ? ((m == n + 4 + e ? 1.0f : 0.0f) - v1[e]) : 0.0f;
            part += v0[e] * v0[e] + v1[e] * v1[e];
          }
          if (!lean) {
            *(f32x4*)(g.C32 + o32) = v0;
            *(f32x4*)(g.C32 + o32 + 4) = v1;
          } else if (tm == tn && m >= n && m < n + 8) {   // the diagonal entry of this row lies in these 8 columns
            g.diag[(long long)b * g.strideDiag + m] = (m - n < 4) ? v0[(m - n) & 3] : v1[(m - n) & 3];
          }
        } else {
          const f32x4 r0 = rin0[EPI == BEPI_POLYQ ? it : 0], r1 = rin1[EPI == BEPI_POLYQ ? it : 0];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v0[e] = g.c1 * r0[e] + alpha * v0[e];
            v1[e] = g.c1 * r1[e] + alpha * v1[e];
          }
        }
        u32x4 pk;
        pk[0] = (unsigned)f2bf(v0[0]) | ((unsigned)f2bf(v0[1]) << 16);
        pk[1] = (unsigned)f2bf(v0[2]) | ((unsigned)f2bf(v0[3]) << 16);
        pk[2] = (unsigned)f2bf(v1[0]) | ((unsigned)f2bf(v1[1]) << 16);
        pk[3] = (unsigned)f2bf(v1[2]) | ((unsigned)f2bf(v1[3]) << 16);
        *(u32x4*)(g.Cb + bb + (long long)m * g.ldcb + n) = pk;
        if (mirror) {
          *(f32x4*)sp = v0;
          *(f32x4*)(sp + 4) = v1;
        }
      }
      if (i + 1 < NB) fetch_r(i + 1);
      if (mirror) {
        // column-wise: 8 consecutive rows of one column = 8 consecutive entries of a mirrored row
#pragma unroll
        for (int it = 0; it < WT / 16; ++it) {
          const int col = it * 16 + cq;
          f32x4 t0, t1;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            t0[e] = strip[(rq * 8 + e) * SW + col];
            t1[e] = strip[(rq * 8 + 4 + e) * SW + col];
          }
          const int mr = n0 + wn0 + col, nr = m0 + wm0 + i * 32 + rq * 8;   // mirrored position
          if (EPI == BEPI_GRAM && !lean) {
            *(f32x4*)(g.C32 + b32 + (long long)mr * g.ldc32 + nr) = t0;
            *(f32x4*)(g.C32 + b32 + (long long)mr * g.ldc32 + nr + 4) = t1;
          }
          u32x4 pk;
          pk[0] = (unsigned)f2bf(t0[0]) | ((unsigned)f2bf(t0[1]) << 16);
          pk[1] = (unsigned)f2bf(t0[2]) | ((unsigned)f2bf(t0[3]) << 16);
          pk[2] = (unsigned)f2bf(t1[0]) | ((unsigned)f2bf(t1[1]) << 16);
          pk[3] = (unsigned)f2bf(t1[2]) | ((unsigned)f2bf(t1[3]) << 16);
          *(u32x4*)(g.Cb + bb + (long long)mr * g.ldcb + nr) = pk;
        }
      }
    }
    if (mirror) part *= 2.0f;
  } else if constexpr (EPI == BEPI_APPLY) {
    // The new iterate goes out in two layouts ([L][S] for the next update, [S][L] for the next
    // Gram product).  Each wave passes its tile through its own LDS strip of 32 rows so that
    // every global access is a 16-byte vector on a contiguous run: row-wise for X (read) and
    // Xa' (write), column-wise for the transposed Xg'.  The LDS ring is free here: no wave reads
    // fragments after the last barrier of the main loop.
    constexpr int SW = WT + 4;                       // strip row stride in floats (16-byte aligned)
    float* strip = (float*)smem + wave * 32 * SW;
    constexpr int LPR = WT / 8, RPI = 64 / LPR;      // lanes per row, rows per instruction
    const int rr = lane / LPR, cc = (lane % LPR) * 8;
    const int cq = lane >> 2, rq = lane & 3;
    const long long base = (long long)b * g.strideCb;
    // The old iterate of row block i + 1 is requested while block i is worked on (and that of
    // block 0 before the accumulators go to LDS): its memory latency is paid once per tile
    // instead of once per block.
    constexpr int ITS = 32 / RPI;
    u32x4 xh[2][ITS], xl[2][ITS];
    const bool has_lo = g.Xlo != nullptr;
    auto fetch_x = [&](int i, int set) {
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const long long o = base + (long long)(m0 + wm0 + i * 32 + it * RPI + rr) * g.ldcb + n0 + wn0 + cc;
        xh[set][it] = *(const u32x4*)(g.Xhi + o);
        xl[set][it] = (u32x4){0u, 0u, 0u, 0u};
        if (has_lo) xl[set][it] = *(const u32x4*)(g.Xlo + o);
      }
    };
    fetch_x(0, 0);
#pragma unroll
    for (int i = 0; i < NB; ++i) {
      if (i + 1 < NB) fetch_x(i + 1, (i + 1) & 1);
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          strip[((r >> 2) * 8 + rbase + (r & 3)) * SW + j * 32 + lr] = acc[i][j][r];
      // row-wise: x' = x_hi + x_lo + coef * acc, split again, keep the high half for the transpose
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const int row = it * RPI + rr;
        float* sp = strip + row * SW + cc;
        const f32x4 a0 = *(const f32x4*)sp, a1 = *(const f32x4*)(sp + 4);
        const long long o = base + (long long)(m0 + wm0 + i * 32 + row) * g.ldcb + n0 + wn0 + cc;
        const u32x4 hi = xh[i & 1][it];
        const u32x4 lo = xl[i & 1][it];
        u32x4 nh, nl;
        f32x4 k0, k1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // two bf16 per 32-bit word: even element in the low half
          const float x0 = __uint_as_float(hi[e] << 16) + __uint_as_float(lo[e] << 16) + coef * (e < 2 ? a0[2 * e] : a1[2 * e - 4]);
          const float x1 = __uint_as_float(hi[e] & 0xFFFF0000u) + __uint_as_float(lo[e] & 0xFFFF0000u) + coef * (e < 2 ? a0[2 * e + 1] : a1[2 * e - 3]);
          const unsigned h0 = f2bf(x0), h1 = f2bf(x1);
          nh[e] = h0 | (h1 << 16);
          nl[e] = (unsigned)f2bf(x0 - bf2f((unsigned short)h0)) | ((unsigned)f2bf(x1 - bf2f((unsigned short)h1)) << 16);
          if (e < 2) { k0[2 * e] = bf2f((unsigned short)h0); k0[2 * e + 1] = bf2f((unsigned short)h1); }
          else { k1[2 * e - 4] = bf2f((unsigned short)h0); k1[2 * e - 3] = bf2f((unsigned short)h1); }
        }
        *(u32x4*)(g.Cb + o) = nh;
        if (g.Cb2) *(u32x4*)(g.Cb2 + o) = nl;
        *(f32x4*)sp = k0;
        *(f32x4*)(sp + 4) = k1;
      }
      // column-wise: 8 consecutive rows of one column = 16 bytes of a row of Xg'
#pragma unroll
      for (int it = 0; it < WT / 16; ++it) {
        const int col = it * 16 + cq;
        u32x4 tv;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const unsigned h0 = f2bf(strip[(rq * 8 + 2 * e) * SW + col]);
          const unsigned h1 = f2bf(strip[(rq * 8 + 2 * e + 1) * SW + col]);
          tv[e] = h0 | (h1 << 16);
        }
        *(u32x4*)(g.Ct + (long long)b * g.strideCt + (long long)(n0 + wn0 + col) * g.ldct + m0 + wm0 + i * 32 + rq * 8) = tv;
      }
    }
  } else {
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int gn = n0 + wn0 + j * 32 + lr;
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int gm = m0 + wm0 + i * 32 + rg * 8 + rbase;  // first of 4 consecutive rows
        if (EPI == BEPI_STORE) {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            g.C32[(long long)b * g.strideC32 + (long long)(gm + e) * g.ldc32 + gn] = acc[i][j][rg * 4 + e];
        } else if (EPI == BEPI_GRAM) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int m = gm + e;
            const float r = (m < g.n_true && gn < g.n_true) ? ((m == gn ? 1.0f : 0.0f) - acc[i][j][rg * 4 + e]) : 0.0f;
            g.C32[(long long)b * g.strideC32 + (long long)m * g.ldc32 + gn] = r;
            g.Cb[(long long)b * g.strideCb + (long long)m * g.ldcb + gn] = f2bf(r);
            part += r * r;
          }
        } else if (EPI == BEPI_POLYQ) {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int m = gm + e;
            const float rin = g.C32[(long long)b * g.strideC32 + (long long)m * g.ldc32 + gn];
            g.Cb[(long long)b * g.strideCb + (long long)m * g.ldcb + gn] = f2bf(g.c1 * rin + alpha * acc[i][j][rg * 4 + e]);
          }
        }
      }
    }
  }
  if (EPI == BEPI_GRAM) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
    float* red = (float*)smem;          // the epilogue strips are dead once every wave is here
    __syncthreads();
    if (lane == 0) red[wave] = part;
    __syncthreads();
    if (t == 0) g.rho_part[(long long)b * per_mat + rem] = red[0] + red[1] + red[2] + red[3];
  }
}

template <int T, int EPI, bool SYM, bool DUAL = false>
int launch_te(const Bf16Desc& g, hipStream_t s) {
  const int tm = g.M / T, tn = g.N / T;
  const int total = (SYM ? tm * (tm + 1) / 2 : tm * tn) * g.batch;
  // ring of STAGES x (A slab + B slab), or of 3 x (A_hi + A_lo + B)
  const size_t lds = DUAL ? (size_t)3 * 3 * T * 64 : (size_t)stages_of(T) * 2 * T * 64;
  const int rc = allow_dynamic_lds((const void*)gemm_bf16_kernel<T, EPI, SYM, DUAL>, (int)lds);
  if (rc != PRISM_OK) return rc;
  hipLaunchKernelGGL((gemm_bf16_kernel<T, EPI, SYM, DUAL>), dim3(total), dim3(NT), lds, s, g);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

template <int T>
int launch_t(const Bf16Desc& g, hipStream_t s) {
  if (g.M % T || g.N % T || g.K % BK || g.lda % 8 || g.ldb % 8) return PRISM_EINVAL;
  if ((g.M / T) * (g.N / T) * g.batch <= 0) return PRISM_EINVAL;
  if (g.sym && (g.M != g.N || g.A != g.B || g.A2)) return PRISM_EINVAL;
  if ((g.epi == BEPI_GRAM || g.epi == BEPI_POLYQ || g.epi == BEPI_STORE) && !g.C32) {
    // without the fp32 matrix: symmetric GRAM with a diagonal array, symmetric POLYQ with R in bf16
    if (!g.sym || (g.epi == BEPI_GRAM && !g.diag) || (g.epi == BEPI_POLYQ && !g.Cin16) || g.epi == BEPI_STORE) return PRISM_EINVAL;
  }
  switch (g.epi) {
    case BEPI_STORE: return launch_te<T, BEPI_STORE, false>(g, s);
    case BEPI_GRAM: return g.sym ? launch_te<T, BEPI_GRAM, true>(g, s) : launch_te<T, BEPI_GRAM, false>(g, s);
    case BEPI_POLYQ: return g.sym ? launch_te<T, BEPI_POLYQ, true>(g, s) : launch_te<T, BEPI_POLYQ, false>(g, s);
    case BEPI_APPLY:
      return (g.A2 && g.K >= 3 * BK && !g.no_dual) ? launch_te<T, BEPI_APPLY, false, true>(g, s) : launch_te<T, BEPI_APPLY, false>(g, s);
  }
  return PRISM_EINVAL;
}

}  // namespace

int launch_gemm_bf16(const Bf16Desc& g0, int tile, hipStream_t s) {
  Bf16Desc g = g0;
  // bytes of all operands of the launch against half the 256 MiB Infinity Cache
  const double operand_bytes = 2.0 * g.batch * ((double)g.M * g.K * (g.A2 ? 2 : 1) + (g.A == g.B ? 0.0 : (double)g.N * g.K));
  const long long tm = g.M / tile, tn = g.N / tile;
  const long long per_mat = g.sym ? tm * (tm + 1) / 2 : tm * tn;
  g.xcd_private = per_mat <= 64 || operand_bytes <= 128.0 * 1024 * 1024;
  static const int no_blocks = ab_switch("PRISM_BF16_NO_XCD_BLOCKS");
  g.xcd_blocks = !no_blocks && !g.sym && per_mat % 256 == 0 && tm % 4 == 0 && tn % 8 == 0;
  if (tile == 256) return launch_t<256>(g, s);
  if (tile == 128) return launch_t<128>(g, s);
  return PRISM_EINVAL;
}

}  // namespace prism
