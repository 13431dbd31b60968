// bf16 GEMMs C = A * B^T on the CDNA4 matrix cores (v_mfma_f32_32x32x16_bf16, fp32
// accumulate) with the epilogues of the PRISM polar iteration fused in (Table 1, rows
// "Newton-Schulz, U V^T": Gram/residual R = I - X^T X, Q = R/2 + alpha R^2, update X + X Q).
//
// The instruction consumes operands with K contiguous (each lane feeds 8 consecutive k of one row).
// An operand may be stored that way ([M][K] / [N][K]) or with K as the slow index ([K][M] / [K][N]);
// the latter is read from LDS with transposing reads.  The polar iteration keeps one copy of the
// iterate, X[L][S]: the Gram product X^T X reads it as [K][M] for both operands, the update X Q reads
// it as [M][K]; R and Q are symmetric and are read as [K][N], which fetches whole cache lines per
// request where the K-contiguous form fetches 64 bytes per row and slab.
//
// One workgroup = 4 wavefronts (2 x 2) computes a TM x TN tile for one matrix; K runs in slabs of
// 32 moved straight from global memory into an LDS ring (no register staging; loads run
// STAGES - 1 slabs ahead to cover the memory latency), in a swizzled layout that keeps the
// 16-byte fragment reads free of bank conflicts.  Three tile shapes:
//   256 x 256  one workgroup per CU, four-deep ring (128 KiB): fewest bytes per flop
//   256 x 128  two workgroups per CU, three-deep rings (2 x 72 KiB): two wavefronts per SIMD, so the
//              matrix pipe has a second wave to issue from whenever one waits at a barrier or for
//              LDS, and the HBM-bound epilogue of one workgroup runs under the main loop of the other
//   128 x 128  three workgroups per CU (3 x 48 KiB), for products too small to fill the chip otherwise
// A launch may cover several shape groups (a descriptor per group): the workgroup index runs over
// the tiles of all groups.
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

// LDS ring depth (loads run STAGES - 1 slabs ahead of the MFMAs) and workgroups per CU
constexpr int stages_of(int TM, int TN) { return (TM == 256 && TN == 256) ? 4 : 3; }
constexpr int wgs_per_cu(int TM, int TN) { return (TM == 256 && TN == 256) ? 1 : (TM == 256 ? 2 : 3); }

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding)
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// KM: both operands are stored with K as the slow index ([K][M] and [K][N]: the Gram product X^T X
// read from the [L][S] iterate itself, no transposed copy).  The slabs then sit in LDS as [k][row]
// and the fragments are read with ds_read_b64_tr_b16, which hands every lane of a 16-lane group four
// consecutive k of one row out of four 32-byte row segments (see below).
// NW wavefronts per workgroup: 4 (2 x 2) or 8 (2 x 4: the 256 x 256 tile with two wavefronts per
// SIMD, each 128 x 64, so that the matrix pipe has a second wave to issue from whenever one waits at
// a barrier, for its fragments or for a slab).
template <int TM, int TN, int EPI, bool SYM, bool KMA, bool KMB, int NW>
__global__ __launch_bounds__(64 * NW, (NW == 8 ? 1 : wgs_per_cu(TM, TN))) void gemm_bf16_kernel(Bf16Multi mg) {
  constexpr bool KM = KMA || KMB;   // some fragment reads are transposing ones
  constexpr int STAGES = stages_of(TM, TN);
  constexpr int WCOLS = NW / 2;                  // wavefronts side by side
  constexpr int WTM = TM / 2, WTN = TN / WCOLS;  // wave tile (2 x WCOLS waves)
  constexpr int NBM = WTM / 32, NBN = WTN / 32;  // 32x32 blocks per wave and dimension
  constexpr int LDA = TM / (16 * NW), LDB = TN / (16 * NW);   // direct-to-LDS load instructions per wave, operand and slab
  static_assert(NW == 4 || (NW == 8 && TM == 256 && TN == 256), "wavefronts per workgroup");
  constexpr int NL = LDA + LDB;                  // ... per wave and slab
  constexpr int OPA_BYTES = TM * 64;             // operand slabs in LDS: rows x 32 bf16, unpadded
  constexpr int BUF_BYTES = (TM + TN) * 64;
  constexpr int RT = TM / TN;                    // SYM: tile columns per tile row height
  static_assert(TM % 64 == 0 && TN % 64 == 0 && (RT == 1 || RT == 2), "tile shape");
  // LDS: ring of STAGES buffers, each [A slab | B slab].  The LDS has 64 banks of 4 bytes and
  // serves a 16-byte read per lane in groups of 16 lanes, so 16 consecutive lanes must cover one
  // 256-byte bank line exactly once.  Four consecutive rows (64 bytes each) share a line; the
  // sixteen 16-byte chunks of line q sit at slot ((row & 3) * 4 + chunk) ^ (q & 15): the fragment
  // reads (16 consecutive rows, same chunk) then hit 16 different slots.
  extern __shared__ __align__(1024) unsigned char smem[];

  // Workgroup -> (group, tile).  The hardware deals consecutive workgroups round-robin to the 8
  // XCDs, each with its own L2.  xcd_private (set by the launcher for small matrices, or when all
  // operands of the launch fit the Infinity Cache together): every XCD gets a contiguous range of
  // tiles, i.e. whole matrices, so that the tiles sharing a panel share an L2 (without this the
  // 768-sized Gram fetched 7x its algorithmic bytes).  Otherwise workgroup i runs tile i: all XCDs
  // sweep the same matrix and share its panels through the Infinity Cache (private ranges measured
  // 20 % slower at 8 x 4096^2, where eight matrices at once overflow that cache).
  int wg = blockIdx.x;
  const int total = mg.tile_start[mg.ngroups];
  if ((total & 7) == 0 && mg.xcd_private) wg = (wg & 7) * (total >> 3) + (wg >> 3);
  int gi = 0;
  while (gi + 1 < mg.ngroups && wg >= mg.tile_start[gi + 1]) ++gi;
  wg -= mg.tile_start[gi];
  const Bf16Desc& g = mg.d[gi];

  // SYM: A == B and the result is symmetric (Gram matrix, R^2): only the tiles that reach the
  // diagonal or lie above it are computed; a tile wholly above the diagonal blocks is also written
  // mirrored.
  const int tiles_m = g.M / TM, tiles_n = g.N / TN;
  const int per_mat = SYM ? RT * tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  const int b = wg / per_mat;
  const int rem = wg - b * per_mat;
  int tm, tn;
  if (SYM) {       // row tm of the upper triangle holds tiles_n - RT * tm tiles
    int left = rem;
    tm = 0;
    while (left >= tiles_n - RT * tm) { left -= tiles_n - RT * tm; ++tm; }
    tn = RT * tm + left;
  } else if (g.xcd_blocks && !mg.xcd_private) {
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
  const float alpha = g.ctrl ? g.ctrl[cb].alpha : 1.0f;

  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);  // uniform: LDS destinations stay scalar
  const int wm0 = (wave / WCOLS) * WTM, wn0 = (wave % WCOLS) * WTN;
  const int m0 = tm * TM, n0 = tn * TN;
  const unsigned short* A1 = g.A + (long long)b * g.strideA + (KMA ? (long long)m0 : (long long)m0 * g.lda);
  const unsigned short* Bb = g.B + (long long)b * g.strideB + (KMB ? (long long)n0 : (long long)n0 * g.ldb);

  const int KT = g.K / BK;

  // Global -> LDS without passing through registers (global_load_lds_dwordx4): one wave
  // instruction moves 64 lanes x 16 bytes into 1 KiB of consecutive LDS = 16 rows of a slab.
  // Lane l fills slot l & 15 of line l >> 4 of those 16 rows and fetches the chunk that belongs
  // there (the line index within the slab is (it * NW + wave) * 4 + (l >> 4)).
  // KM: a slab is 32 k-rows of T consecutive entries; one wave instruction moves 64 / (T / 8) of
  // them.  16-byte unit u of row k holds chunk u ^ (4 (k & 3)) of that row, so that the four row
  // segments a transposing read touches (same chunks, rows 4j .. 4j + 3) fall on different banks.
  const int lq = lane >> 4, lu = (lane & 15) ^ ((wave * 4 + lq) & 15);
  unsigned aoff[LDA], boff[LDB];
  if constexpr (KMA) {
    constexpr int URA = TM / 8;          // 16-byte units per k-row
#pragma unroll
    for (int it = 0; it < LDA; ++it) {
      const int k = (it * NW + wave) * (64 / URA) + lane / URA, c = (lane % URA) ^ (4 * (k & 3));
      aoff[it] = (unsigned)(k * g.lda + c * 8) * 2u;
    }
  } else {
#pragma unroll
    for (int it = 0; it < LDA; ++it) aoff[it] = (unsigned)(((it * NW + wave) * 16 + 4 * lq + (lu >> 2)) * g.lda + (lu & 3) * 8) * 2u;
  }
  if constexpr (KMB) {
    constexpr int URB = TN / 8;
#pragma unroll
    for (int it = 0; it < LDB; ++it) {
      const int k = (it * NW + wave) * (64 / URB) + lane / URB, c = (lane % URB) ^ (4 * (k & 3));
      boff[it] = (unsigned)(k * g.ldb + c * 8) * 2u;
    }
  } else {
#pragma unroll
    for (int it = 0; it < LDB; ++it) boff[it] = (unsigned)(((it * NW + wave) * 16 + 4 * lq + (lu >> 2)) * g.ldb + (lu & 3) * 8) * 2u;
  }
  // load instruction u in [0, NL): first the LDA of A, then the LDB of B
  auto issue_load = [&](int kt, int slot, int u) {
    const long long ka = KMA ? (long long)kt * BK * g.lda : (long long)kt * BK;
    const long long kb = KMB ? (long long)kt * BK * g.ldb : (long long)kt * BK;
    if (u < LDA) {
      unsigned char* dst = smem + slot * BUF_BYTES + wave * 1024 + u * (1024 * NW);
      __builtin_amdgcn_global_load_lds((gptr_t)((const char*)(A1 + ka) + aoff[u]), (lptr_t)dst, 16, 0, 0);
    } else {
      unsigned char* dst = smem + slot * BUF_BYTES + OPA_BYTES + wave * 1024 + (u - LDA) * (1024 * NW);
      __builtin_amdgcn_global_load_lds((gptr_t)((const char*)(Bb + kb) + boff[u - LDA]), (lptr_t)dst, 16, 0, 0);
    }
  };
  auto issue_loads = [&](int kt, int slot) {
#pragma unroll
    for (int u = 0; u < NL; ++u) issue_load(kt, slot, u);
  };

  f32x16 acc[NBM][NBN];
#pragma unroll
  for (int i = 0; i < NBM; ++i)
#pragma unroll
    for (int j = 0; j < NBN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragment addresses: row r = tile row, chunk cc = 2 * kk + (lane >> 5)
  const int lr = lane & 31, lh = lane >> 5;
  // (row block f starts 32 rows = 8 lines further on, which flips bit 3 of the line index; the wave
  // offsets are multiples of 64 rows = 16 lines and leave it alone)
  const unsigned char* Afr = smem + wm0 * 64 + (lr >> 2) * 256;
  const unsigned char* Bfr = smem + OPA_BYTES + wn0 * 64 + (lr >> 2) * 256;
  int koff[2][2];
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int par = 0; par < 2; ++par)
      koff[kk][par] = ((((lr & 3) << 2) + kk * 2 + lh) ^ ((lr >> 2) + 8 * par)) << 4;
  // KM: lane l = (i = l % 16, mb = (l / 16) % 2, kg = l / 32) of row block f reads, for the half r of
  // its eight k, the 8 bytes at row k = 16 kk + 8 kg + 4 r + i / 4, entries 32 f + 16 mb + 4 (i % 4) ..
  // + 3 of the wave's rows; the instruction returns to lane l the entry 32 f + 16 mb + i of rows
  // 16 kk + 8 kg + 4 r .. + 3: eight consecutive k of one row after two reads, the MFMA operand layout.
  int fra[NBM], frb[NBN];
  if constexpr (KMA) {
    const int i = lane & 15, mb = (lane >> 4) & 1, kg = lane >> 5;
#pragma unroll
    for (int f = 0; f < NBM; ++f) {
      const int c = wm0 / 8 + 4 * f + 2 * mb + ((i & 3) >> 1);
      fra[f] = (8 * kg + (i >> 2)) * (TM / 8) * 16 + ((c ^ (4 * (i >> 2))) * 16) + 8 * (i & 1);
    }
  }
  if constexpr (KMB) {
    const int i = lane & 15, mb = (lane >> 4) & 1, kg = lane >> 5;
#pragma unroll
    for (int f = 0; f < NBN; ++f) {
      const int c = wn0 / 8 + 4 * f + 2 * mb + ((i & 3) >> 1);
      frb[f] = OPA_BYTES + (8 * kg + (i >> 2)) * (TN / 8) * 16 + ((c ^ (4 * (i >> 2))) * 16) + 8 * (i & 1);
    }
  }
  // The transposing reads are issued as inline assembly: given as a builtin, the compiler cannot
  // tell them from readers of the slabs still on their way into LDS and waits for every outstanding
  // global load before each one, which empties the ring at every step.  The price: it does not wait
  // for their results either, so every place that consumes fragments says so itself (frag_wait).
  typedef unsigned u32x2v __attribute__((ext_vector_type(2)));
  const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem;
  auto read_tr = [&](int byte_off) {
    u32x2v r;
    asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(r) : "v"(lds0 + (unsigned)byte_off));
    return r;
  };
  // In a kernel with transposing reads the ordinary fragment reads are issued the same way, so that
  // one explicit wait covers both kinds.
  auto plain_frag = [&](const unsigned char* p) {
    if constexpr (KM) {
      u32x4 r;
      asm volatile("ds_read_b128 %0, %1" : "=v"(r) : "v"((unsigned)(size_t)(__attribute__((address_space(3))) const unsigned char*)p));
      return __builtin_bit_cast(bf16x8, r);
    } else {
      return *(const bf16x8*)p;
    }
  };
  auto frag_wait = [&]() {   // KM: all fragment reads issued so far have landed
    if constexpr (KM) {
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  bf16x8 fa[2][NBM], fb[2][NBN];
  constexpr int NF = NBM + NBN;          // fragment reads per sub-step
  constexpr int NM = NBM * NBN;          // MFMAs per sub-step
  // fragment f in [0, NF) of sub-step kk: first the NBM row blocks of A, then the NBN of B
  auto load_frag = [&](int slot, int kk, int f) {
    const int o = slot * BUF_BYTES;
    auto tr_frag = [&](int base, int step) {
      const u32x2v h0 = read_tr(base), h1 = read_tr(base + step);
      const u32x4 v = {h0[0], h0[1], h1[0], h1[1]};
      return __builtin_bit_cast(bf16x8, v);
    };
    // KM operand: rows 16 kk + 4 r of the slab lie (16 kk + 4 r) * (T / 8) * 16 bytes further on
    if (f < NBM) {
      if constexpr (KMA) fa[kk][f] = tr_frag(o + fra[f] + kk * 16 * (TM / 8) * 16, 4 * (TM / 8) * 16);
      else fa[kk][f] = plain_frag(Afr + o + koff[kk][f & 1] + f * 2048);
    } else {
      if constexpr (KMB) fb[kk][f - NBM] = tr_frag(o + frb[f - NBM] + kk * 16 * (TN / 8) * 16, 4 * (TN / 8) * 16);
      else fb[kk][f - NBM] = plain_frag(Bfr + o + koff[kk][(f - NBM) & 1] + (f - NBM) * 2048);
    }
  };
  auto load_frags = [&](int slot, int kk) {
#pragma unroll
    for (int f = 0; f < NF; ++f) load_frag(slot, kk, f);
  };
  auto mfma_one = [&](int set, int m) {
    const int i = m / NBN, j = m % NBN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
  };
  auto mfma_block = [&](int set) {
#pragma unroll
    for (int m = 0; m < NM; ++m) mfma_one(set, m);
  };
  // wait until the loads of slab `kt` have landed: up to STAGES - 2 younger slabs may still be in flight
  auto wait_slab = [&](int kt) {
    const int younger = KT - 1 - kt;
    if (younger >= 2 && STAGES >= 4) wait_vmcnt<2 * NL>();
    else if (younger >= 1) wait_vmcnt<NL>();
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
    if constexpr (KM) __builtin_amdgcn_sched_barrier(0);   // no MFMA may move above the wait for its fragments
  };

  // Main loop.  Slab kt+STAGES-1 is requested during the first half of slab kt (its ring slot was
  // released by the barrier that closed slab kt-1); the fragments of the second half of slab kt
  // are read while its first half computes, and after the single barrier of the slab the first
  // fragments of slab kt+1 are read while the second half computes.  Reads and requests are placed
  // one per MFMA at the head of each half, so that they issue in the shadow of the matrix pipe and
  // the LDS latency of the last read is covered by the MFMAs that follow it.
  static_assert(BK == 32 && STAGES >= 3 && STAGES <= 4, "pipeline written for two sub-steps per slab");
#pragma unroll
  for (int s0 = 0; s0 < STAGES - 1; ++s0)
    if (s0 < KT) issue_loads(s0, s0);
  wait_slab(0);
  ring_barrier();
  load_frags(0, 0);
  int kt = 0, slot = 0;                 // slot = kt mod STAGES
  const int KT_main = KT - (STAGES - 1);
  constexpr int NSTEP = NM > NF ? (NM > NL ? NM : NL) : (NF > NL ? NF : NL);   // interleave steps per half
  for (; kt < KT_main; ++kt) {          // steady state: no conditions inside
    const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
    const int lslot = slot == 0 ? STAGES - 1 : slot - 1;   // slot of slab kt-1 = slot of slab kt+STAGES-1
    frag_wait();                         // fragments of the first half (read during the half before)
    // Every step issues its MFMA first: the first one of a half waits for the fragments read during
    // the half before (long complete), and a read placed ahead of it would add its own LDS latency
    // to that wait (the counter only tells "all reads done").
#pragma unroll
    for (int u = 0; u < NSTEP; ++u) {
      if (u < NM) mfma_one(0, u);
      __builtin_amdgcn_sched_barrier(0);
      if (u < NF) load_frag(slot, 1, u);
      if (u < NL) issue_load(kt + STAGES - 1, lslot, u);
      __builtin_amdgcn_sched_barrier(0);
    }
    wait_vmcnt<(STAGES - 2) * NL>();   // slab kt+1 has landed; the younger ones may be in flight
    ring_barrier();
#pragma unroll
    for (int u = 0; u < NSTEP; ++u) {
      if (u < NM) mfma_one(1, u);
      __builtin_amdgcn_sched_barrier(0);
      if (u < NF) load_frag(nslot, 0, u);
      __builtin_amdgcn_sched_barrier(0);
    }
    slot = nslot;
  }
  for (; kt < KT; ++kt) {               // drain: nothing left to request
    const int nslot = slot == STAGES - 1 ? 0 : slot + 1;
    frag_wait();
    load_frags(slot, 1);
    mfma_block(0);
    if (kt + 1 < KT) wait_slab(kt + 1);
    ring_barrier();
    if (kt + 1 < KT) load_frags(nslot, 0);
    mfma_block(1);
    slot = nslot;
  }

  // epilogue: register r of lane l holds row (r/4)*8 + (l/32)*4 + r%4, column l%32 of a block
  float part = 0.0f;
  const float coef = g.coef_is_alpha ? alpha : 1.0f;
  const int rbase = (lane >> 5) * 4;
  if constexpr (SYM && (EPI == BEPI_GRAM || EPI == BEPI_POLYQ)) {
    // Each wave passes its tile through its own LDS strip of 32 rows (the ring is free after the
    // last barrier): row-wise for the tile itself, column-wise for its mirror image, so that both
    // are written with 16- and 32-byte vectors on contiguous runs.
    constexpr int SW = WTN + 4;
    float* strip = (float*)smem + wave * 32 * SW;
    constexpr int LPR = WTN / 8, RPI = 64 / LPR;
    const int rr = lane / LPR, cc = (lane % LPR) * 8;
    const int cq = lane >> 2, rq = lane & 3;
    const bool mirror = n0 >= m0 + TM;   // wholly above the diagonal blocks (which are computed in full)
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
    for (int i = 0; i < NBM; ++i) {
#pragma unroll
      for (int j = 0; j < NBN; ++j)
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
          } else if (m >= n && m < n + 8) {   // the diagonal entry of this row lies in these 8 columns
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
      if (i + 1 < NBM) fetch_r(i + 1);
      if (mirror) {
        // column-wise: 8 consecutive rows of one column = 8 consecutive entries of a mirrored row
#pragma unroll
        for (int it = 0; it < WTN / 16; ++it) {
          const int col = it * 16 + cq;
          f32x4 t0, t1;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            t0[e] = strip[(rq * 8 + e) * SW + col];
            t1[e] = strip[(rq * 8 + 4 + e) * SW + col];
          }
          const int mr = n0 + wn0 + col, nr = m0 + wm0 + i * 32 + rq * 8;   // mirrored position
          if (EPI == BEPI_GRAM && !lean && !g.upper32) {
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
    // Each wave passes its tile through its own LDS strip of 32 rows so that every global access
    // is a 16-byte vector on a contiguous run of a row of X (read) and X' (write).  The LDS ring is
    // free here: no wave reads fragments after the last barrier of the main loop.
    constexpr int SW = WTN + 4;                      // strip row stride in floats (16-byte aligned)
    float* strip = (float*)smem + wave * 32 * SW;
    constexpr int LPR = WTN / 8, RPI = 64 / LPR;     // lanes per row, rows per instruction
    const int rr = lane / LPR, cc = (lane % LPR) * 8;
    const long long base = (long long)b * g.strideCb;
    // The old iterate of row block i + 1 is requested while block i is worked on (and that of
    // block 0 before the accumulators go to LDS): its memory latency is paid once per tile
    // instead of once per block.
    constexpr int ITS = 32 / RPI;
    u32x4 xh[2][ITS], xl[2][ITS];
    const bool has_lo = g.Xlo != nullptr;
    // Split iterate: the product takes the high half only.  What the low half would contribute,
    // X_lo Q, matters for the small singular values alone, and on their subspace the polynomial
    // Q = R/2 + alpha R^2 (d = 1: alpha R) acts as the scalar c = 1/2 + alpha (alpha), because R is
    // the identity there up to sigma^2.  So X_lo Q is taken as c X_lo here, elementwise; the part
    // left out, X_lo (Q - c I), is second order in the small singular values.  Once the fit has left
    // the upper end of its interval (ctrl.plain: no singular value is small any more) Q tends to
    // zero instead and the term is dropped.
    const float lo_gain = 1.0f + ((has_lo && g.ctrl && !g.ctrl[cb].plain) ? (g.coef_is_alpha ? alpha : 0.5f + alpha) : 0.0f);
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
    for (int i = 0; i < NBM; ++i) {
      if (i + 1 < NBM) fetch_x(i + 1, (i + 1) & 1);
#pragma unroll
      for (int j = 0; j < NBN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r)
          strip[((r >> 2) * 8 + rbase + (r & 3)) * SW + j * 32 + lr] = acc[i][j][r];
      // row-wise: x' = x_hi + lo_gain * x_lo + coef * acc, split again
#pragma unroll
      for (int it = 0; it < ITS; ++it) {
        const int row = it * RPI + rr;
        float* sp = strip + row * SW + cc;
        const f32x4 a0 = *(const f32x4*)sp, a1 = *(const f32x4*)(sp + 4);
        const long long o = base + (long long)(m0 + wm0 + i * 32 + row) * g.ldcb + n0 + wn0 + cc;
        const u32x4 hi = xh[i & 1][it];
        const u32x4 lo = xl[i & 1][it];
        u32x4 nh, nl;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          // two bf16 per 32-bit word: even element in the low half
          const float x0 = __uint_as_float(hi[e] << 16) + lo_gain * __uint_as_float(lo[e] << 16) + coef * (e < 2 ? a0[2 * e] : a1[2 * e - 4]);
          const float x1 = __uint_as_float(hi[e] & 0xFFFF0000u) + lo_gain * __uint_as_float(lo[e] & 0xFFFF0000u) + coef * (e < 2 ? a0[2 * e + 1] : a1[2 * e - 3]);
          const unsigned h0 = f2bf(x0), h1 = f2bf(x1);
          nh[e] = h0 | (h1 << 16);
          nl[e] = (unsigned)f2bf(x0 - bf2f((unsigned short)h0)) | ((unsigned)f2bf(x1 - bf2f((unsigned short)h1)) << 16);
        }
        *(u32x4*)(g.Cb + o) = nh;
        if (g.Cb2) *(u32x4*)(g.Cb2 + o) = nl;
      }
    }
  } else {
    static_assert(EPI == BEPI_STORE && !SYM, "GRAM and POLYQ exist as symmetric products only");
#pragma unroll
    for (int i = 0; i < NBM; ++i)
#pragma unroll
      for (int j = 0; j < NBN; ++j) {
        const int gn = n0 + wn0 + j * 32 + lr;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int gm = m0 + wm0 + i * 32 + rg * 8 + rbase;  // first of 4 consecutive rows
#pragma unroll
          for (int e = 0; e < 4; ++e)
            g.C32[(long long)b * g.strideC32 + (long long)(gm + e) * g.ldc32 + gn] = acc[i][j][rg * 4 + e];
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
    if (t == 0) {
      float sum = (red[0] + red[1]) + (red[2] + red[3]);
      if (NW == 8) sum += (red[4] + red[5]) + (red[6] + red[7]);
      g.rho_part[(long long)b * per_mat + rem] = sum;
    }
  }
}

// tiles of one matrix
template <int TM, int TN, bool SYM>
long long tiles_per_matrix(const Bf16Desc& g) {
  const long long tm = g.M / TM, tn = g.N / TN;
  return SYM ? (TM / TN) * tm * (tm + 1) / 2 : tm * tn;
}

template <int TM, int TN, int EPI, bool SYM, bool KMA, bool KMB, int NW>
int launch_tw(Bf16Multi& mg, hipStream_t s) {
  long long total = 0;
  for (int i = 0; i < mg.ngroups; ++i) {
    mg.tile_start[i] = (int)total;
    total += tiles_per_matrix<TM, TN, SYM>(mg.d[i]) * mg.d[i].batch;
    if (total > 0x7fffffff) return PRISM_EUNSUPPORTED;
  }
  mg.tile_start[mg.ngroups] = (int)total;
  const size_t lds = (size_t)stages_of(TM, TN) * (TM + TN) * 64;   // ring of STAGES x (A slab + B slab)
  const int rc = allow_dynamic_lds((const void*)gemm_bf16_kernel<TM, TN, EPI, SYM, KMA, KMB, NW>, (int)lds);
  if (rc != PRISM_OK) return rc;
  hipLaunchKernelGGL((gemm_bf16_kernel<TM, TN, EPI, SYM, KMA, KMB, NW>), dim3((unsigned)total), dim3(64 * NW), lds, s, mg);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

// 256 x 256 tiles run with eight wavefronts (mg.waves8), every other shape with four
template <int TM, int TN, int EPI, bool SYM, bool KMA = false, bool KMB = false>
int launch_te(Bf16Multi& mg, hipStream_t s) {
  if constexpr (TM == 256 && TN == 256) {
    if (mg.waves8) return launch_tw<TM, TN, EPI, SYM, KMA, KMB, 8>(mg, s);
  }
  return launch_tw<TM, TN, EPI, SYM, KMA, KMB, 4>(mg, s);
}

template <int TM, int TN>
int launch_t(Bf16Multi& mg, hipStream_t s) {
  const int epi = mg.d[0].epi, sym = mg.d[0].sym, km = mg.d[0].km;
  for (int i = 0; i < mg.ngroups; ++i) {
    const Bf16Desc& g = mg.d[i];
    if (g.epi != epi || g.sym != sym || g.km != km) return PRISM_EINVAL;
    if (g.M % TM || g.N % TN || g.K % BK || g.K < BK || g.lda % 8 || g.ldb % 8) return PRISM_EINVAL;
    if ((long long)(g.M / TM) * (g.N / TN) * g.batch <= 0) return PRISM_EINVAL;
    if (g.sym && (g.M != g.N || g.A != g.B)) return PRISM_EINVAL;
    if ((g.epi == BEPI_GRAM || g.epi == BEPI_POLYQ) && !g.sym) return PRISM_EINVAL;   // symmetric products only
    if (g.epi == BEPI_STORE && (g.sym || !g.C32)) return PRISM_EINVAL;
    // without the fp32 matrix: GRAM with a diagonal array, POLYQ with R in bf16
    if (g.epi == BEPI_GRAM && !g.C32 && !g.diag) return PRISM_EINVAL;
    if (g.epi == BEPI_POLYQ && !g.C32 && !g.Cin16) return PRISM_EINVAL;
  }
  // operand layouts (km: bit 0 = A stored [K][M], bit 1 = B stored [K][N]) per kind of product
  switch (epi) {
    case BEPI_STORE:
      if (km == 3) return launch_te<TM, TN, BEPI_STORE, false, true, true>(mg, s);
      if (km == 2) return launch_te<TM, TN, BEPI_STORE, false, false, true>(mg, s);
      if (km == 0) return launch_te<TM, TN, BEPI_STORE, false>(mg, s);
      return PRISM_EINVAL;
    case BEPI_GRAM:
      if (km == 3) return launch_te<TM, TN, BEPI_GRAM, true, true, true>(mg, s);
      if (km == 0) return launch_te<TM, TN, BEPI_GRAM, true>(mg, s);
      return PRISM_EINVAL;
    case BEPI_POLYQ:
      if (km == 3) return launch_te<TM, TN, BEPI_POLYQ, true, true, true>(mg, s);
      if (km == 0) return launch_te<TM, TN, BEPI_POLYQ, true>(mg, s);
      return PRISM_EINVAL;
    case BEPI_APPLY:
      if (km == 2) return launch_te<TM, TN, BEPI_APPLY, false, false, true>(mg, s);
      if (km == 0) return launch_te<TM, TN, BEPI_APPLY, false>(mg, s);
      return PRISM_EINVAL;
  }
  return PRISM_EINVAL;
}

}  // namespace

int launch_gemm_bf16_multi(const Bf16Desc* groups, int ngroups, int tile_m, int tile_n, hipStream_t s) {
  if (ngroups < 1 || ngroups > BF16_MAX_GROUPS) return PRISM_EINVAL;
  Bf16Multi mg = {};
  mg.ngroups = ngroups;
  // bytes of all operands of the launch against half the 256 MiB Infinity Cache
  double operand_bytes = 0.0;
  bool small = true;
  static const int no_blocks = ab_switch("PRISM_BF16_NO_XCD_BLOCKS");
  for (int i = 0; i < ngroups; ++i) {
    Bf16Desc& g = mg.d[i];
    g = groups[i];
    operand_bytes += 2.0 * g.batch * ((double)g.M * g.K + (g.A == g.B ? 0.0 : (double)g.N * g.K));
    const long long tm = g.M / tile_m, tn = g.N / tile_n;
    const long long per_mat = g.sym ? (tile_m / tile_n) * tm * (tm + 1) / 2 : tm * tn;
    if (per_mat > 64) small = false;
    g.xcd_blocks = !no_blocks && !g.sym && per_mat % 256 == 0 && tm % 4 == 0 && tn % 8 == 0;
  }
  mg.xcd_private = small || operand_bytes <= 128.0 * 1024 * 1024;
  static const int waves4 = ab_switch("PRISM_BF16_WAVES4");
  mg.waves8 = !waves4;
  if (tile_m == 256 && tile_n == 256) return launch_t<256, 256>(mg, s);
  if (tile_m == 256 && tile_n == 128) return launch_t<256, 128>(mg, s);
  if (tile_m == 128 && tile_n == 128) return launch_t<128, 128>(mg, s);
  return PRISM_EINVAL;
}

int launch_gemm_bf16(const Bf16Desc& g, int tile_m, int tile_n, hipStream_t s) {
  return launch_gemm_bf16_multi(&g, 1, tile_m, tile_n, s);
}

}  // namespace prism
