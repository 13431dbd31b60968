// Sketch chain V_out = R * V_in (paper Section 4.2 and App. A.1: the products R(R(...(R S^T)))
// that make the fit cost O(n^2 p_s) instead of O(n^3)).  R is n x n fp32, V is n x p_s with the
// sketch width padded to ld = 16, 32 or 64 columns.  The product reads R exactly once and is bound
// by HBM bandwidth, so R never goes through LDS: every lane fetches 16 bytes of its row straight
// into registers and feeds v_mfma_f32_16x16x4_f32; only the small V is staged in LDS and shared by
// the four wavefronts of a workgroup.
//
//   workgroup = 4 wavefronts = 64 rows of R for one matrix, wave w owns rows 16w..16w+15
//   K runs in chunks of 64: lane (i = l % 16, q = l / 16) holds R[row i][k0 + 16 s + 4 q + e],
//   s = 0..3, e = 0..3; MFMA (s, e) pairs it with V[k0 + 16 s + 4 q + e][col] (the order of the
//   four k of one instruction is free as long as both operands agree).
//   V chunk in LDS: Vs[64][LD + 4]; with that stride the four lane groups of a fragment read
//   (rows 4 apart) fall on disjoint bank halves.
//   The loads of R and V run five chunks ahead of the MFMAs (the kernel is latency bound otherwise).
//
// Three kernels: chain_kernel (64-row workgroups, fp32 R), chain_small_kernel (16-row workgroups
// for small batches of small matrices, fp32 or bf16 R) and chain_bf16_kernel (64-row workgroups,
// bf16 R, bf16 matrix cores).
//
// bf16 R (bf16 polar path): R is read from its bf16 copy, half the bytes.  The diagonal of R is
// taken from the fp32 matrix all the same: early on it is 1 - g_ii with g_ii ~ 1/n, which rounds
// to 1 in bf16 and would erase the factor (1 - xi) of the fit objective (Section 4.2), whereas
// rounding the off-diagonal entries perturbs the fitted coefficient by ~1e-5 only.  The kernels
// multiply by the bf16 matrix and add (r_ii - bf16(r_ii)) v_i afterwards.
#include <cstdlib>
#include <type_traits>

#include "common.h"

namespace prism {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
constexpr int NT = 256;
constexpr int KC = 64;     // k per chunk
constexpr int ROWS = 64;   // rows of R per workgroup

typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

// Four consecutive k of one row of R: fp32 as they are, bf16 widened in registers.
template <bool RB> struct RFrag;
template <> struct RFrag<false> {
  typedef float elem;
  f32x4 v;
  __device__ void load(const float* p) { v = *(const f32x4*)p; }
  __device__ float get(int e) const { return v[e]; }
};
template <> struct RFrag<true> {
  typedef unsigned short elem;
  u32x2 v;
  __device__ void load(const unsigned short* p) { v = *(const u32x2*)p; }
  __device__ float get(int e) const {
    const unsigned w = v[e >> 1];
    return __uint_as_float((e & 1) ? (w & 0xFFFF0000u) : (w << 16));
  }
};

__device__ inline float bf16_bits_to_float(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

template <int D, typename F>
__device__ inline void unrolled(F&& f) {
  if constexpr (D > 0) {
    unrolled<D - 1>(f);
    f(std::integral_constant<int, D - 1>{});
  }
}

template <int LD>
__global__ __launch_bounds__(NT, 2) void chain_kernel(const float* __restrict__ R, long long strideR, int ldr,
                                                   const float* __restrict__ Vin, long long strideVin,
                                                   float* __restrict__ Vout, long long strideVout, int n,
                                                   const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int VS = LD + 4;
  constexpr int EK = 4;                // k per 16-byte load
  constexpr int KCH = 16 * EK;         // k per chunk
  __shared__ __align__(16) float Vs[2][KCH][VS];
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int li = lane & 15, lq = lane >> 4;
  const int row0 = blockIdx.x * ROWS + wave * 16;
  const float* Rrow = R + (long long)b * strideR + (long long)(row0 + li) * ldr + EK * lq;
  const float* Vb = Vin + (long long)b * strideVin;

  // Loads return in order, so waiting for one drains every older one.  The chunk of V that is
  // staged in LDS next is therefore requested DEPTH-1 chunks ahead as well, just before the rows
  // of R of the same chunk: when the wave waits for it, the rows of the DEPTH-2 chunks behind it
  // stay in flight (requested one chunk ahead only, that wait emptied the whole ring every chunk).
  constexpr int DEPTH = LD == 64 ? 4 : 6;
  // V chunk loader: KCH x LD floats = KCH * LD / 4 float4, spread over the workgroup
  constexpr int V_LOADS = KCH * LD / 4;
  constexpr int V_IT = (V_LOADS + NT - 1) / NT;
  f32x4 vreg[DEPTH][V_IT];
  f32x4 ra[DEPTH][4];
  const int nchunks = n / KCH;
  // Past the end the last chunk is fetched again (and never used): no branch around the loads, so
  // that the compiler can count how many younger loads may stay in flight at each wait.  (With the
  // loads under a condition it had to assume none were issued and waited for all of them.)
  // The workgroups of one matrix all read the same V; each starts its sweep over k at a chunk of
  // its own, so that at any moment they ask different L2 channels for it.
  const int rot = (int)(blockIdx.x % (unsigned)nchunks);
  auto load_chunk = [&](int slot, int c_want) {   // slot is a compile-time constant at every call site
    int c = (c_want < nchunks ? c_want : nchunks - 1) + rot;
    if (c >= nchunks) c -= nchunks;
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      if (V_LOADS % NT == 0 || idx < V_LOADS) {
        const int kr = idx / (LD / 4), c4 = idx % (LD / 4);
        vreg[slot][it] = *(const f32x4*)(Vb + (long long)(c * KCH + kr) * LD + c4 * 4);
      }
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) ra[slot][s] = *(const f32x4*)(Rrow + c * KCH + 4 * EK * s);
  };
  auto store_v = [&](int slot, int buf) {
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      if (V_LOADS % NT == 0 || idx < V_LOADS) {
        const int kr = idx / (LD / 4), c4 = idx % (LD / 4);
        *(f32x4*)&Vs[buf][kr][c4 * 4] = vreg[slot][it];
      }
    }
  };

  // Eight independent accumulators per wave (k taken round-robin), added up at the end: an MFMA
  // that accumulates into the result of the one before it waits out the whole pipeline latency,
  // and one or two chains of such MFMAs kept the matrix cores half idle.
  constexpr int NACC = 8 / NBLK;
  f32x4 acc[NBLK][NACC];
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int u = 0; u < NACC; ++u) acc[j][u] = (f32x4){0.f, 0.f, 0.f, 0.f};

  // Workgroup barrier without the release fence of __syncthreads(): that fence waits for every
  // outstanding load and would expose the memory latency of the prefetched rows of R at every
  // chunk.  LDS traffic of this wave is complete (lgkmcnt(0)); loads into registers stay in flight.
  auto lds_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d) load_chunk(d, d);
  store_v(0, 0);
  lds_barrier();
  auto step = [&](auto dtag, int c) {   // chunk c, whose rows sit in ring slot d = c % DEPTH
    constexpr int d = decltype(dtag)::value;
    const int cur = c & 1;
    load_chunk((d + DEPTH - 1) % DEPTH, c + DEPTH - 1);
    // The fragments of V are read from LDS one load step ahead of the MFMAs that use them (left
    // to itself the compiler reads each pair right before its two MFMAs and waits every time).
    float vf[2][EK][NBLK];
    auto read_v = [&](int s) {
#pragma unroll
      for (int e = 0; e < EK; ++e)
#pragma unroll
        for (int j = 0; j < NBLK; ++j) vf[s & 1][e][j] = Vs[cur][16 * s + 4 * lq + e][j * 16 + li];
    };
    read_v(0);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 4) read_v(s + 1);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < EK; ++e)
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
          acc[j][(s * EK + e) % NACC] = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[d][s][e], vf[s & 1][e][j], acc[j][(s * EK + e) % NACC], 0, 0, 0);
    }
    store_v((d + 1) % DEPTH, cur ^ 1);   // chunk c + 1 (past the end: the last one again, unused)
    lds_barrier();
  };
  const int nfull = nchunks / DEPTH * DEPTH;
  for (int c0 = 0; c0 < nfull; c0 += DEPTH)
    unrolled<DEPTH>([&](auto dt) { step(dt, c0 + decltype(dt)::value); });
  // the last nchunks % DEPTH chunks
  unrolled<DEPTH - 1>([&](auto dt) {
    if (nfull + decltype(dt)::value < nchunks) step(dt, nfull + decltype(dt)::value);
  });
#pragma unroll
  for (int j = 0; j < NBLK; ++j) {
#pragma unroll
    for (int w = NACC / 2; w > 0; w >>= 1)      // fixed pairwise order
#pragma unroll
      for (int u = 0; u < w; ++u) acc[j][u] += acc[j][u + w];
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + 4 * lq + r, col = j * 16 + li;
      Vout[(long long)b * strideVout + (long long)row * LD + col] = acc[j][0][r];
    }
}

// Large matrices, R from its bf16 copy, on the bf16 matrix cores (v_mfma_f32_16x16x32_bf16): with
// fp32 MFMAs the kernel above is bound by them once R shrinks to two bytes per entry.  V keeps its
// 24 significant bits: every fp32 entry is cut into three bf16 pieces (8 bits each, exact) and R is
// multiplied by each piece; the partial products of two bf16 numbers are exact in fp32, so only the
// accumulation rounds.
//
// The pieces are not cut here (every workgroup would cut all of V again).  Whoever produces a V (this
// kernel for V_1 .. V_{nv-1}, split_planes_kernel for the sketches) also writes it as three bf16
// planes, chunk by chunk of 256 k, as the image of the LDS stage the consumer wants:
//     P[matrix][c = k / 256][plane][column][unit u'][8 k],   u = (k % 256) / 8,  u' = (u & 16) | ((u ^ column) & 15)
// A stage is 3 * LD rows of 512 bytes; the workgroup moves it from global memory straight into LDS
// (global_load_lds_dwordx4, 1 KiB per wave instruction, no registers, no arithmetic).
// A workgroup owns 64 rows of R; wave w takes the k with (k % 256) / 64 = w of every chunk, for all
// 64 rows: its fragments of V (a quarter of the stage) serve four row blocks, so the LDS is read
// a quarter as often as with a wave per 16 rows, and the wave fetches whole 128-byte lines of R.
// The four partial sums are added through LDS in a fixed order at the end.
//   A operand: lane (i = l % 16, g = l / 16) holds R[row 16 q + i][256 c + 64 w + 32 h + 8 g .. + 7], h = 0, 1
//   B operand: lane (j = l % 16, g) reads unit u = 8 w + 4 h + g of column 16 jb + j: with the low bits of
//   the unit index xor-ed by the column the 16 lanes of a group hit 16 different units of their rows.
// R goes straight into registers.  Rows of R and stages of V run STAGES - 1 chunks ahead.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef const void __attribute__((address_space(1)))* gptr_t;
typedef void __attribute__((address_space(3)))* lptr_t;

// three truncations: each piece takes the next 8 significant bits, the last one is exact
__device__ inline void split3(float v, unsigned& h, unsigned& m, unsigned& l) {
  h = __float_as_uint(v) & 0xFFFF0000u;
  const float r1 = v - __uint_as_float(h);
  m = __float_as_uint(r1) & 0xFFFF0000u;
  const float r2 = r1 - __uint_as_float(m);
  l = __float_as_uint(r2) & 0xFFFF0000u;
}

// eight consecutive k (values v[0..7]) of one column -> the 16-byte units of the three planes
__device__ inline void split3x8(const float* v, u32x4& hi, u32x4& mid, u32x4& lo) {
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    unsigned h0, m0, l0, h1, m1, l1;
    split3(v[2 * w], h0, m0, l0);
    split3(v[2 * w + 1], h1, m1, l1);
    hi[w] = (h0 >> 16) | h1;
    mid[w] = (m0 >> 16) | m1;
    lo[w] = (l0 >> 16) | l1;
  }
}

constexpr int PCH = 256;   // k per chunk of the plane layout
// entry offset of the unit that holds (k .. k + 7, column), k a multiple of 8, in plane 0 of its matrix;
// planes 1 and 2 lie LD * 256 and 2 * LD * 256 entries further on
template <int LD> __device__ inline long long plane_offset(int k, int col) {
  const int c = k / PCH, u = (k % PCH) / 8;
  return ((long long)(c * 3) * LD + col) * PCH + (((u & 16) | ((u ^ col) & 15)) * 8);
}

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding)
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}

// RG row groups of 64 rows per workgroup (4 RG wavefronts): with RG = 2 a stage of V serves 128 rows, and
// a launch fills half as many CUs at about the same speed, which leaves the others to whatever else is
// running (the products of another part of the batch).
template <int LD, int RG>
__global__ __launch_bounds__(NT * RG, 1) void chain_planes_kernel(const unsigned short* __restrict__ R, long long strideR, int ldr,
                                                          const float* __restrict__ R32, long long strideR32, int ldr32,
                                                          const float* __restrict__ Vin, long long strideVin,
                                                          const unsigned short* __restrict__ Pin, long long stridePin,
                                                          float* __restrict__ Vout, long long strideVout,
                                                          unsigned short* __restrict__ Pout, long long stridePout, int n,
                                                          const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int STAGES = 3;
  constexpr int STAGE_BYTES = 3 * LD * 512;
  constexpr int NW = 4 * RG;                     // wavefronts
  constexpr int VL = STAGE_BYTES / (1024 * NW);  // direct-to-LDS instructions per wave and chunk
  constexpr int NL = 8 + VL;                     // loads per wave and chunk
  constexpr int WROWS = ROWS * RG;               // rows per workgroup
  static_assert(STAGE_BYTES % (1024 * NW) == 0, "sketch width");
  static_assert(4 * WROWS * (LD + 1) * 4 <= STAGES * STAGE_BYTES, "the partial sums reuse the stages");
  extern __shared__ __align__(1024) unsigned char Vt[];       // [STAGES][STAGE_BYTES]
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63;
  const int wave = __builtin_amdgcn_readfirstlane(t >> 6);   // uniform: LDS destinations stay scalar
  const int li = lane & 15, lq = lane >> 4;
  const int kq = wave & 3, rg = wave >> 2;       // quarter of the k of a chunk, row group
  const int row0 = blockIdx.x * WROWS;           // first row of the workgroup
  const unsigned short* Rmat = R + (long long)b * strideR;
  const unsigned short* Rk = Rmat + 64 * kq + 8 * lq;                         // this lane's k within a chunk
  const long long rrow = (long long)(row0 + ROWS * rg + li) * ldr;             // ... and its row of block q = 0
  const char* Pmat = (const char*)(Pin + (long long)b * stridePin);
  const int poff = wave * 1024 + lane * 16;
  const int nchunks = n / PCH;
  // The workgroups of one matrix all read the same V.  Those that share an L2 (workgroups are dealt
  // round-robin to the 8 XCDs) sweep k in step, so that a chunk of V is fetched once per XCD and
  // found there by the others before the stream of R has pushed it out; the XCDs start at chunks of
  // their own and ask different memory channels at any moment.  The starting chunk is a function of
  // the row alone (128-row block modulo 8: the XCD of a 128-row workgroup when the row blocks of a
  // matrix are a multiple of 8), so that the order of summation, hence the bits of a result, do not
  // depend on the launch a matrix is part of.
  const int rot = (int)((unsigned)(((row0 / (2 * ROWS)) & 7) * nchunks) / 8u);

  u32x4 ra[STAGES][4][2];
  // Requests are unconditional, so that the compiler can count how many younger ones may stay in
  // flight at each wait.  Past the end the row and chunk offsets collapse to zero: the whole wave then
  // fetches the same few bytes (and nobody reads the result).
  auto load_chunk = [&](int slot, int c_want) {   // slot is a compile-time constant at every call site
    const bool valid = c_want < nchunks;          // uniform
    int c = c_want + rot;
    if (c >= nchunks) c -= nchunks;
    const long long pbase = valid ? (long long)c * STAGE_BYTES + poff : 0;
    const int pstep = valid ? 1024 * NW : 0;
#pragma unroll
    for (int i = 0; i < VL; ++i)
      __builtin_amdgcn_global_load_lds((gptr_t)(Pmat + pbase + i * pstep),
                                       (lptr_t)(Vt + slot * STAGE_BYTES + wave * 1024 + i * (1024 * NW)), 16, 0, 0);
    const long long rbase = valid ? rrow + c * PCH : 0;
    const long long qstep = valid ? 16ll * ldr : 0;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int h = 0; h < 2; ++h) ra[slot][q][h] = *(const u32x4*)(Rk + rbase + q * qstep + 32 * h);
  };

  f32x4 acc[4][NBLK][3];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
#pragma unroll
      for (int p = 0; p < 3; ++p) acc[q][j][p] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // Workgroup barrier without the release fence of __syncthreads() (which would wait for every
  // outstanding load): this wave's share of the next stage has landed (vmcnt), its reads of the stage
  // just used are complete (lgkmcnt).
  auto stage_barrier = [&]() {
    wait_vmcnt<NL * (STAGES - 2)>();
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
#pragma unroll
  for (int d = 0; d < STAGES - 1; ++d) load_chunk(d, d);
  stage_barrier();
  // fragment addresses within a stage: row (plane, column 16 jb + li), unit 8 w + 4 h + lq with its low bits xor li
  const unsigned char* fr = Vt + li * 512 + (kq >> 1) * 256;
  const int fu0 = (((8 * kq + lq) ^ li) & 15) * 16, fu1 = (((8 * kq + 4 + lq) ^ li) & 15) * 16;
  auto step = [&](auto dtag, int c) {   // chunk c, in ring slot d = c % STAGES
    constexpr int d = decltype(dtag)::value;
    __builtin_amdgcn_sched_barrier(0);
    load_chunk((d + STAGES - 1) % STAGES, c + STAGES - 1);   // into the stage chunk c - 1 was read from
    __builtin_amdgcn_sched_barrier(0);
    // the fragments of one half of the wave's k at a time (with two wavefronts per SIMD the other one
    // covers the wait)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      u32x4 fb[3][NBLK];
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
          fb[p][j] = *(const u32x4*)(fr + d * STAGE_BYTES + (p * LD + 16 * j) * 512 + (h ? fu1 : fu0));
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q)
            acc[q][j][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ra[d][q][h]),
                                                                   __builtin_bit_cast(bf16x8, fb[p][j]), acc[q][j][p], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    stage_barrier();
  };
  const int nfull = nchunks / STAGES * STAGES;
  for (int c0 = 0; c0 < nfull; c0 += STAGES)
    unrolled<STAGES>([&](auto dt) { step(dt, c0 + decltype(dt)::value); });
  unrolled<STAGES - 1>([&](auto dt) {
    if (nfull + decltype(dt)::value < nchunks) step(dt, nfull + decltype(dt)::value);
  });
  wait_vmcnt<0>();   // the requests past the end write into this workgroup's LDS: none may outlive it
  __syncthreads();   // ... nor the reuse of the stages below
  // partial sums of this wave's k (small pieces first), added up in wave order
  float (*red)[WROWS][LD + 1] = (float (*)[WROWS][LD + 1])Vt;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        red[kq][ROWS * rg + 16 * q + 4 * lq + r][16 * j + li] = (acc[q][j][2][r] + acc[q][j][1][r]) + acc[q][j][0][r];
  __syncthreads();
  // thread = (column, eight consecutive rows): the rows are the k of the next product, so the thread
  // owns one 16-byte unit of each plane of the result
  const int col = t % LD, u8 = t / LD;
  if (u8 < WROWS / 8) {
    const float* Vb = Vin + (long long)b * strideVin;
    float o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int rl = 8 * u8 + e, row = row0 + rl;
      const float v = (red[0][rl][col] + red[1][rl][col]) + (red[2][rl][col] + red[3][rl][col]);
      // exact diagonal minus the rounded one
      const float dfix = R32[(long long)b * strideR32 + (long long)row * ldr32] -
                         bf16_bits_to_float(Rmat[(long long)row * ldr + row]);
      o[e] = v + dfix * Vb[(long long)row * LD + col];
      Vout[(long long)b * strideVout + (long long)row * LD + col] = o[e];
    }
    if (Pout) {
      u32x4 hi, mid, lo;
      split3x8(o, hi, mid, lo);
      unsigned short* P = Pout + (long long)b * stridePout + plane_offset<LD>(row0 + 8 * u8, col);
      *(u32x4*)P = hi;
      *(u32x4*)(P + (long long)LD * PCH) = mid;
      *(u32x4*)(P + 2ll * LD * PCH) = lo;
    }
  }
}

// V [count][n][LD] fp32 -> planes (the sketches of a call, once per call)
template <int LD>
__global__ __launch_bounds__(NT) void split_planes_kernel(const float* __restrict__ V, unsigned short* __restrict__ P, int n) {
  const long long mat = (long long)blockIdx.y * n * LD;
  const int task = blockIdx.x * NT + threadIdx.x;   // (unit of eight k, column)
  const int col = task % LD, u = task / LD;
  if (u >= n / 8) return;
  float v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) v[e] = V[mat + (long long)(8 * u + e) * LD + col];
  u32x4 hi, mid, lo;
  split3x8(v, hi, mid, lo);
  unsigned short* o = P + mat * 3 + plane_offset<LD>(8 * u, col);
  *(u32x4*)o = hi;
  *(u32x4*)(o + (long long)LD * PCH) = mid;
  *(u32x4*)(o + 2ll * LD * PCH) = lo;
}

// Variant for small matrices (n <= 2048), where the kernel above is latency bound for lack of
// workgroups: a workgroup owns only 16 rows of R and its four wavefronts split K between them
// (wave w takes the chunks c = w, w+4, ...), each staging its own chunks of V in a private LDS
// area (no workgroup barrier inside the loop); the four partial sums are added through LDS in a
// fixed order at the end.
template <int LD, bool RB>
__global__ __launch_bounds__(NT, 2) void chain_small_kernel(const typename RFrag<RB>::elem* __restrict__ R, long long strideR, int ldr,
                                                         const float* __restrict__ R32, long long strideR32, int ldr32,
                                                         const float* __restrict__ Vin, long long strideVin,
                                                         float* __restrict__ Vout, long long strideVout, int n,
                                                         const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int VS = LD + 4;
  constexpr int VL = KC * LD / 4 / 64;          // float4 loads per lane for one chunk of V
  __shared__ float Vs[4][2][KC][VS];             // [wave][double buffer]
  __shared__ float red[4][NBLK][4][64];
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int li = lane & 15, lq = lane >> 4;
  const int row0 = blockIdx.x * 16;
  const typename RFrag<RB>::elem* Rrow = R + (long long)b * strideR + (long long)(row0 + li) * ldr + 4 * lq;
  const float* Vb = Vin + (long long)b * strideVin;
  const int nchunks = n / KC;
  const int mine = (nchunks - wave + 3) / 4;     // chunks of this wave

  constexpr int DEPTH = 3;
  RFrag<RB> ra[DEPTH][4];
  f32x4 va[DEPTH][VL];
  auto load = [&](int slot, int i) {             // i-th chunk of this wave; slot is compile time
    if (i < mine) {
      const int c = wave + 4 * i;
#pragma unroll
      for (int s = 0; s < 4; ++s) ra[slot][s].load(Rrow + c * KC + 16 * s);
#pragma unroll
      for (int v = 0; v < VL; ++v) {
        const int idx = lane + 64 * v;
        va[slot][v] = *(const f32x4*)(Vb + (long long)(c * KC + idx / (LD / 4)) * LD + (idx % (LD / 4)) * 4);
      }
    }
  };
  constexpr int NACC = 8 / NBLK;   // independent accumulators, as in the kernel above
  f32x4 acc[NBLK][NACC];
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int u = 0; u < NACC; ++u) acc[j][u] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d) load(d, d);
  for (int i0 = 0; i0 < mine; i0 += DEPTH) {
#pragma unroll
    for (int d = 0; d < DEPTH; ++d) {
      const int i = i0 + d;
      if (i < mine) {                             // uniform within the wave
        load((d + DEPTH - 1) % DEPTH, i + DEPTH - 1);
        const int buf = i & 1;
#pragma unroll
        for (int v = 0; v < VL; ++v) {
          const int idx = lane + 64 * v;
          *(f32x4*)&Vs[wave][buf][idx / (LD / 4)][(idx % (LD / 4)) * 4] = va[d][v];
        }
        // wave-private LDS area: LDS operations of one wave complete in order, no barrier needed
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
          for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int j = 0; j < NBLK; ++j)
              acc[j][(4 * s + e) % NACC] = __builtin_amdgcn_mfma_f32_16x16x4f32(ra[d][s].get(e), Vs[wave][buf][16 * s + 4 * lq + e][j * 16 + li], acc[j][(4 * s + e) % NACC], 0, 0, 0);
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j) {
#pragma unroll
    for (int w = NACC / 2; w > 0; w >>= 1)
#pragma unroll
      for (int u = 0; u < w; ++u) acc[j][u] += acc[j][u + w];
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) red[wave][j][r][lane] = acc[j][0][r];
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int j = 0; j < NBLK; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        float v = (red[0][j][r][lane] + red[1][j][r][lane]) + (red[2][j][r][lane] + red[3][j][r][lane]);
        const int row = row0 + 4 * lq + r, col = j * 16 + li;
        if constexpr (RB) {   // exact diagonal minus the rounded one
          const float dfix = R32[(long long)b * strideR32 + (long long)row * ldr32] -
                             bf16_bits_to_float((unsigned short)R[(long long)b * strideR + (long long)row * ldr + row]);
          v += dfix * Vb[(long long)row * LD + col];
        }
        Vout[(long long)b * strideVout + (long long)row * LD + col] = v;
      }
  }
}

// Matrices of order 64 (after padding): the whole chain V_1 .. V_nv in one launch, one workgroup per
// matrix with R and the current V in LDS.  At this size a product is a few hundred FMAs per thread
// and a call is bound by the number of launches, of which this removes nv - 1 per iteration.
// Thread (row, group of 4 columns): 64 x LD / 4 tasks over 256 threads.
template <int LD>
__global__ __launch_bounds__(NT) void chain_tiny_kernel(const float* __restrict__ R, long long strideR, int ldr,
                                                       const float* __restrict__ V0, long long strideV0,
                                                       float* __restrict__ Vout, long long strideJ, long long strideB,
                                                       int nv, const Ctrl* __restrict__ ctrl) {
  constexpr int N = 64;
  constexpr int TASKS = N * LD / 4, T_IT = TASKS / NT;
  static_assert(TASKS % NT == 0, "sketch width");
  __shared__ float Rs[N][N + 1];
  __shared__ __align__(16) float Vs[2][N][LD];
  const int b = blockIdx.x, t = threadIdx.x;
  if (ctrl && ctrl[b].done) return;
  for (int idx = t; idx < N * N; idx += NT) Rs[idx / N][idx % N] = R[(long long)b * strideR + (long long)(idx / N) * ldr + idx % N];
  for (int idx = t; idx < N * LD / 4; idx += NT)
    *(f32x4*)&Vs[0][idx / (LD / 4)][(idx % (LD / 4)) * 4] = *(const f32x4*)(V0 + (long long)b * strideV0 + (long long)idx * 4);
  __syncthreads();
  int cur = 0;
  for (int j = 0; j < nv; ++j) {
    f32x4 acc[T_IT];
#pragma unroll
    for (int it = 0; it < T_IT; ++it) {
      const int task = t + it * NT, row = task / (LD / 4), c4 = (task % (LD / 4)) * 4;
      f32x4 a = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
      for (int k = 0; k < N; ++k) {
        const float r = Rs[row][k];
        const f32x4 v = *(const f32x4*)&Vs[cur][k][c4];
        a[0] = fmaf(r, v[0], a[0]); a[1] = fmaf(r, v[1], a[1]); a[2] = fmaf(r, v[2], a[2]); a[3] = fmaf(r, v[3], a[3]);
      }
      acc[it] = a;
    }
#pragma unroll
    for (int it = 0; it < T_IT; ++it) {
      const int task = t + it * NT, row = task / (LD / 4), c4 = (task % (LD / 4)) * 4;
      *(f32x4*)&Vs[cur ^ 1][row][c4] = acc[it];
      *(f32x4*)(Vout + (long long)j * strideJ + (long long)b * strideB + (long long)row * LD + c4) = acc[it];
    }
    __syncthreads();
    cur ^= 1;
  }
}

// 64-row workgroups of a launch below which the 16-row kernel is taken
constexpr int small_below(bool rb) { return rb ? 128 : 256; }

template <bool RB>
int launch_chain_t(const typename RFrag<RB>::elem* R, long long strideR, int ldr, const float* R32, long long strideR32,
                   int ldr32, const float* Vin, long long strideVin, float* Vout, long long strideVout, int n, int ld,
                   int batch, const Ctrl* ctrl, hipStream_t s, int sel_batch) {
  if (n % KC || n % ROWS || ldr % 4 || batch <= 0) return PRISM_EINVAL;
  if (sel_batch <= 0) sel_batch = batch;   // the batch size that picks the kernel (a launch over several shape groups
                                           // passes the size of one group, so that every group gets the kernel of its own call)
  // 64-row workgroups leave most CUs idle on small batches of small matrices: 16-row ones there.
  // The bf16 kernels change over earlier: the 64-row one reads V once per 64 rows instead of once per
  // 16 and, beside other kernels, leaves them more of the chip (config 2, 192 workgroups of 64 rows:
  // 9.3 -> 7.5 us per launch and 3.55 -> 3.30 ms per step).
  if (ld <= 32 && (long long)(n / ROWS) * sel_batch < small_below(RB)) {
    const dim3 grid(n / 16, batch), block(NT);
    if (ld == 16) hipLaunchKernelGGL((chain_small_kernel<16, RB>), grid, block, 0, s, R, strideR, ldr, R32, strideR32, ldr32, Vin, strideVin, Vout, strideVout, n, ctrl);
    else hipLaunchKernelGGL((chain_small_kernel<32, RB>), grid, block, 0, s, R, strideR, ldr, R32, strideR32, ldr32, Vin, strideVin, Vout, strideVout, n, ctrl);
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
  }
  const dim3 grid(n / ROWS, batch), block(NT);
  if constexpr (RB) {
    return PRISM_EINVAL;   // large bf16 products take the plane kernel (launch_chain_planes)
  }
  else {
    if (ld == 16) hipLaunchKernelGGL((chain_kernel<16>), grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
    else if (ld == 32) hipLaunchKernelGGL((chain_kernel<32>), grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
    else if (ld == 64) hipLaunchKernelGGL((chain_kernel<64>), grid, block, 0, s, R, strideR, ldr, Vin, strideVin, Vout, strideVout, n, ctrl);
    else return PRISM_EINVAL;
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
  }
}

}  // namespace

// R: [batch][n][ldr] fp32 (n a multiple of 64), Vin/Vout: [n][ld] per matrix (strideVin may be 0)
int launch_chain(const float* R, long long strideR, int ldr, const float* Vin, long long strideVin, float* Vout,
                 long long strideVout, int n, int ld, int batch, const Ctrl* ctrl, hipStream_t s, int sel_batch) {
  return launch_chain_t<false>(R, strideR, ldr, nullptr, 0, 0, Vin, strideVin, Vout, strideVout, n, ld, batch, ctrl, s, sel_batch);
}

// V_j = R V_{j-1}, j = 1 .. nv, for matrices of order 64: V0 [64][ld] per matrix (strideV0 may be 0),
// Vout[j - 1] at Vout + (j - 1) * strideJ + b * strideB
int launch_chain_tiny(const float* R, long long strideR, int ldr, const float* V0, long long strideV0, float* Vout,
                      long long strideJ, long long strideB, int nv, int ld, int batch, const Ctrl* ctrl, hipStream_t s) {
  if (batch <= 0 || nv <= 0) return PRISM_EINVAL;
  if (ld == 16) hipLaunchKernelGGL(chain_tiny_kernel<16>, dim3(batch), dim3(NT), 0, s, R, strideR, ldr, V0, strideV0, Vout, strideJ, strideB, nv, ctrl);
  else if (ld == 32) hipLaunchKernelGGL(chain_tiny_kernel<32>, dim3(batch), dim3(NT), 0, s, R, strideR, ldr, V0, strideV0, Vout, strideJ, strideB, nv, ctrl);
  else if (ld == 64) hipLaunchKernelGGL(chain_tiny_kernel<64>, dim3(batch), dim3(NT), 0, s, R, strideR, ldr, V0, strideV0, Vout, strideJ, strideB, nv, ctrl);
  else return PRISM_EINVAL;
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

// Shapes the bf16 kernels take: sketch width up to 32, rows of Rb in 16-byte loads, and K in chunks
// of 128 unless the 16-row kernel applies.
bool chain_takes_small_kernel(int n, int ld, int batch, bool rb) {
  return ld <= 32 && (long long)(n / ROWS) * batch < small_below(rb);
}

bool chain_bf16_supported(int n, int ld, int batch, int ldr) {
  const bool small = ld <= 32 && (long long)(n / ROWS) * batch < small_below(true);
  return (ld == 16 || ld == 32) && ldr % 8 == 0 && n % KC == 0 && (small || n % PCH == 0);
}

// 64-row kernel for bf16 R: V comes as fp32 (for the diagonal term) and as planes; the result is written
// as fp32 and, when Pout is given, as planes for the next product.  n a multiple of 256.
int launch_chain_planes(const unsigned short* Rb, long long strideR, int ldr, const float* D, long long strideD, int ldd,
                        const float* Vin, long long strideVin, const unsigned short* Pin, long long stridePin, float* Vout,
                        long long strideVout, unsigned short* Pout, long long stridePout, int n, int ld, int batch,
                        const Ctrl* ctrl, hipStream_t s, int sel_batch) {
  if (!Rb || !D || !Vin || !Pin || !Vout || n % PCH || ldr % 8 || batch <= 0 || (ld != 16 && ld != 32)) return PRISM_EINVAL;
  const int lds = 3 * 3 * ld * 512;   // STAGES stages of three planes, 256 k each
  // 128-row workgroups when they still fill at least half the chip (judged by sel_batch, see launch_chain)
  const bool two = n % (2 * ROWS) == 0 && (long long)(n / (2 * ROWS)) * (sel_batch > 0 ? sel_batch : batch) >= 128;
  const void* kern = two ? (ld == 16 ? (const void*)chain_planes_kernel<16, 2> : (const void*)chain_planes_kernel<32, 2>)
                         : (ld == 16 ? (const void*)chain_planes_kernel<16, 1> : (const void*)chain_planes_kernel<32, 1>);
  const int rc = allow_dynamic_lds(kern, lds);
  if (rc != PRISM_OK) return rc;
  const dim3 grid(n / (two ? 2 * ROWS : ROWS), batch), block(two ? 2 * NT : NT);
#define PRISM_LAUNCH_PLANES(LD_, RG_) hipLaunchKernelGGL((chain_planes_kernel<LD_, RG_>), grid, block, lds, s, Rb, strideR, ldr, D, strideD, ldd, Vin, strideVin, Pin, stridePin, Vout, strideVout, Pout, stridePout, n, ctrl)
  if (two) { if (ld == 16) PRISM_LAUNCH_PLANES(16, 2); else PRISM_LAUNCH_PLANES(32, 2); }
  else { if (ld == 16) PRISM_LAUNCH_PLANES(16, 1); else PRISM_LAUNCH_PLANES(32, 1); }
#undef PRISM_LAUNCH_PLANES
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

// V [count][n][ld] fp32 -> bf16 planes [count][n / 128][3][ld][128]
int launch_split_planes(const float* V, unsigned short* P, int n, int ld, int count, hipStream_t s) {
  if (!V || !P || n % PCH || count <= 0 || (ld != 16 && ld != 32)) return PRISM_EINVAL;
  const dim3 grid((unsigned)(((long long)n / 8 * ld + NT - 1) / NT), count), block(NT);
  if (ld == 16) hipLaunchKernelGGL((split_planes_kernel<16>), grid, block, 0, s, V, P, n);
  else hipLaunchKernelGGL((split_planes_kernel<32>), grid, block, 0, s, V, P, n);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

// Same product with R read from its bf16 copy Rb and the diagonal from D (see common.h): the 16-row
// kernel only (chain_takes_small_kernel); larger launches go through launch_chain_planes
int launch_chain_bf16(const unsigned short* Rb, long long strideR, int ldr, const float* D, long long strideD, int ldd,
                      const float* Vin, long long strideVin, float* Vout, long long strideVout, int n, int ld, int batch,
                      const Ctrl* ctrl, hipStream_t s, int sel_batch) {
  if (!Rb || !D || !chain_bf16_supported(n, ld, sel_batch > 0 ? sel_batch : batch, ldr)) return PRISM_EINVAL;
  return launch_chain_t<true>(Rb, strideR, ldr, D, strideD, ldd, Vin, strideVin, Vout, strideVout, n, ld, batch, ctrl, s, sel_batch);
}

}  // namespace prism
