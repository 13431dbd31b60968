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
// 24 significant bits: every fp32 entry is cut into three bf16 pieces (8 bits each, exact), staged
// in LDS as three planes Vt[plane][column][k], and R is multiplied by each plane; the partial
// products of two bf16 numbers are exact in fp32, so only the accumulation rounds.
//   A operand: lane (i = l % 16, g = l / 16) holds R[row i][k0 + 32 s + 8 g .. + 7]: its 16-byte load;
//   B operand: lane (j = l % 16, g) holds the same eight k of column j: one 16-byte LDS read.
//   A row of Vt is 128 k = 256 bytes plus 16 of padding (68 dwords: the 16 columns of a read hit
//   all 64 banks once).
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

template <int LD>
__global__ __launch_bounds__(NT, 2) void chain_bf16_kernel(const unsigned short* __restrict__ R, long long strideR, int ldr,
                                                        const float* __restrict__ R32, long long strideR32, int ldr32,
                                                        const float* __restrict__ Vin, long long strideVin,
                                                        float* __restrict__ Vout, long long strideVout, int n,
                                                        const Ctrl* __restrict__ ctrl) {
  constexpr int NBLK = LD / 16;
  constexpr int KCH = 128;
  constexpr int ROWB = 2 * KCH + 16;             // bytes per (plane, column)
  constexpr int DEPTH = 3;
  constexpr int V_TASKS = LD * (KCH / 8);        // (column, group of 8 k) per chunk
  constexpr int V_IT = V_TASKS / NT;
  static_assert(V_TASKS % NT == 0, "sketch width");
  __shared__ __align__(16) unsigned char Vt[2][3][LD][ROWB];
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int li = lane & 15, lq = lane >> 4;
  const int row0 = blockIdx.x * ROWS + wave * 16;
  const unsigned short* Rrow = R + (long long)b * strideR + (long long)(row0 + li) * ldr + 8 * lq;
  const float* Vb = Vin + (long long)b * strideVin;
  const int nchunks = n / KCH;
  const int rot = (int)(blockIdx.x % (unsigned)nchunks);   // see chain_kernel

  float vreg[DEPTH][V_IT][8];
  u32x4 ra[DEPTH][4];
  auto load_chunk = [&](int slot, int c_want) {   // unconditional, as in chain_kernel
    int c = (c_want < nchunks ? c_want : nchunks - 1) + rot;
    if (c >= nchunks) c -= nchunks;
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      const int col = idx % LD, kg = idx / LD;
#pragma unroll
      for (int e = 0; e < 8; ++e) vreg[slot][it][e] = Vb[(long long)(c * KCH + 8 * kg + e) * LD + col];
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) ra[slot][s] = *(const u32x4*)(Rrow + c * KCH + 32 * s);
  };
  auto store_v = [&](int slot, int buf) {
#pragma unroll
    for (int it = 0; it < V_IT; ++it) {
      const int idx = t + it * NT;
      const int col = idx % LD, kg = idx / LD;
      u32x4 hi, mid, lo;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        unsigned ph[2], pm[2], pl[2];
#pragma unroll
        for (int x = 0; x < 2; ++x) {
          // three truncations: each piece takes the next 8 significant bits, the last one is exact
          const float v = vreg[slot][it][2 * w + x];
          const unsigned h = __float_as_uint(v) & 0xFFFF0000u;
          const float r1 = v - __uint_as_float(h);
          const unsigned m = __float_as_uint(r1) & 0xFFFF0000u;
          const float r2 = r1 - __uint_as_float(m);
          ph[x] = h; pm[x] = m; pl[x] = __float_as_uint(r2);
        }
        hi[w] = (ph[0] >> 16) | ph[1];
        mid[w] = (pm[0] >> 16) | pm[1];
        lo[w] = (pl[0] >> 16) | (pl[1] & 0xFFFF0000u);
      }
      *(u32x4*)&Vt[buf][0][col][16 * kg] = hi;
      *(u32x4*)&Vt[buf][1][col][16 * kg] = mid;
      *(u32x4*)&Vt[buf][2][col][16 * kg] = lo;
    }
  };

  f32x4 acc[NBLK][3];
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int p = 0; p < 3; ++p) acc[j][p] = (f32x4){0.f, 0.f, 0.f, 0.f};
  auto lds_barrier = [&]() {   // see chain_kernel
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
#pragma unroll
  for (int d = 0; d < DEPTH - 1; ++d) load_chunk(d, d);
  store_v(0, 0);
  lds_barrier();
  auto step = [&](auto dtag, int c) {
    constexpr int d = decltype(dtag)::value;
    const int cur = c & 1;
    load_chunk((d + DEPTH - 1) % DEPTH, c + DEPTH - 1);
    // fragments of V one step ahead of their MFMAs (see chain_kernel)
    u32x4 fb[2][3][NBLK];
    auto read_v = [&](int s) {
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < NBLK; ++j) fb[s & 1][p][j] = *(const u32x4*)&Vt[cur][p][j * 16 + li][64 * s + 16 * lq];
    };
    read_v(0);
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      __builtin_amdgcn_sched_barrier(0);
      if (s + 1 < 4) read_v(s + 1);
      __builtin_amdgcn_sched_barrier(0);
      const bf16x8 a = __builtin_bit_cast(bf16x8, ra[d][s]);
#pragma unroll
      for (int p = 0; p < 3; ++p)
#pragma unroll
        for (int j = 0; j < NBLK; ++j)
          acc[j][p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, __builtin_bit_cast(bf16x8, fb[s & 1][p][j]), acc[j][p], 0, 0, 0);
    }
    store_v((d + 1) % DEPTH, cur ^ 1);
    lds_barrier();
  };
  const int nfull = nchunks / DEPTH * DEPTH;
  for (int c0 = 0; c0 < nfull; c0 += DEPTH)
    unrolled<DEPTH>([&](auto dt) { step(dt, c0 + decltype(dt)::value); });
  unrolled<DEPTH - 1>([&](auto dt) {
    if (nfull + decltype(dt)::value < nchunks) step(dt, nfull + decltype(dt)::value);
  });
  float dfix[4];   // exact diagonal minus the rounded one, rows of this lane
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int row = row0 + 4 * lq + r;
    dfix[r] = R32[(long long)b * strideR32 + (long long)row * ldr32] -
              bf16_bits_to_float(R[(long long)b * strideR + (long long)row * ldr + row]);
  }
#pragma unroll
  for (int j = 0; j < NBLK; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = row0 + 4 * lq + r, col = j * 16 + li;
      const float v = (acc[j][2][r] + acc[j][1][r]) + acc[j][0][r];   // small pieces first
      Vout[(long long)b * strideVout + (long long)row * LD + col] = v + dfix[r] * Vb[(long long)row * LD + col];
    }
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
  if constexpr (RB) {   // K in chunks of 128, rows in 16-byte loads
    if (n % 128 || ldr % 8) return PRISM_EINVAL;
    if (ld == 16) hipLaunchKernelGGL((chain_bf16_kernel<16>), grid, block, 0, s, R, strideR, ldr, R32, strideR32, ldr32, Vin, strideVin, Vout, strideVout, n, ctrl);
    else if (ld == 32) hipLaunchKernelGGL((chain_bf16_kernel<32>), grid, block, 0, s, R, strideR, ldr, R32, strideR32, ldr32, Vin, strideVin, Vout, strideVout, n, ctrl);
    else return PRISM_EINVAL;
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
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
  return (ld == 16 || ld == 32) && ldr % 8 == 0 && n % KC == 0 && (small || n % 128 == 0);
}

// Same product with R read from its bf16 copy Rb and the diagonal from D (see common.h)
int launch_chain_bf16(const unsigned short* Rb, long long strideR, int ldr, const float* D, long long strideD, int ldd,
                      const float* Vin, long long strideVin, float* Vout, long long strideVout, int n, int ld, int batch,
                      const Ctrl* ctrl, hipStream_t s, int sel_batch) {
  if (!Rb || !D || !chain_bf16_supported(n, ld, sel_batch > 0 ? sel_batch : batch, ldr)) return PRISM_EINVAL;
  return launch_chain_t<true>(Rb, strideR, ldr, D, strideD, ldd, Vin, strideVin, Vout, strideVout, n, ld, batch, ctrl, s, sel_batch);
}

}  // namespace prism
