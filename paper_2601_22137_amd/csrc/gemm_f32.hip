// fp32 / fp64 GEMMs on the CDNA4 matrix cores (v_mfma_f32_16x16x4_f32, v_mfma_f64_16x16x4_f64)
// with the epilogues of the PRISM iterations fused in (Table 1 of the paper: residual
// R = I - G, polynomial Q = R/2 + alpha R^2, update X + X Q, inverse-Newton factors).
//
// One workgroup = 256 threads = 4 wavefronts computes one TM x TN tile of C for one matrix of
// the batch.  K is consumed in slabs of BK = 16 staged through LDS in K-major order
// (As[k][m], Bs[k][n]) and double buffered: the global loads of slab t+1 are in flight while
// the MFMAs of slab t run.  All operand sizes are padded to tile multiples by the caller, so
// the main loop has no bounds checks; masks are applied in the epilogue only.
#include <type_traits>

#include <cstdlib>

#include "common.h"

namespace prism {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x2 __attribute__((ext_vector_type(2)));

constexpr int BK = 16;
constexpr int NT = 256;

__host__ __device__ constexpr int lds_ld(int t) { return ((t + 31) / 32) * 32 + 16; }

template <typename T> struct Vec16;
template <> struct Vec16<float> { typedef f32x4 type; static constexpr int N = 4; };
template <> struct Vec16<double> { typedef f64x2 type; static constexpr int N = 2; };

__device__ inline f32x4 mfma(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}
__device__ inline f64x4 mfma(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}
template <typename T> struct Acc;
template <> struct Acc<float> { typedef f32x4 type; };
template <> struct Acc<double> { typedef f64x4 type; };

// Row of the 16x16 result held in register r of lane l (column is l % 16).
template <typename TC> __device__ inline int acc_row(int lane, int r);
template <> __device__ inline int acc_row<float>(int lane, int r) { return 4 * (lane >> 4) + r; }
template <> __device__ inline int acc_row<double>(int lane, int r) { return 4 * r + (lane >> 4); }

__device__ inline float apow(float alpha, int p) { return p == 0 ? 1.0f : (p == 1 ? alpha : alpha * alpha); }

// Applies the fused epilogue to one element, stores it, returns its contribution to the residual
// sum; `out` receives the stored value (for the mirrored store of the symmetric variants).
template <typename TC>
__device__ inline TC epilogue(const GemmDesc& g, int b, int i, int j, TC acc, float alpha, TC& out) {
  const long long oc = (long long)b * g.strideC + (long long)i * g.ldc + j;
  switch (g.epi) {
    case EPI_STORE:
      if (g.acc_neg) acc = -acc;
      ((TC*)g.C)[oc] = acc;
      out = acc;
      return 0;
    case EPI_RESIDUAL: {
      TC r = (i < g.n_true && j < g.n_true) ? ((i == j ? (TC)1 : (TC)0) - acc) : (TC)0;
      ((TC*)g.C)[oc] = r;
      out = r;
      return r * r;
    }
    case EPI_POLYQ: {
      const float rin = ((const float*)g.Cin)[(long long)b * g.strideCin + (long long)i * g.ldcin + j];
      const float q = g.c1 * rin + alpha * (float)acc;
      ((float*)g.C)[oc] = q;
      out = (TC)q;
      return 0;
    }
    case EPI_AXPY: {
      const float cin = ((const float*)g.Cin)[(long long)b * g.strideCin + (long long)i * g.ldcin + j];
      const float wc = g.cin_one_minus_alpha ? (1.0f - alpha) : g.c_in * apow(alpha, g.cin_alpha_pow);
      const float wa = g.acc_neg ? -apow(alpha, g.coef_is_alpha) : apow(alpha, g.coef_is_alpha);
      float v = wc * cin + wa * (float)acc;
      if (g.Cin2) v += apow(alpha, g.cin2_alpha_pow) * g.Cin2[(long long)b * g.strideCin + (long long)i * g.ldcin + j];
      ((float*)g.C)[oc] = v;
      out = (TC)v;
      return 0;
    }
    case EPI_MNEXT: {
      const bool in = (i < g.n_true && j < g.n_true);
      if (g.Cin) acc += ((const TC*)g.Cin)[(long long)b * g.strideCin + (long long)i * g.ldcin + j];
      const TC mval = in ? acc : (TC)0;
      ((TC*)g.C)[oc] = mval;
      const TC r = in ? ((i == j ? (TC)1 : (TC)0) - acc) : (TC)0;
      g.R32out[(long long)b * g.strideR + (long long)i * g.ldr + j] = (float)r;
      out = mval;
      return r * r;
    }
  }
  out = 0;
  return 0;
}

template <typename TC, typename TB, int TM, int TN, int WGM, int WGN, bool A_KM, bool SYM>
__global__ __launch_bounds__(NT, 2) void gemm_kernel(GemmDesc g) {
  constexpr int LDA = lds_ld(TM), LDB = lds_ld(TN);
  constexpr int WTM = TM / WGM, WTN = TN / WGN;  // wave tile
  constexpr int BM = WTM / 16, BN = WTN / 16;    // 16x16 blocks per wave
  static_assert(WGM * WGN == 4 && BM >= 1 && BN >= 1, "bad tiling");
  __shared__ TC As[2][BK][LDA];
  __shared__ TC Bs[2][BK][LDB];
  __shared__ TC red[4];

  // SYM (square fp32 products whose exact result is symmetric): only the tiles on and above the
  // diagonal are computed; every off-diagonal tile is also stored mirrored.
  const int tiles_m = g.M / TM, tiles_n = g.N / TN;
  const int per_mat = SYM ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  const int total = per_mat * g.batch;
  int wg = blockIdx.x;
  if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);  // one XCD = one contiguous tile range
  const int b = wg / per_mat;
  const int rem = wg - b * per_mat;
  int tm, tn;
  if (SYM) {
    int left = rem;
    tm = 0;
    while (left >= tiles_m - tm) { left -= tiles_m - tm; ++tm; }
    tn = tm + left;
  } else if (g.tile_blocks) {
    // blocks of 8 x 8 tiles in sequence: the 64 tiles an XCD works on at a time (32 CUs, two workgroups
    // each) share 8 row panels and 8 column panels; row by row they are one row panel and 64 column panels
    const int blk = rem >> 6, w = rem & 63, nbn = tiles_n >> 3;
    tm = (blk / nbn) * 8 + (w >> 3);
    tn = (blk % nbn) * 8 + (w & 7);
  } else {
    tm = rem / tiles_n;
    tn = rem - tm * tiles_n;
  }
  const int cb = g.ctrl_fixed ? 0 : b;   // split-K launches: every batch entry is a part of the same matrix
  if (g.ctrl && g.ctrl[cb].done) return;
  // block Gauss-Jordan: the pivot row / column block has launches of its own
  if ((tm * TM >= g.skip_m0 && tm * TM < g.skip_m1) || (tn * TN >= g.skip_n0 && tn * TN < g.skip_n1)) return;
  const float alpha = g.ctrl ? g.ctrl[cb].alpha : 1.0f;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm0 = (wave / WGN) * WTM, wn0 = (wave % WGN) * WTN;
  const int m0 = tm * TM, n0 = tn * TN;
  const float* Ab = (const float*)g.A + (long long)b * g.strideA;
  const TB* Bb = (const TB*)g.B + (long long)b * g.strideB;

  // staging registers
  constexpr int A_LOADS = TM * BK / 4;                       // float4 loads per slab
  constexpr int A_IT = (A_LOADS + NT - 1) / NT;
  constexpr int BV = Vec16<TB>::N;
  constexpr int B_LOADS = TN * BK / BV;
  constexpr int B_IT = (B_LOADS + NT - 1) / NT;
  // two register sets: the loads of slab t+2 are issued while slab t is multiplied and slab t+1
  // waits in the other set (one slab of MFMAs is shorter than the memory latency under load)
  f32x4 ra[2][A_IT];
  typename Vec16<TB>::type rb[2][B_IT];

  auto load_slab = [&](int set, int k0) {   // set is a compile-time constant at every call site
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int idx = t + it * NT;
      if (A_LOADS % NT == 0 || idx < A_LOADS) {
        if (A_KM) {
          const int kr = idx / (TM / 4), c4 = idx % (TM / 4);
          ra[set][it] = *(const f32x4*)(Ab + (long long)(k0 + kr) * g.lda + m0 + c4 * 4);
        } else {
          const int row = idx / (BK / 4), c4 = idx % (BK / 4);
          ra[set][it] = *(const f32x4*)(Ab + (long long)(m0 + row) * g.lda + k0 + c4 * 4);
        }
      }
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int idx = t + it * NT;
      if (B_LOADS % NT == 0 || idx < B_LOADS) {
        const int kr = idx / (TN / BV), c = idx % (TN / BV);
        rb[set][it] = *(const typename Vec16<TB>::type*)(Bb + (long long)(k0 + kr) * g.ldb + n0 + c * BV);
      }
    }
  };
  auto store_slab = [&](int set, int buf) {
#pragma unroll
    for (int it = 0; it < A_IT; ++it) {
      const int idx = t + it * NT;
      if (A_LOADS % NT == 0 || idx < A_LOADS) {
        if (A_KM) {
          const int kr = idx / (TM / 4), c4 = idx % (TM / 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) As[buf][kr][c4 * 4 + e] = (TC)ra[set][it][e];
        } else {
          const int row = idx / (BK / 4), c4 = idx % (BK / 4);
#pragma unroll
          for (int e = 0; e < 4; ++e) As[buf][c4 * 4 + e][row] = (TC)ra[set][it][e];
        }
      }
    }
#pragma unroll
    for (int it = 0; it < B_IT; ++it) {
      const int idx = t + it * NT;
      if (B_LOADS % NT == 0 || idx < B_LOADS) {
        const int kr = idx / (TN / BV), c = idx % (TN / BV);
#pragma unroll
        for (int e = 0; e < BV; ++e) Bs[buf][kr][c * BV + e] = (TC)rb[set][it][e];
      }
    }
  };

  typename Acc<TC>::type acc[BM][BN];
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j) acc[i][j] = (typename Acc<TC>::type){0, 0, 0, 0};

  // Long fp32 sums are accumulated in two levels (partial sums of 256 terms inside the matrix
  // core accumulator, then added up in registers): the rounding error then grows like the square
  // root of the chunk length instead of that of K, which the 1e-5 parity bar needs at K = 8192.
  constexpr bool FLUSH = sizeof(TC) == 4 && BM * BN <= 16;
  typename Acc<TC>::type ksum[FLUSH ? BM : 1][FLUSH ? BN : 1];
  if (FLUSH) {
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j) ksum[i][j] = (typename Acc<TC>::type){0, 0, 0, 0};
  }
  const int KT = g.K / BK;
  // Past the end the last slab is fetched (and staged) again, unused: no branch around the loads,
  // so that the compiler can count the younger loads that may stay in flight at each wait.
  auto kclamp = [&](int kt) { return (kt < KT ? kt : KT - 1) * BK; };
  // barrier for the LDS tiles only: __syncthreads() would also wait for the loads in flight
  auto lds_barrier = [&]() {
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
  };
  load_slab(0, 0);
  store_slab(0, 0);
  load_slab(1, kclamp(1));
  lds_barrier();
  const int lr = lane & 15, lk = lane >> 4;
  auto slab = [&](auto ptag, int kt) {   // slab kt, P = kt & 1: LDS buffer P, next slab in register set P ^ 1
    constexpr int P = decltype(ptag)::value;
    load_slab(P, kclamp(kt + 2));
    __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of the MFMAs
#pragma unroll
    for (int kk = 0; kk < BK / 4; ++kk) {
      TC a[BM], bb[BN];
#pragma unroll
      for (int i = 0; i < BM; ++i) a[i] = As[P][kk * 4 + lk][wm0 + i * 16 + lr];
#pragma unroll
      for (int j = 0; j < BN; ++j) bb[j] = Bs[P][kk * 4 + lk][wn0 + j * 16 + lr];
#pragma unroll
      for (int i = 0; i < BM; ++i)
#pragma unroll
        for (int j = 0; j < BN; ++j) acc[i][j] = mfma(a[i], bb[j], acc[i][j]);
    }
    store_slab(P ^ 1, P ^ 1);
    lds_barrier();
  };
  // Two nested loops, so that inside the inner one the accumulators are touched by MFMAs only;
  // the partial sums are closed between inner loops.
  constexpr int CHUNK = FLUSH ? 16 : (1 << 30);   // slabs per partial sum (fp32: 256 k); even
  for (int kt0 = 0; kt0 < KT; kt0 += CHUNK) {
    const int kt1 = (FLUSH && kt0 + CHUNK < KT) ? kt0 + CHUNK : KT;
    int kt = kt0;
    for (; kt + 1 < kt1; kt += 2) {
      slab(std::integral_constant<int, 0>{}, kt);
      slab(std::integral_constant<int, 1>{}, kt + 1);
    }
    if (kt < kt1) slab(std::integral_constant<int, 0>{}, kt);
    if (FLUSH) {
#pragma unroll
      for (int i = 0; i < BM; ++i)
#pragma unroll
        for (int j = 0; j < BN; ++j) {
          ksum[i][j] += acc[i][j];
          acc[i][j] = (typename Acc<TC>::type){0, 0, 0, 0};
        }
    }
  }
  if (FLUSH) {
#pragma unroll
    for (int i = 0; i < BM; ++i)
#pragma unroll
      for (int j = 0; j < BN; ++j) acc[i][j] = ksum[i][j];
  }

  TC part = 0;
#pragma unroll
  for (int i = 0; i < BM; ++i)
#pragma unroll
    for (int j = 0; j < BN; ++j) {
      const int gj = n0 + wn0 + j * 16 + lr;
      typename Acc<TC>::type outv;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const int gi = m0 + wm0 + i * 16 + acc_row<TC>(lane, r);
        TC o;
        part += epilogue<TC>(g, b, gi, gj, acc[i][j][r], alpha, o);
        outv[r] = o;
      }
      if (SYM && tm != tn) {
        // the lane holds four consecutive rows of one column: one 16-byte store in the mirror image
        if (g.sym_skew_bound > 0 && ((m0 < g.sym_skew_bound) != (n0 < g.sym_skew_bound))) outv = -outv;
        const int gi0 = m0 + wm0 + i * 16 + 4 * (lane >> 4);
        *(typename Acc<TC>::type*)((TC*)g.C + (long long)b * g.strideC + (long long)gj * g.ldc + gi0) = outv;
      }
    }
  if (SYM && tm != tn) part *= (TC)2;
  if (g.epi == EPI_RESIDUAL || g.epi == EPI_MNEXT) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
    if (lane == 0) red[wave] = part;
    __syncthreads();
    if (t == 0) g.rho_part[(long long)b * per_mat + rem] = (float)(red[0] + red[1] + red[2] + red[3]);
  }
}

template <typename TC, typename TB, int TM, int TN, int WGM, int WGN>
int launch_cfg(const GemmDesc& g, hipStream_t s) {
  if (g.M % TM || g.N % TN || g.K % BK || g.lda % 4 || g.ldb % 4) return PRISM_EINVAL;
  const int tm = g.M / TM, tn = g.N / TN;
  int total = tm * tn * g.batch;
  if (total <= 0) return PRISM_EINVAL;
  if constexpr (sizeof(TC) == 4 && TM == TN) {
    if (g.sym) {
      if (g.M != g.N || g.epi == EPI_MNEXT || g.ldc % 4) return PRISM_EINVAL;
      total = tm * (tm + 1) / 2 * g.batch;
      if (g.a_km)
        hipLaunchKernelGGL((gemm_kernel<TC, TB, TM, TN, WGM, WGN, true, true>), dim3(total), dim3(NT), 0, s, g);
      else
        hipLaunchKernelGGL((gemm_kernel<TC, TB, TM, TN, WGM, WGN, false, true>), dim3(total), dim3(NT), 0, s, g);
      return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
    }
  }
  if (g.sym) return PRISM_EINVAL;
  static const int no_blocks = ab_switch("PRISM_F32_NO_TILE_BLOCKS");
  GemmDesc gb = g;
  gb.tile_blocks = !no_blocks && tm % 8 == 0 && tn % 8 == 0 && tm * tn > 64;
  if (g.a_km)
    hipLaunchKernelGGL((gemm_kernel<TC, TB, TM, TN, WGM, WGN, true, false>), dim3(total), dim3(NT), 0, s, gb);
  else
    hipLaunchKernelGGL((gemm_kernel<TC, TB, TM, TN, WGM, WGN, false, false>), dim3(total), dim3(NT), 0, s, gb);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

}  // namespace

int launch_gemm_f32(const GemmDesc& g, int tile_m, int tile_n, hipStream_t s) {
  if (tile_m == 128 && tile_n == 128) return launch_cfg<float, float, 128, 128, 2, 2>(g, s);
  if (tile_m == 64 && tile_n == 64) return launch_cfg<float, float, 64, 64, 2, 2>(g, s);
  if (tile_m == 128 && tile_n == 64) return launch_cfg<float, float, 128, 64, 4, 1>(g, s);
  if (tile_m == 128 && tile_n == 32) return launch_cfg<float, float, 128, 32, 4, 1>(g, s);
  if (tile_m == 128 && tile_n == 16) return launch_cfg<float, float, 128, 16, 4, 1>(g, s);
  if (tile_m == 64 && tile_n == 32) return launch_cfg<float, float, 64, 32, 4, 1>(g, s);
  if (tile_m == 64 && tile_n == 16) return launch_cfg<float, float, 64, 16, 4, 1>(g, s);
  return PRISM_EINVAL;
}

int launch_gemm_f64a(const GemmDesc& g, int tile_m, int tile_n, hipStream_t s) {
  if (g.a_km) return PRISM_EINVAL;
  if (tile_m == 64 && tile_n == 64) return launch_cfg<double, double, 64, 64, 2, 2>(g, s);
  return PRISM_EINVAL;
}

}  // namespace prism
