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
// slabs of 64 staged through LDS rows padded to 144 bytes (conflict-free 16-byte reads), double
// buffered.  With a second A operand (the low half of a split-bf16 iterate) the K loop simply
// runs over both halves against the same B.
#include "common.h"

namespace prism {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16x4 __attribute__((ext_vector_type(4)));

constexpr int BK = 64;
constexpr int LDK = BK + 8;  // LDS row stride in elements (144 bytes)
constexpr int NT = 256;

__device__ inline unsigned short f2bf(float x) {
  unsigned int u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);  // round to nearest even (inputs are finite here)
  return (unsigned short)(u >> 16);
}
__device__ inline float bf2f(unsigned short h) { return __uint_as_float(((unsigned int)h) << 16); }

template <int T, int EPI>
__global__ __launch_bounds__(NT) void gemm_bf16_kernel(Bf16Desc g) {
  constexpr int WT = T / 2;        // wave tile (2 x 2 waves)
  constexpr int NB = WT / 32;      // 32x32 blocks per wave and dimension
  constexpr int LOADS = T * 8 / NT;  // 16-byte chunks per thread, operand and slab
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned short* As = (unsigned short*)smem;       // [2][T][LDK]
  unsigned short* Bs = As + 2 * T * LDK;            // [2][T][LDK]
  __shared__ float red[4];

  const int tiles_m = g.M / T, tiles_n = g.N / T;
  const int per_mat = tiles_m * tiles_n;
  const int total = per_mat * g.batch;
  int wg = blockIdx.x;
  if ((total & 7) == 0) wg = (wg & 7) * (total >> 3) + (wg >> 3);  // one XCD = contiguous tile range
  const int b = wg / per_mat;
  const int rem = wg - b * per_mat;
  const int tm = rem / tiles_n, tn = rem - tm * tiles_n;
  if (g.ctrl && g.ctrl[b].done) return;
  const float alpha = g.ctrl ? g.ctrl[b].alpha : 1.0f;

  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm0 = (wave >> 1) * WT, wn0 = (wave & 1) * WT;
  const int m0 = tm * T, n0 = tn * T;
  const unsigned short* A1 = g.A + (long long)b * g.strideA + (long long)m0 * g.lda;
  const unsigned short* A2 = g.A2 ? g.A2 + (long long)b * g.strideA + (long long)m0 * g.lda : nullptr;
  const unsigned short* Bb = g.B + (long long)b * g.strideB + (long long)n0 * g.ldb;

  const int KT1 = g.K / BK;
  const int KT = A2 ? 2 * KT1 : KT1;

  u32x4 ra[LOADS], rb[LOADS];
  auto load_slab = [&](int kt) {
    const unsigned short* Ap = (kt < KT1) ? A1 : A2;
    const int k0 = ((kt < KT1) ? kt : kt - KT1) * BK;
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
      const int idx = t + it * NT;
      const int row = idx >> 3, c = idx & 7;
      ra[it] = *(const u32x4*)(Ap + (long long)row * g.lda + k0 + c * 8);
      rb[it] = *(const u32x4*)(Bb + (long long)row * g.ldb + k0 + c * 8);
    }
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int it = 0; it < LOADS; ++it) {
      const int idx = t + it * NT;
      const int row = idx >> 3, c = idx & 7;
      *(u32x4*)(As + ((long long)buf * T + row) * LDK + c * 8) = ra[it];
      *(u32x4*)(Bs + ((long long)buf * T + row) * LDK + c * 8) = rb[it];
    }
  };

  f32x16 acc[NB][NB];
#pragma unroll
  for (int i = 0; i < NB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  load_slab(0);
  store_slab(0);
  __syncthreads();
  const int lr = lane & 31, lk = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) load_slab(kt + 1);
    const unsigned short* Ac = As + ((long long)cur * T + wm0 + lr) * LDK + lk;
    const unsigned short* Bc = Bs + ((long long)cur * T + wn0 + lr) * LDK + lk;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 a[NB], bb[NB];
#pragma unroll
      for (int i = 0; i < NB; ++i) a[i] = *(const bf16x8*)(Ac + i * 32 * LDK + kk * 16);
#pragma unroll
      for (int j = 0; j < NB; ++j) bb[j] = *(const bf16x8*)(Bc + j * 32 * LDK + kk * 16);
#pragma unroll
      for (int i = 0; i < NB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) store_slab(cur ^ 1);
    __syncthreads();
  }

  // epilogue: register r of lane l holds row (r/4)*8 + (l/32)*4 + r%4, column l%32 of a block
  float part = 0.0f;
  const float coef = g.coef_is_alpha ? alpha : 1.0f;
  const int rbase = (lane >> 5) * 4;
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
        } else {  // BEPI_APPLY
          u16x4 tr;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const long long o = (long long)b * g.strideCb + (long long)(gm + e) * g.ldcb + gn;
            float x = bf2f(g.Xhi[o]);
            if (g.Xlo) x += bf2f(g.Xlo[o]);
            x += coef * acc[i][j][rg * 4 + e];
            const unsigned short hi = f2bf(x);
            g.Cb[o] = hi;
            if (g.Cb2) g.Cb2[o] = f2bf(x - bf2f(hi));
            tr[e] = hi;
          }
          *(u16x4*)(g.Ct + (long long)b * g.strideCt + (long long)gn * g.ldct + gm) = tr;
        }
      }
    }
  if (EPI == BEPI_GRAM) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
    if (lane == 0) red[wave] = part;
    __syncthreads();
    if (t == 0) g.rho_part[(long long)b * per_mat + rem] = red[0] + red[1] + red[2] + red[3];
  }
}

template <int T, int EPI>
int launch_te(const Bf16Desc& g, hipStream_t s) {
  const int total = (g.M / T) * (g.N / T) * g.batch;
  const size_t lds = (size_t)4 * T * LDK * sizeof(unsigned short);
  static bool attr_set = false;  // per instantiation
  if (!attr_set) {
    if (hipFuncSetAttribute((const void*)gemm_bf16_kernel<T, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            (int)lds) != hipSuccess) {
      set_last_error("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed");
      return PRISM_EHIP;
    }
    attr_set = true;
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<T, EPI>), dim3(total), dim3(NT), lds, s, g);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

template <int T>
int launch_t(const Bf16Desc& g, hipStream_t s) {
  if (g.M % T || g.N % T || g.K % BK || g.lda % 8 || g.ldb % 8) return PRISM_EINVAL;
  if ((g.M / T) * (g.N / T) * g.batch <= 0) return PRISM_EINVAL;
  switch (g.epi) {
    case BEPI_STORE: return launch_te<T, BEPI_STORE>(g, s);
    case BEPI_GRAM: return launch_te<T, BEPI_GRAM>(g, s);
    case BEPI_POLYQ: return launch_te<T, BEPI_POLYQ>(g, s);
    case BEPI_APPLY: return launch_te<T, BEPI_APPLY>(g, s);
  }
  return PRISM_EINVAL;
}

}  // namespace

int launch_gemm_bf16(const Bf16Desc& g, int tile, hipStream_t s) {
  if (tile == 256) return launch_t<256>(g, s);
  if (tile == 128) return launch_t<128>(g, s);
  return PRISM_EINVAL;
}

}  // namespace prism
