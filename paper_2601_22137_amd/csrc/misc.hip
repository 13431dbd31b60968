// Entry and exit of the PRISM iterations: Frobenius norm of the input, initial iterates
// (paper Section 3: X_0 = A / ||A||_F; App. A.3: X_0 = I / c, M_0 = A / c^p with
// c = (2 ||A||_F / (p+1))^(1/p)), copy into the padded internal layouts, and the final
// un-scaling / copy-out (A^{1/2} = sqrt(s) X, A^{-1/2} = Y / sqrt(s)).  Matrix sign (Section 4)
// starts like the polar factor; the Chebyshev inverse (App. A.4) keeps A_s = A / ||A||_F, starts
// from X_0 = A_s^T and returns X / ||A||_F.
#include <cstdint>

#include "common.h"

namespace prism {
namespace {

constexpr int NT = 256;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ inline unsigned short f2bf(float x) {
  unsigned int u = __float_as_uint(x);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__device__ inline float bf2f(unsigned short h) { return __uint_as_float(((unsigned int)h) << 16); }

__device__ inline double load_src(const void* src, int dt, long long idx) {
  return dt == PRISM_BF16 ? (double)bf2f(((const unsigned short*)src)[idx]) : (double)((const float*)src)[idx];
}

// sumsq_part[b][blockIdx.x] = sum of squares of a strided share of matrix b (fp64).
// An inf or nan entry makes its partial non-finite, which the prepare step reports.
// bx in [0, gx): the share of the matrix, b: the matrix (the launch geometry of a single group, which
// the launches over several groups reproduce so that every matrix gets the same partial sums)
__device__ inline void sumsq_body(const PrepArgs& a, int bx, int b, int gx) {
  const long long total = (long long)a.m * a.n;
  const long long base = (long long)b * total;
  double acc = 0.0;
  const long long first = (long long)bx * NT + threadIdx.x, step = (long long)gx * NT;
  if (a.dt == PRISM_BF16 && (total & 7) == 0) {          // 16-byte loads: 8 bf16 at a time
    const u32x4* v = (const u32x4*)((const unsigned short*)a.src + base);
    for (long long i = first; i < total / 8; i += step) {
      const u32x4 w = v[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const double x0 = (double)__uint_as_float(w[e] << 16), x1 = (double)__uint_as_float(w[e] & 0xFFFF0000u);
        acc += x0 * x0 + x1 * x1;
      }
    }
  } else if (a.dt == PRISM_F32 && (total & 3) == 0) {
    const f32x4* v = (const f32x4*)((const float*)a.src + base);
    for (long long i = first; i < total / 4; i += step) {
      const f32x4 w = v[i];
#pragma unroll
      for (int e = 0; e < 4; ++e) acc += (double)w[e] * (double)w[e];
    }
  } else {
    for (long long i = first; i < total; i += step) {
      const double v = load_src(a.src, a.dt, base + i);
      acc += v * v;
    }
  }
  __shared__ double red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
  if (lane == 0) red[wave] = acc;
  __syncthreads();
  if (threadIdx.x == 0) a.sumsq_part[(long long)b * a.nsum + bx] = red[0] + red[1] + red[2] + red[3];
}
__global__ __launch_bounds__(NT) void sumsq_kernel(PrepArgs a) { sumsq_body(a, blockIdx.x, blockIdx.y, gridDim.x); }
// several shape groups in one launch: workgroup -> (group, matrix, share)
__global__ __launch_bounds__(NT) void sumsq_multi_kernel(PrepMulti m) {
  int w = blockIdx.x, gi = 0;
  while (gi + 1 < m.ngroups && w >= m.start[gi + 1]) ++gi;
  w -= m.start[gi];
  const PrepArgs& a = m.d[gi];
  sumsq_body(a, w % a.nsum, w / a.nsum, a.nsum);
}

// One workgroup per 64 x 64 tile of the padded internal iterate [Lp][Sp].
__global__ __launch_bounds__(NT) void prepare_kernel(PrepArgs a) {
  const int b = blockIdx.y;
  const int tiles_c = a.Sp / 64;
  const int tr = blockIdx.x / tiles_c, tc = blockIdx.x % tiles_c;
  double ss = 0.0;
  for (int i = 0; i < a.nsum; ++i) ss += a.sumsq_part[(long long)b * a.nsum + i];
  const bool finite = (ss == ss) && ss < 1.0e300;
  const bool zero = finite && ss == 0.0;
  const double norm = sqrt(ss);
  double scale = 0.0, cinv = 0.0;
  if (finite && !zero) {
    if (a.fn == PRISM_FN_SQRT_NEWTON) {
      scale = 1.0;                                             // App. A.2 starts from A itself
    } else if (a.fn == PRISM_FN_INV_ROOT) {
      const double cp = 2.0 * norm / (double)(a.root_p + 1);   // c^p
      scale = 1.0 / cp;
      cinv = pow(cp, -1.0 / (double)a.root_p);                 // 1 / c
    } else {
      scale = 1.0 / norm;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    Ctrl c;
    c.done = (finite && !zero) ? 0 : 1;
    c.iters = 0;
    c.status = !finite ? PRISM_INFO_NONFINITE : (zero ? PRISM_INFO_ZERO : PRISM_INFO_BUDGET);
    c.plain = 0;
    c.alpha = 0.0f; c.res0 = 0.0f; c.res1 = 0.0f; c.res2 = 0.0f;
    c.norm = norm; c.scale = scale;
    a.ctrl[b] = c;
    a.info[b].iters = 0;
    a.info[b].status = c.status;
  }
  if (blockIdx.x == 0) {
    for (int i = threadIdx.x; i <= PRISM_MAX_ITERS; i += NT) a.info[b].residual[i] = -1.0f;
    for (int i = threadIdx.x; i < PRISM_MAX_ITERS; i += NT) a.info[b].alpha[i] = 0.0f;
  }

  float rho = 0.0f;
  const long long mat = (long long)a.m * a.n;
  for (int e = threadIdx.x; e < 64 * 64; e += NT) {
    const int lr = e >> 6, lc = e & 63;
    const int r = tr * 64 + lr, c = tc * 64 + lc;   // position in the internal [Lp][Sp] iterate
    double v = 0.0;
    if (r < a.L && c < a.S) {
      const long long si = a.transpose ? ((long long)c * a.n + r) : ((long long)r * a.n + c);
      v = load_src(a.src, a.dt, (long long)b * mat + si) * scale;
    }
    const long long o = (long long)b * a.Lp * a.Sp + (long long)r * a.Sp + c;
    if (a.fn == PRISM_FN_SIGN) {
      a.X32[o] = (float)v;
    } else if (a.fn == PRISM_FN_SQRT_NEWTON) {   // X_0 = M_0 = A, Y_0 = I; the padding of M is the identity
      const bool in = (r < a.S && c < a.S);
      const float eye = (r == c) ? 1.0f : 0.0f;
      a.X32[o] = (float)v;
      a.Y32[o] = in ? eye : 0.0f;
      a.R32[o] = in ? (float)v : eye;
      const double res = in ? ((double)eye - v) : 0.0;
      rho += (float)(res * res);
    } else if (a.fn == PRISM_FN_INVERSE) {
      a.Y32[o] = (float)v;                                                                    // A_s
      a.X32[(long long)b * a.Lp * a.Sp + (long long)c * a.Sp + r] = (float)v;                 // X_0 = A_s^T
    } else if (a.fn == PRISM_FN_POLAR) {
      if (a.dt == PRISM_BF16) {
        const unsigned short hi = f2bf((float)v);
        a.Xa_hi[o] = hi;
        if (a.Xa_lo) a.Xa_lo[o] = f2bf((float)v - bf2f(hi));
      } else {
        a.X32[o] = (float)v;
      }
    } else if (a.fn == PRISM_FN_SQRT) {
      a.X32[o] = (float)v;
      a.Y32[o] = (r == c && r < a.S) ? 1.0f : 0.0f;
    } else {  // inverse root: v = M_0 entry
      const bool in = (r < a.S && c < a.S);
      const double eye = (r == c && in) ? 1.0 : 0.0;
      a.M64[o] = v;
      a.X32[o] = (float)(eye * cinv);
      const double res = in ? (eye - v) : 0.0;
      a.R32[o] = (float)res;
      rho += (float)(res * res);
    }
  }
  if (a.fn == PRISM_FN_INV_ROOT || a.fn == PRISM_FN_SQRT_NEWTON) {
    __shared__ float red[4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) rho += __shfl_down(rho, off, 64);
    if (lane == 0) red[wave] = rho;
    __syncthreads();
    if (threadIdx.x == 0)
      a.rho_part[(long long)b * gridDim.x + blockIdx.x] = red[0] + red[1] + red[2] + red[3];
  }
}

// bf16 polar, both sides multiples of 8: one workgroup per 64 x 64 tile of the CALLER's matrix.
// The tile is read with 16-byte loads along the caller's rows, scaled and split into high and low
// halves; a tall or square matrix goes straight into the internal [Lp][Sp] iterate, a wide one
// (the iterate is its transpose) through an LDS transpose, everything as 16-byte vectors.
__device__ inline void prepare_bf16_body(const PrepArgs& a, int bx, int b) {
  const int tiles_c = (a.transpose ? a.Lp : a.Sp) / 64;             // tiles over the padded, caller-oriented matrix
  const int tr = bx / tiles_c, tc = bx % tiles_c;
  double ss = 0.0;
  for (int i = 0; i < a.nsum; ++i) ss += a.sumsq_part[(long long)b * a.nsum + i];
  const bool finite = (ss == ss) && ss < 1.0e300;
  const bool zero = finite && ss == 0.0;
  const double norm = sqrt(ss);
  const float scale = (finite && !zero) ? (float)(1.0 / norm) : 0.0f;
  if (bx == 0 && threadIdx.x == 0) {
    Ctrl c;
    c.done = (finite && !zero) ? 0 : 1;
    c.iters = 0;
    c.status = !finite ? PRISM_INFO_NONFINITE : (zero ? PRISM_INFO_ZERO : PRISM_INFO_BUDGET);
    c.plain = 0;
    c.alpha = 0.0f; c.res0 = 0.0f; c.res1 = 0.0f; c.res2 = 0.0f;
    c.norm = norm; c.scale = scale;
    a.ctrl[b] = c;
    a.info[b].iters = 0;
    a.info[b].status = c.status;
  }
  if (bx == 0) {
    for (int i = threadIdx.x; i <= PRISM_MAX_ITERS; i += NT) a.info[b].residual[i] = -1.0f;
    for (int i = threadIdx.x; i < PRISM_MAX_ITERS; i += NT) a.info[b].alpha[i] = 0.0f;
  }
  const long long mat_int = (long long)a.Lp * a.Sp;
  __shared__ float tile_hi[64][65], tile_lo[64][65];
  const unsigned short* src = (const unsigned short*)a.src + (long long)b * a.m * a.n;
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int v = threadIdx.x + it * NT;          // 512 vectors of 8 per tile
    const int lr = v >> 3, lc = (v & 7) * 8;
    const int r = tr * 64 + lr, c = tc * 64 + lc;
    u32x4 w = {0u, 0u, 0u, 0u};
    if (r < a.m && c < a.n) w = *(const u32x4*)(src + (long long)r * a.n + c);
    u32x4 hi, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float x0 = __uint_as_float(w[e] << 16) * scale, x1 = __uint_as_float(w[e] & 0xFFFF0000u) * scale;
      const unsigned short h0 = f2bf(x0), h1 = f2bf(x1);
      const unsigned short l0 = f2bf(x0 - bf2f(h0)), l1 = f2bf(x1 - bf2f(h1));
      hi[e] = (unsigned)h0 | ((unsigned)h1 << 16);
      lo[e] = (unsigned)l0 | ((unsigned)l1 << 16);
      if (a.transpose) {
        tile_hi[lc + 2 * e][lr] = bf2f(h0); tile_hi[lc + 2 * e + 1][lr] = bf2f(h1);
        tile_lo[lc + 2 * e][lr] = bf2f(l0); tile_lo[lc + 2 * e + 1][lr] = bf2f(l1);
      }
    }
    if (!a.transpose) {  // rows / columns beyond the caller's matrix but inside the padded array are written as zeros
      const long long o = (long long)b * mat_int + (long long)r * a.Sp + c;
      *(u32x4*)(a.Xa_hi + o) = hi;
      if (a.Xa_lo) *(u32x4*)(a.Xa_lo + o) = lo;
    }
  }
  if (!a.transpose) return;
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int v = threadIdx.x + it * NT;
    const int lc = v >> 3, lr = (v & 7) * 8;      // row lc of the transposed tile, 8 consecutive source rows
    const int r = tr * 64 + lr, c = tc * 64 + lc;
    u32x4 hi, lo;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      hi[e] = (unsigned)f2bf(tile_hi[lc][lr + 2 * e]) | ((unsigned)f2bf(tile_hi[lc][lr + 2 * e + 1]) << 16);
      lo[e] = (unsigned)f2bf(tile_lo[lc][lr + 2 * e]) | ((unsigned)f2bf(tile_lo[lc][lr + 2 * e + 1]) << 16);
    }
    const long long o = (long long)b * mat_int + (long long)c * a.Sp + r;   // internal row = caller's column
    *(u32x4*)(a.Xa_hi + o) = hi;
    if (a.Xa_lo) *(u32x4*)(a.Xa_lo + o) = lo;
  }
}
__global__ __launch_bounds__(NT) void prepare_bf16_kernel(PrepArgs a) { prepare_bf16_body(a, blockIdx.x, blockIdx.y); }
__global__ __launch_bounds__(NT) void prepare_bf16_multi_kernel(PrepMulti m) {
  int w = blockIdx.x, gi = 0;
  while (gi + 1 < m.ngroups && w >= m.start[gi + 1]) ++gi;
  w -= m.start[gi];
  const PrepArgs& a = m.d[gi];
  const int tiles = (a.Lp / 64) * (a.Sp / 64);
  prepare_bf16_body(a, w % tiles, w / tiles);
}

// bf16 polar, both sides multiples of 8: the result is the high half of the iterate.  One workgroup
// per 64 x 64 tile of the caller's matrix: a tall or square one is copied with 16-byte vectors, a
// wide one (the iterate is its transpose) goes through an LDS transpose.
__device__ inline void finalize_bf16_body(const FinalArgs& a, int bx, int b) {
  const Ctrl c = a.ctrl[b];
  if (c.status == PRISM_INFO_NONFINITE || c.status == PRISM_INFO_ZERO) return;
  const int par = c.iters & 1;
  const unsigned short* srcm = a.Xa_hi[par] + (long long)b * a.Lp * a.Sp;
  unsigned short* dst = (unsigned short*)a.dst + (long long)b * a.m * a.n;
  if (!a.transpose && a.Xa_hi[par] == (const unsigned short*)a.dst) return;   // the caller's array was that iterate buffer: in place
  const int tiles_c = (a.n + 63) / 64;
  const int tr = bx / tiles_c, tc = bx % tiles_c;
  if (!a.transpose) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const int v = threadIdx.x + it * NT;
      const int r = tr * 64 + (v >> 3), col = tc * 64 + (v & 7) * 8;
      if (r < a.m && col < a.n) *(u32x4*)(dst + (long long)r * a.n + col) = *(const u32x4*)(srcm + (long long)r * a.Sp + col);
    }
    return;
  }
  // caller's tile (rows tr, columns tc) = transpose of the internal tile (rows tc, columns tr)
  __shared__ unsigned short tile[64][72];
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int v = threadIdx.x + it * NT;
    const int lr = v >> 3, lc = (v & 7) * 8;                 // internal row (caller's column), 8 internal columns
    const int ri = tc * 64 + lr, ci = tr * 64 + lc;
    u32x4 w = {0u, 0u, 0u, 0u};
    if (ri < a.Lp && ci < a.Sp) w = *(const u32x4*)(srcm + (long long)ri * a.Sp + ci);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      tile[lc + 2 * e][lr] = (unsigned short)(w[e] & 0xFFFFu);
      tile[lc + 2 * e + 1][lr] = (unsigned short)(w[e] >> 16);
    }
  }
  __syncthreads();
#pragma unroll
  for (int it = 0; it < 2; ++it) {
    const int v = threadIdx.x + it * NT;
    const int lr = v >> 3, lc = (v & 7) * 8;                 // caller's row within the tile, 8 caller's columns
    const int r = tr * 64 + lr, col = tc * 64 + lc;
    if (r < a.m && col < a.n) {
      u32x4 w;
#pragma unroll
      for (int e = 0; e < 4; ++e) w[e] = (unsigned)tile[lr][lc + 2 * e] | ((unsigned)tile[lr][lc + 2 * e + 1] << 16);
      *(u32x4*)(dst + (long long)r * a.n + col) = w;
    }
  }
}
__global__ __launch_bounds__(NT) void finalize_bf16_kernel(FinalArgs a) { finalize_bf16_body(a, blockIdx.x, blockIdx.y); }
__global__ __launch_bounds__(NT) void finalize_bf16_multi_kernel(FinalMulti m) {
  int w = blockIdx.x, gi = 0;
  while (gi + 1 < m.ngroups && w >= m.start[gi + 1]) ++gi;
  w -= m.start[gi];
  const FinalArgs& a = m.d[gi];
  const int tiles = ((a.m + 63) / 64) * ((a.n + 63) / 64);
  finalize_bf16_body(a, w % tiles, w / tiles);
}

// One thread per element of the caller's array.
__global__ __launch_bounds__(NT) void finalize_kernel(FinalArgs a) {
  const int b = blockIdx.y;
  const Ctrl c = a.ctrl[b];
  if (c.status == PRISM_INFO_NONFINITE || c.status == PRISM_INFO_ZERO) return;
  const int par = c.iters & 1;
  const long long mat = (long long)a.m * a.n;
  const long long i = (long long)blockIdx.x * NT + threadIdx.x;
  if (i >= mat) return;
  const int r = (int)(i / a.n), col = (int)(i % a.n);
  const long long o = (long long)b * a.Lp * a.Sp +
                      (a.transpose ? ((long long)col * a.Sp + r) : ((long long)r * a.Sp + col));
  if (a.fn == PRISM_FN_INVERSE) {
    ((float*)a.dst)[(long long)b * mat + i] = (float)((double)a.X32[par][o] / c.norm);
  } else if (a.fn == PRISM_FN_POLAR) {
    if (a.dt == PRISM_BF16) {
      float x = bf2f(a.Xa_hi[par][o]);
      if (a.Xa_lo[par]) x += bf2f(a.Xa_lo[par][o]);
      ((unsigned short*)a.dst)[(long long)b * mat + i] = f2bf(x);
    } else {
      ((float*)a.dst)[(long long)b * mat + i] = a.X32[par][o];
    }
  } else if (a.fn == PRISM_FN_SQRT_NEWTON) {
    ((float*)a.dst)[(long long)b * mat + i] = a.X32[par][o];
    ((float*)a.dst2)[(long long)b * mat + i] = a.Y32[par][o];
  } else if (a.fn == PRISM_FN_SQRT) {
    const double rs = sqrt(c.norm);
    ((float*)a.dst)[(long long)b * mat + i] = (float)((double)a.X32[par][o] * rs);
    ((float*)a.dst2)[(long long)b * mat + i] = (float)((double)a.Y32[par][o] / rs);
  } else {
    ((float*)a.dst)[(long long)b * mat + i] = a.X32[par][o];
  }
}

__global__ __launch_bounds__(NT) void make_e_kernel(float* E, const float* R, const Ctrl* ctrl, int np) {
  const int b = blockIdx.y;
  if (ctrl[b].done) return;
  const float alpha = ctrl[b].alpha;
  const long long total = (long long)np * np;
  const long long i = (long long)blockIdx.x * NT + threadIdx.x;
  if (i >= total) return;
  E[(long long)b * total + i] = alpha * R[(long long)b * total + i];
}

// One workgroup per 64 x 64 tile on or above the diagonal; thread t: row t / 4, 16 consecutive columns.
__global__ __launch_bounds__(NT) void gram_reduce_kernel(GramReduceArgs a) {
  const int b = blockIdx.y;
  if (a.ctrl[b].done) return;
  const int nt = a.np / 64;
  int left = blockIdx.x, tm = 0;
  while (left >= nt - tm) { left -= nt - tm; ++tm; }
  const int tn = tm + left;
  const int m0 = tm * 64, n0 = tn * 64;
  const long long SS = (long long)a.np * a.np;
  const int r = threadIdx.x >> 2, c0 = (threadIdx.x & 3) * 16;
  __shared__ float tile[64][65];
  {
    f32x4 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
    const float* src = a.part + (long long)b * a.parts * SS + (long long)(m0 + r) * a.np + n0 + c0;
    for (int p = 0; p < a.parts; ++p)
#pragma unroll
      for (int q = 0; q < 4; ++q) acc[q] += *(const f32x4*)(src + (long long)p * SS + 4 * q);
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int m = m0 + r, n = n0 + c0 + 4 * q + e;
        tile[r][c0 + 4 * q + e] = (m < a.n_true && n < a.n_true) ? ((m == n ? 1.0f : 0.0f) - acc[q][e]) : 0.0f;
      }
  }
  __syncthreads();
  const bool diag_tile = tm == tn;
  float part = 0.0f;
  auto emit = [&](int row0, int col0, bool transposed) {   // this thread's 16 entries of the tile at (row0, col0)
    float v[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int c = c0 + e;
      v[e] = transposed ? tile[c][r] : ((diag_tile && c < r) ? tile[c][r] : tile[r][c]);
    }
    const long long o = (long long)b * SS + (long long)(row0 + r) * a.np + col0 + c0;
    if (a.R32) {
#pragma unroll
      for (int q = 0; q < 4; ++q) *(f32x4*)(a.R32 + o + 4 * q) = f32x4{v[4 * q], v[4 * q + 1], v[4 * q + 2], v[4 * q + 3]};
    }
    if (a.Rb) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        u32x4 pk;
#pragma unroll
        for (int e = 0; e < 4; ++e) pk[e] = (unsigned)f2bf(v[8 * h + 2 * e]) | ((unsigned)f2bf(v[8 * h + 2 * e + 1]) << 16);
        *(u32x4*)(a.Rb + o + 8 * h) = pk;
      }
    }
    if (!transposed) {
#pragma unroll
      for (int e = 0; e < 16; ++e) part += v[e] * v[e];
      if (a.diag && diag_tile && r >= c0 && r < c0 + 16) a.diag[(long long)b * a.np + m0 + r] = tile[r][r];
    }
  };
  emit(m0, n0, false);
  if (!diag_tile) { emit(n0, m0, true); part *= 2.0f; }
  __shared__ float red[4];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = part;
  __syncthreads();
  if (threadIdx.x == 0) a.rho_part[(long long)b * gridDim.x + blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

}  // namespace

int gram_reduce_parts(int np) { return (np / 64) * (np / 64 + 1) / 2; }

void launch_gram_reduce(const GramReduceArgs& a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(gram_reduce_kernel, dim3(gram_reduce_parts(a.np), batch), dim3(NT), 0, s, a);
}

void launch_make_e(float* E, const float* R, const Ctrl* ctrl, int batch, int np, hipStream_t s) {
  const long long total = (long long)np * np;
  hipLaunchKernelGGL(make_e_kernel, dim3((unsigned)((total + NT - 1) / NT), batch), dim3(NT), 0, s, E, R, ctrl, np);
}

void launch_sumsq(const PrepArgs& a, hipStream_t s) {
  hipLaunchKernelGGL(sumsq_kernel, dim3(a.nsum, a.batch), dim3(NT), 0, s, a);
}

static bool bf16_vector_path(int fn, int dt, int m, int n, const void* user) {
  return fn == PRISM_FN_POLAR && dt == PRISM_BF16 && m % 8 == 0 && n % 8 == 0 && ((uintptr_t)user & 15) == 0;
}

void launch_prepare(const PrepArgs& a, hipStream_t s) {
  if (bf16_vector_path(a.fn, a.dt, a.m, a.n, a.src)) {
    // tiles over the padded caller-oriented matrix, so that the padding is written too
    const int tiles = (a.Lp / 64) * (a.Sp / 64);
    hipLaunchKernelGGL(prepare_bf16_kernel, dim3(tiles, a.batch), dim3(NT), 0, s, a);
    return;
  }
  const int tiles = (a.Lp / 64) * (a.Sp / 64);
  hipLaunchKernelGGL(prepare_kernel, dim3(tiles, a.batch), dim3(NT), 0, s, a);
}

// The pre-scaling and copy-out steps of several shape groups in one launch each (bf16 polar, every group
// on the 16-byte vector path); false: the caller launches them group by group.
bool launch_prep_multi(const PrepArgs* groups, int ngroups, hipStream_t s) {
  if (ngroups < 2 || ngroups > BF16_MAX_GROUPS) return false;
  PrepMulti ms = {}, mp = {};
  ms.ngroups = mp.ngroups = ngroups;
  long long ts = 0, tp = 0;
  for (int i = 0; i < ngroups; ++i) {
    const PrepArgs& a = groups[i];
    if (!bf16_vector_path(a.fn, a.dt, a.m, a.n, a.src)) return false;
    ms.d[i] = mp.d[i] = a;
    ms.start[i] = (int)ts; mp.start[i] = (int)tp;
    ts += (long long)a.nsum * a.batch;
    tp += (long long)(a.Lp / 64) * (a.Sp / 64) * a.batch;
    if (ts > 0x7fffffff || tp > 0x7fffffff) return false;
  }
  ms.start[ngroups] = (int)ts; mp.start[ngroups] = (int)tp;
  hipLaunchKernelGGL(sumsq_multi_kernel, dim3((unsigned)ts), dim3(NT), 0, s, ms);
  hipLaunchKernelGGL(prepare_bf16_multi_kernel, dim3((unsigned)tp), dim3(NT), 0, s, mp);
  return true;
}

bool launch_finalize_multi(const FinalArgs* groups, int ngroups, hipStream_t s) {
  if (ngroups < 2 || ngroups > BF16_MAX_GROUPS) return false;
  FinalMulti mf = {};
  mf.ngroups = ngroups;
  long long t = 0;
  for (int i = 0; i < ngroups; ++i) {
    const FinalArgs& a = groups[i];
    if (!bf16_vector_path(a.fn, a.dt, a.m, a.n, a.dst)) return false;
    mf.d[i] = a;
    mf.start[i] = (int)t;
    t += (long long)((a.m + 63) / 64) * ((a.n + 63) / 64) * a.batch;
    if (t > 0x7fffffff) return false;
  }
  mf.start[ngroups] = (int)t;
  hipLaunchKernelGGL(finalize_bf16_multi_kernel, dim3((unsigned)t), dim3(NT), 0, s, mf);
  return true;
}

void launch_finalize(const FinalArgs& a, hipStream_t s) {
  if (bf16_vector_path(a.fn, a.dt, a.m, a.n, a.dst)) {
    const int tiles = ((a.m + 63) / 64) * ((a.n + 63) / 64);
    hipLaunchKernelGGL(finalize_bf16_kernel, dim3((unsigned)tiles, a.batch), dim3(NT), 0, s, a);
    return;
  }
  const long long mat = (long long)a.m * a.n;
  hipLaunchKernelGGL(finalize_kernel, dim3((unsigned)((mat + NT - 1) / NT), a.batch), dim3(NT), 0, s, a);
}

namespace {
__global__ __launch_bounds__(256) void scatter_info_kernel(InfoScatter a) {
  const int words = (int)(sizeof(prism_info) / 4);
  for (int g = 0; g < a.ngroups; ++g) {
    if (!a.dst[g]) continue;
    const unsigned* src = (const unsigned*)(a.src + a.first[g]);
    unsigned* dst = (unsigned*)a.dst[g];
    const int n = (a.first[g + 1] - a.first[g]) * words;
    for (int i = blockIdx.x * 256 + threadIdx.x; i < n; i += gridDim.x * 256) dst[i] = src[i];
  }
}
}  // namespace

void launch_scatter_info(const InfoScatter& a, hipStream_t s) {
  static_assert(sizeof(prism_info) % 4 == 0, "reports are copied word by word");
  hipLaunchKernelGGL(scatter_info_kernel, dim3(8), dim3(256), 0, s, a);
}

}  // namespace prism
