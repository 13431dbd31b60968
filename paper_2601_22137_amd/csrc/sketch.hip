// Gaussian sketch generator (paper Section 4.2: S_k is a p_s x n matrix of i.i.d. Gaussian
// entries, fresh for every iteration k).
//
// Entry (r, j) of S_k is a pure function of (seed, k, function tag, r, j):
//   Philox4x32-10 (Salmon et al., SC'11), key = (seed low, seed high), counter = (j, r/4, k, tag);
//   the four output words give rows 4q..4q+3 of column j through two Box-Muller pairs:
//     a = (xa >> 8) + 1, b = xb >> 8,  z = fl32( sqrt(-2 ln(a 2^-24)) * (cos, sin)(2 pi b 2^-24) ).
// The logarithm, cosine and sine are fixed sequences of IEEE binary64 +, -, *, /, sqrt, each
// rounded once; this file must be compiled with floating-point contraction off so that no
// multiply-add pair is fused.  That makes the stream reproducible bit for bit on any machine.
#include "common.h"

#pragma clang fp contract(off)

namespace prism {
namespace {

struct U4 { unsigned int x, y, z, w; };

__device__ inline U4 philox4x32_10(U4 c, unsigned int k0, unsigned int k1) {
  const unsigned int M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const unsigned int hi0 = __umulhi(M0, c.x), lo0 = M0 * c.x;
    const unsigned int hi1 = __umulhi(M1, c.z), lo1 = M1 * c.z;
    U4 n;
    n.x = hi1 ^ c.y ^ k0;
    n.y = lo1;
    n.z = hi0 ^ c.w ^ k1;
    n.w = lo0;
    c = n;
    k0 += W0;
    k1 += W1;
  }
  return c;
}

// sqrt(-2 ln(a 2^-24)), a in [1, 2^24]
__device__ inline double bm_radius(unsigned int a) {
  int e = 31 - __clz((int)a);
  // m = a * 2^-e in [1, 2): exact scaling by a power of two
  double m = (double)a * __longlong_as_double((long long)(1023 - e) << 52);
  if (m > 1.4142135623730951) {
    m = m * 0.5;
    e = e + 1;
  }
  const double f = m - 1.0;
  const double s = f / (2.0 + f);
  const double w = s * s;
  double p = 1.0 / 21.0;
  p = p * w + 1.0 / 19.0;
  p = p * w + 1.0 / 17.0;
  p = p * w + 1.0 / 15.0;
  p = p * w + 1.0 / 13.0;
  p = p * w + 1.0 / 11.0;
  p = p * w + 1.0 / 9.0;
  p = p * w + 1.0 / 7.0;
  p = p * w + 1.0 / 5.0;
  p = p * w + 1.0 / 3.0;
  p = p * w + 1.0;
  const double lnm = (2.0 * s) * p;
  const double lnu = (double)(e - 24) * 0.6931471805599453 + lnm;
  return sqrt(0.0 - 2.0 * lnu);
}

// (cos, sin)(2 pi b 2^-24), b in [0, 2^24)
__device__ inline void bm_cos_sin(unsigned int b, double& cs, double& sn) {
  const unsigned int oct = b >> 21;
  double t = (double)(b & 0x1FFFFFu) * 4.76837158203125e-07;  // 2^-21, exact
  if (oct & 1u) t = 1.0 - t;
  const double x = t * 0.7853981633974483;
  const double y = x * x;
  double c = 1.0 / 20922789888000.0;   // 1/16!
  double s = 1.0 / 355687428096000.0;  // 1/17!
  c = c * y + (-(1.0 / 87178291200.0));   s = s * y + (-(1.0 / 1307674368000.0));  // k = 7
  c = c * y + 1.0 / 479001600.0;          s = s * y + 1.0 / 6227020800.0;          // k = 6
  c = c * y + (-(1.0 / 3628800.0));       s = s * y + (-(1.0 / 39916800.0));       // k = 5
  c = c * y + 1.0 / 40320.0;              s = s * y + 1.0 / 362880.0;              // k = 4
  c = c * y + (-(1.0 / 720.0));           s = s * y + (-(1.0 / 5040.0));           // k = 3
  c = c * y + 1.0 / 24.0;                 s = s * y + 1.0 / 120.0;                 // k = 2
  c = c * y + (-(1.0 / 2.0));             s = s * y + (-(1.0 / 6.0));              // k = 1
  c = c * y + 1.0;                        s = s * y + 1.0;                         // k = 0
  s = s * x;
  switch (oct) {
    case 0: cs = c;  sn = s;  break;
    case 1: cs = s;  sn = c;  break;
    case 2: cs = -s; sn = c;  break;
    case 3: cs = -c; sn = s;  break;
    case 4: cs = -c; sn = -s; break;
    case 5: cs = -s; sn = -c; break;
    case 6: cs = s;  sn = -c; break;
    default: cs = c; sn = -s; break;
  }
}

__device__ inline void box_muller(unsigned int xa, unsigned int xb, float& z0, float& z1) {
  const double r = bm_radius((xa >> 8) + 1u);
  double c, s;
  bm_cos_sin(xb >> 8, c, s);
  z0 = (float)(r * c);
  z1 = (float)(r * s);
}

// v0[rows_total][ld]: row j < n holds column j of S_k (entries r < p_s), everything else zero.
__global__ void sketch_kernel(float* v0, int rows_total, int n, int ld, int p_s, unsigned int k0,
                              unsigned int k1, unsigned int iter, unsigned int tag) {
  const int groups = (ld + 3) / 4;
  const long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long long)rows_total * groups) return;
  iter += blockIdx.y;                                   // one sketch per blockIdx.y
  v0 += (long long)blockIdx.y * rows_total * ld;
  const int j = (int)(idx / groups), q = (int)(idx % groups);
  float z[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  if (j < n && 4 * q < p_s) {
    U4 c;
    c.x = (unsigned int)j; c.y = (unsigned int)q; c.z = iter; c.w = tag;
    const U4 x = philox4x32_10(c, k0, k1);
    box_muller(x.x, x.y, z[0], z[1]);
    box_muller(x.z, x.w, z[2], z[3]);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int r = 4 * q + e;
    if (r < ld) v0[(long long)j * ld + r] = (r < p_s) ? z[e] : 0.0f;
  }
}

__global__ void gauss_parts_kernel(unsigned int first, unsigned int count, double* r, double* c, double* s) {
  const unsigned int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const unsigned int v = first + i;  // v in [0, 2^24)
  r[i] = bm_radius(v + 1u);
  double cc, ss;
  bm_cos_sin(v, cc, ss);
  c[i] = cc;
  s[i] = ss;
}

}  // namespace

void launch_sketch(float* v0, int rows_total, int n, int ld, int p_s, uint64_t seed, int k_first, int k_count, int fn,
                   hipStream_t s) {
  const long long total = (long long)rows_total * ((ld + 3) / 4);
  const int nb = (int)((total + 255) / 256);
  hipLaunchKernelGGL(sketch_kernel, dim3(nb, k_count), dim3(256), 0, s, v0, rows_total, n, ld, p_s,
                     (unsigned int)(seed & 0xFFFFFFFFull), (unsigned int)(seed >> 32), (unsigned int)k_first,
                     (unsigned int)fn);
}

void launch_gauss_parts(uint32_t first, uint32_t count, double* r, double* c, double* sn, hipStream_t s) {
  const int nb = (int)((count + 255) / 256);
  hipLaunchKernelGGL(gauss_parts_kernel, dim3(nb), dim3(256), 0, s, first, count, r, c, sn);
}

}  // namespace prism
