// The per-iteration coefficient fit of PRISM (paper Section 4.2, eq. (4); App. A.1, A.3 and A.4)
// after the sketch chain V_j = R V_{j-1} has been formed:
//   moments_kernel (a few workgroups per matrix) forms the blocks W_i = u_i(R) S^T from the chain
//      (the factor (1 - xi) = G = I - R is applied as V_j - V_{j+1}) and accumulates
//         c_s = sum_{i+l=s} <W_i, W_l>,  m(alpha) = || sum_i alpha^i W_i ||_F^2,
//      in fp64 with a fixed reduction order (results are run-to-run identical);
//   solve_kernel (one workgroup per matrix)
//   1. sums the residual partials, applies the stop rule and records the residual;
//   2. adds up the coefficient partials;
//   3. minimises m over [l, u]: all real roots of m' in the interval are bracketed between the
//      roots of m'' (recursively down to the linear derivative) and found by bisection, then m
//      is compared at the end points and those roots; the smallest alpha wins ties.
// Nothing returns to the host: alpha_k, the done flag and the report stay on the device.
#include "common.h"

namespace prism {
namespace {

constexpr int NT = 256;
constexpr int MAXC = 2 * PRISM_MAX_ROOT + 1;  // coefficients of m

__device__ inline double horner(const double* c, int deg, double x) {
  double v = c[deg];
  for (int i = deg - 1; i >= 0; --i) v = v * x + c[i];
  return v;
}

// Blocks<d>: Newton-Schulz family (polar, square root, sign).  BlocksInv<p>: coupled inverse
// Newton.  BlocksCheb: Chebyshev inverse.
template <int KIND> struct Blocks;
template <> struct Blocks<1> {
  static constexpr int NV = 3, NW = 3;
  __device__ static void make(const double* v, double* w) {  // v[j-1] = V_j
    w[0] = v[0];
    w[1] = -2.0 * (v[0] - v[1]);
    w[2] = -(v[1] - v[2]);
  }
};
template <> struct Blocks<2> {
  static constexpr int NV = 5, NW = 3;
  __device__ static void make(const double* v, double* w) {
    w[0] = (3.0 * v[1] + v[2]) * 0.25;
    w[1] = -((2.0 * v[1] + v[2]) - (2.0 * v[2] + v[3]));
    w[2] = -(v[3] - v[4]);
  }
};
struct BlocksCheb {   // App. A.4: W_0 = R^2 S^T, W_1 = -(R^2 - R^3) S^T
  static constexpr int NV = 3, NW = 2;
  __device__ static void make(const double* v, double* w) {
    w[0] = v[1];
    w[1] = -(v[1] - v[2]);
  }
};
template <int P> struct BlocksInv {
  static constexpr int NV = P + 1, NW = P + 1;
  __device__ static void make(const double* v, double* w) {
    w[0] = v[0];
    double binom = 1.0;
#pragma unroll
    for (int i = 1; i <= P; ++i) {
      binom = binom * (double)(P - i + 1) / (double)i;  // C(P, i), exact for P <= 8
      w[i] = -binom * (v[i - 1] - v[i]);
    }
  }
};

template <class BL>
__device__ void accumulate_coefficients(const SolveArgs& a, int b, int grp, int ngrp, double* c_out /* global, MAXC */) {
  constexpr int NV = BL::NV, NW = BL::NW, NC = 2 * NW - 1;
  double c[NC];
#pragma unroll
  for (int s = 0; s < NC; ++s) c[s] = 0.0;
  const long long total = (long long)a.rows * a.ld;
  const float* base = a.V + (long long)b * a.bstride;
  for (long long idx = (long long)grp * NT + threadIdx.x; idx < total; idx += (long long)ngrp * NT) {
    double v[NV], w[NW];
#pragma unroll
    for (int j = 0; j < NV; ++j) v[j] = (double)base[(long long)j * a.vstride + idx];
    BL::make(v, w);
#pragma unroll
    for (int i = 0; i < NW; ++i)
#pragma unroll
      for (int l = 0; l < NW; ++l) c[i + l] += w[i] * w[l];
  }
  __shared__ double red[4][MAXC];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int s = 0; s < NC; ++s) {
    double x = c[s];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_down(x, off, 64);
    if (lane == 0) red[wave][s] = x;
  }
  __syncthreads();
  if (threadIdx.x < MAXC) {
    const int s = threadIdx.x;
    c_out[s] = (s < NC) ? (red[0][s] + red[1][s] + red[2][s] + red[3][s]) : 0.0;
  }
}

__device__ void accumulate_for(const SolveArgs& a, int b, int grp, int ngrp, double* out) {
  if (a.fn == PRISM_FN_INV_ROOT) {
    switch (a.p) {
      case 1: accumulate_coefficients<BlocksInv<1>>(a, b, grp, ngrp, out); break;
      case 2: accumulate_coefficients<BlocksInv<2>>(a, b, grp, ngrp, out); break;
      case 3: accumulate_coefficients<BlocksInv<3>>(a, b, grp, ngrp, out); break;
      case 4: accumulate_coefficients<BlocksInv<4>>(a, b, grp, ngrp, out); break;
      case 5: accumulate_coefficients<BlocksInv<5>>(a, b, grp, ngrp, out); break;
      case 6: accumulate_coefficients<BlocksInv<6>>(a, b, grp, ngrp, out); break;
      case 7: accumulate_coefficients<BlocksInv<7>>(a, b, grp, ngrp, out); break;
      default: accumulate_coefficients<BlocksInv<8>>(a, b, grp, ngrp, out); break;
    }
  } else if (a.fn == PRISM_FN_INVERSE) {
    accumulate_coefficients<BlocksCheb>(a, b, grp, ngrp, out);
  } else if (a.d == 1) {
    accumulate_coefficients<Blocks<1>>(a, b, grp, ngrp, out);
  } else {
    accumulate_coefficients<Blocks<2>>(a, b, grp, ngrp, out);
  }
}

// grid (groups, batch): partial coefficient sums of one matrix, groups interleaved over the elements
__global__ __launch_bounds__(NT) void moments_kernel(SolveArgs a) {
  const int b = blockIdx.y, grp = blockIdx.x, ngrp = gridDim.x;
  if (a.ctrl[b].done) return;
  accumulate_for(a, b, grp, ngrp, a.cpart + ((long long)b * ngrp + grp) * MAXC);
}

__global__ __launch_bounds__(NT) void solve_kernel(SolveArgs a) {
  const int b = blockIdx.x, t = threadIdx.x;
  Ctrl* ctl = &a.ctrl[b];
  if (ctl->done) return;
  prism_info* info = a.info + b;
  __shared__ int s_stop;
  __shared__ double s_c[MAXC];
  __shared__ double s_q[2 * PRISM_MAX_ROOT][MAXC];   // derivative chain of m'
  __shared__ double s_roots[2][MAXC + 2];
  __shared__ int s_nroots[2];

  // residual: sum of the per-tile partials, every thread a strided share, then a fixed tree
  __shared__ double s_rho[4];
  {
    double part = 0.0;
    for (int i = t; i < a.nparts; i += NT) part += (double)a.rho_part[(long long)b * a.nparts + i];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
    if ((t & 63) == 0) s_rho[t >> 6] = part;
    __syncthreads();
  }
  if (a.phase == 2) {
    if (t == 0) s_stop = 0;          // coefficient only: the stop test of this k has been taken
  } else if (t == 0) {
    const double rho = (s_rho[0] + s_rho[1]) + (s_rho[2] + s_rho[3]);
    const double res = sqrt(rho / (double)a.n);
    info->residual[a.k] = (float)res;
    int status = -1;
    if (!(res == res) || res > 1.0e300) status = PRISM_INFO_DIVERGED;
    else if (a.tol > 0.0 && res <= a.tol) status = PRISM_INFO_CONVERGED;
    else if (a.k == a.max_iters) status = PRISM_INFO_BUDGET;
    else if (a.tol > 0.0 && a.k >= 2 && res > (double)ctl->res1 && ctl->res1 > ctl->res2 && res > (double)ctl->res0)
      status = PRISM_INFO_DIVERGED;
    if (status >= 0) {
      ctl->status = status;
      ctl->iters = a.k;
      ctl->done = 1;
      info->status = status;
      info->iters = a.k;
      s_stop = 1;
    } else {
      if (a.k == 0) ctl->res0 = (float)res;
      ctl->res2 = ctl->res1;
      ctl->res1 = (float)res;
      ctl->iters = a.k + 1;     // the update of this iteration is already enqueued behind us
      info->iters = a.k + 1;
      s_stop = 0;
    }
  }
  __syncthreads();
  if (s_stop || a.phase == 1) return;

  double lo, hi;
  if (a.fn == PRISM_FN_INV_ROOT) { lo = 1.0 / a.p; hi = 2.0 / a.p; }
  else if (a.fn == PRISM_FN_INVERSE) { lo = 0.5; hi = 2.0; }
  else if (a.fn == PRISM_FN_SQRT_NEWTON) { lo = 0.0; hi = 1.0; }
  else if (a.d == 1) { lo = 0.5; hi = 1.0; }
  else { lo = 0.375; hi = 1.45; }

  if (a.mode != 0) {
    if (t == 0) {
      // without a fit: the Taylor coefficient, which is l except for the Chebyshev inverse (1)
      // (and the DB Newton iteration, whose classical coefficient is 1/2)
      const double taylor = (a.fn == PRISM_FN_INVERSE) ? 1.0 : (a.fn == PRISM_FN_SQRT_NEWTON ? 0.5 : lo);
      const float al = (a.mode == 3) ? a.sched_alpha : (float)((a.mode == 1) ? taylor : hi);
      ctl->alpha = al;
      info->alpha[a.k] = al;
    }
    return;
  }

  const int nc = (a.fn == PRISM_FN_INV_ROOT) ? 2 * a.p + 1 : (a.fn == PRISM_FN_INVERSE ? 3 : 5);
  if (a.ngroups == 1 && a.fn != PRISM_FN_SQRT_NEWTON) {   // small matrices: the moments are accumulated right here
    accumulate_for(a, b, 0, 1, a.cpart + (long long)b * MAXC);
    __threadfence_block();
    __syncthreads();
  }
  if (t < MAXC) {   // coefficient s = sum of the group partials, in group order
    double v = 0.0;
    for (int gidx = 0; gidx < a.ngroups; ++gidx) v += a.cpart[((long long)b * a.ngroups + gidx) * MAXC + t];
    s_c[t] = v;
  }
  __syncthreads();

  // ---- minimise m(alpha) = sum_s c_s alpha^s on [lo, hi] ----
  const int deg = nc - 1;   // degree of m
  const int dq = deg - 1;   // degree of m'
  bool usable = true;
  {
    bool all_tiny = true;
    for (int s = 0; s < nc; ++s) {
      const double v = s_c[s];
      if (!(v == v) || fabs(v) > 1.0e300) usable = false;
      if (fabs(v) >= 1.0e-300) all_tiny = false;
    }
    if (all_tiny) usable = false;
  }
  if (!usable) {
    if (t == 0) { ctl->alpha = (float)lo; info->alpha[a.k] = (float)lo; }
    return;
  }
  // derivative chain: s_q[j] = (j+1)-th derivative of m, degree deg-1-j
  if (t == 0) {
    for (int i = 0; i <= dq; ++i) s_q[0][i] = (double)(i + 1) * s_c[i + 1];
    for (int j = 1; j < dq; ++j)
      for (int i = 0; i <= dq - j; ++i) s_q[j][i] = (double)(i + 1) * s_q[j - 1][i + 1];
    // linear level j = dq-1: a0 + a1 x
    const double a0 = s_q[dq - 1][0], a1 = s_q[dq - 1][1];
    int n0 = 0;
    if (a1 != 0.0) {
      const double r = -a0 / a1;
      if (r >= lo && r <= hi) s_roots[(dq - 1) & 1][n0++] = r;
    }
    s_nroots[(dq - 1) & 1] = n0;
  }
  __syncthreads();
  for (int j = dq - 2; j >= 0; --j) {
    const int src = (j + 1) & 1, dst = j & 1;
    const int nr = s_nroots[src];
    const int pdeg = dq - j;
    double found = 0.0;
    int has = 0;
    if (t <= nr) {  // interval t between consecutive roots of the next derivative
      const double xa = (t == 0) ? lo : s_roots[src][t - 1];
      const double xb = (t == nr) ? hi : s_roots[src][t];
      double fa = horner(s_q[j], pdeg, xa);
      const double fb = horner(s_q[j], pdeg, xb);
      if (fa == 0.0) { found = xa; has = 1; }
      else if (t == nr && fb == 0.0) { found = xb; has = 1; }
      else if ((fa < 0.0) != (fb < 0.0) && fb != 0.0) {
        double l = xa, h = xb;
        for (int it = 0; it < 200; ++it) {
          const double mid = 0.5 * (l + h);
          if (mid <= l || mid >= h) break;
          const double fm = horner(s_q[j], pdeg, mid);
          if (fm == 0.0) { l = h = mid; break; }
          if ((fm < 0.0) == (fa < 0.0)) l = mid; else h = mid;
        }
        found = 0.5 * (l + h);
        has = 1;
      }
    }
    __syncthreads();
    __shared__ double s_tmp[MAXC + 2];
    __shared__ int s_has[MAXC + 2];
    if (t <= nr) { s_tmp[t] = found; s_has[t] = has; }
    __syncthreads();
    if (t == 0) {
      int cnt = 0;
      for (int i = 0; i <= nr; ++i)
        if (s_has[i]) s_roots[dst][cnt++] = s_tmp[i];
      s_nroots[dst] = cnt;
    }
    __syncthreads();
  }
  if (t == 0) {
    const int lvl = (dq >= 2) ? 0 : ((dq - 1) & 1);
    const int nr = s_nroots[lvl & 1];
    double best = lo, bestv = horner(s_c, deg, lo);
    for (int i = 0; i < nr; ++i) {
      const double x = s_roots[lvl & 1][i];
      const double v = horner(s_c, deg, x);
      if (v < bestv) { bestv = v; best = x; }
    }
    const double vh = horner(s_c, deg, hi);
    if (vh < bestv) { bestv = vh; best = hi; }
    ctl->alpha = (float)best;
    info->alpha[a.k] = (float)best;
    // The fit has left the upper end of its interval: no eigenvalue of R is close to 1 any more,
    // i.e. no singular value of the iterate is small.  The bf16 polar path stops carrying the low
    // half of the iterate from here on (it exists for the small singular values only).
    if (best < hi - 1e-6) ctl->plain = 1;
  }
}

}  // namespace

void launch_moments(const SolveArgs& a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(moments_kernel, dim3(a.ngroups, batch), dim3(NT), 0, s, a);
}

void launch_solve(const SolveArgs& a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(solve_kernel, dim3(batch), dim3(NT), 0, s, a);
}

}  // namespace prism
