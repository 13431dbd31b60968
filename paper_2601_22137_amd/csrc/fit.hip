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
//      roots of m'' (recursively down to the linear derivative) and found by Newton's method
//      safeguarded by bisection, then m
//      is compared at the end points and those roots; the smallest alpha wins ties.
// Nothing returns to the host: alpha_k, the done flag and the report stay on the device.
//   small_polar_kernel: for fp32 polar factors whose padded iterate is 64 x 64, the whole method
//   (residual, chain, fit, update, for all iterations) in one workgroup per matrix.
#include "common.h"

namespace prism {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));

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

// One workgroup, matrix b: stop rule and coefficient of iteration a.k.  Every return is taken by all
// threads of the workgroup together.
// rho_local (LDS, one double) stands in for the residual partials in global memory and c_local
// (LDS, MAXC doubles) for the coefficient partials when the caller has them on chip.
__device__ void solve_body(const SolveArgs& a, int b, const double* rho_local = nullptr, double* c_local = nullptr) {
  const int t = threadIdx.x;
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
  if (!rho_local) {
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
    const double rho = rho_local ? *rho_local : (s_rho[0] + s_rho[1]) + (s_rho[2] + s_rho[3]);
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

  if (a.fn == PRISM_FN_SQRT_NEWTON) {
    // The fp32 inverse N_k loses about cond(M_k) * eps * sqrt(n) of its accuracy and X, Y inherit
    // that; once it is worthless the iteration would still drive M_k to I and report convergence.
    // Slot 16 of the partials holds ||M_k N_k v - v||^2 for a probe vector v of +-1 entries, an
    // estimate of ||M_k N_k - I||_F^2: above 10 % relative the matrix stops as diverged, before the
    // update that would use N_k.
    if (t == 0) {
      double e2 = 0.0;
      for (int gidx = 0; gidx < a.ngroups; ++gidx) e2 += a.cpart[((long long)b * a.ngroups + gidx) * MAXC + 16];
      if (!(e2 <= 0.01 * (double)a.n)) {
        ctl->status = PRISM_INFO_DIVERGED; ctl->iters = a.k; ctl->done = 1;
        info->status = PRISM_INFO_DIVERGED; info->iters = a.k;
        s_stop = 1;
      }
    }
    __syncthreads();
    if (s_stop) return;
  }

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
  if (c_local) {   // moments straight into LDS
    accumulate_for(a, b, 0, 1, c_local);
    __syncthreads();
    if (t < MAXC) s_c[t] = c_local[t];
  } else {
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
        // Newton's method kept inside the bracket [l, h] (f(l) has the sign of fa): a step that
        // would leave the bracket, or that shrinks too slowly, is replaced by a bisection step.
        // The derivative of level j is level j + 1 of the chain.
        double l = xa, h = xb;
        double x = 0.5 * (l + h), dx = h - l, dxold = dx;
        double fx = horner(s_q[j], pdeg, x), dfx = horner(s_q[j + 1], pdeg - 1, x);
        for (int it = 0; it < 200; ++it) {
          if (fx == 0.0) break;
          if ((fx < 0.0) == (fa < 0.0)) l = x; else h = x;
          const bool leaves = !((((x - h) * dfx - fx) * ((x - l) * dfx - fx)) < 0.0);
          const bool slow = fabs(2.0 * fx) > fabs(dxold * dfx);
          dxold = dx;
          double xn;
          if (leaves || slow) { dx = 0.5 * (h - l); xn = l + dx; }
          else { dx = fx / dfx; xn = x - dx; }
          if (xn == x || !(xn > l && xn < h)) break;   // the bracket is down to neighbouring numbers
          x = xn;
          if (fabs(dx) <= 2.0e-16 * fabs(x)) break;
          fx = horner(s_q[j], pdeg, x);
          dfx = horner(s_q[j + 1], pdeg - 1, x);
        }
        found = x;
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

__global__ __launch_bounds__(NT) void solve_kernel(SolveArgs a) { solve_body(a, blockIdx.x); }

// ---- fp32 polar factor, padded iterate 64 x 64: all iterations in one workgroup ----
// The products run on v_mfma_f32_16x16x4_f32 (A operand: lane l holds A[m = l % 16][k = l / 16], B
// operand B[k = l / 16][n = l % 16], result register r of lane l is D[4 (l / 16) + r][l % 16]); each
// of the four waves owns a 32 x 32 quadrant of a 64 x 64 result (2 x 2 blocks), or 16 rows of a chain
// product.  LDS: X [64][SX], R [64][SR], and a third area for the two chain buffers [64][ldv] and
// later Q [64][SR].  R and Q are symmetric, so they are always read with k as the row index; SR = 80 and
// the chain stride ld + 16 put the four k rows of a fragment read into different banks, SX = 68
// does the same for the reads of X along its rows in X Q.
constexpr int SN = 64, SX = 68, SR = 80;
__host__ __device__ inline int small_ldv(int ld) { return ld == 16 ? 16 : ld + 16; }
// the third area holds Q [64][SR] or the two chain buffers [64][ldv], whichever is larger (58 KiB in
// all for 16 sketch columns, so that two workgroups share a CU; 77 KiB for 64 columns)
// (16 sketch columns: V_0 .. V_5 all stay in LDS, 6 x [64][16], and the moments are taken from there)
inline int small_lds_floats(int ld) {
  const int chain = ld == 16 ? 6 * SN * 16 : 2 * SN * small_ldv(ld);
  return SN * SX + SN * SR + (chain > SN * SR ? chain : SN * SR);
}

// acc[i][j] += sum_k A(k, m) B(k, n) over k = 0 .. 63 for the wave's quadrant; A(k, m) sits at
// As[k * sak + m * sam], B(k, n) at Bs[k * ldb + n]
__device__ inline void small_mma(const float* As, int sak, int sam, const float* Bs, int ldb, int wm0, int wn0,
                                 f32x4 (&acc)[2][2]) {
  const int lr = threadIdx.x & 15, lk = (threadIdx.x & 63) >> 4;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll 4
  for (int k0 = 0; k0 < SN; k0 += 4) {
    float av[2], bv[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) av[i] = As[(k0 + lk) * sak + (wm0 + i * 16 + lr) * sam];
#pragma unroll
    for (int j = 0; j < 2; ++j) bv[j] = Bs[(k0 + lk) * ldb + wn0 + j * 16 + lr];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[i], bv[j], acc[i][j], 0, 0, 0);
  }
}

// Vout = R Vin (R symmetric): wave w forms rows 16 w .. 16 w + 15, all LD columns; the result goes to
// the other LDS buffer and, densely ([64][LD]), to global memory for the moments
template <int LD>
__device__ inline void small_chain_step(const float* Rs, const float* Vin, float* Vout, float* Vglobal) {
  constexpr int NB = LD / 16;
  const int ldv = LD == 16 ? 16 : LD + 16;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, lr = lane & 15, lk = lane >> 4;
  f32x4 acc[NB];
#pragma unroll
  for (int j = 0; j < NB; ++j) acc[j] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
  for (int k0 = 0; k0 < SN; k0 += 4) {
    const float av = Rs[(k0 + lk) * SR + 16 * wave + lr];
#pragma unroll
    for (int j = 0; j < NB; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(av, Vin[(k0 + lk) * ldv + 16 * j + lr], acc[j], 0, 0, 0);
  }
#pragma unroll
  for (int j = 0; j < NB; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      const int row = 16 * wave + 4 * lk + r, col = 16 * j + lr;
      Vout[row * ldv + col] = acc[j][r];
      if (Vglobal) Vglobal[row * LD + col] = acc[j][r];
    }
}

__global__ __launch_bounds__(NT) void small_polar_kernel(SmallPolarArgs a) {
  extern __shared__ float small_lds[];
  float* Xs = small_lds;
  float* Rs = Xs + SN * SX;
  float* Ts = Rs + SN * SR;
  __shared__ double s_part[4];
  __shared__ double s_rho;
  __shared__ double s_coef[MAXC];
  const int b = blockIdx.x, t = threadIdx.x;
  SolveArgs sv = a.sv;
  Ctrl* ctl = &sv.ctrl[b];
  if (ctl->done) return;   // zero or non-finite input: reported by the prepare step
  if (sv.ld == 16) { sv.V = Ts + SN * 16; sv.vstride = SN * 16; sv.bstride = 0; }
  const int lane = t & 63, wave = t >> 6, lr = lane & 15, lk = lane >> 4;
  const int wm0 = (wave >> 1) * 32, wn0 = (wave & 1) * 32;   // this wave's quadrant of a 64 x 64 result
  {
    const float* Xg = a.X[0] + (long long)b * SN * SN;
    for (int idx = t; idx < SN * SN / 4; idx += NT) {
      const int r = idx >> 4, c = (idx & 15) * 4;
      *(f32x4*)&Xs[r * SX + c] = *(const f32x4*)&Xg[r * SN + c];
    }
  }
  __syncthreads();
  f32x4 acc[2][2];
  for (int k = 0; k <= sv.max_iters; ++k) {
    if (k == sv.max_iters && sv.tol <= 0.0) break;
    // R = I - X^T X, zero outside the leading n x n block; rho = ||R||_F^2
    small_mma(Xs, SX, 1, Xs, SX, wm0, wn0, acc);
    double part = 0.0;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = wm0 + i * 16 + 4 * lk + r, col = wn0 + j * 16 + lr;
          const float rv = (row < sv.n && col < sv.n) ? ((row == col ? 1.0f : 0.0f) - acc[i][j][r]) : 0.0f;
          Rs[row * SR + col] = rv;
          part += (double)rv * (double)rv;
        }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) part += __shfl_down(part, off, 64);
    if (lane == 0) s_part[wave] = part;
    __syncthreads();
    if (t == 0) s_rho = (s_part[0] + s_part[1]) + (s_part[2] + s_part[3]);

    // sketch chain V_j = R V_{j-1}, V_0 = S_k^T; the V_j also go to global memory for the moments
    if (a.p_s > 0 && k >= a.first_fit && k < sv.max_iters) {
      const int ld = sv.ld, ldv = small_ldv(ld);
      const float* v0 = a.V0 + (long long)(k - a.first_fit) * SN * ld;
      for (int idx = t; idx < SN * ld / 4; idx += NT) {
        const int r = (idx * 4) / ld, c = (idx * 4) % ld;
        *(f32x4*)&Ts[r * ldv + c] = *(const f32x4*)&v0[idx * 4];
      }
      __syncthreads();
      // between the products only the LDS copies must be in place; the stores to global memory stay
      // in flight until the full barrier below
      auto lds_barrier = [&]() {
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
      };
      if (ld == 16) {   // V_j at Ts + j * 1024: the moments read them from LDS
        for (int j = 1; j <= a.nv; ++j) {
          small_chain_step<16>(Rs, Ts + (j - 1) * SN * 16, Ts + j * SN * 16, nullptr);
          lds_barrier();
        }
      } else {
        float* vin = Ts;
        float* vout = Ts + SN * ldv;
        for (int j = 1; j <= a.nv; ++j) {
          float* vg = const_cast<float*>(a.sv.V) + (long long)(j - 1) * a.sv.vstride + (long long)b * a.sv.bstride;
          if (ld == 32) small_chain_step<32>(Rs, vin, vout, vg);
          else small_chain_step<64>(Rs, vin, vout, vg);
          lds_barrier();
          float* tmp = vin; vin = vout; vout = tmp;
        }
      }
    }
    __threadfence_block();
    __syncthreads();

    sv.k = k;
    sv.mode = k < a.sched_len ? 3 : (a.p_s == 0 ? 1 : (k < a.warm ? 2 : 0));
    sv.sched_alpha = k < a.sched_len ? a.sched[k] : 0.0f;
    solve_body(sv, b, &s_rho, s_coef);
    __threadfence_block();
    __syncthreads();
    if (ctl->done) break;
    const float alpha = ctl->alpha;

    const float* Bm = Rs;
    float wa = alpha;
    if (sv.d == 2) {   // Q = R / 2 + alpha R^2
      small_mma(Rs, SR, 1, Rs, SR, wm0, wn0, acc);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int row = wm0 + i * 16 + 4 * lk + r, col = wn0 + j * 16 + lr;
            Ts[row * SR + col] = 0.5f * Rs[row * SR + col] + alpha * acc[i][j][r];
          }
      __syncthreads();
      Bm = Ts;
      wa = 1.0f;
    }
    // X <- X + wa X B: every wave reads whole rows of X, so all reads end before the first store
    small_mma(Xs, 1, SX, Bm, SR, wm0, wn0, acc);
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int row = wm0 + i * 16 + 4 * lk + r, col = wn0 + j * 16 + lr;
          Xs[row * SX + col] += wa * acc[i][j][r];
        }
    __syncthreads();
  }
  {
    float* Xg = a.X[ctl->iters & 1] + (long long)b * SN * SN;
    for (int idx = t; idx < SN * SN / 4; idx += NT) {
      const int r = idx >> 4, c = (idx & 15) * 4;
      *(f32x4*)&Xg[r * SN + c] = *(const f32x4*)&Xs[r * SX + c];
    }
  }
}

}  // namespace

int launch_small_polar(const SmallPolarArgs& a, int batch, hipStream_t s) {
  if (a.sv.rows != SN || (a.sv.ld != 16 && a.sv.ld != 32 && a.sv.ld != 64) || a.sv.ngroups != 1 || a.sv.nparts != 1 ||
      a.nv < 1 || a.nv > 5 || batch <= 0)
    return PRISM_EINVAL;
  const size_t lds = (size_t)small_lds_floats(a.sv.ld) * sizeof(float);
  const int rc = allow_dynamic_lds((const void*)small_polar_kernel, (int)(small_lds_floats(64) * sizeof(float)));
  if (rc != PRISM_OK) return rc;
  hipLaunchKernelGGL(small_polar_kernel, dim3(batch), dim3(NT), lds, s, a);
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

void launch_moments(const SolveArgs& a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(moments_kernel, dim3(a.ngroups, batch), dim3(NT), 0, s, a);
}

void launch_solve(const SolveArgs& a, int batch, hipStream_t s) {
  hipLaunchKernelGGL(solve_kernel, dim3(batch), dim3(NT), 0, s, a);
}

}  // namespace prism
