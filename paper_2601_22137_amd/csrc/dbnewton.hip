// Pieces of the PRISM DB Newton iteration in product form (paper App. A.2):
//   N_k = M_k^{-1} for symmetric positive definite M_k   (the paper factors M_k; here: in-place
//         block Gauss-Jordan elimination without pivoting, which is stable for SPD matrices)
//   g00 = <D0,D0>, g02 = <D0,D2>, g22 = <D2,D2>,  D0 = M - I, D2 = M + N - 2I
//         (the O(n^2) quantities behind the quartic m(alpha) = ||I - M_{k+1}||_F^2; the printed
//         trace combinations expand these inner products and cancel badly near convergence)
//   M_{k+1} = 2a(1-a) I + (1-a)^2 M_k + a^2 N_k
// Block Gauss-Jordan: for every pivot block k
//   P = A_kk^{-1},  A_kj <- P A_kj  (j != k),  A_ij <- A_ij - A_ik A_kj  (i, j != k),  A_ik <- -A_ik P  (i != k),  A_kk <- P
// with the three block updates as launches of the fp32 GEMM kernel.  Two levels: pivot blocks of
// 512 or 256 (such rank updates are compute bound: >= 64 flop per byte of the matrix they sweep; with
// blocks of 64 the sweep is HBM bound), each inverted by the same
// elimination with blocks of 64, whose 64 x 64 pivots one workgroup inverts in fp64.  With blocks
// of 64 the updates run in place (one 64 x 64 tile covers a block); with the large blocks the new pivot
// row and column panels go to scratch and are copied back.
#include "common.h"

namespace prism {
namespace {

constexpr int NT = 256;
constexpr int BS = 64;   // block size of the elimination

__global__ __launch_bounds__(NT) void copy_kernel(const float* __restrict__ src, float* __restrict__ dst, long long per_mat,
                                                  const Ctrl* __restrict__ ctrl) {
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const long long i = ((long long)blockIdx.x * NT + threadIdx.x) * 4;
  if (i < per_mat) *(float4*)(dst + (long long)b * per_mat + i) = *(const float4*)(src + (long long)b * per_mat + i);
}

// In-place inverse of the 64 x 64 diagonal block k of every matrix.  Thread t owns row t / 4,
// columns 16 (t % 4) .. +15 in registers (fp64); per elimination step the old pivot row and pivot
// column are exchanged through a double-buffered LDS line, one barrier per step.
__global__ __launch_bounds__(NT) void diag_inv_kernel(float* __restrict__ A, long long stride, int ld, int k,
                                                      const Ctrl* __restrict__ ctrl) {
  const int b = blockIdx.x;
  if (ctrl && ctrl[b].done) return;
  __shared__ double rowbuf[2][BS], colbuf[2][BS];
  const int t = threadIdx.x, i = t >> 2, c0 = (t & 3) * 16;
  float* blk = A + (long long)b * stride + (long long)(k * BS + i) * ld + k * BS + c0;
  double v[16];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const float4 x = *(const float4*)(blk + 4 * q);
    v[4 * q] = x.x; v[4 * q + 1] = x.y; v[4 * q + 2] = x.z; v[4 * q + 3] = x.w;
  }
  for (int p = 0; p < BS; ++p) {
    const int buf = p & 1;
    if (i == p) {
#pragma unroll
      for (int e = 0; e < 16; ++e) rowbuf[buf][c0 + e] = v[e];
    }
    if ((p >> 4) == (t & 3)) {
      double f = 0.0;
#pragma unroll
      for (int e = 0; e < 16; ++e) f = (e == (p & 15)) ? v[e] : f;
      colbuf[buf][i] = f;
    }
    __syncthreads();
    const double inv = 1.0 / rowbuf[buf][p];
    const double f = colbuf[buf][i];
    if (i == p) {
#pragma unroll
      for (int e = 0; e < 16; ++e) v[e] = (c0 + e == p) ? inv : v[e] * inv;
    } else {
#pragma unroll
      for (int e = 0; e < 16; ++e) v[e] = (c0 + e == p) ? -f * inv : v[e] - f * (rowbuf[buf][c0 + e] * inv);
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q)
    *(float4*)(blk + 4 * q) = make_float4((float)v[4 * q], (float)v[4 * q + 1], (float)v[4 * q + 2], (float)v[4 * q + 3]);
}

// grid (groups, batch): partial sums of the three inner products over the true n x n part; the
// five coefficient partials are written where the solve kernel adds them up.
__global__ __launch_bounds__(NT) void db_moments_kernel(const float* __restrict__ M, const float* __restrict__ N, int np,
                                                        int n_true, const Ctrl* __restrict__ ctrl, double* __restrict__ cpart) {
  const int b = blockIdx.y, grp = blockIdx.x, ngrp = gridDim.x;
  if (ctrl[b].done) return;
  const long long total = (long long)np * np;
  const float* Mb = M + (long long)b * total;
  const float* Nb = N + (long long)b * total;
  double g00 = 0.0, g02 = 0.0, g22 = 0.0;
  for (long long idx = ((long long)grp * NT + threadIdx.x) * 4; idx < total; idx += (long long)ngrp * NT * 4) {
    const int r = (int)(idx / np), c = (int)(idx % np);
    if (r >= n_true) break;
    const float4 m4 = *(const float4*)(Mb + idx), n4 = *(const float4*)(Nb + idx);
    const float mv[4] = {m4.x, m4.y, m4.z, m4.w}, nv[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c + e < n_true) {
        const double eye = (r == c + e) ? 1.0 : 0.0;
        const double d0 = (double)mv[e] - eye, d2 = (double)mv[e] + (double)nv[e] - 2.0 * eye;
        g00 += d0 * d0; g02 += d0 * d2; g22 += d2 * d2;
      }
    }
  }
  __shared__ double red[4][3];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) {
    g00 += __shfl_down(g00, off, 64); g02 += __shfl_down(g02, off, 64); g22 += __shfl_down(g22, off, 64);
  }
  if (lane == 0) { red[wave][0] = g00; red[wave][1] = g02; red[wave][2] = g22; }
  __syncthreads();
  if (threadIdx.x == 0) {
    const double a = (red[0][0] + red[1][0]) + (red[2][0] + red[3][0]);
    const double c = (red[0][1] + red[1][1]) + (red[2][1] + red[3][1]);
    const double d = (red[0][2] + red[1][2]) + (red[2][2] + red[3][2]);
    double* out = cpart + ((long long)b * ngrp + grp) * 17;
    out[0] = a; out[1] = -4.0 * a; out[2] = 4.0 * a + 2.0 * c; out[3] = -4.0 * c; out[4] = d;
    for (int s = 5; s < 16; ++s) out[s] = 0.0;   // slot 16 belongs to the check of the inverse (db_probe_kernel)
  }
}

// Check of the inverse with one probe vector v of +-1 entries: ||M (N v) - v||^2 estimates
// ||M N - I||_F^2 (its expectation over such v), i.e. the error of N measured against the smallest
// entries of its spectrum, which is what the large components of X = A^(1/2) inherit.  Pass 0: w = N v.
// Pass 1: partial sums of (M w - v)^2 into slot 16 of the coefficient partials, which the solve
// kernel adds up.
// grid (groups, batch); a wave takes 16 rows at a time (16-byte loads, 16 KiB in flight per wave).  The
// padding needs no mask: M and N are the identity there, so padded rows reproduce v exactly.
__device__ inline float probe_entry(int c) { return ((unsigned)c * 2654435761u >> 16) & 1u ? 1.0f : -1.0f; }
constexpr int PR = 16;   // rows per wave and sweep
__global__ __launch_bounds__(NT) void db_probe_kernel(const float* __restrict__ A, int np, const Ctrl* __restrict__ ctrl,
                                                      float* __restrict__ w, double* __restrict__ cpart, int pass) {
  const int b = blockIdx.y, grp = blockIdx.x, ngrp = gridDim.x;
  if (ctrl[b].done) return;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float* Ab = A + (long long)b * np * np;
  float* wb = w + (long long)b * np;
  double err = 0.0;
  for (int r0 = PR * (4 * grp + wave); r0 < np; r0 += 4 * PR * ngrp) {
    double dot[PR];
#pragma unroll
    for (int k = 0; k < PR; ++k) dot[k] = 0.0;
    for (int c = lane * 4; c < np; c += 256) {
      float4 x;
      if (pass == 0) x = make_float4(probe_entry(c), probe_entry(c + 1), probe_entry(c + 2), probe_entry(c + 3));
      else x = *(const float4*)(wb + c);
#pragma unroll
      for (int k = 0; k < PR; ++k) {
        const float4 a = *(const float4*)(Ab + (long long)(r0 + k) * np + c);
        dot[k] += ((double)a.x * (double)x.x + (double)a.y * (double)x.y) + ((double)a.z * (double)x.z + (double)a.w * (double)x.w);
      }
    }
#pragma unroll
    for (int k = 0; k < PR; ++k) {
#pragma unroll
      for (int off = 32; off > 0; off >>= 1) dot[k] += __shfl_down(dot[k], off, 64);
    }
    if (lane == 0) {
#pragma unroll
      for (int k = 0; k < PR; ++k) {
        if (pass == 0) wb[r0 + k] = (float)dot[k];
        else { const double d = dot[k] - (double)probe_entry(r0 + k); err += d * d; }
      }
    }
  }
  if (pass == 1) {
    __shared__ double red[4];
    if (lane == 0) red[wave] = err;
    __syncthreads();
    if (threadIdx.x == 0) cpart[((long long)b * ngrp + grp) * 17 + 16] = (red[0] + red[1]) + (red[2] + red[3]);
  }
}

// grid (parts, batch)
__global__ __launch_bounds__(NT) void db_update_m_kernel(float* __restrict__ M, const float* __restrict__ N, int np, int n_true,
                                                         const Ctrl* __restrict__ ctrl, float* __restrict__ rho_part) {
  const int b = blockIdx.y;
  if (ctrl[b].done) return;
  const double a = (double)ctrl[b].alpha;
  const double wi = 2.0 * a * (1.0 - a), wm = (1.0 - a) * (1.0 - a), wn = a * a;
  const long long total = (long long)np * np;
  float* Mb = M + (long long)b * total;
  const float* Nb = N + (long long)b * total;
  double rho = 0.0;
  for (long long idx = ((long long)blockIdx.x * NT + threadIdx.x) * 4; idx < total; idx += (long long)gridDim.x * NT * 4) {
    const int r = (int)(idx / np), c = (int)(idx % np);
    if (r >= n_true) break;
    float4 m4 = *(const float4*)(Mb + idx);
    const float4 n4 = *(const float4*)(Nb + idx);
    float mv[4] = {m4.x, m4.y, m4.z, m4.w};
    const float nv[4] = {n4.x, n4.y, n4.z, n4.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      if (c + e < n_true) {
        const double eye = (r == c + e) ? 1.0 : 0.0;
        const double mn = wi * eye + wm * (double)mv[e] + wn * (double)nv[e];
        mv[e] = (float)mn;
        const double d = eye - (double)mv[e];
        rho += d * d;
      }
    }
    *(float4*)(Mb + idx) = make_float4(mv[0], mv[1], mv[2], mv[3]);
  }
  __shared__ double red[4];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) rho += __shfl_down(rho, off, 64);
  if (lane == 0) red[wave] = rho;
  __syncthreads();
  if (threadIdx.x == 0) rho_part[(long long)b * gridDim.x + blockIdx.x] = (float)((red[0] + red[1]) + (red[2] + red[3]));
}

// rows [r0, r0 + nr) x cols [c0, c0 + nc) of every matrix: dst <- src (different leading dimensions)
__global__ __launch_bounds__(NT) void panel_copy_kernel(const float* __restrict__ src, long long sstride, int sld,
                                                        float* __restrict__ dst, long long dstride, int dld, int nr, int nc,
                                                        int skip0, int skip1, int skip_rows, const Ctrl* __restrict__ ctrl) {
  const int b = blockIdx.y;
  if (ctrl && ctrl[b].done) return;
  const long long i = ((long long)blockIdx.x * NT + threadIdx.x) * 4;
  if (i >= (long long)nr * nc) return;
  const int r = (int)(i / nc), c = (int)(i % nc);
  const int key = skip_rows ? r : c;
  if (key >= skip0 && key < skip1) return;       // the pivot block itself is already in place
  *(float4*)(dst + (long long)b * dstride + (long long)r * dld + c) = *(const float4*)(src + (long long)b * sstride + (long long)r * sld + c);
}

// In-place inverse of the n x n SPD matrices at A (leading dimension ld, batch stride `stride`)
// by block Gauss-Jordan with blocks of 64; n a multiple of 64.
int gauss_jordan_64(float* A, long long stride, int ld, int n, int batch, const Ctrl* ctrl, hipStream_t s) {
  const int nb = n / BS;
  for (int k = 0; k < nb; ++k) {
    hipLaunchKernelGGL(diag_inv_kernel, dim3(batch), dim3(NT), 0, s, A, stride, ld, k, ctrl);
    if (nb == 1) break;
    float* Pk = A + (long long)k * BS * ld + k * BS;     // diagonal block (now P)
    float* rowk = A + (long long)k * BS * ld;            // block row k
    float* colk = A + k * BS;                            // block column k
    GemmDesc g = {};
    g.batch = batch; g.ctrl = ctrl; g.K = BS; g.epi = EPI_STORE; g.c_in = 1.0f;
    g.strideA = g.strideB = g.strideC = g.strideCin = stride;
    g.lda = g.ldb = g.ldc = g.ldcin = ld;
    GemmDesc r = g;                                      // A_kj <- P A_kj, j != k
    r.A = Pk; r.B = rowk; r.C = rowk; r.M = BS; r.N = n; r.skip_n0 = k * BS; r.skip_n1 = (k + 1) * BS;
    int rc = launch_gemm_f32(r, BS, BS, s);
    if (rc != PRISM_OK) return rc;
    GemmDesc u = g;                                      // A_ij <- A_ij - A_ik A_kj, i, j != k
    u.A = colk; u.B = rowk; u.C = A; u.Cin = A; u.M = n; u.N = n; u.epi = EPI_AXPY; u.acc_neg = 1;
    u.skip_m0 = u.skip_n0 = k * BS; u.skip_m1 = u.skip_n1 = (k + 1) * BS;
    rc = launch_gemm_f32(u, BS, BS, s);
    if (rc != PRISM_OK) return rc;
    GemmDesc c = g;                                      // A_ik <- -A_ik P, i != k
    c.A = colk; c.B = Pk; c.C = colk; c.M = n; c.N = BS; c.acc_neg = 1; c.skip_m0 = k * BS; c.skip_m1 = (k + 1) * BS;
    rc = launch_gemm_f32(c, BS, BS, s);
    if (rc != PRISM_OK) return rc;
  }
  return PRISM_OK;
}

// outer pivot block: 512 or 256 when it divides the order (0: blocks of 64 only)
int outer_block(int np) { return (np > 512 && np % 512 == 0) ? 512 : ((np > 256 && np % 256 == 0) ? 256 : 0); }

}  // namespace

long long spd_inverse_scratch_floats(int np, int batch) { return 2ll * outer_block(np) * np * batch; }

int launch_spd_inverse(const float* M, float* N, int np, int batch, const Ctrl* ctrl, float* panels, hipStream_t s) {
  if (np % BS || batch <= 0) return PRISM_EINVAL;
  const long long per_mat = (long long)np * np;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)((per_mat / 4 + NT - 1) / NT), batch), dim3(NT), 0, s, M, N, per_mat, ctrl);
  if (spd_inverse_scratch_floats(np, batch) == 0) {
    const int rc = gauss_jordan_64(N, per_mat, np, np, batch, ctrl, s);
    if (rc != PRISM_OK) return rc;
    return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
  }
  if (!panels) return PRISM_EINVAL;
  const int OB = outer_block(np);
  float* Trow = panels;                                   // [batch][OB][np]: P A_k,:
  float* Ucol = panels + (long long)batch * OB * np;      // [batch][np][OB]: -A_:,k P
  const long long tstride = (long long)OB * np, ustride = (long long)np * OB;
  for (int k = 0; k < np / OB; ++k) {
    float* Pk = N + (long long)k * OB * np + k * OB;
    float* rowk = N + (long long)k * OB * np;
    float* colk = N + k * OB;
    int rc = gauss_jordan_64(Pk, per_mat, np, OB, batch, ctrl, s);    // P = A_kk^{-1}, in place
    if (rc != PRISM_OK) return rc;
    GemmDesc g = {};
    g.batch = batch; g.ctrl = ctrl; g.K = OB; g.epi = EPI_STORE; g.c_in = 1.0f;
    GemmDesc r = g;                                      // T = P A_k,:
    r.A = Pk; r.strideA = per_mat; r.lda = np; r.B = rowk; r.strideB = per_mat; r.ldb = np;
    r.C = Trow; r.strideC = tstride; r.ldc = np; r.M = OB; r.N = np; r.skip_n0 = k * OB; r.skip_n1 = (k + 1) * OB;
    rc = launch_gemm_f32(r, 128, 128, s);
    if (rc != PRISM_OK) return rc;
    GemmDesc u = g;                                      // A_ij <- A_ij - A_ik T_j, i, j outside the pivot block
    u.A = colk; u.strideA = per_mat; u.lda = np; u.B = Trow; u.strideB = tstride; u.ldb = np;
    u.C = N; u.strideC = per_mat; u.ldc = np; u.Cin = N; u.strideCin = per_mat; u.ldcin = np;
    u.M = np; u.N = np; u.epi = EPI_AXPY; u.acc_neg = 1;
    u.skip_m0 = u.skip_n0 = k * OB; u.skip_m1 = u.skip_n1 = (k + 1) * OB;
    // A half-swept symmetric matrix is symmetric within the swept and within the unswept blocks and
    // antisymmetric between them, and the update keeps that: upper triangle of tiles only
    u.sym = 1; u.sym_skew_bound = k * OB;
    rc = launch_gemm_f32(u, 128, 128, s);
    if (rc != PRISM_OK) return rc;
    GemmDesc c = g;                                      // U = -A_:,k P
    c.A = colk; c.strideA = per_mat; c.lda = np; c.B = Pk; c.strideB = per_mat; c.ldb = np;
    c.C = Ucol; c.strideC = ustride; c.ldc = OB; c.M = np; c.N = OB; c.acc_neg = 1;
    c.skip_m0 = k * OB; c.skip_m1 = (k + 1) * OB;
    rc = launch_gemm_f32(c, 128, 128, s);
    if (rc != PRISM_OK) return rc;
    hipLaunchKernelGGL(panel_copy_kernel, dim3((unsigned)(((long long)OB * np / 4 + NT - 1) / NT), batch), dim3(NT), 0, s,
                       Trow, tstride, np, rowk, per_mat, np, OB, np, k * OB, (k + 1) * OB, 0, ctrl);
    hipLaunchKernelGGL(panel_copy_kernel, dim3((unsigned)(((long long)np * OB / 4 + NT - 1) / NT), batch), dim3(NT), 0, s,
                       Ucol, ustride, OB, colk, per_mat, np, np, OB, k * OB, (k + 1) * OB, 1, ctrl);
  }
  return hipGetLastError() == hipSuccess ? PRISM_OK : PRISM_EHIP;
}

void launch_db_moments(const float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, double* cpart,
                       int ngroups, hipStream_t s) {
  hipLaunchKernelGGL(db_moments_kernel, dim3(ngroups, batch), dim3(NT), 0, s, M, N, np, n_true, ctrl, cpart);
}

void launch_db_probe(const float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, float* w, double* cpart,
                     int ngroups, hipStream_t s) {
  (void)n_true;
  hipLaunchKernelGGL(db_probe_kernel, dim3(ngroups, batch), dim3(NT), 0, s, N, np, ctrl, w, cpart, 0);
  hipLaunchKernelGGL(db_probe_kernel, dim3(ngroups, batch), dim3(NT), 0, s, M, np, ctrl, w, cpart, 1);
}

void launch_db_update_m(float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, float* rho_part,
                        int nparts, hipStream_t s) {
  hipLaunchKernelGGL(db_update_m_kernel, dim3(nparts, batch), dim3(NT), 0, s, M, N, np, n_true, ctrl, rho_part);
}

}  // namespace prism
