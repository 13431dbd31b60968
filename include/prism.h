/*
 * prism.h - C-ABI of the MI355X (gfx950) PRISM library.
 *
 * PRISM accelerates Newton-Schulz-like matrix iterations by fitting, at every
 * iteration, the highest coefficient alpha_k of the update polynomial
 * g_d(R_k; alpha) to the spectrum of the current residual R_k through a
 * sketched least-squares problem (paper Sections 3-4, eq. (2)-(4)).
 * The iterations of Table 1 and Section 4 are provided:
 *
 *   prism_polar        polar factor U V^T          R_k = I - X_k^T X_k
 *   prism_sqrt         A^{1/2} and A^{-1/2}        R_k = I - Y_k X_k   (Theorem 3)
 *   prism_inv_root     A^{-1/p}                    R_k = I - M_k       (App. A.3)
 *   prism_sign         sign(A)                     R_k = I - X_k^2     (Section 4)
 *   prism_inverse      A^{-1} (Chebyshev)          R_k = I - A X_k     (App. A.4)
 *   prism_sqrt_newton  A^{1/2} and A^{-1/2}        R_k = I - M_k       (DB Newton, App. A.2)
 *   prism_run_grouped  any of them over groups of different shapes in one call
 *
 * Conventions common to all entry points
 *   - Every matrix pointer is a DEVICE pointer to row-major, contiguous,
 *     batch-strided data: x[batch][m][n].  The caller owns all of it.  Alignment
 *     to the element size is enough; bf16 arrays aligned to 16 bytes are copied
 *     in and out with vector accesses, and a 256-byte aligned bf16 array whose
 *     sides are tile multiples may be used as scratch for intermediate iterates
 *     between the moment its input has been read and the end of the call.
 *   - `dt` is the storage type of the caller's matrices.  PRISM_F32 computes
 *     with fp32 matrix instructions (the inverse-root recurrence for M_k in
 *     fp64); PRISM_BF16 computes with bf16 matrix instructions accumulating in
 *     fp32 and is available for prism_polar only (the iterate is carried as
 *     a pair of bf16 matrices while small singular values need it).
 *   - `degree` is the degree of the update in X: 3 (d = 1) or 5 (d = 2).
 *   - `sketch_dim` = p_s, the number of rows of the Gaussian sketch S_k
 *     (1..64).  0 disables the fit: alpha_k stays at the Taylor value, which is
 *     the classical iteration.
 *   - `seed` selects the sketch stream; S_k depends only on (seed, k, function)
 *     and is shared by all matrices of the call.
 *   - `tol` > 0: iterate until ||R_k||_F / sqrt(n_R) <= tol (n_R = order of
 *     R_k), at most `max_iters` updates.  `tol` <= 0: exactly `max_iters`
 *     updates.  max_iters <= PRISM_MAX_ITERS.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only
 *     enqueue work on it and return; nothing synchronises with the host and
 *     there is no host round trip per iteration.
 *   - The return value reports errors the host can detect (prism_status).
 *     Numerical outcomes are reported per matrix in prism_info.status.
 *   - Unless a workspace is passed through prism_options, the library keeps
 *     one grow-only device workspace per (device, stream); calls that share
 *     it must be ordered on that stream.  A block that a larger call outgrows
 *     stays allocated (earlier work and captured HIP graphs still point into
 *     it) until prism_release_workspaces().  Exception: prism_run_grouped, and
 *     single-shape calls that the library splits into two half batches (an even
 *     batch >= 8 of matrices with min(m, n) >= 1024 and no caller workspace), run
 *     on four library-owned streams per device, each with a cached workspace of
 *     its own, whatever the caller's stream.  Such calls are enqueued one at a
 *     time (a process-wide lock) and are ordered after one another on those
 *     streams, so eager calls from different caller streams are safe but do not
 *     overlap; HIP graphs captured from such calls share those workspaces and
 *     must not be replayed concurrently with each other or with another such
 *     call.  Pass a workspace through prism_options to keep a call on its own
 *     stream and memory.
 *   - A matrix whose info.status is PRISM_INFO_NONFINITE or PRISM_INFO_ZERO is
 *     left untouched.
 *   - Empty input (batch, m or n equal to 0; a grouped call with no groups) is
 *     valid: the other arguments are checked, nothing is enqueued, no pointer is
 *     read (they may be NULL) and the call returns PRISM_OK.  Negative extents
 *     are PRISM_EINVAL.
 *   - Size limits: at most 2^31 - 1 entries per matrix, counted with both
 *     sides rounded up to the next multiple of 256 (bf16 with min(m, n) >=
 *     512), 128 or 64 (fp32 with min(m, n) <= 256), and batch <=
 *     PRISM_MAX_BATCH matrices per call; beyond them PRISM_EUNSUPPORTED.
 */
#ifndef PRISM_H
#define PRISM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define PRISM_MAX_ITERS 64
#define PRISM_MAX_SKETCH 64
#define PRISM_MAX_ROOT 8
#define PRISM_MAX_BATCH 65535 /* matrices per call (per group of a grouped call) */

typedef enum { PRISM_F32 = 0, PRISM_BF16 = 1 } prism_dtype;

typedef enum {
  PRISM_OK = 0,
  PRISM_EINVAL = 1,       /* null pointer, bad size, degree, root order, budget ... */
  PRISM_EUNSUPPORTED = 2, /* combination not implemented (e.g. bf16 square root) */
  PRISM_ENOMEM = 3,       /* workspace allocation failed or passed workspace too small */
  PRISM_EHIP = 4          /* a HIP runtime call failed */
} prism_status;

/* function ids; also the function tag of the sketch counter */
typedef enum {
  PRISM_FN_POLAR = 1, PRISM_FN_SQRT = 2, PRISM_FN_INV_ROOT = 3, PRISM_FN_SIGN = 4, PRISM_FN_INVERSE = 5,
  PRISM_FN_SQRT_NEWTON = 6
} prism_fn;

enum {
  PRISM_INFO_CONVERGED = 0, /* residual <= tol after `iters` updates */
  PRISM_INFO_BUDGET = 1,    /* max_iters updates done (the normal outcome when tol <= 0) */
  PRISM_INFO_NONFINITE = 2, /* input holds inf or nan */
  PRISM_INFO_ZERO = 3,      /* input is all zero */
  PRISM_INFO_DIVERGED = 4   /* residual non-finite, or rising twice in a row above its start */
};

/* Per-matrix report, written on the device.  residual[k] = ||R_k||_F / sqrt(n_R)
 * for k = 0..iters (residual[max_iters] is not evaluated when tol <= 0 and is
 * set to -1); alpha[k] is the coefficient used by update k. */
typedef struct {
  int32_t iters;
  int32_t status;
  float residual[PRISM_MAX_ITERS + 1];
  float alpha[PRISM_MAX_ITERS];
} prism_info;

enum {
  /* bf16 polar only: keep the iterate X_k in plain bf16 between iterations (one
   * matrix-core pass per update).  By default X_k is carried as a pair of bf16
   * matrices (high + low part, two passes per update), which is what an
   * ill-conditioned input needs to reach its own polar factor. */
  PRISM_FLAG_BF16_PLAIN_ITERATE = 1u,
  /* Scheduling hint, results unchanged: other work of the caller runs on the GPU beside this
   * call (calls for other shapes on other streams).  The bf16 Gram product then takes 256 x 256
   * tiles even when they are too few to fill the chip: they move half the bytes per flop and
   * leave whole CUs to the other work.  prism_run_grouped sets it for its groups. */
  PRISM_FLAG_SHARED_GPU = 2u,
  /* Keep every kernel of the call on the caller's stream: no internal streams (prism_run_grouped
   * then runs its groups, or the one launch sequence over all of them, one after the other; a
   * single-shape call is not split into half batches).  Results unchanged.  For callers that time
   * kernels one by one or must not have work on streams they do not own. */
  PRISM_FLAG_SINGLE_STREAM = 4u
};

typedef struct {
  uint32_t flags;         /* PRISM_FLAG_* */
  int32_t warm_iters;     /* the first warm_iters updates use alpha = u without a fit (App. C) */
  void* workspace;        /* device memory, 256-byte aligned, or NULL for the cached one */
  size_t workspace_bytes; /* size of `workspace` */
  prism_info* info;       /* device array of `batch` entries, or NULL */
  const float* alpha_schedule; /* HOST array, read before the call returns, or NULL: update k <
                                * schedule_len uses alpha_schedule[k] as given (no fit, no clamp);
                                * fixed-coefficient schemes run through the same kernels this way */
  int32_t schedule_len;   /* 0 <= schedule_len <= PRISM_MAX_ITERS */
} prism_options;

/* Frees every cached workspace of the calling process (all devices and streams).  The caller guarantees that no call of the library is in flight and that
 * no HIP graph captured from one will be launched again.  The next call allocates anew. */
int prism_release_workspaces(void);

/* Device bytes a call with these arguments needs (host-only computation). */
int prism_workspace_bytes(int fn, int batch, int m, int n, prism_dtype dt, int degree,
                          int sketch_dim, int root_p, size_t* out_bytes);

/* Polar factor (Table 1, "Newton-Schulz, U V^T"; App. A.1).  x[batch][m][n] is
 * replaced in place by U V^T.  m < n is handled on the transpose. */
int prism_polar(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                int sketch_dim, uint64_t seed, double tol, void* stream);
int prism_polar_ex(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                   int sketch_dim, uint64_t seed, double tol, void* stream,
                   const prism_options* opt);

/* prism_polar_ex for callers that cannot allocate device memory: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the
 * same results as prism_polar_ex on one stream, but every intermediate (iterates, R, Q, sketches,
 * chain vectors, control blocks) lives in a static device array of PRISM_STATIC_SCRATCH_BYTES
 * that is part of the library's code object: each GPU the library runs on holds its own copy
 * until the process ends.  The call makes no hipMalloc / hipFree, creates no stream or event and
 * records no hipMemsetAsync; it enqueues kernels on `stream` and returns.
 *   - opt may be NULL; opt->workspace must be NULL (PRISM_EINVAL otherwise).  opt->info, flags,
 *     warm_iters and the coefficient schedule work as in prism_polar_ex.
 *   - A call whose intermediates need more than the array (prism_workspace_bytes tells; e.g. one
 *     1024 x 1024 bf16 matrix with the split iterate needs 27 MB, sixteen 768 x 768 ones do not
 *     fit) returns PRISM_EUNSUPPORTED before anything is enqueued, with a message in
 *     prism_last_error().
 *   - All calls on one GPU share that GPU's array, which keeps the contents of the last call;
 *     every call initialises what it reads.  Two calls that overlap in time on one GPU (different
 *     streams, or concurrent replays of graphs captured from them) race: order them.
 *   - Timing through prism_profile_enable does not see this call. */
#define PRISM_STATIC_SCRATCH_BYTES (32u << 20)
int prism_polar_static(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                       int sketch_dim, uint64_t seed, double tol, void* stream,
                       const prism_options* opt);

/* Coupled square root (Table 1, "A^{1/2}, A^{-1/2}"; Theorem 3).  a[batch][n][n]
 * symmetric positive definite is replaced by A^{1/2}; inv_out[batch][n][n]
 * receives A^{-1/2}.  m must equal n. */
int prism_sqrt(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int degree,
               int max_iters, int sketch_dim, uint64_t seed, double tol, void* stream);
int prism_sqrt_ex(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int degree,
                  int max_iters, int sketch_dim, uint64_t seed, double tol, void* stream,
                  const prism_options* opt);

/* Coupled inverse Newton (Table 1, "Coupled Inverse Newton"; App. A.3).
 * a[batch][n][n] symmetric positive definite is replaced by A^{-1/root_p},
 * 1 <= root_p <= PRISM_MAX_ROOT.  The update is linear in R_k: degree must be 3. */
int prism_inv_root(void* a, int root_p, int batch, int m, int n, prism_dtype dt, int degree,
                   int max_iters, int sketch_dim, uint64_t seed, double tol, void* stream);
int prism_inv_root_ex(void* a, int root_p, int batch, int m, int n, prism_dtype dt, int degree,
                      int max_iters, int sketch_dim, uint64_t seed, double tol, void* stream,
                      const prism_options* opt);

/* Matrix sign (Section 4, eq. (2)-(4)): x[batch][n][n], square with x^2 symmetric, is replaced
 * in place by sign(x) = x (x^2)^{-1/2}.  X_0 = x / ||x||_F, R_k = I - X_k^2,
 * X_{k+1} = X_k g_d(R_k; alpha_k).  m must equal n; fp32 only (bf16: PRISM_EUNSUPPORTED). */
int prism_sign(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
               int sketch_dim, uint64_t seed, double tol, void* stream);
int prism_sign_ex(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                  int sketch_dim, uint64_t seed, double tol, void* stream,
                  const prism_options* opt);

/* Inverse by the PRISM Chebyshev iteration (Table 1, "Chebyshev"; App. A.4): a[batch][n][n],
 * square and of full rank (symmetry is not needed), is replaced in place by a^{-1}.
 * A_s = a / ||a||_F, X_0 = A_s^T, R_k = I - A_s X_k, X_{k+1} = X_k (I + R_k + alpha_k R_k^2),
 * alpha_k in [1/2, 2] minimises the sketched next residual (a quadratic); sketch_dim = 0
 * keeps alpha_k = 1, the classical iteration.  m must equal n; fp32 only. */
int prism_inverse(void* a, int batch, int m, int n, prism_dtype dt, int max_iters, int sketch_dim,
                  uint64_t seed, double tol, void* stream);
int prism_inverse_ex(void* a, int batch, int m, int n, prism_dtype dt, int max_iters,
                     int sketch_dim, uint64_t seed, double tol, void* stream,
                     const prism_options* opt);

/* Square root and inverse square root by the PRISM DB Newton iteration in product form (Table 1,
 * "DB Newton"; App. A.2): a[batch][n][n] symmetric positive definite is replaced by A^{1/2},
 * inv_out[batch][n][n] receives A^{-1/2}.  M_0 = X_0 = A, Y_0 = I, N_k = M_k^{-1} (block
 * Gauss-Jordan on the device), alpha_k minimises ||I - M_{k+1}||_F^2 over [0, 1] from exact O(n^2)
 * inner products (no sketch); fit = 0 keeps alpha_k = 1/2, the classical iteration.  The stop rule
 * tests ||I - M_k||_F / sqrt(n).  m must equal n; fp32 only; options.warm_iters is ignored.
 * Accuracy: the results inherit the error of the fp32 inverses, about cond(A) * 6e-8 * sqrt(n)
 * (1e-2 at cond 1e4, n = 1024), where prism_sqrt loses about sqrt(cond(A)) * 6e-8 * sqrt(n); a matrix
 * whose inverse misses ||M_k N_k v - v|| <= 0.1 ||v|| for a fixed probe vector v of +-1 entries
 * (checked every iteration) stops with PRISM_INFO_DIVERGED and its current iterate: about cond 1e4
 * at n = 1024; prism_sqrt handles such inputs. */
int prism_sqrt_newton(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int max_iters,
                      int fit, double tol, void* stream);
int prism_sqrt_newton_ex(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt,
                         int max_iters, int fit, double tol, void* stream,
                         const prism_options* opt);

/* ---- one call over groups of different shapes (an optimizer step over all parameters) ----
 *
 * Callers: a Muon-style step orthogonalises the gradient of every weight matrix, a Shampoo-style
 * step takes the inverse root of every preconditioner; the matrices come in a few shapes, each a
 * batch.  The groups are independent.
 *   - bf16 polar factors of up to 8 groups that share min(m, n) (the weight shapes of a layer stack
 *     do: 768 x 768, 768 x 3072, 3072 x 768, 768 x 2304) run as ONE launch sequence over all their
 *     matrices: R_k, Q_k, the chain vectors and the control blocks of every matrix form a single
 *     batch, so R^2, the chain products, the moments and the solve are one launch each for the
 *     whole call, and the Gram product and the update take all shapes in one launch each (the
 *     kernel maps its workgroup index to group, matrix and tile).  When every group's batch is a
 *     multiple of 4 (of 2) the sequence is issued for the quarters (halves) of every group on
 *     internal streams, so that the latency-bound steps of one part run beside the products of
 *     another.
 *   - any other combination runs each group as its own call on one of four internal streams.
 * The internal streams have default priority and fork from and join back into `stream` (event
 * record / wait only: the call stays asynchronous and capturable once the library's workspaces
 * exist, i.e. after one eager call with the same arguments on the same stream).  Every group is
 * computed exactly as by its own single-group call: same kernels, same bits. */
typedef struct {
  void* x;          /* device: [batch][m][n], replaced in place as by the single-group call */
  void* inv_out;    /* device: second output of prism_sqrt / prism_sqrt_newton, else NULL */
  prism_info* info; /* device array of `batch` entries, or NULL */
  int32_t batch, m, n;
} prism_group;

/* fn selects the iteration (PRISM_FN_*); root_p is used by PRISM_FN_INV_ROOT only, degree by the
 * Newton-Schulz family, sketch_dim by all but PRISM_FN_SQRT_NEWTON (where non-zero means "fit").
 * opt may be NULL; its workspace and info fields must be NULL (each internal stream keeps its own
 * cached workspace).  Returns the first error of any group; nothing is enqueued for the groups
 * after it. */
int prism_run_grouped(prism_fn fn, const prism_group* groups, int ngroups, int root_p, prism_dtype dt,
                      int degree, int max_iters, int sketch_dim, uint64_t seed, double tol,
                      void* stream, const prism_options* opt);

/* ---- single steps of the path, exposed for unit tests and profiling ---- */

/* S_k^T (Section 4.2: Gaussian sketch): out[n][sketch_dim] fp32 on the device,
 * unit-variance entries; entry (j, r) depends only on (seed, k, fn, r, j). */
int prism_sketch(float* out, int n, int sketch_dim, uint64_t seed, int k, int fn, void* stream);

/* The two Box-Muller factors for `count` consecutive 24-bit arguments starting
 * at `first`: radius[i] = sqrt(-2 ln((first+i+1) 2^-24)), (cosv, sinv)[i] =
 * (cos, sin)(2 pi (first+i) 2^-24).  Device arrays of doubles. */
int prism_gauss_parts(uint32_t first, uint32_t count, double* radius, double* cosv, double* sinv,
                      void* stream);

/* One product of the sketch chain (Section 4.2, App. A.1): out[batch][n][ld] = R[batch][n][n] *
 * V[batch][n][ld], fp32 device arrays, n a multiple of 64, ld = 16, 32 or 64. */
int prism_chain_product(const float* R, const float* V, float* out, int batch, int n, int ld,
                        void* stream);
/* The same product as the bf16 polar path takes it: the off-diagonal entries of R are read from
 * Rb, its copy in bf16 bit patterns (same shape), the diagonal from R itself:
 * out = (Rb + diag(R - Rb)) * V.  ld = 16 or 32, n a multiple of 64 (of 256 when (n / 64) * batch >= 128);
 * other shapes return PRISM_EUNSUPPORTED (the library then keeps to the fp32 matrix).
 * Launches of (n / 64) * batch >= 128 workgroups read V as three bf16 planes (the exact 8 + 8 + 8 bit
 * split of every fp32 entry, laid out [matrix][k / 256][plane][column][u'][8] with u = (k % 256) / 8,
 * u' = (u & 16) | ((u ^ column) & 15): the image of the kernel's LDS stage) and write their
 * result in that form too, for the next product of the chain: `planes` is device scratch of
 * 2 * batch * n * ld * 3 entries; on return its first half holds the planes of V, the second half
 * those of out.  It may be null for smaller launches, which do not use it. */
int prism_chain_product_bf16(const uint16_t* Rb, const float* R, const float* V, float* out,
                             uint16_t* planes, int batch, int n, int ld, void* stream);

/* Inverse of symmetric positive definite matrices by block Gauss-Jordan elimination without
 * pivoting (the N_k = M_k^{-1} step of DB Newton, App. A.2): out[batch][n][n] = a^{-1}, fp32
 * device arrays, n a multiple of 64, a is left unchanged. */
int prism_spd_inverse(const float* a, float* out, int batch, int n, void* stream);

/* C[batch][M][N] = A * B on the matrix cores, no epilogue.  Device pointers.
 *   prism_gemm_f32 : fp32 in/out; bit 0 of a_km: A is stored [K][M].  B is [K][N].  Bit 1: the
 *                    caller asserts A B is symmetric (M = N, tile-sized); only the tiles on and
 *                    above the diagonal are computed and the rest is their mirror image.
 *   prism_gemm_f64a: A fp32 (promoted), B and C fp64, A stored [M][K].
 *   prism_gemm_bf16_nt: A [M][K], B [N][K] bf16 bit patterns, C fp32 = A B^T.  `tile` = 128, 256
 *                    (square tiles) or 2561 (256 x 128); + 20000: B is stored [K][N] (row length N);
 *                    + 10000: A is stored [K][M] and B [K][N] (row lengths M and N).
 * M, N must be multiples of 128 (bf16: of the tile's sides; fp32 skinny N = 16, 32, 64 also
 * allowed) and K of 64. */
int prism_gemm_f32(const float* A, const float* B, float* C, int batch, int M, int N, int K,
                   int a_km, void* stream);
int prism_gemm_f64a(const float* A, const double* B, double* C, int batch, int M, int N, int K,
                    void* stream);
int prism_gemm_bf16_nt(const uint16_t* A, const uint16_t* B, float* C, int batch, int M, int N,
                       int K, int tile, void* stream);

/* Per-kernel timing for benchmarks: while enabled, every kernel launch of the library is
 * bracketed by a HIP event pair on the caller's stream.  prism_profile_enable(on) also discards
 * what was recorded so far.  prism_profile_collect waits for the recorded events and returns the
 * summed milliseconds and the launch counts per kernel kind (host arrays of PRISM_PROFILE_KINDS
 * entries; nkinds >= PRISM_PROFILE_KINDS).  Meant for a single benchmarking thread; calls from
 * other threads while it is enabled are recorded too (the record list is locked). */
#define PRISM_PROFILE_KINDS 20
int prism_profile_enable(int on);
int prism_profile_collect(double* ms_by_kind, long long* launches_by_kind, int nkinds);

/* Last HIP error string seen by the library on this thread ("" if none). */
const char* prism_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* PRISM_H */
