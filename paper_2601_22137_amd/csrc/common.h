// Internal declarations shared by the translation units of libprism (not part of the C-ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "prism.h"

namespace prism {

// Per-matrix control block, device resident.  Written by the prepare and solve
// kernels, read by every kernel of the iteration (done != 0 => the matrix is skipped).
struct Ctrl {
  int done;      // 0 while iterating
  int iters;     // updates performed
  int status;    // PRISM_INFO_*
  int plain;     // bf16 polar with a split iterate: the fit has left the upper end of its interval (no small
                 // singular value is left): the update stops adding the low half's share of the product
  float alpha;   // coefficient of the update being applied
  float res0;    // residual at k = 0
  float res1;    // residual at k - 1
  float res2;    // residual at k - 2
  double norm;   // ||A||_F of the input
  double scale;  // factor applied to the input when it is copied in
};

// ---- gemm_f32.hip : fp32 / fp64 matrix-core GEMMs with fused epilogues ----
enum EpiKind {
  EPI_STORE = 0,     // C = +-acc
  EPI_RESIDUAL = 1,  // R = I - acc (masked to n x n), rho partial
  EPI_POLYQ = 2,     // Q = c1 * Rin + alpha * acc
  EPI_AXPY = 3,      // C = c_in alpha^a * Cin + alpha^b * Cin2 + alpha^c * acc   (a, b, c in 0..2; Cin2 optional)
  EPI_MNEXT = 4      // fp64: M' = Cin + acc, R32' = I - M' (masked), rho partial
};

struct GemmDesc {
  const void* A; long long strideA; int lda;
  const void* B; long long strideB; int ldb;
  int M, N, K;          // padded sizes: multiples of the tile sizes
  int a_km;             // A stored [K][M] instead of [M][K]
  int sym;              // the exact result is symmetric: compute the upper triangle of tiles, mirror the rest
  int ctrl_fixed;       // ctrl[0] applies to every batch entry (the parts of a split-K product)
  int tile_blocks;      // set by the launcher: tiles are taken in blocks of 8 x 8 (plain products, grids of 8 x 8 multiples)
  int batch;
  // epilogue operands
  int epi;
  int n_true;           // unpadded order for masks
  void* C; long long strideC; int ldc;           // main output (float, or double for EPI_MNEXT / f64 store)
  const void* Cin; long long strideCin; int ldcin;  // extra input (R for POLYQ, X for AXPY)
  float* R32out; long long strideR; int ldr;     // EPI_MNEXT: fp32 residual out
  float c1;             // POLYQ: coefficient of Rin
  float c_in;           // AXPY: coefficient of Cin
  const float* Cin2;    // AXPY: optional second addend, same layout as Cin
  int coef_is_alpha;    // AXPY: power of ctrl.alpha (0, 1, 2) that multiplies acc
  int cin_alpha_pow;    // AXPY: power of ctrl.alpha that multiplies Cin (besides c_in)
  int cin2_alpha_pow;   // AXPY: power of ctrl.alpha that multiplies Cin2
  int cin_one_minus_alpha;  // AXPY: Cin is weighted by (1 - ctrl.alpha) (DB Newton updates)
  int acc_neg;          // STORE, AXPY: acc enters with a minus sign
  int sym_skew_bound;   // sym: the mirror image of a tile gets a minus sign when exactly one of its row and column
                        // blocks lies below this index (half-swept matrices of the block Gauss-Jordan inverse); 0: none
  int skip_m0, skip_m1; // output tiles starting in rows [skip_m0, skip_m1) are left untouched (0, 0: none)
  int skip_n0, skip_n1; // likewise for columns
  float* rho_part;      // [batch][tiles] partial sums of R^2 (RESIDUAL / MNEXT)
  const Ctrl* ctrl;     // may be null (test entry points)
};

// tile: 64 or 128 (square tiles), or skinny N (16/32/64) with tile_m 64/128 for the sketch chain
int launch_gemm_f32(const GemmDesc& g, int tile_m, int tile_n, hipStream_t s);
int launch_gemm_f64a(const GemmDesc& g, int tile_m, int tile_n, hipStream_t s);  // A float, B/C double

// ---- gemm_bf16.hip : bf16 matrix-core NT GEMMs (both operands K-contiguous) ----
enum Bf16Epi {
  BEPI_STORE = 0,   // C(fp32) = acc
  BEPI_GRAM = 1,    // R = I - acc: R32 (fp32) and Rb (bf16), rho partial
  BEPI_POLYQ = 2,   // Q(bf16) = c1 * R32 + alpha * acc
  BEPI_APPLY = 3    // X' = Xhi + (1 + c) Xlo + acc -> Xa_hi', Xa_lo' ([L][S]); acc = Xhi B
};

struct Bf16Desc {
  int km;                                            // bit 0: A stored [K][M], bit 1: B stored [K][N] (lda / ldb: elements between k-rows)
  const uint16_t* A; long long strideA; int lda;    // [M][K]
  const uint16_t* B; long long strideB; int ldb;    // [N][K]
  int M, N, K, batch;
  int epi;
  int sym;                                           // GRAM / POLYQ with A == B: compute the upper triangle of tiles only
  int n_true;                                        // GRAM mask
  float* C32; long long strideC32; int ldc32;        // STORE / GRAM fp32 out; POLYQ fp32 in.  Null with `diag` set:
  int upper32;                                       // GRAM: the fp32 matrix is written in the computed tiles only (no mirror image):
                                                     // enough for the R^2 epilogue and for readers of the diagonal
  float* diag; long long strideDiag;                 // symmetric GRAM writes only the bf16 copy and the fp32 diagonal, POLYQ reads the bf16 copy (Cin)
  const uint16_t* Cin16;                             // POLYQ without C32: R in bf16 (layout of Cb)
  uint16_t* Cb; long long strideCb; int ldcb;        // GRAM: Rb out; POLYQ: Q out; APPLY: Xa_hi' out
  uint16_t* Cb2;                                     // APPLY: Xa_lo' out (null in plain mode)
  const uint16_t* Xhi; const uint16_t* Xlo;          // APPLY: current iterate (same layout as Cb)
  float c1;
  int coef_is_alpha;                                 // APPLY: multiply acc by ctrl.alpha (d = 1)
  float* rho_part;                                   // GRAM: partial sums of R^2, one slot per computed tile: b * tiles + tile
  const Ctrl* ctrl;
  int xcd_blocks;                                    // set by launch_gemm_bf16: 4 x 8 tile blocks per XCD
  int ctrl_fixed;                                    // ctrl[0] applies to every batch entry (the parts of a split-K product)
};
// One launch over up to BF16_MAX_GROUPS products of the same kind (epilogue, symmetry) and
// different shapes: workgroup index -> (group, matrix, tile) through the running tile counts.
constexpr int BF16_MAX_GROUPS = 8;
struct Bf16Multi {
  Bf16Desc d[BF16_MAX_GROUPS];
  int tile_start[BF16_MAX_GROUPS + 1];               // set by the launcher
  int ngroups;
  int xcd_private;                                   // set by the launcher: contiguous tile ranges per XCD
  int waves8;                                        // set by the launcher: 256 x 256 tiles run with eight wavefronts
};
// tile_m x tile_n: 256 x 256, 256 x 128 or 128 x 128; M, N of every group must be multiples of them
int launch_gemm_bf16(const Bf16Desc& g, int tile_m, int tile_n, hipStream_t s);
int launch_gemm_bf16_multi(const Bf16Desc* groups, int ngroups, int tile_m, int tile_n, hipStream_t s);

// ---- sketch.hip ----
// v0[k - k_first][rows_total][ld] for k = k_first .. k_first + k_count - 1
void launch_sketch(float* v0, int rows_total, int n, int ld, int p_s, uint64_t seed, int k_first, int k_count, int fn,
                   hipStream_t s);
void launch_gauss_parts(uint32_t first, uint32_t count, double* r, double* c, double* sn,
                        hipStream_t s);

// ---- chain.hip : V_out = R V_in for the sketch chain (HBM bound; R read once, straight into registers) ----
// sel_batch: the batch size that picks the kernel variant (0: batch).  A launch over the matrices of
// several shape groups passes the size of one group, so that each matrix gets the kernel, hence the
// summation order and the bits, of a call on its own group.
int launch_chain(const float* R, long long strideR, int ldr, const float* Vin, long long strideVin, float* Vout,
                 long long strideVout, int n, int ld, int batch, const Ctrl* ctrl, hipStream_t s, int sel_batch = 0);
// true: (n, ld, batch) takes the 16-row kernels (few workgroups otherwise); rb: the bf16 variants
bool chain_takes_small_kernel(int n, int ld, int batch, bool rb);
// Rb: bf16 copy of R [batch][n][ldr]; D: its exact fp32 diagonal, entry i of matrix b at D[b * strideD + i * ldd]
// (ldd = ld of R + 1 reads it out of the full fp32 matrix, ldd = 1 out of a compact array)
int launch_chain_tiny(const float* R, long long strideR, int ldr, const float* V0, long long strideV0, float* Vout,
                      long long strideJ, long long strideB, int nv, int ld, int batch, const Ctrl* ctrl, hipStream_t s);
bool chain_bf16_supported(int n, int ld, int batch, int ldr);
// bf16 R, launches too large for the 16-row kernel: V is read as three bf16 planes (the exact 8 + 8 + 8 bit
// split of its fp32 entries) laid out [matrix][k / 256][plane][column][unit'][8 k] (chain.hip); Vin (fp32) serves the
// diagonal term; the result goes to Vout (fp32) and, if Pout is given, to planes for the next product.
int launch_chain_planes(const unsigned short* Rb, long long strideR, int ldr, const float* D, long long strideD, int ldd,
                        const float* Vin, long long strideVin, const unsigned short* Pin, long long stridePin, float* Vout,
                        long long strideVout, unsigned short* Pout, long long stridePout, int n, int ld, int batch,
                        const Ctrl* ctrl, hipStream_t s, int sel_batch = 0);
int launch_split_planes(const float* V, unsigned short* P, int n, int ld, int count, hipStream_t s);
int launch_chain_bf16(const unsigned short* Rb, long long strideR, int ldr, const float* D, long long strideD, int ldd,
                      const float* Vin, long long strideVin, float* Vout, long long strideVout, int n, int ld, int batch,
                      const Ctrl* ctrl, hipStream_t s, int sel_batch = 0);

// ---- fit.hip ----
struct SolveArgs {
  int fn;            // PRISM_FN_*
  int k;             // iteration index
  int d;             // NS order (1, 2); unused for inverse root
  int p;             // root order (inverse root)
  int n;             // unpadded order of R
  int rows;          // padded rows of V
  int ld;            // leading dimension (padded sketch columns) of V
  const float* V;    // V_1 .. V_nv: [nv][batch][rows][ld]; V_j at V + (j-1)*vstride
  long long vstride; // elements between V_j and V_{j+1}
  long long bstride; // elements between matrices inside one V_j
  const float* rho_part; int nparts;
  Ctrl* ctrl;
  prism_info* info;
  double tol;
  int max_iters;
  int mode;          // 0 fit, 1 Taylor alpha (no sketch), 2 alpha = u (warm start), 3 alpha = sched_alpha
  float sched_alpha; // mode 3: the caller's coefficient for this update
  int last;          // this is the residual-only evaluation at k = max_iters
  int phase;         // 0: stop test and coefficient; 1: stop test only; 2: coefficient only (DB Newton: the
                     //    inverse that the coefficient needs is computed between the two)
  double* cpart;     // [batch][ngroups][17] partial coefficient sums (moments -> solve)
  int ngroups;
};
void launch_moments(const SolveArgs& a, int batch, hipStream_t s);
void launch_solve(const SolveArgs& a, int batch, hipStream_t s);

// fp32 polar factor of matrices whose padded iterate is 64 x 64: every iteration (residual, sketch
// chain, fit, update) runs inside one workgroup per matrix, the iterate never leaves the LDS and one
// launch replaces the five launches per iteration of the general path.
struct SmallPolarArgs {
  SolveArgs sv;              // k, mode and sched_alpha are filled in per iteration by the kernel;
                             // the residual sum and the moments stay in LDS (rho_part, cpart unused)
  float* X[2];               // [batch][64][64]: input in X[0], result left in X[iterations & 1]
  const float* V0;           // S_k^T for k = first_fit, first_fit + 1, ...: [.][64][ld]
  int nv;                    // products in the chain (2 d + 1)
  int p_s, first_fit, warm, sched_len;
  float sched[PRISM_MAX_ITERS];
};
int launch_small_polar(const SmallPolarArgs& a, int batch, hipStream_t s);

// ---- misc.hip ----
struct PrepArgs {
  int fn; int dt; int batch; int m, n;     // caller's shape
  int S, L, Sp, Lp;                         // short / long side and padded sizes
  int transpose;                            // polar with m < n: internal iterate is the transpose
  int root_p;
  const void* src;
  double* sumsq_part; int nsum;             // [batch][nsum]
  Ctrl* ctrl; prism_info* info;
  // outputs (which are used depends on fn/dt)
  float* X32; float* Y32; double* M64; float* R32;   // fp32 paths (inverse: Y32 = A / ||A||_F)
  uint16_t* Xa_hi; uint16_t* Xa_lo;                  // bf16 polar: iterate [Lp][Sp], high and low halves
  float* rho_part; int tile;                // inverse root: residual of M_0
};
void launch_sumsq(const PrepArgs& a, hipStream_t s);
void launch_prepare(const PrepArgs& a, hipStream_t s);

struct FinalArgs {
  int fn; int dt; int batch; int m, n; int S, L, Sp, Lp; int transpose;
  void* dst; void* dst2;                    // caller's arrays (dst2 = inverse square root)
  const Ctrl* ctrl;
  const float* X32[2]; const float* Y32[2];
  const uint16_t* Xa_hi[2]; const uint16_t* Xa_lo[2];
};
void launch_finalize(const FinalArgs& a, hipStream_t s);
struct PrepMulti { PrepArgs d[BF16_MAX_GROUPS]; int start[BF16_MAX_GROUPS + 1]; int ngroups; };
struct FinalMulti { FinalArgs d[BF16_MAX_GROUPS]; int start[BF16_MAX_GROUPS + 1]; int ngroups; };
// one launch each over several shape groups (bf16 polar); false: not applicable, launch group by group
bool launch_prep_multi(const PrepArgs* groups, int ngroups, hipStream_t s);
bool launch_finalize_multi(const FinalArgs* groups, int ngroups, hipStream_t s);

// The per-matrix reports of a launch sequence over several shape groups sit in one array; each group's
// part goes to the array its caller gave (one launch instead of a copy per group).
struct InfoScatter {
  const prism_info* src;
  prism_info* dst[BF16_MAX_GROUPS];   // null: the group wants no report
  int first[BF16_MAX_GROUPS + 1];     // group g owns matrices [first[g], first[g + 1])
  int ngroups;
};
void launch_scatter_info(const InfoScatter& a, hipStream_t s);

// Second pass of a split-K Gram product: R = I - sum_p part_p (zero outside the leading n x n block),
// summed in part order, exactly symmetric (the lower triangle is the mirror image of the upper one).
struct GramReduceArgs {
  const float* part;        // [batch][parts][np][np]
  int parts, np, n_true;
  float* R32;               // [batch][np][np] or null
  uint16_t* Rb;             // bf16 copy [batch][np][np] or null
  float* diag;              // exact diagonal [batch][np] or null
  float* rho_part;          // [batch][tiles]: tiles = (np / 64) (np / 64 + 1) / 2 partial sums of R^2
  const Ctrl* ctrl;
};
int gram_reduce_parts(int np);
void launch_gram_reduce(const GramReduceArgs& a, int batch, hipStream_t s);
// E = alpha R, one matrix per blockIdx.y; skipped when done
void launch_make_e(float* E, const float* R, const Ctrl* ctrl, int batch, int np, hipStream_t s);

// ---- dbnewton.hip : pieces of the DB Newton iteration (App. A.2) ----
// N = M (copy), then the in-place inverse of the SPD matrices N[batch][np][np] by block Gauss-Jordan.
// panels: scratch of spd_inverse_scratch_floats(np, batch) floats (may be null when that is 0).
long long spd_inverse_scratch_floats(int np, int batch);
int launch_spd_inverse(const float* M, float* N, int np, int batch, const Ctrl* ctrl, float* panels, hipStream_t s);
// partial sums of <D0,D0>, <D0,D2>, <D2,D2> (D0 = M - I, D2 = M + N - 2I) -> the five coefficient partials
void launch_db_moments(const float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, double* cpart,
                       int ngroups, hipStream_t s);
// M <- 2a(1-a) I + (1-a)^2 M + a^2 N (a = ctrl.alpha) on the true n x n part, partial sums of ||I - M'||_F^2
// after launch_db_moments (same ngroups): ||M N v - v||^2 partials into slot 16 of cpart; w: [batch][np] scratch
void launch_db_probe(const float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, float* w, double* cpart,
                     int ngroups, hipStream_t s);
void launch_db_update_m(float* M, const float* N, int np, int n_true, int batch, const Ctrl* ctrl, float* rho_part,
                        int nparts, hipStream_t s);

// A/B switches for development builds: an environment variable selects an alternative kernel
// choice (never a different result contract).  Compiled out, always 0, unless the library is built
// with -DPRISM_AB_SWITCHES; the shipped build does not define it.
#ifdef PRISM_AB_SWITCHES
int ab_switch(const char* name);
#else
inline int ab_switch(const char*) { return 0; }
#endif

void set_last_error(const char* msg);
// Raises the dynamic LDS limit of a kernel to `bytes`, once per (device, kernel); the attribute
// belongs to the device that is current when it is set.  PRISM_OK or PRISM_EHIP.
int allow_dynamic_lds(const void* kernel, int bytes);

// ---- per-kernel timing with HIP events (off unless prism_profile_enable(1)) ----
enum ProfKind {
  PK_PREP = 0, PK_FINAL, PK_SKETCH, PK_CHAIN, PK_SOLVE,
  PK_F32_RESID, PK_F32_POLYQ, PK_F32_APPLY, PK_F32_STORE, PK_F64_MNEXT, PK_MAKE_T,
  PK_BF16_GRAM, PK_BF16_POLYQ, PK_BF16_APPLY, PK_BF16_STORE,
  PK_SPD_INVERSE, PK_DB_MOMENTS, PK_DB_UPDATE_M, PK_F32_SMALL_POLAR, PK_MOMENTS,
  PK_COUNT
};
struct ProfScope {   // records an event pair around the launches made during its lifetime
  ProfScope(int kind, hipStream_t s);
  ~ProfScope();
  int slot; hipStream_t stream;
};

}  // namespace prism
