// Host side of libprism: argument checks, workspace layout and the launch sequences of the
// PRISM iterations (paper Table 1; Section 4; App. A.1, A.3, A.4).  Every call only enqueues kernels on
// the caller's stream: the whole budget of iterations is enqueued up front and each kernel
// skips matrices whose `done` flag the on-device solve step has set, so there is no host
// round trip per iteration.
#include <cstdint>
#include <cstdlib>
#include <map>
#include <mutex>
#include <string>
#include <vector>
#include <utility>

#include "common.h"

namespace prism {

static thread_local std::string g_last_error;
void set_last_error(const char* msg) { g_last_error = msg ? msg : ""; }

#ifdef PRISM_AB_SWITCHES
int ab_switch(const char* name) {
  const char* v = getenv(name);
  return v ? atoi(v) : 0;
}
#endif

int allow_dynamic_lds(const void* kernel, int bytes) {
  static std::mutex mu;
  static std::map<std::pair<int, const void*>, int> granted;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { set_last_error("hipGetDevice failed"); return PRISM_EHIP; }
  std::lock_guard<std::mutex> lock(mu);
  int& have = granted[std::make_pair(dev, kernel)];
  if (have >= bytes) return PRISM_OK;
  if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess) {
    (void)hipGetLastError();
    set_last_error("hipFuncSetAttribute(MaxDynamicSharedMemorySize) failed");
    return PRISM_EHIP;
  }
  have = bytes;
  return PRISM_OK;
}

// ---------------------------------------------------------------- event profiling
static_assert(PK_COUNT == PRISM_PROFILE_KINDS, "prism.h must size the profile arrays for every kernel kind");
namespace {
struct ProfRec { int kind; hipEvent_t a, b; };
bool g_prof_on = false;
thread_local bool t_prof_off = false;   // set while an entry point that must not create HIP objects runs on this thread
std::vector<ProfRec> g_prof;
std::mutex g_prof_mu;   // calls from several host threads may record while profiling is on
}  // namespace

ProfScope::ProfScope(int kind, hipStream_t s) : slot(-1), stream(s) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (!g_prof_on || t_prof_off) return;
  ProfRec r;
  r.kind = kind;
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, s);
  g_prof.push_back(r);
  slot = (int)g_prof.size() - 1;
}
ProfScope::~ProfScope() {
  if (slot < 0) return;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  if (slot < (int)g_prof.size()) (void)hipEventRecord(g_prof[slot].b, stream);
}

namespace {

inline int round_up(int x, int m) { return (x + m - 1) / m * m; }
inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Plan {
  int fn, dt, batch, m, n;
  int S, L, Sp, Lp, transpose;
  int d, p, p_s, ld, nv;
  int tile;        // GEMM tile of the main products
  bool split;      // bf16: iterate carried as high + low part
  int nsum;        // partial sums of the Frobenius norm per matrix
  int max_parts;   // residual partials per matrix
  // byte offsets into the workspace
  size_t o_ctrl, o_info, o_sumsq, o_rho, o_v0, o_v, o_cpart;
  size_t o_vp0, o_vp;                             // bf16 polar: bf16 planes of the sketches and of V_1 .. V_{nv-1}
  bool has_planes;
  int ngroups;     // workgroups per matrix of the moments kernel
  bool shared_gpu; // PRISM_FLAG_SHARED_GPU
  size_t o_x[2], o_y[2], o_r, o_q, o_t[3];        // fp32 paths (o_y doubles as M64 for inverse root)
  size_t o_xhi[2], o_xlo[2], o_rb, o_qb;          // bf16 polar
  int ksplit;      // polar: parts of the K loop of X^T X (0 = one pass); partial products at o_gpart
  size_t o_gpart;
  size_t total;
};

// shared_shapes: the plan of a launch sequence over several shape groups with the same short side;
// the iterate buffers are then laid out per group by the caller (offsets o_x* stay 0)
int make_plan(Plan& P, int fn, int batch, int m, int n, int dt, int degree, int sketch_dim, int root_p,
              unsigned flags, bool shared_shapes = false) {
  if (batch <= 0 || m <= 0 || n <= 0) return PRISM_EINVAL;
  if (degree != 3 && degree != 5) return PRISM_EINVAL;
  if (sketch_dim < 0 || sketch_dim > PRISM_MAX_SKETCH) return PRISM_EINVAL;
  if (dt != PRISM_F32 && dt != PRISM_BF16) return PRISM_EINVAL;
  if (fn < PRISM_FN_POLAR || fn > PRISM_FN_SQRT_NEWTON) return PRISM_EINVAL;
  if (fn != PRISM_FN_POLAR && m != n) return PRISM_EINVAL;
  if (fn == PRISM_FN_INV_ROOT && (root_p < 1 || root_p > PRISM_MAX_ROOT || degree != 3)) return PRISM_EINVAL;
  if (fn != PRISM_FN_POLAR && dt == PRISM_BF16) return PRISM_EUNSUPPORTED;
  if ((long long)m * n > (1ll << 31) - 1) { set_last_error("a matrix may hold at most 2^31 - 1 entries"); return PRISM_EUNSUPPORTED; }
  if (batch > PRISM_MAX_BATCH) { set_last_error("more than PRISM_MAX_BATCH matrices in one group"); return PRISM_EUNSUPPORTED; }
  P = Plan();
  P.fn = fn; P.dt = dt; P.batch = batch; P.m = m; P.n = n;
  P.transpose = (fn == PRISM_FN_POLAR && m < n) ? 1 : 0;
  P.S = m < n ? m : n;
  P.L = m < n ? n : m;
  P.d = degree == 3 ? 1 : 2;
  P.p = fn == PRISM_FN_INV_ROOT ? root_p : 0;
  P.p_s = sketch_dim;
  P.ld = sketch_dim <= 16 ? 16 : (sketch_dim <= 32 ? 32 : 64);
  P.nv = fn == PRISM_FN_INV_ROOT ? root_p + 1 : (fn == PRISM_FN_INVERSE ? 3 : 2 * P.d + 1);
  P.split = (dt == PRISM_BF16) && !(flags & PRISM_FLAG_BF16_PLAIN_ITERATE);
  P.shared_gpu = (flags & PRISM_FLAG_SHARED_GPU) != 0;
  if (dt == PRISM_BF16) {
    P.tile = P.S >= 512 ? 256 : 128;   // padding granularity; the tile is chosen per launch
  } else {
    P.tile = P.S <= 256 ? 64 : 128;
  }
  P.Sp = round_up(P.S, P.tile);
  P.Lp = round_up(P.L, P.tile);
  if ((long long)P.Sp * P.Lp > (1ll << 31) - 1) {   // the kernels keep some offsets within a matrix in 32 bits
    set_last_error("a matrix may hold at most 2^31 - 1 entries after its sides are rounded up to tile multiples");
    return PRISM_EUNSUPPORTED;
  }
  P.nsum = 64;
  const int t0 = (P.Sp / 64) * (P.Lp / 64);   // prepare-step tiles (inverse root residual of M_0)
  P.max_parts = t0;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
  const size_t SS = (size_t)P.Sp * P.Sp, LS = (size_t)P.Lp * P.Sp, B = (size_t)batch;
  P.o_ctrl = take(B * sizeof(Ctrl));
  P.o_info = take(B * sizeof(prism_info));
  P.o_sumsq = take(B * P.nsum * sizeof(double));
  P.o_rho = take(B * P.max_parts * sizeof(float));
  P.o_v0 = take((size_t)PRISM_MAX_ITERS * P.Sp * P.ld * sizeof(float));   // S_k^T for every k, generated once per call
  P.o_v = take((size_t)P.nv * B * P.Sp * P.ld * sizeof(float));
  {
    const long long el = (long long)P.Sp * P.ld;
    P.ngroups = el <= 4096 ? 1 : (int)(el / 4096 > 64 ? 64 : el / 4096);   // 1: done inside the solve kernel
    if (fn == PRISM_FN_SQRT_NEWTON) {   // the moments run over the n x n matrices themselves
      const long long mm = (long long)P.Sp * P.Sp / 65536;
      P.ngroups = mm < 1 ? 1 : (mm > 64 ? 64 : (int)mm);
    }
  }
  P.o_cpart = take(B * P.ngroups * 17 * sizeof(double));
  if (dt == PRISM_BF16 && P.ld <= 32 && P.p_s > 0) {   // operands of the plane chain kernel: 3 x 2 bytes per entry
    P.o_vp0 = take((size_t)PRISM_MAX_ITERS * P.Sp * P.ld * 6);
    P.o_vp = take((size_t)(P.nv - 1) * B * P.Sp * P.ld * 6);
    P.has_planes = true;
  }
  if (dt == PRISM_BF16) {
    for (int i = 0; i < 2 && !shared_shapes; ++i) {
      P.o_xhi[i] = take(B * LS * 2);
      P.o_xlo[i] = P.split ? take(B * LS * 2) : 0;
    }
    P.o_r = take(B * SS * 4);
    P.o_rb = take(B * SS * 2);
    P.o_qb = P.d == 2 ? take(B * SS * 2) : 0;
  } else if (fn == PRISM_FN_POLAR || fn == PRISM_FN_SIGN) {
    for (int i = 0; i < 2; ++i) P.o_x[i] = take(B * LS * 4);
    P.o_r = take(B * SS * 4);
    P.o_q = P.d == 2 ? take(B * SS * 4) : 0;
  } else if (fn == PRISM_FN_SQRT_NEWTON) {
    for (int i = 0; i < 2; ++i) { P.o_x[i] = take(B * SS * 4); P.o_y[i] = take(B * SS * 4); }
    P.o_r = take(B * SS * 4);        // M_k
    P.o_q = take(B * SS * 4);        // N_k = M_k^{-1}
    P.o_t[0] = take((size_t)spd_inverse_scratch_floats(P.Sp, batch) * 4 + 256);   // pivot panels of the inverse
  } else if (fn == PRISM_FN_INVERSE) {
    for (int i = 0; i < 2; ++i) P.o_x[i] = take(B * SS * 4);
    P.o_y[0] = take(B * SS * 4);     // A / ||A||_F
    P.o_r = take(B * SS * 4);
    P.o_q = take(B * SS * 4);
  } else if (fn == PRISM_FN_SQRT) {
    for (int i = 0; i < 2; ++i) { P.o_x[i] = take(B * SS * 4); P.o_y[i] = take(B * SS * 4); }
    P.o_r = take(B * SS * 4);
    P.o_q = P.d == 2 ? take(B * SS * 4) : 0;
  } else {
    for (int i = 0; i < 2; ++i) { P.o_x[i] = take(B * SS * 4); P.o_y[i] = take(B * SS * 8); }
    P.o_r = take(B * SS * 4);
    for (int i = 0; i < 3; ++i) P.o_t[i] = take(B * SS * 4);
  }
  // Polar factor of a few tall matrices: X^T X has few tiles and a long K loop, which would leave
  // most CUs idle; the loop is then cut into parts that run as separate workgroups and a second
  // pass adds the partial products up (in part order, so results stay run-to-run identical).
  P.ksplit = 0; P.o_gpart = 0;
  static const int no_split_k = ab_switch("PRISM_NO_SPLIT_K");
  if (fn == PRISM_FN_POLAR && !no_split_k && !shared_shapes && batch <= 8 && P.Lp >= 8192 && P.Sp > 64) {
    const int tg = dt == PRISM_BF16 ? 128 : P.tile;
    const long long nt = P.Sp / tg, tri = nt * (nt + 1) / 2, full = nt * nt;
    if (tri * batch <= 48) {
      for (int parts = 32; parts >= 2; --parts)
        if (P.Lp % (parts * 32) == 0 && P.Lp / parts >= 1024 && full * batch * parts <= 4096) { P.ksplit = parts; break; }
    }
    if (P.ksplit) P.o_gpart = take(B * P.ksplit * SS * 4);
  }
  P.total = off;
  return PRISM_OK;
}

// Grow-only workspace per (device, stream).  A block that has become too small is kept until
// prism_release_workspaces(): work enqueued earlier, and HIP graphs captured from earlier calls,
// still hold its address.
struct Cached { void* ptr = nullptr; size_t bytes = 0; std::vector<void*> retired; };
std::mutex g_mu;
std::map<std::pair<int, void*>, Cached> g_cache;

int get_workspace(size_t bytes, hipStream_t stream, const prism_options* opt, char** out) {
  if (opt && opt->workspace) {
    if (opt->workspace_bytes < bytes || ((uintptr_t)opt->workspace & 255)) return PRISM_ENOMEM;
    *out = (char*)opt->workspace;
    return PRISM_OK;
  }
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { set_last_error("hipGetDevice failed"); return PRISM_EHIP; }
  std::lock_guard<std::mutex> lock(g_mu);
  Cached& c = g_cache[std::make_pair(dev, (void*)stream)];
  if (c.bytes < bytes) {
    void* fresh = nullptr;
    if (hipMalloc(&fresh, bytes) != hipSuccess) {
      (void)hipGetLastError();
      set_last_error("hipMalloc of the workspace failed");
      return PRISM_ENOMEM;
    }
    if (c.ptr) c.retired.push_back(c.ptr);
    c.ptr = fresh;
    c.bytes = bytes;
  }
  *out = (char*)c.ptr;
  return PRISM_OK;
}

#define CHECK_LAUNCH(expr)                         \
  do {                                             \
    int rc_ = (expr);                              \
    if (rc_ != PRISM_OK) return rc_;               \
  } while (0)

int check_hip() {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { set_last_error(hipGetErrorString(e)); return PRISM_EHIP; }
  return PRISM_OK;
}

struct Run {
  Plan P;
  char* ws;
  hipStream_t s;
  Ctrl* ctrl;
  prism_info* info;
  float* rho;
  float* v0;
  float* v;
  uint16_t* vp0 = nullptr;             // bf16 planes of the sketches / of V_1 .. (bf16 polar, large launches)
  uint16_t* vp = nullptr;
  int max_iters, warm;
  const float* sched; int sched_len;   // caller's coefficients for the leading updates (host array)
  int first_fit;                       // first update whose coefficient is fitted
  double tol;
  uint64_t seed;
  // bf16 polar: the iterate buffers, per shape group (one group for a single-shape call).  All
  // groups share the short side, so R, Q, the chain vectors and the control blocks of all their
  // matrices form one batch (matrices [boff, boff + batch) belong to the group); only the Gram
  // product and the update see the long side, and take all groups in one launch each.
  // Plain iterate, no padding, tall or square input: the caller's array serves as the odd one of
  // the two iterate buffers (the input is consumed by the prepare step before the first update
  // writes there), so that after an odd number of updates the result is in place.
  struct XGroup {
    int batch, boff, m, n, L, Lp, transpose;
    void* x;                                   // caller's array
    uint16_t* Xhi[2]; uint16_t* Xlo[2];        // iterate [Lp][Sp], double buffered
    bool aliased;                              // buffer 1 is the caller's array
  };
  std::vector<XGroup> xg;
  int chain_sel_batch = 0;                     // batch size that picks the chain kernels (0: the whole batch)

  template <typename T> T* at(size_t off) const { return (T*)(ws + off); }

  // sketch + chain V_j = R V_{j-1} (fp32 matrix cores, skinny N = padded sketch width)
  // Rb: bf16 copy of R (bf16 polar path): the products then read it instead of R, except the diagonal,
  // which comes from D (entry i of matrix b at D[b * strideD + i * ldd])
  int chain(const float* R, int k, const uint16_t* Rb = nullptr, const float* D = nullptr, long long strideD = 0,
            int ldd = 0) {
    const int Sp = P.Sp, ld = P.ld;
    const long long vs = (long long)P.batch * Sp * ld;
    if (Sp == 64 && !Rb) {   // whole chain in one launch
      ProfScope ps(PK_CHAIN, s);
      return launch_chain_tiny(R, (long long)Sp * Sp, Sp, v0 + (long long)(k - first_fit) * Sp * ld, 0, v, vs,
                               (long long)Sp * ld, P.nv, ld, P.batch, ctrl, s);
    }
    for (int j = 1; j <= P.nv; ++j) {
      const float* vin = (j == 1) ? v0 + (long long)(k - first_fit) * Sp * ld : v + (j - 2) * vs;
      const long long sin = (j == 1) ? 0 : (long long)Sp * ld;
      ProfScope ps(PK_CHAIN, s);
      if (Rb && planes()) {
        const long long pe = (long long)Sp * ld * 3;   // plane entries per matrix
        const uint16_t* pin = (j == 1) ? vp0 + (long long)(k - first_fit) * pe : vp + (long long)(j - 2) * P.batch * pe;
        uint16_t* pout = j < P.nv ? vp + (long long)(j - 1) * P.batch * pe : nullptr;
        CHECK_LAUNCH(launch_chain_planes(Rb, (long long)Sp * Sp, Sp, D, strideD, ldd, vin, sin, pin, j == 1 ? 0 : pe,
                                         v + (j - 1) * vs, (long long)Sp * ld, pout, pe, Sp, ld, P.batch, ctrl, s, chain_sel_batch));
      } else if (Rb)
        CHECK_LAUNCH(launch_chain_bf16(Rb, (long long)Sp * Sp, Sp, D, strideD, ldd, vin, sin, v + (j - 1) * vs,
                                       (long long)Sp * ld, Sp, ld, P.batch, ctrl, s, chain_sel_batch));
      else
        CHECK_LAUNCH(launch_chain(R, (long long)Sp * Sp, Sp, vin, sin, v + (j - 1) * vs, (long long)Sp * ld, Sp, ld,
                                  P.batch, ctrl, s, chain_sel_batch));
    }
    return PRISM_OK;
  }

  int solve(int k, int nparts, int phase = 0) {
    SolveArgs a = {};
    a.phase = phase;
    a.fn = P.fn; a.k = k; a.d = P.d; a.p = P.p; a.n = P.S; a.rows = P.Sp; a.ld = P.ld;
    a.V = v; a.vstride = (long long)P.batch * P.Sp * P.ld; a.bstride = (long long)P.Sp * P.ld;
    a.rho_part = rho; a.nparts = nparts;
    a.ctrl = ctrl; a.info = info; a.tol = tol; a.max_iters = max_iters;
    a.mode = k < sched_len ? 3 : (P.p_s == 0 ? 1 : (k < warm ? 2 : 0));
    a.sched_alpha = k < sched_len ? sched[k] : 0.0f;
    a.last = (k == max_iters);
    a.cpart = at<double>(P.o_cpart); a.ngroups = P.ngroups;
    if (a.mode == 0 && !a.last && a.ngroups > 1 && P.fn != PRISM_FN_SQRT_NEWTON) {
      ProfScope ps(PK_MOMENTS, s);
      launch_moments(a, P.batch, s);
    }
    {
      ProfScope ps(PK_SOLVE, s);
      launch_solve(a, P.batch, s);
    }
    return check_hip();
  }
  bool fit_needed(int k) const { return P.p_s > 0 && k >= first_fit && k < max_iters; }
  // bf16 chain products too large for the 16-row kernel read V as bf16 planes
  bool planes() const {
    const int sel = chain_sel_batch ? chain_sel_batch : P.batch;
    return vp0 && chain_bf16_supported(P.Sp, P.ld, sel, P.Sp) && !chain_takes_small_kernel(P.Sp, P.ld, sel, true);
  }
};

GemmDesc f32_desc(const Run& r, const float* A, int lda, long long sa, const float* B, int ldb, long long sb,
                  int M, int N, int K, int a_km) {
  GemmDesc g = {};
  g.A = A; g.strideA = sa; g.lda = lda; g.B = B; g.strideB = sb; g.ldb = ldb;
  g.M = M; g.N = N; g.K = K; g.a_km = a_km; g.batch = r.P.batch; g.n_true = r.P.S; g.ctrl = r.ctrl;
  g.c_in = 1.0f;
  return g;
}

// Upper-triangle products with a mirrored lower half.  Taken only where the symmetry does not rest
// on iterates commuting: X^T X, the square of a matrix that was itself stored mirrored, and updates
// whose result never re-enters the residual (X of the inverse root, X and Y of DB Newton).  In the
// coupled square root, the sign and the Chebyshev inverse the iterates commute only up to kappa * eps;
// mirroring there turns that defect into a perturbation the iteration amplifies (divergence from
// kappa ~ 1e3 on), so those keep every tile.
int f32_sym() {
  static const int off = ab_switch("PRISM_F32_NO_SYM");
  return off ? 0 : 1;
}
int sym_parts(int nt, int sym) { return sym ? nt * (nt + 1) / 2 : nt * nt; }

int run_polar_f32(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp, Lp = P.Lp, T = P.tile;
  const long long SS = (long long)Sp * Sp, LS = (long long)Lp * Sp;
  float* X[2] = {r.at<float>(P.o_x[0]), r.at<float>(P.o_x[1])};
  float* R = r.at<float>(P.o_r);
  float* Q = P.d == 2 ? r.at<float>(P.o_q) : nullptr;
  const bool polar = P.fn != PRISM_FN_SIGN;
  const int sym = polar ? f32_sym() : 0;
  const int nparts = sym_parts(Sp / T, sym);
  static const int no_small = ab_switch("PRISM_NO_SMALL_KERNEL");
  if (polar && Sp == 64 && Lp == 64 && P.ngroups == 1 && !no_small) {
    // the whole iteration in one workgroup per matrix, one launch for all iterations: with five
    // launches per iteration a call on such matrices is nothing but launch latency
    SmallPolarArgs sa = {};
    SolveArgs& v = sa.sv;
    v.fn = P.fn; v.d = P.d; v.p = P.p; v.n = P.S; v.rows = Sp; v.ld = P.ld;
    v.V = r.v; v.vstride = (long long)P.batch * Sp * P.ld; v.bstride = (long long)Sp * P.ld;
    v.rho_part = r.rho; v.nparts = 1;
    v.ctrl = r.ctrl; v.info = r.info; v.tol = r.tol; v.max_iters = r.max_iters;
    v.cpart = r.at<double>(P.o_cpart); v.ngroups = 1;
    sa.X[0] = X[0]; sa.X[1] = X[1]; sa.V0 = r.v0; sa.nv = P.nv;
    sa.p_s = P.p_s; sa.first_fit = r.first_fit; sa.warm = r.warm; sa.sched_len = r.sched_len;
    for (int i = 0; i < r.sched_len; ++i) sa.sched[i] = r.sched[i];
    ProfScope ps(PK_F32_SMALL_POLAR, r.s);
    return launch_small_polar(sa, P.batch, r.s);
  }
  int cur = 0;
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    // G = X^T X; matrix sign: G = X X (any square input, all tiles)
    GemmDesc g = f32_desc(r, X[cur], Sp, LS, X[cur], Sp, LS, Sp, Sp, Lp, polar ? 1 : 0);
    g.sym = sym;
    g.epi = EPI_RESIDUAL; g.C = R; g.strideC = SS; g.ldc = Sp; g.rho_part = r.rho;
    if (polar && P.ksplit) {
      ProfScope ps(PK_F32_RESID, r.s);
      const int Kp = Lp / P.ksplit;
      float* gpart = r.at<float>(P.o_gpart);
      for (int b = 0; b < P.batch; ++b) {   // the parts of one matrix are the batch of a plain product
        GemmDesc sp = f32_desc(r, X[cur] + (long long)b * LS, Sp, (long long)Kp * Sp, X[cur] + (long long)b * LS, Sp,
                               (long long)Kp * Sp, Sp, Sp, Kp, 1);
        sp.batch = P.ksplit; sp.epi = EPI_STORE; sp.C = gpart + (long long)b * P.ksplit * SS; sp.strideC = SS; sp.ldc = Sp;
        sp.ctrl = r.ctrl + b; sp.ctrl_fixed = 1;
        CHECK_LAUNCH(launch_gemm_f32(sp, T, T, r.s));
      }
      GramReduceArgs ra = {};
      ra.part = gpart; ra.parts = P.ksplit; ra.np = Sp; ra.n_true = P.S;
      ra.R32 = R; ra.rho_part = r.rho; ra.ctrl = r.ctrl;
      launch_gram_reduce(ra, P.batch, r.s);
      CHECK_LAUNCH(check_hip());
    } else {
      ProfScope ps(PK_F32_RESID, r.s);
      CHECK_LAUNCH(launch_gemm_f32(g, T, T, r.s));
    }
    if (r.fit_needed(k)) CHECK_LAUNCH(r.chain(R, k));
    CHECK_LAUNCH(r.solve(k, (polar && P.ksplit) ? gram_reduce_parts(Sp) : nparts));
    if (k == r.max_iters) break;
    const float* Bop = R;
    if (P.d == 2) {
      GemmDesc q = f32_desc(r, R, Sp, SS, R, Sp, SS, Sp, Sp, Sp, polar ? 1 : 0);  // mirrored R: R^2 = R^T R
      q.sym = sym;
      q.epi = EPI_POLYQ; q.C = Q; q.strideC = SS; q.ldc = Sp; q.Cin = R; q.strideCin = SS; q.ldcin = Sp; q.c1 = 0.5f;
      { ProfScope ps(PK_F32_POLYQ, r.s); CHECK_LAUNCH(launch_gemm_f32(q, T, T, r.s)); }
      Bop = Q;
    }
    GemmDesc a = f32_desc(r, X[cur], Sp, LS, Bop, Sp, SS, Lp, Sp, Sp, 0);      // X + X Q
    a.epi = EPI_AXPY; a.C = X[cur ^ 1]; a.strideC = LS; a.ldc = Sp; a.Cin = X[cur]; a.strideCin = LS; a.ldcin = Sp;
    a.coef_is_alpha = P.d == 1;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(a, T, T, r.s)); }
    cur ^= 1;
  }
  return PRISM_OK;
}

// Tile shape of a bf16 product.  Large tiles move fewer bytes per flop but need enough tiles to give
// every CU work and a K long enough to amortise their epilogue: 128 x 128 (three workgroups per CU)
// below that.  (At K = 768 the bare product is faster with large tiles from 144 tiles on, the update
// GEMM with its three-output epilogue is not.)  Among the large shapes 256 x 128 runs two workgroups
// per CU, which overlap each other's epilogue and barrier waits; 256 x 256 runs one.
struct Tile { int m, n; };
int bf16_tile_forced() {
  static const int forced = ab_switch("PRISM_BF16_TILE");   // 128, 256, or 2561 for 256 x 128
  return forced;
}
Tile bf16_big_tile() {
  static const int big = ab_switch("PRISM_BF16_BIG");       // 2: 256 x 128
  return big == 2 ? Tile{256, 128} : Tile{256, 256};
}
Tile bf16_tile(const Plan& P, int M, int N, int K, bool symmetric) {
  const int forced = bf16_tile_forced();
  if (P.tile != 256) return Tile{128, 128};
  if (forced == 128) return Tile{128, 128};
  if (forced == 256) return Tile{256, 256};
  if (forced == 2561) return Tile{256, 128};
  const long long per_mat = symmetric ? (long long)(M / 256) * (M / 256 + 1) / 2 : (long long)(M / 256) * (N / 256);
  // (32 x 1536^2, five iterations: 3.58 ms with large tiles against 4.18; 64 x 768^2: 1.88 against 1.72)
  return (per_mat * P.batch >= 192 && K >= 1536) ? bf16_big_tile() : Tile{128, 128};
}

int run_polar_bf16(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp;
  const int sym = 1;   // X^T X and the square of the (mirrored, hence exactly symmetric) R: upper triangle of tiles
  const int ng = (int)r.xg.size();
  if (ng < 1 || ng > BF16_MAX_GROUPS) return PRISM_EINVAL;
  // Tile shapes.  One shape per launch: with several groups the Gram product and the update take the
  // large tiles when the launch as a whole has enough of them.
  long long gram256 = 0, upd256 = 0;
  for (const Run::XGroup& x : r.xg) {
    gram256 += (long long)(Sp / 256) * (Sp / 256 + 1) / 2 * x.batch;
    upd256 += (long long)(x.Lp / 256) * (Sp / 256) * x.batch;
  }
  Tile Tg, Ta;
  if (ng == 1) {
    // with other work beside this call, large Gram tiles also when they are few (measured on the
    // Muon-shaped batch of four groups on four streams: 3.96 -> 3.80 ms; alone on the GPU the same
    // choice costs 1.40 instead of 1.07 ms of Gram time per step)
    Tg = bf16_tile(P, Sp, Sp, r.xg[0].Lp, true);
    Ta = bf16_tile(P, r.xg[0].Lp, Sp, Sp, false);
    if (P.tile == 256 && P.shared_gpu && bf16_tile_forced() == 0) Tg = Tile{256, 256};
  } else {
    const bool pad256 = P.tile == 256;
    static const int multi_gram = ab_switch("PRISM_BF16_MULTI_GRAM");   // 1: 128 x 128, 2: 256 x 128, 3: 256 x 256
    static const int multi_upd = ab_switch("PRISM_BF16_MULTI_UPD");
    auto pick = [&](int sw, bool big) {
      if (!pad256 || sw == 1) return Tile{128, 128};
      if (sw == 2) return Tile{256, 128};
      if (sw == 3) return Tile{256, 256};
      return big ? bf16_big_tile() : Tile{128, 128};
    };
    // measured on the Muon-shaped groups (order 768, K from 768 to 3072): 256 x 256 tiles (eight
    // wavefronts) for the Gram products and the updates beat 128 x 128 ones from 96 matrices' worth of
    // tiles on (update: 2.90 against 2.96 ms per step with 256 x 128 tiles)
    Tg = multi_gram ? pick(multi_gram, false) : ((pad256 && gram256 >= 96) ? Tile{256, 256} : Tile{128, 128});
    Ta = multi_upd ? pick(multi_upd, false) : ((pad256 && upd256 >= 96) ? Tile{256, 256} : Tile{128, 128});
  }
  const Tile Tq = (ng == 1) ? Tg : bf16_tile(P, Sp, Sp, Sp, true);
  const long long SS = (long long)Sp * Sp;
  float* R = r.at<float>(P.o_r);
  uint16_t* Rb = r.at<uint16_t>(P.o_rb);
  uint16_t* Qb = P.d == 2 ? r.at<uint16_t>(P.o_qb) : nullptr;
  static const int chain_f32 = ab_switch("PRISM_BF16_CHAIN_F32");
  // The fit can read the bf16 copy of R (plus its exact diagonal) when the chain kernels take the
  // shape; with symmetric tiles the fp32 matrix is then not written at all: the Gram epilogue
  // stores the bf16 copy and the diagonal (at the head of the buffer of R), R^2 reads the copy.
  // Only with the plain bf16 iterate: with the split one the linear term of Q = R/2 + alpha R^2 keeps
  // the fp32 R (taking it from the bf16 copy raises the residual floor by a few 1e-4, which at
  // tol = 1e-2 cost the reduced config-3 case one more iteration than the oracle).
  const int sel = r.chain_sel_batch ? r.chain_sel_batch : P.batch;
  const bool chain_b = !chain_f32 && Sp > 64 && (P.p_s == 0 || chain_bf16_supported(Sp, P.ld, sel, Sp));   // order 64: one-launch fp32 chain
  const bool lean = chain_b && sym && !P.split;
  float* Dg = R;
  const int ntg = Sp / Tg.m;
  const int nparts = (Tg.m / Tg.n) * ntg * (ntg + 1) / 2;   // tiles (= residual partial sums) per matrix
  // launch order of the groups: longest K first, so that the short tiles fill the last round
  int order[BF16_MAX_GROUPS];
  for (int i = 0; i < ng; ++i) order[i] = i;
  for (int i = 1; i < ng; ++i)
    for (int j = i; j > 0 && r.xg[order[j]].Lp > r.xg[order[j - 1]].Lp; --j) { const int t = order[j]; order[j] = order[j - 1]; order[j - 1] = t; }
  int cur = 0;
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    if (P.ksplit) {   // single group of a few tall matrices
      const Run::XGroup& x = r.xg[0];
      const long long LS = (long long)x.Lp * Sp;
      ProfScope ps(PK_BF16_GRAM, r.s);
      const int Kp = x.Lp / P.ksplit;
      const int T1 = (P.tile == 256 && (long long)(Sp / 256) * (Sp / 256) * P.ksplit >= 256) ? 256 : 128;   // square tiles
      float* gpart = r.at<float>(P.o_gpart);
      for (int b = 0; b < P.batch; ++b) {   // the parts of one matrix are the batch of a plain product
        Bf16Desc sp = {};
        // part p = rows [p Kp, (p + 1) Kp) of the [Lp][Sp] iterate, read as [K][M]
        sp.A = x.Xhi[cur] + (long long)b * LS; sp.B = sp.A; sp.strideA = (long long)Kp * Sp; sp.strideB = sp.strideA;
        sp.lda = Sp; sp.ldb = Sp; sp.km = 3;
        sp.M = Sp; sp.N = Sp; sp.K = Kp; sp.batch = P.ksplit; sp.epi = BEPI_STORE;
        sp.C32 = gpart + (long long)b * P.ksplit * SS; sp.strideC32 = SS; sp.ldc32 = Sp;
        sp.ctrl = r.ctrl + b; sp.ctrl_fixed = 1;
        CHECK_LAUNCH(launch_gemm_bf16(sp, T1, T1, r.s));
      }
      GramReduceArgs ra = {};
      ra.part = gpart; ra.parts = P.ksplit; ra.np = Sp; ra.n_true = P.S;
      ra.R32 = lean ? nullptr : R; ra.Rb = Rb; ra.diag = lean ? Dg : nullptr; ra.rho_part = r.rho; ra.ctrl = r.ctrl;
      launch_gram_reduce(ra, P.batch, r.s);
      CHECK_LAUNCH(check_hip());
    } else {
      Bf16Desc gd[BF16_MAX_GROUPS];
      for (int i = 0; i < ng; ++i) {
        const Run::XGroup& x = r.xg[order[i]];
        const long long LS = (long long)x.Lp * Sp;
        Bf16Desc& g = gd[i];
        g = Bf16Desc{};
        g.sym = sym;
        // X^T X straight from the [Lp][Sp] iterate: both operands stored [K][M]
        g.A = x.Xhi[cur]; g.strideA = LS; g.lda = Sp; g.B = x.Xhi[cur]; g.strideB = LS; g.ldb = Sp; g.km = 3;
        g.M = Sp; g.N = Sp; g.K = x.Lp; g.batch = x.batch; g.epi = BEPI_GRAM; g.n_true = P.S;
        g.C32 = lean ? nullptr : R + x.boff * SS; g.strideC32 = SS; g.ldc32 = Sp;
        // with the bf16 chain only the R^2 epilogue and the chain's diagonal read the fp32 matrix: both stay
        // inside the tiles the Gram product computes when its tile rows are whole multiples of those of R^2
        g.upper32 = (chain_b && Tg.m % Tq.m == 0) ? 1 : 0;
        g.Cb = Rb + x.boff * SS; g.strideCb = SS; g.ldcb = Sp;
        g.diag = lean ? Dg + (long long)x.boff * Sp : nullptr; g.strideDiag = Sp;
        g.rho_part = r.rho + (long long)x.boff * nparts; g.ctrl = r.ctrl + x.boff;
      }
      ProfScope ps(PK_BF16_GRAM, r.s);
      CHECK_LAUNCH(launch_gemm_bf16_multi(gd, ng, Tg.m, Tg.n, r.s));
    }
    if (r.fit_needed(k)) {
      if (lean) CHECK_LAUNCH(r.chain(R, k, Rb, Dg, Sp, 1));
      else if (chain_b) CHECK_LAUNCH(r.chain(R, k, Rb, R, SS, Sp + 1));
      else CHECK_LAUNCH(r.chain(R, k));
    }
    CHECK_LAUNCH(r.solve(k, P.ksplit ? gram_reduce_parts(Sp) : nparts));
    if (k == r.max_iters) break;
    const uint16_t* Bop = Rb;
    if (P.d == 2) {   // one launch over the matrices of all groups: R has the same order everywhere
      Bf16Desc q = {};
      q.A = Rb; q.strideA = SS; q.lda = Sp; q.B = Rb; q.strideB = SS; q.ldb = Sp;
      q.km = 3;   // R is symmetric bit for bit: read as [K][M], whose whole-cache-line loads are the faster ones
      q.M = Sp; q.N = Sp; q.K = Sp; q.batch = P.batch; q.epi = BEPI_POLYQ; q.sym = sym;
      q.C32 = lean ? nullptr : R; q.strideC32 = SS; q.ldc32 = Sp; q.Cb = Qb; q.strideCb = SS; q.ldcb = Sp; q.c1 = 0.5f;
      q.Cin16 = lean ? Rb : nullptr;
      q.ctrl = r.ctrl;
      { ProfScope ps(PK_BF16_POLYQ, r.s); CHECK_LAUNCH(launch_gemm_bf16(q, Tq.m, Tq.n, r.s)); }
      Bop = Qb;
    }
    // One pass: the product reads the high half of the iterate only; the epilogue adds the low
    // half's share elementwise (see the kernel) and splits the result again.
    Bf16Desc ad[BF16_MAX_GROUPS];
    for (int i = 0; i < ng; ++i) {
      const Run::XGroup& x = r.xg[order[i]];
      const long long LS = (long long)x.Lp * Sp;
      Bf16Desc& a = ad[i];
      a = Bf16Desc{};
      a.A = x.Xhi[cur]; a.strideA = LS; a.lda = Sp; a.B = Bop + x.boff * SS; a.strideB = SS; a.ldb = Sp;
      a.km = 2;   // Q (d = 1: R) is symmetric: read as [K][N]
      a.M = x.Lp; a.N = Sp; a.K = Sp; a.batch = x.batch; a.epi = BEPI_APPLY;
      a.Cb = x.Xhi[cur ^ 1]; a.Cb2 = x.Xlo[cur ^ 1]; a.strideCb = LS; a.ldcb = Sp;
      a.Xhi = x.Xhi[cur]; a.Xlo = x.Xlo[cur]; a.coef_is_alpha = P.d == 1; a.ctrl = r.ctrl + x.boff;
    }
    { ProfScope ps(PK_BF16_APPLY, r.s); CHECK_LAUNCH(launch_gemm_bf16_multi(ad, ng, Ta.m, Ta.n, r.s)); }
    cur ^= 1;
  }
  return PRISM_OK;
}

int run_sqrt_f32(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp, T = P.tile;
  const long long SS = (long long)Sp * Sp;
  float* X[2] = {r.at<float>(P.o_x[0]), r.at<float>(P.o_x[1])};
  float* Y[2] = {r.at<float>(P.o_y[0]), r.at<float>(P.o_y[1])};
  float* R = r.at<float>(P.o_r);
  float* Q = P.d == 2 ? r.at<float>(P.o_q) : nullptr;
  // X_k and Y_k commute up to kappa * eps only: every product keeps all its tiles.  (Mirroring only
  // Y X and R^2 is stable but costs the root an order of magnitude of accuracy from kappa ~ 1e4 on.)
  const int sym = 0;
  const int nparts = sym_parts(Sp / T, sym);
  int cur = 0;
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    GemmDesc g = f32_desc(r, Y[cur], Sp, SS, X[cur], Sp, SS, Sp, Sp, Sp, 0);    // G = Y X
    g.sym = sym;
    g.epi = EPI_RESIDUAL; g.C = R; g.strideC = SS; g.ldc = Sp; g.rho_part = r.rho;
    { ProfScope ps(PK_F32_RESID, r.s); CHECK_LAUNCH(launch_gemm_f32(g, T, T, r.s)); }
    if (r.fit_needed(k)) CHECK_LAUNCH(r.chain(R, k));
    CHECK_LAUNCH(r.solve(k, nparts));
    if (k == r.max_iters) break;
    const float* Pm = R;
    if (P.d == 2) {
      GemmDesc q = f32_desc(r, R, Sp, SS, R, Sp, SS, Sp, Sp, Sp, 0);
      q.sym = sym;
      q.epi = EPI_POLYQ; q.C = Q; q.strideC = SS; q.ldc = Sp; q.Cin = R; q.strideCin = SS; q.ldcin = Sp; q.c1 = 0.5f;
      { ProfScope ps(PK_F32_POLYQ, r.s); CHECK_LAUNCH(launch_gemm_f32(q, T, T, r.s)); }
      Pm = Q;
    }
    GemmDesc ax = f32_desc(r, X[cur], Sp, SS, Pm, Sp, SS, Sp, Sp, Sp, 0);        // X + X Q
    ax.epi = EPI_AXPY; ax.C = X[cur ^ 1]; ax.strideC = SS; ax.ldc = Sp; ax.Cin = X[cur]; ax.strideCin = SS; ax.ldcin = Sp;
    ax.coef_is_alpha = P.d == 1;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ax, T, T, r.s)); }
    GemmDesc ay = f32_desc(r, Pm, Sp, SS, Y[cur], Sp, SS, Sp, Sp, Sp, 0);        // Y + Q Y
    ay.epi = EPI_AXPY; ay.C = Y[cur ^ 1]; ay.strideC = SS; ay.ldc = Sp; ay.Cin = Y[cur]; ay.strideCin = SS; ay.ldcin = Sp;
    ay.coef_is_alpha = P.d == 1;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ay, T, T, r.s)); }
    cur ^= 1;
  }
  return PRISM_OK;
}

// Chebyshev inverse (App. A.4): R = I - A_s X, Q = R + alpha R^2, X <- X + X Q
int run_inverse_f32(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp, T = P.tile;
  const long long SS = (long long)Sp * Sp;
  float* X[2] = {r.at<float>(P.o_x[0]), r.at<float>(P.o_x[1])};
  const float* As = r.at<float>(P.o_y[0]);
  float* R = r.at<float>(P.o_r);
  float* Q = r.at<float>(P.o_q);
  const int sym = 0;   // A_s X_k is symmetric up to kappa * eps only: all tiles
  const int nparts = sym_parts(Sp / T, sym);
  int cur = 0;
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    GemmDesc g = f32_desc(r, As, Sp, SS, X[cur], Sp, SS, Sp, Sp, Sp, 0);
    g.sym = sym;
    g.epi = EPI_RESIDUAL; g.C = R; g.strideC = SS; g.ldc = Sp; g.rho_part = r.rho;
    { ProfScope ps(PK_F32_RESID, r.s); CHECK_LAUNCH(launch_gemm_f32(g, T, T, r.s)); }
    if (r.fit_needed(k)) CHECK_LAUNCH(r.chain(R, k));
    CHECK_LAUNCH(r.solve(k, nparts));
    if (k == r.max_iters) break;
    GemmDesc q = f32_desc(r, R, Sp, SS, R, Sp, SS, Sp, Sp, Sp, 0);
    q.sym = sym;
    q.epi = EPI_POLYQ; q.C = Q; q.strideC = SS; q.ldc = Sp; q.Cin = R; q.strideCin = SS; q.ldcin = Sp; q.c1 = 1.0f;
    { ProfScope ps(PK_F32_POLYQ, r.s); CHECK_LAUNCH(launch_gemm_f32(q, T, T, r.s)); }
    GemmDesc ax = f32_desc(r, X[cur], Sp, SS, Q, Sp, SS, Sp, Sp, Sp, 0);
    ax.epi = EPI_AXPY; ax.C = X[cur ^ 1]; ax.strideC = SS; ax.ldc = Sp; ax.Cin = X[cur]; ax.strideCin = SS; ax.ldcin = Sp;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ax, T, T, r.s)); }
    cur ^= 1;
  }
  return PRISM_OK;
}

// DB Newton in product form (App. A.2): N = M^{-1}, X <- (1-a) X + a X N, Y likewise,
// M <- 2a(1-a) I + (1-a)^2 M + a^2 N.  The stop test of iteration k runs before the inverse.
int run_sqrt_newton_f32(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp, T = P.tile;
  const long long SS = (long long)Sp * Sp;
  float* X[2] = {r.at<float>(P.o_x[0]), r.at<float>(P.o_x[1])};
  float* Y[2] = {r.at<float>(P.o_y[0]), r.at<float>(P.o_y[1])};
  float* M = r.at<float>(P.o_r);
  float* N = r.at<float>(P.o_q);
  const int nparts0 = (Sp / 64) * (Sp / 64);               // prepare step: one partial per 64 x 64 tile
  const int nparts = nparts0 < 512 ? nparts0 : 512;        // later: the M update
  const int sym = f32_sym();                               // X, Y never re-enter M: mirrored halves are safe
  int cur = 0;
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    CHECK_LAUNCH(r.solve(k, k == 0 ? nparts0 : nparts, 1));
    if (k == r.max_iters) break;
    { ProfScope ps(PK_SPD_INVERSE, r.s); CHECK_LAUNCH(launch_spd_inverse(M, N, Sp, P.batch, r.ctrl, r.at<float>(P.o_t[0]), r.s)); }
    {   // also without a fit: the probe of the inverse shares the partials with the moments
      ProfScope ps(PK_DB_MOMENTS, r.s);
      launch_db_moments(M, N, Sp, P.S, P.batch, r.ctrl, r.at<double>(P.o_cpart), P.ngroups, r.s);
      launch_db_probe(M, N, Sp, P.S, P.batch, r.ctrl, r.v, r.at<double>(P.o_cpart), P.ngroups, r.s);
    }
    CHECK_LAUNCH(r.solve(k, 0, 2));
    GemmDesc ax = f32_desc(r, X[cur], Sp, SS, N, Sp, SS, Sp, Sp, Sp, 0);
    ax.epi = EPI_AXPY; ax.C = X[cur ^ 1]; ax.strideC = SS; ax.ldc = Sp; ax.Cin = X[cur]; ax.strideCin = SS; ax.ldcin = Sp;
    ax.cin_one_minus_alpha = 1; ax.coef_is_alpha = 1; ax.sym = sym;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ax, T, T, r.s)); }
    GemmDesc ay = f32_desc(r, Y[cur], Sp, SS, N, Sp, SS, Sp, Sp, Sp, 0);
    ay.epi = EPI_AXPY; ay.C = Y[cur ^ 1]; ay.strideC = SS; ay.ldc = Sp; ay.Cin = Y[cur]; ay.strideCin = SS; ay.ldcin = Sp;
    ay.cin_one_minus_alpha = 1; ay.coef_is_alpha = 1; ay.sym = sym;
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ay, T, T, r.s)); }
    { ProfScope ps(PK_DB_UPDATE_M, r.s); launch_db_update_m(M, N, Sp, P.S, P.batch, r.ctrl, r.rho, nparts, r.s); }
    CHECK_LAUNCH(check_hip());
    cur ^= 1;
  }
  return PRISM_OK;
}

int run_inv_root_f32(Run& r) {
  const Plan& P = r.P;
  const int Sp = P.Sp, T = P.tile, p = P.p;
  const long long SS = (long long)Sp * Sp;
  float* X[2] = {r.at<float>(P.o_x[0]), r.at<float>(P.o_x[1])};
  double* M[2] = {r.at<double>(P.o_y[0]), r.at<double>(P.o_y[1])};
  float* R = r.at<float>(P.o_r);
  float* Tm[3] = {r.at<float>(P.o_t[0]), r.at<float>(P.o_t[1]), r.at<float>(P.o_t[2])};
  const int nparts0 = (Sp / 64) * (Sp / 64);  // residual of M_0 comes from the prepare step (64 x 64 tiles)
  const int nparts = (Sp / 64) * (Sp / 64);   // later ones from the fp64 product (64 x 64 tiles)
  int cur = 0, mc = 0;   // current X and M buffers
  for (int k = 0; k <= r.max_iters; ++k) {
    if (k == r.max_iters && r.tol <= 0.0) break;
    if (r.fit_needed(k)) CHECK_LAUNCH(r.chain(R, k));
    CHECK_LAUNCH(r.solve(k, k == 0 ? nparts0 : nparts));
    if (k == r.max_iters) break;
    GemmDesc ax = f32_desc(r, X[cur], Sp, SS, R, Sp, SS, Sp, Sp, Sp, 0);         // X (I + alpha R)
    ax.epi = EPI_AXPY; ax.C = X[cur ^ 1]; ax.strideC = SS; ax.ldc = Sp; ax.Cin = X[cur]; ax.strideCin = SS; ax.ldcin = Sp;
    ax.coef_is_alpha = 1; ax.sym = f32_sym();   // X never re-enters M; the power chain below keeps all tiles
    { ProfScope ps(PK_F32_APPLY, r.s); CHECK_LAUNCH(launch_gemm_f32(ax, T, T, r.s)); }
    // (I + alpha R)^q = I + E_q, built on the part beyond the identity so that fp32 rounding acts
    // on the small quantity only: E_1 = alpha R, squaring E <- 2E + E E, times T: E <- E + E_1 + E E_1.
    // E_1 itself is never stored: wherever it is an operand R stands in and the epilogue supplies
    // the powers of alpha.
    auto square = [&](const float* E /* null: E_1 */, float* dst) -> int {
      const float* Eop = E ? E : R;
      GemmDesc sq = f32_desc(r, Eop, Sp, SS, Eop, Sp, SS, Sp, Sp, Sp, 0);
      sq.epi = EPI_AXPY; sq.C = dst; sq.strideC = SS; sq.ldc = Sp; sq.Cin = Eop; sq.strideCin = SS; sq.ldcin = Sp; sq.c_in = 2.0f;
      if (!E) { sq.cin_alpha_pow = 1; sq.coef_is_alpha = 2; }
      ProfScope ps(PK_F32_STORE, r.s);
      return launch_gemm_f32(sq, T, T, r.s);
    };
    auto times_t = [&](const float* U, float* dst) -> int {                      // U + alpha R + alpha U R
      GemmDesc mu = f32_desc(r, U, Sp, SS, R, Sp, SS, Sp, Sp, Sp, 0);
      mu.epi = EPI_AXPY; mu.C = dst; mu.strideC = SS; mu.ldc = Sp; mu.Cin = U; mu.strideCin = SS; mu.ldcin = Sp; mu.c_in = 1.0f;
      mu.Cin2 = R; mu.cin2_alpha_pow = 1; mu.coef_is_alpha = 1;
      ProfScope ps(PK_F32_STORE, r.s);
      return launch_gemm_f32(mu, T, T, r.s);
    };
    auto m_times = [&](const float* E, const double* Min, double* Mout, float* Rout) -> int {   // Mout = Min + E Min in fp64
      GemmDesc mn = {};
      mn.A = E; mn.strideA = SS; mn.lda = Sp; mn.B = Min; mn.strideB = SS; mn.ldb = Sp;
      mn.M = Sp; mn.N = Sp; mn.K = Sp; mn.batch = P.batch; mn.n_true = P.S; mn.ctrl = r.ctrl;
      mn.epi = EPI_MNEXT; mn.C = Mout; mn.strideC = SS; mn.ldc = Sp;
      mn.Cin = Min; mn.strideCin = SS; mn.ldcin = Sp;
      mn.R32out = Rout; mn.strideR = SS; mn.ldr = Sp; mn.rho_part = r.rho;
      ProfScope ps(PK_F64_MNEXT, r.s);
      return launch_gemm_f64a(mn, 64, 64, r.s);
    };
    if (p <= 4) {
      const float* U = nullptr;   // null: E = E_1 = alpha R
      int hb = 0;
      while ((p >> (hb + 1)) != 0) ++hb;
      for (int bit = hb - 1; bit >= 0; --bit) {
        float* dst = (U == Tm[1]) ? Tm[2] : Tm[1];
        CHECK_LAUNCH(square(U, dst));
        U = dst;
        if ((p >> bit) & 1) {
          float* dst2 = (U == Tm[1]) ? Tm[2] : Tm[1];
          CHECK_LAUNCH(times_t(U, dst2));
          U = dst2;
        }
      }
      if (!U) {   // p = 1: E_p = alpha R.  The product below overwrites R, so it cannot read R as an operand
        { ProfScope ps(PK_MAKE_T, r.s); launch_make_e(Tm[0], R, r.ctrl, P.batch, Sp, r.s); }
        CHECK_LAUNCH(check_hip());
        U = Tm[0];
      }
      CHECK_LAUNCH(m_times(U, M[mc], M[mc ^ 1], R));                               // M' = M + E_p M in fp64
      mc ^= 1;
    } else {
      // p = 5 .. 8: (I + alpha R)^p as p / 2 factors (I + E_2), and (I + E_1) for odd p, applied to M
      // one after the other in fp64.  Every squaring in fp32 doubles the rounding error of its operand
      // times (1 + E), and M must stay consistent with X^p A: with one fp32 chain up to E_8 the root of
      // a 1024 x 1024 matrix came out with a relative error of 2e-5, with two factors (I + E_4) 1.6e-5,
      // with factors of order <= 2 6e-6 (p = 8; 4e-6, 2e-6, 1e-6 for p = 7, 6, 5).
      float* E2 = Tm[1];
      CHECK_LAUNCH(square(nullptr, E2));
      int left = p / 2 + (p & 1);
      if (p & 1) {
        { ProfScope ps(PK_MAKE_T, r.s); launch_make_e(Tm[0], R, r.ctrl, P.batch, Sp, r.s); }
        CHECK_LAUNCH(check_hip());
        --left;
        CHECK_LAUNCH(m_times(Tm[0], M[mc], M[mc ^ 1], Tm[2]));   // the residual of an intermediate product goes to a spare array
        mc ^= 1;
      }
      for (; left > 0; --left) {
        CHECK_LAUNCH(m_times(E2, M[mc], M[mc ^ 1], left == 1 ? R : Tm[2]));
        mc ^= 1;
      }
    }
    cur ^= 1;
  }
  return PRISM_OK;
}

// bf16 polar, plain iterate, shapes that need no padding, array aligned like the workspace buffers:
// the caller's array takes the place of buffer 1 of its own orientation
void alias_output(const Plan& P, Run::XGroup& x) {
  static const int no_alias = ab_switch("PRISM_BF16_NO_OUTPUT_ALIAS");
  const int S = x.m < x.n ? x.m : x.n;
  x.aliased = false;
  if (P.split || x.transpose || P.Sp != S || x.Lp != x.L || no_alias || ((uintptr_t)x.x & 255)) return;
  x.Xhi[1] = (uint16_t*)x.x;
  x.aliased = true;
}
// iterate buffers of one shape group in the arguments of the pre-scaling and copy-out kernels
void bf16_prep_final(const Plan& P, const Run::XGroup& x, PrepArgs& pa, FinalArgs& fa) {
  pa.Xa_hi = x.Xhi[0]; pa.Xa_lo = x.Xlo[0];
  for (int i = 0; i < 2; ++i) { fa.Xa_hi[i] = x.Xhi[i]; fa.Xa_lo[i] = x.Xlo[i]; }
  (void)P;
}

int run(int fn, void* a, void* inv_out, int root_p, int batch, int m, int n, int dt, int degree, int max_iters,
        int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt) {
  set_last_error("");
  const bool empty = batch == 0 || m == 0 || n == 0;   // nothing to compute; the arguments are still checked
  if (batch < 0 || m < 0 || n < 0) return PRISM_EINVAL;
  if (!empty && !a) return PRISM_EINVAL;
  if (!empty && (fn == PRISM_FN_SQRT || fn == PRISM_FN_SQRT_NEWTON) && !inv_out) return PRISM_EINVAL;
  if (max_iters < 0 || max_iters > PRISM_MAX_ITERS) return PRISM_EINVAL;
  if (!(tol == tol)) return PRISM_EINVAL;
  if (opt && opt->warm_iters < 0) return PRISM_EINVAL;
  if (opt && (opt->schedule_len < 0 || opt->schedule_len > PRISM_MAX_ITERS || (opt->schedule_len > 0 && !opt->alpha_schedule)))
    return PRISM_EINVAL;
  Run r;
  if (empty) return make_plan(r.P, fn, 1, m ? m : 1, n ? n : 1, dt, degree, sketch_dim, root_p, opt ? opt->flags : 0u);
  int rc = make_plan(r.P, fn, batch, m, n, dt, degree, sketch_dim, root_p, opt ? opt->flags : 0u);
  if (rc != PRISM_OK) return rc;
  r.s = (hipStream_t)stream;
  rc = get_workspace(r.P.total, r.s, opt, &r.ws);
  if (rc != PRISM_OK) return rc;
  const Plan& P = r.P;
  r.ctrl = r.at<Ctrl>(P.o_ctrl);
  r.info = (opt && opt->info) ? opt->info : r.at<prism_info>(P.o_info);
  r.rho = r.at<float>(P.o_rho);
  r.v0 = r.at<float>(P.o_v0);
  r.v = r.at<float>(P.o_v);
  if (P.has_planes) { r.vp0 = r.at<uint16_t>(P.o_vp0); r.vp = r.at<uint16_t>(P.o_vp); }
  r.max_iters = max_iters; r.tol = tol; r.seed = seed; r.warm = opt ? opt->warm_iters : 0;
  r.sched = opt ? opt->alpha_schedule : nullptr;
  r.sched_len = opt ? opt->schedule_len : 0;
  if (fn == PRISM_FN_SQRT_NEWTON) r.warm = 0;   // no upper end to start from: the coefficient is not clamped to a fit interval
  r.first_fit = r.warm > r.sched_len ? r.warm : r.sched_len;

  PrepArgs pa = {};
  pa.fn = fn; pa.dt = dt; pa.batch = batch; pa.m = m; pa.n = n; pa.S = P.S; pa.L = P.L; pa.Sp = P.Sp; pa.Lp = P.Lp;
  pa.transpose = P.transpose; pa.root_p = root_p; pa.src = a;
  pa.sumsq_part = r.at<double>(P.o_sumsq); pa.nsum = P.nsum; pa.ctrl = r.ctrl; pa.info = r.info;
  pa.rho_part = r.rho; pa.tile = P.tile;
  FinalArgs fa = {};
  fa.fn = fn; fa.dt = dt; fa.batch = batch; fa.m = m; fa.n = n; fa.S = P.S; fa.L = P.L; fa.Sp = P.Sp; fa.Lp = P.Lp;
  fa.transpose = P.transpose; fa.dst = a; fa.dst2 = inv_out; fa.ctrl = r.ctrl;
  if (dt == PRISM_BF16) {
    Run::XGroup x = {};
    x.batch = batch; x.boff = 0; x.m = m; x.n = n; x.L = P.L; x.Lp = P.Lp; x.transpose = P.transpose; x.x = a;
    for (int i = 0; i < 2; ++i) {
      x.Xhi[i] = r.at<uint16_t>(P.o_xhi[i]);
      x.Xlo[i] = P.split ? r.at<uint16_t>(P.o_xlo[i]) : nullptr;
    }
    alias_output(P, x);
    r.xg.push_back(x);
    bf16_prep_final(P, x, pa, fa);
  } else {
    pa.X32 = r.at<float>(P.o_x[0]);
    if (fn == PRISM_FN_SQRT || fn == PRISM_FN_INVERSE || fn == PRISM_FN_SQRT_NEWTON) pa.Y32 = r.at<float>(P.o_y[0]);
    if (fn == PRISM_FN_SQRT_NEWTON) pa.R32 = r.at<float>(P.o_r);
    if (fn == PRISM_FN_INV_ROOT) { pa.M64 = r.at<double>(P.o_y[0]); pa.R32 = r.at<float>(P.o_r); }
    for (int i = 0; i < 2; ++i) {
      fa.X32[i] = r.at<float>(P.o_x[i]);
      fa.Y32[i] = (fn == PRISM_FN_SQRT || fn == PRISM_FN_SQRT_NEWTON) ? r.at<float>(P.o_y[i]) : nullptr;
    }
  }
  { ProfScope ps(PK_PREP, r.s); launch_sumsq(pa, r.s); launch_prepare(pa, r.s); }
  if (P.p_s > 0 && max_iters > r.first_fit && fn != PRISM_FN_SQRT_NEWTON) {
    ProfScope ps(PK_SKETCH, r.s);
    launch_sketch(r.v0, P.Sp, P.S, P.ld, P.p_s, seed, r.first_fit, max_iters - r.first_fit, P.fn, r.s);
    if (r.planes()) CHECK_LAUNCH(launch_split_planes(r.v0, r.vp0, P.Sp, P.ld, max_iters - r.first_fit, r.s));
  }
  rc = check_hip();
  if (rc != PRISM_OK) return rc;
  if (dt == PRISM_BF16) rc = run_polar_bf16(r);
  else if (fn == PRISM_FN_POLAR || fn == PRISM_FN_SIGN) rc = run_polar_f32(r);
  else if (fn == PRISM_FN_INVERSE) rc = run_inverse_f32(r);
  else if (fn == PRISM_FN_SQRT_NEWTON) rc = run_sqrt_newton_f32(r);
  else if (fn == PRISM_FN_SQRT) rc = run_sqrt_f32(r);
  else rc = run_inv_root_f32(r);
  if (rc != PRISM_OK) return rc;
  { ProfScope ps(PK_FINAL, r.s); launch_finalize(fa, r.s); }
  return check_hip();
}

// bf16 polar factors of several shape groups that share the short side (the weight gradients of a
// layer stack: 768 x 768, 768 x 3072, 3072 x 768, 768 x 2304): one launch sequence for all of them
// on the caller's stream.  R, Q, the chain vectors and the control blocks of all matrices form one
// batch, so R^2, the chain products, the moments and the solve are single launches over every
// matrix of the call; the Gram product and the update take one descriptor per group in one launch
// each (the kernel maps its workgroup index to group, matrix and tile).  Every matrix goes through
// the kernels its own single-group call would pick.  Returns PRISM_EUNSUPPORTED (nothing enqueued)
// when the groups do not fit this form; the caller then takes the per-group path.
int run_polar_bf16_shapes(const prism_group* groups, int ngroups, int degree, int max_iters, int sketch_dim, uint64_t seed,
                          double tol, void* stream, const prism_options* opt, int batch_scale = 1) {
  static const int off = ab_switch("PRISM_NO_SHARED_SHAPES");
  if (off || ngroups < 2 || ngroups > BF16_MAX_GROUPS) return PRISM_EUNSUPPORTED;
  if (max_iters < 0 || max_iters > PRISM_MAX_ITERS || !(tol == tol)) return PRISM_EINVAL;
  if (opt && (opt->warm_iters < 0 || opt->schedule_len < 0 || opt->schedule_len > PRISM_MAX_ITERS ||
              (opt->schedule_len > 0 && !opt->alpha_schedule)))
    return PRISM_EINVAL;
  const unsigned flags = opt ? opt->flags : 0u;
  Plan Pg[BF16_MAX_GROUPS];
  long long btot = 0;
  for (int g = 0; g < ngroups; ++g) {
    if (groups[g].batch <= 0 || groups[g].m <= 0 || groups[g].n <= 0 || !groups[g].x) return PRISM_EUNSUPPORTED;   // empty or invalid: per-group path
    const int rc = make_plan(Pg[g], PRISM_FN_POLAR, groups[g].batch, groups[g].m, groups[g].n, PRISM_BF16, degree, sketch_dim, 0, flags);
    if (rc != PRISM_OK) return rc;
    if (Pg[g].S != Pg[0].S || Pg[g].Sp != Pg[0].Sp || Pg[g].tile != Pg[0].tile || Pg[g].ksplit) return PRISM_EUNSUPPORTED;
    // every group must get the chain kernels of its own call (batch_scale: the groups passed in are
    // 1 / batch_scale of the caller's groups each)
    const int bg = groups[g].batch * batch_scale, b0 = groups[0].batch * batch_scale;
    if (chain_takes_small_kernel(Pg[g].Sp, Pg[g].ld, bg, true) != chain_takes_small_kernel(Pg[0].Sp, Pg[0].ld, b0, true) ||
        chain_takes_small_kernel(Pg[g].Sp, Pg[g].ld, bg, false) != chain_takes_small_kernel(Pg[0].Sp, Pg[0].ld, b0, false) ||
        chain_bf16_supported(Pg[g].Sp, Pg[g].ld, bg, Pg[g].Sp) != chain_bf16_supported(Pg[0].Sp, Pg[0].ld, b0, Pg[0].Sp))
      return PRISM_EUNSUPPORTED;
    btot += groups[g].batch;
  }
  if (btot > PRISM_MAX_BATCH) return PRISM_EUNSUPPORTED;
  Run r;
  int rc = make_plan(r.P, PRISM_FN_POLAR, (int)btot, Pg[0].S, Pg[0].S, PRISM_BF16, degree, sketch_dim, 0, flags, true);
  if (rc != PRISM_OK) return rc;
  Plan& P = r.P;
  // iterate buffers per group behind the shared part
  size_t off_bytes = P.total;
  auto take = [&](size_t bytes) { size_t o = off_bytes; off_bytes = align256(off_bytes + bytes); return o; };
  size_t o_xhi[BF16_MAX_GROUPS][2], o_xlo[BF16_MAX_GROUPS][2];
  for (int g = 0; g < ngroups; ++g) {
    const size_t bytes = (size_t)groups[g].batch * Pg[g].Lp * Pg[g].Sp * 2;
    for (int i = 0; i < 2; ++i) {
      o_xhi[g][i] = take(bytes);
      o_xlo[g][i] = P.split ? take(bytes) : 0;
    }
  }
  P.total = off_bytes;
  r.s = (hipStream_t)stream;
  rc = get_workspace(P.total, r.s, nullptr, &r.ws);
  if (rc != PRISM_OK) return rc;
  r.ctrl = r.at<Ctrl>(P.o_ctrl);
  r.info = r.at<prism_info>(P.o_info);
  r.rho = r.at<float>(P.o_rho);
  r.v0 = r.at<float>(P.o_v0);
  r.v = r.at<float>(P.o_v);
  if (P.has_planes) { r.vp0 = r.at<uint16_t>(P.o_vp0); r.vp = r.at<uint16_t>(P.o_vp); }
  r.max_iters = max_iters; r.tol = tol; r.seed = seed; r.warm = opt ? opt->warm_iters : 0;
  r.sched = opt ? opt->alpha_schedule : nullptr;
  r.sched_len = opt ? opt->schedule_len : 0;
  r.first_fit = r.warm > r.sched_len ? r.warm : r.sched_len;
  r.chain_sel_batch = groups[0].batch * batch_scale;
  int boff = 0;
  for (int g = 0; g < ngroups; ++g) {
    Run::XGroup x = {};
    x.batch = groups[g].batch; x.boff = boff; x.m = groups[g].m; x.n = groups[g].n;
    x.L = Pg[g].L; x.Lp = Pg[g].Lp; x.transpose = Pg[g].transpose; x.x = groups[g].x;
    for (int i = 0; i < 2; ++i) {
      x.Xhi[i] = r.at<uint16_t>(o_xhi[g][i]);
      x.Xlo[i] = P.split ? r.at<uint16_t>(o_xlo[g][i]) : nullptr;
    }
    alias_output(P, x);
    r.xg.push_back(x);
    boff += x.batch;
  }
  auto group_args = [&](const Run::XGroup& x, PrepArgs& pa, FinalArgs& fa) {
    pa = PrepArgs{}; fa = FinalArgs{};
    pa.fn = PRISM_FN_POLAR; pa.dt = PRISM_BF16; pa.batch = x.batch; pa.m = x.m; pa.n = x.n;
    pa.S = P.S; pa.L = x.L; pa.Sp = P.Sp; pa.Lp = x.Lp; pa.transpose = x.transpose; pa.root_p = 0; pa.src = x.x;
    pa.sumsq_part = r.at<double>(P.o_sumsq) + (long long)x.boff * P.nsum; pa.nsum = P.nsum;
    pa.ctrl = r.ctrl + x.boff; pa.info = r.info + x.boff; pa.rho_part = r.rho; pa.tile = P.tile;
    fa.fn = PRISM_FN_POLAR; fa.dt = PRISM_BF16; fa.batch = x.batch; fa.m = x.m; fa.n = x.n;
    fa.S = P.S; fa.L = x.L; fa.Sp = P.Sp; fa.Lp = x.Lp; fa.transpose = x.transpose; fa.dst = x.x; fa.dst2 = nullptr;
    fa.ctrl = r.ctrl + x.boff;
    bf16_prep_final(P, x, pa, fa);
  };
  PrepArgs pa; FinalArgs fa;
  {
    ProfScope ps(PK_PREP, r.s);
    PrepArgs pas[BF16_MAX_GROUPS];
    int np = 0;
    for (const Run::XGroup& x : r.xg) { group_args(x, pa, fa); pas[np++] = pa; }
    if (!launch_prep_multi(pas, np, r.s))
      for (int i = 0; i < np; ++i) { launch_sumsq(pas[i], r.s); launch_prepare(pas[i], r.s); }
  }
  if (P.p_s > 0 && max_iters > r.first_fit) {
    ProfScope ps(PK_SKETCH, r.s);
    launch_sketch(r.v0, P.Sp, P.S, P.ld, P.p_s, seed, r.first_fit, max_iters - r.first_fit, P.fn, r.s);
    if (r.planes()) CHECK_LAUNCH(launch_split_planes(r.v0, r.vp0, P.Sp, P.ld, max_iters - r.first_fit, r.s));
  }
  rc = check_hip();
  if (rc != PRISM_OK) return rc;
  rc = run_polar_bf16(r);
  if (rc != PRISM_OK) return rc;
  {
    ProfScope ps(PK_FINAL, r.s);
    FinalArgs fas[BF16_MAX_GROUPS];
    int nf = 0;
    for (const Run::XGroup& x : r.xg) { group_args(x, pa, fa); fas[nf++] = fa; }
    if (!launch_finalize_multi(fas, nf, r.s))
      for (int i = 0; i < nf; ++i) launch_finalize(fas[i], r.s);
  }
  rc = check_hip();
  if (rc != PRISM_OK) return rc;
  // the reports were written into one array over all matrices: hand each group its part
  InfoScatter sc = {};
  sc.src = r.info; sc.ngroups = ngroups;
  bool wanted = false;
  boff = 0;
  for (int g = 0; g < ngroups; ++g) {
    sc.dst[g] = groups[g].info; sc.first[g] = (int)boff;
    wanted = wanted || groups[g].info;
    boff += groups[g].batch;
  }
  sc.first[ngroups] = (int)boff;
  if (wanted) launch_scatter_info(sc, r.s);
  return check_hip();
}

// Internal streams of the grouped call, per device, created on first use (default priority).
constexpr int GROUP_STREAMS = 4;
struct Fork {
  hipStream_t streams[GROUP_STREAMS] = {};
  hipEvent_t forked = nullptr, joined[GROUP_STREAMS] = {};
  bool ready = false;
};
std::mutex g_fork_mu;
std::map<int, Fork> g_forks;

int get_fork(Fork** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { set_last_error("hipGetDevice failed"); return PRISM_EHIP; }
  std::lock_guard<std::mutex> lock(g_fork_mu);
  Fork& f = g_forks[dev];
  if (!f.ready) {
    if (hipEventCreateWithFlags(&f.forked, hipEventDisableTiming) != hipSuccess) return PRISM_EHIP;
    for (int i = 0; i < GROUP_STREAMS; ++i) {
      if (hipStreamCreateWithFlags(&f.streams[i], hipStreamNonBlocking) != hipSuccess) return PRISM_EHIP;
      if (hipEventCreateWithFlags(&f.joined[i], hipEventDisableTiming) != hipSuccess) return PRISM_EHIP;
    }
    f.ready = true;
  }
  *out = &f;
  return PRISM_OK;
}

int run_grouped(int fn, const prism_group* groups, int ngroups, int root_p, int dt, int degree, int max_iters,
                int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt, bool from_auto_split = false) {
  set_last_error("");
  if (ngroups == 0) return PRISM_OK;
  if (!groups || ngroups < 0) return PRISM_EINVAL;
  if (opt && (opt->workspace || opt->info)) return PRISM_EINVAL;
  if (fn == PRISM_FN_INVERSE) degree = 5;                     // fixed polynomial
  if (fn == PRISM_FN_SQRT_NEWTON) { degree = 3; sketch_dim = sketch_dim ? 1 : 0; seed = 0; }
  static std::mutex enqueue_mu;      // the internal streams and events are shared by all callers on a device
  std::lock_guard<std::mutex> enqueue_lock(enqueue_mu);
  if (ngroups == 1) {
    prism_options o = opt ? *opt : prism_options{};
    o.info = groups[0].info;
    return run(fn, groups[0].x, groups[0].inv_out, root_p, groups[0].batch, groups[0].m, groups[0].n, dt, degree,
               max_iters, sketch_dim, seed, tol, stream, &o);
  }
  int rc;
  Fork* f = nullptr;
  hipStream_t user = (hipStream_t)stream;
  const bool single_stream = opt && (opt->flags & PRISM_FLAG_SINGLE_STREAM);
  if (fn == PRISM_FN_POLAR && dt == PRISM_BF16 && !from_auto_split) {
    // Groups that share the short side run as one launch sequence over all their matrices.  With
    // many matrices the sequence is issued for four quarters (or two halves) of every group on
    // internal streams: the latency-bound steps of one part (chain, moments, solve, prologues and
    // epilogues of short products) then run beside the products of another.  Measured on the
    // Muon-shaped batch of 64 (replayed from a HIP graph / eager): one sequence 4.00 / 3.93 ms, two
    // halves 3.80 / 3.82, four quarters 3.39 / 4.07, one call per group on four streams 3.40 / 4.09.
    static const int no_halves = ab_switch("PRISM_SHARED_SHAPES_NO_HALVES");
    static const int parts_sw = ab_switch("PRISM_SHARED_SHAPES_PARTS");
    long long btot = 0;
    int common = 4;   // parts every group's batch divides into: 4, else 2, else 1
    for (int gi = 0; gi < ngroups; ++gi) {
      btot += groups[gi].batch;
      while (common > 1 && (groups[gi].batch <= 0 || groups[gi].batch % common)) common >>= 1;
    }
    const int NP = (parts_sw == 2 || parts_sw == 4) ? (common >= parts_sw ? parts_sw : common) : common;
    const bool even = ngroups <= BF16_MAX_GROUPS && NP >= 2 && !single_stream;
    if (!even || btot < 32 || no_halves) {
      rc = run_polar_bf16_shapes(groups, ngroups, degree, max_iters, sketch_dim, seed, tol, stream, opt);
      if (rc != PRISM_EUNSUPPORTED) return rc;
    } else {
      prism_group half[4][BF16_MAX_GROUPS];   // NP <= 4 parts
      for (int gi = 0; gi < ngroups; ++gi) {
        const size_t bytes = (size_t)(groups[gi].batch / NP) * groups[gi].m * groups[gi].n * 2;
        for (int h = 0; h < NP; ++h) {
          half[h][gi] = groups[gi];
          half[h][gi].batch = groups[gi].batch / NP;
          half[h][gi].x = (char*)groups[gi].x + h * bytes;
          half[h][gi].info = groups[gi].info ? groups[gi].info + h * (groups[gi].batch / NP) : nullptr;
        }
      }
      rc = get_fork(&f);
      if (rc != PRISM_OK) return rc;
      if (hipEventRecord(f->forked, user) != hipSuccess) { (void)hipGetLastError(); set_last_error("hipEventRecord failed"); return PRISM_EHIP; }
      int forked = 0, first_error = PRISM_OK;
      for (; forked < NP; ++forked)
        if (hipStreamWaitEvent(f->streams[forked], f->forked, 0) != hipSuccess) { first_error = PRISM_EHIP; break; }
      bool unsupported = false;
      for (int h = 0; h < NP && first_error == PRISM_OK; ++h) {
        first_error = run_polar_bf16_shapes(half[h], ngroups, degree, max_iters, sketch_dim, seed, tol, f->streams[h], opt, NP);
        if (h == 0 && first_error == PRISM_EUNSUPPORTED) { unsupported = true; first_error = PRISM_OK; break; }   // nothing was enqueued
      }
      for (int i = 0; i < forked; ++i) {
        if (hipEventRecord(f->joined[i], f->streams[i]) != hipSuccess || hipStreamWaitEvent(user, f->joined[i], 0) != hipSuccess) {
          (void)hipGetLastError();
          if (first_error == PRISM_OK) { set_last_error("joining an internal stream failed"); first_error = PRISM_EHIP; }
        }
      }
      if (!unsupported) return first_error;
    }
    set_last_error("");
  }
  if (single_stream) {
    for (int gi = 0; gi < ngroups; ++gi) {
      prism_options o = opt ? *opt : prism_options{};
      o.info = groups[gi].info;
      rc = run(fn, groups[gi].x, groups[gi].inv_out, root_p, groups[gi].batch, groups[gi].m, groups[gi].n, dt, degree,
               max_iters, sketch_dim, seed, tol, stream, &o);
      if (rc != PRISM_OK) return rc;
    }
    return PRISM_OK;
  }
  rc = get_fork(&f);
  if (rc != PRISM_OK) return rc;
  const int used = ngroups < GROUP_STREAMS ? ngroups : GROUP_STREAMS;
  // nothing is forked before this record succeeds
  if (hipEventRecord(f->forked, user) != hipSuccess) { (void)hipGetLastError(); set_last_error("hipEventRecord failed"); return PRISM_EHIP; }
  int first_error = PRISM_OK;
  int forked = 0;   // internal streams that wait for the caller's stream: exactly these are joined again below
  for (; forked < used; ++forked)
    if (hipStreamWaitEvent(f->streams[forked], f->forked, 0) != hipSuccess) { first_error = PRISM_EHIP; break; }
  for (int gi = 0; gi < ngroups && first_error == PRISM_OK; ++gi) {
    prism_options o = opt ? *opt : prism_options{};
    o.info = groups[gi].info;
    o.flags |= PRISM_FLAG_SHARED_GPU;
    first_error = run(fn, groups[gi].x, groups[gi].inv_out, root_p, groups[gi].batch, groups[gi].m, groups[gi].n, dt,
                      degree, max_iters, sketch_dim, seed, tol, f->streams[gi % GROUP_STREAMS], &o);
  }
  // Join every forked stream back into the caller's, on every exit: after an error too, and past a
  // failing record or wait of one stream (the others are still joined, so that no forked work is
  // left unordered and a stream capture of the caller is not left with dangling branches).
  for (int i = 0; i < forked; ++i) {
    if (hipEventRecord(f->joined[i], f->streams[i]) != hipSuccess || hipStreamWaitEvent(user, f->joined[i], 0) != hipSuccess) {
      (void)hipGetLastError();
      if (first_error == PRISM_OK) { set_last_error("joining an internal stream failed"); first_error = PRISM_EHIP; }
    }
  }
  return first_error;
}

// Single-shape entry points: a large batch of large matrices is enqueued as two half batches on
// the internal streams, so that the partial last wave of tiles and the latency-bound kernels of one
// half run beside the GEMMs of the other (+3 % on 8 x 4096^2 and 32 x 1024^2).  Every matrix is
// computed exactly as in an unsplit call; an explicit workspace keeps the call on one stream.
int run_auto(int fn, void* a, void* inv_out, int root_p, int batch, int m, int n, int dt, int degree, int max_iters,
             int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt) {
  static const int no_split = ab_switch("PRISM_NO_BATCH_SPLIT");
  const int S = m < n ? m : n;
  if (no_split || !a || batch < 8 || (batch & 1) || S < 1024 || (opt && opt->workspace) || (opt && (opt->flags & PRISM_FLAG_SINGLE_STREAM)) || g_prof_on)
    return run(fn, a, inv_out, root_p, batch, m, n, dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
  const size_t esz = dt == PRISM_BF16 ? 2 : 4;
  const size_t half = (size_t)(batch / 2) * m * n * esz;
  prism_group gr[2];
  for (int h = 0; h < 2; ++h) {
    gr[h].x = (char*)a + h * half;
    gr[h].inv_out = inv_out ? (char*)inv_out + h * half : nullptr;
    gr[h].info = (opt && opt->info) ? opt->info + h * (batch / 2) : nullptr;
    gr[h].batch = batch / 2; gr[h].m = m; gr[h].n = n;
  }
  prism_options o = opt ? *opt : prism_options{};
  o.info = nullptr;
  return run_grouped(fn, gr, 2, root_p, dt, degree, max_iters, sketch_dim, seed, tol, stream, &o, true);
}

}  // namespace
}  // namespace prism

// Device memory of the entry point that allocates nothing: one array per GPU, part of the loaded
// code object, alive until the process ends.  In host code this name only stands for the symbol;
// the device address is looked up once per device and that pointer is what the kernels get.
// (No `used` attribute: the compiler gives a static device variable that host code refers to a
// global symbol in the code object by itself, which is what the runtime's lookup by name needs;
// with the attribute the symbol stays local and the lookup fails.)
static __device__ __align__(256) unsigned char scratch[PRISM_STATIC_SCRATCH_BYTES];

namespace prism {
namespace {
std::mutex g_scratch_mu;
std::map<int, void*> g_scratch_ptr;   // device ordinal -> address of that device's copy of `scratch`

int static_scratch(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); set_last_error("hipGetDevice failed"); return PRISM_EHIP; }
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  auto it = g_scratch_ptr.find(dev);
  if (it == g_scratch_ptr.end()) {
    void* ptr = nullptr;   // the current device is `dev`: the address returned is that of its copy
    const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) {
      (void)hipGetLastError();
      set_last_error("hipGetSymbolAddress of the static scratch array failed");
      return PRISM_EHIP;
    }
    if ((uintptr_t)ptr & 255) { set_last_error("static scratch array is not 256-byte aligned"); return PRISM_EHIP; }
    it = g_scratch_ptr.emplace(dev, ptr).first;
  }
  *out = it->second;
  return PRISM_OK;
}
}  // namespace
}  // namespace prism

using namespace prism;

extern "C" {

const char* prism_last_error(void) { return g_last_error.c_str(); }

int prism_release_workspaces(void) {
  set_last_error("");
  std::lock_guard<std::mutex> lock(g_mu);
  int rc = PRISM_OK, current = 0;
  const bool have_current = hipGetDevice(&current) == hipSuccess;
  for (auto& kv : g_cache) {
    if (hipSetDevice(kv.first.first) != hipSuccess) { rc = PRISM_EHIP; continue; }
    for (void* p : kv.second.retired)
      if (hipFree(p) != hipSuccess) rc = PRISM_EHIP;
    if (kv.second.ptr && hipFree(kv.second.ptr) != hipSuccess) rc = PRISM_EHIP;
  }
  g_cache.clear();
  if (have_current) (void)hipSetDevice(current);
  if (rc != PRISM_OK) { (void)hipGetLastError(); set_last_error("hipFree of a cached workspace failed"); }
  return rc;
}

int prism_profile_enable(int on) {
  std::lock_guard<std::mutex> lock(g_prof_mu);
  for (auto& r : g_prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  g_prof.clear();
  g_prof_on = on != 0;
  return PRISM_OK;
}

int prism_profile_collect(double* ms_by_kind, long long* launches_by_kind, int nkinds) {
  if (!ms_by_kind || !launches_by_kind || nkinds < PK_COUNT) return PRISM_EINVAL;
  std::lock_guard<std::mutex> lock(g_prof_mu);
  for (int i = 0; i < nkinds; ++i) { ms_by_kind[i] = 0.0; launches_by_kind[i] = 0; }
  for (auto& r : g_prof) {
    if (hipEventSynchronize(r.b) != hipSuccess) return PRISM_EHIP;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) return PRISM_EHIP;
    ms_by_kind[r.kind] += ms;
    launches_by_kind[r.kind] += 1;
  }
  return PRISM_OK;
}

int prism_workspace_bytes(int fn, int batch, int m, int n, prism_dtype dt, int degree, int sketch_dim,
                          int root_p, size_t* out_bytes) {
  if (!out_bytes || batch < 0 || m < 0 || n < 0) return PRISM_EINVAL;
  const bool empty = batch == 0 || m == 0 || n == 0;
  Plan P;
  int rc = empty ? make_plan(P, fn, 1, m ? m : 1, n ? n : 1, (int)dt, degree, sketch_dim, root_p, 0u)
                 : make_plan(P, fn, batch, m, n, (int)dt, degree, sketch_dim, root_p, 0u);
  if (rc != PRISM_OK) return rc;
  *out_bytes = empty ? 0 : P.total;
  return PRISM_OK;
}

int prism_polar(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters, int sketch_dim,
                uint64_t seed, double tol, void* stream) {
  return run_auto(PRISM_FN_POLAR, x, nullptr, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, nullptr);
}
int prism_polar_ex(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters, int sketch_dim,
                   uint64_t seed, double tol, void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_POLAR, x, nullptr, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
}
int prism_polar_static(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters, int sketch_dim,
                       uint64_t seed, double tol, void* stream, const prism_options* opt) {
  set_last_error("");
  if (opt && opt->workspace) { set_last_error("prism_polar_static takes no workspace: it uses the static array"); return PRISM_EINVAL; }
  if (batch < 0 || m < 0 || n < 0) return PRISM_EINVAL;
  prism_options o = opt ? *opt : prism_options{};
  if (batch > 0 && m > 0 && n > 0) {
    Plan P;
    const int rc = make_plan(P, PRISM_FN_POLAR, batch, m, n, (int)dt, degree, sketch_dim, 0, o.flags);
    if (rc != PRISM_OK) return rc;
    if (P.total > (size_t)PRISM_STATIC_SCRATCH_BYTES) {
      set_last_error("prism_polar_static: this call needs more than PRISM_STATIC_SCRATCH_BYTES of scratch; use prism_polar_ex");
      return PRISM_EUNSUPPORTED;
    }
    void* ptr = nullptr;
    const int rs = static_scratch(&ptr);
    if (rs != PRISM_OK) return rs;
    o.workspace = ptr;
    o.workspace_bytes = (size_t)PRISM_STATIC_SCRATCH_BYTES;
  }
  // straight to the single-stream driver: no internal streams, no cached workspace, no timing events
  t_prof_off = true;
  const int rc = run(PRISM_FN_POLAR, x, nullptr, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, &o);
  t_prof_off = false;
  return rc;
}

int prism_sqrt(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
               int sketch_dim, uint64_t seed, double tol, void* stream) {
  return run_auto(PRISM_FN_SQRT, a, inv_out, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, nullptr);
}
int prism_sqrt_ex(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                  int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_SQRT, a, inv_out, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
}
int prism_inv_root(void* a, int root_p, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                   int sketch_dim, uint64_t seed, double tol, void* stream) {
  return run_auto(PRISM_FN_INV_ROOT, a, nullptr, root_p, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, nullptr);
}
int prism_inv_root_ex(void* a, int root_p, int batch, int m, int n, prism_dtype dt, int degree, int max_iters,
                      int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_INV_ROOT, a, nullptr, root_p, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
}

int prism_sign(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters, int sketch_dim,
               uint64_t seed, double tol, void* stream) {
  return run_auto(PRISM_FN_SIGN, x, nullptr, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, nullptr);
}
int prism_sign_ex(void* x, int batch, int m, int n, prism_dtype dt, int degree, int max_iters, int sketch_dim,
                  uint64_t seed, double tol, void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_SIGN, x, nullptr, 0, batch, m, n, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
}
int prism_inverse(void* a, int batch, int m, int n, prism_dtype dt, int max_iters, int sketch_dim, uint64_t seed,
                  double tol, void* stream) {
  return run_auto(PRISM_FN_INVERSE, a, nullptr, 0, batch, m, n, (int)dt, 5, max_iters, sketch_dim, seed, tol, stream, nullptr);
}
int prism_inverse_ex(void* a, int batch, int m, int n, prism_dtype dt, int max_iters, int sketch_dim, uint64_t seed,
                     double tol, void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_INVERSE, a, nullptr, 0, batch, m, n, (int)dt, 5, max_iters, sketch_dim, seed, tol, stream, opt);
}

int prism_sqrt_newton(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int max_iters, int fit, double tol,
                      void* stream) {
  return run_auto(PRISM_FN_SQRT_NEWTON, a, inv_out, 0, batch, m, n, (int)dt, 3, max_iters, fit ? 1 : 0, 0, tol, stream, nullptr);
}
int prism_sqrt_newton_ex(void* a, void* inv_out, int batch, int m, int n, prism_dtype dt, int max_iters, int fit, double tol,
                         void* stream, const prism_options* opt) {
  return run_auto(PRISM_FN_SQRT_NEWTON, a, inv_out, 0, batch, m, n, (int)dt, 3, max_iters, fit ? 1 : 0, 0, tol, stream, opt);
}

int prism_spd_inverse(const float* a, float* out, int batch, int n, void* stream) {
  if (!a || !out || batch <= 0 || batch > PRISM_MAX_BATCH || n <= 0 || n % 64) return PRISM_EINVAL;
  char* ws = nullptr;
  const size_t bytes = (size_t)spd_inverse_scratch_floats(n, batch) * 4;
  if (bytes) {
    const int rc = get_workspace(bytes, (hipStream_t)stream, nullptr, &ws);
    if (rc != PRISM_OK) return rc;
  }
  return launch_spd_inverse(a, out, n, batch, nullptr, (float*)ws, (hipStream_t)stream);
}

int prism_run_grouped(prism_fn fn, const prism_group* groups, int ngroups, int root_p, prism_dtype dt, int degree,
                      int max_iters, int sketch_dim, uint64_t seed, double tol, void* stream, const prism_options* opt) {
  return run_grouped((int)fn, groups, ngroups, root_p, (int)dt, degree, max_iters, sketch_dim, seed, tol, stream, opt);
}

int prism_sketch(float* out, int n, int sketch_dim, uint64_t seed, int k, int fn, void* stream) {
  if (!out || n <= 0 || sketch_dim <= 0 || sketch_dim > PRISM_MAX_SKETCH || k < 0) return PRISM_EINVAL;
  launch_sketch(out, n, n, sketch_dim, sketch_dim, seed, k, 1, fn, (hipStream_t)stream);
  return check_hip();
}

int prism_gauss_parts(uint32_t first, uint32_t count, double* radius, double* cosv, double* sinv, void* stream) {
  if (!radius || !cosv || !sinv || count == 0 || (uint64_t)first + count > (1ull << 24)) return PRISM_EINVAL;
  launch_gauss_parts(first, count, radius, cosv, sinv, (hipStream_t)stream);
  return check_hip();
}

int prism_chain_product(const float* R, const float* V, float* out, int batch, int n, int ld, void* stream) {
  if (!R || !V || !out || batch <= 0 || batch > PRISM_MAX_BATCH || n <= 0) return PRISM_EINVAL;
  return launch_chain(R, (long long)n * n, n, V, (long long)n * ld, out, (long long)n * ld, n, ld, batch, nullptr,
                      (hipStream_t)stream);
}

int prism_chain_product_bf16(const uint16_t* Rb, const float* R, const float* V, float* out, uint16_t* planes, int batch,
                             int n, int ld, void* stream) {
  set_last_error("");
  if (!Rb || !R || !V || !out || batch <= 0 || batch > PRISM_MAX_BATCH || n <= 0) return PRISM_EINVAL;
  if (!chain_bf16_supported(n, ld, batch, n)) return PRISM_EUNSUPPORTED;
  hipStream_t s = (hipStream_t)stream;
  if (chain_takes_small_kernel(n, ld, batch, true))
    return launch_chain_bf16(Rb, (long long)n * n, n, R, (long long)n * n, n + 1, V, (long long)n * ld, out,
                             (long long)n * ld, n, ld, batch, nullptr, s);
  if (!planes) return PRISM_EINVAL;
  const long long pe = (long long)n * ld * 3;
  CHECK_LAUNCH(launch_split_planes(V, planes, n, ld, batch, s));
  return launch_chain_planes(Rb, (long long)n * n, n, R, (long long)n * n, n + 1, V, (long long)n * ld, planes, pe, out,
                             (long long)n * ld, planes + (long long)batch * pe, pe, n, ld, batch, nullptr, s);
}

int prism_gemm_f32(const float* A, const float* B, float* C, int batch, int M, int N, int K, int a_km, void* stream) {
  if (!A || !B || !C || batch <= 0 || batch > PRISM_MAX_BATCH || M <= 0 || N <= 0 || K <= 0) return PRISM_EINVAL;
  GemmDesc g = {};
  g.A = A; g.strideA = (long long)M * K; g.lda = (a_km & 1) ? M : K;
  g.B = B; g.strideB = (long long)K * N; g.ldb = N;
  g.M = M; g.N = N; g.K = K; g.a_km = a_km & 1; g.sym = (a_km >> 1) & 1; g.batch = batch; g.epi = EPI_STORE;
  g.C = C; g.strideC = (long long)M * N; g.ldc = N;
  const int tn = (N == 16 || N == 32 || N == 64) ? N : 128;
  return launch_gemm_f32(g, (tn == 64 && M % 128) ? 64 : 128, tn, (hipStream_t)stream);
}

int prism_gemm_f64a(const float* A, const double* B, double* C, int batch, int M, int N, int K, void* stream) {
  if (!A || !B || !C || batch <= 0 || batch > PRISM_MAX_BATCH || M <= 0 || N <= 0 || K <= 0) return PRISM_EINVAL;
  GemmDesc g = {};
  g.A = A; g.strideA = (long long)M * K; g.lda = K;
  g.B = B; g.strideB = (long long)K * N; g.ldb = N;
  g.M = M; g.N = N; g.K = K; g.a_km = 0; g.batch = batch; g.epi = EPI_STORE;
  g.C = C; g.strideC = (long long)M * N; g.ldc = N;
  return launch_gemm_f64a(g, 64, 64, (hipStream_t)stream);
}

int prism_gemm_bf16_nt(const uint16_t* A, const uint16_t* B, float* C, int batch, int M, int N, int K, int tile,
                       void* stream) {
  if (!A || !B || !C || batch <= 0 || batch > PRISM_MAX_BATCH || M <= 0 || N <= 0 || K <= 0) return PRISM_EINVAL;
  Bf16Desc g = {};
  g.A = A; g.strideA = (long long)M * K; g.lda = K;
  g.B = B; g.strideB = (long long)N * K; g.ldb = K;
  g.M = M; g.N = N; g.K = K; g.batch = batch; g.epi = BEPI_STORE;
  g.C32 = C; g.strideC32 = (long long)M * N; g.ldc32 = N;
  if (tile >= 20000) {          // B stored [K][N]
    tile -= 20000;
    g.km = 2; g.ldb = N;
  } else if (tile >= 10000) {   // A stored [K][M] and B stored [K][N]
    tile -= 10000;
    g.km = 3; g.lda = M; g.ldb = N;
  }
  if (tile == 2561) return launch_gemm_bf16(g, 256, 128, (hipStream_t)stream);
  return launch_gemm_bf16(g, tile, tile, (hipStream_t)stream);
}

}  // extern "C"
