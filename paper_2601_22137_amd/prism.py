"""ctypes binding of libprism.so (see include/prism.h).  Argument marshalling only: every
step of the path runs in the HIP kernels.  PyTorch supplies device memory and the stream.

The library must have been built (python -m paper_2601_22137_amd.build); there is no fallback.
"""
import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprism.so")

F32, BF16 = 0, 1
FN_POLAR, FN_SQRT, FN_INV_ROOT, FN_SIGN, FN_INVERSE, FN_SQRT_NEWTON = 1, 2, 3, 4, 5, 6
MAX_ITERS = 64
FLAG_BF16_PLAIN_ITERATE = 1
FLAG_SHARED_GPU = 2
FLAG_SINGLE_STREAM = 4
OK, EINVAL, EUNSUPPORTED, ENOMEM, EHIP = 0, 1, 2, 3, 4
INFO_CONVERGED, INFO_BUDGET, INFO_NONFINITE, INFO_ZERO, INFO_DIVERGED = 0, 1, 2, 3, 4

INFO_DTYPE = np.dtype([("iters", np.int32), ("status", np.int32),
                       ("residual", np.float32, (MAX_ITERS + 1,)), ("alpha", np.float32, (MAX_ITERS,))])

EXPORTS = ("prism_workspace_bytes", "prism_release_workspaces", "prism_polar", "prism_polar_ex", "prism_polar_static", "prism_sqrt", "prism_sqrt_ex",
           "prism_inv_root", "prism_inv_root_ex", "prism_sign", "prism_sign_ex", "prism_inverse", "prism_inverse_ex", "prism_sqrt_newton", "prism_sqrt_newton_ex", "prism_spd_inverse", "prism_run_grouped",
           "prism_sketch", "prism_gauss_parts", "prism_chain_product", "prism_chain_product_bf16", "prism_gemm_f32",
           "prism_gemm_f64a", "prism_gemm_bf16_nt", "prism_profile_enable", "prism_profile_collect",
           "prism_last_error")

PROFILE_KINDS = ("prep", "final", "sketch", "chain", "solve", "f32_resid", "f32_polyq", "f32_apply", "f32_store",
                 "f64_mnext", "make_t", "bf16_gram", "bf16_polyq", "bf16_apply", "bf16_store", "spd_inverse", "db_moments",
                 "db_update_m", "f32_small_polar", "moments")


class Options(ctypes.Structure):
    _fields_ = [("flags", ctypes.c_uint32), ("warm_iters", ctypes.c_int32), ("workspace", ctypes.c_void_p),
                ("workspace_bytes", ctypes.c_size_t), ("info", ctypes.c_void_p),
                ("alpha_schedule", ctypes.POINTER(ctypes.c_float)), ("schedule_len", ctypes.c_int32)]


class Group(ctypes.Structure):
    _fields_ = [("x", ctypes.c_void_p), ("inv_out", ctypes.c_void_p), ("info", ctypes.c_void_p),
                ("batch", ctypes.c_int32), ("m", ctypes.c_int32), ("n", ctypes.c_int32)]


class PrismError(RuntimeError):
    pass


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise PrismError("libprism.so is not built: run `python -m paper_2601_22137_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, u64, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_uint64, ctypes.c_double
        L.prism_last_error.restype = ctypes.c_char_p
        L.prism_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i, ctypes.POINTER(ctypes.c_size_t)]
        L.prism_polar.argtypes = [vp, i, i, i, i, i, i, i, u64, dbl, vp]
        L.prism_polar_ex.argtypes = L.prism_polar.argtypes + [ctypes.POINTER(Options)]
        L.prism_polar_static.argtypes = L.prism_polar_ex.argtypes
        L.prism_sqrt.argtypes = [vp, vp, i, i, i, i, i, i, i, u64, dbl, vp]
        L.prism_sqrt_ex.argtypes = L.prism_sqrt.argtypes + [ctypes.POINTER(Options)]
        L.prism_inv_root.argtypes = [vp, i, i, i, i, i, i, i, i, u64, dbl, vp]
        L.prism_inv_root_ex.argtypes = L.prism_inv_root.argtypes + [ctypes.POINTER(Options)]
        L.prism_sign.argtypes = [vp, i, i, i, i, i, i, i, u64, dbl, vp]
        L.prism_sign_ex.argtypes = L.prism_sign.argtypes + [ctypes.POINTER(Options)]
        L.prism_inverse.argtypes = [vp, i, i, i, i, i, i, u64, dbl, vp]
        L.prism_inverse_ex.argtypes = L.prism_inverse.argtypes + [ctypes.POINTER(Options)]
        L.prism_sqrt_newton.argtypes = [vp, vp, i, i, i, i, i, i, dbl, vp]
        L.prism_sqrt_newton_ex.argtypes = L.prism_sqrt_newton.argtypes + [ctypes.POINTER(Options)]
        L.prism_spd_inverse.argtypes = [vp, vp, i, i, vp]
        L.prism_run_grouped.argtypes = [i, ctypes.POINTER(Group), i, i, i, i, i, i, u64, dbl, vp, ctypes.POINTER(Options)]
        L.prism_sketch.argtypes = [vp, i, i, u64, i, i, vp]
        L.prism_gauss_parts.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vp, vp, vp, vp]
        L.prism_chain_product.argtypes = [vp, vp, vp, i, i, i, vp]
        L.prism_chain_product_bf16.argtypes = [vp, vp, vp, vp, vp, i, i, i, vp]
        L.prism_gemm_f32.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.prism_gemm_f64a.argtypes = [vp, vp, vp, i, i, i, i, vp]
        L.prism_gemm_bf16_nt.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.prism_profile_enable.argtypes = [i]
        L.prism_profile_collect.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_longlong), i]
        _lib = L
    return _lib


def _check(rc):
    if rc != OK:
        names = {EINVAL: "PRISM_EINVAL", EUNSUPPORTED: "PRISM_EUNSUPPORTED", ENOMEM: "PRISM_ENOMEM", EHIP: "PRISM_EHIP"}
        raise PrismError("%s (%s)" % (names.get(rc, rc), lib().prism_last_error().decode()))


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise PrismError("unsupported dtype %s" % t.dtype)


def _batched(t):
    if not (t.is_cuda and t.is_contiguous() and t.dim() == 3):
        raise PrismError("expected a contiguous CUDA tensor [batch, m, n]")
    return t.shape


class _Info:
    def __init__(self, batch, device):
        self.buf = torch.empty(batch * INFO_DTYPE.itemsize, dtype=torch.uint8, device=device)

    def read(self):
        """Synchronises and returns a numpy structured array (one record per matrix)."""
        return self.buf.cpu().numpy().view(INFO_DTYPE).copy()


def _options(info, flags, warm_iters, workspace, alpha_schedule=None):
    o = Options()
    if alpha_schedule is not None and len(alpha_schedule) > 0:
        o._sched = (ctypes.c_float * len(alpha_schedule))(*[float(a) for a in alpha_schedule])   # kept alive by o
        o.alpha_schedule = ctypes.cast(o._sched, ctypes.POINTER(ctypes.c_float))
        o.schedule_len = len(alpha_schedule)
    o.flags = flags
    o.warm_iters = warm_iters
    o.workspace = workspace.data_ptr() if workspace is not None else None
    o.workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    o.info = info.buf.data_ptr()
    return o


def workspace_bytes(fn, batch, m, n, dtype_code, degree, sketch_dim, root_p=0):
    out = ctypes.c_size_t(0)
    _check(lib().prism_workspace_bytes(fn, batch, m, n, dtype_code, degree, sketch_dim, root_p, ctypes.byref(out)))
    return out.value


def polar(x, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, flags=0, warm_iters=0, workspace=None,
          alpha_schedule=None):
    """In place: x[batch, m, n] <- polar factor.  Returns an info handle (.read() synchronises)."""
    b, m, n = _batched(x)
    info = _Info(b, x.device)
    o = _options(info, flags, warm_iters, workspace, alpha_schedule)
    _check(lib().prism_polar_ex(x.data_ptr(), b, m, n, _dtype_code(x), degree, max_iters, sketch_dim, seed, tol,
                                _stream(), ctypes.byref(o)))
    return info


STATIC_SCRATCH_BYTES = 32 << 20


def new_info(batch, device="cuda"):
    """An info handle made ahead of time, for calls that must not allocate (polar_static)."""
    return _Info(batch, device)


def polar_static(x, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, flags=0, warm_iters=0, info=None,
                 alpha_schedule=None):
    """polar() through the entry point that allocates nothing: the library's intermediates live in
    its static device array (STATIC_SCRATCH_BYTES; larger calls raise PRISM_EUNSUPPORTED).  `info` is
    a handle from new_info() made beforehand, or None; nothing is allocated here either."""
    b, m, n = _batched(x)
    o = Options()
    if alpha_schedule is not None and len(alpha_schedule) > 0:
        o._sched = (ctypes.c_float * len(alpha_schedule))(*[float(a) for a in alpha_schedule])
        o.alpha_schedule = ctypes.cast(o._sched, ctypes.POINTER(ctypes.c_float))
        o.schedule_len = len(alpha_schedule)
    o.flags = flags
    o.warm_iters = warm_iters
    o.info = info.buf.data_ptr() if info is not None else None
    _check(lib().prism_polar_static(x.data_ptr(), b, m, n, _dtype_code(x), degree, max_iters, sketch_dim, seed, tol,
                                    _stream(), ctypes.byref(o)))
    return info


def sqrt(a, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, warm_iters=0, workspace=None,
         alpha_schedule=None, flags=0):
    """In place: a <- A^(1/2); returns (A^(-1/2), info handle)."""
    b, m, n = _batched(a)
    inv = torch.empty_like(a)
    info = _Info(b, a.device)
    o = _options(info, flags, warm_iters, workspace, alpha_schedule)
    _check(lib().prism_sqrt_ex(a.data_ptr(), inv.data_ptr(), b, m, n, _dtype_code(a), degree, max_iters, sketch_dim,
                               seed, tol, _stream(), ctypes.byref(o)))
    return inv, info


def inv_root(a, root_p, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, warm_iters=0, workspace=None,
             alpha_schedule=None, flags=0):
    """In place: a <- A^(-1/root_p).  Returns an info handle."""
    b, m, n = _batched(a)
    info = _Info(b, a.device)
    o = _options(info, flags, warm_iters, workspace, alpha_schedule)
    _check(lib().prism_inv_root_ex(a.data_ptr(), root_p, b, m, n, _dtype_code(a), 3, max_iters, sketch_dim, seed,
                                   tol, _stream(), ctypes.byref(o)))
    return info


def sign(x, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, warm_iters=0, workspace=None,
         alpha_schedule=None, flags=0):
    """In place: x[batch, n, n] <- sign(x).  Returns an info handle."""
    b, m, n = _batched(x)
    info = _Info(b, x.device)
    o = _options(info, flags, warm_iters, workspace, alpha_schedule)
    _check(lib().prism_sign_ex(x.data_ptr(), b, m, n, _dtype_code(x), degree, max_iters, sketch_dim, seed, tol,
                               _stream(), ctypes.byref(o)))
    return info


def inverse(a, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, warm_iters=0, workspace=None, alpha_schedule=None, flags=0):
    """In place: a[batch, n, n] <- a^(-1) by the Chebyshev iteration.  Returns an info handle."""
    b, m, n = _batched(a)
    info = _Info(b, a.device)
    o = _options(info, flags, warm_iters, workspace, alpha_schedule)
    _check(lib().prism_inverse_ex(a.data_ptr(), b, m, n, _dtype_code(a), max_iters, sketch_dim, seed, tol,
                                  _stream(), ctypes.byref(o)))
    return info


def sqrt_newton(a, max_iters=30, tol=1e-6, fit=True, workspace=None, alpha_schedule=None, flags=0):
    """In place: a <- A^(1/2) by the DB Newton iteration; returns (A^(-1/2), info handle)."""
    b, m, n = _batched(a)
    inv = torch.empty_like(a)
    info = _Info(b, a.device)
    o = _options(info, flags, 0, workspace, alpha_schedule)
    _check(lib().prism_sqrt_newton_ex(a.data_ptr(), inv.data_ptr(), b, m, n, _dtype_code(a), max_iters, int(bool(fit)), tol,
                                      _stream(), ctypes.byref(o)))
    return inv, info


def run_grouped(fn, xs, degree=5, max_iters=30, sketch_dim=8, seed=22137, tol=1e-6, root_p=0, flags=0, warm_iters=0,
                alpha_schedule=None):
    """One call over tensors of different shapes (each [batch, m, n], all of one dtype), in place.
    Returns (inverse outputs or None per group, info handles per group)."""
    if len(xs) == 0:
        _check(lib().prism_run_grouped(fn, None, 0, root_p, F32, degree, max_iters, sketch_dim, seed, tol, _stream(), None))
        return [], []
    groups = (Group * len(xs))()
    infos, invs = [], []
    two_outputs = fn in (FN_SQRT, FN_SQRT_NEWTON)
    for g, x in zip(groups, xs):
        b, m, n = _batched(x)
        info = _Info(b, x.device)
        inv = torch.empty_like(x) if two_outputs else None
        g.x, g.inv_out, g.info = x.data_ptr(), (inv.data_ptr() if two_outputs else None), info.buf.data_ptr()
        g.batch, g.m, g.n = b, m, n
        infos.append(info)
        invs.append(inv)
    o = Options()
    o.flags, o.warm_iters = flags, warm_iters
    if alpha_schedule is not None and len(alpha_schedule) > 0:
        o._sched = (ctypes.c_float * len(alpha_schedule))(*[float(a) for a in alpha_schedule])
        o.alpha_schedule = ctypes.cast(o._sched, ctypes.POINTER(ctypes.c_float))
        o.schedule_len = len(alpha_schedule)
    _check(lib().prism_run_grouped(fn, groups, len(xs), root_p, _dtype_code(xs[0]), degree, max_iters, sketch_dim, seed, tol,
                                   _stream(), ctypes.byref(o)))
    return invs, infos


# ---- single steps (unit tests, profiling) ----

def spd_inverse(a):
    batch, n, _ = a.shape
    out = torch.empty_like(a)
    _check(lib().prism_spd_inverse(a.data_ptr(), out.data_ptr(), batch, n, _stream()))
    return out


def sketch(n, sketch_dim, seed, k, fn, device="cuda"):
    out = torch.empty((n, sketch_dim), dtype=torch.float32, device=device)
    _check(lib().prism_sketch(out.data_ptr(), n, sketch_dim, seed, k, fn, _stream()))
    return out


def gauss_parts(first, count, device="cuda"):
    r = torch.empty(count, dtype=torch.float64, device=device)
    c = torch.empty_like(r)
    s = torch.empty_like(r)
    _check(lib().prism_gauss_parts(first, count, r.data_ptr(), c.data_ptr(), s.data_ptr(), _stream()))
    return r, c, s


def chain_product(R, V):
    batch, n, ld = V.shape
    out = torch.empty_like(V)
    _check(lib().prism_chain_product(R.data_ptr(), V.data_ptr(), out.data_ptr(), batch, n, ld, _stream()))
    return out


def release_workspaces():
    """Free the library's cached workspaces (nothing may be in flight, no captured graph may be replayed)."""
    torch.cuda.synchronize()
    _check(lib().prism_release_workspaces())


def chain_product_bf16(Rb, R, V, return_planes=False):
    """out = (Rb + diag(R - Rb)) V.  With return_planes also the scratch array of the call: bf16 bit
    patterns [2][batch][n / 256][3][ld][32 units, low four bits xor-ed with the column][8], the planes of V and of out (zeros where the launch is
    small enough for the kernel that does not use them)."""
    batch, n, ld = V.shape
    out = torch.empty_like(V)
    planes = torch.zeros((2, batch, n * ld * 3), dtype=torch.int16, device=V.device)
    _check(lib().prism_chain_product_bf16(Rb.data_ptr(), R.data_ptr(), V.data_ptr(), out.data_ptr(), planes.data_ptr(),
                                          batch, n, ld, _stream()))
    return (out, planes) if return_planes else out


def gemm_f32(A, B, a_km=False, sym=False):
    batch = A.shape[0]
    M, K = (A.shape[2], A.shape[1]) if a_km else (A.shape[1], A.shape[2])
    N = B.shape[2]
    C = torch.empty((batch, M, N), dtype=torch.float32, device=A.device)
    _check(lib().prism_gemm_f32(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, N, K, int(a_km) | (2 if sym else 0), _stream()))
    return C


def gemm_f64a(A, B):
    batch, M, K = A.shape
    N = B.shape[2]
    C = torch.empty((batch, M, N), dtype=torch.float64, device=A.device)
    _check(lib().prism_gemm_f64a(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, N, K, _stream()))
    return C


def gemm_bf16_nt(A, B, tile, km=0):
    """C = A B^T.  km = 0: A [batch][M][K], B [batch][N][K]; km = 2: B is stored [batch][K][N];
    km = 3: A is stored [batch][K][M] and B [batch][K][N]."""
    if km not in (0, 2, 3):
        raise ValueError("km must be 0, 2 or 3")
    batch = A.shape[0]
    K, M = (A.shape[1], A.shape[2]) if km == 3 else (A.shape[2], A.shape[1])
    N = B.shape[2] if km else B.shape[1]
    if (B.shape[1] if km else B.shape[2]) != K or B.shape[0] != batch:
        raise ValueError("operand shapes do not match")
    tile = tile + (10000 if km == 3 else 20000 if km == 2 else 0)
    C = torch.empty((batch, M, N), dtype=torch.float32, device=A.device)
    _check(lib().prism_gemm_bf16_nt(A.data_ptr(), B.data_ptr(), C.data_ptr(), batch, M, N, K, tile, _stream()))
    return C


def profile_enable(on):
    _check(lib().prism_profile_enable(int(on)))


def profile_collect():
    """{kind: (milliseconds, launches)} summed over everything recorded since profile_enable(True)."""
    n = len(PROFILE_KINDS)
    ms = (ctypes.c_double * n)()
    cnt = (ctypes.c_longlong * n)()
    _check(lib().prism_profile_collect(ms, cnt, n))
    return {k: (ms[j], cnt[j]) for j, k in enumerate(PROFILE_KINDS)}
