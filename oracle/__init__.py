"""CPU oracle for the Fast-SNARF articulation path -- TEST INFRASTRUCTURE ONLY.

A ctypes/numpy front end of `fs_oracle.c`.  Only tests, the smoke check and the
benchmark's cpu_baseline leg may import this package; the HIP library never does and
shares no code with it.

Every entry takes `prec` = "f32" (strict single precision, explicit fused multiply-adds in
a fixed order: defines masks and trajectories) or "f64" (truth for root validity and
gradients).  Arrays follow the layouts in the C file's header.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
# FS_ORACLE_LIB: load another build of the same source instead (the sanitizer-instrumented one, in its own process)
_LIB_PATH = os.environ.get("FS_ORACLE_LIB") or os.path.join(_HERE, "libfs_oracle.so")
_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            from . import build as _b
            _b.build()
        _lib = ctypes.CDLL(_LIB_PATH)
    return _lib


def _dt(prec):
    return {"f32": np.float32, "f64": np.float64}[prec]


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def _dims(dims, nb, P):
    return np.array([dims[0], dims[1], dims[2], nb, P], dtype=np.int32)


def _box(lo, hi):
    return np.concatenate([np.asarray(lo, dtype=np.float32).astype(np.float64),
                           np.asarray(hi, dtype=np.float32).astype(np.float64)])


def _fn(name, prec):
    f = getattr(lib(), f"{name}_{prec}")
    f.restype = None
    return f


def precompute(dims, W, B, prec="f64"):
    """Sec. 3.1 "Pre-computing LBS": T [P, V, 12]."""
    dt = _dt(prec)
    W = _c(W, dt)
    B = _c(B, dt)
    P, nb = B.shape[0], B.shape[1]
    V = dims[0] * dims[1] * dims[2]
    T = np.empty((P, V, 12), dtype=dt)
    d = _dims(dims, nb, P)
    _fn("orc_precompute", prec)(_p(d), _p(W), _p(B), _p(T))
    return T


def forward(dims, lo, hi, T, x, pose=None, jac=False, prec="f64"):
    """d(x) = T(x) x (Eq. (4)/(5) with tri-linear T) and optionally dd/dx [9, n]."""
    dt = _dt(prec)
    T = _c(T, dt)
    x = _c(x, dt)
    n = x.shape[1]
    pose = _c(pose, np.int32)
    d = np.empty((3, n), dtype=dt)
    J = np.empty((9, n), dtype=dt) if jac else None
    dm = _dims(dims, 0, T.shape[0])
    bx = _box(lo, hi)
    _fn("orc_forward", prec)(_p(dm), _p(bx), _p(T), _p(x), _p(pose), ctypes.c_int64(n), _p(d), _p(J))
    return (d, J) if jac else d


def init_bone(dims, lo, hi, T, B, xq, pose=None, prec="f32"):
    """Eq. (8): per-bone initial states.  Returns x0 [K,3,N], Jinv0 [K,9,N], valid0 [K,N]."""
    dt = _dt(prec)
    T, B, xq = _c(T, dt), _c(B, dt), _c(xq, dt)
    pose = _c(pose, np.int32)
    P, nb = B.shape[0], B.shape[1]
    N = xq.shape[1]
    x0 = np.empty((nb, 3, N), dtype=dt)
    J0 = np.empty((nb, 9, N), dtype=dt)
    v0 = np.empty((nb, N), dtype=np.uint8)
    dm = _dims(dims, nb, P)
    bx = _box(lo, hi)
    _fn("orc_init_bone", prec)(_p(dm), _p(bx), _p(T), _p(B), _p(xq), _p(pose), ctypes.c_int64(N),
                               _p(x0), _p(J0), _p(v0))
    return x0, J0, v0


def corr_build(dims, lo, hi, T, corr_dims, prec="f32"):
    """Correspondence grid of the voxel-based initialisation.  Returns bbox [P,6], cand [P,ncell,ck]."""
    dt = _dt(prec)
    T = _c(T, dt)
    P = T.shape[0]
    cd = np.asarray(corr_dims, dtype=np.int32)
    ncell = int(cd[0]) * int(cd[1]) * int(cd[2])
    bbox = np.zeros((P, 6), dtype=dt)
    cand = np.empty((P, ncell, int(cd[3])), dtype=np.int32)
    dm = _dims(dims, 0, P)
    bx = _box(lo, hi)
    _fn("orc_corr_build", prec)(_p(dm), _p(bx), _p(T), _p(cd), _p(bbox), _p(cand))
    return bbox, cand


def init_voxel(dims, lo, hi, T, corr_dims, bbox, cand, xq, pose=None, prec="f32"):
    dt = _dt(prec)
    T, xq, bbox = _c(T, dt), _c(xq, dt), _c(bbox, dt)
    cand = _c(cand, np.int32)
    pose = _c(pose, np.int32)
    cd = np.asarray(corr_dims, dtype=np.int32)
    K = int(cd[3])
    N = xq.shape[1]
    x0 = np.empty((K, 3, N), dtype=dt)
    J0 = np.empty((K, 9, N), dtype=dt)
    v0 = np.empty((K, N), dtype=np.uint8)
    dm = _dims(dims, 0, T.shape[0])
    bx = _box(lo, hi)
    _fn("orc_init_voxel", prec)(_p(dm), _p(bx), _p(T), _p(cd), _p(bbox), _p(cand), _p(xq), _p(pose),
                                ctypes.c_int64(N), _p(x0), _p(J0), _p(v0))
    return x0, J0, v0


def solve(dims, lo, hi, T, xq, x0, Jinv0, valid0, pose=None, tol=1e-5, div_thresh=10.0,
          max_iters=50, prec="f32"):
    """Algorithm 1 (variant 2) with Broyden updates.  Returns xc [K,3,N], conv [K,N],
    Jinv [K,9,N], iters [K,N]."""
    dt = _dt(prec)
    T, xq, x0, Jinv0 = _c(T, dt), _c(xq, dt), _c(x0, dt), _c(Jinv0, dt)
    valid0 = _c(valid0, np.uint8)
    pose = _c(pose, np.int32)
    K, _, N = x0.shape
    xc = np.empty((K, 3, N), dtype=dt)
    cv = np.empty((K, N), dtype=np.uint8)
    Jo = np.empty((K, 9, N), dtype=dt)
    it = np.empty((K, N), dtype=np.uint8)
    dm = _dims(dims, 0, T.shape[0])
    bx = _box(lo, hi)
    # tol and div_thresh are rounded to float32 first so that both precisions square the same number
    prm = np.array([np.float32(tol), np.float32(div_thresh), max_iters], dtype=np.float64)
    _fn("orc_solve", prec)(_p(dm), _p(bx), _p(T), _p(prm), _p(xq), _p(pose), ctypes.c_int64(N),
                           ctypes.c_int32(K), _p(x0), _p(Jinv0), _p(valid0), _p(xc), _p(cv), _p(Jo), _p(it))
    return xc, cv, Jo, it


def grad(dims, lo, hi, T, W, B, xc, Jinv, conv, gxc, pose=None, mode=0, prec="f64", want_GT=False):
    """Implicit-differentiation backward.  mode 0: M = Broyden's last J~ (Eq. (15));
    mode 1: M = analytic inverse Jacobian (Eq. (12)).  Returns gW, gB, gxq[, G_T]."""
    dt = _dt(prec)
    T, W, B, xc, gxc = _c(T, dt), _c(W, dt), _c(B, dt), _c(xc, dt), _c(gxc, dt)
    Jinv = _c(Jinv, dt)
    conv = _c(conv, np.uint8)
    pose = _c(pose, np.int32)
    P, nb = B.shape[0], B.shape[1]
    K, _, N = xc.shape
    V = dims[0] * dims[1] * dims[2]
    gW = np.empty((dims[0], dims[1], dims[2], nb), dtype=dt)
    gB = np.empty((P, nb, 12), dtype=dt)
    gxq = np.empty((3, N), dtype=dt)
    GT = np.empty((P, V, 12), dtype=dt) if want_GT else None
    dm = _dims(dims, nb, P)
    bx = _box(lo, hi)
    _fn("orc_grad", prec)(_p(dm), _p(bx), _p(T), _p(W), _p(B), ctypes.c_int32(mode), _p(xc), _p(Jinv),
                          _p(conv), _p(gxc), _p(pose), ctypes.c_int64(N), ctypes.c_int32(K),
                          _p(gW), _p(gB), _p(gxq), _p(GT))
    return (gW, gB, gxq, GT) if want_GT else (gW, gB, gxq)


def dedupe(xc, conv, min_dist, prec="f32"):
    """Sec. 3.1 "Remove Duplicate Correspondences": greedy in lane order.  Returns keep [K,N], count [N]."""
    dt = _dt(prec)
    xc = _c(xc, dt)
    conv = _c(conv, np.uint8)
    K, _, N = xc.shape
    keep = np.empty((K, N), dtype=np.uint8)
    count = np.empty(N, dtype=np.int32)
    _fn("orc_dedupe", prec)(_p(xc), _p(conv), ctypes.c_int64(N), ctypes.c_int32(K),
                            ctypes.c_double(float(np.float32(min_dist))), _p(keep), _p(count))
    return keep, count


def brute_roots(dims, lo, hi, T, xq, starts_per_axis=8, merge_tol=1e-6, max_roots=16):
    """Exhaustive in-box root list per query (float64 checker).  T is one pose [V,12]."""
    T = _c(T, np.float64).reshape(-1, 12)
    xq = _c(xq, np.float64)
    n = xq.shape[1]
    roots = np.full((n, max_roots, 3), np.nan)
    count = np.zeros(n, dtype=np.int32)
    dm = _dims(dims, 0, 1)
    bx = _box(lo, hi)
    f = lib().orc_brute_roots_f64
    f.restype = None
    f(_p(dm), _p(bx), _p(T), _p(xq), ctypes.c_int64(n), ctypes.c_int32(starts_per_axis),
      ctypes.c_double(merge_tol), ctypes.c_int32(max_roots), _p(roots), _p(count))
    return roots, count
