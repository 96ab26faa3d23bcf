"""Thin ctypes binding of the C-ABI library (include/fastsnarf.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch supplies
device memory (`tensor.data_ptr()`) and the current HIP stream.  There is no CPU fallback: if the
library has not been built, `load()` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "csrc", "libfastsnarf.so")

FS_OK, FS_E_ARG, FS_E_SHAPE, FS_E_STATE, FS_E_ALLOC, FS_E_DEVICE, FS_E_UNSUPPORTED = range(7)
STATUS_NAMES = ["FS_OK", "FS_E_ARG", "FS_E_SHAPE", "FS_E_STATE", "FS_E_ALLOC", "FS_E_DEVICE", "FS_E_UNSUPPORTED"]
FS_INIT_BONE, FS_INIT_VOXEL = 0, 1
FS_GRAD_BROYDEN_J, FS_GRAD_EXACT_J = 0, 1

EXPORTS = ["fs_create", "fs_destroy", "fs_set_params", "fs_set_tuning", "fs_set_list_order", "fs_set_spin_limit", "fs_precompute", "fs_init", "fs_solve", "fs_grad",
           "fs_dedupe", "fs_dedupe_noalloc", "fs_get_transforms", "fs_get_corr", "fs_microbench", "fs_set_timing", "fs_get_timing", "fs_last_error",
           "fs_version"]


class GridDesc(ctypes.Structure):
    _fields_ = [("nx", ctypes.c_int32), ("ny", ctypes.c_int32), ("nz", ctypes.c_int32),
                ("n_bones", ctypes.c_int32), ("n_poses", ctypes.c_int32),
                ("lo", ctypes.c_float * 3), ("hi", ctypes.c_float * 3)]


class Params(ctypes.Structure):
    _fields_ = [("tol", ctypes.c_float), ("div_thresh", ctypes.c_float), ("max_iters", ctypes.c_int32),
                ("init_mode", ctypes.c_int32), ("grad_mode", ctypes.c_int32),
                ("corr_nx", ctypes.c_int32), ("corr_ny", ctypes.c_int32), ("corr_nz", ctypes.c_int32),
                ("corr_k", ctypes.c_int32)]


class FsError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS_NAMES[status] if 0 <= status < 7 else status}: {msg}")
        self.status = status


_lib = None


def load():
    """dlopen the HIP library and declare its prototypes.  Raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not found: build it with `python -m paper_2211_15601_amd.build` "
                           "(there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
    L.fs_create.argtypes = [ctypes.POINTER(GridDesc), ctypes.POINTER(Params), vp, ctypes.POINTER(vp)]
    L.fs_destroy.argtypes = [vp]
    L.fs_set_params.argtypes = [vp, ctypes.POINTER(Params)]
    L.fs_precompute.argtypes = [vp, vp, vp]
    L.fs_init.argtypes = [vp, vp, vp, i64, vp, vp, vp]
    L.fs_solve.argtypes = [vp, vp, vp, i64, i32, vp, vp, vp, vp, vp, vp, vp, vp]
    L.fs_grad.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i32, vp, vp, vp, vp]
    L.fs_get_transforms.argtypes = [vp, vp]
    L.fs_get_corr.argtypes = [vp, vp, vp]
    L.fs_last_error.argtypes = [vp]
    L.fs_last_error.restype = ctypes.c_char_p
    L.fs_version.argtypes = []
    L.fs_version.restype = ctypes.c_char_p
    L.fs_set_tuning.argtypes = [vp, i32, i32, i32, i32, i32]
    L.fs_set_spin_limit.argtypes = [vp, i32]
    L.fs_set_list_order.argtypes = [vp, i32]
    L.fs_microbench.argtypes = [i32, i64, ctypes.POINTER(ctypes.c_double)]
    L.fs_set_timing.argtypes = [vp, i32]
    L.fs_get_timing.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i32)]
    L.fs_dedupe.argtypes = [vp, vp, vp, i64, i32, ctypes.c_float, vp, vp, vp, vp, i64]
    L.fs_dedupe_noalloc.argtypes = L.fs_dedupe.argtypes
    for name in EXPORTS:
        if name not in ("fs_last_error", "fs_version"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return ctypes.c_void_p(t.data_ptr())


class Context:
    """One fs_ctx.  Methods mirror the C entry points one to one and return the raw status when
    `check=False`, else raise FsError on a non-OK status."""

    def __init__(self, dims, n_bones, lo, hi, n_poses=1, tol=1e-5, div_thresh=10.0, max_iters=50,
                 init_mode=FS_INIT_BONE, grad_mode=FS_GRAD_BROYDEN_J, corr_dims=(32, 32, 8, 3), stream=None):
        L = load()
        self._L = L
        self.desc = GridDesc(int(dims[0]), int(dims[1]), int(dims[2]), int(n_bones), int(n_poses),
                             (ctypes.c_float * 3)(*[float(v) for v in lo]),
                             (ctypes.c_float * 3)(*[float(v) for v in hi]))
        self.params = Params(float(tol), float(div_thresh), int(max_iters), int(init_mode), int(grad_mode),
                             int(corr_dims[0]), int(corr_dims[1]), int(corr_dims[2]), int(corr_dims[3]))
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.stream = int(stream)
        h = ctypes.c_void_p()
        st = L.fs_create(ctypes.byref(self.desc), ctypes.byref(self.params), ctypes.c_void_p(self.stream),
                         ctypes.byref(h))
        if st != FS_OK:
            raise FsError(st, "fs_create failed")
        self._h = h
        self.K = int(n_bones) if init_mode == FS_INIT_BONE else int(corr_dims[3])
        self.V = int(dims[0]) * int(dims[1]) * int(dims[2])

    def _ret(self, st, check):
        if check and st != FS_OK:
            raise FsError(st, self.last_error())
        return st

    def last_error(self) -> str:
        return self._L.fs_last_error(self._h).decode()

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            self._L.fs_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_params(self, tol=None, div_thresh=None, max_iters=None, grad_mode=None, check=True):
        p = self.params
        if tol is not None: p.tol = float(tol)
        if div_thresh is not None: p.div_thresh = float(div_thresh)
        if max_iters is not None: p.max_iters = int(max_iters)
        if grad_mode is not None: p.grad_mode = int(grad_mode)
        return self._ret(self._L.fs_set_params(self._h, ctypes.byref(p)), check)

    def set_tuning(self, chunk=0, refill_min=0, blocks_per_cu=0, point_major=-1, lds_grid=-1, check=True):
        return self._ret(self._L.fs_set_tuning(self._h, int(chunk), int(refill_min), int(blocks_per_cu),
                                               int(point_major), int(lds_grid)), check)

    def set_list_order(self, by_place, check=True):
        return self._ret(self._L.fs_set_list_order(self._h, int(by_place)), check)

    def set_spin_limit(self, polls, check=True):
        return self._ret(self._L.fs_set_spin_limit(self._h, int(polls)), check)

    def precompute(self, W, B, check=True):
        self.pre_serial = getattr(self, "pre_serial", 0) + 1          # lets a caller tell whose W and B the context holds
        return self._ret(self._L.fs_precompute(self._h, _ptr(W), _ptr(B)), check)

    def init(self, xq, pose, N, x0, Jinv0, valid0, check=True):
        return self._ret(self._L.fs_init(self._h, _ptr(xq), _ptr(pose), N, _ptr(x0), _ptr(Jinv0), _ptr(valid0)), check)

    def solve(self, xq, pose, N, K, x0, Jinv0, valid0, xc, conv, Jinv=None, iters=None, slot=None, check=True):
        self.solve_serial = getattr(self, "solve_serial", 0) + 1      # lets a caller tell whether `slot` is still the last one
        return self._ret(self._L.fs_solve(self._h, _ptr(xq), _ptr(pose), N, K, _ptr(x0), _ptr(Jinv0), _ptr(valid0),
                                          _ptr(xc), _ptr(conv), _ptr(Jinv), _ptr(iters), _ptr(slot)), check)

    def grad(self, W, xc, Jinv, conv, gxc, pose, N, K, gW, gB, gxq=None, slot=None, check=True):
        return self._ret(self._L.fs_grad(self._h, _ptr(W), _ptr(xc), _ptr(Jinv), _ptr(conv), _ptr(gxc), _ptr(pose),
                                         N, K, _ptr(slot), _ptr(gW), _ptr(gB), _ptr(gxq)), check)

    def dedupe(self, xc, conv, N, K, min_dist, keep, offsets, roots=None, lane=None, cap=0, check=True):
        return self._ret(self._L.fs_dedupe(self._h, _ptr(xc), _ptr(conv), N, K, float(min_dist), _ptr(keep),
                                           _ptr(offsets), _ptr(roots), _ptr(lane), cap), check)

    def dedupe_noalloc(self, xc, conv, N, K, min_dist, keep, offsets, roots=None, lane=None, cap=0, check=True):
        return self._ret(self._L.fs_dedupe_noalloc(self._h, _ptr(xc), _ptr(conv), N, K, float(min_dist), _ptr(keep),
                                                   _ptr(offsets), _ptr(roots), _ptr(lane), cap), check)

    def set_timing(self, enable=True, check=True):
        return self._ret(self._L.fs_set_timing(self._h, int(bool(enable))), check)

    def get_timing(self):
        """(summed k_solve milliseconds, launches) since the last call; synchronises the stream."""
        ms, n = ctypes.c_double(), ctypes.c_int32()
        self._ret(self._L.fs_get_timing(self._h, ctypes.byref(ms), ctypes.byref(n)), True)
        return ms.value, n.value

    def get_transforms(self, T, check=True):
        return self._ret(self._L.fs_get_transforms(self._h, _ptr(T)), check)

    def get_corr(self, bbox, cand, check=True):
        return self._ret(self._L.fs_get_corr(self._h, _ptr(bbox), _ptr(cand)), check)


MB_FMA, MB_GATHER_LANE, MB_GATHER_LINE, MB_LDS_GATHER, MB_GATHER_SEGMENT = range(5)


def microbench(which: int, array_bytes: int = 3 << 20) -> float:
    """Run one of the library's micro-benchmarks; returns flop/s (MB_FMA) or 16-byte loads/s."""
    L = load()
    r = ctypes.c_double()
    st = L.fs_microbench(int(which), int(array_bytes), ctypes.byref(r))
    if st != FS_OK:
        raise FsError(st, "fs_microbench failed")
    return r.value


def version() -> str:
    return load().fs_version().decode()
