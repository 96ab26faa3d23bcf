"""The C-ABI library loads without a GPU and exports every symbol the header declares;
argument checks that need no device answer with the documented status codes."""
import ctypes
import os
import re

import pytest

from paper_2211_15601_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(headers=None):
    """Every function the headers under include/ declare."""
    inc = os.path.join(ROOT, "include")
    names = set()
    for h in headers or sorted(f for f in os.listdir(inc) if f.endswith(".h")):
        text = open(os.path.join(inc, h)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(fs_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_header_declares_the_four_calls():
    names = _declared(["fastsnarf.h"])
    # measurement support is declared apart from the articulation path
    assert not {"fs_microbench", "fs_set_timing", "fs_get_timing"} & set(names)
    for n in ("fs_precompute", "fs_init", "fs_solve", "fs_grad", "fs_create", "fs_destroy"):
        assert n in names


def test_library_exports_every_declared_symbol():
    L = binding.load()
    for n in _declared():
        assert hasattr(L, n), n
    assert sorted(binding.EXPORTS) == _declared()
    assert b"gfx950" in L.fs_version()


def test_struct_layouts_match_header():
    assert ctypes.sizeof(binding.GridDesc) == 5 * 4 + 6 * 4
    assert ctypes.sizeof(binding.Params) == 9 * 4


def _create(desc, prm):
    L = binding.load()
    h = ctypes.c_void_p()
    st = L.fs_create(ctypes.byref(desc), ctypes.byref(prm), None, ctypes.byref(h))
    if st == binding.FS_OK:
        L.fs_destroy(h)
    return st, h


def _good():
    d = binding.GridDesc(8, 8, 4, 24, 1, (ctypes.c_float * 3)(-1, -1, -0.25), (ctypes.c_float * 3)(1, 1, 0.25))
    p = binding.Params(1e-5, 10.0, 50, 0, 0, 32, 32, 8, 3)
    return d, p


def test_create_rejects_bad_shapes_before_touching_the_device():
    L = binding.load()
    d, p = _good()
    h = ctypes.c_void_p()
    assert L.fs_create(None, ctypes.byref(p), None, ctypes.byref(h)) == binding.FS_E_ARG
    assert L.fs_create(ctypes.byref(d), ctypes.byref(p), None, None) == binding.FS_E_ARG
    d.nx = 1
    assert _create(d, p)[0] == binding.FS_E_SHAPE
    d, p = _good(); d.n_bones = 65
    assert _create(d, p)[0] == binding.FS_E_SHAPE
    d, p = _good(); d.n_poses = 0
    assert _create(d, p)[0] == binding.FS_E_SHAPE
    d, p = _good(); d.hi[1] = -1.0
    assert _create(d, p)[0] == binding.FS_E_ARG
    d, p = _good(); p.tol = 0.0
    assert _create(d, p)[0] == binding.FS_E_ARG
    d, p = _good(); p.max_iters = 256
    assert _create(d, p)[0] == binding.FS_E_ARG
    d, p = _good(); p.init_mode = 7
    assert _create(d, p)[0] == binding.FS_E_ARG
    d, p = _good(); p.init_mode = 1; p.corr_k = 9
    assert _create(d, p)[0] == binding.FS_E_SHAPE
    d, p = _good()
    st, h = _create(d, p)
    assert st in (binding.FS_OK, binding.FS_E_DEVICE)     # FS_E_DEVICE where there is no GPU


def test_null_context_is_an_argument_error():
    L = binding.load()
    assert L.fs_precompute(None, None, None) == binding.FS_E_ARG
    assert L.fs_solve(None, None, None, 0, 24, None, None, None, None, None, None, None, None) == binding.FS_E_ARG
    assert L.fs_grad(None, None, None, None, None, None, None, 0, 24, None, None, None, None) == binding.FS_E_ARG
    assert L.fs_destroy(None) == binding.FS_OK
    assert L.fs_last_error(None) == b"null context"


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load()
