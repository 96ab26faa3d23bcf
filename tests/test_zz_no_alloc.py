"""fs_dedupe_noalloc (the entry point for callers that cannot allocate device memory) against fs_dedupe, through the
C ABI: same keep mask, offsets, packed roots and lane ids, bit for bit, on two calls in a row, the second with a
smaller input (the scratch array keeps the first call's contents)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_15601_amd import binding, workloads as wl
import gpu_util as gu

pytestmark = pytest.mark.gpu


def _both(ctx, fn_names, xc, cv, N, K, md, cap):
    outs = []
    for name in fn_names:
        keep = torch.full((K, N), 9, dtype=torch.uint8, device=gu.DEV)
        offs = torch.full((N + 1,), -1, dtype=torch.int32, device=gu.DEV)
        roots = torch.full((cap, 3), float("nan"), dtype=torch.float32, device=gu.DEV)
        lane = torch.full((cap,), -1, dtype=torch.int32, device=gu.DEV)
        getattr(ctx, name)(xc, cv, N, K, md, keep, offs, roots, lane, cap)
        torch.cuda.synchronize()
        outs.append((keep, offs, roots, lane))
    return outs


def test_dedupe_noalloc_matches_dedupe_on_two_calls_in_a_row(gpu_lib):
    md = 1e-3
    first = wl.make_config(2, n_points=3 * 4096 + 77, dims=(32, 32, 8))        # four scan tiles, ragged
    second = wl.make_config(3, n_points=16 * 250, dims=(32, 32, 8))            # smaller: one tile, other K
    ctx = None
    for w in (first, second):
        T_ref = oracle.precompute(w.dims, w.W, w.B, prec="f32")
        x0, J0, v0 = gu.oracle_inits(w, T_ref)
        xc_h, cv_h, _, _ = gu.oracle_solve(w, T_ref, x0, J0, v0)
        if ctx is None:
            ctx = gu.GpuRun(w).ctx           # dedupe uses the context for its stream only: one context serves both calls
        N, K = w.N, w.K
        xc, cv = gu.dev(xc_h), gu.dev(cv_h)
        cap = N * K
        (k0, o0, r0, l0), (k1, o1, r1, l1) = _both(ctx, ("dedupe", "dedupe_noalloc"), xc, cv, N, K, md, cap)
        total = int(o0[-1].item())
        assert 0 < total < int(cv_h.sum())
        assert torch.equal(k0, k1) and torch.equal(o0, o1) and torch.equal(l0, l1)
        assert torch.equal(r0[:total].view(torch.int32), r1[:total].view(torch.int32))
        # and both equal the oracle's keep mask
        keep_ref, count_ref = oracle.dedupe(xc_h, cv_h, md, prec="f32")
        np.testing.assert_array_equal(k1.cpu().numpy(), keep_ref)
        np.testing.assert_array_equal(o1.cpu().numpy(), np.concatenate([[0], np.cumsum(count_ref)]).astype(np.int32))
    # empty input and the size limit
    offs = torch.full((1,), -1, dtype=torch.int32, device=gu.DEV)
    ctx.dedupe_noalloc(None, None, 0, 3, md, None, offs, None, None, 0)
    torch.cuda.synchronize()
    assert offs.item() == 0
    big = (1 << 24) + 1
    st = ctx.dedupe_noalloc(xc, cv, big, 1, md, k1, o1, None, None, 0, check=False)
    assert st == binding.FS_E_SHAPE and "scratch" in ctx.last_error()
