"""Pins for the oracle's duplicate removal (Sec. 3.1 "Remove Duplicate Correspondences"): the greedy
rule re-derived in plain numpy, and the properties it must have."""
import numpy as np

import oracle
from paper_2211_15601_amd import workloads as wl


def _greedy(xc, conv, md):
    K, _, N = xc.shape
    keep = np.zeros((K, N), np.uint8)
    for i in range(N):
        kept = []
        for k in range(K):
            if conv[k, i] and all(np.linalg.norm(xc[k, :, i] - xc[j, :, i]) >= md for j in kept):
                kept.append(k)
                keep[k, i] = 1
    return keep


def test_dedupe_matches_numpy_greedy_and_properties():
    w = wl.make_config(1, n_points=300, dims=(16, 16, 4))
    T = oracle.precompute(w.dims, w.W, w.B, prec="f64")
    x0, J0, v0 = oracle.init_bone(w.dims, w.lo, w.hi, T, w.B, w.xq, prec="f64")
    xc, cv, _, _ = oracle.solve(w.dims, w.lo, w.hi, T, w.xq, x0, J0, v0, prec="f64")
    md = 1e-3
    keep, count = oracle.dedupe(xc, cv, md, prec="f64")
    np.testing.assert_array_equal(keep, _greedy(xc, cv, float(np.float32(md))))
    np.testing.assert_array_equal(count, keep.sum(0))
    assert (keep <= cv).all()                         # only converged lanes survive
    assert (count[cv.any(0)] >= 1).all()              # a point with a root keeps at least one
    assert count.mean() < 0.5 * cv.sum(0).mean()      # most of the 24 lanes are duplicates
    for i in range(300):
        ks = np.nonzero(keep[:, i])[0]
        for a in range(len(ks)):                      # kept roots are pairwise at least min_dist apart
            for b in range(a):
                assert np.linalg.norm(xc[ks[a], :, i] - xc[ks[b], :, i]) >= md * (1 - 1e-9)
        for k in np.nonzero(cv[:, i])[0]:             # every converged lane is represented by an earlier or equal kept lane
            assert any(kk <= k and np.linalg.norm(xc[k, :, i] - xc[kk, :, i]) < md for kk in ks)


def test_dedupe_two_distinct_roots_survive():
    # the quadratic of the 2x2x2 closed form has two roots 0.64 apart: both are kept, copies are not
    xc = np.zeros((4, 3, 1))
    xc[0, 0, 0], xc[1, 0, 0], xc[2, 0, 0], xc[3, 0, 0] = 0.2298, 0.8702, 0.2298 + 1e-5, 0.8702 - 1e-5
    cv = np.ones((4, 1), np.uint8)
    keep, count = oracle.dedupe(xc, cv, 1e-3, prec="f64")
    assert keep[:, 0].tolist() == [1, 1, 0, 0] and count[0] == 2
    cv[0, 0] = 0                                      # an unconverged lane never represents anyone
    keep, count = oracle.dedupe(xc, cv, 1e-3, prec="f64")
    assert keep[:, 0].tolist() == [0, 1, 1, 0] and count[0] == 2
