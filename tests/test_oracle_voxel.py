"""Invariants of the oracle's voxel-based initialisation.  The paper does not define this
rule (PARITY UNPINNED by the paper); what is checked here is the rule's own statement,
re-derived by brute force in numpy float64: cell membership, nearest-to-centre first,
greedy canonical separation, at most ck candidates, and the query side."""
import numpy as np

import oracle
from paper_2211_15601_amd import workloads as wl
from helpers import ref_T


def _brute(dims, lo, hi, T1, cd):
    nodes = wl.grid_nodes(dims, lo, hi)
    Tm = T1.reshape(-1, 3, 4)
    Y = np.einsum("vrc,vc->vr", Tm[:, :, :3], nodes) + Tm[:, :, 3]
    blo, bhi = Y.min(0), Y.max(0)
    cs = (bhi - blo) / np.array(cd[:3])
    ci = np.minimum(((Y - blo) / cs).astype(np.int64), np.array(cd[:3]) - 1)
    cell = (ci[:, 0] * cd[1] + ci[:, 1]) * cd[2] + ci[:, 2]
    h = (np.asarray(hi, np.float64) - np.asarray(lo, np.float64)) / (np.array(dims) - 1)
    rs2 = 6.25 * (h ** 2).sum()
    ncell = cd[0] * cd[1] * cd[2]
    out = -np.ones((ncell, cd[3]), dtype=np.int64)
    for c in range(ncell):
        ids = np.nonzero(cell == c)[0]
        if len(ids) == 0:
            continue
        cc = np.array([c // (cd[1] * cd[2]), (c // cd[2]) % cd[1], c % cd[2]])
        ctr = blo + (cc + 0.5) * cs
        key = ((Y[ids] - ctr) ** 2).sum(1)
        acc = []
        for j in np.lexsort((ids, key)):
            v = ids[j]
            if all(((nodes[v] - nodes[a]) ** 2).sum() > rs2 for a in acc):
                acc.append(v)
                if len(acc) == cd[3]:
                    break
        out[c, :len(acc)] = acc
    return np.concatenate([blo, bhi]), out, Y, cell


def test_corr_build_matches_brute_force_rederivation():
    s = wl.random_affine_scene(81, dims=(13, 12, 9), n_bones=4, n_poses=2, max_deg=50.0)
    T = ref_T(s["dims"], s["W"], s["B"])
    cd = (3, 2, 2, 3)
    bbox, cand = oracle.corr_build(s["dims"], s["lo"], s["hi"], T, cd, prec="f64")
    assert cand.shape == (2, 12, 3)
    for p in range(2):
        bb, ref, Y, cell = _brute(s["dims"], s["lo"], s["hi"], T[p], cd)
        np.testing.assert_allclose(bbox[p], bb, atol=1e-12)
        np.testing.assert_array_equal(cand[p], ref)
        assert (cand[p] >= 0).sum() > 18          # several cells hold more than one candidate


def test_corr_candidates_obey_the_rule_on_a_human_scene():
    w = wl.make_config(3, n_points=256, dims=(16, 16, 8))
    T = oracle.precompute(w.dims, w.W, w.B, prec="f32")
    cd = (8, 8, 4, 3)
    bbox, cand = oracle.corr_build(w.dims, w.lo, w.hi, T, cd, prec="f32")
    nodes = wl.grid_nodes(w.dims, w.lo, w.hi)
    Tm = T[0].astype(np.float64).reshape(-1, 3, 4)
    Y = np.einsum("vrc,vc->vr", Tm[:, :, :3], nodes) + Tm[:, :, 3]
    np.testing.assert_allclose(bbox[0, :3], Y.min(0), atol=1e-5)
    np.testing.assert_allclose(bbox[0, 3:], Y.max(0), atol=1e-5)
    cs = (bbox[0, 3:] - bbox[0, :3]).astype(np.float64) / np.array(cd[:3])
    h = (w.hi.astype(np.float64) - w.lo) / (np.array(w.dims) - 1)
    rsep = 2.5 * np.linalg.norm(h)
    seen = 0
    for c in range(cand.shape[1]):
        ids = cand[0, c][cand[0, c] >= 0]
        # -1 entries only at the tail
        assert (cand[0, c][len(ids):] == -1).all()
        cc = np.array([c // (cd[1] * cd[2]), (c // cd[2]) % cd[1], c % cd[2]])
        ctr = bbox[0, :3] + (cc + 0.5) * cs
        for v in ids:
            # the sample's image lies in this cell (up to rounding at the faces)
            assert (np.abs(Y[v] - ctr) <= 0.5 * cs + 1e-5).all()
        for i in range(len(ids)):
            for j in range(i):
                assert np.linalg.norm(nodes[ids[i]] - nodes[ids[j]]) > rsep * (1 - 1e-6)
        key = ((Y[ids] - ctr) ** 2).sum(1)
        assert (np.diff(key) >= -1e-6).all()
        seen += len(ids)
    assert seen > 50


def test_init_voxel_uses_cell_candidates():
    w = wl.make_config(3, n_points=512, dims=(16, 16, 8))
    T = oracle.precompute(w.dims, w.W, w.B, prec="f64")
    cd = (8, 8, 4, 3)
    bbox, cand = oracle.corr_build(w.dims, w.lo, w.hi, T, cd, prec="f64")
    xq = w.xq.astype(np.float64)
    xq[:, 0] = bbox[0, 3:] + 5.0            # far outside: clamps into the last cell
    x0, J0, v0 = oracle.init_voxel(w.dims, w.lo, w.hi, T, cd, bbox, cand, xq, prec="f64")
    nodes = wl.grid_nodes(w.dims, w.lo, w.hi)
    cs = (bbox[0, 3:] - bbox[0, :3]) / np.array(cd[:3])
    ci = np.clip(np.floor((xq.T - bbox[0, :3]) / cs).astype(np.int64), 0, np.array(cd[:3]) - 1)
    cell = (ci[:, 0] * cd[1] + ci[:, 1]) * cd[2] + ci[:, 2]
    assert cell[0] == cd[0] * cd[1] * cd[2] - 1
    for k in range(3):
        ids = cand[0, cell, k]
        has = ids >= 0
        assert (v0[k][~has] == 0).all()
        np.testing.assert_allclose(x0[k][:, has], nodes[ids[has]].T, atol=1e-12)
        ok = v0[k] == 1
        _, J = oracle.forward(w.dims, w.lo, w.hi, T, x0[k][:, ok], jac=True, prec="f64")
        ref = np.linalg.inv(J.T.reshape(-1, 3, 3))
        np.testing.assert_allclose(J0[k][:, ok].T.reshape(-1, 3, 3), ref, rtol=1e-8, atol=1e-8)
    assert v0.mean() > 0.05


def test_voxel_init_recovers_sources_of_posed_points():
    # report (not a parity claim): how often the solve started from the cell candidates finds
    # the canonical source of a posed point
    w = wl.make_config(2, n_points=2048, dims=(32, 32, 8))
    T = oracle.precompute(w.dims, w.W, w.B, prec="f32")
    cd = (16, 16, 4, 3)
    bbox, cand = oracle.corr_build(w.dims, w.lo, w.hi, T, cd, prec="f32")
    x0, J0, v0 = oracle.init_voxel(w.dims, w.lo, w.hi, T, cd, bbox, cand, w.xq, prec="f32")
    xc, cv, _, it = oracle.solve(w.dims, w.lo, w.hi, T, w.xq, x0, J0, v0, prec="f32")
    src = ~np.isnan(w.x_src[0])
    d = np.abs(xc - w.x_src[None]).max(1)
    d[cv == 0] = np.inf
    rate = (d.min(0)[src] < 2e-2).mean()
    print(f"voxel-init recovery of posed sources: {rate:.3f}; mean iters {it[v0 == 1].mean():.2f}")
    assert rate > 0.5
