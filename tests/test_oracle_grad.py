"""Pins for the oracle's implicit-differentiation backward (Eq. (11)/(12), Eq. (15)).

Truth comes from outside the oracle: roots are re-found by an independent float64 Newton
(torch.grid_sample forward + autograd Jacobian) under perturbed parameters and differenced;
an unrolled differentiable Newton gives the same derivative through torch.autograd; one-hot
weights give a closed form."""
import numpy as np
import torch

import oracle
from paper_2211_15601_amd import workloads as wl
from helpers import ref_forward, ref_forward_lerp


def _newton_torch(dims, lo, hi, W, B, xq, x_start, steps=8, create_graph=False, fwd=None):
    """Independent Newton solve of d(x) - x' = 0 for a batch of lanes; W [V,nb], B [nb,12]
    torch float64 (may require grad), xq / x_start [3,n]."""
    T1 = W @ B
    x = x_start
    for _ in range(steps):
        if not x.requires_grad:
            x = x.clone().requires_grad_(True)
        g = (fwd(dims, lo, hi, T1, x) if fwd else ref_forward(dims, lo, hi, T1, x, T_is_tensor=True)) - xq
        cols = [torch.autograd.grad(g[r].sum(), x, create_graph=create_graph, retain_graph=True)[0]
                for r in range(3)]                       # cols[r][j] = dg_r/dx_j  [3,n]
        J = torch.stack(cols, 0).permute(2, 0, 1)        # [n,3,3]
        if not create_graph:
            J, g = J.detach(), g.detach()
        step = torch.linalg.solve(J, g.T[..., None])[..., 0].T
        x = (x if create_graph else x.detach()) - step
    return x


def _setup(seed=71, n=10, dims=(5, 4, 3), nb=3):
    s = wl.random_affine_scene(seed, dims=dims, n_bones=nb, n_points=n, max_deg=35.0)
    lo, hi = s["lo"].astype(np.float64), s["hi"].astype(np.float64)
    rng = np.random.default_rng(seed)
    xs = rng.uniform(lo + 0.1 * (hi - lo), hi - 0.1 * (hi - lo), size=(n, 3)).T
    W = s["W"].astype(np.float64)
    B = s["B"].astype(np.float64)
    T = oracle.precompute(dims, W, B, prec="f64")
    xq = ref_forward(dims, lo, hi, T[0], xs).numpy()
    x0, J0, v0 = oracle.init_bone(dims, lo, hi, T, B, xq, prec="f64")
    xc, cv, Jo, it = oracle.solve(dims, lo, hi, T, xq, x0, J0, v0, prec="f64", tol=1e-10, max_iters=80)
    gx = rng.standard_normal(xc.shape)
    return dict(dims=dims, lo=lo, hi=hi, W=W, B=B, T=T, xq=xq, xc=xc, cv=cv, Jo=Jo, it=it, gx=gx, nb=nb)


def _loss_at(c, W, B, xq):
    """L = sum over converged lanes of g_x . x*(theta), roots re-found by the torch Newton."""
    Wt = torch.as_tensor(W.reshape(-1, c["nb"]))
    Bt = torch.as_tensor(B[0])
    tot = 0.0
    for k in range(c["xc"].shape[0]):
        m = c["cv"][k] == 1
        if not m.any():
            continue
        xr = _newton_torch(c["dims"], c["lo"], c["hi"], Wt, Bt, torch.as_tensor(xq[:, m]),
                           torch.as_tensor(c["xc"][k][:, m]), steps=6)
        tot += float((torch.as_tensor(c["gx"][k][:, m]) * xr.detach()).sum())
    return tot


def test_exact_gradient_matches_finite_differences_of_the_root():
    c = _setup()
    assert c["cv"].mean() > 0.5
    gW, gB, gxq = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"],
                              c["cv"], c["gx"], mode=1, prec="f64")
    rng = np.random.default_rng(1)
    eps = 1e-6
    for trial in range(4):
        dW = rng.standard_normal(c["W"].shape)
        dB = rng.standard_normal(c["B"].shape)
        dq = rng.standard_normal(c["xq"].shape)
        for (aW, aB, aq) in ((1, 0, 0), (0, 1, 0), (0, 0, 1), (1, 1, 1)):
            Lp = _loss_at(c, c["W"] + eps * aW * dW, c["B"] + eps * aB * dB, c["xq"] + eps * aq * dq)
            Lm = _loss_at(c, c["W"] - eps * aW * dW, c["B"] - eps * aB * dB, c["xq"] - eps * aq * dq)
            fd = (Lp - Lm) / (2 * eps)
            an = aW * (gW * dW).sum() + aB * (gB * dB).sum() + aq * (gxq * dq).sum()
            assert abs(fd - an) <= 2e-6 * max(1.0, abs(fd)), (trial, aW, aB, aq, fd, an)


def test_exact_gradient_matches_autograd_through_unrolled_newton():
    c = _setup(seed=72, n=8)
    gW, gB, gxq = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"],
                              c["cv"], c["gx"], mode=1, prec="f64")
    Wt = torch.tensor(c["W"].reshape(-1, c["nb"]), requires_grad=True)
    Bt = torch.tensor(c["B"][0], requires_grad=True)
    qt = torch.tensor(c["xq"], requires_grad=True)
    L = 0.0
    rng = np.random.default_rng(2)
    for k in range(c["xc"].shape[0]):
        m = c["cv"][k] == 1
        if not m.any():
            continue
        start = torch.as_tensor(c["xc"][k][:, m] + 1e-3 * rng.standard_normal((3, int(m.sum()))))
        xr = _newton_torch(c["dims"], c["lo"], c["hi"], Wt, Bt, qt[:, torch.as_tensor(m)], start,
                           steps=6, create_graph=True, fwd=ref_forward_lerp)
        L = L + (torch.as_tensor(c["gx"][k][:, m]) * xr).sum()
    aW, aB, aq = torch.autograd.grad(L, [Wt, Bt, qt])
    np.testing.assert_allclose(gW.reshape(-1, c["nb"]), aW.numpy(), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(gB[0], aB.numpy(), rtol=1e-6, atol=1e-8)
    np.testing.assert_allclose(gxq, aq.numpy(), rtol=1e-6, atol=1e-8)


def test_one_hot_closed_form_both_modes():
    # one-hot weights on bone k: x* = R^{-1}(x' - t); dx* = -R^{-1}(dR x* + dt)
    #  => dL/dR[r][j] = lam_r x*_j, dL/dt_r = lam_r with lam = -R^{-T} g_x; other bones get 0;
    # Broyden's J~ equals R^{-1} here, so both modes must give this.
    s = wl.random_affine_scene(73, dims=(4, 4, 3), n_bones=3, n_points=30)
    k = 1
    W = np.zeros(s["W"].shape); W[..., k] = 1.0
    B = s["B"].astype(np.float64)
    lo, hi = s["lo"], s["hi"]
    T = oracle.precompute(s["dims"], W, B, prec="f64")
    xq = s["x"].astype(np.float64)
    x0, J0, v0 = oracle.init_bone(s["dims"], lo, hi, T, B, xq, prec="f64")
    xc, cv, Jo, it = oracle.solve(s["dims"], lo, hi, T, xq, x0, J0, v0, prec="f64", tol=1e-10)
    assert cv.all()
    rng = np.random.default_rng(4)
    gx = rng.standard_normal(xc.shape)
    R = B[0, k].reshape(3, 4)[:, :3]
    ref = np.zeros((3, 4))
    ref_q = np.zeros_like(xq)
    for kk in range(3):
        lam = -np.linalg.inv(R).T @ gx[kk]                       # [3,n]
        ref[:, :3] += lam @ xc[kk].T
        ref[:, 3] += lam.sum(1)
        ref_q -= lam
    for mode in (0, 1):
        gW, gB, gxq, GT = oracle.grad(s["dims"], lo, hi, T, W, B, xc, Jo, cv, gx, mode=mode, prec="f64",
                                      want_GT=True)
        np.testing.assert_allclose(gB[0, k].reshape(3, 4), ref, rtol=1e-7, atol=1e-7)
        assert np.abs(gB[0, [0, 2]]).max() == 0.0
        np.testing.assert_allclose(gxq, ref_q, rtol=1e-7, atol=1e-7)
        np.testing.assert_allclose(GT[0].sum(0).reshape(3, 4), ref, rtol=1e-7, atol=1e-7)
        np.testing.assert_allclose(gW.reshape(-1, 3), GT[0] @ B[0].T, rtol=1e-10, atol=1e-10)


def test_unconverged_lanes_contribute_nothing():
    c = _setup(seed=74)
    cv = c["cv"].copy()
    base = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"], cv, c["gx"], mode=0)
    gx2 = c["gx"].copy()
    cv[0, :] = 0
    gx2[0] = 1e6                                 # garbage on masked lanes must not leak
    a = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"], cv, gx2, mode=0)
    gx3 = c["gx"].copy(); gx3[0] = 0.0
    b = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"], c["cv"], gx3, mode=0)
    for u, v in zip(a, b):
        np.testing.assert_allclose(u, v, atol=1e-12)
    assert np.abs(base[0] - a[0]).max() > 0


def test_broyden_gradient_gap_is_reported_and_sane():
    # Sec. 3.2 "Approximated Gradient": no error bound is given, so this only guards against
    # gross mistakes (sign, transpose) and prints the gap.  PARITY UNPINNED against truth.
    w = wl.make_config(1, n_points=256, dims=(16, 16, 4))
    T = oracle.precompute(w.dims, w.W, w.B, prec="f64")
    x0, J0, v0 = oracle.init_bone(w.dims, w.lo, w.hi, T, w.B, w.xq, prec="f64")
    xc, cv, Jo, it = oracle.solve(w.dims, w.lo, w.hi, T, w.xq, x0, J0, v0, prec="f64")
    gx = np.random.default_rng(9).standard_normal(xc.shape)
    a = oracle.grad(w.dims, w.lo, w.hi, T, w.W, w.B, xc, Jo, cv, gx, mode=0)
    b = oracle.grad(w.dims, w.lo, w.hi, T, w.W, w.B, xc, Jo, cv, gx, mode=1)
    for name, u, v in zip(("gW", "gB", "gxq"), a, b):
        gap = np.linalg.norm(u - v) / np.linalg.norm(v)
        cos = (u * v).sum() / (np.linalg.norm(u) * np.linalg.norm(v))
        print(f"Broyden-J vs exact-J, {name}: relative L2 gap {gap:.3e}, cosine {cos:.4f}")
        assert cos > 0.5


def test_f32_gradient_close_to_f64():
    c = _setup(seed=75, n=40)
    a = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"], c["cv"], c["gx"],
                    mode=0, prec="f64")
    b = oracle.grad(c["dims"], c["lo"], c["hi"], c["T"], c["W"], c["B"], c["xc"], c["Jo"], c["cv"], c["gx"],
                    mode=0, prec="f32")
    for u, v in zip(a, b):
        assert np.linalg.norm(u - v) <= 1e-5 * np.linalg.norm(u)
