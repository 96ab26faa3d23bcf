"""Independent reference pieces for pinning the oracle (numpy / torch CPU, float64).

Nothing here calls the oracle or the HIP path.
"""
import numpy as np
import torch
import torch.nn.functional as F


def ref_T(dims, W, B):
    """T_v = sum_i w_{v,i} B_i as one float64 matmul per pose -> [P, V, 12]."""
    V = dims[0] * dims[1] * dims[2]
    Wm = np.asarray(W, dtype=np.float64).reshape(V, -1)
    return np.stack([Wm @ np.asarray(Bp, dtype=np.float64) for Bp in B])


def ref_interp_T(dims, lo, hi, T1, x, T_is_tensor=False):
    """Tri-linear lookup of a [V,12] grid at x [3,n] through torch.grid_sample
    (align_corners=True: nodes on the box faces; border padding: clamp to edge)."""
    Tt = T1 if T_is_tensor else torch.as_tensor(np.asarray(T1, dtype=np.float64))
    vol = Tt.reshape(dims[0], dims[1], dims[2], 12).permute(3, 0, 1, 2)[None]   # [1,12,D=nx,H=ny,W=nz]
    xt = x if torch.is_tensor(x) else torch.as_tensor(np.asarray(x, dtype=np.float64))
    lo_t = torch.as_tensor(np.asarray(lo, dtype=np.float64))
    hi_t = torch.as_tensor(np.asarray(hi, dtype=np.float64))
    c = 2.0 * (xt - lo_t[:, None]) / (hi_t - lo_t)[:, None] - 1.0               # [3,n]
    grid = torch.stack([c[2], c[1], c[0]], dim=-1)[None, None, None]            # x->W(nz) y->H z->D(nx)
    out = F.grid_sample(vol, grid, mode="bilinear", padding_mode="border", align_corners=True)
    return out[0, :, 0, 0, :]                                                   # [12, n]


def ref_forward(dims, lo, hi, T1, x, T_is_tensor=False):
    """d(x) = T(x) x with T from grid_sample; returns torch [3,n] float64."""
    xt = x if torch.is_tensor(x) else torch.as_tensor(np.asarray(x, dtype=np.float64))
    Tx = ref_interp_T(dims, lo, hi, T1, xt, T_is_tensor).reshape(3, 4, -1)
    return (Tx[:, :3, :] * xt[None]).sum(1) + Tx[:, 3, :]


def inv_rigid_apply(B12, xp):
    """B^{-1} x' for a 3x4 [R|t] given as 12 numbers, float64; xp [3,n]."""
    M = np.asarray(B12, dtype=np.float64).reshape(3, 4)
    return np.linalg.solve(M[:, :3], np.asarray(xp, dtype=np.float64) - M[:, 3:4])


def ref_forward_lerp(dims, lo, hi, T1, x):
    """d(x) = T(x) x with T from nested 1-D lerps (z, then y, then x) on gathered nodes; pure torch
    indexing ops, so it is twice differentiable (grid_sample is not).  T1 [V,12], x [3,n] tensors."""
    n = torch.tensor(dims, dtype=torch.float64)
    lo_t = torch.as_tensor(np.asarray(lo, dtype=np.float64))
    hi_t = torch.as_tensor(np.asarray(hi, dtype=np.float64))
    u = (x - lo_t[:, None]) / (hi_t - lo_t)[:, None] * (n - 1)[:, None]
    u = torch.minimum(torch.maximum(u, torch.zeros_like(u)), (n - 1)[:, None].expand_as(u))
    i0 = torch.minimum(u.detach().floor(), (n - 2)[:, None].expand_as(u)).long()
    f = u - i0
    G = T1.reshape(dims[0], dims[1], dims[2], 12)

    def node(a, b, c):
        return G[i0[0] + a, i0[1] + b, i0[2] + c]            # [n,12]

    def lerp(p, q, t):
        return p + (q - p) * t[:, None]
    c00 = lerp(node(0, 0, 0), node(0, 0, 1), f[2])
    c01 = lerp(node(0, 1, 0), node(0, 1, 1), f[2])
    c10 = lerp(node(1, 0, 0), node(1, 0, 1), f[2])
    c11 = lerp(node(1, 1, 0), node(1, 1, 1), f[2])
    Tx = lerp(lerp(c00, c01, f[1]), lerp(c10, c11, f[1]), f[0]).T.reshape(3, 4, -1)
    return (Tx[:, :3, :] * x[None]).sum(1) + Tx[:, 3, :]
