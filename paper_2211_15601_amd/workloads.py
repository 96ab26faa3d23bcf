"""Seeded synthetic workloads: human-shaped skinning scenes and query point sets.

This module only *synthesises inputs* (weight grids, bone transforms, query points,
upstream gradients).  It holds none of the solver's arithmetic: no tri-linear
lookup, no root finding, no gradients.  Both the CPU oracle's tests and the HIP
path's tests / benchmark draw their inputs from here, so that the two are compared
on identical bytes.

The scenes stand in for the paper's SMPL-posed humans (Sec. 4.1 "Dataset": per-frame
point sets, half uniform in space and half near the surface; 200k-point batches in
Sec. 3), which are not available offline.  Shapes follow the paper: 24 bones, a
64x64x16 weight grid over a box that is flat along z (Sec. 3.1 "Voxel-based
Skinning Field").

Query points of the "forward-skinned" kind are produced the way a posed scan would
be: a canonical sample is moved by linear blend skinning (Eq. 2 / Eq. 3) using the
*continuous* weight function the grid was sampled from, in float64 numpy.  They are
therefore close to, but not exactly on, the image of the gridded field.
"""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

N_BONES = 24
BOX_LO = np.array([-1.0, -1.0, -0.25], dtype=np.float32)
BOX_HI = np.array([1.0, 1.0, 0.25], dtype=np.float32)
WEIGHT_SIGMA2 = 0.02  # w_b(x) ~ exp(-dist^2 / 0.02)

INIT_BONE = 0
INIT_VOXEL = 1


@dataclasses.dataclass
class Workload:
    name: str
    dims: tuple            # (nx, ny, nz)
    n_bones: int
    n_poses: int
    lo: np.ndarray         # [3] float32
    hi: np.ndarray         # [3] float32
    W: np.ndarray          # [nx, ny, nz, n_bones] float32
    B: np.ndarray          # [P, n_bones, 12] float32, row-major 3x4
    xq: np.ndarray         # [3, N] float32 (SoA)
    pose: np.ndarray       # [N] int32
    x_src: np.ndarray      # [3, N] float32 canonical source, NaN where none
    tol: float
    div_thresh: float
    max_iters: int
    init_mode: int
    K: int
    corr_dims: tuple       # (cx, cy, cz, ck)
    gxc_seed: Optional[int] = None   # seed of the upstream gradients (training config)
    seg_a: Optional[np.ndarray] = None
    seg_b: Optional[np.ndarray] = None

    @property
    def N(self) -> int:
        return int(self.xq.shape[1])

    def upstream_grads(self) -> np.ndarray:
        """[K, 3, N] float32 ~ N(0, 1)."""
        rng = np.random.default_rng(self.gxc_seed if self.gxc_seed is not None else 77)
        return rng.standard_normal((self.K, 3, self.N), dtype=np.float32)


# ----------------------------------------------------------------------------- geometry

def _rot(axis: np.ndarray, angle: float) -> np.ndarray:
    """Rodrigues rotation matrix (float64)."""
    a = axis / np.linalg.norm(axis)
    Kx = np.array([[0, -a[2], a[1]], [a[2], 0, -a[0]], [-a[1], a[0], 0]])
    return np.eye(3) + np.sin(angle) * Kx + (1 - np.cos(angle)) * (Kx @ Kx)


def _rand_axis(rng) -> np.ndarray:
    v = rng.standard_normal(3)
    return v / np.linalg.norm(v)


def random_segments(rng, n=N_BONES):
    """n random bone segments inside the canonical box."""
    lo, hi = BOX_LO.astype(np.float64) * 0.9, BOX_HI.astype(np.float64) * 0.9
    a = rng.uniform(lo, hi, size=(n, 3))
    d = rng.standard_normal((n, 3))
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    d[:, 2] *= 0.3
    b = np.clip(a + d * rng.uniform(0.1, 0.4, size=(n, 1)), lo, hi)
    return a, b


def human_skeleton(rng):
    """A procedural 24-bone skeleton (not SMPL's): root, spine/head, two arms, two legs.

    Returns (seg_a, seg_b, parent): proximal joint, distal end, parent index (-1 root).
    """
    j = lambda s=0.1: 1.0 + rng.uniform(-s, s)
    zj = lambda: rng.uniform(-0.02, 0.02)
    a = np.zeros((N_BONES, 3))
    b = np.zeros((N_BONES, 3))
    parent = np.full(N_BONES, -1, dtype=np.int64)
    a[0] = (0.0, -0.05, 0.0)
    b[0] = (0.0, 0.05, 0.0)
    # spine + head, bones 1..5, up +y
    cur = b[0].copy()
    for i in range(1, 6):
        a[i] = cur
        cur = cur + np.array([0.0, 0.15 * j(), zj()])
        b[i] = cur
        parent[i] = i - 1
    shoulder = b[3].copy()
    # arms: 6..10 along +x, 11..15 along -x, both hanging off bone 3
    for first, sgn in ((6, 1.0), (11, -1.0)):
        cur = shoulder.copy()
        for i in range(first, first + 5):
            a[i] = cur
            cur = cur + np.array([sgn * 0.16 * j(), -0.01 * j(), zj()])
            b[i] = cur
            parent[i] = i - 1 if i > first else 3
    # legs: 16..20 (five bones) and 21..23 (three bones), from the root, down -y
    for first, cnt, x0, ln in ((16, 5, 0.12, 0.16), (21, 3, -0.12, 0.27)):
        cur = np.array([x0, -0.05, 0.0])
        for i in range(first, first + cnt):
            a[i] = cur
            cur = cur + np.array([0.01 * (j() - 1.0), -ln * j(), zj()])
            b[i] = cur
            parent[i] = i - 1 if i > first else 0
    lo, hi = BOX_LO.astype(np.float64) * 0.97, BOX_HI.astype(np.float64) * 0.97
    return np.clip(a, lo, hi), np.clip(b, lo, hi), parent


def independent_bone_transforms(rng, n=N_BONES, max_deg=30.0, max_t=0.1) -> np.ndarray:
    """[n, 12] float64: random rotation (axis uniform, angle U[0,max_deg]) + translation."""
    out = np.zeros((n, 12))
    for i in range(n):
        R = _rot(_rand_axis(rng), np.deg2rad(rng.uniform(0.0, max_deg)))
        t = rng.uniform(-max_t, max_t, size=3)
        out[i] = np.concatenate([R, t[:, None]], axis=1).reshape(12)
    return out


def chain_bone_transforms(rng, seg_a, parent, max_deg=45.0) -> np.ndarray:
    """[n, 12] float64 world transforms: local rotation about each bone's proximal joint,
    composed along the kinematic tree.  The rest pose is the canonical pose, so the
    world transform of a bone is directly its skinning transform."""
    n = len(parent)
    G = np.zeros((n, 4, 4))
    for i in range(n):
        R = _rot(_rand_axis(rng), np.deg2rad(rng.uniform(0.0, max_deg)))
        L = np.eye(4)
        L[:3, :3] = R
        L[:3, 3] = seg_a[i] - R @ seg_a[i]
        G[i] = L if parent[i] < 0 else G[parent[i]] @ L
    return G[:, :3, :].reshape(n, 12)


def seg_dist2(x: np.ndarray, a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Squared distance from points x [M,3] to segments (a[n,3], b[n,3]) -> [M,n]."""
    ab = b - a
    L2 = np.maximum((ab * ab).sum(1), 1e-12)
    ap = x[:, None, :] - a[None]
    t = np.clip((ap * ab[None]).sum(2) / L2[None], 0.0, 1.0)
    d = ap - t[..., None] * ab[None]
    return (d * d).sum(2)


def skin_weights(x: np.ndarray, a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Continuous weight field: normalised exp(-dist^2/0.02), float64, [M, n]."""
    d2 = seg_dist2(x, a, b)
    z = -(d2 - d2.min(axis=1, keepdims=True)) / WEIGHT_SIGMA2
    w = np.exp(z)
    return w / w.sum(axis=1, keepdims=True)


def grid_nodes(dims, lo=BOX_LO, hi=BOX_HI) -> np.ndarray:
    """Node positions [nx*ny*nz, 3] float64, z fastest; nodes sit on the box faces."""
    ax = [np.linspace(float(lo[i]), float(hi[i]), dims[i]) for i in range(3)]
    X, Y, Z = np.meshgrid(*ax, indexing="ij")
    return np.stack([X, Y, Z], -1).reshape(-1, 3)


def weight_grid(dims, a, b, chunk=65536) -> np.ndarray:
    nodes = grid_nodes(dims)
    out = np.empty((nodes.shape[0], a.shape[0]), dtype=np.float32)
    for s in range(0, nodes.shape[0], chunk):
        out[s:s + chunk] = skin_weights(nodes[s:s + chunk], a, b).astype(np.float32)
    return out.reshape(dims[0], dims[1], dims[2], a.shape[0])


def pose_points(x: np.ndarray, a, b, B12: np.ndarray, chunk=131072) -> np.ndarray:
    """Move canonical points x [M,3] with linear blend skinning under the continuous
    weight field (stand-in for posing a scan). float64."""
    out = np.empty_like(x)
    Bm = B12.reshape(-1, 3, 4)
    for s in range(0, x.shape[0], chunk):
        xs = x[s:s + chunk]
        w = skin_weights(xs, a, b)                       # [m, n]
        T = np.einsum("mn,nrc->mrc", w, Bm)               # [m, 3, 4]
        out[s:s + chunk] = np.einsum("mrc,mc->mr", T[:, :, :3], xs) + T[:, :, 3]
    return out


def deformed_bbox(dims, W, B12):
    """Bounding box of the grid nodes moved by their own blended transform."""
    nodes = grid_nodes(dims)
    Wm = W.reshape(-1, W.shape[-1]).astype(np.float64)
    T = (Wm @ B12.astype(np.float64)).reshape(-1, 3, 4)
    y = np.einsum("vrc,vc->vr", T[:, :, :3], nodes) + T[:, :, 3]
    return y.min(0), y.max(0)


def _ray_points(rng, n_rays, n_samples, blo, bhi) -> np.ndarray:
    """n_rays x n_samples points, equally spaced between a ray's entry into and exit
    from the box [blo, bhi]; ray-major order. Returns [n_rays*n_samples, 3]."""
    ctr = 0.5 * (blo + bhi)
    rad = 0.75 * np.linalg.norm(bhi - blo)
    d = rng.standard_normal((n_rays, 3))
    d /= np.linalg.norm(d, axis=1, keepdims=True)
    org = ctr + rad * d
    tgt = rng.uniform(blo, bhi, size=(n_rays, 3))
    dirv = tgt - org
    dirv /= np.linalg.norm(dirv, axis=1, keepdims=True)
    with np.errstate(divide="ignore", invalid="ignore"):
        inv = 1.0 / dirv
        t0 = (blo - org) * inv
        t1 = (bhi - org) * inv
    tn = np.nanmax(np.minimum(t0, t1), axis=1)
    tf = np.nanmin(np.maximum(t0, t1), axis=1)
    tf = np.maximum(tf, tn)
    s = (np.arange(n_samples) + 0.5) / n_samples
    t = tn[:, None] + (tf - tn)[:, None] * s[None]
    pts = org[:, None, :] + t[..., None] * dirv[:, None, :]
    return pts.reshape(-1, 3)


def _mixed_points(rng, n, a, b, B12, blo, bhi, frac_skinned):
    n_sk = int(round(n * frac_skinned))
    xs = rng.uniform(BOX_LO.astype(np.float64), BOX_HI.astype(np.float64), size=(n_sk, 3))
    xp = pose_points(xs, a, b, B12)
    xu = rng.uniform(blo, bhi, size=(n - n_sk, 3))
    pts = np.concatenate([xp, xu], 0)
    src = np.concatenate([xs, np.full((n - n_sk, 3), np.nan)], 0)
    perm = rng.permutation(n)
    return pts[perm], src[perm]


# ----------------------------------------------------------------------------- configs

CONFIG_SEEDS = {1: 1001, 2: 1002, 3: 1003, 4: 1004, 5: 1005}
CONFIG_NAMES = {1: "tiny", 2: "smpl_scale", 3: "ray_batch", 4: "training", 5: "multi_pose"}


def make_config(cfg: int, n_points: Optional[int] = None, dims: Optional[tuple] = None,
                seed: Optional[int] = None, n_poses: Optional[int] = None) -> Workload:
    """Build one of the five benchmark configurations.

    n_points / dims / n_poses shrink a configuration for parity tests; the recipe
    (skeleton, pose distribution, point mix) is unchanged.
    """
    if cfg not in CONFIG_SEEDS:
        raise ValueError(f"unknown config {cfg}")
    rng = np.random.default_rng(CONFIG_SEEDS[cfg] if seed is None else seed)
    tol, div = 1e-5, 10.0
    corr = (32, 32, 8, 3)
    if cfg == 1:
        dims = dims or (16, 16, 4)
        N = n_points or 4096
        a, b = random_segments(rng)
        W = weight_grid(dims, a, b)
        B = independent_bone_transforms(rng)[None]
        xs = rng.uniform(BOX_LO.astype(np.float64), BOX_HI.astype(np.float64), size=(N, 3))
        pts, src = pose_points(xs, a, b, B[0]), xs
        pose = np.zeros(N, dtype=np.int32)
        max_iters, mode, K = 50, INIT_BONE, N_BONES
    elif cfg == 2:
        dims = dims or (64, 64, 16)
        N = n_points or 65536
        a, b, parent = human_skeleton(rng)
        W = weight_grid(dims, a, b)
        B = chain_bone_transforms(rng, a, parent, 45.0)[None]
        blo, bhi = deformed_bbox(dims, W, B[0])
        pts, src = _mixed_points(rng, N, a, b, B[0], blo, bhi, 0.5)
        pose = np.zeros(N, dtype=np.int32)
        max_iters, mode, K = 50, INIT_BONE, N_BONES
    elif cfg in (3, 4):
        dims = dims or (64, 64, 16)
        n_samples = 256
        N = n_points or (1048576 if cfg == 3 else 2097152)
        n_rays = max(1, N // n_samples)
        if n_rays * n_samples != N:
            n_samples = N // n_rays
            N = n_rays * n_samples
        a, b, parent = human_skeleton(rng)
        W = weight_grid(dims, a, b)
        B = chain_bone_transforms(rng, a, parent, 45.0)[None]
        blo, bhi = deformed_bbox(dims, W, B[0])
        pts = _ray_points(rng, n_rays, n_samples, blo, bhi)
        src = np.full_like(pts, np.nan)
        pose = np.zeros(N, dtype=np.int32)
        max_iters, mode, K = 30, INIT_VOXEL, 3
    else:
        dims = dims or (128, 128, 32)
        P = n_poses or 8
        per = (n_points or 524288 * P) // P
        N = per * P
        a, b, parent = human_skeleton(rng)
        W = weight_grid(dims, a, b)
        B = np.stack([chain_bone_transforms(rng, a, parent, 60.0) for _ in range(P)])
        pts_l, src_l, pose_l = [], [], []
        for p in range(P):
            blo, bhi = deformed_bbox(dims, W, B[p])
            pp, ss = _mixed_points(rng, per, a, b, B[p], blo, bhi, 0.5)
            pts_l.append(pp)
            src_l.append(ss)
            pose_l.append(np.full(per, p, dtype=np.int32))
        pts, src, pose = np.concatenate(pts_l), np.concatenate(src_l), np.concatenate(pose_l)
        max_iters, mode, K = 50, INIT_VOXEL, 3
    return Workload(
        name=CONFIG_NAMES[cfg], dims=tuple(dims), n_bones=N_BONES, n_poses=B.shape[0],
        lo=BOX_LO.copy(), hi=BOX_HI.copy(), W=np.ascontiguousarray(W, dtype=np.float32),
        B=np.ascontiguousarray(B, dtype=np.float32),
        xq=np.ascontiguousarray(pts.T, dtype=np.float32), pose=pose,
        x_src=np.ascontiguousarray(src.T, dtype=np.float32),
        tol=tol, div_thresh=div, max_iters=max_iters, init_mode=mode, K=K, corr_dims=corr,
        gxc_seed=(CONFIG_SEEDS[cfg] + 5000) if cfg == 4 else None, seg_a=a, seg_b=b)


def random_affine_scene(seed: int, dims=(6, 5, 4), n_bones=4, n_poses=1, n_points=64,
                        max_deg=25.0, lo=(-1.0, -0.8, -0.5), hi=(1.0, 0.9, 0.6)):
    """A small generic scene for unit tests: random convex weights, random rigid bones,
    uniform points in a slightly enlarged box.  Returns a dict of float32/float64 arrays."""
    rng = np.random.default_rng(seed)
    lo = np.asarray(lo, dtype=np.float32)
    hi = np.asarray(hi, dtype=np.float32)
    W = rng.uniform(0.05, 1.0, size=(*dims, n_bones))
    W /= W.sum(-1, keepdims=True)
    B = np.stack([independent_bone_transforms(rng, n_bones, max_deg, 0.15) for _ in range(n_poses)])
    ext = 0.1 * (hi - lo).astype(np.float64)
    x = rng.uniform(lo.astype(np.float64) - ext, hi.astype(np.float64) + ext, size=(n_points, 3))
    pose = rng.integers(0, n_poses, size=n_points).astype(np.int32)
    return dict(dims=tuple(dims), n_bones=n_bones, n_poses=n_poses, lo=lo, hi=hi,
                W=W.astype(np.float32), B=B.astype(np.float32),
                x=np.ascontiguousarray(x.T.astype(np.float32)), pose=pose)
