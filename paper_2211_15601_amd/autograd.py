"""torch.autograd hook over the C-ABI calls: forward = fs_precompute + fs_solve, backward = fs_grad.

This is the seam through which a skinning-weight model trained by distillation (paper, Sec. 3.2
"Distilling Smooth Skinning Fields": an MLP evaluated on the grid nodes gives the weight grid each
iteration) would receive its gradient: `dL/dW` flows on into whatever produced `W`.  Only argument
marshalling happens here; all arithmetic runs in the HIP kernels.
"""
from __future__ import annotations

import torch

from . import binding


class CorrespondenceSearch(torch.autograd.Function):
    """roots, conv = CorrespondenceSearch.apply(ctx_handle, W, B, xq, pose)

    W [nx,ny,nz,n_b], B [P,n_b,12], xq [3,N] float32 CUDA tensors; pose [N] int32 or None.
    Returns xc [K,3,N] and conv [K,N] (uint8, not differentiable).  Gradients are returned for
    W, B and xq; lanes that did not converge receive none (Eq. (11)/(12), Eq. (15))."""

    @staticmethod
    def forward(ctx, fs: binding.Context, W, B, xq, pose):
        N, K = xq.shape[1], fs.K
        xc = torch.empty((K, 3, N), dtype=torch.float32, device=xq.device)
        conv = torch.empty((K, N), dtype=torch.uint8, device=xq.device)
        Jinv = torch.empty((K, 9, N), dtype=torch.float32, device=xq.device)
        W, B, xq = W.contiguous(), B.contiguous(), xq.contiguous()
        fs.precompute(W, B)
        slot = torch.empty((K, N), dtype=torch.int32, device=xq.device)
        fs.solve(xq, pose, N, K, None, None, None, xc, conv, Jinv, None, slot)
        ctx.fs = fs
        ctx.slot, ctx.serial, ctx.pre_serial = slot, fs.solve_serial, fs.pre_serial
        ctx.pose = pose
        ctx.save_for_backward(W, B, xc, Jinv, conv)
        ctx.shapes = (W.shape, B.shape)
        ctx.mark_non_differentiable(conv)
        return xc, conv

    @staticmethod
    def backward(ctx, g_xc, _g_conv):
        W, B, xc, Jinv, conv = ctx.saved_tensors
        fs = ctx.fs
        # fs_grad multiplies by the bone transforms (and, in exact-J mode, reads the transform grid) of the last
        # fs_precompute on the context: if another forward has replaced them since, put this one's back
        if fs.pre_serial != ctx.pre_serial:
            fs.precompute(W, B)
            ctx.pre_serial = fs.pre_serial
        K, _, N = xc.shape
        gW = torch.empty(ctx.shapes[0], dtype=torch.float32, device=xc.device)
        gB = torch.empty(ctx.shapes[1], dtype=torch.float32, device=xc.device)
        gxq = torch.empty((3, N), dtype=torch.float32, device=xc.device)
        # the solve's per-cell bookkeeping is reusable only while no other solve ran on the context
        slot = ctx.slot if (N > 0 and fs.solve_serial == ctx.serial) else None
        fs.grad(W, xc, Jinv, conv, g_xc.contiguous(), ctx.pose, N, K, gW, gB, gxq, slot)
        return None, gW, gB, gxq, None
