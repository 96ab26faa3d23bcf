#!/usr/bin/env python3
"""Benchmark of the Fast-SNARF articulation hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch that is already resident in
HBM: fs_precompute -> fs_solve (initial states computed inside the kernel; J~ and iteration counts
kept) -> fs_grad.  `--unfused` materialises the initial states with fs_init first.
Workload: the SMPL-scale single-pose configuration (24 bones, 64x64x16 weight grid,
65,536 query points x 24 per-bone initial states, max 50 iterations, tol 1e-5).

Prints ONE JSON line.  `value` = converged (point, init) root solves per second over the whole
step.  `roofline` describes the Broyden kernel (k_solve_ws, or k_solve when the grid fits in LDS: the dominant
one), timed by the library with
HIP events around that kernel on the stream it runs on.  `cpu_baseline` is the CPU oracle timed on
this machine's host cores.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# algorithmic fp32 operation counts of the method (one fused multiply-add = 2), from the arithmetic
# the solver is defined by: one field evaluation and residual, one Broyden update, one step
FLOP_EVAL = 237      # locate 12, corner weights 19, 8x12 tri-linear blend 180, T x 18, g 3, |g|^2 5
FLOP_UPDATE = 63     # dg 3, v = J~^T dx 15, u = dx - J~ dg 18, v.dg 5, divide 1, u/den 3, rank-one 18
FLOP_STEP = 18       # dx = -J~ g 15, x + dx 3
LOADS_EVAL = 24      # 8 corner records x 3 rows of 16 bytes
PEAK_FP32_TFLOPS = 157.3            # published fp32 vector peak (needs packed fp32 instructions)
PEAK_FP32_UNPACKED_TFLOPS = 78.6    # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz: one FMA per lane per clock
# HBM traffic of one launch of the Broyden kernel on the default workload, from rocprofv3 FETCH_SIZE / WRITE_SIZE
# (profiles/k_solve_config2_hbm_traffic.md); None for other workloads.  The second figure is the same
# kernel without the per-cell counting of converged lanes (--no-slots).
SOLVE_TRAFFIC_BYTES = {2: 274.3e6}
SOLVE_TRAFFIC_BYTES_NO_SLOTS = {2: 199.1e6}
# L1 (vector cache) accesses and L1 -> L2 read requests of one launch of the Broyden kernel on the default
# workload, from rocprofv3 TCP_TOTAL_CACHE_ACCESSES_sum / TCP_TCC_READ_REQ_sum
# (profiles/k_solve_config2_gather_path.md): the per-lane 16-byte gathers the texture path actually served,
# after the same-cell reuse and the skipping of weight-zero corners.
SOLVE_L1_ACCESSES = {2: 131.3e6}
SOLVE_L1_TO_L2_REQUESTS = {2: 26.6e6}


def resolution_sweep(torch, binding, wl, dev):
    """Articulation time (fs_precompute + fs_solve, fused initial states, roots + masks only) against the
    resolution of the weight grid, 200k points of the SMPL-scale scene."""
    for dims in ((16, 16, 4), (32, 32, 8), (64, 64, 16), (128, 128, 32)):
        w = wl.make_config(2, n_points=200000, dims=dims)
        N, K = w.N, w.K
        ctx = binding.Context(w.dims, w.n_bones, w.lo, w.hi, tol=w.tol, div_thresh=w.div_thresh, max_iters=w.max_iters)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        W, B, xq = up(w.W), up(w.B), up(w.xq)
        xc = torch.empty((K, 3, N), dtype=torch.float32, device=dev)
        cv = torch.empty((K, N), dtype=torch.uint8, device=dev)
        it = torch.empty((K, N), dtype=torch.uint8, device=dev)

        def run():
            ctx.precompute(W, B)
            ctx.solve(xq, None, N, K, None, None, None, xc, cv, None, it)
        for _ in range(3):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(10):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 10
        print(json.dumps({"sweep": "grid resolution", "grid": list(dims), "grid_bytes": dims[0] * dims[1] * dims[2] * 48,
                          "points": N, "inits": K, "articulation_ms": ms, "points_per_s": N / (ms * 1e-3),
                          "converged_pairs": int(cv.sum().item()),
                          "lane_iterations": int(it.to(torch.int64).sum().item()) + N * K}))
        ctx.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="workload configuration 1..5 (default 2: SMPL-scale)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-grad", action="store_true", help="leave fs_grad out of the step")
    ap.add_argument("--no-slots", action="store_true",
                    help="fs_grad counts lanes per cell itself instead of reusing fs_solve's counts")
    ap.add_argument("--probe-copy-mib", type=int, default=0,
                    help="after the timed region copy this many MiB device to device once (a kernel of known "
                         "traffic, for calibrating the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    ap.add_argument("--resolution-sweep", action="store_true",
                    help="instead of the benchmark: time fs_precompute + fs_solve for 200k posed points x 24 inits on "
                         "weight grids of 16x16x4 .. 128x128x32 (the shape of the paper's grid-resolution ablation, "
                         "Table 2) and print one JSON line per grid")
    ap.add_argument("--unfused", action="store_true",
                    help="materialise the initial states with fs_init instead of computing them inside fs_solve")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (lanes are independent: several GPUs would each take a share "
              "of the points and a copy of the transform grid); rerun with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2211_15601_amd import binding, workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    binding.load()
    dev = "cuda:0"
    torch.cuda.set_device(0)

    if args.resolution_sweep:
        resolution_sweep(torch, binding, wl, dev)
        return

    w = wl.make_config(args.config)
    N, K = w.N, w.K
    ctx = binding.Context(w.dims, w.n_bones, w.lo, w.hi, n_poses=w.n_poses, tol=w.tol, div_thresh=w.div_thresh,
                          max_iters=w.max_iters, init_mode=w.init_mode, grad_mode=binding.FS_GRAD_BROYDEN_J,
                          corr_dims=w.corr_dims)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    W, B, xq = up(w.W), up(w.B), up(w.xq)
    pose = up(w.pose) if w.n_poses > 1 else None
    gxc = up(w.upstream_grads())
    f32, u8 = torch.float32, torch.uint8
    x0 = torch.empty((K, 3, N), dtype=f32, device=dev)
    J0 = torch.empty((K, 9, N), dtype=f32, device=dev)
    v0 = torch.empty((K, N), dtype=u8, device=dev)
    xc = torch.empty((K, 3, N), dtype=f32, device=dev)
    Jo = torch.empty((K, 9, N), dtype=f32, device=dev)
    cv = torch.empty((K, N), dtype=u8, device=dev)
    it = torch.empty((K, N), dtype=u8, device=dev)
    gW = torch.empty(w.W.shape, dtype=f32, device=dev)
    gB = torch.empty(w.B.shape, dtype=f32, device=dev)
    gxq = torch.empty((3, N), dtype=f32, device=dev)
    slot = None if args.no_slots else torch.empty((K, N), dtype=torch.int32, device=dev)
    # with the cell positions handed on, J~ can stay in the library's result records
    Jarg = None if slot is not None else Jo

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []

    def step(record):
        e = [ev() for _ in range(5)] if record else None
        if record: e[0].record()
        ctx.precompute(W, B)
        if record: e[1].record()
        if args.unfused:
            ctx.init(xq, pose, N, x0, J0, v0)
        if record: e[2].record()
        if args.unfused:
            ctx.solve(xq, pose, N, K, x0, J0, v0, xc, cv, Jarg, it, slot)
        else:
            ctx.solve(xq, pose, N, K, None, None, None, xc, cv, Jarg, it, slot)
        if record: e[3].record()
        if not args.no_grad:
            ctx.grad(W, xc, Jarg, cv, gxc, pose, N, K, gW, gB, gxq, slot)
        if record: e[4].record()
        if record: marks.append(e)

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    ctx.set_timing(True)          # HIP events around the Broyden kernel itself, on its stream
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps

    kernel_ms_total, kernel_launches = ctx.get_timing()
    ctx.set_timing(False)
    solve_kernel_ms = kernel_ms_total / max(kernel_launches, 1)
    # per-call breakdown from a second, untimed pass (the event records between the calls cost a few
    # microseconds each and stay out of the timed region)
    for _ in range(min(args.steps, 20)):
        step(True)
    torch.cuda.synchronize()
    phases = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in marks])   # ms
    pre_ms, init_ms, solve_ms, grad_ms = phases.mean(0)

    ctx.init(xq, pose, N, x0, J0, v0)                 # (untimed) validity flags for the lane-iteration count
    torch.cuda.synchronize()
    conv = int(cv.sum().item())
    valid = int(v0.sum().item())
    steps_total = int(it.to(torch.int64)[v0 == 1].sum().item())
    evals = steps_total + valid                       # field evaluations = active lane-iterations
    flops = evals * FLOP_EVAL + steps_total * (FLOP_UPDATE + FLOP_STEP)
    achieved = flops / (solve_kernel_ms * 1e-3) / 1e12

    # transform grids (all poses) of at most 64 KiB are held in LDS by k_solve; larger ones go to k_solve_ws
    grid_in_lds = w.n_poses * w.dims[0] * w.dims[1] * w.dims[2] * 48 <= 64 * 1024
    out = {
        "metric": "converged (point, init) root solves/sec",
        "value": conv / (ms_per_step * 1e-3),
        "unit": "solves/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"config {args.config} ({w.name}): grid {w.dims[0]}x{w.dims[1]}x{w.dims[2]}, "
                               f"{w.n_bones} bones, {w.n_poses} pose(s), {N} points x {K} inits, "
                               f"max_iters {w.max_iters}, tol {w.tol}",
                   "step": "fs_precompute + " + ("fs_init + fs_solve" if args.unfused else "fs_solve (initial states fused)")
                           + ("" if args.no_grad else " + fs_grad")
                           + ("" if slot is None else (", cell positions handed from the solve to the backward"
                                                       + (", J~ kept in the library" if Jarg is None else ""))),
                   "pairs": N * K, "valid_pairs": valid, "converged_pairs": conv,
                   "lane_iterations": evals},
        "breakdown_ms": {"fs_precompute": float(pre_ms), "fs_init": float(init_ms), "fs_solve": float(solve_ms),
                         "fs_grad": float(grad_ms)},
        "solve_only": {"converged_solves_per_s": conv / (solve_ms * 1e-3),
                       "lane_iterations_per_s": evals / (solve_ms * 1e-3)},
        "roofline": {"kernel": "k_solve" if grid_in_lds else "k_solve_ws", "bound": "alu", "achieved": achieved, "peak": PEAK_FP32_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / PEAK_FP32_TFLOPS, "traffic": None,
                     "flop_per_launch": flops, "avg_launch_ms": float(solve_kernel_ms), "launches_timed": kernel_launches},
    }

    # ceilings of the solve kernel measured on this device by the library's micro-benchmarks
    grid_bytes = int(w.n_poses * w.dims[0] * w.dims[1] * w.dims[2] * 48)
    fma = binding.microbench(binding.MB_FMA)
    gl = binding.microbench(binding.MB_GATHER_LANE, max(grid_bytes, 4096))
    gline = binding.microbench(binding.MB_GATHER_LINE, max(grid_bytes, 4096))
    glds = binding.microbench(binding.MB_LDS_GATHER)
    loads = evals * LOADS_EVAL / (solve_kernel_ms * 1e-3)
    out["roofline"].update({
        "peak_unpacked": PEAK_FP32_UNPACKED_TFLOPS, "frac_unpacked": achieved / PEAK_FP32_UNPACKED_TFLOPS,
        "measured_fma_tflops": fma / 1e12,
        "gather_path": {"algorithmic_16B_loads_per_s": loads,
                        "ceiling_lane_random_gather_same_footprint": gl, "frac_of_lane_gather": loads / gl,
                        "ceiling_line_coalesced_gather_same_footprint": gline,
                        "ceiling_lds_lane_random_gather": glds, "footprint_bytes": grid_bytes},
        "traffic": (SOLVE_TRAFFIC_BYTES_NO_SLOTS if args.no_slots else SOLVE_TRAFFIC_BYTES).get(args.config)})
    if args.config in SOLVE_L1_ACCESSES and not args.no_slots and not args.unfused:
        # the texture path's own roofline: served gathers per second against the ceiling measured on this device for
        # the kernel's mix of L1 hits (lane-random gathers from an L1-resident array) and L2 hits (from an array of
        # the grid's size)
        acc, req = SOLVE_L1_ACCESSES[args.config], SOLVE_L1_TO_L2_REQUESTS[args.config]
        hit = 1.0 - req / acc
        g1 = binding.microbench(binding.MB_GATHER_LANE, 8192)
        blended = 1.0 / (hit / g1 + (1.0 - hit) / gl)
        served = acc / (solve_kernel_ms * 1e-3)
        out["roofline"]["gather_path"].update({
            "l1_accesses_per_launch": acc, "l1_hit_rate": hit, "served_16B_gathers_per_s": served,
            "ceiling_lane_random_gather_l1_resident": g1, "ceiling_for_this_hit_rate": blended,
            "frac_of_ceiling_for_this_hit_rate": served / blended})

    if args.probe_copy_mib > 0:
        a = torch.empty(args.probe_copy_mib << 18, dtype=f32, device=dev)
        b = torch.ones(args.probe_copy_mib << 18, dtype=f32, device=dev)
        torch.cuda.synchronize()
        a.copy_(b)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        import oracle
        ncores = int(os.environ.get("OMP_NUM_THREADS", len(os.sched_getaffinity(0))))
        pz = w.pose if w.n_poses > 1 else None
        best = None
        for rep in range(2):
            c0 = time.perf_counter()
            T = oracle.precompute(w.dims, w.W, w.B, prec="f32")
            if w.init_mode == 0:
                a0, b0, c0v = oracle.init_bone(w.dims, w.lo, w.hi, T, w.B, w.xq, pose=pz, prec="f32")
            else:
                bb, cd = oracle.corr_build(w.dims, w.lo, w.hi, T, w.corr_dims, prec="f32")
                a0, b0, c0v = oracle.init_voxel(w.dims, w.lo, w.hi, T, w.corr_dims, bb, cd, w.xq, pose=pz, prec="f32")
            oxc, ocv, oJ, oit = oracle.solve(w.dims, w.lo, w.hi, T, w.xq, a0, b0, c0v, pose=pz, tol=w.tol,
                                             div_thresh=w.div_thresh, max_iters=w.max_iters, prec="f32")
            if not args.no_grad:
                oracle.grad(w.dims, w.lo, w.hi, T, w.W, w.B, oxc, oJ, ocv, w.upstream_grads(), pose=pz, mode=0, prec="f32")
            dt = time.perf_counter() - c0
            best = dt if best is None else min(best, dt)
        out["cpu_baseline"] = {"value": int(ocv.sum()) / best, "unit": "solves/s", "cores": ncores, "kind": "oracle",
                               "sample": "the whole workload of this run, same step (strict-fp32 oracle, best of 2 passes)",
                               "seconds": best}
        out["parity_spot_check"] = {"conv_equal": bool((ocv == cv.cpu().numpy()).all())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
