#!/usr/bin/env python3
"""Benchmark of the Fast-SNARF articulation hot path on one MI355X.

One "step" = one pass of the whole path over one synthetic batch that is already resident in
HBM: fs_precompute -> fs_solve (initial states computed inside the kernel; iteration counts kept,
J~ left in the library's result records) -> fs_grad.  `--unfused` materialises the initial states
with fs_init first.

Headline workload (default `--config 5`): the largest single-GPU configuration, the multi-pose batch
(8 poses, 24 bones each, 128x128x32 weight grid = 192 MiB of transform grids, 524,288 points per pose,
voxel-based initial states with up to 3 candidates, max 50 iterations, tol 1e-5).  The other four
configurations are timed too and reported, shorter, under `per_config`.

Prints ONE JSON line.  `value` = converged (point, init) root solves per second over the whole
step.  `roofline` describes the Broyden kernel (k_solve_ws, or k_solve when the grid fits in LDS: the
dominant one), timed by the library with HIP events around that kernel on the stream it runs on.
`cpu_baseline` is the CPU oracle timed on this machine's host cores.
"""
import argparse
import json
import os
import re
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
BYTES_EVAL = 384     # ... = 8 x 48 bytes gathered per field evaluation
PEAK_FP32_TFLOPS = 157.3            # published fp32 vector peak (needs packed fp32 instructions)
PEAK_FP32_UNPACKED_TFLOPS = 78.6    # 256 CUs x 4 SIMDs x 16 lanes x 2 flop x 2.4 GHz: one FMA per lane per clock
PEAK_HBM_BPS = 8.0e12
LDS_GRID_MAX = 148 * 1024           # transform grids (all poses) up to this size are held in LDS by k_solve


def profile_value(cfg, key):
    """A figure measured with rocprofv3 and committed under profiles/ (a line `key: number` in the summary of the
    Broyden kernel on this configuration); None where no such run was made."""
    path = os.path.join(ROOT, "profiles", f"k_solve_config{cfg}_counters.md")
    try:
        with open(path) as f:
            m = re.search(rf"^{re.escape(key)}\s*:\s*([0-9.eE+-]+)\s*$", f.read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def pct(a):
    a = np.asarray(a, dtype=np.float64)
    return {"median": float(np.median(a)), "p10": float(np.percentile(a, 10)), "p90": float(np.percentile(a, 90))}


class Case:
    """One configuration resident on the device: context, inputs, outputs."""

    def __init__(self, cfg, args, torch, binding, wl, dev):
        self.cfg, self.args, self.torch, self.binding = cfg, args, torch, binding
        w = self.w = wl.make_config(cfg)
        N, K = self.N, self.K = w.N, w.K
        self.ctx = binding.Context(w.dims, w.n_bones, w.lo, w.hi, n_poses=w.n_poses, tol=w.tol, div_thresh=w.div_thresh,
                                   max_iters=w.max_iters, init_mode=w.init_mode, grad_mode=binding.FS_GRAD_BROYDEN_J,
                                   corr_dims=w.corr_dims)
        self.ctx.set_list_order({"input": 0, "place": 1, "place-xcd": 2}[getattr(args, "list_order", "input")])
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        self.W, self.B, self.xq = up(w.W), up(w.B), up(w.xq)
        self.pose = up(w.pose) if w.n_poses > 1 else None
        self.gxc = up(w.upstream_grads())
        f32, u8 = torch.float32, torch.uint8
        e = lambda shape, dt: torch.empty(shape, dtype=dt, device=dev)
        self.x0, self.J0, self.v0 = e((K, 3, N), f32), e((K, 9, N), f32), e((K, N), u8)
        self.xc, self.cv, self.it = e((K, 3, N), f32), e((K, N), u8), e((K, N), u8)
        self.gW, self.gB, self.gxq = e(w.W.shape, f32), e(w.B.shape, f32), e((3, N), f32)
        self.slot = None if args.no_slots else e((K, N), torch.int32)
        # with the cell positions handed on, J~ can stay in the library's result records
        self.Jarg = None if self.slot is not None else e((K, 9, N), f32)
        self.grid_bytes = int(w.n_poses * w.dims[0] * w.dims[1] * w.dims[2] * 48)
        self.kernel = "k_solve" if self.grid_bytes <= LDS_GRID_MAX else "k_solve_ws"

    def step(self, marks=None):
        a, c, t = self.args, self.ctx, self.torch
        ev = [t.cuda.Event(enable_timing=True) for _ in range(5)] if marks is not None else None
        if ev: ev[0].record()
        c.precompute(self.W, self.B)
        if ev: ev[1].record()
        if a.unfused:
            c.init(self.xq, self.pose, self.N, self.x0, self.J0, self.v0)
        if ev: ev[2].record()
        if a.unfused:
            c.solve(self.xq, self.pose, self.N, self.K, self.x0, self.J0, self.v0, self.xc, self.cv, self.Jarg, self.it, self.slot)
        else:
            c.solve(self.xq, self.pose, self.N, self.K, None, None, None, self.xc, self.cv, self.Jarg, self.it, self.slot)
        if ev: ev[3].record()
        if not a.no_grad:
            c.grad(self.W, self.xc, self.Jarg, self.cv, self.gxc, self.pose, self.N, self.K, self.gW, self.gB, self.gxq, self.slot)
        if ev:
            ev[4].record()
            marks.append(ev)

    def measure(self, steps, warmup, launches):
        """Wall-clock of `steps` whole steps, the Broyden kernel's own time (HIP events inside the library, on the
        stream it is launched on) over the same steps, then `launches` more steps with events between the calls
        for the per-call statistics."""
        t, c = self.torch, self.ctx
        for _ in range(warmup):
            self.step()
        t.cuda.synchronize()
        c.set_timing(True)
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        t.cuda.synchronize()
        t1 = time.perf_counter()
        kms, kn = c.get_timing()
        c.set_timing(False)
        self.ms_per_step = (t1 - t0) * 1e3 / steps
        self.kernel_ms, self.kernel_launches = kms / max(kn, 1), kn
        marks = []
        for _ in range(launches):
            self.step(marks)
        t.cuda.synchronize()
        ph = np.array([[e[i].elapsed_time(e[i + 1]) for i in range(4)] for e in marks])   # ms
        self.calls = {"fs_precompute": pct(ph[:, 0]), "fs_solve": pct(ph[:, 2]), "fs_grad": pct(ph[:, 3]),
                      "step": pct(ph.sum(1)), "launches": launches}
        if self.args.unfused:
            self.calls["fs_init"] = pct(ph[:, 1])
        # (untimed) validity flags for the count of field evaluations
        c.init(self.xq, self.pose, self.N, self.x0, self.J0, self.v0)
        t.cuda.synchronize()
        valid = self.v0 == 1
        self.conv = int(self.cv.sum(dtype=t.int64).item())
        self.valid = int(valid.sum().item())
        its = self.it[valid].to(t.int64)
        self.steps_total = int(its.sum().item())
        self.evals = self.steps_total + self.valid            # field evaluations = active lane-iterations
        self.iter_hist = t.bincount(its, minlength=self.w.max_iters + 1).cpu().tolist()
        self.flops = self.evals * FLOP_EVAL + self.steps_total * (FLOP_UPDATE + FLOP_STEP)

    def workload(self):
        w = self.w
        return (f"config {self.cfg} ({w.name}): grid {w.dims[0]}x{w.dims[1]}x{w.dims[2]}, {w.n_bones} bones, "
                f"{w.n_poses} pose(s), {self.N} points x {self.K} inits "
                f"({'one per bone' if w.init_mode == 0 else 'voxel-based candidates'}), max_iters {w.max_iters}, tol {w.tol}")

    def roofline(self):
        ks = self.kernel_ms * 1e-3
        achieved = self.flops / ks / 1e12
        traffic = profile_value(self.cfg, "hbm_bytes_per_launch") if not (self.args.no_slots or self.args.unfused) else None
        r = {"kernel": self.kernel, "bound": "alu", "achieved": achieved, "peak": PEAK_FP32_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_FP32_TFLOPS, "traffic": traffic,
             "peak_unpacked": PEAK_FP32_UNPACKED_TFLOPS, "frac_unpacked": achieved / PEAK_FP32_UNPACKED_TFLOPS,
             "flop_per_launch": self.flops, "evaluations_per_launch": self.evals,
             "avg_launch_ms": float(self.kernel_ms), "launches_timed": self.kernel_launches,
             "evaluations_per_s": self.evals / ks,
             "algorithmic_gather_bytes_per_s": self.evals * BYTES_EVAL / ks}
        if traffic is not None:
            r["hbm"] = {"counter_bytes_per_launch": traffic, "achieved_bytes_per_s": traffic / ks,
                        "frac_of_peak": traffic / ks / PEAK_HBM_BPS}
        return r

    def close(self):
        self.ctx.close()


def resolution_sweep(torch, binding, wl, dev):
    """Articulation time (fs_precompute + fs_solve, fused initial states, roots + masks only) against the
    resolution of the weight grid, 200k points of the SMPL-scale scene."""
    out = []
    for dims in ((16, 16, 4), (16, 16, 8), (32, 32, 8), (64, 64, 16), (128, 128, 32)):
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
        out.append({"sweep": "grid resolution", "grid": list(dims), "grid_bytes": dims[0] * dims[1] * dims[2] * 48,
                    "grid_in_lds": dims[0] * dims[1] * dims[2] * 48 <= LDS_GRID_MAX,
                    "points": N, "inits": K, "articulation_ms": ms, "points_per_s": N / (ms * 1e-3),
                    "converged_pairs": int(cv.sum().item()),
                    "lane_iterations": int(it.to(torch.int64).sum().item()) + N * K})
        ctx.close()
    return out


def cpu_baseline(case, args):
    """The CPU oracle (strict fp32: the arithmetic the parity tests hold the GPU to; then float64 once) running the
    same step on the same inputs on this machine's host cores."""
    import oracle
    w = case.w
    ncores = int(os.environ.get("OMP_NUM_THREADS", len(os.sched_getaffinity(0))))
    pz = w.pose if w.n_poses > 1 else None
    gx = w.upstream_grads()

    def one(prec):
        c0 = time.perf_counter()
        T = oracle.precompute(w.dims, w.W, w.B, prec=prec)
        if w.init_mode == 0:
            a0, b0, c0v = oracle.init_bone(w.dims, w.lo, w.hi, T, w.B, w.xq, pose=pz, prec=prec)
        else:
            bb, cd = oracle.corr_build(w.dims, w.lo, w.hi, T, w.corr_dims, prec=prec)
            a0, b0, c0v = oracle.init_voxel(w.dims, w.lo, w.hi, T, w.corr_dims, bb, cd, w.xq, pose=pz, prec=prec)
        oxc, ocv, oJ, oit = oracle.solve(w.dims, w.lo, w.hi, T, w.xq, a0, b0, c0v, pose=pz, tol=w.tol,
                                         div_thresh=w.div_thresh, max_iters=w.max_iters, prec=prec)
        if not args.no_grad:
            oracle.grad(w.dims, w.lo, w.hi, T, w.W, w.B, oxc, oJ, ocv, gx, pose=pz, mode=0, prec=prec)
        return time.perf_counter() - c0, ocv
    best, ocv = None, None
    for _ in range(2):
        dt, ocv = one("f32")
        best = dt if best is None else min(best, dt)
    dt64, ocv64 = one("f64")
    base = {"value": int(ocv.sum()) / best, "unit": "solves/s", "cores": ncores, "kind": "oracle",
            "sample": "the whole workload of this run, same step (strict-fp32 oracle, best of 2 passes)",
            "seconds": best,
            "float64_oracle": {"value": int(ocv64.sum()) / dt64, "seconds": dt64, "converged_pairs": int(ocv64.sum())}}
    return base, {"conv_equal": bool((ocv == case.cv.cpu().numpy()).all())}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=5,
                    help="headline workload configuration 1..5 (default 5: multi-pose, the largest that one GPU takes)")
    ap.add_argument("--launches", type=int, default=100,
                    help="extra steps, after the timed region, with HIP events between the fs_* calls (median / p10 / p90 per call)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="time the headline configuration only")
    ap.add_argument("--no-microbench", action="store_true", help="skip the library's micro-benchmarks of the gather ceilings")
    ap.add_argument("--no-grad", action="store_true", help="leave fs_grad out of the step")
    ap.add_argument("--no-slots", action="store_true",
                    help="fs_grad counts lanes per cell itself instead of reusing fs_solve's counts")
    ap.add_argument("--probe-copy-mib", type=int, default=0,
                    help="after the timed region copy this many MiB device to device once (a kernel of known "
                         "traffic, for calibrating the FETCH_SIZE / WRITE_SIZE counters under rocprofv3)")
    ap.add_argument("--no-sweep", action="store_true", help="leave the grid-resolution sweep out of the JSON line")
    ap.add_argument("--resolution-sweep", action="store_true",
                    help="instead of the benchmark: time fs_precompute + fs_solve for 200k posed points x 24 inits on "
                         "weight grids of 16x16x4 .. 128x128x32 (the shape of the paper's grid-resolution ablation, "
                         "Table 2) and print one JSON line per grid")
    ap.add_argument("--list-order", choices=("input", "place", "place-xcd"), default="input",
                    help="order of the (point, candidate) pair list of voxel-based solves: as the points come (default), "
                         "ordered by pose and correspondence cell on the device, or ordered and cut into one range "
                         "per XCD (fs_set_list_order 0 / 1 / 2)")
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
        for r in resolution_sweep(torch, binding, wl, dev):
            print(json.dumps(r))
        return

    case = Case(args.config, args, torch, binding, wl, dev)
    case.measure(args.steps, args.warmup, args.launches)
    w = case.w
    out = {
        "metric": "converged (point, init) root solves/sec",
        "value": case.conv / (case.ms_per_step * 1e-3),
        "unit": "solves/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": case.ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": case.workload(),
                   "step": "fs_precompute + " + ("fs_init + fs_solve" if args.unfused else "fs_solve (initial states fused)")
                           + ("" if args.no_grad else " + fs_grad")
                           + ("" if case.slot is None else (", cell positions handed from the solve to the backward"
                                                            + (", J~ kept in the library" if case.Jarg is None else ""))),
                   "list_order": args.list_order,
                   "pairs": case.N * case.K, "valid_pairs": case.valid, "converged_pairs": case.conv,
                   "lane_iterations": case.evals},
        "calls_ms": case.calls,
        "solve_only": {"converged_solves_per_s": case.conv / (case.calls["fs_solve"]["median"] * 1e-3),
                       "lane_iterations_per_s": case.evals / (case.calls["fs_solve"]["median"] * 1e-3)},
        "iteration_histogram": case.iter_hist,
        "roofline": case.roofline(),
    }
    if case.slot is not None:
        # one position in its grid cell's list per converged lane, handed out by integer atomics inside the Broyden kernel
        # (requests of one wave for the same cell are sent as one atomic)
        out["slot_requests_per_s"] = case.conv / (case.kernel_ms * 1e-3)

    if not args.no_microbench:
        # Ceilings of the Broyden kernel measured on this device by the library's micro-benchmarks.  The kernel's own
        # access pattern is FS_MB_GATHER_SEGMENT: every SIMD lane reads the six 16-byte pieces of a random pair of adjacent
        # 48-byte records.  Its rate depends on where the records come from, so it is measured for an array the size of
        # one pose's transform grid (what all waves work on at a time when the points are grouped by pose) and of all of them.
        pose_bytes = max(case.grid_bytes // w.n_poses, 4096)
        gb = max(case.grid_bytes, 4096)
        ks = case.kernel_ms * 1e-3
        loads = case.evals * LOADS_EVAL / ks
        seg_pose = binding.microbench(binding.MB_GATHER_SEGMENT, pose_bytes)
        seg_all = seg_pose if gb == pose_bytes else binding.microbench(binding.MB_GATHER_SEGMENT, gb)
        gp = {"algorithmic_16B_loads_per_s": loads, "grid_bytes": case.grid_bytes, "grid_bytes_per_pose": pose_bytes,
              # rates of the library's micro-benchmarks on this device: references for the kernel's gather path, not bounds
              # (the kernel's lanes are not independent random readers: neighbouring evaluations of a lane share cache lines)
              "reference_rates_16B_loads_per_s": {
                  "segment_gather_one_pose_grid": seg_pose, "segment_gather_whole_grid": seg_all,
                  "line_coalesced_gather_whole_grid": binding.microbench(binding.MB_GATHER_LINE, gb),
                  "lane_random_gather_whole_grid": binding.microbench(binding.MB_GATHER_LANE, gb),
                  "segment_gather_l1_resident": binding.microbench(binding.MB_GATHER_SEGMENT, 8192),
                  "lds_lane_random_gather": binding.microbench(binding.MB_LDS_GATHER)}}
        issued = profile_value(args.config, "l1_accesses_per_launch") if not (args.no_slots or args.unfused) else None
        if issued is not None:
            # loads the kernel really issues (rocprofv3 TCP_TOTAL_CACHE_ACCESSES, profiles/): fewer than the algorithmic
            # 24 per evaluation, since a lane that stays in its grid cell keeps the 8 records in registers
            gp.update({"issued_16B_loads_per_launch": issued, "issued_16B_loads_per_s": issued / ks,
                       # the vector cache of a CU takes one access (a 64-byte block) per clock: 256 CUs at 2.4 GHz
                       "l1_accesses_per_clk_per_cu": issued / (ks * 2.4e9 * 256), "l1_peak_accesses_per_clk_per_cu": 1.0})
        out["roofline"].update({"measured_fma_tflops": binding.microbench(binding.MB_FMA) / 1e12, "gather_path": gp})

    if args.probe_copy_mib > 0:
        a = torch.empty(args.probe_copy_mib << 18, dtype=torch.float32, device=dev)
        b = torch.ones(args.probe_copy_mib << 18, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        a.copy_(b)
        torch.cuda.synchronize()

    if not args.no_cpu_baseline:
        out["cpu_baseline"], out["parity_spot_check"] = cpu_baseline(case, args)
    case.close()
    del case
    torch.cuda.empty_cache()

    if not args.no_per_config:
        per = {}
        for cfg in (1, 2, 3, 4, 5):
            if cfg == args.config:
                continue
            c = Case(cfg, args, torch, binding, wl, dev)
            c.measure(max(10, min(args.steps, 50)), max(3, args.warmup), min(args.launches, 50))
            r = c.roofline()
            per[str(cfg)] = {"workload": c.workload(), "ms_per_step": c.ms_per_step,
                             "value": c.conv / (c.ms_per_step * 1e-3),
                             "converged_pairs": c.conv, "valid_pairs": c.valid, "lane_iterations": c.evals,
                             "calls_ms": {k: (v["median"] if isinstance(v, dict) else v) for k, v in c.calls.items()},
                             "kernel": r["kernel"], "kernel_ms": r["avg_launch_ms"], "evaluations_per_s": r["evaluations_per_s"],
                             "tflops": r["achieved"], "frac": r["frac"], "frac_unpacked": r["frac_unpacked"],
                             "traffic": r["traffic"]}
            c.close()
            del c
            torch.cuda.empty_cache()
        out["per_config"] = per
    if not args.no_sweep and not args.no_per_config:
        # fs_precompute + fs_solve (roots, masks, iteration counts) for 200 000 points x 24 initial states against the
        # resolution of the grid: the shape of the paper's grid-resolution ablation (Table 2)
        out["resolution_sweep"] = [{k: r[k] for k in ("grid", "grid_bytes", "grid_in_lds", "articulation_ms", "points_per_s")}
                                   for r in resolution_sweep(torch, binding, wl, dev)]
    print(json.dumps(out))


if __name__ == "__main__":
    main()
