/*
 * fastsnarf.h -- C ABI of the MI355X-native Fast-SNARF articulation library.
 *
 * The library maps deformed-space query points x' back to canonical space by solving
 * d(x) - x' = 0 with Broyden's method from several initial states per point, where
 * d(x) = T(x) x and T(x) is the tri-linear interpolation of a per-voxel grid of blended
 * bone transforms (paper: Sec. 2 "Correspondence Search", "Handling Multiple
 * Correspondences"; Sec. 3.1 "Voxel-based Correspondence Search"; Algorithm 1, variant 2).
 *
 * Equation numbers below count the paper's numbered display lines from the occupancy-field
 * definition (1)-(2): (4) LBS, (5) forward map, (6) root equation, (7) quasi-Newton step,
 * (8) initial states, (9) root set, (11) chain rule, (12) implicit differentiation,
 * (13) per-voxel transforms T_v, (15) approximated inverse Jacobian.
 *
 * General conventions
 *  - Every pointer named d_* is a DEVICE pointer owned by the caller, 16-byte aligned, valid on
 *    the context's device.  The library reads / writes it only through work enqueued on the
 *    context's stream during the call and keeps no reference afterwards.
 *  - All calls enqueue on the context's HIP stream and return without synchronising; results are
 *    ready when the stream reaches that point.  Argument and state errors are reported at once
 *    through the return code; a failed launch is reported by the call that made it; a solve whose
 *    kernel gave up one of its bounded waits (fs_set_spin_limit) is reported by the calls after it.
 *    No exceptions or aborts cross this boundary.  fs_last_error() gives a readable message.
 *  - All arithmetic is IEEE fp32.  Point sets are structure-of-arrays: xq is [3][N]; per-lane
 *    arrays are [K][c][N] (lane = (initial state k, point n)), c = 3 for positions, 9 for a
 *    row-major 3x3.  Node index v = (ix*ny + iy)*nz + iz; grid nodes lie ON the box faces:
 *    node (ix,iy,iz) sits at lo + (ix,iy,iz) * (hi-lo)/(n-1).  Outside the box the field is
 *    extended by clamping each coordinate to the box (constant along that axis).
 *  - Point order in and out is the caller's; any reordering is internal.
 *  - A context must not be used from two threads at once.
 */
#ifndef FASTSNARF_H
#define FASTSNARF_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct fs_ctx fs_ctx; /* opaque: owns the transform grids, inverse bone transforms,
                                 correspondence grids and gradient scratch */

typedef enum {
    FS_OK = 0,
    FS_E_ARG = 1,         /* null / misaligned / non-device pointer, bad enum value          */
    FS_E_SHAPE = 2,       /* size out of range or inconsistent with the context              */
    FS_E_STATE = 3,       /* call order: e.g. fs_solve before fs_precompute                  */
    FS_E_ALLOC = 4,       /* device allocation failed                                        */
    FS_E_DEVICE = 5,      /* HIP runtime error (no device, failed launch); unfinished solve  */
    FS_E_UNSUPPORTED = 6
} fs_status;

enum { FS_INIT_BONE = 0, FS_INIT_VOXEL = 1 };
enum { FS_GRAD_BROYDEN_J = 0, FS_GRAD_EXACT_J = 1 };
enum { FS_MAX_BONES = 64, FS_MAX_POSES = 64, FS_MAX_CORR_K = 8 };

typedef struct {
    int32_t nx, ny, nz;   /* grid nodes per axis, each >= 2                                  */
    int32_t n_bones;      /* 1 .. FS_MAX_BONES                                               */
    int32_t n_poses;      /* 1 .. FS_MAX_POSES: poses solved side by side on one weight grid */
    float lo[3], hi[3];   /* canonical box, hi > lo                                          */
} fs_grid_desc;

typedef struct {
    float tol;            /* convergence threshold eps of Eq. (9), > 0                       */
    float div_thresh;     /* divergence threshold of the per-iteration filter, > tol         */
    int32_t max_iters;    /* 0 .. 255 Broyden steps after the initial evaluation             */
    int32_t init_mode;    /* FS_INIT_BONE: K = n_bones; FS_INIT_VOXEL: K = corr_k            */
    int32_t grad_mode;    /* FS_GRAD_BROYDEN_J or FS_GRAD_EXACT_J                            */
    int32_t corr_nx, corr_ny, corr_nz; /* correspondence grid cells (voxel init), each >= 1   */
    int32_t corr_k;       /* candidates kept per cell, 1 .. FS_MAX_CORR_K                    */
} fs_params;

/* Create a context on the current HIP device.  `hip_stream` is a hipStream_t (NULL = the
 * default stream).  Allocates the library-owned grids (n_poses * V * 48 bytes and smaller) and
 * one word of pinned host memory.  On failure *out is NULL. */
fs_status fs_create(const fs_grid_desc *desc, const fs_params *params, void *hip_stream, fs_ctx **out);

/* Free everything the context owns.  Synchronises the stream first.  NULL is allowed. */
fs_status fs_destroy(fs_ctx *ctx);

/* Replace the solve / gradient parameters (tol, div_thresh, max_iters, grad_mode only;
 * init_mode and the correspondence-grid shape are fixed at creation). */
fs_status fs_set_params(fs_ctx *ctx, const fs_params *params);

/* Launch-shape knobs of the solve kernel; results never depend on them.  chunk = lanes a wave draws
 * from the work cursor at a time (8..4096; every draw is one atomic on a single counter, which serves about
 * 1e8 of them per second, so small chunks make the counter the bottleneck), refill_min = idle SIMD lanes that trigger a refill
 * (1..64; until it is set: 8, 24 for grids of more than 32 MiB, 32 for a grid held in LDS),
 * blocks_per_cu = resident 256-thread blocks per compute unit (capped by what the occupancy
 * query reports; until it is set the library takes 2, or 3 where it solves the shorter list of
 * voxel-based candidates on a grid of at most 32 MiB, or holds the grid in LDS); for these a value of 0
 * keeps the current setting.  point_major = 1: consecutive SIMD
 * lanes take the K initial states of one point, 0: consecutive points with the same initial state,
 * -1: keep.  lds_grid = 1: transform grids of at most 148 KiB (all poses; blocks of 4 waves up to 60 KiB, above that one block of 12 waves per CU) are copied into LDS by every
 * block of the solve and read from there, 0: always read through the caches, -1: keep. */
fs_status fs_set_tuning(fs_ctx *ctx, int32_t chunk, int32_t refill_min, int32_t blocks_per_cu, int32_t point_major,
                        int32_t lds_grid);

/* Order in which fs_solve works through the (point, candidate) pairs of voxel-based initial states computed inside the
 * kernel; results never depend on it.  by_place = 0 (default): the order of the points.  1: batches of at least 65,536
 * points are first ordered by pose and column of correspondence cells with a counting sort, so that lanes at work at the
 * same time read neighbouring parts of the transform grid.  2: as 1, and the ordered list is cut into 8 ranges, one per
 * XCD with a cursor of its own (blocks whose range is used up take chunks from the others), so that every XCD's L2
 * sees one stretch of one pose's grid.  Measured on the 8-pose batch of 4.2 M points (Broyden kernel alone):
 * 0: 1.36 ms, 8.6 GB read from beyond the L2 (hit rate 0.47); 1: 1.26 ms, 6.8 GB; 2: 1.29 ms, 2.9 GB (hit rate 0.72).
 * The kernel is limited by the vector cache in front of the L2, not by what the L2 misses, and the sort costs
 * 0.09 ms: over the whole step 1 gained 2 % on that batch and lost 7 % on batches of 1 M points.  (With the kernel as it
 * is now -- consumers that ask for their next records ahead of time -- order 1 takes it from 1.32 to 1.29 ms and the
 * step from 2.77 to 2.79 ms.)  Hence the default. */
fs_status fs_set_list_order(fs_ctx *ctx, int32_t by_place);

/* The waves of a block of the solve kernel hand work to each other through queues in LDS (one wave prepares
 * initial states, the others iterate).  The preparing wave's wait for room in those queues is bounded: when it has
 * polled `polls` times in vain (about 0.2 us each; default 2^22) it gives up and leaves, and the iterating waves,
 * which wait for nothing but that wave, finish what they hold and leave too, so the kernel always ends.
 * The call during which that happened returns FS_OK (nothing is synchronised), its results are incomplete,
 * and every later call on the context that uses the device returns FS_E_DEVICE: destroy the context.  No healthy run
 * comes near the default; the limit exists for tests of this path (polls = 0: the preparing wave gives up the first
 * time it finds every queue full).  polls >= 0. */
fs_status fs_set_spin_limit(fs_ctx *ctx, int32_t polls);

/* Pre-compute linear blend skinning on the grid nodes, Eq. (13) / Sec. 3.1 "Pre-computing
 * LBS": T[p][v] = sum_b W[v][b] * B[p][b], bones accumulated in index order with fused
 * multiply-adds.  Also inverts every bone transform for Eq. (8) and, for FS_INIT_VOXEL,
 * rebuilds the correspondence grid of every pose.
 *   d_W [nx][ny][nz][n_bones]  skinning weights on the grid nodes (used as given)
 *   d_B [n_poses][n_bones][12] bone transforms, row-major 3x4 [R|t] */
fs_status fs_precompute(fs_ctx *ctx, const float *d_W, const float *d_B);

/* Initial states.
 * FS_INIT_BONE, Eq. (8): lane k starts at x0 = B_k^{-1} x' with J~0 = (dd/dx at x0)^{-1} (analytic
 *   Jacobian of the tri-linear field, 3x3 adjugate inverse); valid0 = 0 if B_k or the Jacobian is
 *   singular (|det| < 1e-12).
 * FS_INIT_VOXEL (not defined by the paper; rule of this library): x' is clamped into the pose's
 *   deformed bounding box, lane k starts at the k-th candidate node of its cell of the
 *   correspondence grid; valid0 = 0 where the cell holds fewer candidates.
 *   d_xq [3][N]; d_pose [N] pose index per point, or NULL when n_poses == 1
 *   out: d_x0 [K][3][N], d_Jinv0 [K][9][N], d_valid0 [K][N] (0/1).  N == 0 is a no-op. */
fs_status fs_init(fs_ctx *ctx, const float *d_xq, const int32_t *d_pose, int64_t N,
                  float *d_x0, float *d_Jinv0, uint8_t *d_valid0);

/* Broyden root finding, Eq. (7) with the inverse-Jacobian rank-one update, Algorithm 1
 * (variant 2), one lane per (initial state, point).  A lane stops when |d(x)-x'|^2 < tol^2
 * (converged, Eq. (9)), when !(|d(x)-x'|^2 < div_thresh^2) (diverged or NaN), or after max_iters
 * steps (Sec. 3.1 "Custom CUDA Kernel": per-iteration filtering).
 *   K must equal n_bones (FS_INIT_BONE) or corr_k (FS_INIT_VOXEL); K*N < 2^31.
 *   d_x0, d_Jinv0, d_valid0 all NULL: the kernel computes the initial states of the context's
 *   init_mode itself (same arithmetic as fs_init, bit-identical results) and fs_init is not needed.
 *   out: d_xc [K][3][N] last iterate; d_conv [K][N] 1 = converged; d_Jinv [K][9][N] last J~ (may be
 *   NULL); d_iters [K][N] steps taken (may be NULL).  Lanes with valid0 == 0 return x0, conv 0.
 *   d_slot [K][N] (may be NULL): bookkeeping for fs_grad.  The kernel counts its converged lanes per
 *   grid cell of x* as they finish and writes each lane's arrival position in its cell (-1 where
 *   conv == 0); the counts, and the solve's result records (roots, masks, J~), stay in the context
 *   until the next fs_solve.  The positions depend on the order in which lanes finish, so they differ
 *   from run to run; any run's set is a valid input of fs_grad.  With d_slot, d_Jinv may be NULL:
 *   J~ is then not written out at all and fs_grad takes it from the context. */
fs_status fs_solve(fs_ctx *ctx, const float *d_xq, const int32_t *d_pose, int64_t N, int32_t K,
                   const float *d_x0, const float *d_Jinv0, const uint8_t *d_valid0,
                   float *d_xc, uint8_t *d_conv, float *d_Jinv, uint8_t *d_iters, int32_t *d_slot);

/* Backward by implicit differentiation, Eq. (11)/(12); with FS_GRAD_BROYDEN_J the inverse
 * Jacobian is Broyden's last J~ (Sec. 3.2 "Approximated Gradient", Eq. (15)), with
 * FS_GRAD_EXACT_J it is recomputed analytically at x*.  Only lanes with conv == 1 contribute.
 *   in : d_xc, d_Jinv (may be NULL for FS_GRAD_EXACT_J, or with d_slot), d_conv, d_gxc [K][3][N] = dL/dx*,
 *        d_W as given to fs_precompute
 *        d_slot: NULL, or the array the last fs_solve on this context wrote (same N, K, and d_xc,
 *        d_conv, d_pose as that call left them; FS_E_STATE otherwise where it can be told).  The
 *        pass that sorts the lanes by grid cell then reuses the solve's counts instead of counting
 *        again, and roots, masks and J~ are read from the result records that solve left in the
 *        context (one contiguous record per pair) rather than from d_xc / d_conv / d_Jinv; d_Jinv may
 *        then be NULL for FS_GRAD_BROYDEN_J too.  The sums are the same up to the order of the fp32
 *        additions.
 *   out: d_gW [nx][ny][nz][n_bones] = dL/dW (summed over poses), d_gB [n_poses][n_bones][12],
 *        d_gxq [3][N] = dL/dx' (may be NULL).  Outputs are overwritten.  No floating-point atomics are
 *        used, but the order in which the lanes of a grid cell are added follows the order in which
 *        they were counted (integer atomics), so dL/dW and dL/dB vary in the last bits from run to run. */
fs_status fs_grad(fs_ctx *ctx, const float *d_W, const float *d_xc, const float *d_Jinv,
                  const uint8_t *d_conv, const float *d_gxc, const int32_t *d_pose, int64_t N, int32_t K,
                  const int32_t *d_slot, float *d_gW, float *d_gB, float *d_gxq);

/* Duplicate removal, Sec. 3.1 "Remove Duplicate Correspondences": different initial states often reach
 * the same root, and the canonical field should be queried once per distinct root.  The paper detects
 * duplicates by distance in canonical space without stating the rule; here, per point, lanes are
 * visited in increasing k and a converged lane is kept iff no lane kept before it lies closer than
 * min_dist (Euclidean, strict <).
 *   in : d_xc [K][3][N], d_conv [K][N]
 *   out: d_keep [K][N] 0/1; d_offsets [N+1]: point n owns packed entries offsets[n] .. offsets[n+1],
 *        offsets[N] = number of kept roots; d_roots [cap][3] and d_lane [cap] (either may be NULL): the
 *        kept roots and their lane index k in that order.  Entries beyond cap are not written, so the
 *        caller compares offsets[N] with cap.  K <= 64.  N == 0 writes offsets[0] = 0. */
fs_status fs_dedupe(fs_ctx *ctx, const float *d_xc, const uint8_t *d_conv, int64_t N, int32_t K, float min_dist,
                    uint8_t *d_keep, int32_t *d_offsets, float *d_roots, int32_t *d_lane, int64_t cap);

/* fs_dedupe for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments, same results (bit for bit) as fs_dedupe.  The partial sums of
 * its prefix scan live in a fixed 16 KiB device array inside the library (one copy per GPU, held until the process
 * ends) instead of a context buffer that grows on demand, so this call never allocates, frees or synchronises.
 * Limit: N <= 16,777,216 points (4096 scan tiles of 4096); larger N returns FS_E_SHAPE and touches nothing.
 * The context's device must be the current device.  All calls on one GPU share that array, whatever their context
 * or stream: calls that overlap on one GPU race; calls on one stream, or otherwise ordered, do not (every call
 * overwrites what it reads before reading it, nothing is carried over from the call before). */
fs_status fs_dedupe_noalloc(fs_ctx *ctx, const float *d_xc, const uint8_t *d_conv, int64_t N, int32_t K, float min_dist,
                            uint8_t *d_keep, int32_t *d_offsets, float *d_roots, int32_t *d_lane, int64_t cap);

/* Copy library-owned state out for inspection (device to device, on the stream).
 *   fs_get_transforms: d_T [n_poses][V][12], the pre-computed grid in node order.
 *   fs_get_corr: d_bbox [n_poses][6] (lo xyz, hi xyz), d_cand [n_poses][ncell][corr_k] node index
 *   or -1, cell index = (cx*corr_ny + cy)*corr_nz + cz.  FS_E_STATE unless FS_INIT_VOXEL. */
fs_status fs_get_transforms(fs_ctx *ctx, float *d_T);
fs_status fs_get_corr(fs_ctx *ctx, float *d_bbox, int32_t *d_cand);

/* Message for the last non-OK status returned on this context ("" if none). */
const char *fs_last_error(const fs_ctx *ctx);

/* Library version string. */
const char *fs_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FASTSNARF_H */
