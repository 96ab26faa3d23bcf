/*
 * fastsnarf_bench.h -- measurement support of the Fast-SNARF articulation library.
 *
 * Nothing here is part of the articulation path (include/fastsnarf.h): these calls exist for the
 * benchmark, which reports the Broyden kernel's own launch time and the measured ceilings of the
 * device it ran on beside the published ones.
 */
#ifndef FASTSNARF_BENCH_H
#define FASTSNARF_BENCH_H

#include "fastsnarf.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Timing of the Broyden kernel alone (k_solve, without the unpacking of its results): while enabled,
 * every fs_solve brackets that kernel with two HIP events on the context's stream.  fs_get_timing
 * synchronises the stream, returns the summed elapsed milliseconds and the number of launches since
 * the last call, and releases the events. */
fs_status fs_set_timing(fs_ctx *ctx, int32_t enable);
fs_status fs_get_timing(fs_ctx *ctx, double *solve_kernel_ms, int32_t *launches);

/* Micro-benchmarks of the ceilings that bound
 * fs_solve on the current device, run on the default stream, synchronising.
 *   FS_MB_FMA          *result = fp32 flop/s of independent fused multiply-add chains
 *   FS_MB_GATHER_LANE  *result = 16-byte loads per second when every SIMD lane reads its own random
 *                      address inside an array of array_bytes (the tri-linear lookup's access pattern)
 *   FS_MB_GATHER_LINE  same, but 8 adjacent lanes share one aligned 128-byte line
 *   FS_MB_LDS_GATHER   16-byte loads per second, every lane its own random address in 48 KiB of LDS
 *   FS_MB_GATHER_SEGMENT  16-byte loads per second when every lane reads the six pieces of a random pair of adjacent
 *                      48-byte records with six consecutive instructions: the solve kernel's own pattern (two
 *                      z-neighbours of the transform grid), so that this is its ceiling for a grid of array_bytes
 * array_bytes is used by the three global gathers only (4 KiB .. 4 GiB). */
enum { FS_MB_FMA = 0, FS_MB_GATHER_LANE = 1, FS_MB_GATHER_LINE = 2, FS_MB_LDS_GATHER = 3, FS_MB_GATHER_SEGMENT = 4 };
fs_status fs_microbench(int32_t which, int64_t array_bytes, double *result);

#ifdef __cplusplus
}
#endif
#endif /* FASTSNARF_BENCH_H */
