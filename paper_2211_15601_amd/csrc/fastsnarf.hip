// C ABI of the Fast-SNARF articulation library (see include/fastsnarf.h): argument checks,
// context-owned device buffers and kernel launches.  gfx950 only.
#include "../../include/fastsnarf.h"
#include "../../include/fastsnarf_bench.h"
#include "fs_kernels.hpp"

#include <hip/hip_runtime.h>
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <utility>
#include <vector>

using namespace fs;

struct fs_ctx {
    fs_grid_desc desc;
    fs_params prm;
    hipStream_t stream;
    int device;
    GridP G;
    CorrP C;
    bool have_T;
    // device buffers owned by the context
    float *T;          // [P][V][12]
    float *Bdev;       // [P][nb][12] copy of the bone transforms of the last precompute
    float *Binv;       // [P][nb][12]
    uint8_t *Bok;      // [P][nb]
    float *GT;         // [P][V][12] gradient w.r.t. the transform grid (allocated on first fs_grad)
    // correspondence grid (voxel init)
    float *Y;          // [P][V][3]
    unsigned *bb_ord;  // [P][EXTENT_BLOCKS][6]: per-block extents of the node images (k_corr_extent)
    float *bbox;       // [P][6]
    int *cell_of;      // [P][V]
    int *count;        // [P*ncell + 1] counts, then offsets
    int *fill;         // [P][V] arrival slot of a node inside its cell
    float4 *order;     // [P][V] the nodes sorted by correspondence cell: {image[3], node index}
    int32_t *cand;     // [P][ncell][ck]
    uint8_t *ccnt;     // [P][ncell] number of candidates of a correspondence cell
    float4 *cinit;     // [P][ncell][ck][4] initial state of every candidate (k_corr_init)
    unsigned *cursor;  // work cursor of the solve kernel
    int *gcount;       // [P*ncells + 1] per-cell lane counts, then offsets (backward)
    int *gcount_solve; // [P*ncells + 1] per-cell counts of converged lanes written by the last fs_solve that gave slots
    long long slots_N; // N of that fs_solve (0: none)
    int slots_K;
    bool slots_list;   // that solve drew its pairs from the candidate list: pairs without a candidate have no record
    int *gpos;         // [K*N] position of a lane inside its cell's list (grows on demand)
    float *grec;       // [K*N][8] cell-sorted {x*, lambda, cell} records (grows on demand)
    size_t gcap;       // lanes gpos / grec can hold
    float *gpart;      // [P][gb_blocks][nb*12] partial sums of dL/dB, one per block of k_grad_bones_mfma
    int gb_blocks;
    float4 *srec;      // per-pair result records of the solve kernel (grows on demand)
    size_t srec_cap;   // float4 entries srec can hold
    int *scan_sums;    // tile sums of the prefix scans
    int *voffs;        // [N + 1] candidates per point, then offsets (fused voxel solve; grows on demand)
    uint8_t *vcnt;     // [N] candidates per point
    int *vgcell;       // [N] pose * ncell + correspondence cell of every point
    int2 *vlist;       // [K*N] pairs that have a candidate: {point, cell << 3 | k}
    size_t vcap;       // points voffs / vcnt / vgcell / vlist can hold
    int *vhist;        // [buckets][blocks] + 1: counts, then places, of the counting sort that orders the list by place
    size_t vhist_cap;
    int scan_cap;      // tiles scan_sums can hold
    int n_cus, occ_blocks_per_cu, occ_ws_blocks_per_cu, occ_vx_blocks_per_cu, chunk, refill_min, blocks_per_cu, point_major, lds_grid;
    bool lds_big;      // the grid is larger than 60 KiB and fits the LDS of a CU as one block of 12 waves
    int sort_list;     // order the list of (point, candidate) pairs by place (large voxel-mode batches)
    int xcd_ranges;    // with an ordered list: one range of it, and one cursor, per XCD
    int spin_limit;    // polls for room in its consumers' queues before the producer wave of a solve block gives up
    int pre_serial;    // number of the last fs_precompute; cursor[CUR_NONFINITE] == pre_serial: that grid has an entry that is not finite
    int *gave_up;      // pinned host word, mapped into the device: a wave that gave up sets it
    int *gave_up_dev;  // the device's address of it
    // optional timing of the Broyden kernel alone (events on the context's stream)
    bool timing;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> *timed;
    // caller pointers the runtime has already confirmed as memory of this device (direct-mapped by address)
    const void *ptr_seen[128];
    char err[256];
};

constexpr int FS_NOALLOC_TILES = 4096;
static __device__ __align__(256) int scratch[FS_NOALLOC_TILES + 64];     // see scratch_on_device()

namespace {

fs_status fail(fs_ctx *c, fs_status s, const char *fmt, ...)
{
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof c->err, fmt, ap);
        va_end(ap);
    }
    return s;
}

// Null, alignment and "is memory of this context's device".  The last needs a lookup in the runtime (about a
// microsecond; a step makes some thirty such checks and a small step lasts 150 us), so a pointer that passed it
// once is remembered per context: a training or serving loop passes the same buffers again and again.  A
// remembered pointer whose memory the caller has freed since is the caller's error, as it would be one
// instruction after a fresh check.
bool device_ptr_ok(fs_ctx *c, const void *p, bool nullable)
{
    if (!p) return nullable;
    const uintptr_t u = reinterpret_cast<uintptr_t>(p);
    if ((u & 15u) != 0) return false;
    const size_t h = (size_t)((u >> 4) ^ (u >> 11) ^ (u >> 20)) & 127u;
    if (c->ptr_seen[h] == p) return true;
    hipPointerAttribute_t a;
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();
        return false;
    }
    if (a.type != hipMemoryTypeDevice && a.type != hipMemoryTypeManaged) return false;
    if (a.device != c->device) return false;
    c->ptr_seen[h] = p;
    return true;
}

#define FS_CHECK_PTR(ctx, p, nullable)                                                            \
    do {                                                                                          \
        if (!device_ptr_ok((ctx), (p), (nullable)))                                               \
            return fail((ctx), FS_E_ARG, "%s: " #p " must be a 16-byte aligned device pointer%s", \
                        __func__, (nullable) ? " or NULL" : "");                                  \
    } while (0)

fs_status launch_status(fs_ctx *c, const char *what)
{
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(c, FS_E_DEVICE, "%s: %s", what, hipGetErrorString(e));
    return FS_OK;
}

// A wave of the solve kernel that waited too long for its block's work queue has left early: the results
// of that call are incomplete.  Seen by the first call that comes after the kernel has run; the context
// stays in error from then on.
fs_status check_gave_up(fs_ctx *c, const char *what)
{
    if (c->gave_up && *static_cast<volatile int *>(c->gave_up))
        return fail(c, FS_E_DEVICE, "%s: an earlier fs_solve did not finish (a wave of its kernel gave up waiting for its block's work queue); create a new context", what);
    return FS_OK;
}

template <class Tp>
bool dev_alloc(Tp **p, size_t count)
{
    *p = nullptr;
    if (count == 0) return true;
    if (hipMalloc(reinterpret_cast<void **>(p), count * sizeof(Tp)) != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        return false;
    }
    return true;
}

bool params_ok(const fs_params *p, char *why, size_t n)
{
    if (!(p->tol > 0.0f) || !(p->div_thresh > p->tol) || !std::isfinite(p->div_thresh)) {
        snprintf(why, n, "need 0 < tol < div_thresh < inf");
        return false;
    }
    if (p->max_iters < 0 || p->max_iters > 255) { snprintf(why, n, "max_iters must be in 0..255"); return false; }
    if (p->grad_mode != FS_GRAD_BROYDEN_J && p->grad_mode != FS_GRAD_EXACT_J) {
        snprintf(why, n, "bad grad_mode");
        return false;
    }
    return true;
}

int grid1d(long long n, int block) { return (int)((n + block - 1) / block); }

void free_all(fs_ctx *c)
{
    void *ptrs[] = {c->T, c->Bdev, c->Binv, c->Bok, c->GT, c->Y, c->bb_ord, c->bbox,
                    c->cell_of, c->count, c->fill, c->order, c->cand, c->cursor, c->gcount, c->gcount_solve, c->gpos, c->grec, c->scan_sums, c->srec, c->gpart, c->voffs, c->vlist, c->cinit, c->vcnt, c->vgcell, c->vhist, c->ccnt};
    for (void *p : ptrs)
        if (p) (void)hipFree(p);
}

// exclusive scan of src[0..n) into a[0..n) (src == nullptr: in place) on the context's stream,
// a[n] = total; *also_zero (may be null) is cleared on the way
fs_status scan_exclusive(fs_ctx *c, int n, int *a, const int *src = nullptr, int *also_zero = nullptr)
{
    if (n <= 0) {
        k_fill_zero_i32<<<1, 64, 0, c->stream>>>(1, a);
        if (also_zero) k_fill_zero_i32<<<1, 64, 0, c->stream>>>(1, also_zero);
        return FS_OK;
    }
    const int m = (n + SCAN_TILE - 1) / SCAN_TILE;
    if (m + 1 > c->scan_cap) {
        (void)hipStreamSynchronize(c->stream);
        if (c->scan_sums) (void)hipFree(c->scan_sums);
        c->scan_cap = 0;
        if (!dev_alloc(&c->scan_sums, (size_t)m + 1)) return fail(c, FS_E_ALLOC, "out of device memory (scan)");
        c->scan_cap = m + 1;
    }
    k_scan_tile_sums<<<m, 1024, 0, c->stream>>>(n, src ? src : a, c->scan_sums);
    if (m <= 4096) {
        k_scan_tiles<false><<<m, 1024, 0, c->stream>>>(n, src ? src : a, a, c->scan_sums, m, also_zero);
    } else {
        k_scan_sums<<<1, 1024, 0, c->stream>>>(m, c->scan_sums, also_zero);
        k_scan_tiles<true><<<m, 1024, 0, c->stream>>>(n, src ? src : a, a, c->scan_sums, m, nullptr);
    }
    return FS_OK;
}

// ---- scratch memory of fs_dedupe_noalloc: a file-scope device array instead of a context-owned allocation ----
// The prefix scan over the per-point counts of kept roots needs one partial sum per tile of SCAN_TILE points.
// FS_NOALLOC_MAX_N points = FS_NOALLOC_TILES tiles; every GPU the library runs on holds its own 16 KiB copy of the
// array until the process ends.  In host code the array's name is only a handle for hipGetSymbolAddress: the
// device address is looked up once per device (with that device current) and kept in g_scratch_ptr.
constexpr long long FS_NOALLOC_MAX_N = (long long)FS_NOALLOC_TILES * SCAN_TILE;     // 2^24 points
constexpr int FS_MAX_DEVICES = 64;
int *g_scratch_ptr[FS_MAX_DEVICES];       // device address of `scratch` on device i, nullptr until looked up
std::mutex g_scratch_mutex;

// address of `scratch` on the context's device (which must be the current one); nullptr on failure
int *scratch_on_device(fs_ctx *c)
{
    if (c->device < 0 || c->device >= FS_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[c->device]) {
        int cur = -1;
        if (hipGetDevice(&cur) != hipSuccess || cur != c->device) {
            (void)hipGetLastError();
            return nullptr;
        }
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return nullptr;
        }
        g_scratch_ptr[c->device] = static_cast<int *>(p);
    }
    return g_scratch_ptr[c->device];
}

#ifndef FS_TPN8_AT
#define FS_TPN8_AT 8
#endif
// largest transform grid (all poses) kept in LDS by the solve: a block may ask for 64 KiB in all, and k_solve has 4 KiB of
// its own (the parked cell-position requests of its four waves)
constexpr size_t FS_LDS_GRID_MAX = 60 * 1024;
// ... by one block of 12 waves per CU: the CU's 160 KiB less the 12 KiB of parked requests of those waves
constexpr int FS_LDS_BIG_WAVES = 12;
constexpr size_t FS_LDS_GRID_MAX_BIG = 148 * 1024;

int lanes_K(const fs_ctx *c) { return c->prm.init_mode == FS_INIT_BONE ? c->desc.n_bones : c->prm.corr_k; }

}  // namespace

extern "C" {

const char *fs_version(void) { return "fastsnarf-mi355x 0.1 (gfx950)"; }

const char *fs_last_error(const fs_ctx *ctx) { return ctx ? ctx->err : "null context"; }

fs_status fs_create(const fs_grid_desc *desc, const fs_params *params, void *hip_stream, fs_ctx **out)
{
    if (out) *out = nullptr;
    if (!desc || !params || !out) return FS_E_ARG;
    if (desc->nx < 2 || desc->ny < 2 || desc->nz < 2 || desc->n_bones < 1 || desc->n_bones > FS_MAX_BONES ||
        desc->n_poses < 1 || desc->n_poses > FS_MAX_POSES)
        return FS_E_SHAPE;
    const long long V = (long long)desc->nx * desc->ny * desc->nz;
    if ((long long)desc->n_poses * V * 12 >= (1ll << 31)) return FS_E_SHAPE;   /* grid offsets are 32-bit */
    if (desc->n_poses * desc->n_bones > 1024) return FS_E_UNSUPPORTED;   /* bone tables are staged in 48 KiB of LDS */
    for (int a = 0; a < 3; ++a)
        if (!(desc->hi[a] > desc->lo[a]) || !std::isfinite(desc->hi[a]) || !std::isfinite(desc->lo[a])) return FS_E_ARG;
    char why[128];
    if (!params_ok(params, why, sizeof why)) return FS_E_ARG;
    if (params->init_mode != FS_INIT_BONE && params->init_mode != FS_INIT_VOXEL) return FS_E_ARG;
    if (params->init_mode == FS_INIT_VOXEL) {
        if (params->corr_nx < 1 || params->corr_ny < 1 || params->corr_nz < 1 || params->corr_k < 1 ||
            params->corr_k > FS_MAX_CORR_K)
            return FS_E_SHAPE;
        if ((long long)params->corr_nx * params->corr_ny * params->corr_nz * desc->n_poses >= (1ll << 24)) return FS_E_SHAPE;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return FS_E_DEVICE;
    }
    fs_ctx *c = new (std::nothrow) fs_ctx;
    if (!c) return FS_E_ALLOC;
    std::memset(c, 0, sizeof *c);
    c->desc = *desc;
    c->prm = *params;
    c->stream = static_cast<hipStream_t>(hip_stream);
    c->device = dev;
    GridP &G = c->G;
    G.nx = desc->nx; G.ny = desc->ny; G.nz = desc->nz; G.nb = desc->n_bones; G.P = desc->n_poses;
    G.sy = desc->nz * 12;
    G.sx = desc->ny * desc->nz * 12;
    G.V = V;
    G.mag_ny = div_magic((unsigned)desc->ny);
    G.mag_nz = div_magic((unsigned)desc->nz);
    G.mag_V = div_magic((unsigned)V);          // n_poses * V * 12 < 2^31
    const int n[3] = {desc->nx, desc->ny, desc->nz};
    for (int a = 0; a < 3; ++a) {
        G.lo[a] = desc->lo[a];
        G.hi[a] = desc->hi[a];
        G.inv_h[a] = (float)(n[a] - 1) / (desc->hi[a] - desc->lo[a]);
        G.h[a] = (desc->hi[a] - desc->lo[a]) / (float)(n[a] - 1);
        G.m[a] = (float)(n[a] - 1);
    }
    const size_t P = desc->n_poses, nb = desc->n_bones;
    bool ok = dev_alloc(&c->T, P * V * 12) && dev_alloc(&c->Bdev, P * nb * 12) && dev_alloc(&c->Binv, P * nb * 12) &&
              dev_alloc(&c->Bok, P * nb) && dev_alloc(&c->cursor, CUR_WORDS);
    if (ok) ok = hipMemset(c->cursor, 0, CUR_WORDS * sizeof(unsigned)) == hipSuccess;
    {
        int per_cu = 0, cus = 0;
        int per_cu_ws = 0;
        // resident blocks of the LDS-grid kernel with the LDS this context's grid needs (the grid's size never changes)
        const size_t gb = (size_t)desc->n_poses * V * 48;
        if (gb > FS_LDS_GRID_MAX && gb <= FS_LDS_GRID_MAX_BIG) {
            // the device must grant one block that much LDS; else the grid is read through the caches
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_solve<true, true, FS_LDS_BIG_WAVES>, 64 * FS_LDS_BIG_WAVES, gb) != hipSuccess) per_cu = 0;
            c->lds_big = per_cu >= 1;
            (void)hipGetLastError();
            if (c->lds_big) {       // more dynamic LDS than the default limit of a block: say so for every variant
                const void *fns[] = {(const void *)k_solve<true, true, FS_LDS_BIG_WAVES>, (const void *)k_solve<true, false, FS_LDS_BIG_WAVES>,
                                     (const void *)k_solve<false, true, FS_LDS_BIG_WAVES>, (const void *)k_solve<false, false, FS_LDS_BIG_WAVES>};
                for (const void *f : fns)
                    if (hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, (int)gb) != hipSuccess) {
                        (void)hipGetLastError();
                        c->lds_big = false;
                    }
            }
            per_cu = 1;
        } else if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, k_solve<true, true>, 256, gb <= FS_LDS_GRID_MAX ? gb : 0) != hipSuccess || per_cu < 1) per_cu = 1;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_ws, k_solve_ws<true, true, FS_WS_CONSUMERS, false>, 64 * (FS_WS_CONSUMERS + 1), 0) != hipSuccess || per_cu_ws < 1) per_cu_ws = 2;
        c->occ_ws_blocks_per_cu = per_cu_ws;
        int per_cu_vx = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu_vx, k_solve_ws<true, true, FS_VX_CONSUMERS, false>, 64 * (FS_VX_CONSUMERS + 1), 0) != hipSuccess || per_cu_vx < 1) per_cu_vx = 2;
        c->occ_vx_blocks_per_cu = per_cu_vx;
        c->spin_limit = 1 << 22;   /* x about 0.2 us per poll */
        c->blocks_per_cu = 0;      /* 0: chosen per call */
        c->point_major = 1;
        c->lds_grid = 1;
        c->sort_list = 0;
        c->xcd_ranges = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
        (void)hipGetLastError();
        c->n_cus = cus;
        c->occ_blocks_per_cu = per_cu;
        c->chunk = 128;
        c->refill_min = 0;         /* 0: chosen per call */
    }
    if (ok && params->init_mode == FS_INIT_VOXEL) {
        CorrP &C = c->C;
        C.cx = params->corr_nx; C.cy = params->corr_ny; C.cz = params->corr_nz; C.ck = params->corr_k;
        C.ncell = C.cx * C.cy * C.cz;
        ok = dev_alloc(&c->Y, P * V * 3) && dev_alloc(&c->bb_ord, P * EXTENT_BLOCKS * 6) && dev_alloc(&c->bbox, P * 6) &&
             dev_alloc(&c->cell_of, P * V) && dev_alloc(&c->count, P * C.ncell + 1) && dev_alloc(&c->fill, P * V) &&
             dev_alloc(&c->order, P * V) && dev_alloc(&c->cand, P * (size_t)C.ncell * C.ck) && dev_alloc(&c->ccnt, P * (size_t)C.ncell) &&
             dev_alloc(&c->cinit, P * (size_t)C.ncell * C.ck * 4);
    }
    if (ok) {
        ok = hipHostMalloc(reinterpret_cast<void **>(&c->gave_up), sizeof(int), hipHostMallocMapped) == hipSuccess;
        if (ok) {
            *c->gave_up = 0;
            ok = hipHostGetDevicePointer(reinterpret_cast<void **>(&c->gave_up_dev), c->gave_up, 0) == hipSuccess;
        }
        if (!ok) (void)hipGetLastError();
    }
    if (!ok) {
        free_all(c);
        if (c->gave_up) (void)hipHostFree(c->gave_up);
        delete c;
        return FS_E_ALLOC;
    }
    *out = c;
    return FS_OK;
}

fs_status fs_destroy(fs_ctx *ctx)
{
    if (!ctx) return FS_OK;
    (void)hipStreamSynchronize(ctx->stream);
    if (ctx->timed) {
        for (auto &e : *ctx->timed) {
            (void)hipEventDestroy(e.first);
            (void)hipEventDestroy(e.second);
        }
        delete ctx->timed;
    }
    free_all(ctx);
    if (ctx->gave_up) (void)hipHostFree(ctx->gave_up);
    delete ctx;
    return FS_OK;
}

fs_status fs_set_params(fs_ctx *ctx, const fs_params *params)
{
    if (!ctx) return FS_E_ARG;
    if (!params) return fail(ctx, FS_E_ARG, "fs_set_params: params is NULL");
    char why[128];
    if (!params_ok(params, why, sizeof why)) return fail(ctx, FS_E_ARG, "fs_set_params: %s", why);
    ctx->prm.tol = params->tol;
    ctx->prm.div_thresh = params->div_thresh;
    ctx->prm.max_iters = params->max_iters;
    ctx->prm.grad_mode = params->grad_mode;
    return FS_OK;
}

fs_status fs_set_tuning(fs_ctx *ctx, int32_t chunk, int32_t refill_min, int32_t blocks_per_cu, int32_t point_major, int32_t lds_grid)
{
    if (!ctx) return FS_E_ARG;
    if ((chunk != 0 && (chunk < 8 || chunk > 4096)) || (refill_min != 0 && (refill_min < 1 || refill_min > 64)) ||
        blocks_per_cu < 0 || blocks_per_cu > 32 || point_major < -1 || point_major > 1 || lds_grid < -1 || lds_grid > 1)
        return fail(ctx, FS_E_ARG, "fs_set_tuning: value out of range");
    if (chunk) ctx->chunk = chunk;
    if (refill_min) ctx->refill_min = refill_min;
    if (blocks_per_cu) ctx->blocks_per_cu = blocks_per_cu;
    if (point_major >= 0) ctx->point_major = point_major;
    if (lds_grid >= 0) ctx->lds_grid = lds_grid;
    return FS_OK;
}

fs_status fs_set_list_order(fs_ctx *ctx, int32_t by_place)
{
    if (!ctx) return FS_E_ARG;
    if (by_place < 0 || by_place > 2) return fail(ctx, FS_E_ARG, "fs_set_list_order: by_place must be 0, 1 or 2");
    ctx->sort_list = by_place != 0;
    ctx->xcd_ranges = by_place == 2;
    return FS_OK;
}

fs_status fs_set_spin_limit(fs_ctx *ctx, int32_t polls)
{
    if (!ctx) return FS_E_ARG;
    if (polls < 0) return fail(ctx, FS_E_ARG, "fs_set_spin_limit: polls must be >= 0");
    ctx->spin_limit = polls;
    return FS_OK;
}

fs_status fs_precompute(fs_ctx *ctx, const float *d_W, const float *d_B)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_precompute"); if (gs != FS_OK) return gs; }
    FS_CHECK_PTR(ctx, d_W, false);
    FS_CHECK_PTR(ctx, d_B, false);
    const GridP &G = ctx->G;
    hipStream_t st = ctx->stream;
    ++ctx->pre_serial;
    const bool voxel = ctx->prm.init_mode == FS_INIT_VOXEL;
    if (voxel) {
        const int ncp0 = G.P * ctx->C.ncell;
        k_corr_reset<<<grid1d(ncp0, 256), 256, 0, st>>>(G.P, ctx->C.ncell, ctx->count);
    }
    k_precompute<<<dim3(grid1d(G.V, 256), (G.P + PRE_POSES - 1) / PRE_POSES), 256, 0, st>>>(G, d_W, d_B, ctx->T, ctx->Bdev, ctx->Binv, ctx->Bok,
                                                   reinterpret_cast<int *>(ctx->cursor + CUR_NONFINITE), ctx->pre_serial,
                                                   voxel ? ctx->Y : nullptr);
    if (voxel) {
        const CorrP &C = ctx->C;
        const int ncp = G.P * C.ncell;
        const dim3 gv(grid1d(G.V, 256), G.P);
        const int eblk = std::min(grid1d(G.V, 256), EXTENT_BLOCKS);
        k_corr_extent<<<dim3(eblk, G.P), 256, 0, st>>>(G, ctx->Y, ctx->bb_ord);
        k_corr_bbox<<<G.P, 384, 0, st>>>(eblk, ctx->bb_ord, ctx->bbox);
        k_corr_count<<<gv, 256, 0, st>>>(G, C, ctx->Y, ctx->bbox, ctx->cell_of, ctx->count, ctx->fill);
        { fs_status ss = scan_exclusive(ctx, ncp, ctx->count); if (ss != FS_OK) return ss; }
        k_corr_scatter<<<gv, 256, 0, st>>>(G, C, ctx->Y, ctx->cell_of, ctx->count, ctx->fill, ctx->order);
        k_corr_select<<<grid1d((long long)ncp * WAVE, 256), 256, 0, st>>>(G, C, ctx->Y, ctx->bbox, ctx->count, ctx->order, ctx->cand, ctx->ccnt);
        k_corr_init<<<grid1d((long long)ncp * C.ck, 256), 256, 0, st>>>(G, C, ctx->T, ctx->cand, ctx->cinit);
    }
    fs_status s = launch_status(ctx, "fs_precompute");
    if (s == FS_OK) ctx->have_T = true;
    return s;
}

fs_status fs_init(fs_ctx *ctx, const float *d_xq, const int32_t *d_pose, int64_t N, float *d_x0, float *d_Jinv0,
                  uint8_t *d_valid0)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_init"); if (gs != FS_OK) return gs; }
    if (!ctx->have_T) return fail(ctx, FS_E_STATE, "fs_init: call fs_precompute first");
    const int K = lanes_K(ctx);
    if (N < 0 || (long long)N * K >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "fs_init: need 0 <= N and K*N < 2^31");
    if (N == 0) return FS_OK;
    if (ctx->desc.n_poses > 1 && !d_pose) return fail(ctx, FS_E_ARG, "fs_init: d_pose is required when n_poses > 1");
    FS_CHECK_PTR(ctx, d_xq, false);
    FS_CHECK_PTR(ctx, d_pose, true);
    FS_CHECK_PTR(ctx, d_x0, false);
    FS_CHECK_PTR(ctx, d_Jinv0, false);
    FS_CHECK_PTR(ctx, d_valid0, false);
    const long long total = (long long)N * K;
    if (ctx->prm.init_mode == FS_INIT_BONE)
        k_init_bone<<<grid1d(total, 256), 256, 0, ctx->stream>>>(ctx->G, ctx->T, ctx->Binv, ctx->Bok, d_xq, d_pose, N,
                                                                 d_x0, d_Jinv0, d_valid0);
    else
        k_init_voxel<<<grid1d(total, 256), 256, 0, ctx->stream>>>(ctx->G, ctx->C, ctx->bbox, ctx->cinit, d_xq, d_pose, N,
                                                                  d_x0, d_Jinv0, d_valid0);
    return launch_status(ctx, "fs_init");
}

fs_status fs_solve(fs_ctx *ctx, const float *d_xq, const int32_t *d_pose, int64_t N, int32_t K, const float *d_x0,
                   const float *d_Jinv0, const uint8_t *d_valid0, float *d_xc, uint8_t *d_conv, float *d_Jinv,
                   uint8_t *d_iters, int32_t *d_slot)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_solve"); if (gs != FS_OK) return gs; }
    if (!ctx->have_T) return fail(ctx, FS_E_STATE, "fs_solve: call fs_precompute first");
    if (K != lanes_K(ctx)) return fail(ctx, FS_E_SHAPE, "fs_solve: K = %d but the init mode produces %d lanes per point", K, lanes_K(ctx));
    if (N < 0 || (long long)N * K >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "fs_solve: need 0 <= N and K*N < 2^31");
    if (N == 0) return FS_OK;
    if (ctx->desc.n_poses > 1 && !d_pose) return fail(ctx, FS_E_ARG, "fs_solve: d_pose is required when n_poses > 1");
    FS_CHECK_PTR(ctx, d_xq, false);
    FS_CHECK_PTR(ctx, d_pose, true);
    const bool fused = d_x0 == nullptr;
    if (fused && (d_Jinv0 || d_valid0))
        return fail(ctx, FS_E_ARG, "fs_solve: d_x0, d_Jinv0 and d_valid0 must be all NULL (fused initial states) or all set");
    if (!fused) {
        FS_CHECK_PTR(ctx, d_x0, false);
        FS_CHECK_PTR(ctx, d_Jinv0, false);
        FS_CHECK_PTR(ctx, d_valid0, false);
    }
    FS_CHECK_PTR(ctx, d_xc, false);
    FS_CHECK_PTR(ctx, d_conv, false);
    FS_CHECK_PTR(ctx, d_Jinv, true);
    FS_CHECK_PTR(ctx, d_iters, true);
    FS_CHECK_PTR(ctx, d_slot, true);
    SolveP S;
    S.N = N;
    S.total = (long long)N * K;
    S.max_iters = ctx->prm.max_iters;
    S.tol2 = ctx->prm.tol * ctx->prm.tol;
    S.div2 = ctx->prm.div_thresh * ctx->prm.div_thresh;
    S.K = K;
    S.point_major = ctx->point_major;
    S.chunk = ctx->chunk;
    S.spin_limit = ctx->spin_limit;
    const long long chunks = (S.total + S.chunk - 1) / S.chunk;
    const size_t grid_bytes = (size_t)ctx->G.P * ctx->G.V * 48;
    const bool lds_big = ctx->lds_grid && ctx->lds_big && grid_bytes > FS_LDS_GRID_MAX && grid_bytes <= FS_LDS_GRID_MAX_BIG;
    const bool lds = (ctx->lds_grid && grid_bytes <= FS_LDS_GRID_MAX) || lds_big;
    // Launch shape.  Grid in LDS (k_solve): latency / ALU bound, every wave the registers allow, refill at 32 idle
    // lanes.  Grid read through the caches (k_solve_ws, bound by the vector-memory path): blocks of one producer and
    // several consumers, 2 blocks per CU (measured: more waves that compute Eq. (8) only thrash the L1).
    const bool voxel_list = fused && ctx->prm.init_mode == FS_INIT_VOXEL;     // the solve draws from the list of pairs that have a candidate
    // fused voxel-based candidates: the producer only looks initial states up (k_corr_init computed them once per pose)
    const bool vx = !lds && voxel_list;
    const int wpb = lds_big ? FS_LDS_BIG_WAVES : (lds ? 4 : 1);       // waves of a block that draw chunks from the cursor
    const int auto_blocks = lds ? 3 : 2;
    const int want_blocks = ctx->blocks_per_cu ? (lds ? std::max(ctx->blocks_per_cu, 3) : ctx->blocks_per_cu) : auto_blocks;
    const int occ = lds ? ctx->occ_blocks_per_cu : (vx ? ctx->occ_vx_blocks_per_cu : ctx->occ_ws_blocks_per_cu);
    const int per_cu = lds_big ? 1 : std::max(1, std::min(want_blocks, occ));
    // consumers of k_solve_ws refill from their queue at 8 idle lanes (8 ... 24: within 1 % on grids the L2 holds; 32 and
    // more lose 3 ... 40 %); on grids beyond it at 24 (1.34 instead of 1.37 ms on the 8-pose batch; 48: 1.38)
    S.refill_min = ctx->refill_min ? ctx->refill_min : (lds ? 32 : (grid_bytes > (32u << 20) ? 24 : 8));
    S.prefetch = grid_bytes > (32u << 20);
    const int blocks = (int)std::min<long long>(grid1d(chunks, wpb), (long long)per_cu * ctx->n_cus);
    InitP I;
    I.mode = ctx->prm.init_mode;
    I.Binv = ctx->Binv;
    I.Bok = ctx->Bok;
    I.C = ctx->C;
    I.bbox = ctx->bbox;
    I.cand = ctx->cand;
    I.ccnt = ctx->ccnt;
    I.cinit = ctx->cinit;
    const bool with_J = d_Jinv != nullptr || d_slot != nullptr;     // with d_slot alone J~ stays in the result records
    const size_t need = (size_t)S.total * (with_J ? 4 : 1);
    if (need > ctx->srec_cap) {
        (void)hipStreamSynchronize(ctx->stream);
        if (ctx->srec) (void)hipFree(ctx->srec);
        ctx->srec = nullptr;
        ctx->srec_cap = 0;
        if (!dev_alloc(&ctx->srec, need)) return fail(ctx, FS_E_ALLOC, "fs_solve: out of device memory for %zu result records", (size_t)S.total);
        ctx->srec_cap = need;
    }
    hipStream_t st = ctx->stream;
    const int2 *list = nullptr;
    const int *list_len = nullptr;
    S.xcd_ranges = 0;
    if (voxel_list) {
        if ((size_t)N > ctx->vcap) {
            (void)hipStreamSynchronize(st);
            for (void *q : {(void *)ctx->voffs, (void *)ctx->vlist, (void *)ctx->vcnt, (void *)ctx->vgcell})
                if (q) (void)hipFree(q);
            ctx->voffs = ctx->vgcell = nullptr;
            ctx->vlist = nullptr;
            ctx->vcnt = nullptr;
            ctx->vcap = 0;
            if (!dev_alloc(&ctx->voffs, (size_t)N + 1) || !dev_alloc(&ctx->vlist, (size_t)N * K) ||
                !dev_alloc(&ctx->vcnt, (size_t)N) || !dev_alloc(&ctx->vgcell, (size_t)N))
                return fail(ctx, FS_E_ALLOC, "fs_solve: out of device memory for the pair list");
            ctx->vcap = (size_t)N;
        }
        k_voxel_count<<<grid1d(N, 256), 256, sizeof(float) * 6 * ctx->G.P, st>>>(ctx->G, I, N, d_xq, d_pose, ctx->voffs, ctx->vcnt, ctx->vgcell);
        // On request (fs_set_list_order) large batches are ordered by place (pose, then column of correspondence cells)
        // with a counting sort; small ones, or correspondence grids with more columns than the sort's LDS counters hold,
        // keep the order of the points.
        const int nb = ctx->G.P * ctx->C.cx * ctx->C.cy;
        const long long sblk = (N + SORT_TILE - 1) / SORT_TILE;
        const bool sorted = ctx->sort_list && N >= 4 * SORT_TILE && nb <= SORT_MAX_BUCKETS && (long long)nb * sblk < (1ll << 24);
        if (sorted) {
            const size_t need_h = (size_t)nb * sblk + 1;
            if (need_h > ctx->vhist_cap) {
                (void)hipStreamSynchronize(st);
                if (ctx->vhist) (void)hipFree(ctx->vhist);
                ctx->vhist = nullptr;
                ctx->vhist_cap = 0;
                if (!dev_alloc(&ctx->vhist, need_h)) return fail(ctx, FS_E_ALLOC, "fs_solve: out of device memory for the pair list");
                ctx->vhist_cap = need_h;
            }
            k_sort_hist<<<(unsigned)sblk, 1024, nb * sizeof(int), st>>>(N, ctx->C.cz, nb, ctx->vgcell, ctx->vcnt, ctx->vhist);
            { fs_status ss = scan_exclusive(ctx, (int)((long long)nb * sblk), ctx->vhist); if (ss != FS_OK) return ss; }
            k_sort_scatter<<<(unsigned)sblk, 1024, nb * sizeof(int), st>>>(N, ctx->C.cz, nb, ctx->vgcell, ctx->vcnt, ctx->vhist, ctx->vlist);
            list_len = ctx->vhist + (long long)nb * sblk;
            S.xcd_ranges = (!lds && ctx->xcd_ranges) ? 1 : 0;
        } else {
            { fs_status ss = scan_exclusive(ctx, (int)N, ctx->voffs); if (ss != FS_OK) return ss; }
            k_voxel_expand<<<grid1d(N, 256), 256, 0, st>>>(N, ctx->voffs, ctx->vgcell, ctx->vlist);
            list_len = ctx->voffs + N;
        }
        list = ctx->vlist;
    }
    const int ncell = (ctx->G.nx - 1) * (ctx->G.ny - 1) * (ctx->G.nz - 1);
    int *cell_count = nullptr;
    ctx->slots_N = 0;
    // every wave that draws chunks (all four of a k_solve block, the producer of a k_solve_ws block) owns the
    // chunk of its own number to begin with; the shared cursor starts behind those
    const unsigned drawers = (unsigned)(blocks * wpb);
    if (d_slot) {
        const long long ncp = (long long)ctx->G.P * ncell;
        if (ncp + 1 >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "fs_solve: too many grid cells for d_slot");
        if (!ctx->gcount_solve && !dev_alloc(&ctx->gcount_solve, (size_t)ncp + 1)) return fail(ctx, FS_E_ALLOC, "fs_solve: out of device memory");
        k_fill_zero_i32<<<(int)std::min<long long>(grid1d(ncp + 1, 256), 4096), 256, 0, st>>>(ncp + 1, ctx->gcount_solve, ctx->cursor, drawers, (unsigned)S.chunk);
        cell_count = ctx->gcount_solve;
    } else {
        k_reset_cursor<<<1, 64, 0, st>>>(ctx->cursor, drawers, (unsigned)S.chunk);
    }
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    if (ctx->timing && hipEventCreate(&ev0) == hipSuccess && hipEventCreate(&ev1) == hipSuccess) (void)hipEventRecord(ev0, st);
    if (lds) {
#define FS_LAUNCH_SOLVE(F, J, NW)                                                                                      \
    k_solve<F, J, NW><<<dim3(blocks), dim3(NW * WAVE), grid_bytes, st>>>(ctx->G, S, I, ctx->T, d_xq, d_pose, d_x0,     \
                                                                         d_Jinv0, d_valid0, ctx->srec, ctx->cursor,    \
                                                                         list, list_len, cell_count, ncell)
        if (lds_big) {
            if (fused && with_J) FS_LAUNCH_SOLVE(true, true, FS_LDS_BIG_WAVES);
            else if (fused) FS_LAUNCH_SOLVE(true, false, FS_LDS_BIG_WAVES);
            else if (with_J) FS_LAUNCH_SOLVE(false, true, FS_LDS_BIG_WAVES);
            else FS_LAUNCH_SOLVE(false, false, FS_LDS_BIG_WAVES);
        } else {
            if (fused && with_J) FS_LAUNCH_SOLVE(true, true, 4);
            else if (fused) FS_LAUNCH_SOLVE(true, false, 4);
            else if (with_J) FS_LAUNCH_SOLVE(false, true, 4);
            else FS_LAUNCH_SOLVE(false, false, 4);
        }
#undef FS_LAUNCH_SOLVE
    } else {
#define FS_LAUNCH_SOLVE(F, J, NC, Z)                                                                                   \
    k_solve_ws<F, J, NC, Z><<<dim3(blocks), dim3((NC + 1) * WAVE), 0, st>>>(                                           \
        ctx->G, S, I, ctx->T, d_xq, d_pose, d_x0, d_Jinv0, d_valid0, ctx->srec, ctx->cursor, list, list_len, cell_count,  \
        ncell, ctx->gave_up_dev, reinterpret_cast<const int *>(ctx->cursor + CUR_NONFINITE), ctx->pre_serial)
        // Z = true: contexts with one state per bone.  Many of those lanes start outside the box (51 % of the
        // evaluations on the SMPL-scale scene have a clamped coordinate): the consumers skip the corner records of
        // weight zero (kernel -8 %).  Z = false: voxel-based candidates, which start inside it, where the bookkeeping
        // costs more than it saves (+15 %); with fused initial states the producer reads them from the table
        const bool skip = ctx->prm.init_mode == FS_INIT_BONE;
        if (skip) {
            if (fused && with_J) FS_LAUNCH_SOLVE(true, true, FS_WS_CONSUMERS, true);
            else if (fused) FS_LAUNCH_SOLVE(true, false, FS_WS_CONSUMERS, true);
            else if (with_J) FS_LAUNCH_SOLVE(false, true, FS_WS_CONSUMERS, true);
            else FS_LAUNCH_SOLVE(false, false, FS_WS_CONSUMERS, true);
        } else {
            if (fused && with_J) FS_LAUNCH_SOLVE(true, true, FS_VX_CONSUMERS, false);
            else if (fused) FS_LAUNCH_SOLVE(true, false, FS_VX_CONSUMERS, false);
            else if (with_J) FS_LAUNCH_SOLVE(false, true, FS_WS_CONSUMERS, false);
            else FS_LAUNCH_SOLVE(false, false, FS_WS_CONSUMERS, false);
        }
#undef FS_LAUNCH_SOLVE
    }
    if (ev0 && ev1) {
        (void)hipEventRecord(ev1, st);
        ctx->timed->emplace_back(ev0, ev1);
    }
    const dim3 ub(grid1d(N, 256), K);       // one thread per pair: x = point, y = initial state
    if (with_J && voxel_list)
        k_solve_unpack<true, true><<<ub, 256, 0, st>>>(N, S.total, ctx->vcnt, ctx->srec, d_xc, d_conv, d_Jinv, d_iters, d_slot);
    else if (with_J)
        k_solve_unpack<true, false><<<ub, 256, 0, st>>>(N, S.total, nullptr, ctx->srec, d_xc, d_conv, d_Jinv, d_iters, d_slot);
    else if (voxel_list)
        k_solve_unpack<false, true><<<ub, 256, 0, st>>>(N, S.total, ctx->vcnt, ctx->srec, d_xc, d_conv, d_Jinv, d_iters, d_slot);
    else
        k_solve_unpack<false, false><<<ub, 256, 0, st>>>(N, S.total, nullptr, ctx->srec, d_xc, d_conv, d_Jinv, d_iters, d_slot);
    fs_status lst = launch_status(ctx, "fs_solve");
    if (lst == FS_OK && d_slot) {
        ctx->slots_N = N;
        ctx->slots_K = K;
        ctx->slots_list = list != nullptr;
    }
    return lst;
}

fs_status fs_grad(fs_ctx *ctx, const float *d_W, const float *d_xc, const float *d_Jinv, const uint8_t *d_conv,
                  const float *d_gxc, const int32_t *d_pose, int64_t N, int32_t K, const int32_t *d_slot, float *d_gW,
                  float *d_gB, float *d_gxq)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_grad"); if (gs != FS_OK) return gs; }
    if (!ctx->have_T) return fail(ctx, FS_E_STATE, "fs_grad: call fs_precompute first");
    if (K < 1 || K > FS_MAX_BONES) return fail(ctx, FS_E_SHAPE, "fs_grad: K out of range");
    if (N < 0 || (long long)N * K >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "fs_grad: need 0 <= N and K*N < 2^31");
    if (ctx->desc.n_poses > 1 && !d_pose && N > 0) return fail(ctx, FS_E_ARG, "fs_grad: d_pose is required when n_poses > 1");
    const int mode = ctx->prm.grad_mode;
    FS_CHECK_PTR(ctx, d_W, false);
    FS_CHECK_PTR(ctx, d_gW, false);
    FS_CHECK_PTR(ctx, d_gB, false);
    FS_CHECK_PTR(ctx, d_gxq, true);
    if (N > 0) {
        FS_CHECK_PTR(ctx, d_xc, false);
        FS_CHECK_PTR(ctx, d_Jinv, mode == FS_GRAD_EXACT_J || d_slot != nullptr);
        FS_CHECK_PTR(ctx, d_conv, false);
        FS_CHECK_PTR(ctx, d_gxc, false);
        FS_CHECK_PTR(ctx, d_pose, true);
    }
    FS_CHECK_PTR(ctx, d_slot, true);
    if (d_slot && (ctx->slots_N != N || ctx->slots_K != K || N == 0))
        return fail(ctx, FS_E_STATE, "fs_grad: d_slot must come from the last fs_solve on this context with the same N and K");
    const bool from_rec = d_slot != nullptr;
    const GridP &G = ctx->G;
    const int ncell = (G.nx - 1) * (G.ny - 1) * (G.nz - 1);
    const long long ncp = (long long)G.P * ncell;
    if (ncp + 1 >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "fs_grad: too many grid cells");
    if (!ctx->GT && !dev_alloc(&ctx->GT, (size_t)G.P * G.V * 12)) return fail(ctx, FS_E_ALLOC, "fs_grad: out of device memory");
    if (!ctx->gcount && !dev_alloc(&ctx->gcount, (size_t)ncp + 1)) return fail(ctx, FS_E_ALLOC, "fs_grad: out of device memory");
    if (!ctx->gpart) {
        ctx->gb_blocks = (int)std::min<long long>(grid1d(G.V, 256), 1024);      // 4 waves each, >= 16 node quads per wave
        if (!dev_alloc(&ctx->gpart, (size_t)G.P * ctx->gb_blocks * G.nb * 12)) return fail(ctx, FS_E_ALLOC, "fs_grad: out of device memory");
    }
    const size_t lanes = (size_t)N * K;
    if (lanes > ctx->gcap) {
        (void)hipStreamSynchronize(ctx->stream);
        if (ctx->gpos) (void)hipFree(ctx->gpos);
        if (ctx->grec) (void)hipFree(ctx->grec);
        ctx->gpos = nullptr; ctx->grec = nullptr; ctx->gcap = 0;
        if (!dev_alloc(&ctx->gpos, lanes) || !dev_alloc(&ctx->grec, std::max<size_t>(lanes, PIECE_MIN) * GREC))
            return fail(ctx, FS_E_ALLOC, "fs_grad: out of device memory for %zu lanes", lanes);
        ctx->gcap = lanes;
    }
    hipStream_t st = ctx->stream;
    const int *pos = ctx->gpos, *counts = nullptr;
    if (d_slot) {
        // the solve already counted its converged lanes per cell and gave each its slot; its counts are
        // left as they are, so the backward can be repeated
        pos = d_slot;
        counts = ctx->gcount_solve;
    } else {
        k_fill_zero_i32<<<(int)std::min<long long>(grid1d(ncp + 1, 256), 4096), 256, 0, st>>>(ncp + 1, ctx->gcount);
        if (N > 0) k_grad_count<<<grid1d((long long)N * K, 256), 256, 0, st>>>(G, d_xc, d_conv, d_pose, N, K, ncell, ctx->gcount, ctx->gpos);
    }
    { fs_status ss = scan_exclusive(ctx, (int)ncp, ctx->gcount, counts); if (ss != FS_OK) return ss; }
    if (N > 0) {
        // small batches: several threads share a point's lanes so that the chip has enough threads in flight
        const int groups = N >= (1 << 19) ? 1 : (K >= 8 ? 8 : (K >= 4 ? 4 : (K >= 2 ? 2 : 1)));
        const dim3 rg(grid1d(N, 256 / groups));
        float4 *grec4 = reinterpret_cast<float4 *>(ctx->grec);
#define FS_LAUNCH_RECORDS(R, E)                                                                                       \
    k_grad_records<R, E><<<rg, 256, 0, st>>>(G, ctx->T, d_xc, d_Jinv, d_conv, d_gxc, d_pose, N, K, ncell, ctx->gcount, pos, \
                                             grec4, d_gxq, groups, (R) ? ctx->srec : nullptr,                          \
                                             ((R) && ctx->slots_list) ? ctx->vcnt : nullptr)
        // from_rec: the solve's own result records are still in the context: one 64-byte read per pair
        if (from_rec && mode != 0) FS_LAUNCH_RECORDS(true, true);
        else if (from_rec && groups == 1)     // large batches: three lanes of a point in flight, stage by stage
            k_grad_records<true, false, 3><<<rg, 256, 0, st>>>(G, ctx->T, d_xc, d_Jinv, d_conv, d_gxc, d_pose, N, K, ncell, ctx->gcount,
                                                               pos, grec4, d_gxq, groups, ctx->srec, ctx->slots_list ? ctx->vcnt : nullptr);
        else if (from_rec) FS_LAUNCH_RECORDS(true, false);
        else if (mode != 0) FS_LAUNCH_RECORDS(false, true);
        else FS_LAUNCH_RECORDS(false, false);
#undef FS_LAUNCH_RECORDS
    }
    if (N > 0) k_grad_pieces<<<grid1d((long long)lanes, PIECE_R), 64 * PIECE_WAVES, 0, st>>>(G, ncp, ctx->gcount, ctx->grec);
    // crowded grids: one thread per (node, adjacent cell); sparse ones: one thread per node, which walks the 4 cells at
    // its height and hands their share for the node above to the next SIMD lane
    const long long nodes = (long long)G.P * G.V;
    if ((long long)lanes >= FS_TPN8_AT * nodes)
        k_grad_nodes_p<8><<<grid1d(nodes * 8, 256), 256, 0, st>>>(G, ncell, ctx->gcount, ctx->grec, ctx->GT);
    else
        k_grad_nodes_z<<<grid1d(nodes, 256), 256, 0, st>>>(G, ncell, ctx->gcount, ctx->grec, ctx->GT);
    // (dL/dW on a second stream beside dL/dB, joined before the call returns: both kernels then take twice as long,
    // 156 + 132 us instead of 77 + 79 on the 8-pose grid, and the step gains nothing.)
    k_grad_weights_node<<<grid1d(G.V * ((G.nb + 7) / 8), 256), 256, sizeof(float) * G.P * G.nb * 12, st>>>(G, ctx->GT, ctx->Bdev, d_gW);
    const int nout = G.nb * 12, nparts = ctx->gb_blocks * 4;
    const dim3 gbg(ctx->gb_blocks, (G.P + GB_POSES - 1) / GB_POSES);
    switch ((G.nb + 15) / 16) {
    case 1: k_grad_bones_mfma<1><<<gbg, 256, 0, st>>>(G, d_W, ctx->GT, ctx->gpart, nparts); break;
    case 2: k_grad_bones_mfma<2><<<gbg, 256, 0, st>>>(G, d_W, ctx->GT, ctx->gpart, nparts); break;
    case 3: k_grad_bones_mfma<3><<<gbg, 256, 0, st>>>(G, d_W, ctx->GT, ctx->gpart, nparts); break;
    default: k_grad_bones_mfma<4><<<gbg, 256, 0, st>>>(G, d_W, ctx->GT, ctx->gpart, nparts); break;
    }
    k_grad_bones_final<<<G.P * nout, 64, 0, st>>>(G.P, ctx->gb_blocks, nout, ctx->gpart, d_gB);
    return launch_status(ctx, "fs_grad");
}

// shared body of fs_dedupe and fs_dedupe_noalloc: `sums` = nullptr: the tile sums of the scan live in the context's
// buffer, which grows on demand; otherwise they live in `sums` (room for FS_NOALLOC_TILES) and nothing is allocated
static fs_status dedupe_impl(fs_ctx *ctx, const char *who, int *sums, const float *d_xc, const uint8_t *d_conv, int64_t N,
                             int32_t K, float min_dist, uint8_t *d_keep, int32_t *d_offsets, float *d_roots, int32_t *d_lane,
                             int64_t cap)
{
    if (K < 1 || K > FS_MAX_BONES) return fail(ctx, FS_E_SHAPE, "%s: K must be in 1..%d", who, (int)FS_MAX_BONES);
    if (N < 0 || (long long)N * K >= (1ll << 31)) return fail(ctx, FS_E_SHAPE, "%s: need 0 <= N and K*N < 2^31", who);
    if (sums && N > FS_NOALLOC_MAX_N)
        return fail(ctx, FS_E_SHAPE, "%s: N = %lld exceeds the %lld points its fixed scratch memory is sized for; use fs_dedupe",
                    who, (long long)N, FS_NOALLOC_MAX_N);
    if (!(min_dist >= 0.0f) || !std::isfinite(min_dist)) return fail(ctx, FS_E_ARG, "%s: min_dist must be finite and >= 0", who);
    if (cap < 0) return fail(ctx, FS_E_SHAPE, "%s: cap must be >= 0", who);
    FS_CHECK_PTR(ctx, d_offsets, false);
    FS_CHECK_PTR(ctx, d_roots, true);
    FS_CHECK_PTR(ctx, d_lane, true);
    hipStream_t st = ctx->stream;
    if (N > 0) {
        FS_CHECK_PTR(ctx, d_xc, false);
        FS_CHECK_PTR(ctx, d_conv, false);
        FS_CHECK_PTR(ctx, d_keep, false);
        k_dedupe<<<grid1d(N, 256), 256, 0, st>>>(N, K, min_dist * min_dist, d_xc, d_conv, d_keep, d_offsets);
    }
    if (sums) {
        // at most FS_NOALLOC_TILES tiles: every block of the second pass adds up the tile sums before its own, all
        // of which the first pass has just written (nothing of an earlier call is read)
        if (N > 0) {
            const int m = (int)((N + SCAN_TILE - 1) / SCAN_TILE);
            k_scan_tile_sums<<<m, 1024, 0, st>>>((int)N, d_offsets, sums);
            k_scan_tiles<false><<<m, 1024, 0, st>>>((int)N, d_offsets, d_offsets, sums, m, nullptr);
        } else {
            k_fill_zero_i32<<<1, 64, 0, st>>>(1, d_offsets, nullptr);
        }
    } else {
        fs_status ss = scan_exclusive(ctx, (int)N, d_offsets);
        if (ss != FS_OK) return ss;
    }
    if (N > 0 && (d_roots || d_lane))
        k_pack_roots<<<grid1d(N, 256), 256, 0, st>>>(N, K, cap, d_xc, d_keep, d_offsets, d_roots, d_lane);
    return launch_status(ctx, who);
}

fs_status fs_dedupe(fs_ctx *ctx, const float *d_xc, const uint8_t *d_conv, int64_t N, int32_t K, float min_dist,
                    uint8_t *d_keep, int32_t *d_offsets, float *d_roots, int32_t *d_lane, int64_t cap)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_dedupe"); if (gs != FS_OK) return gs; }
    return dedupe_impl(ctx, "fs_dedupe", nullptr, d_xc, d_conv, N, K, min_dist, d_keep, d_offsets, d_roots, d_lane, cap);
}

fs_status fs_dedupe_noalloc(fs_ctx *ctx, const float *d_xc, const uint8_t *d_conv, int64_t N, int32_t K, float min_dist,
                            uint8_t *d_keep, int32_t *d_offsets, float *d_roots, int32_t *d_lane, int64_t cap)
{
    if (!ctx) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_dedupe_noalloc"); if (gs != FS_OK) return gs; }
    int *sums = scratch_on_device(ctx);
    if (!sums) return fail(ctx, FS_E_DEVICE, "fs_dedupe_noalloc: the address of the library's scratch array could not be obtained "
                                             "(the context's device must be the current one)");
    return dedupe_impl(ctx, "fs_dedupe_noalloc", sums, d_xc, d_conv, N, K, min_dist, d_keep, d_offsets, d_roots, d_lane, cap);
}

fs_status fs_set_timing(fs_ctx *ctx, int32_t enable)
{
    if (!ctx) return FS_E_ARG;
    if (enable && !ctx->timed) {
        ctx->timed = new (std::nothrow) std::vector<std::pair<hipEvent_t, hipEvent_t>>();
        if (!ctx->timed) return fail(ctx, FS_E_ALLOC, "fs_set_timing: out of host memory");
    }
    ctx->timing = enable != 0;
    return FS_OK;
}

fs_status fs_get_timing(fs_ctx *ctx, double *solve_kernel_ms, int32_t *launches)
{
    if (!ctx || !solve_kernel_ms || !launches) return FS_E_ARG;
    { fs_status gs = check_gave_up(ctx, "fs_get_timing"); if (gs != FS_OK) return gs; }
    *solve_kernel_ms = 0.0;
    *launches = 0;
    if (!ctx->timed) return FS_OK;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return launch_status(ctx, "fs_get_timing");
    for (auto &e : *ctx->timed) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, e.first, e.second) == hipSuccess) {
            *solve_kernel_ms += ms;
            ++*launches;
        }
        (void)hipEventDestroy(e.first);
        (void)hipEventDestroy(e.second);
    }
    (void)hipGetLastError();
    ctx->timed->clear();
    return FS_OK;
}

fs_status fs_get_transforms(fs_ctx *ctx, float *d_T)
{
    if (!ctx) return FS_E_ARG;
    if (!ctx->have_T) return fail(ctx, FS_E_STATE, "fs_get_transforms: call fs_precompute first");
    FS_CHECK_PTR(ctx, d_T, false);
    if (hipMemcpyAsync(d_T, ctx->T, sizeof(float) * ctx->G.P * ctx->G.V * 12, hipMemcpyDeviceToDevice, ctx->stream) != hipSuccess)
        return launch_status(ctx, "fs_get_transforms");
    return FS_OK;
}

fs_status fs_get_corr(fs_ctx *ctx, float *d_bbox, int32_t *d_cand)
{
    if (!ctx) return FS_E_ARG;
    if (ctx->prm.init_mode != FS_INIT_VOXEL) return fail(ctx, FS_E_STATE, "fs_get_corr: context was not created with FS_INIT_VOXEL");
    if (!ctx->have_T) return fail(ctx, FS_E_STATE, "fs_get_corr: call fs_precompute first");
    FS_CHECK_PTR(ctx, d_bbox, false);
    FS_CHECK_PTR(ctx, d_cand, false);
    hipError_t e = hipMemcpyAsync(d_bbox, ctx->bbox, sizeof(float) * ctx->G.P * 6, hipMemcpyDeviceToDevice, ctx->stream);
    if (e == hipSuccess)
        e = hipMemcpyAsync(d_cand, ctx->cand, sizeof(int32_t) * ctx->G.P * (size_t)ctx->C.ncell * ctx->C.ck,
                           hipMemcpyDeviceToDevice, ctx->stream);
    if (e != hipSuccess) return launch_status(ctx, "fs_get_corr");
    return FS_OK;
}

}  // extern "C"
