// HIP kernels of the articulation path for gfx950 (wave64).
#pragma once
#include "fs_field.hpp"

namespace fs {

constexpr int WAVE = 64;

// pose index of point n, forced into [0, P) so that a bad index in the caller's array cannot send
// a kernel outside the transform grids
__device__ __forceinline__ int pose_of(const int32_t *__restrict__ pose, long long n, int P)
{
    if (!pose) return 0;
    const int p = pose[n];
    return p < 0 ? 0 : (p >= P ? P - 1 : p);
}
constexpr int FS_MAX_CORR_K_DEV = 8;

// ------------------------------------------------------------------------------------------------
// Pre-computed LBS (Eq. (13)): one thread per node, all poses.  The bone transforms are read with
// wave-uniform addresses, i.e. through the scalar cache into SGPR operands of the multiply-adds.
// Reads W once (96 B / node for 24 bones), writes 48 B per node and pose.
// ------------------------------------------------------------------------------------------------
// Every lane of a wave holds one row of NF floats (NF = 12: a 48-byte record; NF = 3: a point) of a tile whose rows are
// contiguous in memory (row r of the wave's tile at dst + r * NF).  Stored straight from registers, a row goes out as
// 16-byte pieces at a 48-byte stride: partial writes of cache lines, for which the L2 first fetches the line (on the
// 8-pose 128x128x32 grid k_precompute fetched 386 MB to read 50 MB of weights).  Through LDS the tile leaves as whole,
// consecutive 16-byte pieces from consecutive lanes.  nrows = valid rows of the wave's tile (wave-uniform; <= 0: none).
// s_tile: 64 * NF floats of LDS that belong to this wave alone, so no barrier between waves is needed; all 64 lanes
// must call.
template <int NF>
__device__ __forceinline__ void wave_store_rows(float *__restrict__ dst, const float (&v)[NF], int nrows, float *s_tile)
{
    const int lane = threadIdx.x & 63;
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // s_tile may still be read from the call before
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int e = 0; e < NF; ++e) s_tile[lane * NF + e] = v[e];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
    __builtin_amdgcn_wave_barrier();
    const int n4 = nrows * NF / 4, tail = nrows * NF - n4 * 4;
    if ((reinterpret_cast<uintptr_t>(dst) & 15u) == 0) {
        for (int i = lane; i < n4; i += 64)
            reinterpret_cast<float4 *>(dst)[i] = reinterpret_cast<const float4 *>(s_tile)[i];
        if (lane < tail) dst[n4 * 4 + lane] = s_tile[n4 * 4 + lane];
    } else {
        for (int i = lane; i < nrows * NF; i += 64) dst[i] = s_tile[i];
    }
}

__device__ __forceinline__ void bone_inverse(int i, const float *__restrict__ B, float *__restrict__ Bcopy,
                                             float *__restrict__ Binv, uint8_t *__restrict__ ok);

// monotone float <-> uint mapping so that min / max can use integer atomics (exact, order-free)
__device__ __forceinline__ unsigned f2ord(float f)
{
    const unsigned u = __float_as_uint(f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float ord2f(unsigned o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7fffffffu) : ~o);
}

// The first n_poses*n_bones threads also invert their bone's linear part for Eq. (8) and keep a copy
// of the bone transforms for the backward.
// Y (may be null; voxel-based initial states): the image y_v = T_v x_v of every node is written as well -- the
// correspondence grid is built on those, and the transforms are in registers here anyway (a pass of its own would
// read all of T again).
#ifndef FS_PRE_POSES
#define FS_PRE_POSES 4
#endif
constexpr int PRE_POSES = FS_PRE_POSES;     // poses that share one pass over a node's weights (8-pose grid: 2 -> 144 us, 4 -> 105, 8 -> 138)
__global__ __launch_bounds__(256) void k_precompute(GridP G, const float *__restrict__ W,
                                                    const float *__restrict__ B, float *__restrict__ T,
                                                    float *__restrict__ Bcopy, float *__restrict__ Binv,
                                                    uint8_t *__restrict__ Bok, int *__restrict__ nonfinite,
                                                    int serial, float *__restrict__ Y)
{
    // *nonfinite = serial (the number of this call) tells the solve that this grid holds an entry that is not
    // finite: a record with weight zero may then not be skipped (0 * inf is not 0)
    __shared__ __attribute__((aligned(16))) float s_tiles[4][64 * 12];
    float *s_tile = s_tiles[threadIdx.x >> 6];
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x, v0 = v - (threadIdx.x & 63);   // v0: the wave's first node
    if (blockIdx.y == 0)
        for (long long i = v; i < (long long)G.P * G.nb; i += (long long)gridDim.x * blockDim.x)
            bone_inverse((int)i, B, Bcopy, Binv, Bok);
    const bool live = v < G.V;                   // the last wave: its other lanes stay for the wave-wide stores
    const int nrows = (int)min(64ll, G.V - v0);
    const float *w = W + (live ? v : 0) * G.nb;
    const bool vec = (G.nb & 3) == 0;        // weight rows are 16-byte aligned: read them four at a time
    float xv[3] = {0.0f, 0.0f, 0.0f};
    if (Y && live) node_pos(G, v, xv);
    // four poses share one pass over the node's weights; per pose the sum runs over the bones in order,
    // first term a product, the rest fused multiply-adds
    // blockIdx.y = group of PRE_POSES poses: twice the waves of one block per node tile, in different phases of
    // load, arithmetic and store at any one time
    for (int p0 = blockIdx.y * PRE_POSES; p0 < G.P; p0 += gridDim.y * PRE_POSES) {
        const int np = min(PRE_POSES, G.P - p0);
        float acc[PRE_POSES][12];
#pragma unroll
        for (int q = 0; q < PRE_POSES; ++q)
#pragma unroll
            for (int e = 0; e < 12; ++e) acc[q][e] = 0.0f;
        if (live) {
            for (int b0 = 0; b0 < G.nb; b0 += 4) {
                float wv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
                if (vec) {
                    const float4 w4 = *reinterpret_cast<const float4 *>(w + b0);
                    wv[0] = w4.x; wv[1] = w4.y; wv[2] = w4.z; wv[3] = w4.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (b0 + j < G.nb) wv[j] = w[b0 + j];
                }
#pragma unroll
                for (int q = 0; q < PRE_POSES; ++q) {
                    if (q < np) {
                        const float *Bp = B + (long long)(p0 + q) * G.nb * 12;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            if (b0 + j < G.nb) {
                                if (b0 == 0 && j == 0) {
#pragma unroll
                                    for (int e = 0; e < 12; ++e) acc[q][e] = wv[0] * Bp[e];
                                } else {
#pragma unroll
                                    for (int e = 0; e < 12; ++e) acc[q][e] = FS_FMA(wv[j], Bp[(b0 + j) * 12 + e], acc[q][e]);
                                }
                            }
                        }
                    }
                }
            }
        }
#pragma unroll
        for (int q = 0; q < PRE_POSES; ++q) {
            if (q < np) {                        // wave-uniform
                if (live) {
                    float big = 0.0f;
#pragma unroll
                    for (int e = 0; e < 12; ++e) big = __builtin_fmaxf(big, __builtin_fabsf(acc[q][e]) < __builtin_inff() ? 0.0f : 1.0f);
                    if (big != 0.0f) *nonfinite = serial;
                }
                wave_store_rows<12>(T + ((long long)(p0 + q) * G.V + v0) * 12, acc[q], nrows, s_tile);
                if (Y) {
                    float y[3] = {0.0f, 0.0f, 0.0f};
                    if (live) apply12(acc[q], xv, y);
                    wave_store_rows<3>(Y + ((long long)(p0 + q) * G.V + v0) * 3, y, nrows, s_tile);
                }
            }
        }
    }
}

// Inverse of one bone's linear part for Eq. (8): Binv [P][nb][12] = 9 inverse entries + t, ok flag.
__device__ __forceinline__ void bone_inverse(int i, const float *__restrict__ B, float *__restrict__ Bcopy,
                                             float *__restrict__ Binv, uint8_t *__restrict__ ok)
{
    const float *b = B + i * 12;
    for (int e = 0; e < 12; ++e) Bcopy[i * 12 + e] = b[e];
    const float R[9] = {b[0], b[1], b[2], b[4], b[5], b[6], b[8], b[9], b[10]};
    float Ri[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    const bool good = inv3(R, Ri);
    for (int e = 0; e < 9; ++e) Binv[i * 12 + e] = Ri[e];
    Binv[i * 12 + 9] = b[3];
    Binv[i * 12 + 10] = b[7];
    Binv[i * 12 + 11] = b[11];
    ok[i] = good ? 1 : 0;
}

// ------------------------------------------------------------------------------------------------
// Initial states.  One thread per lane q = k*N + n.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void write_init(long long q, long long N, int k, long long n, const float x0[3],
                                           const float Ji[9], bool ok, float *__restrict__ o_x0,
                                           float *__restrict__ o_J, uint8_t *__restrict__ o_v)
{
#pragma unroll
    for (int r = 0; r < 3; ++r) o_x0[((long long)k * 3 + r) * N + n] = x0[r];
#pragma unroll
    for (int e = 0; e < 9; ++e) o_J[((long long)k * 9 + e) * N + n] = ok ? Ji[e] : 0.0f;
    o_v[q] = ok ? 1 : 0;
}

__global__ __launch_bounds__(256) void k_init_bone(GridP G, const float *__restrict__ T,
                                                   const float *__restrict__ Binv, const uint8_t *__restrict__ Bok,
                                                   const float *__restrict__ xq, const int32_t *__restrict__ pose,
                                                   long long N, float *__restrict__ o_x0, float *__restrict__ o_J,
                                                   uint8_t *__restrict__ o_v)
{
    const long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= N * G.nb) return;
    const int k = (int)(q / N);
    const long long n = q - (long long)k * N;
    const int p = pose_of(pose, n, G.P);
    const float *bi = Binv + ((long long)p * G.nb + k) * 12;
    float x0[3] = {0, 0, 0}, Ji[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    bool ok = Bok[p * G.nb + k] != 0;
    if (ok) {
        const float y[3] = {xq[n] - bi[9], xq[N + n] - bi[10], xq[2 * N + n] - bi[11]};
#pragma unroll
        for (int r = 0; r < 3; ++r)
            x0[r] = FS_FMA(bi[r * 3 + 0], y[0], FS_FMA(bi[r * 3 + 1], y[1], bi[r * 3 + 2] * y[2]));
        float d[3], J[9];
        field_dJ(T + (long long)p * G.V * 12, G, x0, d, J);
        ok = inv3(J, Ji);
    }
    write_init(q, N, k, n, x0, Ji, ok, o_x0, o_J, o_v);
}

struct CorrP {
    int cx, cy, cz, ck;
    int ncell;
};

__device__ __forceinline__ int cell_coord(float y, float blo, float cs, int n)
{
    if (!(cs > 0.0f)) return 0;
    float t = (y - blo) / cs;
    if (!(t >= 0.0f)) t = 0.0f;
    if (t > (float)(n - 1)) t = (float)(n - 1);
    return (int)t;
}

__device__ __forceinline__ int cell_index(const CorrP &C, const float *__restrict__ bb, const float y[3])
{
    const float cs0 = (bb[3] - bb[0]) / (float)C.cx;
    const float cs1 = (bb[4] - bb[1]) / (float)C.cy;
    const float cs2 = (bb[5] - bb[2]) / (float)C.cz;
    return (cell_coord(y[0], bb[0], cs0, C.cx) * C.cy + cell_coord(y[1], bb[1], cs1, C.cy)) * C.cz +
           cell_coord(y[2], bb[2], cs2, C.cz);
}

__global__ __launch_bounds__(256) void k_init_voxel(GridP G, CorrP C, const float *__restrict__ bbox,
                                                    const float4 *__restrict__ cinit, const float *__restrict__ xq,
                                                    const int32_t *__restrict__ pose, long long N,
                                                    float *__restrict__ o_x0, float *__restrict__ o_J,
                                                    uint8_t *__restrict__ o_v)
{
    // the candidate's initial state was computed once per pose by k_corr_init
    const long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= N * C.ck) return;
    const int k = (int)(q / N);
    const long long n = q - (long long)k * N;
    const int p = pose_of(pose, n, G.P);
    const float y[3] = {xq[n], xq[N + n], xq[2 * N + n]};
    const int cell = cell_index(C, bbox + p * 6, y);
    const float4 *ci = cinit + (((long long)p * C.ncell + cell) * C.ck + k) * 4;
    const float4 a = ci[0], b = ci[1], c = ci[2], d = ci[3];
    const float x0[3] = {a.x, a.y, a.z};
    const float Ji[9] = {b.w, c.x, c.y, c.z, c.w, d.x, d.y, d.z, d.w};
    write_init(q, N, k, n, x0, Ji, (__float_as_int(a.w) & 1) != 0, o_x0, o_J, o_v);
}

// ------------------------------------------------------------------------------------------------
// Correspondence grid build (voxel-based initialisation).
// ------------------------------------------------------------------------------------------------
__global__ void k_corr_reset(int P, int ncell, int *__restrict__ count)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < P * ncell) count[i] = 0;
    if (i == 0) count[P * ncell] = 0;
}

// Bounding box per pose of the images of all nodes, in two steps without atomics: every block leaves the extent of its
// share of the nodes in bb_part[p][block][6] (ordered-integer images of the floats: min x, y, z, max x, y, z), then one
// wave per pose and entry reduces the blocks' values.  (With atomicMin / atomicMax on the 6 words of a pose -- all in
// one cache line -- the atomics were the cost of the kernel: about 3 ns each, 37 of its 40 us on the 8-pose grid with
// 256 blocks per pose, 145 us with 1024.)
constexpr int EXTENT_BLOCKS = 512;      // blocks per pose at most
__global__ __launch_bounds__(256) void k_corr_extent(GridP G, const float *__restrict__ Y, unsigned *__restrict__ bb_part)
{
    __shared__ unsigned smn[4][3], smx[4][3];
    const int p = blockIdx.y;
    unsigned mn[3] = {0xffffffffu, 0xffffffffu, 0xffffffffu}, mx[3] = {0u, 0u, 0u};
    for (long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x; v < G.V; v += (long long)gridDim.x * blockDim.x) {
        const float *y = Y + ((long long)p * G.V + v) * 3;
#pragma unroll
        for (int a = 0; a < 3; ++a) {
            const unsigned ov = f2ord(y[a]);
            mn[a] = min(mn[a], ov);
            mx[a] = max(mx[a], ov);
        }
    }
#pragma unroll
    for (int a = 0; a < 3; ++a) {
#pragma unroll
        for (int sft = 32; sft >= 1; sft >>= 1) {
            mn[a] = min(mn[a], (unsigned)__shfl_xor((int)mn[a], sft));
            mx[a] = max(mx[a], (unsigned)__shfl_xor((int)mx[a], sft));
        }
    }
    const int wid = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int a = 0; a < 3; ++a) { smn[wid][a] = mn[a]; smx[wid][a] = mx[a]; }
    }
    __syncthreads();
    if (threadIdx.x < 3) {
        const int a = threadIdx.x;
        unsigned *o = bb_part + ((long long)p * gridDim.x + blockIdx.x) * 6;
        o[a] = min(min(smn[0][a], smn[1][a]), min(smn[2][a], smn[3][a]));
        o[3 + a] = max(max(smx[0][a], smx[1][a]), max(smx[2][a], smx[3][a]));
    }
}

// one block of 6 waves per pose: wave e reduces entry e over the nblk blocks of k_corr_extent
__global__ __launch_bounds__(384) void k_corr_bbox(int nblk, const unsigned *__restrict__ bb_part, float *__restrict__ bbox)
{
    const int p = blockIdx.x, e = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const bool is_min = e < 3;
    unsigned r = is_min ? 0xffffffffu : 0u;
    for (int b = lane; b < nblk; b += 64) {
        const unsigned t = bb_part[((long long)p * nblk + b) * 6 + e];
        r = is_min ? min(r, t) : max(r, t);
    }
#pragma unroll
    for (int sft = 32; sft >= 1; sft >>= 1) {
        const unsigned o = (unsigned)__shfl_xor((int)r, sft);
        r = is_min ? min(r, o) : max(r, o);
    }
    if (lane == 0) bbox[p * 6 + e] = ord2f(r);
}

// Neighbouring nodes have neighbouring images, so the 64 nodes of a wave fall into a handful of cells: the
// lanes of a wave that share a cell are counted together and one of them adds the group to the cell's
// counter (device-scope atomics are executed outside the L2 and are the cost of this kernel).
__global__ __launch_bounds__(256) void k_corr_count(GridP G, CorrP C, const float *__restrict__ Y,
                                                    const float *__restrict__ bbox, int *__restrict__ cell_of,
                                                    int *__restrict__ count, int *__restrict__ slot)
{
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int p = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const bool valid = v < G.V;
    int c = -1;
    if (valid) {
        const float *yp = Y + ((long long)p * G.V + v) * 3;
        const float y[3] = {yp[0], yp[1], yp[2]};
        c = cell_index(C, bbox + p * 6, y);
        cell_of[(long long)p * G.V + v] = c;
    }
    int leader = lane, rank = 0, members = 1;
    unsigned long long todo = __ballot(valid);
    while (todo) {
        const int first = __ffsll((long long)todo) - 1;
        const int key = __shfl(c, first);
        const unsigned long long same = __ballot(valid && c == key);
        if (valid && c == key) {
            leader = first;
            rank = __popcll(same & ((1ull << lane) - 1ull));
            members = __popcll(same);
        }
        todo &= ~same;
    }
    int base = 0;
    if (valid && leader == lane) base = atomicAdd(count + p * C.ncell + c, members);
    base = __shfl(base, leader);
    if (valid) slot[(long long)p * G.V + v] = base + rank;      // a position inside the cell's list
}

// Exclusive prefix sum of a[0..n) in place, a[n] = total.  Three launches: per-tile sums (tile = 4096
// entries), a single-block scan of the tile sums, then every tile scans itself from its carry-in.
constexpr int SCAN_TILE = 4096;   // 1024 threads x 4 entries

__device__ __forceinline__ int block_exclusive_scan_1024(int v, int *total)
{
    __shared__ int wsum[16];
    const int lane = threadIdx.x & 63, wid = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const int o = __shfl_up(inc, d);
        if (lane >= d) inc += o;
    }
    __syncthreads();                       // wsum may still be read by a previous call
    if (lane == 63) wsum[wid] = inc;
    __syncthreads();
    int carry = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int x = wsum[w];
        if (w < wid) carry += x;
        tot += x;
    }
    *total = tot;
    return carry + inc - v;
}

__global__ __launch_bounds__(1024) void k_scan_tile_sums(int n, const int *__restrict__ a, int *__restrict__ sums)
{
    const long long base = (long long)blockIdx.x * SCAN_TILE + threadIdx.x * 4;
    int v = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        if (base + e < n) v += a[base + e];
    int tot;
    block_exclusive_scan_1024(v, &tot);
    if (threadIdx.x == 0) sums[blockIdx.x] = tot;
}

// sums[0..m) -> exclusive scan in place, sums[m] = total (one block, loops over m in steps of 1024);
// also clears *also_zero when given (saves the caller a launch)
__global__ __launch_bounds__(1024) void k_scan_sums(int m, int *__restrict__ sums, int *__restrict__ also_zero)
{
    if (also_zero && threadIdx.x == 0) *also_zero = 0;
    int run = 0;
    for (int s0 = 0; s0 < m; s0 += 1024) {
        const int i = s0 + threadIdx.x;
        const int v = i < m ? sums[i] : 0;
        int tot;
        const int ex = block_exclusive_scan_1024(v, &tot);
        if (i < m) sums[i] = run + ex;
        run += tot;
    }
    if (threadIdx.x == 0) sums[m] = run;
}

// out[i] = exclusive prefix of a (out may be a itself), out[n] = total.  SCANNED: sums holds the exclusive scan
// of the tile sums (k_scan_sums ran); otherwise it holds the raw tile sums and every block adds up the ones
// before its own tile itself (worth it while there are few tiles: one launch less).
template <bool SCANNED>
__global__ __launch_bounds__(1024) void k_scan_tiles(int n, const int *a, int *out, const int *__restrict__ sums, int m,
                                                     int *__restrict__ also_zero)
{
    const long long base = (long long)blockIdx.x * SCAN_TILE + threadIdx.x * 4;
    int e4[4], v = 0;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        e4[e] = base + e < n ? a[base + e] : 0;
        v += e4[e];
    }
    int carry_in, grand = 0;
    if (SCANNED) {
        carry_in = sums[blockIdx.x];
        if (blockIdx.x == 0 && threadIdx.x == 0) grand = sums[m];
    } else {
        int before = 0, all = 0;
        for (int j = threadIdx.x; j < m; j += 1024) {
            const int x = sums[j];
            all += x;
            if (j < (int)blockIdx.x) before += x;
        }
        int t0, t1;
        (void)block_exclusive_scan_1024(before, &t0);
        (void)block_exclusive_scan_1024(all, &t1);
        carry_in = t0;
        grand = t1;
        if (also_zero && blockIdx.x == 0 && threadIdx.x == 0) *also_zero = 0;
    }
    int tot;
    int run = carry_in + block_exclusive_scan_1024(v, &tot);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        if (base + e < n) out[base + e] = run;
        run += e4[e];
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) out[n] = grand;
}

// Every node goes to its place in its cell's list as {image[3], node index}: the selection below then reads its
// samples as consecutive 16-byte entries.  (With a list of node indices alone every sample cost three gathered 4-byte
// loads of its image in each of the three passes: k_corr_select 127 us on the 8-pose grid.)
__global__ __launch_bounds__(256) void k_corr_scatter(GridP G, CorrP C, const float *__restrict__ Y,
                                                      const int *__restrict__ cell_of, const int *__restrict__ offset,
                                                      const int *__restrict__ slot, float4 *__restrict__ sample)
{
    const long long v = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int p = blockIdx.y;
    if (v >= G.V) return;
    const long long i = (long long)p * G.V + v;
    const int c = p * C.ncell + cell_of[i];
    const float *y = Y + i * 3;
    sample[offset[c] + slot[i]] = make_float4(y[0], y[1], y[2], __int_as_float((int)v));
}

// One wave per cell.  Candidate j is the sample with the smallest (distance^2 of its image to the
// cell centre, node index) among those farther than r_sep (canonical distance) from candidates
// 0..j-1: the same set, in the same order, as visiting the samples by increasing key and accepting
// greedily.
__global__ __launch_bounds__(256) void k_corr_select(GridP G, CorrP C, const float *__restrict__ Y,
                                                     const float *__restrict__ bbox, const int *__restrict__ offset,
                                                     const float4 *__restrict__ sample, int32_t *__restrict__ cand,
                                                     uint8_t *__restrict__ ccnt)
{
    // accepted candidates' positions, per wave: the same for all lanes and indexed by a loop counter -- in registers
    // that indexing turns into chains of selects, from LDS it is one broadcast read per candidate
    __shared__ float4 s_acc[4][FS_MAX_CORR_K_DEV];
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int lane = threadIdx.x & 63, wib = threadIdx.x >> 6;
    if (wave >= G.P * C.ncell) return;
    const int p = wave / C.ncell, c = wave - p * C.ncell;
    const float *bb = bbox + p * 6;
    const int beg = offset[wave], end = offset[wave + 1];
    const int ciz = c % C.cz, ciy = (c / C.cz) % C.cy, cix = c / (C.cz * C.cy);
    const float cs0 = (bb[3] - bb[0]) / (float)C.cx;
    const float cs1 = (bb[4] - bb[1]) / (float)C.cy;
    const float cs2 = (bb[5] - bb[2]) / (float)C.cz;
    const float ctr[3] = {FS_FMA((float)cix + 0.5f, cs0, bb[0]), FS_FMA((float)ciy + 0.5f, cs1, bb[1]),
                          FS_FMA((float)ciz + 0.5f, cs2, bb[2])};
    const float rs2 = 6.25f * FS_FMA(G.h[2], G.h[2], FS_FMA(G.h[1], G.h[1], G.h[0] * G.h[0]));
    int na = 0;
    int32_t *out = cand + (long long)wave * C.ck;
    for (int j = 0; j < C.ck; ++j) {
        float bkey = __builtin_inff();
        int bv = 0x7fffffff;
        for (int s = beg + lane; s < end; s += WAVE) {
            const float4 sm = sample[s];
            const int v = __float_as_int(sm.w);
            float x[3];
            node_pos(G, v, x);
            bool far = true;
            for (int a = 0; a < na; ++a) {
                const float4 ac = s_acc[wib][a];
                const float ex = x[0] - ac.x, ey = x[1] - ac.y, ez = x[2] - ac.z;
                const float d2 = FS_FMA(ez, ez, FS_FMA(ey, ey, ex * ex));
                if (!(d2 > rs2)) far = false;
            }
            if (!far) continue;
            const float dx = sm.x - ctr[0], dy = sm.y - ctr[1], dz = sm.z - ctr[2];
            const float key = FS_FMA(dz, dz, FS_FMA(dy, dy, dx * dx));
            if (key < bkey || (key == bkey && v < bv)) { bkey = key; bv = v; }
        }
#pragma unroll
        for (int s = 32; s >= 1; s >>= 1) {
            const float ok = __shfl_xor(bkey, s);
            const int ov = __shfl_xor(bv, s);
            if (ok < bkey || (ok == bkey && ov < bv)) { bkey = ok; bv = ov; }
        }
        if (bv == 0x7fffffff) break;     // wave-uniform
        float xa[3];
        node_pos(G, bv, xa);
        if (lane == 0) s_acc[wib][na] = make_float4(xa[0], xa[1], xa[2], 0.0f);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        ++na;
        if (lane == 0) out[j] = bv;
    }
    if (lane == 0) {
        for (int j = na; j < C.ck; ++j) out[j] = -1;
        ccnt[wave] = (uint8_t)na;            // candidates of this cell (they are packed at the front)
    }
}

// Initial state of every candidate of the correspondence grid, once per fs_precompute instead of once per pair: a
// candidate is a grid node, so its x0, its image d(x0) and J~0 = (dd/dx at x0)^-1 depend on the pose alone, not on
// the query point.  Entry (4 float4) of candidate k of cell gc, at [(gc * ck + k) * 4]:
// {x0[3], flags | d(x0)[3], J~0[0] | J~0[1..4] | J~0[5..8]}, flags (integer bits) = 0: no such candidate,
// 1: usable, 2: Jacobian singular (J~0 = 0), plus the linear index of x0's grid cell << 2.
// Same arithmetic as a lane computing it for itself (node_pos, the 8 corner records of x0's cell,
// jacobian_from_corners, inv3).
__global__ __launch_bounds__(256) void k_corr_init(GridP G, CorrP C, const float *__restrict__ T,
                                                   const int32_t *__restrict__ cand, float4 *__restrict__ cinit)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= (long long)G.P * C.ncell * C.ck) return;
    const int p = (int)(i / ((long long)C.ncell * C.ck));
    const int v = cand[i];
    float x0[3] = {0, 0, 0}, d[3] = {0, 0, 0}, Ji[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    int flags = 0;
    if (v >= 0) {
        node_pos(G, v, x0);
        const float *Tp = T + (long long)p * G.V * 12;
        const Cell c0 = locate(G, x0);
        float q[8][12], Jac[9];
#pragma unroll
        for (int c = 0; c < 8; ++c) load12(Tp + c0.base + corner_off(G, c), q[c]);
        jacobian_from_corners(G, c0, q, x0, d, Jac);
        const bool ok = inv3(Jac, Ji);
        if (!ok) {
#pragma unroll
            for (int e = 0; e < 9; ++e) Ji[e] = 0.0f;
        }
        flags = (ok ? 1 : 2) | (cell_linear(G, c0) << 2);
    }
    float4 *o = cinit + i * 4;
    o[0] = make_float4(x0[0], x0[1], x0[2], __int_as_float(flags));
    o[1] = make_float4(d[0], d[1], d[2], Ji[0]);
    o[2] = make_float4(Ji[1], Ji[2], Ji[3], Ji[4]);
    o[3] = make_float4(Ji[5], Ji[6], Ji[7], Ji[8]);
}

// ------------------------------------------------------------------------------------------------
// Broyden solve.  Lanes are persistent: a wave draws chunks of consecutive lanes q = k*N + n from a
// global cursor and hands a new one to each SIMD lane that has finished, so that a wave does not
// idle behind its slowest trajectory and the grid drains only once, at the very end.  Every loop
// iteration evaluates the field once per active lane: for a freshly loaded lane at x0, otherwise
// at x + dx followed by the rank-one update of J~.
// ------------------------------------------------------------------------------------------------
struct SolveP {
    long long N;
    long long total;     // K * N
    int chunk;           // lanes drawn from the global cursor at a time
    int refill_min;      // refill when at least this many SIMD lanes are idle
    int max_iters;
    float tol2, div2;
    int K;
    int point_major;     // order in which pairs are handed out
    int spin_limit;      // producer / consumer kernel: polls of a work queue before a wave gives up
    int xcd_ranges;      // producer / consumer kernel: the list is cut into 8 ranges, one per XCD, each with its own cursor
    int prefetch;        // producer / consumer kernel: consumers ask for the next cell's records at the end of a pass
};

// What the fused variant needs to compute initial states itself (same arithmetic as k_init_*).
struct InitP {
    int mode;                 // 0: one state per bone (Eq. (8)); 1: candidates of the correspondence grid
    const float *Binv;        // [P][nb][12]
    const uint8_t *Bok;       // [P][nb]
    CorrP C;
    const float *bbox;        // [P][6]
    const int32_t *cand;      // [P][ncell][ck]
    const uint8_t *ccnt;      // [P][ncell]: number of candidates of the cell
    const float4 *cinit;      // [P][ncell][ck][4]: initial state of every candidate (k_corr_init)
};

// Result record of one pair.  WITH_J: 16 floats {x*[3], flags | pos, J~[0..2] | J~[3..6] | J~[7], J~[8], pad[2]}, else 4 floats
// {x*[3], flags}; flags = conv | iters << 8 (as an integer bit pattern).  `pos` (the lane's position in its grid cell's
// list, for the backward) is not written here but later, by flush_slots, for converged lanes only: this store leaves
// that word alone, so the two never write the same address.  x*, flags and pos share the record's first 32-byte sector.
template <bool WITH_J>
__device__ __forceinline__ void write_record(float4 *__restrict__ rec, long long pq, const float x[3], const float J[9],
                                             int flags)
{
    if (WITH_J) {
        float4 *o = rec + pq * 4;
        o[0] = make_float4(x[0], x[1], x[2], __int_as_float(flags));
        float *j = reinterpret_cast<float *>(o) + 5;
        j[0] = J[0];
        j[1] = J[1];
        j[2] = J[2];
        o[2] = make_float4(J[3], J[4], J[5], J[6]);
        o[3] = make_float4(J[7], J[8], 0.0f, 0.0f);
    } else {
        rec[pq] = make_float4(x[0], x[1], x[2], __int_as_float(flags));
    }
}
constexpr int REC_POS = 4;      // float index of `pos` inside a 16-float record

__device__ __forceinline__ void read_record_J(const float4 *__restrict__ r, float (&J)[9])
{
    const float4 b = r[1], c = r[2], d = r[3];
    J[0] = b.y; J[1] = b.z; J[2] = b.w; J[3] = c.x; J[4] = c.y; J[5] = c.z; J[6] = c.w; J[7] = d.x; J[8] = d.y;
}

// Voxel-based initial states leave most lanes without a candidate (a ray sample in empty space has
// none).  Pre-pass for the fused solve: candidates per point, prefix sum, then the list of pairs
// that do have one, so that the solve kernel draws only those.
// Per pose the lower corner of the box of node images and the size of a correspondence cell are put into LDS once per
// block (the arithmetic of cell_index), and the number of candidates of a cell is one byte written by k_corr_select:
// with the six box entries and the three candidate slots read per point through the vector cache -- nine gathered
// loads of four bytes -- this kernel took 77 us on the 8-pose batch.
__global__ __launch_bounds__(256) void k_voxel_count(GridP G, InitP I, long long N, const float *__restrict__ xq,
                                                     const int32_t *__restrict__ pose, int *__restrict__ cnt,
                                                     uint8_t *__restrict__ cnt8, int *__restrict__ gcell)
{
    extern __shared__ float s_pose[];            // [P][6]: lower corner, cell size
    for (int i = threadIdx.x; i < G.P * 3; i += blockDim.x) {
        const int p = i / 3, a = i - 3 * p;
        const float *bb = I.bbox + p * 6;
        const int na = a == 0 ? I.C.cx : (a == 1 ? I.C.cy : I.C.cz);
        s_pose[p * 6 + a] = bb[a];
        s_pose[p * 6 + 3 + a] = (bb[3 + a] - bb[a]) / (float)na;
    }
    __syncthreads();
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const int p = pose_of(pose, n, G.P);
    const float *sp = s_pose + p * 6;
    const int ci = (cell_coord(xq[n], sp[0], sp[3], I.C.cx) * I.C.cy + cell_coord(xq[N + n], sp[1], sp[4], I.C.cy)) * I.C.cz +
                   cell_coord(xq[2 * N + n], sp[2], sp[5], I.C.cz);
    const int gc = p * I.C.ncell + ci;
    const int m = I.ccnt[gc];
    cnt[n] = m;
    cnt8[n] = (uint8_t)m;
    gcell[n] = gc;
}

// list entry of a pair: {point n, (pose * ncell + correspondence cell) << 3 | k}
__global__ __launch_bounds__(256) void k_voxel_expand(long long N, const int *__restrict__ offs, const int *__restrict__ gcell,
                                                      int2 *__restrict__ list)
{
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    const int b = offs[n], e = offs[n + 1], gc = gcell[n];
    for (int j = b; j < e; ++j) list[j] = make_int2((int)n, (gc << 3) | (j - b));
}

// The list of pairs, ordered by place: all pairs whose query point falls into the same column of correspondence cells
// (bucket = (pose * ncell + cell) / cz, i.e. the cell index without its fastest coordinate) are made neighbours, so
// that the lanes at work at any one time -- on every XCD, since all blocks draw from one cursor -- read the same
// stretch of one pose's transform grid and of the candidate table, and the caches serve what memory served before.
// A counting sort without global atomics: every block counts the candidates of its tile of SORT_TILE points per
// bucket in LDS and leaves the counts in hist[bucket][block]; an exclusive scan over that matrix (bucket-major)
// gives every (bucket, block) the place where its pairs start; the blocks then hand out places within that from LDS
// counters.  The order inside a bucket is the order in which the lanes of a block arrive: any order is a valid list.
constexpr int SORT_TILE = 16384;          // points per block
constexpr int SORT_MAX_BUCKETS = 16384;   // 64 KiB of LDS counters

__global__ __launch_bounds__(1024) void k_sort_hist(long long N, int cz, int nb, const int *__restrict__ gcell,
                                                    const uint8_t *__restrict__ cnt8, int *__restrict__ hist)
{
    extern __shared__ int s_cnt[];
    for (int i = threadIdx.x; i < nb; i += blockDim.x) s_cnt[i] = 0;
    __syncthreads();
    const long long n0 = (long long)blockIdx.x * SORT_TILE, n1 = min(N, n0 + SORT_TILE);
    for (long long n = n0 + threadIdx.x; n < n1; n += blockDim.x) {
        const int c = cnt8[n];
        if (c) atomicAdd(&s_cnt[gcell[n] / cz], c);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < nb; i += blockDim.x) hist[(long long)i * gridDim.x + blockIdx.x] = s_cnt[i];
}

// list entry of a pair: {point n, (pose * ncell + correspondence cell) << 3 | k}
__global__ __launch_bounds__(1024) void k_sort_scatter(long long N, int cz, int nb, const int *__restrict__ gcell,
                                                       const uint8_t *__restrict__ cnt8, const int *__restrict__ start,
                                                       int2 *__restrict__ list)
{
    extern __shared__ int s_cnt[];
    for (int i = threadIdx.x; i < nb; i += blockDim.x) s_cnt[i] = start[(long long)i * gridDim.x + blockIdx.x];
    __syncthreads();
    const long long n0 = (long long)blockIdx.x * SORT_TILE, n1 = min(N, n0 + SORT_TILE);
    for (long long n = n0 + threadIdx.x; n < n1; n += blockDim.x) {
        const int c = cnt8[n];
        if (!c) continue;
        const int gc = gcell[n];
        const int at = atomicAdd(&s_cnt[gc / cz], c);
        for (int k = 0; k < c; ++k) list[at + k] = make_int2((int)n, (gc << 3) | k);
    }
}

// records -> caller's layout: one thread per pair q = k*N + n, consecutive threads consecutive n.
// NOCAND: the solve ran with fused voxel-based initial states and wrote no record for lanes whose
// cell holds no k-th candidate (cand_cnt[n] = candidates of point n, packed at the front);
// those get the answer of an invalid lane (x0 = 0, J~ = 0, not converged).
// o_slot (may be null): the positions of the converged lanes in their grid cells' lists, which the solve kernel
// left in the records, -1 for every other lane.
template <bool WITH_J, bool NOCAND>
__global__ __launch_bounds__(256) void k_solve_unpack(long long N, long long total, const uint8_t *__restrict__ cand_cnt,
                                                      const float4 *__restrict__ rec, float *__restrict__ o_x,
                                                      uint8_t *__restrict__ o_conv, float *__restrict__ o_J,
                                                      uint8_t *__restrict__ o_it, int32_t *__restrict__ o_slot)
{
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x, k = blockIdx.y;      // grid: points x initial states
    if (n >= N) return;
    const long long pq = k * N + n;
    bool have = true;
    if (NOCAND) have = k < cand_cnt[n];
    float4 a = make_float4(0.0f, 0.0f, 0.0f, 0.0f), b = a;
    if (have) a = WITH_J ? rec[pq * 4] : rec[pq];
    o_x[(k * 3 + 0) * N + n] = a.x;
    o_x[(k * 3 + 1) * N + n] = a.y;
    o_x[(k * 3 + 2) * N + n] = a.z;
    const int flags = __float_as_int(a.w);
    o_conv[pq] = (uint8_t)(flags & 1);
    if (o_it) o_it[pq] = (uint8_t)(flags >> 8);
    if (WITH_J && (o_slot || o_J) && have) b = rec[pq * 4 + 1];
    if (WITH_J && o_slot) o_slot[pq] = (flags & 1) ? __float_as_int(b.x) : -1;
    if (WITH_J && o_J) {
        float J[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
        if (have) {
            const float4 c = rec[pq * 4 + 2], d = rec[pq * 4 + 3];
            J[0] = b.y; J[1] = b.z; J[2] = b.w; J[3] = c.x; J[4] = c.y; J[5] = c.z; J[6] = c.w; J[7] = d.x; J[8] = d.y;
        }
#pragma unroll
        for (int e = 0; e < 9; ++e) o_J[(k * 9 + e) * N + n] = J[e];
    }
}

// Words of the context's cursor array: CUR_ALL is the work cursor of the solve kernels; CUR_NONFINITE holds the serial
// number of the last fs_precompute whose grid had an entry that is not finite.
// CUR_XCD + j (j = 0 .. 7): the cursor of the j-th eighth of an ordered pair list, relative to the start of that eighth.
constexpr int CUR_ALL = 0, CUR_NONFINITE = 2, CUR_XCD = 4, CUR_WORDS = 12, N_XCD = 8;

// The blocks of the solve kernel own their first chunk without asking: the shared cursor starts behind `nblocks`
// chunks, the cursor of range j behind one chunk for every block b with b mod 8 = j.
__device__ __forceinline__ void reset_cursors(unsigned *__restrict__ cursor, int i, unsigned nblocks, unsigned chunk)
{
    if (i == 0) cursor[CUR_ALL] = nblocks * chunk;
    if (i < N_XCD) cursor[CUR_XCD + i] = ((nblocks + (N_XCD - 1) - (unsigned)i) / N_XCD) * chunk;
}

__global__ void k_reset_cursor(unsigned *__restrict__ cursor, unsigned nblocks, unsigned chunk)
{
    if (blockIdx.x == 0) reset_cursors(cursor, (int)threadIdx.x, nblocks, chunk);
}

// The parked requests of one wave: entry i = {cell, pair}, one per SIMD lane.  Lanes of one point that reach
// the same root are neighbours in the wave and finish within a few passes of each other, so many entries name
// the same cell: those are counted together and one lane adds the group to the cell's counter.
constexpr int PEND = 128;       // requests a wave parks before it sends them
constexpr int PEND_SEND = 112;  // ... at least this many

__device__ __forceinline__ void flush_slots(int (&pend)[2][PEND], int npend, int lane, int *__restrict__ cell_count,
                                            float4 *__restrict__ rec)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the LDS writes of the wave's other lanes
    __builtin_amdgcn_wave_barrier();
    // two rounds of 64 entries; the atomics of both are on their way before either answer is used
    bool valid[2];
    int pq[2], leader[2], rank[2], base[2];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        valid[b] = 64 * b + lane < npend;
        const int c = valid[b] ? pend[0][64 * b + lane] : -1;
        pq[b] = valid[b] ? pend[1][64 * b + lane] : 0;
        int members = 1;
        leader[b] = lane;
        rank[b] = 0;
        unsigned long long todo = __ballot(valid[b]);
        while (todo) {
            const int first = __ffsll((long long)todo) - 1;
            const int key = __builtin_amdgcn_readlane(c, first);
            const unsigned long long same = __ballot(valid[b] && c == key);
            if (valid[b] && c == key) {
                leader[b] = first;
                rank[b] = __popcll(same & ((1ull << lane) - 1ull));
                members = __popcll(same);
            }
            todo &= ~same;
        }
        base[b] = 0;
        if (valid[b] && leader[b] == lane) base[b] = atomicAdd(cell_count + c, members);
    }
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int bs = __shfl(base[b], leader[b]);
        // into the pair's own result record (written a few passes ago, still in the L2), not into an array of its own
        if (valid[b]) reinterpret_cast<int *>(rec)[(long long)pq[b] * 16 + REC_POS] = bs + rank[b];
    }
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // before the entries are overwritten
    __builtin_amdgcn_wave_barrier();
}

// Broyden solve for a transform grid (all poses) small enough to be held in LDS: every block copies it there
// first and all corner records are then read from LDS, where per-lane addresses cost far less than in the
// vector memory path.  Every wave does everything:
// FUSED = false: initial states are read from x0 / J0 / valid0.  FUSED = true: a lane computes its
// initial state when it picks up a pair (Sec. 3.1 "Custom CUDA Kernel": the kernel first computes the
// initialisation states); the corner records fetched for the Jacobian then also serve the first
// evaluation of the field, and the 53 bytes per pair of initial state never touch memory.
//
// Results leave the kernel as one contiguous record per pair (lanes finish at different times, so
// writing the caller's structure-of-arrays layout from here would touch 14 cache lines per pair with
// 4 bytes each); k_solve_unpack then moves the records into that layout with coalesced stores.
// (record layout: see write_record).
// NW = waves per block.  4: grids of up to 60 KiB, three blocks per CU, each with its own copy.  12: larger grids, up
// to what one block may hold of the CU's 160 KiB: one block per CU, the same 3 waves per SIMD, one copy.
template <bool FUSED, bool WITH_J, int NW = 4>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 3 : 1) void k_solve(GridP G, SolveP S, InitP I, const float *__restrict__ Tglobal,
                                               const float *__restrict__ xq, const int32_t *__restrict__ pose,
                                               const float *__restrict__ x0, const float *__restrict__ J0,
                                               const uint8_t *__restrict__ valid0, float4 *__restrict__ rec,
                                               unsigned *__restrict__ cursor, const int2 *__restrict__ list,
                                               const int *__restrict__ list_len, int *__restrict__ cell_count,
                                               int ncell)
{
    extern __shared__ float4 s_grid[];
    // converged lanes waiting for their position in their grid cell's list: {cell, pair} per wave
    __shared__ int s_pend[NW][2][PEND];
    {
        const int n4 = (int)((long long)G.P * G.V * 3);      // float4 per record: 3
        const float4 *src = reinterpret_cast<const float4 *>(Tglobal);
        for (int i = threadIdx.x; i < n4; i += blockDim.x) s_grid[i] = src[i];
        __syncthreads();
    }
    const float *T = reinterpret_cast<const float *>(s_grid);
    // with a list only the pairs list[0 .. *list_len) ({point, cell << 3 | k}) are solved
    const long long total = list ? (long long)*list_len : S.total;
    const int lane = threadIdx.x & 63;
    // wave-uniform: the wave's current chunk is [next, c1).  The first chunk of wave w is chunk w (the cursor
    // starts behind these): 2048 waves asking one counter at once would wait 9 ns each, one after the other.
    long long next = (long long)__builtin_amdgcn_readfirstlane((int)((blockIdx.x * blockDim.x + threadIdx.x) >> 6)) * S.chunk;
    long long c1 = min(total, next + S.chunk);
    bool exhausted = false;          // wave-uniform: the global cursor has run past the end
    const long long N = S.N;

    bool active = false, fresh = false;
    long long n = 0;
    int k = 0, it = 0, pz = 0;
    const float *Tp = T;
    float xp[3] = {0, 0, 0}, x[3] = {0, 0, 0}, xt[3] = {0, 0, 0}, g[3] = {0, 0, 0}, dx[3] = {0, 0, 0};
    float J[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    float q[8][12];                  // corner records of the lane's current cell, kept across iterations
    long long held = -1;             // grid offset of the cell whose corners q holds (-1: none)
    int npend = 0;                   // wave-uniform: entries of s_pend in use
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));

    while (true) {
        unsigned long long idle = __ballot(!active);
        int nidle = __popcll(idle);
        // hand out pairs until fewer than refill_min lanes are idle: a pair whose initial state is
        // invalid is answered on the spot and its lane asks again
        while (!exhausted && nidle >= S.refill_min) {
            if (next >= c1) {
                unsigned b = 0;
                if (lane == 0) b = atomicAdd(cursor + CUR_ALL, (unsigned)S.chunk);
                b = (unsigned)__builtin_amdgcn_readfirstlane((int)b);
                if ((long long)b >= total) {
                    exhausted = true;
                } else {
                    next = b;
                    c1 = min(total, (long long)b + S.chunk);
                }
            }
            if (!exhausted) {
                const int rank = __popcll(idle & ((1ull << lane) - 1ull));
                const long long pq = next + rank;
                if (!active && pq < c1) {
                    // K * N < 2^31: 32-bit division
                    if (list) {
                        const int2 e = list[pq];
                        n = e.x;
                        k = e.y & 7;
                    } else if (S.point_major) {   // consecutive SIMD lanes: the K initial states of one point
                        n = (unsigned)pq / (unsigned)S.K;
                        k = (int)((unsigned)pq - (unsigned)n * (unsigned)S.K);
                    } else {                      // consecutive SIMD lanes: consecutive points, same initial state
                        k = (int)((unsigned)pq / (unsigned)N);
                        n = (unsigned)pq - (unsigned)k * (unsigned)N;
                    }
                    const int p = pose_of(pose, n, G.P);
                    pz = p;
                    Tp = T + (long long)p * G.V * 12;
                    it = 0;
                    held = -1;
                    bool ok, norec = false;     // norec: no record needed, k_solve_unpack knows the answer
#pragma unroll
                    for (int r = 0; r < 3; ++r) xp[r] = xq[r * N + n];
                    if (FUSED) {
#pragma unroll
                        for (int r = 0; r < 3; ++r) xt[r] = 0.0f;
#pragma unroll
                        for (int e = 0; e < 9; ++e) J[e] = 0.0f;
                        if (I.mode == 0) {
                            const float *bi = I.Binv + ((long long)p * G.nb + k) * 12;
                            ok = I.Bok[p * G.nb + k] != 0;
                            if (ok) {
                                const float y[3] = {xp[0] - bi[9], xp[1] - bi[10], xp[2] - bi[11]};
#pragma unroll
                                for (int r = 0; r < 3; ++r)
                                    xt[r] = FS_FMA(bi[r * 3 + 0], y[0], FS_FMA(bi[r * 3 + 1], y[1], bi[r * 3 + 2] * y[2]));
                            }
                        } else {
                            const int cidx = cell_index(I.C, I.bbox + p * 6, xp);
                            const int v = I.cand[((long long)p * I.C.ncell + cidx) * I.C.ck + k];
                            ok = v >= 0;
                            norec = !ok;
                            if (ok) node_pos(G, v, xt);
                        }
                        if (ok) {
                            const Cell c0 = locate(G, xt);
#pragma unroll
                            for (int c = 0; c < 8; ++c) load12(Tp + c0.base + corner_off(G, c), q[c]);
                            held = (long long)(Tp - T) + c0.base;
                            float d0[3], Jac[9];
                            jacobian_from_corners(G, c0, q, xt, d0, Jac);
                            ok = inv3(Jac, J);
                            if (!ok) {
#pragma unroll
                                for (int e = 0; e < 9; ++e) J[e] = 0.0f;
                            }
                        }
                    } else {
#pragma unroll
                        for (int r = 0; r < 3; ++r) xt[r] = x0[((long long)k * 3 + r) * N + n];
#pragma unroll
                        for (int e = 0; e < 9; ++e) J[e] = J0[((long long)k * 9 + e) * N + n];
                        ok = valid0[(long long)k * N + n] != 0;
                    }
                    if (ok) {
                        active = true;
                        fresh = true;
                    } else if (!norec) {
                        write_record<WITH_J>(rec, (long long)k * N + n, xt, J, 0);
                    }
                }
                next += min((long long)nidle, c1 - next);
            }
            idle = __ballot(!active);
            nidle = __popcll(idle);
        }
        if (!__any(active)) {
            if (exhausted) break;
            continue;
        }
        bool want_slot = false;
        int slot_cell = 0;
        if (active) {
            float d[3], gn[3];
            // steps shrink as a lane converges, so it often stays in the cell it was in: reload the
            // 8 corner records only when the cell changed
            const Cell cell = locate(G, xt);
            const long long want = (long long)(Tp - T) + cell.base;
            if (want != held) {
#pragma unroll
                for (int c = 0; c < 8; ++c) load12(Tp + cell.base + corner_off(G, c), q[c]);
                held = want;
            }
            blend_apply(cell, q, xt, d);
#pragma unroll
            for (int r = 0; r < 3; ++r) gn[r] = d[r] - xp[r];
            if (!fresh) {
                float dg[3], v[3], u[3];
#pragma unroll
                for (int r = 0; r < 3; ++r) dg[r] = gn[r] - g[r];
#pragma unroll
                for (int c = 0; c < 3; ++c) v[c] = FS_FMA(dx[2], J[6 + c], FS_FMA(dx[1], J[3 + c], dx[0] * J[c]));
#pragma unroll
                for (int r = 0; r < 3; ++r)
                    u[r] = dx[r] - FS_FMA(J[r * 3 + 2], dg[2], FS_FMA(J[r * 3 + 1], dg[1], J[r * 3] * dg[0]));
                const float den = FS_FMA(v[2], dg[2], FS_FMA(v[1], dg[1], v[0] * dg[0]));
                if (den != 0.0f && __builtin_fabsf(den) < __builtin_inff()) {
                    const float rinv = 1.0f / den;
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        const float s = u[r] * rinv;
#pragma unroll
                        for (int c = 0; c < 3; ++c) J[r * 3 + c] = FS_FMA(s, v[c], J[r * 3 + c]);
                    }
                }
                ++it;
            }
            fresh = false;
#pragma unroll
            for (int r = 0; r < 3; ++r) { x[r] = xt[r]; g[r] = gn[r]; }
            const float r2 = FS_FMA(g[2], g[2], FS_FMA(g[1], g[1], g[0] * g[0]));
            const bool conv = r2 < S.tol2;
            const bool done = conv || !(r2 < S.div2) || it >= S.max_iters;
            if (done) {
                write_record<WITH_J>(rec, (long long)k * N + n, x, J, (conv ? 1 : 0) | (it << 8));
                if (WITH_J && cell_count && conv) {
                    want_slot = true;
                    slot_cell = pz * ncell + cell_linear(G, cell);
                }
                active = false;
            } else {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    dx[r] = -FS_FMA(J[r * 3 + 2], g[2], FS_FMA(J[r * 3 + 1], g[1], J[r * 3] * g[0]));
                    xt[r] = x[r] + dx[r];
                }
            }
        }
        // For the backward every converged lane needs its arrival position in the list of its grid cell: one
        // returning atomic on the cell's counter.  A wave would wait for that answer in every pass (a few of
        // its lanes finish in each), so the requests are parked in LDS and sent 112 or more at a time, one per cell and round of 64.
        if (WITH_J && cell_count) {
            const unsigned long long m = __ballot(want_slot);
            if (m) {
                if (npend + __popcll(m) > PEND) {
                    flush_slots(s_pend[wib], npend, lane, cell_count, rec);
                    npend = 0;
                }
                if (want_slot) {
                    const int at = npend + __popcll(m & ((1ull << lane) - 1ull));
                    s_pend[wib][0][at] = slot_cell;
                    s_pend[wib][1][at] = (int)((long long)k * N + n);
                }
                npend += __popcll(m);
            }
            if (npend >= PEND_SEND) {
                flush_slots(s_pend[wib], npend, lane, cell_count, rec);
                npend = 0;
            }
        }
    }
    if (WITH_J && cell_count && npend > 0) flush_slots(s_pend[wib], npend, lane, cell_count, rec);
}

// ------------------------------------------------------------------------------------------------
// Broyden solve (Eq. (7) with the rank-one update of J~, Algorithm 1 variant 2, per-iteration filter of
// Sec. 3.1 "Custom CUDA Kernel") with the work divided between the waves of a block.  One wave (the producer) prepares
// pairs 64 at a time, every SIMD lane busy: initial state, first evaluation of the field, first step; pairs
// that end there (invalid state, converged or diverged at x0) it answers itself.  The other waves (the
// consumers) only iterate: each owns a queue of prepared states {x', x, g, dx, J~, pair} in LDS, its idle
// lanes pick states up with a few LDS reads, and its loop holds nothing but the Broyden step.  The producer
// gives every batch to the consumer whose queue is emptiest.  Neither role ever holds the other's registers.
// Queues: single producer, single consumer; tail is written by the producer only, head by the consumer only.
// Every wait ends: a producer that has polled S.spin_limit times in vain for room in its consumers' queues raises
// *give_up (host-visible) and leaves; it raises s_done on every way out, and its consumers, which wait for
// nothing else, finish what their queues hold and leave too.
// ------------------------------------------------------------------------------------------------
constexpr int WS_RING = 128;                 // entries per queue (two batches)
constexpr int FS_WS_CONSUMERS = 3;           // measured: a producer that computes Eq. (8) keeps up with three consumers, not with four
// A producer that only looks up voxel-based candidates could serve more consumers, but more iterating waves per CU
// only compete for the vector cache: measured on the multi-pose / training / ray batches, kernel ms with 2 blocks per
// CU: 3 consumers 1.73 / 0.175 / 0.120, 4 consumers 1.87 / 0.196 / 0.124, 5 consumers 1.92 / 0.213 / 0.138.
constexpr int FS_VX_CONSUMERS = 3;
constexpr int ST_XP = 0, ST_X = 3, ST_G = 6, ST_DX = 9, ST_J = 12, ST_N = 21, ST_K = 22, ST_P = 23, ST_FIELDS = 24;

__device__ __forceinline__ int lds_load_acquire(const int *p)
{
    return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP);
}
__device__ __forceinline__ void lds_store_release(int *p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
}

__device__ __forceinline__ void park_slots(bool want_slot, int slot_cell, int pair, int (&pend)[2][PEND], int &npend, int lane,
                                           int *__restrict__ cell_count, float4 *__restrict__ rec)
{
    const unsigned long long m = __ballot(want_slot);
    if (m) {
        if (npend + __popcll(m) > PEND) {
            flush_slots(pend, npend, lane, cell_count, rec);
            npend = 0;
        }
        if (want_slot) {
            const int at = npend + __popcll(m & ((1ull << lane) - 1ull));
            pend[0][at] = slot_cell;
            pend[1][at] = pair;
        }
        npend += __popcll(m);
    }
    if (npend >= PEND_SEND) {
        flush_slots(pend, npend, lane, cell_count, rec);
        npend = 0;
    }
}

// ---- result records of k_solve_ws leave through LDS ---------------------------------------------------------------
// A lane that finishes does not store its 64-byte record itself (four 16-byte stores to an address of its own: four
// vector-memory instructions in nearly every pass of the wave, each of which reaches memory as a partial write of a
// 32-byte sector).  The wave parks finished records in LDS, OUT_PEND per wave, together with the grid cell of the
// converged ones; when OUT_SEND have gathered it asks for their positions in their cells' lists (one atomic per cell
// and round of 64, as flush_slots does), puts each position into its record, and writes the records out with four
// consecutive lanes per record: every record reaches memory once, whole, as 64 contiguous bytes.
constexpr int OUT_PEND = 128, OUT_SEND = 112;
struct OutQ {
    float4 rec[OUT_PEND][4];
    int cell[OUT_PEND];      // grid cell (pose * ncell + cell) of a converged lane that wants a position, else -1
    int pair[OUT_PEND];
};

__device__ __forceinline__ void out_flush(OutQ &q, int npend, int lane, int *__restrict__ cell_count, float4 *__restrict__ rec)
{
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // the LDS writes of the wave's other lanes
    __builtin_amdgcn_wave_barrier();
    if (cell_count) {
        // two rounds of 64 entries; the atomics of both are on their way before either answer is used
        bool valid[2];
        int leader[2], rank[2], base[2];
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int c = 64 * b + lane < npend ? q.cell[64 * b + lane] : -1;
            valid[b] = c >= 0;
            int members = 1;
            leader[b] = lane;
            rank[b] = 0;
            unsigned long long todo = __ballot(valid[b]);
            while (todo) {
                const int first = __ffsll((long long)todo) - 1;
                const int key = __builtin_amdgcn_readlane(c, first);
                const unsigned long long same = __ballot(valid[b] && c == key);
                if (valid[b] && c == key) {
                    leader[b] = first;
                    rank[b] = __popcll(same & ((1ull << lane) - 1ull));
                    members = __popcll(same);
                }
                todo &= ~same;
            }
            base[b] = 0;
            if (valid[b] && leader[b] == lane) base[b] = atomicAdd(cell_count + c, members);
        }
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int bs = __shfl(base[b], leader[b]);
            if (valid[b]) reinterpret_cast<int *>(&q.rec[64 * b + lane][1])[0] = bs + rank[b];
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
    for (int i = lane; i < npend * 4; i += 64) rec[(long long)q.pair[i >> 2] * 4 + (i & 3)] = q.rec[i >> 2][i & 3];
    __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");      // before the entries are overwritten
    __builtin_amdgcn_wave_barrier();
}

// park the record of every lane with `want` (wave-wide call); cell < 0: no position wanted
__device__ __forceinline__ void out_park(bool want, const float x[3], const float J[9], int flags, int cell, int pair, OutQ &q,
                                         int &npend, int lane, int *__restrict__ cell_count, float4 *__restrict__ rec)
{
    const unsigned long long m = __ballot(want);
    if (m) {
        if (npend + __popcll(m) > OUT_PEND) {
            out_flush(q, npend, lane, cell_count, rec);
            npend = 0;
        }
        if (want) {
            const int at = npend + __popcll(m & ((1ull << lane) - 1ull));
            q.rec[at][0] = make_float4(x[0], x[1], x[2], __int_as_float(flags));
            q.rec[at][1] = make_float4(__int_as_float(-1), J[0], J[1], J[2]);
            q.rec[at][2] = make_float4(J[3], J[4], J[5], J[6]);
            q.rec[at][3] = make_float4(J[7], J[8], 0.0f, 0.0f);
            q.cell[at] = cell;
            q.pair[at] = pair;
        }
        npend += __popcll(m);
    }
    if (npend >= OUT_SEND) {
        out_flush(q, npend, lane, cell_count, rec);
        npend = 0;
    }
}

// ---- corner records with zero weight need not be fetched ------------------------------------------------
// A coordinate outside the box is clamped, so its fraction is exactly 0 or 1 and the four corners on the far
// side of that axis get the weight 0: their records contribute 0 * T_c, i.e. nothing but possibly the sign of
// an exact zero.  A consumer of k_solve_ws may fetch only the other corners (bit c of the mask below); the
// registers of the skipped ones keep whatever finite record (or the initial zeros) they held before.  If a
// blended entry then comes out as an exact zero, the skipped records are fetched and the evaluation is
// repeated, so that even the sign of that zero is the one the full sum has.
// Corners that can have a non-zero weight: along a clamped axis only the side the point was clamped to
// (fraction 0: offset 0, fraction 1: offset 1).  An axis that merely happens to have fraction 0 keeps both sides.
__device__ __forceinline__ int corners_needed(const Cell &c)
{
    const int mx = c.cl[0] ? (c.f[0] == 0.0f ? 0x55 : 0xAA) : 0xFF;
    const int my = c.cl[1] ? (c.f[1] == 0.0f ? 0x33 : 0xCC) : 0xFF;
    const int mz = c.cl[2] ? (c.f[2] == 0.0f ? 0x0F : 0xF0) : 0xFF;
    return mx & my & mz;
}

// Issue order of the 24 loads of a cell.  The two z-neighbours of an (x, y) corner are 96 contiguous bytes, i.e. six
// 16-byte pieces in one or two cache lines; FS_LOAD_ORDER 1 issues the six pieces of a corner pair back to back
// (the compiler barrier keeps that order), 0 leaves the order to the compiler (four pieces of each pair, then the
// rest), 2 issues piece by piece across the four pairs (accesses of a lane to one line four instructions apart).
// Measured, Broyden kernel on the multi-pose / SMPL-scale batches: order 2: 2.20 / 0.42 ms, order 0: 1.69 / 0.35 ms:
// the vector cache rewards accesses to one line that follow each other closely.
#ifndef FS_LOAD_ORDER
#define FS_LOAD_ORDER 1
#endif
__device__ __forceinline__ void load_corners(const float *__restrict__ Tcell, const GridP &G, int mask, float (&q)[8][12])
{
#if FS_LOAD_ORDER == 0
#pragma unroll
    for (int c = 0; c < 8; ++c)
        if ((mask >> c) & 1) load12(Tcell + corner_off(G, c), q[c]);
#else
#pragma unroll
    for (int i = 0; i < 24; ++i) {
        const int j = FS_LOAD_ORDER == 1 ? i % 6 : i / 4, s4 = FS_LOAD_ORDER == 1 ? i / 6 : i % 4;
        const int c = s4 + 4 * (j / 3), e = 4 * (j % 3);
        if ((mask >> c) & 1) {
            const float4 v = *reinterpret_cast<const float4 *>(Tcell + corner_off(G, c) + e);
            q[c][e] = v.x; q[c][e + 1] = v.y; q[c][e + 2] = v.z; q[c][e + 3] = v.w;
        }
        if ((FS_LOAD_ORDER == 1 ? i % 6 == 5 : i % 4 == 3)) asm volatile("" ::: "memory");
    }
#endif
}

// all eight corner records of a cell
__device__ __forceinline__ void load_cell(const float *__restrict__ Tcell, const GridP &G, float (&q)[8][12])
{
    load_corners(Tcell, G, 0xFF, q);
}

// blend_apply that also tells whether one of the 12 blended entries is an exact zero
__device__ __forceinline__ bool blend_apply_z(const Cell &c, const float (&q)[8][12], const float x[3], float d[3])
{
    float om[8];
    corner_weights(c, om);
    float T[12];
#pragma unroll
    for (int e = 0; e < 12; ++e) T[e] = om[0] * q[0][e];
#pragma unroll
    for (int k = 1; k < 8; ++k)
#pragma unroll
        for (int e = 0; e < 12; ++e) T[e] = FS_FMA(om[k], q[k][e], T[e]);
    apply12(T, x, d);
    float m = __builtin_fabsf(T[0]);
#pragma unroll
    for (int e = 1; e < 12; ++e) m = __builtin_fminf(m, __builtin_fabsf(T[e]));
    return m == 0.0f;
}

template <bool FUSED, bool WITH_J, int NCONS, bool SKIP>
__global__ __launch_bounds__(64 * (NCONS + 1), 2) void k_solve_ws(GridP G, SolveP S, InitP I, const float *__restrict__ T,
                                               const float *__restrict__ xq, const int32_t *__restrict__ pose,
                                               const float *__restrict__ x0, const float *__restrict__ J0,
                                               const uint8_t *__restrict__ valid0, float4 *__restrict__ rec,
                                               unsigned *__restrict__ cursor, const int2 *__restrict__ list,
                                               const int *__restrict__ list_len, int *__restrict__ cell_count,
                                               int ncell, int *__restrict__ give_up,
                                               const int *__restrict__ nonfinite, int serial)
{
    __shared__ float s_ring[NCONS][ST_FIELDS][WS_RING];
    __shared__ int s_tail[NCONS], s_head[NCONS], s_done;
    __shared__ OutQ s_out[WITH_J ? NCONS + 1 : 1];      // records on their way out, per wave (only full records are parked)
    if (threadIdx.x < NCONS) {
        s_tail[threadIdx.x] = 0;
        s_head[threadIdx.x] = 0;
    }
    if (threadIdx.x == 0) s_done = 0;
    __syncthreads();
    const long long total = list ? (long long)*list_len : S.total;
    const int lane = threadIdx.x & 63;
    const int wib = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long N = S.N;
    int npend = 0;                   // wave-uniform: entries of the wave's s_out in use
    OutQ &outq = s_out[WITH_J ? wib : 0];

    if (wib == NCONS) {
        // ------------------------------------------------ producer ------------------------------------------------
        // the first chunk of block b is chunk b; the shared cursor starts behind those.  (One cursor for the whole chip
        // on purpose: all XCDs then work through the same stretch of the points at the same time, and what one of them
        // brought into the memory-side cache serves the others.  With a cursor per XCD over its own eighth of the
        // points -- one pose per XCD on the multi-pose batch -- the kernel was 13 % slower: eight transform grids
        // instead of one compete for that cache.)
        //
        // On request the list, ordered by place, is cut into 8 ranges, one per XCD (blocks go to the XCDs in turn, so
        // block b runs on XCD b mod 8); a block whose range is used up takes chunks from the next ranges in turn.  The
        // XCD's own L2 then serves 0.72 instead of 0.47 of the requests and a third of the bytes come from beyond it,
        // but the kernel is no faster (1.29 against 1.26 ms with the ordered list behind one cursor): the vector cache
        // in front of the L2 is the limit.
        const bool ranges = S.xcd_ranges != 0;
        const int home = (int)(blockIdx.x & (N_XCD - 1));
        const long long per = ((total + (long long)N_XCD * S.chunk - 1) / ((long long)N_XCD * S.chunk)) * S.chunk;
        long long next, c1;
        if (ranges) {
            const long long r1 = min(total, (home + 1) * per);
            next = home * per + (long long)(blockIdx.x >> 3) * S.chunk;
            c1 = min(r1, next + S.chunk);
        } else {
            next = (long long)blockIdx.x * S.chunk;
            c1 = min(total, next + S.chunk);
        }
        int alive = 0;                    // ranges home, home + 1, ... home + alive - 1 are known to be used up
        int tails[NCONS];
#pragma unroll
        for (int c = 0; c < NCONS; ++c) tails[c] = 0;
        bool lost = false;
        const bool prod_skip = SKIP && __builtin_amdgcn_readfirstlane(*nonfinite) != serial;
        while (!lost) {
            if (next >= c1) {
                if (ranges) {
                    bool got = false;
                    while (alive < N_XCD) {
                        const int j = (home + alive) & (N_XCD - 1);
                        unsigned b = 0;
                        if (lane == 0) b = atomicAdd(cursor + CUR_XCD + j, (unsigned)S.chunk);
                        b = (unsigned)__builtin_amdgcn_readfirstlane((int)b);
                        const long long r1 = min(total, (j + 1) * per), at = j * per + (long long)b;
                        if ((long long)b < per && at < r1) {
                            next = at;
                            c1 = min(r1, at + S.chunk);
                            got = true;
                            break;
                        }
                        ++alive;
                    }
                    if (!got) break;
                } else {
                    unsigned b = 0;
                    if (lane == 0) b = atomicAdd(cursor + CUR_ALL, (unsigned)S.chunk);
                    b = (unsigned)__builtin_amdgcn_readfirstlane((int)b);
                    if ((long long)b >= total) break;
                    next = b;
                    c1 = min(total, (long long)b + S.chunk);
                }
            }
            const long long pq = next + lane;
            next += min(64ll, c1 - next);
            bool keep = false, want_out = false;
            int out_cell = -1, out_flags = 0, pair = 0;
            int nn = 0, nk = 0, np = 0;
            float nxp[3] = {0, 0, 0}, nx[3] = {0, 0, 0}, ng[3] = {0, 0, 0}, ndx[3] = {0, 0, 0};
            float nJ[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
            if (pq < c1) {
                const unsigned upq = (unsigned)pq;        // K * N < 2^31
                int gcell = -1;                           // pose * ncell + correspondence cell, when the list gives it
                if (list) {
                    const int2 e = list[pq];
                    nn = e.x;
                    nk = e.y & 7;
                    gcell = e.y >> 3;
                } else if (S.point_major) {   // consecutive SIMD lanes: the K initial states of one point
                    nn = (int)(upq / (unsigned)S.K);
                    nk = (int)(upq - (unsigned)nn * (unsigned)S.K);
                } else {                      // consecutive SIMD lanes: consecutive points, same initial state
                    nk = (int)(upq / (unsigned)N);
                    nn = (int)(upq - (unsigned)nk * (unsigned)N);
                }
                np = pose_of(pose, nn, G.P);
                pair = (int)((long long)nk * N + nn);
                const float *Tn = T + (long long)np * G.V * 12;
                bool ok, norec = false;     // norec: no record needed, k_solve_unpack knows the answer
                float d[3] = {0, 0, 0};
                int c0lin = 0;              // grid cell of the initial state
#pragma unroll
                for (int r = 0; r < 3; ++r) nxp[r] = xq[r * N + nn];
                if (FUSED && SKIP) {
                    // one state per bone, Eq. (8)
                    const float *bi = I.Binv + ((long long)np * G.nb + nk) * 12;
                    ok = I.Bok[np * G.nb + nk] != 0;
                    if (ok) {
                        const float y[3] = {nxp[0] - bi[9], nxp[1] - bi[10], nxp[2] - bi[11]};
#pragma unroll
                        for (int r = 0; r < 3; ++r)
                            nx[r] = FS_FMA(bi[r * 3 + 0], y[0], FS_FMA(bi[r * 3 + 1], y[1], bi[r * 3 + 2] * y[2]));
                        const Cell c0 = locate(G, nx);
                        c0lin = cell_linear(G, c0);
                        float qn[8][12];
                        // corner records of weight zero contribute nothing to the Jacobian either (the derivative of
                        // their weight vanishes along the clamped axis by definition and carries the zero factor
                        // along the others): fetch the rest, zeros in their place, and if an entry of the blend
                        // or of the Jacobian comes out as an exact zero, do it again with all eight
                        const int need = prod_skip ? corners_needed(c0) : 0xFF;
#pragma unroll
                        for (int c = 0; c < 8; ++c) {
#pragma unroll
                            for (int e = 0; e < 12; ++e) qn[c][e] = 0.0f;
                        }
                        load_corners(Tn + c0.base, G, need, qn);
                        float Jac[9];
                        jacobian_from_corners(G, c0, qn, nx, d, Jac);
                        if (need != 0xFF) {
                            float d2[3];
                            bool z = blend_apply_z(c0, qn, nx, d2);      // the same blend as inside the Jacobian
                            float m = __builtin_fabsf(Jac[0]);
#pragma unroll
                            for (int e = 1; e < 9; ++e) m = __builtin_fminf(m, __builtin_fabsf(Jac[e]));
                            z = z || m == 0.0f;
                            if (z) {
                                load_corners(Tn + c0.base, G, 0xFF & ~need, qn);
                                jacobian_from_corners(G, c0, qn, nx, d, Jac);
                            }
                        }
                        ok = inv3(Jac, nJ);
                        if (!ok) {
#pragma unroll
                            for (int e = 0; e < 9; ++e) nJ[e] = 0.0f;
                        }
                    }
                } else if (FUSED) {
                    // voxel-based candidates: x0, d(x0) and J~0 of a candidate do not depend on the query point and
                    // were computed once per pose (k_corr_init); a lane only looks its candidate up
                    if (gcell < 0) gcell = np * I.C.ncell + cell_index(I.C, I.bbox + np * 6, nxp);
                    const float4 *ci = I.cinit + ((long long)gcell * I.C.ck + nk) * 4;
                    const float4 a = ci[0], b = ci[1], c = ci[2], e = ci[3];
                    const int fl = __float_as_int(a.w);
                    ok = (fl & 1) != 0;
                    norec = (fl & 3) == 0;
                    c0lin = fl >> 2;
                    nx[0] = a.x; nx[1] = a.y; nx[2] = a.z;
                    d[0] = b.x; d[1] = b.y; d[2] = b.z;
                    nJ[0] = b.w; nJ[1] = c.x; nJ[2] = c.y; nJ[3] = c.z; nJ[4] = c.w;
                    nJ[5] = e.x; nJ[6] = e.y; nJ[7] = e.z; nJ[8] = e.w;
                } else {
#pragma unroll
                    for (int r = 0; r < 3; ++r) nx[r] = x0[((long long)nk * 3 + r) * N + nn];
#pragma unroll
                    for (int e = 0; e < 9; ++e) nJ[e] = J0[((long long)nk * 9 + e) * N + nn];
                    ok = valid0[(long long)nk * N + nn] != 0;
                    if (ok) {
                        const Cell c0 = locate(G, nx);
                        c0lin = cell_linear(G, c0);
                        float qn[8][12];
#pragma unroll
                        for (int c = 0; c < 8; ++c) load12(Tn + c0.base + corner_off(G, c), qn[c]);
                        blend_apply(c0, qn, nx, d);
                    }
                }
                if (ok) {
#pragma unroll
                    for (int r = 0; r < 3; ++r) ng[r] = d[r] - nxp[r];
                    const float r2 = FS_FMA(ng[2], ng[2], FS_FMA(ng[1], ng[1], ng[0] * ng[0]));
                    const bool conv = r2 < S.tol2;
                    if (conv || !(r2 < S.div2) || 0 >= S.max_iters) {
                        if (WITH_J) {
                            want_out = true;
                            out_flags = conv ? 1 : 0;
                            if (cell_count && conv) out_cell = np * ncell + c0lin;
                        } else {
                            write_record<false>(rec, pair, nx, nJ, conv ? 1 : 0);
                        }
                    } else {
                        keep = true;
#pragma unroll
                        for (int r = 0; r < 3; ++r)
                            ndx[r] = -FS_FMA(nJ[r * 3 + 2], ng[2], FS_FMA(nJ[r * 3 + 1], ng[1], nJ[r * 3] * ng[0]));
                    }
                }
                if (!ok && !norec) {
                    if (WITH_J) want_out = true;         // out_flags = 0, no position
                    else write_record<false>(rec, pair, nx, nJ, 0);
                }
            }
            const unsigned long long km = __ballot(keep);
            const int nkeep = __popcll(km);
            if (nkeep > 0) {
                // the consumer with the emptiest queue takes the batch; wait while none has room
                int best = 0, room = -1, spins = 0;
                while (true) {
#pragma unroll
                    for (int c = 0; c < NCONS; ++c) {
                        const int r = WS_RING - (tails[c] - __builtin_amdgcn_readfirstlane(lds_load_acquire(&s_head[c])));
                        if (r > room) { room = r; best = c; }
                    }
                    if (room >= nkeep) break;
                    room = -1;
                    if (++spins > S.spin_limit) { lost = true; break; }
                    __builtin_amdgcn_s_sleep(8);
                }
                if (lost) break;
                int tl = 0;
#pragma unroll
                for (int c = 0; c < NCONS; ++c) if (c == best) tl = tails[c];
                if (keep) {
                    const int at = (tl + __popcll(km & ((1ull << lane) - 1ull))) & (WS_RING - 1);
                    float (&ring)[ST_FIELDS][WS_RING] = s_ring[best];
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        ring[ST_XP + r][at] = nxp[r];
                        ring[ST_X + r][at] = nx[r];
                        ring[ST_G + r][at] = ng[r];
                        ring[ST_DX + r][at] = ndx[r];
                    }
#pragma unroll
                    for (int e = 0; e < 9; ++e) ring[ST_J + e][at] = nJ[e];
                    ring[ST_N][at] = __int_as_float(nn);
                    ring[ST_K][at] = __int_as_float(nk);
                    ring[ST_P][at] = __int_as_float(np);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                __builtin_amdgcn_wave_barrier();
                tl += nkeep;
#pragma unroll
                for (int c = 0; c < NCONS; ++c) if (c == best) tails[c] = tl;
                if (lane == 0) lds_store_release(&s_tail[best], tl);
            }
            if (WITH_J) out_park(want_out, nx, nJ, out_flags, out_cell, pair, outq, npend, lane, cell_count, rec);
        }
        if (lost && lane == 0) *give_up = 1;
        if (WITH_J && npend > 0) out_flush(outq, npend, lane, cell_count, rec);
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
        if (lane == 0) lds_store_release(&s_done, 1);
        return;
    }

    // ---------------------------------------------------- consumer ----------------------------------------------------
    float (&ring)[ST_FIELDS][WS_RING] = s_ring[wib];
    bool active = false;
    int n = 0, k = 0, it = 0, pz = 0, head = 0;
    const float *Tp = T;
    float xp[3] = {0, 0, 0}, x[3] = {0, 0, 0}, xt[3] = {0, 0, 0}, g[3] = {0, 0, 0}, dx[3] = {0, 0, 0};
    float J[9] = {0, 0, 0, 0, 0, 0, 0, 0, 0};
    float q[8][12];                  // corner records of the lane's current cell, kept across iterations
    long long held = -1;             // grid offset of the cell whose corners q holds (-1: none)
    int held_mask = 0;               // SKIP: which of them
    // SKIP needs a grid of finite entries (k_precompute says if this one is not)
    const bool may_skip = SKIP && __builtin_amdgcn_readfirstlane(*nonfinite) != serial;
    if (SKIP) {
#pragma unroll
        for (int c = 0; c < 8; ++c)
#pragma unroll
            for (int e = 0; e < 12; ++e) q[c][e] = 0.0f;
    }
    bool run = true;                 // wave-uniform
    while (run) {
        const unsigned long long idle = __ballot(!active);
        const int nidle = __popcll(idle);
        if (nidle >= S.refill_min) {
            const int tail = __builtin_amdgcn_readfirstlane(lds_load_acquire(&s_tail[wib]));
            const int avail = tail - head;
            if (avail > 0) {
                const int rank = __popcll(idle & ((1ull << lane) - 1ull));
                if (!active && rank < avail) {
                    const int e = (head + rank) & (WS_RING - 1);
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        xp[r] = ring[ST_XP + r][e];
                        x[r] = ring[ST_X + r][e];
                        g[r] = ring[ST_G + r][e];
                        dx[r] = ring[ST_DX + r][e];
                    }
#pragma unroll
                    for (int c = 0; c < 9; ++c) J[c] = ring[ST_J + c][e];
                    n = __float_as_int(ring[ST_N][e]);
                    k = __float_as_int(ring[ST_K][e]);
                    pz = __float_as_int(ring[ST_P][e]);
#pragma unroll
                    for (int r = 0; r < 3; ++r) xt[r] = x[r] + dx[r];
                    Tp = T + (long long)pz * G.V * 12;
                    it = 0;
                    held = -1;
                    active = true;
                }
                head += min(nidle, avail);
                __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "workgroup");      // the reads above are done
                __builtin_amdgcn_wave_barrier();
                if (lane == 0) lds_store_release(&s_head[wib], head);
            }
        }
        if (!__any(active)) {
            // nothing in flight: more to come?  (s_done is read before the tail: the producer raises it last)
            const int d = __builtin_amdgcn_readfirstlane(lds_load_acquire(&s_done));
            const int tail = __builtin_amdgcn_readfirstlane(lds_load_acquire(&s_tail[wib]));
            // a consumer waits for nothing but its own block's producer, whose waits are all bounded and which
            // raises s_done on every way out: this loop ends when the producer has
            if (tail == head) {
                if (d) run = false;
                else __builtin_amdgcn_s_sleep(8);
            }
        }
        bool want_out = false;
        int out_cell = -1, out_flags = 0;
        if (active) {
            float d[3], gn[3];
            const Cell cell = locate(G, xt);
            const long long want = (long long)(Tp - T) + cell.base;
            if (SKIP) {
                const int need = may_skip ? corners_needed(cell) : 0xFF;
                if (want != held) {
                    held = want;
                    held_mask = 0;
                }
                if (need & ~held_mask) {
                    load_corners(Tp + cell.base, G, need & ~held_mask, q);
                    held_mask |= need;
                }
                if (blend_apply_z(cell, q, xt, d) && held_mask != 0xFF) {
                    load_corners(Tp + cell.base, G, 0xFF & ~held_mask, q);
                    held_mask = 0xFF;
                    blend_apply(cell, q, xt, d);
                }
            } else {
                if (want != held) {
                    load_cell(Tp + cell.base, G, q);
                    held = want;
                }
                blend_apply(cell, q, xt, d);
            }
#pragma unroll
            for (int r = 0; r < 3; ++r) gn[r] = d[r] - xp[r];
            float dg[3], v[3], u[3];
#pragma unroll
            for (int r = 0; r < 3; ++r) dg[r] = gn[r] - g[r];
#pragma unroll
            for (int c = 0; c < 3; ++c) v[c] = FS_FMA(dx[2], J[6 + c], FS_FMA(dx[1], J[3 + c], dx[0] * J[c]));
#pragma unroll
            for (int r = 0; r < 3; ++r)
                u[r] = dx[r] - FS_FMA(J[r * 3 + 2], dg[2], FS_FMA(J[r * 3 + 1], dg[1], J[r * 3] * dg[0]));
            const float den = FS_FMA(v[2], dg[2], FS_FMA(v[1], dg[1], v[0] * dg[0]));
            if (den != 0.0f && __builtin_fabsf(den) < __builtin_inff()) {
                const float rinv = 1.0f / den;
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const float sc = u[r] * rinv;
#pragma unroll
                    for (int c = 0; c < 3; ++c) J[r * 3 + c] = FS_FMA(sc, v[c], J[r * 3 + c]);
                }
            }
            ++it;
#pragma unroll
            for (int r = 0; r < 3; ++r) { x[r] = xt[r]; g[r] = gn[r]; }
            const float r2 = FS_FMA(g[2], g[2], FS_FMA(g[1], g[1], g[0] * g[0]));
            const bool conv = r2 < S.tol2;
            const bool done = conv || !(r2 < S.div2) || it >= S.max_iters;
            if (done) {
                if (WITH_J) {
                    want_out = true;
                    out_flags = (conv ? 1 : 0) | (it << 8);
                    if (cell_count && conv) out_cell = pz * ncell + cell_linear(G, cell);
                } else {
                    write_record<false>(rec, (long long)k * N + n, x, J, (conv ? 1 : 0) | (it << 8));
                }
                active = false;
            } else {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    dx[r] = -FS_FMA(J[r * 3 + 2], g[2], FS_FMA(J[r * 3 + 1], g[1], J[r * 3] * g[0]));
                    xt[r] = x[r] + dx[r];
                }
                if (!SKIP && S.prefetch) {
                    // the corner records the next pass will need are asked for now: they travel while this pass parks
                    // its results and the next one looks for work (q is free: its records went into d above).  On the
                    // 8-pose grid, whose records come from beyond the L2: 1.34 -> 1.32 ms; on a grid the L2 holds the
                    // second cell lookup costs more than the head start gains (0.172 -> 0.186 ms), hence the switch
                    const Cell cn = locate(G, xt);
                    const long long wn = (long long)(Tp - T) + cn.base;
                    if (wn != held) {
                        load_cell(Tp + cn.base, G, q);
                        held = wn;
                    }
                }
            }
        }
        if (WITH_J) out_park(want_out, x, J, out_flags, out_cell, (int)((long long)k * N + n), outq, npend, lane, cell_count, rec);
    }
    if (WITH_J && npend > 0) out_flush(outq, npend, lane, cell_count, rec);
}

// ------------------------------------------------------------------------------------------------
// Backward (Eq. (11)/(12), (15)).
// ------------------------------------------------------------------------------------------------
// The gradient w.r.t. the transform grid, G_T[p][v] = sum over converged lanes of
// omega_corner * lambda (x) [x*; 1], is accumulated without floating-point atomics (device-scope
// atomics leave the L2 on this chip and are slow): converged lanes are counting-sorted by the grid
// cell of x* (pass 1 below, or the positions k_solve hands out), crowded cells are summed once per
// corner (k_grad_pieces), and every grid node then adds what its 8 adjacent cells hold (k_grad_nodes_p).

// a[0..n) = 0; `cursors` (may be null): the solve kernels' work cursor is reset on the way (as k_reset_cursor does)
__global__ void k_fill_zero_i32(long long n, int *__restrict__ a, unsigned *__restrict__ cursors = nullptr,
                                unsigned nblocks = 0u, unsigned chunk = 0u)
{
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long stride = (long long)gridDim.x * blockDim.x;
    if (cursors && i < N_XCD) reset_cursors(cursors, (int)i, nblocks, chunk);
    for (; i < n; i += stride) a[i] = 0;
}

// pass 1 (only when the solve did not hand out positions): one thread per lane; position of the lane
// inside its cell's list (arrival order)
__global__ __launch_bounds__(256) void k_grad_count(GridP G, const float *__restrict__ xc,
                                                    const uint8_t *__restrict__ conv, const int32_t *__restrict__ pose,
                                                    long long N, int K, int ncell, int *__restrict__ count,
                                                    int *__restrict__ pos)
{
    const long long q = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= N * K) return;
    if (!conv[q]) return;
    const int k = (int)(q / N);
    const long long n = q - (long long)k * N;
    const float x[3] = {xc[((long long)k * 3 + 0) * N + n], xc[((long long)k * 3 + 1) * N + n],
                        xc[((long long)k * 3 + 2) * N + n]};
    const Cell c = locate(G, x);
    const int p = pose_of(pose, n, G.P);
    pos[q] = atomicAdd(count + p * ncell + cell_linear(G, c), 1);
}

// pass 2: a few threads per point share its lanes: lambda = -M^T g_x; the 32-byte record {x*[3], lambda[3],
// cell, 0} goes to the lane's slot of the cell-sorted list (one aligned sector per record);
// dL/dx' = sum_k M^T g_x without atomics.
constexpr int GREC = 8;           // floats per record
// FROM_REC: roots, masks, J~ and positions are taken from the result records the last solve left in the
// context (one contiguous 64-byte record per pair) instead of the caller's arrays; when that solve drew its
// pairs from the candidate list, only the first cand_cnt[n] lanes of point n have a record.
// EXACT: lambda from the inverse of the exact Jacobian at x* (mode != 0) instead of J~; a kernel of its own so that
// the J~ path does not carry the registers of a field evaluation (117 -> what the compiler reports now).
// REC_DEPTH (with FROM_REC and the J~ gradient only): lanes of a point in flight together, see below; 1 = one by one.
// Measured: depth 3 takes k_grad_records from 425 to 376 us on the 8-pose batch (one thread per point) and from 41 to
// 52 us on the SMPL-scale batch (8 threads per point, 5 instead of 8 waves per SIMD), hence a choice per launch.
template <bool FROM_REC, bool EXACT, int REC_DEPTH = 1>
__global__ __launch_bounds__(256) void k_grad_records(GridP G, const float *__restrict__ T,
                                                      const float *__restrict__ xc, const float *__restrict__ Jinv,
                                                      const uint8_t *__restrict__ conv, const float *__restrict__ gxc,
                                                      const int32_t *__restrict__ pose, long long N, int K, int ncell,
                                                      const int *__restrict__ offset, const int *__restrict__ pos,
                                                      float4 *__restrict__ rec, float *__restrict__ gxq, int groups,
                                                      const float4 *__restrict__ srec, const uint8_t *__restrict__ cand_cnt)
{
    // `groups` (a power of two <= 8) threads share a point and take its lanes k = g, g + groups, ...;
    // consecutive threads of a group are consecutive points, so every load is coalesced
    __shared__ float s_gq[256 * 3];
    const int ppb = 256 / groups;                 // points per block
    const int g = threadIdx.x / ppb, i = threadIdx.x - g * ppb;
    const long long n = (long long)blockIdx.x * ppb + i;
    float gq[3] = {0.0f, 0.0f, 0.0f};
    if (n < N) {
        const int p = pose_of(pose, n, G.P);
        const int nk = (FROM_REC && cand_cnt) ? min(K, (int)cand_cnt[n]) : K;
        if constexpr (FROM_REC && !EXACT && REC_DEPTH > 1) {
            // REC_DEPTH lanes of the point at a time, stage by stage, so that the dependent loads of a stage (record head,
            // rest of the record and g_x, cell offsets) travel together
            for (int k0 = g; k0 < nk; k0 += REC_DEPTH * groups) {
                float4 ra[REC_DEPTH], rb[REC_DEPTH], rc[REC_DEPTH], rd[REC_DEPTH];
                float gx[REC_DEPTH][3];
                bool on[REC_DEPTH];
                long long q[REC_DEPTH];
#pragma unroll
                for (int u = 0; u < REC_DEPTH; ++u) {
                    const int k = k0 + u * groups;
                    on[u] = k < nk;
                    q[u] = (long long)(on[u] ? k : 0) * N + n;
                    ra[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    if (on[u]) ra[u] = srec[q[u] * 4];
                }
#pragma unroll
                for (int u = 0; u < REC_DEPTH; ++u) {
                    on[u] = on[u] && (__float_as_int(ra[u].w) & 1);
                    rb[u] = rc[u] = rd[u] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    gx[u][0] = gx[u][1] = gx[u][2] = 0.0f;
                    if (on[u]) {
                        rb[u] = srec[q[u] * 4 + 1];
                        rc[u] = srec[q[u] * 4 + 2];
                        rd[u] = srec[q[u] * 4 + 3];
                        const int k = k0 + u * groups;
#pragma unroll
                        for (int r = 0; r < 3; ++r) gx[u][r] = gxc[((long long)k * 3 + r) * N + n];
                    }
                }
                float lam[REC_DEPTH][3];
                int cl[REC_DEPTH], o0[REC_DEPTH], o1[REC_DEPTH];
#pragma unroll
                for (int u = 0; u < REC_DEPTH; ++u) {
                    const float M[9] = {rb[u].y, rb[u].z, rb[u].w, rc[u].x, rc[u].y, rc[u].z, rc[u].w, rd[u].x, rd[u].y};
                    const float x[3] = {ra[u].x, ra[u].y, ra[u].z};
                    cl[u] = 0;
                    o0[u] = o1[u] = 0;
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        lam[u][r] = -FS_FMA(M[6 + r], gx[u][2], FS_FMA(M[3 + r], gx[u][1], M[r] * gx[u][0]));
                        if (on[u]) gq[r] -= lam[u][r];
                    }
                    if (on[u]) {
                        const Cell c = locate(G, x);
                        cl[u] = p * ncell + cell_linear(G, c);
                        o0[u] = offset[cl[u]];
                        o1[u] = offset[cl[u] + 1];
                    }
                }
#pragma unroll
                for (int u = 0; u < REC_DEPTH; ++u) {
                    const int pq = __float_as_int(rb[u].x);      // the position the solve kernel left in the record
                    const long long slot = (long long)o0[u] + pq;
                    if (!on[u] || pq < 0 || slot >= o1[u]) continue;
                    rec[slot * 2] = make_float4(ra[u].x, ra[u].y, ra[u].z, lam[u][0]);
                    rec[slot * 2 + 1] = make_float4(lam[u][1], lam[u][2], __int_as_float(cl[u]), 0.0f);
                }
            }
        } else
        for (int k = g; k < nk; k += groups) {
            const long long q = (long long)k * N + n;
            float x[3], gx[3], M[9];
            int pq;
            if (FROM_REC) {
                const float4 a = srec[q * 4];
                if (!(__float_as_int(a.w) & 1)) continue;
                x[0] = a.x; x[1] = a.y; x[2] = a.z;
                pq = __float_as_int(srec[q * 4 + 1].x);      // the position the solve kernel left in the record
                if (!EXACT) read_record_J(srec + q * 4, M);
            } else {
                if (!conv[q]) continue;
#pragma unroll
                for (int r = 0; r < 3; ++r) x[r] = xc[((long long)k * 3 + r) * N + n];
                pq = pos[q];
                if (!EXACT) {
#pragma unroll
                    for (int e = 0; e < 9; ++e) M[e] = Jinv[((long long)k * 9 + e) * N + n];
                }
            }
#pragma unroll
            for (int r = 0; r < 3; ++r) gx[r] = gxc[((long long)k * 3 + r) * N + n];
            bool ok = true;
            if (EXACT) {
                float d[3], J[9];
                field_dJ(T + (long long)p * G.V * 12, G, x, d, J);
                ok = inv3(J, M);
            }
            float lam[3] = {0.0f, 0.0f, 0.0f};
            if (ok) {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    lam[r] = -FS_FMA(M[6 + r], gx[2], FS_FMA(M[3 + r], gx[1], M[r] * gx[0]));
                    gq[r] -= lam[r];
                }
            }
            const Cell c = locate(G, x);
            const int cl = p * ncell + cell_linear(G, c);
            const long long slot = (long long)offset[cl] + pq;
            // positions that do not belong to these roots (a caller mixing arrays of different solves)
            // must not send the store outside the cell's part of the list
            if (pq < 0 || slot >= offset[cl + 1]) continue;
            rec[slot * 2] = make_float4(x[0], x[1], x[2], lam[0]);
            rec[slot * 2 + 1] = make_float4(lam[1], lam[2], __int_as_float(cl), 0.0f);
        }
    }
    if (!gxq) return;
#pragma unroll
    for (int r = 0; r < 3; ++r) s_gq[threadIdx.x * 3 + r] = gq[r];
    __syncthreads();
    if (g == 0 && n < N) {
        for (int h = 1; h < groups; ++h)
#pragma unroll
            for (int r = 0; r < 3; ++r) gq[r] += s_gq[(h * ppb + i) * 3 + r];
#pragma unroll
        for (int r = 0; r < 3; ++r) gxq[r * N + n] = gq[r];
    }
}

// fraction of x along one axis inside the cell that starts at node i0: what locate() returns for a point of
// that cell (same clamping, same subtraction), without looking the cell up again
__device__ __forceinline__ float frac_in_cell(float x, float lo, float inv_h, float m, int i0)
{
    float u = (x - lo) * inv_h;
    u = !(u >= 0.0f) ? 0.0f : (u > m ? m : u);
    return u - (float)i0;
}

// contribution of sorted record s, which lies in the cell with origin (cx, cy, cz), to the node that is that
// cell's corner (da, db, dc)
__device__ __forceinline__ void grad_accumulate(const GridP &G, const float *__restrict__ rec, int s, int cx, int cy, int cz,
                                                int da, int db, int dc, float (&acc)[12])
{
    const float4 *r = reinterpret_cast<const float4 *>(rec + (long long)s * GREC);
    const float4 r0 = r[0], r1 = r[1];
    const float x[3] = {r0.x, r0.y, r0.z};
    const float lam[3] = {r0.w, r1.x, r1.y};
    const float fx = frac_in_cell(x[0], G.lo[0], G.inv_h[0], G.m[0], cx);
    const float fy = frac_in_cell(x[1], G.lo[1], G.inv_h[1], G.m[1], cy);
    const float fz = frac_in_cell(x[2], G.lo[2], G.inv_h[2], G.m[2], cz);
    const float wx = da ? fx : 1.0f - fx;
    const float wy = db ? fy : 1.0f - fy;
    const float wz = dc ? fz : 1.0f - fz;
    const float om = (wx * wy) * wz;
#pragma unroll
    for (int rr = 0; rr < 3; ++rr) {
        const float wl = om * lam[rr];
        acc[rr * 4 + 0] = FS_FMA(wl, x[0], acc[rr * 4 + 0]);
        acc[rr * 4 + 1] = FS_FMA(wl, x[1], acc[rr * 4 + 1]);
        acc[rr * 4 + 2] = FS_FMA(wl, x[2], acc[rr * 4 + 2]);
        acc[rr * 4 + 3] += wl;
    }
}

__device__ __forceinline__ int adjacent_cell(const GridP &G, int ncell, int p, int ix, int iy, int iz, int cn)
{
    const int cx = ix - (cn & 1), cy = iy - ((cn >> 1) & 1), cz = iz - ((cn >> 2) & 1);
    if (cx < 0 || cy < 0 || cz < 0 || cx > G.nx - 2 || cy > G.ny - 2 || cz > G.nz - 2) return -1;
    return p * ncell + (cx * (G.ny - 1) + cy) * (G.nz - 1) + cz;
}

// pass 3.  The cell-sorted record list is cut at every multiple of PIECE_R; a piece is what one cell owns
// of one such range.  A piece of at least PIECE_MIN records is replaced, in place, by its sums for the
// 8 corners of the cell (8 x 12 floats = the storage of 12 records), so that a node later reads 12
// floats per piece instead of every record of a crowded cell; shorter pieces stay as records.
constexpr int PIECE_R = 256;
constexpr int PIECE_MIN = 96 / GREC;
constexpr int PIECE_RPL = PIECE_R / 64;   // records per SIMD lane when a wave scans its range
constexpr int PIECE_WAVES = 2;            // waves per range
constexpr int PIECE_OWN = PIECE_R / PIECE_WAVES;   // records a wave loads and expands
constexpr int PIECE_LOAD = PIECE_OWN / 64;         // ... per SIMD lane

// One block of PIECE_WAVES waves per range: the waves share the loading and expanding of the records and
// take the long pieces in turn.  Every record of the range is expanded once (SIMD lane = record) into its 8 corner
// weights omega_c and its 12 products lambda_r [x*; 1]_j, staged in LDS; the sums of a piece are then the
// matrix product  S[c][rj] = sum_t omega_c(t) * (lambda_r [x;1]_j)(t),  an 8 x len by len x 12 contraction,
// taken four records at a time by the 16x16x4 fp32 MFMA (rows 8..15 and columns 12..15 are zero padding).
// Operand layout of that instruction: lane 16k+i supplies A[i][k] and B[k][i]; lane 16g+j receives
// D[4g+q][j] in accumulator register q.
constexpr int PIECE_ROW = 20;     // floats per staged record: 8 weights + 12 products
#ifndef FS_PIECES_VALU
#define FS_PIECES_VALU 0
#endif
typedef float v4f __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(64 * PIECE_WAVES) void k_grad_pieces(GridP G, long long ncp, const int *__restrict__ offset, float *rec)
{
    __shared__ float4 sm4[PIECE_R * PIECE_ROW / 4];
    __shared__ int s_cell[PIECE_R];
    float *sm = reinterpret_cast<float *>(sm4);
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const long long s = (long long)blockIdx.x * PIECE_R;
    const long long total = offset[ncp];
    if (s >= total) return;
    const int e = (int)min((long long)PIECE_R, total - s);
    // each wave loads and expands its share of the range: SIMD lane l of wave w holds records
    // PIECE_OWN * w + l, PIECE_OWN * w + 64 + l, ...
    float4 r0[PIECE_LOAD], r1[PIECE_LOAD];
#pragma unroll
    for (int b = 0; b < PIECE_LOAD; ++b) {
        const int t = PIECE_OWN * w + 64 * b + lane;
        r0[b] = r1[b] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (t < e) {
            const float4 *r = reinterpret_cast<const float4 *>(rec + (s + t) * GREC);
            r0[b] = r[0];
            r1[b] = r[1];
        }
        s_cell[t] = t < e ? __float_as_int(r1[b].z) : -1;
    }
    __syncthreads();
    // every wave finds the pieces of the whole range (same data, same result): lane l looks at records
    // l, 64 + l, 128 + l, ...; a record starts a piece if its cell differs from the one before it (the
    // first of the range always does)
    int c[PIECE_RPL];
    bool f[PIECE_RPL];
#pragma unroll
    for (int b = 0; b < PIECE_RPL; ++b) c[b] = s_cell[64 * b + lane];
#pragma unroll
    for (int b = 0; b < PIECE_RPL; ++b) {
        int prev = __shfl_up(c[b], 1);
        if (lane == 0) prev = -2;
        if (b > 0) {
            const int last = __shfl(c[b - 1], 63);
            if (lane == 0) prev = last;
        }
        f[b] = 64 * b + lane < e && c[b] != prev;
    }
    // next piece start after each record: suffix minimum of the start positions, batch by batch from the end
    int len[PIECE_RPL];
    int later = e;                       // first piece start in later batches
    bool any_long = false;
#pragma unroll
    for (int b = PIECE_RPL - 1; b >= 0; --b) {
        int suf = f[b] ? 64 * b + lane : e;          // first start in lanes >= this one of batch b
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int o = __shfl_down(suf, d);
            if (lane + d < 64) suf = min(suf, o);
        }
        int nxt = __shfl_down(suf, 1);               // ... in lanes after this one
        if (lane == 63) nxt = e;
        nxt = min(nxt, later);
        len[b] = f[b] ? nxt - (64 * b + lane) : 0;
        any_long = any_long || len[b] >= PIECE_MIN;
        later = min(later, __shfl(suf, 0));
    }
    if (!__any(any_long)) return;       // nothing to summarise here (sparse lists end here); same in every wave
    // expand the records
#pragma unroll
    for (int b = 0; b < PIECE_LOAD; ++b) {
        const int t = PIECE_OWN * w + 64 * b + lane;
        float4 o[5];
#pragma unroll
        for (int h = 0; h < 5; ++h) o[h] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (t < e) {
            const float x[3] = {r0[b].x, r0[b].y, r0[b].z};
            const float lam[3] = {r0[b].w, r1[b].x, r1[b].y};
            const Cell cl = locate(G, x);
            float om[8];
            corner_weights(cl, om);
            o[0] = make_float4(om[0], om[1], om[2], om[3]);
            o[1] = make_float4(om[4], om[5], om[6], om[7]);
#pragma unroll
            for (int rr = 0; rr < 3; ++rr) o[2 + rr] = make_float4(lam[rr] * x[0], lam[rr] * x[1], lam[rr] * x[2], lam[rr]);
        }
#pragma unroll
        for (int h = 0; h < 5; ++h) sm4[t * (PIECE_ROW / 4) + h] = o[h];
    }
    __syncthreads();
    const int col = lane & 15, kq = lane >> 4;
    int turn = 0;                        // the waves take the long pieces in turn
#pragma unroll
    for (int i = 0; i < PIECE_RPL; ++i) {
        unsigned long long m = __ballot(len[i] >= PIECE_MIN);
        while (m) {
            const int src = __ffsll((long long)m) - 1;
            m &= m - 1ull;
            const bool mine = turn == w;
            turn = turn + 1 == PIECE_WAVES ? 0 : turn + 1;
            if (!mine) continue;
            const int ps = 64 * i + src, pe = ps + __shfl(len[i], src);
            // four groups per pass into four accumulators: their LDS reads are in flight together and no
            // MFMA waits for the one before it; records outside the piece enter as zeros
#if FS_PIECES_VALU
            // the same sums with vector FMAs, for comparison: lane (kq, col) takes rows 2 kq, 2 kq + 1 of column col
            {
                float a0 = 0.0f, a1 = 0.0f, b0 = 0.0f, b1 = 0.0f;
                if (col < 12) {
                    int t = ps;
                    for (; t + 1 < pe; t += 2) {
                        const float2 w0 = *reinterpret_cast<const float2 *>(sm + t * PIECE_ROW + 2 * kq);
                        const float2 w1 = *reinterpret_cast<const float2 *>(sm + (t + 1) * PIECE_ROW + 2 * kq);
                        const float p0 = sm[t * PIECE_ROW + 8 + col], p1 = sm[(t + 1) * PIECE_ROW + 8 + col];
                        a0 = FS_FMA(w0.x, p0, a0); a1 = FS_FMA(w0.y, p0, a1);
                        b0 = FS_FMA(w1.x, p1, b0); b1 = FS_FMA(w1.y, p1, b1);
                    }
                    if (t < pe) {
                        const float2 w0 = *reinterpret_cast<const float2 *>(sm + t * PIECE_ROW + 2 * kq);
                        const float p0 = sm[t * PIECE_ROW + 8 + col];
                        a0 = FS_FMA(w0.x, p0, a0); a1 = FS_FMA(w0.y, p0, a1);
                    }
                    float *o = rec + (s + ps) * GREC + (2 * kq) * 12 + col;
                    o[0] = a0 + b0;
                    o[12] = a1 + b1;
                }
                continue;
            }
#endif
            v4f acc4[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) acc4[u] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
            const int g1 = (pe - 1) >> 2;
            for (int g = ps >> 2; g <= g1; g += 4) {
                float av[4], bv[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int t = 4 * (g + u) + kq;
                    const bool in = t >= ps && t < pe;          // pe <= PIECE_R
                    av[u] = (in && col < 8) ? sm[t * PIECE_ROW + col] : 0.0f;
                    bv[u] = (in && col < 12) ? sm[t * PIECE_ROW + 8 + col] : 0.0f;
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) acc4[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[u], bv[u], acc4[u], 0, 0, 0);
            }
            const v4f acc = (acc4[0] + acc4[1]) + (acc4[2] + acc4[3]);
            if (kq < 2 && col < 12) {
                float *o = rec + (s + ps) * GREC + (4 * kq) * 12 + col;
                o[0] = acc[0];
                o[12] = acc[1];
                o[24] = acc[2];
                o[36] = acc[3];
            }
        }
    }
}

// G_T of every node from the pieces of its 8 adjacent cells; TPN threads share a node (1, or 8 = one
// per adjacent cell followed by a butterfly sum).
// Measured on the multi-pose batch (7.7 M records over 4.2 M nodes, TPN = 1: 450 us) and not adopted: a block per brick
// of 4 x 4 x 16 nodes that first copies the records of the cells around it into LDS and gathers from there, same loops:
// 450 .. 518 us (fewer resident threads, three barriers per block); the same with one loop over all records of a node's
// 8 cells instead of a loop per cell: 751 us (the bookkeeping costs more than the shorter loop saves); a block per brick
// that adds every record's 8 x 12 contributions into LDS sums with LDS float atomics: 4.5 ms (about 0.5 SIMD lanes per
// clock and CU).
template <int TPN>
__global__ __launch_bounds__(256) void k_grad_nodes_p(GridP G, int ncell, const int *__restrict__ offset,
                                                      const float *__restrict__ rec, float *__restrict__ GT)
{
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long i = t / TPN;
    const int sub = (int)(t - i * TPN);
    if (i >= (long long)G.P * G.V) return;
    const int p = (int)div_by((unsigned)i, (unsigned)G.V, G.mag_V);          // P * V < 2^31
    const unsigned v = (unsigned)(i - (long long)p * G.V), tz = div_by(v, (unsigned)G.nz, G.mag_nz);
    const int iz = (int)(v - tz * (unsigned)G.nz), ix = (int)div_by(tz, (unsigned)G.ny, G.mag_ny);
    const int iy = (int)(tz - (unsigned)ix * (unsigned)G.ny);
    float acc[12];
#pragma unroll
    for (int e = 0; e < 12; ++e) acc[e] = 0.0f;
    for (int cn = sub; cn < 8; cn += TPN) {
        const int c = adjacent_cell(G, ncell, p, ix, iy, iz, cn);
        if (c < 0) continue;
        const int a = offset[c], b = offset[c + 1];
        if (a == b) continue;
        for (int j = a / PIECE_R; j <= (b - 1) / PIECE_R; ++j) {
            const int ps = max(a, j * PIECE_R), pe = min(b, (j + 1) * PIECE_R);
            if (pe - ps >= PIECE_MIN) {
                const float4 *q = reinterpret_cast<const float4 *>(rec + (long long)ps * GREC + cn * 12);
#pragma unroll
                for (int h = 0; h < 3; ++h) {
                    const float4 u = q[h];
                    acc[4 * h] += u.x;
                    acc[4 * h + 1] += u.y;
                    acc[4 * h + 2] += u.z;
                    acc[4 * h + 3] += u.w;
                }
            } else {
                for (int s = ps; s < pe; ++s)
                    grad_accumulate(G, rec, s, ix - (cn & 1), iy - ((cn >> 1) & 1), iz - ((cn >> 2) & 1), cn & 1, (cn >> 1) & 1,
                                    (cn >> 2) & 1, acc);
            }
        }
    }
    if (TPN > 1) {
#pragma unroll
        for (int e = 0; e < 12; ++e) {
#pragma unroll
            for (int d = TPN >> 1; d >= 1; d >>= 1) acc[e] += __shfl_xor(acc[e], d);
        }
    }
    if (sub == 0) {
        float4 *o = reinterpret_cast<float4 *>(GT + i * 12);
        o[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        o[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
        o[2] = make_float4(acc[8], acc[9], acc[10], acc[11]);
    }
}

// What the records of cell (cx, cy, cz), list entries [a, b), add to the two nodes at its (x, y) corner `ab`
// (= a + 2b): `lo` is the node at cz, `hi` the one at cz + 1.  Pieces that k_grad_pieces replaced by their corner
// sums enter as those sums.  Either output may be switched off.
// one record {x*, lambda} of the cell with origin (cx, cy, cz): its share for the cell's (x, y) corner `ab` at the lower
// z (into lo) and at the upper z (into hi)
template <bool LO, bool HI>
__device__ __forceinline__ void grad_record_pair(const GridP &G, const float4 r0, const float4 r1, int ab, int cx, int cy,
                                                 int cz, float (&lo)[12], float (&hi)[12])
{
    const float x[3] = {r0.x, r0.y, r0.z};
    const float lam[3] = {r0.w, r1.x, r1.y};
    const float fx = frac_in_cell(x[0], G.lo[0], G.inv_h[0], G.m[0], cx);
    const float fy = frac_in_cell(x[1], G.lo[1], G.inv_h[1], G.m[1], cy);
    const float fz = frac_in_cell(x[2], G.lo[2], G.inv_h[2], G.m[2], cz);
    const float wxy = ((ab & 1) ? fx : 1.0f - fx) * ((ab & 2) ? fy : 1.0f - fy);
    const float w0 = wxy * (1.0f - fz), w1 = wxy * fz;
#pragma unroll
    for (int rr = 0; rr < 3; ++rr) {
        if (LO) {
            const float wl = w0 * lam[rr];
            lo[rr * 4 + 0] = FS_FMA(wl, x[0], lo[rr * 4 + 0]);
            lo[rr * 4 + 1] = FS_FMA(wl, x[1], lo[rr * 4 + 1]);
            lo[rr * 4 + 2] = FS_FMA(wl, x[2], lo[rr * 4 + 2]);
            lo[rr * 4 + 3] += wl;
        }
        if (HI) {
            const float wl = w1 * lam[rr];
            hi[rr * 4 + 0] = FS_FMA(wl, x[0], hi[rr * 4 + 0]);
            hi[rr * 4 + 1] = FS_FMA(wl, x[1], hi[rr * 4 + 1]);
            hi[rr * 4 + 2] = FS_FMA(wl, x[2], hi[rr * 4 + 2]);
            hi[rr * 4 + 3] += wl;
        }
    }
}

template <bool LO, bool HI>
__device__ __forceinline__ void grad_cell_pair(const GridP &G, const float *__restrict__ rec, int a, int b, int ab, int cx,
                                               int cy, int cz, float (&lo)[12], float (&hi)[12])
{
    for (int j = a / PIECE_R; j <= (b - 1) / PIECE_R; ++j) {
        const int ps = max(a, j * PIECE_R), pe = min(b, (j + 1) * PIECE_R);
        if (pe - ps >= PIECE_MIN) {
            const float4 *q0 = reinterpret_cast<const float4 *>(rec + (long long)ps * GREC + ab * 12);
            const float4 *q1 = q0 + 12;                   // corner ab + 4
#pragma unroll
            for (int h = 0; h < 3; ++h) {
                if (LO) {
                    const float4 u = q0[h];
                    lo[4 * h] += u.x; lo[4 * h + 1] += u.y; lo[4 * h + 2] += u.z; lo[4 * h + 3] += u.w;
                }
                if (HI) {
                    const float4 u = q1[h];
                    hi[4 * h] += u.x; hi[4 * h + 1] += u.y; hi[4 * h + 2] += u.z; hi[4 * h + 3] += u.w;
                }
            }
        } else {
            for (int s = ps; s < pe; ++s) {
                const float4 *r = reinterpret_cast<const float4 *>(rec + (long long)s * GREC);
                grad_record_pair<LO, HI>(G, r[0], r[1], ab, cx, cy, cz, lo, hi);
            }
        }
    }
}

// G_T of every node for sparse lists (a few records per cell): one thread per node, consecutive SIMD lanes consecutive
// nodes along z.  A node-by-node gather over its 8 adjacent cells reads every record 8 times, and a wave runs as long
// as the sum over the 8 cells of the longest list among its lanes.  Here a lane walks only the 4 cells at its own height
// (cz = iz), adds each record's share for the lower z-corner to its own node and collects the share for the upper
// z-corner, which belongs to the node above it: the next SIMD lane, which receives it with one shuffle per entry.  Every
// record is read 4 times and the loops are half as long.  A lane whose lower neighbour sits in another wave (lane 0 of
// a wave that starts inside a column) walks that neighbour's 4 cells itself.
__global__ __launch_bounds__(256) void k_grad_nodes_z(GridP G, int ncell, const int *__restrict__ offset,
                                                      const float *__restrict__ rec, float *__restrict__ GT)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const int lane = threadIdx.x & 63;
    const bool valid = i < (long long)G.P * G.V;
    int p = 0, ix = 0, iy = 0, iz = 0;
    if (valid) {
        p = (int)div_by((unsigned)i, (unsigned)G.V, G.mag_V);          // P * V < 2^31
        const unsigned v = (unsigned)(i - (long long)p * G.V), t = div_by(v, (unsigned)G.nz, G.mag_nz);
        iz = (int)(v - t * (unsigned)G.nz);
        ix = (int)div_by(t, (unsigned)G.ny, G.mag_ny);
        iy = (int)(t - (unsigned)ix * (unsigned)G.ny);
    }
    float acc[12], up[12];
#pragma unroll
    for (int e = 0; e < 12; ++e) acc[e] = up[e] = 0.0f;
    if (valid && iz <= G.nz - 2) {
        // Cells with fewer than PIECE_MIN records hold records only (no sums): those of the 4 cells are walked side by
        // side, record j of each in one round, so that a round's loads travel together and the loop is as long as the
        // longest of the four lists instead of their sum (two records of each cell per round: 309 instead of 270 us, the
        // extra registers cost two of six waves per SIMD).  The other cells follow one by one.
        int a[4], b[4];
        bool small[4];
        int rounds = 0;
#pragma unroll
        for (int ab = 0; ab < 4; ++ab) {
            const int cx = ix - (ab & 1), cy = iy - (ab >> 1);
            a[ab] = b[ab] = 0;
            if (!(cx < 0 || cy < 0 || cx > G.nx - 2 || cy > G.ny - 2)) {
                const int c = p * ncell + (cx * (G.ny - 1) + cy) * (G.nz - 1) + iz;
                a[ab] = offset[c];
                b[ab] = offset[c + 1];
            }
            small[ab] = b[ab] - a[ab] < PIECE_MIN;
            if (small[ab]) rounds = max(rounds, b[ab] - a[ab]);
        }
        for (int j = 0; j < rounds; ++j) {
            float4 r0[4], r1[4];
            bool on[4];
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) {
                on[ab] = small[ab] && a[ab] + j < b[ab];
                const float4 *r = reinterpret_cast<const float4 *>(rec + (long long)(on[ab] ? a[ab] + j : 0) * GREC);
                r0[ab] = r1[ab] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (on[ab]) { r0[ab] = r[0]; r1[ab] = r[1]; }
            }
#pragma unroll
            for (int ab = 0; ab < 4; ++ab)
                if (on[ab]) grad_record_pair<true, true>(G, r0[ab], r1[ab], ab, ix - (ab & 1), iy - (ab >> 1), iz, acc, up);
        }
#pragma unroll
        for (int ab = 0; ab < 4; ++ab)
            if (!small[ab]) grad_cell_pair<true, true>(G, rec, a[ab], b[ab], ab, ix - (ab & 1), iy - (ab >> 1), iz, acc, up);
    }
    // what the node below collected for this one (lane - 1 is node i - 1: the same column when iz > 0)
    const bool from_lane = lane > 0 && valid && iz > 0;
#pragma unroll
    for (int e = 0; e < 12; ++e) {
        const float below = __shfl_up(up[e], 1);
        if (from_lane) acc[e] += below;
    }
    if (valid && iz > 0 && !from_lane) {
        for (int ab = 0; ab < 4; ++ab) {
            const int cx = ix - (ab & 1), cy = iy - (ab >> 1);
            if (cx < 0 || cy < 0 || cx > G.nx - 2 || cy > G.ny - 2) continue;
            const int c = p * ncell + (cx * (G.ny - 1) + cy) * (G.nz - 1) + iz - 1;
            const int a = offset[c], b = offset[c + 1];
            if (a != b) grad_cell_pair<false, true>(G, rec, a, b, ab, cx, cy, iz - 1, up, acc);
        }
    }
    // the wave's 64 records are contiguous: they leave as whole cache lines
    __shared__ __attribute__((aligned(16))) float s_tiles[4][64 * 12];
    const long long i0 = i - lane;
    wave_store_rows<12>(GT + i0 * 12, acc, (int)min(64ll, (long long)G.P * G.V - i0), s_tiles[threadIdx.x >> 6]);
}

// gW[v][b] = sum_p sum_e G_T[p][v][e] B[p][b][e]: one thread per node and group of 8 bones (groups of a node
// in neighbouring threads, so the node's G_T records come from the same cache lines and the stores are
// contiguous); the bone transforms are staged in LDS.
__global__ __launch_bounds__(256) void k_grad_weights_node(GridP G, const float *__restrict__ GT,
                                                           const float *__restrict__ B, float *__restrict__ gW)
{
    extern __shared__ float sB[];
    const int nB = G.P * G.nb * 12;
    for (int i = threadIdx.x; i < nB; i += blockDim.x) sB[i] = B[i];
    __syncthreads();
    const int nch = (G.nb + 7) / 8;
    const long long t = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    const long long v = t / nch;
    const int b0 = (int)(t - v * nch) * 8;
    if (v >= G.V) return;
    float acc[8];
#pragma unroll
    for (int bb = 0; bb < 8; ++bb) acc[bb] = 0.0f;
    for (int p = 0; p < G.P; ++p) {
        float gt[12];
        load12(GT + ((long long)p * G.V + v) * 12, gt);
#pragma unroll
        for (int bb = 0; bb < 8; ++bb) {
            if (b0 + bb < G.nb) {
                const float4 *Bp = reinterpret_cast<const float4 *>(sB + ((long long)p * G.nb + b0 + bb) * 12);
                const float4 u0 = Bp[0], u1 = Bp[1], u2 = Bp[2];
                const float bq[12] = {u0.x, u0.y, u0.z, u0.w, u1.x, u1.y, u1.z, u1.w, u2.x, u2.y, u2.z, u2.w};
#pragma unroll
                for (int e = 0; e < 12; ++e) acc[bb] = FS_FMA(gt[e], bq[e], acc[bb]);
            }
        }
    }
    float *o = gW + v * G.nb + b0;
    if ((G.nb & 3) == 0 && b0 + 8 <= G.nb) {
        reinterpret_cast<float4 *>(o)[0] = make_float4(acc[0], acc[1], acc[2], acc[3]);
        reinterpret_cast<float4 *>(o)[1] = make_float4(acc[4], acc[5], acc[6], acc[7]);
    } else {
#pragma unroll
        for (int bb = 0; bb < 8; ++bb)
            if (b0 + bb < G.nb) o[bb] = acc[bb];
    }
}

// gB[p][b][e] = sum_v W[v][b] G_T[p][v][e]: per pose an n_b x V by V x 12 product with a long inner dimension.
// Each wave walks its share of the nodes four at a time with the 16x16x4 fp32 MFMA (A = 16 bones x 4 nodes of
// W^T, B = 4 nodes x 12 entries of G_T), up to 8 poses against the same weights; a block of 4 waves writes one
// partial result [n_b][12] per pose (part[p][block]) and k_grad_bones_final adds the partials.  MT = number of 16-bone tiles.
constexpr int GB_POSES = 8;
#ifndef FS_GB_QUADS
#define FS_GB_QUADS 4
#endif
constexpr int GB_QUADS = FS_GB_QUADS;
template <int MT>
__global__ __launch_bounds__(256) void k_grad_bones_mfma(GridP G, const float *__restrict__ W,
                                                         const float *__restrict__ GT, float *__restrict__ part,
                                                         int nparts)
{
    const int lane = threadIdx.x & 63;
    const int wave = (blockIdx.x * blockDim.x + threadIdx.x) >> 6;      // < nparts
    const int p0 = blockIdx.y * GB_POSES;
    const int np = min(GB_POSES, G.P - p0);
    const int col = lane & 15, kq = lane >> 4;
    const long long quads = (G.V + 3) / 4;
    v4f acc[GB_POSES][MT];
#pragma unroll
    for (int pc = 0; pc < GB_POSES; ++pc)
#pragma unroll
        for (int mt = 0; mt < MT; ++mt) acc[pc][mt] = (v4f){0.0f, 0.0f, 0.0f, 0.0f};
    // GB_QUADS node quads per pass: their loads are in flight together
    for (long long q = wave; q < quads; q += (long long)GB_QUADS * nparts) {
        float a[GB_QUADS][MT], bv[GB_QUADS][GB_POSES];
#pragma unroll
        for (int u = 0; u < GB_QUADS; ++u) {
            const long long v = (q + (long long)u * nparts) * 4 + kq;
            const bool inv = v < G.V;
#pragma unroll
            for (int mt = 0; mt < MT; ++mt)
                a[u][mt] = (inv && mt * 16 + col < G.nb) ? W[v * G.nb + mt * 16 + col] : 0.0f;
#pragma unroll
            for (int pc = 0; pc < GB_POSES; ++pc)
                bv[u][pc] = (pc < np && inv && col < 12) ? GT[((long long)(p0 + pc) * G.V + v) * 12 + col] : 0.0f;
        }
#pragma unroll
        for (int pc = 0; pc < GB_POSES; ++pc) {
            if (pc < np) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt)
#pragma unroll
                    for (int u = 0; u < GB_QUADS; ++u)
                        acc[pc][mt] = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u][mt], bv[u][pc], acc[pc][mt], 0, 0, 0);
            }
        }
    }
    // the block's 4 waves add their results in LDS, pose by pose; wave 0 writes the block's partial
    __shared__ v4f s_acc[3][MT][64];
    const int nout = G.nb * 12, wib = threadIdx.x >> 6;
#pragma unroll
    for (int pc = 0; pc < GB_POSES; ++pc) {
        if (pc < np) {                                  // np is the same for the whole block
            if (wib > 0) {
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) s_acc[wib - 1][mt][lane] = acc[pc][mt];
            }
            __syncthreads();
            if (wib == 0) {
                float *o = part + ((long long)(p0 + pc) * gridDim.x + blockIdx.x) * nout;
#pragma unroll
                for (int mt = 0; mt < MT; ++mt) {
                    const v4f t = acc[pc][mt] + s_acc[0][mt][lane] + s_acc[1][mt][lane] + s_acc[2][mt][lane];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int b = mt * 16 + 4 * kq + r;
                        if (b < G.nb && col < 12) o[b * 12 + col] = t[r];
                    }
                }
            }
            __syncthreads();
        }
    }
}

// sum of the per-block partial results of k_grad_bones_mfma: one wave per output
__global__ __launch_bounds__(64) void k_grad_bones_final(int P, int nblk, int nout, const float *__restrict__ part,
                                                         float *__restrict__ gB)
{
    const int i = blockIdx.x;
    if (i >= P * nout) return;
    const int p = i / nout, o = i - p * nout;
    float a = 0.0f;
    for (int b = threadIdx.x; b < nblk; b += WAVE) a += part[((long long)p * nblk + b) * nout + o];
#pragma unroll
    for (int s = 32; s >= 1; s >>= 1) a += __shfl_xor(a, s);
    if (threadIdx.x == 0) gB[i] = a;
}

// ------------------------------------------------------------------------------------------------
// Duplicate removal (Sec. 3.1 "Remove Duplicate Correspondences") and packing of the surviving roots.
// One thread per point; lanes in increasing k; a converged lane is kept iff no lane kept before it is
// closer than min_dist.  The kept set lives in a 64-bit mask; kept roots are re-read when needed.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_dedupe(long long N, int K, float md2, const float *__restrict__ xc,
                                                const uint8_t *__restrict__ conv, uint8_t *__restrict__ keep,
                                                int *__restrict__ count)
{
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    unsigned long long kept = 0ull;
    for (int k = 0; k < K; ++k) {
        bool kp = conv[(long long)k * N + n] != 0;
        if (kp) {
            const float x0 = xc[((long long)k * 3 + 0) * N + n], x1 = xc[((long long)k * 3 + 1) * N + n],
                        x2 = xc[((long long)k * 3 + 2) * N + n];
            unsigned long long m = kept;
            while (m && kp) {
                const int j = __builtin_ctzll(m);
                m &= m - 1ull;
                const float e0 = x0 - xc[((long long)j * 3 + 0) * N + n], e1 = x1 - xc[((long long)j * 3 + 1) * N + n],
                            e2 = x2 - xc[((long long)j * 3 + 2) * N + n];
                const float d2 = FS_FMA(e2, e2, FS_FMA(e1, e1, e0 * e0));
                if (d2 < md2) kp = false;
            }
        }
        if (kp) kept |= 1ull << k;
        keep[(long long)k * N + n] = kp ? 1 : 0;
    }
    count[n] = __popcll(kept);
}

// packed list: roots [total][3] and lane index k, point n owns entries offsets[n] .. offsets[n+1]
__global__ __launch_bounds__(256) void k_pack_roots(long long N, int K, long long cap, const float *__restrict__ xc,
                                                    const uint8_t *__restrict__ keep, const int *__restrict__ offsets,
                                                    float *__restrict__ roots, int32_t *__restrict__ lane)
{
    const long long n = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    long long o = offsets[n];
    for (int k = 0; k < K; ++k) {
        if (!keep[(long long)k * N + n]) continue;
        if (o < cap) {
            if (roots) {
                roots[o * 3 + 0] = xc[((long long)k * 3 + 0) * N + n];
                roots[o * 3 + 1] = xc[((long long)k * 3 + 1) * N + n];
                roots[o * 3 + 2] = xc[((long long)k * 3 + 2) * N + n];
            }
            if (lane) lane[o] = k;
        }
        ++o;
    }
}

}  // namespace fs
