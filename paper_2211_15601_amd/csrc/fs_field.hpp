// Device-side field arithmetic: tri-linear lookup of the transform grid, forward map d(x) = T(x) x,
// analytic Jacobian, 3x3 inverse.  IEEE fp32 throughout; every multiply-add that is meant to be
// fused is an explicit __builtin_fmaf and the file is compiled with -ffp-contract=off, so the
// rounding sequence is fixed by the source text.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fs {

struct GridP {
    int nx, ny, nz, nb, P;
    int sx, sy;          // float strides between x- and y-neighbours (z-neighbours are 12 apart)
    long long V;         // nodes per pose
    float lo[3], hi[3], inv_h[3], h[3], m[3];   // m = n-1 as float
    unsigned mag_ny, mag_nz, mag_V;             // floor(2^32 / ny), floor(2^32 / nz), floor(2^32 / V), at most 2^32 - 1 (div_magic)
};

// v / d for a divisor that is the same for the whole launch, with m = div_magic(d) = min(floor(2^32 / d), 2^32 - 1):
// the high half of v * m is the quotient or one less (v * m / 2^32 > v / d - 1), which one comparison settles.
// The machine has no integer divide: v / d in plain C costs about 35 instructions, this 5.
__host__ __device__ inline unsigned div_magic(unsigned d)
{
    const unsigned long long m = (1ull << 32) / (d ? d : 1u);
    return m > 0xffffffffull ? 0xffffffffu : (unsigned)m;
}
__device__ __forceinline__ unsigned div_by(unsigned v, unsigned d, unsigned m)
{
    unsigned q = __umulhi(v, m);
    if (v - q * d >= d) ++q;
    return q;
}

#define FS_FMA(a, b, c) __builtin_fmaf((a), (b), (c))
#define FS_DET_EPS 1e-12f

struct Cell {
    int base;        // float offset of corner (0,0,0) inside one pose's grid
    int ci[3];       // the cell's index along x, y, z
    float f[3];
    bool cl[3];      // coordinate was clamped to the box along this axis
};

__device__ __forceinline__ void locate_axis(float x, float lo, float inv_h, float m, int n, int &i0, float &f, bool &cl)
{
    float u = (x - lo) * inv_h;
    bool below = !(u >= 0.0f);          // also true for NaN
    bool above = u > m;
    cl = below || above;
    u = below ? 0.0f : (above ? m : u);
    int i = (int)__builtin_floorf(u);
    i = i > n - 2 ? n - 2 : i;
    i0 = i;
    f = u - (float)i;
}

__device__ __forceinline__ Cell locate(const GridP &G, const float x[3])
{
    Cell c;
    int ix, iy, iz;
    locate_axis(x[0], G.lo[0], G.inv_h[0], G.m[0], G.nx, ix, c.f[0], c.cl[0]);
    locate_axis(x[1], G.lo[1], G.inv_h[1], G.m[1], G.ny, iy, c.f[1], c.cl[1]);
    locate_axis(x[2], G.lo[2], G.inv_h[2], G.m[2], G.nz, iz, c.f[2], c.cl[2]);
    c.base = ix * G.sx + iy * G.sy + iz * 12;
    c.ci[0] = ix;
    c.ci[1] = iy;
    c.ci[2] = iz;
    return c;
}

// linear index of the cell among the (nx-1)(ny-1)(nz-1) cells of one pose
__device__ __forceinline__ int cell_linear(const GridP &G, const Cell &c)
{
    return (c.ci[0] * (G.ny - 1) + c.ci[1]) * (G.nz - 1) + c.ci[2];
}

// corner c = a + 2b + 4cz with offsets (a, b, cz) along (x, y, z)
__device__ __forceinline__ int corner_off(const GridP &G, int c)
{
    return (c & 1) * G.sx + ((c >> 1) & 1) * G.sy + ((c >> 2) & 1) * 12;
}

__device__ __forceinline__ void load12(const float *__restrict__ p, float (&o)[12])
{
    const float4 a = *reinterpret_cast<const float4 *>(p);
    const float4 b = *reinterpret_cast<const float4 *>(p + 4);
    const float4 c = *reinterpret_cast<const float4 *>(p + 8);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
    o[8] = c.x; o[9] = c.y; o[10] = c.z; o[11] = c.w;
}

__device__ __forceinline__ void corner_weights(const Cell &c, float (&om)[8])
{
    const float wx[2] = {1.0f - c.f[0], c.f[0]};
    const float wy[2] = {1.0f - c.f[1], c.f[1]};
    const float wz[2] = {1.0f - c.f[2], c.f[2]};
#pragma unroll
    for (int k = 0; k < 8; ++k) om[k] = (wx[k & 1] * wy[(k >> 1) & 1]) * wz[(k >> 2) & 1];
}

__device__ __forceinline__ void apply12(const float (&T)[12], const float x[3], float d[3])
{
#pragma unroll
    for (int r = 0; r < 3; ++r)
        d[r] = FS_FMA(T[r * 4 + 0], x[0], FS_FMA(T[r * 4 + 1], x[1], FS_FMA(T[r * 4 + 2], x[2], T[r * 4 + 3])));
}

// Blend the 8 corner transforms q[c] (c = a + 2b + 4cz) with the tri-linear weights of `c` in corner
// order (first term a product, the rest fused multiply-adds) and apply the result to x: Eq. (4)/(5).
__device__ __forceinline__ void blend_apply(const Cell &c, const float (&q)[8][12], const float x[3], float d[3])
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
}

// Forward map of Eq. (5) with T(x) interpolated from the grid of one pose (Tp).
__device__ __forceinline__ void field_d(const float *__restrict__ Tp, const GridP &G, const float x[3], float d[3])
{
    const Cell c = locate(G, x);
    float q[8][12];
#pragma unroll
    for (int k = 0; k < 8; ++k) load12(Tp + c.base + corner_off(G, k), q[k]);
    blend_apply(c, q, x, d);
}

// Forward map plus spatial Jacobian dd/dx (row-major 3x3) from the 8 corner records q of cell c:
// interpolated rotation part plus the derivative of the interpolation weights applied to every
// corner's image of x; no weight derivative along an axis on which the lookup was clamped.
__device__ __forceinline__ void jacobian_from_corners(const GridP &G, const Cell &c, const float (&q)[8][12],
                                                      const float x[3], float d[3], float J[9])
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
    const float wx[2] = {1.0f - c.f[0], c.f[0]};
    const float wy[2] = {1.0f - c.f[1], c.f[1]};
    const float wz[2] = {1.0f - c.f[2], c.f[2]};
#pragma unroll
    for (int r = 0; r < 3; ++r)
#pragma unroll
        for (int j = 0; j < 3; ++j) J[r * 3 + j] = T[r * 4 + j];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const int a = k & 1, b = (k >> 1) & 1, cz = (k >> 2) & 1;
        float dc[3];
        apply12(q[k], x, dc);
        float dw[3];
        dw[0] = c.cl[0] ? 0.0f : (a ? G.inv_h[0] : -G.inv_h[0]) * (wy[b] * wz[cz]);
        dw[1] = c.cl[1] ? 0.0f : (b ? G.inv_h[1] : -G.inv_h[1]) * (wx[a] * wz[cz]);
        dw[2] = c.cl[2] ? 0.0f : (cz ? G.inv_h[2] : -G.inv_h[2]) * (wx[a] * wy[b]);
#pragma unroll
        for (int r = 0; r < 3; ++r)
#pragma unroll
            for (int j = 0; j < 3; ++j) J[r * 3 + j] = FS_FMA(dw[j], dc[r], J[r * 3 + j]);
    }
}

__device__ __forceinline__ void field_dJ(const float *__restrict__ Tp, const GridP &G, const float x[3],
                                         float d[3], float J[9])
{
    const Cell c = locate(G, x);
    float q[8][12];
#pragma unroll
    for (int k = 0; k < 8; ++k) load12(Tp + c.base + corner_off(G, k), q[k]);
    jacobian_from_corners(G, c, q, x, d, J);
}

// Adjugate / determinant inverse of a row-major 3x3; false if |det| < 1e-12 or NaN.
__device__ __forceinline__ bool inv3(const float m[9], float o[9])
{
    const float c00 = FS_FMA(m[4], m[8], -(m[5] * m[7]));
    const float c01 = FS_FMA(m[5], m[6], -(m[3] * m[8]));
    const float c02 = FS_FMA(m[3], m[7], -(m[4] * m[6]));
    const float det = FS_FMA(m[0], c00, FS_FMA(m[1], c01, m[2] * c02));
    if (!(__builtin_fabsf(det) >= FS_DET_EPS)) return false;
    const float r = 1.0f / det;
    o[0] = c00 * r;
    o[3] = c01 * r;
    o[6] = c02 * r;
    o[1] = FS_FMA(m[2], m[7], -(m[1] * m[8])) * r;
    o[4] = FS_FMA(m[0], m[8], -(m[2] * m[6])) * r;
    o[7] = FS_FMA(m[1], m[6], -(m[0] * m[7])) * r;
    o[2] = FS_FMA(m[1], m[5], -(m[2] * m[4])) * r;
    o[5] = FS_FMA(m[2], m[3], -(m[0] * m[5])) * r;
    o[8] = FS_FMA(m[0], m[4], -(m[1] * m[3])) * r;
    return true;
}

// Canonical position of node v (V < 2^28: 32-bit arithmetic; a 64-bit division costs some hundred instructions).
__device__ __forceinline__ void node_pos(const GridP &G, long long v64, float x[3])
{
    const unsigned v = (unsigned)v64, nz = (unsigned)G.nz, ny = (unsigned)G.ny;
    const unsigned t = div_by(v, nz, G.mag_nz);
    const int iz = (int)(v - t * nz);
    const unsigned ixu = div_by(t, ny, G.mag_ny);
    const int iy = (int)(t - ixu * ny), ix = (int)ixu;
    x[0] = FS_FMA((float)ix, G.h[0], G.lo[0]);
    x[1] = FS_FMA((float)iy, G.h[1], G.lo[1]);
    x[2] = FS_FMA((float)iz, G.h[2], G.lo[2]);
}

}  // namespace fs
