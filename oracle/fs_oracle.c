/*
 * fs_oracle.c -- TEST INFRASTRUCTURE, NOT THE PRODUCT.
 *
 * A plain, slow, step-by-step CPU implementation of the Fast-SNARF articulation
 * path: per-voxel blended transforms, multi-start initial guesses, Broyden root
 * finding of d(x) - x' = 0, and the implicit-differentiation backward.  Only the
 * tests, the smoke check and the benchmark's cpu_baseline leg may call it.  It
 * shares no code with the HIP library.
 *
 * The file is compiled twice: -DORC_F32 gives the "strict fp32" build (every
 * multiply-add is an explicit fmaf in a fixed order; this build defines what the
 * convergence masks and trajectories are), the default gives the float64 build
 * (used to judge root validity and gradients).  Compile with -ffp-contract=off.
 *
 * What follows the paper and where:
 *   orc_precompute  -- Sec. 3.1 "Pre-computing LBS", T_v = sum_i w_{v,i} B_i
 *   field_eval      -- Eq. (4)/(5) (LBS, forward map) with T(x) from tri-linear interpolation of {T_v}
 *                      (Sec. 3.1 "Voxel-based Skinning Field")
 *   orc_init_bone   -- Eq. (8) (initial states): x0_i = B_i^{-1} x', J0_i = dd/dx at x0_i
 *   orc_solve       -- Eq. (7) (quasi-Newton step) with Broyden's inverse-Jacobian update, Algorithm 1
 *                      (variant 2), convergence set of Eq. (9), per-iteration
 *                      divergence / convergence filter of Sec. 3.1 "Custom CUDA Kernel"
 *   orc_grad        -- Eq. (11)/(12) (chain rule, implicit differentiation; exact inverse Jacobian) and Sec. 3.2
 *                      "Approximated Gradient", Eq. (15) (Broyden's last J~)
 *   orc_corr_build / orc_init_voxel -- the voxel-based initialisation; the paper
 *                      does not define it, the rule is this project's own.
 *   orc_dedupe      -- Sec. 3.1 "Remove Duplicate Correspondences" (greedy rule of this project)
 *   orc_brute_roots -- exhaustive dense search + Newton polish, a checker only.
 *
 * Parity pins: every function here is pinned by tests/test_oracle_*.py (closed forms,
 * library cross-checks, finite differences, brute force) except:
 *   - orc_grad in Broyden-J mode: the paper gives no error bound between J~ and the
 *     true inverse Jacobian, so its distance to the exact gradient is only reported:
 *     "parity unpinned" against truth (pinned in exact-J mode).
 *   - orc_corr_build / orc_init_voxel: rule not in the paper: "parity unpinned";
 *     only its own invariants (separation, cell membership, brute-force
 *     re-derivation of the greedy choice) are tested.
 *
 * Equation numbers count every numbered display line of the paper from the occupancy-field
 * definition (1)-(2) onward: (3) weight field, (4) LBS, (5) forward map, (6) root equation,
 * (7) quasi-Newton step, (8) initial states, (9) root set, (10) max aggregation, (11) chain rule,
 * (12) implicit differentiation, (13) T_v, (14)-(15) approximated inverse Jacobian.
 *
 * Layouts: W [nx][ny][nz][nb]; node index v = (ix*ny + iy)*nz + iz; B [P][nb][12]
 * row-major 3x4; T [P][V][12]; points SoA [3][N]; per-lane arrays [K][c][N].
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef ORC_F32
typedef float real;
#define FMA(a, b, c) fmaf((a), (b), (c))
#define FLOOR(a) floorf(a)
#define FABS(a) fabsf(a)
#define NAME(n) n##_f32
#else
typedef double real;
#define FMA(a, b, c) fma((a), (b), (c))
#define FLOOR(a) floor(a)
#define FABS(a) fabs(a)
#define NAME(n) n##_f64
#endif

#define DET_EPS ((real)1e-12)

typedef struct {
    int32_t n[3];
    int32_t nb, P;
    int64_t V;
    real lo[3], hi[3], inv_h[3], h[3];
} grid_t;

static grid_t make_grid(const int32_t *dims, const double *box)
{
    grid_t g;
    for (int a = 0; a < 3; ++a) {
        g.n[a] = dims[a];
        g.lo[a] = (real)box[a];
        g.hi[a] = (real)box[3 + a];
        g.inv_h[a] = (real)(dims[a] - 1) / (g.hi[a] - g.lo[a]);
        g.h[a] = (g.hi[a] - g.lo[a]) / (real)(dims[a] - 1);
    }
    g.nb = dims[3];
    g.P = dims[4];
    g.V = (int64_t)dims[0] * dims[1] * dims[2];
    return g;
}

/* ---- Sec. 3.1 "Pre-computing LBS": T_v = sum_i w_{v,i} B_i, bones in index order ---- */
void NAME(orc_precompute)(const int32_t *dims, const real *W, const real *B, real *T)
{
    const int64_t V = (int64_t)dims[0] * dims[1] * dims[2];
    const int nb = dims[3], P = dims[4];
    for (int p = 0; p < P; ++p) {
#pragma omp parallel for schedule(static)
        for (int64_t v = 0; v < V; ++v) {
            for (int e = 0; e < 12; ++e) {
                real acc = W[v * nb] * B[((int64_t)p * nb) * 12 + e];
                for (int b = 1; b < nb; ++b)
                    acc = FMA(W[v * nb + b], B[((int64_t)p * nb + b) * 12 + e], acc);
                T[((int64_t)p * V + v) * 12 + e] = acc;
            }
        }
    }
}

/* ---- cell location for tri-linear interpolation: nodes on the box faces, clamp to edge ---- */
typedef struct {
    int i0[3];
    real f[3];
    int clamped[3];
} loc_t;

static loc_t locate(const grid_t *g, const real *x)
{
    loc_t L;
    for (int a = 0; a < 3; ++a) {
        real m = (real)(g->n[a] - 1);
        real u = (x[a] - g->lo[a]) * g->inv_h[a];
        L.clamped[a] = 0;
        if (!(u >= (real)0)) { u = (real)0; L.clamped[a] = 1; }
        else if (u > m) { u = m; L.clamped[a] = 1; }
        int i = (int)FLOOR(u);
        if (i > g->n[a] - 2) i = g->n[a] - 2;
        L.i0[a] = i;
        L.f[a] = u - (real)i;
    }
    return L;
}

/* corner c = a + 2 b + 4 cz : offsets (a, b, cz) along (x, y, z) */
static void corner_weights(const loc_t *L, real *om)
{
    real wx[2] = { (real)1 - L->f[0], L->f[0] };
    real wy[2] = { (real)1 - L->f[1], L->f[1] };
    real wz[2] = { (real)1 - L->f[2], L->f[2] };
    for (int c = 0; c < 8; ++c)
        om[c] = (wx[c & 1] * wy[(c >> 1) & 1]) * wz[(c >> 2) & 1];
}

static const real *corner_ptr(const grid_t *g, const real *Tp, const loc_t *L, int c)
{
    int64_t ix = L->i0[0] + (c & 1), iy = L->i0[1] + ((c >> 1) & 1), iz = L->i0[2] + ((c >> 2) & 1);
    return Tp + ((ix * g->n[1] + iy) * g->n[2] + iz) * 12;
}

static void apply12(const real *T, const real *x, real *d)
{
    for (int r = 0; r < 3; ++r)
        d[r] = FMA(T[r * 4 + 0], x[0], FMA(T[r * 4 + 1], x[1], FMA(T[r * 4 + 2], x[2], T[r * 4 + 3])));
}

/* Eq. (4)/(5): T(x) by tri-linear interpolation of the pre-computed grid, d = T(x) x.
 * Optionally the spatial Jacobian dd/dx (row-major 3x3): the interpolated rotation part
 * plus the derivative of the interpolation weights acting on each corner's image of x.
 * Along an axis where the lookup was clamped the field is constant, so that part is 0. */
static void field_eval(const grid_t *g, const real *Tp, const real *x, real *d, real *J, real *Tout)
{
    loc_t L = locate(g, x);
    real om[8], T[12];
    corner_weights(&L, om);
    const real *C0 = corner_ptr(g, Tp, &L, 0);
    for (int e = 0; e < 12; ++e) T[e] = om[0] * C0[e];
    for (int c = 1; c < 8; ++c) {
        const real *C = corner_ptr(g, Tp, &L, c);
        for (int e = 0; e < 12; ++e) T[e] = FMA(om[c], C[e], T[e]);
    }
    apply12(T, x, d);
    if (Tout) memcpy(Tout, T, sizeof T);
    if (!J) return;
    real wx[2] = { (real)1 - L.f[0], L.f[0] };
    real wy[2] = { (real)1 - L.f[1], L.f[1] };
    real wz[2] = { (real)1 - L.f[2], L.f[2] };
    for (int r = 0; r < 3; ++r)
        for (int j = 0; j < 3; ++j) J[r * 3 + j] = T[r * 4 + j];
    for (int c = 0; c < 8; ++c) {
        int a = c & 1, b = (c >> 1) & 1, cz = (c >> 2) & 1;
        real dc[3];
        apply12(corner_ptr(g, Tp, &L, c), x, dc);
        real dw[3];
        dw[0] = L.clamped[0] ? (real)0 : (a ? g->inv_h[0] : -g->inv_h[0]) * (wy[b] * wz[cz]);
        dw[1] = L.clamped[1] ? (real)0 : (b ? g->inv_h[1] : -g->inv_h[1]) * (wx[a] * wz[cz]);
        dw[2] = L.clamped[2] ? (real)0 : (cz ? g->inv_h[2] : -g->inv_h[2]) * (wx[a] * wy[b]);
        for (int r = 0; r < 3; ++r)
            for (int j = 0; j < 3; ++j) J[r * 3 + j] = FMA(dw[j], dc[r], J[r * 3 + j]);
    }
}

/* inverse of a row-major 3x3 by adjugate / determinant; returns 0 if (near) singular */
static int inv3(const real *m, real *o)
{
    real c00 = FMA(m[4], m[8], -(m[5] * m[7]));
    real c01 = FMA(m[5], m[6], -(m[3] * m[8]));
    real c02 = FMA(m[3], m[7], -(m[4] * m[6]));
    real det = FMA(m[0], c00, FMA(m[1], c01, m[2] * c02));
    if (!(FABS(det) >= DET_EPS)) return 0;
    real r = (real)1 / det;
    o[0] = c00 * r;
    o[3] = c01 * r;
    o[6] = c02 * r;
    o[1] = FMA(m[2], m[7], -(m[1] * m[8])) * r;
    o[4] = FMA(m[0], m[8], -(m[2] * m[6])) * r;
    o[7] = FMA(m[1], m[6], -(m[0] * m[7])) * r;
    o[2] = FMA(m[1], m[5], -(m[2] * m[4])) * r;
    o[5] = FMA(m[2], m[3], -(m[0] * m[5])) * r;
    o[8] = FMA(m[0], m[4], -(m[1] * m[3])) * r;
    return 1;
}

/* forward map and Jacobian for tests: x [3][n] -> d [3][n], J [9][n] (may be NULL) */
void NAME(orc_forward)(const int32_t *dims, const double *box, const real *T, const real *x,
                       const int32_t *pose, int64_t n, real *d, real *J)
{
    grid_t g = make_grid(dims, box);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n; ++i) {
        real xi[3] = { x[i], x[n + i], x[2 * n + i] }, di[3], Ji[9];
        const real *Tp = T + (int64_t)(pose ? pose[i] : 0) * g.V * 12;
        field_eval(&g, Tp, xi, di, J ? Ji : NULL, NULL);
        for (int r = 0; r < 3; ++r) d[r * n + i] = di[r];
        if (J) for (int e = 0; e < 9; ++e) J[e * n + i] = Ji[e];
    }
}

/* J~0 = (dd/dx at x0)^{-1}; returns validity */
static int init_jinv(const grid_t *g, const real *Tp, const real *x0, real *Jinv)
{
    real d[3], J[9];
    field_eval(g, Tp, x0, d, J, NULL);
    return inv3(J, Jinv);
}

/* ---- Eq. (8): one initial state per bone ---- */
void NAME(orc_init_bone)(const int32_t *dims, const double *box, const real *T, const real *B,
                         const real *xq, const int32_t *pose, int64_t N,
                         real *x0, real *Jinv0, uint8_t *valid0)
{
    grid_t g = make_grid(dims, box);
    const int K = g.nb;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const int p = pose ? pose[i] : 0;
        const real *Tp = T + (int64_t)p * g.V * 12;
        for (int k = 0; k < K; ++k) {
            const real *Bk = B + ((int64_t)p * g.nb + k) * 12;
            real R[9] = { Bk[0], Bk[1], Bk[2], Bk[4], Bk[5], Bk[6], Bk[8], Bk[9], Bk[10] }, Ri[9];
            real xs[3] = { 0, 0, 0 }, Ji[9] = { 0, 0, 0, 0, 0, 0, 0, 0, 0 };
            int ok = inv3(R, Ri);
            if (ok) {
                real y[3] = { xq[i] - Bk[3], xq[N + i] - Bk[7], xq[2 * N + i] - Bk[11] };
                for (int r = 0; r < 3; ++r)
                    xs[r] = FMA(Ri[r * 3 + 0], y[0], FMA(Ri[r * 3 + 1], y[1], Ri[r * 3 + 2] * y[2]));
                ok = init_jinv(&g, Tp, xs, Ji);
                if (!ok) memset(Ji, 0, sizeof Ji);
            }
            for (int r = 0; r < 3; ++r) x0[((int64_t)k * 3 + r) * N + i] = xs[r];
            for (int e = 0; e < 9; ++e) Jinv0[((int64_t)k * 9 + e) * N + i] = Ji[e];
            valid0[(int64_t)k * N + i] = (uint8_t)ok;
        }
    }
}

/* ---- Broyden root finding, one lane per (point, initial state) ----
 * Eq. (7) with the inverse Jacobian replaced by J~, which receives the rank-one
 * "good Broyden" update in inverse (Sherman-Morrison) form after every step:
 *   J~ += (dx - J~ dg) (dx^T J~) / (dx^T J~ dg).
 * A lane stops when |g|^2 < tol^2 (Eq. (9), strict), when !(|g|^2 < div^2)
 * (divergence filter; also catches NaN), or after max_iters steps. */
void NAME(orc_solve)(const int32_t *dims, const double *box, const real *T, const double *prm,
                     const real *xq, const int32_t *pose, int64_t N, int32_t K,
                     const real *x0, const real *Jinv0, const uint8_t *valid0,
                     real *xc, uint8_t *conv, real *Jinv, uint8_t *iters)
{
    grid_t g = make_grid(dims, box);
    const real tol = (real)prm[0], dv = (real)prm[1];
    const real tol2 = tol * tol, div2 = dv * dv;
    const int max_iters = (int)prm[2];
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < N; ++i) {
        const real *Tp = T + (int64_t)(pose ? pose[i] : 0) * g.V * 12;
        const real xp[3] = { xq[i], xq[N + i], xq[2 * N + i] };
        for (int k = 0; k < K; ++k) {
            real x[3], J[9], gv[3], d[3];
            for (int r = 0; r < 3; ++r) x[r] = x0[((int64_t)k * 3 + r) * N + i];
            for (int e = 0; e < 9; ++e) J[e] = Jinv0[((int64_t)k * 9 + e) * N + i];
            int it = 0, cv = 0;
            if (valid0[(int64_t)k * N + i]) {
                field_eval(&g, Tp, x, d, NULL, NULL);
                for (int r = 0; r < 3; ++r) gv[r] = d[r] - xp[r];
                real r2 = FMA(gv[2], gv[2], FMA(gv[1], gv[1], gv[0] * gv[0]));
                if (r2 < tol2) cv = 1;
                else if (r2 < div2) {
                    while (it < max_iters) {
                        real dx[3], xn[3], gn[3], dg[3], v[3], u[3];
                        for (int r = 0; r < 3; ++r)
                            dx[r] = -FMA(J[r * 3 + 2], gv[2], FMA(J[r * 3 + 1], gv[1], J[r * 3] * gv[0]));
                        for (int r = 0; r < 3; ++r) xn[r] = x[r] + dx[r];
                        field_eval(&g, Tp, xn, d, NULL, NULL);
                        for (int r = 0; r < 3; ++r) { gn[r] = d[r] - xp[r]; dg[r] = gn[r] - gv[r]; }
                        for (int c = 0; c < 3; ++c)
                            v[c] = FMA(dx[2], J[6 + c], FMA(dx[1], J[3 + c], dx[0] * J[c]));
                        for (int r = 0; r < 3; ++r)
                            u[r] = dx[r] - FMA(J[r * 3 + 2], dg[2], FMA(J[r * 3 + 1], dg[1], J[r * 3] * dg[0]));
                        real den = FMA(v[2], dg[2], FMA(v[1], dg[1], v[0] * dg[0]));
                        if (den != (real)0 && isfinite(den)) {
                            real rinv = (real)1 / den;
                            for (int r = 0; r < 3; ++r) {
                                real s = u[r] * rinv;
                                for (int c = 0; c < 3; ++c) J[r * 3 + c] = FMA(s, v[c], J[r * 3 + c]);
                            }
                        }
                        for (int r = 0; r < 3; ++r) { x[r] = xn[r]; gv[r] = gn[r]; }
                        ++it;
                        r2 = FMA(gv[2], gv[2], FMA(gv[1], gv[1], gv[0] * gv[0]));
                        if (r2 < tol2) { cv = 1; break; }
                        if (!(r2 < div2)) break;
                    }
                }
            }
            for (int r = 0; r < 3; ++r) xc[((int64_t)k * 3 + r) * N + i] = x[r];
            conv[(int64_t)k * N + i] = (uint8_t)cv;
            if (Jinv) for (int e = 0; e < 9; ++e) Jinv[((int64_t)k * 9 + e) * N + i] = J[e];
            if (iters) iters[(int64_t)k * N + i] = (uint8_t)it;
        }
    }
}

/* ---- Backward by implicit differentiation ----
 * Eq. (12): dx* / dtheta = -(dd/dx*)^{-1} dd/dtheta.  With g_x = dL/dx*, lambda = -M^T g_x
 * (M = Broyden's last J~ for mode 0, Sec. 3.2 "Approximated Gradient"; M = analytic
 * (dd/dx*)^{-1} for mode 1) the gradient w.r.t. a corner transform entry T_c[r][j] is
 * omega_c lambda_r x*_j (j<3) and omega_c lambda_r (j=3).  The voxel-transform gradient G_T is
 * then pulled back through T_v = sum_i w_{v,i} B_i to the raw weights and to the 12 entries of
 * every bone transform.  dL/dx' = +M^T g_x, summed over the point's converged lanes. */
void NAME(orc_grad)(const int32_t *dims, const double *box, const real *T, const real *W,
                    const real *B, int32_t mode, const real *xc, const real *Jinv,
                    const uint8_t *conv, const real *gxc, const int32_t *pose, int64_t N, int32_t K,
                    real *gW, real *gB, real *gxq, real *GT_out)
{
    grid_t g = make_grid(dims, box);
    const int nb = g.nb;
    real *GT = (real *)calloc((size_t)g.P * g.V * 12, sizeof(real));
    if (gxq) memset(gxq, 0, sizeof(real) * 3 * N);
    for (int64_t i = 0; i < N; ++i) {
        const int p = pose ? pose[i] : 0;
        const real *Tp = T + (int64_t)p * g.V * 12;
        real *Gp = GT + (int64_t)p * g.V * 12;
        for (int k = 0; k < K; ++k) {
            if (!conv[(int64_t)k * N + i]) continue;
            real x[3], M[9], gx[3], lam[3];
            for (int r = 0; r < 3; ++r) {
                x[r] = xc[((int64_t)k * 3 + r) * N + i];
                gx[r] = gxc[((int64_t)k * 3 + r) * N + i];
            }
            if (mode == 0) {
                for (int e = 0; e < 9; ++e) M[e] = Jinv[((int64_t)k * 9 + e) * N + i];
            } else {
                real d[3], J[9];
                field_eval(&g, Tp, x, d, J, NULL);
                if (!inv3(J, M)) continue;
            }
            for (int r = 0; r < 3; ++r)
                lam[r] = -FMA(M[6 + r], gx[2], FMA(M[3 + r], gx[1], M[r] * gx[0]));
            if (gxq) for (int r = 0; r < 3; ++r) gxq[r * N + i] -= lam[r];
            loc_t L = locate(&g, x);
            real om[8];
            corner_weights(&L, om);
            for (int c = 0; c < 8; ++c) {
                real *G = Gp + (corner_ptr(&g, Tp, &L, c) - Tp);
                for (int r = 0; r < 3; ++r) {
                    real wl = om[c] * lam[r];
                    G[r * 4 + 0] += wl * x[0];
                    G[r * 4 + 1] += wl * x[1];
                    G[r * 4 + 2] += wl * x[2];
                    G[r * 4 + 3] += wl;
                }
            }
        }
    }
    /* gW[v][b] = sum_p sum_e G_T[p][v][e] B[p][b][e] */
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < g.V; ++v)
        for (int b = 0; b < nb; ++b) {
            real acc = 0;
            for (int p = 0; p < g.P; ++p)
                for (int e = 0; e < 12; ++e)
                    acc = FMA(GT[((int64_t)p * g.V + v) * 12 + e], B[((int64_t)p * nb + b) * 12 + e], acc);
            gW[v * nb + b] = acc;
        }
    /* gB[p][b][e] = sum_v W[v][b] G_T[p][v][e] */
    for (int p = 0; p < g.P; ++p)
        for (int b = 0; b < nb; ++b)
            for (int e = 0; e < 12; ++e) {
                real acc = 0;
                for (int64_t v = 0; v < g.V; ++v)
                    acc = FMA(W[v * nb + b], GT[((int64_t)p * g.V + v) * 12 + e], acc);
                gB[((int64_t)p * nb + b) * 12 + e] = acc;
            }
    if (GT_out) memcpy(GT_out, GT, sizeof(real) * (size_t)g.P * g.V * 12);
    free(GT);
}

/* ---- Voxel-based initialisation (rule of this project; the paper has none) ----
 * Build, per pose: every transform-grid node x_v is a sample; its image y_v = T_v x_v is
 * binned into a (cx, cy, cz) grid over the bounding box of all images.  Per cell the samples
 * are visited by increasing squared distance of y_v to the cell centre (ties: lower v) and
 * accepted when their canonical position is farther than r_sep = 2.5 |h| from every accepted
 * one (2.5, not 2: for equal spacings no lattice vector has squared length 6.25 |h|^2, so the
 * test never sits on a rounding tie); at most ck are kept.  cand[p][cell][j] = node index or -1. */
typedef struct { real key; int64_t v; } keyed_t;

static int keyed_cmp(const void *a, const void *b)
{
    const keyed_t *p = (const keyed_t *)a, *q = (const keyed_t *)b;
    if (p->key < q->key) return -1;
    if (p->key > q->key) return 1;
    return (p->v > q->v) - (p->v < q->v);
}

static void node_pos(const grid_t *g, int64_t v, real *x)
{
    int64_t iz = v % g->n[2], iy = (v / g->n[2]) % g->n[1], ix = v / ((int64_t)g->n[2] * g->n[1]);
    x[0] = FMA((real)ix, g->h[0], g->lo[0]);
    x[1] = FMA((real)iy, g->h[1], g->lo[1]);
    x[2] = FMA((real)iz, g->h[2], g->lo[2]);
}

static int cell_coord(real y, real blo, real cs, int n)
{
    if (!(cs > (real)0)) return 0;
    real t = (y - blo) / cs;
    if (!(t >= (real)0)) t = (real)0;
    if (t > (real)(n - 1)) t = (real)(n - 1);
    return (int)t;
}

void NAME(orc_corr_build)(const int32_t *dims, const double *box, const real *T,
                          const int32_t *cdims, real *bbox, int32_t *cand)
{
    grid_t g = make_grid(dims, box);
    const int cx = cdims[0], cy = cdims[1], cz = cdims[2], ck = cdims[3];
    const int64_t ncell = (int64_t)cx * cy * cz;
    const real rs2 = (real)6.25 * FMA(g.h[2], g.h[2], FMA(g.h[1], g.h[1], g.h[0] * g.h[0]));
    real *Y = (real *)malloc(sizeof(real) * 3 * g.V);
    int64_t *cell_of = (int64_t *)malloc(sizeof(int64_t) * g.V);
    int64_t *count = (int64_t *)malloc(sizeof(int64_t) * (ncell + 1));
    int64_t *order = (int64_t *)malloc(sizeof(int64_t) * g.V);
    keyed_t *buf = (keyed_t *)malloc(sizeof(keyed_t) * g.V);
    for (int p = 0; p < g.P; ++p) {
        const real *Tp = T + (int64_t)p * g.V * 12;
        real *bb = bbox + p * 6;
        for (int64_t v = 0; v < g.V; ++v) {
            real x[3];
            node_pos(&g, v, x);
            apply12(Tp + v * 12, x, Y + 3 * v);
            for (int a = 0; a < 3; ++a) {
                if (v == 0 || Y[3 * v + a] < bb[a]) bb[a] = Y[3 * v + a];
                if (v == 0 || Y[3 * v + a] > bb[3 + a]) bb[3 + a] = Y[3 * v + a];
            }
        }
        real cs[3] = { (bb[3] - bb[0]) / (real)cx, (bb[4] - bb[1]) / (real)cy, (bb[5] - bb[2]) / (real)cz };
        memset(count, 0, sizeof(int64_t) * (ncell + 1));
        for (int64_t v = 0; v < g.V; ++v) {
            int64_t c = ((int64_t)cell_coord(Y[3 * v], bb[0], cs[0], cx) * cy +
                         cell_coord(Y[3 * v + 1], bb[1], cs[1], cy)) * cz +
                        cell_coord(Y[3 * v + 2], bb[2], cs[2], cz);
            cell_of[v] = c;
            count[c + 1]++;
        }
        for (int64_t c = 0; c < ncell; ++c) count[c + 1] += count[c];
        int64_t *fill = (int64_t *)calloc(ncell, sizeof(int64_t));
        for (int64_t v = 0; v < g.V; ++v) order[count[cell_of[v]] + fill[cell_of[v]]++] = v;
        free(fill);
        for (int64_t c = 0; c < ncell; ++c) {
            int32_t *out = cand + ((int64_t)p * ncell + c) * ck;
            for (int j = 0; j < ck; ++j) out[j] = -1;
            int64_t n = count[c + 1] - count[c];
            if (n == 0) continue;
            int ciz = (int)(c % cz), ciy = (int)((c / cz) % cy), cix = (int)(c / ((int64_t)cz * cy));
            real ctr[3] = { FMA((real)cix + (real)0.5, cs[0], bb[0]),
                            FMA((real)ciy + (real)0.5, cs[1], bb[1]),
                            FMA((real)ciz + (real)0.5, cs[2], bb[2]) };
            for (int64_t s = 0; s < n; ++s) {
                int64_t v = order[count[c] + s];
                real dx = Y[3 * v] - ctr[0], dy = Y[3 * v + 1] - ctr[1], dz = Y[3 * v + 2] - ctr[2];
                buf[s].key = FMA(dz, dz, FMA(dy, dy, dx * dx));
                buf[s].v = v;
            }
            qsort(buf, (size_t)n, sizeof(keyed_t), keyed_cmp);
            int na = 0;
            real acc[8][3];
            for (int64_t s = 0; s < n && na < ck && na < 8; ++s) {
                real x[3];
                node_pos(&g, buf[s].v, x);
                int ok = 1;
                for (int j = 0; j < na; ++j) {
                    real ex = x[0] - acc[j][0], ey = x[1] - acc[j][1], ez = x[2] - acc[j][2];
                    real d2 = FMA(ez, ez, FMA(ey, ey, ex * ex));
                    if (!(d2 > rs2)) { ok = 0; break; }
                }
                if (ok) {
                    memcpy(acc[na], x, sizeof x);
                    out[na++] = (int32_t)buf[s].v;
                }
            }
        }
    }
    free(Y); free(cell_of); free(count); free(order); free(buf);
}

/* Query: x' is clamped into the pose's bounding box, its cell's candidates become the
 * initial states x0 = x_v, with J~0 as in Eq. (8). */
void NAME(orc_init_voxel)(const int32_t *dims, const double *box, const real *T,
                          const int32_t *cdims, const real *bbox, const int32_t *cand,
                          const real *xq, const int32_t *pose, int64_t N,
                          real *x0, real *Jinv0, uint8_t *valid0)
{
    grid_t g = make_grid(dims, box);
    const int cx = cdims[0], cy = cdims[1], cz = cdims[2], ck = cdims[3];
    const int64_t ncell = (int64_t)cx * cy * cz;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        const int p = pose ? pose[i] : 0;
        const real *Tp = T + (int64_t)p * g.V * 12;
        const real *bb = bbox + p * 6;
        real cs[3] = { (bb[3] - bb[0]) / (real)cx, (bb[4] - bb[1]) / (real)cy, (bb[5] - bb[2]) / (real)cz };
        int64_t c = ((int64_t)cell_coord(xq[i], bb[0], cs[0], cx) * cy +
                     cell_coord(xq[N + i], bb[1], cs[1], cy)) * cz +
                    cell_coord(xq[2 * N + i], bb[2], cs[2], cz);
        for (int k = 0; k < ck; ++k) {
            int32_t v = cand[((int64_t)p * ncell + c) * ck + k];
            real xs[3] = { 0, 0, 0 }, Ji[9] = { 0, 0, 0, 0, 0, 0, 0, 0, 0 };
            int ok = 0;
            if (v >= 0) {
                node_pos(&g, v, xs);
                ok = init_jinv(&g, Tp, xs, Ji);
                if (!ok) memset(Ji, 0, sizeof Ji);
            }
            for (int r = 0; r < 3; ++r) x0[((int64_t)k * 3 + r) * N + i] = xs[r];
            for (int e = 0; e < 9; ++e) Jinv0[((int64_t)k * 9 + e) * N + i] = Ji[e];
            valid0[(int64_t)k * N + i] = (uint8_t)ok;
        }
    }
}

/* ---- Duplicate removal (Sec. 3.1 "Remove Duplicate Correspondences") ----
 * Different initial states often reach the same root.  The paper detects duplicates "by their
 * relative distances in canonical space" without giving the rule; here: per point the lanes are
 * visited in increasing k, and a converged lane is kept iff no lane kept before it lies closer than
 * min_dist (Euclidean, strict <).  keep [K][N] 0/1, count [N]. */
void NAME(orc_dedupe)(const real *xc, const uint8_t *conv, int64_t N, int32_t K, double min_dist,
                      uint8_t *keep, int32_t *count)
{
    const real md = (real)min_dist, md2 = md * md;
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        int c = 0;
        for (int k = 0; k < K; ++k) {
            int kp = 0;
            if (conv[(int64_t)k * N + i]) {
                kp = 1;
                for (int j = 0; j < k && kp; ++j) {
                    if (!keep[(int64_t)j * N + i]) continue;
                    real e0 = xc[((int64_t)k * 3 + 0) * N + i] - xc[((int64_t)j * 3 + 0) * N + i];
                    real e1 = xc[((int64_t)k * 3 + 1) * N + i] - xc[((int64_t)j * 3 + 1) * N + i];
                    real e2 = xc[((int64_t)k * 3 + 2) * N + i] - xc[((int64_t)j * 3 + 2) * N + i];
                    real d2 = FMA(e2, e2, FMA(e1, e1, e0 * e0));
                    if (d2 < md2) kp = 0;
                }
            }
            keep[(int64_t)k * N + i] = (uint8_t)kp;
            c += kp;
        }
        count[i] = c;
    }
}

#ifndef ORC_F32
/* ---- Exhaustive root search (checker only, float64) ----
 * For each query point: from a dense lattice of s^3 starts inside every grid cell run Newton
 * with the analytic Jacobian, keep iterates that converge to |d(x)-x'| < 1e-12 inside the
 * (closed) box, and merge those closer than merge_tol.  roots [n][max_roots][3], count [n]. */
void orc_brute_roots_f64(const int32_t *dims, const double *box, const double *T,
                         const double *xq, int64_t n, int32_t s, double merge_tol,
                         int32_t max_roots, double *roots, int32_t *count)
{
    grid_t g = make_grid(dims, box);
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n; ++i) {
        const double xp[3] = { xq[i], xq[n + i], xq[2 * n + i] };
        double *R = roots + i * max_roots * 3;
        int nr = 0;
        for (int cx = 0; cx < g.n[0] - 1; ++cx)
        for (int cy = 0; cy < g.n[1] - 1; ++cy)
        for (int cz = 0; cz < g.n[2] - 1; ++cz)
        for (int a = 0; a < s; ++a)
        for (int b = 0; b < s; ++b)
        for (int c = 0; c < s; ++c) {
            double x[3] = { g.lo[0] + (cx + (a + 0.5) / s) * g.h[0],
                            g.lo[1] + (cy + (b + 0.5) / s) * g.h[1],
                            g.lo[2] + (cz + (c + 0.5) / s) * g.h[2] };
            int ok = 0;
            for (int it = 0; it < 40; ++it) {
                double d[3], J[9], Ji[9];
                field_eval(&g, T, x, d, J, NULL);
                double gv[3] = { d[0] - xp[0], d[1] - xp[1], d[2] - xp[2] };
                double r2 = gv[0] * gv[0] + gv[1] * gv[1] + gv[2] * gv[2];
                if (r2 < 1e-24) { ok = 1; break; }
                if (!(r2 < 1e6) || !inv3(J, Ji)) break;
                for (int r = 0; r < 3; ++r)
                    x[r] -= Ji[r * 3] * gv[0] + Ji[r * 3 + 1] * gv[1] + Ji[r * 3 + 2] * gv[2];
            }
            if (!ok) continue;
            int inside = 1;
            for (int r = 0; r < 3; ++r)
                if (x[r] < g.lo[r] - 1e-9 || x[r] > g.hi[r] + 1e-9) inside = 0;
            if (!inside) continue;
            int dup = 0;
            for (int j = 0; j < nr; ++j) {
                double e0 = x[0] - R[3 * j], e1 = x[1] - R[3 * j + 1], e2 = x[2] - R[3 * j + 2];
                if (e0 * e0 + e1 * e1 + e2 * e2 < merge_tol * merge_tol) { dup = 1; break; }
            }
            if (!dup && nr < max_roots) { memcpy(R + 3 * nr, x, sizeof x); ++nr; }
        }
        count[i] = nr;
    }
}
#endif
