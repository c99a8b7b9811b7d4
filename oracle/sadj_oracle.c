/*
 * sadj_oracle.c -- plain, slow, single-threaded CPU oracle for the adjoint of a
 * stencil loop.  TEST INFRASTRUCTURE ONLY: it may be built and called from tests/,
 * from the smoke check and from the benchmark's cpu_baseline leg, never from the
 * product path.  It shares no code, header, table or helper with the HIP library.
 *
 * What it computes (paper Section 3.2, first two listings, and Section 3.3.1):
 * the conventional reverse-mode adjoint of a gather stencil loop
 *     for i in I:  r[i] = f(u[i+o_1], ..., u[i+o_M], passive data)
 * is the scatter loop
 *     for i in I:  for each read offset o:  u_bar[i+o] += (df_i/du_{i+o}) * r_bar[i]
 * i.e. u_bar_out = u_bar_in + J^T r_bar with J the Jacobian of the primal loop.
 * The oracle is that scatter written out.  It contains no gather form, no index
 * shifting, no core/remainder split and no boundary rule: what happens at the
 * boundary emerges from the primal iteration space I alone.
 *
 * Stencils:
 *  - linear variable-coefficient wave step in 1, 2 or 3 dimensions with a star
 *    Laplacian of radius R (paper Section 4.1 for R=1 in 3-D; the script in its
 *    first figure defines r = 2u - u_prev + c*D*(u_xx+u_yy+u_zz); D is folded
 *    into c here):        r[i] = 2 u[i] - u_prev[i] + c[i] * sum_o w_o u[i+o]
 *  - 1-D upwinded Burgers step (paper Section 4.2, its generating script):
 *    r[i] = u[i] - C*(max(u[i],0)*(u[i]-u[i-1]) + min(u[i],0)*(u[i+1]-u[i]))
 *                + D*(u[i-1] - 2u[i] + u[i+1])
 *  - the 1-D worked example of paper Section 3.2 with arbitrary, possibly
 *    asymmetric, three-point weights:  r[i] = c[i]*(wm*u[i-1] + w0*u[i] + wp*u[i+1])
 *
 * Conventions: arrays are dense, x fastest: index = x + nx*(y + ny*z).  The primal
 * iteration space is I = prod_d [R, n_d-1-R] over the first `ndim` axes (paper:
 * bounds [1,n-2] for R=1); unused axes must have extent 1.  Loops run in ascending
 * lexicographic order (z outer, x inner); per iteration the reads are visited
 * centre first, then offsets -R..-1,+1..+R along x, then y, then z.  Everything is
 * fp64.  `scale`, when non-NULL, receives sum |contribution| per output index: the
 * magnitude against which a differently ordered summation may be compared.
 *
 * Pins (tests/test_oracle_*.py): polynomial exactness of the weights, a library
 * correlation for the primal, dot-product test against the tangent loops, central
 * finite differences, an assembled dense Jacobian transposed by a library mat-vec,
 * the paper's printed 1-D remainder statements and merged core loop, the paper's
 * printed Burgers and 3-D wave gather core loops, the symmetric constant-c case,
 * the conservation sum, zero rows of J^T, NaN poisoning, and brute force over all
 * sizes 2R+1..4R+3.
 */
#include <math.h>
#include <stddef.h>

#define ORACLE_OK 0
#define ORACLE_BAD_ARG 1

/* Standard central finite-difference weights of the second derivative on a unit
 * grid, w[0] centre, w[k] at distance k (orders 2, 4, 6, 8). */
static int star_weights(int R, double w[5])
{
    switch (R) {
    case 1: w[0] = -2.0;          w[1] = 1.0; return 0;
    case 2: w[0] = -5.0 / 2.0;    w[1] = 4.0 / 3.0; w[2] = -1.0 / 12.0; return 0;
    case 3: w[0] = -49.0 / 18.0;  w[1] = 3.0 / 2.0; w[2] = -3.0 / 20.0; w[3] = 1.0 / 90.0; return 0;
    case 4: w[0] = -205.0 / 72.0; w[1] = 8.0 / 5.0; w[2] = -1.0 / 5.0;  w[3] = 8.0 / 315.0;
            w[4] = -1.0 / 560.0; return 0;
    default: return 1;
    }
}

int oracle_star_weights(int R, double *w) { return star_weights(R, w) ? ORACLE_BAD_ARG : ORACLE_OK; }

typedef struct { long n[3]; long stride[3]; long lo[3], hi[3]; int ndim; int R; double w[5]; } grid_t;

static int grid_init(grid_t *g, int ndim, int R, long nx, long ny, long nz)
{
    if (ndim < 1 || ndim > 3) return 1;
    if (star_weights(R, g->w)) return 1;
    g->ndim = ndim; g->R = R;
    g->n[0] = nx; g->n[1] = ny; g->n[2] = nz;
    g->stride[0] = 1; g->stride[1] = nx; g->stride[2] = nx * ny;
    for (int d = 0; d < 3; ++d) {
        if (g->n[d] < 1) return 1;
        if (d < ndim) {
            if (g->n[d] < 2 * R + 1) return 1;       /* empty primal interior */
            g->lo[d] = R; g->hi[d] = g->n[d] - 1 - R;
        } else {
            if (g->n[d] != 1) return 1;
            g->lo[d] = 0; g->hi[d] = 0;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------- wave: primal */
/* r[i] = 2u[i] - u_prev[i] + c[i]*Lap_w(u)[i] for i in I; r outside I untouched.
 * (Section 4.1; the listing there prints "+=", the script says lhs = rhs: assign.) */
int oracle_wave_primal(int ndim, int R, long nx, long ny, long nz,
                       const double *u, const double *u_prev, const double *c, double *r)
{
    grid_t g;
    if (!u || !u_prev || !c || !r || grid_init(&g, ndim, R, nx, ny, nz)) return ORACLE_BAD_ARG;
    for (long z = g.lo[2]; z <= g.hi[2]; ++z)
    for (long y = g.lo[1]; y <= g.hi[1]; ++y)
    for (long x = g.lo[0]; x <= g.hi[0]; ++x) {
        long i = x + nx * (y + ny * z);
        double lap = (double)ndim * g.w[0] * u[i];
        for (int d = 0; d < ndim; ++d) {
            for (int k = -R; k <= R; ++k) {
                if (k == 0) continue;
                lap += g.w[k < 0 ? -k : k] * u[i + k * g.stride[d]];
            }
        }
        r[i] = 2.0 * u[i] - u_prev[i] + c[i] * lap;
    }
    return ORACLE_OK;
}

/* Forward-mode (tangent) loop: r_dot = J_u u_dot + J_uprev u_prev_dot.  The wave
 * stencil is linear in (u, u_prev), so the tangent has the primal's form. */
int oracle_wave_tangent(int ndim, int R, long nx, long ny, long nz, const double *c,
                        const double *u_dot, const double *u_prev_dot, double *r_dot)
{
    grid_t g;
    if (!u_dot || !u_prev_dot || !c || !r_dot || grid_init(&g, ndim, R, nx, ny, nz)) return ORACLE_BAD_ARG;
    for (long z = g.lo[2]; z <= g.hi[2]; ++z)
    for (long y = g.lo[1]; y <= g.hi[1]; ++y)
    for (long x = g.lo[0]; x <= g.hi[0]; ++x) {
        long i = x + nx * (y + ny * z);
        double d_centre = 2.0 + c[i] * (double)ndim * g.w[0];
        double acc = d_centre * u_dot[i];
        for (int d = 0; d < ndim; ++d)
            for (int k = -R; k <= R; ++k) {
                if (k == 0) continue;
                acc += (c[i] * g.w[k < 0 ? -k : k]) * u_dot[i + k * g.stride[d]];
            }
        r_dot[i] = acc - u_prev_dot[i];
    }
    return ORACLE_OK;
}

/* --------------------------------------------------------------- wave: adjoint */
/* Scatter adjoint (Section 3.2 second listing; Section 4.1 third listing without
 * the atomics):  for i in I:
 *     u_bar[i]      += (2 + c[i]*ndim*w_0) * r_bar[i]
 *     u_bar[i+o]    += (c[i]*w_o) * r_bar[i]            for every off-centre read o
 *     u_prev_bar[i] -= r_bar[i]                          (if u_prev_bar != NULL)
 * c is passive: no c_bar.  r_bar is read only. */
int oracle_wave_adjoint(int ndim, int R, long nx, long ny, long nz,
                        const double *c, const double *r_bar,
                        double *u_bar, double *u_prev_bar, double *scale)
{
    grid_t g;
    if (!c || !r_bar || !u_bar || grid_init(&g, ndim, R, nx, ny, nz)) return ORACLE_BAD_ARG;
    for (long z = g.lo[2]; z <= g.hi[2]; ++z)
    for (long y = g.lo[1]; y <= g.hi[1]; ++y)
    for (long x = g.lo[0]; x <= g.hi[0]; ++x) {
        long i = x + nx * (y + ny * z);
        double rb = r_bar[i];
        double t = (2.0 + c[i] * (double)ndim * g.w[0]) * rb;
        u_bar[i] += t;
        if (scale) scale[i] += fabs(t);
        for (int d = 0; d < ndim; ++d)
            for (int k = -R; k <= R; ++k) {
                if (k == 0) continue;
                long j = i + k * g.stride[d];
                t = (c[i] * g.w[k < 0 ? -k : k]) * rb;
                u_bar[j] += t;
                if (scale) scale[j] += fabs(t);
            }
        if (u_prev_bar) u_prev_bar[i] -= rb;
    }
    return ORACLE_OK;
}

/* Reverse sweep of a time loop of wave steps u^{k+1} = step(u^k, u^{k-1}), where a step
 * assigns the new state on I only (cells outside I are inputs of their own).  Reverse
 * mode visits the steps last to first; for the step that produced u^{k+1}:
 *     lam^k += (d step/d u^k)^T lam^{k+1},   lam^{k-1} += (d step/d u^{k-1})^T lam^{k+1},
 * which is the scatter adjoint above with r_bar = lam^{k+1}.  lam[0], lam[1], lam[2] are
 * lam^{K+1}, lam^K, lam^{K-1} on entry; the adjoint of every older state starts from zero.
 * Three buffers rotate: step s reads lam[s%3], updates lam[(s+1)%3] and lam[(s+2)%3];
 * from s = 1 on the latter is the consumed buffer of the previous step and is zeroed
 * first (it now stands for an older state).  (Paper Sections 3.1 and 4: chain rule over
 * a solver that performs many such steps.) */
int oracle_wave_adjoint_steps(int ndim, int R, long nx, long ny, long nz, long nsteps,
                              const double *c, double *lam0, double *lam1, double *lam2)
{
    double *lam[3] = {lam0, lam1, lam2};
    if (!c || !lam0 || !lam1 || !lam2 || nsteps < 0) return ORACLE_BAD_ARG;
    const long n = nx * ny * nz;
    for (long s = 0; s < nsteps; ++s) {
        double *a = lam[s % 3], *b = lam[(s + 1) % 3], *p = lam[(s + 2) % 3];
        if (s > 0)
            for (long i = 0; i < n; ++i) p[i] = 0.0;
        int rc = oracle_wave_adjoint(ndim, R, nx, ny, nz, c, a, b, p, NULL);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* ------------------------------------------------------------------ Burgers 1-D */
static double pos(double a) { return a > 0.0 ? a : 0.0; }   /* max(a,0) */
static double neg(double a) { return a < 0.0 ? a : 0.0; }   /* min(a,0) */

/* r[i] for i in [1, n-2] (Section 4.2, the upwind formula and the script). */
int oracle_burgers_primal(long n, double C, double D, const double *u, double *r)
{
    if (!u || !r || n < 3) return ORACLE_BAD_ARG;
    for (long i = 1; i <= n - 2; ++i) {
        double conv = pos(u[i]) * (u[i] - u[i - 1]) + neg(u[i]) * (u[i + 1] - u[i]);
        r[i] = u[i] - C * conv + D * (u[i - 1] - 2.0 * u[i] + u[i + 1]);
    }
    return ORACLE_OK;
}

/* Partial derivatives of one Burgers iteration with respect to its three reads.
 * d max(a,0)/da and d min(a,0)/da are both taken as 1 at a == 0, which is what
 * the paper's printed adjoint does ((u>=0)?1:0 and (-u>=0)?1:0). */
static void burgers_partials(double C, double D, double um, double u0, double up,
                             double *dm, double *d0, double *dp)
{
    double dpos = (u0 >= 0.0) ? 1.0 : 0.0;
    double dneg = (-u0 >= 0.0) ? 1.0 : 0.0;
    *dm = C * pos(u0) + D;
    *dp = -C * neg(u0) + D;
    *d0 = 1.0 - C * (dpos * (u0 - um) + pos(u0) + dneg * (up - u0) - neg(u0)) - 2.0 * D;
}

int oracle_burgers_tangent(long n, double C, double D, const double *u,
                           const double *u_dot, double *r_dot)
{
    if (!u || !u_dot || !r_dot || n < 3) return ORACLE_BAD_ARG;
    for (long i = 1; i <= n - 2; ++i) {
        double dm, d0, dp;
        burgers_partials(C, D, u[i - 1], u[i], u[i + 1], &dm, &d0, &dp);
        r_dot[i] = dm * u_dot[i - 1] + d0 * u_dot[i] + dp * u_dot[i + 1];
    }
    return ORACLE_OK;
}

/* Scatter adjoint; the stencil is nonlinear so the primal u is read (Section 3.1). */
int oracle_burgers_adjoint(long n, double C, double D, const double *u,
                           const double *r_bar, double *u_bar, double *scale)
{
    if (!u || !r_bar || !u_bar || n < 3) return ORACLE_BAD_ARG;
    for (long i = 1; i <= n - 2; ++i) {
        double dm, d0, dp;
        burgers_partials(C, D, u[i - 1], u[i], u[i + 1], &dm, &d0, &dp);
        double rb = r_bar[i];
        u_bar[i]     += d0 * rb;
        u_bar[i - 1] += dm * rb;
        u_bar[i + 1] += dp * rb;
        if (scale) {
            scale[i]     += fabs(d0 * rb);
            scale[i - 1] += fabs(dm * rb);
            scale[i + 1] += fabs(dp * rb);
        }
    }
    return ORACLE_OK;
}

/* Time loop of Burgers steps u^{t+1} = step(u^t) on I (elements 0 and n-1 of every state
 * are inputs of their own).  states: rows u^0 .. u^{nsteps}, row length n. */
int oracle_burgers_primal_steps(long n, long nsteps, double C, double D, double *states)
{
    if (!states || nsteps < 0) return ORACLE_BAD_ARG;
    for (long t = 0; t < nsteps; ++t) {
        int rc = oracle_burgers_primal(n, C, D, states + t * n, states + (t + 1) * n);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* Reverse sweep over the steps last-1, ..., last-nsteps (chain rule, Section 3.1; the
 * nonlinear step needs the stored primal state u^t, Section 4.2).  lam[0] is the adjoint
 * of u^{last}, lam[1] holds what the objective adds directly to the adjoint of u^{last-1};
 * adjoints of older states start from zero.  Two buffers alternate: reverse step s reads
 * lam[s%2] as r_bar and accumulates into lam[(s+1)%2], which from s = 1 on is zeroed first. */
int oracle_burgers_adjoint_steps(long n, long last, long nsteps, double C, double D,
                                 const double *states, double *lam0, double *lam1)
{
    double *lam[2] = {lam0, lam1};
    if (!states || !lam0 || !lam1 || nsteps < 0 || nsteps > last) return ORACLE_BAD_ARG;
    for (long s = 0; s < nsteps; ++s) {
        long t = last - 1 - s;
        double *a = lam[s % 2], *b = lam[(s + 1) % 2];
        if (s > 0)
            for (long i = 0; i < n; ++i) b[i] = 0.0;
        int rc = oracle_burgers_adjoint(n, C, D, states + t * n, a, b, NULL);
        if (rc != ORACLE_OK) return rc;
    }
    return ORACLE_OK;
}

/* ------------------------- dense 3^d box stencil with arbitrary (asymmetric) weights */
/* Primal  r[i] = c[i] * sum_{o in {-1,0,1}^d} w[o] * u[i+o]   for i in I = prod [1, n_d-2]
 * (the dense stencils whose adjoint loop-nest counts Section 3.3.4 quotes: 3 points in
 * 1-D -- the worked example of Section 3.2 --, 3x3 in 2-D, 3x3x3 in 3-D).  w is indexed
 * (ox+1) + 3*(oy+1) + 9*(oz+1); unused axes have extent 1 and only offset 0.
 * Scatter adjoint:  u_bar[i+o] += w[o] * c[i] * r_bar[i]. */
static int box_check(int ndim, long nx, long ny, long nz)
{
    const long n[3] = {nx, ny, nz};
    if (ndim < 1 || ndim > 3) return 1;
    for (int d = 0; d < 3; ++d) {
        if (d < ndim ? n[d] < 3 : n[d] != 1) return 1;
    }
    return 0;
}

int oracle_box_primal(int ndim, long nx, long ny, long nz, const double *w,
                      const double *u, const double *c, double *r)
{
    if (!w || !u || !c || !r || box_check(ndim, nx, ny, nz)) return ORACLE_BAD_ARG;
    const int ry = ndim >= 2, rz = ndim >= 3;
    for (long z = rz; z <= nz - 1 - rz; ++z)
    for (long y = ry; y <= ny - 1 - ry; ++y)
    for (long x = 1; x <= nx - 2; ++x) {
        double s = 0.0;
        for (int oz = -rz; oz <= rz; ++oz)
        for (int oy = -ry; oy <= ry; ++oy)
        for (int ox = -1; ox <= 1; ++ox)
            s += w[(ox + 1) + 3 * (oy + 1) + 9 * (oz + 1)] * u[(x + ox) + nx * ((y + oy) + ny * (z + oz))];
        const long i = x + nx * (y + ny * z);
        r[i] = c[i] * s;
    }
    return ORACLE_OK;
}

int oracle_box_adjoint(int ndim, long nx, long ny, long nz, const double *w,
                       const double *c, const double *r_bar, double *u_bar, double *scale)
{
    if (!w || !c || !r_bar || !u_bar || box_check(ndim, nx, ny, nz)) return ORACLE_BAD_ARG;
    const int ry = ndim >= 2, rz = ndim >= 3;
    for (long z = rz; z <= nz - 1 - rz; ++z)
    for (long y = ry; y <= ny - 1 - ry; ++y)
    for (long x = 1; x <= nx - 2; ++x) {
        const long i = x + nx * (y + ny * z);
        for (int oz = -rz; oz <= rz; ++oz)
        for (int oy = -ry; oy <= ry; ++oy)
        for (int ox = -1; ox <= 1; ++ox) {
            const double t = w[(ox + 1) + 3 * (oy + 1) + 9 * (oz + 1)] * c[i] * r_bar[i];
            const long j = (x + ox) + nx * ((y + oy) + ny * (z + oz));
            u_bar[j] += t;
            if (scale) scale[j] += fabs(t);
        }
    }
    return ORACLE_OK;
}

/* ---------------------------- 3-D star stencil of radius R with arbitrary weights */
/* Primal r[i] = c[i]*(w_0 u[i] + sum_{d} sum_{o=-R..R, o!=0} w_{d,o} u[i + o e_d]) for i in I
 * (the general linear star; Sections 3.2-3.3 treat exactly this: one derivative expression
 * per read offset).  w: 1 + 6R values: centre, then per axis x, y, z the offsets
 * -R..-1, +1..+R.  Scatter adjoint: u_bar[i + o e_d] += w_{d,o} c[i] r_bar[i]. */
static double star_w_at(const double *w, int R, int d, int o)
{
    return w[1 + d * 2 * R + (o < 0 ? o + R : o + R - 1)];
}

int oracle_star3d_primal(int R, long nx, long ny, long nz, const double *w,
                         const double *u, const double *c, double *r)
{
    grid_t g;
    if (!w || !u || !c || !r || grid_init(&g, 3, R, nx, ny, nz)) return ORACLE_BAD_ARG;
    for (long z = g.lo[2]; z <= g.hi[2]; ++z)
    for (long y = g.lo[1]; y <= g.hi[1]; ++y)
    for (long x = g.lo[0]; x <= g.hi[0]; ++x) {
        long i = x + nx * (y + ny * z);
        double s = w[0] * u[i];
        for (int d = 0; d < 3; ++d)
            for (int o = -R; o <= R; ++o)
                if (o != 0) s += star_w_at(w, R, d, o) * u[i + o * g.stride[d]];
        r[i] = c[i] * s;
    }
    return ORACLE_OK;
}

int oracle_star3d_adjoint(int R, long nx, long ny, long nz, const double *w,
                          const double *c, const double *r_bar, double *u_bar, double *scale)
{
    grid_t g;
    if (!w || !c || !r_bar || !u_bar || grid_init(&g, 3, R, nx, ny, nz)) return ORACLE_BAD_ARG;
    for (long z = g.lo[2]; z <= g.hi[2]; ++z)
    for (long y = g.lo[1]; y <= g.hi[1]; ++y)
    for (long x = g.lo[0]; x <= g.hi[0]; ++x) {
        long i = x + nx * (y + ny * z);
        double rb = r_bar[i];
        double t = (c[i] * w[0]) * rb;
        u_bar[i] += t;
        if (scale) scale[i] += fabs(t);
        for (int d = 0; d < 3; ++d)
            for (int o = -R; o <= R; ++o) {
                if (o == 0) continue;
                long j = i + o * g.stride[d];
                t = (c[i] * star_w_at(w, R, d, o)) * rb;
                u_bar[j] += t;
                if (scale) scale[j] += fabs(t);
            }
    }
    return ORACLE_OK;
}

/* --------------------------------------- 1-D three-point example, general weights */
/* Primal r[i] = c[i]*(wm*u[i-1] + w0*u[i] + wp*u[i+1]) for i in [lo,hi], arrays of
 * length len (Section 3.2: weights (2,-3,4), i in [1,n-1], arrays of length n+1). */
int oracle_lin3_primal(long len, long lo, long hi, double wm, double w0, double wp,
                       const double *c, const double *u, double *r)
{
    if (!c || !u || !r || lo < 1 || hi > len - 2 || lo > hi) return ORACLE_BAD_ARG;
    for (long i = lo; i <= hi; ++i)
        r[i] = c[i] * (wm * u[i - 1] + w0 * u[i] + wp * u[i + 1]);
    return ORACLE_OK;
}

int oracle_lin3_adjoint(long len, long lo, long hi, double wm, double w0, double wp,
                        const double *c, const double *r_bar, double *u_bar)
{
    if (!c || !r_bar || !u_bar || lo < 1 || hi > len - 2 || lo > hi) return ORACLE_BAD_ARG;
    for (long i = lo; i <= hi; ++i) {
        u_bar[i - 1] += wm * c[i] * r_bar[i];
        u_bar[i]     += w0 * c[i] * r_bar[i];
        u_bar[i + 1] += wp * c[i] * r_bar[i];
    }
    return ORACLE_OK;
}

/* ------------------ 1-D three-point stencil with a caller-supplied loop body (callbacks) */
/* Section 3.3.1: the loop body may be an uninterpreted function f of the three reads
 * (and of a passive value p[i]); its adjoint then refers to the partial derivatives of f
 * as functions too.  Primal r[i] = f(u[i-1], u[i], u[i+1], p[i]) for i in [1, n-2];
 * conventional scatter adjoint, iteration by iteration:
 *     u_bar[i-1] += df/d(um) * r_bar[i];  u_bar[i] += df/d(u0) * r_bar[i];  u_bar[i+1] += df/d(up) * r_bar[i]
 * with the partials evaluated at (u[i-1], u[i], u[i+1], p[i]).  p may be NULL (then 0 is passed). */
typedef double (*oracle_body_fn)(double um, double u0, double up, double p);
typedef void (*oracle_body_partials_fn)(double um, double u0, double up, double p,
                                        double *dm, double *d0, double *dp);

int oracle_stencil1d_primal(long n, oracle_body_fn f, const double *u, const double *p, double *r)
{
    if (!f || !u || !r || n < 3) return ORACLE_BAD_ARG;
    for (long i = 1; i <= n - 2; ++i)
        r[i] = f(u[i - 1], u[i], u[i + 1], p ? p[i] : 0.0);
    return ORACLE_OK;
}

int oracle_stencil1d_adjoint(long n, oracle_body_partials_fn df, const double *u, const double *p,
                             const double *r_bar, double *u_bar, double *scale)
{
    if (!df || !u || !r_bar || !u_bar || n < 3) return ORACLE_BAD_ARG;
    for (long i = 1; i <= n - 2; ++i) {
        double dm, d0, dp;
        df(u[i - 1], u[i], u[i + 1], p ? p[i] : 0.0, &dm, &d0, &dp);
        double rb = r_bar[i];
        u_bar[i - 1] += dm * rb;
        u_bar[i]     += d0 * rb;
        u_bar[i + 1] += dp * rb;
        if (scale) {
            scale[i - 1] += fabs(dm * rb);
            scale[i]     += fabs(d0 * rb);
            scale[i + 1] += fabs(dp * rb);
        }
    }
    return ORACLE_OK;
}

/* ---- star-shaped loop body supplied by the caller, 1 to 3 dimensions (paper Section 3.3.1:
 * the loop body as an uninterpreted function of its reads, its partial derivatives as
 * uninterpreted functions too; the paper's example there is two-dimensional).
 *   primal   r[i] = f(v, p[i])   for i in I,   v[0] = u[i], and for the axes x, y, z in turn
 *            v[1 + a*2R + m], m = 0..2R-1, = u at the offsets -R..-1, +1..+R along axis a
 *   adjoint  for i in I (ascending): for every read k:  u_bar[i + o_k] += d_k * r_bar[i],
 *            (d_0 .. d_{2R*ndim}) = the partials of f with respect to v at iteration i
 * `parity unpinned` does not apply: pinned against the wave, free-weight star and three-point
 * callback loops of this file and against finite differences (tests/test_oracle_starfn.py). */
typedef double (*oracle_star_body_fn)(const double *v, double p);
typedef void (*oracle_star_partials_fn)(const double *v, double p, double *d);

static long star_offsets(int ndim, int R, long nx, long ny, long *off)
{
    long stride[3] = {1, nx, nx * ny};
    long n = 0;
    off[n++] = 0;
    for (int a = 0; a < ndim; ++a) {
        for (int k = -R; k <= R; ++k)
            if (k != 0) off[n++] = k * stride[a];
    }
    return n;
}

int oracle_starfn_primal(int ndim, int radius, long nx, long ny, long nz, oracle_star_body_fn f,
                         const double *u, const double *p, double *r)
{
    if (!f || !u || !r || ndim < 1 || ndim > 3 || radius < 1 || radius > 4) return ORACLE_BAD_ARG;
    if (ndim < 3 && nz != 1) return ORACLE_BAD_ARG;
    if (ndim < 2 && ny != 1) return ORACLE_BAD_ARG;
    const long R = radius;
    const long n[3] = {nx, ny, nz};
    for (int a = 0; a < ndim; ++a)
        if (n[a] < 2 * R + 1) return ORACLE_BAD_ARG;
    long off[25];
    const long nread = star_offsets(ndim, radius, nx, ny, off);
    const long zlo = ndim >= 3 ? R : 0, zhi = ndim >= 3 ? nz - 1 - R : 0;
    const long ylo = ndim >= 2 ? R : 0, yhi = ndim >= 2 ? ny - 1 - R : 0;
    double v[25];
    for (long z = zlo; z <= zhi; ++z)
        for (long y = ylo; y <= yhi; ++y)
            for (long x = R; x <= nx - 1 - R; ++x) {
                const long i = x + nx * (y + ny * z);
                for (long k = 0; k < nread; ++k) v[k] = u[i + off[k]];
                r[i] = f(v, p ? p[i] : 0.0);
            }
    return ORACLE_OK;
}

int oracle_starfn_adjoint(int ndim, int radius, long nx, long ny, long nz, oracle_star_partials_fn df,
                          const double *u, const double *p, const double *r_bar, double *u_bar, double *scale)
{
    if (!df || !u || !r_bar || !u_bar || ndim < 1 || ndim > 3 || radius < 1 || radius > 4) return ORACLE_BAD_ARG;
    if (ndim < 3 && nz != 1) return ORACLE_BAD_ARG;
    if (ndim < 2 && ny != 1) return ORACLE_BAD_ARG;
    const long R = radius;
    const long n[3] = {nx, ny, nz};
    for (int a = 0; a < ndim; ++a)
        if (n[a] < 2 * R + 1) return ORACLE_BAD_ARG;
    long off[25];
    const long nread = star_offsets(ndim, radius, nx, ny, off);
    const long zlo = ndim >= 3 ? R : 0, zhi = ndim >= 3 ? nz - 1 - R : 0;
    const long ylo = ndim >= 2 ? R : 0, yhi = ndim >= 2 ? ny - 1 - R : 0;
    double v[25], d[25];
    for (long z = zlo; z <= zhi; ++z)
        for (long y = ylo; y <= yhi; ++y)
            for (long x = R; x <= nx - 1 - R; ++x) {
                const long i = x + nx * (y + ny * z);
                for (long k = 0; k < nread; ++k) v[k] = u[i + off[k]];
                df(v, p ? p[i] : 0.0, d);
                const double rb = r_bar[i];
                for (long k = 0; k < nread; ++k) {
                    u_bar[i + off[k]] += d[k] * rb;
                    if (scale) scale[i + off[k]] += fabs(d[k] * rb);
                }
            }
    return ORACLE_OK;
}
