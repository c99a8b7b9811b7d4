/*
 * sadj_stencil_star.hpp -- primal and gather-form adjoint of a USER-SUPPLIED star-shaped
 * stencil loop of radius 1 on a 2-D or 3-D grid (5-point / 7-point star), for one AMD MI355X
 * (gfx950).  Header only, HIP C++17; include it from a .hip file compiled with
 * hipcc --offload-arch=gfx950.  The 1-D counterpart is sadj_stencil1d.hpp.
 *
 * What it is for (paper Section 3.3.1, the paragraph on large loop bodies; its example,
 * r[i,j] = f(a, b) with a = u[i-1,j], b = u[i,j-1], is two-dimensional): the loop body is an
 * uninterpreted function of the values it reads,
 *     r[i] = f(v, p[i])                                         for i in I = prod_d [1, n_d-2],
 * and the adjoint refers to its partial derivatives as uninterpreted functions too.  Here
 * both are member functions of a device functor, and the kernels below are the same for every
 * body: a new nonlinear 2-D or 3-D stencil needs a functor, not a kernel.
 *
 * Reads.  v[0] = u[i]; then for the axes x, y (and z) in turn the neighbours at -1 and +1:
 *     v = { u[i], u[i-ex], u[i+ex], u[i-ey], u[i+ey] (, u[i-ez], u[i+ez]) },  NREAD = 1 + 2*ndim.
 * A body that reads fewer cells ignores the others and returns zero partials for them.
 *
 * The functor F (trivially copyable, passed by value to the kernel) provides
 *     static constexpr int  ndim;           // 2 or 3
 *     static constexpr bool uses_passive;   // does the body read a passive array p[i]?
 *     static constexpr bool df_uses_u;      // do the partials depend on u (nonlinear body)?
 *     __device__ T    f (const T (&v)[NREAD], T p) const;                    // loop body
 *     __device__ void df(const T (&v)[NREAD], T p, T (&d)[NREAD]) const;     // d[k] = df/dv[k]
 * Only u is active: there is no p_bar (Section 3.3.1, the list of active variables).  With
 * df_uses_u == false (a body linear in u, Section 3.1) the adjoint loads no u, passes zeros
 * for v and accepts u == nullptr.
 *
 * What is computed.
 *   primal_star:   r[i] = f(v(i), p[i]) for i in I; r outside I is left untouched.
 *   adjoint_star:  u_bar[j] += sum_k d_k(j - o_k) * r_bar[j - o_k] [j - o_k in I]   for all j,
 *   o_k the offset of read k and d_k(i) the k-th partial at iteration i: the scatter
 *   u_bar[i + o_k] += d_k(i) r_bar[i] after index shifting (Section 3.3.2).  The shifted
 *   derivative calls read u up to two cells away from j in every combination the star of a
 *   star produces -- e.g. u[j + ex - ey], an index no primal iteration at j touches.  Every
 *   partial is evaluated ONCE per primal iteration: the thread that owns cell i evaluates
 *   df there, multiplies by r_bar[i], keeps the terms for its own column (centre, z-1, z+1)
 *   in registers and hands the four in-plane terms to its neighbours through LDS; the
 *   iterations in the one-cell ring around a tile are evaluated a second time by the tile
 *   they send a term into.  Every u_bar[j] is written by exactly one thread, no atomics; the
 *   result is reproducible bit for bit.  Values of r_bar and p outside I never influence the
 *   result, not even NaN, and whatever df returns for a point outside I is discarded by a
 *   select.
 *
 * Mapping.  An x-y tile of 64 x 32 (fp32: 128 x 32) cells per 512-thread workgroup, 16 bytes
 * per lane, two rows per thread; in 3-D the workgroup marches along z with three running
 * sums per owned cell, the last three (primal: four) planes of u staged in LDS with a two-cell border.
 * Tiles whose iterations, ring included, all lie in I run without guards (core, Section
 * 3.3.3); the others run the guarded instantiation (remainder, Section 3.3.4); one dispatch.
 * Workgroup ids are mapped so that each of the 8 XCDs works on neighbouring tiles.
 *
 * Arguments: DEVICE pointers, dense arrays with x fastest (element (x,y,z) at
 * x + nx*(y + ny*z)), nx*ny*nz elements each (nz = 1 and ignored in 2-D), owned by the caller
 * and valid until the work queued on `stream` has finished; p may be nullptr iff
 * !F::uses_passive, the adjoint's u iff !F::df_uses_u.  r and u_bar must not overlap the inputs.
 * Requirements: every extent >= 3; nx a multiple of 16 bytes' worth of elements and all
 * arrays 16-byte aligned; nx*ny < 2^28.  Returns hipErrorInvalidValue for bad arguments
 * (nothing is enqueued), else the status of the launch.  Asynchronous.
 */
#ifndef SADJ_STENCIL_STAR_HPP
#define SADJ_STENCIL_STAR_HPP

#include <hip/hip_runtime.h>
#include <cstdint>

namespace sadj {
namespace star_detail {

// Cells per thread and threads per workgroup.  A 3-D march overlaps the loads of the next plane
// with the arithmetic of this one inside a workgroup; a 2-D grid has a single plane per tile, so
// there the tile is half as high, which lets three workgroups share a compute unit and overlap
// each other instead.
template <class T, int ND> struct Shape {
    static constexpr int PX = 16 / (int)sizeof(T), PY = ND == 3 ? 2 : 1, BX = 32, BY = 16;
    static constexpr int TX = BX * PX, TY = BY * PY, NT = BX * BY;
    static constexpr int ULX = TX + 4, ULY = TY + 4, UPLANE = ULX * ULY;     // u: tile + border of 2
    static constexpr int TLX = TX + 2, TLY = TY + 2, TPLANE = TLX * TLY;     // terms: tile + ring of 1
    static constexpr int NBORDER = UPLANE - TX * TY;                         // border cells of u
    static constexpr int US = (NBORDER + NT - 1) / NT;                       // border slots per thread
    static constexpr int NRING = 2 * TX + 2 * TY;                            // ring iterations (no corners)
    static constexpr int RS = (NRING + NT - 1) / NT;                         // ring slots per thread
};

template <class T, class F> struct Args {
    F fn;
    const T *u, *p, *r_bar;   // r_bar: adjoint only
    T *out;                   // primal: r, adjoint: u_bar
    int nx, ny, nz;
    int ntx, nty, ntz, zchunk, total;
};

// Workgroups are dealt to the 8 XCDs round-robin by hardware id; each XCD has its own L2.
// Logical id such that every XCD owns a contiguous range (neighbouring tiles share an L2).
__host__ __device__ inline int xcd_range_id(int hw, int total)
{
    const int xcd = hw % 8, idx = hw / 8, base = total / 8, rem = total % 8;
    return xcd * base + (xcd < rem ? xcd : rem) + idx;
}

template <class T, int N> struct alignas(sizeof(T) * N) Vec { T v[N]; };
template <class T, int N> __device__ __forceinline__ Vec<T, N> ldv(const T *p, bool stream)
{
    typedef T VT __attribute__((ext_vector_type(N)));
    const VT t = stream ? __builtin_nontemporal_load(reinterpret_cast<const VT *>(p)) : *reinterpret_cast<const VT *>(p);
    Vec<T, N> r;
#pragma unroll
    for (int e = 0; e < N; ++e) r.v[e] = t[e];
    return r;
}
template <class T, int N> __device__ __forceinline__ void stv(T *p, const Vec<T, N> &v)
{
    typedef T VT __attribute__((ext_vector_type(N)));
    VT t;
#pragma unroll
    for (int e = 0; e < N; ++e) t[e] = v.v[e];
    __builtin_nontemporal_store(t, reinterpret_cast<VT *>(p));
}

// The march of one workgroup over planes of its tile.  ADJ: adjoint (else primal).  GUARD:
// the tile touches the remainder (iterations outside I, cells outside the grid).
template <class T, class F, bool ADJ, bool GUARD>
__device__ __forceinline__ void march(const Args<T, F> &a, int tix, int tiy, int zs, int ze, T *su, T *st)
{
    using S = Shape<T, F::ndim>;
    constexpr int ND = F::ndim, NREAD = 1 + 2 * ND;
    constexpr int PX = S::PX, PY = S::PY, TX = S::TX, TY = S::TY, NT = S::NT;
    constexpr int ULX = S::ULX, TLX = S::TLX, US = S::US, RS = S::RS;
    constexpr int ZR = ND == 3 ? 1 : 0;                 // reach of the star along the march axis
    // planes of u held in LDS: the three a step reads; the primal, which has no second barrier
    // per step, keeps a fourth so that the plane being replaced is never one being read
    constexpr int NU = ND == 3 ? (ADJ ? 3 : 4) : 1;
    constexpr int NACC = 2 * ZR + 1;                    // running sums per owned cell
    constexpr bool NEED_U = !ADJ || F::df_uses_u;
    using V = Vec<T, PX>;

    const int tid = threadIdx.x, tx = tid % S::BX, ty = tid / S::BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;
    const int x = x0 + tx * PX;

    // ---- owned cells (a vector of PX cells is entirely inside or outside the grid: nx % PX == 0)
    size_t ooff[PY];
    bool oin[PY], oI[PY][PX];
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        const int y = y0 + ty * PY + p;
        oin[p] = GUARD ? (x < nx && y < ny) : true;
        ooff[p] = oin[p] ? (size_t)y * nx + x : 0;
#pragma unroll
        for (int e = 0; e < PX; ++e) oI[p][e] = GUARD ? (x + e >= 1 && x + e <= nx - 2 && y >= 1 && y <= ny - 2) : true;
    }
    // ---- border cells of the u tile (everything of the (TX+4) x (TY+4) block that is not owned)
    size_t boff[US];
    int blds[US];
    bool bslot[US];
#pragma unroll
    for (int s = 0; s < US; ++s) {
        const int h = tid + s * NT;
        // rows 0,1 and TY+2,TY+3 in full, then the two columns left and right of the middle rows
        int lx, ly;
        if (h < 4 * ULX) { ly = h / ULX; lx = h - ly * ULX; if (ly >= 2) ly += TY; }
        else { const int h2 = h - 4 * ULX; ly = 2 + h2 / 4; const int k = h2 % 4; lx = k < 2 ? k : k + TX; }
        bslot[s] = h < S::NBORDER;
        int gx = x0 - 2 + lx, gy = y0 - 2 + ly;
        gx = gx < 0 ? 0 : (gx > nx - 1 ? nx - 1 : gx);          // clamped: such values feed only discarded iterations
        gy = gy < 0 ? 0 : (gy > ny - 1 ? ny - 1 : gy);
        boff[s] = bslot[s] ? (size_t)gy * nx + gx : 0;
        blds[s] = bslot[s] ? ly * ULX + lx : 0;
    }
    // ---- ring iterations around the tile (adjoint): the cells left, right, below and above it
    size_t roff[RS];
    int rlx[RS], rly[RS];
    bool rI[RS], rslot[RS];
    if (ADJ) {
#pragma unroll
        for (int s = 0; s < RS; ++s) {
            const int h = tid + s * NT;
            int lx, ly;                                          // in term-plane coordinates (origin x0-1, y0-1)
            if (h < 2 * TX) { ly = h < TX ? 0 : TY + 1; lx = 1 + (h < TX ? h : h - TX); }
            else { const int h2 = h - 2 * TX; lx = h2 < TY ? 0 : TX + 1; ly = 1 + (h2 < TY ? h2 : h2 - TY); }
            rslot[s] = h < S::NRING;
            const int gx = x0 - 1 + lx, gy = y0 - 1 + ly;
            rI[s] = rslot[s] && gx >= 1 && gx <= nx - 2 && gy >= 1 && gy <= ny - 2;
            roff[s] = rI[s] ? (size_t)gy * nx + gx : 0;
            rlx[s] = rslot[s] ? lx : 0;
            rly[s] = rslot[s] ? ly : 0;
        }
    }

    auto plane_in_I = [&](int z) { return ND == 2 ? true : (z >= 1 && z <= nz - 2); };

    // ---- staging registers (one plane ahead)
    V gu[PY], gp[PY], gr[PY], gb[PY];
    T gub[US], gpr[RS], grr[RS];
#pragma unroll
    for (int p = 0; p < PY; ++p) { gu[p] = V{}; gp[p] = V{}; gr[p] = V{}; gb[p] = V{}; }
#pragma unroll
    for (int s = 0; s < US; ++s) gub[s] = T(0);
#pragma unroll
    for (int s = 0; s < RS; ++s) { gpr[s] = T(0); grr[s] = T(0); }

    T acc[PY][PX][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e)
#pragma unroll
            for (int k = 0; k < NACC; ++k) acc[p][e][k] = T(0);

    // iteration planes that matter: the adjoint's outputs [zs, ze) receive terms from
    // iterations zs-ZR .. ze-1+ZR; the primal's outputs are its own iterations
    const int it0 = ADJ ? zs - ZR : zs, it1 = ADJ ? ze - 1 + ZR : ze - 1;

    auto load_u_plane = [&](int z) {                    // plane z of u into the staging registers
        if (!NEED_U) return;
        if (z < 0 || z > nz - 1) return;
        const T *up = a.u + (size_t)z * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) gu[p] = ldv<T, PX>(up + ooff[p], false);
#pragma unroll
        for (int s = 0; s < US; ++s) gub[s] = up[boff[s]];
    };
    auto store_u_plane = [&](int z) {                   // staging registers -> ring slot of plane z
        if (!NEED_U) return;
        if (z < 0 || z > nz - 1) return;
        T *sb = su + ((z + NU) % NU) * S::UPLANE;
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) sb[(2 + ty * PY + p) * ULX + 2 + tx * PX + e] = gu[p].v[e];
#pragma unroll
        for (int s = 0; s < US; ++s)
            if (bslot[s]) sb[blds[s]] = gub[s];
    };
    auto load_rest = [&](int z) {                       // what iteration plane z needs besides u
        if (z > it1) return;
        if (plane_in_I(z)) {
            if (F::uses_passive) {
                const T *pp = a.p + (size_t)z * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) gp[p] = ldv<T, PX>(pp + ooff[p], !ADJ);
                if (ADJ) {
#pragma unroll
                    for (int s = 0; s < RS; ++s) gpr[s] = pp[roff[s]];
                }
            }
            if (ADJ) {
                const T *rp = a.r_bar + (size_t)z * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) gr[p] = ldv<T, PX>(rp + ooff[p], false);
#pragma unroll
                for (int s = 0; s < RS; ++s) grr[s] = rp[roff[s]];
            }
        }
        if (ADJ) {
            const int zo = z - ZR;                       // the output plane this step completes
            if (zo >= zs && zo < ze) {
                const T *bp = a.out + (size_t)zo * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) gb[p] = ldv<T, PX>(bp + ooff[p], true);
            }
        }
    };
    // reads of the iteration at LDS position (lx, ly) of the u tile, plane z
    auto reads = [&](int lx, int ly, int z, T (&v)[NREAD]) {
        if (!NEED_U) {
#pragma unroll
            for (int k = 0; k < NREAD; ++k) v[k] = T(0);
            return;
        }
        const T *sb = su + ((z + NU) % NU) * S::UPLANE + ly * ULX + lx;
        v[0] = sb[0]; v[1] = sb[-1]; v[2] = sb[1]; v[3] = sb[-ULX]; v[4] = sb[ULX];
        if constexpr (ND == 3) {
            v[NREAD - 2] = su[((z - 1 + NU) % NU) * S::UPLANE + ly * ULX + lx];
            v[NREAD - 1] = su[((z + 1 + NU) % NU) * S::UPLANE + ly * ULX + lx];
        }
    };

    // ---- prime the ring: planes it0-1 and it0 synchronously, plane it0+1 stays in flight
    if (NEED_U) {
        for (int z = it0 - ZR; z <= it0; ++z) {
            load_u_plane(z);
            store_u_plane(z);
        }
        if (ND == 3) load_u_plane(it0 + 1);
    }
    load_rest(it0);

    for (int zi = it0; zi <= it1; ++zi) {
        const bool zin = plane_in_I(zi);
        if (ND == 3) store_u_plane(zi + 1);
        // consume the staged values of this step
        V cp[PY], cr[PY], cb[PY];
        T cpr[RS], crr[RS];
#pragma unroll
        for (int p = 0; p < PY; ++p) { cp[p] = gp[p]; cr[p] = gr[p]; cb[p] = gb[p]; }
#pragma unroll
        for (int s = 0; s < RS; ++s) { cpr[s] = gpr[s]; crr[s] = grr[s]; }
        if (ND == 3) load_u_plane(zi + 2);
        load_rest(zi + 1);
        __syncthreads();                                 // plane zi+1 of u is in the ring
        if (!ADJ) {
            if (zin) {
                T *rp = a.out + (size_t)zi * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) {
                    V o;
                    bool all = true;
#pragma unroll
                    for (int e = 0; e < PX; ++e) {
                        T v[NREAD];
                        reads(2 + tx * PX + e, 2 + ty * PY + p, zi, v);
                        o.v[e] = a.fn.f(v, F::uses_passive ? cp[p].v[e] : T(0));
                        all = all && oI[p][e];
                    }
                    if (!GUARD || all) {
                        stv<T, PX>(rp + ooff[p], o);
                    } else {
#pragma unroll
                        for (int e = 0; e < PX; ++e)
                            if (oI[p][e]) rp[ooff[p] + e] = o.v[e];
                    }
                }
            }
            continue;
        }
        // ---- adjoint: evaluate the partials once per iteration, form the terms
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    T v[NREAD], d[NREAD];
                    reads(2 + tx * PX + e, 2 + ty * PY + p, zi, v);
                    a.fn.df(v, F::uses_passive ? cp[p].v[e] : T(0), d);
                    const T rb = cr[p].v[e];
                    const bool ok = oI[p][e];
                    T t[NREAD];
#pragma unroll
                    for (int k = 0; k < NREAD; ++k) t[k] = ok ? d[k] * rb : T(0);
                    acc[p][e][ZR] += t[0];
                    if constexpr (ND == 3) {
                        acc[p][e][0] += t[NREAD - 2];      // read of u[z-1]: lands one plane below
                        acc[p][e][2] += t[NREAD - 1];      // read of u[z+1]: lands one plane above
                    }
                    const int li = (1 + ty * PY + p) * TLX + 1 + tx * PX + e;
#pragma unroll
                    for (int k = 0; k < 4; ++k) st[k * S::TPLANE + li] = t[1 + k];
                }
#pragma unroll
            for (int s = 0; s < RS; ++s) {
                T v[NREAD], d[NREAD];
                reads(1 + rlx[s], 1 + rly[s], zi, v);
                a.fn.df(v, F::uses_passive ? cpr[s] : T(0), d);
                const T rb = crr[s];
                if (rslot[s]) {
                    const int li = rly[s] * TLX + rlx[s];
#pragma unroll
                    for (int k = 0; k < 4; ++k) st[k * S::TPLANE + li] = rI[s] ? d[1 + k] * rb : T(0);
                }
            }
        }
        __syncthreads();                                 // the terms of plane zi are in LDS
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const int li = (1 + ty * PY + p) * TLX + 1 + tx * PX + e;
                    // term of read k of the iteration at j - o_k: reads at -ex, +ex, -ey, +ey
                    const T s = (st[0 * S::TPLANE + li + 1] + st[1 * S::TPLANE + li - 1]) +
                                (st[2 * S::TPLANE + li + TLX] + st[3 * S::TPLANE + li - TLX]);
                    acc[p][e][ZR] += s;
                }
        }
        const int zo = zi - ZR;
        if (zo >= zs && zo < ze) {
            T *bp = a.out + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = cb[p].v[e] + acc[p][e][0];
                if (!GUARD || oin[p]) stv<T, PX>(bp + ooff[p], o);
            }
        }
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) {
#pragma unroll
                for (int k = 0; k < NACC - 1; ++k) acc[p][e][k] = acc[p][e][k + 1];
                acc[p][e][NACC - 1] = T(0);
            }
    }
}

template <class T, class F, bool ADJ>
__global__ __launch_bounds__((Shape<T, F::ndim>::NT)) void kernel(Args<T, F> a)
{
    using S = Shape<T, F::ndim>;
    constexpr int NU = F::ndim == 3 ? (ADJ ? 3 : 4) : 1;
    constexpr bool NEED_U = !ADJ || F::df_uses_u;
    __shared__ T su[NEED_U ? NU * S::UPLANE : 1];
    __shared__ T st[ADJ ? 4 * S::TPLANE : 1];
    const int L = xcd_range_id(blockIdx.x, a.total);
    const int tiles = a.ntx * a.nty;
    const int tiz = L / tiles, t = L - tiz * tiles;
    const int tiy = t / a.ntx, tix = t - tiy * a.ntx;
    const int zs = tiz * a.zchunk;
    const int ze = zs + a.zchunk < a.nz ? zs + a.zchunk : a.nz;
    // core tile: its iterations and the ring around it lie in I, its border of two lies in the grid
    const int x0 = tix * S::TX, y0 = tiy * S::TY;
    const bool core = x0 >= 2 && x0 + S::TX + 2 <= a.nx && y0 >= 2 && y0 + S::TY + 2 <= a.ny;
    if (core) march<T, F, ADJ, false>(a, tix, tiy, zs, ze, su, st);
    else      march<T, F, ADJ, true>(a, tix, tiy, zs, ze, su, st);
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <class T, class F, bool ADJ>
hipError_t launch(Args<T, F> a, hipStream_t stream)
{
    using S = Shape<T, F::ndim>;
    if (a.nx < 3 || a.ny < 3 || (F::ndim == 3 && a.nz < 3)) return hipErrorInvalidValue;
    if ((long)a.nx * a.ny >= (1L << 28) || a.nx % S::PX != 0) return hipErrorInvalidValue;
    if (!aligned16(a.u) || !aligned16(a.p) || !aligned16(a.r_bar) || !aligned16(a.out)) return hipErrorInvalidValue;
    if (F::ndim == 2) a.nz = 1;
    a.ntx = (a.nx + S::TX - 1) / S::TX;
    a.nty = (a.ny + S::TY - 1) / S::TY;
    const long tiles = (long)a.ntx * a.nty;
    // z-chunks: as many as it takes to give every compute unit a workgroup, each at least 16 planes
    int dev = 0, ncu = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) ncu = v;
    }
    long chunks = 1;
    if (F::ndim == 3) {
        // fewest rounds of ncu workgroups, chunks of at least 16 planes
        long best = -1;
        const long maxc = a.nz / 16 > 0 ? a.nz / 16 : 1;
        for (long c = 1; c <= maxc && c <= 64; ++c) {
            const long cost = (tiles * c + ncu - 1) / ncu * ((a.nz + c - 1) / c + 2);
            if (best < 0 || cost < best) { best = cost; chunks = c; }
        }
    }
    a.zchunk = (int)((a.nz + chunks - 1) / chunks);
    a.ntz = (a.nz + a.zchunk - 1) / a.zchunk;
    const long total = tiles * a.ntz;
    if (total > 0x3fffffffL) return hipErrorInvalidValue;
    a.total = (int)total;
    hipLaunchKernelGGL((kernel<T, F, ADJ>), dim3((unsigned)total), dim3(S::NT), 0, stream, a);
    return hipGetLastError();
}

}  // namespace star_detail

// r[i] = f(v(i), p[i]) on I.  2-D: pass nz = 1.
template <class T, class F>
hipError_t primal_star(const F &fn, int nx, int ny, int nz, const T *u, const T *p, T *r, hipStream_t stream)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "float or double");
    static_assert(F::ndim == 2 || F::ndim == 3, "two or three dimensions");
    if (!u || !r || (F::uses_passive && !p)) return hipErrorInvalidValue;
    star_detail::Args<T, F> a{fn, u, F::uses_passive ? p : nullptr, nullptr, r, nx, ny, nz, 0, 0, 0, 0, 0};
    return star_detail::launch<T, F, false>(a, stream);
}

// u_bar += (dr/du)^T r_bar, as a gather.  2-D: pass nz = 1.
template <class T, class F>
hipError_t adjoint_star(const F &fn, int nx, int ny, int nz, const T *u, const T *p, const T *r_bar, T *u_bar,
                        hipStream_t stream)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "float or double");
    static_assert(F::ndim == 2 || F::ndim == 3, "two or three dimensions");
    if ((F::df_uses_u && !u) || !r_bar || !u_bar || (F::uses_passive && !p)) return hipErrorInvalidValue;
    star_detail::Args<T, F> a{fn, F::df_uses_u ? u : nullptr, F::uses_passive ? p : nullptr, r_bar, u_bar,
                              nx, ny, nz, 0, 0, 0, 0, 0};
    return star_detail::launch<T, F, true>(a, stream);
}

}  // namespace sadj
#endif /* SADJ_STENCIL_STAR_HPP */
