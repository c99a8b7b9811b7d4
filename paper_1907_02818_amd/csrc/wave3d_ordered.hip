// 3-D linear wave stencil of radius R: gather-form adjoint that adds the terms of every
// u_bar[j] in the order, and with the rounding, of the sequential scatter adjoint.
//
// Paper Section 3.5: the method assumes that the contributions to an output index may be
// reordered, notes that floating point does not honour this, and observes that a gather
// can respect any order the user chooses and still run in parallel, because all updates
// of an index sit in one iteration.  The order offered here is the one a conventional
// reverse-mode tool produces when its scatter loop runs sequentially (Section 3.2):
// primal iterations i in ascending memory order (z slowest, x fastest), iteration i adding
//     (2 + c[i]*3*w_0) * r_bar[i]     to u_bar[i]
//     (c[i]*w_|k|) * r_bar[i]         to u_bar[i + k e_d],  k != 0, d = x, y, z
// one rounded product and one rounded addition each, no fused multiply-add.  Output j
// receives at most one term per iteration, so its terms arrive in the order of their
// source cell:
//     (x,y,z-R) .. (x,y,z-1),  (x,y-R,z) .. (x,y-1,z),  (x-R,y,z) .. (x-1,y,z),  (x,y,z),
//     (x+1,y,z) .. (x+R,y,z),  (x,y+1,z) .. (x,y+R,z),  (x,y,z+1) .. (x,y,z+R),
// starting from the incoming u_bar[j]; sources outside I contribute nothing (they are
// skipped, not added as zeros, so that even the sign of a zero result is the scatter's).
// In fp64 the result equals the sequential scatter adjoint bit for bit.
//
// Mapping.  Same z-march as the default kernel (a workgroup owns an x-y tile, 2R+1 running
// sums per owned cell in registers, ascending source planes), with three differences:
// LDS holds the finished terms (c*w_k)*r_bar of every staged cell, one plane per |k| (a term
// is (c*w)*r_bar, not w*(c*r_bar), so the product c*r_bar cannot be shared between the k);
// a running sum is initialised with u_bar when it is created, R planes before its own
// plane arrives, instead of adding u_bar at the end; and contraction of multiply-add is
// off.
#include "launch.hpp"
#include "tile3d.hpp"

#pragma clang fp contract(off)

namespace sadj {

template <class T, int R, int BX, int BY, int PY, bool GUARD, bool UPREV>
__device__ __forceinline__ void adj3d_march_ordered(const March3dArgs &a, int tix, int tiy, int zs, int ze,
                                                    T *__restrict__ lds)
{
    using G = Tile3d<T, R, BX, BY, PY, 1>;
    constexpr int TX = G::TX, TY = G::TY, LX = G::LX, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;

    const T *__restrict__ cg = static_cast<const T *>(a.in0);
    const T *__restrict__ rg = static_cast<const T *>(a.in1);
    T *__restrict__ ug = static_cast<T *>(a.out0);
    T *__restrict__ upg = static_cast<T *>(a.out1);

    // owned cells (x, y0 + ty*PY + p) and halo slots (tile3d.hpp; halo slots are loaded wherever the
    // cell lies in the grid, their use is decided per term); per owned cell, which of its sources
    // lie in I: bit R+d of xbits: x+d in I_x;  bit R+d of ybits[p]: y_p+d in I_y
    TileAddr<1, PY, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, nx, ny, R, R, LX, 0 /* cell (0,0) is a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
    const int x = x0 + tx;
    uint32_t ooff[PY], ybits[PY], xbits = 0;
    bool ostore[PY];
#pragma unroll
    for (int d = -R; d <= R; ++d)
        if (!GUARD || (x + d >= R && x + d < nx - R)) xbits |= 1u << (R + d);
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        const int y = y0 + ty * PY + p;
        ostore[p] = ad.own_grid[p];
        ooff[p] = ad.own_off[p];
        ybits[p] = 0;
#pragma unroll
        for (int d = -R; d <= R; ++d)
            if (!GUARD || (y + d >= R && y + d < ny - R)) ybits[p] |= 1u << (R + d);
    }
    uint32_t hoff[HS];
    int hlds[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) { hoff[s] = ad.halo_off[s]; hlds[s] = ad.halo_lds[s]; }
    auto xin = [&](int d) { return !GUARD || ((xbits >> (R + d)) & 1u); };
    auto yin = [&](int p, int d) { return !GUARD || ((ybits[p] >> (R + d)) & 1u); };

    T acc[PY][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int k = 0; k < NACC; ++k) acc[p][k] = T(0);

    T sc[PY], sr[PY], su[PY], sp[PY], shc[HS], shr[HS];
#pragma unroll
    for (int p = 0; p < PY; ++p) sc[p] = sr[p] = su[p] = sp[p] = T(0);
#pragma unroll
    for (int s = 0; s < HS; ++s) shc[s] = shr[s] = T(0);

    const int zi0 = zs - R, zi1 = ze - 1 + R;       // source planes that reach outputs [zs, ze)
    auto plane_in_I = [&](int z) { return z >= R && z < nz - R; };

    // everything step z consumes: plane z of c and r_bar (if in I), u_bar of plane z+R
    // (the running sum created in step z), u_prev_bar of plane z
    auto issue = [&](int z) {
        if (z > zi1) return;
        if (plane_in_I(z)) {
            const T *cp = cg + (size_t)z * plane;
            const T *rp = rg + (size_t)z * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) { sc[p] = ld_off(cp, ooff[p]); sr[p] = ld_off(rp, ooff[p]); }
#pragma unroll
            for (int s = 0; s < HS; ++s) { shc[s] = ld_off(cp, hoff[s]); shr[s] = ld_off(rp, hoff[s]); }
            if (UPREV && z >= zs && z < ze) {
                const T *pp = upg + (size_t)z * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) sp[p] = ld_stream<T, true>(pp, ooff[p]);
            }
        }
        const int zn = z + R;
        if (zn >= zs && zn < ze) {
            const T *up = ug + (size_t)zn * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) su[p] = ld_stream<T, true>(up, ooff[p]);
        }
    };

    // LDS holds, per |k| = 1..R, the plane of finished terms P_k = (c w_k) r_bar of the
    // staged cells: a term is formed once per source cell and read by the (up to) four
    // in-plane neighbours at distance k.  One buffer, two barriers per plane (NBUF = 2 would
    // save a barrier but the LDS is better spent on a second workgroup per CU).
    constexpr int NBUF = 1;
    int buf = 0;
    issue(zi0);
    for (int zi = zi0; zi <= zi1; ++zi) {
        const bool zin = plane_in_I(zi);
        const int zo = zi - R, zn = zi + R;
        T *lp = lds + (NBUF == 2 ? buf : 0) * (R * G::PLANE);
        // the running sum of output plane zi+R starts from the incoming u_bar
        if (zn >= zs && zn < ze) {
#pragma unroll
            for (int p = 0; p < PY; ++p) acc[p][NACC - 1] = su[p];
        }
        T cc[PY], rv[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) { cc[p] = sc[p]; rv[p] = sr[p]; }
        if (zin) {
            if (NBUF == 1) __syncthreads();         // all reads of the previous plane are done
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                const bool own = xin(0) && yin(p, 0);
                const int cell = (R + ty * PY + p) * LX + R + tx;
#pragma unroll
                for (int k = 1; k <= R; ++k) {
                    const T t = (cc[p] * T(star_w<R>(k))) * rv[p];
                    lp[(k - 1) * G::PLANE + cell] = t;
                    // this plane lies above the output planes zi-R .. zi-1 (for them it is the
                    // source "z+k") and below zi+1 .. zi+R (source "z-k"): one term each
                    acc[p][R - k] = own ? acc[p][R - k] + t : acc[p][R - k];
                    acc[p][R + k] = own ? acc[p][R + k] + t : acc[p][R + k];
                }
            }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
#pragma unroll
                for (int k = 1; k <= R; ++k) lp[(k - 1) * G::PLANE + hlds[s]] = (shc[s] * T(star_w<R>(k))) * shr[s];
            }
            if (UPREV && zi >= zs && zi < ze) {
                T *pp = upg + (size_t)zi * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p)
                    if (ostore[p] && xin(0) && yin(p, 0)) st_stream<T, true>(pp, ooff[p], sp[p] - rv[p]);
            }
        }
        issue(zi + 1);
        if (zin) {
            __syncthreads();
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                const int lrow = R + ty * PY + p, lcol = R + tx;
                // in-plane terms of output plane zi, in ascending order of the source cell
                T s = acc[p][R];
#pragma unroll
                for (int k = R; k >= 1; --k) {      // (x, y-k)
                    const T t = lp[(k - 1) * G::PLANE + (lrow - k) * LX + lcol];
                    s = (xin(0) && yin(p, -k)) ? s + t : s;
                }
#pragma unroll
                for (int k = R; k >= 1; --k) {      // (x-k, y)
                    const T t = lp[(k - 1) * G::PLANE + lrow * LX + lcol - k];
                    s = (xin(-k) && yin(p, 0)) ? s + t : s;
                }
                {
                    const T t = (T(2) + cc[p] * T(3) * T(star_w<R>(0))) * rv[p];
                    s = (xin(0) && yin(p, 0)) ? s + t : s;
                }
#pragma unroll
                for (int k = 1; k <= R; ++k) {      // (x+k, y)
                    const T t = lp[(k - 1) * G::PLANE + lrow * LX + lcol + k];
                    s = (xin(k) && yin(p, 0)) ? s + t : s;
                }
#pragma unroll
                for (int k = 1; k <= R; ++k) {      // (x, y+k)
                    const T t = lp[(k - 1) * G::PLANE + (lrow + k) * LX + lcol];
                    s = (xin(0) && yin(p, k)) ? s + t : s;
                }
                acc[p][R] = s;
            }
            buf ^= 1;
        }
        if (zo >= zs) {                             // zo <= ze-1 because zi <= zi1
            T *up = ug + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p)
                if (ostore[p]) st_stream<T, true>(up, ooff[p], acc[p][0]);
        }
#pragma unroll
        for (int p = 0; p < PY; ++p) {
#pragma unroll
            for (int k = 0; k < NACC - 1; ++k) acc[p][k] = acc[p][k + 1];
            acc[p][NACC - 1] = T(0);
        }
    }
}

template <class T, int R, int BX, int BY, int PY, bool UPREV>
__global__ __launch_bounds__(BX *BY) void adj_wave3d_ordered_kernel(March3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY, 1>;
    constexpr int NBUF = 1;
    __shared__ T lds[NBUF * R * G::PLANE];          // per |k| a plane of finished terms, see the march
    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);
    const int x0 = tix * G::TX, y0 = tiy * G::TY;
    const bool core = x0 >= 2 * R && x0 + G::TX + 2 * R <= a.nx && y0 >= 2 * R && y0 + G::TY + 2 * R <= a.ny;
    if (core) adj3d_march_ordered<T, R, BX, BY, PY, false, UPREV>(a, tix, tiy, zs, ze, lds);
    else      adj3d_march_ordered<T, R, BX, BY, PY, true, UPREV>(a, tix, tiy, zs, ze, lds);
}

// 64 x 16 tile, 256 threads, one LDS buffer: two workgroups share a CU, so that one computes
// while the other waits for memory.  Measured at 512^3 fp64 against one workgroup of 512
// threads on a 64 x 32 tile with two buffers: radius 4 1.22 vs 1.41 ms, radius 1 0.74 vs 0.82 ms.
template <class T, int R>
static hipError_t launch_ordered_T(March3dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    constexpr int BX = 64, BY = 4, PY = 4;
    using G = Tile3d<T, R, BX, BY, PY, 1>;
    static_assert(sizeof(T) * R * G::PLANE <= 80 * 1024, "two workgroups must fit into the LDS of a CU");
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, R, opt, 2);
    dim3 grid(a.map.total_blocks), block(G::NT);
    // exactly two per CU: request LDS up to just over a third of a CU's 160 KB
    constexpr size_t static_lds = sizeof(T) * R * G::PLANE, third = 54 * 1024;
    unsigned pad = static_lds < third ? (unsigned)(third - static_lds) : 0;
    if (opt.lds_pad > 0) pad = (unsigned)opt.lds_pad;
    if (opt.lds_pad < 0) pad = 0;
    if (a.out1) hipLaunchKernelGGL((adj_wave3d_ordered_kernel<T, R, BX, BY, PY, true>), grid, block, pad, stream, a);
    else        hipLaunchKernelGGL((adj_wave3d_ordered_kernel<T, R, BX, BY, PY, false>), grid, block, pad, stream, a);
    return hipGetLastError();
}

hipError_t launch_adjoint_wave3d_ordered(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                         const void *r_bar, void *u_bar, void *u_prev_bar,
                                         const LaunchOptions &opt, hipStream_t stream)
{
    March3dArgs a{};
    a.in0 = c; a.in1 = r_bar; a.out0 = u_bar; a.out1 = u_prev_bar;
    a.nx = nx; a.ny = ny; a.nz = nz;
    if (is_f64) {
        switch (radius) {
        case 1: return launch_ordered_T<double, 1>(a, opt, stream);
        case 2: return launch_ordered_T<double, 2>(a, opt, stream);
        case 3: return launch_ordered_T<double, 3>(a, opt, stream);
        default: return launch_ordered_T<double, 4>(a, opt, stream);
        }
    }
    switch (radius) {
    case 1: return launch_ordered_T<float, 1>(a, opt, stream);
    case 2: return launch_ordered_T<float, 2>(a, opt, stream);
    case 3: return launch_ordered_T<float, 3>(a, opt, stream);
    default: return launch_ordered_T<float, 4>(a, opt, stream);
    }
}

}  // namespace sadj
