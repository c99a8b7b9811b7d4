// 2-D linear wave stencil, 5-point star (radius 1): primal and gather-form adjoint.
//
// Adjoint: with q = c*r_bar on I and 0 elsewhere,
//     u_bar[j] += 2 r_bar[j] [j in I] + q[j-ex] + q[j+ex] + q[j-ey] + q[j+ey] - 4 q[j]
// (paper Section 4.1 gather listing reduced to two dimensions; Sections 3.3.2-3.3.4).
//
// Mapping to CDNA4.  Each 64-lane wave owns a strip of 64*PX columns (PX elements
// = 16 bytes per lane, x is unit stride) and marches down y.  An arriving row of q
// contributes its x-neighbours and centre to the running sum of the same output row
// and q itself to the sums of the rows above and below, so a lane keeps three
// running sums per owned column; x-neighbours travel between lanes with wave
// shuffles and the two cells beside the strip are loaded by lanes 0 and 63.  There
// is no LDS; waves exchange nothing, but those of a workgroup meet at a barrier every few
// rows so that they stream neighbouring pieces of the same rows (plan_row_march).  Waves whose reads all lie in I
// run the unguarded instantiation (core); waves touching the first/last columns or
// rows run the guarded one, where unused cells are replaced by zero with a select
// (the if-guarded remainder variant of Section 3.3.4).
#include "common.hpp"
#include "launch.hpp"
#include "tile3d.hpp"

#include <type_traits>

namespace sadj {

struct Wave2dArgs {
    const void *c, *r_bar;
    void *u_bar, *u_prev_bar;
    const void *u, *u_prev;
    void *r;
    int nx, ny;
    int ychunk;
};


// D rows of loads are kept in flight per wave.  In the steady part of the march every
// row of a step is known to exist, so that part is compiled without branches and the
// compiler can count exactly which loads may still be outstanding.
template <int D>
__device__ __forceinline__ RowMarch adj2d_rows(int ys, int ye, int ny)
{
    // steady steps yi in [lo, hi]: rows yi and yi+D lie in I and in this chunk's input
    // range; output rows yi-1 and yi+D-1 (for u_prev_bar: yi and yi+D) belong to the chunk
    return plan_row_march(ys - 1, ye, ys + 1, min(ny - 1, ye) - 1 - D, D);
}

template <class T, int PX, int D, bool GUARD, bool UPREV>
__device__ __forceinline__ void adj2d_strip(const Wave2dArgs &a, int xs, int ys, int ye, int lane, const RowMarch rm)
{
    constexpr int W = 64 * PX;
    using V = Vec<T, PX>;
    const int nx = a.nx, ny = a.ny;
    const T *__restrict__ cg = static_cast<const T *>(a.c);
    const T *__restrict__ rg = static_cast<const T *>(a.r_bar);
    T *__restrict__ ug = static_cast<T *>(a.u_bar);
    T *__restrict__ pg = static_cast<T *>(a.u_prev_bar);

    const int x = xs + lane * PX;
    const bool active = GUARD ? (x < nx) : true;
    const int xc = active ? x : xs;
    bool xin[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) xin[e] = GUARD ? (x + e >= 1 && x + e <= nx - 2) : true;
    const int hx = lane < 32 ? xs - 1 : xs + W;
    const bool hin = GUARD ? (hx >= 1 && hx <= nx - 2) : true;
    const int hxc = hin ? hx : xs;
    const bool edge_lane = lane == 0 || lane == 63;

    T acc[PX][3];
#pragma unroll
    for (int e = 0; e < PX; ++e) acc[e][0] = acc[e][1] = acc[e][2] = T(0);
    V sc[D], sr[D], su[D], sp[D];
    T shc[D], shr[D];
#pragma unroll
    for (int d = 0; d < D; ++d) {
        sc[d] = V{}; sr[d] = V{}; su[d] = V{}; sp[d] = V{};
        shc[d] = shr[d] = T(0);
    }

    const int yi0 = ys - 1, yi1 = ye;            // input rows that reach output rows [ys, ye)
    auto row_in_I = [&](int y) { return y >= 1 && y <= ny - 2; };

    auto issue = [&](int y, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        if (!STEADY && y > yi1) return;
        if (STEADY || row_in_I(y)) {
            const T *cp = cg + (size_t)y * nx;
            const T *rp = rg + (size_t)y * nx;
            sc[d] = ld_vec<T, PX>(cp + xc);           // plain: streaming c or r_bar measured 2-3 points slower
            sr[d] = ld_vec<T, PX>(rp + xc);
            if (edge_lane) { shc[d] = cp[hxc]; shr[d] = rp[hxc]; }   // only lanes 0 and 63 use the value
            if (UPREV) {
                if (STEADY || (y >= ys && y < ye)) sp[d] = ld_vec_stream<T, PX>(pg + (size_t)y * nx + xc);
            }
        }
        const int yo = y - 1;
        if (STEADY || yo >= ys) su[d] = ld_vec_stream<T, PX>(ug + (size_t)yo * nx + xc);
    };

    auto step = [&](int yi, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        const bool rin = STEADY || row_in_I(yi);
        const int yo = yi - 1;
        const V cu = su[d];
        if (rin) {
            T q[PX], rr[PX];
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                rr[e] = GUARD ? (xin[e] ? sr[d].v[e] : T(0)) : sr[d].v[e];
                q[e] = GUARD ? (xin[e] ? sc[d].v[e] * sr[d].v[e] : T(0)) : sc[d].v[e] * sr[d].v[e];
            }
            const T qh = GUARD ? (hin ? shc[d] * shr[d] : T(0)) : shc[d] * shr[d];
            if (UPREV) {
                if ((STEADY || (yi >= ys && yi < ye)) && active) {
                    V o;
#pragma unroll
                    for (int e = 0; e < PX; ++e) o.v[e] = sp[d].v[e] - rr[e];
                    st_vec_stream<T, PX>(pg + (size_t)yi * nx + x, o);
                }
            }
            T left, right;
            wave_neighbours<T, PX>(q, qh, lane, left, right);
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                const T l = e == 0 ? left : q[e - 1];
                const T r = e == PX - 1 ? right : q[e + 1];
                acc[e][1] += (T(-4) * q[e] + (l + r)) + T(2) * rr[e];
                acc[e][0] += q[e];
                acc[e][2] += q[e];
            }
        }
        issue(yi + D, dc, steady);
        if ((STEADY || yo >= ys) && active) {
            V o;
#pragma unroll
            for (int e = 0; e < PX; ++e) o.v[e] = cu.v[e] + acc[e][0];
            st_vec_stream<T, PX>(ug + (size_t)yo * nx + x, o);
        }
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            acc[e][0] = acc[e][1];
            acc[e][1] = acc[e][2];
            acc[e][2] = T(0);
        }
    };
    using No = std::integral_constant<bool, false>;
    using Yes = std::integral_constant<bool, true>;
    auto step_any = [&](int yi, int d) {
        if (D == 1 || d == 0) step(yi, std::integral_constant<int, 0>{}, No{});
        else if (D == 2 || d == 1) step(yi, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, No{});
        else if (D == 3 || d == 2) step(yi, std::integral_constant<int, (D > 2 ? 2 : 0)>{}, No{});
        else step(yi, std::integral_constant<int, (D > 3 ? 3 : 0)>{}, No{});
    };
    issue(yi0, std::integral_constant<int, 0>{}, No{});
    if (D > 1) issue(yi0 + 1, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, No{});
    if (D > 2) issue(yi0 + 2, std::integral_constant<int, (D > 2 ? 2 : 0)>{}, No{});
    if (D > 3) issue(yi0 + 3, std::integral_constant<int, (D > 3 ? 3 : 0)>{}, No{});

    int yi = yi0, d = 0;
    for (; yi < rm.pre_end; ++yi) {
        step_any(yi, d);
        d = d + 1 == D ? 0 : d + 1;
    }
    for (int group = 1; group <= rm.steady; ++group) {
        step(yi, std::integral_constant<int, 0>{}, Yes{});
        if (D > 1) step(yi + 1, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, Yes{});
        if (D > 2) step(yi + 2, std::integral_constant<int, (D > 2 ? 2 : 0)>{}, Yes{});
        if (D > 3) step(yi + 3, std::integral_constant<int, (D > 3 ? 3 : 0)>{}, Yes{});
        yi += D;
        row_march_sync(group);
    }
    for (; yi <= yi1; ++yi) {
        step_any(yi, d);
        d = d + 1 == D ? 0 : d + 1;
    }
}

template <class T, int PX, int D, int WAVES, bool UPREV>
__global__ __launch_bounds__(64 * WAVES) void adj_wave2d_kernel(Wave2dArgs a)
{
    constexpr int W = 64 * PX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int xs = (blockIdx.x * WAVES + wave) * W;
    const int ys = blockIdx.y * a.ychunk;
    const int ye = min(ys + a.ychunk, a.ny);
    const RowMarch rm = adj2d_rows<D>(ys, ye, a.ny);
    if (xs >= a.nx) {                           // wave-uniform: a strip outside the grid
        row_march_idle(rm);
        return;
    }
    const bool core = xs >= 2 && xs + W <= a.nx - 2 && ys >= 2 && ye <= a.ny - 2;
    if (core) adj2d_strip<T, PX, D, false, UPREV>(a, xs, ys, ye, lane, rm);
    else      adj2d_strip<T, PX, D, true, UPREV>(a, xs, ys, ye, lane, rm);
}

// ------------------------------------------------------------------------- primal
// r = 2u - u_prev + c*(u[x-1]+u[x+1]+u[y-1]+u[y+1]-4u) on I (paper Section 4.1 in two
// dimensions).  Same march applied to u, with the same D-row load pipeline; u of the
// completing row is the previous step's row and is kept in registers.  c, u_prev and r
// are streamed.  Only cells of I are stored; reads of u never leave the grid.
// GUARD = false: strips whose columns all lie in I (and hence in the grid): no lane is
// masked anywhere in the march.  GUARD = true: the first and the last strip of a row.
template <int D>
__device__ __forceinline__ RowMarch primal2d_rows(int ys, int ye)
{
    return plan_row_march(ys - 1, ye, ys + 1, ye - D, D);   // steady: rows yi-1 >= ys and yi+D <= ye
}

template <class T, int PX, int D, bool GUARD>
__device__ __forceinline__ void primal2d_strip(const Wave2dArgs &a, int xs, int ys, int ye, int lane, const RowMarch rm)
{
    constexpr int W = 64 * PX;
    using V = Vec<T, PX>;
    const int nx = a.nx;
    const T *__restrict__ ug = static_cast<const T *>(a.u);
    const T *__restrict__ pg = static_cast<const T *>(a.u_prev);
    const T *__restrict__ cg = static_cast<const T *>(a.c);
    T *__restrict__ rg = static_cast<T *>(a.r);

    const int x = xs + lane * PX;
    const bool active = GUARD ? (x < nx) : true;
    const int xc = active ? x : xs;
    bool xin[PX], all_in = true;
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        xin[e] = GUARD ? (x + e >= 1 && x + e <= nx - 2) : true;
        all_in = all_in && xin[e];
    }
    const int hx = lane < 32 ? xs - 1 : xs + W;
    const int hxc = (!GUARD || (hx >= 0 && hx < nx)) ? hx : xs;
    const bool edge_lane = lane == 0 || lane == 63;

    T acc[PX][3], uq[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) { acc[e][0] = acc[e][1] = acc[e][2] = T(0); uq[e] = T(0); }
    V su[D], scc[D], spp[D];
    T sh[D];
#pragma unroll
    for (int d = 0; d < D; ++d) { su[d] = V{}; scc[d] = V{}; spp[d] = V{}; sh[d] = T(0); }

    const int yi0 = ys - 1, yi1 = ye;                     // all inside the grid
    auto issue = [&](int y, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        if (!STEADY && y > yi1) return;
        const T *up = ug + (size_t)y * nx;
        su[d] = ld_vec_stream<T, PX>(up + xc);
        if (edge_lane) sh[d] = up[hxc];                    // only lanes 0 and 63 use the value
        const int yo = y - 1;
        if (STEADY || yo >= ys) {
            scc[d] = ld_vec_stream<T, PX>(cg + (size_t)yo * nx + xc);
            spp[d] = ld_vec_stream<T, PX>(pg + (size_t)yo * nx + xc);
        }
    };
    auto step = [&](int yi, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        const int yo = yi - 1;
        T u0[PX];
#pragma unroll
        for (int e = 0; e < PX; ++e) u0[e] = su[d].v[e];
        const T uh = sh[d];
        const V cc = scc[d], pp = spp[d];
        issue(yi + D, dc, steady);
        T left, right;
        wave_neighbours<T, PX>(u0, uh, lane, left, right);
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            const T l = e == 0 ? left : u0[e - 1];
            const T r = e == PX - 1 ? right : u0[e + 1];
            acc[e][1] += T(-4) * u0[e] + (l + r);
            acc[e][0] += u0[e];
            acc[e][2] += u0[e];
        }
        if ((STEADY || yo >= ys) && active) {
            V o;
#pragma unroll
            for (int e = 0; e < PX; ++e) o.v[e] = T(2) * uq[e] - pp.v[e] + cc.v[e] * acc[e][0];
            T *rp = rg + (size_t)yo * nx + x;
            if (!GUARD || all_in) {
                st_vec_stream<T, PX>(rp, o);
            } else {                                       // r outside I stays untouched
#pragma unroll
                for (int e = 0; e < PX; ++e)
                    if (xin[e]) rp[e] = o.v[e];
            }
        }
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            acc[e][0] = acc[e][1];
            acc[e][1] = acc[e][2];
            acc[e][2] = T(0);
            uq[e] = u0[e];
        }
    };
    using No = std::integral_constant<bool, false>;
    using Yes = std::integral_constant<bool, true>;
    auto step_any = [&](int yi, int d) {
        if (D == 1 || d == 0) step(yi, std::integral_constant<int, 0>{}, No{});
        else step(yi, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, No{});
    };
    static_assert(D <= 2, "primal_wave2d_kernel: D is 1 or 2");
    issue(yi0, std::integral_constant<int, 0>{}, No{});
    if (D > 1) issue(yi0 + 1, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, No{});
    int yi = yi0, d = 0;
    for (; yi < rm.pre_end; ++yi) {
        step_any(yi, d);
        d = d + 1 == D ? 0 : d + 1;
    }
    for (int group = 1; group <= rm.steady; ++group) {
        step(yi, std::integral_constant<int, 0>{}, Yes{});
        if (D > 1) step(yi + 1, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, Yes{});
        yi += D;
        row_march_sync(group);
    }
    for (; yi <= yi1; ++yi) {
        step_any(yi, d);
        d = d + 1 == D ? 0 : d + 1;
    }
}

template <class T, int PX, int D, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void primal_wave2d_kernel(Wave2dArgs a)
{
    constexpr int W = 64 * PX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int xs = (blockIdx.x * WAVES + wave) * W;
    const int ys = 1 + blockIdx.y * a.ychunk;             // output rows cover [1, ny-1)
    const int ye = min(ys + a.ychunk, a.ny - 1);
    const RowMarch rm = primal2d_rows<D>(ys, ye);
    if (xs >= a.nx) {                                     // wave-uniform: a strip outside the grid
        row_march_idle(rm);
        return;
    }
    if (xs >= 1 && xs + W <= a.nx - 1) primal2d_strip<T, PX, D, false>(a, xs, ys, ye, lane, rm);
    else                               primal2d_strip<T, PX, D, true>(a, xs, ys, ye, lane, rm);
}


// ------------------------------------------------------------ tile form of the adjoint
// One workgroup per tile of TX x TY outputs, no march: q on the tile and the ring around it is
// staged in LDS once, and the loads of one workgroup overlap the arithmetic of the others that
// share its compute unit (small tiles, several workgroups per CU).  Every tile re-reads a ring of
// c and r_bar (found in L2 where the neighbour runs on the same XCD).  Measured a few points
// slower than the strip march where that is at its best and a little faster where it is not
// (see launch_adj2d).
template <class T, int PX, int TY, bool GUARD, bool UPREV>
__device__ __forceinline__ void adj2d_tile(const Wave2dArgs &a, int tix, int tiy, T *__restrict__ sq)
{
    using G = Tile3d<T, 1, 32, TY, 1, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, LX = G::LX, HS = G::HS;
    const int tid = threadIdx.x, tx = tid % 32, ty = tid / 32;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ cg = static_cast<const T *>(a.c);
    const T *__restrict__ rg = static_cast<const T *>(a.r_bar);
    T *__restrict__ ug = static_cast<T *>(a.u_bar);
    T *__restrict__ pg = static_cast<T *>(a.u_prev_bar);

    TileAddr<PX, 1, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, a.nx, a.ny, 1, 1, LX, 0 /* a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
    bool any = false;
#pragma unroll
    for (int e = 0; e < PX; ++e) any = any || ad.own_I[0][e];
    const uint32_t ooff = ad.own_off[0], coff = (!GUARD || any) ? ooff : ad.dummy;
    const V vc = ld_vec_off<T, PX, false>(cg, coff), vr = ld_vec_off<T, PX, false>(rg, coff);
    T hc[HS], hr[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const uint32_t off = ad.halo_I[s] ? ad.halo_off[s] : ad.dummy;
        hc[s] = ld_off(cg, off);
        hr[s] = ld_off(rg, off);
    }
    const V vu = ld_vec_off<T, PX, true>(ug, ooff);
    V vp{};
    if (UPREV) vp = ld_vec_off<T, PX, true>(pg, ooff);
    T q[PX], rm[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const bool in = ad.own_I[0][e];
        rm[e] = GUARD ? (in ? vr.v[e] : T(0)) : vr.v[e];
        q[e] = GUARD ? (in ? vc.v[e] * vr.v[e] : T(0)) : vc.v[e] * vr.v[e];
        sq[(1 + ty) * LX + 1 + tx * PX + e] = q[e];
    }
#pragma unroll
    for (int s = 0; s < HS; ++s) sq[ad.halo_lds[s]] = GUARD ? (ad.halo_I[s] ? hc[s] * hr[s] : T(0)) : hc[s] * hr[s];
    __syncthreads();
    V o, op;
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T *at = sq + (1 + ty) * LX + 1 + tx * PX + e;
        const T left = e > 0 ? q[e - 1] : at[-1], right = e < PX - 1 ? q[e + 1] : at[1];
        const T s = T(2.0 * star_w<1>(0)) * q[e] + T(star_w<1>(1)) * (left + right) + T(star_w<1>(1)) * (at[-LX] + at[LX]);
        o.v[e] = vu.v[e] + (s + T(2) * rm[e]);
        op.v[e] = vp.v[e] - rm[e];
    }
    if (!GUARD || ad.own_grid[0]) {
        st_vec_off<T, PX, true>(ug, ooff, o);
        if (UPREV) st_vec_off<T, PX, true>(pg, ooff, op);
    }
}

template <class T, int PX, int TY, bool UPREV>
__global__ __launch_bounds__(32 * TY) void adj_wave2d_tile_kernel(Wave2dArgs a, int ntx, int total)
{
    using G = Tile3d<T, 1, 32, TY, 1, PX>;
    __shared__ T sq[G::PLANE];
    const int L = xcd_contiguous_id(blockIdx.x, total);
    const int tiy = L / ntx, tix = L - tiy * ntx;
    const int x0 = tix * G::TX, y0 = tiy * TY;
    const bool core = x0 >= 2 && x0 + G::TX + 2 <= a.nx && y0 >= 2 && y0 + TY + 2 <= a.ny;
    if (core) adj2d_tile<T, PX, TY, false, UPREV>(a, tix, tiy, sq);
    else      adj2d_tile<T, PX, TY, true, UPREV>(a, tix, tiy, sq);
}

template <class T, int PX, int TY>
static hipError_t launch_adj2d_tile(const Wave2dArgs &a, hipStream_t stream)
{
    constexpr int TX = 32 * PX;
    const long ntx = (a.nx + TX - 1) / TX, nty = (a.ny + TY - 1) / TY;
    if (ntx * nty > 0x3fffffffL) return hipErrorNotSupported;
    const int total = (int)(ntx * nty);
    dim3 grid(total), block(32 * TY);
    if (a.u_prev_bar) hipLaunchKernelGGL((adj_wave2d_tile_kernel<T, PX, TY, true>), grid, block, 0, stream, a, (int)ntx, total);
    else              hipLaunchKernelGGL((adj_wave2d_tile_kernel<T, PX, TY, false>), grid, block, 0, stream, a, (int)ntx, total);
    return hipGetLastError();
}


// Tile form of the primal: u on the tile and its ring staged in LDS, one workgroup per tile.
template <class T, int PX, int TY, bool GUARD>
__device__ __forceinline__ void primal2d_tile(const Wave2dArgs &a, int tix, int tiy, T *__restrict__ sq)
{
    using G = Tile3d<T, 1, 32, TY, 1, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, LX = G::LX, HS = G::HS;
    const int tid = threadIdx.x, tx = tid % 32, ty = tid / 32;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ ug = static_cast<const T *>(a.u);
    const T *__restrict__ pg = static_cast<const T *>(a.u_prev);
    const T *__restrict__ cg = static_cast<const T *>(a.c);
    T *__restrict__ rg = static_cast<T *>(a.r);

    TileAddr<PX, 1, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, a.nx, a.ny, 1, 1, LX, 0 /* a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
    bool any = false, all = true;
#pragma unroll
    for (int e = 0; e < PX; ++e) { any = any || ad.own_I[0][e]; all = all && ad.own_I[0][e]; }
    const uint32_t ooff = ad.own_off[0], coff = (!GUARD || any) ? ooff : ad.dummy;
    const V vu = ld_vec_off<T, PX, false>(ug, ooff);       // u is read on the whole grid
    T hu[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) hu[s] = ld_off(ug, ad.halo_off[s]);
    const V vc = ld_vec_off<T, PX, true>(cg, coff), vp = ld_vec_off<T, PX, true>(pg, coff);
#pragma unroll
    for (int e = 0; e < PX; ++e) sq[(1 + ty) * LX + 1 + tx * PX + e] = vu.v[e];
#pragma unroll
    for (int s = 0; s < HS; ++s) sq[ad.halo_lds[s]] = hu[s];
    __syncthreads();
    if (GUARD && !any) return;
    V o;
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T *at = sq + (1 + ty) * LX + 1 + tx * PX + e;
        const T left = e > 0 ? vu.v[e - 1] : at[-1], right = e < PX - 1 ? vu.v[e + 1] : at[1];
        const T lap = T(2.0 * star_w<1>(0)) * vu.v[e] + T(star_w<1>(1)) * (left + right) + T(star_w<1>(1)) * (at[-LX] + at[LX]);
        o.v[e] = T(2) * vu.v[e] - vp.v[e] + vc.v[e] * lap;
    }
    if (!GUARD || all) {
        st_vec_off<T, PX, true>(rg, ooff, o);
    } else {                                               // r outside I stays untouched
        T *rp = reinterpret_cast<T *>(reinterpret_cast<char *>(rg) + ooff);
#pragma unroll
        for (int e = 0; e < PX; ++e)
            if (ad.own_I[0][e]) rp[e] = o.v[e];
    }
}

template <class T, int PX, int TY>
__global__ __launch_bounds__(32 * TY) void primal_wave2d_tile_kernel(Wave2dArgs a, int ntx, int total)
{
    using G = Tile3d<T, 1, 32, TY, 1, PX>;
    __shared__ T sq[G::PLANE];
    const int L = xcd_contiguous_id(blockIdx.x, total);
    const int tiy = L / ntx, tix = L - tiy * ntx;
    const int x0 = tix * G::TX, y0 = tiy * TY;
    const bool core = x0 >= 1 && x0 + G::TX + 1 <= a.nx && y0 >= 1 && y0 + TY + 1 <= a.ny;
    if (core) primal2d_tile<T, PX, TY, false>(a, tix, tiy, sq);
    else      primal2d_tile<T, PX, TY, true>(a, tix, tiy, sq);
}

template <class T, int PX, int TY>
static hipError_t launch_pri2d_tile(const Wave2dArgs &a, hipStream_t stream)
{
    constexpr int TX = 32 * PX;
    const long ntx = (a.nx + TX - 1) / TX, nty = (a.ny + TY - 1) / TY;
    if (ntx * nty > 0x3fffffffL) return hipErrorNotSupported;
    const int total = (int)(ntx * nty);
    hipLaunchKernelGGL((primal_wave2d_tile_kernel<T, PX, TY>), dim3(total), dim3(32 * TY), 0, stream, a, (int)ntx, total);
    return hipGetLastError();
}

// ------------------------------------------------------------------------ launchers
static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

static inline int auto_ychunk(int bx, int rows, long opt_ychunk)
{
    int ychunk = (int)opt_ychunk;
    if (ychunk <= 0) {
        // one workgroup per CU and never more workgroups than CUs: few waves, each with D rows
        // in flight, marching long columns, so that the set of rows being streamed at any moment
        // stays small.  (Rounding the number of chunks up instead left a few workgroups for a
        // second round that ran almost alone: 9000^2 measured 47 % of peak instead of 64 %.)
        int dev = 0, ncu = 256, v = 0;
        if (hipGetDevice(&dev) == hipSuccess &&
            hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
            ncu = v;
        const int chunks = bx >= ncu ? 1 : ncu / bx;
        ychunk = (rows + chunks - 1) / chunks;
        if (ychunk < 16) ychunk = 16;
    }
    if (ychunk > rows) ychunk = rows;
    return ychunk;
}

template <class T, int PX, int D, int WAVES>
static hipError_t launch_adj2d_cfg(Wave2dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    constexpr int W = 64 * PX;
    const int nstrips = (a.nx + W - 1) / W;
    const int bx = (nstrips + WAVES - 1) / WAVES;
    const int ychunk = auto_ychunk(bx, a.ny, opt.ychunk2d);
    a.ychunk = ychunk;
    if ((a.ny + ychunk - 1) / ychunk > 65535) return hipErrorNotSupported;     // a user-set "wave2d.ychunk" too small for ny
    dim3 grid(bx, (a.ny + ychunk - 1) / ychunk), block(64 * WAVES);
    if (a.u_prev_bar) hipLaunchKernelGGL((adj_wave2d_kernel<T, PX, D, WAVES, true>), grid, block, 0, stream, a);
    else              hipLaunchKernelGGL((adj_wave2d_kernel<T, PX, D, WAVES, false>), grid, block, 0, stream, a);
    return hipGetLastError();
}

// "wave2d.variant": 0 (automatic) the tile form with 8 rows per tile; 1 the strip march (two rows
// of loads in flight per wave, eight waves per workgroup; "wave2d.ychunk" applies); 2 the tile
// form with 16 rows per tile.  Measured fp64 adjoint, % of 8 TB/s, strip march / tiles of 8 rows:
// 8192^2 72.5 / 76, 9000^2 65 / 72, 10000^2 65 / 73, 7000^2 64.5 / 70-73, 6144^2 61 / 73,
// 8192 x 9216 66.5 / 73-76, 2048^2 65 / 72, 9001^2 (one cell per lane) 62 / 65; primal the same
// picture (8192^2 72.8 / 73.4, 7000^2 63.6 / 75.4); tiles of 16 rows within 2 points of 8 rows,
// tiles of 4 and of 32 rows 1-3 points lower.  Other strip-march shapes that were tried (one or
// four rows in flight, four or sixteen waves per workgroup) were never better than the one kept.
template <class T, int PX>
static hipError_t launch_adj2d(const Wave2dArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    switch (opt.variant2d) {
    default:
    case 0: return launch_adj2d_tile<T, PX, 8>(a, stream);
    case 1: return launch_adj2d_cfg<T, PX, 2, 8>(a, opt, stream);
    case 2: return launch_adj2d_tile<T, PX, 16>(a, stream);
    }
}

template <class T, int PX>
static hipError_t launch_pri2d(const Wave2dArgs &a0, const LaunchOptions &opt, hipStream_t stream)
{
    if (opt.variant2d == 2) return launch_pri2d_tile<T, PX, 16>(a0, stream);
    if (opt.variant2d != 1) return launch_pri2d_tile<T, PX, 8>(a0, stream);
    constexpr int WAVES = 8, D = 2;
    Wave2dArgs a = a0;
    constexpr int W = 64 * PX;
    const int nstrips = (a.nx + W - 1) / W;
    const int bx = (nstrips + WAVES - 1) / WAVES;
    const int rows = a.ny - 2;
    a.ychunk = auto_ychunk(bx, rows, opt.ychunk2d);
    if ((rows + a.ychunk - 1) / a.ychunk > 65535) return hipErrorNotSupported;
    dim3 grid(bx, (rows + a.ychunk - 1) / a.ychunk), block(64 * WAVES);
    hipLaunchKernelGGL((primal_wave2d_kernel<T, PX, D, WAVES>), grid, block, 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_adjoint_wave2d(int is_f64, int nx, int ny, const void *c, const void *r_bar,
                                 void *u_bar, void *u_prev_bar, const LaunchOptions &opt, hipStream_t stream)
{
    Wave2dArgs a{};
    a.c = c; a.r_bar = r_bar; a.u_bar = u_bar; a.u_prev_bar = u_prev_bar;
    a.nx = nx; a.ny = ny;
    const bool al = aligned16(c) && aligned16(r_bar) && aligned16(u_bar) && aligned16(u_prev_bar);
    if (is_f64) {
        if (al && nx % 2 == 0) return launch_adj2d<double, 2>(a, opt, stream);
        return launch_adj2d<double, 1>(a, opt, stream);
    }
    if (al && nx % 4 == 0) return launch_adj2d<float, 4>(a, opt, stream);
    return launch_adj2d<float, 1>(a, opt, stream);
}

hipError_t launch_primal_wave2d(int is_f64, int nx, int ny, const void *u, const void *u_prev,
                                const void *c, void *r, const LaunchOptions &opt, hipStream_t stream)
{
    Wave2dArgs a{};
    a.u = u; a.u_prev = u_prev; a.c = c; a.r = r;
    a.nx = nx; a.ny = ny;
    const bool al = aligned16(u) && aligned16(u_prev) && aligned16(c) && aligned16(r);
    if (is_f64) {
        if (al && nx % 2 == 0) return launch_pri2d<double, 2>(a, opt, stream);
        return launch_pri2d<double, 1>(a, opt, stream);
    }
    if (al && nx % 4 == 0) return launch_pri2d<float, 4>(a, opt, stream);
    return launch_pri2d<float, 1>(a, opt, stream);
}

}  // namespace sadj
