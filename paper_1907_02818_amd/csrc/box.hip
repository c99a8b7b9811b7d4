// Dense 3^d box stencils with arbitrary (asymmetric) weights: primal and gather-form
// adjoint in 2-D and 3-D (the 1-D case lives with the other wave-per-segment kernels).
//
//   primal   r[i]      = c[i] * sum_{o in {-1,0,1}^d} w[o] u[i+o]                 for i in I
//   adjoint  u_bar[j] += sum_o w[o] * c[j-o] r_bar[j-o]  [j-o in I]               for all j
//
// These are the dense stencils for which paper Section 3.3.4 counts 5 / 25 / 125 adjoint
// loop nests; the 1-D instance with weights (2,-3,4) is the worked example of Section
// 3.2.  Index shifting (Section 3.3.2) turns the scatter into a gather over the
// point-mirrored weight table: u_bar[j] += sum_o' w[-o'] q[j+o'] with q = c*r_bar masked
// to I.  The launcher mirrors the table on the host, so primal and adjoint are the same
// gather  out[j] <- sum_o W[o] S[j+o]  over a staged field S (u, or q), and share one
// kernel body per dimension:
//   2-D: one workgroup per small tile, S on the tile and its ring staged in LDS once (default);
//        or (option "wave2d.variant" 1) a wave owns a strip of columns and marches down y, an
//        arriving row of S feeding three running sums, x-neighbours by wave shuffles.
//   3-D: a workgroup owns an x-y tile and marches along z; an arriving plane of S is
//        staged in LDS with a full halo ring (a box reads the corners) and feeds three
//        running sums per owned cell.
// Cells whose reads all lie in I take the unguarded instantiation; the others the
// guarded one (selects, never multiplications by zero).
#include "launch.hpp"
#include "tile3d.hpp"

#include <type_traits>

namespace sadj {

struct BoxArgs {
    const void *in0, *in1;      // adjoint: c, r_bar          primal: u, c
    void *out;                  // adjoint: u_bar (accumulated)   primal: r (assigned on I)
    int nx, ny, nz;
    int chunk;                  // 2-D: output rows per march
    TileMap map;                // 3-D: workgroup id -> tile and planes
    double w[27];               // gather weights W[(ox+1) + 3(oy+1) + 9(oz+1)]
};

// ------------------------------------------------------------------------------ 2-D
// D rows of loads in flight per wave; the steady part of the march has no branches so
// that the wait counters know which loads may still be outstanding.
template <int D>
__device__ __forceinline__ RowMarch box2d_rows(int ys, int ye, int ny)
{
    // steady steps yi in [lo, hi]: rows yi and yi+D exist and lie in I; output rows yi-1 and
    // yi+D-1 belong to this chunk and (primal) to I
    return plan_row_march(ys - 1, ye, max(ys + 1, 2), min(ny - 1, ye) - 1 - D, D);
}

template <class T, int PX, int D, bool ADJ, bool GUARD>
__device__ __forceinline__ void box2d_strip(const BoxArgs &a, int xs, int ys, int ye, int lane, const RowMarch rm)
{
    constexpr int W = 64 * PX;
    using V = Vec<T, PX>;
    const int nx = a.nx, ny = a.ny;
    const T *__restrict__ g0 = static_cast<const T *>(a.in0);
    const T *__restrict__ g1 = static_cast<const T *>(a.in1);
    T *__restrict__ og = static_cast<T *>(a.out);
    T wt[3][3];                                     // wt[oy+1][ox+1]
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < 3; ++i) wt[j][i] = (T)a.w[i + 3 * j + 9];

    const int x = xs + lane * PX;
    const bool active = x < nx;
    const int xc = active ? x : xs;
    bool xin[PX], all_in = true;
#pragma unroll
    for (int e = 0; e < PX; ++e) { xin[e] = x + e >= 1 && x + e <= nx - 2; all_in = all_in && xin[e]; }
    const int hx = lane < 32 ? xs - 1 : xs + W;
    const bool hgrid = hx >= 0 && hx < nx;
    const bool hin = hx >= 1 && hx <= nx - 2;
    const int hxc = hgrid ? hx : xs;
    const bool edge_lane = lane == 0 || lane == 63;

    T acc[PX][3];
#pragma unroll
    for (int e = 0; e < PX; ++e) acc[e][0] = acc[e][1] = acc[e][2] = T(0);
    V s0[D], s1[D], so[D];
    T sh0[D], sh1[D];
#pragma unroll
    for (int d = 0; d < D; ++d) { s0[d] = V{}; s1[d] = V{}; so[d] = V{}; sh0[d] = sh1[d] = T(0); }

    // rows of S that exist: adjoint: rows of I (q is zero elsewhere); primal: all grid rows
    auto row_used = [&](int y) { return ADJ ? (y >= 1 && y <= ny - 2) : (y >= 0 && y < ny); };
    const int yi0 = ys - 1, yi1 = ye;

    // everything step y consumes: row y of the staged field, and for output row y-1 the
    // array it is combined with (adjoint: u_bar, primal: c)
    auto issue = [&](int y, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        if (!STEADY && y > yi1) return;
        if (STEADY || row_used(y)) {
            // adjoint: c and r_bar through L2 (streaming either measured 2 points slower);
            // primal: u streamed (3 points faster)
            s0[d] = ADJ ? ld_vec<T, PX>(g0 + (size_t)y * nx + xc) : ld_vec_stream<T, PX>(g0 + (size_t)y * nx + xc);
            if (ADJ) s1[d] = ld_vec<T, PX>(g1 + (size_t)y * nx + xc);
            if (edge_lane) {                        // only lanes 0 and 63 use the values
                sh0[d] = g0[(size_t)y * nx + hxc];
                if (ADJ) sh1[d] = g1[(size_t)y * nx + hxc];
            }
        }
        const int yo = y - 1;
        if (STEADY || yo >= ys)
            so[d] = ADJ ? ld_vec_stream<T, PX>(og + (size_t)yo * nx + xc) : ld_vec_stream<T, PX>(g1 + (size_t)yo * nx + xc);
    };
    auto step = [&](int yi, auto dc, auto steady) {
        constexpr int d = decltype(dc)::value;
        constexpr bool STEADY = decltype(steady)::value;
        const bool rin = STEADY || row_used(yi);
        const int yo = yi - 1;
        const V cur_out = so[d];
        if (rin) {
            T s[PX], sh;
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                if (ADJ) s[e] = (!GUARD || xin[e]) ? s0[d].v[e] * s1[d].v[e] : T(0);
                else     s[e] = s0[d].v[e];
            }
            if (ADJ) sh = (!GUARD || hin) ? sh0[d] * sh1[d] : T(0);
            else     sh = sh0[d];
            T left, right;
            wave_neighbours<T, PX>(s, sh, lane, left, right);
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                const T l = e == 0 ? left : s[e - 1];
                const T r = e == PX - 1 ? right : s[e + 1];
                // S row yi sits at offset oy = yi - yo of output row yo: k = 0: yo = yi-1 (oy=+1),
                // k = 1: yo = yi, k = 2: yo = yi+1 (oy=-1)
#pragma unroll
                for (int k = 0; k < 3; ++k)
                    acc[e][k] += (wt[2 - k][0] * l + wt[2 - k][1] * s[e]) + wt[2 - k][2] * r;
            }
        }
        issue(yi + D, dc, steady);
        if ((STEADY || yo >= ys) && (!GUARD || active)) {
            V o;
            if (ADJ) {
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = cur_out.v[e] + acc[e][0];
                st_vec_stream<T, PX>(og + (size_t)yo * nx + x, o);
            } else if (STEADY || (yo >= 1 && yo <= ny - 2)) {
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = cur_out.v[e] * acc[e][0];
                T *rp = og + (size_t)yo * nx + x;
                if (all_in) {
                    st_vec_stream<T, PX>(rp, o);
                } else {                              // r outside I stays untouched
#pragma unroll
                    for (int e = 0; e < PX; ++e)
                        if (xin[e]) rp[e] = o.v[e];
                }
            }
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
    static_assert(D <= 2, "box2d_strip: D is 1 or 2");
    auto step_any = [&](int yi, int d) {
        if (D == 1 || d == 0) step(yi, std::integral_constant<int, 0>{}, No{});
        else step(yi, std::integral_constant<int, (D > 1 ? 1 : 0)>{}, No{});
    };
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

template <class T, int PX, bool ADJ, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void box2d_kernel(BoxArgs a)
{
    constexpr int W = 64 * PX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int xs = (blockIdx.x * WAVES + wave) * W;
    const int ys = blockIdx.y * a.chunk;
    const int ye = min(ys + a.chunk, a.ny);
    const RowMarch rm = box2d_rows<2>(ys, ye, a.ny);
    if (xs >= a.nx) {                               // wave-uniform: a strip outside the grid
        row_march_idle(rm);
        return;
    }
    const bool core = xs >= 2 && xs + W <= a.nx - 2 && ys >= 2 && ye <= a.ny - 2;
    if (core) box2d_strip<T, PX, 2, ADJ, false>(a, xs, ys, ye, lane, rm);
    else      box2d_strip<T, PX, 2, ADJ, true>(a, xs, ys, ye, lane, rm);
}

// ------------------------------------------------------------------------------ 3-D
template <class T, int BX, int BY, int PY, int PX>
struct BoxTile {
    static constexpr int TX = BX * PX, TY = BY * PY, NT = BX * BY;
    static constexpr int LX = TX + 2, LY = TY + 2, PLANE = LX * LY;
    static constexpr int NH = PLANE - TX * TY;          // full ring, corners included
    static constexpr int HS = (NH + NT - 1) / NT;
    // ring cell h -> LDS coordinates: row 0, row LY-1, then the two side columns
    __device__ static __forceinline__ bool halo_cell(int h, int &lx, int &ly)
    {
        if (h < LX) { lx = h; ly = 0; }
        else if (h < 2 * LX) { lx = h - LX; ly = LY - 1; }
        else { const int h2 = h - 2 * LX; lx = (h2 & 1) ? LX - 1 : 0; ly = 1 + (h2 >> 1); }
        return h < NH;
    }
};

// Tile form of the 2-D kernels (the default; see wave2d.hip for the measurements that made it
// so): one workgroup per tile of TX x TY outputs, no march.  The staged field S (u, or q) on the
// tile and the full ring around it goes to LDS once; a thread owns PX cells of one row.
template <class T, int PX, int TY, bool ADJ, bool GUARD>
__device__ __forceinline__ void box2d_tile(const BoxArgs &a, int tix, int tiy, T *__restrict__ sq)
{
    using G = BoxTile<T, 32, TY, 1, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, LX = G::LX, HS = G::HS;
    const int tid = threadIdx.x, tx = tid % 32, ty = tid / 32;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ g0 = static_cast<const T *>(a.in0);
    const T *__restrict__ g1 = static_cast<const T *>(a.in1);
    T *__restrict__ og = static_cast<T *>(a.out);
    T wt[3][3];                                     // wt[oy+1][ox+1]
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int i = 0; i < 3; ++i) wt[j][i] = (T)a.w[i + 3 * j + 9];

    TileAddr<PX, 1, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, a.nx, a.ny, 1, 1, LX, -1, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid + s * G::NT, lx, ly); });
    bool any = false, all = true;
#pragma unroll
    for (int e = 0; e < PX; ++e) { any = any || ad.own_I[0][e]; all = all && ad.own_I[0][e]; }
    const uint32_t ooff = ad.own_off[0];
    // adjoint: c and r_bar are used on I only; primal: u is read on the whole grid, c on I
    const uint32_t ioff = (!GUARD || any) ? ooff : ad.dummy;
    const V v0 = ld_vec_off<T, PX, false>(g0, ADJ ? ioff : ooff);
    const V v1 = ld_vec_off<T, PX, !ADJ>(g1, ioff);
    T h0[HS], h1[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const bool use = ADJ ? ad.halo_I[s] : ad.halo_grid[s];
        const uint32_t off = use ? ad.halo_off[s] : ad.dummy;
        h0[s] = ld_off(g0, off);
        h1[s] = ADJ ? ld_off(g1, off) : T(0);
    }
    V vo{};
    if (ADJ) vo = ld_vec_off<T, PX, true>(og, ooff);
    T sv[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        if (ADJ) sv[e] = (!GUARD || ad.own_I[0][e]) ? v0.v[e] * v1.v[e] : T(0);
        else     sv[e] = v0.v[e];
        sq[(1 + ty) * LX + 1 + tx * PX + e] = sv[e];
    }
#pragma unroll
    for (int s = 0; s < HS; ++s)
        if (ad.halo_lds[s] >= 0) sq[ad.halo_lds[s]] = ADJ ? ((!GUARD || ad.halo_I[s]) ? h0[s] * h1[s] : T(0)) : h0[s];
    __syncthreads();
    if (!ADJ && GUARD && !any) return;
    V o;
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T *at = sq + (1 + ty) * LX + 1 + tx * PX + e;
        T s = T(0);
#pragma unroll
        for (int j = 0; j < 3; ++j)
#pragma unroll
            for (int i = 0; i < 3; ++i) s += wt[j][i] * at[(j - 1) * LX + (i - 1)];
        o.v[e] = ADJ ? vo.v[e] + s : v1.v[e] * s;
    }
    if (ADJ) {
        if (!GUARD || ad.own_grid[0]) st_vec_off<T, PX, true>(og, ooff, o);
    } else if (!GUARD || all) {
        st_vec_off<T, PX, true>(og, ooff, o);
    } else {                                               // r outside I stays untouched
        T *rp = reinterpret_cast<T *>(reinterpret_cast<char *>(og) + ooff);
#pragma unroll
        for (int e = 0; e < PX; ++e)
            if (ad.own_I[0][e]) rp[e] = o.v[e];
    }
}

template <class T, int PX, int TY, bool ADJ>
__global__ __launch_bounds__(32 * TY) void box2d_tile_kernel(BoxArgs a, int ntx, int total)
{
    using G = BoxTile<T, 32, TY, 1, PX>;
    __shared__ T sq[G::PLANE];
    const int L = xcd_contiguous_id(blockIdx.x, total);
    const int tiy = L / ntx, tix = L - tiy * ntx;
    const int x0 = tix * G::TX, y0 = tiy * TY;
    const bool core = x0 >= 2 && x0 + G::TX + 2 <= a.nx && y0 >= 2 && y0 + TY + 2 <= a.ny;
    if (core) box2d_tile<T, PX, TY, ADJ, false>(a, tix, tiy, sq);
    else      box2d_tile<T, PX, TY, ADJ, true>(a, tix, tiy, sq);
}

template <class T, int PX, bool ADJ>
static hipError_t launch_box2d_tile(const BoxArgs &a, hipStream_t stream)
{
    constexpr int TY = 8, TX = 32 * PX;
    const long ntx = cdiv_i(a.nx, TX), nty = cdiv_i(a.ny, TY);
    if (ntx * nty > 0x3fffffffL) return hipErrorNotSupported;
    const int total = (int)(ntx * nty);
    hipLaunchKernelGGL((box2d_tile_kernel<T, PX, TY, ADJ>), dim3(total), dim3(32 * TY), 0, stream, a, (int)ntx, total);
    return hipGetLastError();
}

// A thread owns PX consecutive cells in x (one 16-byte memory instruction where PX > 1; nx is
// then a multiple of PX, so a vector lies entirely inside or outside the grid) times PY rows.
template <class T, int BX, int BY, int PY, int PX, bool ADJ, bool GUARD>
__device__ __forceinline__ void box3d_march(const BoxArgs &a, int tix, int tiy, int zs, int ze, T *__restrict__ sq)
{
    using G = BoxTile<T, BX, BY, PY, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, TY = G::TY, LX = G::LX, HS = G::HS;
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ g0 = static_cast<const T *>(a.in0);
    const T *__restrict__ g1 = static_cast<const T *>(a.in1);
    T *__restrict__ og = static_cast<T *>(a.out);
    T wt[27];
#pragma unroll
    for (int i = 0; i < 27; ++i) wt[i] = (T)a.w[i];
    // owned cells and halo slots (tile3d.hpp); the halo is the full ring of width 1, corners included.
    // ouse: cell in I (x,y); ostore: cell receives output
    TileAddr<PX, PY, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, nx, ny, 1, 1, LX, -1, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid + s * G::NT, lx, ly); });
    uint32_t ooff[PY];
    bool ouse[PY][PX], ostore[PY][PX], ovec[PY];
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        ovec[p] = true;
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            ouse[p][e] = ad.own_I[p][e];
            ostore[p][e] = ADJ ? ad.own_grid[p] : ouse[p][e];
            ovec[p] = ovec[p] && ostore[p][e];
        }
        ooff[p] = ad.own_off[p];
    }
    uint32_t hoff[HS];
    int hlds[HS];
    bool huse[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        huse[s] = ADJ ? ad.halo_I[s] : ad.halo_grid[s];
        hoff[s] = ad.halo_off[s];
        hlds[s] = ad.halo_lds[s];
    }

    T acc[PY][PX][3];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e) acc[p][e][0] = acc[p][e][1] = acc[p][e][2] = T(0);
    V n0[PY], n1[PY], nout[PY];
    T nh0[HS], nh1[HS];
#pragma unroll
    for (int p = 0; p < PY; ++p) { n0[p] = V{}; n1[p] = V{}; nout[p] = V{}; }
#pragma unroll
    for (int s = 0; s < HS; ++s) nh0[s] = nh1[s] = T(0);

    auto plane_used = [&](int z) { return ADJ ? (z >= 1 && z <= nz - 2) : (z >= 0 && z < nz); };
    auto load_plane = [&](int z) {
        const T *p0 = g0 + (size_t)z * plane;
        const T *p1 = g1 + (size_t)z * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) {
            n0[p] = ld_vec_off<T, PX, false>(p0, ooff[p]);
            if (ADJ) n1[p] = ld_vec_off<T, PX, false>(p1, ooff[p]);
        }
#pragma unroll
        for (int s = 0; s < HS; ++s) { nh0[s] = ld_off(p0, hoff[s]); if (ADJ) nh1[s] = ld_off(p1, hoff[s]); }
    };
    auto load_out = [&](int zo) {
        const T *po = (ADJ ? static_cast<const T *>(og) : g1) + (size_t)zo * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) nout[p] = ld_vec_off<T, PX, true>(po, ooff[p]);
    };
    const int zi0 = zs - 1, zi1 = ze;
    if (plane_used(zi0)) load_plane(zi0);
    int buf = 0;
    for (int zi = zi0; zi <= zi1; ++zi) {
        const bool zin = plane_used(zi);
        const int zo = zi - 1;
        T *sb = sq + buf * G::PLANE;
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    T s;
                    if (ADJ) s = ouse[p][e] ? n0[p].v[e] * n1[p].v[e] : T(0);
                    else     s = n0[p].v[e];
                    sb[(1 + ty * PY + p) * LX + 1 + tx * PX + e] = s;
                }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                T v;
                if (ADJ) v = huse[s] ? nh0[s] * nh1[s] : T(0);
                else     v = huse[s] ? nh0[s] : T(0);
                if (hlds[s] >= 0) sb[hlds[s]] = v;
            }
        }
        V cur_out[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) cur_out[p] = nout[p];
        if (zi + 1 <= zi1) {
            if (plane_used(zi + 1)) load_plane(zi + 1);
            if (zo + 1 >= zs) load_out(zo + 1);
        }
        if (zin) {
            __syncthreads();
            // rows ty*PY .. ty*PY+PY+1 of the LDS plane, PX + 2 columns each
            T win[PY + 2][PX + 2];
#pragma unroll
            for (int i = 0; i < PY + 2; ++i)
#pragma unroll
                for (int j = 0; j < PX + 2; ++j) win[i][j] = sb[(ty * PY + i) * LX + tx * PX + j];
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e)
#pragma unroll
                    for (int k = 0; k < 3; ++k) {   // k = 0: zo = zi-1 (oz=+1), 1: zo = zi, 2: zo = zi+1 (oz=-1)
                        const T *w9 = wt + 9 * (2 - k);
                        T s = T(0);
#pragma unroll
                        for (int oy = 0; oy < 3; ++oy)
#pragma unroll
                            for (int ox = 0; ox < 3; ++ox) s += w9[ox + 3 * oy] * win[p + oy][e + ox];
                        acc[p][e][k] += s;
                    }
            buf ^= 1;
        }
        if (zo >= zs && (ADJ || (zo >= 1 && zo <= nz - 2))) {
            T *po = og + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e)
                    o.v[e] = ADJ ? cur_out[p].v[e] + acc[p][e][0] : cur_out[p].v[e] * acc[p][e][0];
                if (!GUARD || ovec[p]) {
                    st_vec_off<T, PX, true>(po, ooff[p], o);
                } else {                             // a vector that straddles the boundary of I (primal)
#pragma unroll
                    for (int e = 0; e < PX; ++e)
                        if (ostore[p][e]) st_stream<T, true>(po, ooff[p] + e * (uint32_t)sizeof(T), o.v[e]);
                }
            }
        }
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                acc[p][e][0] = acc[p][e][1];
                acc[p][e][1] = acc[p][e][2];
                acc[p][e][2] = T(0);
            }
    }
}

template <class T, int BX, int BY, int PY, int PX, bool ADJ>
__global__ __launch_bounds__(BX *BY) void box3d_kernel(BoxArgs a)
{
    using G = BoxTile<T, BX, BY, PY, PX>;
    __shared__ T sq[2 * G::PLANE];
    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);
    const int x0 = tix * G::TX, y0 = tiy * G::TY;
    const bool core = x0 >= 2 && x0 + G::TX + 2 <= a.nx && y0 >= 2 && y0 + G::TY + 2 <= a.ny;
    if (core) box3d_march<T, BX, BY, PY, PX, ADJ, false>(a, tix, tiy, zs, ze, sq);
    else      box3d_march<T, BX, BY, PY, PX, ADJ, true>(a, tix, tiy, zs, ze, sq);
}

static inline bool box_aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <class T, int PX, bool ADJ>
static hipError_t launch_box2d(BoxArgs a, hipStream_t stream)
{
    constexpr int WAVES = 8, W = 64 * PX;
    const int nstrips = cdiv_i(a.nx, W);
    const int bx = cdiv_i(nstrips, WAVES);
    int dev = 0, ncu = 256, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        ncu = v;
    // one workgroup of 8 waves per CU, each wave with two rows in flight; never more workgroups
    // than CUs (a few left for a second round would run almost alone)
    const int chunks = bx >= ncu ? 1 : ncu / bx;
    int chunk = cdiv_i(a.ny, chunks);
    if (chunk < 16) chunk = 16;
    if (chunk > a.ny) chunk = a.ny;
    a.chunk = chunk;
    dim3 grid(bx, cdiv_i(a.ny, chunk)), block(64 * WAVES);
    hipLaunchKernelGGL((box2d_kernel<T, PX, ADJ, WAVES>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <class T, bool ADJ, int BX, int BY, int PY, int PX>
static hipError_t launch_box3d_shape(BoxArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = BoxTile<T, BX, BY, PY, PX>;
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, 1, opt);
    const unsigned pad = one_workgroup_per_cu_pad(sizeof(T) * 2 * G::PLANE, opt.lds_pad);
    hipLaunchKernelGGL((box3d_kernel<T, BX, BY, PY, PX, ADJ>), dim3(a.map.total_blocks), dim3(G::NT), pad, stream, a);
    return hipGetLastError();
}

// Adjoint: 16 bytes per lane where nx and the alignment allow it (as the wave kernels), else one cell.
template <class T, bool ADJ>
static hipError_t launch_box3d(const BoxArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    constexpr int PXV = 16 / sizeof(T);
    const bool ok = a.nx % PXV == 0 && box_aligned16(a.in0) && box_aligned16(a.in1) && box_aligned16(a.out);
    // rows that are not cache-line multiples: 256 x 16 tiles, as the radius-1 wave kernels
    // (wide_tile_for_unaligned_rows); 128 x 4 threads, two cells per lane, four rows per thread
    const uintptr_t all_ptrs = reinterpret_cast<uintptr_t>(a.in0) | reinterpret_cast<uintptr_t>(a.in1) |
                               reinterpret_cast<uintptr_t>(a.out);
    const bool ok2 = a.nx % 2 == 0 && all_ptrs % (2 * sizeof(T)) == 0;
    if (ok2 && opt.variant == 0 && wide_tile_for_unaligned_rows(a.nx, sizeof(T), 1, false) == 256)
        return launch_box3d_shape<T, ADJ, 128, 4, 4, 2>(a, opt, stream);
    // the primal (24 bytes per cell) measured 2 points faster with the one-cell shape
    if (ok && ADJ && opt.variant != 3) return launch_box3d_shape<T, ADJ, 32, 16, 2, PXV>(a, opt, stream);
    return launch_box3d_shape<T, ADJ, 64, 8, 4, 1>(a, opt, stream);
}

template <bool ADJ>
static hipError_t launch_box_nd(int is_f64, int ndim, const BoxArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    if (ndim == 3) return is_f64 ? launch_box3d<double, ADJ>(a, opt, stream) : launch_box3d<float, ADJ>(a, opt, stream);
    const bool al = box_aligned16(a.in0) && box_aligned16(a.in1) && box_aligned16(a.out);
    if (opt.variant2d == 1) {                       // the strip march
        if (is_f64) return (al && a.nx % 2 == 0) ? launch_box2d<double, 2, ADJ>(a, stream) : launch_box2d<double, 1, ADJ>(a, stream);
        return (al && a.nx % 4 == 0) ? launch_box2d<float, 4, ADJ>(a, stream) : launch_box2d<float, 1, ADJ>(a, stream);
    }
    if (is_f64) return (al && a.nx % 2 == 0) ? launch_box2d_tile<double, 2, ADJ>(a, stream) : launch_box2d_tile<double, 1, ADJ>(a, stream);
    return (al && a.nx % 4 == 0) ? launch_box2d_tile<float, 4, ADJ>(a, stream) : launch_box2d_tile<float, 1, ADJ>(a, stream);
}

// w: 27 gather weights indexed (ox+1) + 3(oy+1) + 9(oz+1) (already mirrored for the adjoint)
hipError_t launch_box(int adjoint, int is_f64, int ndim, int nx, int ny, int nz, const double *w,
                      const void *in0, const void *in1, void *out, const LaunchOptions &opt, hipStream_t stream)
{
    BoxArgs a{};
    a.in0 = in0; a.in1 = in1; a.out = out;
    a.nx = nx; a.ny = ny; a.nz = nz;
    for (int i = 0; i < 27; ++i) a.w[i] = w[i];
    return adjoint ? launch_box_nd<true>(is_f64, ndim, a, opt, stream) : launch_box_nd<false>(is_f64, ndim, a, opt, stream);
}

}  // namespace sadj
