// 3-D linear wave stencil of radius R: primal and gather-form adjoint kernels.
//
// Adjoint (paper Section 4.1, gather listing; Sections 3.3.2-3.3.4 for shifting,
// core and remainder):  with q[i] = c[i]*r_bar[i] for i in I and q[i] = 0 elsewhere,
//     u_bar[j] += 2 r_bar[j] [j in I] + sum_o w_o q[j-o]
// which is the same star applied to q, because the weights are symmetric.  The
// product c*r_bar is formed once per staged element instead of once per term.
//
// Mapping to CDNA4.  A workgroup owns an x-y tile of TX x TY outputs and marches
// along z.  Each arriving plane of q is staged in LDS (tile + halo of width R, no
// corners: a star never reads them) and contributes
//   - its in-plane star to the accumulator of the same output plane,
//   - w_k * q(x,y) to the accumulators of the output planes z-k and z+k,
// so a thread keeps 2R+1 running sums per owned point in registers and LDS holds
// only the plane that has just arrived (two buffers, one barrier per plane).  An
// output plane is complete R steps after its own plane arrived; u_bar is then
// read-modify-written once.  Global loads of plane z+1 are issued before the LDS
// phase of plane z.  x is the unit-stride direction of memory and of the lanes.
//
// Regions.  The unguarded instantiation (GUARD=false) runs on whole tiles whose
// reads all lie in I: every staged element is loaded unconditionally.  The guarded
// instantiation (GUARD=true) serves the remainder slabs: an element is used iff it
// lies in I (and is needed by the slab); unused elements are replaced by zero with
// a select, never by a multiplication, so NaN outside I cannot leak.  This is the
// if-guarded remainder variant of Section 3.3.4; because the guards are per-thread
// constants in x,y and wave-uniform in z, they cost a few selects per plane.
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

struct Wave3dArgs {
    const void *c, *r_bar;
    void *u_bar, *u_prev_bar;
    const void *u, *u_prev;    // primal only
    void *r;                   // primal only
    int nx, ny, nz;
    int zchunk;
    int nregions;
    int unguarded_regions;     // the first `unguarded_regions` regions need no guards
    int total_blocks;
    int remap;                 // 1: XCD-contiguous logical ids
    Region reg[kMaxRegions];
};

template <class T, int R, int BX, int BY, int PY>
struct Tile3d {
    static constexpr int TX = BX, TY = BY * PY, NT = BX * BY;
    static constexpr int LX = TX + 2 * R, LY = TY + 2 * R;
    static constexpr int NH = 2 * R * TX + 2 * R * TY;     // halo cells without corners
    static constexpr int HS = (NH + NT - 1) / NT;          // halo slots per thread
    static constexpr int LDS_ELEMS = 2 * LY * LX;
};

// ------------------------------------------------------------------------ adjoint
template <class T, int R, int BX, int BY, int PY, bool GUARD, bool UPREV>
__device__ __forceinline__ void adj3d_tile(const Wave3dArgs &a, const Box &bx, int tix, int tiy,
                                           int tiz, T *__restrict__ sq)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    constexpr int TX = G::TX, TY = G::TY, NT = G::NT, LX = G::LX, LY = G::LY, NH = G::NH, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = bx.x0 + tix * TX, y0 = bx.y0 + tiy * TY;
    const int zs = bx.z0 + tiz * a.zchunk;
    const int ze = min(zs + a.zchunk, bx.z1);

    const T *__restrict__ cg = static_cast<const T *>(a.c);
    const T *__restrict__ rg = static_cast<const T *>(a.r_bar);
    T *__restrict__ ug = static_cast<T *>(a.u_bar);
    T *__restrict__ upg = static_cast<T *>(a.u_prev_bar);

    // A cell that is always inside the grid: unused slots load it and discard it.
    const uint32_t dummy = (uint32_t)((size_t)y0 * nx + x0) * sizeof(T);

    // ---- owned points: x = x0+tx, y = y0 + ty*PY + p
    uint32_t ooff[PY];
    bool ouse[PY], ostore[PY];
    const int x = x0 + tx;
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        const int y = y0 + ty * PY + p;
        if (GUARD) {
            ouse[p] = x >= R && x < nx - R && y >= R && y < ny - R && x < bx.x1 + R && y < bx.y1 + R;
            ostore[p] = x < bx.x1 && y < bx.y1;
        } else {
            ouse[p] = true;
            ostore[p] = true;
        }
        ooff[p] = (ouse[p] || ostore[p]) ? (uint32_t)((size_t)y * nx + x) * sizeof(T) : dummy;
    }
    // ---- halo slots
    uint32_t hoff[HS];
    int hlds[HS];
    bool huse[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const int h = tid + s * NT;
        int lx, ly;
        if (h < 2 * R * TX) {
            const int row = h / TX;
            lx = R + h % TX;
            ly = row < R ? row : row + TY;
        } else {
            const int h2 = h - 2 * R * TX;
            const int k = h2 % (2 * R);
            lx = k < R ? k : k + TX;
            ly = R + h2 / (2 * R);
        }
        const int gx = x0 - R + lx, gy = y0 - R + ly;
        bool use = h < NH;
        if (GUARD)
            use = use && gx >= R && gx < nx - R && gy >= R && gy < ny - R && gx < bx.x1 + R && gy < bx.y1 + R;
        huse[s] = use;
        hoff[s] = use ? (uint32_t)((size_t)gy * nx + gx) * sizeof(T) : dummy;
        hlds[s] = h < NH ? ly * LX + lx : 0;      // cell (0,0) is a corner nobody reads
    }

    T acc[PY][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int k = 0; k < NACC; ++k) acc[p][k] = T(0);

    T nc[PY], nr[PY], nhc[HS], nhr[HS], nu[PY], nup[PY];
#pragma unroll
    for (int p = 0; p < PY; ++p) { nc[p] = nr[p] = nu[p] = nup[p] = T(0); }
#pragma unroll
    for (int s = 0; s < HS; ++s) { nhc[s] = nhr[s] = T(0); }

    const int zi0 = zs - R, zi1 = ze - 1 + R;
    auto plane_in_I = [&](int z) { return GUARD ? (z >= R && z < nz - R) : true; };
    auto load_plane = [&](int z) {
        const T *cp = cg + (size_t)z * plane;
        const T *rp = rg + (size_t)z * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) { nc[p] = ld_off(cp, ooff[p]); nr[p] = ld_off(rp, ooff[p]); }
#pragma unroll
        for (int s = 0; s < HS; ++s) { nhc[s] = ld_off(cp, hoff[s]); nhr[s] = ld_off(rp, hoff[s]); }
        if (UPREV) {
            if (z >= zs && z < ze) {
                const T *pp = upg + (size_t)z * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) nup[p] = ld_off(pp, ooff[p]);
            }
        }
    };
    if (plane_in_I(zi0)) load_plane(zi0);

    int buf = 0;
    for (int zi = zi0; zi <= zi1; ++zi) {
        const bool zin = plane_in_I(zi);
        const int zo = zi - R;
        T *sb = sq + buf * (LY * LX);
        T qo[PY], ro[PY];
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                const T rr = GUARD ? (ouse[p] ? nr[p] : T(0)) : nr[p];
                const T qq = GUARD ? (ouse[p] ? nc[p] * nr[p] : T(0)) : nc[p] * nr[p];
                ro[p] = rr;
                qo[p] = qq;
                sb[(R + ty * PY + p) * LX + R + tx] = qq;
            }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                const T qq = GUARD ? (huse[s] ? nhc[s] * nhr[s] : T(0)) : nhc[s] * nhr[s];
                sb[hlds[s]] = qq;
            }
            if (UPREV) {
                if (zi >= zs && zi < ze) {
                    T *pp = upg + (size_t)zi * plane;
#pragma unroll
                    for (int p = 0; p < PY; ++p)
                        if (!GUARD || (ouse[p] && ostore[p])) st_off(pp, ooff[p], nup[p] - ro[p]);
                }
            }
        }
        // u_bar of the plane that completes in this step was fetched one step ago
        T cu[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) cu[p] = nu[p];
        // issue the global loads of the next step before the LDS phase of this one
        if (zi + 1 <= zi1 && plane_in_I(zi + 1)) load_plane(zi + 1);
        if (zo + 1 >= zs) {        // zo+1 <= ze-1 whenever zi+1 <= zi1
            if (zi + 1 <= zi1) {
                const T *up = ug + (size_t)(zo + 1) * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) nu[p] = ld_off(up, ooff[p]);
            }
        }
        if (zin) {
            __syncthreads();
            T col[PY + 2 * R];
#pragma unroll
            for (int i = 0; i < PY + 2 * R; ++i) col[i] = sb[(ty * PY + i) * LX + R + tx];
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                const T *row = sb + (R + ty * PY + p) * LX + R + tx;
                T s = T(3.0 * star_w<R>(0)) * qo[p];
#pragma unroll
                for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (row[-k] + row[k]);
#pragma unroll
                for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (col[R + p - k] + col[R + p + k]);
                acc[p][R] += s + T(2) * ro[p];
#pragma unroll
                for (int k = 1; k <= R; ++k) {
                    acc[p][R - k] += T(star_w<R>(k)) * qo[p];
                    acc[p][R + k] += T(star_w<R>(k)) * qo[p];
                }
            }
            buf ^= 1;
        }
        if (zo >= zs) {
            T *up = ug + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p)
                if (!GUARD || ostore[p]) st_off(up, ooff[p], cu[p] + acc[p][0]);
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
__global__ __launch_bounds__(BX *BY) void adj_wave3d_kernel(Wave3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    __shared__ T sq[G::LDS_ELEMS];
    const int L = a.remap ? xcd_contiguous_id(blockIdx.x, a.total_blocks) : (int)blockIdx.x;
    int ri = 0;
    while (ri + 1 < a.nregions && L >= a.reg[ri + 1].first_block) ++ri;
    const Region rg = a.reg[ri];
    const int l = L - rg.first_block;
    const int tix = l % rg.ntx;
    const int t = l / rg.ntx;
    const int tiy = t % rg.nty;
    const int tiz = t / rg.nty;
    if (ri < a.unguarded_regions)
        adj3d_tile<T, R, BX, BY, PY, false, UPREV>(a, rg.box, tix, tiy, tiz, sq);
    else
        adj3d_tile<T, R, BX, BY, PY, true, UPREV>(a, rg.box, tix, tiy, tiz, sq);
}

// Guarded-only and unguarded-only entry points for the one-dispatch-per-region mode
// (so that a profiler shows the core and the remainder kernels separately).
template <class T, int R, int BX, int BY, int PY, bool UPREV>
__global__ __launch_bounds__(BX *BY) void adj_wave3d_core_kernel(Wave3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    __shared__ T sq[G::LDS_ELEMS];
    const int L = a.remap ? xcd_contiguous_id(blockIdx.x, a.total_blocks) : (int)blockIdx.x;
    const Region rg = a.reg[0];
    const int tix = L % rg.ntx;
    const int t = L / rg.ntx;
    adj3d_tile<T, R, BX, BY, PY, false, UPREV>(a, rg.box, tix, t % rg.nty, t / rg.nty, sq);
}
template <class T, int R, int BX, int BY, int PY, bool UPREV>
__global__ __launch_bounds__(BX *BY) void adj_wave3d_remainder_kernel(Wave3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    __shared__ T sq[G::LDS_ELEMS];
    const int L = a.remap ? xcd_contiguous_id(blockIdx.x, a.total_blocks) : (int)blockIdx.x;
    const Region rg = a.reg[0];
    const int tix = L % rg.ntx;
    const int t = L / rg.ntx;
    adj3d_tile<T, R, BX, BY, PY, true, UPREV>(a, rg.box, tix, t % rg.nty, t / rg.nty, sq);
}

// --------------------------------------------------------------- region construction
static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

static void add_region(Wave3dArgs &a, Box b, int TX, int TY, int zchunk)
{
    if (b.x1 <= b.x0 || b.y1 <= b.y0 || b.z1 <= b.z0) return;
    Region &r = a.reg[a.nregions++];
    r.box = b;
    r.ntx = cdiv(b.x1 - b.x0, TX);
    r.nty = cdiv(b.y1 - b.y0, TY);
    r.ntz = cdiv(b.z1 - b.z0, zchunk);
    r.first_block = a.total_blocks;
    a.total_blocks += r.ntx * r.nty * r.ntz;
}

// Core region = the largest box of whole tiles (anchored at multiples of TX, TY)
// inside K = prod [2R, n-2R); remainder = up to six slabs covering the rest.
static void build_regions(Wave3dArgs &a, int R, int TX, int TY, int zchunk)
{
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    a.nregions = 0;
    a.total_blocks = 0;
    a.unguarded_regions = 0;
    a.zchunk = zchunk;
    int cx0 = cdiv(2 * R, TX) * TX, cx1 = ((nx - 2 * R) / TX) * TX;
    int cy0 = cdiv(2 * R, TY) * TY, cy1 = ((ny - 2 * R) / TY) * TY;
    int cz0 = 2 * R, cz1 = nz - 2 * R;
    const bool has_core = cx1 > cx0 && cy1 > cy0 && cz1 > cz0;
    if (!has_core) {
        add_region(a, Box{0, nx, 0, ny, 0, nz}, TX, TY, zchunk);
        return;
    }
    add_region(a, Box{cx0, cx1, cy0, cy1, cz0, cz1}, TX, TY, zchunk);
    a.unguarded_regions = 1;
    add_region(a, Box{0, nx, 0, ny, 0, cz0}, TX, TY, zchunk);           // z-low slab
    add_region(a, Box{0, nx, 0, ny, cz1, nz}, TX, TY, zchunk);          // z-high slab
    add_region(a, Box{0, nx, 0, cy0, cz0, cz1}, TX, TY, zchunk);        // y-low slab
    add_region(a, Box{0, nx, cy1, ny, cz0, cz1}, TX, TY, zchunk);       // y-high slab
    add_region(a, Box{0, cx0, cy0, cy1, cz0, cz1}, TX, TY, zchunk);     // x-low slab
    add_region(a, Box{cx1, nx, cy0, cy1, cz0, cz1}, TX, TY, zchunk);    // x-high slab
}

template <class T, int R, int BX, int BY, int PY>
static hipError_t launch_adjoint_cfg(Wave3dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    int zchunk = opt.zchunk > 0 ? (int)opt.zchunk : 64;
    build_regions(a, R, G::TX, G::TY, zchunk);
    a.remap = 1;
    const bool uprev = a.u_prev_bar != nullptr;
    if (opt.fused) {
        if (uprev)
            hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, true>), dim3(a.total_blocks), dim3(G::NT), 0, stream, a);
        else
            hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, false>), dim3(a.total_blocks), dim3(G::NT), 0, stream, a);
        return hipGetLastError();
    }
    // one dispatch per region: regions are disjoint, so any order is valid
    for (int i = 0; i < a.nregions; ++i) {
        Wave3dArgs b = a;
        b.nregions = 1;
        b.reg[0] = a.reg[i];
        b.reg[0].first_block = 0;
        b.total_blocks = a.reg[i].ntx * a.reg[i].nty * a.reg[i].ntz;
        const bool core = i < a.unguarded_regions;
        dim3 grid(b.total_blocks), block(G::NT);
        if (core) {
            if (uprev) hipLaunchKernelGGL((adj_wave3d_core_kernel<T, R, BX, BY, PY, true>), grid, block, 0, stream, b);
            else       hipLaunchKernelGGL((adj_wave3d_core_kernel<T, R, BX, BY, PY, false>), grid, block, 0, stream, b);
        } else {
            if (uprev) hipLaunchKernelGGL((adj_wave3d_remainder_kernel<T, R, BX, BY, PY, true>), grid, block, 0, stream, b);
            else       hipLaunchKernelGGL((adj_wave3d_remainder_kernel<T, R, BX, BY, PY, false>), grid, block, 0, stream, b);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

template <class T, int R>
static hipError_t launch_adjoint_T(const Wave3dArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    switch (opt.variant) {
    default:
    case 0: return launch_adjoint_cfg<T, R, 64, 4, 4>(a, opt, stream);
    case 1: return launch_adjoint_cfg<T, R, 64, 8, 2>(a, opt, stream);
    case 2: return launch_adjoint_cfg<T, R, 64, 4, 2>(a, opt, stream);
    case 3: return launch_adjoint_cfg<T, R, 32, 8, 4>(a, opt, stream);
    }
}

// ------------------------------------------------------------------------- primal
// r[i] = 2u[i] - u_prev[i] + c[i]*Lap_w(u)[i] on I (paper Section 4.1, primal
// listing).  Same marching scheme as the adjoint, applied to u itself: a plane of u
// is staged in LDS, its in-plane star and its z contributions are added to 2R+1
// running sums per owned point; when a plane completes, c and u_prev of that plane
// are combined with the sum and with u of that plane, which is kept in a register
// queue of depth R+1.  Tiles are anchored at 0 and outputs are masked to I; reads
// of u never leave the grid for outputs in I, so only the tile halo needs clamping.
template <class T, int R, int BX, int BY, int PY>
__global__ __launch_bounds__(BX *BY) void primal_wave3d_kernel(Wave3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    constexpr int TX = G::TX, TY = G::TY, NT = G::NT, LX = G::LX, LY = G::LY, NH = G::NH, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    __shared__ T sq[G::LDS_ELEMS];
    const int L = a.remap ? xcd_contiguous_id(blockIdx.x, a.total_blocks) : (int)blockIdx.x;
    const Region rgn = a.reg[0];
    const int tix = L % rgn.ntx;
    const int tt = L / rgn.ntx;
    const int tiy = tt % rgn.nty, tiz = tt / rgn.nty;

    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;
    const int zs = rgn.box.z0 + tiz * a.zchunk;
    const int ze = min(zs + a.zchunk, rgn.box.z1);
    const T *__restrict__ ug = static_cast<const T *>(a.u);
    const T *__restrict__ pg = static_cast<const T *>(a.u_prev);
    const T *__restrict__ cg = static_cast<const T *>(a.c);
    T *__restrict__ rg = static_cast<T *>(a.r);
    const uint32_t dummy = (uint32_t)((size_t)y0 * nx + x0) * sizeof(T);

    uint32_t ooff[PY];
    bool ostore[PY];
    const int x = x0 + tx;
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        const int y = y0 + ty * PY + p;
        ostore[p] = x >= R && x < nx - R && y >= R && y < ny - R;
        const bool ingrid = x < nx && y < ny;
        ooff[p] = ingrid ? (uint32_t)((size_t)y * nx + x) * sizeof(T) : dummy;
    }
    uint32_t hoff[HS];
    int hlds[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        const int h = tid + s * NT;
        int lx, ly;
        if (h < 2 * R * TX) {
            const int row = h / TX;
            lx = R + h % TX;
            ly = row < R ? row : row + TY;
        } else {
            const int h2 = h - 2 * R * TX;
            const int k = h2 % (2 * R);
            lx = k < R ? k : k + TX;
            ly = R + h2 / (2 * R);
        }
        const int gx = x0 - R + lx, gy = y0 - R + ly;
        const bool ingrid = h < NH && gx >= 0 && gx < nx && gy >= 0 && gy < ny;
        hoff[s] = ingrid ? (uint32_t)((size_t)gy * nx + gx) * sizeof(T) : dummy;
        hlds[s] = h < NH ? ly * LX + lx : 0;
    }

    T acc[PY][NACC], uq[PY][R + 1];
#pragma unroll
    for (int p = 0; p < PY; ++p) {
#pragma unroll
        for (int k = 0; k < NACC; ++k) acc[p][k] = T(0);
#pragma unroll
        for (int k = 0; k <= R; ++k) uq[p][k] = T(0);
    }
    T nuo[PY], nh[HS], ncc[PY], npp[PY];
#pragma unroll
    for (int p = 0; p < PY; ++p) { nuo[p] = ncc[p] = npp[p] = T(0); }
#pragma unroll
    for (int s = 0; s < HS; ++s) nh[s] = T(0);

    const int zi0 = zs - R, zi1 = ze - 1 + R;      // all inside [0, nz)
    auto load_plane = [&](int z) {
        const T *up = ug + (size_t)z * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) nuo[p] = ld_off(up, ooff[p]);
#pragma unroll
        for (int s = 0; s < HS; ++s) nh[s] = ld_off(up, hoff[s]);
    };
    load_plane(zi0);
    int buf = 0;
    for (int zi = zi0; zi <= zi1; ++zi) {
        const int zo = zi - R;
        T *sb = sq + buf * (LY * LX);
        T uo[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) {
            uo[p] = nuo[p];
            sb[(R + ty * PY + p) * LX + R + tx] = uo[p];
        }
#pragma unroll
        for (int s = 0; s < HS; ++s) sb[hlds[s]] = nh[s];
        T cc[PY], pp[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) { cc[p] = ncc[p]; pp[p] = npp[p]; }
        if (zi + 1 <= zi1) {
            load_plane(zi + 1);
            if (zo + 1 >= zs) {
                const T *cp = cg + (size_t)(zo + 1) * plane;
                const T *qp = pg + (size_t)(zo + 1) * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p) { ncc[p] = ld_off(cp, ooff[p]); npp[p] = ld_off(qp, ooff[p]); }
            }
        }
        __syncthreads();
        T col[PY + 2 * R];
#pragma unroll
        for (int i = 0; i < PY + 2 * R; ++i) col[i] = sb[(ty * PY + i) * LX + R + tx];
#pragma unroll
        for (int p = 0; p < PY; ++p) {
            const T *row = sb + (R + ty * PY + p) * LX + R + tx;
            T s = T(3.0 * star_w<R>(0)) * uo[p];
#pragma unroll
            for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (row[-k] + row[k]);
#pragma unroll
            for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (col[R + p - k] + col[R + p + k]);
            acc[p][R] += s;
#pragma unroll
            for (int k = 1; k <= R; ++k) {
                acc[p][R - k] += T(star_w<R>(k)) * uo[p];
                acc[p][R + k] += T(star_w<R>(k)) * uo[p];
            }
            uq[p][R] = uo[p];
        }
        buf ^= 1;
        if (zo >= zs) {
            T *rp = rg + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p)
                if (ostore[p]) st_off(rp, ooff[p], T(2) * uq[p][0] - pp[p] + cc[p] * acc[p][0]);
        }
#pragma unroll
        for (int p = 0; p < PY; ++p) {
#pragma unroll
            for (int k = 0; k < NACC - 1; ++k) acc[p][k] = acc[p][k + 1];
            acc[p][NACC - 1] = T(0);
#pragma unroll
            for (int k = 0; k < R; ++k) uq[p][k] = uq[p][k + 1];
        }
    }
}

template <class T, int R, int BX, int BY, int PY>
static hipError_t launch_primal_cfg(Wave3dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = Tile3d<T, R, BX, BY, PY>;
    const int zchunk = opt.zchunk > 0 ? (int)opt.zchunk : 64;
    a.nregions = 0;
    a.total_blocks = 0;
    a.unguarded_regions = 0;
    a.zchunk = zchunk;
    a.remap = 1;
    add_region(a, Box{0, a.nx, 0, a.ny, R, a.nz - R}, G::TX, G::TY, zchunk);
    hipLaunchKernelGGL((primal_wave3d_kernel<T, R, BX, BY, PY>), dim3(a.total_blocks), dim3(G::NT), 0, stream, a);
    return hipGetLastError();
}

hipError_t launch_primal_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *u,
                                const void *u_prev, const void *c, void *r, const LaunchOptions &opt,
                                hipStream_t stream)
{
    Wave3dArgs a{};
    a.u = u; a.u_prev = u_prev; a.c = c; a.r = r;
    a.nx = nx; a.ny = ny; a.nz = nz;
    if (is_f64) {
        if (radius == 1) return launch_primal_cfg<double, 1, 64, 4, 4>(a, opt, stream);
        return launch_primal_cfg<double, 4, 64, 4, 4>(a, opt, stream);
    }
    if (radius == 1) return launch_primal_cfg<float, 1, 64, 4, 4>(a, opt, stream);
    return launch_primal_cfg<float, 4, 64, 4, 4>(a, opt, stream);
}


hipError_t launch_adjoint_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                 const void *r_bar, void *u_bar, void *u_prev_bar,
                                 const LaunchOptions &opt, hipStream_t stream)
{
    Wave3dArgs a{};
    a.c = c; a.r_bar = r_bar; a.u_bar = u_bar; a.u_prev_bar = u_prev_bar;
    a.nx = nx; a.ny = ny; a.nz = nz;
    if (is_f64) {
        if (radius == 1) return launch_adjoint_T<double, 1>(a, opt, stream);
        return launch_adjoint_T<double, 4>(a, opt, stream);
    }
    if (radius == 1) return launch_adjoint_T<float, 1>(a, opt, stream);
    return launch_adjoint_T<float, 4>(a, opt, stream);
}

}  // namespace sadj
