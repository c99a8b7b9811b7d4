// 3-D linear wave stencil of radius R: primal kernel.
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

struct Wave3dArgs {
    const void *u, *u_prev, *c;
    void *r;
    int nx, ny, nz;
    int zchunk;
    int total_blocks;
    int remap;                 // 1: XCD-contiguous logical ids
    Region reg[1];
};

template <class T, int R, int BX, int BY, int PY>
struct Tile3d {
    static constexpr int TX = BX, TY = BY * PY, NT = BX * BY;
    static constexpr int LX = TX + 2 * R, LY = TY + 2 * R;
    static constexpr int NH = 2 * R * TX + 2 * R * TY;     // halo cells without corners
    static constexpr int HS = (NH + NT - 1) / NT;          // halo slots per thread
    static constexpr int LDS_ELEMS = 2 * LY * LX;
};

static inline int cdiv(int a, int b) { return (a + b - 1) / b; }

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
    a.zchunk = zchunk;
    a.remap = 1;
    Region &rg = a.reg[0];
    rg.box = Box{0, a.nx, 0, a.ny, R, a.nz - R};
    rg.ntx = cdiv(a.nx, G::TX);
    rg.nty = cdiv(a.ny, G::TY);
    rg.ntz = cdiv(a.nz - 2 * R, zchunk);
    rg.first_block = 0;
    a.total_blocks = rg.ntx * rg.nty * rg.ntz;
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


}  // namespace sadj
