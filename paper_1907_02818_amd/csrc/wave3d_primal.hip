// 3-D linear wave stencil of radius R: primal kernel.
//
//     r[i] = 2 u[i] - u_prev[i] + c[i] * sum_o w_o u[i+o]        for i in I
// (paper Section 4.1, primal listing and generating script; r is assigned on I and
// left untouched elsewhere).
//
// Same march as the adjoint kernel (wave3d_adjoint.hip), applied to u itself: a
// workgroup owns an x-y tile and walks along z; each arriving plane of u is staged in
// LDS with its halo and adds its in-plane star to the running sum of its own output
// plane and w_k*u(x,y) to the sums of planes z-k and z+k (2R+1 running sums per owned
// point, in registers).  When plane z-R completes, c and u_prev of that plane (fetched
// together with plane z of u) and u of that plane are combined with the sum.  u of the
// last R+1 planes is not kept in registers: the LDS ring holds R+2 planes and the
// thread reads its own cell of plane z-R back from it.
//
// u is the only array with reuse (halo cells shared with neighbouring tiles); c,
// u_prev and r are streamed with non-temporal accesses so that they do not displace u
// from L2.  Workgroups are mapped to XCD patches and sized to one resident wave, as
// in the adjoint kernel.  Reads of u never leave the grid for outputs in I, so the only
// guards are address clamps for tiles that stick out of the grid and the store mask.
#include "launch.hpp"
#include "tile3d.hpp"

namespace sadj {

template <class T, int R, int BX, int BY, int PY, int PX, bool NTS>
__global__ __launch_bounds__(BX *BY) void primal_wave3d_kernel(March3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, TY = G::TY, LX = G::LX, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    constexpr int NB = R + 2;                       // LDS ring of planes
    __shared__ T sq[NB * G::PLANE];

    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);

    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ ug = static_cast<const T *>(a.in0);
    const T *__restrict__ pg = static_cast<const T *>(a.in1);
    const T *__restrict__ cg = static_cast<const T *>(a.in2);
    T *__restrict__ rg = static_cast<T *>(a.out0);
    // owned cells x = x0 + tx*PX + e, y = y0 + ty*PY + p and halo slots (tile3d.hpp): r is written on I,
    // u is read wherever it lies in the grid
    TileAddr<PX, PY, HS, true> ad;
    ad.init(tx, ty, x0, y0, nx, ny, R, R, LX, 0 /* cell (0,0) is a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
    uint32_t ooff[PY];
    bool ostore[PY][PX], oall[PY];
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        oall[p] = true;
#pragma unroll
        for (int e = 0; e < PX; ++e) { ostore[p][e] = ad.own_I[p][e]; oall[p] = oall[p] && ostore[p][e]; }
        ooff[p] = ad.own_off[p];
    }
    uint32_t hoff[HS];
    int hlds[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) { hoff[s] = ad.halo_off[s]; hlds[s] = ad.halo_lds[s]; }

    T acc[PY][PX][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e)
#pragma unroll
            for (int k = 0; k < NACC; ++k) acc[p][e][k] = T(0);

    V su[PY], scc[PY], spp[PY];
    T sh[HS];
#pragma unroll
    for (int p = 0; p < PY; ++p) { su[p] = V{}; scc[p] = V{}; spp[p] = V{}; }
#pragma unroll
    for (int s = 0; s < HS; ++s) sh[s] = T(0);

    // output planes of this chunk that lie in I; input planes that reach them
    const int zo0 = max(zs, R), zo1 = min(ze, nz - R) - 1;
    if (zo0 > zo1) return;                          // block-uniform: nothing to do
    const int zi0 = zo0 - R, zi1 = zo1 + R;         // all inside [0, nz)

    auto issue = [&](int z) {
        if (z > zi1) return;
        const T *up = ug + (size_t)z * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) su[p] = ld_vec_off<T, PX, false>(up, ooff[p]);
#pragma unroll
        for (int s = 0; s < HS; ++s) sh[s] = ld_off(up, hoff[s]);
        const int zo = z - R;
        if (zo >= zo0) {
            const T *cp = cg + (size_t)zo * plane;
            const T *pp = pg + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                scc[p] = ld_vec_off<T, PX, NTS>(cp, ooff[p]);
                spp[p] = ld_vec_off<T, PX, NTS>(pp, ooff[p]);
            }
        }
    };

    issue(zi0);
    int buf = 0, bufo = R % NB;                      // ring slots of plane zi and of plane zi-R
    for (int zi = zi0; zi <= zi1; ++zi) {
        const int zo = zi - R;
        T *sb = sq + buf * G::PLANE;
        T uo[PY][PX];
        V cc[PY], pp[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) {
            cc[p] = scc[p];
            pp[p] = spp[p];
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                uo[p][e] = su[p].v[e];
                sb[(R + ty * PY + p) * LX + R + tx * PX + e] = uo[p][e];
            }
        }
#pragma unroll
        for (int s = 0; s < HS; ++s) sb[hlds[s]] = sh[s];
        issue(zi + 1);
        __syncthreads();
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            T col[PY + 2 * R];
#pragma unroll
            for (int i = 0; i < PY + 2 * R; ++i) col[i] = sb[(ty * PY + i) * LX + R + tx * PX + e];
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                const T *row = sb + (R + ty * PY + p) * LX + R + tx * PX + e;
                T s = T(3.0 * star_w<R>(0)) * uo[p][e];
#pragma unroll
                for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (row[-k] + row[k]);
#pragma unroll
                for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (col[R + p - k] + col[R + p + k]);
                acc[p][e][R] += s;
#pragma unroll
                for (int k = 1; k <= R; ++k) {
                    acc[p][e][R - k] += T(star_w<R>(k)) * uo[p][e];
                    acc[p][e][R + k] += T(star_w<R>(k)) * uo[p][e];
                }
            }
        }
        if (zo >= zo0) {
            // own cells of plane zo were written to ring slot `bufo` R steps ago
            const T *so = sq + bufo * G::PLANE;
            T *rp = rg + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T uc = so[(R + ty * PY + p) * LX + R + tx * PX + e];
                    o.v[e] = T(2) * uc - pp[p].v[e] + cc[p].v[e] * acc[p][e][0];
                }
                if (oall[p]) {
                    st_vec_off<T, PX, NTS>(rp, ooff[p], o);
                } else {                              // r outside I stays untouched
#pragma unroll
                    for (int e = 0; e < PX; ++e)
                        if (ostore[p][e]) st_stream<T, NTS>(rp, ooff[p] + e * (uint32_t)sizeof(T), o.v[e]);
                }
            }
            bufo = bufo + 1 == NB ? 0 : bufo + 1;
        }
        buf = buf + 1 == NB ? 0 : buf + 1;
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

static inline bool aligned_to_p(const void *p, size_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

template <class T, int R, int BX, int BY, int PY, int PX>
static hipError_t launch_primal_cfg(March3dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    if constexpr ((R + 2) * G::PLANE * sizeof(T) > 160 * 1024) {
        return launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream);      // ring would not fit the 160 KB LDS
    } else {
    if (PX > 1) {
        const size_t al = PX * sizeof(T);
        const bool ok = a.nx % PX == 0 && aligned_to_p(a.in0, al) && aligned_to_p(a.in1, al) &&
                        aligned_to_p(a.in2, al) && aligned_to_p(a.out0, al);
        if (!ok) return launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream);
    }
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, R, opt);
    const unsigned pad = one_workgroup_per_cu_pad(sizeof(T) * (R + 2) * G::PLANE, opt.lds_pad);
    hipLaunchKernelGGL((primal_wave3d_kernel<T, R, BX, BY, PY, PX, true>), dim3(a.map.total_blocks), dim3(G::NT), pad,
                       stream, a);
    return hipGetLastError();
    }
}

// Same shape numbering as the adjoint kernel (option "wave3d.variant").
template <class T, int R>
static hipError_t launch_primal_T(const March3dArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    long v = opt.variant;
    if (v == 0) {
        v = sizeof(T) == 8 ? 3 : 8;              // measured best per dtype
        const int wide = wide_tile_for_unaligned_rows(a.nx, sizeof(T), R, false);
        if (R == 1 && wide == 256) v = 10;
        else if (R > 1 && wide) v = 5;
    }
    if constexpr (R == 2 || R == 3) {            // the default shapes only
        if constexpr (sizeof(T) == 8) {
            return v == 5 ? launch_primal_cfg<T, R, 64, 8, 2, 2>(a, opt, stream) : launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream);
        } else {
            return v == 3 ? launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream)
                 : v == 5 ? launch_primal_cfg<T, R, 64, 8, 2, 4>(a, opt, stream)
                          : launch_primal_cfg<T, R, 64, 8, 4, 2>(a, opt, stream);
        }
    } else {
        switch (v) {
        default:
        case 1: return launch_primal_cfg<T, R, 32, 16, 2, 2>(a, opt, stream);
        case 2: return launch_primal_cfg<T, R, 32, 16, 2, 4>(a, opt, stream);
        case 3: return launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream);
        case 5:                                  // rows of 1 KB, 16 rows
            if constexpr (sizeof(T) == 8) return launch_primal_cfg<T, R, 64, 8, 2, 2>(a, opt, stream);
            else return launch_primal_cfg<T, R, 64, 8, 2, 4>(a, opt, stream);
        case 8: return launch_primal_cfg<T, R, 64, 8, 4, 2>(a, opt, stream);
        case 10:                                 // radius 1: 256 x 16 tile (see wide_tile_for_unaligned_rows)
            if constexpr (R == 1) return launch_primal_cfg<T, R, 128, 4, 4, 2>(a, opt, stream);
            else return launch_primal_cfg<T, R, 64, 8, 4, 1>(a, opt, stream);
        }
    }
}

hipError_t launch_primal_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *u,
                                const void *u_prev, const void *c, void *r, const LaunchOptions &opt,
                                hipStream_t stream)
{
    March3dArgs a{};
    a.in0 = u; a.in1 = u_prev; a.in2 = c; a.out0 = r;
    a.nx = nx; a.ny = ny; a.nz = nz;
    if (is_f64) {
        switch (radius) {
        case 1: return launch_primal_T<double, 1>(a, opt, stream);
        case 2: return launch_primal_T<double, 2>(a, opt, stream);
        case 3: return launch_primal_T<double, 3>(a, opt, stream);
        default: return launch_primal_T<double, 4>(a, opt, stream);
        }
    }
    switch (radius) {
    case 1: return launch_primal_T<float, 1>(a, opt, stream);
    case 2: return launch_primal_T<float, 2>(a, opt, stream);
    case 3: return launch_primal_T<float, 3>(a, opt, stream);
    default: return launch_primal_T<float, 4>(a, opt, stream);
    }
}

}  // namespace sadj
