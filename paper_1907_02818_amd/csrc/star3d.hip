// 3-D star stencils of radius R with arbitrary (asymmetric) weights: primal and gather-form
// adjoint.
//
//   primal   r[i]      = c[i] * ( w_0 u[i] + sum_{d in x,y,z} sum_{o=-R..R, o!=0} w_{d,o} u[i + o e_d] )   i in I
//   adjoint  u_bar[j] += w_0 q[j] + sum_d sum_o w_{d,o} q[j - o e_d],   q = c*r_bar on I, 0 elsewhere
//
// This is the general linear stencil of the paper's method restricted to a star (Sections
// 3.2-3.3: one derivative expression per read offset, shifted by -o so that all of them
// write u_bar[j]); with asymmetric weights -- upwind-biased differences, for instance -- the
// shift shows as mirrored weights, w_{d,o} multiplying the value at j - o e_d, exactly what
// the worked 1-D example with weights (2,-3,4) displays.  The launcher mirrors the table on
// the host, so both directions are the same gather  out[j] <- sum_o W[o] S[j+o]  over a
// staged field S (u for the primal, q for the adjoint) and share the kernel body.
//
// Mapping: the z-march of the wave kernels (a workgroup owns a 64 x 32 x-y tile, the arriving
// plane of S is staged in LDS with a halo of width R without corners, 2R+1 running sums per
// owned cell in registers), with the weights as kernel arguments.
#include "launch.hpp"
#include "tile3d.hpp"

namespace sadj {

struct StarArgs {
    const void *in0, *in1;      // adjoint: c, r_bar          primal: u, c
    void *out;                  // adjoint: u_bar (accumulated)   primal: r (assigned on I)
    int nx, ny, nz;
    TileMap map;                // workgroup id -> tile and planes
    double w0;                  // centre weight
    double w[3][8];             // gather weights W[d][idx], idx: offsets -R..-1 -> 0..R-1, +1..+R -> R..2R-1
};

template <class T, int R, int BX, int BY, int PY, int PX, bool ADJ, bool GUARD>
__device__ __forceinline__ void star3d_march(const StarArgs &a, int tix, int tiy, int zs, int ze, T *__restrict__ sq)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, TY = G::TY, LX = G::LX, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;
    const T *__restrict__ g0 = static_cast<const T *>(a.in0);
    const T *__restrict__ g1 = static_cast<const T *>(a.in1);
    T *__restrict__ og = static_cast<T *>(a.out);
    const T w0 = (T)a.w0;
    T wx[2 * R], wy[2 * R], wz[2 * R];
#pragma unroll
    for (int i = 0; i < 2 * R; ++i) { wx[i] = (T)a.w[0][i]; wy[i] = (T)a.w[1][i]; wz[i] = (T)a.w[2][i]; }
    // owned cells x = x0 + tx*PX + e, y = y0 + ty*PY + p and halo slots (tile3d.hpp).  ouse: cell in I
    // (x,y); ostore: cell receives output; the primal reads u wherever it lies in the grid (outside it
    // reads as 0, never used by cells of I), the adjoint uses c and r_bar on I only
    TileAddr<PX, PY, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, nx, ny, R, R, LX, 0 /* cell (0,0) is a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
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

    T acc[PY][PX][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e)
#pragma unroll
            for (int k = 0; k < NACC; ++k) acc[p][e][k] = T(0);
    V n0[PY], n1[PY], nout[PY];
    T nh0[HS], nh1[HS];
#pragma unroll
    for (int p = 0; p < PY; ++p) { n0[p] = V{}; n1[p] = V{}; nout[p] = V{}; }
#pragma unroll
    for (int s = 0; s < HS; ++s) nh0[s] = nh1[s] = T(0);

    // planes of S that exist: adjoint: planes of I (q is zero elsewhere); primal: all planes
    auto plane_used = [&](int z) { return ADJ ? (z >= R && z < nz - R) : (z >= 0 && z < nz); };
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
    // what the completing output plane is combined with: adjoint: u_bar, primal: c
    auto load_out = [&](int zo) {
        const T *po = (ADJ ? static_cast<const T *>(og) : g1) + (size_t)zo * plane;
#pragma unroll
        for (int p = 0; p < PY; ++p) nout[p] = ld_vec_off<T, PX, true>(po, ooff[p]);
    };
    const int zi0 = zs - R, zi1 = ze - 1 + R;       // source planes that reach outputs [zs, ze)
    if (plane_used(zi0)) load_plane(zi0);
    int buf = 0;
    for (int zi = zi0; zi <= zi1; ++zi) {
        const bool zin = plane_used(zi);
        const int zo = zi - R;
        T *sb = sq + buf * G::PLANE;
        T own[PY][PX];
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    if (ADJ) own[p][e] = ouse[p][e] ? n0[p].v[e] * n1[p].v[e] : T(0);
                    else     own[p][e] = n0[p].v[e];
                    sb[(R + ty * PY + p) * LX + R + tx * PX + e] = own[p][e];
                }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                T v;
                if (ADJ) v = huse[s] ? nh0[s] * nh1[s] : T(0);
                else     v = huse[s] ? nh0[s] : T(0);
                sb[hlds[s]] = v;
            }
        }
        V cur_out[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) cur_out[p] = nout[p];
        if (zi + 1 <= zi1) {
            if (plane_used(zi + 1)) load_plane(zi + 1);
            if (zo + 1 >= zs) load_out(zo + 1);     // zo+1 <= ze-1 because zi+1 <= zi1
        }
        if (zin) {
            __syncthreads();
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T *row = sb + (R + ty * PY + p) * LX + R + tx * PX + e;
                    T s = w0 * own[p][e];
#pragma unroll
                    for (int k = 1; k <= R; ++k) s += wx[R - k] * row[-k] + wx[R + k - 1] * row[k];
#pragma unroll
                    for (int k = 1; k <= R; ++k) s += wy[R - k] * row[-k * LX] + wy[R + k - 1] * row[k * LX];
                    acc[p][e][R] += s;
                    // S(zi) sits at offset o = zi - z' of output plane z' = zi - o: running sum R - o
#pragma unroll
                    for (int k = 1; k <= R; ++k) {
                        acc[p][e][R - k] += wz[R + k - 1] * own[p][e];     // o = +k
                        acc[p][e][R + k] += wz[R - k] * own[p][e];         // o = -k
                    }
                }
            buf ^= 1;
        }
        if (zo >= zs && (ADJ || (zo >= R && zo < nz - R))) {
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
#pragma unroll
                for (int k = 0; k < NACC - 1; ++k) acc[p][e][k] = acc[p][e][k + 1];
                acc[p][e][NACC - 1] = T(0);
            }
    }
}

template <class T, int R, int BX, int BY, int PY, int PX, bool ADJ>
__global__ __launch_bounds__(BX *BY) void star3d_kernel(StarArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    __shared__ T sq[2 * G::PLANE];
    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);
    const int x0 = tix * G::TX, y0 = tiy * G::TY;
    // core tile: own cells and halo cells all inside I in x and y
    const bool core = x0 >= 2 * R && x0 + G::TX + 2 * R <= a.nx && y0 >= 2 * R && y0 + G::TY + 2 * R <= a.ny;
    if (core) star3d_march<T, R, BX, BY, PY, PX, ADJ, false>(a, tix, tiy, zs, ze, sq);
    else      star3d_march<T, R, BX, BY, PY, PX, ADJ, true>(a, tix, tiy, zs, ze, sq);
}

template <class T, int R, bool ADJ, int BX, int BY, int PY, int PX>
static hipError_t launch_star_shape(StarArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, R, opt);
    const unsigned pad = one_workgroup_per_cu_pad(sizeof(T) * 2 * G::PLANE, opt.lds_pad);
    hipLaunchKernelGGL((star3d_kernel<T, R, BX, BY, PY, PX, ADJ>), dim3(a.map.total_blocks), dim3(G::NT), pad, stream, a);
    return hipGetLastError();
}

static inline bool star_aligned(const void *p, size_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

// 16 bytes per lane (two doubles / four floats), 32 x 16 threads, two rows per thread, as the
// wave kernels; needs nx to be a multiple of the vector length and vector-aligned arrays,
// otherwise 64 x 8 threads with one cell per lane and four rows.  One workgroup per CU (a
// 64 x 16 tile with two workgroups per CU measured 4-11 points slower for the radius-3 and -4
// primal at 512^3).
template <class T, int R, bool ADJ>
static hipError_t launch_star_TR(const StarArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    constexpr int PXV = 16 / sizeof(T);
    const bool ok = a.nx % PXV == 0 && star_aligned(a.in0, 16) && star_aligned(a.in1, 16) && star_aligned(a.out, 16);
    // the primal measured 2-6 points faster with the one-cell shape for radius 1 and 2, and for
    // radius 3 in fp32 (512^3: 63 vs 58 %); 10-12 points slower for radius 4 and radius 3 fp64
    const bool wide = ADJ || R == 4 || (R == 3 && sizeof(T) == 8);
    // rows that are not cache-line multiples: tiles of 16 rows with long rows, as the wave kernels
    // (wide_tile_for_unaligned_rows): radius 1 256 cells, two per lane, four rows per thread;
    // larger radii 1 KB, 16 bytes per lane, two rows per thread
    if (opt.variant == 0) {
        const int wide_tx = wide_tile_for_unaligned_rows(a.nx, sizeof(T), R, false);
        if constexpr (R == 1) {
            const bool ok2 = a.nx % 2 == 0 && star_aligned(a.in0, 2 * sizeof(T)) && star_aligned(a.in1, 2 * sizeof(T)) &&
                             star_aligned(a.out, 2 * sizeof(T));
            if (ok2 && wide_tx == 256) return launch_star_shape<T, R, ADJ, 128, 4, 4, 2>(a, opt, stream);
        } else {
            if (ok && wide_tx) return launch_star_shape<T, R, ADJ, 64, 8, 2, PXV>(a, opt, stream);
        }
    }
    if (ok && wide && opt.variant != 3) return launch_star_shape<T, R, ADJ, 32, 16, 2, PXV>(a, opt, stream);
    return launch_star_shape<T, R, ADJ, 64, 8, 4, 1>(a, opt, stream);
}

template <class T, bool ADJ>
static hipError_t launch_star_T(int radius, const StarArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    switch (radius) {
    case 1: return launch_star_TR<T, 1, ADJ>(a, opt, stream);
    case 2: return launch_star_TR<T, 2, ADJ>(a, opt, stream);
    case 3: return launch_star_TR<T, 3, ADJ>(a, opt, stream);
    default: return launch_star_TR<T, 4, ADJ>(a, opt, stream);
    }
}

// w0, w[d][idx]: the GATHER table (already mirrored by the caller for the adjoint);
// idx enumerates the offsets -R..-1, +1..+R of axis d (x, y, z).
hipError_t launch_star3d(int adjoint, int is_f64, int radius, int nx, int ny, int nz, double w0,
                         const double (*w)[8], const void *in0, const void *in1, void *out,
                         const LaunchOptions &opt, hipStream_t stream)
{
    StarArgs a{};
    a.in0 = in0; a.in1 = in1; a.out = out;
    a.nx = nx; a.ny = ny; a.nz = nz;
    a.w0 = w0;
    for (int d = 0; d < 3; ++d)
        for (int i = 0; i < 8; ++i) a.w[d][i] = i < 2 * radius ? w[d][i] : 0.0;
    if (adjoint) return is_f64 ? launch_star_T<double, true>(radius, a, opt, stream) : launch_star_T<float, true>(radius, a, opt, stream);
    return is_f64 ? launch_star_T<double, false>(radius, a, opt, stream) : launch_star_T<float, false>(radius, a, opt, stream);
}

}  // namespace sadj
