// Two reverse steps of a time loop of radius-1 wave steps in one pass over the data.
//
// What is computed.  A solver repeats u^{k+1} = 2 u^k - u^{k-1} + c * Lap(u^k) on I (paper
// Section 4.1; Section 4 notes that such solvers take many steps).  With a = lam^{k+1},
// b = lam^k and m the indicator of I, one reverse step in gather form (Sections 3.3.2-3.3.4) is
//     a' = b + 2 a m + S(q),   q = c a m,        b' = -a m
// where S is the 7-point star with the second-difference weights (symmetric, so the gather
// uses the same table).  Two steps in a row give
//     a'' = -a m + 2 a' m + S(q'),   q' = c a' m,   b'' = -a' m
// and a' itself is never needed in memory.  This kernel reads a, b, c once and writes a'' and
// b'' once: 40 bytes per cell (fp64) for two steps where two single-step launches move 80.
//
// How.  The z-march of the single-step adjoint (wave3d_adjoint.hip) run as a two-stage pipeline.
// Stage 1 stages plane z of q in LDS on the tile plus a frame of width 2 and keeps three running
// sums per cell for a' on the tile AND on the ring of cells around it (a thread owns PX x PY tile
// cells; the first 2 TX + 2 TY threads own one ring cell each).  A plane of a' is complete one
// step after its q plane arrived; b is added, q' = c a' m is formed on tile and ring and staged
// in a second LDS plane, from which stage 2 forms a'' on the tile with three more running sums.
// Both LDS planes are double-buffered and one barrier per step serves both stages: stage 2 works
// one step behind stage 1.  Values outside I are replaced by zero with selects, never by a
// multiplication, so NaN outside I cannot leak (Section 3.3.4: guarded remainder; tiles whose
// frame lies in I in x and y run an unguarded instantiation).
//
// The outputs must be arrays other than a and b: neighbouring workgroups read the frame of a and
// the ring of b while this one writes.
#include "launch.hpp"
#include "tile3d.hpp"

#include <type_traits>

namespace sadj {

struct PairArgs {
    const void *c, *a, *b;
    void *out_a, *out_b;
    int nx, ny, nz;
    TileMap map;
};

template <class T, int BX, int BY, int PY, int PX> struct PairTile {
    static constexpr int TX = BX * PX, TY = BY * PY, NT = BX * BY;
    static constexpr int LX1 = TX + 4, LY1 = TY + 4, PLANE1 = LX1 * LY1;   // q:  origin (x0-2, y0-2)
    static constexpr int LX2 = TX + 2, LY2 = TY + 2, PLANE2 = LX2 * LY2;   // q': origin (x0-1, y0-1)
    static constexpr int NRING = 2 * TX + 2 * TY;                           // ring cells without corners: a' is formed there
    static constexpr int NFRAME = NRING + 4 + 2 * TX + 2 * TY;              // + ring corners + the arms two cells out
    static constexpr int HS = (NFRAME + NT - 1) / NT;
    static_assert(NRING <= NT, "one ring cell per thread at most");

    // Frame slot s of thread tid -> coordinates in the q plane; false if the slot is unused.
    // Slots 0 .. NRING-1 are the ring (rows above and below, then the columns left and right),
    // then its four corners, then the rows and columns two cells out.
    __device__ static __forceinline__ bool frame_cell(int tid, int s, int &lx, int &ly)
    {
        int h = tid + s * NT;
        const bool used = h < NFRAME;
        if (h < 2 * TX) {
            lx = 2 + h % TX;
            ly = h < TX ? 1 : TY + 2;
        } else if (h < NRING) {
            h -= 2 * TX;
            lx = (h & 1) ? TX + 2 : 1;
            ly = 2 + h / 2;
        } else if (h < NRING + 4) {
            h -= NRING;
            lx = (h & 1) ? TX + 2 : 1;
            ly = (h & 2) ? TY + 2 : 1;
        } else if (h < NRING + 4 + 2 * TX) {
            h -= NRING + 4;
            lx = 2 + h % TX;
            ly = h < TX ? 0 : TY + 3;
        } else {
            h -= NRING + 4 + 2 * TX;
            lx = (h & 1) ? TX + 3 : 0;
            ly = 2 + h / 2;
        }
        return used;
    }
};

template <class T, int BX, int BY, int PY, int PX, bool GUARD>
__device__ __forceinline__ void pair_march(const PairArgs &a, int tix, int tiy, int zs, int ze, T *__restrict__ sq1,
                                           T *__restrict__ sq2)
{
    using G = PairTile<T, BX, BY, PY, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, TY = G::TY, LX1 = G::LX1, LX2 = G::LX2, HS = G::HS;
    constexpr T W0 = T(3.0 * star_w<1>(0)), W1 = T(star_w<1>(1));
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;

    const T *__restrict__ cg = static_cast<const T *>(a.c);
    const T *__restrict__ ag = static_cast<const T *>(a.a);
    const T *__restrict__ bg = static_cast<const T *>(a.b);
    T *__restrict__ oag = static_cast<T *>(a.out_a);
    T *__restrict__ obg = static_cast<T *>(a.out_b);

    TileAddr<PX, PY, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, nx, ny, 1, 2, LX1, 0 /* plane corner, never read */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::frame_cell(tid, s, lx, ly); });
    const uint32_t dummy = ad.dummy;
    uint32_t ooff[PY], coff[PY];
    bool ouse[PY][PX], ostore[PY];
#pragma unroll
    for (int p = 0; p < PY; ++p) {
        ostore[p] = ad.own_grid[p];
        ooff[p] = ad.own_off[p];
        bool any = false;
#pragma unroll
        for (int e = 0; e < PX; ++e) { ouse[p][e] = ad.own_I[p][e]; any = any || ouse[p][e]; }
        coff[p] = (!GUARD || any) ? ooff[p] : dummy;
    }
    uint32_t hoff[HS];
    int hlds[HS];
    bool huse[HS];
#pragma unroll
    for (int s = 0; s < HS; ++s) {
        huse[s] = ad.halo_I[s];
        hoff[s] = huse[s] ? ad.halo_off[s] : dummy;
        hlds[s] = ad.halo_lds[s];
    }
    // the ring cell of this thread (slot 0 of the first NRING threads); whole waves have one or none
    const bool ring = tid < G::NRING;
    int rlx, rly;
    G::frame_cell(tid, 0, rlx, rly);
    const int ring1 = rly * LX1 + rlx;                   // in the q plane
    const int ring2 = (rly - 1) * LX2 + (rlx - 1);       // in the q' plane
    const bool ruse = ring && huse[0];

    // running sums: index 0 = the plane that completes in this step
    T acc1[PY][PX][3], acc1r[3], acc2[PY][PX][3];
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        acc1r[k] = T(0);
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) acc1[p][e][k] = acc2[p][e][k] = T(0);
    }
    // carried from the previous step: c and a m of its plane, and what stage 2 consumes one step late
    T c_prev[PY][PX], c_prev_r = T(0), am_prev[PY][PX], q2[PY][PX], q2r = T(0), a1m[PY][PX];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e) c_prev[p][e] = am_prev[p][e] = q2[p][e] = a1m[p][e] = T(0);
    bool q2_valid = false;

    // values in flight for the next step
    V sa[PY], sc[PY], sb[PY];
    T sha[HS], shc[HS], sbr = T(0);
#pragma unroll
    for (int p = 0; p < PY; ++p) { sa[p] = V{}; sc[p] = V{}; sb[p] = V{}; }
#pragma unroll
    for (int s = 0; s < HS; ++s) sha[s] = shc[s] = T(0);

    auto plane_in_I = [&](int z) { return z >= 1 && z < nz - 1; };
    const int zi0 = zs - 2, zi1 = ze + 1;        // q planes that reach the outputs [zs, ze)
    // a' of plane z is wanted for z in [zs-1, ze] and only on I
    auto a1_wanted = [&](int z) { return z >= zs - 1 && z <= ze && plane_in_I(z); };

    // request what step z consumes: a and c of plane z (tile and frame), b of plane z-1 (tile and ring)
    // `steady` (a std::bool_constant): the caller knows that every condition on the plane index
    // holds, so the step has no branches on them (measured 2 % faster than the generic step alone)
    auto issue = [&](int z, auto steady) {
        constexpr bool ST = decltype(steady)::value;
        if (ST || (z <= zi1 && plane_in_I(z))) {
            const T *cp = cg + (size_t)z * plane;
            const T *ap = ag + (size_t)z * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                sc[p] = ld_vec_off<T, PX, false>(cp, coff[p]);
                sa[p] = ld_vec_off<T, PX, false>(ap, coff[p]);
            }
#pragma unroll
            for (int s = 0; s < HS; ++s) { shc[s] = ld_off(cp, hoff[s]); sha[s] = ld_off(ap, hoff[s]); }
        }
        if (ST || a1_wanted(z - 1)) {
            const T *bp = bg + (size_t)(z - 1) * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) sb[p] = ld_vec_off<T, PX, false>(bp, coff[p]);
            if (ring) sbr = ld_off(bp, hoff[0]);
        }
    };

    issue(zi0, std::false_type{});
    int buf = 0;
    auto step = [&](int zi, auto steady) {
        constexpr bool ST = decltype(steady)::value;
        const bool zin = ST || (zi <= zi1 && plane_in_I(zi));
        T *s1 = sq1 + buf * G::PLANE1;
        T *s2 = sq2 + buf * G::PLANE2;
        T qo[PY][PX], am[PY][PX], cc[PY][PX], qr = T(0), amr = T(0), ccr = T(0);
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T cv = sc[p].v[e], av = sa[p].v[e];
                    cc[p][e] = cv;
                    am[p][e] = GUARD ? (ouse[p][e] ? av : T(0)) : av;
                    qo[p][e] = GUARD ? (ouse[p][e] ? cv * av : T(0)) : cv * av;
                    s1[(2 + ty * PY + p) * LX1 + 2 + tx * PX + e] = qo[p][e];
                }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                const T qq = GUARD ? (huse[s] ? shc[s] * sha[s] : T(0)) : shc[s] * sha[s];
                s1[hlds[s]] = qq;
                if (s == 0) { qr = qq; ccr = shc[0]; amr = GUARD ? (huse[0] ? sha[0] : T(0)) : sha[0]; }
            }
        } else {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) cc[p][e] = am[p][e] = qo[p][e] = T(0);
        }
        const bool stage2 = ST || q2_valid;       // q' of plane zi-2 was formed in the previous step
        if (stage2) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) s2[(1 + ty * PY + p) * LX2 + 1 + tx * PX + e] = q2[p][e];
            if (ring) s2[ring2] = q2r;
        }
        V cb[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) cb[p] = sb[p];
        const T cbr = sbr;
        issue(zi + 1, steady);
        __syncthreads();

        // ---- stage 2: q' of plane zi-2 -> a'' sums of planes zi-3, zi-2, zi-1
        if (stage2) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T *at = s2 + (1 + ty * PY + p) * LX2 + 1 + tx * PX + e;
                    const T left = e > 0 ? q2[p][e - 1] : at[-1];
                    const T right = e < PX - 1 ? q2[p][e + 1] : at[1];
                    const T up = p > 0 ? q2[p - 1][e] : at[-LX2];
                    const T down = p < PY - 1 ? q2[p + 1][e] : at[LX2];
                    const T s = W0 * q2[p][e] + W1 * (left + right) + W1 * (up + down);
                    acc2[p][e][1] += s + T(2) * a1m[p][e];
                    acc2[p][e][0] += W1 * q2[p][e];
                    acc2[p][e][2] += W1 * q2[p][e];
                }
        }
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) acc2[p][e][2] -= am_prev[p][e];      // -a m of plane zi-1
        const int zo2 = zi - 3;
        if (ST || (zo2 >= zs && zo2 < ze)) {
            T *op = oag + (size_t)zo2 * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = acc2[p][e][0];
                if (!GUARD || ostore[p]) st_vec_off<T, PX, true>(op, ooff[p], o);
            }
        }

        // ---- stage 1: q of plane zi -> a' sums of planes zi-1, zi, zi+1
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T *at = s1 + (2 + ty * PY + p) * LX1 + 2 + tx * PX + e;
                    const T left = e > 0 ? qo[p][e - 1] : at[-1];
                    const T right = e < PX - 1 ? qo[p][e + 1] : at[1];
                    const T up = p > 0 ? qo[p - 1][e] : at[-LX1];
                    const T down = p < PY - 1 ? qo[p + 1][e] : at[LX1];
                    const T s = W0 * qo[p][e] + W1 * (left + right) + W1 * (up + down);
                    acc1[p][e][1] += s + T(2) * am[p][e];
                    acc1[p][e][0] += W1 * qo[p][e];
                    acc1[p][e][2] += W1 * qo[p][e];
                }
            if (ring) {
                const T *at = s1 + ring1;
                const T s = W0 * qr + W1 * (at[-1] + at[1]) + W1 * (at[-LX1] + at[LX1]);
                acc1r[1] += s + T(2) * amr;
                acc1r[0] += W1 * qr;
                acc1r[2] += W1 * qr;
            }
        }
        // a' of plane zi-1 is complete: form q' and -a' m from it
        const int zo1 = zi - 1;
        q2_valid = ST || a1_wanted(zo1);
        if (q2_valid) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T a1 = acc1[p][e][0] + cb[p].v[e];
                    a1m[p][e] = GUARD ? (ouse[p][e] ? a1 : T(0)) : a1;
                    q2[p][e] = GUARD ? (ouse[p][e] ? c_prev[p][e] * a1 : T(0)) : c_prev[p][e] * a1;
                }
            const T a1r = acc1r[0] + cbr;
            q2r = GUARD ? (ruse ? c_prev_r * a1r : T(0)) : c_prev_r * a1r;
        } else {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) a1m[p][e] = q2[p][e] = T(0);
            q2r = T(0);
        }
        if (ST || (zo1 >= zs && zo1 < ze)) {         // b'' = -a' m; zero on planes outside I
            T *op = obg + (size_t)zo1 * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = -a1m[p][e];
                if (!GUARD || ostore[p]) st_vec_off<T, PX, true>(op, ooff[p], o);
            }
        }
        // next step
        acc1r[0] = acc1r[1]; acc1r[1] = acc1r[2]; acc1r[2] = T(0);
        c_prev_r = ccr;
#pragma unroll
        for (int p = 0; p < PY; ++p)
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                acc1[p][e][0] = acc1[p][e][1]; acc1[p][e][1] = acc1[p][e][2]; acc1[p][e][2] = T(0);
                acc2[p][e][0] = acc2[p][e][1]; acc2[p][e][1] = acc2[p][e][2]; acc2[p][e][2] = T(0);
                c_prev[p][e] = cc[p][e];
                am_prev[p][e] = am[p][e];
            }
        buf ^= 1;
    };
    // steady steps: planes zi-2 .. zi+1 lie in I, and the output planes zi-3 and zi-1 in this chunk
    const int lo = max(zs + 3, 3), hi = min(ze, nz - 3);
    int zi = zi0;
    for (; zi <= zi1 + 1 && zi < lo; ++zi) step(zi, std::false_type{});
    __builtin_amdgcn_s_waitcnt(0x0F70);          // enter the steady loop with nothing outstanding (vmcnt(0))
    for (; zi <= hi; ++zi) step(zi, std::true_type{});
    for (; zi <= zi1 + 1; ++zi) step(zi, std::false_type{});
}

template <class T, int BX, int BY, int PY, int PX>
__global__ __launch_bounds__(BX *BY) void adj_wave3d_pair_kernel(PairArgs a)
{
    using G = PairTile<T, BX, BY, PY, PX>;
    __shared__ T sq1[2 * G::PLANE1];
    __shared__ T sq2[2 * G::PLANE2];
    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);
    // core tile: the tile and its frame lie in I in x and y
    const int x0 = tix * G::TX, y0 = tiy * G::TY;
    const bool core = x0 >= 3 && x0 + G::TX + 3 <= a.nx && y0 >= 3 && y0 + G::TY + 3 <= a.ny;
    if (core) pair_march<T, BX, BY, PY, PX, false>(a, tix, tiy, zs, ze, sq1, sq2);
    else      pair_march<T, BX, BY, PY, PX, true>(a, tix, tiy, zs, ze, sq1, sq2);
}

template <class T, int PX>
static hipError_t launch_pair(PairArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    constexpr int BX = 32, BY = 16, PY = 2;
    using G = PairTile<T, BX, BY, PY, PX>;
    const size_t al = PX * sizeof(T);
    const void *arrays[5] = {a.c, a.a, a.b, a.out_a, a.out_b};
    for (const void *p : arrays)
        if (reinterpret_cast<uintptr_t>(p) % al != 0) return hipErrorNotSupported;
    if (a.nx % PX != 0) return hipErrorNotSupported;
    // each chunk marches 4 planes beyond its own: plan as a march of radius 2
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, 2, opt);
    const size_t lds = sizeof(T) * 2 * (G::PLANE1 + G::PLANE2);
    const unsigned pad = one_workgroup_per_cu_pad(lds, opt.lds_pad);
    hipLaunchKernelGGL((adj_wave3d_pair_kernel<T, BX, BY, PY, PX>), dim3(a.map.total_blocks), dim3(G::NT), pad, stream, a);
    return hipGetLastError();
}

// whole vectors per lane: nx a multiple of the vector length and every array aligned to it
bool adjoint_wave3d_pair_supported(int is_f64, int nx, const void *c, const void *p0, const void *p1, const void *p2,
                                   const void *p3)
{
    const size_t al = 16;
    const int px = is_f64 ? 2 : 4;
    const void *arrays[5] = {c, p0, p1, p2, p3};
    for (const void *p : arrays)
        if (reinterpret_cast<uintptr_t>(p) % al != 0) return false;
    return nx % px == 0;
}

hipError_t launch_adjoint_wave3d_pair(int is_f64, int nx, int ny, int nz, const void *c, const void *a, const void *b,
                                      void *out_a, void *out_b, const LaunchOptions &opt, hipStream_t stream)
{
    PairArgs p{};
    p.c = c; p.a = a; p.b = b; p.out_a = out_a; p.out_b = out_b;
    p.nx = nx; p.ny = ny; p.nz = nz;
    return is_f64 ? launch_pair<double, 2>(p, opt, stream) : launch_pair<float, 4>(p, opt, stream);
}

}  // namespace sadj
