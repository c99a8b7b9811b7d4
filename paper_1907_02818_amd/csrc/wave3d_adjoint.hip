// 3-D linear wave stencil of radius R: gather-form adjoint kernel.
//
// What is computed (paper Section 4.1, gather listing, generalised to radius R;
// Sections 3.3.2-3.3.4 for index shifting, core and remainder).  With
//     q[i] = c[i]*r_bar[i] for i in I,   q[i] = 0 elsewhere,
//     u_bar[j] += 2 r_bar[j] [j in I] + sum_o w_o q[j-o]
// i.e. the same star applied to q, because the weights are symmetric; the product
// c*r_bar is formed once per staged element instead of once per term.  Optionally
// u_prev_bar[j] -= r_bar[j] for j in I (accumulate mode), or u_prev_bar[j] = -r_bar[j]
// for j in I and 0 elsewhere (assign mode, used when a time loop recycles a buffer).
//
// Mapping to CDNA4.  The x-y plane is cut into tiles of TX x TY outputs; a workgroup
// owns one tile and marches along z.  Each arriving plane of q is staged in LDS
// (tile + halo of width R, no corners: a star never reads them) and contributes
//   - its in-plane star to the running sum of the same output plane,
//   - w_k * q(x,y) to the running sums of the output planes z-k and z+k,
// so a thread keeps 2R+1 running sums per owned point in registers and LDS holds
// only the plane that has just arrived (two buffers, one barrier per plane).  An
// output plane is complete R steps after its own plane arrived; u_bar is then
// read-modify-written once.  x is the unit-stride direction of memory and lanes.
//
// Memory pipeline.  Global loads run D planes ahead of the arithmetic: the values of
// plane z+D (c and r_bar on tile and halo, u_bar of plane z+D-R) are requested as
// soon as the registers of plane z have been consumed, so D planes are in flight
// per workgroup.  The z loop is unrolled D times; the stage index is a compile-time
// constant, hence no register copies.
//
// HBM traffic.  The chip is bound by traffic that misses the 4 MB L2 of an XCD, so
// halo cells must be found in L2.  Workgroup ids are mapped such that, within each
// round of resident workgroups, every XCD owns a compact patch of neighbouring tiles
// (block_to_tile), and the number of z-chunks is chosen so that the dispatch is one
// round (one workgroup per CU) or as few full rounds as possible; the workgroups of a
// round start together, do identical work per plane and hence move through z in near
// lockstep: a halo cell is fetched from memory by whichever tile asks first and is an
// L2 hit for its neighbour.  u_bar is streamed with non-temporal loads and stores so
// that it does not displace c and r_bar from L2.
//
// Regions (Section 3.3.4).  Tiles whose reads in x and y all lie in I run the
// unguarded instantiation (core): every staged element is loaded and used
// unconditionally.  Tiles that touch the first/last 2R columns or rows run the
// guarded instantiation (remainder): an element is used iff it lies in I, otherwise
// it is replaced by zero with a select -- never by a multiplication, so NaN outside
// I cannot leak.  Along z the same rule is applied per plane with a wave-uniform
// (scalar) test in both instantiations: planes outside I are skipped.  The regions
// are disjoint and need no ordering, so they share one dispatch.
#include "launch.hpp"
#include "tile3d.hpp"

#include <type_traits>

namespace sadj {

template <class T> __device__ __forceinline__ T mul_rounded(T a, T b)
{
#pragma clang fp contract(off)
    return a * b;
}

// acc + (2 r + (3 w_0 q + sum_k w_k xs_k + sum_k w_k ys_k)) with every multiply-add explicit
// and contraction of the remaining operations off.
template <class T, int R>
__device__ __forceinline__ T pinned_centre(T q, T r, const T (&xs)[R], const T (&ys)[R], T acc)
{
#pragma clang fp contract(off)
    T s = T(3.0 * star_w<R>(0)) * q;
#pragma unroll
    for (int k = 1; k <= R; ++k) s = __builtin_fmaf(T(star_w<R>(k)), xs[k - 1], s);
#pragma unroll
    for (int k = 1; k <= R; ++k) s = __builtin_fmaf(T(star_w<R>(k)), ys[k - 1], s);
    return acc + __builtin_fmaf(T(2), r, s);
}

template <class T, int R, int BX, int BY, int PY, int PX, int D, bool NTU, bool GUARD, int UPREV>
__device__ __forceinline__ void adj3d_march(const March3dArgs &a, int tix, int tiy, int zs, int ze,
                                            T *__restrict__ sq)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    using V = Vec<T, PX>;
    constexpr int TX = G::TX, TY = G::TY, LX = G::LX, LY = G::LY, HS = G::HS;
    constexpr int NACC = 2 * R + 1;
    // A branch-free middle part of the march.  With a branch around the stores the number of
    // outstanding stores at the next wait for loads is unknown, and the compiler waits for all
    // memory operations, the stores of the previous plane included, before it touches the
    // loaded values; without the branch two stores stay in flight across the loop end.
    // Measured at 512^3 .. 1000^3: fp32 with u_bar only gains 1-6 points; fp64 loses 1-8 (the
    // wait keeps waves and workgroups closer together, which is worth more there) and the
    // u_prev_bar variants lose more, so only the fp32 u_bar-only kernels have it.  Their
    // arithmetic is written with explicit fused multiply-adds (PINNED), so that the two
    // instantiations of a step round alike and no bit depends on where the z-chunks are cut.
    constexpr bool STEADY_PHASE = D == 1 && sizeof(T) == 4 && UPREV == 0;
    constexpr bool PINNED = STEADY_PHASE;
    const int tid = threadIdx.x;
    const int tx = tid % BX, ty = tid / BX;
    const int nx = a.nx, ny = a.ny, nz = a.nz;
    const size_t plane = (size_t)nx * ny;
    const int x0 = tix * TX, y0 = tiy * TY;

    const T *__restrict__ cg = static_cast<const T *>(a.in0);
    const T *__restrict__ rg = static_cast<const T *>(a.in1);
    T *__restrict__ ug = static_cast<T *>(a.out0);
    T *__restrict__ upg = static_cast<T *>(a.out1);

    // owned cells x = x0 + tx*PX + e, y = y0 + ty*PY + p and halo slots (tile3d.hpp); c and r_bar are
    // used on I only, and not fetched at all where none of a vector's cells lies in I
    TileAddr<PX, PY, HS, GUARD> ad;
    ad.init(tx, ty, x0, y0, nx, ny, R, R, LX, 0 /* cell (0,0) is a corner nobody reads */, (uint32_t)sizeof(T),
            [&](int s, int &lx, int &ly) { return G::halo_cell(tid, s, lx, ly); });
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

    T acc[PY][PX][NACC];
#pragma unroll
    for (int p = 0; p < PY; ++p)
#pragma unroll
        for (int e = 0; e < PX; ++e)
#pragma unroll
            for (int k = 0; k < NACC; ++k) acc[p][e][k] = T(0);

    // D stages of values in flight
    V sc[D][PY], sr[D][PY], su[D][PY], sp[D][PY];
    T shc[D][HS], shr[D][HS];
#pragma unroll
    for (int d = 0; d < D; ++d) {
#pragma unroll
        for (int p = 0; p < PY; ++p) { sc[d][p] = V{}; sr[d][p] = V{}; su[d][p] = V{}; sp[d][p] = V{}; }
#pragma unroll
        for (int s = 0; s < HS; ++s) { shc[d][s] = shr[d][s] = T(0); }
    }

    const int zi0 = zs - R, zi1 = ze - 1 + R;     // input planes that reach outputs [zs, ze)
    auto plane_in_I = [&](int z) { return z >= R && z < nz - R; };

    // Request everything step `z` will consume into stage d.
    // `steady` (a std::bool_constant): the caller knows that every condition below holds, so
    // the code has no branches and the compiler can count exactly which loads and stores are
    // outstanding at each wait (see the loop at the end).
    auto issue = [&](int z, int d, auto steady) {
        constexpr bool ST = decltype(steady)::value;
        if (!ST && z > zi1) return;
        if (ST || plane_in_I(z)) {
            const T *cp = cg + (size_t)z * plane;
            const T *rp = rg + (size_t)z * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                sc[d][p] = ld_vec_off<T, PX, false>(cp, coff[p]);
                sr[d][p] = ld_vec_off<T, PX, false>(rp, coff[p]);
            }
#pragma unroll
            for (int s = 0; s < HS; ++s) { shc[d][s] = ld_off(cp, hoff[s]); shr[d][s] = ld_off(rp, hoff[s]); }
            if (UPREV == 1) {                      // accumulate mode reads u_prev_bar; assign mode does not
                if (ST || (z >= zs && z < ze)) {
                    const T *pp = upg + (size_t)z * plane;
#pragma unroll
                    for (int p = 0; p < PY; ++p) sp[d][p] = ld_vec_off<T, PX, NTU>(pp, ooff[p]);
                }
            }
        }
        const int zo = z - R;
        if (ST || zo >= zs) {                      // zo <= ze-1 because z <= zi1
            const T *up = ug + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) su[d][p] = ld_vec_off<T, PX, NTU>(up, ooff[p]);
        }
    };

    int buf = 0;
    auto step = [&](int zi, int d, auto steady) {
        constexpr bool ST = decltype(steady)::value;
        const bool zin = ST || plane_in_I(zi);
        const int zo = zi - R;
        T *sb = sq + buf * (LY * LX);
        T qo[PY][PX], ro[PY][PX];
        V cu[PY];
#pragma unroll
        for (int p = 0; p < PY; ++p) cu[p] = su[d][p];
        if (zin) {
#pragma unroll
            for (int p = 0; p < PY; ++p)
#pragma unroll
                for (int e = 0; e < PX; ++e) {
                    const T cc = sc[d][p].v[e], rv = sr[d][p].v[e];
                    ro[p][e] = GUARD ? (ouse[p][e] ? rv : T(0)) : rv;
                    // PINNED: a product rounded on its own, never fused into a later addition
                    // (for radius 1 the z-terms are acc + 1.0 * q, which would otherwise invite it)
                    const T cr = PINNED ? mul_rounded(cc, rv) : cc * rv;
                    qo[p][e] = GUARD ? (ouse[p][e] ? cr : T(0)) : cr;
                    sb[(R + ty * PY + p) * LX + R + tx * PX + e] = qo[p][e];
                }
#pragma unroll
            for (int s = 0; s < HS; ++s) {
                const T qq = GUARD ? (huse[s] ? shc[d][s] * shr[d][s] : T(0)) : shc[d][s] * shr[d][s];
                sb[hlds[s]] = qq;
            }
            if (UPREV) {
                if (ST || (zi >= zs && zi < ze)) {
                    T *pp = upg + (size_t)zi * plane;
#pragma unroll
                    for (int p = 0; p < PY; ++p) {
                        V o;
#pragma unroll
                        for (int e = 0; e < PX; ++e) o.v[e] = (UPREV == 1 ? sp[d][p].v[e] : T(0)) - ro[p][e];
                        if (!GUARD || ostore[p]) st_vec_off<T, PX, NTU>(pp, ooff[p], o);
                    }
                }
            }
        } else if (UPREV == 2) {
            // assign mode: planes of this chunk outside I receive zeros
            if (zi >= zs && zi < ze) {
                T *pp = upg + (size_t)zi * plane;
#pragma unroll
                for (int p = 0; p < PY; ++p)
                    if (!GUARD || ostore[p]) st_vec_off<T, PX, NTU>(pp, ooff[p], V{});
            }
        }
        // the registers of stage d are free again: request plane zi+D
        issue(zi + D, d, steady);
        if (zin) {
            __syncthreads();
#pragma unroll
            for (int e = 0; e < PX; ++e) {
                T col[PY + 2 * R];
#pragma unroll
                for (int i = 0; i < PY + 2 * R; ++i) col[i] = sb[(ty * PY + i) * LX + R + tx * PX + e];
#pragma unroll
                for (int p = 0; p < PY; ++p) {
                    const T *row = sb + (R + ty * PY + p) * LX + R + tx * PX + e;
                    if constexpr (PINNED) {
                        // every multiply-add written out, so that the generic and the branch-free
                        // instantiation of this step round alike
                        T xs[R], ys[R];
#pragma unroll
                        for (int k = 1; k <= R; ++k) { xs[k - 1] = row[-k] + row[k]; ys[k - 1] = col[R + p - k] + col[R + p + k]; }
                        acc[p][e][R] = pinned_centre<T, R>(qo[p][e], ro[p][e], xs, ys, acc[p][e][R]);
#pragma unroll
                        for (int k = 1; k <= R; ++k) {
                            acc[p][e][R - k] = __builtin_fmaf(T(star_w<R>(k)), qo[p][e], acc[p][e][R - k]);
                            acc[p][e][R + k] = __builtin_fmaf(T(star_w<R>(k)), qo[p][e], acc[p][e][R + k]);
                        }
                    } else {
                        T s = T(3.0 * star_w<R>(0)) * qo[p][e];
#pragma unroll
                        for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (row[-k] + row[k]);
#pragma unroll
                        for (int k = 1; k <= R; ++k) s += T(star_w<R>(k)) * (col[R + p - k] + col[R + p + k]);
                        acc[p][e][R] += s + T(2) * ro[p][e];
#pragma unroll
                        for (int k = 1; k <= R; ++k) {
                            acc[p][e][R - k] += T(star_w<R>(k)) * qo[p][e];
                            acc[p][e][R + k] += T(star_w<R>(k)) * qo[p][e];
                        }
                    }
                }
            }
            buf ^= 1;
        }
        if (ST || zo >= zs) {
            T *up = ug + (size_t)zo * plane;
#pragma unroll
            for (int p = 0; p < PY; ++p) {
                V o;
#pragma unroll
                for (int e = 0; e < PX; ++e) o.v[e] = cu[p].v[e] + acc[p][e][0];
                if (!GUARD || ostore[p]) st_vec_off<T, PX, NTU>(up, ooff[p], o);
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
    };

    using Generic = std::false_type;
    using Steady = std::true_type;
#pragma unroll
    for (int d = 0; d < D; ++d) issue(zi0 + d, d, Generic{});
    if constexpr (STEADY_PHASE) {
        // Steady steps zi in [lo, hi]: planes zi and zi+1 lie in I and in this chunk's input
        // range, and the output planes zi-R and zi+1-R belong to the chunk.
        const int lo = zs + R;
        const int hi = min(nz - R - 2, ze - 2);
        int zi = zi0;
        for (; zi <= zi1 && zi < lo; ++zi) step(zi, 0, Generic{});
        // Enter the steady loop with nothing outstanding: otherwise the unknown number of loads
        // that the generic steps may have left pending is carried into the loop header, and
        // every iteration waits for all its memory operations there (vmcnt(0); expcnt and
        // lgkmcnt untouched).
        __builtin_amdgcn_s_waitcnt(0x0F70);
        for (; zi <= hi; ++zi) step(zi, 0, Steady{});
        for (; zi <= zi1; ++zi) step(zi, 0, Generic{});
    } else {
        for (int zb = zi0; zb <= zi1; zb += D) {
#pragma unroll
            for (int d = 0; d < D; ++d)
                if (zb + d <= zi1) step(zb + d, d, Generic{});
        }
    }
}

// REM selects how the remainder (Section 3.3.4) is treated:
//   0  one dispatch; a block-uniform test picks the unguarded (core) or the guarded body
//   1  every tile runs the guarded body: all shifted statements everywhere, reads outside
//      I yield zero -- the zero-padding strategy without owning the caller's memory
//   2  core tiles only   } two disjoint dispatches, each with a single body and no
//   3  remainder tiles only } choice between bodies (the split-nests strategy at tile level)
template <class T, int R, int BX, int BY, int PY, int PX, int D, bool NTU, int UPREV, int REM>
__global__ __launch_bounds__(BX *BY) void adj_wave3d_kernel(March3dArgs a)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    __shared__ T sq[2 * G::PLANE];
    int tix, tiy, zs, ze;
    block_to_tile(a.map, blockIdx.x, tix, tiy, zs, ze);
    // core tile: own cells and halo cells all inside I in x and y
    const int x0 = tix * G::TX, y0 = tiy * G::TY;
    const bool core = x0 >= 2 * R && x0 + G::TX + 2 * R <= a.nx && y0 >= 2 * R && y0 + G::TY + 2 * R <= a.ny;
    if (REM == 0) {
        if (core) adj3d_march<T, R, BX, BY, PY, PX, D, NTU, false, UPREV>(a, tix, tiy, zs, ze, sq);
        else      adj3d_march<T, R, BX, BY, PY, PX, D, NTU, true, UPREV>(a, tix, tiy, zs, ze, sq);
    } else if (REM == 1) {
        adj3d_march<T, R, BX, BY, PY, PX, D, NTU, true, UPREV>(a, tix, tiy, zs, ze, sq);
    } else if (REM == 2) {
        if (core) adj3d_march<T, R, BX, BY, PY, PX, D, NTU, false, UPREV>(a, tix, tiy, zs, ze, sq);
    } else {
        if (!core) adj3d_march<T, R, BX, BY, PY, PX, D, NTU, true, UPREV>(a, tix, tiy, zs, ze, sq);
    }
}

static inline bool aligned_to(const void *p, size_t n) { return (reinterpret_cast<uintptr_t>(p) % n) == 0; }

template <class T, int R, int BX, int BY, int PY, int PX, int D, bool NTU>
static hipError_t launch_cfg(March3dArgs a, const LaunchOptions &opt, hipStream_t stream)
{
    using G = Tile3d<T, R, BX, BY, PY, PX>;
    if (PX > 1) {
        // PX cells per lane and memory instruction need whole vectors: nx a multiple of
        // PX and every array aligned to the vector size; otherwise use a PX = 1 shape
        const size_t al = PX * sizeof(T);
        const bool ok = a.nx % PX == 0 && aligned_to(a.in0, al) && aligned_to(a.in1, al) &&
                        aligned_to(a.out0, al) && aligned_to(a.out1, al);
        if (!ok) return launch_cfg<T, R, 64, 8, 4, 1, 1, true>(a, opt, stream);
    }
    plan_march(a.map, a.nx, a.ny, a.nz, G::TX, G::TY, R, opt);
    dim3 grid(a.map.total_blocks), block(G::NT);
    const unsigned pad = one_workgroup_per_cu_pad(sizeof(T) * 2 * G::PLANE, opt.lds_pad);
    if (opt.remainder != 0) {
        // the strategy study is built for the two default shapes and u_bar only
        if constexpr (BX == 32 && BY == 16 && D == 1 && NTU) {
            if (a.out1) return hipErrorNotSupported;
            if (opt.remainder == 1) {
                hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 0, 1>), grid, block, pad, stream, a);
            } else {
                hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 0, 2>), grid, block, pad, stream, a);
                hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 0, 3>), grid, block, pad, stream, a);
            }
            return hipGetLastError();
        } else {
            return hipErrorNotSupported;
        }
    }
    if (!a.out1)                hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 0, 0>), grid, block, pad, stream, a);
    else if (a.out1_assign == 0) hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 1, 0>), grid, block, pad, stream, a);
    else                        hipLaunchKernelGGL((adj_wave3d_kernel<T, R, BX, BY, PY, PX, D, NTU, 2, 0>), grid, block, pad, stream, a);
    return hipGetLastError();
}

// Tile shapes <BX, BY, PY, PX, D, NT>.  Variant 0 picks the measured best per dtype:
// 16 bytes per lane and memory instruction (two doubles / four floats), tile rows of
// 512 bytes, 32 rows, 32 x 16 threads (a wave covers two rows), one workgroup per CU.
//   1  fp64 default: 64 x 32 tile, two doubles per lane
//   2  fp32 default: 128 x 32 tile, four floats per lane
//   3  one cell per lane (64 x 32 tile, 8- or 4-byte accesses): the fallback for odd nx or
//      unaligned arrays, and the fp64 choice when u_prev_bar is read and written as well
//   5  rows of 1 KB, 16 rows: for rows that are not cache-line multiples
//   10, 11  radius 1 only: 16 rows of 256 / 512 cells (see wide_tile_for_unaligned_rows)
// (Shapes tried and removed: two planes in flight, u_bar without the streaming hint, a
// 64 x 16 tile with 256 threads, a 128 x 32 tile with eight cells per thread -- none
// was the best anywhere.)
static inline long choose_adjoint_shape(bool is_f64, int radius, int nx, bool u_prev_accumulated, const LaunchOptions &opt)
{
    long v = opt.variant;
    if (v != 0) return v;
    // measured best: 16 bytes per lane (1 for fp64, 2 for fp32); fp64 with u_prev_bar read and
    // written as well: the one-cell shape with fewer registers per cell (3).  (fp32 with
    // u_prev_bar: shape 2 measured 3-16 points faster than an 8-byte shape at 256^3 .. 896^3.)
    v = is_f64 ? (u_prev_accumulated ? 3 : 1) : 2;
    if (opt.remainder == 0) {
        const int wide = wide_tile_for_unaligned_rows(nx, is_f64 ? 8 : 4, radius, !is_f64);
        if (radius == 1 && wide == 512) v = 11;
        else if (radius == 1 && wide == 256) v = 10;
        else if (wide) v = 5;
    }
    return v;
}

// Tile extents (cells) and cells per lane of a shape, for the host-side description of the plan.
static inline void shape_extents(long v, bool is_f64, int radius, int &TX, int &TY, int &PX)
{
    const int px16 = is_f64 ? 2 : 4;
    switch (v) {
    case 2: TX = 128; TY = 32; PX = 4; break;
    case 3: TX = 64; TY = 32; PX = 1; break;
    case 5: TX = 64 * px16; TY = 16; PX = px16; break;
    case 10: if (radius == 1) { TX = 256; TY = 16; PX = 2; break; } TX = 64; TY = 32; PX = 2; break;
    case 11: if (radius == 1 && !is_f64) { TX = 512; TY = 16; PX = 4; break; } TX = 64; TY = 32; PX = 2; break;
    default: TX = 64; TY = 32; PX = 2; break;      // 1 and anything unknown: the fp64 default shape
    }
}

template <class T, int R>
static hipError_t launch_T(const March3dArgs &a, const LaunchOptions &opt, hipStream_t stream)
{
    const long v = choose_adjoint_shape(sizeof(T) == 8, R, a.nx, a.out1 && !a.out1_assign, opt);
    if constexpr (R == 2 || R == 3) {            // the default shapes of the dtype only
        if constexpr (sizeof(T) == 8) {
            return v == 3 ? launch_cfg<T, R, 64, 8, 4, 1, 1, true>(a, opt, stream)
                 : v == 5 ? launch_cfg<T, R, 64, 8, 2, 2, 1, true>(a, opt, stream)
                          : launch_cfg<T, R, 32, 16, 2, 2, 1, true>(a, opt, stream);
        } else {
            return v == 3 ? launch_cfg<T, R, 64, 8, 4, 1, 1, true>(a, opt, stream)
                 : v == 5 ? launch_cfg<T, R, 64, 8, 2, 4, 1, true>(a, opt, stream)
                          : launch_cfg<T, R, 32, 16, 2, 4, 1, true>(a, opt, stream);
        }
    } else {
        switch (v) {
        default:
        case 1: return launch_cfg<T, R, 32, 16, 2, 2, 1, true>(a, opt, stream);     // fp64 default
        case 2: return launch_cfg<T, R, 32, 16, 2, 4, 1, true>(a, opt, stream);     // fp32 default
        case 3: return launch_cfg<T, R, 64, 8, 4, 1, 1, true>(a, opt, stream);      // one cell per lane
        case 5:                                                                     // rows of 1 KB, 16 rows
            if constexpr (sizeof(T) == 8) return launch_cfg<T, R, 64, 8, 2, 2, 1, true>(a, opt, stream);
            else return launch_cfg<T, R, 64, 8, 2, 4, 1, true>(a, opt, stream);
        // radius 1 only: 16 rows of 256 or 512 cells
        case 10:
            if constexpr (R == 1) return launch_cfg<T, R, 128, 4, 4, 2, 1, true>(a, opt, stream);  // 256 x 16 tile, PX = 2
            else return launch_cfg<T, R, 32, 16, 2, 2, 1, true>(a, opt, stream);
        case 11:
            if constexpr (R == 1 && sizeof(T) == 4) return launch_cfg<T, R, 128, 4, 4, 4, 1, true>(a, opt, stream);   // 512 x 16 tile, PX = 4
            else return launch_cfg<T, R, 32, 16, 2, 2, 1, true>(a, opt, stream);
        }
    }
}

void describe_march_plan(int is_f64, int radius, int nx, int ny, int nz, int with_u_prev_bar, const LaunchOptions &opt,
                         long *plan, int *tiles, long max_blocks)
{
    // the shape launch_T takes for 16-byte aligned arrays and an nx that allows whole vectors;
    // otherwise the one-cell shape
    long v = choose_adjoint_shape(is_f64 != 0, radius, nx, with_u_prev_bar != 0, opt);
    int TX, TY, PX;
    shape_extents(v, is_f64 != 0, radius, TX, TY, PX);
    if (nx % PX != 0) shape_extents(3, is_f64 != 0, radius, TX, TY, PX);
    March3dArgs a{};
    a.nx = nx; a.ny = ny; a.nz = nz;
    TileMap &m = a.map;
    plan_march(m, nx, ny, nz, TX, TY, radius, opt);
    plan[0] = m.ntx; plan[1] = m.nty; plan[2] = TX; plan[3] = TY; plan[4] = m.total_blocks;
    plan[5] = m.tiles_a; plan[6] = m.ntz_a; plan[7] = m.ntz;
    if (!tiles) return;
    for (int b = 0; b < m.total_blocks && b < max_blocks; ++b) {
        int tix, tiy, zs, ze;
        block_to_tile(m, b, tix, tiy, zs, ze);
        tiles[4 * b] = tix; tiles[4 * b + 1] = tiy; tiles[4 * b + 2] = zs; tiles[4 * b + 3] = ze;
    }
}

hipError_t launch_adjoint_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                 const void *r_bar, void *u_bar, void *u_prev_bar, int u_prev_bar_assign,
                                 const LaunchOptions &opt, hipStream_t stream)
{
    March3dArgs a{};
    a.in0 = c; a.in1 = r_bar; a.out0 = u_bar; a.out1 = u_prev_bar;
    a.out1_assign = u_prev_bar_assign;
    a.nx = nx; a.ny = ny; a.nz = nz;
    if (is_f64) {
        switch (radius) {
        case 1: return launch_T<double, 1>(a, opt, stream);
        case 2: return launch_T<double, 2>(a, opt, stream);
        case 3: return launch_T<double, 3>(a, opt, stream);
        default: return launch_T<double, 4>(a, opt, stream);
        }
    }
    switch (radius) {
    case 1: return launch_T<float, 1>(a, opt, stream);
    case 2: return launch_T<float, 2>(a, opt, stream);
    case 3: return launch_T<float, 3>(a, opt, stream);
    default: return launch_T<float, 4>(a, opt, stream);
    }
}

}  // namespace sadj
