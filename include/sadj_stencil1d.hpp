/*
 * sadj_stencil1d.hpp -- primal and gather-form adjoint of a USER-SUPPLIED three-point
 * stencil loop on a 1-D grid, for one AMD MI355X (gfx950).  Header only, HIP C++17;
 * include it from a .hip file compiled with hipcc --offload-arch=gfx950.
 *
 * What it is for (paper Section 3.3.1, the paragraph on large loop bodies): instead of a
 * concrete expression the user hands over an uninterpreted function
 *     r[i] = f(a, b, c)(a = u[i-1], b = u[i], c = u[i+1])          for i in I = [1, n-2]
 * and the adjoint refers to its partial derivatives as uninterpreted calls as well; a back
 * end substitutes a hand-written or AD-generated derivative routine.  Here both are the
 * member functions of a device functor, and the kernel body below is the same for every
 * stencil: a new nonlinear stencil needs a functor, not a kernel.
 *
 * The functor F (trivially copyable, passed by value to the kernel) provides
 *     static constexpr bool uses_passive;   // does the loop body read a passive array p[i]?
 *     static constexpr bool df_uses_u;      // do the partials depend on u (nonlinear body)?
 *     __device__ T f (T um, T u0, T up, T p) const;                        // loop body
 *     __device__ void df(T um, T u0, T up, T p, T &dm, T &d0, T &dp) const; // its partials
 * with (um, u0, up) = (u[i-1], u[i], u[i+1]), p = p[i] (0 if !uses_passive), and
 * (dm, d0, dp) = the partial derivatives of f with respect to um, u0, up at that point.
 * Only u is active: there is no p_bar (Section 3.3.1, list of active variables).  If the
 * body is linear in u its partials do not read u (Section 3.1: only a nonlinear statement
 * makes the adjoint read primal values); with df_uses_u == false the adjoint skips those
 * loads, passes zeros for (um, u0, up) and accepts u == nullptr.
 *
 * What is computed.
 *   primal_stencil1d:   r[i] = f(u[i-1], u[i], u[i+1], p[i])  for i in I; r[0], r[n-1] untouched.
 *   adjoint_stencil1d:  u_bar[j] += dp(j-1) r_bar[j-1] [j-1 in I] + d0(j) r_bar[j] [j in I]
 *                                 + dm(j+1) r_bar[j+1] [j+1 in I]      for all j in [0, n-1],
 *   where d*(i) are the partials evaluated at iteration i.  This is the scatter
 *   u_bar[i+o] += (df_i/du_{i+o}) r_bar[i] after index shifting (Section 3.3.2): the shifted
 *   derivative calls read u at j-2 .. j+2, indices the primal at j never touched.  Every
 *   partial is evaluated once per primal iteration (the terms d*(i) r_bar[i] are formed
 *   by the lane that owns cell i and handed to the neighbouring lanes), every u_bar[j] is
 *   written by exactly one lane, no atomics; the result is reproducible bit for bit.
 *   Values of r_bar outside I never influence the result, not even NaN; partials that f
 *   returns for iterations outside I are discarded by selects.
 *
 * Mapping.  A 64-lane wave owns 64*PX consecutive cells (PX = 16 bytes per lane when all
 * arrays are 16-byte aligned, else 1).  Terms travel between lanes by wave shuffles; the
 * terms of the two cells beside the segment are evaluated by lanes 0 and 63.  Segments
 * whose reads all lie inside the array and whose iterations all lie in I run without any
 * guard (core, Section 3.3.3); the first and the last segment(s) run the guarded
 * instantiation (remainder, Section 3.3.4); both share one dispatch.
 *
 * Arguments: DEVICE pointers to n elements each, owned by the caller and valid until the
 * work queued on `stream` has finished; p may be nullptr iff !F::uses_passive; the
 * adjoint's u may be nullptr iff !F::df_uses_u.  r and
 * u_bar must not overlap the inputs.  n >= 3.  Returns hipErrorInvalidValue for bad
 * arguments (nothing is enqueued), else the status of the launch.  Asynchronous.
 */
#ifndef SADJ_STENCIL1D_HPP
#define SADJ_STENCIL1D_HPP

#include <hip/hip_runtime.h>
#include <cstdint>

namespace sadj {
namespace stencil1d_detail {

constexpr int kWaves = 4;     // waves per workgroup

template <class T, class F> struct Args {
    F fn;
    const T *u, *p, *r_bar;   // r_bar: adjoint only
    T *out;                   // primal: r, adjoint: u_bar
    long n;
    long core_segs;           // core waves handle segments 1 .. core_segs
    long core_blocks;         // workgroups [0, core_blocks) are core, the rest remainder
    long rem_segs;            // remainder waves: index 0 -> segment 0, k > 0 -> segment core_segs + k
};

// PX consecutive cells from x.  Unguarded: one memory instruction, with the streaming
// (non-temporal) hint: every array of a call is touched exactly once, and keeping these
// lines out of the way in L2 measured 5-9 points faster.  Guarded: element-wise, indices
// clamped into the array (the values of clamped reads are discarded later).
template <class T, int PX, bool GUARD>
__device__ __forceinline__ void load_cells(const T *g, long x, long n, T (&v)[PX])
{
    if (!GUARD) {
        typedef T VT __attribute__((ext_vector_type(PX)));
        const VT t = __builtin_nontemporal_load(reinterpret_cast<const VT *>(g + x));
#pragma unroll
        for (int e = 0; e < PX; ++e) v[e] = t[e];
    } else {
#pragma unroll
        for (int e = 0; e < PX; ++e) v[e] = g[x + e < n ? x + e : n - 1];
    }
}
template <class T, int PX, bool GUARD>
__device__ __forceinline__ void store_cells(T *g, long x, const T (&v)[PX], const bool (&ok)[PX])
{
    if (!GUARD) {
        typedef T VT __attribute__((ext_vector_type(PX)));
        VT t;
#pragma unroll
        for (int e = 0; e < PX; ++e) t[e] = v[e];
        __builtin_nontemporal_store(t, reinterpret_cast<VT *>(g + x));
    } else {
#pragma unroll
        for (int e = 0; e < PX; ++e)
            if (ok[e]) g[x + e] = v[e];
    }
}
// One cell, loaded by lanes 0 and 63 only (the others get 0).
template <class T, bool GUARD> __device__ __forceinline__ T load_edge(const T *g, long i, long n, int lane)
{
    if (GUARD) i = i < 0 ? 0 : (i > n - 1 ? n - 1 : i);
    T v = T(0);
    if (lane == 0 || lane == 63) v = g[i];
    return v;
}
__device__ __forceinline__ bool in_I(long i, long n) { return i >= 1 && i <= n - 2; }

template <class T, class F, int PX, bool GUARD>
__device__ __forceinline__ void primal_segment(const Args<T, F> &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T uv[PX], pv[PX];
    load_cells<T, PX, GUARD>(a.u, x, n, uv);
    if (F::uses_passive) load_cells<T, PX, GUARD>(a.p, x, n, pv);
    const T uh = load_edge<T, GUARD>(a.u, hx, n, lane);
    const T from_left = __shfl_up(uv[PX - 1], 1), from_right = __shfl_down(uv[0], 1);
    const T left = lane == 0 ? uh : from_left, right = lane == 63 ? uh : from_right;
    T out[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T um = e == 0 ? left : uv[e - 1];
        const T up = e == PX - 1 ? right : uv[e + 1];
        ok[e] = GUARD ? in_I(x + e, n) : true;
        out[e] = a.fn.f(um, uv[e], up, F::uses_passive ? pv[e] : T(0));
    }
    store_cells<T, PX, GUARD>(a.out, x, out, ok);
}

template <class T, class F, int PX, bool GUARD>
__device__ __forceinline__ void adjoint_segment(const Args<T, F> &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;             // the cell beside the segment
    const long hx2 = lane < 32 ? xs - 2 : xs + W + 1;        // and the one beyond it
    T uv[PX], pv[PX], rv[PX], bv[PX];
    if (F::df_uses_u) {
        load_cells<T, PX, GUARD>(a.u, x, n, uv);
    } else {
#pragma unroll
        for (int e = 0; e < PX; ++e) uv[e] = T(0);
    }
    load_cells<T, PX, GUARD>(a.r_bar, x, n, rv);
    load_cells<T, PX, GUARD>(a.out, x, n, bv);
    if (F::uses_passive) load_cells<T, PX, GUARD>(a.p, x, n, pv);
    const T uh = F::df_uses_u ? load_edge<T, GUARD>(a.u, hx, n, lane) : T(0);
    const T uh2 = F::df_uses_u ? load_edge<T, GUARD>(a.u, hx2, n, lane) : T(0);
    const T rh = load_edge<T, GUARD>(a.r_bar, hx, n, lane);
    const T ph = F::uses_passive ? load_edge<T, GUARD>(a.p, hx, n, lane) : T(0);

    const T from_left = __shfl_up(uv[PX - 1], 1), from_right = __shfl_down(uv[0], 1);
    const T left = lane == 0 ? uh : from_left, right = lane == 63 ? uh : from_right;

    // terms of the iterations this lane owns: to u_bar[i-1], u_bar[i], u_bar[i+1]
    T tm[PX], t0[PX], tp[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T um = e == 0 ? left : uv[e - 1];
        const T up = e == PX - 1 ? right : uv[e + 1];
        T dm, d0, dp;
        a.fn.df(um, uv[e], up, F::uses_passive ? pv[e] : T(0), dm, d0, dp);
        const bool in = GUARD ? in_I(x + e, n) : true;
        ok[e] = GUARD ? (x + e < n) : true;
        tm[e] = in ? dm * rv[e] : T(0);
        t0[e] = in ? d0 * rv[e] : T(0);
        tp[e] = in ? dp * rv[e] : T(0);
    }
    // the iteration beside the segment: lane 0 needs its term to u_bar[xs] (dp of cell
    // xs-1), lane 63 its term to u_bar[xs+W-1] (dm of cell xs+W)
    T th;
    {
        const bool lo = lane < 32;
        const T um = lo ? uh2 : uv[PX - 1];
        const T up = lo ? uv[0] : uh2;
        T dm, d0, dp;
        a.fn.df(um, uh, up, ph, dm, d0, dp);
        const bool in = GUARD ? in_I(hx, n) : true;
        th = in ? (lo ? dp : dm) * rh : T(0);
    }
    const T tl = __shfl_up(tp[PX - 1], 1), tr = __shfl_down(tm[0], 1);
    const T term_left = lane == 0 ? th : tl;      // from iteration x-1
    const T term_right = lane == 63 ? th : tr;    // from iteration x+PX
    T out[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T l = e == 0 ? term_left : tp[e - 1];
        const T r = e == PX - 1 ? term_right : tm[e + 1];
        out[e] = bv[e] + ((l + t0[e]) + r);
    }
    store_cells<T, PX, GUARD>(a.out, x, out, ok);
}

template <class T, class F, int PX, bool ADJ>
__global__ __launch_bounds__(64 * kWaves) void kernel(Args<T, F> a)
{
    constexpr int W = 64 * PX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long b = blockIdx.x;
    if (b < a.core_blocks) {                       // block-uniform; the kernel has no barrier
        const long local = b * kWaves + wave;
        if (local >= a.core_segs) return;
        if (ADJ) adjoint_segment<T, F, PX, false>(a, (1 + local) * W, lane);
        else     primal_segment<T, F, PX, false>(a, (1 + local) * W, lane);
    } else {
        const long local = (b - a.core_blocks) * kWaves + wave;
        if (local >= a.rem_segs) return;
        const long seg = local == 0 ? 0 : a.core_segs + local;
        if (ADJ) adjoint_segment<T, F, PX, true>(a, seg * W, lane);
        else     primal_segment<T, F, PX, true>(a, seg * W, lane);
    }
}

// Core: segments 1 .. s_hi, those with xs >= W and xs + W <= n - 2: own cells and both
// neighbouring cells lie in I, and the reads at xs-2 and xs+W+1 lie inside the array.
// Remainder: segment 0 and segments s_hi+1 .. nseg-1.
template <class T, class F, int PX, bool ADJ>
hipError_t launch(Args<T, F> a, hipStream_t stream)
{
    constexpr int W = 64 * PX;
    const long nseg = (a.n + W - 1) / W;
    long s_hi = (a.n - 2) / W - 1;
    if (s_hi < 1) s_hi = 0;
    a.core_segs = s_hi;
    a.core_blocks = (a.core_segs + kWaves - 1) / kWaves;
    a.rem_segs = 1 + (nseg - 1 - s_hi);
    const long blocks = a.core_blocks + (a.rem_segs + kWaves - 1) / kWaves;
    if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((kernel<T, F, PX, ADJ>), dim3((unsigned)blocks), dim3(64 * kWaves), 0, stream, a);
    return hipGetLastError();
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

template <class T, class F, bool ADJ>
hipError_t dispatch(const Args<T, F> &a, hipStream_t stream)
{
    constexpr int PXV = 16 / sizeof(T);
    const bool al = aligned16(a.u) && aligned16(a.p) && aligned16(a.r_bar) && aligned16(a.out);
    return al ? launch<T, F, PXV, ADJ>(a, stream) : launch<T, F, 1, ADJ>(a, stream);
}

}  // namespace stencil1d_detail

template <class T, class F>
hipError_t primal_stencil1d(const F &fn, long n, const T *u, const T *p, T *r, hipStream_t stream)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "float or double");
    if (n < 3 || !u || !r || (F::uses_passive && !p)) return hipErrorInvalidValue;
    stencil1d_detail::Args<T, F> a{fn, u, F::uses_passive ? p : nullptr, nullptr, r, n, 0, 0, 0};
    return stencil1d_detail::dispatch<T, F, false>(a, stream);
}

template <class T, class F>
hipError_t adjoint_stencil1d(const F &fn, long n, const T *u, const T *p, const T *r_bar, T *u_bar,
                             hipStream_t stream)
{
    static_assert(sizeof(T) == 4 || sizeof(T) == 8, "float or double");
    if (n < 3 || (F::df_uses_u && !u) || !r_bar || !u_bar || (F::uses_passive && !p)) return hipErrorInvalidValue;
    stencil1d_detail::Args<T, F> a{fn, F::df_uses_u ? u : nullptr, F::uses_passive ? p : nullptr, r_bar, u_bar, n, 0, 0, 0};
    return stencil1d_detail::dispatch<T, F, true>(a, stream);
}

}  // namespace sadj
#endif /* SADJ_STENCIL1D_HPP */
