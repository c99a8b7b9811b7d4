// 1-D stencils: linear 3-point wave step and upwinded Burgers step, primal and
// gather-form adjoint (paper Sections 3.2, 4.1 in one dimension, and 4.2).
//
// Mapping to CDNA4.  A 64-lane wave owns a segment of 64*PX consecutive cells, PX
// cells (16 bytes) per lane.  Neighbour values travel between lanes with wave
// shuffles; the two cells beside the segment are loaded by lanes 0 and 63.  No LDS,
// no barrier, no atomics: each output cell is written by exactly one lane.
//
// Regions (Sections 3.3.3, 3.3.4).  The core waves cover the segments whose reads
// all lie in the primal iteration space I = [1, n-2]; they run an instantiation that
// is compiled without any guard.  The remainder waves cover the first and the last
// segment(s) with the guarded instantiation: a term is kept iff its primal iteration
// exists, unused values are replaced by zero with a select (never multiplied by zero),
// and loads are element-wise and clamped into the array.  Core and remainder are
// disjoint and unordered, so they share one dispatch: the first workgroups are core,
// the last one or two are remainder.
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

struct Args1d {
    const void *a0, *a1, *a2;   // inputs (meaning depends on the kernel)
    void *o0, *o1;              // outputs
    long n;
    double C, D;
    double w[3];                // box stencil: gather weights at offsets -1, 0, +1
    long core_segs;             // core waves handle segments 1 .. core_segs
    long core_blocks;           // workgroups [0, core_blocks) are core, the rest remainder
    long rem_segs;              // remainder waves: index 0 -> segment 0, k>0 -> segment core_segs + k
};

constexpr int kWaves1d = 4;
constexpr bool kStreamStores = true;
enum Op1d { OP_ADJ_WAVE, OP_ADJ_WAVE_UPREV, OP_PRI_WAVE, OP_PRI_BURGERS, OP_ADJ_BURGERS, OP_ADJ_BOX, OP_PRI_BOX,
            OP_ADJ_BURGERS_ASSIGN, OP_PRI_BURGERS_KEEP_ENDS };

// Load PX consecutive cells starting at x.  Unguarded: one vector load.  Guarded:
// element-wise, indices clamped to [0, n-1].
template <class T, int PX, bool GUARD, bool STREAM = false>
__device__ __forceinline__ void load_cells(const T *p, long x, long n, T (&v)[PX])
{
    if (!GUARD) {
        const Vec<T, PX> t = STREAM ? ld_vec_stream<T, PX>(p + x) : ld_vec<T, PX>(p + x);
#pragma unroll
        for (int e = 0; e < PX; ++e) v[e] = t.v[e];
    } else {
#pragma unroll
        for (int e = 0; e < PX; ++e) {
            const long i = x + e < n ? x + e : n - 1;
            v[e] = p[i];
        }
    }
}
// The cell beside a wave's segment; only lanes 0 and 63 use it, so only they load it.
template <class T, bool GUARD> __device__ __forceinline__ T load_cell(const T *p, long i, long n, int lane)
{
    if (GUARD) i = i < 0 ? 0 : (i > n - 1 ? n - 1 : i);
    T v = T(0);
    if (lane == 0 || lane == 63) v = p[i];
    return v;
}
template <class T, int PX, bool GUARD>
__device__ __forceinline__ void store_cells(T *p, long x, long n, const T (&v)[PX], const bool (&ok)[PX])
{
    if (!GUARD) {
        Vec<T, PX> t;
#pragma unroll
        for (int e = 0; e < PX; ++e) t.v[e] = v[e];
        if (kStreamStores) st_vec_stream<T, PX>(p + x, t);
        else st_vec<T, PX>(p + x, t);
    } else {
#pragma unroll
        for (int e = 0; e < PX; ++e)
            if (ok[e]) p[x + e] = v[e];
    }
}

// ------------------------------------------------------------------- wave, adjoint
// u_bar[j] += 2 r_bar[j] [j in I] + q[j-1] - 2 q[j] + q[j+1],  q = c*r_bar on I, else 0.
template <class T, int PX, bool GUARD, bool UPREV>
__device__ __forceinline__ void adj_wave1d_segment(const Args1d &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const T *cg = static_cast<const T *>(a.a0);
    const T *rg = static_cast<const T *>(a.a1);
    T *ug = static_cast<T *>(a.o0);
    T *pg = static_cast<T *>(a.o1);
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T cv[PX], rv[PX], uv[PX], pv[PX];
    load_cells<T, PX, GUARD, true>(cg, x, n, cv);
    load_cells<T, PX, GUARD, true>(rg, x, n, rv);
    load_cells<T, PX, GUARD, true>(ug, x, n, uv);
    if (UPREV) load_cells<T, PX, GUARD, true>(pg, x, n, pv);
    const T hc = load_cell<T, GUARD>(cg, hx, n, lane), hr = load_cell<T, GUARD>(rg, hx, n, lane);
    T q[PX], rr[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const bool in = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
        ok[e] = GUARD ? (x + e < n) : true;
        rr[e] = in ? rv[e] : T(0);
        q[e] = in ? cv[e] * rv[e] : T(0);
    }
    const bool hin = GUARD ? (hx >= 1 && hx <= n - 2) : true;
    const T qh = hin ? hc * hr : T(0);
    T left, right;
    wave_neighbours<T, PX>(q, qh, lane, left, right);
    T out[PX], pout[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T l = e == 0 ? left : q[e - 1];
        const T r = e == PX - 1 ? right : q[e + 1];
        out[e] = uv[e] + ((T(-2) * q[e] + (l + r)) + T(2) * rr[e]);
        if (UPREV) pout[e] = pv[e] - rr[e];
    }
    store_cells<T, PX, GUARD>(ug, x, n, out, ok);
    if (UPREV) store_cells<T, PX, GUARD>(pg, x, n, pout, ok);
}

// -------------------------------------------------------------------- wave, primal
// r[i] = 2u[i] - u_prev[i] + c[i]*(u[i-1] - 2u[i] + u[i+1]) for i in I.
template <class T, int PX, bool GUARD>
__device__ __forceinline__ void pri_wave1d_segment(const Args1d &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const T *ug = static_cast<const T *>(a.a0);
    const T *pg = static_cast<const T *>(a.a1);
    const T *cg = static_cast<const T *>(a.a2);
    T *rg = static_cast<T *>(a.o0);
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T uv[PX], pv[PX], cv[PX];
    load_cells<T, PX, GUARD, true>(ug, x, n, uv);
    load_cells<T, PX, GUARD, true>(pg, x, n, pv);
    load_cells<T, PX, GUARD, true>(cg, x, n, cv);
    const T uh = load_cell<T, GUARD>(ug, hx, n, lane);
    T left, right;
    wave_neighbours<T, PX>(uv, uh, lane, left, right);
    T out[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T l = e == 0 ? left : uv[e - 1];
        const T r = e == PX - 1 ? right : uv[e + 1];
        ok[e] = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
        out[e] = T(2) * uv[e] - pv[e] + cv[e] * (T(-2) * uv[e] + (l + r));
    }
    store_cells<T, PX, GUARD>(rg, x, n, out, ok);
}

// ------------------------------------------------ three-point stencil, general weights
// primal   r[i] = c[i]*(w[-1] u[i-1] + w[0] u[i] + w[+1] u[i+1])            for i in I
// adjoint  u_bar[j] += W[-1] q[j-1] + W[0] q[j] + W[+1] q[j+1], q = c*r_bar on I, else 0,
// with W the mirrored table W[o] = w[-o] (paper Section 3.2: the worked example with
// weights (2,-3,4), whose outer weights trade places in the adjoint).  a.w holds the
// gather weights, i.e. w for the primal and W for the adjoint.
template <class T, int PX, bool GUARD, bool ADJ>
__device__ __forceinline__ void box1d_segment(const Args1d &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const T wm = (T)a.w[0], w0 = (T)a.w[1], wp = (T)a.w[2];
    const T *g0 = static_cast<const T *>(a.a0);      // adjoint: c      primal: u
    const T *g1 = static_cast<const T *>(a.a1);      // adjoint: r_bar  primal: c
    T *og = static_cast<T *>(a.o0);
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T v0[PX], v1[PX], vo[PX];
    load_cells<T, PX, GUARD, true>(g0, x, n, v0);
    load_cells<T, PX, GUARD, true>(g1, x, n, v1);
    if (ADJ) load_cells<T, PX, GUARD, true>(og, x, n, vo);
    T sh = load_cell<T, GUARD>(g0, hx, n, lane);
    if (ADJ) {
        const T h1 = load_cell<T, GUARD>(g1, hx, n, lane);
        const bool hin = GUARD ? (hx >= 1 && hx <= n - 2) : true;
        sh = hin ? sh * h1 : T(0);
    }
    T s[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const bool in = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
        if (ADJ) { s[e] = in ? v0[e] * v1[e] : T(0); ok[e] = GUARD ? (x + e < n) : true; }
        else     { s[e] = v0[e]; ok[e] = in; }
    }
    T left, right;
    wave_neighbours<T, PX>(s, sh, lane, left, right);
    T out[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T l = e == 0 ? left : s[e - 1];
        const T r = e == PX - 1 ? right : s[e + 1];
        const T sum = (wm * l + w0 * s[e]) + wp * r;
        out[e] = ADJ ? vo[e] + sum : v1[e] * sum;
    }
    store_cells<T, PX, GUARD>(og, x, n, out, ok);
}

// ----------------------------------------------------------------- Burgers, primal
template <class T> __device__ __forceinline__ T pos_part(T v) { return v > T(0) ? v : T(0); }
template <class T> __device__ __forceinline__ T neg_part(T v) { return v < T(0) ? v : T(0); }

// KEEP_ENDS: the two end cells, which no iteration writes, receive the input's end values
// (boundary data held fixed from one state of a time loop to the next).
template <class T, int PX, bool GUARD, bool KEEP_ENDS = false>
__device__ __forceinline__ void pri_burgers_segment(const Args1d &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const T C = (T)a.C, D = (T)a.D;
    const T *ug = static_cast<const T *>(a.a0);
    T *rg = static_cast<T *>(a.o0);
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T uv[PX];
    load_cells<T, PX, GUARD, true>(ug, x, n, uv);
    const T uh = load_cell<T, GUARD>(ug, hx, n, lane);
    T left, right;
    wave_neighbours<T, PX>(uv, uh, lane, left, right);
    T out[PX];
    bool ok[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T um = e == 0 ? left : uv[e - 1];
        const T up = e == PX - 1 ? right : uv[e + 1];
        const T u0 = uv[e];
        const bool in = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
        ok[e] = (GUARD && KEEP_ENDS) ? (x + e < n) : in;
        const T conv = pos_part(u0) * (u0 - um) + neg_part(u0) * (up - u0);
        const T val = u0 - C * conv + D * (um - T(2) * u0 + up);
        out[e] = (GUARD && KEEP_ENDS) ? (in ? val : u0) : val;
    }
    store_cells<T, PX, GUARD>(rg, x, n, out, ok);
}

// ---------------------------------------------------------------- Burgers, adjoint
// u_bar[j] += g_-(j+1) r_bar[j+1] [j+1 in I] + g_0(j) r_bar[j] [j in I] + g_+(j-1) r_bar[j-1] [j-1 in I]
//   g_-(i) = C max(u_i,0) + D,  g_+(i) = -C min(u_i,0) + D,
//   g_0(i) = 1 - 2D - C( [u_i>=0](u_i-u_{i-1}) + max(u_i,0) + [-u_i>=0](u_{i+1}-u_i) - min(u_i,0) )
// The primal u is read at j-1, j, j+1 (shifted reads, Section 3.3.2).
// ASSIGN: u_bar[j] = (the three terms) instead of +=, for a time loop that recycles a
// buffer whose accumulated value is known to be zero (u_bar is then not read).
// The three terms of one u_bar[j]; (um, u0, up) = u[j-1], u[j], u[j+1], (rm, r0, rp) = r_bar at
// the same cells with zeros where the iteration does not exist.  One function with
// contraction into fused multiply-adds switched off, shared by the single-step kernel and the
// kernel that fuses several reverse steps of a time loop, so that both round every cell alike
// and the fused sweep reproduces the step-by-step sweep bit for bit.
template <class T> __device__ __forceinline__ T burgers_adjoint_terms(T um, T u0, T up, T rm, T r0, T rp, T C, T D, bool in0)
{
#pragma clang fp contract(off)
    const T dpos = u0 >= T(0) ? T(1) : T(0);
    const T dneg = -u0 >= T(0) ? T(1) : T(0);
    const T g0 = T(1) - C * (dpos * (u0 - um) + pos_part(u0) + dneg * (up - u0) - neg_part(u0)) - T(2) * D;
    const T from_right = (C * pos_part(up) + D) * rp;      // iteration j+1 read u[j] as its left cell
    const T from_left = (-C * neg_part(um) + D) * rm;      // iteration j-1 read u[j] as its right cell
    return from_right + (in0 ? g0 * r0 : T(0)) + from_left;
}

template <class T, int PX, bool GUARD, bool ASSIGN>
__device__ __forceinline__ void adj_burgers_segment(const Args1d &a, long xs, int lane)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const T C = (T)a.C, D = (T)a.D;
    const T *ug = static_cast<const T *>(a.a0);
    const T *rg = static_cast<const T *>(a.a1);
    T *bg = static_cast<T *>(a.o0);
    const long x = xs + (long)lane * PX;
    const long hx = lane < 32 ? xs - 1 : xs + W;
    T uv[PX], rv[PX], bv[PX];
    load_cells<T, PX, GUARD, true>(ug, x, n, uv);
    load_cells<T, PX, GUARD, true>(rg, x, n, rv);
    if (!ASSIGN) load_cells<T, PX, GUARD, true>(bg, x, n, bv);
    const T uh = load_cell<T, GUARD>(ug, hx, n, lane);
    T rh = load_cell<T, GUARD>(rg, hx, n, lane);
    bool ok[PX], in[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        in[e] = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
        ok[e] = GUARD ? (x + e < n) : true;
        rv[e] = in[e] ? rv[e] : T(0);       // r_bar outside I is never used
    }
    if (GUARD) rh = (hx >= 1 && hx <= n - 2) ? rh : T(0);
    T ul, ur, rl, rr;
    wave_neighbours<T, PX>(uv, uh, lane, ul, ur);
    wave_neighbours<T, PX>(rv, rh, lane, rl, rr);
    T out[PX];
#pragma unroll
    for (int e = 0; e < PX; ++e) {
        const T um = e == 0 ? ul : uv[e - 1];
        const T up = e == PX - 1 ? ur : uv[e + 1];
        const T rm = e == 0 ? rl : rv[e - 1];
        const T rp = e == PX - 1 ? rr : rv[e + 1];
        const T terms = burgers_adjoint_terms(um, uv[e], up, rm, rv[e], rp, C, D, in[e]);
        out[e] = ASSIGN ? terms : bv[e] + terms;
    }
    store_cells<T, PX, GUARD>(bg, x, n, out, ok);
}

// ------------------------------------------- Burgers, several reverse steps in one pass
// A reverse sweep over stored states applies lam <- J(u^t)^T lam for t = T, T-1, ...; done
// step by step each application reads u^t and lam and writes lam: 24 bytes per cell and step
// (fp64).  Here a wave applies M consecutive steps to a window of cells held in registers:
// lam is read once, the M states once each, lam written once -- (16 + 8M)/M bytes per cell and
// step.  A cell's value after k steps depends on k cells to either side, so a window of W cells
// yields W - 2H finished cells (H >= M, a multiple of the cells per lane so that whole lanes
// are either finished or not); neighbouring windows overlap by 2H cells, which are computed
// twice.  All M steps are in assign mode (the target starts from zero), as from the second
// step of a sweep on; lam outside I is never used (masked to zero at every step).  Input and
// output must be different buffers (windows read cells their neighbours write): M is odd, so
// the alternating buffers of the sweep stay in step.
constexpr int kFuseM = 5;        // reverse steps per pass
constexpr int kFuseH = 8;        // cells recomputed on either side of a window

struct FusedArgs {
    const void *u[kFuseM];       // states of the steps in the order they are applied: u^t, u^{t-1}, ...
    const void *lam_in;
    void *lam_out;
    long n;
    double C, D;
    long core_lo, core_hi;       // windows core_lo .. core_hi-1 need no guard
    long core_blocks, nwin;
};

template <class T, bool GUARD>
__device__ __forceinline__ void adj_burgers_fused_window(const FusedArgs &a, long w, int lane)
{
    constexpr int PXL = 32 / (int)sizeof(T);            // cells per lane: two 16-byte accesses
    constexpr int PXV = 16 / (int)sizeof(T);
    constexpr int W = 64 * PXL, V = W - 2 * kFuseH;
    const long n = a.n;
    const T C = (T)a.C, D = (T)a.D;
    const long x = w * V - kFuseH + (long)lane * PXL;  // first cell of this lane (may lie outside the array)
    auto load = [&](const void *base, T (&v)[PXL]) {
        const T *p = static_cast<const T *>(base);
        if (!GUARD) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const Vec<T, PXV> t = ld_vec_stream<T, PXV>(p + x + h * PXV);
#pragma unroll
                for (int e = 0; e < PXV; ++e) v[h * PXV + e] = t.v[e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < PXL; ++e) {
                long i = x + e;
                i = i < 0 ? 0 : (i > n - 1 ? n - 1 : i);
                v[e] = p[i];
            }
        }
    };
    bool in[PXL];
#pragma unroll
    for (int e = 0; e < PXL; ++e) in[e] = GUARD ? (x + e >= 1 && x + e <= n - 2) : true;
    T lam[PXL], uv[kFuseM][PXL];
    load(a.lam_in, lam);
#pragma unroll
    for (int s = 0; s < kFuseM; ++s) load(a.u[s], uv[s]);
#pragma unroll
    for (int s = 0; s < kFuseM; ++s) {
#pragma unroll
        for (int e = 0; e < PXL; ++e) lam[e] = in[e] ? lam[e] : T(0);      // lam outside I is never used
        // neighbours across lanes; the window's two end lanes get zeros, which only reach cells
        // that are discarded
        T ul = __shfl_up(uv[s][PXL - 1], 1), ur = __shfl_down(uv[s][0], 1);
        T ll = __shfl_up(lam[PXL - 1], 1), lr = __shfl_down(lam[0], 1);
        ul = lane == 0 ? T(0) : ul;  ll = lane == 0 ? T(0) : ll;
        ur = lane == 63 ? T(0) : ur; lr = lane == 63 ? T(0) : lr;
        T next[PXL];
#pragma unroll
        for (int e = 0; e < PXL; ++e) {
            const T um = e == 0 ? ul : uv[s][e - 1];
            const T up = e == PXL - 1 ? ur : uv[s][e + 1];
            const T rm = e == 0 ? ll : lam[e - 1];
            const T rp = e == PXL - 1 ? lr : lam[e + 1];
            next[e] = burgers_adjoint_terms(um, uv[s][e], up, rm, lam[e], rp, C, D, in[e]);
        }
#pragma unroll
        for (int e = 0; e < PXL; ++e) lam[e] = next[e];
    }
    T *out = static_cast<T *>(a.lam_out);
    if (!GUARD) {
        if (lane >= kFuseH / PXL && lane < 64 - kFuseH / PXL) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                Vec<T, PXV> t;
#pragma unroll
                for (int e = 0; e < PXV; ++e) t.v[e] = lam[h * PXV + e];
                st_vec_stream<T, PXV>(out + x + h * PXV, t);
            }
        }
    } else {
#pragma unroll
        for (int e = 0; e < PXL; ++e) {
            const long i = x + e;
            if (i >= w * V && i < (w + 1) * V && i < n) out[i] = lam[e];
        }
    }
}

template <class T>
__global__ __launch_bounds__(64 * kWaves1d) void adj_burgers_fused_kernel(FusedArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long b = blockIdx.x;
    if (b < a.core_blocks) {                       // block-uniform; no barrier in this kernel
        const long w = a.core_lo + b * kWaves1d + wave;
        if (w >= a.core_hi) return;
        adj_burgers_fused_window<T, false>(a, w, lane);
    } else {
        // remainder windows: 0 .. core_lo-1 and core_hi .. nwin-1
        long k = (b - a.core_blocks) * kWaves1d + wave;
        const long w = k < a.core_lo ? k : a.core_hi + (k - a.core_lo);
        if (w >= a.nwin) return;
        adj_burgers_fused_window<T, true>(a, w, lane);
    }
}

static inline bool aligned16_1d(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <class T>
static hipError_t launch_fused_T(FusedArgs a, hipStream_t stream)
{
    constexpr int PXL = 32 / (int)sizeof(T);
    constexpr int W = 64 * PXL, V = W - 2 * kFuseH;
    a.nwin = (a.n + V - 1) / V;
    // core window w: all its cells w*V-H .. w*V-H+W-1 lie in I = [1, n-2]
    a.core_lo = 1;
    a.core_hi = (a.n - 2 - W + 1 + kFuseH) / V + 1;          // largest w with w*V - H + W - 1 <= n-2, plus one
    if (a.n - 2 - W + 1 + kFuseH < V) a.core_hi = 1;         // no core window
    if (a.core_hi > a.nwin) a.core_hi = a.nwin;
    if (a.core_hi < a.core_lo) a.core_hi = a.core_lo;
    a.core_blocks = (a.core_hi - a.core_lo + kWaves1d - 1) / kWaves1d;
    const long rem = a.nwin - (a.core_hi - a.core_lo);
    const long blocks = a.core_blocks + (rem + kWaves1d - 1) / kWaves1d;
    if (blocks > 0x7fffffffL) return hipErrorNotSupported;
    hipLaunchKernelGGL((adj_burgers_fused_kernel<T>), dim3((unsigned)blocks), dim3(64 * kWaves1d), 0, stream, a);
    return hipGetLastError();
}

int burgers_fused_steps() { return kFuseM; }

// kFuseM reverse steps in assign mode: lam_out = J(u[M-1])^T ... J(u[0])^T lam_in.
// hipErrorNotSupported (nothing enqueued) if an array is not 16-byte aligned.
hipError_t launch_adjoint_burgers1d_fused(int is_f64, long n, double C, double D, const void *const *u,
                                          const void *lam_in, void *lam_out, hipStream_t stream)
{
    FusedArgs a{};
    for (int s = 0; s < kFuseM; ++s) {
        a.u[s] = u[s];
        if (!aligned16_1d(u[s])) return hipErrorNotSupported;
    }
    if (!aligned16_1d(lam_in) || !aligned16_1d(lam_out)) return hipErrorNotSupported;
    a.lam_in = lam_in; a.lam_out = lam_out; a.n = n; a.C = C; a.D = D;
    return is_f64 ? launch_fused_T<double>(a, stream) : launch_fused_T<float>(a, stream);
}

// -------------------------------------------------------------------------- kernels
template <class T, int PX, bool GUARD, int OP>
__device__ __forceinline__ void run_segment(const Args1d &a, long xs, int lane)
{
    if (OP == OP_ADJ_WAVE) adj_wave1d_segment<T, PX, GUARD, false>(a, xs, lane);
    else if (OP == OP_ADJ_WAVE_UPREV) adj_wave1d_segment<T, PX, GUARD, true>(a, xs, lane);
    else if (OP == OP_PRI_WAVE) pri_wave1d_segment<T, PX, GUARD>(a, xs, lane);
    else if (OP == OP_PRI_BURGERS) pri_burgers_segment<T, PX, GUARD>(a, xs, lane);
    else if (OP == OP_PRI_BURGERS_KEEP_ENDS) pri_burgers_segment<T, PX, GUARD, true>(a, xs, lane);
    else if (OP == OP_ADJ_BOX) box1d_segment<T, PX, GUARD, true>(a, xs, lane);
    else if (OP == OP_PRI_BOX) box1d_segment<T, PX, GUARD, false>(a, xs, lane);
    else if (OP == OP_ADJ_BURGERS_ASSIGN) adj_burgers_segment<T, PX, GUARD, true>(a, xs, lane);
    else adj_burgers_segment<T, PX, GUARD, false>(a, xs, lane);
}

template <class T, int PX, int OP>
__global__ __launch_bounds__(64 * kWaves1d) void stencil1d_kernel(Args1d a)
{
    constexpr int W = 64 * PX;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long b = blockIdx.x;
    if (b < a.core_blocks) {                       // block-uniform; no barrier in this kernel
        const long local = b * kWaves1d + wave;
        if (local >= a.core_segs) return;
        run_segment<T, PX, false, OP>(a, (1 + local) * W, lane);
    } else {
        const long local = (b - a.core_blocks) * kWaves1d + wave;
        if (local >= a.rem_segs) return;
        const long seg = local == 0 ? 0 : a.core_segs + local;
        run_segment<T, PX, true, OP>(a, seg * W, lane);
    }
}

// Core: segments 1 .. s_hi (all reads inside I, whole vectors inside the array).
// Remainder: segment 0 and segments s_hi+1 .. nseg-1.
template <class T, int PX, int OP>
static hipError_t launch_1d(Args1d a, hipStream_t stream)
{
    constexpr int W = 64 * PX;
    const long n = a.n;
    const long nseg = (n + W - 1) / W;
    long s_hi = (n - 2) / W - 1;                  // last segment with xs + W <= n-2
    if (s_hi < 1) s_hi = 0;                       // no core segment
    a.core_segs = s_hi;
    a.core_blocks = (a.core_segs + kWaves1d - 1) / kWaves1d;
    a.rem_segs = 1 + (nseg - 1 - s_hi);
    const long rem_blocks = (a.rem_segs + kWaves1d - 1) / kWaves1d;
    dim3 grid((unsigned)(a.core_blocks + rem_blocks));
    hipLaunchKernelGGL((stencil1d_kernel<T, PX, OP>), grid, dim3(64 * kWaves1d), 0, stream, a);
    return hipGetLastError();
}

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

template <int OP>
static hipError_t dispatch_1d(int is_f64, const Args1d &a, hipStream_t stream)
{
    const bool al = aligned16(a.a0) && aligned16(a.a1) && aligned16(a.a2) && aligned16(a.o0) && aligned16(a.o1);
    if (is_f64) return al ? launch_1d<double, 2, OP>(a, stream) : launch_1d<double, 1, OP>(a, stream);
    return al ? launch_1d<float, 4, OP>(a, stream) : launch_1d<float, 1, OP>(a, stream);
}

hipError_t launch_adjoint_wave1d(int is_f64, long n, const void *c, const void *r_bar, void *u_bar,
                                 void *u_prev_bar, hipStream_t stream)
{
    Args1d a{};
    a.a0 = c; a.a1 = r_bar; a.o0 = u_bar; a.o1 = u_prev_bar; a.n = n;
    return u_prev_bar ? dispatch_1d<OP_ADJ_WAVE_UPREV>(is_f64, a, stream)
                      : dispatch_1d<OP_ADJ_WAVE>(is_f64, a, stream);
}
hipError_t launch_primal_wave1d(int is_f64, long n, const void *u, const void *u_prev, const void *c,
                                void *r, hipStream_t stream)
{
    Args1d a{};
    a.a0 = u; a.a1 = u_prev; a.a2 = c; a.o0 = r; a.n = n;
    return dispatch_1d<OP_PRI_WAVE>(is_f64, a, stream);
}
hipError_t launch_adjoint_burgers1d(int is_f64, long n, double C, double D, const void *u,
                                    const void *r_bar, void *u_bar, int assign, hipStream_t stream)
{
    Args1d a{};
    a.a0 = u; a.a1 = r_bar; a.o0 = u_bar; a.n = n; a.C = C; a.D = D;
    return assign ? dispatch_1d<OP_ADJ_BURGERS_ASSIGN>(is_f64, a, stream) : dispatch_1d<OP_ADJ_BURGERS>(is_f64, a, stream);
}
hipError_t launch_primal_burgers1d(int is_f64, long n, double C, double D, const void *u, void *r,
                                   hipStream_t stream, int keep_ends)
{
    Args1d a{};
    a.a0 = u; a.o0 = r; a.n = n; a.C = C; a.D = D;
    return keep_ends ? dispatch_1d<OP_PRI_BURGERS_KEEP_ENDS>(is_f64, a, stream) : dispatch_1d<OP_PRI_BURGERS>(is_f64, a, stream);
}

hipError_t launch_box1d(int adjoint, int is_f64, long n, const double *w, const void *in0, const void *in1,
                        void *out, hipStream_t stream)
{
    Args1d a{};
    a.a0 = in0; a.a1 = in1; a.o0 = out; a.n = n;
    a.w[0] = w[0]; a.w[1] = w[1]; a.w[2] = w[2];
    return adjoint ? dispatch_1d<OP_ADJ_BOX>(is_f64, a, stream) : dispatch_1d<OP_PRI_BOX>(is_f64, a, stream);
}

}  // namespace sadj
