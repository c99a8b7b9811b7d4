// The library's own 1-D stencils expressed as functors of the generic three-point
// stencil kernel (include/sadj_stencil1d.hpp): the loop body and its partial derivatives
// are the only stencil-specific code, the kernel body is shared (paper Section 3.3.1,
// uninterpreted loop-body function and derivative calls).
#include "../../include/sadj_stencil1d.hpp"
#include "launch.hpp"

namespace sadj {

// Upwinded Burgers step (Section 4.2):
//   f = u0 - C (max(u0,0)(u0-um) + min(u0,0)(up-u0)) + D (um - 2 u0 + up);
// max/min differentiate to the indicator functions [u0 >= 0], [-u0 >= 0] as in the
// paper's printed adjoint.
template <class T> struct BurgersUpwind {
    static constexpr bool uses_passive = false;
    static constexpr bool df_uses_u = true;
    T C, D;
    __device__ __forceinline__ T f(T um, T u0, T up, T) const
    {
        const T pos = u0 > T(0) ? u0 : T(0), neg = u0 < T(0) ? u0 : T(0);
        return u0 - C * (pos * (u0 - um) + neg * (up - u0)) + D * (um - T(2) * u0 + up);
    }
    __device__ __forceinline__ void df(T um, T u0, T up, T, T &dm, T &d0, T &dp) const
    {
        const T pos = u0 > T(0) ? u0 : T(0), neg = u0 < T(0) ? u0 : T(0);
        const T dpos = u0 >= T(0) ? T(1) : T(0), dneg = -u0 >= T(0) ? T(1) : T(0);
        dm = C * pos + D;
        dp = -C * neg + D;
        d0 = T(1) - C * (dpos * (u0 - um) + pos + dneg * (up - u0) - neg) - T(2) * D;
    }
};

// Linear three-point stencil with free weights and a passive coefficient (Section 3.2's
// worked example has weights (2,-3,4)):  f = p (wm um + w0 u0 + wp up).
template <class T> struct Weighted3 {
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = false;
    T wm, w0, wp;
    __device__ __forceinline__ T f(T um, T u0, T up, T p) const { return p * ((wm * um + w0 * u0) + wp * up); }
    __device__ __forceinline__ void df(T, T, T, T p, T &dm, T &d0, T &dp) const
    {
        dm = p * wm; d0 = p * w0; dp = p * wp;
    }
};

hipError_t launch_burgers1d_functor(int adjoint, int is_f64, long n, double C, double D, const void *u,
                                    const void *r_bar, void *out, hipStream_t stream)
{
    if (is_f64) {
        const BurgersUpwind<double> fn{C, D};
        return adjoint ? adjoint_stencil1d<double>(fn, n, (const double *)u, nullptr, (const double *)r_bar, (double *)out, stream)
                       : primal_stencil1d<double>(fn, n, (const double *)u, nullptr, (double *)out, stream);
    }
    const BurgersUpwind<float> fn{(float)C, (float)D};
    return adjoint ? adjoint_stencil1d<float>(fn, n, (const float *)u, nullptr, (const float *)r_bar, (float *)out, stream)
                   : primal_stencil1d<float>(fn, n, (const float *)u, nullptr, (float *)out, stream);
}

// w: PRIMAL weights at offsets -1, 0, +1 (the generic adjoint does the mirroring itself:
// the term of iteration i to u_bar[i-1] carries dm = p w[-1]).
hipError_t launch_weighted3_functor(int adjoint, int is_f64, long n, const double *w, const void *u,
                                    const void *c, const void *r_bar, void *out, hipStream_t stream)
{
    if (is_f64) {
        const Weighted3<double> fn{w[0], w[1], w[2]};
        return adjoint ? adjoint_stencil1d<double>(fn, n, (const double *)u, (const double *)c, (const double *)r_bar, (double *)out, stream)
                       : primal_stencil1d<double>(fn, n, (const double *)u, (const double *)c, (double *)out, stream);
    }
    const Weighted3<float> fn{(float)w[0], (float)w[1], (float)w[2]};
    return adjoint ? adjoint_stencil1d<float>(fn, n, (const float *)u, (const float *)c, (const float *)r_bar, (float *)out, stream)
                   : primal_stencil1d<float>(fn, n, (const float *)u, (const float *)c, (float *)out, stream);
}

}  // namespace sadj
