// A user-side stencil built on the public header alone: a made-up nonlinear three-point
// loop body with a passive coefficient,
//     f(um, u0, up, p) = u0 + p (sin(up) - sin(um)) u0 + um up / 2,
// and its hand-derived partials (the derivative of sin is the statement-level rule of
// paper Section 3.1).  No kernel is written here: the functor is all the generic
// primal / gather-adjoint kernels of sadj_stencil1d.hpp need (Section 3.3.1).
#include "sadj_stencil1d.hpp"

template <class T> struct SineFlux {
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = true;
    __device__ T f(T um, T u0, T up, T p) const { return u0 + p * (sin(up) - sin(um)) * u0 + T(0.5) * um * up; }
    __device__ void df(T um, T u0, T up, T p, T &dm, T &d0, T &dp) const
    {
        dm = -p * cos(um) * u0 + T(0.5) * up;
        d0 = T(1) + p * (sin(up) - sin(um));
        dp = p * cos(up) * u0 + T(0.5) * um;
    }
};

// is_f64: 1 = double, 0 = float.  Device pointers; stream = hipStream_t.  Returns the hipError_t.
extern "C" int sine_flux_primal(int is_f64, long n, const void *u, const void *p, void *r, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (is_f64) return (int)sadj::primal_stencil1d<double>(SineFlux<double>{}, n, (const double *)u, (const double *)p, (double *)r, st);
    return (int)sadj::primal_stencil1d<float>(SineFlux<float>{}, n, (const float *)u, (const float *)p, (float *)r, st);
}

extern "C" int sine_flux_adjoint(int is_f64, long n, const void *u, const void *p, const void *r_bar, void *u_bar,
                                 void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (is_f64)
        return (int)sadj::adjoint_stencil1d<double>(SineFlux<double>{}, n, (const double *)u, (const double *)p,
                                                    (const double *)r_bar, (double *)u_bar, st);
    return (int)sadj::adjoint_stencil1d<float>(SineFlux<float>{}, n, (const float *)u, (const float *)p,
                                               (const float *)r_bar, (float *)u_bar, st);
}
