// The library's own free-weight 7-point star (sadj_*_star3d, radius 1) written as a functor
// for the generic kernels of include/sadj_stencil_star.hpp (paper Section 3.3.1: loop body and
// partial derivatives as uninterpreted functions).  Option "star3d.functor" = 1 routes the
// radius-1 star calls through them, so that the hook is measured and parity-tested on a
// stencil the library also implements by hand.
#include "../../include/sadj_stencil_star.hpp"
#include "launch.hpp"

namespace sadj {

namespace {

// r = p * (w[0] v[0] + sum_k w[k] v[k]);  linear in u: the partials do not read u.
template <class T> struct WeightedStar7 {
    static constexpr int ndim = 3;
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = false;
    T w[7];                       // primal weights in read order: centre, x-1, x+1, y-1, y+1, z-1, z+1
    __device__ T f(const T (&v)[7], T p) const
    {
        T s = w[0] * v[0];
#pragma unroll
        for (int k = 1; k < 7; ++k) s += w[k] * v[k];
        return p * s;
    }
    __device__ void df(const T (&)[7], T p, T (&d)[7]) const
    {
#pragma unroll
        for (int k = 0; k < 7; ++k) d[k] = p * w[k];
    }
};

template <class T>
hipError_t run(int adjoint, int nx, int ny, int nz, const double *w, const void *in0, const void *in1, void *out,
               hipStream_t stream)
{
    WeightedStar7<T> fn;
    for (int k = 0; k < 7; ++k) fn.w[k] = (T)w[k];
    hipError_t e;
    if (adjoint)      // (c, r_bar) -> u_bar
        e = adjoint_star<T>(fn, nx, ny, nz, (const T *)nullptr, (const T *)in0, (const T *)in1, (T *)out, stream);
    else              // (u, c) -> r
        e = primal_star<T>(fn, nx, ny, nz, (const T *)in0, (const T *)in1, (T *)out, stream);
    // the header refuses what it cannot run (alignment, nx not a multiple of the vector width)
    return e == hipErrorInvalidValue ? hipErrorNotSupported : e;
}

}  // namespace

// w: the caller's PRIMAL weights, centre, then x-1, x+1, y-1, y+1, z-1, z+1.
hipError_t launch_star7_functor(int adjoint, int is_f64, int nx, int ny, int nz, const double *w, const void *in0,
                                const void *in1, void *out, hipStream_t stream)
{
    return is_f64 ? run<double>(adjoint, nx, ny, nz, w, in0, in1, out, stream)
                  : run<float>(adjoint, nx, ny, nz, w, in0, in1, out, stream);
}

}  // namespace sadj
