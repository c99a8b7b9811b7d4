// User-side stencils in two and three dimensions built on the public header alone
// (sadj_stencil_star.hpp): the bodies of star_bodies.py, written separately for the device.
//   kind 0  soft_wave     f = 2 v0 + p (1 + BETA v0^2) (sum of neighbours - 2 ndim v0)   (made up; nonlinear)
//   kind 1  pair_product  f = a b + p a,  a = u[x-1, y], b = u[x, y-1]   (2-D; the example of paper Section 3.3.1)
//   kind 2  lin_wave      f = 2 v0 + p (sum of neighbours - 2 ndim v0)   (the library's wave step without u_prev)
// No kernel is written here: a functor is all the generic kernels need.
#include "sadj_stencil_star.hpp"

template <class T, int ND> struct SoftWave {
    static constexpr int ndim = ND;
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = true;
    static constexpr int NREAD = 1 + 2 * ND;
    T beta;
    __device__ T lap(const T (&v)[NREAD]) const
    {
        T s = T(0);
#pragma unroll
        for (int k = 1; k < NREAD; ++k) s += v[k];
        return s - T(2 * ND) * v[0];
    }
    __device__ T f(const T (&v)[NREAD], T p) const { return T(2) * v[0] + p * (T(1) + beta * v[0] * v[0]) * lap(v); }
    __device__ void df(const T (&v)[NREAD], T p, T (&d)[NREAD]) const
    {
        const T g = T(1) + beta * v[0] * v[0];
#pragma unroll
        for (int k = 1; k < NREAD; ++k) d[k] = p * g;
        d[0] = T(2) + p * (T(2) * beta * v[0] * lap(v) - T(2 * ND) * g);
    }
};

template <class T> struct PairProduct {
    static constexpr int ndim = 2;
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = true;
    __device__ T f(const T (&v)[5], T p) const { return v[1] * v[3] + p * v[1]; }
    __device__ void df(const T (&v)[5], T p, T (&d)[5]) const
    {
        d[0] = T(0); d[1] = v[3] + p; d[2] = T(0); d[3] = v[1]; d[4] = T(0);
    }
};

template <class T, int ND> struct LinWave {
    static constexpr int ndim = ND;
    static constexpr bool uses_passive = true;
    static constexpr bool df_uses_u = false;
    static constexpr int NREAD = 1 + 2 * ND;
    __device__ T f(const T (&v)[NREAD], T p) const
    {
        T s = T(0);
#pragma unroll
        for (int k = 1; k < NREAD; ++k) s += v[k];
        return T(2) * v[0] + p * (s - T(2 * ND) * v[0]);
    }
    __device__ void df(const T (&)[NREAD], T p, T (&d)[NREAD]) const
    {
#pragma unroll
        for (int k = 1; k < NREAD; ++k) d[k] = p;
        d[0] = T(2) - T(2 * ND) * p;
    }
};

template <class T, class F>
static int run(const F &fn, int adjoint, int nx, int ny, int nz, const void *u, const void *p, const void *r_bar,
               void *out, hipStream_t st)
{
    if (adjoint)
        return (int)sadj::adjoint_star<T>(fn, nx, ny, nz, (const T *)u, (const T *)p, (const T *)r_bar, (T *)out, st);
    return (int)sadj::primal_star<T>(fn, nx, ny, nz, (const T *)u, (const T *)p, (T *)out, st);
}

template <class T>
static int pick(int kind, int adjoint, int ndim, int nx, int ny, int nz, const void *u, const void *p,
                const void *r_bar, void *out, hipStream_t st)
{
    const T beta = T(0.3);
    if (kind == 0 && ndim == 2) return run<T>(SoftWave<T, 2>{beta}, adjoint, nx, ny, 1, u, p, r_bar, out, st);
    if (kind == 0 && ndim == 3) return run<T>(SoftWave<T, 3>{beta}, adjoint, nx, ny, nz, u, p, r_bar, out, st);
    if (kind == 1 && ndim == 2) return run<T>(PairProduct<T>{}, adjoint, nx, ny, 1, u, p, r_bar, out, st);
    if (kind == 2 && ndim == 2) return run<T>(LinWave<T, 2>{}, adjoint, nx, ny, 1, u, p, r_bar, out, st);
    if (kind == 2 && ndim == 3) return run<T>(LinWave<T, 3>{}, adjoint, nx, ny, nz, u, p, r_bar, out, st);
    return (int)hipErrorInvalidValue;
}

// is_f64: 1 = double, 0 = float.  Device pointers; stream = hipStream_t.  Returns the hipError_t.
// Primal: out = r (u, p read).  Adjoint: out = u_bar (u, p, r_bar read; u may be NULL for kind 2).
extern "C" int star_example(int kind, int adjoint, int is_f64, int ndim, int nx, int ny, int nz, const void *u,
                            const void *p, const void *r_bar, void *out, void *stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (is_f64) return pick<double>(kind, adjoint, ndim, nx, ny, nz, u, p, r_bar, out, st);
    return pick<float>(kind, adjoint, ndim, nx, ny, nz, u, p, r_bar, out, st);
}
