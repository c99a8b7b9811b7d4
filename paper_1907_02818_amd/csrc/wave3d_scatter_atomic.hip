// Contrast kernel, not the method: the conventional scatter adjoint of the 3-D wave
// stencil (paper Sections 1 and 3.2) parallelised over primal iterations with atomic
// updates -- the baseline whose poor scaling the paper reports for OpenMP atomics
// (Section 4.1) -- so that the gather kernels can be compared with it on the same GPU.
// One thread per primal iteration i in I:
//     u_bar[i]         += (2 + 3 w_0 c[i]) r_bar[i]
//     u_bar[i + k e_d] += w_|k| c[i] r_bar[i]          k = -R..R, k != 0, d = x, y, z
// every update a hardware floating-point atomic add in device memory (vector memory
// instructions; requires ordinary, coarse-grained device allocations).  The order in
// which the 6R+1 updates of one element arrive is not fixed, so results differ in the
// last bits from run to run -- the property Section 3.5 contrasts with the gather.
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

template <class T, int R>
__global__ __launch_bounds__(256) void scatter_atomic_kernel(const T *__restrict__ c, const T *__restrict__ r_bar,
                                                             T *u_bar, int nx, int ny, int nz)
{
    const int x = R + blockIdx.x * 64 + (threadIdx.x & 63);
    const int y = R + blockIdx.y * 4 + (threadIdx.x >> 6);
    const int z = R + blockIdx.z;
    if (x >= nx - R || y >= ny - R || z >= nz - R) return;
    const size_t sy = (size_t)nx, sz = (size_t)nx * ny;
    const size_t i = x + sy * y + sz * z;
    const T rb = r_bar[i];
    const T q = c[i] * rb;
    unsafeAtomicAdd(u_bar + i, T(2) * rb + T(3.0 * star_w<R>(0)) * q);
#pragma unroll
    for (int k = 1; k <= R; ++k) {
        const T t = T(star_w<R>(k)) * q;
        unsafeAtomicAdd(u_bar + i - k, t);
        unsafeAtomicAdd(u_bar + i + k, t);
        unsafeAtomicAdd(u_bar + i - k * sy, t);
        unsafeAtomicAdd(u_bar + i + k * sy, t);
        unsafeAtomicAdd(u_bar + i - k * sz, t);
        unsafeAtomicAdd(u_bar + i + k * sz, t);
    }
}

template <class T, int R>
static hipError_t launch_scatter_T(int nx, int ny, int nz, const void *c, const void *r_bar, void *u_bar,
                                   hipStream_t stream)
{
    const int ix = nx - 2 * R, iy = ny - 2 * R, iz = nz - 2 * R;   // extents of I, all >= 1
    if (iz > 65535 || (iy + 3) / 4 > 65535) return hipErrorNotSupported;
    dim3 grid((ix + 63) / 64, (iy + 3) / 4, iz), block(256);
    hipLaunchKernelGGL((scatter_atomic_kernel<T, R>), grid, block, 0, stream, static_cast<const T *>(c),
                       static_cast<const T *>(r_bar), static_cast<T *>(u_bar), nx, ny, nz);
    return hipGetLastError();
}

hipError_t launch_adjoint_wave3d_scatter_atomic(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                                const void *r_bar, void *u_bar, hipStream_t stream)
{
    if (is_f64) {
        switch (radius) {
        case 1: return launch_scatter_T<double, 1>(nx, ny, nz, c, r_bar, u_bar, stream);
        case 2: return launch_scatter_T<double, 2>(nx, ny, nz, c, r_bar, u_bar, stream);
        case 3: return launch_scatter_T<double, 3>(nx, ny, nz, c, r_bar, u_bar, stream);
        default: return launch_scatter_T<double, 4>(nx, ny, nz, c, r_bar, u_bar, stream);
        }
    }
    switch (radius) {
    case 1: return launch_scatter_T<float, 1>(nx, ny, nz, c, r_bar, u_bar, stream);
    case 2: return launch_scatter_T<float, 2>(nx, ny, nz, c, r_bar, u_bar, stream);
    case 3: return launch_scatter_T<float, 3>(nx, ny, nz, c, r_bar, u_bar, stream);
    default: return launch_scatter_T<float, 4>(nx, ny, nz, c, r_bar, u_bar, stream);
    }
}

}  // namespace sadj
