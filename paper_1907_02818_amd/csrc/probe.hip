// Streaming yardstick with the adjoint kernels' access mix: two arrays read, one array
// read and written, every element touched once, no reuse and no halo:
//     out[i] += a[i] * b[i] .
// It bounds what any kernel with that mix of streams can reach on this memory system; the
// benchmark reports the adjoint kernels against it next to the nominal HBM peak.
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

// VB = bytes per lane and memory instruction; UNR vectors per thread, a workgroup of WG threads
// covers a contiguous piece of WG*UNR vectors; NT = streaming (non-temporal) loads and stores:
// 0 none, 1 all arrays, 2 `out` only.
template <class T, int VB, int UNR, int NT, int WG>
__global__ __launch_bounds__(WG) void stream_probe_kernel(const T *__restrict__ a, const T *__restrict__ b,
                                                          T *__restrict__ out, size_t n)
{
    constexpr int N = VB / (int)sizeof(T);
    using V = Vec<T, N>;
    const size_t nvec = n / N;
    const size_t base = (size_t)blockIdx.x * WG * UNR + threadIdx.x;
    V va[UNR], vb[UNR], vo[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = base + (size_t)u * WG;
        if (i < nvec) {
            va[u] = NT == 1 ? ld_vec_stream<T, N>(a + i * N) : ld_vec<T, N>(a + i * N);
            vb[u] = NT == 1 ? ld_vec_stream<T, N>(b + i * N) : ld_vec<T, N>(b + i * N);
            vo[u] = NT ? ld_vec_stream<T, N>(out + i * N) : ld_vec<T, N>(out + i * N);
        }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
        const size_t i = base + (size_t)u * WG;
        if (i < nvec) {
#pragma unroll
            for (int e = 0; e < N; ++e) vo[u].v[e] += va[u].v[e] * vb[u].v[e];
            if (NT) st_vec_stream<T, N>(out + i * N, vo[u]);
            else st_vec<T, N>(out + i * N, vo[u]);
        }
    }
    // the last n % N elements
    if (blockIdx.x == 0 && threadIdx.x < n - nvec * N) {
        const size_t i = nvec * N + threadIdx.x;
        out[i] += a[i] * b[i];
    }
}

template <class T, int VB, int UNR, int NT, int WG>
static hipError_t launch_probe(const void *a, const void *b, void *out, size_t n, hipStream_t stream)
{
    constexpr int N = VB / (int)sizeof(T);
    const size_t nvec = n / N;
    const size_t blocks = (nvec + WG * UNR - 1) / (WG * UNR);
    if (blocks > 0x7fffffffu) return hipErrorNotSupported;
    hipLaunchKernelGGL((stream_probe_kernel<T, VB, UNR, NT, WG>), dim3((unsigned)(blocks ? blocks : 1)), dim3(WG), 0, stream,
                       static_cast<const T *>(a), static_cast<const T *>(b), static_cast<T *>(out), n);
    return hipGetLastError();
}

hipError_t launch_stream_probe(int is_f64, int shape, size_t n, const void *a, const void *b, void *out,
                               hipStream_t stream)
{
    // shape 0: 256 threads, 8 bytes per lane, one vector per thread; shape 1: 256 threads, 16 bytes
    // per lane, four vectors per thread, streaming hints; shape 2: single-wave workgroups, one
    // 16-byte vector per lane and array, streaming hints on `out` only -- the fastest found in a
    // sweep of workgroup sizes 64..1024, 1..8 vectors per thread, contiguous pieces of 1..256 KB per
    // workgroup, persistent workgroups walking regions of their own, and either order of
    // workgroup ids over the XCDs (6.4-6.6 TB/s where shape 1 measured 6.0-6.2)
    if (is_f64) return shape == 0 ? launch_probe<double, 8, 1, 0, 256>(a, b, out, n, stream)
                     : shape == 1 ? launch_probe<double, 16, 4, 1, 256>(a, b, out, n, stream)
                                  : launch_probe<double, 16, 1, 2, 64>(a, b, out, n, stream);
    return shape == 0 ? launch_probe<float, 8, 1, 0, 256>(a, b, out, n, stream)
         : shape == 1 ? launch_probe<float, 16, 4, 1, 256>(a, b, out, n, stream)
                      : launch_probe<float, 16, 1, 2, 64>(a, b, out, n, stream);
}

}  // namespace sadj
