// Shared device/host helpers of libsadj (HIP, gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sadj {

// Central finite-difference weights of the second derivative on a unit grid
// (orders 2, 4, 6 and 8 for radius 1 .. 4), the nearest double of each rational; w(0) is the per-axis
// centre weight.
template <int R> __host__ __device__ constexpr double star_w(int k);
template <> __host__ __device__ constexpr double star_w<1>(int k) { return k == 0 ? -2.0 : 1.0; }
template <> __host__ __device__ constexpr double star_w<2>(int k)
{
    return k == 0 ? -5.0 / 2.0 : k == 1 ? 4.0 / 3.0 : -1.0 / 12.0;
}
template <> __host__ __device__ constexpr double star_w<3>(int k)
{
    return k == 0 ? -49.0 / 18.0 : k == 1 ? 3.0 / 2.0 : k == 2 ? -3.0 / 20.0 : 1.0 / 90.0;
}
template <> __host__ __device__ constexpr double star_w<4>(int k)
{
    return k == 0 ? -205.0 / 72.0
         : k == 1 ? 8.0 / 5.0
         : k == 2 ? -1.0 / 5.0
         : k == 3 ? 8.0 / 315.0
                  : -1.0 / 560.0;
}

// Workgroups are dealt to the 8 XCDs round-robin by their linear id, and each XCD
// has its own L2.  Map the hardware id to a logical id such that every XCD works
// on one contiguous range of logical ids (so that neighbouring tiles, which share
// halo cells, meet in the same L2).  Bijective for any total.
__host__ __device__ __forceinline__ int xcd_contiguous_id(int hw_id, int total)
{
    constexpr int NXCD = 8;
    const int xcd = hw_id % NXCD;
    const int idx = hw_id / NXCD;
    const int base = total / NXCD;
    const int rem = total % NXCD;
    const int start = xcd * base + (xcd < rem ? xcd : rem);
    return start + idx;
}

template <class T> __device__ __forceinline__ T ld_off(const T *base, uint32_t byte_off)
{
    return *reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + byte_off);
}


// N consecutive elements moved with one (up to 16-byte) memory instruction.
template <class T, int N> struct alignas(sizeof(T) * N) Vec { T v[N]; };

template <class T, int N> __device__ __forceinline__ Vec<T, N> ld_vec(const T *p)
{
    return *reinterpret_cast<const Vec<T, N> *>(p);
}
template <class T, int N> __device__ __forceinline__ void st_vec(T *p, const Vec<T, N> &v)
{
    *reinterpret_cast<Vec<T, N> *>(p) = v;
}

// Streaming (non-temporal) variants for data that is touched exactly once.
template <class T, int N> __device__ __forceinline__ Vec<T, N> ld_vec_stream(const T *p)
{
    typedef T VT __attribute__((ext_vector_type(N)));
    const VT t = __builtin_nontemporal_load(reinterpret_cast<const VT *>(p));
    Vec<T, N> r;
#pragma unroll
    for (int e = 0; e < N; ++e) r.v[e] = t[e];
    return r;
}
template <class T, int N> __device__ __forceinline__ void st_vec_stream(T *p, const Vec<T, N> &v)
{
    typedef T VT __attribute__((ext_vector_type(N)));
    VT t;
#pragma unroll
    for (int e = 0; e < N; ++e) t[e] = v.v[e];
    __builtin_nontemporal_store(t, reinterpret_cast<VT *>(p));
}

// Neighbour exchange inside a 64-lane wave whose lanes own PX consecutive elements
// each: left = element just before this lane's first, right = element just after
// its last.  `halo` holds, in lane 0, the element before the wave's segment and, in
// lane 63, the element after it.
template <class T, int PX>
__device__ __forceinline__ void wave_neighbours(const T (&v)[PX], T halo, int lane, T &left, T &right)
{
    const T from_left = __shfl_up(v[PX - 1], 1);
    const T from_right = __shfl_down(v[0], 1);
    left = lane == 0 ? halo : from_left;        // selects, so that left/right stay in registers
    right = lane == 63 ? halo : from_right;
}

// Row march of the 2-D strip kernels.  A wave steps through the input rows yi0 .. yi1 of its
// row chunk: single steps up to row pre_end, then `steady` groups of D branch-free steps,
// then single steps again.  The plan depends on the chunk only, not on the strip, so all
// waves of a workgroup (adjacent strips of one chunk) share it.  They meet at a workgroup
// barrier every kRowSync steady groups: left alone the waves drift apart by many rows, and
// keeping the eight adjacent strips within a few rows of each other makes the rows they
// stream contiguous pieces of memory (8192^2 fp64 adjoint 71.7 -> 74.3 % of peak, 8192 x
// 16384 65 -> 72 %).  Waves whose strip lies outside the grid do no work but still arrive at
// every barrier (row_march_idle), so the count of arrivals is the same for all.
struct RowMarch { int pre_end, steady; };
constexpr int kRowSync = 4;

__host__ __device__ __forceinline__ RowMarch plan_row_march(int yi0, int yi1, int lo, int hi, int D)
{
    // single steps until row lo is reached and the slot index is back at 0, or the rows run out
    int yi = yi0, d = 0;
    while (yi <= yi1 && (yi < lo || d != 0)) {
        ++yi;
        d = d + 1 == D ? 0 : d + 1;
    }
    RowMarch m;
    m.pre_end = yi;
    m.steady = hi - yi + 1 >= D ? (hi - yi + 1) / D : 0;     // groups yi .. yi+D-1 with yi+D-1 <= hi
    return m;
}

__device__ __forceinline__ void row_march_sync(int group)     // group = 1, 2, ... steady
{
    if (group % kRowSync == 0) __builtin_amdgcn_s_barrier();
}

__device__ __forceinline__ void row_march_idle(const RowMarch &m)
{
    for (int k = m.steady / kRowSync; k > 0; --k) __builtin_amdgcn_s_barrier();
}

}  // namespace sadj
