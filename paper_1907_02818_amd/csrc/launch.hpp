// Internal launcher interface between the C ABI (api.hip) and the kernel files.
#pragma once
#include <hip/hip_runtime.h>

namespace sadj {

struct LaunchOptions {
    long zchunk = 0;     // wave3d: output planes per workgroup (0 = automatic)
    long variant = 0;    // wave3d: tile-shape variant
    long ychunk2d = 0;   // wave2d: output rows per wave (0 = automatic)
    long variant2d = 0;  // wave2d: pipeline depth / workgroup size variant
    long xcd_map = 0;    // wave3d: workgroup id -> logical id (0 = automatic, see block_to_tile)
    long band = 0;       // wave3d: tile rows per band of the tile numbering (0 = rows of tiles)
    long lds_pad = 0;    // 3-D marches: dynamic LDS bytes requested to limit workgroups per CU (0 = automatic, -1 = none)
    long split = 0;      // 3-D marches: 0 = left-over tiles may be cut finer than the rest, 1 = all tiles cut alike
    long remainder = 0;  // wave3d adjoint: remainder strategy (0 guarded where needed, 1 guarded everywhere, 2 split dispatches)
};

hipError_t launch_adjoint_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                 const void *r_bar, void *u_bar, void *u_prev_bar, int u_prev_bar_assign,
                                 const LaunchOptions &opt, hipStream_t stream);
// Same result up to rounding; terms added in the order and rounding of the sequential scatter.
hipError_t launch_adjoint_wave3d_ordered(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                         const void *r_bar, void *u_bar, void *u_prev_bar,
                                         const LaunchOptions &opt, hipStream_t stream);
// Contrast baseline: conventional scatter with atomic updates (not the method).
hipError_t launch_adjoint_wave3d_scatter_atomic(int is_f64, int radius, int nx, int ny, int nz, const void *c,
                                                const void *r_bar, void *u_bar, hipStream_t stream);
// Two reverse steps of a time loop of radius-1 wave steps in one pass: with a = lam^{k+1},
// b = lam^k: out_a = lam^{k-1}, out_b = -(lam^k after the first step) on I, 0 elsewhere.  out_a and
// out_b must be arrays other than a and b.  hipErrorNotSupported (nothing enqueued) where
// adjoint_wave3d_pair_supported is false.
bool adjoint_wave3d_pair_supported(int is_f64, int nx, const void *c, const void *p0, const void *p1, const void *p2,
                                   const void *p3);
hipError_t launch_adjoint_wave3d_pair(int is_f64, int nx, int ny, int nz, const void *c, const void *a, const void *b,
                                      void *out_a, void *out_b, const LaunchOptions &opt, hipStream_t stream);
hipError_t launch_primal_wave3d(int is_f64, int radius, int nx, int ny, int nz, const void *u,
                                const void *u_prev, const void *c, void *r,
                                const LaunchOptions &opt, hipStream_t stream);

hipError_t launch_adjoint_wave2d(int is_f64, int nx, int ny, const void *c, const void *r_bar,
                                 void *u_bar, void *u_prev_bar, const LaunchOptions &opt, hipStream_t stream);
hipError_t launch_primal_wave2d(int is_f64, int nx, int ny, const void *u, const void *u_prev,
                                const void *c, void *r, const LaunchOptions &opt, hipStream_t stream);

hipError_t launch_adjoint_wave1d(int is_f64, long n, const void *c, const void *r_bar, void *u_bar,
                                 void *u_prev_bar, hipStream_t stream);
hipError_t launch_primal_wave1d(int is_f64, long n, const void *u, const void *u_prev, const void *c,
                                void *r, hipStream_t stream);

// assign != 0: u_bar = J^T r_bar (u_bar is not read) instead of u_bar += J^T r_bar
hipError_t launch_adjoint_burgers1d(int is_f64, long n, double C, double D, const void *u,
                                    const void *r_bar, void *u_bar, int assign, hipStream_t stream);
// burgers_fused_steps() consecutive reverse steps of a time loop in one pass, all in assign mode:
// lam_out = J(u[M-1])^T ... J(u[0])^T lam_in (u[0] is the state of the step applied first).
// lam_in and lam_out must differ.  hipErrorNotSupported (nothing enqueued) if an array is not
// 16-byte aligned.
int burgers_fused_steps();
hipError_t launch_adjoint_burgers1d_fused(int is_f64, long n, double C, double D, const void *const *u,
                                          const void *lam_in, void *lam_out, hipStream_t stream);

// keep_ends != 0: r[0] = u[0] and r[n-1] = u[n-1] as well (boundary data carried to the next state)
hipError_t launch_primal_burgers1d(int is_f64, long n, double C, double D, const void *u, void *r,
                                   hipStream_t stream, int keep_ends = 0);

// The same 1-D stencils as instantiations of the generic functor kernel
// (include/sadj_stencil1d.hpp); w = PRIMAL weights at offsets -1, 0, +1.
hipError_t launch_burgers1d_functor(int adjoint, int is_f64, long n, double C, double D, const void *u,
                                    const void *r_bar, void *out, hipStream_t stream);
hipError_t launch_weighted3_functor(int adjoint, int is_f64, long n, const double *w, const void *u,
                                    const void *c, const void *r_bar, void *out, hipStream_t stream);

// The radius-1 free-weight star through the generic functor kernels of
// include/sadj_stencil_star.hpp; w = the caller's PRIMAL weights (centre, x-1, x+1, y-1, y+1,
// z-1, z+1).  hipErrorNotSupported (nothing enqueued) if nx or the alignment rule it out.
hipError_t launch_star7_functor(int adjoint, int is_f64, int nx, int ny, int nz, const double *w, const void *in0,
                                const void *in1, void *out, hipStream_t stream);

// 3-D star stencil with free weights; w0 / w[d][idx] is the gather table (mirrored by the caller
// for the adjoint), idx enumerating the offsets -R..-1, +1..+R of axis d.
hipError_t launch_star3d(int adjoint, int is_f64, int radius, int nx, int ny, int nz, double w0,
                         const double (*w)[8], const void *in0, const void *in1, void *out,
                         const LaunchOptions &opt, hipStream_t stream);

// Host-side view of how the 3-D adjoint decomposes a grid (for tests): fills plan[0..7] =
// tiles in x, tiles in y, tile width, tile height, workgroups, tiles of the first group,
// z-chunks per tile of the first group, z-chunks per tile of the others; and, if `tiles` is
// not null, for every workgroup id (tile x, tile y, first plane, one past the last plane).
void describe_march_plan(int is_f64, int radius, int nx, int ny, int nz, int with_u_prev_bar, const LaunchOptions &opt,
                         long *plan, int *tiles, long max_blocks);

// Streaming yardstick out[i] += a[i]*b[i] over n elements (two launch shapes, see probe.hip).
hipError_t launch_stream_probe(int is_f64, int shape, size_t n, const void *a, const void *b, void *out,
                               hipStream_t stream);

// Dense 3^d box stencils; w = gather weights (mirrored by the caller for the adjoint).
hipError_t launch_box1d(int adjoint, int is_f64, long n, const double *w, const void *in0, const void *in1,
                        void *out, hipStream_t stream);
hipError_t launch_box(int adjoint, int is_f64, int ndim, int nx, int ny, int nz, const double *w,
                      const void *in0, const void *in1, void *out, const LaunchOptions &opt, hipStream_t stream);

}  // namespace sadj
