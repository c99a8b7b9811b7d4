/*
 * sadj.h -- C ABI of libsadj: primal stencil loops and their gather-form adjoints
 * on one AMD MI355X (gfx950).
 *
 * Problem statement (paper Sections 3.2 and 3.3): a primal stencil loop computes
 *     r[i] = f(u[i+o_1], ..., u[i+o_M]; passive data)        for i in I
 * on a dense 1-, 2- or 3-D grid.  Its reverse-mode adjoint is
 *     u_bar += (dr/du)^T r_bar .
 * Conventional AD writes that as a scatter u_bar[i+o] += ... over i in I, which
 * races when parallelised.  Every sadj_adjoint_* call instead evaluates the
 * index-shifted gather form (Section 3.3.2): each element of u_bar is produced by
 * exactly one GPU thread, which sums the terms (df_{j-o}/du_j) * r_bar[j-o] over the
 * offsets o whose primal iteration j-o exists (j-o in I).  No atomics are used and
 * the result is bitwise reproducible from run to run (Section 3.5).  The grid is
 * covered by a core region, where all terms exist (Section 3.3.3), and by boundary /
 * remainder regions, where a subset exists (Section 3.3.4); the regions are
 * disjoint, so they need no ordering among themselves.
 *
 * General conventions
 *  - Every array argument is a DEVICE pointer owned by the caller; it must stay valid
 *    until the work queued on `stream` has finished.  The library allocates nothing
 *    and keeps no reference after the work has run.
 *  - Arrays are dense with x fastest: element (x,y,z) lives at x + nx*(y + ny*z);
 *    every array of a call has nx*ny*nz elements of the call's dtype.
 *  - Primal iteration space: I = prod_d [R, n_d-1-R] with R the stencil radius
 *    (the paper's loop bounds [1,n-2] for R=1).  Every extent must be >= 2R+1,
 *    otherwise SADJ_ERR_SIZE.  Grids whose core region is empty (n_d < 4R+1) are valid.
 *    Limits: nx*ny <= 2^28 elements and every extent <= 2^30.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    are asynchronous: they enqueue kernels and return.
 *  - Primal calls ASSIGN r on I and leave r outside I untouched.
 *  - Adjoint calls ACCUMULATE into u_bar (and u_prev_bar) over the whole grid;
 *    r_bar is read only; values of r_bar, c (and u_prev) outside I never influence
 *    the result, not even when they are NaN.  c is passive: there is no c_bar.
 *  - An output array must not overlap any input array of the same call (Section 3.4:
 *    read and write sets are disjoint) -> SADJ_ERR_ALIAS.
 *  - Errors are return codes; argument checks happen before anything is enqueued, so
 *    a failed call has no effect.  No function throws or aborts.
 *  - Calls may be made from several threads at once; one GPU (the current HIP device of the
 *    calling thread).  The launch options (sadj_set_option) are process-wide, not per thread or
 *    per call: every call works with one consistent snapshot of them, taken when it starts, so
 *    two threads cannot use different settings at the same time, and an option changed while
 *    calls are being made applies to the calls that start afterwards.
 *
 * Star Laplacian weights (standard central second-derivative weights, centre first):
 * R=1: (-2, 1); R=2: (-5/2, 4/3, -1/12); R=3: (-49/18, 3/2, -3/20, 1/90);
 * R=4: (-205/72, 8/5, -1/5, 8/315, -1/560) per axis; the centre weight is multiplied by
 * the number of dimensions.  Grid spacing and time step are folded into c.
 */
#ifndef SADJ_H
#define SADJ_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SADJ_OK = 0,
    SADJ_ERR_NULL = 1,        /* a required pointer is NULL                              */
    SADJ_ERR_SIZE = 2,        /* an extent is < 2R+1 or above the documented limits, or
                                 (sadj_check_array) an array runs past its allocation    */
    SADJ_ERR_ALIAS = 3,       /* an output array overlaps an input array                 */
    SADJ_ERR_UNSUPPORTED = 4, /* dtype or radius not built, unknown option               */
    SADJ_ERR_DEVICE = 5       /* HIP reported an error when enqueueing, or
                                 (sadj_check_array) memory the device cannot access      */
} sadj_status;

typedef enum { SADJ_F32 = 0, SADJ_F64 = 1 } sadj_dtype;

/* Static, NUL-terminated description of a status code (never NULL). */
const char *sadj_status_string(sadj_status status);

/* Library version as a static string, e.g. "0.1.0". */
const char *sadj_version(void);

/* HIP's description of the error behind the calling thread's most recent
 * SADJ_ERR_DEVICE ("no error" if there was none).  Static string, never NULL. */
const char *sadj_last_device_error(void);

/* ---- linear variable-coefficient wave step ---------------------------------------
 * Primal (paper Section 4.1, the generating script):
 *     r[i] = 2 u[i] - u_prev[i] + c[i] * sum_o w_o u[i+o]            for i in I
 * Adjoint (Section 4.1, gather listing, generalised to radius R and merged into one
 * update per index as in the last listing of Section 3.2):
 *     u_bar[j]      += 2 r_bar[j] [j in I] + sum_o w_o * c[j-o] r_bar[j-o] [j-o in I]
 *     u_prev_bar[j] -= r_bar[j] [j in I]            (skipped when u_prev_bar is NULL)
 * The linear stencil's adjoint does not need the primal u (Section 3.1).
 * 1-D and 2-D: radius 1 (3- and 5-point).  3-D: radius 1 .. 4 (7-, 13-, 19- and 25-point
 * stars; radius 1 is the paper's test case, radius 4 the benchmark's; the launch-shape
 * variants of "wave3d.variant" exist for radius 1 and 4, other radii use the default shape).
 */
sadj_status sadj_primal_wave1d(sadj_dtype dtype, long n,
                               const void *u, const void *u_prev, const void *c, void *r,
                               void *stream);
sadj_status sadj_adjoint_wave1d(sadj_dtype dtype, long n,
                                const void *c, const void *r_bar,
                                void *u_bar, void *u_prev_bar /* nullable */, void *stream);

sadj_status sadj_primal_wave2d(sadj_dtype dtype, long nx, long ny,
                               const void *u, const void *u_prev, const void *c, void *r,
                               void *stream);
sadj_status sadj_adjoint_wave2d(sadj_dtype dtype, long nx, long ny,
                                const void *c, const void *r_bar,
                                void *u_bar, void *u_prev_bar /* nullable */, void *stream);

sadj_status sadj_primal_wave3d(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                               const void *u, const void *u_prev, const void *c, void *r,
                               void *stream);
sadj_status sadj_adjoint_wave3d(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                const void *c, const void *r_bar,
                                void *u_bar, void *u_prev_bar /* nullable */, void *stream);

/* ---- contrast baseline (NOT the method): conventional scatter with atomic updates ----------
 * Computes the same u_bar += J^T r_bar as sadj_adjoint_wave3d (u_prev_bar not offered),
 * but the way conventional reverse mode parallelised with atomics does (paper Sections 1
 * and 3.2; the OpenMP-atomics baseline of Section 4.1): one GPU thread per primal
 * iteration i in I scatters its 6R+1 terms with hardware atomic adds.  It exists so that
 * the gather kernels can be compared with it on the same hardware.  The order of the
 * additions into one element is not fixed: results vary in the last bits from run to run.
 * Arrays must be ordinary (coarse-grained) device allocations.  Same argument rules and
 * errors as sadj_adjoint_wave3d; additionally nz - 2R and (ny - 2R)/4 must not exceed
 * 65535 (SADJ_ERR_UNSUPPORTED).
 */
sadj_status sadj_adjoint_wave3d_atomic_scatter(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                               const void *c, const void *r_bar, void *u_bar, void *stream);

/* ---- reverse sweep of a time loop of 3-D wave steps -----------------------------------
 * A solver runs many steps u^{k+1} = step(u^k, u^{k-1}) (the paper measures one step and
 * notes that such solvers take many, Section 4); each step assigns u^{k+1} on I only, so
 * cells of u^{k+1} outside I are inputs, not functions of earlier states.  With lam^k
 * the adjoint of state u^k, the reverse sweep of one step is
 *     lam^k     += (d step / d u^k)^T     lam^{k+1}        (the gather of sadj_adjoint_wave3d)
 *     lam^{k-1} += (d step / d u^{k-1})^T lam^{k+1}  =  lam^{k-1} - lam^{k+1} on I .
 * This call performs `nsteps` such reverse steps with three rotating buffers.  On entry
 * lam0 = lam^{K+1}, lam1 = lam^K, lam2 = lam^{K-1} (whatever the objective contributes to
 * them directly; often lam2 is zero).  Step s = 0, 1, ... reads a = lam[s%3] and updates
 * b = lam[(s+1)%3] and p = lam[(s+2)%3]; from s = 1 on, p is the buffer whose content
 * was consumed by the previous step, and it is ASSIGNED: p = -a on I, 0 elsewhere (the
 * adjoint of a state that the objective does not touch directly starts from zero).
 * After the call: lam[nsteps%3] = lam^{K+1-nsteps}, lam[(nsteps+1)%3] = lam^{K-nsteps},
 * and lam[(nsteps+2)%3] holds consumed data.  nsteps = 0 does nothing.  One kernel per
 * step is enqueued on `stream`; the four arrays must be mutually non-overlapping.
 */
sadj_status sadj_adjoint_wave3d_steps(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                      long nsteps, const void *c,
                                      void *lam0, void *lam1, void *lam2, void *stream);

/* The same reverse sweep with a fourth array to work in, so that two steps can share one pass
 * over the data.  Writing a = lam^{k+1}, b = lam^k and m for the indicator of I, one reverse step
 * is a' = b + 2 a m + S(c a m), b' = -a m (S: the gather of sadj_adjoint_wave3d without its
 * centre term 2 r_bar); two steps are a'' = -a m + 2 a' m + S(c a' m), b'' = -a' m, and a' need
 * not reach memory: a, b and c are read once and a'', b'' written once per two steps (40 bytes
 * per cell in fp64 instead of 80).  a'' and b'' cannot be written over a or b, because other
 * workgroups still read their halo cells; hence the fourth array.
 *   Arguments, entry and exit state of lam0, lam1, lam2 and errors are those of
 * sadj_adjoint_wave3d_steps; `work` is a device array of the same size and dtype, not overlapping
 * the others (NULL -> SADJ_ERR_NULL), whose contents on entry are ignored and on exit undefined,
 * as are those of lam[(nsteps+2)%3].  Step 0 accumulates into lam2 and runs alone; from then on
 * pairs of steps are fused, and the last few launches are chosen such that the results land in
 * the documented buffers (at most three single steps after the first; sadj_describe_wave3d_sweep
 * shows the choice).  Fused pairs exist for radius 1 where nx is a multiple of 16 bytes' worth
 * of elements and all five arrays are 16-byte aligned; otherwise, with nsteps < 3, or with
 * option "wave3d.fuse" 1, the call is sadj_adjoint_wave3d_steps and `work` is not touched.
 * Fused and single steps add the same terms in a different order: results agree to rounding,
 * not bit for bit.
 */
sadj_status sadj_adjoint_wave3d_steps_fused(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                            long nsteps, const void *c,
                                            void *lam0, void *lam1, void *lam2, void *work, void *stream);

/* Diagnostic (host only, no device access): the launches of sadj_adjoint_wave3d_steps_fused
 * after step 0 when pairs can be fused.  Buffers are numbered 0..2 = lam0..lam2, 3 = work.
 * *body_pairs fused pairs alternate (a, b) = (1, 2) -> results in (0, 3) -> results in (1, 2)
 * ...; then *tail_len launches follow, five ints each in `tail` (room for 12 launches):
 * fused (1 or 0), a, b, and the output buffers (fused: a'', b''; single: the buffer that
 * receives -a m, then -1).  *body_pairs = -1: single steps over lam0..lam2 only (nsteps < 3).
 */
sadj_status sadj_describe_wave3d_sweep(long nsteps, long *body_pairs, int *tail_len, int *tail);

/* ---- dense 3^d box stencils with arbitrary weights --------------------------------------
 * Primal:   r[i] = c[i] * sum_{o in {-1,0,1}^ndim} w[o] u[i+o]              for i in I = prod [1, n_d-2]
 * Adjoint:  u_bar[j] += sum_o w[o] * c[j-o] r_bar[j-o] [j-o in I]           for all j
 * These are the dense stencils of paper Section 3.3.4 (3 points in 1-D, 3x3, 3x3x3); the
 * 1-D case with weights (2,-3,4) is the worked example of Section 3.2, whose outer
 * weights change sides in the adjoint.  The weights may be asymmetric: the adjoint
 * gathers with the point-mirrored table (index shifting, Section 3.3.2).
 * `weights` is a HOST pointer to 3^ndim doubles, x fastest: entry (ox+1) + 3*(oy+1) +
 * 9*(oz+1) (only the axes that exist); it is read during the call and converted to dtype.
 * ndim = 1, 2 or 3; extents of unused axes are ignored.  Other conventions as above.
 */
sadj_status sadj_primal_box(sadj_dtype dtype, int ndim, long nx, long ny, long nz,
                            const double *weights /* host */,
                            const void *u, const void *c, void *r, void *stream);
sadj_status sadj_adjoint_box(sadj_dtype dtype, int ndim, long nx, long ny, long nz,
                             const double *weights /* host */,
                             const void *c, const void *r_bar, void *u_bar, void *stream);

/* ---- 1-D upwinded Burgers step -----------------------------------------------------
 * Primal (paper Section 4.2, upwind formula and generating script), i in [1, n-2]:
 *     r[i] = u[i] - C*(max(u[i],0)*(u[i]-u[i-1]) + min(u[i],0)*(u[i+1]-u[i]))
 *                 + D*(u[i-1] - 2u[i] + u[i+1])
 * Adjoint (Section 4.2, gather listing): nonlinear, so the primal u is read, at
 * shifted indices (Section 3.3.2); with g_-(i), g_0(i), g_+(i) the partial derivatives
 * of iteration i with respect to u[i-1], u[i], u[i+1],
 *     u_bar[j] += g_-(j+1) r_bar[j+1] [j+1 in I] + g_0(j) r_bar[j] [j in I]
 *               + g_+(j-1) r_bar[j-1] [j-1 in I]
 * d max(a,0)/da and d min(a,0)/da are both 1 at a == 0, as in the paper's listing.
 * C and D are converted to dtype before use.
 */
sadj_status sadj_primal_burgers1d(sadj_dtype dtype, long n, double C, double D,
                                  const void *u, void *r, void *stream);
sadj_status sadj_adjoint_burgers1d(sadj_dtype dtype, long n, double C, double D,
                                   const void *u, const void *r_bar, void *u_bar,
                                   void *stream);

/* ---- 3-D star stencils of radius 1..4 with arbitrary weights --------------------------------
 * The general linear star: one free weight per read offset, e.g. upwind-biased differences.
 *   primal   r[i]      = c[i] * ( w_0 u[i] + sum_{d=x,y,z} sum_{o=-R..R, o!=0} w_{d,o} u[i + o e_d] )  for i in I
 *   adjoint  u_bar[j] += w_0 q[j] + sum_d sum_o w_{d,o} q[j - o e_d],  q = c*r_bar on I, 0 elsewhere, for all j
 * (Sections 3.2-3.3: the term of read offset o is shifted by -o, so an asymmetric table
 * appears mirrored in the adjoint, as in the worked 1-D example.)  `weights` is a HOST array
 * of 1 + 6R doubles read during the call: the centre weight, then for the axes x, y, z in
 * turn the 2R weights of the offsets -R, .., -1, +1, .., +R; they are converted to dtype.
 * Same conventions and errors as the wave calls (primal assigns r on I, adjoint accumulates
 * into u_bar, c and r_bar outside I never used).  With the symmetric Laplacian weights the
 * adjoint equals sadj_adjoint_wave3d without its 2 r_bar term.
 */
sadj_status sadj_primal_star3d(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                               const double *weights /* host, 1 + 6*radius */,
                               const void *u, const void *c, void *r, void *stream);
sadj_status sadj_adjoint_star3d(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                const double *weights /* host, 1 + 6*radius */,
                                const void *c, const void *r_bar, void *u_bar, void *stream);

/* ---- time loop of Burgers steps: store every state, then sweep backwards -------------------
 * The Burgers stencil is nonlinear, so the reverse sweep of step u^t -> u^{t+1} needs the
 * primal state u^t (paper Section 3.1: a nonlinear statement's adjoint reads primal values;
 * Section 4.2).  With 288 GB of HBM the states of a 1-D solver are simply all kept:
 *
 * sadj_primal_burgers1d_steps: `states` holds nsteps+1 rows of n elements, row t = u^t.
 *   Row 0 is the initial state; for t = 0 .. nsteps-1 the call assigns row t+1 on I = [1, n-2]
 *   from row t.  Elements 0 and n-1 of every row are inputs (boundary data), never written.
 *
 * sadj_adjoint_burgers1d_steps: reverse sweep over the steps last-1, last-2, ..., last-nsteps
 *   (step t maps row t to row t+1; rows last-nsteps .. last-1 of `states` are read).  On entry
 *   lam0 = adjoint of u^{last}, lam1 = whatever the objective contributes directly to the
 *   adjoint of u^{last-1} (often zero).  Reverse step s = 0, 1, ... reads lam[s%2] and
 *   updates lam[(s+1)%2] with (d step_t / d u^t)^T lam[s%2], t = last-1-s: accumulated for
 *   s = 0, ASSIGNED for s >= 1 (the buffer's old content, the adjoint of a later state, is
 *   consumed; adjoints of earlier states start from zero).  As in every adjoint call, values
 *   of lam[s%2] outside I are never used.  After the call lam[nsteps%2] holds the adjoint of
 *   u^{last-nsteps}.  nsteps = 0 does nothing; nsteps > last -> SADJ_ERR_SIZE.  lam0, lam1 and
 *   the rows read must not overlap.  One kernel per step is enqueued (fewer where steps are fused, see
 *   option "burgers1d.fuse").
 */
sadj_status sadj_primal_burgers1d_steps(sadj_dtype dtype, long n, long nsteps, double C, double D,
                                        void *states, void *stream);
sadj_status sadj_adjoint_burgers1d_steps(sadj_dtype dtype, long n, long last, long nsteps, double C, double D,
                                         const void *states, void *lam0, void *lam1, void *stream);

/* ---- time loop of Burgers steps with checkpoints: keep every k-th state, recompute the rest ------
 * At the size of the paper's own Burgers experiment (10^9 cells, Section 4.2) one state is 8 GB,
 * so a long time loop cannot keep every state; the standard remedy stores every `every`-th state
 * (a checkpoint) and recomputes the states in between, one segment at a time, while sweeping
 * backwards.  Both calls run the kernels of the single-step calls; the reverse sweep's result
 * equals that of sadj_adjoint_burgers1d_steps over a full history bit for bit.
 * Boundary data: elements 0 and n-1 of every state equal those of u^0 (held fixed in time).
 *
 * sadj_primal_burgers1d_ckpt: `ckpt` holds nsteps/every + 1 rows of n elements; row 0 = u^0 on
 *   entry; on return row j = u^{j*every}.  `work`: 2 rows of scratch.  u_final (nullable, n
 *   elements) receives u^{nsteps}.  nsteps+1 kernels (and one copy) are enqueued.
 *
 * sadj_adjoint_burgers1d_ckpt: reverse sweep over the steps nsteps-1 .. 0.  On entry lam0 =
 *   adjoint of u^{nsteps}, lam1 = what the objective contributes directly to the adjoint of
 *   u^{nsteps-1} (often zero); rotation and assign/accumulate rules as in
 *   sadj_adjoint_burgers1d_steps; after the call lam[nsteps%2] holds the adjoint of u^0.  `work`:
 *   scratch of at least (every-1)*n elements (work_bytes states its size; may be NULL when
 *   every == 1) that receives the recomputed states of one segment at a time.
 *   Errors: every < 1, work_bytes too small -> SADJ_ERR_SIZE; ckpt, lam0, lam1, work overlapping
 *   -> SADJ_ERR_ALIAS.  Roughly (2 - 1/every) kernels per step are enqueued.
 */
sadj_status sadj_primal_burgers1d_ckpt(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                       void *ckpt, void *work, void *u_final /* nullable */, void *stream);
sadj_status sadj_adjoint_burgers1d_ckpt(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                        const void *ckpt, void *work, size_t work_bytes,
                                        void *lam0, void *lam1, void *stream);

/* ---- the checkpointed reverse sweep for callers that cannot allocate ------------------------
 * For callers that may not obtain device memory at the time of the call -- code recorded into a
 * HIP graph, tight serving loops, harnesses that forbid allocation -- and therefore cannot hand
 * over a `work` array: sadj_adjoint_burgers1d_ckpt with its scratch taken from a fixed array
 * that lives in the library's device image (sadj_static_scratch_bytes() bytes, 64 MiB; every GPU
 * that loads the library holds its own copy until the process ends).  The call allocates and
 * frees nothing; the first call on a device looks up that device's copy of the array.
 * Arguments, result and errors as sadj_adjoint_burgers1d_ckpt without `work`/`work_bytes`;
 * additionally (every-1)*n*sizeof(element) > sadj_static_scratch_bytes() -> SADJ_ERR_SIZE, nothing
 * enqueued.  The scratch keeps the last call's contents; every element a call reads it has
 * written before, so nothing needs clearing.  All calls on one GPU share the one array: calls
 * whose work overlaps in time on the same GPU (different streams or threads) race and must be
 * serialised by the caller.
 */
sadj_status sadj_adjoint_burgers1d_ckpt_static(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                               const void *ckpt, void *lam0, void *lam1, void *stream);
size_t sadj_static_scratch_bytes(void);

/* ---- diagnostic: how a 3-D adjoint call is cut into workgroups ----------------------------
 * Section 3.3.4 requires the loop nests (here: workgroups) to be disjoint and to cover every
 * output index exactly once.  This host-only call reports the decomposition that
 * sadj_adjoint_wave3d uses under the current options for 16-byte aligned arrays (with_u_prev_bar:
 * whether u_prev_bar is passed, which selects another tile shape in fp64), so that a test can
 * check that property without a GPU: plan[0..7] = tiles along x, tiles along y, tile width, tile
 * height (cells), number of workgroups, and how the tiles are cut along z: the first
 * plan[5] tiles (in tile numbering order) into plan[6] chunks each, all others into
 * plan[7] chunks each (plan[5] = 0: every tile alike).  If `tiles` is not NULL it receives,
 * for each of the first max_blocks workgroup ids, four ints: tile x, tile y, first plane,
 * one past the last plane.  `plan` and `tiles` are HOST pointers.  Nothing is launched.
 */
sadj_status sadj_describe_wave3d_plan(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                      int with_u_prev_bar, long *plan /* host, 8 */, int *tiles /* host, 4*max_blocks, nullable */,
                                      long max_blocks);

/* ---- launch options -------------------------------------------------------------------
 * Process-wide integer options that select among equivalent launch strategies; they
 * never change what is computed, only how the regions are mapped to kernels.  Every
 * setting is deterministic (same inputs, same bits).  Settings that select another
 * kernel shape or instruction sequence ("*.variant", "wave2d.ychunk", "wave3d.order",
 * "stencil1d.functor", "star3d.functor") may round differently from each other within the usual
 * floating-point tolerance; "wave3d.zchunk", "wave3d.split", "wave3d.xcdmap",
 * "wave3d.band" and "wave3d.ldspad" only move work between workgroups and leave every
 * bit of the 3-D results unchanged.
 *   "wave3d.zchunk"  planes of output per workgroup along z (default 0 = automatic).
 *   "wave3d.split"   0 (default): where the x-y tiles do not fill whole rounds of one workgroup
 *                    per compute unit, the left-over tiles may be cut into more z-chunks than
 *                    the others so that they fill a round of their own; 1: all tiles are cut
 *                    alike.  Ignored when "wave3d.zchunk" is set.
 *   "wave3d.variant" tile shape of sadj_adjoint_wave3d (default 0 = automatic): 1 = 64 x 32 cells, two
 *                    cells per lane; 2 = 128 x 32, four cells per lane; 3 = 64 x 32, one cell per
 *                    lane; 5 = rows of 1 KB x 16 rows; 10 / 11 = 256 / 512 cells x 16 rows (radius
 *                    1).  Other values select shape 1.
 *   "wave2d.variant" kernel form of the 2-D wave and 2-D box calls: 0 (default) one workgroup per tile of 8 rows,
 *                    no march; 1 the strip march (a wave marches down y over a strip of columns);
 *                    2 tiles of 16 rows.
 *   "wave2d.ychunk"  strip march only: rows of output per wave along y (default 0 = automatic); a
 *                    value that would need more than 65535 row chunks makes the 2-D calls return
 *                    SADJ_ERR_UNSUPPORTED.
 *   "wave3d.xcdmap"  how workgroups of the 3-D marching kernels are assigned to x-y tiles:
 *                    0/1 (default) per round of resident workgroups every XCD (chiplet with
 *                    its own L2) owns a contiguous range of tiles, 2 one contiguous range
 *                    per XCD over the whole dispatch, 3 tiles dealt round-robin to XCDs.
 *   "wave3d.band"    numbering of the tiles of a plane: k > 0 bands of k tile rows with y
 *                    fastest inside a band (1: plain rows of tiles, x fastest); 0 (default)
 *                    automatic: rows of tiles, or bands of 8 where a row has 32 or more tiles
 *                    and the plane at least 8 tile rows.
 *   "wave3d.ldspad"  dynamic LDS bytes requested per workgroup of the 3-D marching kernels,
 *                    which limits how many workgroups share a CU: 0 (default) as much as
 *                    keeps it at one workgroup per CU, -1 none, n > 0 exactly n (<= 65536).
 *   "wave3d.remainder" treatment of the boundary / remainder regions (Section 3.3.4) by
 *                    sadj_adjoint_wave3d:  0 (default) one dispatch, tiles that touch the
 *                    remainder run guarded statements, core tiles unguarded ones;
 *                    1 every tile runs the guarded statements (as if the inputs were
 *                    zero-padded); 2 core tiles and remainder tiles in two disjoint
 *                    dispatches.  1 and 2 serve to measure the strategies; they need
 *                    u_prev_bar == NULL, variant 0-2, nx a multiple of 16 bytes' worth of
 *                    elements and 16-byte aligned arrays, else SADJ_ERR_UNSUPPORTED.
 *   "stencil1d.functor" 1: sadj_*_burgers1d and the 1-D sadj_*_box run through the generic
 *                    functor kernel of sadj_stencil1d.hpp instead of their own (default 0).
 *   "star3d.functor" 1: radius-1 calls of sadj_*_star3d run through the generic functor kernels of
 *                    sadj_stencil_star.hpp where nx and the arrays' alignment allow 16-byte
 *                    accesses (default 0: their own kernel).
 *   "burgers1d.fuse" 0 (default): the reverse sweeps of the Burgers time loop
 *                    (sadj_adjoint_burgers1d_steps, sadj_adjoint_burgers1d_ckpt*) apply runs of five
 *                    assigned steps in one pass over the data (lam read and written once per
 *                    five states read, instead of once per state) where all arrays are 16-byte
 *                    aligned; 1: one kernel per step.  Same result bit for bit.
 *   "wave3d.fuse"    0 (default): sadj_adjoint_wave3d_steps_fused fuses pairs of steps where it can;
 *                    1: it runs single steps only.
 *   "wave3d.order"   order in which sadj_adjoint_wave3d adds the terms of one u_bar[j]
 *                    (Section 3.5: a gather can respect an order the user chooses and
 *                    stay parallel).  0 (default): the kernel's own fixed order, fastest.
 *                    1: the order and rounding of the sequential scatter adjoint that
 *                    conventional reverse mode produces (Section 3.2) -- starting from the
 *                    incoming u_bar[j], terms by ascending memory index of their primal
 *                    iteration i, each term (c[i]*w)*r_bar[i] and each addition rounded
 *                    separately; in fp64 the result equals that sequential loop bit for
 *                    bit.  Both orders are deterministic.  "wave3d.variant" and
 *                    "wave3d.remainder" do not apply to order 1; other entry points
 *                    ignore this option.
 *   "check.pointers" 1: before anything is enqueued, every array argument of every entry
 *                    point is checked with sadj_check_array (below); a call with a failing
 *                    array returns that status and launches nothing.  Default 0: pointers
 *                    are trusted, as the conventions above say (the check costs a few
 *                    runtime queries per array).
 * Unknown names or out-of-range values give SADJ_ERR_UNSUPPORTED and change nothing.
 * sadj_get_option returns SADJ_OK and stores the value, or SADJ_ERR_UNSUPPORTED.
 */
sadj_status sadj_set_option(const char *name, long value);
sadj_status sadj_get_option(const char *name, long *value);

/* ---- measurement yardstick: a plain streaming kernel with the adjoint's access mix -----------
 * out[i] += a[i] * b[i] for i in [0, n): two arrays read, one array read and written, every
 * element touched once -- the streams of a wave adjoint call (c, r_bar, u_bar; Section 4.1's
 * gather listing) without any stencil, halo or reuse.  Its rate is the ceiling this memory
 * system offers to that mix of streams; the benchmark quotes the adjoint kernels against it as
 * well as against the nominal HBM peak.  `shape` selects the launch shape: 0 = 256 threads, 8 bytes
 * per lane, one access per thread; 1 = 256 threads, 16 bytes per lane, four accesses per thread,
 * streaming hints; 2 = single-wave workgroups, one 16-byte access per lane, the fastest found.
 * a, b, out: DEVICE arrays of n elements, 16-byte aligned (else SADJ_ERR_UNSUPPORTED), out not
 * overlapping a or b.  n < 1 or n > 2^40 -> SADJ_ERR_SIZE.  Asynchronous on `stream`.
 */
sadj_status sadj_stream_probe(sadj_dtype dtype, int shape, long n,
                              const void *a, const void *b, void *out, void *stream);

/* ---- diagnostic: can a kernel on the current device use this array? ------------------------
 * For callers that want wrong pointers or sizes turned into a status instead of a GPU memory
 * fault.  Queries the HIP runtime; enqueues nothing.  SADJ_OK: [p, p+bytes) lies inside one
 * allocation of device, managed or pinned host memory that the current device can access.
 * SADJ_ERR_DEVICE: the runtime does not know the pointer (pageable host memory, a stale or
 * made-up address), or it belongs to a device the current one cannot access.  SADJ_ERR_SIZE:
 * the range runs past the end of the allocation p points into.  SADJ_ERR_NULL: p is NULL.
 * An allocation here is what the runtime handed out: with a caching allocator on top (torch's),
 * a tensor smaller than its block passes for the block's size.
 */
sadj_status sadj_check_array(const void *p /* device or host */, size_t bytes);

#ifdef __cplusplus
}
#endif
#endif /* SADJ_H */
