// C ABI of libsadj: argument validation and dispatch.  See include/sadj.h for the
// contract of every entry point.
#include "../../include/sadj.h"
#include "launch.hpp"

#include <atomic>
#include <cstdint>
#include <cstring>
#include <mutex>

namespace {

std::atomic<long> g_zchunk{0}, g_variant{0}, g_ychunk2d{0}, g_variant2d{0}, g_remainder{0}, g_order{0}, g_functor1d{0}, g_functor_star{0}, g_burgers_fuse{0}, g_wave_fuse{0}, g_xcdmap{0}, g_band{0}, g_ldspad{0}, g_split{0};

// Options are set one at a time; a call takes one consistent snapshot of all of them under
// the same lock the setters hold, so it never sees a combination that was not in force at
// some moment.
std::mutex g_option_mutex;

sadj::LaunchOptions current_options()
{
    std::lock_guard<std::mutex> lock(g_option_mutex);
    sadj::LaunchOptions o;
    o.zchunk = g_zchunk.load();
    o.variant = g_variant.load();
    o.ychunk2d = g_ychunk2d.load();
    o.variant2d = g_variant2d.load();
    o.remainder = g_remainder.load();
    o.split = g_split.load();
    o.xcd_map = g_xcdmap.load();
    o.band = g_band.load();
    o.lds_pad = g_ldspad.load();
    return o;
}

constexpr long kMaxExtent = 1L << 30;
constexpr long kMaxPlane = 1L << 28;   // elements; keeps in-plane byte offsets below 2^32

struct Span { const void *p; size_t bytes; };

bool overlaps(const Span &a, const Span &b)
{
    if (!a.p || !b.p || a.bytes == 0 || b.bytes == 0) return false;
    const uintptr_t a0 = (uintptr_t)a.p, b0 = (uintptr_t)b.p;
    return a0 < b0 + b.bytes && b0 < a0 + a.bytes;
}

bool dtype_ok(sadj_dtype d) { return d == SADJ_F32 || d == SADJ_F64; }
size_t elem(sadj_dtype d) { return d == SADJ_F64 ? 8 : 4; }

std::atomic<long> g_check_pointers{0};

// Optional argument check (option "check.pointers"): the whole array must lie in memory a
// kernel on the current device can access (device, managed or pinned host memory) and inside
// one allocation.  Queries only; nothing is enqueued.
sadj_status check_span_memory(const Span &a)
{
    if (!a.p || a.bytes == 0) return SADJ_OK;
    hipPointerAttribute_t attr{};
    hipError_t e = hipPointerGetAttributes(&attr, a.p);
    if (e != hipSuccess) { (void)hipGetLastError(); return SADJ_ERR_DEVICE; }   // not known to the runtime
    if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged && attr.type != hipMemoryTypeHost)
        return SADJ_ERR_DEVICE;                                                  // pageable host memory
    if (attr.type == hipMemoryTypeDevice) {
        int dev = -1;
        if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return SADJ_ERR_DEVICE; }
        if (attr.device != dev) {
            int peer = 0;
            if (hipDeviceCanAccessPeer(&peer, dev, attr.device) != hipSuccess || !peer) {
                (void)hipGetLastError();
                return SADJ_ERR_DEVICE;
            }
        }
    }
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    e = hipMemGetAddressRange(&base, &size, const_cast<void *>(a.p));
    if (e != hipSuccess) { (void)hipGetLastError(); return SADJ_ERR_DEVICE; }
    const uintptr_t b0 = (uintptr_t)base, p0 = (uintptr_t)a.p;
    if (p0 < b0 || a.bytes > size || p0 - b0 > size - a.bytes) return SADJ_ERR_SIZE;
    return SADJ_OK;
}

// Outputs must not overlap inputs, nor each other; with "check.pointers" on, every array must
// also be memory the device can access, in full.
template <size_t NI, size_t NO>
sadj_status check_arrays(const Span (&in)[NI], const Span (&out)[NO])
{
    for (size_t o = 0; o < NO; ++o) {
        for (size_t i = 0; i < NI; ++i)
            if (overlaps(out[o], in[i])) return SADJ_ERR_ALIAS;
        for (size_t o2 = o + 1; o2 < NO; ++o2)
            if (overlaps(out[o], out[o2])) return SADJ_ERR_ALIAS;
    }
    if (g_check_pointers.load() == 1) {
        for (size_t i = 0; i < NI; ++i) { const sadj_status s = check_span_memory(in[i]); if (s != SADJ_OK) return s; }
        for (size_t o = 0; o < NO; ++o) { const sadj_status s = check_span_memory(out[o]); if (s != SADJ_OK) return s; }
    }
    return SADJ_OK;
}

sadj_status check_extents(int radius, long nx, long ny, long nz, int ndim)
{
    const long n[3] = {nx, ny, nz};
    for (int d = 0; d < ndim; ++d)
        if (n[d] < 2L * radius + 1 || n[d] > kMaxExtent) return SADJ_ERR_SIZE;
    if (ndim >= 2 && nx * ny > kMaxPlane) return SADJ_ERR_SIZE;
    return SADJ_OK;
}

thread_local hipError_t g_last_hip_error = hipSuccess;

sadj_status from_hip(hipError_t e)
{
    if (e == hipSuccess) return SADJ_OK;
    if (e == hipErrorNotSupported) return SADJ_ERR_UNSUPPORTED;   // a launcher declined before enqueueing
    g_last_hip_error = e;
    return SADJ_ERR_DEVICE;
}

// An earlier, unrelated HIP call of this thread may have left a sticky error code
// behind; drop it so that the check after our launch reports our launch only.
void clear_stale_hip_error() { (void)hipGetLastError(); }

}  // namespace

namespace {

// Reverse steps s0, s0+1, ... of a sweep over the states state(0), state(1), ... (in the order
// they are applied).  Step s reads lam[s%2] and updates lam[(s+1)%2]: accumulated for s = 0,
// assigned from then on.  Runs of assigned steps are fused, several steps per pass over the
// data, unless option "burgers1d.fuse" is 1 or the arrays' alignment rules it out; the result is
// the same bit for bit.  Returns the number of steps done in `s0`.
template <class StateOf>
sadj_status burgers_reverse_steps(sadj_dtype dtype, long n, double C, double D, long count, StateOf state, void *const (&lam)[2],
                                  long &s0, hipStream_t st)
{
    const int f64 = dtype == SADJ_F64;
    const int M = sadj::burgers_fused_steps();
    const bool fuse = g_burgers_fuse.load() == 0;
    long k = 0;
    while (k < count) {
        const long s = s0 + k;
        if (fuse && s > 0 && count - k >= M) {
            const void *u[16];
            for (int i = 0; i < M; ++i) u[i] = state(k + i);
            const hipError_t e = sadj::launch_adjoint_burgers1d_fused(f64, n, C, D, u, lam[s % 2], lam[(s + M) % 2], st);
            if (e == hipSuccess) { k += M; continue; }
            if (e != hipErrorNotSupported) return from_hip(e);
        }
        const hipError_t e = sadj::launch_adjoint_burgers1d(f64, n, C, D, state(k), lam[s % 2], lam[(s + 1) % 2], s > 0 ? 1 : 0, st);
        if (e != hipSuccess) return from_hip(e);
        ++k;
    }
    s0 += count;
    return SADJ_OK;
}

// Reverse sweep over all nsteps steps with recomputation; `work` holds every-1 rows.
sadj_status burgers_ckpt_reverse(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                 const void *ckpt, void *work, void *lam0, void *lam1, hipStream_t st)
{
    const size_t row = (size_t)n * elem(dtype);
    const int f64 = dtype == SADJ_F64;
    void *const lam[2] = {lam0, lam1};
    const char *cb = static_cast<const char *>(ckpt);
    char *wb = static_cast<char *>(work);
    long s = 0;                                             // reverse steps done
    for (long seg = (nsteps - 1) / every; seg >= 0 && nsteps > 0; --seg) {
        const long t0 = seg * every, t1 = t0 + every < nsteps ? t0 + every : nsteps;
        // states u^{t0+1} .. u^{t1-1} into work rows 0 .. t1-t0-2 (u^{t0} is the checkpoint itself)
        auto state = [&](long t) -> const char * { return t == t0 ? cb + (size_t)seg * row : wb + (size_t)(t - t0 - 1) * row; };
        for (long t = t0; t + 1 < t1; ++t) {
            hipError_t e = sadj::launch_primal_burgers1d(f64, n, C, D, state(t), wb + (size_t)(t - t0) * row, st, 1);
            if (e != hipSuccess) return from_hip(e);
        }
        // reverse steps t1-1 .. t0 over these states
        auto applied = [&](long k) -> const void * { return state(t1 - 1 - k); };
        if (sadj_status rs = burgers_reverse_steps(dtype, n, C, D, t1 - t0, applied, lam, s, st); rs != SADJ_OK) return rs;
    }
    return SADJ_OK;
}

// Order of launches of a reverse sweep of wave steps that may use a fourth array.
// Buffers 0..2 are the caller's lam arrays, 3 is the work array.  A state is the pair (A, B) of
// buffers that hold lam^{k+1} and lam^k.  A single step updates B in place and assigns -A m to
// a buffer F outside {A, B}: (A, B) -> (B, F).  A fused pair of steps writes both results to the
// two buffers outside {A, B}: (A, B) -> (F, G).  After the first step (which accumulates into
// lam2 and is always single) the state is (1, 2); the sweep must end in (n%3, (n+1)%3).  The
// body alternates pairs (1,2) -> (0,3) -> (1,2) ...; the last few steps are chosen by exhaustive
// dynamic programming so that the end state is met with as many pairs as possible.
struct WaveStepLaunch { int pair, a, b, o0, o1; };   // single: o0 = F;  pair: o0 <- a'', o1 <- b''

constexpr int kTailMax = 12;

struct WaveSweepPlan {
    bool plain = true;                 // single steps rotating the caller's three buffers, work unused
    long body_pairs = 0;               // else: pairs alternating (1,2) -> (0,3) -> (1,2) ..., then the tail
    int tail_len = 0;
    WaveStepLaunch tail[kTailMax];
};

inline int state_id(int a, int b) { return a * 4 + b; }

// Launches for steps 1 .. nsteps-1 (step 0 is not part of the plan).
WaveSweepPlan plan_wave_sweep(long nsteps)
{
    WaveSweepPlan plan;
    const long m = nsteps - 1;
    if (m < 2) return plan;
    const int ta = (int)(nsteps % 3), tb = (int)((nsteps + 1) % 3);
    const int tmax = (int)(m < kTailMax ? m : kTailMax);
    // best[t][state]: most pairs on a way from state to the target in exactly t steps, -1 if none
    int best[kTailMax + 1][16], choice[kTailMax + 1][16][3];
    for (int t = 0; t <= tmax; ++t)
        for (int s = 0; s < 16; ++s) best[t][s] = -1;
    best[0][state_id(ta, tb)] = 0;
    for (int t = 1; t <= tmax; ++t)
        for (int a = 0; a < 4; ++a)
            for (int b = 0; b < 4; ++b) {
                if (a == b) continue;
                int fr[2], nf = 0;
                for (int f = 0; f < 4; ++f)
                    if (f != a && f != b) fr[nf++] = f;
                int &bst = best[t][state_id(a, b)];
                int *ch = choice[t][state_id(a, b)];
                for (int i = 0; i < 2; ++i) {
                    const int v = best[t - 1][state_id(b, fr[i])];
                    if (v >= 0 && v > bst) { bst = v; ch[0] = 0; ch[1] = fr[i]; ch[2] = -1; }
                    if (t >= 2) {
                        const int w = best[t - 2][state_id(fr[i], fr[1 - i])];
                        if (w >= 0 && w + 1 > bst) { bst = w + 1; ch[0] = 1; ch[1] = fr[i]; ch[2] = fr[1 - i]; }
                    }
                }
            }
    auto body_state = [](long pairs, int &a, int &b) { if (pairs % 2 == 0) { a = 1; b = 2; } else { a = 0; b = 3; } };
    long q = m / 2;
    int t = 0, a = 1, b = 2;
    bool found = false;
    for (; q >= 0 && m - 2 * q <= tmax; --q) {
        t = (int)(m - 2 * q);
        body_state(q, a, b);
        if (best[t][state_id(a, b)] >= 0) { found = true; break; }
    }
    if (!found) return plan;           // plain stays set: single steps over three buffers
    plan.plain = false;
    plan.body_pairs = q;
    while (t > 0) {
        const int *ch = choice[t][state_id(a, b)];
        WaveStepLaunch &l = plan.tail[plan.tail_len++];
        if (ch[0] == 0) { l = {0, a, b, ch[1], -1}; const int nb = ch[1]; a = b; b = nb; t -= 1; }
        else            { l = {1, a, b, ch[1], ch[2]}; a = ch[1]; b = ch[2]; t -= 2; }
    }
    return plan;
}

// Scratch memory of the entry point that must not allocate: a fixed array in device memory,
// one copy per GPU that loads the library, held until the process ends.  The array's name is
// a host-side handle only; the device address of the current GPU's copy is looked up once per
// device and used from then on.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<void *> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

sadj_status static_scratch_of_current_device(void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { g_last_hip_error = e; (void)hipGetLastError(); return SADJ_ERR_DEVICE; }
    if (dev < 0 || dev >= kMaxDevices) return SADJ_ERR_UNSUPPORTED;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));       // of the current device's copy
            if (e != hipSuccess || !p) { g_last_hip_error = e; (void)hipGetLastError(); return SADJ_ERR_DEVICE; }
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return SADJ_OK;
}

// library_work: `work` is the library's own scratch array (not an argument of the caller, so
// the optional pointer check does not apply to it; overlap with the caller's arrays cannot occur)
sadj_status burgers_ckpt_args(sadj_dtype dtype, long n, long nsteps, long every, const void *ckpt, const void *work,
                              size_t work_bytes, void *lam0, void *lam1, bool library_work = false)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!ckpt || !lam0 || !lam1) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent || nsteps < 0 || nsteps > kMaxExtent || every < 1 || every > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t row = (size_t)n * elem(dtype);
    const size_t need = (size_t)(every - 1) * row;
    if (need > 0 && !work) return SADJ_ERR_NULL;
    if (work_bytes < need) return SADJ_ERR_SIZE;
    const Span in[1] = {{ckpt, (size_t)((nsteps - 1 > 0 ? nsteps - 1 : 0) / every + 1) * row}};
    const Span out[3] = {{lam0, row}, {lam1, row}, {work, library_work ? 0 : need}};
    return check_arrays(in, out);
}

}  // namespace

extern "C" {

const char *sadj_status_string(sadj_status s)
{
    switch (s) {
    case SADJ_OK: return "ok";
    case SADJ_ERR_NULL: return "a required pointer is NULL";
    case SADJ_ERR_SIZE: return "grid extent below 2*radius+1 or above the supported limit";
    case SADJ_ERR_ALIAS: return "an output array overlaps an input array";
    case SADJ_ERR_UNSUPPORTED: return "unsupported dtype, radius or option";
    case SADJ_ERR_DEVICE: return "HIP error while enqueueing";
    }
    return "unknown status";
}

const char *sadj_version(void) { return "0.1.0"; }

const char *sadj_last_device_error(void) { return hipGetErrorString(g_last_hip_error); }

// Diagnostic: the check that "check.pointers" applies to every array argument.
sadj_status sadj_check_array(const void *p, size_t bytes)
{
    if (!p) return SADJ_ERR_NULL;
    return check_span_memory({p, bytes});
}

sadj_status sadj_set_option(const char *name, long value)
{
    if (!name) return SADJ_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_option_mutex);
    if (!std::strcmp(name, "wave3d.zchunk")) {
        if (value < 0 || value > kMaxExtent) return SADJ_ERR_UNSUPPORTED;
        g_zchunk = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.variant")) {
        if (value < 0 || value > 63) return SADJ_ERR_UNSUPPORTED;
        g_variant = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave2d.ychunk")) {
        if (value < 0 || value > kMaxExtent) return SADJ_ERR_UNSUPPORTED;
        g_ychunk2d = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave2d.variant")) {
        if (value < 0 || value > 2) return SADJ_ERR_UNSUPPORTED;
        g_variant2d = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "check.pointers")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_check_pointers = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.split")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_split = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.remainder")) {
        if (value < 0 || value > 2) return SADJ_ERR_UNSUPPORTED;
        g_remainder = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.xcdmap")) {
        if (value < 0 || value > 3) return SADJ_ERR_UNSUPPORTED;
        g_xcdmap = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.ldspad")) {
        if (value < -1 || value > 65536) return SADJ_ERR_UNSUPPORTED;
        g_ldspad = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.band")) {
        if (value < 0 || value > 4096) return SADJ_ERR_UNSUPPORTED;
        g_band = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.order")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_order = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "stencil1d.functor")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_functor1d = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "star3d.functor")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_functor_star = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "burgers1d.fuse")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_burgers_fuse = value;
        return SADJ_OK;
    }
    if (!std::strcmp(name, "wave3d.fuse")) {
        if (value < 0 || value > 1) return SADJ_ERR_UNSUPPORTED;
        g_wave_fuse = value;
        return SADJ_OK;
    }

    return SADJ_ERR_UNSUPPORTED;
}

sadj_status sadj_get_option(const char *name, long *value)
{
    if (!name || !value) return SADJ_ERR_NULL;
    if (!std::strcmp(name, "wave3d.zchunk")) { *value = g_zchunk; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.variant")) { *value = g_variant; return SADJ_OK; }
    if (!std::strcmp(name, "wave2d.ychunk")) { *value = g_ychunk2d; return SADJ_OK; }
    if (!std::strcmp(name, "wave2d.variant")) { *value = g_variant2d; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.remainder")) { *value = g_remainder; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.split")) { *value = g_split; return SADJ_OK; }
    if (!std::strcmp(name, "check.pointers")) { *value = g_check_pointers; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.order")) { *value = g_order; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.xcdmap")) { *value = g_xcdmap; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.band")) { *value = g_band; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.ldspad")) { *value = g_ldspad; return SADJ_OK; }
    if (!std::strcmp(name, "stencil1d.functor")) { *value = g_functor1d; return SADJ_OK; }
    if (!std::strcmp(name, "star3d.functor")) { *value = g_functor_star; return SADJ_OK; }
    if (!std::strcmp(name, "burgers1d.fuse")) { *value = g_burgers_fuse; return SADJ_OK; }
    if (!std::strcmp(name, "wave3d.fuse")) { *value = g_wave_fuse; return SADJ_OK; }
    return SADJ_ERR_UNSUPPORTED;
}

// ---------------------------------------------------------------------------- wave
static sadj_status primal_wave(int ndim, sadj_dtype dtype, int radius, long nx, long ny, long nz,
                               const void *u, const void *u_prev, const void *c, void *r, void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!u || !u_prev || !c || !r) return SADJ_ERR_NULL;
    sadj_status s = check_extents(radius, nx, ny, nz, ndim);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[3] = {{u, bytes}, {u_prev, bytes}, {c, bytes}};
    const Span out[1] = {{r, bytes}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int f64 = dtype == SADJ_F64;
    clear_stale_hip_error();
    switch (ndim) {
    case 1: return from_hip(sadj::launch_primal_wave1d(f64, nx, u, u_prev, c, r, st));
    case 2: return from_hip(sadj::launch_primal_wave2d(f64, (int)nx, (int)ny, u, u_prev, c, r, current_options(), st));
    default: return from_hip(sadj::launch_primal_wave3d(f64, radius, (int)nx, (int)ny, (int)nz, u, u_prev, c, r,
                                                        current_options(), st));
    }
}

static sadj_status adjoint_wave(int ndim, sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                const void *c, const void *r_bar, void *u_bar, void *u_prev_bar,
                                void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!c || !r_bar || !u_bar) return SADJ_ERR_NULL;
    sadj_status s = check_extents(radius, nx, ny, nz, ndim);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[2] = {{c, bytes}, {r_bar, bytes}};
    const Span out[2] = {{u_bar, bytes}, {u_prev_bar, u_prev_bar ? bytes : 0}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int f64 = dtype == SADJ_F64;
    clear_stale_hip_error();
    switch (ndim) {
    case 1: return from_hip(sadj::launch_adjoint_wave1d(f64, nx, c, r_bar, u_bar, u_prev_bar, st));
    case 2: return from_hip(sadj::launch_adjoint_wave2d(f64, (int)nx, (int)ny, c, r_bar, u_bar, u_prev_bar, current_options(), st));
    default:
        if (g_order.load() == 1)
            return from_hip(sadj::launch_adjoint_wave3d_ordered(f64, radius, (int)nx, (int)ny, (int)nz, c, r_bar, u_bar,
                                                                u_prev_bar, current_options(), st));
        return from_hip(sadj::launch_adjoint_wave3d(f64, radius, (int)nx, (int)ny, (int)nz, c, r_bar, u_bar,
                                                    u_prev_bar, 0, current_options(), st));
    }
}

sadj_status sadj_primal_wave1d(sadj_dtype dtype, long n, const void *u, const void *u_prev, const void *c,
                               void *r, void *stream)
{
    return primal_wave(1, dtype, 1, n, 1, 1, u, u_prev, c, r, stream);
}
sadj_status sadj_adjoint_wave1d(sadj_dtype dtype, long n, const void *c, const void *r_bar, void *u_bar,
                                void *u_prev_bar, void *stream)
{
    return adjoint_wave(1, dtype, 1, n, 1, 1, c, r_bar, u_bar, u_prev_bar, stream);
}
sadj_status sadj_primal_wave2d(sadj_dtype dtype, long nx, long ny, const void *u, const void *u_prev,
                               const void *c, void *r, void *stream)
{
    return primal_wave(2, dtype, 1, nx, ny, 1, u, u_prev, c, r, stream);
}
sadj_status sadj_adjoint_wave2d(sadj_dtype dtype, long nx, long ny, const void *c, const void *r_bar,
                                void *u_bar, void *u_prev_bar, void *stream)
{
    return adjoint_wave(2, dtype, 1, nx, ny, 1, c, r_bar, u_bar, u_prev_bar, stream);
}
sadj_status sadj_primal_wave3d(sadj_dtype dtype, int radius, long nx, long ny, long nz, const void *u,
                               const void *u_prev, const void *c, void *r, void *stream)
{
    if (radius < 1 || radius > 4) return SADJ_ERR_UNSUPPORTED;
    return primal_wave(3, dtype, radius, nx, ny, nz, u, u_prev, c, r, stream);
}
sadj_status sadj_adjoint_wave3d(sadj_dtype dtype, int radius, long nx, long ny, long nz, const void *c,
                                const void *r_bar, void *u_bar, void *u_prev_bar, void *stream)
{
    if (radius < 1 || radius > 4) return SADJ_ERR_UNSUPPORTED;
    return adjoint_wave(3, dtype, radius, nx, ny, nz, c, r_bar, u_bar, u_prev_bar, stream);
}

// Diagnostic: the decomposition sadj_adjoint_wave3d would use (no launch, no device access
// beyond reading the CU count).
sadj_status sadj_describe_wave3d_plan(sadj_dtype dtype, int radius, long nx, long ny, long nz, int with_u_prev_bar,
                                      long *plan, int *tiles, long max_blocks)
{
    if (radius < 1 || radius > 4 || !dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!plan) return SADJ_ERR_NULL;
    sadj_status s = check_extents(radius, nx, ny, nz, 3);
    if (s != SADJ_OK) return s;
    sadj::describe_march_plan(dtype == SADJ_F64, radius, (int)nx, (int)ny, (int)nz, with_u_prev_bar, current_options(),
                              plan, tiles, max_blocks);
    (void)hipGetLastError();       // a machine without a GPU leaves an error code behind; it is not ours to keep
    return SADJ_OK;
}

// Contrast baseline, not the method: scatter with atomic updates.
sadj_status sadj_adjoint_wave3d_atomic_scatter(sadj_dtype dtype, int radius, long nx, long ny, long nz,
                                               const void *c, const void *r_bar, void *u_bar, void *stream)
{
    if (radius < 1 || radius > 4) return SADJ_ERR_UNSUPPORTED;
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!c || !r_bar || !u_bar) return SADJ_ERR_NULL;
    sadj_status s = check_extents(radius, nx, ny, nz, 3);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[2] = {{c, bytes}, {r_bar, bytes}};
    const Span out[1] = {{u_bar, bytes}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    clear_stale_hip_error();
    return from_hip(sadj::launch_adjoint_wave3d_scatter_atomic(dtype == SADJ_F64, radius, (int)nx, (int)ny, (int)nz, c,
                                                               r_bar, u_bar, static_cast<hipStream_t>(stream)));
}

// Reverse sweep of a time loop of wave steps.
static sadj_status wave_steps_args(sadj_dtype dtype, int radius, long nx, long ny, long nz, long nsteps, const void *c,
                                   void *lam0, void *lam1, void *lam2, void *work)
{
    if (radius < 1 || radius > 4) return SADJ_ERR_UNSUPPORTED;
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!c || !lam0 || !lam1 || !lam2) return SADJ_ERR_NULL;
    if (nsteps < 0) return SADJ_ERR_SIZE;
    sadj_status s = check_extents(radius, nx, ny, nz, 3);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[1] = {{c, bytes}};
    const Span out[4] = {{lam0, bytes}, {lam1, bytes}, {lam2, bytes}, {work, work ? bytes : 0}};
    return check_arrays(in, out);
}

// Single steps k0 .. nsteps-1 rotating three buffers.
static sadj_status wave_steps_plain(int f64, int radius, long nx, long ny, long nz, long k0, long nsteps, const void *c,
                                    void *const (&lam)[3], const sadj::LaunchOptions &opt, hipStream_t st)
{
    for (long k = k0; k < nsteps; ++k) {
        void *a = lam[k % 3], *b = lam[(k + 1) % 3], *p = lam[(k + 2) % 3];
        // the buffer that receives -a was the r_bar of the previous step: it is dead and is assigned
        hipError_t e = sadj::launch_adjoint_wave3d(f64, radius, (int)nx, (int)ny, (int)nz, c, a, b, p, k > 0 ? 1 : 0,
                                                   opt, st);
        if (e != hipSuccess) return from_hip(e);
    }
    return SADJ_OK;
}

sadj_status sadj_adjoint_wave3d_steps(sadj_dtype dtype, int radius, long nx, long ny, long nz, long nsteps,
                                      const void *c, void *lam0, void *lam1, void *lam2, void *stream)
{
    if (sadj_status s = wave_steps_args(dtype, radius, nx, ny, nz, nsteps, c, lam0, lam1, lam2, nullptr); s != SADJ_OK) return s;
    void *const lam[3] = {lam0, lam1, lam2};
    clear_stale_hip_error();
    sadj::LaunchOptions opt = current_options();
    opt.remainder = 0;   // the strategy variants exist for the single-step call only
    return wave_steps_plain(dtype == SADJ_F64, radius, nx, ny, nz, 0, nsteps, c, lam, opt, static_cast<hipStream_t>(stream));
}

// The same sweep with a fourth array to work in: pairs of steps run fused where the kernel exists.
sadj_status sadj_adjoint_wave3d_steps_fused(sadj_dtype dtype, int radius, long nx, long ny, long nz, long nsteps,
                                            const void *c, void *lam0, void *lam1, void *lam2, void *work, void *stream)
{
    if (!work) return SADJ_ERR_NULL;
    if (sadj_status s = wave_steps_args(dtype, radius, nx, ny, nz, nsteps, c, lam0, lam1, lam2, work); s != SADJ_OK) return s;
    void *const lam[3] = {lam0, lam1, lam2};
    void *const buf[4] = {lam0, lam1, lam2, work};
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int f64 = dtype == SADJ_F64;
    clear_stale_hip_error();
    sadj::LaunchOptions opt = current_options();
    opt.remainder = 0;
    const bool fusable = radius == 1 && g_wave_fuse.load() == 0 &&
                         sadj::adjoint_wave3d_pair_supported(f64, (int)nx, c, lam0, lam1, lam2, work);
    const WaveSweepPlan plan = fusable ? plan_wave_sweep(nsteps) : WaveSweepPlan{};
    if (plan.plain) return wave_steps_plain(f64, radius, nx, ny, nz, 0, nsteps, c, lam, opt, st);
    // step 0 accumulates into lam2, which may hold the objective's own contribution
    if (sadj_status s = wave_steps_plain(f64, radius, nx, ny, nz, 0, 1, c, lam, opt, st); s != SADJ_OK) return s;
    auto run = [&](const WaveStepLaunch &l) {
        return l.pair ? sadj::launch_adjoint_wave3d_pair(f64, (int)nx, (int)ny, (int)nz, c, buf[l.a], buf[l.b], buf[l.o0],
                                                         buf[l.o1], opt, st)
                      : sadj::launch_adjoint_wave3d(f64, radius, (int)nx, (int)ny, (int)nz, c, buf[l.a], buf[l.b], buf[l.o0], 1,
                                                    opt, st);
    };
    for (long i = 0; i < plan.body_pairs; ++i) {
        const WaveStepLaunch l = i % 2 == 0 ? WaveStepLaunch{1, 1, 2, 0, 3} : WaveStepLaunch{1, 0, 3, 1, 2};
        if (hipError_t e = run(l); e != hipSuccess) return from_hip(e);
    }
    for (int i = 0; i < plan.tail_len; ++i)
        if (hipError_t e = run(plan.tail[i]); e != hipSuccess) return from_hip(e);
    return SADJ_OK;
}

// Diagnostic: the launches sadj_adjoint_wave3d_steps_fused makes after step 0 when pairs can be fused.
sadj_status sadj_describe_wave3d_sweep(long nsteps, long *body_pairs, int *tail_len, int *tail /* 5 ints per launch, 12 launches */)
{
    if (!body_pairs || !tail_len || !tail) return SADJ_ERR_NULL;
    if (nsteps < 0) return SADJ_ERR_SIZE;
    const WaveSweepPlan plan = plan_wave_sweep(nsteps);
    *body_pairs = plan.plain ? -1 : plan.body_pairs;
    *tail_len = plan.tail_len;
    for (int i = 0; i < plan.tail_len; ++i) {
        const WaveStepLaunch &l = plan.tail[i];
        const int v[5] = {l.pair, l.a, l.b, l.o0, l.o1};
        for (int k = 0; k < 5; ++k) tail[5 * i + k] = v[k];
    }
    return SADJ_OK;
}

// Streaming yardstick with the adjoint's access mix (two arrays read, one read and written).
sadj_status sadj_stream_probe(sadj_dtype dtype, int shape, long n, const void *a, const void *b, void *out,
                              void *stream)
{
    if (!dtype_ok(dtype) || shape < 0 || shape > 2) return SADJ_ERR_UNSUPPORTED;
    if (!a || !b || !out) return SADJ_ERR_NULL;
    if (n < 1 || n > (1L << 40)) return SADJ_ERR_SIZE;
    const size_t bytes = (size_t)n * elem(dtype);
    const Span in[2] = {{a, bytes}, {b, bytes}};
    const Span outs[1] = {{out, bytes}};
    if (sadj_status al = check_arrays(in, outs); al != SADJ_OK) return al;
    // vector accesses need 16-byte aligned arrays
    if (((uintptr_t)a | (uintptr_t)b | (uintptr_t)out) % 16 != 0) return SADJ_ERR_UNSUPPORTED;
    clear_stale_hip_error();
    return from_hip(sadj::launch_stream_probe(dtype == SADJ_F64, shape, (size_t)n, a, b, out,
                                              static_cast<hipStream_t>(stream)));
}

// ------------------------------------------------------------ dense 3^d box stencils
static sadj_status box_call(int adjoint, sadj_dtype dtype, int ndim, long nx, long ny, long nz,
                            const double *weights, const void *in0, const void *in1, void *out, void *stream)
{
    if (!dtype_ok(dtype) || ndim < 1 || ndim > 3) return SADJ_ERR_UNSUPPORTED;
    if (!weights || !in0 || !in1 || !out) return SADJ_ERR_NULL;
    if (ndim < 3) nz = 1;
    if (ndim < 2) ny = 1;
    sadj_status s = check_extents(1, nx, ny, nz, ndim);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[2] = {{in0, bytes}, {in1, bytes}};
    const Span outs[1] = {{out, bytes}};
    if (sadj_status al = check_arrays(in, outs); al != SADJ_OK) return al;
    // expand the caller's 3^ndim table to 27 entries (x fastest); the adjoint gathers with
    // the point-mirrored table W[o] = w[-o] (index shifting)
    double full[27] = {0};
    const int ey = ndim >= 2 ? 1 : 0, ez = ndim >= 3 ? 1 : 0;
    int k = 0;
    for (int oz = -ez; oz <= ez; ++oz)
        for (int oy = -ey; oy <= ey; ++oy)
            for (int ox = -1; ox <= 1; ++ox) full[(ox + 1) + 3 * (oy + 1) + 9 * (oz + 1)] = weights[k++];
    double gather[27];
    for (int i = 0; i < 27; ++i) gather[i] = adjoint ? full[26 - i] : full[i];
    hipStream_t st = static_cast<hipStream_t>(stream);
    clear_stale_hip_error();
    if (ndim == 1 && g_functor1d.load() == 1)      // primal: (u, c) -> r;  adjoint: (c, r_bar) -> u_bar, u not needed
        return from_hip(adjoint ? sadj::launch_weighted3_functor(1, dtype == SADJ_F64, nx, full + 12, nullptr, in0, in1, out, st)
                                : sadj::launch_weighted3_functor(0, dtype == SADJ_F64, nx, full + 12, in0, in1, nullptr, out, st));
    if (ndim == 1) return from_hip(sadj::launch_box1d(adjoint, dtype == SADJ_F64, nx, gather + 12, in0, in1, out, st));
    return from_hip(sadj::launch_box(adjoint, dtype == SADJ_F64, ndim, (int)nx, (int)ny, (int)nz, gather, in0, in1, out,
                                     current_options(), st));
}

sadj_status sadj_primal_box(sadj_dtype dtype, int ndim, long nx, long ny, long nz, const double *weights,
                            const void *u, const void *c, void *r, void *stream)
{
    return box_call(0, dtype, ndim, nx, ny, nz, weights, u, c, r, stream);
}

sadj_status sadj_adjoint_box(sadj_dtype dtype, int ndim, long nx, long ny, long nz, const double *weights,
                             const void *c, const void *r_bar, void *u_bar, void *stream)
{
    return box_call(1, dtype, ndim, nx, ny, nz, weights, c, r_bar, u_bar, stream);
}

// --------------------------------------------- 3-D star stencils with free weights
static sadj_status star_call(int adjoint, sadj_dtype dtype, int radius, long nx, long ny, long nz,
                             const double *weights, const void *in0, const void *in1, void *out, void *stream)
{
    if (!dtype_ok(dtype) || radius < 1 || radius > 4) return SADJ_ERR_UNSUPPORTED;
    if (!weights || !in0 || !in1 || !out) return SADJ_ERR_NULL;
    sadj_status s = check_extents(radius, nx, ny, nz, 3);
    if (s != SADJ_OK) return s;
    const size_t bytes = (size_t)nx * ny * nz * elem(dtype);
    const Span in[2] = {{in0, bytes}, {in1, bytes}};
    const Span outs[1] = {{out, bytes}};
    if (sadj_status al = check_arrays(in, outs); al != SADJ_OK) return al;
    // caller's table: centre, then per axis the offsets -R..-1, +1..+R; the adjoint gathers
    // with the mirrored table W[d][o] = w[d][-o] (index shifting)
    double w[3][8] = {};
    const int n = 2 * radius;
    for (int d = 0; d < 3; ++d)
        for (int i = 0; i < n; ++i) w[d][i] = weights[1 + d * n + (adjoint ? n - 1 - i : i)];
    clear_stale_hip_error();
    if (radius == 1 && g_functor_star.load() == 1) {
        const hipError_t e = sadj::launch_star7_functor(adjoint, dtype == SADJ_F64, (int)nx, (int)ny, (int)nz, weights, in0,
                                                        in1, out, static_cast<hipStream_t>(stream));
        if (e != hipErrorNotSupported) return from_hip(e);      // else: the hand-written kernel takes the call
    }
    return from_hip(sadj::launch_star3d(adjoint, dtype == SADJ_F64, radius, (int)nx, (int)ny, (int)nz, weights[0], w, in0,
                                        in1, out, current_options(), static_cast<hipStream_t>(stream)));
}

sadj_status sadj_primal_star3d(sadj_dtype dtype, int radius, long nx, long ny, long nz, const double *weights,
                               const void *u, const void *c, void *r, void *stream)
{
    return star_call(0, dtype, radius, nx, ny, nz, weights, u, c, r, stream);
}

sadj_status sadj_adjoint_star3d(sadj_dtype dtype, int radius, long nx, long ny, long nz, const double *weights,
                                const void *c, const void *r_bar, void *u_bar, void *stream)
{
    return star_call(1, dtype, radius, nx, ny, nz, weights, c, r_bar, u_bar, stream);
}

// ------------------------------------------------------------------------- Burgers
sadj_status sadj_primal_burgers1d(sadj_dtype dtype, long n, double C, double D, const void *u, void *r,
                                  void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!u || !r) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t bytes = (size_t)n * elem(dtype);
    const Span in[1] = {{u, bytes}};
    const Span out[1] = {{r, bytes}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    clear_stale_hip_error();
    if (g_functor1d.load() == 1)
        return from_hip(sadj::launch_burgers1d_functor(0, dtype == SADJ_F64, n, C, D, u, nullptr, r, static_cast<hipStream_t>(stream)));
    return from_hip(sadj::launch_primal_burgers1d(dtype == SADJ_F64, n, C, D, u, r, static_cast<hipStream_t>(stream)));
}

sadj_status sadj_adjoint_burgers1d(sadj_dtype dtype, long n, double C, double D, const void *u,
                                   const void *r_bar, void *u_bar, void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!u || !r_bar || !u_bar) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t bytes = (size_t)n * elem(dtype);
    const Span in[2] = {{u, bytes}, {r_bar, bytes}};
    const Span out[1] = {{u_bar, bytes}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    clear_stale_hip_error();
    if (g_functor1d.load() == 1)
        return from_hip(sadj::launch_burgers1d_functor(1, dtype == SADJ_F64, n, C, D, u, r_bar, u_bar,
                                                       static_cast<hipStream_t>(stream)));
    return from_hip(sadj::launch_adjoint_burgers1d(dtype == SADJ_F64, n, C, D, u, r_bar, u_bar, 0,
                                                   static_cast<hipStream_t>(stream)));
}

// Time loop of Burgers steps: forward sweep that stores every state, reverse sweep over them.
sadj_status sadj_primal_burgers1d_steps(sadj_dtype dtype, long n, long nsteps, double C, double D, void *states,
                                        void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!states) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent || nsteps < 0 || nsteps > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t row = (size_t)n * elem(dtype);
    if (g_check_pointers.load() == 1)
        if (sadj_status m = check_span_memory({states, (size_t)(nsteps + 1) * row}); m != SADJ_OK) return m;
    clear_stale_hip_error();
    char *base = static_cast<char *>(states);
    for (long t = 0; t < nsteps; ++t) {
        hipError_t e = sadj::launch_primal_burgers1d(dtype == SADJ_F64, n, C, D, base + (size_t)t * row,
                                                     base + (size_t)(t + 1) * row, static_cast<hipStream_t>(stream));
        if (e != hipSuccess) return from_hip(e);
    }
    return SADJ_OK;
}

sadj_status sadj_adjoint_burgers1d_steps(sadj_dtype dtype, long n, long last, long nsteps, double C, double D,
                                         const void *states, void *lam0, void *lam1, void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!states || !lam0 || !lam1) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent || nsteps < 0 || last < 0 || nsteps > last || last > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t row = (size_t)n * elem(dtype);
    // states u^{last-nsteps} .. u^{last-1} are read; lam0, lam1 are written
    const Span in[1] = {{static_cast<const char *>(states) + (size_t)(last - nsteps) * row, (size_t)nsteps * row}};
    const Span out[2] = {{lam0, row}, {lam1, row}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    clear_stale_hip_error();
    void *const lam[2] = {lam0, lam1};
    const char *base = static_cast<const char *>(states);
    // reverse step s undoes the primal step u^t -> u^{t+1}, t = last-1-s; lam[(s+1)%2] receives
    // lam^t; from s = 1 on it is the consumed buffer and is assigned
    auto applied = [&](long s) -> const void * { return base + (size_t)(last - 1 - s) * row; };
    long done = 0;
    return burgers_reverse_steps(dtype, n, C, D, nsteps, applied, lam, done, static_cast<hipStream_t>(stream));
}

// Time loop with checkpoints: every `every`-th state is kept, the others are recomputed
// segment by segment during the reverse sweep.
sadj_status sadj_primal_burgers1d_ckpt(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                       void *ckpt, void *work, void *u_final, void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (!ckpt || !work) return SADJ_ERR_NULL;
    if (n < 3 || n > kMaxExtent || nsteps < 0 || nsteps > kMaxExtent || every < 1 || every > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t row = (size_t)n * elem(dtype);
    const long rows = nsteps / every + 1;
    const Span in[1] = {{ckpt, (size_t)rows * row}};
    const Span out[2] = {{work, 2 * row}, {u_final, u_final ? row : 0}};
    if (sadj_status al = check_arrays(in, out); al != SADJ_OK) return al;
    clear_stale_hip_error();
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int f64 = dtype == SADJ_F64;
    char *cb = static_cast<char *>(ckpt), *wb = static_cast<char *>(work);
    const char *cur = cb;                                   // u^0
    for (long t = 0; t < nsteps; ++t) {
        // u^{t+1} goes to its checkpoint row if it has one, else to the work row not holding u^t
        char *dst = (t + 1) % every == 0 ? cb + (size_t)((t + 1) / every) * row : wb + (size_t)((t + 1) % 2) * row;
        hipError_t e = sadj::launch_primal_burgers1d(f64, n, C, D, cur, dst, st, 1);
        if (e != hipSuccess) return from_hip(e);
        cur = dst;
    }
    if (u_final) {
        hipError_t e = hipMemcpyAsync(u_final, cur, row, hipMemcpyDeviceToDevice, st);
        if (e != hipSuccess) return from_hip(e);
    }
    return SADJ_OK;
}

sadj_status sadj_adjoint_burgers1d_ckpt(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                        const void *ckpt, void *work, size_t work_bytes, void *lam0, void *lam1,
                                        void *stream)
{
    if (sadj_status s = burgers_ckpt_args(dtype, n, nsteps, every, ckpt, work, work_bytes, lam0, lam1); s != SADJ_OK) return s;
    clear_stale_hip_error();
    return burgers_ckpt_reverse(dtype, n, nsteps, every, C, D, ckpt, work, lam0, lam1, static_cast<hipStream_t>(stream));
}

// The same reverse sweep for callers that cannot allocate: the recomputed states go to the
// library's fixed scratch array.
sadj_status sadj_adjoint_burgers1d_ckpt_static(sadj_dtype dtype, long n, long nsteps, long every, double C, double D,
                                               const void *ckpt, void *lam0, void *lam1, void *stream)
{
    if (!dtype_ok(dtype)) return SADJ_ERR_UNSUPPORTED;
    if (n < 3 || n > kMaxExtent || every < 1 || every > kMaxExtent) return SADJ_ERR_SIZE;
    const size_t need = (size_t)(every - 1) * (size_t)n * elem(dtype);
    if (need > kStaticScratchBytes) return SADJ_ERR_SIZE;
    void *work = nullptr;
    if (sadj_status s = static_scratch_of_current_device(&work); s != SADJ_OK) return s;
    if (sadj_status s = burgers_ckpt_args(dtype, n, nsteps, every, ckpt, work, kStaticScratchBytes, lam0, lam1, true); s != SADJ_OK)
        return s;
    clear_stale_hip_error();
    return burgers_ckpt_reverse(dtype, n, nsteps, every, C, D, ckpt, work, lam0, lam1, static_cast<hipStream_t>(stream));
}

size_t sadj_static_scratch_bytes(void) { return kStaticScratchBytes; }

}  // extern "C"
