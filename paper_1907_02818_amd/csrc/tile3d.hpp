// Geometry shared by the 3-D marching kernels: an x-y tile of TX x TY cells owned by a
// workgroup of BX x BY threads (PX consecutive cells in x times PY consecutive rows
// per thread), staged in LDS with a
// halo of width R on all four sides (corners omitted: a star never reads them).
#pragma once
#include "common.hpp"
#include "launch.hpp"

namespace sadj {

template <class T, int R, int BX, int BY, int PY, int PX = 1>
struct Tile3d {
    static constexpr int TX = BX * PX, TY = BY * PY, NT = BX * BY;
    static constexpr int LX = TX + 2 * R, LY = TY + 2 * R;      // LDS plane extents
    static constexpr int PLANE = LX * LY;
    static constexpr int NH = 2 * R * TX + 2 * R * TY;          // halo cells without corners
    static constexpr int HS = (NH + NT - 1) / NT;               // halo slots per thread

    // Halo slot s of thread tid -> LDS coordinates (lx, ly); false if the slot is unused.
    // Slots 0 .. 2R*TX-1 are the R rows above and below the tile (x fastest), the rest
    // are the R columns left and right of it.
    __device__ static __forceinline__ bool halo_cell(int tid, int s, int &lx, int &ly)
    {
        const int h = tid + s * NT;
        if (h < 2 * R * TX) {
            const int row = h / TX;
            lx = R + h % TX;
            ly = row < R ? row : row + TY;
        } else {
            const int h2 = h - 2 * R * TX;
            const int k = h2 % (2 * R);
            lx = k < R ? k : k + TX;
            ly = R + h2 / (2 * R);
        }
        return h < NH;
    }
};

struct March3dArgs {
    const void *in0, *in1, *in2;   // adjoint: c, r_bar, -      primal: u, u_prev, c
    void *out0, *out1;             // adjoint: u_bar, u_prev_bar (nullable)   primal: r, -
    int out1_assign;               // adjoint: 1 = u_prev_bar is assigned (-r_bar on I, 0 elsewhere), 0 = accumulated
    int nx, ny, nz;
    int ntx, nty, ntz;             // tiles along x and y, chunks along z
    int zchunk;                    // output planes per chunk
    int total_blocks;
    int xcd_map, band;             // workgroup id -> tile mapping, see block_to_tile
    int round_blocks;              // workgroups resident at a time
};

// Workgroup id -> (tile x, tile y, z-chunk).
// Logical ids.  Workgroups are dealt to the 8 XCDs round-robin by hardware id and run in
// rounds of round_blocks (what the chip holds at a time).  xcd_map 1: within each round
// every XCD owns a contiguous range of logical ids, so all XCDs work on neighbouring tiles
// of the same chunk at a time and tiles that share halo cells meet in one L2 (default).
// xcd_map 2: one contiguous range per XCD over the whole dispatch (the same thing when
// there is a single round; with several rounds the XCDs drift to different z-chunks,
// measured 3-5 % slower).  xcd_map 3: logical id = hardware id (neighbouring tiles on
// different XCDs).
// Tiles of a chunk are numbered x fastest (band = 0) or in bands of `band` tile rows with
// y fastest inside a band, which makes the 32 tiles an XCD holds a compact patch.
template <class Args>
__host__ __device__ __forceinline__ void block_to_tile(const Args &a, int hw_id, int &tix, int &tiy, int &tiz)
{
    int L;
    if (a.xcd_map == 3) {
        L = hw_id;
    } else if (a.xcd_map == 2) {
        L = xcd_contiguous_id(hw_id, a.total_blocks);
    } else {
        const int round = hw_id / a.round_blocks;
        const int first = round * a.round_blocks;
        const int left = a.total_blocks - first;
        const int m = a.round_blocks < left ? a.round_blocks : left;
        L = first + xcd_contiguous_id(hw_id - first, m);
    }
    const int tiles = a.ntx * a.nty;
    tiz = L / tiles;
    const int t = L - tiz * tiles;
    if (a.band > 0) {
        const int b = t / (a.ntx * a.band);
        const int r = t - b * a.ntx * a.band;
        const int rows_left = a.nty - b * a.band;
        const int h = a.band < rows_left ? a.band : rows_left;
        tix = r / h;
        tiy = b * a.band + (r - tix * h);
    } else {
        tiy = t / a.ntx;
        tix = t - tiy * a.ntx;
    }
}

static inline int cdiv_i(int a, int b) { return (a + b - 1) / b; }

// Choose the number of z-chunks.  Each CU holds wg_per_cu workgroups of these kernels at a
// time (one, except where a kernel is built to overlap two), so the dispatch runs in rounds
// of `ncu` = CUs x wg_per_cu workgroups, each marching zchunk + 2R planes
// (the 2R planes beyond a chunk are read by two chunks).  Minimise rounds * planes per
// workgroup; ties go to fewer chunks.  With tiles*chunks == ncu this is the single
// resident wave in which neighbouring tiles move through z in lockstep.
static inline void plan_march(March3dArgs &a, int TX, int TY, int R, const LaunchOptions &opt, int wg_per_cu = 1)
{
    a.ntx = cdiv_i(a.nx, TX);
    a.nty = cdiv_i(a.ny, TY);
    int dev = 0, ncu = 256, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        ncu = v;
    a.xcd_map = opt.xcd_map > 0 ? (int)opt.xcd_map : 1;
    a.band = (int)opt.band;
    // ids are made XCD-contiguous per group of one workgroup per CU, also where two groups
    // are resident together (measured better than one contiguous range per XCD over both)
    a.round_blocks = ncu >= 8 ? ncu - ncu % 8 : 8;
    ncu *= wg_per_cu;                                  // workgroups resident at a time
    int zchunk = (int)opt.zchunk;
    if (zchunk <= 0) {
        const long tiles = (long)a.ntx * a.nty;
        long best_cost = -1;
        int best_chunks = 1;
        const int max_chunks = a.nz / (4 * R) > 0 ? a.nz / (4 * R) : 1;   // chunks of at least 4R planes
        for (int c = 1; c <= max_chunks && c <= 64; ++c) {
            const long rounds = (tiles * c + ncu - 1) / ncu;
            const long cost = rounds * (cdiv_i(a.nz, c) + 2 * R);
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best_chunks = c; }
        }
        zchunk = cdiv_i(a.nz, best_chunks);
    }
    if (zchunk > a.nz) zchunk = a.nz;
    if (zchunk < 1) zchunk = 1;
    // the grid is one-dimensional: keep the number of workgroups a valid int
    while ((long)a.ntx * a.nty * cdiv_i(a.nz, zchunk) > 0x3fffffffL && zchunk < a.nz) zchunk *= 2;
    if (zchunk > a.nz) zchunk = a.nz;
    a.zchunk = zchunk;
    a.ntz = cdiv_i(a.nz, zchunk);
    a.total_blocks = a.ntx * a.nty * a.ntz;
}

// The marching kernels are planned for one workgroup per CU (rounds of ncu workgroups that
// move through z together).  Kernels that need few registers and little LDS would otherwise
// be packed two or more to a CU, which measured 2-9 % slower at grid sizes with several
// rounds; requesting unused dynamic LDS up to more than half of a CU's 160 KB keeps them at
// one.  Returns the dynamic LDS bytes to request for a kernel with `static_lds` bytes.
static inline unsigned one_workgroup_per_cu_pad(size_t static_lds, long override_bytes)
{
    if (override_bytes > 0) return (unsigned)override_bytes;
    if (override_bytes < 0) return 0;
    constexpr size_t half = 80 * 1024, max_dynamic = 64 * 1024;
    if (static_lds > half) return 0;
    const size_t want = half + 2048 - static_lds;
    return (unsigned)(want < max_dynamic ? want : max_dynamic);
}

template <class T, bool NT> __device__ __forceinline__ T ld_stream(const T *base, uint32_t byte_off)
{
    const T *p = reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + byte_off);
    return NT ? __builtin_nontemporal_load(p) : *p;
}
template <class T, bool NT> __device__ __forceinline__ void st_stream(T *base, uint32_t byte_off, T v)
{
    T *p = reinterpret_cast<T *>(reinterpret_cast<char *>(base) + byte_off);
    if (NT) __builtin_nontemporal_store(v, p);
    else *p = v;
}

// PX consecutive cells at a 32-bit byte offset from a uniform base pointer.
template <class T, int N, bool NT> __device__ __forceinline__ Vec<T, N> ld_vec_off(const T *base, uint32_t byte_off)
{
    const T *p = reinterpret_cast<const T *>(reinterpret_cast<const char *>(base) + byte_off);
    return NT ? ld_vec_stream<T, N>(p) : ld_vec<T, N>(p);
}
template <class T, int N, bool NT> __device__ __forceinline__ void st_vec_off(T *base, uint32_t byte_off, const Vec<T, N> &v)
{
    T *p = reinterpret_cast<T *>(reinterpret_cast<char *>(base) + byte_off);
    if (NT) st_vec_stream<T, N>(p, v);
    else st_vec<T, N>(p, v);
}

}  // namespace sadj
