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

// Per-thread addressing of a marching kernel's tile, computed once before the march and shared
// by the 3-D kernels (wave adjoint and primal, free-weight star, box, scatter-order adjoint).
// A thread owns PX consecutive cells in x times PY consecutive rows and HS halo slots.  For
// each it gets the byte offset inside an x-y plane and two predicates: "lies in the grid" and
// "lies in the primal iteration space I in x and y" (at least `margin` cells from the grid's
// edge).  Offsets of owned vectors outside the grid and of halo slots that are unused or
// outside the grid point at `dummy`, a cell that is always inside the grid, so that a load
// through them is harmless; which of the two predicates decides about a cell's value is the
// kernel's business (an adjoint uses c and r_bar on I only, a primal reads u on the whole
// grid).  GUARD = false (core tiles: everything lies in I) folds all predicates to constants.
template <int PX, int PY, int HS, bool GUARD> struct TileAddr {
    uint32_t dummy;
    uint32_t own_off[PY];     // owned vector of row p (nx is a multiple of PX: inside or outside the grid as a whole)
    bool own_grid[PY];
    bool own_I[PY][PX];
    uint32_t halo_off[HS];
    bool halo_grid[HS], halo_I[HS];
    int halo_lds[HS];

    // halo_cell(s, lx, ly) -> does slot s of this thread exist, and its LDS coordinates; the LDS
    // plane has row length LX and its origin `halo` cells left of and above the tile.
    template <class HaloCell>
    __device__ __forceinline__ void init(int tx, int ty, int x0, int y0, int nx, int ny, int margin, int halo, int LX,
                                         int unused_lds, uint32_t elem_bytes, HaloCell halo_cell)
    {
        dummy = (uint32_t)((size_t)y0 * nx + x0) * elem_bytes;
        const int x = x0 + tx * PX;
#pragma unroll
        for (int p = 0; p < PY; ++p) {
            const int y = y0 + ty * PY + p;
            own_grid[p] = GUARD ? (x < nx && y < ny) : true;
#pragma unroll
            for (int e = 0; e < PX; ++e)
                own_I[p][e] = GUARD ? (x + e >= margin && x + e < nx - margin && y >= margin && y < ny - margin) : true;
            own_off[p] = own_grid[p] ? (uint32_t)((size_t)y * nx + x) * elem_bytes : dummy;
        }
#pragma unroll
        for (int s = 0; s < HS; ++s) {
            int lx, ly;
            const bool slot = halo_cell(s, lx, ly);
            const int gx = x0 - halo + lx, gy = y0 - halo + ly;
            halo_grid[s] = slot && (!GUARD || (gx >= 0 && gx < nx && gy >= 0 && gy < ny));
            halo_I[s] = slot && (!GUARD || (gx >= margin && gx < nx - margin && gy >= margin && gy < ny - margin));
            halo_off[s] = halo_grid[s] ? (uint32_t)((size_t)gy * nx + gx) * elem_bytes : dummy;
            halo_lds[s] = slot ? ly * LX + lx : unused_lds;
        }
    }
};

// Workgroup id -> (x-y tile, range of planes) of a 3-D march; filled by plan_march.
// The tiles are numbered 0 .. ntx*nty-1 (see `band`).  The first tiles_a of them are cut
// into ntz_a chunks of zchunk_a planes, the others into ntz chunks of zchunk planes;
// workgroup ids run over the first group, then over the second, within a group over
// all tiles of chunk 0, then chunk 1, ...
struct TileMap {
    int ntx, nty, nz;
    int tiles_a, ntz_a, zchunk_a, blocks_a;   // first group (tiles_a = 0: none)
    int ntz, zchunk;                          // second group
    int total_blocks;
    int xcd_map, band;                        // see block_to_tile
    int round_blocks;                         // workgroups per round of XCD-contiguous ids
};

struct March3dArgs {
    const void *in0, *in1, *in2;   // adjoint: c, r_bar, -      primal: u, u_prev, c
    void *out0, *out1;             // adjoint: u_bar, u_prev_bar (nullable)   primal: r, -
    int out1_assign;               // adjoint: 1 = u_prev_bar is assigned (-r_bar on I, 0 elsewhere), 0 = accumulated
    int nx, ny, nz;
    TileMap map;
};

// Workgroup id -> (tile x, tile y, planes zs .. ze-1).
// Logical ids.  Workgroups are dealt to the 8 XCDs round-robin by hardware id and run in
// rounds of round_blocks (what the chip holds at a time).  xcd_map 1: within each round
// every XCD owns a contiguous range of logical ids, so all XCDs work on neighbouring tiles
// of the same chunk at a time and tiles that share halo cells meet in one L2 (default).
// xcd_map 2: one contiguous range per XCD over the whole dispatch (the same thing when
// there is a single round; with several rounds the XCDs drift to different z-chunks,
// measured 3-5 % slower).  xcd_map 3: logical id = hardware id (neighbouring tiles on
// different XCDs).
// Tiles are numbered x fastest (band = 0) or in bands of `band` tile rows with
// y fastest inside a band, which makes the 32 tiles an XCD holds a compact patch
// (plan_march chooses, see there).
__host__ __device__ __forceinline__ void block_to_tile(const TileMap &m, int hw_id, int &tix, int &tiy, int &zs, int &ze)
{
    int L;
    if (m.xcd_map == 3) {
        L = hw_id;
    } else if (m.xcd_map == 2) {
        L = xcd_contiguous_id(hw_id, m.total_blocks);
    } else {
        const int round = hw_id / m.round_blocks;
        const int first = round * m.round_blocks;
        const int left = m.total_blocks - first;
        const int n = m.round_blocks < left ? m.round_blocks : left;
        L = first + xcd_contiguous_id(hw_id - first, n);
    }
    int t, zchunk;
    if (L < m.blocks_a) {
        const int tiz = L / m.tiles_a;
        t = L - tiz * m.tiles_a;
        zchunk = m.zchunk_a;
        zs = tiz * zchunk;
    } else {
        const int tiles_b = m.ntx * m.nty - m.tiles_a;
        const int Lb = L - m.blocks_a;
        const int tiz = Lb / tiles_b;
        t = m.tiles_a + (Lb - tiz * tiles_b);
        zchunk = m.zchunk;
        zs = tiz * zchunk;
    }
    ze = zs + zchunk < m.nz ? zs + zchunk : m.nz;
    if (m.band > 0) {
        const int b = t / (m.ntx * m.band);
        const int r = t - b * m.ntx * m.band;
        const int rows_left = m.nty - b * m.band;
        const int h = m.band < rows_left ? m.band : rows_left;
        tix = r / h;
        tiy = b * m.band + (r - tix * h);
    } else {
        tiy = t / m.ntx;
        tix = t - tiy * m.ntx;
    }
}

static inline int cdiv_i(int a, int b) { return (a + b - 1) / b; }

// Cut the grid into workgroups.  Each CU holds wg_per_cu workgroups of these kernels at a
// time (one, except where a kernel is built to overlap two), so the dispatch runs in rounds
// of `ncu` = CUs x wg_per_cu workgroups, each marching its chunk + 2R planes (the 2R planes
// beyond a chunk are read by two chunks).  The model of the run time is the sum over rounds
// of the planes a workgroup of that round marches.  Candidates: every tile cut into the same
// number of chunks; or the tiles that fill whole rounds with few (long) chunks each cut
// alike and only the left-over tiles cut finer, so that they fill one more round instead of
// leaving most CUs idle (768^3 with 64 x 32 tiles: 256 tiles march all 768 planes, the
// other 32 are cut into 8 chunks of 96: 768 + 96 + 2*2R = 880 plane times instead of 9 rounds
// of 96 + 2R, 936).  Ties go to fewer workgroups.  With tiles*chunks == ncu this is the single
// resident wave in which neighbouring tiles move through z in lockstep.
static inline void plan_march(TileMap &m, int nx, int ny, int nz, int TX, int TY, int R, const LaunchOptions &opt,
                              int wg_per_cu = 1)
{
    m = TileMap{};
    m.ntx = cdiv_i(nx, TX);
    m.nty = cdiv_i(ny, TY);
    m.nz = nz;
    int dev = 0, ncu = 256, v = 0;
    if (hipGetDevice(&dev) == hipSuccess &&
        hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0)
        ncu = v;
    m.xcd_map = opt.xcd_map > 0 ? (int)opt.xcd_map : 1;
    // rows of 32 or more tiles: one XCD's 32 tiles would be a single thin strip whose halo rows
    // are all fetched a second time by the XCDs above and below; bands of 8 rows make the patch
    // 4 x 8 tiles (2048-wide and wider planes measured 2-4 points faster).  Only where the plane
    // has the 8 tile rows of a full band; with fewer rows no order measured better than another.
    m.band = opt.band > 0 ? (int)opt.band : (m.ntx >= 32 && m.nty >= 8 ? 8 : 0);
    // ids are made XCD-contiguous per group of one workgroup per CU, also where two groups
    // are resident together (measured better than one contiguous range per XCD over both)
    m.round_blocks = ncu >= 8 ? ncu - ncu % 8 : 8;
    ncu *= wg_per_cu;                                  // workgroups resident at a time
    const long tiles = (long)m.ntx * m.nty;
    // chunks of at least 4R planes; at most 64 of them, or what fills the chip where the grid has few tiles
    const long chunk_cap = tiles * 64 >= ncu ? 64 : (ncu + tiles - 1) / tiles;
    const int max_chunks = nz / (4 * R) > 0 ? (int)(nz / (4 * R) < chunk_cap ? nz / (4 * R) : chunk_cap) : 1;
    int zchunk = (int)opt.zchunk;
    if (zchunk <= 0) {
        long best_cost = -1, best_blocks = 0;
        int best_a = 0, best_ca = 1, best_cb = 1;
        auto consider = [&](long tiles_a, int ca, int cb) {
            const long blocks = tiles_a * ca + (tiles - tiles_a) * cb;
            const long cost = (tiles_a * ca + ncu - 1) / ncu * (cdiv_i(nz, ca) + 2 * R) +
                              ((tiles - tiles_a) * cb + ncu - 1) / ncu * (cdiv_i(nz, cb) + 2 * R);
            if (best_cost < 0 || cost < best_cost || (cost == best_cost && blocks < best_blocks)) {
                best_cost = cost; best_blocks = blocks; best_a = (int)tiles_a; best_ca = ca; best_cb = cb;
            }
        };
        for (int c = 1; c <= max_chunks; ++c) consider(0, 1, c);
        if (opt.split == 0 && tiles < 0x3fffffffL / 64) {
            for (int ca = 1; ca <= max_chunks && ca <= 8; ++ca) {
                // the largest number of tiles whose ca chunks fill whole rounds
                long g = ncu, x = ca;
                while (x) { const long r = g % x; g = x; x = r; }
                const long step = ncu / g;
                const long tiles_a = tiles / step * step;
                if (tiles_a == 0 || tiles_a == tiles) continue;
                for (int cb = ca + 1; cb <= max_chunks; ++cb) consider(tiles_a, ca, cb);
            }
        }
        m.tiles_a = best_a;
        m.ntz_a = best_a ? best_ca : 0;
        m.zchunk_a = best_a ? cdiv_i(nz, best_ca) : 0;
        zchunk = cdiv_i(nz, best_cb);
    }
    if (zchunk > nz) zchunk = nz;
    if (zchunk < 1) zchunk = 1;
    // the grid is one-dimensional: keep the number of workgroups a valid int
    while (tiles * cdiv_i(nz, zchunk) > 0x3fffffffL && zchunk < nz) zchunk *= 2;
    if (zchunk > nz) zchunk = nz;
    m.zchunk = zchunk;
    m.ntz = cdiv_i(nz, zchunk);
    if (m.tiles_a) m.ntz_a = cdiv_i(nz, m.zchunk_a);
    m.blocks_a = m.tiles_a * m.ntz_a;
    m.total_blocks = m.blocks_a + (int)(tiles - m.tiles_a) * m.ntz;
}

// Rows whose length in bytes is not a multiple of the 128-byte cache line (nx = 1000 in fp64:
// every other row starts in the middle of a line).  Tile rows then begin and end inside a line
// on most rows, and tiles with long rows (fewer row ends per byte) measured faster than the
// default shapes, while for line-aligned rows they measured equal or slower.
//
// Radius 1 keeps three running sums per cell, so eight cells per lane fit the register file:
// tiles of 256 (fp32 adjoint: 512) cells x 16 rows measured 4-10 points faster (500^3, 1000^3,
// 200 x 700 x 1500, both dtypes, adjoint and primal).  Larger radii stay at four fp64 (eight
// fp32) cells per lane and trade tile rows for width: 1 KB x 16 rows instead of 512 B x 32
// (radius 4 fp64 at 500^3, 1000^3, 250 x 900 x 1100, 300 x 300 x 1250: adjoint +2 to +5
// points, with u_prev_bar +3 to +7, primal +3 to +6).
//
// Returns the tile width in cells to use, or 0 for the default shape; a width qualifies if its
// tiles cover nx with at most 10 % idle columns.
static inline int wide_tile_for_unaligned_rows(int nx, size_t elem_bytes, int radius, bool allow_512)
{
    if (((size_t)nx * elem_bytes) % 128 == 0) return 0;
    auto fills = [nx](int tx) { return 10L * nx >= 9L * cdiv_i(nx, tx) * tx; };
    if (radius == 1) {
        if (allow_512 && fills(512)) return 512;
        return fills(256) ? 256 : 0;
    }
    const int tx = (int)(1024 / elem_bytes);
    return fills(tx) ? tx : 0;
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
