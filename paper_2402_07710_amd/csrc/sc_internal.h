// Internal definitions shared by the HIP translation units of libsc (gfx950 only).
// Nothing here is visible through the C ABI; the public contract is include/sc.h.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdlib.h>

#include "sc.h"

namespace sc {

constexpr int WAVE = 64;                      // CDNA wavefront
constexpr int TILE = 64;                      // output rows per kernel-map tile (= one wavefront)
constexpr uint64_t KEY_EMPTY = ~0ull;         // epoch field 0xff: no build ever uses it
constexpr uint32_t KMAP_MAGIC = 0x70614d6bu;

// ---- coordinate keys ------------------------------------------------------------------------
// The paper linearises (x,y,z) into one dense-array index (Section III-C.1 eq. 6); the batch
// index is part of the coordinate (Section II-A), so here the batch (8 bits) and the three 16-bit
// coordinates are packed into the low 56 bits of one 64-bit word.  The top 8 bits of a stored
// word carry the epoch of the build that wrote it: a slot whose epoch is not the table's current
// one is free, whatever else it holds, so a table that is built again needs no refill.
constexpr int KEY_EPOCH_SHIFT = 56;
__host__ __device__ inline uint64_t pack_key(int b, int x, int y, int z) {
    return ((uint64_t)(uint32_t)b << 48) | ((uint64_t)(uint32_t)x << 32) |
           ((uint64_t)(uint32_t)y << 16) | (uint64_t)(uint32_t)z;
}
__host__ __device__ inline uint64_t epoch_tag(uint32_t epoch) { return (uint64_t)epoch << KEY_EPOCH_SHIFT; }
__host__ __device__ inline bool same_epoch(uint64_t word, uint64_t tag) { return ((word ^ tag) >> KEY_EPOCH_SHIFT) == 0; }
__host__ __device__ inline bool in_domain(int v) { return (unsigned)v <= (unsigned)SC_COORD_MAX; }
__host__ __device__ inline bool in_domain4(int b, int x, int y, int z) {
    return (unsigned)b <= (unsigned)SC_BATCH_MAX && in_domain(x) && in_domain(y) && in_domain(z);
}

// Probe sequence of a key.  The table is cut into regions of 64 slots; a 4x4x4 block of cells
// owns one region per attempt t (a hash of the block's coordinates and t) and a cell sits at its
// own place inside the region (its 6 low coordinate bits, turned by 6 bits of the same hash).  Cells of one block therefore never
// collide with each other, the 27 neighbours of a voxel fall into at most 8 regions, and voxels
// that are close in space read the same cache lines of the table.  After REHASH_MAX attempts the
// sequence continues linearly, so it visits every slot and always ends at an empty one.
constexpr uint32_t REHASH_MAX = 32;
__host__ __device__ inline uint32_t mix_block(uint32_t hi, uint32_t lo, uint32_t t) {
    uint32_t h = hi * 0x85ebca6bu ^ lo * 0xc2b2ae35u ^ (t + 1u) * 0x9e3779b9u;
    h ^= h >> 15; h *= 0x2c1b3c6du;
    h ^= h >> 12; h *= 0x297a2d39u;
    h ^= h >> 15;
    return h;
}
__host__ __device__ inline uint32_t probe_slot(uint64_t key, uint32_t t, uint32_t mask) {
    const uint32_t hi = (uint32_t)(key >> 32) & 0xfffffffcu;          // b, x >> 2
    const uint32_t lo = (uint32_t)key & 0xfffcfffcu;                  // y >> 2, z >> 2
    const uint32_t local = (((uint32_t)(key >> 32) & 3u) << 4) | (((uint32_t)(key >> 16) & 3u) << 2) | ((uint32_t)key & 3u);
    const uint32_t tt = t < REHASH_MAX ? t : REHASH_MAX - 1;
    // the place inside the region is turned by six more bits of the block's hash: one turn for the
    // whole block and attempt, so its cells still never collide with each other, but voxel sets
    // on a coarse lattice (every coordinate a multiple of 2 or 4, as after down-sampling at the
    // original scale) no longer all ask for the same few places of every region
    const uint32_t h = mix_block(hi, lo, tt);
    const uint32_t slot = ((h << 6) | (local ^ (h >> 26))) + (t - tt);
    return slot & mask;
}

// Slots for n keys at `per_key` slots each: the next power of two, at least 1024.
inline uint64_t hash_capacity(int64_t n, uint64_t per_key) {
    uint64_t cap = 1024;
    while (cap < per_key * (uint64_t)(n < 0 ? 0 : n)) cap <<= 1;
    return cap;
}
// Capacity of the location table.  Probe chains decide the cost of the build and of the kernel
// map (every extra attempt is one more dependent round trip for the whole wavefront), and memory
// is cheap.  What a sparser table costs is its fill - and a table that is built again skips the
// fill as long as it has at most NO_FILL_SLOTS_MAX slots (sc_hash_rebuild).  So: 32 slots per key
// while that stays within the no-fill size, never fewer than 8.  Measured, whole layers with the
// table reused: ~53k voxels 8n 33.5 us, 16n 31.0, 32n 29.8; ~110k voxels 8n 78.4, 16n 73.0, 32n
// 70.3; 10^6 voxels (filled every time) 8n 900, 16n 929, 32n 990.  (When every build still
// filled the table, ~53k voxels: 2n 121 us, 4n 46, 8n 37, 16n 36.5.)
constexpr uint64_t NO_FILL_SLOTS_MAX = 1ull << 22;      // 64 MiB of slots
inline uint64_t table_capacity(int64_t n) {
    const uint64_t dense = hash_capacity(n, 8), sparse = hash_capacity(n, 32);
    const uint64_t capped = sparse < NO_FILL_SLOTS_MAX ? sparse : NO_FILL_SLOTS_MAX;
    return dense > capped ? dense : capped;
}

// One 16-byte slot per key: {epoch | key (8 bytes), value (4), unused (4)}, so a probe is one
// 16-byte load that brings the key and the row index together.  A 256-byte header precedes the
// slots: the table's capacity (fixed by the build that filled it), the epoch of the last build,
// and the first error a build without a fill came across (tagged with its epoch, so it needs no
// reset: stale tags never match).
struct TableHeader {
    uint32_t mask;            // capacity - 1
    uint32_t epoch;           // of the last build (0 after sc_hash_build)
    uint32_t err_tag;         // (epoch << 8) | -status of a build with epoch >= 1, or 0
    uint32_t pad[61];
};
static_assert(sizeof(TableHeader) == 256, "table header");
struct HashTable {            // view of a caller-owned table buffer
    TableHeader* hdr;
    uint4* slots;             // [cap]: x,y = epoch | key (low, high), z = value
    uint32_t mask;            // cap - 1 of a table for n keys (what the header of a fresh table says)
};
inline HashTable table_view(void* p, int64_t n) {
    HashTable t;
    t.hdr = (TableHeader*)p;
    t.slots = (uint4*)((char*)p + sizeof(TableHeader));
    t.mask = (uint32_t)(table_capacity(n) - 1);
    return t;
}
__host__ __device__ inline uint64_t slot_key(const uint4& s) { return (uint64_t)s.x | ((uint64_t)s.y << 32); }

// Probe for `key` among the slots of the epoch in `tag`; returns the stored value or -1.  The
// table is never full.
__device__ inline int32_t table_find(const uint4* __restrict__ slots, uint32_t mask, uint64_t key, uint64_t tag) {
    for (uint32_t t = 0; t <= mask + REHASH_MAX; ++t) {
        const uint4 s = slots[probe_slot(key, t, mask)];
        const uint64_t cur = slot_key(s);
        if (cur == (key | tag)) return (int32_t)s.z;
        if (!same_epoch(cur, tag)) return -1;
    }
    return -1;
}

__device__ inline void latch_status(sc_counts* counts, int code) {
    atomicCAS(&counts->status, 0, code);
}

// every slot <- {EMPTY, val_init}; optionally *counts reset (defined in sc_hash.hip)
int launch_table_fill(uint4* slots, uint64_t cap, int32_t val_init, sc_counts* counts, int64_t n_in, hipStream_t s,
                      TableHeader* th = nullptr, uint32_t epoch = 0);
// what a later build on `table` has to report: the error of an epoch >= 1 build, if any
__device__ inline void fold_table_error(const TableHeader* th, sc_counts* counts) {
    const uint32_t e = th->epoch, tag = th->err_tag;
    if (e != 0 && (tag >> 8) == e) latch_status(counts, -(int)(tag & 0xffu));
}

// ---- dense location table (sc_grid.hip) -------------------------------------------------------
// One 8-byte cell {row (low 32 bits), epoch (high 32 bits)} per site of the box, z fastest.
struct GridDims {
    int32_t B, X, Y, Z;
};
__host__ __device__ inline int64_t grid_cells(GridDims d) { return (int64_t)d.B * d.X * d.Y * d.Z; }
__device__ inline bool grid_inside(GridDims d, int b, int x, int y, int z) {
    return (unsigned)b < (unsigned)d.B && (unsigned)x < (unsigned)d.X && (unsigned)y < (unsigned)d.Y &&
           (unsigned)z < (unsigned)d.Z;
}
__device__ inline int64_t grid_index(GridDims d, int b, int x, int y, int z) {
    return (((int64_t)b * d.X + x) * d.Y + y) * d.Z + z;
}

// Where a convolution kernel finds the neighbours of its rows: the offset table of a kernel-map
// blob (mask + nbr), or - fused layers - the dense location table itself, looked up on the fly.
struct MapSource {
    const uint32_t* gmask;
    const int32_t* nbr;
    const int4* coords;
    const unsigned long long* cells;
    GridDims dims;
    uint32_t epoch;
};
// The K^3 neighbours of `row` (its own index at the centre), straight from the dense table:
// what k_kmap_subm_grid stores as the row's column of the offset table.
template <int K>
__device__ inline void grid_neighbours(const MapSource& ms, int64_t row, int64_t n, int32_t (&e)[K * K * K]) {
    constexpr int K3 = K * K * K, pad = (K - 1) / 2, centre = (K3 - 1) / 2;
    const bool valid = row < n;
    int4 c = make_int4(-1, 0, 0, 0);
    if (valid) c = ms.coords[row];
    const bool ok = valid && grid_inside(ms.dims, c.x, c.y, c.z, c.w);
    const int64_t base = ok ? grid_index(ms.dims, c.x, c.y, c.z, c.w) : 0;
    unsigned long long got[K3];
    bool look[K3];
#pragma unroll
    for (int k = 0; k < K3; ++k) {
        const int dx = k / (K * K) - pad, dy = (k / K) % K - pad, dz = k % K - pad;
        look[k] = ok && k != centre && (unsigned)(c.y + dx) < (unsigned)ms.dims.X &&
                  (unsigned)(c.z + dy) < (unsigned)ms.dims.Y && (unsigned)(c.w + dz) < (unsigned)ms.dims.Z;
        got[k] = look[k] ? ms.cells[base + ((int64_t)dx * ms.dims.Y + dy) * ms.dims.Z + dz] : 0ull;
    }
#pragma unroll
    for (int k = 0; k < K3; ++k) {
        if (k == centre) e[k] = valid ? (int32_t)row : -1;
        else e[k] = (look[k] && (uint32_t)(got[k] >> 32) == ms.epoch) ? (int32_t)(uint32_t)got[k] : -1;
    }
}

// The same for every fourth offset only, k = first + 4u (u = 0..ceil(K^3/4)-1; entries past K^3 are
// -1): four lanes that serve one row share the look-ups instead of repeating them.
template <int K>
__device__ inline void grid_neighbours_quarter(const MapSource& ms, int64_t row, int64_t n, int first,
                                               int32_t (&e)[(K * K * K + 3) / 4]) {
    constexpr int K3 = K * K * K, pad = (K - 1) / 2, centre = (K3 - 1) / 2, NQ = (K3 + 3) / 4;
    const bool valid = row < n;
    int4 c = make_int4(-1, 0, 0, 0);
    if (valid) c = ms.coords[row];
    const bool ok = valid && grid_inside(ms.dims, c.x, c.y, c.z, c.w);
    const int64_t base = ok ? grid_index(ms.dims, c.x, c.y, c.z, c.w) : 0;
    unsigned long long got[NQ];
    bool look[NQ];
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = first + 4 * u;
        const int dx = k / (K * K) - pad, dy = (k / K) % K - pad, dz = k % K - pad;
        look[u] = ok && k < K3 && k != centre && (unsigned)(c.y + dx) < (unsigned)ms.dims.X &&
                  (unsigned)(c.z + dy) < (unsigned)ms.dims.Y && (unsigned)(c.w + dz) < (unsigned)ms.dims.Z;
        got[u] = look[u] ? ms.cells[base + ((int64_t)dx * ms.dims.Y + dy) * ms.dims.Z + dz] : 0ull;
    }
#pragma unroll
    for (int u = 0; u < NQ; ++u) {
        const int k = first + 4 * u;
        if (k == centre) e[u] = valid ? (int32_t)row : -1;
        else e[u] = (look[u] && (uint32_t)(got[u] >> 32) == ms.epoch) ? (int32_t)(uint32_t)got[u] : -1;
    }
}

// ---- kernel-map blob ------------------------------------------------------------------------
// header | mask[T][4][mw] (uint32) | nbr[T][K3][TILE] (int32)
// Outputs are cut into tiles of 64 consecutive rows.  nbr[t][k][j] is the input row paired with
// output row 64t+j at offset k, or -1: the paper's offset table (Section III-C.2), stored
// offset-major inside a tile so that the 16 rows an MFMA group takes are 64 contiguous bytes.
// Bit k of mask[t][q] (word k/32) says whether any of the rows 16q..16q+15 of tile t has a
// neighbour at offset k; the convolution skips the groups whose bit is clear.
struct KmapHeader {
    uint32_t magic;
    int32_t K, stride, mode;
    int64_t n_in, n_out_bound;
    int64_t tiles;
    int32_t mw, reserved;
};
struct KmapLayout {
    int64_t tiles;        // T = ceil(n_out_bound / TILE)
    int K3;
    int mw;               // mask words per (tile, quarter) = ceil(K3 / 32)
    size_t off_mask;      // byte offsets inside the blob
    size_t off_nbr;
    size_t bytes;
};
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline KmapLayout kmap_layout(int64_t n_out_bound, int K) {
    KmapLayout L;
    L.K3 = K * K * K;
    L.mw = (L.K3 + 31) / 32;
    L.tiles = (n_out_bound + TILE - 1) / TILE;
    L.off_mask = 256;
    L.off_nbr = align_up(L.off_mask + (size_t)L.tiles * 4 * L.mw * sizeof(uint32_t), 256);
    L.bytes = align_up(L.off_nbr + (size_t)L.tiles * L.K3 * TILE * sizeof(int32_t), 256);
    return L;
}

// Workgroup -> work unit, XCD-aware.  MI355X hands consecutive workgroups to its 8 XCDs in turn
// and every XCD has its own L2.  Units (tiles of consecutive rows) that are close in index are
// close in space, so each XCD is given one contiguous eighth of the units: the slice of the
// location table and of the feature rows it touches is then fetched into one L2, not eight.
// Launch xcd_grid(units) workgroups; a workgroup whose unit is >= units has nothing to do.
constexpr int NUM_XCD = 8;
inline unsigned xcd_grid(int64_t units) { return (unsigned)((units + NUM_XCD - 1) / NUM_XCD * NUM_XCD); }
__device__ inline int64_t xcd_unit(unsigned block, unsigned grid) {
    const unsigned chunk = grid / NUM_XCD;
    return (int64_t)(block % NUM_XCD) * chunk + block / NUM_XCD;
}
// The same when the grid was sized for a bound and only `units` units exist (output rows are
// counted on the device): the units that exist are dealt out in eighths, so all XCDs work, and a
// workgroup without a unit gets -1.  Needs gridDim.x >= xcd_grid(units).
__device__ inline int64_t xcd_unit_of(unsigned block, int64_t units) {
    const int64_t chunk = (units + NUM_XCD - 1) / NUM_XCD;
    const int64_t u = (int64_t)(block % NUM_XCD) * chunk + block / NUM_XCD;
    return (block / NUM_XCD < chunk && u < units) ? u : -1;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

#define SC_HIP_CHECK_LAUNCH()                        \
    do {                                             \
        if (hipGetLastError() != hipSuccess) return SC_EHIP; \
    } while (0)

// ---- phase marks inside kernels (development builds with -DSC_TRACE only) ----------------------
// SC_MARK(i) stores the 100 MHz wall clock of the calling wavefront's first lane into
// trace[workgroup][i]; it compiles to nothing in the product build.
#ifdef SC_TRACE
extern __device__ long long* g_trace_buf;
#define SC_MARK(i)                                                                              \
    do {                                                                                        \
        if (g_trace_buf != nullptr && threadIdx.x == 0) g_trace_buf[(size_t)blockIdx.x * 16 + (i)] = wall_clock64(); \
    } while (0)
#else
#define SC_MARK(i) do { } while (0)
#endif

// ---- optional per-kernel timing (sc_profile_enable / sc_profile_read) --------------------------
enum KernelId {
    KID_TABLE_FILL = 0, KID_HASH_INSERT, KID_HASH_LOOKUP, KID_KMAP_HEADER, KID_KMAP_SUBM, KID_FILL_I32,
    KID_STRIDED_INSERT, KID_STRIDED_FLAGS, KID_SCAN_BLOCKS, KID_STRIDED_PAIRS, KID_KMAP_FROM_OFT,
    KID_COUNT_PAIRS, KID_EXPORT, KID_WEIGHT_PACK, KID_CONV_MFMA, KID_CONV_F32, KID_GRID_CLEAR, KID_GRID_INSERT,
    KID_GRID_LOOKUP, KID_KMAP_GRID, KID_MISC, KID_COUNT
};
extern bool g_profile_on;
// A fresh pair of events for one launch of `kernel_id`; false if none could be created.
bool profile_events(int kernel_id, hipEvent_t* begin, hipEvent_t* end);

// Launch a kernel.  When profiling is on, the launch carries a pair of events that the runtime
// stamps with the dispatch's own begin and end times (hipExtLaunchKernelGGL), the same clock a
// profiler's kernel trace reports.
#define SC_LAUNCH(kid, kernel, grid, block, lds, stream, ...)                                      \
    do {                                                                                           \
        hipEvent_t sc_ev0_, sc_ev1_;                                                               \
        if (sc::g_profile_on && sc::profile_events(kid, &sc_ev0_, &sc_ev1_))                       \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, sc_ev0_, sc_ev1_, 0, __VA_ARGS__); \
        else                                                                                       \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                     \
        if (hipGetLastError() != hipSuccess) return SC_EHIP;                                       \
    } while (0)

}  // namespace sc
