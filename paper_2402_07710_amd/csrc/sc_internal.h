// Internal definitions shared by the HIP translation units of libsc (gfx950 only).
// Nothing here is visible through the C ABI; the public contract is include/sc.h.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sc.h"

namespace sc {

constexpr int WAVE = 64;                      // CDNA wavefront
constexpr int TILE = 64;                      // output rows per kernel-map tile (= one wavefront)
constexpr uint64_t KEY_EMPTY = ~0ull;         // (65535,65535,65535,65535): outside the domain
constexpr uint32_t ENTRY_ROW_BITS = 26;       // kernel-map entry = in_row | out_slot << 26
constexpr uint32_t ENTRY_ROW_MASK = (1u << ENTRY_ROW_BITS) - 1;
constexpr uint32_t KMAP_MAGIC = 0x70614d6bu;

// ---- coordinate keys ------------------------------------------------------------------------
// The paper linearises (x,y,z) into one dense-array index (Section III-C.1 eq. 6); the batch
// index is part of the coordinate (Section II-A), so here all four 16-bit fields are packed
// into one 64-bit key instead.
__host__ __device__ inline uint64_t pack_key(int b, int x, int y, int z) {
    return ((uint64_t)(uint32_t)b << 48) | ((uint64_t)(uint32_t)x << 32) |
           ((uint64_t)(uint32_t)y << 16) | (uint64_t)(uint32_t)z;
}
__host__ __device__ inline bool in_domain(int v) { return (unsigned)v <= (unsigned)SC_COORD_MAX; }
__host__ __device__ inline bool in_domain4(int b, int x, int y, int z) {
    return in_domain(b) && in_domain(x) && in_domain(y) && in_domain(z);
}

// Home slot of a key.  Keys that differ only in the low bits of z share one hash of the
// remaining bits and sit side by side, so the z-neighbours a kernel-map probe asks for fall
// into the same or the adjacent 32-byte sector of the key array.
constexpr int HASH_RUN_LOG2 = 2;
__host__ __device__ inline uint32_t home_slot(uint64_t key, uint32_t mask) {
    uint64_t g = key >> HASH_RUN_LOG2;
    g *= 0x9E3779B97F4A7C15ull;
    g ^= g >> 29;
    g *= 0xBF58476D1CE4E5B9ull;
    g ^= g >> 32;
    return (((uint32_t)g << HASH_RUN_LOG2) | ((uint32_t)key & ((1u << HASH_RUN_LOG2) - 1))) & mask;
}

// capacity: power of two >= 2n, at least 1024 slots
inline uint64_t hash_capacity(int64_t n) {
    uint64_t cap = 1024;
    while (cap < 2ull * (uint64_t)(n < 0 ? 0 : n)) cap <<= 1;
    return cap;
}

struct HashTable {            // view of a caller-owned table buffer
    uint64_t* keys;           // [cap]
    int32_t* vals;            // [cap]
    uint32_t mask;            // cap - 1
};
inline HashTable table_view(void* p, int64_t n) {
    uint64_t cap = hash_capacity(n);
    HashTable t;
    t.keys = (uint64_t*)p;
    t.vals = (int32_t*)((char*)p + cap * sizeof(uint64_t));
    t.mask = (uint32_t)(cap - 1);
    return t;
}

// Probe for `key`; returns the stored value or -1.  Linear probing, table never full.
__device__ inline int32_t table_find(const uint64_t* __restrict__ keys, const int32_t* __restrict__ vals,
                                     uint32_t mask, uint64_t key) {
    uint32_t slot = home_slot(key, mask);
    for (uint32_t step = 0; step <= mask; ++step) {
        uint64_t cur = keys[slot];
        if (cur == key) return vals[slot];
        if (cur == KEY_EMPTY) return -1;
        slot = (slot + 1) & mask;
    }
    return -1;
}

__device__ inline void latch_status(sc_counts* counts, int code) {
    atomicCAS(&counts->status, 0, code);
}

// keys <- EMPTY, optionally vals <- val_init and *counts reset (defined in sc_hash.hip)
int launch_table_fill(uint64_t* keys, int32_t* vals, uint64_t cap, int fill_vals, int32_t val_init,
                      sc_counts* counts, int64_t n_in, hipStream_t s);

// ---- kernel-map blob ------------------------------------------------------------------------
// header | start[T][sstride] (uint16) | entries[T][TILE*K3] (uint32)
// start[t][k] .. start[t][k+1] delimit tile t's pairs of offset k inside entries[t][...].
struct KmapHeader {
    uint32_t magic;
    int32_t K, stride, mode;
    int64_t n_in, n_out_bound;
    int64_t tiles;
    int32_t sstride, reserved;
};
struct KmapLayout {
    int64_t tiles;        // T = ceil(n_out_bound / TILE)
    int K3;
    int sstride;          // uint16 per tile in start[], multiple of 32
    size_t off_start;     // byte offsets inside the blob
    size_t off_entries;
    size_t bytes;
};
inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline KmapLayout kmap_layout(int64_t n_out_bound, int K) {
    KmapLayout L;
    L.K3 = K * K * K;
    L.tiles = (n_out_bound + TILE - 1) / TILE;
    L.sstride = (int)align_up((size_t)L.K3 + 1, 32);
    L.off_start = 256;
    L.off_entries = align_up(L.off_start + (size_t)L.tiles * L.sstride * sizeof(uint16_t), 256);
    L.bytes = align_up(L.off_entries + (size_t)L.tiles * TILE * L.K3 * sizeof(uint32_t), 256);
    return L;
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }

#define SC_HIP_CHECK_LAUNCH()                        \
    do {                                             \
        if (hipGetLastError() != hipSuccess) return SC_EHIP; \
    } while (0)

// ---- optional per-kernel timing (sc_profile_enable / sc_profile_read) --------------------------
enum KernelId {
    KID_TABLE_FILL = 0, KID_HASH_INSERT, KID_HASH_LOOKUP, KID_KMAP_HEADER, KID_KMAP_SUBM, KID_FILL_I32,
    KID_STRIDED_INSERT, KID_STRIDED_FLAGS, KID_SCAN_BLOCKS, KID_STRIDED_PAIRS, KID_KMAP_FROM_OFT,
    KID_COUNT_PAIRS, KID_EXPORT, KID_WEIGHT_PACK, KID_CONV_MFMA, KID_CONV_F32, KID_MISC, KID_COUNT
};
extern bool g_profile_on;
void profile_mark(int kernel_id, hipStream_t s, bool after);

// Launch a kernel; when profiling is on, bracket it with a pair of HIP events on the same stream.
#define SC_LAUNCH(kid, kernel, grid, block, lds, stream, ...)                    \
    do {                                                                         \
        if (sc::g_profile_on) sc::profile_mark(kid, stream, false);              \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);       \
        if (sc::g_profile_on) sc::profile_mark(kid, stream, true);               \
        if (hipGetLastError() != hipSuccess) return SC_EHIP;                     \
    } while (0)

}  // namespace sc
