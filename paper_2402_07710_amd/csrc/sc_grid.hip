// Dense location table (paper Section III-C.1: the "large array" form of the location table, which
// the paper prefers when the domain is small enough; its eq. 6 linearises the coordinate).
//
// One 8-byte cell per site of a box B x X x Y x Z: {row (low 32 bits), epoch (high 32 bits)}.  A
// cell counts as occupied only if its epoch equals the epoch of the current build, so a build is
// one scatter of n cells with no fill before it and no clean-up after it: cells written by
// earlier builds are simply stale.  The array is cleared once, when it is allocated.  With 288 GB
// of HBM the 1408 x 1600 x 41 LiDAR box (0.7 GB) and a 512^3 box (1 GB) both fit with room to
// spare; a look-up is one index computation and one 8-byte load instead of a probe sequence.
// The linear index runs z fastest (the paper's eq. 6 runs x fastest; the order is free, and the
// short vertical axis of LiDAR boxes keeps a 3x3x3 neighbourhood within a few cache lines this way).
#include "sc_internal.h"

namespace sc {

__global__ void __launch_bounds__(256)
k_grid_clear(uint4* __restrict__ blob16, int64_t n16) {
    const int64_t nthr = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += nthr) blob16[i] = make_uint4(0, 0, 0, 0);
}

// One thread per point: cell <- {row, epoch}, a plain 8-byte store as in the paper's own table
// kernel (no read of the cell, so the scatter moves 8 bytes per point and not a cache line each
// way).  The first workgroup also resets the counts block.  Nothing is checked here: a row outside
// the box writes nothing, and of two rows with one coordinate the later store wins; both cases are
// found - and latched into counts->status - by the kernel-map build, which reads every row's own
// cell anyway.
__global__ void __launch_bounds__(256)
k_grid_insert(const int4* __restrict__ coords, int64_t n, unsigned long long* __restrict__ cells, GridDims dims,
              uint32_t epoch, sc_counts* counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.x == 0) {
        int32_t* w = reinterpret_cast<int32_t*>(counts);
        for (int j = threadIdx.x; j < (int)(sizeof(sc_counts) / 4); j += blockDim.x) w[j] = 0;
        __syncthreads();
        if (threadIdx.x == 0) counts->n_in = n;
    }
    if (i >= n) return;
    const int4 c = coords[i];
    if (grid_inside(dims, c.x, c.y, c.z, c.w))
        cells[grid_index(dims, c.x, c.y, c.z, c.w)] = ((unsigned long long)epoch << 32) | (uint32_t)i;
}

__global__ void __launch_bounds__(64)
k_kmap_header_set(KmapHeader* hdr, KmapHeader value, sc_counts* counts, int64_t n_out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *hdr = value;
        counts->n_out = n_out;
    }
}

__global__ void __launch_bounds__(256)
k_grid_lookup(const unsigned long long* __restrict__ cells, GridDims dims, uint32_t epoch, const int4* __restrict__ query,
              int64_t nq, int32_t* __restrict__ rows) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nq) return;
    const int4 c = query[i];
    int32_t r = -1;
    if (grid_inside(dims, c.x, c.y, c.z, c.w)) {
        const unsigned long long v = cells[grid_index(dims, c.x, c.y, c.z, c.w)];
        if ((uint32_t)(v >> 32) == epoch) r = (int32_t)(uint32_t)v;
    }
    rows[i] = r;
}

// Submanifold offset table from the dense array (Section III-C.2): the same tile layout and group
// masks as the hash-table build.  One workgroup of WPT wavefronts per 64-row tile, lane = row,
// offsets dealt to the wavefronts round-robin; a wavefront issues the loads of all its offsets
// at once (they are independent and there is nothing to re-probe).
template <int K, int WPT>
__global__ void __launch_bounds__(64 * WPT)
k_kmap_subm_grid(const int4* __restrict__ coords, int64_t n, const unsigned long long* __restrict__ cells, GridDims dims,
                 uint32_t epoch, uint32_t* __restrict__ gmask, int32_t* __restrict__ nbr, sc_counts* counts,
                 KmapHeader* hdr, KmapHeader hdr_value) {
    constexpr int K3 = K * K * K, pad = (K - 1) / 2, centre = (K3 - 1) / 2;
    constexpr int PER = (K3 + WPT - 1) / WPT;        // offsets per wavefront
    constexpr int MW = (K3 + 31) / 32;
    __shared__ uint32_t mask_s[4 * MW];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t tile = xcd_unit(blockIdx.x, gridDim.x);
    if (tile * TILE >= n) return;                    // padding workgroup of the XCD-aware grid
    if (threadIdx.x < 4 * MW) mask_s[threadIdx.x] = 0u;
    const int64_t row = tile * TILE + lane;
    const bool valid = row < n;
    int4 c = make_int4(-1, 0, 0, 0);
    if (valid) c = coords[row];
    if (tile == 0 && threadIdx.x == 0) {
        counts->n_out = n;
        *hdr = hdr_value;
    }
    __syncthreads();
    const bool row_ok = valid && grid_inside(dims, c.x, c.y, c.z, c.w);
    const int64_t base = row_ok ? grid_index(dims, c.x, c.y, c.z, c.w) : 0;

    unsigned long long got[PER];
    bool look[PER];
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int k = w + u * WPT;
        const int dx = k / (K * K) - pad, dy = (k / K) % K - pad, dz = k % K - pad;
        look[u] = k < K3 && row_ok && (unsigned)(c.y + dx) < (unsigned)dims.X &&
                  (unsigned)(c.z + dy) < (unsigned)dims.Y && (unsigned)(c.w + dz) < (unsigned)dims.Z;
        const int64_t idx = base + ((int64_t)dx * dims.Y + dy) * dims.Z + dz;
        got[u] = look[u] ? cells[idx] : 0ull;
    }
    int32_t* tile_nbr = nbr + tile * (int64_t)(K3 * TILE);
#pragma unroll
    for (int u = 0; u < PER; ++u) {
        const int k = w + u * WPT;
        if (k < K3) {
            int32_t found = -1;
            if (look[u] && (uint32_t)(got[u] >> 32) == epoch) found = (int32_t)(uint32_t)got[u];
            if (k == centre && valid) {
                // a row's own cell must name the row: otherwise the row lies outside the box (it
                // was never stored) or another row with the same coordinate overwrote it
                if (!row_ok) latch_status(counts, SC_ERANGE);
                else if (found != (int32_t)row) latch_status(counts, SC_EDUP);
                found = (int32_t)row;
            }
            tile_nbr[k * TILE + lane] = found;
            const uint64_t vote = __ballot(found >= 0);
            if (lane < 4 && ((vote >> (16 * lane)) & 0xffffull) != 0) atomicOr(&mask_s[lane * MW + (k >> 5)], 1u << (k & 31));
        }
    }
    __syncthreads();
    if (threadIdx.x < 4 * MW) gmask[tile * (4 * MW) + threadIdx.x] = mask_s[threadIdx.x];
}

static bool dims_ok(int32_t B, int32_t X, int32_t Y, int32_t Z) {
    if (B < 1 || X < 1 || Y < 1 || Z < 1) return false;
    if (B > SC_COORD_MAX + 1 || X > SC_COORD_MAX + 1 || Y > SC_COORD_MAX + 1 || Z > SC_COORD_MAX + 1) return false;
    const long double cells = (long double)B * X * Y * Z;
    return cells <= (long double)SC_GRID_CELLS_MAX;
}

template <int K>
static int launch_kmap_grid(int64_t tiles, hipStream_t s, const int4* coords, int64_t n, const unsigned long long* cells,
                            GridDims dims, uint32_t epoch, uint32_t* gmask, int32_t* nbr, sc_counts* counts,
                            KmapHeader* hdr, KmapHeader hv) {
    SC_LAUNCH(KID_KMAP_GRID, (k_kmap_subm_grid<K, 8>), dim3(xcd_grid(tiles)), dim3(512), 0, s, coords, n, cells, dims, epoch,
              gmask, nbr, counts, hdr, hv);
    return SC_OK;
}

}  // namespace sc

using namespace sc;

extern "C" size_t sc_grid_bytes(int32_t B, int32_t X, int32_t Y, int32_t Z) {
    if (!dims_ok(B, X, Y, Z)) return 0;
    return align_up((size_t)grid_cells(GridDims{B, X, Y, Z}) * 8, 256);
}

extern "C" int sc_grid_clear(void* d_grid, size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z, void* stream) {
    const size_t need = sc_grid_bytes(B, X, Y, Z);
    if (need == 0 || d_grid == nullptr || !aligned16(d_grid)) return SC_EINVAL;
    if (grid_bytes < need) return SC_ECAP;
    const int64_t n16 = (int64_t)(need / 16);
    int64_t blocks = (n16 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    SC_LAUNCH(KID_GRID_CLEAR, k_grid_clear, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (uint4*)d_grid, n16);
    return SC_OK;
}

extern "C" int sc_grid_build(const int32_t* d_coords, int64_t n, void* d_grid, size_t grid_bytes, int32_t B, int32_t X,
                             int32_t Y, int32_t Z, uint32_t epoch, sc_counts* d_counts, void* stream) {
    const size_t need = sc_grid_bytes(B, X, Y, Z);
    if (need == 0 || n < 0 || n > SC_N_MAX || d_grid == nullptr || d_counts == nullptr || epoch == 0) return SC_EINVAL;
    if (n > 0 && d_coords == nullptr) return SC_EINVAL;
    if (!aligned16(d_coords) || !aligned16(d_grid) || !aligned16(d_counts)) return SC_EINVAL;
    if (grid_bytes < need) return SC_ECAP;
    const unsigned blocks = n > 0 ? (unsigned)((n + 255) / 256) : 1u;
    SC_LAUNCH(KID_GRID_INSERT, k_grid_insert, dim3(blocks), dim3(256), 0, (hipStream_t)stream, (const int4*)d_coords, n,
              (unsigned long long*)d_grid, (GridDims{B, X, Y, Z}), epoch, d_counts);
    return SC_OK;
}

extern "C" int sc_grid_lookup(const void* d_grid, int32_t B, int32_t X, int32_t Y, int32_t Z, uint32_t epoch,
                              const int32_t* d_query, int64_t n_query, int32_t* d_rows, void* stream) {
    if (sc_grid_bytes(B, X, Y, Z) == 0 || d_grid == nullptr || n_query < 0 || epoch == 0) return SC_EINVAL;
    if (n_query == 0) return SC_OK;
    if (d_query == nullptr || d_rows == nullptr || !aligned16(d_query) || !aligned16(d_grid)) return SC_EINVAL;
    SC_LAUNCH(KID_GRID_LOOKUP, k_grid_lookup, dim3((unsigned)((n_query + 255) / 256)), dim3(256), 0, (hipStream_t)stream,
              (const unsigned long long*)d_grid, (GridDims{B, X, Y, Z}), epoch,
              (const int4*)d_query, n_query, d_rows);
    return SC_OK;
}

extern "C" int sc_kmap_build_grid(const int32_t* d_coords, int64_t n, const void* d_grid, size_t grid_bytes, int32_t B,
                                  int32_t X, int32_t Y, int32_t Z, uint32_t epoch, int K, void* d_kmap, size_t kmap_bytes,
                                  sc_counts* d_counts, void* stream) {
    const size_t need = sc_grid_bytes(B, X, Y, Z);
    if (need == 0 || n < 0 || n > SC_N_MAX || d_grid == nullptr || d_kmap == nullptr || d_counts == nullptr || epoch == 0)
        return SC_EINVAL;
    if (K < 1 || K > SC_K_MAX || K % 2 == 0) return SC_EINVAL;
    if (n > 0 && d_coords == nullptr) return SC_EINVAL;
    if (!aligned16(d_coords) || !aligned16(d_grid) || !aligned16(d_kmap) || !aligned16(d_counts)) return SC_EINVAL;
    if (grid_bytes < need) return SC_ECAP;
    if (kmap_bytes < sc_kmap_bytes(n, K, 1, SC_SUBM)) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    const KmapLayout L = kmap_layout(n, K);
    KmapHeader hv = {KMAP_MAGIC, K, 1, SC_SUBM, n, n, L.tiles, L.mw, 0};
    KmapHeader* hdr = (KmapHeader*)d_kmap;
    if (n == 0) {
        SC_LAUNCH(KID_KMAP_HEADER, k_kmap_header_set, dim3(1), dim3(64), 0, s, hdr, hv, d_counts, (int64_t)0);
        return SC_OK;
    }
    uint32_t* gmask = (uint32_t*)((char*)d_kmap + L.off_mask);
    int32_t* nbr = (int32_t*)((char*)d_kmap + L.off_nbr);
    const unsigned long long* cells = (const unsigned long long*)d_grid;
    const GridDims dims{B, X, Y, Z};
    switch (K) {
        case 1: return launch_kmap_grid<1>(L.tiles, s, (const int4*)d_coords, n, cells, dims, epoch, gmask, nbr, d_counts, hdr, hv);
        case 3: return launch_kmap_grid<3>(L.tiles, s, (const int4*)d_coords, n, cells, dims, epoch, gmask, nbr, d_counts, hdr, hv);
        case 5: return launch_kmap_grid<5>(L.tiles, s, (const int4*)d_coords, n, cells, dims, epoch, gmask, nbr, d_counts, hdr, hv);
        case 7: return launch_kmap_grid<7>(L.tiles, s, (const int4*)d_coords, n, cells, dims, epoch, gmask, nbr, d_counts, hdr, hv);
    }
    return SC_EINVAL;
}
