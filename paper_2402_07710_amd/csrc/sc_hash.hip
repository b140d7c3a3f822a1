// Location table: coordinate -> input row (paper Section III-C.1).
//
// The paper scatters the row index into a dense X*Y*Z array (or a hash table for large
// domains) with one thread per point.  Here the table is an open-addressing hash table in HBM,
// keyed on the packed 64-bit (b,x,y,z) and claimed with one 64-bit compare-and-swap per point:
// a 1408x1600x41 LiDAR grid would need 369 MB as a dense int array against ~2 MB of table.
#include "sc_internal.h"

namespace sc {

// every slot <- {EMPTY, val_init}; block 0 also resets the counts block.
__global__ void __launch_bounds__(256)
k_table_fill(uint4* __restrict__ slots, uint64_t cap, int32_t val_init, sc_counts* counts, int64_t n_in) {
    const uint64_t nthr = (uint64_t)gridDim.x * blockDim.x;
    const uint4 empty = make_uint4(0xffffffffu, 0xffffffffu, (uint32_t)val_init, 0u);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cap; i += nthr) slots[i] = empty;
    if (counts != nullptr && blockIdx.x == 0) {
        int32_t* w = reinterpret_cast<int32_t*>(counts);
        for (int i = threadIdx.x; i < (int)(sizeof(sc_counts) / 4); i += blockDim.x) w[i] = 0;
        __syncthreads();
        if (threadIdx.x == 0) counts->n_in = n_in;
    }
}

// One thread per point: walk the key's probe sequence and claim the first empty slot with one
// 64-bit compare-and-swap.  (Reading several slots of the sequence ahead with plain loads and
// then claiming the first that looked empty was measured slower: the extra loads cost more than
// the compare-and-swap round trips they save at a load factor <= 1/4.)
__global__ void __launch_bounds__(256)
k_hash_insert(const int4* __restrict__ coords, int64_t n, uint4* slots, uint32_t mask, sc_counts* counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int4 c = coords[i];
    if (!in_domain4(c.x, c.y, c.z, c.w)) {
        latch_status(counts, SC_ERANGE);
        return;
    }
    const uint64_t key = pack_key(c.x, c.y, c.z, c.w);
    for (uint32_t t = 0; t <= mask + REHASH_MAX; ++t) {
        const uint32_t slot = probe_slot(key, t, mask);
        const uint64_t cur = atomicCAS(reinterpret_cast<unsigned long long*>(&slots[slot]),
                                       (unsigned long long)KEY_EMPTY, (unsigned long long)key);
        if (cur == KEY_EMPTY) {
            reinterpret_cast<int32_t*>(&slots[slot])[2] = (int32_t)i;
            return;
        }
        if (cur == key) {
            latch_status(counts, SC_EDUP);
            return;
        }
    }
    latch_status(counts, SC_EFULL);
}

__global__ void __launch_bounds__(256)
k_hash_lookup(const uint4* __restrict__ slots, uint32_t mask, const int4* __restrict__ query, int64_t nq,
              int32_t* __restrict__ rows) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nq) return;
    const int4 c = query[i];
    int32_t r = -1;
    if (in_domain4(c.x, c.y, c.z, c.w)) r = table_find(slots, mask, pack_key(c.x, c.y, c.z, c.w));
    rows[i] = r;
}

int launch_table_fill(uint4* slots, uint64_t cap, int32_t val_init, sc_counts* counts, int64_t n_in, hipStream_t s) {
    unsigned blocks = (unsigned)((cap + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    SC_LAUNCH(KID_TABLE_FILL, k_table_fill, dim3(blocks), dim3(256), 0, s, slots, cap, val_init, counts, n_in);
    return SC_OK;
}

}  // namespace sc

using namespace sc;

extern "C" size_t sc_hash_bytes(int64_t n) {
    if (n < 0 || n > SC_N_MAX) return 0;
    return (size_t)hash_capacity(n) * sizeof(uint4);
}

extern "C" int sc_hash_build(const int32_t* d_coords, int64_t n, void* d_table, size_t table_bytes,
                             sc_counts* d_counts, void* stream) {
    if (n < 0 || n > SC_N_MAX || d_table == nullptr || d_counts == nullptr) return SC_EINVAL;
    if (n > 0 && d_coords == nullptr) return SC_EINVAL;
    if (!aligned16(d_coords) || !aligned16(d_table) || !aligned16(d_counts)) return SC_EINVAL;
    if (table_bytes < sc_hash_bytes(n)) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    HashTable t = table_view(d_table, n);
    if (int rc = launch_table_fill(t.slots, (uint64_t)t.mask + 1, 0, d_counts, n, s)) return rc;
    if (n > 0)
        SC_LAUNCH(KID_HASH_INSERT, k_hash_insert, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                  (const int4*)d_coords, n, t.slots, t.mask, d_counts);
    return SC_OK;
}

extern "C" int sc_hash_lookup(const void* d_table, int64_t n_table, const int32_t* d_query, int64_t n_query,
                              int32_t* d_rows, void* stream) {
    if (d_table == nullptr || n_table < 0 || n_table > SC_N_MAX || n_query < 0) return SC_EINVAL;
    if (n_query == 0) return SC_OK;
    if (d_query == nullptr || d_rows == nullptr || !aligned16(d_query) || !aligned16(d_table)) return SC_EINVAL;
    HashTable t = table_view(const_cast<void*>(d_table), n_table);
    hipStream_t s = (hipStream_t)stream;
    SC_LAUNCH(KID_HASH_LOOKUP, k_hash_lookup, dim3((unsigned)((n_query + 255) / 256)), dim3(256), 0, s,
              (const uint4*)t.slots, t.mask, (const int4*)d_query, n_query, d_rows);
    return SC_OK;
}

extern "C" const char* sc_strerror(int status) {
    switch (status) {
        case SC_OK: return "ok";
        case SC_EINVAL: return "invalid argument";
        case SC_ERANGE: return "coordinate outside the key domain";
        case SC_EDUP: return "duplicate input coordinate";
        case SC_ECAP: return "buffer too small";
        case SC_EHIP: return "HIP runtime error";
        case SC_EFULL: return "hash table full";
        default: return "unknown status";
    }
}
