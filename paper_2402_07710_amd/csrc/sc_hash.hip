// Location table: coordinate -> input row (paper Section III-C.1).
//
// The paper scatters the row index into a dense X*Y*Z array (or a hash table for large
// domains) with one thread per point.  Here the table is an open-addressing hash table in HBM,
// keyed on the packed 64-bit (b,x,y,z) and claimed with one 64-bit compare-and-swap per point:
// a 1408x1600x41 LiDAR grid would need 369 MB as a dense int array against ~2 MB of table.
// Stored keys carry the epoch of their build in the top byte, so a table can be built again and
// again without being refilled: what an older build left behind reads as free.
#include "sc_internal.h"

namespace sc {

// every slot <- {EMPTY, val_init}; block 0 also resets the counts block.
__global__ void __launch_bounds__(256)
k_table_fill(uint4* __restrict__ slots, uint64_t cap, int32_t val_init, sc_counts* counts, int64_t n_in, TableHeader* th,
             uint32_t epoch) {
    const uint64_t nthr = (uint64_t)gridDim.x * blockDim.x;
    const uint4 empty = make_uint4(0xffffffffu, 0xffffffffu, (uint32_t)val_init, 0u);
    for (uint64_t i = (uint64_t)blockIdx.x * blockDim.x + threadIdx.x; i < cap; i += nthr) slots[i] = empty;
    if (counts != nullptr && blockIdx.x == 0) {
        int32_t* w = reinterpret_cast<int32_t*>(counts);
        for (int i = threadIdx.x; i < (int)(sizeof(sc_counts) / 4); i += blockDim.x) w[i] = 0;
        __syncthreads();
        if (threadIdx.x == 0) counts->n_in = n_in;
    }
    if (th != nullptr && blockIdx.x == 0 && threadIdx.x == 0) {
        th->mask = (uint32_t)(cap - 1);
        th->epoch = epoch;
        th->err_tag = 0;
    }
}

// One thread per point: walk the key's probe sequence and claim the first free slot with a
// 64-bit compare-and-swap.  The first attempt on a slot expects the filled-in empty word and so
// doubles as the read: in a freshly filled table it succeeds at once; otherwise it returns what
// the slot holds, and if that belongs to another epoch a second compare-and-swap replaces it.
// (Reading several slots of the sequence ahead with plain loads and then claiming the first that
// looked empty was measured slower: the extra loads cost more than the round trips they save at
// a load factor <= 1/8.)
// FRESH: the table was filled and *counts reset just before (epoch 0); errors go to *counts.
// Otherwise block 0 resets *counts and writes the header itself, and errors are left in the
// header under the epoch's tag, because a latch into *counts could race with that reset.
template <int FRESH>
__global__ void __launch_bounds__(256)
k_hash_insert(const int4* __restrict__ coords, int64_t n, uint4* slots, uint32_t mask_fresh, uint32_t epoch,
              TableHeader* th, sc_counts* counts) {
    // without a fill, workgroups are dealt to the XCDs the way the map build deals its tiles: the
    // slots a row claims are then in the L2 that will probe for them (~53k voxels: 9.7 -> 8.4 us;
    // after a fill the table is spread over the caches already and the plain order is faster)
    const int64_t i = (FRESH ? (int64_t)blockIdx.x : xcd_unit(blockIdx.x, gridDim.x)) * blockDim.x + threadIdx.x;
    const uint32_t mask = FRESH ? mask_fresh : th->mask;      // a table keeps the capacity it was filled with
    if (!FRESH && blockIdx.x == 0) {
        int32_t* w = reinterpret_cast<int32_t*>(counts);
        for (int j = threadIdx.x; j < (int)(sizeof(sc_counts) / 4); j += blockDim.x) w[j] = 0;
        __syncthreads();
        if (threadIdx.x == 0) {
            counts->n_in = n;
            th->epoch = epoch;
        }
    }
    auto report = [&](int code) {
        if (FRESH) {
            latch_status(counts, code);
            return;
        }
        // the tag of another epoch is stale whatever its value (epochs need not be used in rising
        // order): replace it; within this epoch keep the largest code
        const uint32_t mine_tag = (epoch << 8) | (uint32_t)(-code);
        uint32_t seen = th->err_tag;
        while ((seen >> 8) != epoch || seen < mine_tag) {
            const uint32_t prev = atomicCAS(&th->err_tag, seen, mine_tag);
            if (prev == seen) break;
            seen = prev;
        }
    };
    if (i >= n) return;
    if (!FRESH && (uint64_t)n * 4 > (uint64_t)mask + 1) {      // more rows than this table was made for
        report(SC_ECAP);
        return;
    }
    const int4 c = coords[i];
    if (!in_domain4(c.x, c.y, c.z, c.w)) {
        report(SC_ERANGE);
        return;
    }
    const uint64_t key = pack_key(c.x, c.y, c.z, c.w), tag = epoch_tag(epoch), mine = key | tag;
    for (uint32_t t = 0; t <= mask + REHASH_MAX; ++t) {
        unsigned long long* word = reinterpret_cast<unsigned long long*>(&slots[probe_slot(key, t, mask)]);
        // what to expect there: the empty word in a fresh table; otherwise look first (a load is
        // much cheaper than a compare-and-swap that fails)
        uint64_t expect = KEY_EMPTY;
        if (!FRESH) {
            expect = *reinterpret_cast<const volatile unsigned long long*>(word);
            if (expect == mine) {
                report(SC_EDUP);
                return;
            }
            if (same_epoch(expect, tag)) continue;  // taken by another key of this build: next attempt
        }
        for (;;) {      // ends: the word only ever changes from another epoch to this one, once
            const uint64_t cur = atomicCAS(word, (unsigned long long)expect, (unsigned long long)mine);
            if (cur == expect) {
                reinterpret_cast<int32_t*>(word)[2] = (int32_t)i;
                return;
            }
            if (cur == mine) {
                report(SC_EDUP);
                return;
            }
            if (same_epoch(cur, tag)) break;        // taken by another key of this build: next attempt
            expect = cur;
        }
    }
    report(SC_EFULL);
}

__global__ void __launch_bounds__(256)
k_hash_lookup(const uint4* __restrict__ slots, const TableHeader* __restrict__ th,
              const int4* __restrict__ query, int64_t nq, int32_t* __restrict__ rows) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= nq) return;
    const int4 c = query[i];
    int32_t r = -1;
    if (in_domain4(c.x, c.y, c.z, c.w)) r = table_find(slots, th->mask, pack_key(c.x, c.y, c.z, c.w), epoch_tag(th->epoch));
    rows[i] = r;
}

int launch_table_fill(uint4* slots, uint64_t cap, int32_t val_init, sc_counts* counts, int64_t n_in, hipStream_t s,
                      TableHeader* th, uint32_t epoch) {
    unsigned blocks = (unsigned)((cap + 255) / 256);
    if (blocks > 2048) blocks = 2048;
    SC_LAUNCH(KID_TABLE_FILL, k_table_fill, dim3(blocks), dim3(256), 0, s, slots, cap, val_init, counts, n_in, th, epoch);
    return SC_OK;
}

}  // namespace sc

using namespace sc;

extern "C" size_t sc_hash_bytes(int64_t n) {
    if (n < 0 || n > SC_N_MAX) return 0;
    return (size_t)table_capacity(n) * sizeof(uint4) + sizeof(TableHeader);
}

static int hash_build(const int32_t* d_coords, int64_t n, void* d_table, size_t table_bytes, int epoch,
                      sc_counts* d_counts, void* stream) {
    if (n < 0 || n > SC_N_MAX || d_table == nullptr || d_counts == nullptr) return SC_EINVAL;
    if (n > 0 && d_coords == nullptr) return SC_EINVAL;
    if (!aligned16(d_coords) || !aligned16(d_table) || !aligned16(d_counts)) return SC_EINVAL;
    if (table_bytes < sc_hash_bytes(n)) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    HashTable t = table_view(d_table, n);
    // A build with an epoch >= 1 may skip the fill.  It does so for tables up to 64 MiB; above
    // that the fill pays for itself: written front to back it leaves the table in the last-level
    // cache, where the scattered inserts and the 26 probes per row of the map build then find it
    // (measured at 10^6 rows, 256 MiB of table: insert + map build 199 us without the fill, 183 us with).
    if (epoch == 0 || (uint64_t)t.mask + 1 > NO_FILL_SLOTS_MAX) {
        if (int rc = launch_table_fill(t.slots, (uint64_t)t.mask + 1, 0, d_counts, n, s, t.hdr, (uint32_t)epoch)) return rc;
        if (n > 0)
            SC_LAUNCH(KID_HASH_INSERT, k_hash_insert<1>, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s,
                      (const int4*)d_coords, n, t.slots, t.mask, (uint32_t)epoch, t.hdr, d_counts);
    } else {
        // at least one workgroup: it also resets the counts and stamps the header
        SC_LAUNCH(KID_HASH_INSERT, k_hash_insert<0>, dim3(xcd_grid((n + 255) / 256 > 0 ? (n + 255) / 256 : 1)), dim3(256), 0,
                  s, (const int4*)d_coords, n, t.slots, t.mask, (uint32_t)epoch, t.hdr, d_counts);
    }
    return SC_OK;
}

extern "C" int sc_hash_build(const int32_t* d_coords, int64_t n, void* d_table, size_t table_bytes,
                             sc_counts* d_counts, void* stream) {
    return hash_build(d_coords, n, d_table, table_bytes, 0, d_counts, stream);
}

extern "C" int sc_hash_rebuild(const int32_t* d_coords, int64_t n, void* d_table, size_t table_bytes, int epoch,
                               sc_counts* d_counts, void* stream) {
    if (epoch < 1 || epoch > SC_HASH_EPOCH_MAX) return SC_EINVAL;
    return hash_build(d_coords, n, d_table, table_bytes, epoch, d_counts, stream);
}

extern "C" int sc_hash_lookup(const void* d_table, int64_t n_table, const int32_t* d_query, int64_t n_query,
                              int32_t* d_rows, void* stream) {
    if (d_table == nullptr || n_table < 0 || n_table > SC_N_MAX || n_query < 0) return SC_EINVAL;
    if (n_query == 0) return SC_OK;
    if (d_query == nullptr || d_rows == nullptr || !aligned16(d_query) || !aligned16(d_table)) return SC_EINVAL;
    HashTable t = table_view(const_cast<void*>(d_table), n_table);
    hipStream_t s = (hipStream_t)stream;
    SC_LAUNCH(KID_HASH_LOOKUP, k_hash_lookup, dim3((unsigned)((n_query + 255) / 256)), dim3(256), 0, s,
              (const uint4*)t.slots, (const TableHeader*)t.hdr, (const int4*)d_query, n_query, d_rows);
    return SC_OK;
}

extern "C" int64_t sc_hash_probe_slot(int32_t b, int32_t x, int32_t y, int32_t z, uint32_t attempt, int64_t n) {
    if (n < 0 || n > SC_N_MAX || !in_domain4(b, x, y, z)) return -1;
    return (int64_t)probe_slot(pack_key(b, x, y, z), attempt, (uint32_t)(table_capacity(n) - 1));
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
