// Offset table / kernel map (paper Section III-C.2 for submanifold layers, Section III-B
// eq. 1-5 and Section III-D for strided layers).
//
// The paper writes a dense N x K^3 table of neighbour rows (-1 where there is none) with one
// thread per point probing the location table K^3 times in a loop, and for strided layers counts
// the distinct output cells with an atomic exchange on a status table plus an atomic counter.
// Here the table is the same offset table, laid out for the matrix cores: outputs are cut into
// tiles of 64 rows, a tile stores its K^3 x 64 neighbour rows offset-major, and a bit per
// (16-row group, offset) records whether the group has any neighbour there, so the convolution
// only touches groups that exist.  Look-ups are issued many at a time (they are independent), not
// one after the other.  Strided layers number their output cells in order of first occurrence
// (min input row per cell + prefix sum), so the result does not depend on thread timing, unlike
// an atomic counter.  The plain per-offset pair lists are produced on demand (sc_kmap_export) by
// ballot + prefix-count compaction of the table.
#include <cstdlib>

#include "sc_internal.h"

namespace sc {

__device__ inline uint64_t lanemask_lt() { return (1ull << (threadIdx.x & 63)) - 1ull; }

__global__ void __launch_bounds__(64)
k_kmap_header(KmapHeader* hdr, KmapHeader value) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *hdr = value;
}

__global__ void __launch_bounds__(64)
k_set_n_out(sc_counts* counts, int64_t n_out) {
    if (threadIdx.x == 0 && blockIdx.x == 0) counts->n_out = n_out;
}

// Submanifold: output row = input row.  One workgroup of WPT wavefronts per 64-row tile; lane =
// row, and the K^3 offsets are dealt to the wavefronts CH at a time.  The probes of a row do not
// depend on each other, so a wavefront issues the loads of its CH offsets together and afterwards
// re-probes only the offsets whose slot held another key: a tile's K^3 x 64 look-ups cost a few
// memory round trips instead of K^3.  Each wavefront then stores its offsets' 64 results as one
// 256-byte line of the tile and votes (ballot) on which 16-row groups have a neighbour.
template <int K, int WPT, int CH, int AT>
__global__ void __launch_bounds__(64 * WPT)
k_kmap_subm(const int4* __restrict__ coords, int64_t n, const uint4* __restrict__ slots,
            const TableHeader* __restrict__ th, uint32_t* __restrict__ gmask, int32_t* __restrict__ nbr,
            sc_counts* counts, KmapHeader* hdr, KmapHeader hdr_value) {
    constexpr int K3 = K * K * K, pad = (K - 1) / 2, centre = (K3 - 1) / 2;
    constexpr int PER_PASS = WPT * CH;
    constexpr int PASSES = (K3 + PER_PASS - 1) / PER_PASS;
    constexpr int MW = (K3 + 31) / 32;
    __shared__ uint32_t mask_s[4 * MW];

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t tile = xcd_unit(blockIdx.x, gridDim.x);
    SC_MARK(0);
    if (tile * TILE >= n) return;                    // padding workgroup of the XCD-aware grid
    if (threadIdx.x < 4 * MW) mask_s[threadIdx.x] = 0u;
    const int64_t row = tile * TILE + lane;
    const bool valid = row < n;
    int4 c = make_int4(0, 0, 0, 0);
    if (valid) c = coords[row];
    const uint32_t mask = th->mask;
    const uint64_t tag = epoch_tag(th->epoch);       // slots of other epochs are free
    if (tile == 0 && threadIdx.x == 0) {
        counts->n_out = n;
        *hdr = hdr_value;
        fold_table_error(th, counts);
    }
    __syncthreads();

    auto neighbour_key = [&](int k, bool& inside) -> uint64_t {
        const int dx = k / (K * K) - pad, dy = (k / K) % K - pad, dz = k % K - pad;
        const int x = c.y + dx, y = c.z + dy, z = c.w + dz;
        inside = in_domain(x) && in_domain(y) && in_domain(z);
        return pack_key(c.x, x, y, z);
    };
    auto load_slot = [&](uint32_t slot) -> uint3 { return *reinterpret_cast<const uint3*>(&slots[slot]); };

    int32_t* tile_nbr = nbr + tile * (int64_t)(K3 * TILE);
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int k_base = (p * WPT + w) * CH;
        uint32_t pending = 0;          // bit u: offset k_base+u still has to be looked up
        int32_t found[CH];
        uint3 got[CH][AT];             // AT consecutive attempts of the probe sequence per round
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int k = k_base + u;
            bool inside;
            const uint64_t key = neighbour_key(k, inside);
            found[u] = -1;
            if (valid && k < K3) {
                if (k == centre) found[u] = (int32_t)row;                  // the centre is the row itself
                else if (inside) pending |= 1u << u;
            }
            // the first AT attempts of every offset at once (harmless loads where nothing is pending)
#pragma unroll
            for (int a = 0; a < AT; ++a) got[u][a] = load_slot(probe_slot(key, a, mask));
        }
        SC_MARK(1);
        for (uint32_t t = 0; __any(pending != 0); t += AT) {   // ends: every probe sequence reaches an empty slot
            if (t == AT) SC_MARK(2);
            if (t > 0) {
#pragma unroll
                for (int u = 0; u < CH; ++u) {
                    if (pending & (1u << u)) {
                        bool inside;
                        const uint64_t key = neighbour_key(k_base + u, inside);
#pragma unroll
                        for (int a = 0; a < AT; ++a) got[u][a] = load_slot(probe_slot(key, t + a, mask));
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < CH; ++u) {
                if (pending & (1u << u)) {
                    bool inside;
                    const uint64_t key = neighbour_key(k_base + u, inside);
#pragma unroll
                    for (int a = 0; a < AT; ++a) {
                        if (pending & (1u << u)) {
                            const uint64_t cur = (uint64_t)got[u][a].x | ((uint64_t)got[u][a].y << 32);
                            if (cur == (key | tag)) { found[u] = (int32_t)got[u][a].z; pending &= ~(1u << u); }
                            else if (!same_epoch(cur, tag)) pending &= ~(1u << u);
                        }
                    }
                }
            }
        }
        SC_MARK(3);
#pragma unroll
        for (int u = 0; u < CH; ++u) {
            const int k = k_base + u;
            if (k < K3) {
                tile_nbr[k * TILE + lane] = found[u];
                const uint64_t vote = __ballot(found[u] >= 0);
                if (lane < 4 && ((vote >> (16 * lane)) & 0xffffull) != 0) atomicOr(&mask_s[lane * MW + (k >> 5)], 1u << (k & 31));
            }
        }
    }
    __syncthreads();
    SC_MARK(4);
    if (threadIdx.x < 4 * MW) gmask[tile * (4 * MW) + threadIdx.x] = mask_s[threadIdx.x];
    SC_MARK(5);
}

// ---- strided layers with K == stride ---------------------------------------------------------
// scratch: output-cell table (key -> min input row of the cell), slot_of[n], flag words,
// in-block word prefix, block sums / prefixes.
struct StridedScratch {
    uint4* oslots;           // output-cell table: {key, min input row}
    uint32_t omask;
    int32_t* slot_of;        // [n]
    uint64_t* flagword;      // [ceil(n/64)]  bit i%64 set iff input i is the first of its cell
    int32_t* word_prefix;    // [ceil(n/64)]  flags before this word inside its 1024-block
    int32_t* block_sum;      // [nblk]
    int32_t* block_prefix;   // [nblk]
    size_t bytes;
};
// n = entries of slot_of / flag bits (inputs, or candidates for K != stride); slots_per_key sizes
// the output-cell table: 8 when every entry is a distinct cell at worst (K == stride: n cells),
// 2 for candidate lists, whose n is a bound that real voxel sets stay far below
inline StridedScratch strided_scratch(void* p, int64_t n, uint64_t slots_per_key = 8) {
    StridedScratch s;
    const uint64_t cap = hash_capacity(n, slots_per_key);
    const int64_t words = (n + 63) / 64, nblk = (n + 1023) / 1024;
    size_t off = 0;
    char* b = (char*)p;
    s.oslots = (uint4*)(b + off); off = align_up(off + cap * 16, 256);
    s.omask = (uint32_t)(cap - 1);
    s.slot_of = (int32_t*)(b + off); off = align_up(off + (size_t)n * 4, 256);
    s.flagword = (uint64_t*)(b + off); off = align_up(off + (size_t)words * 8, 256);
    s.word_prefix = (int32_t*)(b + off); off = align_up(off + (size_t)words * 4, 256);
    s.block_sum = (int32_t*)(b + off); off = align_up(off + (size_t)nblk * 4, 256);
    s.block_prefix = (int32_t*)(b + off); off = align_up(off + (size_t)nblk * 4, 256);
    s.bytes = off + 256;
    return s;
}

// One pass that prepares a strided build: output table <- empty, offset table <- -1.
__global__ void __launch_bounds__(256)
k_strided_fill(uint4* __restrict__ oslots, uint64_t cap, int4* __restrict__ nbr16, int64_t nbr_vec, sc_counts* counts,
               int reset, int64_t n_in, const TableHeader* th) {
    const int64_t nthr = (int64_t)gridDim.x * blockDim.x;
    const int64_t tid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (reset && blockIdx.x == 0) {                  // a build without a location table starts the counts block itself
        int32_t* w = reinterpret_cast<int32_t*>(counts);
        for (int i = threadIdx.x; i < (int)(sizeof(sc_counts) / 4); i += blockDim.x) w[i] = 0;
        __syncthreads();
        if (threadIdx.x == 0) counts->n_in = n_in;
    }
    // after a location-table build that could not report into the counts block, report for it
    if (th != nullptr && tid == 0) fold_table_error(th, counts);
    const uint4 empty = make_uint4(0xffffffffu, 0xffffffffu, 0x7fffffffu, 0u);
    for (int64_t i = tid; i < (int64_t)cap; i += nthr) oslots[i] = empty;
    for (int64_t i = tid; i < nbr_vec; i += nthr) nbr16[i] = make_int4(-1, -1, -1, -1);
}

// Each input claims (or finds) the slot of its output cell floor(p/s) (eq. 2, eq. 4) and
// lowers the slot's value to its own row index.
__global__ void __launch_bounds__(256)
k_strided_insert(const int4* __restrict__ coords, int64_t n, int s, uint4* oslots, uint32_t omask,
                 int32_t* __restrict__ slot_of, sc_counts* counts) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int4 c = coords[i];
    int32_t myslot = -1;
    if (!in_domain4(c.x, c.y, c.z, c.w)) {
        latch_status(counts, SC_ERANGE);
    } else {
        const uint64_t key = pack_key(c.x, c.y / s, c.z / s, c.w / s);
        for (uint32_t t = 0; t <= omask + REHASH_MAX; ++t) {
            const uint32_t slot = probe_slot(key, t, omask);
            const uint64_t cur = atomicCAS(reinterpret_cast<unsigned long long*>(&oslots[slot]),
                                           (unsigned long long)KEY_EMPTY, (unsigned long long)key);
            if (cur == KEY_EMPTY || cur == key) {
                myslot = (int32_t)slot;
                break;
            }
        }
        if (myslot >= 0) atomicMin(reinterpret_cast<int32_t*>(&oslots[myslot]) + 2, (int32_t)i);
        else latch_status(counts, SC_EFULL);
    }
    slot_of[i] = myslot;
}

// flag(i) = input i is the first (lowest row) of its cell; one bit per input, plus the
// exclusive prefix of the flag counts of the 16 words of each 1024-input block.
__global__ void __launch_bounds__(1024)
k_strided_flags(int64_t n, const int32_t* __restrict__ slot_of, const uint4* __restrict__ oslots,
                uint64_t* __restrict__ flagword, int32_t* __restrict__ word_prefix,
                int32_t* __restrict__ block_sum) {
    __shared__ int32_t wave_count[16];
    const int64_t i = (int64_t)blockIdx.x * 1024 + threadIdx.x;
    bool first = false;
    if (i < n) {
        const int32_t sl = slot_of[i];
        first = sl >= 0 && (int32_t)oslots[sl].z == (int32_t)i;
    }
    const uint64_t vote = __ballot(first);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    if (lane == 0) wave_count[wave] = __popcll(vote);
    __syncthreads();
    if (lane == 0) {
        int32_t before = 0;
        for (int w = 0; w < wave; ++w) before += wave_count[w];
        const int64_t word = (int64_t)blockIdx.x * 16 + wave;
        if (word * 64 < n) {
            flagword[word] = vote;
            word_prefix[word] = before;
        }
        if (wave == 15) block_sum[blockIdx.x] = before + wave_count[15];
    }
}

// Exclusive prefix of the block sums (one workgroup walks the array), total -> counts->n_out.
__global__ void __launch_bounds__(1024)
k_scan_blocks(const int32_t* __restrict__ block_sum, int32_t* __restrict__ block_prefix, int64_t nblk,
              sc_counts* counts) {
    __shared__ int32_t part[1024];
    __shared__ int32_t carry_s;
    if (threadIdx.x == 0) carry_s = 0;
    __syncthreads();
    for (int64_t base = 0; base < nblk; base += 1024) {
        const int64_t i = base + threadIdx.x;
        const int32_t v = i < nblk ? block_sum[i] : 0;
        part[threadIdx.x] = v;
        __syncthreads();
        for (int off = 1; off < 1024; off <<= 1) {           // Hillis-Steele inclusive scan
            int32_t add = threadIdx.x >= (unsigned)off ? part[threadIdx.x - off] : 0;
            __syncthreads();
            part[threadIdx.x] += add;
            __syncthreads();
        }
        const int32_t carry = carry_s;
        if (i < nblk) block_prefix[i] = carry + part[threadIdx.x] - v;
        __syncthreads();
        if (threadIdx.x == 1023) carry_s = carry + part[1023];
        __syncthreads();
    }
    if (threadIdx.x == 0) counts->n_out = carry_s;
}

// Exclusive prefix of the per-block counts, computed by every workgroup for itself into LDS (the
// counts of a few hundred to a few thousand 1024-input blocks: cheaper than a kernel of its own,
// which is one workgroup long).  Returns the total.  All threads of the workgroup call it.
constexpr int SCAN_IN_PAIRS_MAX = 4096;              // blocks (4 M inputs); more: k_scan_blocks
__device__ inline int32_t block_prefix_to_lds(const int32_t* __restrict__ block_sum, int nblk, int32_t* prefix_s,
                                              int32_t* wave_s) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int per = (nblk + (int)blockDim.x - 1) / (int)blockDim.x;
    const int lo = threadIdx.x * per, hi = lo + per < nblk ? lo + per : nblk;
    int32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += block_sum[i];
    int32_t incl = sum;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int32_t v = __shfl_up(incl, off);
        if (lane >= off) incl += v;
    }
    if (lane == 63) wave_s[wave] = incl;
    __syncthreads();
    int32_t before = 0, total = 0;
    for (int w = 0; w < nwaves; ++w) {
        if (w < wave) before += wave_s[w];
        total += wave_s[w];
    }
    int32_t run = before + incl - sum;
    for (int i = lo; i < hi; ++i) {
        prefix_s[i] = run;
        run += block_sum[i];
    }
    __syncthreads();
    return total;
}

// Every input finds its output row (rank of its cell's first input among all first inputs),
// its in-cell offset (eq. 3) and kernel offset (eq. 5), and records itself in the offset table.
// SCAN: the prefix of the block counts is made here (block_prefix is then unused) and workgroup 0
// writes the number of output rows.
template <int SCAN>
__global__ void __launch_bounds__(256)
k_strided_pairs(const int4* __restrict__ coords, int64_t n, int s, int K3,
                const int32_t* __restrict__ slot_of, const uint4* __restrict__ oslots,
                const uint64_t* __restrict__ flagword, const int32_t* __restrict__ word_prefix,
                const int32_t* __restrict__ block_prefix, const int32_t* __restrict__ block_sum, int nblk,
                int32_t* __restrict__ nbr, int4* __restrict__ out_coords, sc_counts* counts, KmapHeader* hdr,
                KmapHeader hdr_value) {
    __shared__ int32_t prefix_s[SCAN ? SCAN_IN_PAIRS_MAX : 1];
    __shared__ int32_t wave_s[4];
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i == 0) *hdr = hdr_value;
    if constexpr (SCAN) {
        const int32_t total = block_prefix_to_lds(block_sum, nblk, prefix_s, wave_s);
        if (i == 0) counts->n_out = total;
        block_prefix = prefix_s;
    }
    if (i >= n) return;
    const int32_t sl = slot_of[i];
    if (sl < 0) return;
    const int32_t r = (int32_t)oslots[sl].z;                   // first input of this cell
    const int32_t o = block_prefix[r >> 10] + word_prefix[r >> 6] +
                      __popcll(flagword[r >> 6] & ((1ull << (r & 63)) - 1ull));
    const int4 c = coords[i];
    const int qx = c.y / s, qy = c.z / s, qz = c.w / s;
    const int k = ((c.y - qx * s) * s + (c.z - qy * s)) * s + (c.w - qz * s);
    const int64_t tile = o >> 6;
    const int j = o & 63;
    // distinct inputs own distinct (output row, offset) cells, so a plain store is enough; repeated
    // input coordinates are the location table's business (sc_hash_build latches SC_EDUP)
    nbr[(tile * K3 + k) * TILE + j] = (int32_t)i;
    if (r == (int32_t)i) out_coords[o] = make_int4(c.x, qx, qy, qz);
}

// ---- strided layers with K != stride -------------------------------------------------------------
// An input p pairs with output cell q at offset d whenever p = q*s + d, d in [0,K)^3 (the
// enumeration of Algorithm 1's getOutputCoord with no padding), so it can belong to up to
// MAXC = ceil(K/s)^3 cells.  Its valid (offset, cell) candidates are numbered j = 0.. in
// ascending offset order; candidate id c = i*MAXC + j therefore orders all candidates by input
// row and then by offset, and a cell's number is the rank of its lowest candidate id among all
// cells' lowest ids: the same first-occurrence numbering as for K == stride, found with the same
// flag / prefix kernels run over candidates instead of inputs.
// offset table <- -1 for the tiles that hold the counts->n_out output rows
__global__ void __launch_bounds__(256)
k_fill_rows(int4* __restrict__ nbr16, int K3, const sc_counts* __restrict__ counts) {
    const int64_t vec = (counts->n_out + TILE - 1) / TILE * K3 * (TILE / 4);
    const int64_t nthr = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < vec; i += nthr) nbr16[i] = make_int4(-1, -1, -1, -1);
}

// Candidate j of the input at c, or k < 0 if it has fewer.  Along one axis the offsets that can
// pair coordinate p with a cell are d = p mod s, p mod s + s, ... below K and not above p (the
// cell coordinate (p - d)/s must not be negative); candidates are numbered with x slowest and z
// fastest, offsets ascending, i.e. in ascending order of the offset number k.
struct Candidate {
    int k;                 // offset number, -1: no such candidate
    int qx, qy, qz;        // the output cell
};
__device__ inline int axis_options(int p, int K, int s) {
    const int top = p < K - 1 ? p : K - 1;
    return (top - p % s) / s + 1;                  // p mod s <= top always: s <= K and p mod s <= p
}
__device__ inline Candidate candidate(const int4 c, int K, int s, int j) {
    const int cy = axis_options(c.z, K, s), cz = axis_options(c.w, K, s), cx = axis_options(c.y, K, s);
    Candidate r;
    r.k = -1; r.qx = r.qy = r.qz = 0;
    if (j >= cx * cy * cz) return r;
    const int dz = c.w % s + (j % cz) * s, dy = c.z % s + ((j / cz) % cy) * s, dx = c.y % s + (j / (cz * cy)) * s;
    r.k = (dx * K + dy) * K + dz;
    r.qx = (c.y - dx) / s; r.qy = (c.z - dy) / s; r.qz = (c.w - dz) / s;
    return r;
}

// One thread per candidate (input i = id / maxc, candidate j = id % maxc): the inputs' candidates
// are independent, and with a thread each their compare-and-swaps are all in flight together.
__global__ void __launch_bounds__(256)
k_gstrided_insert(const int4* __restrict__ coords, int64_t n, int K, int s, int maxc, uint4* oslots, uint32_t omask,
                  int32_t* __restrict__ cand_slot, sc_counts* counts) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id >= n * maxc) return;
    const int64_t i = id / maxc;
    const int j = (int)(id - i * maxc);
    const int4 c = coords[i];
    int32_t myslot = -1;
    if (!in_domain4(c.x, c.y, c.z, c.w)) {
        if (j == 0) latch_status(counts, SC_ERANGE);
    } else {
        const Candidate q = candidate(c, K, s, j);
        if (q.k >= 0) {
            const uint64_t key = pack_key(c.x, q.qx, q.qy, q.qz);
            for (uint32_t t = 0; t <= omask + REHASH_MAX; ++t) {
                const uint32_t slot = probe_slot(key, t, omask);
                const uint64_t cur = atomicCAS(reinterpret_cast<unsigned long long*>(&oslots[slot]),
                                               (unsigned long long)KEY_EMPTY, (unsigned long long)key);
                if (cur == KEY_EMPTY || cur == key) {
                    myslot = (int32_t)slot;
                    break;
                }
            }
            if (myslot >= 0) atomicMin(reinterpret_cast<int32_t*>(&oslots[myslot]) + 2, (int32_t)id);
            else latch_status(counts, SC_EFULL);
        }
    }
    cand_slot[id] = myslot;
}

__global__ void __launch_bounds__(256)
k_gstrided_pairs(const int4* __restrict__ coords, int64_t n, int K, int s, int maxc,
                 const int32_t* __restrict__ cand_slot, const uint4* __restrict__ oslots,
                 const uint64_t* __restrict__ flagword, const int32_t* __restrict__ word_prefix,
                 const int32_t* __restrict__ block_prefix, int32_t* __restrict__ nbr,
                 int4* __restrict__ out_coords, KmapHeader* hdr, KmapHeader hdr_value) {
    const int64_t id = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (id == 0) *hdr = hdr_value;
    if (id >= n * maxc) return;
    const int32_t sl = cand_slot[id];
    if (sl < 0) return;
    const int64_t i = id / maxc;
    const int4 c = coords[i];
    const Candidate q = candidate(c, K, s, (int)(id - i * maxc));
    const int32_t r = (int32_t)oslots[sl].z;                   // the cell's first candidate
    const int32_t o = block_prefix[r >> 10] + word_prefix[r >> 6] +
                      __popcll(flagword[r >> 6] & ((1ull << (r & 63)) - 1ull));
    // one input per (output row, offset): a plain store
    nbr[((int64_t)(o >> 6) * (K * K * K) + q.k) * TILE + (o & 63)] = (int32_t)i;
    if (r == (int32_t)id) out_coords[o] = make_int4(c.x, q.qx, q.qy, q.qz);
}

// Group masks of a finished offset table: one workgroup per tile; its four wavefronts share the
// offset lines, eight lines in flight each, vote on them and merge their bits in LDS.
__global__ void __launch_bounds__(256)
k_masks_from_table(const int32_t* __restrict__ nbr, int K3, int mw, int64_t tiles, uint32_t* __restrict__ gmask,
                   const sc_counts* __restrict__ counts, int inverse) {
    __shared__ uint32_t mask_s[4 * ((343 + 31) / 32)];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;
    // tiles past the last output row (inverse maps: the last fine row) are never read
    if (tile >= tiles || tile * TILE >= (inverse ? counts->n_in : counts->n_out)) return;
    if (threadIdx.x < 4 * mw) mask_s[threadIdx.x] = 0u;
    __syncthreads();
    const int32_t* tile_nbr = nbr + tile * (int64_t)K3 * TILE;
    for (int k0 = w * 8; k0 < K3; k0 += 32) {       // the eight lines k0..k0+7 lie in one mask word
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = k0 + u < K3 ? tile_nbr[(k0 + u) * TILE + lane] : -1;
        uint32_t bits = 0;                          // lanes 0..3: group `lane`
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint64_t vote = __ballot(v[u] >= 0);
            if (lane < 4 && ((vote >> (16 * lane)) & 0xffffull) != 0) bits |= 1u << ((k0 + u) & 31);
        }
        if (lane < 4 && bits) atomicOr(&mask_s[lane * mw + (k0 >> 5)], bits);
    }
    __syncthreads();
    if (threadIdx.x < 4 * mw) gmask[tile * (4 * mw) + threadIdx.x] = mask_s[threadIdx.x];
}

// ---- reading a map back -----------------------------------------------------------------------
__global__ void __launch_bounds__(256)
k_counts_clear_pairs(sc_counts* counts) {
    for (int i = threadIdx.x; i < 343; i += blockDim.x) counts->per_offset[i] = 0;
    if (threadIdx.x == 0) counts->n_pairs = 0;
}

// One wavefront per (tile, offset) line of the table: count the rows that have a neighbour.
__global__ void __launch_bounds__(256)
k_count_pairs(const int32_t* __restrict__ nbr, int K3, int64_t tiles_bound, sc_counts* counts, int inverse) {
    __shared__ int32_t hist[343];
    for (int i = threadIdx.x; i < K3; i += blockDim.x) hist[i] = 0;
    __syncthreads();
    int64_t tiles = ((inverse ? counts->n_in : counts->n_out) + TILE - 1) / TILE;
    if (tiles > tiles_bound) tiles = tiles_bound;
    const int64_t items = tiles * K3;
    const int lane = threadIdx.x & 63;
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t it = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); it < items; it += nwaves) {
        const int k = (int)(it % K3);
        const int c = __popcll(__ballot(nbr[it * TILE + lane] >= 0));
        if (lane == 0 && c) atomicAdd(&hist[k], c);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < K3; i += blockDim.x) {
        if (hist[i]) {
            atomicAdd(&counts->per_offset[i], hist[i]);
            atomicAdd((unsigned long long*)&counts->n_pairs, (unsigned long long)hist[i]);
        }
    }
}

// Plain pair lists: one workgroup per offset k walks the tiles in order, 16 tiles (one per
// wavefront) at a time; the rows with a neighbour are compacted by ballot + prefix count behind
// those of the earlier tiles, so the pairs of an offset come out ordered by output row.
__global__ void __launch_bounds__(1024)
k_export(const int32_t* __restrict__ nbr, int K3, int64_t tiles, const int32_t* __restrict__ offset_start,
         int32_t* __restrict__ pairs_in, int32_t* __restrict__ pairs_out) {
    __shared__ int32_t cnt_s[16];
    __shared__ int32_t carry_s;
    const int k = blockIdx.x;
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    if (threadIdx.x == 0) carry_s = offset_start[k];
    __syncthreads();
    for (int64_t t0 = 0; t0 < tiles; t0 += 16) {
        const int64_t t = t0 + w;
        int32_t v = -1;
        if (t < tiles) v = nbr[(t * K3 + k) * TILE + lane];
        const uint64_t vote = __ballot(v >= 0);
        if (lane == 0) cnt_s[w] = __popcll(vote);
        __syncthreads();
        int32_t base = carry_s;
        for (int ww = 0; ww < w; ++ww) base += cnt_s[ww];
        if (v >= 0) {
            const int32_t dst = base + __popcll(vote & lanemask_lt());
            pairs_in[dst] = v;
            pairs_out[dst] = (int32_t)(t * TILE + lane);
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            int32_t total = 0;
            for (int ww = 0; ww < 16; ++ww) total += cnt_s[ww];
            carry_s += total;
        }
        __syncthreads();
    }
}

struct StartArg {
    int32_t v[344];
};
__global__ void __launch_bounds__(256)
k_write_starts(StartArg a, int count, int32_t* __restrict__ dst) {
    for (int i = threadIdx.x; i < count; i += blockDim.x) dst[i] = a.v[i];
}

// Inverse layer (Section III-E): the pairs of a strided map with input and output swapped.
// One wavefront per coarse tile and offset line: row i of the fine set learns its coarse parent.
__global__ void __launch_bounds__(256)
k_transpose_scatter(const int32_t* __restrict__ nbr, int K3, const sc_counts* __restrict__ counts,
                    int32_t* __restrict__ inv_nbr, KmapHeader* hdr, KmapHeader hdr_value) {
    const int lane = threadIdx.x & 63;
    if (blockIdx.x == 0 && threadIdx.x == 0) *hdr = hdr_value;
    const int64_t tiles = (counts->n_out + TILE - 1) / TILE;
    const int64_t items = tiles * K3;
    const int64_t nwaves = (int64_t)gridDim.x * (blockDim.x >> 6);
    for (int64_t it = (int64_t)blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6); it < items; it += nwaves) {
        const int64_t t = it / K3;
        const int k = (int)(it - t * K3);
        const int32_t i = nbr[it * TILE + lane];
        if (i >= 0) inv_nbr[((int64_t)(i >> 6) * K3 + k) * TILE + (i & 63)] = (int32_t)(t * TILE + lane);
    }
}

// candidates per input of a strided layer: ceil(K/s)^3
static int strided_maxc(int K, int stride) {
    const int m = (K + stride - 1) / stride;
    return m * m * m;
}

static bool kmap_args_ok(int64_t n, int K, int stride, int mode) {
    if (n < 0 || n > SC_N_MAX || K < 1 || K > SC_K_MAX) return false;
    if (mode == SC_SUBM) return stride == 1 && (K % 2) == 1;
    if (mode == SC_INVERSE) return K == stride && K >= 2 && K <= 4;
    if (mode == SC_STRIDED) {
        if (K < 2 || stride < 1 || stride > K) return false;
        return n * (int64_t)strided_maxc(K, stride) <= SC_N_MAX;     // candidate ids and output rows fit
    }
    return false;
}
static bool strided_fast(int K, int stride) { return K == stride && K <= 4; }

}  // namespace sc

using namespace sc;

extern "C" int64_t sc_out_bound(int64_t n, int K, int stride, int mode) {
    if (!kmap_args_ok(n, K, stride, mode)) return -1;
    return mode == SC_STRIDED ? n * (int64_t)strided_maxc(K, stride) : n;
}

extern "C" size_t sc_kmap_bytes(int64_t n, int K, int stride, int mode) {
    if (!kmap_args_ok(n, K, stride, mode)) return 0;
    return kmap_layout(sc_out_bound(n, K, stride, mode), K).bytes;
}

extern "C" size_t sc_kmap_scratch_bytes(int64_t n, int K, int stride, int mode) {
    if (!kmap_args_ok(n, K, stride, mode)) return 0;
    if (mode == SC_SUBM) return 256;
    if (mode == SC_STRIDED && !strided_fast(K, stride))
        return strided_scratch(nullptr, sc_out_bound(n, K, stride, mode), 2).bytes;    // one entry per candidate
    return strided_scratch(nullptr, n).bytes;
}

static int kmap_build(const int32_t* d_coords, int64_t n, const void* d_table, int K, int stride, int mode,
                      int32_t* d_out_coords, void* d_kmap, size_t kmap_bytes, void* d_scratch, size_t scratch_bytes,
                      sc_counts* d_counts, void* stream) {
    if (!kmap_args_ok(n, K, stride, mode) || mode == SC_INVERSE) return SC_EINVAL;   // inverse maps: sc_kmap_transpose
    if (d_kmap == nullptr || d_counts == nullptr || (n > 0 && d_coords == nullptr)) return SC_EINVAL;
    if (!aligned16(d_coords) || !aligned16(d_kmap) || !aligned16(d_counts) || !aligned16(d_out_coords) ||
        !aligned16(d_scratch) || !aligned16(d_table))
        return SC_EINVAL;
    if (mode == SC_SUBM && d_table == nullptr) return SC_EINVAL;
    if (mode == SC_STRIDED && (d_out_coords == nullptr || d_scratch == nullptr)) return SC_EINVAL;
    if (kmap_bytes < sc_kmap_bytes(n, K, stride, mode)) return SC_ECAP;
    if (scratch_bytes < sc_kmap_scratch_bytes(n, K, stride, mode) && mode == SC_STRIDED) return SC_ECAP;

    hipStream_t s = (hipStream_t)stream;
    const int64_t bound = sc_out_bound(n, K, stride, mode);
    const KmapLayout L = kmap_layout(bound, K);
    uint32_t* gmask = (uint32_t*)((char*)d_kmap + L.off_mask);
    int32_t* nbr = (int32_t*)((char*)d_kmap + L.off_nbr);
    KmapHeader h{};
    h.magic = KMAP_MAGIC; h.K = K; h.stride = stride; h.mode = mode;
    h.n_in = n; h.n_out_bound = bound; h.tiles = L.tiles; h.mw = L.mw;
    if (n == 0) {
        if (mode == SC_STRIDED && d_table == nullptr)
            SC_LAUNCH(KID_FILL_I32, k_strided_fill, dim3(1), dim3(256), 0, s, (uint4*)nullptr, (uint64_t)0, (int4*)nullptr,
                      (int64_t)0, d_counts, 1, (int64_t)0, (const TableHeader*)nullptr);
        SC_LAUNCH(KID_KMAP_HEADER, k_kmap_header, dim3(1), dim3(64), 0, s, (KmapHeader*)d_kmap, h);
        SC_LAUNCH(KID_MISC, k_set_n_out, dim3(1), dim3(64), 0, s, d_counts, (int64_t)0);
        return SC_OK;
    }

    if (mode == SC_SUBM) {
        HashTable t = table_view(const_cast<void*>(d_table), n);
#define SC_SUBM_LAUNCH(KV, WPT, CH, AT)                                                                           \
    SC_LAUNCH(KID_KMAP_SUBM, (k_kmap_subm<KV, WPT, CH, AT>), dim3(xcd_grid(L.tiles)), dim3(64 * WPT), 0, s,      \
              (const int4*)d_coords, n, (const uint4*)t.slots, (const TableHeader*)t.hdr, gmask, nbr, d_counts,          \
              (KmapHeader*)d_kmap, h)
        switch (K) {
            case 1: SC_SUBM_LAUNCH(1, 1, 1, 1); break;
            case 3: SC_SUBM_LAUNCH(3, 8, 4, 1); break;
            case 5: SC_SUBM_LAUNCH(5, 8, 4, 1); break;
            case 7: SC_SUBM_LAUNCH(7, 8, 4, 1); break;
            default: return SC_EINVAL;
        }
#undef SC_SUBM_LAUNCH
        if (d_out_coords != nullptr && d_out_coords != d_coords) {
            if (hipMemcpyAsync(d_out_coords, d_coords, (size_t)n * 16, hipMemcpyDeviceToDevice, s) != hipSuccess)
                return SC_EHIP;
        }
        return SC_OK;
    }

    const TableHeader* table_hdr = (const TableHeader*)d_table;
    if (!strided_fast(K, stride)) {
        // strided, general K and stride: the same pipeline over candidates (input, offset)
        const int maxc = strided_maxc(K, stride);
        const int64_t nc = n * maxc;
        StridedScratch g = strided_scratch(d_scratch, nc, 2);
        const uint64_t gcap = (uint64_t)g.omask + 1;
        const int64_t gvec = (int64_t)((L.bytes - L.off_nbr) / 16);
        {
            // the offset table is filled further down, once the number of output rows is known: the
            // bound is ceil(K/s)^3 rows per input, real sets need about one
            unsigned fb = (unsigned)((gcap + 255) / 256);
            if (fb > 4096) fb = 4096;
            SC_LAUNCH(KID_FILL_I32, k_strided_fill, dim3(fb), dim3(256), 0, s, g.oslots, gcap, (int4*)nbr, (int64_t)0,
                      d_counts, d_table == nullptr ? 1 : 0, n, table_hdr);
        }
        const int64_t gblk = (nc + 1023) / 1024;
        const unsigned gg = (unsigned)((nc + 255) / 256);
        SC_LAUNCH(KID_STRIDED_INSERT, k_gstrided_insert, dim3(gg), dim3(256), 0, s, (const int4*)d_coords, n, K, stride,
                  maxc, g.oslots, g.omask, g.slot_of, d_counts);
        SC_LAUNCH(KID_STRIDED_FLAGS, k_strided_flags, dim3((unsigned)gblk), dim3(1024), 0, s, nc,
                  (const int32_t*)g.slot_of, (const uint4*)g.oslots, g.flagword, g.word_prefix, g.block_sum);
        SC_LAUNCH(KID_SCAN_BLOCKS, k_scan_blocks, dim3(1), dim3(1024), 0, s, (const int32_t*)g.block_sum,
                  g.block_prefix, gblk, d_counts);
        {
            unsigned fb = (unsigned)((gvec + 255) / 256);
            if (fb > 2048) fb = 2048;
            SC_LAUNCH(KID_FILL_I32, k_fill_rows, dim3(fb), dim3(256), 0, s, (int4*)nbr, L.K3, (const sc_counts*)d_counts);
        }
        SC_LAUNCH(KID_STRIDED_PAIRS, k_gstrided_pairs, dim3(gg), dim3(256), 0, s, (const int4*)d_coords, n, K, stride,
                  maxc, (const int32_t*)g.slot_of, (const uint4*)g.oslots, (const uint64_t*)g.flagword,
                  (const int32_t*)g.word_prefix, (const int32_t*)g.block_prefix, nbr, (int4*)d_out_coords,
                  (KmapHeader*)d_kmap, h);
        SC_LAUNCH(KID_KMAP_FROM_OFT, k_masks_from_table, dim3((unsigned)L.tiles), dim3(256), 0, s,
                  (const int32_t*)nbr, L.K3, L.mw, L.tiles, gmask, (const sc_counts*)d_counts, 0);
        return SC_OK;
    }

    // strided, K == stride
    StridedScratch sc_ = strided_scratch(d_scratch, n);
    const uint64_t cap = (uint64_t)sc_.omask + 1;
    const int64_t nbr_vec = (int64_t)((L.bytes - L.off_nbr) / 16);
    {
        int64_t work = (int64_t)cap > nbr_vec ? (int64_t)cap : nbr_vec;
        unsigned fb = (unsigned)((work + 255) / 256);
        if (fb > 4096) fb = 4096;
        SC_LAUNCH(KID_FILL_I32, k_strided_fill, dim3(fb), dim3(256), 0, s, sc_.oslots, cap, (int4*)nbr, nbr_vec,
                  d_counts, d_table == nullptr ? 1 : 0, n, table_hdr);
    }
    const int64_t nblk = (n + 1023) / 1024;
    const unsigned gb = (unsigned)((n + 255) / 256);
    SC_LAUNCH(KID_STRIDED_INSERT, k_strided_insert, dim3(gb), dim3(256), 0, s, (const int4*)d_coords, n, stride,
              sc_.oslots, sc_.omask, sc_.slot_of, d_counts);
    SC_LAUNCH(KID_STRIDED_FLAGS, k_strided_flags, dim3((unsigned)nblk), dim3(1024), 0, s, n,
              (const int32_t*)sc_.slot_of, (const uint4*)sc_.oslots, sc_.flagword, sc_.word_prefix, sc_.block_sum);
    if (nblk <= SCAN_IN_PAIRS_MAX) {
        SC_LAUNCH(KID_STRIDED_PAIRS, k_strided_pairs<1>, dim3(gb), dim3(256), 0, s, (const int4*)d_coords, n, stride, L.K3,
                  (const int32_t*)sc_.slot_of, (const uint4*)sc_.oslots, (const uint64_t*)sc_.flagword,
                  (const int32_t*)sc_.word_prefix, (const int32_t*)nullptr, (const int32_t*)sc_.block_sum, (int)nblk, nbr,
                  (int4*)d_out_coords, d_counts, (KmapHeader*)d_kmap, h);
    } else {
        SC_LAUNCH(KID_SCAN_BLOCKS, k_scan_blocks, dim3(1), dim3(1024), 0, s, (const int32_t*)sc_.block_sum,
                  sc_.block_prefix, nblk, d_counts);
        SC_LAUNCH(KID_STRIDED_PAIRS, k_strided_pairs<0>, dim3(gb), dim3(256), 0, s, (const int4*)d_coords, n, stride, L.K3,
                  (const int32_t*)sc_.slot_of, (const uint4*)sc_.oslots, (const uint64_t*)sc_.flagword,
                  (const int32_t*)sc_.word_prefix, (const int32_t*)sc_.block_prefix, (const int32_t*)sc_.block_sum,
                  (int)nblk, nbr, (int4*)d_out_coords, d_counts, (KmapHeader*)d_kmap, h);
    }
    SC_LAUNCH(KID_KMAP_FROM_OFT, k_masks_from_table, dim3((unsigned)L.tiles), dim3(256), 0, s,
              (const int32_t*)nbr, L.K3, L.mw, L.tiles, gmask, (const sc_counts*)d_counts, 0);
    return SC_OK;
}

extern "C" int sc_kmap_build(const int32_t* d_coords, int64_t n, const void* d_table, int K, int stride, int mode,
                             int32_t* d_out_coords, void* d_kmap, size_t kmap_bytes, void* d_scratch,
                             size_t scratch_bytes, sc_counts* d_counts, void* stream) {
    return kmap_build(d_coords, n, d_table, K, stride, mode, d_out_coords, d_kmap, kmap_bytes, d_scratch, scratch_bytes,
                      d_counts, stream);
}

// ---- the same build for callers that cannot allocate ------------------------------------------
// The scratch of a strided build (output-cell table, per-input slots, flag words, prefixes) lives
// in one device array of the library instead of a caller's buffer.  Every device holds its own
// copy of the array at its own address; the name below is only a host-side handle, so the
// address is asked for once per device (with that device current) and that pointer is what the
// kernels receive.  The build clears what it needs itself (k_strided_fill), so the contents a
// previous call left behind do not matter; two calls that overlap on one device would race.
static __device__ __align__(256) unsigned char scratch[SC_NOALLOC_SCRATCH_BYTES];

static int noalloc_scratch(void** out) {
    constexpr int MAX_DEVICES = 64;
    static void* ptr[MAX_DEVICES] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SC_EHIP;
    if (ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return SC_EHIP;
        ptr[dev] = p;
    }
    *out = ptr[dev];
    return SC_OK;
}

extern "C" int sc_kmap_build_noalloc(const int32_t* d_coords, int64_t n, const void* d_table, int K, int stride,
                                     int mode, int32_t* d_out_coords, void* d_kmap, size_t kmap_bytes,
                                     sc_counts* d_counts, void* stream) {
    if (!kmap_args_ok(n, K, stride, mode) || mode == SC_INVERSE) return SC_EINVAL;
    const size_t need = sc_kmap_scratch_bytes(n, K, stride, mode);
    if (need > (size_t)SC_NOALLOC_SCRATCH_BYTES) return SC_ECAP;
    void* p = nullptr;
    if (int rc = noalloc_scratch(&p)) return rc;
    return kmap_build(d_coords, n, d_table, K, stride, mode, d_out_coords, d_kmap, kmap_bytes, p,
                      (size_t)SC_NOALLOC_SCRATCH_BYTES, d_counts, stream);
}

extern "C" int sc_kmap_transpose(const void* d_kmap, int64_t n, int K, int stride, const sc_counts* d_counts,
                                 void* d_kmap_inv, size_t kmap_inv_bytes, void* stream) {
    if (!kmap_args_ok(n, K, stride, SC_STRIDED)) return SC_EINVAL;
    if (d_kmap == nullptr || d_kmap_inv == nullptr || d_counts == nullptr || d_kmap == d_kmap_inv) return SC_EINVAL;
    if (!aligned16(d_kmap) || !aligned16(d_kmap_inv) || !aligned16(d_counts)) return SC_EINVAL;
    if (kmap_inv_bytes < sc_kmap_bytes(n, K, stride, SC_INVERSE)) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    const KmapLayout L = kmap_layout(n, K);          // same shape for both directions when K == stride
    KmapHeader h{};
    h.magic = KMAP_MAGIC; h.K = K; h.stride = stride; h.mode = SC_INVERSE;
    h.n_in = n; h.n_out_bound = n; h.tiles = L.tiles; h.mw = L.mw;
    if (n == 0) {
        SC_LAUNCH(KID_KMAP_HEADER, k_kmap_header, dim3(1), dim3(64), 0, s, (KmapHeader*)d_kmap_inv, h);
        return SC_OK;
    }
    const int32_t* nbr = (const int32_t*)((const char*)d_kmap + L.off_nbr);
    int32_t* inv_nbr = (int32_t*)((char*)d_kmap_inv + L.off_nbr);
    uint32_t* inv_mask = (uint32_t*)((char*)d_kmap_inv + L.off_mask);
    const int64_t nbr_vec = (int64_t)((L.bytes - L.off_nbr) / 16);
    unsigned fb = (unsigned)((nbr_vec + 255) / 256);
    if (fb > 4096) fb = 4096;
    SC_LAUNCH(KID_FILL_I32, k_strided_fill, dim3(fb), dim3(256), 0, s, (uint4*)nullptr, (uint64_t)0, (int4*)inv_nbr,
              nbr_vec, (sc_counts*)nullptr, 0, (int64_t)0, (const TableHeader*)nullptr);
    int64_t items = L.tiles * L.K3;
    unsigned gb = (unsigned)((items + 3) / 4);
    if (gb > 4096) gb = 4096;
    SC_LAUNCH(KID_MISC, k_transpose_scatter, dim3(gb), dim3(256), 0, s, nbr, L.K3, d_counts, inv_nbr,
              (KmapHeader*)d_kmap_inv, h);
    SC_LAUNCH(KID_KMAP_FROM_OFT, k_masks_from_table, dim3((unsigned)L.tiles), dim3(256), 0, s,
              (const int32_t*)inv_nbr, L.K3, L.mw, L.tiles, inv_mask, d_counts, 1);
    return SC_OK;
}

extern "C" int sc_counts_read(sc_counts* d_counts, sc_counts* h_counts, const void* d_kmap, int64_t n, int K,
                              int stride, int mode, void* stream) {
    if (d_counts == nullptr || h_counts == nullptr) return SC_EINVAL;
    hipStream_t s = (hipStream_t)stream;
    if (d_kmap != nullptr) {
        if (!kmap_args_ok(n, K, stride, mode)) return SC_EINVAL;
        const KmapLayout L = kmap_layout(sc_out_bound(n, K, stride, mode), K);
        SC_LAUNCH(KID_MISC, k_counts_clear_pairs, dim3(1), dim3(256), 0, s, d_counts);
        if (L.tiles > 0) {
            int64_t items = L.tiles * L.K3;
            unsigned gb = (unsigned)((items + 3) / 4);
            if (gb > 2048) gb = 2048;
            SC_LAUNCH(KID_COUNT_PAIRS, k_count_pairs, dim3(gb), dim3(256), 0, s,
                      (const int32_t*)((const char*)d_kmap + L.off_nbr), L.K3, L.tiles, d_counts,
                      mode == SC_INVERSE ? 1 : 0);
        }
    }
    if (hipMemcpyAsync(h_counts, d_counts, sizeof(sc_counts), hipMemcpyDeviceToHost, s) != hipSuccess) return SC_EHIP;
    if (hipStreamSynchronize(s) != hipSuccess) return SC_EHIP;
    return h_counts->status < 0 ? h_counts->status : SC_OK;
}

extern "C" int sc_kmap_export(const void* d_kmap, int64_t n, int K, int stride, int mode, const sc_counts* h_counts,
                              int32_t* d_pairs_in, int32_t* d_pairs_out, int32_t* d_offset_start, void* stream) {
    if (d_kmap == nullptr || h_counts == nullptr || d_offset_start == nullptr) return SC_EINVAL;
    if (!kmap_args_ok(n, K, stride, mode)) return SC_EINVAL;
    if (h_counts->n_pairs > 0 && (d_pairs_in == nullptr || d_pairs_out == nullptr)) return SC_EINVAL;
    if (h_counts->n_pairs > 0x7fffffffLL) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    const KmapLayout L = kmap_layout(sc_out_bound(n, K, stride, mode), K);
    StartArg h_start{};
    int32_t acc = 0;
    for (int k = 0; k < L.K3; ++k) {
        h_start.v[k] = acc;
        acc += h_counts->per_offset[k];
    }
    h_start.v[L.K3] = acc;
    if ((int64_t)acc != h_counts->n_pairs) return SC_EINVAL;
    SC_LAUNCH(KID_MISC, k_write_starts, dim3(1), dim3(256), 0, s, h_start, L.K3 + 1, d_offset_start);
    const int64_t tiles = ((mode == SC_INVERSE ? h_counts->n_in : h_counts->n_out) + TILE - 1) / TILE;
    if (tiles > 0 && acc > 0)
        SC_LAUNCH(KID_EXPORT, k_export, dim3((unsigned)L.K3), dim3(1024), 0, s,
                  (const int32_t*)((const char*)d_kmap + L.off_nbr), L.K3, tiles, (const int32_t*)d_offset_start,
                  d_pairs_in, d_pairs_out);
    return SC_OK;
}
