// Compute step: out[o] = sum_k sum_{(i,o) in M_k} in[i] . W[k]   (paper Algorithm 2).
//
// The paper's kernel gives one thread one (output row, output channel) and walks K^3 x C_in
// scalar FMAs with one output channel's weights cached in shared memory, so every gathered
// feature row is re-read C_out times.  Here a wavefront owns 16 consecutive output rows (a
// quarter of a kernel-map tile).  For every offset k at which that group has a neighbour (one
// bit test) it gathers the 16 input rows straight into MFMA operand registers, 16 bytes per
// lane, zero where a row has no neighbour, and multiplies them by W[k] on the matrix cores
// (v_mfma_f32_16x16x32, fp32 accumulation).  Because an output row keeps its place in the group
// for every offset, the accumulators stay in registers for the whole layer: no atomics, no
// scatter, one conversion and one store per output row.  Groups without a neighbour at k are
// skipped; on surface-like voxel sets this issues about 1.8x the MACs that exist.
// A layer of ~10^5 voxels is a few microseconds of matrix work, so what decides its time is how
// many loads are in flight: the kernels below issue the offset-table reads of all K^3 offsets,
// then all feature gathers, before the first multiply.
#include "sc_internal.h"

namespace sc {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Packed weights: W [K3][C_in][C_out] (16-bit elements) as MFMA A-operand tiles of W[k]^T.  A tile
// is 64 lanes x 16 bytes: lane l of tile (k, cb, ks) holds W[k][ks*32 + 8*(l/16) + j][cb*16 + l%16],
// j = 0..7.  Inside one offset k the tiles are ordered by 64-channel half of C_in first, then
// output block, then 32-channel slice of the half, so the tiles a kernel needs for one half of the
// input channels are one contiguous piece: tile number wtile(KS, CB, cb, ks) below (for C_in = 32
// there is one slice and the order is just cb).
__host__ __device__ constexpr int wtile(int KS, int CB, int cb, int ks) {
    return KS == 1 ? cb : ((ks >> 1) * CB + cb) * 2 + (ks & 1);
}
__global__ void __launch_bounds__(256)
k_weight_pack(const uint16_t* __restrict__ w, uint4* __restrict__ wp, int K3, int C_in, int C_out) {
    const int KS = C_in / 32, CB = C_out / 16;
    const int64_t total = (int64_t)K3 * CB * KS * 64;
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= total) return;
    const int lane = (int)(t & 63);
    int64_t rest = t >> 6;
    const int ks = (int)(rest % KS); rest /= KS;
    const int cb = (int)(rest % CB);
    const int k = (int)(rest / CB);
    const int co = cb * 16 + (lane & 15);
    const int ci0 = ks * 32 + 8 * (lane >> 4);
    const uint16_t* src = w + ((int64_t)k * C_in + ci0) * C_out + co;
    uint32_t v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        v[j] = (uint32_t)src[(int64_t)(2 * j) * C_out] | ((uint32_t)src[(int64_t)(2 * j + 1) * C_out] << 16);
    wp[((int64_t)k * CB * KS + wtile(KS, CB, cb, ks)) * 64 + lane] = make_uint4(v[0], v[1], v[2], v[3]);
}

// Workgroup barrier for data exchanged through LDS only.  __syncthreads() also waits until every
// outstanding global load of the wavefront has returned (vmcnt(0)), which would drain the gathers
// and weight fetches that were issued ahead on purpose; here only the wavefront's LDS operations
// have to be complete before it arrives.
__device__ inline void lds_barrier() {
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

template <int DT>
__device__ inline f32x4 mfma16x16x32(uint4 a, uint4 b, f32x4 c) {
    if constexpr (DT == SC_F16)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

__device__ inline uint32_t f32_to_bf16_rne(float f) {
    uint32_t u = __builtin_bit_cast(uint32_t, f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;     // NaN stays NaN
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}
template <int DT>
__device__ inline uint32_t pack2(float lo, float hi) {
    if constexpr (DT == SC_F16) {
        const _Float16 a = (_Float16)lo, b = (_Float16)hi;              // round to nearest even
        return (uint32_t)__builtin_bit_cast(uint16_t, a) | ((uint32_t)__builtin_bit_cast(uint16_t, b) << 16);
    } else {
        return f32_to_bf16_rne(lo) | (f32_to_bf16_rne(hi) << 16);
    }
}

// Store one accumulator block: the lane holds channels cb*16 + 4*qq .. +3 of output row `row`.
template <int DT>
__device__ inline void store_acc(void* __restrict__ out, int out_f32, int64_t row, int C_out, int col, f32x4 d) {
    if (out_f32) {
        *reinterpret_cast<float4*>(reinterpret_cast<float*>(out) + row * C_out + col) = make_float4(d[0], d[1], d[2], d[3]);
    } else {
        *reinterpret_cast<uint2*>(reinterpret_cast<uint16_t*>(out) + row * C_out + col) =
            make_uint2(pack2<DT>(d[0], d[1]), pack2<DT>(d[2], d[3]));
    }
}

// ---- small layers: all of W resident in LDS ----------------------------------------------------
// One wavefront per 16 output rows, NT tiles (4*NT wavefronts) per workgroup.  The workgroup
// copies the weights of all K3 offsets into LDS once, re-laying them out as MFMA operand tiles on
// the way, so no separate packing pass is needed; meanwhile every wavefront has its K3 offset-table lines and then all its feature
// gathers in flight.  KS = C_in/32, CB = C_out/16.
// FUSED: there is no kernel map; the K^3 neighbours of a row are looked up in the dense location
// table right here (one index computation and one 8-byte load each, all in flight together), and
// the group's mask is a vote over what was found.  n_out_cap is then the number of rows.
// UP: the inverse (up-sampling) layer of a K == stride layer, straight from that layer's own map
// (Section III-E: the same pairs with input and output swapped).  The wavefront's 16 rows are
// coarse rows, read in place; entry k of a row's table column names the fine row that receives
// row . W[k].  Every fine row has exactly one parent, so results are stored, not accumulated, and
// nothing needs to be transposed first.
template <int DT, int K3, int KS, int CB, int NT, int FUSED, int UP = 0, int WPACKED = 0>
__global__ void __launch_bounds__(256 * NT)
k_conv_rows16(const uint16_t* __restrict__ feat, const uint4* __restrict__ wraw, void* __restrict__ out, int out_f32,
              const MapSource ms, const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    static_assert(K3 <= 32, "one mask word per group");
    static_assert(!FUSED || K3 == 27, "fused look-ups: 3x3x3 layers");
    static_assert(!(FUSED && UP), "one or the other");
    const uint32_t* __restrict__ gmask = ms.gmask;
    const int32_t* __restrict__ nbr = ms.nbr;
    constexpr int C_in = KS * 32, C_out = CB * 16;
    extern __shared__ __align__(16) uint4 w_lds[];                   // [K3][CB][KS][64]
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int r = lane & 15, qq = lane >> 4;
    const int q = wv & 3;
    SC_MARK(0);
    int64_t n_out = n_out_cap;
    if (!FUSED && *n_out_ptr < n_out) n_out = *n_out_ptr;
    // the grid covers the caller's row capacity; the rows that exist are spread over all XCDs and
    // a workgroup that gets none leaves at once (the whole workgroup, before any barrier)
    const int64_t unit = xcd_unit_of(blockIdx.x, (n_out + NT * TILE - 1) / (NT * TILE));
    if (unit < 0) return;
    const int64_t tile = unit * NT + (wv >> 2);
    const int64_t row = tile * TILE + q * 16 + r;
    const bool group_ok = tile * TILE + q * 16 < n_out;             // uniform per wavefront

    // the group's offset-table lines (all K3 of them) and its mask word: one round trip
    int32_t e[K3];
    uint32_t m = 0;
    if constexpr (FUSED) {
        // the four lanes that serve a row look up every fourth offset each and trade the results
        // through LDS (a wavefront's LDS operations execute in order: no barrier needed)
        __shared__ int32_t found_s[FUSED ? 4 * NT : 1][28][16];
        if (group_ok) {
            int32_t part[7];
            grid_neighbours_quarter<3>(ms, row, n_out, qq, part);
#pragma unroll
            for (int u = 0; u < 7; ++u) found_s[wv][qq + 4 * u][r] = part[u];
#pragma unroll
            for (int k = 0; k < K3; ++k) e[k] = found_s[wv][k][r];
#pragma unroll
            for (int k = 0; k < K3; ++k) m |= (__ballot(e[k] >= 0) != 0ull ? 1u : 0u) << k;
        } else {
#pragma unroll
            for (int k = 0; k < K3; ++k) e[k] = -1;
        }
    } else if (group_ok) {
        const int32_t* line = nbr + tile * (int64_t)(K3 * TILE) + q * 16 + r;
#pragma unroll
        for (int k = 0; k < K3; ++k) e[k] = line[k * TILE];
        m = gmask[tile * 4 + q];
    } else {
#pragma unroll
        for (int k = 0; k < K3; ++k) e[k] = -1;
    }
    // weights -> LDS as operand tiles (every thread helps, also wavefronts without rows): the
    // thread that fills (tile, lane) reads its 8 input channels of one output channel (2-byte
    // loads, 128 contiguous bytes per wavefront) and writes them as one 16-byte LDS store
    if constexpr (WPACKED) {
        // the caller packed the weights once (sc_conv_weight_pack): the tiles are copied as they are
        for (int i = threadIdx.x; i < K3 * CB * KS * 64; i += 256 * NT) w_lds[i] = wraw[i];
    } else {
        const uint16_t* w16 = reinterpret_cast<const uint16_t*>(wraw);
        for (int i = threadIdx.x; i < K3 * CB * KS * 64; i += 256 * NT) {
            const int ln = i & 63;
            int rest = i >> 6;
            const int ks = rest % KS; rest /= KS;
            const int cb = rest % CB;
            const int k = rest / CB;
            const uint16_t* src = w16 + ((int64_t)k * C_in + ks * 32 + 8 * (ln >> 4)) * C_out + cb * 16 + (ln & 15);
            uint32_t v[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) v[j] = (uint32_t)src[(2 * j) * C_out] | ((uint32_t)src[(2 * j + 1) * C_out] << 16);
            w_lds[i] = make_uint4(v[0], v[1], v[2], v[3]);
        }
    }
    SC_MARK(1);
    m = __builtin_amdgcn_readfirstlane(m);

    if constexpr (UP) {
        uint4 own[KS];                       // the coarse row itself: no gather
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            own[ks] = (group_ok && row < n_out) ? reinterpret_cast<const uint4*>(feat + row * C_in)[qq + ks * 4]
                                                : make_uint4(0, 0, 0, 0);
        __syncthreads();
        SC_MARK(2);
#pragma unroll
        for (int k = 0; k < K3; ++k) {
            if (m & (1u << k)) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) {
                    f32x4 d = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        d = mfma16x16x32<DT>(w_lds[((k * CB + cb) * KS + ks) * 64 + lane], own[ks], d);
                    if (e[k] >= 0) store_acc<DT>(out, out_f32, e[k], C_out, cb * 16 + qq * 4, d);
                }
            }
        }
        SC_MARK(3);
        SC_MARK(4);
        SC_MARK(5);
        return;
    }
    // every gather of the group in flight at once
    uint4 fb[K3][KS];
#pragma unroll
    for (int k = 0; k < K3; ++k) {
        if (m & (1u << k)) {
            const uint4* frow = reinterpret_cast<const uint4*>(feat + (int64_t)(e[k] < 0 ? 0 : e[k]) * C_in) + qq;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) fb[k][ks] = e[k] >= 0 ? frow[ks * 4] : make_uint4(0, 0, 0, 0);
        }
    }
    __syncthreads();
    SC_MARK(2);

    f32x4 acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int k = 0; k < K3; ++k) {
        if (m & (1u << k)) {
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    acc[cb] = mfma16x16x32<DT>(w_lds[((k * CB + cb) * KS + ks) * 64 + lane], fb[k][ks], acc[cb]);
        }
    }
    SC_MARK(3);
    if (group_ok && row < n_out) {
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) store_acc<DT>(out, out_f32, row, C_out, cb * 16 + qq * 4, acc[cb]);
    }
    SC_MARK(4);
    SC_MARK(5);
}

// A row of zeros that stands in for "no neighbour" in the streaming kernels: a lane without an
// input row reads its operand from here, so every lane issues every load.  The compiler can then
// count, at each use, exactly how many younger loads may still be in flight (s_waitcnt vmcnt(n));
// a load that is skipped under a condition makes that count unknown and every wait becomes
// vmcnt(0), which drains the loads that were issued ahead on purpose.
__device__ __align__(256) uint4 g_zero_row[32];      // 512 bytes: a row of up to 256 16-bit channels

// ---- larger layers: W[k] streamed through LDS, one offset at a time ------------------------------
// One wavefront per 64-row tile (four 16-row groups), NWV tiles per workgroup.  The workgroup
// walks the K3 offsets in lockstep; W[k] reaches the matrix cores through a double-buffered LDS
// tile, each weight operand read once and applied to every group of the wavefront that has a
// neighbour at k.  Everything else is arranged so that loads stay in flight across steps:
//  * the tile's offset-table lines are copied to LDS once, up front, so the loop reads neighbour
//    indices through the LDS counter and never has to wait on the vector-memory counter for them
//    (that counter retires in order: waiting for a young index load would drain every older
//    gather and weight fetch with it);
//  * gathered rows live in a ring of D register slots: as soon as a 32-channel slice of slot
//    k % D has been used it is refilled with the rows of offset k + D;
//  * W[k + D] is fetched into registers at the top of step k and stored to LDS at the end of step
//    k + D - 1;
//  * every load is issued by every lane (rows without a neighbour read the zero row), only the
//    multiplies are skipped, so all waits are exact counts.
// Accumulators (64 rows x C_out per wavefront) never leave the registers.  KS = C_in/32,
// CB = C_out/16.
// Rows are gathered in the operand's own lane order (16 rows x four 16-byte pieces of a 32-channel
// slice per load: 64 contiguous bytes of a row).  Gathering whole 128-byte rows with eight
// consecutive lanes per row is cheaper for the address unit, but the rows then have to pass
// through LDS to reach operand layout; k_conv_direct64 does that for 64 input channels, where a
// row is one line.  For wider rows the extra LDS traffic costs more than the gather saves, and an
// in-register shuffle (lane-swap + quad-permute instructions, 20 VALU operations per 16 bytes)
// was measured slower than either.
// FUSED: as in k_conv_rows16, the offset-table lines come from the dense location table directly.
template <int DT, int K3, int KS, int CB, int NWV, int D, int FUSED>
__global__ void __launch_bounds__(64 * NWV, 2)
k_conv_stream(const uint16_t* __restrict__ feat, const uint4* wp, void* __restrict__ out, int out_f32,
              const MapSource ms, const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    static_assert(K3 <= 32, "one mask word per group");
    static_assert(!FUSED || K3 == 27, "fused look-ups: 3x3x3 layers");
    const uint32_t* __restrict__ gmask = ms.gmask;
    const int32_t* __restrict__ nbr = ms.nbr;
    constexpr int NTH = 64 * NWV;
    constexpr int C_in = KS * 32, C_out = CB * 16;
    constexpr int WK = CB * KS * 64;                  // uint4 per packed W[k]
    static_assert(WK % NTH == 0, "a weight matrix is a whole number of passes of the workgroup");
    constexpr int WPT = WK / NTH;                     // uint4 per thread per W[k]
    constexpr int CBG = CB < 4 ? CB : 4;              // weight operands held at a time
    static_assert(CB % CBG == 0, "whole operand batches");
    extern __shared__ __align__(16) uint4 smem[];     // w_lds[2][WK] | e_lds[NWV][K3][64]

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    const int r = lane & 15, qq = lane >> 4;
    uint4* w_lds = smem;
    int32_t* e_lds = reinterpret_cast<int32_t*>(smem + 2 * WK) + wv * (K3 * TILE);
    SC_MARK(0);
    int64_t n_out = n_out_cap;
    if (!FUSED && *n_out_ptr < n_out) n_out = *n_out_ptr;
    // the grid covers the caller's row capacity; the rows that exist are spread over all XCDs and
    // a workgroup that gets none leaves at once (the same decision in every wavefront, before
    // any barrier)
    // a workgroup's tiles are spread over the whole row range (tile = wavefront * units + unit):
    // its steps last as long as its busiest wavefront's, and neighbouring tiles are alike in how
    // many offsets they take part in (10^6 voxels, 128 channels: -2 %)
    const int64_t units = (n_out + NWV * TILE - 1) / (NWV * TILE);
    const int64_t unit = xcd_unit_of(blockIdx.x, units);
    if (unit < 0) return;
    const int64_t tile = wv * units + unit;
    const bool tile_ok = tile * TILE < n_out;

    uint32_t mg[4] = {0u, 0u, 0u, 0u};
    {   // the tile's offset-table lines -> LDS (read back below by other lanes of this wavefront)
        int32_t v[K3];
        if constexpr (FUSED) {
            if (tile_ok) {
                grid_neighbours<3>(ms, tile * TILE + lane, n_out, v);
#pragma unroll
                for (int k = 0; k < K3; ++k) {
                    const uint64_t vote = __ballot(v[k] >= 0);
#pragma unroll
                    for (int g = 0; g < 4; ++g) mg[g] |= (((vote >> (16 * g)) & 0xffffull) != 0ull ? 1u : 0u) << k;
                }
            } else {
#pragma unroll
                for (int k = 0; k < K3; ++k) v[k] = -1;
            }
        } else if (tile_ok) {
            const int32_t* line = nbr + tile * (int64_t)(K3 * TILE) + lane;
#pragma unroll
            for (int k = 0; k < K3; ++k) v[k] = line[k * TILE];
#pragma unroll
            for (int g = 0; g < 4; ++g) mg[g] = gmask[tile * 4 + g];
        } else {
#pragma unroll
            for (int k = 0; k < K3; ++k) v[k] = -1;
        }
#pragma unroll
        for (int k = 0; k < K3; ++k) e_lds[k * TILE + lane] = v[k];
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) mg[g] = __builtin_amdgcn_readfirstlane(mg[g]);
    SC_MARK(1);

    const u32x4* wsrc = reinterpret_cast<const u32x4*>(wp) + threadIdx.x;
    u32x4 wr[D][WPT];
#pragma unroll
    for (int j = 0; j < D && j < K3; ++j)
#pragma unroll
        for (int i = 0; i < WPT; ++i) wr[j][i] = wsrc[(int64_t)j * WK + i * NTH];

    // a lane gathers row lane % 16 of a group, the (lane / 16)-th 16-byte piece of a 32-channel slice
    auto rowptr = [&](int32_t e) -> const uint4* {
        return (e >= 0 ? reinterpret_cast<const uint4*>(feat + (int64_t)e * C_in) : g_zero_row) + qq;
    };
    uint4 fb[D][4][KS];
#pragma unroll
    for (int j = 0; j < D && j < K3; ++j) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint4* frow = rowptr(e_lds[j * TILE + g * 16 + r]);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) fb[j][g][ks] = frow[ks * 4];
        }
    }
    f32x4 acc[4][CB];
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int cb = 0; cb < CB; ++cb) acc[g][cb] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < WPT; ++i) reinterpret_cast<u32x4*>(w_lds)[threadIdx.x + i * NTH] = wr[0][i];
    lds_barrier();
    SC_MARK(2);

#pragma unroll
    for (int k = 0; k < K3; ++k) {
        const bool more = k + D < K3;
        if (more) {
#pragma unroll
            for (int i = 0; i < WPT; ++i) wr[k % D][i] = wsrc[(int64_t)(k + D) * WK + i * NTH];
        }
        int32_t e4[4] = {-1, -1, -1, -1};
        if (more) {
#pragma unroll
            for (int g = 0; g < 4; ++g) e4[g] = e_lds[(k + D) * TILE + g * 16 + r];
        }
        __builtin_amdgcn_sched_barrier(0);            // the fetches are issued here, not next to their use
        const uint4* wk = w_lds + (k & 1) * WK + lane;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int c0 = 0; c0 < CB; c0 += CBG) {
                uint4 a[CBG];
#pragma unroll
                for (int c = 0; c < CBG; ++c) a[c] = wk[wtile(KS, CB, c0 + c, ks) * 64];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    if ((mg[g] >> k) & 1u) {
#pragma unroll
                        for (int c = 0; c < CBG; ++c)
                            acc[g][c0 + c] = mfma16x16x32<DT>(a[c], fb[k % D][g][ks], acc[g][c0 + c]);
                    }
                }
            }
            if (more && D == 1) {   // this slice is free: refill it with the rows of offset k + D
#pragma unroll
                for (int g = 0; g < 4; ++g) fb[k % D][g][ks] = rowptr(e4[g])[ks * 4];
            }
        }
        if (more && D > 1) {
            // with a deeper ring there is no hurry: refill the whole slot at once, so that the loads
            // which share a cache line (the 64-byte slices of one row) are issued back to back
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint4* frow = rowptr(e4[g]);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) fb[k % D][g][ks] = frow[ks * 4];
            }
        }
        if (k + 1 < K3) {
#pragma unroll
            for (int i = 0; i < WPT; ++i)
                reinterpret_cast<u32x4*>(w_lds)[((k + 1) & 1) * WK + threadIdx.x + i * NTH] = wr[(k + 1) % D][i];
            lds_barrier();
        }
    }
    SC_MARK(3);
    if (tile_ok) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int64_t row = tile * TILE + g * 16 + r;
            if (row < n_out) {
#pragma unroll
                for (int cb = 0; cb < CB; ++cb) store_acc<DT>(out, out_f32, row, C_out, cb * 16 + qq * 4, acc[g][cb]);
            }
        }
    }
    SC_MARK(4);
    SC_MARK(5);
}

// ---- 64 input channels: independent wavefronts, weights straight from global memory ---------------
// One wavefront per 64-row tile as in k_conv_stream, but nothing is shared between the wavefronts
// of a workgroup: no weight tile in LDS, no barrier.  A layer of ~10^5 voxels keeps every CU busy
// with a handful of wavefronts, each of which walks its K^3 offsets as one chain; what a step of
// that chain costs is the latency of what it has to wait for, so everything a step needs is
// requested one to two steps ahead and a wavefront never waits for another one.
//  * A wavefront walks only the offsets at which its tile has a neighbour at all (about 60 % of
//    the 27 on surface-like sets), in increasing order, taken from the tile's masks bit by bit.
//  * Multiplies are v_mfma_f32_32x32x16 on the two 32-row halves of the tile.  SKIP = 1: a half
//    without a neighbour at offset k is skipped, and so are its loads (tests and branches in
//    every step, exact wait counts that depend on the tile).  SKIP = 0: such a half is rows of
//    zeros like any row without a neighbour, and a step is one straight line of code, the same
//    for every offset and tile; the host picks the form by how full the CUs are.
//  * The weight operand of that instruction (32 output channels x 16 input channels) is read
//    straight from the packed 16x32 tiles in global memory, one step ahead: both forms keep 8
//    input channels of one output channel in 16 bytes, so only the addresses differ, and a load
//    touches eight whole 128-byte lines.  Every wavefront of the chip reads the same 8 KB per
//    offset: L1 and L2 hits.
//  * Gathers are buffer loads, eight lanes on the eight 16-byte pieces of one 128-byte row: the
//    address is one shift-or (row << 7 | byte in row), and "no neighbour" (row -1) lands beyond
//    the buffer's range, where the hardware returns zeros without touching memory.  The rows
//    land in a ring of three register slots and pass through a 4 KB staging area in LDS (swizzled
//    16-byte slots) to come back in operand layout, one step before they are multiplied.
//  * Loads inside the loop are inline assembly, so that the compiler places no waits of its own
//    for them: which loads are issued depends on the tile, and the one wait per step names the
//    exact number of younger loads that may stay in flight (the counter retires in order).
//    Registers written by such a load are handed back to the compiler through an empty asm
//    statement right after the wait that covers them.
//  * In program order the staging operations of offset k+1 sit between the multiplies of offset
//    k: a wavefront's LDS operations then run in the shadow of its own matrix instructions.
// The feature array must be smaller than 4 GiB (32-bit buffer offsets); the host checks and falls
// back to k_conv_stream otherwise.  The number of tiles per workgroup is the launch's block size
// / 64 (any value up to 8): the host picks it so that the workgroups spread evenly over the CUs.
typedef float f32x16 __attribute__((ext_vector_type(16)));
template <int DT>
__device__ inline f32x16 mfma32x32x16(u32x4 a, u32x4 b, f32x16 c) {
    if constexpr (DT == SC_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
template <int N> struct IntC { static constexpr int value = N; };
constexpr int DIRECT_LINES(int K3) { return K3 + 1; }                // table lines kept in LDS per wavefront
constexpr int DIRECT_STAGE = 32 * 128;                               // bytes of a wavefront's staging area

template <int DT, int K3, int FUSED, int SKIP>
__global__ void __launch_bounds__(512, 1)
k_conv_direct64(const uint16_t* __restrict__ feat, const uint4* wp, void* __restrict__ out, int out_f32,
                const MapSource ms, const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    static_assert(K3 <= 31, "one mask word per half, and one more bit that is never set");
    static_assert(!FUSED || K3 == 27, "fused look-ups: 3x3x3 layers");
    const uint32_t* __restrict__ gmask = ms.gmask;
    const int32_t* __restrict__ nbr = ms.nbr;
    constexpr int MB = 2, C_out = 64, RB = 128;       // 32-channel output blocks, bytes per feature row
    constexpr int KE = DIRECT_LINES(K3);               // the real lines, then one line of "no neighbour"
    extern __shared__ __align__(16) uint4 smem[];     // stage[NWV][32 rows x 128 B] | e_lds[NWV][KE][64]

    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, NWV = blockDim.x >> 6;
    const int r32 = lane & 31, hh = lane >> 5;
    char* stage = reinterpret_cast<char*>(smem) + wv * DIRECT_STAGE;
    int32_t* e_lds = reinterpret_cast<int32_t*>(reinterpret_cast<char*>(smem) + NWV * DIRECT_STAGE) + wv * (KE * TILE);
    int64_t n_out = n_out_cap;
    if (!FUSED && *n_out_ptr < n_out) n_out = *n_out_ptr;
    // a workgroup's tiles are spread over the whole row range (tile = wavefront * units + unit):
    // neighbouring tiles are alike in how many offsets they take part in, and the kernel ends with
    // its slowest workgroup
    const int64_t units = (n_out + (int64_t)NWV * TILE - 1) / ((int64_t)NWV * TILE);
    const int64_t unit = xcd_unit_of(blockIdx.x, units);
    if (unit < 0) return;
    SC_MARK(0);
    const int64_t tile = wv * units + unit;
    const bool tile_ok = tile * TILE < n_out;

    uint32_t mg[2] = {0u, 0u};                         // which offsets each 32-row half takes part in (bits < K3)
    if constexpr (FUSED) {
        int32_t v[K3];
        if (tile_ok) {
            grid_neighbours<3>(ms, tile * TILE + lane, n_out, v);
#pragma unroll
            for (int k = 0; k < K3; ++k) {
                const uint64_t vote = __ballot(v[k] >= 0);
#pragma unroll
                for (int g = 0; g < 2; ++g) mg[g] |= (((vote >> (32 * g)) & 0xffffffffull) != 0ull ? 1u : 0u) << k;
            }
        } else {
#pragma unroll
            for (int k = 0; k < K3; ++k) v[k] = -1;
        }
#pragma unroll
        for (int k = 0; k < K3; ++k) e_lds[k * TILE + lane] = v[k];
    } else {
        // the tile's K3 table lines are one contiguous piece of the map: 16 bytes per lane and load
        constexpr int LINE16 = K3 * TILE / 4;          // 16-byte pieces
        constexpr int PASSES = (LINE16 + 63) / 64;
        u32x4 v[PASSES];
        const u32x4* line = reinterpret_cast<const u32x4*>(nbr + tile * (int64_t)(K3 * TILE));
#pragma unroll
        for (int i = 0; i < PASSES; ++i)
            v[i] = (tile_ok && i * 64 + lane < LINE16) ? line[i * 64 + lane] : u32x4{~0u, ~0u, ~0u, ~0u};
        if (tile_ok) {
#pragma unroll
            for (int g = 0; g < 2; ++g) mg[g] = gmask[tile * 4 + 2 * g] | gmask[tile * 4 + 2 * g + 1];
        }
#pragma unroll
        for (int i = 0; i < PASSES; ++i)
            if (i * 64 + lane < LINE16) reinterpret_cast<u32x4*>(e_lds)[i * 64 + lane] = v[i];
    }
#pragma unroll
    for (int k = K3; k < KE; ++k) e_lds[k * TILE + lane] = -1;
#pragma unroll
    for (int g = 0; g < 2; ++g) mg[g] = __builtin_amdgcn_readfirstlane(mg[g]);
    auto pattern_at = [&](int k) -> uint32_t { return SKIP ? ((mg[0] >> k) & 1u) | (((mg[1] >> k) & 1u) << 1) : 3u; };
    auto halves_at = [&](int k) -> uint32_t { return ((mg[0] >> k) & 1u) + ((mg[1] >> k) & 1u); };
    // The wavefront walks only the offsets its tile takes part in, in increasing order; K3 stands
    // for "no further offset": no bit of the masks, a table line of "no neighbour".  k0 is the
    // offset of the step at hand, k1..k4 the ones after it (what is requested ahead).
    uint32_t rest = mg[0] | mg[1];
    const int n_steps = __builtin_popcount(rest);
    auto next_offset = [&]() -> int {
        const int k = rest != 0u ? __builtin_ctz(rest) : K3;
        rest &= rest - 1u;
        return k;
    };
    int k0 = next_offset(), k1 = next_offset(), k2 = next_offset(), k3 = next_offset(), k4 = next_offset();

    // gathers: instruction i of a half reads its rows 8i .. 8i+7, eight lanes per row
    const int row8 = lane >> 3, piece = lane & 7;
    // buffer descriptor over the feature array: offsets at or above 0xFFFFFF80 (row -1) read as zeros
    u32x4 rs;
    {
        const uint64_t fa = (uint64_t)feat;
        rs[0] = __builtin_amdgcn_readfirstlane((uint32_t)fa);
        rs[1] = __builtin_amdgcn_readfirstlane((uint32_t)(fa >> 32) & 0xffffu);
        rs[2] = __builtin_amdgcn_readfirstlane(0xFFFFFF80u);
        rs[3] = __builtin_amdgcn_readfirstlane(0x00020000u);
    }
    const uint32_t pbyte = piece << 4;
    // staging area: [32 rows][128 bytes], the 16-byte slots of a row swizzled with the row number;
    // the multiply's operand for 16-channel slice s is piece 2s + (lane / 32) of row lane % 32
    int st_w[4], st_r[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        st_w[i] = (8 * i + row8) * RB + ((piece ^ row8) << 4);
        st_r[i] = r32 * RB + (((2 * i + hh) ^ (r32 & 7)) << 4);
    }
    const int32_t* e_mine = e_lds + row8;
    // row numbers of offset k for this lane's eight loads (read from LDS well ahead of their use), and
    // the byte offsets made of them
    auto row_numbers = [&](uint32_t (&e)[2][4], int k) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) e[g][i] = (uint32_t)e_mine[k * TILE + g * 32 + i * 8];
    };
    auto row_offsets = [&](uint32_t (&off)[2][4], const uint32_t (&e)[2][4]) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) off[g][i] = (e[g][i] << 7) | pbyte;
    };
    // the rows of one offset for the halves named by pat: four loads per half, skipped as a whole otherwise
    auto gather = [&](u32x4 (&dst)[2][4], const uint32_t (&off)[2][4], uint32_t pat) {
#pragma unroll
        for (int g = 0; g < 2; ++g)
            if constexpr (!SKIP)
                asm volatile(
                    "buffer_load_dwordx4 %[d0], %[o0], %[rs], 0 offen\n\t"
                    "buffer_load_dwordx4 %[d1], %[o1], %[rs], 0 offen\n\t"
                    "buffer_load_dwordx4 %[d2], %[o2], %[rs], 0 offen\n\t"
                    "buffer_load_dwordx4 %[d3], %[o3], %[rs], 0 offen"
                    : [d0] "+v"(dst[g][0]), [d1] "+v"(dst[g][1]), [d2] "+v"(dst[g][2]), [d3] "+v"(dst[g][3])
                    : [o0] "v"(off[g][0]), [o1] "v"(off[g][1]), [o2] "v"(off[g][2]), [o3] "v"(off[g][3]), [rs] "s"(rs));
            else
            asm volatile(
                "s_bitcmp1_b32 %[pat], %[bit]\n\t"
                "s_cbranch_scc0 .Lsc_skip_%=\n\t"
                "buffer_load_dwordx4 %[d0], %[o0], %[rs], 0 offen\n\t"
                "buffer_load_dwordx4 %[d1], %[o1], %[rs], 0 offen\n\t"
                "buffer_load_dwordx4 %[d2], %[o2], %[rs], 0 offen\n\t"
                "buffer_load_dwordx4 %[d3], %[o3], %[rs], 0 offen\n"
                ".Lsc_skip_%=:"
                : [d0] "+v"(dst[g][0]), [d1] "+v"(dst[g][1]), [d2] "+v"(dst[g][2]), [d3] "+v"(dst[g][3])
                : [o0] "v"(off[g][0]), [o1] "v"(off[g][1]), [o2] "v"(off[g][2]), [o3] "v"(off[g][3]), [rs] "s"(rs),
                  [pat] "s"(pat), [bit] "n"(g)
                : "scc");
    };
    // the eight weight operands of offset k (slice sl, output block mb), skipped if the tile takes no part
    const int a_lane = 2048 * ((lane >> 4) & 1) + 256 * hh + 16 * (lane & 15);
    const char* w_lane = reinterpret_cast<const char*>(wp) + a_lane;
    auto load_weights = [&](u32x4 (&dst)[4][MB], int k, uint32_t pat) {
        const char* p0 = w_lane + (int64_t)(k < K3 ? k : K3 - 1) * (4 * MB * 1024);
        const char* p1 = p0 + 4096;
        if constexpr (!SKIP)
            asm volatile(
                "global_load_dwordx4 %[d0], %[p0], off\n\t"
                "global_load_dwordx4 %[d1], %[p1], off\n\t"
                "global_load_dwordx4 %[d2], %[p0], off offset:512\n\t"
                "global_load_dwordx4 %[d3], %[p1], off offset:512\n\t"
                "global_load_dwordx4 %[d4], %[p0], off offset:1024\n\t"
                "global_load_dwordx4 %[d5], %[p1], off offset:1024\n\t"
                "global_load_dwordx4 %[d6], %[p0], off offset:1536\n\t"
                "global_load_dwordx4 %[d7], %[p1], off offset:1536"
                : [d0] "+v"(dst[0][0]), [d1] "+v"(dst[0][1]), [d2] "+v"(dst[1][0]), [d3] "+v"(dst[1][1]),
                  [d4] "+v"(dst[2][0]), [d5] "+v"(dst[2][1]), [d6] "+v"(dst[3][0]), [d7] "+v"(dst[3][1])
                : [p0] "v"(p0), [p1] "v"(p1));
        else
        asm volatile(
            "s_cmp_eq_u32 %[pat], 0\n\t"
            "s_cbranch_scc1 .Lsc_skipw_%=\n\t"
            "global_load_dwordx4 %[d0], %[p0], off\n\t"
            "global_load_dwordx4 %[d1], %[p1], off\n\t"
            "global_load_dwordx4 %[d2], %[p0], off offset:512\n\t"
            "global_load_dwordx4 %[d3], %[p1], off offset:512\n\t"
            "global_load_dwordx4 %[d4], %[p0], off offset:1024\n\t"
            "global_load_dwordx4 %[d5], %[p1], off offset:1024\n\t"
            "global_load_dwordx4 %[d6], %[p0], off offset:1536\n\t"
            "global_load_dwordx4 %[d7], %[p1], off offset:1536\n"
            ".Lsc_skipw_%=:"
            : [d0] "+v"(dst[0][0]), [d1] "+v"(dst[0][1]), [d2] "+v"(dst[1][0]), [d3] "+v"(dst[1][1]),
              [d4] "+v"(dst[2][0]), [d5] "+v"(dst[2][1]), [d6] "+v"(dst[3][0]), [d7] "+v"(dst[3][1])
            : [p0] "v"(p0), [p1] "v"(p1), [pat] "s"(pat)
            : "scc");
    };
    // wait until at most 4 n loads are outstanding (n: halves fetched by the step before)
    auto wait_younger = [&](uint32_t n) {
        if (!SKIP || n == 2u) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        else if (n == 0u) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        else asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
    };
    // hand the registers of finished loads back to the compiler
    auto pin = [&](u32x4 (&slot)[2][4]) {
        asm volatile("" : "+v"(slot[0][0]), "+v"(slot[0][1]), "+v"(slot[0][2]), "+v"(slot[0][3]),
                          "+v"(slot[1][0]), "+v"(slot[1][1]), "+v"(slot[1][2]), "+v"(slot[1][3]));
    };
    auto pin_w = [&](u32x4 (&w)[4][MB]) {
        asm volatile("" : "+v"(w[0][0]), "+v"(w[0][1]), "+v"(w[1][0]), "+v"(w[1][1]),
                          "+v"(w[2][0]), "+v"(w[2][1]), "+v"(w[3][0]), "+v"(w[3][1]));
    };
    u32x4 fb[3][2][4], a[2][4][MB];
#pragma unroll
    for (int j = 0; j < 3; ++j)
#pragma unroll
        for (int g = 0; g < 2; ++g)
#pragma unroll
            for (int i = 0; i < 4; ++i) fb[j][g][i] = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int sl = 0; sl < 4; ++sl)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) a[j][sl][mb] = u32x4{0u, 0u, 0u, 0u};
    // before the loop: the weights of the first offset and the rows of the first three, all complete at its start
    load_weights(a[0], k0, pattern_at(k0));
    {
        const int kj[3] = {k0, k1, k2};
#pragma unroll
        for (int j = 0; j < 3; ++j) {
            uint32_t e[2][4], off[2][4];
            row_numbers(e, kj[j]);
            row_offsets(off, e);
            gather(fb[j], off, pattern_at(kj[j]));
        }
    }
    uint32_t e_next[2][4];               // row numbers of the offset the next step fetches
    row_numbers(e_next, k3);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int j = 0; j < 3; ++j) pin(fb[j]);
    pin_w(a[0]);
    f32x16 acc[2][MB];
#pragma unroll
    for (int g = 0; g < 2; ++g)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 16; ++j) acc[g][mb][j] = 0.f;
    // rows of the first offset: load layout -> operand layout through the staging area (one half after
    // the other through the same 4 KB: a wavefront's LDS operations execute in order)
    {
        const uint32_t pat0 = pattern_at(k0);
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            if ((pat0 >> g) & 1u) {
#pragma unroll
                for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(stage + st_w[i]) = fb[0][g][i];
#pragma unroll
                for (int sl = 0; sl < 4; ++sl) fb[0][g][sl] = *reinterpret_cast<const u32x4*>(stage + st_r[sl]);
            }
        }
    }
    SC_MARK(1);
    SC_MARK(2);

    // One step, for offset k0.  At its start the rows of k0 are in ring slot S in operand layout and
    // its weights are in a[AB] (possibly still on their way: the wait comes first); the rows of k1
    // are in slot S1 in load layout, those of k2 in flight.  Loads in issue order:
    // ... weights k0, rows k2 | weights k1, rows k3: what may stay in flight at the top of the step
    // are the rows of k2, four loads per half that takes part.  Then the weights of k1 are
    // requested, the multiplies of k0 are issued slice by slice with the staging of k1 between
    // them (half 0 is written in slice 0 and read back in slice 1, half 1 in slices 2 and 3), the
    // freed slot is refilled with the rows of k3, and the row numbers of k4 are read from LDS.
    auto step = [&](auto slot_c, auto ab_c) {
        constexpr int S = decltype(slot_c)::value, S1 = (S + 1) % 3, AB = decltype(ab_c)::value;
        const uint32_t pat = pattern_at(k0), pat1 = pattern_at(k1), pat3 = pattern_at(k3);
        wait_younger(halves_at(k2));
        // every LDS operation of the step before is complete from here on (staging reads, row
        // numbers): said in a form the compiler's wait-count pass sees, it places no LDS waits
        // between the multiplies below, where they would also wait for the staging of this step
        __builtin_amdgcn_s_waitcnt(0xc07f);      // lgkmcnt(0), the other counters left alone
        pin(fb[S1]);
        pin_w(a[AB]);
        load_weights(a[1 - AB], k1, pat1);
#pragma unroll
        for (int sl = 0; sl < 4; ++sl) {
#pragma unroll
            for (int g = 0; g < 2; ++g) {
                if ((pat >> g) & 1u) {
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) acc[g][mb] = mfma32x32x16<DT>(a[AB][sl][mb], fb[S][g][sl], acc[g][mb]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (g == 0) {
                    const int h = sl >> 1;          // the half whose staging falls into this slice
                    if ((pat1 >> h) & 1u) {
                        if ((sl & 1) == 0) {
#pragma unroll
                            for (int i = 0; i < 4; ++i) *reinterpret_cast<u32x4*>(stage + st_w[i]) = fb[S1][h][i];
                        } else {
#pragma unroll
                            for (int i = 0; i < 4; ++i) fb[S1][h][i] = *reinterpret_cast<const u32x4*>(stage + st_r[i]);
                        }
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        uint32_t off[2][4];
        row_offsets(off, e_next);
        gather(fb[S], off, pat3);
        row_numbers(e_next, k4);        // on their way while the next step starts
        k0 = k1; k1 = k2; k2 = k3; k3 = k4;
        k4 = next_offset();
    };
    // six steps per trip, so that ring slots (three) and weight registers (two sets) are constants;
    // steps past the last offset find K3 everywhere and do nothing
#pragma unroll 1
    for (int i = 0; i < n_steps; i += 6) {
        step(IntC<0>{}, IntC<0>{});
        step(IntC<1>{}, IntC<1>{});
        step(IntC<2>{}, IntC<0>{});
        step(IntC<0>{}, IntC<1>{});
        step(IntC<1>{}, IntC<0>{});
        step(IntC<2>{}, IntC<1>{});
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");      // nothing of the loop's loads is left in flight
    SC_MARK(3);
    // the accumulator block of a lane: output row lane % 32 of the half, channels
    // 32 mb + 8 q + 4 (lane / 32) .. + 3 for q = 0..3
    if (tile_ok) {
#pragma unroll
        for (int g = 0; g < 2; ++g) {
            const int64_t row = tile * TILE + g * 32 + r32;
            if (row < n_out) {
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        store_acc<DT>(out, out_f32, row, C_out, mb * 32 + 8 * q + 4 * hh,
                                      f32x4{acc[g][mb][4 * q], acc[g][mb][4 * q + 1], acc[g][mb][4 * q + 2], acc[g][mb][4 * q + 3]});
            }
        }
    }
    SC_MARK(4);
    SC_MARK(5);
}

// ---- any shape: weights read from global memory, offsets walked by mask bit --------------------
// One wavefront per 16 output rows, one tile per workgroup.  C_in = 32*KS (KS <= 8),
// C_out = 16*CB (CB <= 16), any K3 <= 343.
constexpr int KS_MAX = 8, CB_MAX = 16;
template <int DT>
__global__ void __launch_bounds__(256)
k_conv_rows16_any(const uint16_t* __restrict__ feat, const uint4* __restrict__ wp, void* __restrict__ out,
                  int out_f32, const uint32_t* __restrict__ gmask, const int32_t* __restrict__ nbr, int K3, int mw,
                  int KS, int CB, const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    const int C_in = KS * 32, C_out = CB * 16;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int r = lane & 15, qq = lane >> 4;
    const int64_t tile = blockIdx.x;
    int64_t n_out = *n_out_ptr;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row = tile * TILE + q * 16 + r;
    if (tile * TILE + q * 16 >= n_out) return;                       // uniform per wavefront

    f32x4 acc[CB_MAX];
#pragma unroll
    for (int cb = 0; cb < CB_MAX; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int32_t* line = nbr + tile * (int64_t)K3 * TILE + q * 16 + r;
    for (int wi = 0; wi < mw; ++wi) {
        uint32_t m = gmask[(tile * 4 + q) * mw + wi];
        while (m) {
            const int k = wi * 32 + __builtin_ctz(m);
            m &= m - 1;
            const int32_t e = line[(int64_t)k * TILE];
            uint4 fb[KS_MAX];
            const uint4* frow = reinterpret_cast<const uint4*>(feat + (int64_t)(e < 0 ? 0 : e) * C_in) + qq;
#pragma unroll
            for (int ks = 0; ks < KS_MAX; ++ks)
                if (ks < KS) fb[ks] = e >= 0 ? frow[ks * 4] : make_uint4(0, 0, 0, 0);
            const uint4* wk = wp + (int64_t)k * CB * KS * 64 + lane;
#pragma unroll
            for (int cb = 0; cb < CB_MAX; ++cb) {
                if (cb < CB) {
#pragma unroll
                    for (int ks = 0; ks < KS_MAX; ++ks)
                        if (ks < KS) acc[cb] = mfma16x16x32<DT>(wk[wtile(KS, CB, cb, ks) * 64], fb[ks], acc[cb]);
                }
            }
        }
    }
    if (row < n_out) {
#pragma unroll
        for (int cb = 0; cb < CB_MAX; ++cb)
            if (cb < CB) store_acc<DT>(out, out_f32, row, C_out, cb * 16 + qq * 4, acc[cb]);
    }
}

// ---- fp32 features and weights -------------------------------------------------------------------
// Same scheme with the fp32 matrix instruction (v_mfma_f32_16x16x4_f32: true fp32 products and
// sums): one wavefront per 16 output rows, offsets walked by mask bit, operands read straight from
// the [K3][C_in][C_out] weights and the feature rows, four input channels per step.  Any C_in,
// C_out <= 256 (edges are zero-filled).
__global__ void __launch_bounds__(256)
k_conv_f32(const float* __restrict__ feat, const float* __restrict__ w, float* __restrict__ out,
           const uint32_t* __restrict__ gmask, const int32_t* __restrict__ nbr, int K3, int mw, int C_in, int C_out,
           const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int r = lane & 15, qq = lane >> 4;
    const int CB = (C_out + 15) / 16;
    const int64_t tile = blockIdx.x;
    int64_t n_out = *n_out_ptr;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row = tile * TILE + q * 16 + r;
    if (tile * TILE + q * 16 >= n_out) return;                       // uniform per wavefront

    f32x4 acc[CB_MAX];
#pragma unroll
    for (int cb = 0; cb < CB_MAX; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int32_t* line = nbr + tile * (int64_t)K3 * TILE + q * 16 + r;
    for (int wi = 0; wi < mw; ++wi) {
        uint32_t m = gmask[(tile * 4 + q) * mw + wi];
        while (m) {
            const int k = wi * 32 + __builtin_ctz(m);
            m &= m - 1;
            const int32_t e = line[(int64_t)k * TILE];
            const float* frow = feat + (int64_t)(e < 0 ? 0 : e) * C_in;
            const float* wk = w + (int64_t)k * C_in * C_out;
            for (int ci0 = 0; ci0 < C_in; ci0 += 4) {
                const int ci = ci0 + qq;
                const bool ci_ok = ci < C_in;
                const float b = (e >= 0 && ci_ok) ? frow[ci] : 0.f;
#pragma unroll
                for (int cb = 0; cb < CB_MAX; ++cb) {
                    if (cb < CB) {
                        const int co = cb * 16 + r;
                        const float a = (ci_ok && co < C_out) ? wk[(int64_t)ci * C_out + co] : 0.f;
                        acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc[cb], 0, 0, 0);
                    }
                }
            }
        }
    }
    if (row < n_out) {
        float* orow = out + row * C_out;
#pragma unroll
        for (int cb = 0; cb < CB_MAX; ++cb) {
            if (cb < CB) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int co = cb * 16 + qq * 4 + i;
                    if (co < C_out) orow[co] = acc[cb][i];
                }
            }
        }
    }
}

// fp32 layers with few channels (C_in = 16*CI16 <= 64, C_out = 16*CB <= 64, K^3 <= 32): the same
// instruction, loads batched.  A lane reads 16 bytes (4 channels) of its row per 16-channel chunk
// and feeds component j to the j-th of four multiplies, so input channel 16c + 4q + j sits at
// position q of multiply (c, j); the weight operand is read to match.  The offsets that exist are
// taken four at a time: their four table entries are in flight together, then all their feature
// loads, so a group costs two dependent round trips per batch instead of two per offset.
template <int CI16, int CB>
__global__ void __launch_bounds__(256)
k_conv_f32_small(const float* __restrict__ feat, const float* __restrict__ w, float* __restrict__ out,
                 const uint32_t* __restrict__ gmask, const int32_t* __restrict__ nbr, int K3,
                 const int64_t* __restrict__ n_out_ptr, int64_t n_out_cap) {
    constexpr int C_in = 16 * CI16, C_out = 16 * CB, NB = 4;
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int r = lane & 15, qq = lane >> 4;
    const int64_t tile = blockIdx.x;
    int64_t n_out = *n_out_ptr;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row = tile * TILE + q * 16 + r;
    if (tile * TILE + q * 16 >= n_out) return;                       // uniform per wavefront

    f32x4 acc[CB];
#pragma unroll
    for (int cb = 0; cb < CB; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int32_t* line = nbr + tile * (int64_t)K3 * TILE + q * 16 + r;
    uint32_t m = __builtin_amdgcn_readfirstlane(gmask[tile * 4 + q]);
    while (m) {
        int kk[NB];
        int32_t e[NB];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            kk[j] = m ? __builtin_ctz(m) : -1;
            if (m) m &= m - 1;
            e[j] = kk[j] >= 0 ? line[kk[j] * TILE] : -1;
        }
        float4 f[NB][CI16];
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            const float4* frow = reinterpret_cast<const float4*>(feat + (int64_t)(e[j] < 0 ? 0 : e[j]) * C_in) + qq;
#pragma unroll
            for (int c = 0; c < CI16; ++c) f[j][c] = e[j] >= 0 ? frow[c * 4] : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int j = 0; j < NB; ++j) {
            if (kk[j] >= 0) {                                        // uniform
                const float* wk = w + (int64_t)kk[j] * C_in * C_out + r;
#pragma unroll
                for (int c = 0; c < CI16; ++c) {
                    const float b[4] = {f[j][c].x, f[j][c].y, f[j][c].z, f[j][c].w};
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const float* wrow = wk + (int64_t)(c * 16 + 4 * qq + t) * C_out;
#pragma unroll
                        for (int cb = 0; cb < CB; ++cb)
                            acc[cb] = __builtin_amdgcn_mfma_f32_16x16x4f32(wrow[cb * 16], b[t], acc[cb], 0, 0, 0);
                    }
                }
            }
        }
    }
    if (row < n_out) {
        float* orow = out + row * C_out;
#pragma unroll
        for (int cb = 0; cb < CB; ++cb)
            *reinterpret_cast<float4*>(orow + cb * 16 + qq * 4) = make_float4(acc[cb][0], acc[cb][1], acc[cb][2], acc[cb][3]);
    }
}

// Large dynamic LDS has to be allowed per kernel, once on every device the kernel runs on: a flag
// per device (a repeated call would be harmless, so a race between host threads is too).
constexpr int MAX_DEVICES = 64;
static int allow_lds(const void* fn, size_t lds, bool (&done)[MAX_DEVICES]) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return SC_EHIP;
    if (!done[dev]) {
        if (hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SC_EHIP;
        done[dev] = true;
    }
    return SC_OK;
}

template <int DT, int K3, int KS, int CB, int NT, int FUSED, int UP = 0, int WPACKED = 0>
static int launch_rows16(int64_t tiles, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out, int out_f32,
                         const MapSource& ms, const int64_t* counts, int64_t n_out_cap) {
    auto fn = k_conv_rows16<DT, K3, KS, CB, NT, FUSED, UP, WPACKED>;
    const size_t lds = (size_t)K3 * CB * KS * 64 * sizeof(uint4);
    static bool allowed[MAX_DEVICES] = {};  // per instantiation
    if (int rc = allow_lds((const void*)fn, lds, allowed)) return rc;
    const dim3 grid(xcd_grid((tiles + NT - 1) / NT));
    SC_LAUNCH(KID_CONV_MFMA, fn, grid, dim3(256 * NT), lds, s, feat, wp, out, out_f32, ms, counts, n_out_cap);
    return SC_OK;
}

// Shapes whose packed weights fit in LDS as a whole.  The resident kernel's LDS layout of the
// weights is the packed layout itself (tile (k, cb, ks) at ((k CB + cb) KS + ks): one 64-channel
// half at most), so packed weights are copied and raw ones re-laid out on the way in.
static bool resident_shape(int K3, int C_in, int C_out, bool fused) {
    if (K3 == 27 && C_in == 32 && C_out == 32) return true;
    if (fused) return false;
    return K3 == 8 && ((C_in == 32 && C_out == 64) || (C_in == 32 && C_out == 32) || (C_in == 64 && C_out == 64) ||
                       (C_in == 64 && C_out == 32));
}
template <int DT, int FUSED, int WPACKED>
static int launch_resident(int K3, int C_in, int C_out, int64_t tiles, hipStream_t s, const uint16_t* feat,
                           const uint4* wp, void* out, int out_f32, const MapSource& ms, const int64_t* counts,
                           int64_t n_out_cap, bool* handled) {
    *handled = true;
#define SC_ROWS16(K3V, KSV, CBV, NTV) \
    return launch_rows16<DT, K3V, KSV, CBV, NTV, FUSED, 0, WPACKED>(tiles, s, feat, wp, out, out_f32, ms, counts, n_out_cap)
    // four tiles per workgroup once every CU still gets a workgroup: the weights are re-laid out
    // half as often and no CU hosts two workgroups while another hosts one (cfg2: 11.9 -> 10.6 us)
    if (K3 == 27 && C_in == 32 && C_out == 32 && tiles >= 512) SC_ROWS16(27, 1, 2, 4);
    if (K3 == 27 && C_in == 32 && C_out == 32) SC_ROWS16(27, 1, 2, 2);
    if constexpr (!FUSED) {
        if (K3 == 8 && C_in == 32 && C_out == 64) SC_ROWS16(8, 1, 4, 2);
        if (K3 == 8 && C_in == 32 && C_out == 32) SC_ROWS16(8, 1, 2, 2);
        if (K3 == 8 && C_in == 64 && C_out == 64) SC_ROWS16(8, 2, 4, 2);
        if (K3 == 8 && C_in == 64 && C_out == 32) SC_ROWS16(8, 2, 2, 2);      // the up-sampling twin of 32 -> 64
    }
#undef SC_ROWS16
    *handled = false;
    return SC_OK;
}

template <int DT, int K3, int KS, int CB, int NWV, int D, int FUSED>
static int launch_stream(int64_t tiles, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out, int out_f32,
                         const MapSource& ms, const int64_t* counts, int64_t n_out_cap) {
    auto fn = k_conv_stream<DT, K3, KS, CB, NWV, D, FUSED>;
    const size_t lds = (size_t)2 * CB * KS * 64 * sizeof(uint4) +
                       (size_t)NWV * K3 * TILE * sizeof(int32_t);
    static bool allowed[MAX_DEVICES] = {};
    if (int rc = allow_lds((const void*)fn, lds, allowed)) return rc;
    SC_LAUNCH(KID_CONV_MFMA, fn, dim3(xcd_grid((tiles + NWV - 1) / NWV)), dim3(64 * NWV), lds, s, feat, wp, out, out_f32,
              ms, counts, n_out_cap);
    return SC_OK;
}

// Tiles per workgroup for k_conv_direct64: its wavefronts are independent, so any count up to 8
// (two wavefronts per SIMD at its register use) works; the workgroups should land on the CUs evenly.
// Up to 8 tiles per CU: one workgroup per CU with ceil(tiles / CUs) wavefronts (measured on ~110 k
// voxels: 31.4 us with 7, 33.3 with 8, 35.1 with 4); beyond that, four (261 k voxels: 62.6 us
// with 4, 64.0 with 8, 78.1 with 7).
static int direct_tiles_per_workgroup(int64_t tiles, int* cu_count_out) {
    static int cu_count[MAX_DEVICES] = {};      // per device, asked once (a race between host threads stores the same value)
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess && dev >= 0 && dev < MAX_DEVICES) {
        if (cu_count[dev] == 0) {
            int n = 0;
            cu_count[dev] = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0 ? n : 256;
        }
        cus = cu_count[dev];
    }
    *cu_count_out = cus;
    if (tiles > (int64_t)cus * 8) return 4;
    const int64_t per_cu = (tiles + cus - 1) / cus;
    return per_cu < 1 ? 1 : (int)per_cu;
}
// SKIP = 1: halves of a tile without a neighbour at an offset are skipped together with their loads
// (tests and branches in every step); SKIP = 0: a step is one straight line of code that treats
// them as rows of zeros (about a sixth more loads, staging and multiplies on surface-like sets,
// half the instructions).  The straight line wins while a CU has few wavefronts and the time is
// one wavefront's walk over its offsets (14 k voxels: 15.2 against 19.2 us, 55 k: 20.8 against
// 22.8), the skipping form once the CUs are full (110 k: 32.1 against 35.7, 261 k: 63.9 against 68.7).
template <int DT, int K3, int FUSED, int SKIP>
static int launch_direct64_as(int64_t tiles, int nwv, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out,
                              int out_f32, const MapSource& ms, const int64_t* counts, int64_t n_out_cap) {
    auto fn = k_conv_direct64<DT, K3, FUSED, SKIP>;
    const size_t per_wave = DIRECT_STAGE + DIRECT_LINES(K3) * TILE * sizeof(int32_t);
    static bool allowed[MAX_DEVICES] = {};
    if (int rc = allow_lds((const void*)fn, 8 * per_wave, allowed)) return rc;
    SC_LAUNCH(KID_CONV_MFMA, fn, dim3(xcd_grid((tiles + nwv - 1) / nwv)), dim3(64 * nwv), nwv * per_wave, s, feat, wp, out,
              out_f32, ms, counts, n_out_cap);
    return SC_OK;
}
template <int DT, int K3, int FUSED>
static int launch_direct64(int64_t tiles, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out, int out_f32,
                           const MapSource& ms, const int64_t* counts, int64_t n_out_cap) {
    int cus = 256;
    const int nwv = direct_tiles_per_workgroup(tiles, &cus);
    if (tiles <= (int64_t)cus * 4)
        return launch_direct64_as<DT, K3, FUSED, 0>(tiles, nwv, s, feat, wp, out, out_f32, ms, counts, n_out_cap);
    return launch_direct64_as<DT, K3, FUSED, 1>(tiles, nwv, s, feat, wp, out, out_f32, ms, counts, n_out_cap);
}

// Up-sampling straight from the strided layer's map: shapes with a dedicated kernel.
template <int DT>
static int launch_up(int K3, int C_in, int C_out, int64_t tiles, hipStream_t s, const uint16_t* feat, const uint4* wp,
                     void* out, int out_f32, const MapSource& ms, const int64_t* counts, int64_t n_out_cap,
                     bool* handled) {
    *handled = true;
#define SC_UP16(K3V, KSV, CBV) \
    return launch_rows16<DT, K3V, KSV, CBV, 2, 0, 1>(tiles, s, feat, wp, out, out_f32, ms, counts, n_out_cap)
    if (K3 == 8 && C_in == 64 && C_out == 32) SC_UP16(8, 2, 2);
    if (K3 == 8 && C_in == 32 && C_out == 32) SC_UP16(8, 1, 2);
    if (K3 == 8 && C_in == 64 && C_out == 64) SC_UP16(8, 2, 4);
    if (K3 == 8 && C_in == 128 && C_out == 64) SC_UP16(8, 4, 4);
    if (K3 == 27 && C_in == 32 && C_out == 32) SC_UP16(27, 1, 2);
#undef SC_UP16
    *handled = false;
    return SC_OK;
}

// Shapes with a streaming kernel.
template <int DT, int FUSED>
static int launch_streamed(int K3, int C_in, int C_out, int64_t tiles, hipStream_t s, const uint16_t* feat,
                           const uint4* wp, void* out, int out_f32, const MapSource& ms, const int64_t* counts,
                           int64_t n_out_cap, bool feat_small, bool* handled) {
    *handled = true;
    // 64 input channels: the kernel with 32-bit buffer offsets where the feature array allows it
    if (K3 == 27 && C_in == 64 && C_out == 64 && feat_small)
        return launch_direct64<DT, 27, FUSED>(tiles, s, feat, wp, out, out_f32, ms, counts, n_out_cap);
#define SC_STREAM(K3V, KSV, CBV, NWV, DV) \
    return launch_stream<DT, K3V, KSV, CBV, NWV, DV, FUSED>(tiles, s, feat, wp, out, out_f32, ms, counts, n_out_cap)
    if (K3 == 27 && C_in == 64 && C_out == 64) SC_STREAM(27, 2, 4, 4, 3);       // feature arrays of 4 GiB and more
    if (K3 == 27 && C_in == 128 && C_out == 128) SC_STREAM(27, 4, 8, 8, 1);
    if (K3 == 27 && C_in == 32 && C_out == 64) SC_STREAM(27, 1, 4, 4, 3);
    if (K3 == 27 && C_in == 64 && C_out == 128) SC_STREAM(27, 2, 8, 4, 2);
    if constexpr (!FUSED) {
        if (K3 == 8 && C_in == 64 && C_out == 128) SC_STREAM(8, 2, 8, 4, 2);
        if (K3 == 8 && C_in == 128 && C_out == 128) SC_STREAM(8, 4, 8, 8, 1);
    }
#undef SC_STREAM
    *handled = false;
    return SC_OK;
}

static bool mfma_channels_ok(int C_in, int C_out) {
    return (C_in == 32 || C_in == 64 || C_in == 128 || C_in == 256) && C_out >= 16 && C_out <= 256 && C_out % 16 == 0;
}

// Packed form of 16-bit weights [K3][C_in][C_out] for sc_conv_fwd's kernels (operand tiles, see k_weight_pack).
static int pack_weights(int K3, int C_in, int C_out, const void* d_weight, void* d_packed, hipStream_t s) {
    const int64_t pack_threads = (int64_t)K3 * (C_out / 16) * (C_in / 32) * 64;
    SC_LAUNCH(KID_WEIGHT_PACK, k_weight_pack, dim3((unsigned)((pack_threads + 255) / 256)), dim3(256), 0, s,
              (const uint16_t*)d_weight, (uint4*)d_packed, K3, C_in, C_out);
    return SC_OK;
}

// A 16-bit layer.  `packed`: d_weight is what sc_conv_weight_pack made; otherwise the raw weights,
// which the resident kernels re-lay out themselves and the others have packed into the workspace
// first.  FUSED (dense table, no map) always takes raw weights.
template <int FUSED>
static int conv_16bit(int dtype_in, int K3, int mw, int C_in, int C_out, int64_t tiles, hipStream_t s, const void* d_feat_in,
                      const void* d_weight, bool packed, void* d_workspace, void* d_feat_out,
                      int out_f32, const MapSource& ms, const int64_t* n_out_ptr, int64_t n_out_cap, int64_t feat_rows) {
    const uint16_t* feat = (const uint16_t*)d_feat_in;
    bool handled = false;
    int rc;
    if (resident_shape(K3, C_in, C_out, FUSED)) {
        if (packed)
            rc = dtype_in == SC_F16 ? launch_resident<SC_F16, FUSED, 1>(K3, C_in, C_out, tiles, s, feat, (const uint4*)d_weight,
                                                                       d_feat_out, out_f32, ms, n_out_ptr, n_out_cap, &handled)
                                    : launch_resident<SC_BF16, FUSED, 1>(K3, C_in, C_out, tiles, s, feat, (const uint4*)d_weight,
                                                                        d_feat_out, out_f32, ms, n_out_ptr, n_out_cap, &handled);
        else
            rc = dtype_in == SC_F16 ? launch_resident<SC_F16, FUSED, 0>(K3, C_in, C_out, tiles, s, feat, (const uint4*)d_weight,
                                                                       d_feat_out, out_f32, ms, n_out_ptr, n_out_cap, &handled)
                                    : launch_resident<SC_BF16, FUSED, 0>(K3, C_in, C_out, tiles, s, feat, (const uint4*)d_weight,
                                                                        d_feat_out, out_f32, ms, n_out_ptr, n_out_cap, &handled);
        return rc;
    }
    const bool stream_shape = (K3 == 27 && ((C_in == 64 && C_out == 64) || (C_in == 128 && C_out == 128) ||
                                            (C_in == 32 && C_out == 64) || (C_in == 64 && C_out == 128))) ||
                              (!FUSED && K3 == 8 && ((C_in == 64 && C_out == 128) || (C_in == 128 && C_out == 128)));
    if (FUSED && !stream_shape) return SC_EINVAL;     // no fused kernel for this shape: use the three calls
    const uint4* wp = (const uint4*)d_weight;
    if (!packed) {
        if (int prc = pack_weights(K3, C_in, C_out, d_weight, d_workspace, s)) return prc;
        wp = (const uint4*)d_workspace;
    }
    // rows that a 32-bit byte offset can address, with room for the "no neighbour" offsets above them
    const bool feat_small = feat_rows * (int64_t)C_in * 2 < 0xFFFFFF80ll;
    rc = dtype_in == SC_F16 ? launch_streamed<SC_F16, FUSED>(K3, C_in, C_out, tiles, s, feat, wp, d_feat_out, out_f32, ms,
                                                            n_out_ptr, n_out_cap, feat_small, &handled)
                            : launch_streamed<SC_BF16, FUSED>(K3, C_in, C_out, tiles, s, feat, wp, d_feat_out, out_f32, ms,
                                                             n_out_ptr, n_out_cap, feat_small, &handled);
    if (handled || rc != SC_OK) return rc;
    if (FUSED) return SC_EINVAL;
    if (dtype_in == SC_F16)
        SC_LAUNCH(KID_CONV_MFMA, k_conv_rows16_any<SC_F16>, dim3((unsigned)tiles), dim3(256), 0, s, feat, wp, d_feat_out, out_f32,
                  ms.gmask, ms.nbr, K3, mw, C_in / 32, C_out / 16, n_out_ptr, n_out_cap);
    else
        SC_LAUNCH(KID_CONV_MFMA, k_conv_rows16_any<SC_BF16>, dim3((unsigned)tiles), dim3(256), 0, s, feat, wp, d_feat_out, out_f32,
                  ms.gmask, ms.nbr, K3, mw, C_in / 32, C_out / 16, n_out_ptr, n_out_cap);
    return SC_OK;
}

}  // namespace sc

using namespace sc;

extern "C" size_t sc_conv_workspace_bytes(int K, int C_in, int C_out, int dtype_in) {
    if (K < 1 || K > SC_K_MAX || C_in < 1 || C_out < 1) return 0;
    if (dtype_in == SC_F32) return 0;
    return align_up((size_t)K * K * K * C_in * C_out * 2, 256);
}

static int conv_fwd(const void* d_feat_in, int64_t n_map, const void* d_weight, bool packed, void* d_feat_out,
                    int64_t n_out_cap, const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts, int K, int stride,
                    int mode, int C_in, int C_out, int dtype_in, int dtype_out, void* d_workspace, size_t workspace_bytes,
                    void* stream) {
    if (n_map < 0 || n_map > SC_N_MAX || n_out_cap < 0 || K < 1 || K > SC_K_MAX || C_in < 1 || C_out < 1) return SC_EINVAL;
    if (d_weight == nullptr || d_kmap == nullptr || d_counts == nullptr) return SC_EINVAL;
    if ((n_map > 0 && d_feat_in == nullptr) || (n_out_cap > 0 && d_feat_out == nullptr)) return SC_EINVAL;
    if (!aligned16(d_feat_in) || !aligned16(d_weight) || !aligned16(d_feat_out) || !aligned16(d_kmap) ||
        !aligned16(d_counts) || !aligned16(d_workspace))
        return SC_EINVAL;
    if (dtype_in != SC_F32 && dtype_in != SC_F16 && dtype_in != SC_BF16) return SC_EINVAL;
    if (dtype_out != SC_F32 && dtype_out != dtype_in) return SC_EINVAL;
    const int64_t bound = sc_out_bound(n_map, K, stride, mode);
    if (bound < 0) return SC_EINVAL;
    if (kmap_bytes < sc_kmap_bytes(n_map, K, stride, mode)) return SC_ECAP;
    // rows of the output: what the map build counted, or (inverse layers) the rows it was built from
    const int64_t* n_out_ptr = mode == SC_INVERSE ? &d_counts->n_in : &d_counts->n_out;
    const KmapLayout L = kmap_layout(bound, K);
    int64_t tiles = (n_out_cap + TILE - 1) / TILE;
    if (tiles > L.tiles) tiles = L.tiles;
    if (tiles == 0) return SC_OK;
    const uint32_t* gmask = (const uint32_t*)((const char*)d_kmap + L.off_mask);
    const int32_t* nbr = (const int32_t*)((const char*)d_kmap + L.off_nbr);
    hipStream_t s = (hipStream_t)stream;

    if (dtype_in == SC_F32) {           // fp32 weights are used as they are: packed == raw
        if (C_out > 256) return SC_EINVAL;
        if (L.K3 <= 32 && C_in % 16 == 0 && C_in <= 64 && C_out % 16 == 0 && C_out <= 64) {
#define SC_F32_SMALL(CI, CBV)                                                                                         \
    if (C_in == 16 * CI && C_out == 16 * CBV) {                                                                       \
        SC_LAUNCH(KID_CONV_F32, (k_conv_f32_small<CI, CBV>), dim3((unsigned)tiles), dim3(256), 0, s,                  \
                  (const float*)d_feat_in, (const float*)d_weight, (float*)d_feat_out, gmask, nbr, L.K3, n_out_ptr,   \
                  n_out_cap);                                                                                         \
        return SC_OK;                                                                                                 \
    }
            SC_F32_SMALL(1, 1) SC_F32_SMALL(1, 2) SC_F32_SMALL(2, 1) SC_F32_SMALL(2, 2) SC_F32_SMALL(2, 4)
            SC_F32_SMALL(4, 2) SC_F32_SMALL(4, 4)
#undef SC_F32_SMALL
        }
        SC_LAUNCH(KID_CONV_F32, k_conv_f32, dim3((unsigned)tiles), dim3(256), 0, s, (const float*)d_feat_in,
                  (const float*)d_weight, (float*)d_feat_out, gmask, nbr, L.K3, L.mw, C_in, C_out, n_out_ptr,
                  n_out_cap);
        return SC_OK;
    }

    if (!mfma_channels_ok(C_in, C_out)) return SC_EINVAL;
    if (!packed) {
        const size_t need = sc_conv_workspace_bytes(K, C_in, C_out, dtype_in);
        if (d_workspace == nullptr || workspace_bytes < need) return SC_ECAP;
    }
    const MapSource ms{gmask, nbr, nullptr, nullptr, GridDims{0, 0, 0, 0}, 0u};
    // rows of the input feature array: the map's inputs, or (inverse layers) at most the strided map's bound
    const int64_t feat_rows = n_map > bound ? n_map : bound;
    return conv_16bit<0>(dtype_in, L.K3, L.mw, C_in, C_out, tiles, s, d_feat_in, d_weight, packed, d_workspace,
                         d_feat_out, dtype_out == SC_F32, ms, n_out_ptr, n_out_cap, feat_rows);
}

extern "C" int sc_conv_fwd(const void* d_feat_in, int64_t n_map, const void* d_weight, void* d_feat_out,
                           int64_t n_out_cap, const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts, int K,
                           int stride, int mode, int C_in, int C_out, int dtype_in, int dtype_out, void* d_workspace,
                           size_t workspace_bytes, void* stream) {
    return conv_fwd(d_feat_in, n_map, d_weight, false, d_feat_out, n_out_cap, d_kmap, kmap_bytes, d_counts, K, stride, mode,
                    C_in, C_out, dtype_in, dtype_out, d_workspace, workspace_bytes, stream);
}

extern "C" int sc_conv_fwd_packed(const void* d_feat_in, int64_t n_map, const void* d_packed, void* d_feat_out,
                                  int64_t n_out_cap, const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts,
                                  int K, int stride, int mode, int C_in, int C_out, int dtype_in, int dtype_out,
                                  void* stream) {
    return conv_fwd(d_feat_in, n_map, d_packed, true, d_feat_out, n_out_cap, d_kmap, kmap_bytes, d_counts, K, stride, mode,
                    C_in, C_out, dtype_in, dtype_out, nullptr, 0, stream);
}

extern "C" size_t sc_conv_packed_bytes(int K, int C_in, int C_out, int dtype_in) {
    if (K < 1 || K > SC_K_MAX || C_in < 1 || C_out < 1) return 0;
    if (dtype_in == SC_F32) return align_up((size_t)K * K * K * C_in * C_out * 4, 256);
    if (dtype_in != SC_F16 && dtype_in != SC_BF16) return 0;
    return align_up((size_t)K * K * K * C_in * C_out * 2, 256);
}

extern "C" int sc_conv_weight_pack(const void* d_weight, int K, int C_in, int C_out, int dtype_in, void* d_packed,
                                   size_t packed_bytes, void* stream) {
    const size_t need = sc_conv_packed_bytes(K, C_in, C_out, dtype_in);
    if (need == 0 || d_weight == nullptr || d_packed == nullptr || !aligned16(d_weight) || !aligned16(d_packed))
        return SC_EINVAL;
    if (packed_bytes < need) return SC_ECAP;
    hipStream_t s = (hipStream_t)stream;
    const int K3 = K * K * K;
    if (dtype_in == SC_F32) {
        if (C_out > 256) return SC_EINVAL;
        return hipMemcpyAsync(d_packed, d_weight, (size_t)K3 * C_in * C_out * 4, hipMemcpyDeviceToDevice, s) == hipSuccess
                   ? SC_OK : SC_EHIP;
    }
    if (!mfma_channels_ok(C_in, C_out)) return SC_EINVAL;
    return pack_weights(K3, C_in, C_out, d_weight, d_packed, s);
}

extern "C" int sc_conv_up_fwd(const void* d_feat_coarse, int64_t n_map, const void* d_weight, void* d_feat_fine,
                              const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts, int K, int C_in,
                              int C_out, int dtype_in, int dtype_out, void* stream) {
    if (n_map < 0 || n_map > SC_N_MAX || K < 2 || K > 4 || C_in < 1 || C_out < 1) return SC_EINVAL;
    if (d_weight == nullptr || d_kmap == nullptr || d_counts == nullptr) return SC_EINVAL;
    if (n_map > 0 && (d_feat_coarse == nullptr || d_feat_fine == nullptr)) return SC_EINVAL;
    if (!aligned16(d_feat_coarse) || !aligned16(d_weight) || !aligned16(d_feat_fine) || !aligned16(d_kmap) ||
        !aligned16(d_counts))
        return SC_EINVAL;
    if (dtype_in != SC_F16 && dtype_in != SC_BF16) return SC_EINVAL;
    if (dtype_out != SC_F32 && dtype_out != dtype_in) return SC_EINVAL;
    if (kmap_bytes < sc_kmap_bytes(n_map, K, K, SC_STRIDED)) return SC_ECAP;
    const KmapLayout L = kmap_layout(sc_out_bound(n_map, K, K, SC_STRIDED), K);
    if (L.tiles == 0) return SC_OK;
    MapSource ms{};
    ms.gmask = (const uint32_t*)((const char*)d_kmap + L.off_mask);
    ms.nbr = (const int32_t*)((const char*)d_kmap + L.off_nbr);
    bool handled = false;
    // the kernel walks the coarse rows: counts->n_out of them, at most the map's bound
    const int rc = dtype_in == SC_F16
                       ? launch_up<SC_F16>(L.K3, C_in, C_out, L.tiles, (hipStream_t)stream, (const uint16_t*)d_feat_coarse,
                                           (const uint4*)d_weight, d_feat_fine, dtype_out == SC_F32 ? 1 : 0, ms,
                                           &d_counts->n_out, n_map, &handled)
                       : launch_up<SC_BF16>(L.K3, C_in, C_out, L.tiles, (hipStream_t)stream, (const uint16_t*)d_feat_coarse,
                                            (const uint4*)d_weight, d_feat_fine, dtype_out == SC_F32 ? 1 : 0, ms,
                                            &d_counts->n_out, n_map, &handled);
    if (rc != SC_OK) return rc;
    return handled ? SC_OK : SC_EINVAL;
}

extern "C" int sc_conv_fwd_grid(const void* d_feat_in, const int32_t* d_coords, int64_t n, const void* d_grid,
                                size_t grid_bytes, int32_t B, int32_t X, int32_t Y, int32_t Z, uint32_t epoch,
                                const void* d_weight, void* d_feat_out, int K, int C_in, int C_out, int dtype_in,
                                int dtype_out, void* d_workspace, size_t workspace_bytes, void* stream) {
    const size_t gneed = sc_grid_bytes(B, X, Y, Z);
    if (gneed == 0 || n < 0 || n > SC_N_MAX || epoch == 0 || K != 3) return SC_EINVAL;
    if (d_weight == nullptr || d_grid == nullptr) return SC_EINVAL;
    if (n > 0 && (d_feat_in == nullptr || d_feat_out == nullptr || d_coords == nullptr)) return SC_EINVAL;
    if (!aligned16(d_feat_in) || !aligned16(d_weight) || !aligned16(d_feat_out) || !aligned16(d_grid) ||
        !aligned16(d_coords) || !aligned16(d_workspace))
        return SC_EINVAL;
    if (dtype_in != SC_F16 && dtype_in != SC_BF16) return SC_EINVAL;
    if (dtype_out != SC_F32 && dtype_out != dtype_in) return SC_EINVAL;
    if (grid_bytes < gneed) return SC_ECAP;
    const size_t need = sc_conv_workspace_bytes(K, C_in, C_out, dtype_in);
    if (d_workspace == nullptr || workspace_bytes < need) return SC_ECAP;
    if (n == 0) return SC_OK;
    const MapSource ms{nullptr, nullptr, (const int4*)d_coords, (const unsigned long long*)d_grid, GridDims{B, X, Y, Z}, epoch};
    if (!mfma_channels_ok(C_in, C_out)) return SC_EINVAL;
    return conv_16bit<1>(dtype_in, 27, 1, C_in, C_out, (n + TILE - 1) / TILE, (hipStream_t)stream, d_feat_in, d_weight,
                         false, d_workspace, d_feat_out, dtype_out == SC_F32, ms, nullptr, n, n);
}
