// Compute step: out[o] = sum_k sum_{(i,o) in M_k} in[i] . W[k]   (paper Algorithm 2).
//
// The paper's kernel gives one thread one (output row, output channel) and walks K^3 x C_in
// scalar FMAs with one output channel's weights cached in shared memory, so every gathered
// feature row is re-read C_out times.  Here a wavefront owns one 64-row output tile of the
// kernel map.  For each offset k it takes the tile's pairs 16 at a time, gathers their input
// rows straight into MFMA operand registers (16 bytes per lane), multiplies them by W[k] on the
// matrix cores (v_mfma_f32_16x16x32, fp32 accumulation) and adds the 16 x C_out result into the
// tile's fp32 accumulators in LDS at the rows the pairs name.  Only pairs that exist are
// multiplied, every offset of a row is summed on-chip, and each output row is written once,
// converted once, with no global atomics.
#include <cstdlib>

#include "sc_internal.h"

namespace sc {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int LDS_PAD = 4;   // floats added to each accumulator row (rotates LDS banks)

// W [K3][C_in][C_out] (16-bit elements) -> MFMA A-operand tiles of W[k]^T:
// wp[((k*CB + cb)*KS + ks)*64 + lane] holds W[k][ks*32 + 8*(lane/16) + j][cb*16 + lane%16], j = 0..7
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
    wp[t] = make_uint4(v[0], v[1], v[2], v[3]);
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

// One wavefront per output tile.  KS = C_in / 32.
template <int DT, int KS>
__global__ void __launch_bounds__(64)
k_conv_mfma(const uint16_t* __restrict__ feat, const uint4* __restrict__ wp, void* __restrict__ out, int out_f32,
            const uint16_t* __restrict__ start, const uint32_t* __restrict__ entries, int sstride, int K3,
            int C_out, const sc_counts* __restrict__ counts, int64_t n_out_cap) {
    extern __shared__ __align__(16) float acc_lds[];      // [TILE][C_out + LDS_PAD]
    constexpr int C_in = KS * 32;
    const int LS = C_out + LDS_PAD;
    const int CB = C_out / 16;
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    int64_t n_out = counts->n_out;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row0 = tile * TILE;
    if (row0 >= n_out) return;

    for (int i = lane; i < TILE * LS / 4; i += WAVE) reinterpret_cast<float4*>(acc_lds)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();

    const uint16_t* st = start + tile * sstride;
    const uint32_t* en = entries + tile * (int64_t)(TILE * K3);
    const int r = lane & 15, q = lane >> 4;

    for (int k = 0; k < K3; ++k) {
        const int s0 = st[k], s1 = st[k + 1];
        for (int g = s0; g < s1; g += 16) {
            const bool active = g + r < s1;
            uint32_t e = 0;
            if (active) e = en[g + r];
            const uint32_t in_row = e & ENTRY_ROW_MASK, slot = e >> ENTRY_ROW_BITS;
            uint4 fb[KS];
            const uint4* frow = reinterpret_cast<const uint4*>(feat + (int64_t)in_row * C_in) + q;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) fb[ks] = active ? frow[ks * 4] : make_uint4(0, 0, 0, 0);
            const uint4* wk = wp + (int64_t)k * CB * KS * 64 + lane;
            for (int cb = 0; cb < CB; ++cb) {
                f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) acc = mfma16x16x32<DT>(wk[(cb * KS + ks) * 64], fb[ks], acc);
                if (active) {
                    float4* p = reinterpret_cast<float4*>(&acc_lds[slot * LS + cb * 16 + q * 4]);
                    float4 v = *p;
                    v.x += acc[0]; v.y += acc[1]; v.z += acc[2]; v.w += acc[3];
                    *p = v;
                }
            }
        }
    }
    __syncthreads();

    const int rows = (int)((n_out - row0) < TILE ? (n_out - row0) : TILE);
    if (out_f32) {
        const int per_row = C_out / 4;
        float4* dst = reinterpret_cast<float4*>(out) + row0 * per_row;
        for (int i = lane; i < rows * per_row; i += WAVE) {
            const int rr = i / per_row, c4 = i - rr * per_row;
            dst[i] = *reinterpret_cast<const float4*>(&acc_lds[rr * LS + c4 * 4]);
        }
    } else {
        const int per_row = C_out / 8;
        uint4* dst = reinterpret_cast<uint4*>(out) + row0 * per_row;
        for (int i = lane; i < rows * per_row; i += WAVE) {
            const int rr = i / per_row, c8 = i - rr * per_row;
            const float4 a = *reinterpret_cast<const float4*>(&acc_lds[rr * LS + c8 * 8]);
            const float4 b = *reinterpret_cast<const float4*>(&acc_lds[rr * LS + c8 * 8 + 4]);
            dst[i] = make_uint4(pack2<DT>(a.x, a.y), pack2<DT>(a.z, a.w), pack2<DT>(b.x, b.y), pack2<DT>(b.z, b.w));
        }
    }
}

// Same computation for the common shapes, organised for memory-level parallelism.  A layer of
// ~10^5 voxels is a few microseconds of matrix work, so what decides the time is how many loads
// are in flight, not how many flops are issued.  One workgroup of SPLIT wavefronts owns a tile:
//   - the tile's offset starts and all of its pairs are copied into LDS once;
//   - the tile's MFMA groups (16 pairs of one offset) are dealt round-robin to the wavefronts;
//   - a wavefront takes G groups at a time: it reads their pairs from LDS, issues the feature
//     gathers and the weight-tile loads of all G groups back to back, and only then multiplies;
//   - every wavefront adds into its own fp32 accumulator tile in LDS (no atomics, fixed order),
//     and the SPLIT partial tiles are summed in wavefront order when the row is written.
// KS = C_in / 32, CB = C_out / 16; needs K^3 <= 27.
constexpr int CONV_K3_MAX = 27;
template <int DT, int KS, int CB, int SPLIT, int G>
__global__ void __launch_bounds__(64 * SPLIT)
k_conv_mfma_tile(const uint16_t* __restrict__ feat, const uint4* __restrict__ wp, void* __restrict__ out, int out_f32,
                 const uint16_t* __restrict__ start, const uint32_t* __restrict__ entries, int sstride, int K3,
                 const sc_counts* __restrict__ counts, int64_t n_out_cap) {
    constexpr int C_in = KS * 32, C_out = CB * 16, LS = C_out + LDS_PAD;
    constexpr int MAX_GROUPS = CONV_K3_MAX + TILE * CONV_K3_MAX / 16;
    extern __shared__ __align__(16) float acc_lds[];                  // [SPLIT][TILE][LS]
    __shared__ uint32_t ent_s[TILE * CONV_K3_MAX];
    __shared__ uint32_t grp_s[MAX_GROUPS];                            // group -> first pair | past-the-end pair << 16
    __shared__ uint8_t grp_k[MAX_GROUPS];                             // group -> offset k
    __shared__ int32_t st_s[CONV_K3_MAX + 1];
    __shared__ int32_t ng_s;

    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const int64_t tile = blockIdx.x;
    int64_t n_out = counts->n_out;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row0 = tile * TILE;
    if (row0 >= n_out) return;

    const uint16_t* st = start + tile * sstride;
    const uint32_t* en = entries + tile * (int64_t)(TILE * K3);
    if (threadIdx.x <= K3) st_s[threadIdx.x] = st[threadIdx.x];
    float* acc = acc_lds + w * (TILE * LS);
    for (int i = lane; i < TILE * LS / 4; i += WAVE) reinterpret_cast<float4*>(acc)[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    __syncthreads();
    const int E = st_s[K3];
    for (int i = threadIdx.x; i < E; i += 64 * SPLIT) ent_s[i] = en[i];
    if (w == 0) {          // the tile's group list: offset k has ceil(count/16) groups
        int cnt = 0, s0 = 0;
        if (lane < K3) { s0 = st_s[lane]; cnt = st_s[lane + 1] - s0; }
        const int ng = (cnt + 15) >> 4;
        int incl = ng;
#pragma unroll
        for (int off = 1; off < WAVE; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const int gbase = incl - ng;
        for (int j = 0; j < ng; ++j) {
            grp_s[gbase + j] = (uint32_t)(s0 + 16 * j) | ((uint32_t)(s0 + cnt) << 16);
            grp_k[gbase + j] = (uint8_t)lane;
        }
        if (lane == WAVE - 1) ng_s = incl;
    }
    __syncthreads();
    const int NG = ng_s;
    const int r = lane & 15, q = lane >> 4;

    for (int b0 = w; b0 < NG; b0 += SPLIT * G) {
        uint32_t e[G];
        int kk[G];
        bool act[G];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const int gi = b0 + j * SPLIT;
            const bool have = gi < NG;
            const uint32_t info = have ? grp_s[gi] : 0u;
            kk[j] = have ? (int)grp_k[gi] : 0;
            const int g0 = (int)(info & 0xffffu), g1 = (int)(info >> 16);
            act[j] = have && (g0 + r < g1);
            e[j] = act[j] ? ent_s[g0 + r] : 0u;
        }
        uint4 fb[G][KS];
        uint4 wa[G][CB][KS];
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const uint4* frow = reinterpret_cast<const uint4*>(feat + (int64_t)(e[j] & ENTRY_ROW_MASK) * C_in) + q;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) fb[j][ks] = act[j] ? frow[ks * 4] : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const uint4* wk = wp + (int64_t)kk[j] * (CB * KS * 64) + lane;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) wa[j][cb][ks] = wk[(cb * KS + ks) * 64];
        }
#pragma unroll
        for (int j = 0; j < G; ++j) {
            const uint32_t slot = e[j] >> ENTRY_ROW_BITS;
#pragma unroll
            for (int cb = 0; cb < CB; ++cb) {
                f32x4 d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) d = mfma16x16x32<DT>(wa[j][cb][ks], fb[j][ks], d);
                if (act[j]) {
                    float4* p = reinterpret_cast<float4*>(&acc[slot * LS + cb * 16 + q * 4]);
                    float4 v = *p;
                    v.x += d[0]; v.y += d[1]; v.z += d[2]; v.w += d[3];
                    *p = v;
                }
            }
        }
    }
    __syncthreads();

    const int rows = (int)((n_out - row0) < TILE ? (n_out - row0) : TILE);
    constexpr int per_row = C_out / 8;                                // 8 channels per thread per step
    for (int i = threadIdx.x; i < rows * per_row; i += 64 * SPLIT) {
        const int rr = i / per_row, c8 = i - rr * per_row;
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
#pragma unroll
        for (int ww = 0; ww < SPLIT; ++ww) {
            const float* src = acc_lds + ww * (TILE * LS) + rr * LS + c8 * 8;
            const float4 x = *reinterpret_cast<const float4*>(src), y = *reinterpret_cast<const float4*>(src + 4);
            a.x += x.x; a.y += x.y; a.z += x.z; a.w += x.w;
            b.x += y.x; b.y += y.y; b.z += y.z; b.w += y.w;
        }
        if (out_f32) {
            float4* dst = reinterpret_cast<float4*>(out) + (row0 * per_row + i) * 2;
            dst[0] = a;
            dst[1] = b;
        } else {
            reinterpret_cast<uint4*>(out)[row0 * per_row + i] =
                make_uint4(pack2<DT>(a.x, a.y), pack2<DT>(a.z, a.w), pack2<DT>(b.x, b.y), pack2<DT>(b.z, b.w));
        }
    }
}

// fp32 features and weights: plain FMA, one wavefront per tile, lanes over output channels.
__global__ void __launch_bounds__(64)
k_conv_f32(const float* __restrict__ feat, const float* __restrict__ w, float* __restrict__ out,
           const uint16_t* __restrict__ start, const uint32_t* __restrict__ entries, int sstride, int K3,
           int C_in, int C_out, const sc_counts* __restrict__ counts, int64_t n_out_cap) {
    extern __shared__ __align__(16) float acc_lds[];      // [TILE][C_out]
    const int lane = threadIdx.x;
    const int64_t tile = blockIdx.x;
    int64_t n_out = counts->n_out;
    if (n_out > n_out_cap) n_out = n_out_cap;
    const int64_t row0 = tile * TILE;
    if (row0 >= n_out) return;
    for (int i = lane; i < TILE * C_out; i += WAVE) acc_lds[i] = 0.f;
    __syncthreads();
    const uint16_t* st = start + tile * sstride;
    const uint32_t* en = entries + tile * (int64_t)(TILE * K3);
    // lanes = (pair within a group of PG pairs) x (output channel), PG * CL = 64
    int CL = 1;
    while (CL < C_out && CL < 64) CL <<= 1;
    const int PG = 64 / CL;
    const int pl = lane / CL, cl = lane - pl * CL;
    for (int k = 0; k < K3; ++k) {
        const int s0 = st[k], s1 = st[k + 1];
        const float* wk = w + (int64_t)k * C_in * C_out;
        for (int g = s0; g < s1; g += PG) {
            const bool active = g + pl < s1;
            uint32_t e = 0;
            if (active) e = en[g + pl];
            const float* f = feat + (int64_t)(e & ENTRY_ROW_MASK) * C_in;
            const uint32_t slot = e >> ENTRY_ROW_BITS;
            if (active) {
                for (int co = cl; co < C_out; co += CL) {
                    float s = 0.f;
                    for (int ci = 0; ci < C_in; ++ci) s = fmaf(f[ci], wk[(int64_t)ci * C_out + co], s);
                    acc_lds[slot * C_out + co] += s;
                }
            }
        }
    }
    __syncthreads();
    const int rows = (int)((n_out - row0) < TILE ? (n_out - row0) : TILE);
    float* dst = out + row0 * C_out;
    for (int i = lane; i < rows * C_out; i += WAVE) dst[i] = acc_lds[i];
}

template <int DT>
static int launch_mfma(int KS, dim3 grid, size_t lds, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out,
                       int out_f32, const uint16_t* start, const uint32_t* entries, int sstride, int K3, int C_out,
                       const sc_counts* counts, int64_t n_out_cap) {
#define SC_LAUNCH_KS(KSV)                                                                                           \
    case KSV: {                                                                                                     \
        auto fn = k_conv_mfma<DT, KSV>;                                                                             \
        if (lds > 48 * 1024 &&                                                                                      \
            hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) \
            return SC_EHIP;                                                                                         \
        SC_LAUNCH(KID_CONV_MFMA, fn, grid, dim3(64), lds, s, feat, wp, out, out_f32, start, entries, sstride, K3, C_out,  \
                           counts, n_out_cap);                                                                      \
        break;                                                                                                      \
    }
    switch (KS) {
        SC_LAUNCH_KS(1)
        SC_LAUNCH_KS(2)
        SC_LAUNCH_KS(4)
        SC_LAUNCH_KS(8)
        default: return SC_EINVAL;
    }
#undef SC_LAUNCH_KS
    return SC_OK;
}

template <int DT, int KS, int CB, int SPLIT, int G>
static int launch_tile(dim3 grid, hipStream_t s, const uint16_t* feat, const uint4* wp, void* out, int out_f32,
                       const uint16_t* start, const uint32_t* entries, int sstride, int K3, const sc_counts* counts,
                       int64_t n_out_cap) {
    auto fn = k_conv_mfma_tile<DT, KS, CB, SPLIT, G>;
    const size_t lds = (size_t)SPLIT * TILE * (CB * 16 + LDS_PAD) * sizeof(float);
    static bool attr_set = false;           // once per instantiation; the value never changes
    if (!attr_set) {
        if (hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)
            return SC_EHIP;
        attr_set = true;
    }
    SC_LAUNCH(KID_CONV_MFMA, fn, grid, dim3(64 * SPLIT), lds, s, feat, wp, out, out_f32, start, entries, sstride, K3,
              counts, n_out_cap);
    return SC_OK;
}

// Shapes with a tile kernel: (C_in, C_out) in {(32,32), (32,64), (64,64), (128,128)}, K^3 <= 27.
// `split` wavefronts share a tile when the layer is too small to fill the GPU otherwise.
template <int DT>
static int launch_tile_shape(int C_in, int C_out, int64_t tiles, hipStream_t s, const uint16_t* feat, const uint4* wp,
                             void* out, int out_f32, const uint16_t* start, const uint32_t* entries, int sstride,
                             int K3, const sc_counts* counts, int64_t n_out_cap, bool* handled) {
    *handled = true;
    const dim3 grid((unsigned)tiles);
    static const int force_split = getenv("SC_CONV_SPLIT") ? atoi(getenv("SC_CONV_SPLIT")) : 0;
    int split = tiles < 2048 ? 4 : (tiles < 8192 ? 2 : 1);
    if (force_split) split = force_split;
#define SC_TILE(KSV, CBV, SP, GV) \
    return launch_tile<DT, KSV, CBV, SP, GV>(grid, s, feat, wp, out, out_f32, start, entries, sstride, K3, counts, n_out_cap)
    if (C_in == 32 && C_out == 32) {
        if (split == 4) SC_TILE(1, 2, 4, 8);
        if (split == 2) SC_TILE(1, 2, 2, 8);
        SC_TILE(1, 2, 1, 8);
    }
    if (C_in == 32 && C_out == 64) {
        if (split == 4) SC_TILE(1, 4, 4, 4);
        if (split == 2) SC_TILE(1, 4, 2, 4);
        SC_TILE(1, 4, 1, 4);
    }
    if (C_in == 64 && C_out == 64) {
        if (split == 4) SC_TILE(2, 4, 4, 2);
        if (split == 2) SC_TILE(2, 4, 2, 2);
        SC_TILE(2, 4, 1, 2);
    }
    if (C_in == 128 && C_out == 128) {
        if (split >= 2) SC_TILE(4, 8, 2, 1);
        SC_TILE(4, 8, 1, 1);
    }
#undef SC_TILE
    *handled = false;
    return SC_OK;
}

static bool mfma_channels_ok(int C_in, int C_out) {
    return (C_in == 32 || C_in == 64 || C_in == 128 || C_in == 256) && C_out >= 16 && C_out <= 256 && C_out % 16 == 0;
}

}  // namespace sc

using namespace sc;

extern "C" size_t sc_conv_workspace_bytes(int K, int C_in, int C_out, int dtype_in) {
    if (K < 1 || K > SC_K_MAX || C_in < 1 || C_out < 1) return 0;
    if (dtype_in == SC_F32) return 0;
    return align_up((size_t)K * K * K * C_in * C_out * 2, 256);
}

extern "C" int sc_conv_fwd(const void* d_feat_in, int64_t n_in, const void* d_weight, void* d_feat_out,
                           int64_t n_out_cap, const void* d_kmap, size_t kmap_bytes, const sc_counts* d_counts, int K,
                           int stride, int mode, int C_in, int C_out, int dtype_in, int dtype_out, void* d_workspace,
                           size_t workspace_bytes, void* stream) {
    if (n_in < 0 || n_in > SC_N_MAX || n_out_cap < 0 || K < 1 || K > SC_K_MAX || C_in < 1 || C_out < 1) return SC_EINVAL;
    if (d_weight == nullptr || d_kmap == nullptr || d_counts == nullptr) return SC_EINVAL;
    if ((n_in > 0 && d_feat_in == nullptr) || (n_out_cap > 0 && d_feat_out == nullptr)) return SC_EINVAL;
    if (!aligned16(d_feat_in) || !aligned16(d_weight) || !aligned16(d_feat_out) || !aligned16(d_kmap) ||
        !aligned16(d_counts) || !aligned16(d_workspace))
        return SC_EINVAL;
    if (dtype_in != SC_F32 && dtype_in != SC_F16 && dtype_in != SC_BF16) return SC_EINVAL;
    if (dtype_out != SC_F32 && dtype_out != dtype_in) return SC_EINVAL;
    const int64_t bound = sc_out_bound(n_in, K, stride, mode);
    if (bound < 0) return SC_EINVAL;
    if (kmap_bytes < sc_kmap_bytes(n_in, K, stride, mode)) return SC_ECAP;
    const KmapLayout L = kmap_layout(bound, K);
    int64_t tiles = (n_out_cap + TILE - 1) / TILE;
    if (tiles > L.tiles) tiles = L.tiles;
    if (tiles == 0) return SC_OK;
    const uint16_t* start = (const uint16_t*)((const char*)d_kmap + L.off_start);
    const uint32_t* entries = (const uint32_t*)((const char*)d_kmap + L.off_entries);
    hipStream_t s = (hipStream_t)stream;

    if (dtype_in == SC_F32) {
        if (C_out > 256) return SC_EINVAL;
        const size_t lds = (size_t)TILE * C_out * sizeof(float);
        if (lds > 48 * 1024 && hipFuncSetAttribute((const void*)k_conv_f32, hipFuncAttributeMaxDynamicSharedMemorySize,
                                                   (int)lds) != hipSuccess)
            return SC_EHIP;
        SC_LAUNCH(KID_CONV_F32, k_conv_f32, dim3((unsigned)tiles), dim3(64), lds, s, (const float*)d_feat_in,
                           (const float*)d_weight, (float*)d_feat_out, start, entries, L.sstride, L.K3, C_in, C_out,
                           d_counts, n_out_cap);
        return SC_OK;
    }

    if (!mfma_channels_ok(C_in, C_out)) return SC_EINVAL;
    const size_t need = sc_conv_workspace_bytes(K, C_in, C_out, dtype_in);
    if (d_workspace == nullptr || workspace_bytes < need) return SC_ECAP;
    const int64_t pack_threads = (int64_t)L.K3 * (C_out / 16) * (C_in / 32) * 64;
    SC_LAUNCH(KID_WEIGHT_PACK, k_weight_pack, dim3((unsigned)((pack_threads + 255) / 256)), dim3(256), 0, s,
                       (const uint16_t*)d_weight, (uint4*)d_workspace, L.K3, C_in, C_out);
    const int out_f32 = dtype_out == SC_F32;
    static const bool no_tile = getenv("SC_CONV_GENERIC") != nullptr;
    if (L.K3 <= CONV_K3_MAX && !no_tile) {
        bool handled = false;
        int rc;
        if (dtype_in == SC_F16)
            rc = launch_tile_shape<SC_F16>(C_in, C_out, tiles, s, (const uint16_t*)d_feat_in, (const uint4*)d_workspace,
                                           d_feat_out, out_f32, start, entries, L.sstride, L.K3, d_counts, n_out_cap,
                                           &handled);
        else
            rc = launch_tile_shape<SC_BF16>(C_in, C_out, tiles, s, (const uint16_t*)d_feat_in, (const uint4*)d_workspace,
                                            d_feat_out, out_f32, start, entries, L.sstride, L.K3, d_counts, n_out_cap,
                                            &handled);
        if (handled || rc != SC_OK) return rc;
    }
    const size_t lds = (size_t)TILE * (C_out + LDS_PAD) * sizeof(float);
    if (dtype_in == SC_F16)
        return launch_mfma<SC_F16>(C_in / 32, dim3((unsigned)tiles), lds, s, (const uint16_t*)d_feat_in,
                                   (const uint4*)d_workspace, d_feat_out, out_f32, start, entries, L.sstride, L.K3,
                                   C_out, d_counts, n_out_cap);
    return launch_mfma<SC_BF16>(C_in / 32, dim3((unsigned)tiles), lds, s, (const uint16_t*)d_feat_in,
                                (const uint4*)d_workspace, d_feat_out, out_f32, start, entries, L.sstride, L.K3, C_out,
                                d_counts, n_out_cap);
}
