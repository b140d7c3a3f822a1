// CPU oracle for sparse 3-D convolution over voxel coordinates.  TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, obviously-correct statement of what the sparse-convolution path computes,
// written from the paper's definitions (Section II-B: submanifold convolution keeps the output
// sites equal to the input sites; Section III-B eq. 1-5: the stride-s cell mapping and the
// numbering of kernel offsets; Section III-C "Create Offset Table" and its figure: which
// neighbour lands in which column; Algorithm 2: the sum over offsets and input channels).
// Ordered std::map lookups and a triple loop per offset in double precision; no blocking, no
// fusion, no cleverness.  It shares nothing with the GPU library: only tests, the smoke check
// and the benchmark's cpu_baseline leg may link or call it.
//
// Definition implemented here (coordinates p = (b,x,y,z), all >= 0, rows distinct):
//   offsets d in {0..K-1}^3 are numbered k = dX*K^2 + dY*K + dZ                (eq. 5)
//   pad = (K-1)/2 for submanifold layers (stride 1, K odd), 0 for strided layers
//   output sites Q: submanifold: Q = inputs, same order;
//                   strided: every q >= 0 with q*s + d = p_i for some input i and offset d
//                   (for K = s this is the set of cells floor(p/s), eq. 2 and eq. 4), numbered
//                   in order of first occurrence (inputs ascending, then k ascending)
//   pair (in=i, out=o) belongs to offset k  <=>  p_i = q_o*s + d_k - pad, batch equal
//   F_out[o][co] = sum_k sum_{(i,o) in M_k} sum_ci F_in[i][ci] * W[k][ci][co]  (Algorithm 2)
//
// Pins (tests/test_oracle_*.py, all CPU): dense zero-padded 3-D correlation masked to active
// sites on tiny grids, the paper's two worked figures, eq. 1-5 examples, pair symmetry, centre
// identity, delta weights, closed-form pair counts, an isolated-voxel case equal to one matrix
// product, linearity / permutation / translation / batch invariances, and an out-major
// evaluation in Algorithm 2's loop order written separately in numpy.

#include <array>
#include <cstdint>
#include <cstring>
#include <map>
#include <vector>

namespace {

using Coord = std::array<int32_t, 4>;   // b, x, y, z — std::array orders lexicographically

enum { OR_OK = 0, OR_EINVAL = -1, OR_EDUP = -2, OR_ENEG = -3, OR_ECAP = -4 };

bool decode_offset(int k, int K, int d[3]) {
    d[0] = k / (K * K);
    d[1] = (k / K) % K;
    d[2] = k % K;
    return true;
}

}  // namespace

extern "C" {

// Kernel map (rulebook) by direct lookup.
//   coords      [n][4] int32 (b,x,y,z)
//   mode        0 = submanifold (stride must be 1, K odd), 1 = strided
//   out_coords  [out_cap][4]  receives the output sites (submanifold: a copy of coords)
//   pair_in/pair_out [pair_cap]  pairs grouped by offset k, inside one offset ordered by
//                                output index ascending
//   offset_start [K^3+1]  pairs of offset k are [offset_start[k], offset_start[k+1])
int sc_oracle_kmap(const int32_t* coords, int64_t n, int K, int stride, int mode,
                   int32_t* out_coords, int64_t out_cap, int64_t* n_out,
                   int32_t* pair_in, int32_t* pair_out, int64_t pair_cap,
                   int64_t* offset_start) {
    if (n < 0 || K < 1 || stride < 1 || (mode != 0 && mode != 1)) return OR_EINVAL;
    if (mode == 0 && (stride != 1 || K % 2 == 0)) return OR_EINVAL;
    const int K3 = K * K * K;
    const int pad = (mode == 0) ? (K - 1) / 2 : 0;

    std::map<Coord, int32_t> in_index;
    for (int64_t i = 0; i < n; ++i) {
        Coord p{coords[4 * i], coords[4 * i + 1], coords[4 * i + 2], coords[4 * i + 3]};
        for (int a = 0; a < 4; ++a)
            if (p[a] < 0) return OR_ENEG;
        if (!in_index.emplace(p, (int32_t)i).second) return OR_EDUP;
    }

    // output sites
    std::vector<Coord> outs;
    if (mode == 0) {
        outs.reserve(n);
        for (int64_t i = 0; i < n; ++i)
            outs.push_back({coords[4 * i], coords[4 * i + 1], coords[4 * i + 2], coords[4 * i + 3]});
    } else {
        std::map<Coord, int32_t> out_index;
        for (int64_t i = 0; i < n; ++i) {
            for (int k = 0; k < K3; ++k) {
                int d[3];
                decode_offset(k, K, d);
                Coord q{coords[4 * i], 0, 0, 0};
                bool ok = true;
                for (int a = 0; a < 3; ++a) {
                    int32_t t = coords[4 * i + 1 + a] - d[a];       // = q*s must hold
                    if (t < 0 || t % stride != 0) { ok = false; break; }
                    q[1 + a] = t / stride;
                }
                if (!ok) continue;
                if (out_index.emplace(q, (int32_t)outs.size()).second) outs.push_back(q);
            }
        }
    }
    *n_out = (int64_t)outs.size();
    if ((int64_t)outs.size() > out_cap) return OR_ECAP;
    for (size_t o = 0; o < outs.size(); ++o)
        for (int a = 0; a < 4; ++a) out_coords[4 * o + a] = outs[o][a];

    // pairs, offset by offset
    int64_t total = 0;
    for (int k = 0; k < K3; ++k) {
        offset_start[k] = total;
        int d[3];
        decode_offset(k, K, d);
        for (size_t o = 0; o < outs.size(); ++o) {
            Coord p{outs[o][0],
                    outs[o][1] * stride + d[0] - pad,
                    outs[o][2] * stride + d[1] - pad,
                    outs[o][3] * stride + d[2] - pad};
            auto it = in_index.find(p);
            if (it == in_index.end()) continue;
            if (total >= pair_cap) return OR_ECAP;
            pair_in[total] = it->second;
            pair_out[total] = (int32_t)o;
            ++total;
        }
    }
    offset_start[K3] = total;
    return OR_OK;
}

// Output features from a kernel map: one triple loop per offset (pairs x C_in x C_out),
// accumulated in double into a zero-initialised output.  `threads` > 1 splits the output
// columns over OpenMP threads (each column is still summed in the same order).
//   feat_in [n_in][C_in], weight [K3][C_in][C_out], feat_out [n_out][C_out]
int sc_oracle_conv(const double* feat_in, int64_t n_in, const double* weight, int K3,
                   int C_in, int C_out, const int32_t* pair_in, const int32_t* pair_out,
                   const int64_t* offset_start, double* feat_out, int64_t n_out, int threads) {
    if (n_in < 0 || n_out < 0 || K3 < 1 || C_in < 1 || C_out < 1) return OR_EINVAL;
    std::memset(feat_out, 0, sizeof(double) * (size_t)n_out * C_out);
    for (int64_t e = 0; e < offset_start[K3]; ++e)
        if (pair_in[e] < 0 || pair_in[e] >= n_in || pair_out[e] < 0 || pair_out[e] >= n_out)
            return OR_EINVAL;
    if (threads < 1) threads = 1;
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int t = 0; t < threads; ++t) {
        const int co_lo = (int)((int64_t)C_out * t / threads);
        const int co_hi = (int)((int64_t)C_out * (t + 1) / threads);
        for (int k = 0; k < K3; ++k) {
            const double* Wk = weight + (size_t)k * C_in * C_out;
            for (int64_t e = offset_start[k]; e < offset_start[k + 1]; ++e) {
                const double* fi = feat_in + (size_t)pair_in[e] * C_in;
                double* fo = feat_out + (size_t)pair_out[e] * C_out;
                for (int ci = 0; ci < C_in; ++ci)
                    for (int co = co_lo; co < co_hi; ++co)
                        fo[co] += fi[ci] * Wk[(size_t)ci * C_out + co];
            }
        }
    }
    return OR_OK;
}

}  // extern "C"
