// Driver for the CPU oracle under AddressSanitizer / UndefinedBehaviorSanitizer (host code only).
// Runs the oracle's two entry points on seeded pseudo-random inputs of several shapes, including
// empty input, a single voxel, strided layers with K != stride and capacity errors, and checks
// basic invariants; any sanitizer report aborts the process.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <set>
#include <array>
#include <vector>

extern "C" {
int sc_oracle_kmap(const int32_t* coords, int64_t n, int K, int stride, int mode, int32_t* out_coords, int64_t out_cap,
                   int64_t* n_out, int32_t* pair_in, int32_t* pair_out, int64_t pair_cap, int64_t* offset_start);
int sc_oracle_conv(const double* feat_in, int64_t n_in, const double* weight, int K3, int C_in, int C_out,
                   const int32_t* pair_in, const int32_t* pair_out, const int64_t* offset_start, double* feat_out,
                   int64_t n_out, int threads);
}

static uint64_t rng_state = 0x9e3779b97f4a7c15ull;
static uint32_t rnd() {
    rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17;
    return (uint32_t)(rng_state >> 32);
}
#define REQUIRE(c) do { if (!(c)) { std::fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

static int run_case(int n, int grid, int K, int stride, int mode, int C_in, int C_out) {
    std::set<std::array<int32_t, 4>> seen;
    std::vector<int32_t> coords;
    while ((int)seen.size() < n) {
        std::array<int32_t, 4> c{(int32_t)(rnd() % 2), (int32_t)(rnd() % grid), (int32_t)(rnd() % grid), (int32_t)(rnd() % grid)};
        if (seen.insert(c).second) coords.insert(coords.end(), c.begin(), c.end());
    }
    const int K3 = K * K * K;
    const int m = (K + stride - 1) / stride;
    const int64_t out_cap = mode == 0 ? n : (int64_t)n * m * m * m, pair_cap = (int64_t)n * K3;
    std::vector<int32_t> out_coords((size_t)out_cap * 4 + 4), pin((size_t)pair_cap + 1), pout((size_t)pair_cap + 1);
    std::vector<int64_t> ost(K3 + 1);
    int64_t n_out = -1;
    int rc = sc_oracle_kmap(coords.data(), n, K, stride, mode, out_coords.data(), out_cap, &n_out, pin.data(), pout.data(),
                            pair_cap, ost.data());
    REQUIRE(rc == 0);
    REQUIRE(n_out >= 0 && n_out <= out_cap && ost[0] == 0 && ost[K3] <= pair_cap);
    for (int64_t e = 0; e < ost[K3]; ++e) REQUIRE(pin[e] >= 0 && pin[e] < n && pout[e] >= 0 && pout[e] < n_out);
    if (mode == 0) REQUIRE(n_out == n && ost[(K3 - 1) / 2 + 1] - ost[(K3 - 1) / 2] == n);      // centre offset: every row with itself
    std::vector<double> f((size_t)n * C_in + 1), w((size_t)K3 * C_in * C_out), o((size_t)n_out * C_out + 1);
    for (auto& v : f) v = (double)(rnd() % 2001) / 1000.0 - 1.0;
    for (auto& v : w) v = (double)(rnd() % 2001) / 1000.0 - 1.0;
    rc = sc_oracle_conv(f.data(), n, w.data(), K3, C_in, C_out, pin.data(), pout.data(), ost.data(), o.data(), n_out, 2);
    REQUIRE(rc == 0);
    // capacity errors are reported, not written past
    if (n > 1) {
        int64_t n_out2 = 0;
        rc = sc_oracle_kmap(coords.data(), n, K, stride, mode, out_coords.data(), 0, &n_out2, pin.data(), pout.data(), pair_cap, ost.data());
        REQUIRE(rc != 0);
        rc = sc_oracle_kmap(coords.data(), n, K, stride, mode, out_coords.data(), out_cap, &n_out2, pin.data(), pout.data(), 0, ost.data());
        REQUIRE(rc != 0 || ost[K3] == 0);
    }
    return 0;
}

int main() {
    const int cases[][7] = {{0, 8, 3, 1, 0, 4, 4},   {1, 8, 3, 1, 0, 3, 5},    {300, 8, 3, 1, 0, 8, 8},  {200, 6, 5, 1, 0, 2, 3},
                            {150, 9, 2, 2, 1, 4, 6}, {150, 9, 3, 2, 1, 4, 6},  {100, 9, 3, 1, 1, 2, 2},  {64, 5, 7, 1, 0, 1, 1},
                            {120, 10, 4, 2, 1, 3, 3}, {90, 10, 5, 3, 1, 2, 4}};
    for (const auto& c : cases)
        if (run_case(c[0], c[1], c[2], c[3], c[4], c[5], c[6])) { std::fprintf(stderr, "case n=%d K=%d s=%d failed\n", c[0], c[2], c[3]); return 1; }
    std::puts("oracle under sanitizers: ok");
    return 0;
}
