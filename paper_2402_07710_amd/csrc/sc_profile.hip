// Optional per-kernel timing: every launch carries a pair of HIP events stamped with the
// dispatch's begin and end, so a benchmark can report the duration of each kernel without an
// external profiler.
#include <algorithm>
#include <vector>

#include "sc_internal.h"

namespace sc {

#ifdef SC_TRACE
__device__ long long* g_trace_buf = nullptr;
#endif

bool g_profile_on = false;

namespace {
struct Mark {
    int kid;
    hipEvent_t begin, end;
};
std::vector<Mark> g_marks;
std::vector<hipEvent_t> g_pool;      // events ready for reuse
const char* const KERNEL_NAMES[KID_COUNT] = {
    "k_table_fill", "k_hash_insert", "k_hash_lookup", "k_kmap_header", "k_kmap_subm", "k_strided_fill",
    "k_strided_insert", "k_strided_flags", "k_scan_blocks", "k_strided_pairs", "k_masks_from_table",
    "k_count_pairs", "k_export", "k_weight_pack", "k_conv_mfma", "k_conv_f32", "k_grid_clear", "k_grid_insert",
    "k_grid_lookup", "k_kmap_subm_grid", "misc"};

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

bool profile_events(int kernel_id, hipEvent_t* begin, hipEvent_t* end) {
    Mark m{kernel_id, take_event(), take_event()};
    if (m.begin == nullptr || m.end == nullptr) return false;
    g_marks.push_back(m);
    *begin = m.begin;
    *end = m.end;
    return true;
}

}  // namespace sc

using namespace sc;

extern "C" int sc_profile_enable(int enable) {
    for (Mark& m : g_marks) {
        g_pool.push_back(m.begin);
        g_pool.push_back(m.end);
    }
    g_marks.clear();
    g_profile_on = enable != 0;
    return SC_OK;
}

extern "C" int sc_profile_read(sc_profile_entry* h_entries, int max_entries) {
    if (h_entries == nullptr || max_entries < 0) return SC_EINVAL;
    if (hipDeviceSynchronize() != hipSuccess) return SC_EHIP;
    std::vector<float> samples[KID_COUNT];
    for (const Mark& m : g_marks) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, m.begin, m.end) != hipSuccess) return SC_EHIP;
        samples[m.kid].push_back(ms);
    }
    int n = 0;
    for (int k = 0; k < KID_COUNT && n < max_entries; ++k) {
        std::vector<float>& v = samples[k];
        if (v.empty()) continue;
        double total = 0.0;
        for (float ms : v) total += ms;
        std::sort(v.begin(), v.end());
        h_entries[n].name = KERNEL_NAMES[k];
        h_entries[n].launches = (int64_t)v.size();
        h_entries[n].total_ms = total;
        h_entries[n].median_ms = v.size() % 2 ? v[v.size() / 2] : 0.5 * (v[v.size() / 2 - 1] + v[v.size() / 2]);
        ++n;
    }
    return n;
}

// What the matrix cores of this device sustain on a loop of independent 16x16x32 fp16 multiplies
// with operands in registers: the measured counterpart of the published peak.
namespace sc {
typedef _Float16 pk_f16x8 __attribute__((ext_vector_type(8)));
typedef float pk_f32x4 __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256)
k_mfma_peak(float* sink, int iters) {
    pk_f16x8 a, b;
    for (int i = 0; i < 8; ++i) { a[i] = (_Float16)(threadIdx.x * 0.001f + i); b[i] = (_Float16)(i * 0.5f); }
    pk_f32x4 acc[8];
    for (int j = 0; j < 8; ++j) acc[j] = pk_f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, acc[j], 0, 0, 0);
    }
    float s = 0.f;
    for (int j = 0; j < 8; ++j) s += acc[j][0] + acc[j][1] + acc[j][2] + acc[j][3];
    if (s == 12345.678f) sink[0] = s;      // keeps the loop alive; never true for these operands in practice
}
}  // namespace sc

extern "C" int sc_profile_mfma_peak(double* h_tflops) {
    if (h_tflops == nullptr) return SC_EINVAL;
    float* d_sink = nullptr;
    if (hipMalloc(&d_sink, 256) != hipSuccess) return SC_EHIP;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    int rc = SC_OK;
    if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) rc = SC_EHIP;
    const int iters = 4096, blocks = 256 * 8;       // 8 workgroups of 4 wavefronts per compute unit
    double best = 0.0;
    for (int rep = 0; rep < 4 && rc == SC_OK; ++rep) {
        hipEventRecord(e0, nullptr);
        hipLaunchKernelGGL(k_mfma_peak, dim3(blocks), dim3(256), 0, nullptr, d_sink, iters);
        hipEventRecord(e1, nullptr);
        float ms = 0.f;
        if (hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess || ms <= 0.f) rc = SC_EHIP;
        else {
            const double flop = (double)blocks * 4 * iters * 8 * (2.0 * 16 * 16 * 32);
            best = std::max(best, flop / (ms * 1e-3) / 1e12);
        }
    }
    if (e0) hipEventDestroy(e0);
    if (e1) hipEventDestroy(e1);
    hipFree(d_sink);
    *h_tflops = best;
    return rc;
}

#ifdef SC_TRACE
extern "C" int sc_trace_set(void* d_buf) {
    long long* p = (long long*)d_buf;
    return hipMemcpyToSymbol(HIP_SYMBOL(sc::g_trace_buf), &p, sizeof(p)) == hipSuccess ? SC_OK : SC_EHIP;
}
#endif
