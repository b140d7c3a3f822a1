// Optional per-kernel timing: every launch carries a pair of HIP events stamped with the
// dispatch's begin and end, so a benchmark can report the duration of each kernel without an
// external profiler.
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
    int64_t launches[KID_COUNT] = {0};
    double total[KID_COUNT] = {0.0};
    for (const Mark& m : g_marks) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, m.begin, m.end) != hipSuccess) return SC_EHIP;
        launches[m.kid] += 1;
        total[m.kid] += ms;
    }
    int n = 0;
    for (int k = 0; k < KID_COUNT && n < max_entries; ++k) {
        if (launches[k] == 0) continue;
        h_entries[n].name = KERNEL_NAMES[k];
        h_entries[n].launches = launches[k];
        h_entries[n].total_ms = total[k];
        ++n;
    }
    return n;
}

#ifdef SC_TRACE
extern "C" int sc_trace_set(void* d_buf) {
    long long* p = (long long*)d_buf;
    return hipMemcpyToSymbol(HIP_SYMBOL(sc::g_trace_buf), &p, sizeof(p)) == hipSuccess ? SC_OK : SC_EHIP;
}
#endif
