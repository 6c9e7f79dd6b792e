// Optional per-kernel timing with HIP events, for benchmarks: when switched on, every kernel
// launch of the library is bracketed by two events on the launch stream.  Off by default, so
// the hot path records nothing and allocates nothing.
#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"

namespace pa {

static const char* const kKernelNames[kProfKernels] = {"match_prefixes", "extend_plan",        "extend_attention",
                                                       "extend_merge",   "extend_attention_f32", "append_kv",
                                                       "gather_kv",      "calib_copy",           "calib_mfma"};

struct ProfRecord {
    hipEvent_t start, stop;
    int kernel;
};

static std::mutex g_prof_mu;
static bool g_prof_on = false;
static bool g_prof_clock = false;
static std::vector<ProfRecord> g_prof_records;  // events are reused across enable() calls
static size_t g_prof_used = 0;
constexpr size_t kProfMaxRecords = 1 << 16;

bool prof_clock_enabled() {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    return g_prof_on && g_prof_clock;
}

bool prof_begin(int kernel, hipStream_t stream, size_t* slot) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof_on || g_prof_used >= kProfMaxRecords) return false;
    if (g_prof_used == g_prof_records.size()) {
        ProfRecord r{};
        if (hipEventCreate(&r.start) != hipSuccess) return false;
        if (hipEventCreate(&r.stop) != hipSuccess) { (void)hipEventDestroy(r.start); return false; }
        g_prof_records.push_back(r);
    }
    *slot = g_prof_used++;
    g_prof_records[*slot].kernel = kernel;
    (void)hipEventRecord(g_prof_records[*slot].start, stream);
    return true;
}

void prof_end(size_t slot, hipStream_t stream) {
    std::lock_guard<std::mutex> lk(g_prof_mu);
    (void)hipEventRecord(g_prof_records[slot].stop, stream);
}

}  // namespace pa

extern "C" int pa_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(pa::g_prof_mu);
    if (on) pa::g_prof_used = 0;
    pa::g_prof_on = on != 0;
    pa::g_prof_clock = on == 2;
    return PA_OK;
}

extern "C" int pa_profile_read(const char* kernel, double* total_ms, int64_t* launches) {
    PA_REQUIRE(kernel != nullptr, "pa_profile_read: kernel name is NULL");
    int id = -1;
    for (int i = 0; i < pa::kProfKernels; ++i)
        if (std::strcmp(kernel, pa::kKernelNames[i]) == 0) id = i;
    PA_REQUIRE(id >= 0, "pa_profile_read: unknown kernel '%s'", kernel);
    std::lock_guard<std::mutex> lk(pa::g_prof_mu);
    double ms = 0.0;
    int64_t n = 0;
    for (size_t i = 0; i < pa::g_prof_used; ++i) {
        const pa::ProfRecord& r = pa::g_prof_records[i];
        if (r.kernel != id) continue;
        PA_HIP(hipEventSynchronize(r.stop));
        float x = 0.f;
        PA_HIP(hipEventElapsedTime(&x, r.start, r.stop));
        ms += x;
        ++n;
    }
    if (total_ms) *total_ms = ms;
    if (launches) *launches = n;
    return PA_OK;
}

extern "C" int pa_profile_clock(void* workspace, int reset, double* shader_mhz) {
    PA_REQUIRE(workspace != nullptr, "pa_profile_clock: workspace is NULL");
    unsigned char* at = static_cast<unsigned char*>(workspace) + pa::kClockProbeOffset;
    unsigned long long c[2] = {0, 0};
    PA_HIP(hipDeviceSynchronize());
    if (reset) {
        PA_HIP(hipMemcpy(at, c, sizeof c, hipMemcpyHostToDevice));
        if (shader_mhz) *shader_mhz = 0.0;
        return PA_OK;
    }
    PA_HIP(hipMemcpy(c, at, sizeof c, hipMemcpyDeviceToHost));
    if (shader_mhz) *shader_mhz = c[1] ? 100.0 * static_cast<double>(c[0]) / static_cast<double>(c[1]) : 0.0;
    return PA_OK;
}
