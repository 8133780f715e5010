// Status strings, thread-local error text and version of libdfgnn.
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <vector>

#include "common.hpp"

namespace dfgnn {
static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_error, sizeof(g_error), fmt, ap);
    va_end(ap);
}
void clear_error() { g_error[0] = '\0'; }

// ---- optional per-kernel timing -------------------------------------------------------------------
namespace {
struct TimingRecord { const char* label; hipEvent_t start, stop; };
bool g_timing = false;
std::vector<TimingRecord> g_records;  // used records: [0, g_used)
size_t g_used = 0;
constexpr size_t kMaxRecords = 1 << 16;
}  // namespace

KernelTimer::KernelTimer(const char* label, hipStream_t st) : slot(-1), stream(st) {
    if (!g_timing || g_used >= kMaxRecords) return;
    if (g_used == g_records.size()) {
        TimingRecord r{label, nullptr, nullptr};
        if (hipEventCreate(&r.start) != hipSuccess || hipEventCreate(&r.stop) != hipSuccess) return;
        g_records.push_back(r);
    }
    slot = (int)g_used++;
    g_records[slot].label = label;
    (void)hipEventRecord(g_records[slot].start, stream);
}
KernelTimer::~KernelTimer() {
    if (slot >= 0) (void)hipEventRecord(g_records[slot].stop, stream);
}
}  // namespace dfgnn

extern "C" int dfgnn_timing_enable(int enable) {
    dfgnn::clear_error();
    dfgnn::g_timing = enable != 0;
    dfgnn::g_used = 0;
    return DFGNN_OK;
}

extern "C" int dfgnn_timing_collect(int max_labels, const char** labels, double* total_ms, int64_t* launches, int* n_labels) {
    using namespace dfgnn;
    clear_error();
    DFGNN_REQUIRE(n_labels != nullptr && (max_labels == 0 || (labels && total_ms && launches)), DFGNN_EINVAL,
                  "NULL argument");
    int n = 0;
    for (size_t r = 0; r < g_used; ++r) {
        DFGNN_HIP(hipEventSynchronize(g_records[r].stop));
        float ms = 0.f;
        DFGNN_HIP(hipEventElapsedTime(&ms, g_records[r].start, g_records[r].stop));
        int k = 0;
        while (k < n && std::strcmp(labels[k], g_records[r].label) != 0) ++k;
        if (k == n) {
            DFGNN_REQUIRE(n < max_labels, DFGNN_EWORKSPACE, "more than %d distinct kernel labels", max_labels);
            labels[n] = g_records[r].label;
            total_ms[n] = 0.0;
            launches[n] = 0;
            ++n;
        }
        total_ms[k] += ms;
        launches[k] += 1;
    }
    g_used = 0;
    *n_labels = n;
    return DFGNN_OK;
}

extern "C" const char* dfgnn_status_string(int status) {
    switch (status) {
    case DFGNN_OK: return "DFGNN_OK";
    case DFGNN_EINVAL: return "DFGNN_EINVAL: invalid argument";
    case DFGNN_EUNSUPPORTED: return "DFGNN_EUNSUPPORTED: shape, dtype or alignment not supported";
    case DFGNN_EWORKSPACE: return "DFGNN_EWORKSPACE: caller-provided buffer too small";
    case DFGNN_EHIP: return "DFGNN_EHIP: HIP runtime error";
    default: return "unknown dfgnn status";
    }
}

extern "C" const char* dfgnn_last_error(void) { return dfgnn::g_error; }

#ifndef DFGNN_BUILD_ID
#define DFGNN_BUILD_ID "unknown"
#endif
// the tag makes the id readable from the library file without loading it
static const char kBuildTag[] = "DFGNN_BUILD_ID=" DFGNN_BUILD_ID;
extern "C" const char* dfgnn_build_id(void) { return kBuildTag + sizeof("DFGNN_BUILD_ID=") - 1; }

extern "C" int dfgnn_version(int* major, int* minor) {
    if (major) *major = 0;
    if (minor) *minor = 1;
    return DFGNN_OK;
}
