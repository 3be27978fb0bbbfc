// Optional per-kernel timing with HIP events on the caller's stream, for benchmarks.
// Off by default; while on, every kernel launch of the layer calls is bracketed by two
// events (created on demand, so the no-allocation guarantee of the layer calls does not
// hold while profiling).
#include "rgnn_internal.h"

#include <stdio.h>
#include <string.h>
#include <atomic>
#include <map>
#include <mutex>

namespace rgnn {

struct Record { const char* name; hipEvent_t a, b; };
static std::atomic<bool> g_on{false};
static char g_only[64] = "";       // name filter in force while profiling is on (empty: every kernel)
static char g_only_next[64] = "";  // the filter rgnn_profile_start() will put in force
static std::vector<Record> g_rec;
static std::mutex g_mu;

const char* wgrad_label(const char* label) {
    static std::mutex mu;
    static std::map<std::string, std::string> names;
    std::lock_guard<std::mutex> lk(mu);
    auto it = names.find(label);
    if (it == names.end()) it = names.emplace(label, std::string(label) + ".wgrad").first;
    return it->second.c_str();
}

KernelTimer::KernelTimer(hipStream_t st, const char* name) : st_(st), idx_(-1) {
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_only[0] && strcmp(g_only, name) != 0) return;
    Record r{name, nullptr, nullptr};
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    (void)hipEventRecord(r.a, st_);
    idx_ = (int)g_rec.size();
    g_rec.push_back(r);
}
KernelTimer::~KernelTimer() {
    if (idx_ < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    (void)hipEventRecord(g_rec[idx_].b, st_);
}

}  // namespace rgnn

using namespace rgnn;

extern "C" rgnn_status_t rgnn_profile_start(void) {
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto& r : g_rec) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    g_rec.clear();
    memcpy(g_only, g_only_next, sizeof(g_only));
    g_on = true;
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_profile_select(const char* name) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (name && strlen(name) >= sizeof(g_only_next)) RGNN_FAIL(RGNN_EINVAL, "rgnn_profile_select: the name is longer than %zu characters", sizeof(g_only_next) - 1);
    memset(g_only_next, 0, sizeof(g_only_next));
    if (name) strcpy(g_only_next, name);
    return RGNN_OK;
}

extern "C" rgnn_status_t rgnn_profile_stop(char* report, size_t report_bytes) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = false;
    RGNN_HIP(hipDeviceSynchronize());
    std::vector<const char*> order;
    std::map<std::string, std::pair<int, double>> agg;
    for (auto& r : g_rec) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) ms = 0.f;
        auto it = agg.find(r.name);
        if (it == agg.end()) { order.push_back(r.name); agg[r.name] = {1, (double)ms}; }
        else { it->second.first++; it->second.second += ms; }
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_rec.clear();
    size_t off = 0;
    if (report && report_bytes) report[0] = 0;
    for (const char* n : order) {
        char line[160];
        const int len = snprintf(line, sizeof(line), "%s %d %.6f\n", n, agg[n].first, agg[n].second);
        if (report && off + (size_t)len + 1 <= report_bytes) { memcpy(report + off, line, (size_t)len + 1); off += (size_t)len; }
    }
    return RGNN_OK;
}
