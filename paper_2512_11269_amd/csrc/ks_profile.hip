// Per-kernel timing with HIP events, off by default.  Used by the benchmark to report each kernel's achieved
// bandwidth and arithmetic rate next to its algorithmic traffic and work; event pairs are recorded on the
// stream the kernel runs on.
#include <stdio.h>
#include <string.h>

#include <atomic>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "ks_internal.hpp"

namespace ks {

namespace {
struct Record {
    const char* name;
    double bytes, ops;
    hipEvent_t start, stop;
};
std::atomic<int> g_enabled{0};
std::mutex g_mu;
std::vector<Record> g_records;
}  // namespace

ProfScope::ProfScope(const char* name, double bytes, hipStream_t s, double ops) : slot(-1), stream(s) {
    if (!g_enabled.load(std::memory_order_relaxed)) return;
    Record r{name, bytes, ops, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess) return;
    if (hipEventCreate(&r.stop) != hipSuccess) {
        (void)hipEventDestroy(r.start);
        return;
    }
    (void)hipEventRecord(r.start, s);
    std::lock_guard<std::mutex> lock(g_mu);
    slot = (int)g_records.size();
    g_records.push_back(r);
}

ProfScope::~ProfScope() {
    if (slot < 0) return;
    std::lock_guard<std::mutex> lock(g_mu);
    (void)hipEventRecord(g_records[slot].stop, stream);
}

}  // namespace ks

using namespace ks;

extern "C" int ks_profile_enable(int on) {
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto& r : g_records) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_records.clear();
    g_enabled.store(on ? 1 : 0);
    return KS_OK;
}

extern "C" int ks_profile_report(char* buf, size_t buflen) {
    if (!buf || buflen == 0) return KS_EINVAL;
    std::lock_guard<std::mutex> lock(g_mu);
    struct Agg { double ms = 0, bytes = 0, ops = 0; long count = 0; };
    std::map<std::string, Agg> agg;
    std::vector<std::string> order;
    for (auto& r : g_records) {
        if (hipEventSynchronize(r.stop) != hipSuccess) return KS_EHIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return KS_EHIP;
        if (!agg.count(r.name)) order.push_back(r.name);
        Agg& a = agg[r.name];
        a.ms += ms;
        a.bytes += r.bytes;
        a.ops += r.ops;
        a.count += 1;
    }
    std::string out = "[";
    for (size_t i = 0; i < order.size(); ++i) {
        const Agg& a = agg[order[i]];
        char line[320];
        snprintf(line, sizeof(line),
                 "%s{\"kernel\": \"%s\", \"launches\": %ld, \"total_ms\": %.6f, \"total_bytes\": %.0f, \"total_ops\": %.0f}",
                 i ? ", " : "", order[i].c_str(), a.count, a.ms, a.bytes, a.ops);
        out += line;
    }
    out += "]";
    if (out.size() + 1 > buflen) return KS_EINVAL;
    memcpy(buf, out.c_str(), out.size() + 1);
    return KS_OK;
}
