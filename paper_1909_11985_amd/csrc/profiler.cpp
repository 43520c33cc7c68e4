#include "profiler.h"

#include <cstdio>
#include <cstdlib>
#include <deque>
#include <map>
#include <string>
#include <vector>

namespace edl {

namespace {
struct Rec {
    const char* label;
    double flops, bytes;
    hipEvent_t a, b;
};
bool g_on = false;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_pool;

hipEvent_t take_event() {
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}
}  // namespace

void prof_enable(bool on) { g_on = on; }
bool prof_enabled() { return g_on; }

const char* prof_shape_label(const char* base, long long M, int C) {
    static const bool by_shape = getenv("EDL_PROFILE_BY_SHAPE") != nullptr;
    if (!by_shape || !g_on) return base;
    static std::deque<std::string> names;   // a deque keeps the strings where they are
    char buf[160];
    snprintf(buf, sizeof(buf), "%s M=%lld C=%d", base, M, C);
    for (const std::string& n : names)
        if (n == buf) return n.c_str();
    names.emplace_back(buf);
    return names.back().c_str();
}

void prof_begin(const char* label, double flops, double bytes, hipStream_t st) {
    Rec r{label, flops, bytes, take_event(), take_event()};
    (void)hipEventRecord(r.a, st);
    g_recs.push_back(r);
}

void prof_end(hipStream_t st) {
    if (!g_recs.empty()) (void)hipEventRecord(g_recs.back().b, st);
}

long prof_report(char* buf, size_t cap) {
    struct Agg { long n = 0; double ms = 0, flops = 0, bytes = 0; };
    std::map<std::string, Agg> agg;
    bool bad = false;
    for (Rec& r : g_recs) {
        if (hipEventSynchronize(r.b) != hipSuccess) bad = true;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) bad = true;
        Agg& a = agg[r.label];
        a.n += 1; a.ms += ms; a.flops += r.flops; a.bytes += r.bytes;
        g_pool.push_back(r.a);
        g_pool.push_back(r.b);
    }
    g_recs.clear();
    if (bad) return -1;
    std::string out = "[";
    bool first = true;
    char line[256];
    for (auto& kv : agg) {
        snprintf(line, sizeof(line), "%s{\"name\":\"%s\",\"launches\":%ld,\"ms\":%.6f,\"flops\":%.6e,\"bytes\":%.6e}",
                 first ? "" : ",", kv.first.c_str(), kv.second.n, kv.second.ms, kv.second.flops, kv.second.bytes);
        out += line;
        first = false;
    }
    out += "]";
    if (buf && cap) snprintf(buf, cap, "%s", out.c_str());
    return (long)out.size();
}

}  // namespace edl
