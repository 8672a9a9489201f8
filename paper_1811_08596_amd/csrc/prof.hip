// Optional per-kernel timing: when switched on, every launch made by the library is bracketed by two HIP
// events recorded on the launch stream, so a benchmark can read each kernel's average duration over its own
// timed region.  Off by default; when off a launch costs one predictable branch.
#include "internal.h"

#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

namespace fftsp {
namespace prof {
namespace {
struct Record {
    const char* name;
    hipEvent_t start, stop;
};
constexpr size_t kMaxRecords = 1 << 15;
bool g_on = false;
std::vector<Record> g_rec;            // used records
std::vector<hipEvent_t> g_pool;       // created events, reused across enable() calls
size_t g_pool_used = 0;
std::mutex g_mu;

hipEvent_t take_event()
{
    if (g_pool_used == g_pool.size()) {
        hipEvent_t e;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        g_pool.push_back(e);
    }
    return g_pool[g_pool_used++];
}
}  // namespace

bool enabled() { return g_on; }

int begin(const char* name, hipStream_t s)
{
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_rec.size() >= kMaxRecords) return -1;
    Record r{name, take_event(), take_event()};
    if (!r.start || !r.stop) return -1;
    (void)hipEventRecord(r.start, s);
    g_rec.push_back(r);
    return (int)g_rec.size() - 1;
}

void end(int id, hipStream_t s)
{
    if (id < 0) return;
    std::lock_guard<std::mutex> lock(g_mu);
    (void)hipEventRecord(g_rec[(size_t)id].stop, s);
}

void enable(bool on)
{
    std::lock_guard<std::mutex> lock(g_mu);
    g_on = on;
    g_rec.clear();
    g_pool_used = 0;
}

// "name calls total_ms" per line, in first-launch order
std::string report()
{
    (void)hipDeviceSynchronize();
    std::lock_guard<std::mutex> lock(g_mu);
    struct Acc {
        const char* name;
        long calls;
        double ms;
    };
    std::vector<Acc> acc;
    for (const Record& r : g_rec) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) continue;
        size_t i = 0;
        for (; i < acc.size(); ++i)
            if (std::strcmp(acc[i].name, r.name) == 0) break;
        if (i == acc.size()) acc.push_back(Acc{r.name, 0, 0.0});
        acc[i].calls += 1;
        acc[i].ms += ms;
    }
    std::string out;
    char line[256];
    for (const Acc& a : acc) {
        std::snprintf(line, sizeof line, "%s %ld %.6f\n", a.name, a.calls, a.ms);
        out += line;
    }
    return out;
}

}  // namespace prof
}  // namespace fftsp
