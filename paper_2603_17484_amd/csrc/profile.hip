// Per-kernel timing with HIP events on the launch stream (l2a_profile_enable / l2a_profile_read).
#include <vector>

#include "common.hpp"

namespace l2a {
namespace {
struct Record {
    const char* name;
    hipEvent_t start, stop;
};
bool g_enabled = false;
std::vector<Record> g_log;
std::vector<hipEvent_t> g_pool;

hipEvent_t get_event() {
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

void profile_begin(const char* name, hipStream_t st) {
    if (!g_enabled) return;
    Record r{name, get_event(), get_event()};
    (void)hipEventRecord(r.start, st);
    g_log.push_back(r);
}

void profile_end(hipStream_t st) {
    if (!g_enabled || g_log.empty()) return;
    (void)hipEventRecord(g_log.back().stop, st);
}
}  // namespace l2a

extern "C" {
void l2a_profile_enable(int on) { l2a::g_enabled = on != 0; }

int l2a_profile_read(l2a_kernel_time* out, int max) {
    using namespace l2a;
    const int n = (int)g_log.size();
    for (int i = 0; i < n; ++i) {
        float ms = 0.f;
        (void)hipEventSynchronize(g_log[i].stop);
        (void)hipEventElapsedTime(&ms, g_log[i].start, g_log[i].stop);
        if (out && i < max) {
            out[i].name = g_log[i].name;
            out[i].ms = ms;
        }
        g_pool.push_back(g_log[i].start);
        g_pool.push_back(g_log[i].stop);
    }
    g_log.clear();
    return n;
}
}
