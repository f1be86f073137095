// Per-kernel timing with HIP events on the launch stream (l2a_profile_enable / l2a_profile_read).
#include <atomic>
#include <mutex>
#include <vector>

#include "common.hpp"

namespace l2a {
namespace {
struct Record {
    const char* name;
    hipEvent_t start, stop;
};
std::mutex g_mu;  // guards the log and the event pool
std::atomic<bool> g_enabled{false};
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

// begin/end bracket one launch on one thread.  While timing is on, the lock is held from begin to
// end, so that the record at the back of the log is still this launch's when its stop event is
// recorded; while it is off (the normal case) neither takes the lock.
bool profile_begin(const char* name, hipStream_t st) {
    if (!g_enabled.load(std::memory_order_relaxed)) return false;
    g_mu.lock();
    Record r{name, get_event(), get_event()};
    (void)hipEventRecord(r.start, st);
    g_log.push_back(r);
    return true;
}

void profile_end(hipStream_t st) {
    (void)hipEventRecord(g_log.back().stop, st);
    g_mu.unlock();
}
}  // namespace l2a

extern "C" {
void l2a_profile_enable(int on) {
    l2a::g_enabled.store(on != 0);
}

int l2a_profile_read(l2a_kernel_time* out, int max) {
    using namespace l2a;
    std::lock_guard<std::mutex> lock(g_mu);
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
