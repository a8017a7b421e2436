// Status strings and per-kernel event timing of libsdp_hip.so.
#include <atomic>
#include <map>
#include <mutex>
#include <string>
#include <vector>

#include "sdp_internal.h"

namespace sdp {
namespace {

struct Pending {
    const char* name;
    hipEvent_t start, stop;
};

std::mutex g_mu;
std::atomic<bool> g_on{false}; // read on every launch without the lock
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_free;
std::map<std::string, std::pair<int64_t, double>> g_totals; // name -> (calls, ms)
std::vector<const char*> g_names;                            // insertion order, static strings
std::string g_filter;                                        // empty = every kernel

hipEvent_t take_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}

// fold finished launches into the totals; waits for each stop event
void drain_locked() {
    for (Pending& p : g_pending) {
        float ms = 0.f;
        if (p.start && p.stop && hipEventSynchronize(p.stop) == hipSuccess &&
            hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            auto it = g_totals.find(p.name);
            if (it == g_totals.end()) {
                g_names.push_back(p.name);
                it = g_totals.emplace(p.name, std::make_pair((int64_t)0, 0.0)).first;
            }
            it->second.first += 1;
            it->second.second += ms;
        }
        if (p.start) g_free.push_back(p.start);
        if (p.stop) g_free.push_back(p.stop);
    }
    g_pending.clear();
}

} // namespace

bool profiling_on() { return g_on.load(std::memory_order_relaxed); }

bool profiling_wants(const char* name) {
    if (!profiling_on()) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    return g_filter.empty() || g_filter == name;
}

// For launches that carry their own start / stop events (hipExtLaunchKernel): hands out the pair and files it
// with the pending launches; false when this kernel is not being timed.
bool profile_launch_events(const char* name, hipEvent_t* start, hipEvent_t* stop) {
    if (!profiling_on() || !profiling_wants(name)) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    Pending p{name, take_event(), take_event()};
    if (!p.start || !p.stop) {
        if (p.start) g_free.push_back(p.start);
        if (p.stop) g_free.push_back(p.stop);
        return false;
    }
    g_pending.push_back(p);
    *start = p.start, *stop = p.stop;
    return true;
}

void profile_begin(const char* name, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    Pending p{name, take_event(), take_event()};
    if (p.start) (void)hipEventRecord(p.start, s);
    g_pending.push_back(p);
}

void profile_end(hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_pending.empty()) return;
    Pending& p = g_pending.back();
    if (p.stop) (void)hipEventRecord(p.stop, s);
}

} // namespace sdp

extern "C" const char* sdp_status_string(int status) {
    switch (status) {
    case SDP_OK: return "ok";
    case SDP_ERR_INVALID_ARG: return "invalid argument";
    case SDP_ERR_SHAPE: return "inconsistent or unsupported shape";
    case SDP_ERR_WORKSPACE: return "workspace missing or too small";
    case SDP_ERR_UNCOVERED: return "coverage impossible: K * p < F";
    case SDP_ERR_UNSUPPORTED: return "unsupported combination";
    case SDP_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

extern "C" int sdp_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(sdp::g_mu);
    sdp::g_on.store(on != 0, std::memory_order_relaxed);
    return SDP_OK;
}

extern "C" int sdp_profile_filter(const char* name) {
    std::lock_guard<std::mutex> lk(sdp::g_mu);
    sdp::g_filter = name ? name : "";
    return SDP_OK;
}

extern "C" int sdp_profile_reset(void) {
    std::lock_guard<std::mutex> lk(sdp::g_mu);
    sdp::drain_locked();
    sdp::g_totals.clear();
    sdp::g_names.clear();
    return SDP_OK;
}

extern "C" int sdp_profile_read(int cap, const char** names, int64_t* calls, double* ms) {
    if (cap < 0 || (cap > 0 && (!names || !calls || !ms))) return SDP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(sdp::g_mu);
    sdp::drain_locked();
    int n = 0;
    for (const char* nm : sdp::g_names) {
        if (n >= cap) break;
        const auto& t = sdp::g_totals[nm];
        names[n] = nm;
        calls[n] = t.first;
        ms[n] = t.second;
        ++n;
    }
    return n;
}
