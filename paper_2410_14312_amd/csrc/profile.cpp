// Per-kernel-class timing: when enabled, every launch of the stage executor is bracketed by two
// timing events on its own stream; tmps_profile_read() adds up the elapsed times per class.
#include "profile.h"

#include <mutex>
#include <vector>

#include "common.h"

namespace tmps {

namespace {
struct Span {
    int kc;
    hipEvent_t a, b;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Span> g_spans;
std::vector<hipEvent_t> g_free;
thread_local hipEvent_t t_open = nullptr;

hipEvent_t get_event() {
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    (void)hipEventCreate(&e);
    return e;
}
}  // namespace

bool profile_on() { return g_on; }

void profile_begin(int, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    t_open = get_event();
    if (t_open) (void)hipEventRecord(t_open, s);
}

void profile_end(int kc, hipStream_t s) {
    std::lock_guard<std::mutex> lk(g_mu);
    hipEvent_t b = get_event();
    if (b) (void)hipEventRecord(b, s);
    if (t_open && b) g_spans.push_back(Span{kc, t_open, b});
    t_open = nullptr;
}

bool profile_kernel_begin(KernelEvents& ev) {
    if (!g_on) return false;
    std::lock_guard<std::mutex> lk(g_mu);
    ev.start = get_event();
    ev.stop = get_event();
    return ev.start && ev.stop;
}

void profile_kernel_end(int kc, const KernelEvents& ev) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_spans.push_back(Span{kc, ev.start, ev.stop});
}

}  // namespace tmps

using namespace tmps;

extern "C" int tmps_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = on != 0;
    return TMPS_OK;
}

extern "C" int tmps_profile_read(double* total_ms, int64_t* launches, int n_classes) {
    if (!total_ms || !launches || n_classes < kcCount)
        return fail(TMPS_ECAP, "tmps_profile_read needs arrays of at least %d entries", (int)kcCount);
    std::lock_guard<std::mutex> lk(g_mu);
    for (int i = 0; i < n_classes; ++i) {
        total_ms[i] = 0.0;
        launches[i] = 0;
    }
    for (const Span& sp : g_spans) {
        TMPS_HIP(hipEventSynchronize(sp.b));
        float ms = 0.0f;
        TMPS_HIP(hipEventElapsedTime(&ms, sp.a, sp.b));
        total_ms[sp.kc] += ms;
        launches[sp.kc] += 1;
        g_free.push_back(sp.a);
        g_free.push_back(sp.b);
    }
    g_spans.clear();
    return kcCount;
}
