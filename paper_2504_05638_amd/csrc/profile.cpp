// Optional per-kernel timing with HIP events on the caller's stream, plus cached device
// properties.  Events are host-side objects: nothing here allocates device memory.
#include <string.h>

#include <atomic>
#include <mutex>
#include <vector>

#include "tagc_internal.h"

namespace tagc {

namespace {

struct Rec {
    const char *name;
    hipEvent_t a, b;
};

std::mutex g_mu;
bool g_on = false;
std::vector<Rec> g_recs;
std::vector<hipEvent_t> g_free;
Rec g_open{nullptr, nullptr, nullptr};

hipEvent_t get_event()
{
    if (!g_free.empty()) {
        hipEvent_t e = g_free.back();
        g_free.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

}  // namespace

void profile_begin(const char *name, hipStream_t s)
{
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    g_open.name = name;
    g_open.a = get_event();
    g_open.b = get_event();
    if (g_open.a) (void)hipEventRecord(g_open.a, s);
}

void profile_end(hipStream_t s)
{
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_open.name) return;
    if (g_open.b) (void)hipEventRecord(g_open.b, s);
    if (g_open.a && g_open.b) g_recs.push_back(g_open);
    g_open = Rec{nullptr, nullptr, nullptr};
}

int device_cu_count()
{
    static int cached[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess ||
            n <= 0)
            n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}

}  // namespace tagc

using namespace tagc;

extern "C" int tagc_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = on != 0;
    return TAGC_OK;
}

extern "C" int tagc_profile_read(const char **names, double *total_ms, uint64_t *launches,
                                 uint32_t cap)
{
    std::lock_guard<std::mutex> lk(g_mu);
    uint32_t n = 0;
    int rc = TAGC_OK;
    for (Rec &r : g_recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess ||
            hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess)
            rc = TAGC_EHIP;
        g_free.push_back(r.a);
        g_free.push_back(r.b);
        uint32_t i = 0;
        for (; i < n; ++i)
            if (names && names[i] == r.name) break;
        if (i == n) {
            if (n >= cap || !names || !total_ms || !launches) continue;
            names[n] = r.name;
            total_ms[n] = 0.0;
            launches[n] = 0;
            ++n;
        }
        total_ms[i] += ms;
        launches[i] += 1;
    }
    g_recs.clear();
    return rc ? rc : int(n);
}
