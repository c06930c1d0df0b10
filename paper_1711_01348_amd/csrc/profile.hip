#include "profile.h"

#include <atomic>
#include <cstring>
#include <mutex>
#include <vector>

#include "../../include/tad.h"

namespace tad {

static std::mutex g_mu;
static char g_name[64] = {0};
static std::atomic<bool> g_armed{false};
static std::vector<hipEvent_t> g_start, g_stop;
static int g_used = 0, g_seen = 0, g_every = 1;
static const int kMaxLaunches = 4096;

ProfileScope::ProfileScope(const char *name) : start(nullptr), stop(nullptr) {
    if (!g_armed) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_armed || std::strcmp(name, g_name) != 0 || g_used >= kMaxLaunches) return;
    if (g_seen++ % g_every != 0) return;
    start = g_start[g_used];
    stop = g_stop[g_used];
    ++g_used;
}

}  // namespace tad

using namespace tad;

extern "C" {

int tad_profile_begin(const char *kernel_name, int every) {
    if (!kernel_name || std::strlen(kernel_name) >= sizeof g_name || every < 1) return TAD_EINVAL;
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_start.empty()) {
        g_start.resize(kMaxLaunches);
        g_stop.resize(kMaxLaunches);
        for (int i = 0; i < kMaxLaunches; ++i) {
            if (hipEventCreate(&g_start[i]) != hipSuccess || hipEventCreate(&g_stop[i]) != hipSuccess) {
                g_start.clear();
                g_stop.clear();
                return TAD_EDEVICE;
            }
        }
    }
    std::strcpy(g_name, kernel_name);
    g_used = 0;
    g_seen = 0;
    g_every = every;
    g_armed = true;
    return TAD_OK;
}

int tad_profile_end(double *total_ms, int *launches) {
    if (!total_ms || !launches) return TAD_EINVAL;
    std::lock_guard<std::mutex> lk(g_mu);
    g_armed = false;
    double sum = 0.0;
    for (int i = 0; i < g_used; ++i) {
        float ms = 0.f;
        if (hipEventSynchronize(g_stop[i]) != hipSuccess) return TAD_EDEVICE;
        if (hipEventElapsedTime(&ms, g_start[i], g_stop[i]) != hipSuccess) return TAD_EDEVICE;
        sum += ms;
    }
    *total_ms = sum;
    *launches = g_used;
    g_used = 0;
    return TAD_OK;
}

}  // extern "C"
