// Optional per-kernel timing with HIP events on the launching stream.
//
// When switched on, every kernel launch of the library is bracketed by two events recorded on
// the stream the kernel runs on; heta_profile_read waits for them and returns, per kernel
// name, the number of launches, the summed duration and the algorithmic bytes / flops the
// launch sites declared.  Off by default: the only cost then is one branch per launch.
#include <cstring>
#include <mutex>
#include <string>

#include "heta_internal.h"

namespace heta {

namespace {
struct Pending {
    int kernel;
    hipEvent_t start, stop;
    double bytes, flops;
};
struct Stat {
    std::string name;
    int64_t launches = 0;
    double ms = 0, bytes = 0, flops = 0;
};
std::mutex g_mu;
bool g_on = false;
std::vector<Pending> g_pending;
std::vector<hipEvent_t> g_pool;
std::vector<Stat> g_stats;

int kernel_id(const char *name)
{
    for (size_t i = 0; i < g_stats.size(); ++i)
        if (g_stats[i].name == name) return static_cast<int>(i);
    Stat s;
    s.name = name;
    g_stats.push_back(s);
    return static_cast<int>(g_stats.size()) - 1;
}

hipEvent_t get_event()
{
    if (!g_pool.empty()) {
        hipEvent_t e = g_pool.back();
        g_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void drain()
{
    for (auto &p : g_pending) {
        float ms = 0.f;
        if (hipEventSynchronize(p.stop) == hipSuccess && hipEventElapsedTime(&ms, p.start, p.stop) == hipSuccess) {
            Stat &s = g_stats[p.kernel];
            s.launches += 1;
            s.ms += ms;
            s.bytes += p.bytes;
            s.flops += p.flops;
        }
        g_pool.push_back(p.start);
        g_pool.push_back(p.stop);
    }
    g_pending.clear();
}
} // namespace

bool profiling_on() { return g_on; }

ProfScope::ProfScope(const char *name, hipStream_t st, double bytes, double flops) : active_(false), stream_(st)
{
    if (!g_on || !name) return; // a null name = a launch site that must not create events
    std::lock_guard<std::mutex> lk(g_mu);
    Pending p;
    p.kernel = kernel_id(name);
    p.start = get_event();
    p.stop = get_event();
    p.bytes = bytes;
    p.flops = flops;
    if (!p.start || !p.stop) return;
    if (hipEventRecord(p.start, st) != hipSuccess) return;
    g_pending.push_back(p);
    index_ = g_pending.size() - 1;
    active_ = true;
}

ProfScope::~ProfScope()
{
    if (!active_) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (index_ < g_pending.size()) (void)hipEventRecord(g_pending[index_].stop, stream_);
}

} // namespace heta

using namespace heta;

extern "C" {

heta_status heta_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = on != 0;
    return HETA_OK;
}

heta_status heta_profile_reset(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    drain();
    for (auto &s : g_stats) {
        s.launches = 0;
        s.ms = s.bytes = s.flops = 0;
    }
    return HETA_OK;
}

heta_status heta_profile_read(heta_kernel_stat *out, int32_t capacity, int32_t *n_out)
{
    if (!n_out || capacity < 0 || (capacity > 0 && !out))
        return fail(HETA_ERR_INVALID_ARG, "heta_profile_read: bad arguments");
    std::lock_guard<std::mutex> lk(g_mu);
    drain();
    int32_t n = 0;
    for (const auto &s : g_stats) {
        if (s.launches == 0) continue;
        if (n < capacity) {
            heta_kernel_stat &o = out[n];
            std::memset(&o, 0, sizeof o);
            std::strncpy(o.name, s.name.c_str(), sizeof(o.name) - 1);
            o.launches = s.launches;
            o.total_ms = s.ms;
            o.algorithmic_bytes = s.bytes;
            o.flops = s.flops;
        }
        ++n;
    }
    *n_out = n;
    return HETA_OK;
}

} // extern "C"
