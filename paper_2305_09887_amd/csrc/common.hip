// Error reporting and version of libtma.
#include "common.hpp"

#include <mutex>
#include <string>
#include <vector>

namespace tma {

char *error_buffer()
{
    static thread_local char buf[512] = {0};
    return buf;
}

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(error_buffer(), 512, fmt, ap);
    va_end(ap);
    return code;
}

// ---- per-kernel event timing ------------------------------------------------
namespace {
struct Sample {
    std::string name;
    hipEvent_t start, stop;
};
struct Entry {
    std::string name;
    int64_t launches;
    double total_ms;
};
std::mutex g_mu;
bool g_on = false;
std::string g_filter;
std::vector<Sample> g_samples;
std::vector<Entry> g_entries;
std::vector<std::string> g_sequence;   // names of the timed launches of the last window, in launch order
}  // namespace

KernelTimer::KernelTimer(const char *name, hipStream_t stream) : slot_(-1), stream_(stream)
{
    if (!g_on) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_on) return;
    if (!g_filter.empty() && g_filter != name) return;
    Sample s;
    s.name = name;
    if (hipEventCreate(&s.start) != hipSuccess) return;
    if (hipEventCreate(&s.stop) != hipSuccess) {
        (void)hipEventDestroy(s.start);
        return;
    }
    (void)hipEventRecord(s.start, stream);
    g_samples.push_back(s);
    slot_ = int(g_samples.size()) - 1;
}

KernelTimer::~KernelTimer()
{
    if (slot_ < 0) return;
    std::lock_guard<std::mutex> lk(g_mu);
    if (slot_ < int(g_samples.size())) (void)hipEventRecord(g_samples[slot_].stop, stream_);
}

}  // namespace tma

extern "C" int tma_profile_begin(const char *kernel_filter)
{
    using namespace tma;
    std::lock_guard<std::mutex> lk(g_mu);
    for (auto &s : g_samples) {
        (void)hipEventDestroy(s.start);
        (void)hipEventDestroy(s.stop);
    }
    g_samples.clear();
    g_entries.clear();
    g_filter = kernel_filter ? kernel_filter : "";
    g_on = true;
    return TMA_OK;
}

extern "C" int tma_profile_end(void)
{
    using namespace tma;
    std::lock_guard<std::mutex> lk(g_mu);
    g_on = false;
    g_entries.clear();
    g_sequence.clear();
    int rc = TMA_OK;
    for (auto &s : g_samples) {
        g_sequence.push_back(s.name);
        float ms = 0.0f;
        hipError_t e = hipEventSynchronize(s.stop);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, s.start, s.stop);
        if (e != hipSuccess) {
            rc = fail(TMA_ERR_HIP, "tma_profile_end: %s", hipGetErrorString(e));
        } else {
            size_t i = 0;
            while (i < g_entries.size() && g_entries[i].name != s.name) ++i;
            if (i == g_entries.size()) g_entries.push_back(Entry{s.name, 0, 0.0});
            g_entries[i].launches += 1;
            g_entries[i].total_ms += double(ms);
        }
        (void)hipEventDestroy(s.start);
        (void)hipEventDestroy(s.stop);
    }
    g_samples.clear();
    return rc;
}

extern "C" int tma_profile_sequence_count(void)
{
    std::lock_guard<std::mutex> lk(tma::g_mu);
    return int(tma::g_sequence.size());
}

extern "C" int tma_profile_sequence_entry(int index, const char **name_out)
{
    using namespace tma;
    std::lock_guard<std::mutex> lk(g_mu);
    TMA_REQUIRE(index >= 0 && index < int(g_sequence.size()) && name_out, TMA_ERR_INVALID_ARG,
                "tma_profile_sequence_entry: index %d", index);
    *name_out = g_sequence[index].c_str();
    return TMA_OK;
}

extern "C" int tma_profile_count(void)
{
    std::lock_guard<std::mutex> lk(tma::g_mu);
    return int(tma::g_entries.size());
}

extern "C" int tma_profile_entry(int index, const char **name_out, int64_t *launches_out, double *total_ms_out)
{
    using namespace tma;
    std::lock_guard<std::mutex> lk(g_mu);
    TMA_REQUIRE(index >= 0 && index < int(g_entries.size()), TMA_ERR_INVALID_ARG, "tma_profile_entry: index %d", index);
    TMA_REQUIRE(name_out && launches_out && total_ms_out, TMA_ERR_INVALID_ARG, "tma_profile_entry: NULL argument");
    *name_out = g_entries[index].name.c_str();
    *launches_out = g_entries[index].launches;
    *total_ms_out = g_entries[index].total_ms;
    return TMA_OK;
}

extern "C" int tma_version(void) { return 100; }

extern "C" uint64_t tma_mix64(uint64_t seed, uint64_t unit) { return tma::splitmix64_at(seed, unit); }

extern "C" const char *tma_last_error(void) { return tma::error_buffer(); }
