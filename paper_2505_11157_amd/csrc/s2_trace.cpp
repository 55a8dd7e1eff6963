// Per-launch timing for benchmarks: HIP events around each kernel launch, on the launch stream.
// Off by default; when off the hooks cost one branch.  Not thread safe (a benchmarking aid).
#include <atomic>
#include <vector>

#include "s2_internal.h"

namespace {

struct Entry {
    const char *name;
    double pairs;
    hipEvent_t start, stop;
};

bool g_enabled = false;
std::vector<Entry> g_entries;

}  // namespace

void s2_trace_begin(const char *name, double pairs, hipStream_t st)
{
    if (!g_enabled) return;
    Entry e{name, pairs, nullptr, nullptr};
    if (hipEventCreate(&e.start) != hipSuccess || hipEventCreate(&e.stop) != hipSuccess) return;
    (void)hipEventRecord(e.start, st);
    g_entries.push_back(e);
}

void s2_trace_end(hipStream_t st)
{
    if (!g_enabled || g_entries.empty()) return;
    (void)hipEventRecord(g_entries.back().stop, st);
}

extern "C" int s2_trace_enable(int on)
{
    const int prev = g_enabled ? 1 : 0;
    g_enabled = on != 0;
    return prev;
}

extern "C" void s2_trace_reset(void)
{
    for (auto &e : g_entries) {
        (void)hipEventDestroy(e.start);
        (void)hipEventDestroy(e.stop);
    }
    g_entries.clear();
}

extern "C" int s2_trace_count(void) { return int(g_entries.size()); }

extern "C" int s2_trace_get(int index, const char **name, float *ms, double *pairs)
{
    if (index < 0 || index >= int(g_entries.size())) return s2_fail(S2_ERR_INVALID_ARG, "trace index out of range");
    Entry &e = g_entries[index];
    if (hipEventSynchronize(e.stop) != hipSuccess) return s2_fail(S2_ERR_DEVICE, "trace event not recorded");
    float t = 0.f;
    if (hipEventElapsedTime(&t, e.start, e.stop) != hipSuccess) return s2_fail(S2_ERR_DEVICE, "trace event not recorded");
    if (name) *name = e.name;
    if (ms) *ms = t;
    if (pairs) *pairs = e.pairs;
    return S2_OK;
}

// Test-only dispatch switches (s2_debug_control in the C ABI).
namespace {
std::atomic<unsigned> g_debug{0u};
}

bool s2_debug_flag(unsigned bit) { return (g_debug.load(std::memory_order_relaxed) & bit) != 0; }

extern "C" unsigned s2_debug_control(unsigned set_bits, unsigned clear_bits)
{
    unsigned cur = g_debug.load(), next;
    do {
        next = (cur | set_bits) & ~clear_bits;
    } while (!g_debug.compare_exchange_weak(cur, next));
    return next;
}
