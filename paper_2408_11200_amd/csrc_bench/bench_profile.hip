// Per-kernel event timing for benchmarks (kan_bench.h): two launch hooks that bracket every kernel
// launch of the layer library with a pair of HIP events, and the read-out of the totals per kernel
// family.  This file belongs to the benchmark library, not to the layer library.
#include <hip/hip_runtime.h>
#include <string.h>
#include <vector>
#include "kan_bench.h"

namespace {
struct Record { const char *family; hipEvent_t e0, e1; bool closed; };
bool g_on = false;
std::vector<Record> g_records;
constexpr size_t kMaxRecords = 8192;
bool g_open = false;     // a "before" without its "after"

void clear()
{
    for (Record &r : g_records) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    g_records.clear();
    g_open = false;
}
}  // namespace

extern "C" void kan_profile_before(const char *family, void *stream)
{
    if (!g_on || g_records.size() >= kMaxRecords) return;
    Record r;
    r.family = family;
    r.closed = false;
    if (hipEventCreate(&r.e0) != hipSuccess) return;
    if (hipEventCreate(&r.e1) != hipSuccess) { (void)hipEventDestroy(r.e0); return; }
    (void)hipEventRecord(r.e0, (hipStream_t)stream);
    g_records.push_back(r);
    g_open = true;
}

extern "C" void kan_profile_after(const char *family, void *stream)
{
    (void)family;
    if (!g_open || g_records.empty()) return;
    (void)hipEventRecord(g_records.back().e1, (hipStream_t)stream);
    g_records.back().closed = true;
    g_open = false;
}

extern "C" int kan_profile_enable(int on)
{
    if (on) clear();
    g_on = on != 0;
    return KAN_OK;
}

extern "C" int kan_profile_read(kan_kernel_time *out, int capacity)
{
    if (capacity < 0 || (capacity > 0 && !out)) return KAN_ERR_INVALID_ARG;
    int n = 0;
    for (Record &r : g_records) {
        if (!r.closed) continue;
        if (hipEventSynchronize(r.e1) != hipSuccess) return KAN_ERR_HIP;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, r.e0, r.e1) != hipSuccess) return KAN_ERR_HIP;
        int at = -1;
        for (int q = 0; q < n && q < capacity; ++q)
            if (strcmp(out[q].name, r.family) == 0) { at = q; break; }
        if (at < 0) {
            if (n < capacity) { out[n].name = r.family; out[n].total_ms = 0.0; out[n].launches = 0; at = n; }
            ++n;
        }
        if (at >= 0) { out[at].total_ms += ms; out[at].launches += 1; }
    }
    return n;
}
