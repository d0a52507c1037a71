// Optional per-kernel timing with HIP events (measurement only; see tt_profile_begin in the public header).
#include <hip/hip_runtime.h>
#include <vector>
#include "tt_internal.h"

namespace tt {
namespace {
struct Entry {
    tt_kernel_record rec;
    hipEvent_t start = nullptr, stop = nullptr;
};
struct State {
    bool on = false;
    bool failed = false;
    std::vector<Entry> entries;
};
thread_local State g_state;

void release(State &st)
{
    for (Entry &e : st.entries) {
        if (e.start) (void)hipEventDestroy(e.start);
        if (e.stop) (void)hipEventDestroy(e.stop);
        e.start = e.stop = nullptr;
    }
}
} // namespace

ProfileScope::ProfileScope(void *stream_, int kernel, int count, int64_t d0, int64_t d1, int64_t d2, uint64_t bytes,
                           uint64_t flops)
    : slot(-1), stream(stream_)
{
    State &st = g_state;
    if (!st.on) return;
    Entry e;
    e.rec.kernel = kernel;
    e.rec.count = count;
    e.rec.d0 = d0; e.rec.d1 = d1; e.rec.d2 = d2;
    e.rec.bytes = bytes;
    e.rec.flops = flops;
    e.rec.ms = 0.0f;
    if (hipEventCreate(&e.start) != hipSuccess || hipEventCreate(&e.stop) != hipSuccess ||
        hipEventRecord(e.start, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) {
        st.failed = true;
        if (e.start) (void)hipEventDestroy(e.start);
        if (e.stop) (void)hipEventDestroy(e.stop);
        return;
    }
    st.entries.push_back(e);
    slot = (int)st.entries.size() - 1;
}

ProfileScope::~ProfileScope()
{
    if (slot < 0) return;
    State &st = g_state;
    if (hipEventRecord(st.entries[slot].stop, reinterpret_cast<hipStream_t>(stream)) != hipSuccess) st.failed = true;
}
} // namespace tt

extern "C" tt_status tt_profile_begin(void)
{
    tt::State &st = tt::g_state;
    tt::release(st);
    st.entries.clear();
    st.failed = false;
    st.on = true;
    return TT_OK;
}

extern "C" tt_status tt_profile_end(int *n_records)
{
    tt::State &st = tt::g_state;
    st.on = false;
    bool ok = !st.failed;
    for (tt::Entry &e : st.entries) {
        if (hipEventSynchronize(e.stop) != hipSuccess || hipEventElapsedTime(&e.rec.ms, e.start, e.stop) != hipSuccess) ok = false;
    }
    tt::release(st);
    if (n_records) *n_records = (int)st.entries.size();
    return ok ? TT_OK : TT_EDEVICE;
}

extern "C" tt_status tt_profile_get(int index, tt_kernel_record *out)
{
    tt::State &st = tt::g_state;
    if (!out || index < 0 || index >= (int)st.entries.size()) return TT_EINVAL;
    *out = st.entries[index].rec;
    return TT_OK;
}
