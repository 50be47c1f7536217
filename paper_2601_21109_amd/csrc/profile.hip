// Optional per-kernel timing with HIP events, for benchmarks.  Off by default; when on, every
// launch of a tracked kernel is bracketed by an event pair recorded on the launch stream.
#include "common.h"

namespace cwl {
namespace {

constexpr int kPairs = 256;   // event pairs per slot; later launches reuse them round-robin

struct Slot {
    hipEvent_t start[kPairs], stop[kPairs];
    int64_t launches;
    bool made;
};

Slot g_slots[CWL_PROF_SLOTS];
bool g_on = false;

}  // namespace

void prof_begin(int slot, hipStream_t st) {
    if (!g_on) return;
    Slot& s = g_slots[slot];
    hipEventRecord(s.start[s.launches % kPairs], st);
}

void prof_end(int slot, hipStream_t st) {
    if (!g_on) return;
    Slot& s = g_slots[slot];
    hipEventRecord(s.stop[s.launches % kPairs], st);
    s.launches += 1;
}

}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_profile_enable(int32_t on) {
    if (on) {
        for (int i = 0; i < CWL_PROF_SLOTS; ++i) {
            Slot& s = g_slots[i];
            if (!s.made) {
                for (int p = 0; p < kPairs; ++p) {
                    if (hipEventCreate(&s.start[p]) != hipSuccess) return CWL_ERR_DEVICE;
                    if (hipEventCreate(&s.stop[p]) != hipSuccess) return CWL_ERR_DEVICE;
                }
                s.made = true;
            }
            s.launches = 0;
        }
    }
    g_on = on != 0;
    return CWL_OK;
}

extern "C" cwl_status cwl_profile_read(int32_t slot, double* total_ms, int64_t* launches) {
    if (slot < 0 || slot >= CWL_PROF_SLOTS || !total_ms || !launches) return CWL_ERR_INVALID_ARG;
    Slot& s = g_slots[slot];
    *total_ms = 0.0;
    *launches = 0;
    if (!s.made) return CWL_OK;
    const int64_t n = s.launches < kPairs ? s.launches : kPairs;
    for (int64_t p = 0; p < n; ++p) {
        if (hipEventSynchronize(s.stop[p]) != hipSuccess) return CWL_ERR_DEVICE;
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, s.start[p], s.stop[p]) != hipSuccess) return CWL_ERR_DEVICE;
        *total_ms += ms;
    }
    *launches = n;
    return CWL_OK;
}
