// Optional per-kernel timing with HIP events, for benchmarks.  Off by default; when a slot is on,
// every launch of its kernel is bracketed by an event pair recorded on the launch stream.  An event
// record between two kernels costs idle time on the stream, hence the per-slot mask.
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
uint32_t g_mask = 0;          // bit i: slot i records

}  // namespace

void prof_begin(int slot, hipStream_t st) {
    if (!(g_mask >> slot & 1u)) return;
    Slot& s = g_slots[slot];
    (void)hipEventRecord(s.start[s.launches % kPairs], st);   // measurement aid: a failed record shows as a failed read
}

void prof_end(int slot, hipStream_t st) {
    if (!(g_mask >> slot & 1u)) return;
    Slot& s = g_slots[slot];
    (void)hipEventRecord(s.stop[s.launches % kPairs], st);
    s.launches += 1;
}

}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_profile_enable(int32_t slot_mask) {
    if (slot_mask < 0 || slot_mask >= (1 << CWL_PROF_SLOTS)) return CWL_ERR_INVALID_ARG;
    if (slot_mask) {
        for (int i = 0; i < CWL_PROF_SLOTS; ++i) {
            Slot& s = g_slots[i];
            if (!s.made) {
                for (int p = 0; p < kPairs; ++p) {
                    // timing only: without the system-scope fence a recorded event would otherwise
                    // put between two kernels
                    if (hipEventCreateWithFlags(&s.start[p], hipEventDisableSystemFence) != hipSuccess) return CWL_ERR_DEVICE;
                    if (hipEventCreateWithFlags(&s.stop[p], hipEventDisableSystemFence) != hipSuccess) return CWL_ERR_DEVICE;
                }
                s.made = true;
            }
            s.launches = 0;
        }
    }
    g_mask = (uint32_t)slot_mask;
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
