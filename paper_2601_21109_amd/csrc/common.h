// Shared host/device helpers of the ChunkWise LoRA HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cwl.h"

#define CWL_RETURN_IF_LAUNCH_FAILED()                        \
    do {                                                     \
        if (hipGetLastError() != hipSuccess) return CWL_ERR_DEVICE; \
    } while (0)

namespace cwl {

constexpr int kWave = 64;                 // CDNA wavefront width
constexpr int32_t kQMax = 1 << 20;        // clamp of a quantised score
constexpr int64_t kQThresholdMax = 1 << 21;  // clamp of a quantised threshold: never reachable

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Set-once launch state (a kernel's dynamic-LDS limit, the number of compute units, the address of
// a device symbol) belongs to a (kernel, device) pair, so it is remembered per device, indexed by
// the current device's ordinal.  Not synchronised: two host threads that make the first call on a
// device at the same moment both do the same idempotent set-up.
constexpr int kMaxDevices = 64;

inline int device_slot() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

struct PerDeviceFlag {
    bool done[kMaxDevices] = {};
};

// raises a kernel's dynamic shared-memory limit on the current device, the first time it is asked to
inline cwl_status ensure_dynamic_lds(const void* kernel, int bytes, PerDeviceFlag& flag) {
    const int dev = device_slot();
    if (dev < 0) return CWL_ERR_DEVICE;
    if (!flag.done[dev]) {
        if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes) != hipSuccess)
            return CWL_ERR_DEVICE;
        flag.done[dev] = true;
    }
    return CWL_OK;
}

// Score -> Q10 fixed-point nats, q = floor(h*1024 + 0.5) in fp32.  h*1024 is exact, so a fused
// multiply-add gives the same value as a separate multiply and add.
__host__ __device__ inline int32_t quantise_score(float h, bool* is_nan) {
    if (h != h) {
        *is_nan = true;
        return 0;
    }
    if (!(h > 0.0f)) return 0;
    float f = floorf(h * 1024.0f + 0.5f);
    if (f >= (float)kQMax) return kQMax;
    return (int32_t)f;
}

inline int64_t quantise_threshold(float h) {
    if (h != h) return kQThresholdMax;
    if (!(h > 0.0f)) return 0;
    float f = floorf(h * 1024.0f + 0.5f);
    if (f >= (float)kQThresholdMax) return kQThresholdMax;
    return (int64_t)f;
}

// the selector's thresholds, quantised like the scores (kernel argument)
struct TauTable {
    int64_t tau_q[CWL_MAX_LADDER];
};

// K-1 ascending thresholds in nats -> table; CWL_ERR_INVALID_ARG for NaN or descending entries
inline cwl_status fill_tau_table(const float* thresholds, int32_t K, TauTable* t) {
    *t = TauTable{};
    for (int32_t j = 0; j < K - 1; ++j) {
        if (thresholds[j] != thresholds[j]) return CWL_ERR_INVALID_ARG;
        if (j > 0 && thresholds[j] < thresholds[j - 1]) return CWL_ERR_INVALID_ARG;
        t->tau_q[j] = quantise_threshold(thresholds[j]);
    }
    return CWL_OK;
}

// length bounds of the chunker
inline cwl_status check_chunk_params(const cwl_chunk_params* p) {
    if (!p) return CWL_ERR_NULL;
    if (p->l_min < 1 || p->l_max < p->l_min) return CWL_ERR_INVALID_ARG;
    if ((int64_t)p->l_max < 2 * (int64_t)p->l_min - 1) return CWL_ERR_INFEASIBLE;
    return CWL_OK;
}

// sequence b: validated (first row, length); a malformed entry yields length 0
__device__ __forceinline__ void seq_extent(const int32_t* seq_offsets, int32_t b, int64_t n_rows,
                                           int64_t* base, int64_t* T, bool* bad) {
    const int64_t s = seq_offsets[b], e = seq_offsets[b + 1];
    if (s < 0 || e < s || e > n_rows) {
        *bad = true;
        *base = 0;
        *T = 0;
    } else {
        *base = s;
        *T = e - s;
    }
}

// 64-bit integers through the 32-bit wavefront shuffles
__device__ __forceinline__ int64_t shfl_up_i64(int64_t v, int delta) {
    int lo = __shfl_up((int)(v & 0xffffffffll), delta);
    int hi = __shfl_up((int)(v >> 32), delta);
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

// sum over the 64 lanes of a wavefront; every lane gets the result
__device__ __forceinline__ int64_t wave_sum_i64(int64_t v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int lo = __shfl_xor((int)(v & 0xffffffffll), off);
        int hi = __shfl_xor((int)(v >> 32), off);
        v += ((int64_t)hi << 32) | (uint32_t)lo;
    }
    return v;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t bits16) {
    return __uint_as_float(bits16 << 16);
}

// optional event timing around tracked kernels (profile.hip); no-ops unless enabled
void prof_begin(int slot, hipStream_t st);
void prof_end(int slot, hipStream_t st);

// cwl_partition_chunks with the path chosen from a caller-supplied average sequence length
cwl_status partition_chunks_avg_len(const float* entropy, int64_t n_rows, const int32_t* seq_offsets,
                                    int32_t n_seqs, const cwl_chunk_params* p, int32_t* chunk_offsets,
                                    int32_t* chunk_start, int32_t* chunk_len, int64_t* chunk_sum, int32_t cap,
                                    int32_t* status_word, void* workspace, size_t workspace_bytes, void* stream,
                                    int64_t avg_len);

}  // namespace cwl
