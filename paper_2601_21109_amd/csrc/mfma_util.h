// Small device helpers shared by the bf16 matrix-core kernels (gfx950 only).
#pragma once
#include "linear_common.h"

namespace cwl {
namespace mfma {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// One wave-wide 1 KiB global -> LDS transfer: lane l's 16 bytes land at lds_wave_base + 16 l.
__device__ __forceinline__ void load_lds_16(const void* gptr, char* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)gptr,
        (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// s_waitcnt with explicit counts (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] |
// vmcnt[5:4] at [15:14]); expcnt is left at its maximum.
template <int VM, int LGKM>
__device__ __forceinline__ void wait_cnt() {
    static_assert(VM >= 0 && VM < 64 && LGKM >= 0 && LGKM < 16, "counter range");
    __builtin_amdgcn_s_waitcnt((VM & 15) | (7 << 4) | ((LGKM & 15) << 8) | ((VM >> 4) << 14));
}

// Workgroup id -> (row tile, column tile).  Consecutive workgroup ids go round-robin over the 8
// XCDs, each with its own L2, so XCD x is given the x-th contiguous eighth of a tile order in
// which GROUP_M row tiles sweep all column tiles before moving on: the 32 tiles in flight on one
// XCD form an 8 x 4 patch that shares 8 x panels and 4 weight panels.
// (wg: the workgroup's index among those of the GEMM; a launch may carry other workgroups in front)
__device__ __forceinline__ bool tile_coords(int64_t wg, int tiles_m, int tiles_n, int* bm, int* bn) {
    constexpr int kXcd = 8, GROUP_M = 8;
    const int64_t n_tiles = (int64_t)tiles_m * tiles_n;
    const int64_t per_xcd = (n_tiles + kXcd - 1) / kXcd;
    const int64_t tile = (wg % kXcd) * per_xcd + wg / kXcd;
    if (tile >= n_tiles) return false;
    const int64_t band_size = (int64_t)GROUP_M * tiles_n;
    const int64_t band = tile / band_size;
    const int64_t in_band = tile % band_size;
    const int64_t first_m = band * GROUP_M;
    const int64_t gm = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    *bm = (int)(first_m + in_band % gm);
    *bn = (int)(in_band / gm);
    return true;
}

}  // namespace mfma
}  // namespace cwl
