// bf16 matrix-core path of cwl_chunkwise_lora_linear (see linear_common.h for the formulation).
//
// One "TN" GEMM kernel, C[m, n] = sum_k A[m, k] B[n, k], both operands K-contiguous, is used
// twice: as the shrink (A = x, B = A^T, epilogue multiplies by the gate and writes uhat) and as
// the main product over the concatenated reduction dimension [x | uhat] . [W^T | B^T]^T, where a
// row tile only walks ceil(r_tile / 16) MFMA steps of the second part.
//
// Data path (gfx950): global -> LDS with global_load_lds_dwordx4 (no staging registers), two
// LDS stages of BK = 64; LDS rows are 128 bytes with the 16-byte chunk index XOR-swizzled by
// (row / 2) % 8 so that ds_read_b128 of 16 consecutive rows touches 16 distinct bank groups;
// v_mfma_f32_32x32x16_bf16 with fp32 accumulators.  The weight fragment is the MFMA's first
// operand, so each lane ends up with 4 consecutive output columns of one row and stores 8 bytes.
#include "linear_common.h"

namespace cwl {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int BK = 64;            // elements of K per LDS stage
constexpr int ROW_BYTES = BK * 2;  // 128

__device__ __forceinline__ void load_lds_16(const void* gptr, char* lds_wave_base) {
    __builtin_amdgcn_global_load_lds(
        (const __attribute__((address_space(1))) void*)gptr,
        (__attribute__((address_space(3))) void*)lds_wave_base, 16, 0, 0);
}

// Workgroup id -> (row tile, column tile).  Consecutive workgroup ids go round-robin over the 8
// XCDs, each with its own L2, so XCD x is given the x-th contiguous eighth of a tile order in
// which GROUP_M row tiles sweep all column tiles before moving on: the tiles in flight on one
// XCD share a few x panels and walk the same weight panels.
__device__ __forceinline__ bool tile_coords(int tiles_m, int tiles_n, int* bm, int* bn) {
    constexpr int kXcd = 8, GROUP_M = 8;
    const int64_t n_tiles = (int64_t)tiles_m * tiles_n;
    const int64_t per_xcd = (n_tiles + kXcd - 1) / kXcd;
    const int64_t wg = blockIdx.x;
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

template <int BM, int BN, int WM, int WN, int EPI>
__global__ void __launch_bounds__(WM * WN * 64) gemm_bf16_tn_kernel(GemmArgs a) {
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;     // wave tile
    constexpr int MI = TM / 32, NI = TN / 32;     // 32x32 MFMA blocks per wave tile
    constexpr int ROWS = BM + BN;
    constexpr int LOADS = ROWS / 8 / NW;          // 1 KiB load instructions per wave per stage
    constexpr int STAGE_BYTES = ROWS * ROW_BYTES;
    static_assert(ROWS % (8 * NW) == 0, "tile rows must split evenly over the waves");
    static_assert(BM % 16 == 0 && BN % 16 == 0 && TM % 32 == 0 && TN % 32 == 0, "tile shape");
    static_assert(BM % kRankBlock == 0, "row tile must cover whole rank blocks");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int bm, bn;
    if (!tile_coords(a.tiles_m, a.tiles_n, &bm, &bn)) return;
    const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // largest effective rank among the rows of this tile
    int32_t r_tile = 0;
    if (a.blk_r) {
        const int64_t n_blk = (a.M + kRankBlock - 1) / kRankBlock;
#pragma unroll
        for (int i = 0; i < BM / kRankBlock; ++i) {
            const int64_t blk = m0 / kRankBlock + i;
            if (blk < n_blk) {
                const int32_t r = a.blk_r[blk];
                r_tile = r > r_tile ? r : r_tile;
            }
        }
    }
    // ---- loader set-up: instruction j of this wave fills rows 8j .. 8j+7 of the stage ----
    const __bf16* gp[LOADS];          // current global address of this lane's 16 bytes
    int32_t grow[LOADS];              // row in the second operand pair (grouped row / column)
    int lchunk[LOADS];
    bool is_a[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int j = wave * LOADS + i;
        const int row_cat = 8 * j + (lane >> 3);
        is_a[i] = (8 * j) < BM;                       // wave-uniform
        const int r = is_a[i] ? row_cat : row_cat - BM;
        lchunk[i] = (lane & 7) ^ ((r >> 1) & 7);
        if (is_a[i]) {
            int64_t g = m0 + r;
            if (g > a.M - 1) g = a.M - 1;
            grow[i] = (int32_t)g;
            const int64_t t = a.perm ? (int64_t)a.perm[g] : g;
            gp[i] = static_cast<const __bf16*>(a.A1) + t * a.lda1 + lchunk[i] * 8;
        } else {
            int64_t n = n0 + r;
            if (n > a.N - 1) n = a.N - 1;
            grow[i] = (int32_t)n;
            gp[i] = static_cast<const __bf16*>(a.B1) + n * a.ldb1 + lchunk[i] * 8;
        }
    }

    auto issue_loads = [&](int stage) {
        char* base = smem + stage * STAGE_BYTES + wave * LOADS * 1024;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            load_lds_16(gp[i], base + i * 1024);
            gp[i] += BK;
        }
    };

    // ---- fragment addressing ----
    const int l32 = lane & 31, h = lane >> 5;
    const int sw = (l32 >> 1) & 7;
    int koff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = ((2 * kk + h) ^ sw) * 16;
    const int a_base = (wm * TM + l32) * ROW_BYTES;
    const int b_base = BM * ROW_BYTES + (wn * TN + l32) * ROW_BYTES;

    f32x16 acc[NI][MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.0f;

    // shrink: output columns (adapter directions) at or beyond the block's largest effective rank
    // are gated to zero anyway, so their MFMAs are skipped; a rank-0 block skips the whole loop
    bool ni_on[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) ni_on[ni] = true;
    int KS = a.K1 / BK;                               // stages of the first part
    if (EPI == EPI_GATE && a.gate_blk_r) {
        const int32_t r_blk = a.gate_blk_r[m0 / kRankBlock];
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) ni_on[ni] = (wn * TN + ni * 32) < r_blk;
        if (r_blk == 0) KS = 0;
    }
    const int TS = (r_tile + BK - 1) / BK;            // stages of the second part
    const int S = KS + TS;
    const int last_steps = (r_tile - (TS - 1) * BK + 15) / 16;   // MFMA k-steps of the last stage

    auto compute = [&](int stage, int steps) {
        const char* sb = smem + stage * STAGE_BYTES;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            if (kk < steps) {   // steps is 4 (a constant after inlining) except in the last stage
                bf16x8 af[MI], bfr[NI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    af[mi] = *reinterpret_cast<const bf16x8*>(sb + a_base + mi * 32 * ROW_BYTES + koff[kk]);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    bfr[ni] = *reinterpret_cast<const bf16x8*>(sb + b_base + ni * 32 * ROW_BYTES + koff[kk]);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    if (ni_on[ni])
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
                            acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ni], af[mi], acc[ni][mi], 0, 0, 0);
            }
        }
    };

    // ---- main loop: two LDS stages, loads of stage s+1 overlap the MFMAs of stage s ----
    // Only the last stage of the second part can be partial; it is peeled off the loop.
    const int n_full = (TS > 0) ? S - 1 : S;
    if (S > 0) issue_loads(0);
    for (int s = 0; s < n_full; ++s) {
        __syncthreads();   // waits for this wave's loads, then for everyone's
        if (s + 1 < S) {
            if (s + 1 == KS) {
                // switch the loaders to the second operand pair (uhat, B^T)
#pragma unroll
                for (int i = 0; i < LOADS; ++i) {
                    if (is_a[i])
                        gp[i] = static_cast<const __bf16*>(a.A2) + (int64_t)grow[i] * a.lda2 + lchunk[i] * 8;
                    else
                        gp[i] = static_cast<const __bf16*>(a.B2) + (int64_t)grow[i] * a.ldb2 + lchunk[i] * 8;
                }
            }
            issue_loads((s + 1) & 1);
        }
        compute(s & 1, 4);
    }
    if (TS > 0) {
        __syncthreads();
        compute((S - 1) & 1, last_steps);
    }

    // ---- epilogue ----
    // accumulator register v of block (ni, mi): column n = ni*32 + 8*(v/4) + 4*h + v%4,
    // row m = mi*32 + l32 (relative to the wave tile)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int64_t g = m0 + wm * TM + mi * 32 + l32;
        if (g >= a.M) continue;
        const int64_t t = a.perm ? (int64_t)a.perm[g] : g;
        TokMeta mt = {0, 0, 0.0f, 0.0f};
        if (EPI == EPI_GATE) mt = a.meta[t];
        __bf16* crow = static_cast<__bf16*>(a.C) + (EPI == EPI_GATE ? g : t) * a.ldc;
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int64_t n = n0 + wn * TN + ni * 32 + q * 8 + h * 4;
                if (n >= a.N) continue;     // N is a multiple of 8: the 4 columns are in or out together
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    float v = acc[ni][mi][q * 4 + e];
                    if (EPI == EPI_GATE) {
                        const int32_t i = (int32_t)n + e;
                        const float gate = (i < mt.r_prev ? mt.g_prev : 0.0f) + (i < mt.r_cur ? mt.g_cur : 0.0f);
                        v *= gate;
                    }
                    o[e] = (__bf16)v;
                }
                *reinterpret_cast<bf16x4*>(crow + n) = o;
            }
        }
    }
}

template <int BM, int BN, int WM, int WN, int EPI>
cwl_status launch_cfg(GemmArgs a, hipStream_t st) {
    constexpr int smem_bytes = 2 * (BM + BN) * ROW_BYTES;
    auto kern = gemm_bf16_tn_kernel<BM, BN, WM, WN, EPI>;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                hipFuncAttributeMaxDynamicSharedMemorySize, smem_bytes) != hipSuccess)
            return CWL_ERR_DEVICE;
        attr_set = true;
    }
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t n_tiles = (int64_t)a.tiles_m * a.tiles_n;
    if (n_tiles <= 0) return CWL_OK;
    const int64_t grid = (n_tiles + 7) / 8 * 8;
    if (grid >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    kern<<<dim3((unsigned)grid), dim3(WM * WN * 64), smem_bytes, st>>>(a);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace

cwl_status launch_shrink_bf16(const GemmArgs& a, hipStream_t st) {
    switch (a.N) {
        case 64: return launch_cfg<64, 64, 2, 2, EPI_GATE>(a, st);
        case 128: return launch_cfg<64, 128, 2, 2, EPI_GATE>(a, st);
        case 192: return launch_cfg<64, 192, 2, 2, EPI_GATE>(a, st);
        case 256: return launch_cfg<64, 256, 2, 2, EPI_GATE>(a, st);
        default: return CWL_ERR_UNSUPPORTED;
    }
}

cwl_status launch_main_bf16(const GemmArgs& a, hipStream_t st) {
    return launch_cfg<256, 256, 2, 4, EPI_STORE>(a, st);
}

}  // namespace cwl
