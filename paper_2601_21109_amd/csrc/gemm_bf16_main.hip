// Main bf16 product of cwl_chunkwise_lora_linear: y = [x | uhat] . [W^T | B^T]^T (see
// linear_common.h for the formulation), one 256 x 256 output tile per workgroup of 4 waves.
//
// Design (gfx950), with the measurements that led to it:
//   * Four waves, one per SIMD, each owning a 128 x 128 quarter of the tile: a k-step of 32 needs
//     16 fragment reads (ds_read_b128) for 64 MFMAs, a third less LDS traffic than eight waves of
//     128 x 64.  v_mfma_f32_16x16x32_bf16 with the 256 fp32 accumulators in AGPRs; on this
//     power-limited part the 16x16x32 shape sustained a higher clock than 32x32x16 on the same data.
//   * A stage covers 64 elements of the reduction dimension, so every global_load_lds_dwordx4
//     fetches whole 128-byte lines (8 rows x 128 B per instruction).  The x half and the weight
//     half of a stage are separate 32 KiB "slots"; five slots form the ring (160 KiB, all of a
//     compute unit's LDS): two are being consumed, three are in flight.  After the barrier that
//     retires stage s the two buffers it held take the weight half of stage s+2 and then the x
//     half of stage s+3.
//   * Load instructions are never issued as a burst.  The address unit takes one 64-lane
//     instruction every ~18 cycles and a wave stays in issue until its loads are taken; bursts
//     after the barrier held the MFMAs back for more than a thousand cycles per stage.  Here
//     every load sits between MFMAs (one per six), as do the LDS reads (two per MFMA at the
//     start of a k-step), by way of sched_group_barrier.
//   * Loads use a scalar base plus a 32-bit lane offset, so the reduction loop advances two
//     scalar pointers and does no vector address arithmetic.
//   * LDS rows are 128 B with the 16-byte chunk index XORed by (row / 2) % 8: the ds_read_b128
//     of a fragment (16 rows x 4 chunks) is conflict-free.
//   * One workgroup barrier per stage, between its two k-steps; fragments are double buffered
//     in registers across k-steps.
//   * Epilogue through LDS: the tile is written as bf16 into a 256 x 512 B image and read back
//     row-wise, so each global store instruction writes two whole 512-byte row segments.
//   * The second reduction part (uhat . B^T) walks only ceil(r_tile / 64) stages, r_tile = largest
//     effective rank among the tile's rows; uhat is zero beyond a row's own rank.
// Rows gathered through a permutation (rank grouping) are served by the general kernel in
// gemm_bf16.hip instead: its loaders keep 64-bit lane addresses.
#include <type_traits>

#include "mfma_util.h"

namespace cwl {
namespace {

using namespace mfma;

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int TM = 128, TN = 128;                   // per wave (2 x 2 waves)
constexpr int MB = TM / 16, NB = TN / 16;           // 16 x 16 MFMA blocks per wave tile
constexpr int ROW_BYTES = BK * 2;                   // 128
constexpr int SLOT_BYTES = 256 * ROW_BYTES;         // 32 KiB: 256 rows of one operand
constexpr int NSLOT = 5;
constexpr int LPW = 8;                              // load instructions per wave per slot
constexpr int SMEM_BYTES = NSLOT * SLOT_BYTES;
constexpr int64_t kMaxLd = (int64_t)1 << 22;        // keeps 256 rows x ld x 2 bytes inside 32 bits
static_assert(BM * BN * 2 <= SMEM_BYTES, "the output image reuses the ring");

__global__ void __launch_bounds__(256) main_bf16_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int bm, bn;
    if (!tile_coords(a.tiles_m, a.tiles_n, &bm, &bn)) return;
    const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;

    // largest effective rank among the rows of this tile: length of the second reduction part
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
    const int KS = a.K1 / BK;                        // stages of the first part (>= 1)
    const int S = KS + (r_tile + BK - 1) / BK;       // plus those of the second part

    // ---- loaders: wave w fills rows 64w .. 64w+63 of a slot, instruction i rows 64w+8i .. +7 ----
    // address = scalar (first row of the tile, current k) + lane offset; rows past the end of the
    // matrix are clamped to its last row (their products are never stored)
    uint32_t voffA[LPW], voffB[LPW];
    const char* sA;
    const char* sB;
    auto set_A = [&](const void* base, int64_t ld) {
        sA = static_cast<const char*>(base) + m0 * ld * 2;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = wave * 64 + i * 8 + (lane >> 3);
            const int ch = (lane & 7) ^ ((r >> 1) & 7);
            int64_t g = m0 + r;
            if (g > a.M - 1) g = a.M - 1;
            voffA[i] = (uint32_t)(((g - m0) * ld + ch * 8) * 2);
        }
    };
    auto set_B = [&](const void* base, int64_t ld) {
        sB = static_cast<const char*>(base) + n0 * ld * 2;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = wave * 64 + i * 8 + (lane >> 3);
            const int ch = (lane & 7) ^ ((r >> 1) & 7);
            int64_t n = n0 + r;
            if (n > a.N - 1) n = a.N - 1;
            voffB[i] = (uint32_t)(((n - n0) * ld + ch * 8) * 2);
        }
    };
    set_A(a.A1, a.lda1);
    set_B(a.B1, a.ldb1);
    int cntA = 0, cntB = 0;                          // slots requested per operand = next stage
    auto slot_A = [&](int buf, auto checked) {
        if (checked.value && cntA == KS) set_A(a.A2, a.lda2);      // from x to uhat
        char* base = smem + buf * SLOT_BYTES + wave * LPW * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            uint32_t v = voffA[i];
            asm volatile("" : "+v"(v));   // keeps the zero-extension at the load, which then takes
                                          // the scalar-base + 32-bit-offset form
            load_lds_16(sA + v, base + i * 1024);
        }
        sA += ROW_BYTES;
        ++cntA;
    };
    auto slot_B = [&](int buf, auto checked) {
        if (checked.value && cntB == KS) set_B(a.B2, a.ldb2);      // from W^T to B^T
        char* base = smem + buf * SLOT_BYTES + wave * LPW * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            uint32_t v = voffB[i];
            asm volatile("" : "+v"(v));
            load_lds_16(sB + v, base + i * 1024);
        }
        sB += ROW_BYTES;
        ++cntB;
    };
    constexpr std::true_type kChecked{};
    constexpr std::false_type kUnchecked{};

    // ---- fragment addressing: lane l reads row l % 16 of a block, chunk 4 kk + l / 16 ----
    const int l16 = lane & 15, g4 = lane >> 4;
    int koff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) koff[kk] = ((kk * 4 + g4) ^ (l16 >> 1)) * 16;
    const int a_base = (wm * TM + l16) * ROW_BYTES;
    const int b_base = (wn * TN + l16) * ROW_BYTES;

    f32x4 acc[NB][MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 4; ++v) acc[nb][mb][v] = 0.0f;

    bf16x8 af[2][MB], bfr[2][NB];
    auto read_frags = [&](int bufA, int bufB, int kk, int f) {
        const char* sa = smem + bufA * SLOT_BYTES + a_base + koff[kk];
        const char* sb = smem + bufB * SLOT_BYTES + b_base + koff[kk];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            bfr[f][i] = *reinterpret_cast<const bf16x8*>(sb + i * 16 * ROW_BYTES);
            af[f][i] = *reinterpret_cast<const bf16x8*>(sa + i * 16 * ROW_BYTES);
        }
    };
    // the weight fragment is the first operand: a lane ends with 4 consecutive output columns
    auto mfma_step = [&](int f) {
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                acc[nb][mb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(bfr[f][nb], af[f][mb], acc[nb][mb], 0, 0, 0);
    };
    // a k-step: 64 MFMAs, the 16 LDS reads of the next k-step among the first eight, the slot's
    // eight loads one per six MFMAs after that
    auto order_step = [&](bool with_loads) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 6, 0);
            if (with_loads) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto next_buf = [](int v) { return v + 1 == NSLOT ? 0 : v + 1; };

    // ---- prologue: slots x0 w0 x1 w1 x2 into buffers 0..4 ----
    slot_A(0, kChecked);
    slot_B(1, kChecked);
    if (S > 1) { slot_A(2, kChecked); slot_B(3, kChecked); }
    if (S > 2) { slot_A(4, kChecked); wait_cnt<3 * LPW, 15>(); }
    else wait_cnt<0, 15>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    int bA = 0, bB = 1;               // buffers of the stage being computed
    int pA = 0;                       // buffer released at the previous barrier for the x half of stage s+2
    read_frags(bA, bB, 0, 0);

    // Stage s: k-step 0 (requesting the x half of stage s+2), barrier, k-step 1 (requesting the
    // weight half of stage s+2).  At the barrier everything but that x half must have landed.
    auto stage_general = [&](int s) {
        const int nA = next_buf(bB), nB = next_buf(nA);
        read_frags(bA, bB, 1, 1);
        if (s >= 1 && s + 2 < S) slot_A(pA, kChecked);
        mfma_step(0);
        order_step(false);
        if (s + 1 < S) {
            if (s + 2 < S) wait_cnt<LPW, 0>();
            else wait_cnt<0, 0>();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            read_frags(nA, nB, 0, 0);
            if (s + 2 < S) slot_B(bA, kChecked);
        }
        mfma_step(1);
        order_step(false);
        pA = bB; bA = nA; bB = nB;
    };
    int s = 0;
    if (S > 0) { stage_general(0); s = 1; }
    // steady state: both requests of the stage exist and neither starts the second reduction
    // part (stage KS-2 does), so the body is one branch-free block
    const int steady_end = (KS - 3 < S - 3) ? KS - 3 : S - 3;      // last steady stage
    for (; s <= steady_end; ++s) {
        const int nA = next_buf(bB), nB = next_buf(nA);
        read_frags(bA, bB, 1, 1); slot_A(pA, kUnchecked); mfma_step(0); order_step(true);
        wait_cnt<LPW, 0>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(nA, nB, 0, 0); slot_B(bA, kUnchecked); mfma_step(1); order_step(true);
        pA = bB; bA = nA; bB = nB;
    }
    for (; s < S; ++s) stage_general(s);

    // ---- epilogue through LDS ----
    // accumulator register v of block (nb, mb): column nb*16 + 4*(l/16) + v, row mb*16 + l%16
    // (relative to the wave tile).  Image: row r at r*512; 16-byte chunk c (8 columns) is stored
    // at chunk c ^ (r % 16) and its two 8-byte halves are swapped when bit 4 of r is set: the
    // 16 rows x 2 halves written by 32 lanes of one ds_write_b64 hit every bank once.
    wait_cnt<0, 0>();
    __builtin_amdgcn_s_barrier();                    // every wave has finished reading the ring
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        const int r = wm * TM + mb * 16 + l16;
        char* rowp = smem + r * 512 + ((((r >> 4) & 1) ^ (g4 & 1)) << 3);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int c = wn * (TN / 8) + nb * 2 + (g4 >> 1);
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[nb][mb][e];
            *reinterpret_cast<bf16x4*>(rowp + ((c ^ (r & 15)) << 4)) = o;
        }
    }
    wait_cnt<0, 0>();
    __builtin_amdgcn_s_barrier();
    // wave w writes rows 64w .. 64w+63, two rows (2 x 512 B) per store instruction
    const int c = lane & 31;
    const int64_t n = n0 + c * 8;                    // N is a multiple of 8: a chunk is in or out whole
#pragma unroll 4
    for (int it = 0; it < 32; ++it) {
        const int r = wave * 64 + it * 2 + (lane >> 5);
        const int64_t g = m0 + r;
        if (g >= a.M || n >= a.N) continue;
        const u32x4 v = *reinterpret_cast<const u32x4*>(smem + r * 512 + ((c ^ (r & 15)) << 4));
        const bool flip = (r >> 4) & 1;
        u32x4 o;
        o[0] = flip ? v[2] : v[0];
        o[1] = flip ? v[3] : v[1];
        o[2] = flip ? v[0] : v[2];
        o[3] = flip ? v[1] : v[3];
        *reinterpret_cast<u32x4*>(static_cast<__bf16*>(a.C) + g * a.ldc + n) = o;
    }
}

}  // namespace

cwl_status launch_main_bf16(const GemmArgs& a_in, hipStream_t st) {
    if (a_in.perm) return launch_main_bf16_general(a_in, st);
    GemmArgs a = a_in;
    if (a.K1 < BK || a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
    if (a.lda1 > kMaxLd || a.ldb1 > kMaxLd || a.lda2 > kMaxLd || a.ldb2 > kMaxLd) return CWL_ERR_UNSUPPORTED;
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(main_bf16_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, SMEM_BYTES) != hipSuccess)
            return CWL_ERR_DEVICE;
        attr_set = true;
    }
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t n_tiles = (int64_t)a.tiles_m * a.tiles_n;
    if (n_tiles <= 0) return CWL_OK;
    const int64_t grid = (n_tiles + 7) / 8 * 8;
    if (grid >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    main_bf16_kernel<<<dim3((unsigned)grid), dim3(256), SMEM_BYTES, st>>>(a);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace cwl
