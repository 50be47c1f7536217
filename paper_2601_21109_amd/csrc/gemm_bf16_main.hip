// Main bf16 product of cwl_chunkwise_lora_linear: y = [x | uhat] . [W^T | B^T]^T (see
// linear_common.h for the formulation), one 256 x 256 output tile per workgroup of 8 waves.
//
// Data path (gfx950):
//   * A stage covers 64 elements of the reduction dimension, so every global_load_lds_dwordx4
//     fetches whole 128-byte lines (8 rows x 128 B per instruction).  The x half and the weight
//     half of a stage are separate 32 KiB "slots"; five slots form the ring (160 KiB, all of a
//     compute unit's LDS): two are being consumed, three are in flight.  Slots are issued in the
//     order x0 w0 x1 w1 ...; after the barrier that retires stage s the two buffers it held take
//     the weight half of stage s+2 and the x half of stage s+3.
//   * LDS rows are 128 B with the 16-byte chunk index XORed by (row / 2) % 8: the ds_read_b128
//     of a fragment (32 rows x 2 chunks) is conflict-free.
//   * Fragments are double buffered in registers across the four k-steps of a stage; the single
//     workgroup barrier of a stage sits before the last k-step.
//   * A stage's eight load instructions per wave are not issued as a burst: the address unit
//     takes one 64-lane instruction every ~18 cycles, a wave stays in issue until its loads are
//     taken, and with all eight waves bursting together that held the MFMAs back for more than
//     a thousand cycles per stage.  Two loads go into every k-step, each between MFMAs.
//   * v_mfma_f32_32x32x16_bf16, fp32 accumulators, weight fragment as the first operand.
//   * Epilogue through LDS: the tile is written as bf16 into a 256 x 512 B image and read back
//     row-wise, so each global store instruction writes two whole 512-byte row segments instead
//     of 16-byte pieces of 32 different rows.
//   * The second reduction part (uhat . B^T) walks only ceil(r_tile / 64) stages, r_tile = largest
//     effective rank among the tile's rows; uhat is zero beyond a row's own rank.
#include <type_traits>

#include "mfma_util.h"

namespace cwl {
namespace {

using namespace mfma;

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WM = 2, WN = 4;                       // wave grid
constexpr int TM = BM / WM, TN = BN / WN;           // 128 x 64 per wave
constexpr int MI = TM / 32, NI = TN / 32;           // 4 x 2 MFMA blocks
constexpr int ROW_BYTES = BK * 2;                   // 128
constexpr int SLOT_BYTES = 256 * ROW_BYTES;         // 32 KiB: 256 rows of one operand
constexpr int NSLOT = 5;
constexpr int LOADS = 4;                            // load instructions per wave per slot
constexpr int SMEM_BYTES = NSLOT * SLOT_BYTES;
static_assert(BM == 256 && BN == 256, "one slot holds 256 rows");
static_assert(BM * BN * 2 <= SMEM_BYTES, "the output image reuses the ring");

__global__ void __launch_bounds__(512) main_bf16_kernel(GemmArgs a) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int bm, bn;
    if (!tile_coords(a.tiles_m, a.tiles_n, &bm, &bn)) return;
    const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave / WN, wn = wave % WN;

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

    // ---- loaders: wave w fills rows 32w .. 32w+31 of a slot, 8 rows per instruction ----
    const __bf16* gpA[LOADS];
    const __bf16* gpB[LOADS];
    int32_t rowA[LOADS], rowB[LOADS];                // grouped row / output column, clamped
    int lchunk[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int r = wave * 32 + i * 8 + (lane >> 3);
        lchunk[i] = (lane & 7) ^ ((r >> 1) & 7);
        int64_t g = m0 + r;
        if (g > a.M - 1) g = a.M - 1;
        rowA[i] = (int32_t)g;
        const int64_t t = a.perm ? (int64_t)a.perm[g] : g;
        gpA[i] = static_cast<const __bf16*>(a.A1) + t * a.lda1 + lchunk[i] * 8;
        int64_t n = n0 + r;
        if (n > a.N - 1) n = a.N - 1;
        rowB[i] = (int32_t)n;
        gpB[i] = static_cast<const __bf16*>(a.B1) + n * a.ldb1 + lchunk[i] * 8;
    }
    // Loads are requested two instructions ("a pair") at a time so that they can sit between MFMAs:
    // a wave that issues a burst of loads is held until the address unit has taken them all, and
    // its MFMAs wait behind them.  cntA / cntB count pairs; pair 2t of an operand starts stage t.
    int cntA = 0, cntB = 0;
    auto switch_A = [&]() {           // from x to uhat
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            gpA[i] = static_cast<const __bf16*>(a.A2) + (int64_t)rowA[i] * a.lda2 + lchunk[i] * 8;
    };
    auto switch_B = [&]() {           // from W^T to B^T
#pragma unroll
        for (int i = 0; i < LOADS; ++i)
            gpB[i] = static_cast<const __bf16*>(a.B2) + (int64_t)rowB[i] * a.ldb2 + lchunk[i] * 8;
    };
    auto pair_A = [&](int buf, int pair, auto checked) {
        if (checked.value && cntA == 2 * KS) switch_A();
        char* base = smem + buf * SLOT_BYTES + wave * LOADS * 1024;
#pragma unroll
        for (int i = 2 * pair; i < 2 * pair + 2; ++i) {
            load_lds_16(gpA[i], base + i * 1024);
            gpA[i] += BK;
        }
        ++cntA;
    };
    auto pair_B = [&](int buf, int pair, auto checked) {
        if (checked.value && cntB == 2 * KS) switch_B();
        char* base = smem + buf * SLOT_BYTES + wave * LOADS * 1024;
#pragma unroll
        for (int i = 2 * pair; i < 2 * pair + 2; ++i) {
            load_lds_16(gpB[i], base + i * 1024);
            gpB[i] += BK;
        }
        ++cntB;
    };
    constexpr std::true_type kChecked{};
    constexpr std::false_type kUnchecked{};
    auto issue_A = [&](int buf) { pair_A(buf, 0, kChecked); pair_A(buf, 1, kChecked); };
    auto issue_B = [&](int buf) { pair_B(buf, 0, kChecked); pair_B(buf, 1, kChecked); };

    // ---- fragment addressing ----
    const int l32 = lane & 31, h = lane >> 5;
    const int sw = (l32 >> 1) & 7;
    int koff[4];
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) koff[kk] = ((2 * kk + h) ^ sw) * 16;
    const int a_base = (wm * TM + l32) * ROW_BYTES;
    const int b_base = (wn * TN + l32) * ROW_BYTES;

    f32x16 acc[NI][MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.0f;

    bf16x8 af[2][MI], bfr[2][NI];
    auto read_frags = [&](int bufA, int bufB, int kk, int f) {
        const char* sa = smem + bufA * SLOT_BYTES;
        const char* sb = smem + bufB * SLOT_BYTES;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            af[f][mi] = *reinterpret_cast<const bf16x8*>(sa + a_base + mi * 32 * ROW_BYTES + koff[kk]);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            bfr[f][ni] = *reinterpret_cast<const bf16x8*>(sb + b_base + ni * 32 * ROW_BYTES + koff[kk]);
    };
    auto mfma_step = [&](int f) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[f][ni], af[f][mi], acc[ni][mi], 0, 0, 0);
    };
    // issue order inside a k-step: one MFMA (its operands are already in registers), the LDS reads
    // of the next k-step, then the remaining MFMAs with the step's two loads spaced out among them
    auto order_step = [&](bool with_loads) {
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        __builtin_amdgcn_sched_group_barrier(0x100, MI + NI, 0);
        if (with_loads) {
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 3, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
        } else {
            __builtin_amdgcn_sched_group_barrier(0x008, MI * NI - 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto next_buf = [](int v) { return v + 1 == NSLOT ? 0 : v + 1; };

    // ---- prologue: slots x0 w0 x1 w1 x2 into buffers 0..4 ----
    issue_A(0);
    issue_B(1);
    if (S > 1) { issue_A(2); issue_B(3); }
    if (S > 2) { issue_A(4); wait_cnt<3 * LOADS, 15>(); }
    else wait_cnt<0, 15>();
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_sched_barrier(0);
    int bA = 0, bB = 1;               // buffers of the stage being computed
    int pB = 0, pA = 0;               // buffers released at the previous barrier: they take the weight
                                      // half of stage s+1 (second pair still to request) and the x half of s+2
    read_frags(bA, bB, 0, 0);

    // Stage s, k-steps 0..2, barrier, k-step 3.  Requests in program order: weights of stage s+1
    // (second pair), x of stage s+2 (both pairs), barrier, weights of stage s+2 (first pair).  At
    // the barrier everything but the x half just requested must have landed.
    auto stage_general = [&](int s) {
        const int nA = next_buf(bB), nB = next_buf(nA);
        const bool pendB = s >= 1 && s + 1 < S, pendA = s >= 1 && s + 2 < S, newB = s + 2 < S;
        read_frags(bA, bB, 1, 1); if (pendB) pair_B(pB, 1, kChecked); mfma_step(0); order_step(false);
        read_frags(bA, bB, 2, 0); if (pendA) pair_A(pA, 0, kChecked); mfma_step(1); order_step(false);
        read_frags(bA, bB, 3, 1); if (pendA) pair_A(pA, 1, kChecked); mfma_step(0); order_step(false);
        if (s + 1 < S) {
            if (s + 2 < S) wait_cnt<LOADS, 0>();
            else wait_cnt<0, 0>();
            __builtin_amdgcn_s_barrier();
            __builtin_amdgcn_sched_barrier(0);
            read_frags(nA, nB, 0, 0);
            if (newB) pair_B(bA, 0, kChecked);
        }
        mfma_step(1);
        __builtin_amdgcn_sched_barrier(0);
        pB = bA; pA = bB; bA = nA; bB = nB;
    };
    int s = 0;
    if (S > 0) { stage_general(0); s = 1; }
    // steady state: no request of this stage starts the second reduction part (that happens in
    // stage KS-2) and all of them exist, so the body is one branch-free block
    const int steady_end = (KS - 3 < S - 3) ? KS - 3 : S - 3;      // last steady stage
    for (; s <= steady_end; ++s) {
        const int nA = next_buf(bB), nB = next_buf(nA);
        read_frags(bA, bB, 1, 1); pair_B(pB, 1, kUnchecked); mfma_step(0); order_step(true);
        read_frags(bA, bB, 2, 0); pair_A(pA, 0, kUnchecked); mfma_step(1); order_step(true);
        read_frags(bA, bB, 3, 1); pair_A(pA, 1, kUnchecked); mfma_step(0); order_step(true);
        wait_cnt<LOADS, 0>();
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
        read_frags(nA, nB, 0, 0); pair_B(bA, 0, kUnchecked); mfma_step(1); order_step(true);
        pB = bA; pA = bB; bA = nA; bB = nB;
    }
    for (; s < S; ++s) stage_general(s);

    // ---- epilogue through LDS ----
    // accumulator register v of block (ni, mi): column n = ni*32 + 8*(v/4) + 4*h + v%4, row
    // m = mi*32 + l32 (relative to the wave tile).  Image: row r at r*512; 16-byte chunk c (8
    // columns) is stored at chunk c ^ (r % 16) and its two 8-byte halves are swapped when bit 4
    // of r is set, which makes the 32-row ds_write_b64 of one (ni, q) hit every bank once.
    wait_cnt<0, 0>();
    __builtin_amdgcn_s_barrier();                    // every wave has finished reading the ring
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int r = wm * TM + mi * 32 + l32;
        char* rowp = smem + r * 512 + ((((r >> 4) & 1) ^ h) << 3);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int c = wn * (TN / 8) + ni * 4 + q;
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)acc[ni][mi][q * 4 + e];
                *reinterpret_cast<bf16x4*>(rowp + ((c ^ (r & 15)) << 4)) = o;
            }
    }
    wait_cnt<0, 0>();
    __builtin_amdgcn_s_barrier();
    // wave w writes rows 32w .. 32w+31, two rows (2 x 512 B) per store instruction
    const int c = lane & 31;
    const int64_t n = n0 + c * 8;                    // N is a multiple of 8: a chunk is in or out whole
#pragma unroll 4
    for (int it = 0; it < 16; ++it) {
        const int r = wave * 32 + it * 2 + (lane >> 5);
        const int64_t g = m0 + r;
        if (g >= a.M || n >= a.N) continue;
        const int64_t t = a.perm ? (int64_t)a.perm[g] : g;
        const u32x4 v = *reinterpret_cast<const u32x4*>(smem + r * 512 + ((c ^ (r & 15)) << 4));
        const bool flip = (r >> 4) & 1;
        u32x4 o;
        o[0] = flip ? v[2] : v[0];
        o[1] = flip ? v[3] : v[1];
        o[2] = flip ? v[0] : v[2];
        o[3] = flip ? v[1] : v[3];
        *reinterpret_cast<u32x4*>(static_cast<__bf16*>(a.C) + t * a.ldc + n) = o;
    }
}

}  // namespace

cwl_status launch_main_bf16(const GemmArgs& a_in, hipStream_t st) {
    GemmArgs a = a_in;
    if (a.K1 < BK || a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
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
    main_bf16_kernel<<<dim3((unsigned)grid), dim3(512), SMEM_BYTES, st>>>(a);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace cwl
