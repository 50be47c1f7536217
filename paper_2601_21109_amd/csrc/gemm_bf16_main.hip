// Main bf16 product of cwl_chunkwise_lora_linear: y = [x | uhat] . [W^T | B^T]^T (see
// linear_common.h for the formulation), 256 x 256 output tiles, persistent workgroups of 4 waves.
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
//   * One workgroup per compute unit walks its tiles (XCD-aware order) and the ring keeps running
//     across tile boundaries: when a tile's epilogue ends, the next tile's first stage is in LDS.
//   * Load instructions are never issued as a burst.  The address unit takes one 64-lane
//     instruction every ~18 cycles and a wave stays in issue until its loads are taken; bursts
//     after the barrier held the MFMAs back for more than a thousand cycles per stage.  Here
//     every load sits between MFMAs (one per four), as do the LDS reads (one per MFMA at the
//     start of a k-step), by way of sched_group_barrier.
//   * Loads use a scalar base plus a 32-bit lane offset, so the reduction loop advances two
//     scalar pointers and does no vector address arithmetic.
//   * LDS rows are 128 B with the 16-byte chunk index XORed by (row / 2) % 8: the ds_read_b128
//     of a fragment (16 rows x 4 chunks) is conflict-free.
//   * One workgroup barrier per stage, between its two k-steps; fragments are double buffered
//     in registers across k-steps.
//   * Epilogue through LDS without a barrier: every wave turns its own quarter, 16 rows at a time,
//     into 256-byte row segments through the 8 KiB of the free slot that it fills itself as a
//     loader, so each global store writes four whole segments with consecutive lanes on
//     consecutive addresses (the store unit takes 52 B per cycle that way, 16 B per cycle when the
//     lanes of a segment are 16 apart as in the MFMA layout), and no 64-bit multiply per store.
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

// Virtual workgroup v -> (row tile, column tile), the XCD-aware order of mfma::tile_coords with
// the index passed in: a persistent workgroup b walks v = b, b + gridDim.x, ... and so stays in
// the band of the XCD it runs on (gridDim.x is a multiple of 8).
__device__ __forceinline__ bool tile_of(int32_t v, int32_t n_virtual, int32_t tiles_m, int32_t tiles_n,
                                        int32_t* bm, int32_t* bn) {
    constexpr int32_t kXcd = 8, GROUP_M = 8;
    if (v >= n_virtual) return false;
    const int32_t n_tiles = tiles_m * tiles_n;
    const int32_t per_xcd = (n_tiles + kXcd - 1) / kXcd;
    const int32_t tile = (v % kXcd) * per_xcd + v / kXcd;
    if (tile >= n_tiles) return false;
    const int32_t band_size = GROUP_M * tiles_n;
    const int32_t band = tile / band_size, in_band = tile % band_size;
    const int32_t first_m = band * GROUP_M;
    const int32_t gm = (tiles_m - first_m < GROUP_M) ? tiles_m - first_m : GROUP_M;
    *bm = first_m + in_band % gm;
    *bn = in_band / gm;
    return true;
}

// GATE: the shrink of a group of projections on many rows, uhat = (x . [A_1 .. A_P]) (.) G: one
// reduction part, and the epilogue multiplies every value by its row's gate for its direction
// (column modulo a.gate_period) before rounding, as the shrink kernels of gemm_bf16.hip do.
template <bool GATE>
__global__ void __launch_bounds__(256) main_bf16_kernel(GemmArgs a, int32_t n_virtual) {
    extern __shared__ __attribute__((aligned(1024))) char smem[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1, wn = wave & 1;
    const int32_t v_step = (int32_t)gridDim.x;
    const int KS = a.K1 / BK;                        // stages of the first reduction part (>= 1)

    // stages of a row tile: the first part plus ceil(r_tile / 64), r_tile = largest effective
    // rank among the tile's rows.  The table holds four entries (one per 64 rows) for every started
    // group of 256 rows, so a tile reads its four with one aligned scalar load.
    typedef __attribute__((ext_vector_type(4))) int i32x4;
    auto stages_of = [&](int32_t bm) -> int {
        int32_t r_tile = 0;
        if (a.blk_r) {
            const i32x4 q = *reinterpret_cast<const i32x4*>(a.blk_r + 4 * (int64_t)bm);
            const int32_t q01 = q[0] > q[1] ? q[0] : q[1], q23 = q[2] > q[3] ? q[2] : q[3];
            r_tile = q01 > q23 ? q01 : q23;
        }
        return KS + (r_tile + BK - 1) / BK;
    };

    // ---- loaders ----
    // Wave w fills rows 64w .. 64w+63 of a slot, instruction i rows 64w+8i .. +7.  Address =
    // scalar (first row of the tile, current k) + 32-bit lane offset; rows past the end of the
    // matrix are clamped to its last row (their products are never stored).  The loader walks
    // (tile, stage) on its own, two stages ahead of the MFMAs: the ring does not drain at a tile
    // boundary.  Every stage requests exactly one x slot and one weight slot (the x slot half a
    // stage before the weight slot), so the reduction loop has a single branch-free body and one
    // walker serves both operands; what changes between stages (second reduction part, next tile)
    // is patched into the loader state after the body.  A loader that has run out of tiles keeps
    // re-requesting its last slots into buffers nobody reads (stepL = 0), which only happens in
    // the last two stages of the kernel.
    uint32_t voffA[LPW], voffB[LPW];
    const char* sA = nullptr;
    const char* sB = nullptr;
    int32_t vL = (int32_t)blockIdx.x;
    int cntL = 0, SL = 0;                            // stages requested of the loader's tile, stages it has
    int stepL = ROW_BYTES;
    int64_t m0A = 0, n0B = 0;
    bool validL = false;
    // (the lane index is made opaque where rarely-run code derives addresses from it: otherwise the
    // compiler computes all of that once, ahead of the tile loop, and the values crowd the register file)
    auto set_A = [&](const void* base, int64_t ld) {
        sA = static_cast<const char*>(base) + m0A * ld * 2;
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = wave * 64 + i * 8 + (ln >> 3);
            const int ch = (ln & 7) ^ ((r >> 1) & 7);
            int64_t g = m0A + r;
            if (g > a.M - 1) g = a.M - 1;
            voffA[i] = (uint32_t)(((g - m0A) * ld + ch * 8) * 2);
        }
    };
    auto set_B = [&](const void* base, int64_t ld) {
        sB = static_cast<const char*>(base) + n0B * ld * 2;
        int ln = lane;
        asm volatile("" : "+v"(ln));
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int r = wave * 64 + i * 8 + (ln >> 3);
            const int ch = (ln & 7) ^ ((r >> 1) & 7);
            int64_t n = n0B + r;
            if (n > a.N - 1) n = a.N - 1;
            voffB[i] = (uint32_t)(((n - n0B) * ld + ch * 8) * 2);
        }
    };
    auto tile_L = [&]() {
        int32_t bm = 0, bn = 0;
        validL = tile_of(vL, n_virtual, a.tiles_m, a.tiles_n, &bm, &bn);
        if (validL) {
            m0A = (int64_t)bm * BM;
            n0B = (int64_t)bn * BN;
            SL = stages_of(bm);
            cntL = 0;
            set_A(a.A1, a.lda1);
            set_B(a.B1, a.ldb1);
        } else {
            sA -= ROW_BYTES;          // stay on the last slots requested
            sB -= ROW_BYTES;
            stepL = 0;
        }
    };
    // after a stage's two requests: move the loader to its next tile, or to the second reduction part
    auto patch_L = [&]() {
        if (validL) {
            if (cntL == SL) { vL += v_step; tile_L(); }
            else if (cntL == KS) {
                set_A(a.A2, a.lda2);                           // from x to uhat
                set_B(a.B2, a.ldb2);                           // from W^T to B^T
            }
        }
    };
    // one slot = 8 load instructions per wave
    auto slot_A = [&](int buf) {
        char* base = smem + buf * SLOT_BYTES + wave * LPW * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            asm volatile("" : "+v"(voffA[i]));   // keeps the zero-extension at the load, which then takes
                                                 // the scalar-base + 32-bit-offset form (in place: no copy)
            load_lds_16(sA + voffA[i], base + i * 1024);
        }
        sA += stepL;
    };
    auto slot_B = [&](int buf) {                 // the second request of a stage: counts it
        char* base = smem + buf * SLOT_BYTES + wave * LPW * 1024;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            asm volatile("" : "+v"(voffB[i]));
            load_lds_16(sB + voffB[i], base + i * 1024);
        }
        sB += stepL;
        ++cntL;
    };

    // ---- fragment addressing: lane l reads row l % 16 of a block, chunk 4 kk + l / 16 ----
    const int l16 = lane & 15, g4 = lane >> 4;
    int koff[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) koff[kk] = ((kk * 4 + g4) ^ (l16 >> 1)) * 16;
    const int a_base = (wm * TM + l16) * ROW_BYTES;
    const int b_base = (wn * TN + l16) * ROW_BYTES;

    f32x4 acc[NB][MB];
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
    // a k-step: 64 MFMAs; the 16 LDS reads of the next k-step one per MFMA at the start, then the
    // slot's eight loads one per four MFMAs (two reads per MFMA measured 5 % slower: with one wave
    // per SIMD whatever is issued between two MFMAs has to fit into the 16 cycles the first one runs)
    auto order_step = [&]() {
#pragma unroll
        for (int j = 0; j < 16; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 16, 0);
        __builtin_amdgcn_sched_barrier(0);
    };
    auto zero_acc = [&]() {
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
#pragma unroll
                for (int v = 0; v < 4; ++v) acc[nb][mb][v] = 0.0f;
    };
    auto next_buf = [](int v) { return v + 1 == NSLOT ? 0 : v + 1; };
    auto sync = [&]() {
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- this workgroup's first tile; prologue: slots x0 w0 x1 w1 into buffers 0..3 ----
    int32_t vC = (int32_t)blockIdx.x, bm = 0, bn = 0;
    if (!tile_of(vC, n_virtual, a.tiles_m, a.tiles_n, &bm, &bn)) return;
    tile_L();
    slot_A(0); slot_B(1); patch_L();
    slot_A(2); slot_B(3); patch_L();
    wait_cnt<2 * LPW, 15>();          // stage 0 has landed
    sync();
    int bA = 0, bB = 1;               // buffers of the stage being computed
    int pA = 4;                       // buffer that takes the next x slot (two stages ahead)
    read_frags(bA, bB, 0, 0);

    while (true) {                    // tiles of this workgroup
        const int S = stages_of(bm);
        const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;
        zero_acc();
        // Stage body: k-step 0 (requesting the x slot two stages ahead), barrier, k-step 1
        // (requesting the weight slot two stages ahead into the x buffer just released).  At the
        // barrier everything but the x slot just requested has landed: the next stage, which may
        // be the next tile's first; its first fragments are read during k-step 1.  With one wave per
        // SIMD whatever follows the last MFMA of a stage is not hidden by anything, so the loader
        // patches run only after the stages that can need them.
        auto stage = [&](bool patch) {
            const int nA = next_buf(bB), nB = next_buf(nA);
            read_frags(bA, bB, 1, 1); slot_A(pA); mfma_step(0); order_step();
            wait_cnt<LPW, 0>();
            sync();
            read_frags(nA, nB, 0, 0); slot_B(bA); mfma_step(1); order_step();
            if (patch) patch_L();
            pA = bB; bA = nA; bB = nB;
        };
        // The first stage is peeled out of the loops: with the cleared accumulators entering a loop
        // directly, the compiler shuffled them between registers in every iteration.
        stage(true);
        int s = 1;
        // stages whose requests (stage s+2 of this tile) stay inside the first reduction part
        const int plain_end = (KS < S ? KS : S) - 4;
        for (; s <= plain_end; ++s) stage(false);
        for (; s < S; ++s) stage(true);

        // ---- epilogue: every wave stages its own quarter through its own 8 KiB of buffer pA ----
        // pA (the weight buffer of the stage just finished) is the one free buffer here: every wave
        // finished reading it before the barrier of that stage, and the next request into it comes
        // with the next stage body, where wave w fills bytes [8192 w, 8192 w + 8192) -- the same
        // 8 KiB it stages through here.  So the epilogue needs no barrier at either end, and the
        // waves drift apart over it (they meet again at the barrier of the next stage).
        //
        // The 8 KiB are two images of 16 rows x 256 B (one block row of the wave's 128 columns as
        // bf16).  Block row q is written from the MFMA layout (accumulator register v of block
        // (nb, q): column nb*16 + 4*(l/16) + v, row l%16) with ds_write_b64 and read back row-wise
        // with ds_read_b128, so a global store covers four whole 256-byte row segments with
        // consecutive lanes on consecutive addresses (stored straight from the MFMA layout the
        // lanes of a 64-byte piece are 16 apart and the store unit takes them one lane at a time:
        // 16 B per cycle against 52).  The LDS unit executes one wave's instructions in order, so
        // block row q+2 is written into the image block row q was just read from without a wait
        // between them; only the read data is waited for.  A 16-byte chunk c of image row r sits
        // at chunk c ^ r: the 16 rows x 2 halves written by 32 lanes of a ds_write_b64 hit every
        // bank once.
        //
        // The accumulators are read with inline assembly (left to itself the compiler copies all
        // 256 out of the AGPRs first, which leaves no vector registers for the fragments that
        // live across the epilogue).  The compiler does not insert the wait states an MFMA result
        // needs before a vector instruction may read it into inline assembly; the instructions
        // since the last MFMA already cover them, the explicit ones make that independent of
        // scheduling.
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("s_nop 15");
        asm volatile("s_nop 15");
        __builtin_amdgcn_sched_barrier(0);
        {
            int le = lane;
            asm volatile("" : "+v"(le));
            const int l16e = le & 15, g4e = le >> 4;
            char* stg = smem + pA * SLOT_BYTES + wave * 8192;
            // GATE: the gate entries of this lane's eight rows (one per block row), and the direction
            // of the wave's first column (wave-uniform; block nb starts 16 nb further on, modulo the
            // period, which is a multiple of 64)
            TokMeta mt[GATE ? MB : 1];
            int32_t dir0 = 0;
            if constexpr (GATE) {
#pragma unroll
                for (int q = 0; q < MB; ++q) {
                    int64_t g = m0 + wm * TM + q * 16 + l16e;
                    if (g > a.M - 1) g = a.M - 1;
                    mt[q] = a.meta[g];
                }
                dir0 = (int32_t)((n0 + wn * TN) % a.gate_period);
            }
            auto put = [&](auto qc) {
                constexpr int q = decltype(qc)::value;
                char* rowp = stg + (q & 1) * 4096 + l16e * 256 + ((g4e & 1) << 3);
                int32_t dir = dir0;                  // direction of block nb's first column
#pragma unroll
                for (int nb = 0; nb < NB; ++nb) {
                    float x0, x1, x2, x3;
                    asm volatile("v_accvgpr_read_b32 %0, %4\n\tv_accvgpr_read_b32 %1, %5\n\t"
                                 "v_accvgpr_read_b32 %2, %6\n\tv_accvgpr_read_b32 %3, %7"
                                 : "=v"(x0), "=v"(x1), "=v"(x2), "=v"(x3)
                                 : "a"(acc[nb][q][0]), "a"(acc[nb][q][1]), "a"(acc[nb][q][2]), "a"(acc[nb][q][3])
                                 : "memory");
                    if constexpr (GATE) {
                        const TokMeta& m = mt[q];
                        const int32_t i0 = dir + 4 * g4e;
                        x0 *= (i0 < m.r_prev ? m.g_prev : 0.0f) + (i0 < m.r_cur ? m.g_cur : 0.0f);
                        x1 *= (i0 + 1 < m.r_prev ? m.g_prev : 0.0f) + (i0 + 1 < m.r_cur ? m.g_cur : 0.0f);
                        x2 *= (i0 + 2 < m.r_prev ? m.g_prev : 0.0f) + (i0 + 2 < m.r_cur ? m.g_cur : 0.0f);
                        x3 *= (i0 + 3 < m.r_prev ? m.g_prev : 0.0f) + (i0 + 3 < m.r_cur ? m.g_cur : 0.0f);
                        dir += 16;
                        if (dir >= a.gate_period) dir -= a.gate_period;
                    }
                    bf16x4 o;
                    o[0] = (__bf16)x0; o[1] = (__bf16)x1; o[2] = (__bf16)x2; o[3] = (__bf16)x3;
                    *reinterpret_cast<bf16x4*>(rowp + (((nb * 2 + (g4e >> 1)) ^ l16e) << 4)) = o;
                }
            };
            // read side: an instruction covers image rows 4 it + l/16, lane l%16 takes chunk l%16
            const int cch = le & 15, rsub = le >> 4;
            const int64_t n = n0 + wn * TN + cch * 8;               // N is a multiple of 8: a chunk is in or out whole
            const int64_t grow0 = m0 + wm * TM + rsub;              // row of (q = 0, it = 0)
            const int64_t left64 = a.M - grow0;
            const int rows_left = left64 > BM ? BM : (int)left64;
            const bool col_ok = n < a.N;
            char* cp = reinterpret_cast<char*>(static_cast<__bf16*>(a.C) + grow0 * a.ldc + n);
            const int64_t pitch4 = a.ldc * 8;                       // bytes from row r to row r + 4
            auto pass = [&](auto qc) {
                constexpr int q = decltype(qc)::value;
                u32x4 v[4];
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    const int r = it * 4 + rsub;
                    v[it] = *reinterpret_cast<const u32x4*>(stg + (q & 1) * 4096 + r * 256 + ((cch ^ r) << 4));
                }
                if constexpr (q + 2 < MB) put(std::integral_constant<int, q + 2>{});
#pragma unroll
                for (int it = 0; it < 4; ++it) {
                    if (col_ok && q * 16 + it * 4 < rows_left) *reinterpret_cast<u32x4*>(cp) = v[it];
                    cp += pitch4;
                }
            };
            put(std::integral_constant<int, 0>{});
            put(std::integral_constant<int, 1>{});
            pass(std::integral_constant<int, 0>{}); pass(std::integral_constant<int, 1>{});
            pass(std::integral_constant<int, 2>{}); pass(std::integral_constant<int, 3>{});
            pass(std::integral_constant<int, 4>{}); pass(std::integral_constant<int, 5>{});
            pass(std::integral_constant<int, 6>{}); pass(std::integral_constant<int, 7>{});
        }
        vC += v_step;
        if (!tile_of(vC, n_virtual, a.tiles_m, a.tiles_n, &bm, &bn)) break;
    }
    wait_cnt<0, 0>();                                 // nothing of this wave's is still on its way into LDS
}

}  // namespace

// compute units of the current device, rounded down to a multiple of 8 (0: error)
static int persistent_grid_limit() {
    static int n_cu_of[kMaxDevices] = {};
    const int dev = device_slot();
    if (dev < 0) return 0;
    if (n_cu_of[dev] == 0) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v < 8)
            return 0;
        n_cu_of[dev] = v / 8 * 8;
    }
    return n_cu_of[dev];
}

bool shrink_wide_bf16_serves(const GemmArgs& a) {
    return !a.perm && a.M >= kShrinkTallRows && a.N >= 192 && a.gate_period >= 64 &&
           a.gate_period % 64 == 0 && a.lda1 <= kMaxLd && a.ldb1 <= kMaxLd && a.K1 >= BK && a.K1 % BK == 0;
}

cwl_status launch_shrink_wide_bf16(const GemmArgs& a_in, hipStream_t st) {
    if (!shrink_wide_bf16_serves(a_in) || !a_in.meta) return CWL_ERR_UNSUPPORTED;
    GemmArgs a = a_in;
    a.blk_r = nullptr;                                 // one reduction part
    a.A2 = a.B2 = nullptr;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(main_bf16_kernel<true>), SMEM_BYTES, lds_set) != CWL_OK)
        return CWL_ERR_DEVICE;
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t n_tiles = (int64_t)a.tiles_m * a.tiles_n;
    const int64_t n_virtual = (n_tiles + 7) / 8 * 8;
    if (n_virtual >= (int64_t)1 << 30) return CWL_ERR_UNSUPPORTED;
    const int n_cu = persistent_grid_limit();
    if (n_cu == 0) return CWL_ERR_DEVICE;
    const int64_t grid = n_virtual < n_cu ? n_virtual : n_cu;
    main_bf16_kernel<true><<<dim3((unsigned)grid), dim3(256), SMEM_BYTES, st>>>(a, (int32_t)n_virtual);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

cwl_status launch_main_bf16(const GemmArgs& a_in, hipStream_t st) {
    GemmArgs a = a_in;
    // gathered rows, and leading dimensions whose 256-row offsets do not fit 32 bits, take the
    // general kernel (64-bit lane addresses)
    if (a.perm || a.lda1 > kMaxLd || a.ldb1 > kMaxLd || a.lda2 > kMaxLd || a.ldb2 > kMaxLd)
        return launch_main_bf16_general(a_in, st);
    if (a.K1 < BK || a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(main_bf16_kernel<false>), SMEM_BYTES, lds_set) != CWL_OK)
        return CWL_ERR_DEVICE;
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t n_tiles = (int64_t)a.tiles_m * a.tiles_n;
    if (n_tiles <= 0) return CWL_OK;
    // with tiles for a quarter of the compute units at most, 128 x 128 tiles fill the chip instead
    if (n_tiles <= 64) return launch_main_bf16_tile128(a_in, st);
    // up to half of them: 256 x 128 tiles, again twice as many
    if (n_tiles <= 128) return launch_main_bf16_tile256x128(a_in, st);
    const int64_t n_virtual = (n_tiles + 7) / 8 * 8;       // workgroup slots, 8 XCDs round-robin
    if (n_virtual >= (int64_t)1 << 30) return CWL_ERR_UNSUPPORTED;
    // persistent: one workgroup per compute unit (160 KiB of LDS each), a multiple of 8 of them
    const int n_cu = persistent_grid_limit();
    if (n_cu == 0) return CWL_ERR_DEVICE;
    const int64_t grid = n_virtual < n_cu ? n_virtual : n_cu;
    main_bf16_kernel<false><<<dim3((unsigned)grid), dim3(256), SMEM_BYTES, st>>>(a, (int32_t)n_virtual);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace cwl
