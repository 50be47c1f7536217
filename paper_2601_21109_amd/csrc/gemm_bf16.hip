// bf16 matrix-core shrink of cwl_chunkwise_lora_linear (see linear_common.h for the formulation).
//
// A "TN" GEMM kernel, C[m, n] = sum_k A[m, k] B[n, k], both operands K-contiguous, with tile
// shape, wave grid and ring depth as template parameters.  The library uses it as the shrink
// (A = x, B = A^T, epilogue multiplies by the gate and writes uhat); with EPI_STORE it also
// computes the two-part product [x | uhat] . [W^T | B^T]^T, which the 256 x 256 kernel in
// gemm_bf16_main.hip specialises.
//
// Data path (gfx950):
//   * global -> LDS with global_load_lds_dwordx4 (no staging registers) into a ring of NST
//     stages of BK = 32 or 64 (LDS rows of 64 or 128 bytes, the 16-byte chunk index XOR-swizzled
//     with the row so that the ds_read_b128 of a fragment touches all 64 banks once).  NST - 1 stages are
//     in flight while one is consumed: the L2 / fabric latency under load is far longer than one
//     stage of MFMA work, and a two-stage scheme measured latency-bound.
//   * LDS -> registers with ds_read_b128, fragments double buffered: the two k-steps of a stage
//     alternate between two register sets, the next set is fetched while the MFMAs of the
//     current one run.
//   * v_mfma_f32_32x32x16_bf16, fp32 accumulators.  The weight fragment is the MFMA's first
//     operand, so each lane ends with 4 consecutive output columns of one row (8-byte stores).
//   * one workgroup barrier per stage, placed between the two k-steps: by then this wave's
//     fragment reads of the stage are in registers and its loads of the next stage have landed.
#include "mfma_util.h"
#include "token_meta.h"
#include "partition_seq.h"

namespace cwl {
namespace {

using namespace mfma;

typedef __attribute__((ext_vector_type(4))) float f32x4;

// BK = elements of K per LDS stage: 32 (64-byte LDS rows, chunk index XORed with (row / 4) % 4) or
// 64 (128-byte rows, (row / 2) % 8).  With 64 every load instruction fetches whole 128-byte lines,
// which is what a kernel that streams its operand once from HBM wants.
// (vid: workgroup index of the GEMM proper; a launch may carry other workgroups in front)
template <int BM, int BN, int WM, int WN, int NST, int EPI, int BK = 32>
__device__ __forceinline__ void gemm_bf16_tn_body(const GemmArgs& a, const int vid) {
    static_assert(BK == 32 || BK == 64, "stage depth");
    constexpr int ROW_BYTES = BK * 2;
    constexpr int CHUNKS = ROW_BYTES / 16;        // 16-byte chunks per LDS row
    constexpr int RPI = 1024 / ROW_BYTES;         // rows per load instruction
    constexpr int SW_SHIFT = (BK == 32) ? 2 : 1;  // swizzle = (row >> SW_SHIFT) % CHUNKS
    constexpr int KSTEPS = BK / 16;               // MFMA k-steps per stage
    constexpr int NW = WM * WN;
    constexpr int TM = BM / WM, TN = BN / WN;     // wave tile
    constexpr int MI = TM / 32, NI = TN / 32;     // 32x32 MFMA blocks per wave tile
    constexpr int ROWS = BM + BN;
    constexpr int LOADS = ROWS / RPI / NW;        // 1 KiB load instructions per wave per stage
    constexpr int STAGE_BYTES = ROWS * ROW_BYTES;
    constexpr int N_DS = MI + NI, N_MFMA = MI * NI;
    static_assert(ROWS % (RPI * NW) == 0 && BM % RPI == 0, "tile rows must split evenly over the waves");
    static_assert(BM % 16 == 0 && BN % 16 == 0 && TM % 32 == 0 && TN % 32 == 0, "tile shape");
    static_assert(EPI == EPI_PARTIAL || BM % kRankBlock == 0, "row tile must cover whole rank blocks");
    static_assert(NST >= 2 && (NST - 1) * LOADS < 64, "ring depth");

    extern __shared__ __attribute__((aligned(1024))) char smem[];

    int bm, bn;
    int split = 0;
    if (EPI == EPI_PARTIAL) {
        // few row tiles, the splits of a tile on consecutive workgroup ids (with 8 splits, split s
        // always runs on XCD s and the x slice it reads stays in that L2)
        const int tile = vid / a.splits;
        split = vid % a.splits;
        if (tile >= a.tiles_m * a.tiles_n) return;
        bm = tile % a.tiles_m;
        bn = tile / a.tiles_m;
    } else if (!tile_coords(vid, a.tiles_m, a.tiles_n, &bm, &bn)) {
        return;
    }
    const int64_t m0 = (int64_t)bm * BM, n0 = (int64_t)bn * BN;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: stage addresses stay in SGPRs
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
    // shrink: output columns (adapter directions) at or beyond the block's largest effective rank
    // are gated to zero anyway, so their MFMAs are skipped; a rank-0 block skips the whole loop
    bool ni_on[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) ni_on[ni] = true;
    int KS = a.K1 / BK;                               // stages of the first part
    if (EPI == EPI_GATE && a.gate_blk_r) {
        const int64_t n_blk = (a.M + kRankBlock - 1) / kRankBlock;
        int32_t r_blk = 0;
#pragma unroll
        for (int i = 0; i < BM / kRankBlock; ++i) {
            const int64_t blk = m0 / kRankBlock + i;
            if (blk < n_blk) {
                const int32_t r = a.gate_blk_r[blk];
                r_blk = r > r_blk ? r : r_blk;
            }
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int32_t c = (int32_t)n0 + wn * TN + ni * 32;      // 32 columns never straddle two adapters
            ni_on[ni] = (a.gate_period > 0 ? c % a.gate_period : c) < r_blk;
        }
        if (r_blk == 0) KS = 0;
    }
    int k_first = 0;                                  // first stage of this workgroup's slice
    int k_wrap = -1;                                  // stages issued when a rotated walk wraps to stage 0
    // Shrink with 256-row tiles (65536 rows and more, token order): all workgroups would walk the
    // same columns of x at the same time, rows one leading dimension apart, which a few memory
    // channels then serve (3.8 TB/s); tile bm starts its walk at stage bm % KS and wraps around
    // instead (4.5 TB/s).  The fp32 sums of a row then run in a rotated order.
    if ((EPI == EPI_GATE || EPI == EPI_RAW) && BM == 256 && !a.perm && KS > 1) {
        k_first = bm % KS;
        k_wrap = KS - k_first;
    }
    if (EPI == EPI_PARTIAL) {
        k_first = split * a.ks_per_split;
        int k_end = k_first + a.ks_per_split;
        if (k_end > KS) k_end = KS;
        KS = k_end > k_first ? k_end - k_first : 0;
    }
    const int TS = (r_tile + BK - 1) / BK;            // stages of the second part (uhat columns
                                                      // beyond a row's rank are zero)
    const int S = KS + TS;

    // ---- loader set-up: instruction j of this wave fills rows RPI j .. RPI j + RPI - 1 of the stage ----
    const __bf16* gp[LOADS];          // current global address of this lane's 16 bytes
    int32_t grow[LOADS];              // row in the second operand pair (grouped row / column)
    int lchunk[LOADS];
    bool is_a[LOADS];
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
        const int j = wave * LOADS + i;
        const int row_cat = RPI * j + lane / CHUNKS;
        is_a[i] = (RPI * j) < BM;                     // wave-uniform
        const int r = is_a[i] ? row_cat : row_cat - BM;
        lchunk[i] = (lane % CHUNKS) ^ ((r >> SW_SHIFT) % CHUNKS);
        if (is_a[i]) {
            int64_t g = m0 + r;
            if (g > a.M - 1) g = a.M - 1;
            grow[i] = (int32_t)g;
            const int64_t t = a.perm ? (int64_t)a.perm[g] : g;
            gp[i] = static_cast<const __bf16*>(a.A1) + t * a.lda1 + lchunk[i] * 8 + (int64_t)k_first * BK;
        } else {
            int64_t n = n0 + r;
            if (n > a.N - 1) n = a.N - 1;
            grow[i] = (int32_t)n;
            gp[i] = static_cast<const __bf16*>(a.B1) + n * a.ldb1 + lchunk[i] * 8 + (int64_t)k_first * BK;
        }
    }
    int issued = 0;                   // stages issued so far (wave-uniform)
    auto issue_next = [&](int buf) {
        if (issued == KS) {
            // switch the loaders to the second operand pair (uhat, B^T)
#pragma unroll
            for (int i = 0; i < LOADS; ++i) {
                if (is_a[i])
                    gp[i] = static_cast<const __bf16*>(a.A2) + (int64_t)grow[i] * a.lda2 + lchunk[i] * 8;
                else
                    gp[i] = static_cast<const __bf16*>(a.B2) + (int64_t)grow[i] * a.ldb2 + lchunk[i] * 8;
            }
        }
        char* base = smem + buf * STAGE_BYTES + wave * LOADS * 1024;
#pragma unroll
        for (int i = 0; i < LOADS; ++i) {
            load_lds_16(gp[i], base + i * 1024);
            gp[i] += BK;
        }
        ++issued;
        if ((EPI == EPI_GATE || EPI == EPI_RAW) && issued == k_wrap) {
#pragma unroll
            for (int i = 0; i < LOADS; ++i) gp[i] -= a.K1;
        }
    };

    // ---- fragment addressing ----
    const int l32 = lane & 31, h = lane >> 5;
    const int sw = (l32 >> SW_SHIFT) % CHUNKS;
    int koff[KSTEPS];
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) koff[kk] = ((2 * kk + h) ^ sw) * 16;
    const int a_base = (wm * TM + l32) * ROW_BYTES;
    const int b_base = BM * ROW_BYTES + (wn * TN + l32) * ROW_BYTES;

    f32x16 acc[NI][MI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[ni][mi][v] = 0.0f;

    bf16x8 af[2][MI], bfr[2][NI];
    auto read_frags = [&](int buf, int kk, int f) {
        const char* sb = smem + buf * STAGE_BYTES;
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
            af[f][mi] = *reinterpret_cast<const bf16x8*>(sb + a_base + mi * 32 * ROW_BYTES + koff[kk]);
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            bfr[f][ni] = *reinterpret_cast<const bf16x8*>(sb + b_base + ni * 32 * ROW_BYTES + koff[kk]);
    };
    auto mfma_step = [&](int f) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
            if (EPI != EPI_GATE || ni_on[ni])
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    acc[ni][mi] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[f][ni], af[f][mi], acc[ni][mi], 0, 0, 0);
    };
    // issue order inside a group: one MFMA (its operands are already in registers), then the LDS
    // reads of the next k-step, then the rest
    auto order_first_half = [&]() {
        if (EPI == EPI_STORE) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, N_DS, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA - 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto order_second_half = [&]() {
        if (EPI == EPI_STORE) {
            __builtin_amdgcn_sched_group_barrier(0x100, N_DS, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x020, LOADS, 0);
            __builtin_amdgcn_sched_group_barrier(0x008, N_MFMA - 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    };
    auto stage_barrier = [&]() {
        __builtin_amdgcn_s_barrier();
        __builtin_amdgcn_sched_barrier(0);
    };

    // ---- prologue: fill the ring, wait for stage 0 ----
#pragma unroll
    for (int p = 0; p < NST; ++p)
        if (p < S) issue_next(p);
    if (S >= NST) wait_cnt<(NST - 1) * LOADS, 15>();
    else wait_cnt<0, 15>();
    stage_barrier();
    if (S > 0) read_frags(0, 0, 0);
    int buf = 0;
    int s = 0;
    // A stage is KSTEPS k-steps of 16; fragments alternate between two register sets, the next
    // k-step's set is fetched while the MFMAs of the current one run.  The stage's one barrier
    // sits before its last k-step.
    // ---- steady state: stage s releases its buffer to stage s + NST ----
    for (; s + NST < S; ++s) {
        const int nxt = (buf + 1 == NST) ? 0 : buf + 1;
#pragma unroll
        for (int kk = 0; kk + 1 < KSTEPS; ++kk) {
            read_frags(buf, kk + 1, (kk + 1) & 1);
            mfma_step(kk & 1);
            order_first_half();
        }
        wait_cnt<(NST - 2) * LOADS, 0>();   // my reads of this stage are in registers, my loads of
        stage_barrier();                    // stage s+1 have landed ... and everybody's
        read_frags(nxt, 0, 0);
        issue_next(buf);
        mfma_step((KSTEPS - 1) & 1);
        order_second_half();
        buf = nxt;
    }
    // ---- drain: nothing left to issue ----
    for (; s < S; ++s) {
        const int nxt = (buf + 1 == NST) ? 0 : buf + 1;
#pragma unroll
        for (int kk = 0; kk + 1 < KSTEPS; ++kk) {
            read_frags(buf, kk + 1, (kk + 1) & 1);
            mfma_step(kk & 1);
            order_first_half();
        }
        if (s + 1 < S) {
            wait_cnt<0, 0>();
            stage_barrier();
            read_frags(nxt, 0, 0);
        }
        mfma_step((KSTEPS - 1) & 1);
        __builtin_amdgcn_sched_barrier(0);
        buf = nxt;
    }

    // ---- epilogue ----
    // accumulator register v of block (ni, mi): column n = ni*32 + 8*(v/4) + 4*h + v%4,
    // row m = mi*32 + l32 (relative to the wave tile)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int64_t g = m0 + wm * TM + mi * 32 + l32;
        if (g >= a.M) continue;
        if (EPI == EPI_PARTIAL || EPI == EPI_RAW) {
            float* prow = a.partial + split * a.partial_stride + g * a.ldp;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const int64_t n = n0 + wn * TN + ni * 32 + q * 8 + h * 4;
                    if (n >= a.N) continue;
                    f32x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = acc[ni][mi][q * 4 + e];
                    *reinterpret_cast<f32x4*>(prow + n) = o;
                }
            continue;
        }
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
                        const int32_t i = (a.gate_period > 0 ? (int32_t)(n % a.gate_period) : (int32_t)n) + e;
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

template <int BM, int BN, int WM, int WN, int NST, int EPI, int BK = 32>
__global__ void __launch_bounds__(WM * WN * 64) gemm_bf16_tn_kernel(GemmArgs a) {
    gemm_bf16_tn_body<BM, BN, WM, WN, NST, EPI, BK>(a, (int)blockIdx.x);
}

// Split-reduction launch: the first job.n_blocks workgroups fill the rows' gate table, 256 tokens
// each (the chain of dependent lookups takes as long as a short product and runs beside it; each
// wavefront also reduces the largest effective rank of its 64 rows into job.blk_r), the
// workgroups after them compute the partial products.
template <int BM, int BN, int WM, int WN, int NST>
__global__ void __launch_bounds__(WM * WN * 64) partial_bf16_kernel(GemmArgs a, MetaJob job) {
    static_assert(WM * WN * 64 == 256, "a gate-table block is 256 tokens");
    if ((int)blockIdx.x < job.n_blocks) {
        __shared__ int32_t lad_ranks[CWL_MAX_LADDER];
        __shared__ float lad_scales[CWL_MAX_LADDER];
        ladder_to_lds(job.lad, lad_ranks, lad_scales);
        __syncthreads();
        const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
        TokMeta m = {0, 0, 0.0f, 0.0f};
        if (t < a.M) {
            m = token_meta_of(t, job.seq_offsets, job.n_seqs, job.chunk_offsets, job.chunk_start,
                              job.chunk_len, job.rank_idx, job.chunk_cap, job.lad.K, lad_ranks, lad_scales,
                              job.blend_w);
            job.meta[t] = m;
        }
        if (job.blk_r) {
            int32_t r_eff = m.r_cur > m.r_prev ? m.r_cur : m.r_prev;
#pragma unroll
            for (int off = 32; off >= 1; off >>= 1) {
                const int32_t o = __shfl_xor(r_eff, off);
                r_eff = o > r_eff ? o : r_eff;
            }
            const int64_t blk = t / kRankBlock;
            if ((threadIdx.x & 63) == 0) job.blk_r[blk] = r_eff;   // all four entries of the 256 rows
        }
        return;
    }
    gemm_bf16_tn_body<BM, BN, WM, WN, NST, EPI_PARTIAL, 64>(a, (int)blockIdx.x - job.n_blocks);
}

template <int BM, int BN, int WM, int WN, int NST>
cwl_status launch_partial_cfg(GemmArgs a, const MetaJob& job, hipStream_t st) {
    constexpr int BK = 64;
    constexpr int smem_bytes = NST * (BM + BN) * BK * 2;
    static_assert(smem_bytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    if (a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
    if (a.splits < 1 || a.ks_per_split < 1 || !a.partial) return CWL_ERR_INVALID_ARG;
    auto kern = partial_bf16_kernel<BM, BN, WM, WN, NST>;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem_bytes, lds_set) != CWL_OK) return CWL_ERR_DEVICE;
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    if (job.n_blocks < 0 || (job.n_blocks > 0 && !job.meta)) return CWL_ERR_INVALID_ARG;
    const int64_t grid = (int64_t)a.tiles_m * a.tiles_n * a.splits + job.n_blocks;
    if (grid >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    kern<<<dim3((unsigned)grid), dim3(WM * WN * 64), smem_bytes, st>>>(a, job);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

// The short-sequence chunker and the ungated shrink in one launch: workgroups 0 .. n_seqs - 1 chunk
// one sequence each (a chain of dependent look-ups on one wavefront: 20-odd microseconds during which
// the chip would otherwise idle), the workgroups behind them compute x A, which needs the memory
// bandwidth and nothing the chunker produces.  Both parts use the launch's dynamic LDS from its start.
template <int BM, int BN, int WM, int WN, int NST>
__global__ void __launch_bounds__(WM * WN * 64) seq_shrink_raw_kernel(GemmArgs a, part::SeqJob job) {
    static_assert(WM * WN * 64 == part::kThreads, "the chunker's workgroup");
    if ((int)blockIdx.x < job.n_seqs) {
        extern __shared__ __attribute__((aligned(1024))) char smem[];
        part::partition_seq_body(job, (int32_t)blockIdx.x, smem);
        return;
    }
    // A head start for the chunker: its first loads (scores, offsets) are a short chain of round trips to
    // memory, which the product's stream would queue behind its own.  Measured on 8 sequences x 2048 tokens
    // beside 256 product tiles: no delay 29.4 us, 0.8 us 28.0, 1.7 us 27.0, 3.4 us 27.0, 6.8 us 30.1
    // (chunker alone 20.4, product alone 23.2).
    __builtin_amdgcn_s_sleep(96);
    gemm_bf16_tn_body<BM, BN, WM, WN, NST, EPI_RAW, 64>(a, (int)blockIdx.x - job.n_seqs);
}

template <int BM, int BN, int WM, int WN, int NST>
cwl_status launch_seq_shrink_cfg(part::SeqJob job, GemmArgs a, hipStream_t st) {
    constexpr int BK = 64;
    constexpr int smem_bytes = NST * (BM + BN) * BK * 2;
    static_assert(2 * smem_bytes <= 160 * 1024, "two workgroups per compute unit, so that the chunker's fit beside the product's");
    if (a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
    auto kern = seq_shrink_raw_kernel<BM, BN, WM, WN, NST>;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem_bytes, lds_set) != CWL_OK) return CWL_ERR_DEVICE;
    job.lds_tokens = (int32_t)(smem_bytes / part::kSeqLdsPerToken);
    a.tiles_m = (int32_t)((a.M + BM - 1) / BM);
    a.tiles_n = (int32_t)((a.N + BN - 1) / BN);
    const int64_t n_tiles = (int64_t)a.tiles_m * a.tiles_n;
    const int64_t grid = (n_tiles + 7) / 8 * 8 + job.n_seqs;
    if (grid >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    kern<<<dim3((unsigned)grid), dim3(WM * WN * 64), smem_bytes, st>>>(a, job);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

template <int BM, int BN, int WM, int WN, int NST, int EPI, int BK = 32>
cwl_status launch_cfg(GemmArgs a, hipStream_t st) {
    constexpr int smem_bytes = NST * (BM + BN) * BK * 2;
    static_assert(smem_bytes <= 160 * 1024, "LDS budget of a gfx950 compute unit");
    if (a.K1 % BK != 0) return CWL_ERR_UNSUPPORTED;
    auto kern = gemm_bf16_tn_kernel<BM, BN, WM, WN, NST, EPI, BK>;
    static PerDeviceFlag lds_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(kern), smem_bytes, lds_set) != CWL_OK) return CWL_ERR_DEVICE;
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
    // 64-row tiles (one rank block), all padded directions as columns.  The shrink streams x once
    // from HBM: stages of BK = 64 (whole 128-byte lines per load instruction) and rings deep enough
    // to cover the memory latency with bytes in flight.
    // Every workgroup re-reads A^T from L2, as many bytes as it reads of x when the tile is 64 x 64;
    // with enough rows to keep all compute units busy, 256-row tiles quarter that.
    // Several adapters side by side (a group of projections) are column tiles of the same launch: the
    // tile order keeps the column tiles of eight row tiles on one XCD at the same time, so x comes
    // from HBM once and from that L2 for the other column tiles.
    if (a.M >= kShrinkTallRows) {
        if (a.N % 128 == 0) return launch_cfg<256, 128, 2, 2, 3, EPI_GATE, 64>(a, st);
        if (a.N % 64 == 0) return launch_cfg<256, 64, 2, 2, 4, EPI_GATE, 64>(a, st);
    }
    switch (a.N) {
        case 64: return launch_cfg<64, 64, 2, 2, 6, EPI_GATE, 64>(a, st);
        case 128: return launch_cfg<64, 128, 2, 2, 4, EPI_GATE, 64>(a, st);
        case 192: return launch_cfg<64, 192, 2, 2, 4, EPI_GATE, 64>(a, st);
        case 256: return launch_cfg<64, 256, 2, 2, 3, EPI_GATE, 64>(a, st);
        default: return CWL_ERR_UNSUPPORTED;
    }
}

// The shrink without its gate: x A in fp32, every direction, the same tiles, rings and order of
// summation as launch_shrink_bf16 (a.partial [M, a.ldp] receives it; token order only).
cwl_status launch_shrink_raw_bf16(const GemmArgs& a, hipStream_t st) {
    if (a.perm || !a.partial) return CWL_ERR_INVALID_ARG;
    if (a.M >= kShrinkTallRows) {
        if (a.N % 128 == 0) return launch_cfg<256, 128, 2, 2, 3, EPI_RAW, 64>(a, st);
        if (a.N % 64 == 0) return launch_cfg<256, 64, 2, 2, 4, EPI_RAW, 64>(a, st);
    }
    switch (a.N) {
        case 64: return launch_cfg<64, 64, 2, 2, 6, EPI_RAW, 64>(a, st);
        case 128: return launch_cfg<64, 128, 2, 2, 4, EPI_RAW, 64>(a, st);
        case 192: return launch_cfg<64, 192, 2, 2, 4, EPI_RAW, 64>(a, st);
        case 256: return launch_cfg<64, 256, 2, 2, 3, EPI_RAW, 64>(a, st);
        default: return CWL_ERR_UNSUPPORTED;
    }
}

cwl_status launch_seq_shrink_raw_bf16(const part::SeqJob& job, const GemmArgs& a, hipStream_t st) {
    if (a.perm || !a.partial || a.M >= kShrinkTallRows || job.n_seqs < 1) return CWL_ERR_UNSUPPORTED;
    // rings of 64 and 72 KiB (the one-pass shrink's own are deeper; its stream runs as fast on these)
    if (a.N == 64) return launch_seq_shrink_cfg<64, 64, 2, 2, 4>(job, a, st);
    if (a.N == 128) return launch_seq_shrink_cfg<64, 128, 2, 2, 3>(job, a, st);
    return CWL_ERR_UNSUPPORTED;
}

// fp32 partial products over slices of the reduction dimension, for a few hundred rows at most: the
// tile shape comes with the plan (small_rows_plan), the rings are shallow enough for two or three
// workgroups per compute unit.
cwl_status launch_partial_bf16(const GemmArgs& a, const MetaJob& job, hipStream_t st) {
    if (a.M_tile == 256) return launch_partial_cfg<256, 128, 2, 2, 3>(a, job, st);
    if (a.M_tile == 32) return launch_partial_cfg<32, 128, 1, 4, 3>(a, job, st);
    if (a.M <= 64 && a.three_per_cu) return launch_partial_cfg<64, 64, 2, 2, 3>(a, job, st);
    if (a.M <= 64) return launch_partial_cfg<64, 64, 2, 2, 4>(a, job, st);
    if (a.N_tile == 64 && a.three_per_cu) return launch_partial_cfg<128, 64, 2, 2, 2>(a, job, st);
    if (a.N_tile == 64) return launch_partial_cfg<128, 64, 2, 2, 3>(a, job, st);
    return launch_partial_cfg<128, 128, 2, 2, 4>(a, job, st);
}

// Two-part product with 64-bit lane addresses (rows gathered through a.perm).
cwl_status launch_main_bf16_general(const GemmArgs& a, hipStream_t st) {
    return launch_cfg<256, 256, 2, 4, 4, EPI_STORE>(a, st);
}


// The same with 128 x 128 tiles, four waves and stages of 64: for products with too few 256 x 256
// tiles to occupy the compute units.
cwl_status launch_main_bf16_tile128(const GemmArgs& a, hipStream_t st) {
    return launch_cfg<128, 128, 2, 2, 4, EPI_STORE, 64>(a, st);
}

cwl_status launch_main_bf16_tile256x128(const GemmArgs& a, hipStream_t st) {
    return launch_cfg<256, 128, 2, 2, 3, EPI_STORE, 64>(a, st);
}

}  // namespace cwl
