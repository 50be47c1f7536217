// Types shared by the pieces of cwl_chunkwise_lora_linear (gfx950 only).
//
// The adapter and the cross-fade are written as one gated product.  With u_t = x_t A (all r_max
// stored directions) and the per-token, per-direction gate
//      G[t, i] = g_prev(t) * [i < r_prev(t)] + g_cur(t) * [i < r_cur(t)]
// (g_cur = s_cur outside a cross-fade window; inside it g_cur = lambda * s_cur and
// g_prev = (1 - lambda) * s_prev), the layer of Sec. III-C / III-D is
//      y_t = x_t W + (u_t * G[t, :]) B .
// So a "shrink" GEMM produces uhat = (x A) * G and the main GEMM runs over the concatenated
// reduction dimension [x | uhat] . [W ; B]; a row tile only walks as much of the second part as
// the largest rank among its rows needs.
#pragma once
#include "common.h"

namespace cwl {

struct TokMeta {          // 16 bytes per token
    int32_t r_cur, r_prev;
    float g_cur, g_prev;
};

struct Ladder {
    int32_t ranks[CWL_MAX_LADDER];
    float scales[CWL_MAX_LADDER];
    int32_t K;
};

constexpr int kRankBlock = 64;    // rows per entry of the block-rank table
constexpr int64_t kShrinkTallRows = 65536;   // from this many rows up the bf16 shrink uses 256-row tiles
constexpr int kRankPad = 64;      // the stored rank dimension is padded to a multiple of this

inline int32_t padded_rank(int32_t r_max) {
    int32_t r = r_max < 1 ? 1 : r_max;
    return (r + kRankPad - 1) / kRankPad * kRankPad;
}

// Operands of one "TN" GEMM launch: C[m, n] = sum_k A1[m,k] B1[n,k] + sum_{k<r(tile)} A2[m,k] B2[n,k].
// Row m of the tile space is "grouped row" g; the token it stands for is perm[g] (g when perm is
// NULL).  A1 and C and meta are indexed by token, A2 and blk_r by grouped row.
struct GemmArgs {
    const void* A1;
    int64_t lda1;
    const void* B1;
    int64_t ldb1;
    int32_t K1;
    const void* A2;
    int64_t lda2;
    const void* B2;
    int64_t ldb2;
    const int32_t* blk_r;   // [ceil(M / kRankBlock)] largest effective rank per block of rows:
                            // length of the second reduction part of a row tile (NULL: none)
    const int32_t* gate_blk_r;  // EPI_GATE only: same table, limits the output columns computed
    int64_t M, N;
    void* C;
    int64_t ldc;
    const TokMeta* meta;
    const int32_t* perm;
    int32_t tiles_m, tiles_n;
    // EPI_PARTIAL (split reduction): workgroup v computes stages [split * ks_per_split, + ks_per_split)
    // of the first part for tile v / splits, split = v % splits, and leaves its fp32 tile at
    // partial[split * partial_stride + m * ldp + n]
    int32_t splits, ks_per_split;
    float* partial;
    int64_t ldp, partial_stride;
    int32_t N_tile;         // EPI_PARTIAL: column tile the plan was made for (64 or 128)
    int32_t M_tile;         // EPI_PARTIAL: row tile of the plan (256: tiles of 256 x 128; else by M and N_tile)
    int32_t three_per_cu;   // EPI_PARTIAL, M <= 64: the plan counts on three workgroups per compute unit (shallower ring)
    int32_t gate_period;    // EPI_GATE: output column n is direction n % gate_period of its adapter (several
                            // adapters of one padded rank side by side); 0: direction n
};

// EPI_STORE: C = result in the launch's element type.  EPI_GATE: C[g, n] = result * G[perm[g], n].
// EPI_PARTIAL: fp32 partial sums of a slice of the reduction dimension (see GemmArgs).
// EPI_RAW: the product in fp32 at partial[m * ldp + n], no gate (the first phase of the two-phase call).
enum { EPI_STORE = 0, EPI_GATE = 1, EPI_PARTIAL = 2, EPI_RAW = 3 };

cwl_status launch_gemm_f32(const GemmArgs& a, int epi, hipStream_t st);
cwl_status launch_shrink_bf16(const GemmArgs& a, hipStream_t st);   // a.N = padded rank
cwl_status launch_shrink_raw_bf16(const GemmArgs& a, hipStream_t st);   // x A in fp32, ungated (EPI_RAW)
// the same product (64-row tiles, a.N = 64 or 128) behind the job.n_seqs workgroups of the short-sequence
// chunker in one launch; CWL_ERR_UNSUPPORTED for other shapes
namespace part { struct SeqJob; }
cwl_status launch_seq_shrink_raw_bf16(const part::SeqJob& job, const GemmArgs& a, hipStream_t st);
cwl_status launch_main_bf16(const GemmArgs& a, hipStream_t st);
// shrink of several adapters side by side (a.N >= 192 directions, gate period a.gate_period) on
// kShrinkTallRows rows or more, token order: the persistent 256 x 256 kernel with a gated epilogue
bool shrink_wide_bf16_serves(const GemmArgs& a);
cwl_status launch_shrink_wide_bf16(const GemmArgs& a, hipStream_t st);
cwl_status launch_main_bf16_general(const GemmArgs& a, hipStream_t st);   // any a.perm
cwl_status launch_main_bf16_tile128(const GemmArgs& a, hipStream_t st);   // 128 x 128 tiles
cwl_status launch_main_bf16_tile256x128(const GemmArgs& a, hipStream_t st);
// the gate table of rows 0 .. M-1, filled by the first workgroups of a split-reduction launch
struct MetaJob {
    const int32_t* seq_offsets;
    const int32_t* chunk_offsets;
    const int32_t* chunk_start;
    const int32_t* chunk_len;
    const int32_t* rank_idx;
    int32_t n_seqs, chunk_cap, blend_w;
    Ladder lad;
    TokMeta* meta;           // [M]
    int32_t* blk_r;          // [ceil(M / 64)] largest effective rank per 64 rows, or NULL
    int32_t n_blocks;        // ceil(M / 256), or 0: the caller brought the gate entries
};
cwl_status launch_partial_bf16(const GemmArgs& a, const MetaJob& job, hipStream_t st);   // EPI_PARTIAL

// ---- few rows (linear_small.hip): bf16, packed weights, token order ----
constexpr int64_t kSmallRows = 512;
struct SmallPlan {
    int32_t splits, ks_per_split, n_tile, m_tile, three_per_cu;
    int64_t ldp, partial_stride;      // elements
    size_t partial_bytes;
};
// Projections that share x, side by side: projection p owns output columns [col0[p], col0[p] + cols[p])
// of the wide product and directions [p R, (p + 1) R) of the concatenated adapters (R = padded rank).
constexpr int kMaxGroup = CWL_MAX_GROUP;
struct GroupCols {
    int32_t n_proj;
    int64_t col0[kMaxGroup], cols[kMaxGroup];
};
// d->d_out: all output columns; the concatenated adapters have grp.n_proj * padded_rank(d->r_max) directions
SmallPlan small_rows_plan(const cwl_linear_desc* d, int32_t n_proj);
// wt_at: W^T [d_out, d_in] directly followed by A^T [n_proj * padded rank, d_in]; bt: B^T [d_out, padded rank]
cwl_status run_small_rows(const cwl_linear_desc* d, const GroupCols& grp, const void* x, const void* wt_at,
                          const void* bt, const int32_t* seq_offsets, int32_t n_seqs,
                          const int32_t* chunk_offsets, const int32_t* chunk_start, const int32_t* chunk_len,
                          const int32_t* rank_idx, int32_t chunk_cap, void* y, float* partial, TokMeta* meta,
                          const TokMeta* gate, hipStream_t st);   // gate != NULL: use these entries, leave the chunk table alone

// ---- one row (linear_gemv.hip): bf16, token order, a projection or a group of them ----
bool gemv_rows_serves(const cwl_linear_desc* d);
// wt / at / bt: W^T, A^T, B^T of the packed weights; u: (projections x padded rank) floats of scratch; meta: one
// entry of scratch, filled from the chunk table when gate is NULL
cwl_status run_gemv_rows(const cwl_linear_desc* d, const GroupCols& grp, const void* x, const void* wt, const void* at, const void* bt,
                         const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
                         const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                         int32_t chunk_cap, const TokMeta* gate, void* y, float* u, TokMeta* meta, hipStream_t st);

}  // namespace cwl
