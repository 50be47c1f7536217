// cwl_chunkwise_lora_linear for a few rows (decode steps, short prompts), bf16, packed weights.
//
// With a few hundred rows at most the layer is bound by streaming the weights once from HBM, and a grid of
// output tiles alone is far too small to have enough bytes in flight.  Two launches:
//   1. Partial products and gate table.  W^T and A^T lie back to back in the packed weights, so
//      P = x . [W | A] is one product with d_out + R output columns.  It is cut into tiles of 64
//      or 128 columns and into slices of the reduction dimension, one workgroup each (several
//      hundred in all, small_rows_plan), every one leaving an fp32 tile in the workspace (the matrix-core kernel of
//      gemm_bf16.hip with the EPI_PARTIAL epilogue).  One or two more workgroups of the same
//      launch look up the rows' gate entries (token_meta.h): a chain of dependent loads that
//      takes as long as the products.
//   2. Fix-up.  Per 16 rows x 128 columns:
//      uhat = gate * (sum over slices of the last R columns of P), rounded to bf16 as on the
//      large path, then y = sum over slices of P + uhat . B with the matrix cores (B^T fragments
//      straight from global memory), rounded once to bf16.
// Sums over slices run in slice order: the result does not depend on scheduling.
// (Formulation: linear_common.h; Sec. III-C / III-D of arxiv 2601.21109.)
#include "mfma_util.h"
#include "token_meta.h"

namespace cwl {
namespace {

using namespace mfma;

typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kFixRows = 16, kFixCols = 128;      // outputs of one fix-up workgroup (4 waves x 2 blocks)
constexpr int kUhPad = 8;                         // bf16 elements of padding per uhat row in LDS
constexpr int kMaxRankPadded = (CWL_MAX_RANK + kRankPad - 1) / kRankPad * kRankPad;

// SP: compile-time bound on the number of slices (the sums are unrolled to it; slices past the
// real count re-read slice 0 and are dropped).  All addresses are clamped into the buffers instead
// of being predicated, so the kernel is straight-line code and every load is in flight before the
// first value is needed: with a few hundred bytes per thread it is pure memory latency.
template <int SP>
__global__ void __launch_bounds__(256)
small_fixup_kernel(int64_t n_rows, int64_t d_out_all, GroupCols grp, int32_t R, const float* __restrict__ partial,
                   int32_t splits, int64_t ldp, int64_t pstride, const __bf16* __restrict__ Bt_all,
                   const TokMeta* __restrict__ meta, __bf16* __restrict__ y_all, int64_t ldy) {
    // projection blockIdx.z of the group: its columns of the wide product, its directions of the
    // concatenated adapters (columns d_out_all + proj R ... of the partial products), its rows of B^T
    const int proj = blockIdx.z;
    int64_t pc0 = 0, d_out = 0;
#pragma unroll
    for (int q = 0; q < kMaxGroup; ++q)
        if (q == proj) { pc0 = grp.col0[q]; d_out = grp.cols[q]; }
    if ((int64_t)blockIdx.x * kFixCols >= d_out) return;
    const int64_t u_col0 = d_out_all + (int64_t)proj * R;
    const __bf16* Bt = Bt_all + pc0 * R;
    __bf16* y = y_all + pc0;
    const float* part_w = partial + pc0;                            // this projection's columns of x W
    extern __shared__ __attribute__((aligned(16))) char dyn[];      // uhat: kFixRows x (R + kUhPad) bf16
    __bf16* uh = reinterpret_cast<__bf16*>(dyn);
    const int ldu = R + kUhPad;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t row0 = (int64_t)blockIdx.y * kFixRows;
    const int64_t col0 = (int64_t)blockIdx.x * kFixCols;
    int64_t soff[SP];                                               // slice offsets, clamped
#pragma unroll
    for (int s = 0; s < SP; ++s) soff[s] = (s < splits ? s : 0) * pstride;

    // (a) raw u = sum over the slices of x A, in slice order.  Thread (w, l) takes rows w, w+4,
    // w+8, w+12 of the 16 and directions l, l+64, ...
    float u_raw[4][kMaxRankPadded / 64];
    TokMeta mt[4];
#pragma unroll
    for (int mj = 0; mj < 4; ++mj) {
        int64_t g = row0 + wave + 4 * mj;
        if (g > n_rows - 1) g = n_rows - 1;
        mt[mj] = meta[g];
#pragma unroll
        for (int ij = 0; ij < kMaxRankPadded / 64; ++ij) {
            u_raw[mj][ij] = 0.0f;
            if (ij * 64 < R) {                                      // uniform
                const float* p = partial + g * ldp + u_col0 + ij * 64 + lane;
                float v[SP];
#pragma unroll
                for (int s = 0; s < SP; ++s) v[s] = p[soff[s]];
#pragma unroll
                for (int s = 0; s < SP; ++s) u_raw[mj][ij] += s < splits ? v[s] : 0.0f;
            }
        }
    }
    // (b) this lane's slice sums of x W and its B^T fragments (first MFMA operand: a lane ends
    // with 4 consecutive columns of row lane % 16)
    const int l16 = lane & 15, g4 = lane >> 4;
    const int64_t g = row0 + l16;
    const int64_t gc = g > n_rows - 1 ? n_rows - 1 : g;
    f32x4 sum[2];
    bf16x8 wf[2][kMaxRankPadded / 32];
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t cb = col0 + wave * 32 + b * 16;
        int64_t n = cb + g4 * 4;
        if (n > d_out - 4) n = d_out - 4;                        // columns past the end are not stored
        const float* p = part_w + gc * ldp + n;
        f32x4 v[SP];
#pragma unroll
        for (int s = 0; s < SP; ++s) v[s] = *reinterpret_cast<const f32x4*>(p + soff[s]);
        sum[b] = (f32x4){0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int s = 0; s < SP; ++s)
            if (s < splits) sum[b] += v[s];
        int64_t wrow = cb + l16;
        if (wrow > d_out - 1) wrow = d_out - 1;
#pragma unroll
        for (int k = 0; k < kMaxRankPadded / 32; ++k)
            if (k * 32 < R) wf[b][k] = *reinterpret_cast<const bf16x8*>(Bt + wrow * R + k * 32 + g4 * 8);
    }
    // uhat = gate * u, rounded to bf16
#pragma unroll
    for (int mj = 0; mj < 4; ++mj)
#pragma unroll
        for (int ij = 0; ij < kMaxRankPadded / 64; ++ij)
            if (ij * 64 < R) {
                const int i = ij * 64 + lane;
                const float gate = (i < mt[mj].r_prev ? mt[mj].g_prev : 0.0f) + (i < mt[mj].r_cur ? mt[mj].g_cur : 0.0f);
                uh[(wave + 4 * mj) * ldu + i] = (__bf16)(u_raw[mj][ij] * gate);
            }
    __syncthreads();

    // y block (16 rows x 16 columns) = sum of slices + uhat . B
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int64_t cb = col0 + wave * 32 + b * 16;
        f32x4 acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
        for (int k = 0; k < kMaxRankPadded / 32; ++k)
            if (k * 32 < R) {
                const bf16x8 xf = *reinterpret_cast<const bf16x8*>(uh + l16 * ldu + k * 32 + g4 * 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[b][k], xf, acc, 0, 0, 0);
            }
        const int64_t n = cb + g4 * 4;
        if (g < n_rows && n < d_out) {                           // d_out % 8 == 0: 4 columns in or out together
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (__bf16)(sum[b][e] + acc[e]);
            *reinterpret_cast<bf16x4*>(y + g * ldy + n) = o;
        }
    }
}

template <int SP>
cwl_status launch_fixup(const cwl_linear_desc* d, const GroupCols& grp, int32_t R, const SmallPlan& p,
                        const float* partial, const void* bt, const TokMeta* meta, void* y, hipStream_t st) {
    int64_t widest = 0;
    for (int q = 0; q < grp.n_proj; ++q) widest = grp.cols[q] > widest ? grp.cols[q] : widest;
    const dim3 grid((unsigned)((widest + kFixCols - 1) / kFixCols), (unsigned)((d->n_rows + kFixRows - 1) / kFixRows),
                    (unsigned)grp.n_proj);
    const size_t lds = sizeof(__bf16) * kFixRows * (size_t)(R + kUhPad);
    small_fixup_kernel<SP><<<grid, dim3(256), lds, st>>>(
        d->n_rows, d->d_out, grp, R, partial, p.splits, p.ldp, p.partial_stride, static_cast<const __bf16*>(bt),
        meta, static_cast<__bf16*>(y), d->ldy);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace

// How the reduction dimension is cut for n_rows <= kSmallRows.  Enough workgroups to have the
// weights in flight everywhere (about two per compute unit), at least four stages of 64 each, and
// partial sums that stay well below the bytes of the weights themselves.
SmallPlan small_rows_plan(const cwl_linear_desc* d, int32_t n_proj) {
    SmallPlan p = {};
    const int64_t R = (int64_t)n_proj * padded_rank(d->r_max);     // directions of all adapters side by side
    const int64_t n_cols = d->d_out + R;
    int64_t bm = d->n_rows <= 64 ? 64 : 128;
    p.n_tile = d->n_rows <= 256 ? 64 : 128;           // from 257 rows the tile count suffices with 128 x 128
    int64_t tiles = (n_cols + p.n_tile - 1) / p.n_tile * ((d->n_rows + bm - 1) / bm);
    int64_t bytes_cap = d->d_in / (4 * d->n_rows);    // partial sums <= half the weights' bytes
    if (p.n_tile == 128 && tiles * 2 > 256) {
        // 128 x 128 tiles (one workgroup per compute unit) that cannot even be cut in two within one round of
        // workgroups: tiles of 256 x 128 instead, a third fewer bytes per flop, and the reduction dimension cut
        // further (partial sums up to the weights' bytes)
        bm = 256;
        tiles = (n_cols + 127) / 128 * ((d->n_rows + 255) / 256);
        bytes_cap = d->d_in / (2 * d->n_rows);
    }
    p.m_tile = (int32_t)bm;
    const int64_t stages = d->d_in / 64;
    if (d->n_rows <= 16 && (n_cols + 127) / 128 <= 64 && stages >= 8 && stages <= 64) {
        // Up to 16 rows, up to 8192 columns, d_in up to 4096: tiles of 32 rows x 128 columns in 8 slices.  Every column tile re-reads
        // its slice of x, and what bounds the launch is the bytes that go into LDS: with 128 columns per tile x is
        // a fifth of them instead of half.  Whole calls from a HIP graph, 4096 -> 4096: 12.0 / 13.0 / 14.5 us for
        // 2 / 8 / 16 rows against 13.7 / 14.4 / 15.4 us with 64 x 64 tiles in 4 slices (4 slices of the wide tiles:
        // 15.2 / 17.8 / 18.7 us, 15 slices: 13.8 / 15.4 / 17.7 us); 4096 -> 6144: 16.4 / 18.8 against 17.5 / 19.0 us
        // for 2 / 16 rows; at 32 rows the two are level.  Longer reductions stay with the 64 x 64 tiles: 8192 -> 4096
        // is level (19.1 / 21.8 against 18.7 / 21.2 us; 12 slices 17.2 / 21.2), 11008 -> 4096 slower with 8, 12 or 15
        // slices (25.7, 24.7, 23.0 us against 22.5 us for 2 rows; 28.4, 28.5, 27.0 against 25.1 us for 16).
        // For 17 to 64 rows tiles of 64 rows x 128 columns gave nothing (6 slices: 15.2 / 15.8 / 17.0 us for 17 / 32 /
        // 64 rows against 15.3 / 16.1 / 17.6 us; 8 slices and 4096 -> 6144 slower).
        p.n_tile = 128;
        p.m_tile = 32;
        p.ks_per_split = (int32_t)((stages + 7) / 8);
        p.splits = (int32_t)((stages + p.ks_per_split - 1) / p.ks_per_split);
        p.ldp = n_cols;
        p.partial_stride = d->n_rows * n_cols;
        p.partial_bytes = sizeof(float) * (size_t)p.splits * (size_t)p.partial_stride;
        return p;
    }
    int64_t s = (p.n_tile == 64 ? 512 : 256) / tiles;   // what fits at once: two (one) workgroups per compute unit
    if (p.n_tile == 64 && s < 3) {
        // wide outputs leave room for one or two slices only (173 tiles of 4096 -> 11008: 346 workgroups on 256
        // compute units); with a ring one stage shallower three workgroups fit on a unit, and 4 slices of
        // 4096 -> 11008 stream the weights 20 % faster than 2 (64 rows: 19 against 24 us; 256 rows: 39 against 47).
        // With three slices or more already, the deeper ring is the better one.
        s = 768 / tiles;
        p.three_per_cu = 1;
    }
    // Slices shorter than sixteen stages do not make the products any faster, they only give the fix-up more to
    // add (4096 -> 4096, 64 rows: 7 slices 11.0 + 7.5 us, 4 slices 10.7 + 6.5 us; 128 rows: 14.5 + 8.4 against
    // 14.1 + 6.7 us)
    if (p.n_tile == 64) {
        const int64_t cap = stages / 16 > 2 ? stages / 16 : 2;
        if (s > cap) s = cap;
    }
    if (s > stages / 4) s = stages / 4;
    if (s > bytes_cap) s = bytes_cap;
    if (s > 32) s = 32;
    if (s < 1) s = 1;
    p.ks_per_split = (int32_t)((stages + s - 1) / s);
    p.splits = (int32_t)((stages + p.ks_per_split - 1) / p.ks_per_split);
    p.ldp = n_cols;
    p.partial_stride = d->n_rows * n_cols;
    p.partial_bytes = sizeof(float) * (size_t)p.splits * (size_t)p.partial_stride;
    return p;
}

cwl_status run_small_rows(const cwl_linear_desc* d, const GroupCols& grp, const void* x, const void* wt_at,
                          const void* bt, const int32_t* seq_offsets, int32_t n_seqs,
                          const int32_t* chunk_offsets, const int32_t* chunk_start, const int32_t* chunk_len,
                          const int32_t* rank_idx, int32_t chunk_cap, void* y, float* partial, TokMeta* meta,
                          const TokMeta* gate, hipStream_t st) {
    if (d->dt != CWL_BF16 || d->n_rows < 1 || d->n_rows > kSmallRows) return CWL_ERR_UNSUPPORTED;
    const SmallPlan p = small_rows_plan(d, grp.n_proj);
    const int32_t R = padded_rank(d->r_max);                       // of one adapter

    GemmArgs pa = {};
    pa.A1 = x;          pa.lda1 = d->ldx;
    pa.B1 = wt_at;      pa.ldb1 = d->d_in;
    pa.K1 = (int32_t)d->d_in;
    pa.M = d->n_rows;   pa.N = d->d_out + (int64_t)grp.n_proj * R;
    pa.N_tile = p.n_tile;
    pa.M_tile = p.m_tile;
    pa.three_per_cu = p.three_per_cu;
    pa.splits = p.splits;
    pa.ks_per_split = p.ks_per_split;
    pa.partial = partial;
    pa.ldp = p.ldp;
    pa.partial_stride = p.partial_stride;
    MetaJob job = {};
    job.seq_offsets = seq_offsets;
    job.chunk_offsets = chunk_offsets;
    job.chunk_start = chunk_start;
    job.chunk_len = chunk_len;
    job.rank_idx = rank_idx;
    job.n_seqs = n_seqs;
    job.chunk_cap = chunk_cap;
    job.blend_w = d->blend_w;
    job.lad.K = d->K;
    for (int32_t k = 0; k < d->K; ++k) {
        job.lad.ranks[k] = d->ranks[k];
        job.lad.scales[k] = d->scales[k];
    }
    job.meta = meta;
    job.n_blocks = gate ? 0 : (int32_t)((d->n_rows + 255) / 256);
    prof_begin(CWL_PROF_MAIN, st);
    cwl_status s = launch_partial_bf16(pa, job, st);
    prof_end(CWL_PROF_MAIN, st);
    if (s != CWL_OK) return s;

    for (int q = 0; q < grp.n_proj; ++q)
        if (grp.cols[q] < 8) return CWL_ERR_UNSUPPORTED;
    prof_begin(CWL_PROF_META, st);
    const TokMeta* mt = gate ? gate : meta;
    if (p.splits <= 2) s = launch_fixup<2>(d, grp, R, p, partial, bt, mt, y, st);
    else if (p.splits <= 4) s = launch_fixup<4>(d, grp, R, p, partial, bt, mt, y, st);
    else if (p.splits <= 8) s = launch_fixup<8>(d, grp, R, p, partial, bt, mt, y, st);
    else if (p.splits <= 16) s = launch_fixup<16>(d, grp, R, p, partial, bt, mt, y, st);
    else s = launch_fixup<32>(d, grp, R, p, partial, bt, mt, y, st);
    prof_end(CWL_PROF_META, st);
    if (s != CWL_OK) return s;
    return CWL_OK;
}

}  // namespace cwl
