// The layer on ONE row (a decode step of a single sequence): y = x W + uhat B as matrix-vector products
// on the vector ALUs (Sec. III-C / III-D of arxiv 2601.21109; Sec. III-A, III-F run the scheduler at each
// decode step).
//
// With one row the layer is one pass over the weights, and the tiled paths spend their time elsewhere: the
// split-reduction path streams W^T through a few hundred workgroups that each cover a slice of d_in, leaves
// fp32 partial tiles in memory and needs a second kernel to add them up.  Here nothing is split: the packed
// weights are K-contiguous, so output column n is the dot product of x with one contiguous row of W^T.  A
// wavefront owns two columns, walks their rows 1 KiB at a time (16 bytes per lane, consecutive lanes on
// consecutive addresses, 8 to 16 KiB in flight per wavefront), reads x with the same lane pattern (a few KiB
// that stay in the caches), multiplies with v_dot2_f32_bf16 (two bf16 products and an fp32 add per lane) and
// reduces over the lanes once at the end; the adapter's term is R more reduction elements per column (the gated
// x A, rounded to bf16 once, against the column's row of B^T).  The same kernel without that term computes
// u = x A first (its "columns" are the R rows of A^T: half a megabyte), in a launch of a few workgroups plus
// one that looks up the row's gate entry with scalar loads.  Two launches like the split path, but no partial
// sums and no second pass over them.
#include "linear_common.h"
#include "token_meta.h"

namespace cwl {
namespace {

constexpr int kThreads = 256;

typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

struct GemvArgs {
    const uint16_t* x;      // [K]
    const uint16_t* Wt;     // [N, K]: row n holds output column n, K-contiguous
    int64_t K, N;
    // second launch only (ADAPTER):
    const float* u;         // [n_proj R] x A of every adapter, fp32
    int32_t R;
    int32_t n_proj;         // projections side by side: columns [col0[p], col0[p + 1]) use directions [p R, p R + R)
    int64_t col0[kMaxGroup];
    const uint16_t* Bt;     // [N, R]
    const TokMeta* gate;    // the row's gate entry
    uint16_t* y;            // [N] bf16
    // first launch only: u out, and the gate entry when it comes from a chunk table
    float* out32;           // [N]
    MetaJob job;            // job.n_blocks == 1: one more workgroup fills job.meta[0]
};

// eight bf16 products of two 16-byte vectors added to acc, two per instruction (v_dot2_f32_bf16, fp32 sum)
__device__ __forceinline__ float dot2(uint32_t a, uint32_t b, float acc) {
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, a), __builtin_bit_cast(bf16x2, b), acc, false);
}
__device__ __forceinline__ float dot8(const u32x4& a, const u32x4& b, float acc) {
    // (the words are taken out by name: a bit cast of a[i] under a loop index read word 0 four times)
    acc = dot2(a.x, b.x, acc);
    acc = dot2(a.y, b.y, acc);
    acc = dot2(a.z, b.z, acc);
    return dot2(a.w, b.w, acc);
}

// kColsPerWave: two for the layer itself (a workgroup then writes eight columns with one 16-byte store; x is
// read once for both), one for x A, whose 64 to 256 "columns" are all the parallelism that launch has.
template <bool ADAPTER>
__global__ void __launch_bounds__(kThreads) gemv_row_kernel(GemvArgs a) {
    constexpr int kColsPerWave = ADAPTER ? 2 : 1;
    constexpr int kColsPerBlock = kColsPerWave * (kThreads / 64);
    __shared__ float outs[kColsPerBlock];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_col_blocks = (int)((a.N + kColsPerBlock - 1) / kColsPerBlock);
    if (!ADAPTER && (int)blockIdx.x >= n_col_blocks) {
        // the extra workgroup of the first launch: the row's gate entry from the chunk table.  The row index
        // is the same in every lane, so the look-ups are scalar loads (a chain of about nine, each a fraction
        // of a vector load's latency).
        __shared__ int32_t lad_ranks[CWL_MAX_LADDER];
        __shared__ float lad_scales[CWL_MAX_LADDER];
        ladder_to_lds(a.job.lad, lad_ranks, lad_scales);
        __syncthreads();
        const int64_t t = __builtin_amdgcn_readfirstlane(0);
        const TokMeta m = token_meta_of(t, a.job.seq_offsets, a.job.n_seqs, a.job.chunk_offsets, a.job.chunk_start,
                                        a.job.chunk_len, a.job.rank_idx, a.job.chunk_cap, a.job.lad.K, lad_ranks,
                                        lad_scales, a.job.blend_w);
        if (tid == 0) a.job.meta[0] = m;
        return;
    }
    const int K = (int)a.K;
    const int64_t j0 = (int64_t)blockIdx.x * kColsPerBlock + wave * kColsPerWave;
    const uint16_t* wrow[kColsPerWave];
#pragma unroll
    for (int c = 0; c < kColsPerWave; ++c) {
        int64_t j = j0 + c;
        if (j > a.N - 1) j = a.N - 1;              // a column past the end repeats the last one and is not stored
        wrow[c] = a.Wt + j * a.K;
    }
    // The adapter's operands are asked for first and used last: the row's gate entry, eight directions of
    // x A per lane (on R / 8 lanes), the same eight entries of the two columns' rows of B^T.
    TokMeta mt = {0, 0, 0.0f, 0.0f};
    f32x4 ua = {0.0f, 0.0f, 0.0f, 0.0f}, ub = {0.0f, 0.0f, 0.0f, 0.0f};
    u32x4 bv[kColsPerWave];
    const int i0 = lane * 8;
    const bool lora_lane = ADAPTER && i0 < a.R;
    if (ADAPTER) {
        mt = a.gate[0];
#pragma unroll
        for (int c = 0; c < kColsPerWave; ++c) bv[c] = u32x4{0u, 0u, 0u, 0u};
        if (lora_lane) {
            // the workgroup's eight columns belong to one projection (column counts are multiples of eight)
            int proj = 0;
            for (int q = 1; q < a.n_proj; ++q)
                if (j0 >= a.col0[q]) proj = q;
            const float* up = a.u + (int64_t)proj * a.R + i0;
            ua = *reinterpret_cast<const f32x4*>(up);
            ub = *reinterpret_cast<const f32x4*>(up + 4);
#pragma unroll
            for (int c = 0; c < kColsPerWave; ++c) {
                int64_t j = j0 + c;
                if (j > a.N - 1) j = a.N - 1;
                bv[c] = *reinterpret_cast<const u32x4*>(a.Bt + j * a.R + i0);
            }
        }
    }

    float acc[kColsPerWave];
#pragma unroll
    for (int c = 0; c < kColsPerWave; ++c) acc[c] = 0.0f;

    // Walk the reduction dimension 512 elements at a time, four such steps per trip.  Nothing is staged and
    // nothing waits for a barrier; the loads of the next trip are issued before the products of the current.
    constexpr int UN = 4;
    u32x4 w[2][UN][kColsPerWave], xv[2][UN];
    auto load_trip = [&](int buf, int k0) {
#pragma unroll
        for (int s = 0; s < UN; ++s) {
            const int k = k0 + s * 512 + lane * 8;
            xv[buf][s] = u32x4{0u, 0u, 0u, 0u};
            if (k < K) xv[buf][s] = *reinterpret_cast<const u32x4*>(a.x + k);
#pragma unroll
            for (int c = 0; c < kColsPerWave; ++c) {
                w[buf][s][c] = u32x4{0u, 0u, 0u, 0u};
                if (k < K) w[buf][s][c] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(wrow[c] + k));
            }
        }
    };
    auto use_trip = [&](int buf) {       // (elements past the end were loaded as zeros)
#pragma unroll
        for (int s = 0; s < UN; ++s)
#pragma unroll
            for (int c = 0; c < kColsPerWave; ++c) acc[c] = dot8(w[buf][s][c], xv[buf][s], acc[c]);
    };
    load_trip(0, 0);
    for (int k0 = 0; k0 < K; k0 += 2 * 512 * UN) {       // two trips per iteration: the buffers alternate by name
        load_trip(1, k0 + 512 * UN);
        use_trip(0);
        load_trip(0, k0 + 2 * 512 * UN);
        use_trip(1);
    }
    if (ADAPTER) {
        // uhat = (x A) (.) G rounded to bf16 once, as the tiled paths round it: R more reduction elements
        const float uu[8] = {ua.x, ua.y, ua.z, ua.w, ub.x, ub.y, ub.z, ub.w};
        uint32_t uw[4];
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            float v[2];
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int i = i0 + 2 * h + e;
                const float g = (i < mt.r_prev ? mt.g_prev : 0.0f) + (i < mt.r_cur ? mt.g_cur : 0.0f);
                v[e] = lora_lane ? uu[2 * h + e] * g : 0.0f;
            }
            const __bf16 lo = (__bf16)v[0], hi = (__bf16)v[1];
            uw[h] = (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
        }
#pragma unroll
        for (int c = 0; c < kColsPerWave; ++c) {
            acc[c] = dot2(bv[c].x, uw[0], acc[c]);
            acc[c] = dot2(bv[c].y, uw[1], acc[c]);
            acc[c] = dot2(bv[c].z, uw[2], acc[c]);
            acc[c] = dot2(bv[c].w, uw[3], acc[c]);
        }
    }
    // sum over the lanes, always in the same order
#pragma unroll
    for (int c = 0; c < kColsPerWave; ++c) {
        float v = acc[c];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) outs[wave * kColsPerWave + c] = v;
    }
    __syncthreads();
    // one thread writes the workgroup's eight columns
    if (tid == 0) {
        const int64_t n0 = (int64_t)blockIdx.x * kColsPerBlock;
        if constexpr (ADAPTER) {
            static_assert(kColsPerBlock == 8, "the 16-byte store below");
            uint16_t o[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const __bf16 b = (__bf16)outs[i];
                o[i] = __builtin_bit_cast(uint16_t, b);
            }
            uint16_t* dst = a.y + n0;
            if (n0 + kColsPerBlock <= a.N) {
                u32x4 p;
                p.x = (uint32_t)o[0] | ((uint32_t)o[1] << 16);
                p.y = (uint32_t)o[2] | ((uint32_t)o[3] << 16);
                p.z = (uint32_t)o[4] | ((uint32_t)o[5] << 16);
                p.w = (uint32_t)o[6] | ((uint32_t)o[7] << 16);
                *reinterpret_cast<u32x4*>(dst) = p;
            } else {
                for (int i = 0; i < kColsPerBlock && n0 + i < a.N; ++i) dst[i] = o[i];
            }
        } else {
            for (int i = 0; i < kColsPerBlock && n0 + i < a.N; ++i) a.out32[n0 + i] = outs[i];
        }
    }
}

template <bool ADAPTER>
cwl_status launch_gemv_row(const GemvArgs& a, hipStream_t st) {
    constexpr int kColsPerBlock = (ADAPTER ? 2 : 1) * (kThreads / 64);
    const int64_t blocks = (a.N + kColsPerBlock - 1) / kColsPerBlock + ((!ADAPTER && a.job.n_blocks > 0) ? 1 : 0);
    if (blocks >= (int64_t)1 << 31) return CWL_ERR_UNSUPPORTED;
    gemv_row_kernel<ADAPTER><<<dim3((unsigned)blocks), dim3(kThreads), 0, st>>>(a);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

}  // namespace

// bf16, token order, ONE row.  More rows stay with the split-reduction path (14.2 to 15.8 us for 2 to 16 rows of
// 4096 -> 4096 from a HIP graph): a form of this kernel with x staged in LDS took 15.1 / 18.5 / 26.6 us for 2 / 4 /
// 8 rows (v_dot2_f32_bf16 issues at about a quarter of the vector rate), and the same walk on the matrix cores
// (v_mfma_f32_4x4x4_16b_bf16, block b of a 128-element k-step on elements [8 b, 8 b + 8), so that a column's
// lanes read 256 contiguous bytes) 15.9 / 16.9 / 21.4 / 39.6 us for 2 / 4 / 8 / 16 rows: every further row of x
// costs about half a microsecond of loads there.  A third form took 16 rows per instruction
// (v_mfma_f32_16x16x32_bf16, a workgroup per 16 output columns, its four wavefronts a quarter of d_in each, both
// fragments straight from memory in the instruction's layout with every load issued before the first product):
// 16.1 / 16.7 / 17.9 / 20.3 us for 2 / 4 / 8 / 16 rows (kernels: x A 7.2 to 10.0 us on its four workgroups next
// to the gate look-ups, the layer 8.4 to 10.7 us against 6.4 us for one row here): a fragment load touches 16 rows
// of W^T with 64 bytes each where this kernel's loads are 1 KiB of one row, and every wavefront re-reads x.
// A reduction of more than 8192 elements stays with the split path too: a wavefront walks its rows of W^T
// (and, in the first launch, of A^T) from end to end, 11008 -> 4096 took 24.4 us here against 22.7 us there.
bool gemv_rows_serves(const cwl_linear_desc* d) {
    if (d->dt != CWL_BF16 || d->group_rows != 0 || d->n_rows != 1) return false;
    return d->d_in % 8 == 0 && d->d_out % 8 == 0 && d->d_in <= 8192;
}

// wt / at / bt: W^T [d_out, d_in], A^T [n_proj R, d_in], B^T [d_out, R] of the packed weights (d_out: the columns
// of all projections of the group); u: n_proj R floats of scratch;
// meta: one gate entry of scratch (used when `gate` is NULL: then the chunk table is looked up)
cwl_status run_gemv_rows(const cwl_linear_desc* d, const GroupCols& grp, const void* x, const void* wt, const void* at, const void* bt,
                         const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
                         const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                         int32_t chunk_cap, const TokMeta* gate, void* y, float* u, TokMeta* meta, hipStream_t st) {
    const int32_t R = padded_rank(d->r_max);
    GemvArgs a1 = {};
    a1.x = static_cast<const uint16_t*>(x);
    a1.Wt = static_cast<const uint16_t*>(at);
    a1.K = d->d_in;
    a1.N = (int64_t)grp.n_proj * R;
    a1.R = R;
    a1.out32 = u;
    if (!gate) {
        a1.job.seq_offsets = seq_offsets;
        a1.job.chunk_offsets = chunk_offsets;
        a1.job.chunk_start = chunk_start;
        a1.job.chunk_len = chunk_len;
        a1.job.rank_idx = rank_idx;
        a1.job.n_seqs = n_seqs;
        a1.job.chunk_cap = chunk_cap;
        a1.job.blend_w = d->blend_w;
        a1.job.lad.K = d->K;
        for (int32_t k = 0; k < d->K; ++k) {
            a1.job.lad.ranks[k] = d->ranks[k];
            a1.job.lad.scales[k] = d->scales[k];
        }
        a1.job.meta = meta;
        a1.job.n_blocks = 1;
    }
    prof_begin(CWL_PROF_META, st);
    cwl_status s = launch_gemv_row<false>(a1, st);
    prof_end(CWL_PROF_META, st);
    if (s != CWL_OK) return s;
    GemvArgs a2 = {};
    a2.x = a1.x;
    a2.Wt = static_cast<const uint16_t*>(wt);
    a2.K = d->d_in;
    a2.N = d->d_out;
    a2.u = u;
    a2.R = R;
    a2.n_proj = grp.n_proj;
    for (int32_t q = 0; q < grp.n_proj; ++q) a2.col0[q] = grp.col0[q];
    a2.Bt = static_cast<const uint16_t*>(bt);
    a2.gate = gate ? gate : meta;
    a2.y = static_cast<uint16_t*>(y);
    prof_begin(CWL_PROF_MAIN, st);
    s = launch_gemv_row<true>(a2, st);
    prof_end(CWL_PROF_MAIN, st);
    return s;
}

}  // namespace cwl
