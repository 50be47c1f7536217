// cwl_chunkwise_lora_linear: host side and the small helper kernels (token gate table, rank
// grouping, weight re-layout).  The GEMMs themselves are in gemm_f32.hip / gemm_bf16.hip; the
// formulation is described in linear_common.h.  (Sec. III-C / III-D of arxiv 2601.21109.)
#include "linear_common.h"
#include "token_meta.h"
#include "partition_seq.h"

// Scratch memory of cwl_chunkwise_lora_linear_packed_static: held in every GPU's memory from the
// moment the library is loaded there.  In host code this name is only a handle for
// hipGetSymbolAddress, never a device address; kernels get the looked-up pointer as an argument.
static __device__ __align__(256) unsigned char scratch[CWL_STATIC_SCRATCH_BYTES];

namespace cwl {
namespace {

constexpr int kSortThreads = 512;
constexpr int kBuckets = CWL_MAX_LADDER + 1;

__device__ __forceinline__ int bucket_of(int32_t r_eff, const Ladder& lad) {
    // larger rank -> smaller bucket id; rank 0 -> last bucket.  The loop runs over the fixed
    // capacity with constant indices so that the ladder stays in scalar registers.
    int n_ge = 0;
#pragma unroll
    for (int k = 0; k < CWL_MAX_LADDER; ++k)
        n_ge += (k < lad.K && lad.ranks[k] > 0 && lad.ranks[k] >= r_eff) ? 1 : 0;
    return r_eff > 0 ? (n_ge > 0 ? n_ge - 1 : 0) : kBuckets - 1;
}


// ------------------------------------------------------------------------------------------
// Per-token gate table (token_meta.h has the lookup).
// A block of 256 threads covers 4 rank blocks of 64 rows; in token order (no grouping) each
// wavefront also reduces the largest effective rank of its 64 rows into blk_r.  The table has four
// entries for every started group of 256 rows (0 for blocks past the last row), so that a 256-row
// tile reads its four with one aligned 16-byte load.
// ------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
token_meta_kernel(int64_t n_rows, const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                  const int32_t* __restrict__ chunk_offsets, const int32_t* __restrict__ chunk_start,
                  const int32_t* __restrict__ chunk_len, const int32_t* __restrict__ rank_idx,
                  int32_t chunk_cap, Ladder lad, int32_t blend_w, TokMeta* __restrict__ meta,
                  int32_t* __restrict__ blk_r /* may be NULL */, int32_t* __restrict__ r_eff_out /* may be NULL */) {
    // the ladder is indexed by a per-thread rung: keep a copy in LDS
    __shared__ int32_t lad_ranks[CWL_MAX_LADDER];
    __shared__ float lad_scales[CWL_MAX_LADDER];
    ladder_to_lds(lad, lad_ranks, lad_scales);
    __syncthreads();
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    TokMeta m = {0, 0, 0.0f, 0.0f};
    if (t < n_rows)
        m = token_meta_of(t, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                          chunk_cap, lad.K, lad_ranks, lad_scales, blend_w);
    int32_t r_eff = m.r_cur > m.r_prev ? m.r_cur : m.r_prev;
    if (t < n_rows) {
        meta[t] = m;
        if (r_eff_out) r_eff_out[t] = r_eff | (bucket_of(r_eff, lad) << 16);   // rank and its sort bucket
    }
    if (blk_r) {
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int32_t o = __shfl_xor(r_eff, off);
            r_eff = o > r_eff ? o : r_eff;
        }
        const int64_t blk = t / kRankBlock;
        if ((threadIdx.x & 63) == 0) blk_r[blk] = r_eff;        // all four entries of the 256 rows, 0 past the end
    }
}

// ------------------------------------------------------------------------------------------
// Rank grouping: a stable counting sort of the token rows by effective rank, largest first, so
// that row tiles are rank-homogeneous (only the few tiles that straddle two buckets mix ranks)
// and the tiles with the longest reduction are scheduled first.  One workgroup of 512 threads;
// bucket ids are staged in LDS a segment at a time, each thread owns a contiguous slice of it.
// ------------------------------------------------------------------------------------------
constexpr int kSortSeg = 32768;     // tokens staged in LDS at a time (one byte each)

// sum over the block of kBuckets counters per thread; result in tot[] (LDS), valid after the call
__device__ void block_bucket_sums(const int32_t (&cnt)[kBuckets], int32_t (*wave_tot)[kSortThreads / 64],
                                  int32_t* tot) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) {
        int32_t v = cnt[b];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) wave_tot[b][wave] = v;
    }
    __syncthreads();
    if (tid < kBuckets) {
        int32_t run = 0;
        for (int w = 0; w < kSortThreads / 64; ++w) run += wave_tot[tid][w];
        tot[tid] = run;
    }
    __syncthreads();
}

// stage the bucket ids of one segment in LDS: 8 independent loads in flight per thread
__device__ __forceinline__ void stage_buckets(const int32_t* __restrict__ packed, int seg_len, uint8_t* bk) {
    for (int base = threadIdx.x; base < seg_len; base += 8 * kSortThreads) {
        int32_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * kSortThreads;
            v[u] = i < seg_len ? packed[i] : 0;
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = base + u * kSortThreads;
            if (i < seg_len) bk[i] = (uint8_t)(v[u] >> 16);
        }
    }
}

// counts of one thread's contiguous slice [i0, i1) of the staged segment, run by run (tokens of one
// chunk share a bucket); the bucket index is only known at run time, so every update is a compare
// against all bucket ids and the counters stay in registers
__device__ __forceinline__ void count_slice(const uint8_t* bk, int i0, int i1, int32_t (&cnt)[kBuckets]) {
    for (int i = i0; i < i1;) {
        const int bkt = bk[i];
        int j = i + 1;
        while (j < i1 && bk[j] == bkt) ++j;
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) cnt[b] += (b == bkt) ? (j - i) : 0;
        i = j;
    }
}

__global__ void __launch_bounds__(kSortThreads)
group_rows_kernel(int64_t n_rows, const int32_t* __restrict__ r_eff /* rank | bucket << 16 */,
                  int32_t* __restrict__ perm) {
    constexpr int kWaves = kSortThreads / 64;
    __shared__ uint8_t bk[kSortSeg];                 // bucket id of every token of the segment
    __shared__ int32_t wave_tot[kBuckets][kWaves];
    __shared__ int32_t tot[kBuckets];
    __shared__ int32_t run_base[kBuckets];           // next free slot of every bucket
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const bool one_segment = n_rows <= kSortSeg;

    // pass 1: bucket totals -> first slot of every bucket
    int32_t cnt[kBuckets];
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) cnt[b] = 0;
    for (int64_t seg0 = 0; seg0 < n_rows; seg0 += kSortSeg) {
        const int seg_len = (int)((n_rows - seg0 < kSortSeg) ? n_rows - seg0 : kSortSeg);
        stage_buckets(r_eff + seg0, seg_len, bk);
        __syncthreads();
        const int per = (seg_len + kSortThreads - 1) / kSortThreads;
        const int i0 = tid * per < seg_len ? tid * per : seg_len;
        const int i1 = i0 + per < seg_len ? i0 + per : seg_len;
        count_slice(bk, i0, i1, cnt);
        if (!one_segment) __syncthreads();
    }
    block_bucket_sums(cnt, wave_tot, tot);
    if (tid == 0) {
        int32_t run = 0;
        for (int b = 0; b < kBuckets; ++b) {
            run_base[b] = run;
            run += tot[b];
        }
    }
    __syncthreads();

    // pass 2: segment by segment; inside a segment every thread owns a contiguous slice, so the
    // order (segment, thread, position in slice) is token order and the sort is stable
    for (int64_t seg0 = 0; seg0 < n_rows; seg0 += kSortSeg) {
        const int seg_len = (int)((n_rows - seg0 < kSortSeg) ? n_rows - seg0 : kSortSeg);
        if (!one_segment) {
            stage_buckets(r_eff + seg0, seg_len, bk);
            __syncthreads();
        }
        const int per = (seg_len + kSortThreads - 1) / kSortThreads;
        const int i0 = tid * per < seg_len ? tid * per : seg_len;
        const int i1 = i0 + per < seg_len ? i0 + per : seg_len;
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) cnt[b] = 0;
        count_slice(bk, i0, i1, cnt);
        // exclusive scan over threads, bucket by bucket: shuffles inside a wave, LDS across waves
        int32_t excl[kBuckets];
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) {
            int32_t v = cnt[b];
#pragma unroll
            for (int off = 1; off < 64; off <<= 1) {
                const int32_t o = __shfl_up(v, off);
                if (lane >= off) v += o;
            }
            excl[b] = v - cnt[b];
            if (lane == 63) wave_tot[b][wave] = v;
        }
        __syncthreads();
        if (tid < kBuckets) {
            int32_t run = 0;
            for (int w = 0; w < kWaves; ++w) {
                const int32_t c = wave_tot[tid][w];
                wave_tot[tid][w] = run;
                run += c;
            }
            tot[tid] = run;
        }
        __syncthreads();
        int32_t pos[kBuckets];
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) pos[b] = run_base[b] + wave_tot[b][wave] + excl[b];
        for (int i = i0; i < i1;) {
            const int bkt = bk[i];
            int j = i + 1;
            while (j < i1 && bk[j] == bkt) ++j;
            int32_t p = 0;
#pragma unroll
            for (int b = 0; b < kBuckets; ++b)
                if (b == bkt) { p = pos[b]; pos[b] = p + (j - i); }
            for (int k = i; k < j; ++k) perm[p + (k - i)] = (int32_t)(seg0 + k);
            i = j;
        }
        __syncthreads();
        if (tid < kBuckets) run_base[tid] += tot[tid];
        __syncthreads();
    }
}

// The same sort spread over the chip, for up to kParSortBlocks * kParSortRows rows: workgroup g owns
// rows [2048 g, 2048 g + 2048), thread i of it eight consecutive rows.  First launch: bucket counts
// per workgroup.  Second launch: every workgroup adds up, from all the counts, where its rows of
// every bucket begin (buckets before it in all workgroups, its own bucket in the workgroups before
// it), ranks its own rows by an exclusive scan over its threads, bucket by bucket, and writes them.
// Order inside a bucket is row order, as in the one-workgroup kernel.
constexpr int kParSortRows = 2048;
constexpr int kParSortBlocks = 1024;

__global__ void __launch_bounds__(256)
sort_count_kernel(int64_t n_rows, const int32_t* __restrict__ r_eff, int32_t* __restrict__ counts /* [blocks][kBuckets] */) {
    __shared__ int32_t wave_tot[kBuckets][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * kParSortRows + tid * 8;
    int32_t cnt[kBuckets];
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) cnt[b] = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int32_t bkt = (i0 + u < n_rows) ? (r_eff[i0 + u] >> 16) : -1;
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) cnt[b] += (b == bkt) ? 1 : 0;
    }
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) {
        int32_t v = cnt[b];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) wave_tot[b][wave] = v;
    }
    __syncthreads();
    if (tid < kBuckets)
        counts[(int64_t)blockIdx.x * kBuckets + tid] = wave_tot[tid][0] + wave_tot[tid][1] + wave_tot[tid][2] + wave_tot[tid][3];
}

__global__ void __launch_bounds__(256)
sort_scatter_kernel(int64_t n_rows, const int32_t* __restrict__ r_eff, const int32_t* __restrict__ counts,
                    int32_t n_blocks, int32_t* __restrict__ perm) {
    __shared__ int32_t wave_tot[kBuckets][4];
    __shared__ int32_t base_sh[kBuckets];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int32_t me = (int32_t)blockIdx.x;
    // first slot of every bucket's rows of this workgroup
    int32_t before[kBuckets];
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) before[b] = 0;
    const int32_t n_entries = n_blocks * kBuckets;
    for (int32_t e = tid; e < n_entries; e += 256) {
        const int32_t blk = e / kBuckets, bb = e - blk * kBuckets;
        const int32_t c = counts[e];
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) before[b] += (bb < b || (bb == b && blk < me)) ? c : 0;
    }
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) {
        int32_t v = before[b];
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
        if (lane == 0) wave_tot[b][wave] = v;
    }
    __syncthreads();
    if (tid < kBuckets) base_sh[tid] = wave_tot[tid][0] + wave_tot[tid][1] + wave_tot[tid][2] + wave_tot[tid][3];
    __syncthreads();
    // this thread's rows, their buckets, and its counts
    const int64_t i0 = (int64_t)me * kParSortRows + tid * 8;
    int32_t bkt[8];
    int32_t cnt[kBuckets];
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) cnt[b] = 0;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        bkt[u] = (i0 + u < n_rows) ? (r_eff[i0 + u] >> 16) : -1;
#pragma unroll
        for (int b = 0; b < kBuckets; ++b) cnt[b] += (b == bkt[u]) ? 1 : 0;
    }
    // exclusive scan over the threads, bucket by bucket
    int32_t pos[kBuckets];
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) {
        int32_t v = cnt[b];
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int32_t o = __shfl_up(v, off);
            if (lane >= off) v += o;
        }
        pos[b] = v - cnt[b];
        if (lane == 63) wave_tot[b][wave] = v;     // (read above before the last barrier)
    }
    __syncthreads();
#pragma unroll
    for (int b = 0; b < kBuckets; ++b) {
        int32_t run = base_sh[b];
        for (int w = 0; w < wave; ++w) run += wave_tot[b][w];
        pos[b] += run;
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        if (bkt[u] < 0) continue;
        int32_t p = 0;
#pragma unroll
        for (int b = 0; b < kBuckets; ++b)
            if (b == bkt[u]) { p = pos[b]; pos[b] = p + 1; }
        perm[p] = (int32_t)(i0 + u);
    }
}

__global__ void __launch_bounds__(256)
block_rank_kernel(int64_t n_rows, const int32_t* __restrict__ r_eff, const int32_t* __restrict__ perm,
                  int32_t* __restrict__ blk_r) {
    const int64_t g = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int32_t r = 0;
    if (g < n_rows) r = r_eff[perm[g]] & 0xffff;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const int32_t o = __shfl_xor(r, off);
        r = o > r ? o : r;
    }
    const int64_t blk = g / kRankBlock;
    if ((threadIdx.x & 63) == 0) blk_r[blk] = r;
}

// largest effective rank per block of 64 rows, from gate entries the caller supplies (ranks
// clipped to [0, r_max]: the table bounds how far the reduction loops walk)
__global__ void __launch_bounds__(256)
block_rank_from_gate_kernel(int64_t n_rows, const TokMeta* __restrict__ gate, int32_t r_max,
                            int32_t* __restrict__ blk_r) {
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
    int32_t r = 0;
    if (t < n_rows) {
        const TokMeta m = gate[t];
        r = m.r_cur > m.r_prev ? m.r_cur : m.r_prev;
        r = r < 0 ? 0 : (r > r_max ? r_max : r);
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        const int32_t o = __shfl_xor(r, off);
        r = o > r ? o : r;
    }
    const int64_t blk = t / kRankBlock;
    if ((threadIdx.x & 63) == 0) blk_r[blk] = r;
}

// ------------------------------------------------------------------------------------------
// Split shrink.  With fewer than ~16k rows the shrink's grid of 64-row tiles leaves most compute
// units idle while each workgroup walks the whole reduction dimension (21 us at d_in = 4096
// whatever the row count).  Then x A is computed as fp32 partial products over slices of the
// reduction dimension (the EPI_PARTIAL launch, which also fills the gate table), and this kernel
// sums the slices in slice order, applies the gate and rounds to bf16: uhat, as the one-pass
// shrink writes it.  A thread owns 4 consecutive directions of one row; straight-line code with
// SP (compile-time bound on the slices) loads in flight.
// ------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) float f32x4_t;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4_t;

template <int SP>
__global__ void __launch_bounds__(256)
shrink_fixup_kernel(int64_t n_rows, int32_t R, const float* __restrict__ partial, int32_t splits,
                    int64_t pstride, const TokMeta* __restrict__ meta, const int32_t* __restrict__ perm,
                    __bf16* __restrict__ uhat) {
    const int64_t idx = (int64_t)blockIdx.x * 256 + threadIdx.x;      // over n_rows * R / 4
    const int per_row = R / 4;
    int64_t g = idx / per_row;
    const int i0 = (int)(idx % per_row) * 4;
    const bool live = g < n_rows;
    if (!live) g = n_rows - 1;
    const float* p = partial + g * R + i0;
    f32x4_t v[SP];
#pragma unroll
    for (int s = 0; s < SP; ++s) v[s] = *reinterpret_cast<const f32x4_t*>(p + (s < splits ? s : 0) * pstride);
    const TokMeta mt = meta[perm ? (int64_t)perm[g] : g];     // partial and uhat: grouped row; meta: token
    f32x4_t u = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
    for (int s = 0; s < SP; ++s)
        if (s < splits) u += v[s];
    bf16x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const int i = i0 + e;
        const float gate = (i < mt.r_prev ? mt.g_prev : 0.0f) + (i < mt.r_cur ? mt.g_cur : 0.0f);
        o[e] = (__bf16)(u[e] * gate);
    }
    if (live) *reinterpret_cast<bf16x4_t*>(uhat + g * R + i0) = o;
}

template <int SP>
cwl_status launch_shrink_fixup(int64_t n_rows, int32_t R, const float* partial, int32_t splits,
                               int64_t pstride, const TokMeta* meta, const int32_t* perm, void* uhat,
                               hipStream_t st) {
    const int64_t n_thr = n_rows * (R / 4);
    shrink_fixup_kernel<SP><<<dim3((unsigned)((n_thr + 255) / 256)), dim3(256), 0, st>>>(
        n_rows, R, partial, splits, pstride, meta, perm, static_cast<__bf16*>(uhat));
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

// ------------------------------------------------------------------------------------------
// Second phase of the two-phase call: the gate of Sec. III-C / III-D applied to a product x A that
// an earlier launch left in fp32 (one slice, or the slices of a split reduction, added here in slice
// order).  A workgroup owns one rank block of 64 rows: wavefront 0 looks up the rows' gate entries
// (one row per lane, a chain of dependent loads) and their largest effective rank, meanwhile all
// four wavefronts have their first 64 directions of the product in flight; then every thread gates
// four consecutive directions of a row at a time and writes uhat in the layer's element type, rounded
// once as the one-pass shrink rounds it.  The grid covers whole groups of 256 rows, so blk_r gets its
// four entries per started group (0 past the last row).
// ------------------------------------------------------------------------------------------
__device__ __forceinline__ void store_gated4(__bf16* dst, const f32x4_t& v) {
    bf16x4_t o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = (__bf16)v[e];
    *reinterpret_cast<bf16x4_t*>(dst) = o;
}
__device__ __forceinline__ void store_gated4(float* dst, const f32x4_t& v) { *reinterpret_cast<f32x4_t*>(dst) = v; }

template <int SP, typename OutT>
__global__ void __launch_bounds__(256)
gate_product_kernel(int64_t n_rows, int32_t R, const float* __restrict__ u, int32_t splits, int64_t pstride,
                    const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                    const int32_t* __restrict__ chunk_offsets, const int32_t* __restrict__ chunk_start,
                    const int32_t* __restrict__ chunk_len, const int32_t* __restrict__ rank_idx,
                    int32_t chunk_cap, Ladder lad, int32_t blend_w, OutT* __restrict__ uhat,
                    int32_t* __restrict__ blk_r) {
    __shared__ int32_t lad_ranks[CWL_MAX_LADDER];
    __shared__ float lad_scales[CWL_MAX_LADDER];
    __shared__ TokMeta sm[kRankBlock];
    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * kRankBlock;
    // pass p covers directions [64 p, 64 p + 64) of the 64 rows: 1024 groups of four, four per thread
    auto load_pass = [&](int pass, f32x4_t (&v)[4][SP]) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int f = j * 256 + tid;
            int64_t g = row0 + f / 16;
            if (g > n_rows - 1) g = n_rows - 1;
            const float* p = u + g * R + pass * 64 + (f % 16) * 4;
#pragma unroll
            for (int sl = 0; sl < SP; ++sl)
                v[j][sl] = *reinterpret_cast<const f32x4_t*>(p + (sl < splits ? sl : 0) * pstride);
        }
    };
    f32x4_t v[4][SP];
    if (row0 < n_rows) load_pass(0, v);
    ladder_to_lds(lad, lad_ranks, lad_scales);
    __syncthreads();
    if (tid < kRankBlock) {
        const int64_t t = row0 + tid;
        TokMeta m = {0, 0, 0.0f, 0.0f};
        if (t < n_rows)
            m = token_meta_of(t, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap,
                              lad.K, lad_ranks, lad_scales, blend_w);
        sm[tid] = m;
        int32_t r_eff = m.r_cur > m.r_prev ? m.r_cur : m.r_prev;
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
            const int32_t o = __shfl_xor(r_eff, off);
            r_eff = o > r_eff ? o : r_eff;
        }
        if (tid == 0) blk_r[blockIdx.x] = r_eff;
    }
    __syncthreads();
    if (row0 >= n_rows) return;
    const int passes = R / 64;
    for (int pass = 0; pass < passes; ++pass) {
        if (pass > 0) load_pass(pass, v);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int f = j * 256 + tid;
            const int64_t g = row0 + f / 16;
            const int i0 = pass * 64 + (f % 16) * 4;
            const TokMeta mt = sm[f / 16];
            f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int sl = 0; sl < SP; ++sl)
                if (sl < splits) acc += v[j][sl];
            f32x4_t o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int i = i0 + e;
                const float gate = (i < mt.r_prev ? mt.g_prev : 0.0f) + (i < mt.r_cur ? mt.g_cur : 0.0f);
                o[e] = acc[e] * gate;
            }
            if (g < n_rows) store_gated4(uhat + g * R + i0, o);
        }
    }
}

template <int SP, typename OutT>
cwl_status launch_gate_product(const cwl_linear_desc* d, int32_t R, const float* u, int32_t splits, int64_t pstride,
                               const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
                               const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                               int32_t chunk_cap, const Ladder& lad, void* uhat, int32_t* blk_r, hipStream_t st) {
    const unsigned blocks = (unsigned)((d->n_rows + 255) / 256 * 4);
    gate_product_kernel<SP, OutT><<<dim3(blocks), dim3(256), 0, st>>>(
        d->n_rows, R, u, splits, pstride, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
        chunk_cap, lad, d->blend_w, static_cast<OutT*>(uhat), blk_r);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

// slices of the reduction dimension for the split shrink; splits < 2: keep the one-pass shrink
// (rows gathered through a permutation are read through it; the gate table is then made first)
SmallPlan shrink_split_plan(const cwl_linear_desc* d) {
    SmallPlan p = {};
    p.splits = 1;
    if (d->dt != CWL_BF16 || d->n_rows >= 16384) return p;
    const int64_t R = padded_rank(d->r_max);
    const int64_t tiles = (d->n_rows + 127) / 128 * (R / 64);
    const int64_t stages = d->d_in / 64;
    int64_t s = 512 / tiles;
    if (s > stages / 4) s = stages / 4;
    if (s > 32) s = 32;
    if (s < 2) return p;
    p.n_tile = 64;
    p.ks_per_split = (int32_t)((stages + s - 1) / s);
    p.splits = (int32_t)((stages + p.ks_per_split - 1) / p.ks_per_split);
    p.ldp = R;
    p.partial_stride = d->n_rows * R;
    p.partial_bytes = sizeof(float) * (size_t)p.splits * (size_t)p.partial_stride;
    return p;
}

// ------------------------------------------------------------------------------------------
// Weight re-layout: dst[c, r] = src[r, c] (zero where the source has no element), so that every
// GEMM operand is contiguous along the reduction dimension.
// ------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256)
transpose_pad_kernel(const T* __restrict__ src, int64_t src_rows, int64_t src_cols, int64_t lds_,
                     T* __restrict__ dst, int64_t dst_rows, int64_t dst_cols, int64_t ldd) {
    __shared__ T tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;       // 32 x 8
    const int64_t c0 = (int64_t)blockIdx.x * 32;                  // source column / dst row
    const int64_t r0 = (int64_t)blockIdx.y * 32;                  // source row / dst column
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t r = r0 + ty + i * 8, c = c0 + tx;
        tile[ty + i * 8][tx] = (r < src_rows && c < src_cols) ? src[r * lds_ + c] : T(0);
    }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t dr = c0 + ty + i * 8, dc = r0 + tx;
        if (dr < dst_rows && dc < dst_cols) dst[dr * ldd + dc] = tile[tx][ty + i * 8];
    }
}

template <typename T>
cwl_status transpose_pad(const void* src, int64_t src_rows, int64_t src_cols, int64_t ld_src,
                         void* dst, int64_t dst_rows, int64_t dst_cols, hipStream_t st) {
    if (dst_rows <= 0 || dst_cols <= 0) return CWL_OK;
    const dim3 grid((unsigned)((dst_rows + 31) / 32), (unsigned)((dst_cols + 31) / 32));
    if (grid.y > 65535u) return CWL_ERR_UNSUPPORTED;
    transpose_pad_kernel<T><<<grid, dim3(256), 0, st>>>(static_cast<const T*>(src), src_rows, src_cols,
                                                       ld_src, static_cast<T*>(dst), dst_rows,
                                                       dst_cols, dst_cols);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

// ---- layouts -------------------------------------------------------------------------------
struct PackedLayout {       // byte offsets into the packed weight blob
    size_t wt, at, bt, total;
    int32_t R;
};

// n_proj projections side by side (d->d_out: all their columns): W^T [d_out, d_in], the adapters'
// A^T one after the other [n_proj R, d_in], B^T [d_out, R] (row n: the column of its own adapter)
PackedLayout packed_layout(const cwl_linear_desc* d, int32_t n_proj = 1) {
    PackedLayout L;
    const size_t es = d->dt == CWL_F32 ? 4 : 2;
    L.R = padded_rank(d->r_max);
    size_t off = 0;
    L.wt = off; off = align_up(off + es * (size_t)d->d_out * (size_t)d->d_in, 256);
    L.at = off; off = align_up(off + es * (size_t)n_proj * (size_t)L.R * (size_t)d->d_in, 256);
    L.bt = off; off = align_up(off + es * (size_t)d->d_out * (size_t)L.R, 256);
    L.total = off;
    return L;
}

struct WsLayout {           // byte offsets into the linear workspace
    size_t meta, blk_r, r_eff, perm, uhat, partial, total;
};

// the few-row path: bf16, token order, and the packed W^T and A^T back to back
bool small_rows_path(const cwl_linear_desc* d, const PackedLayout& P) {
    return d->dt == CWL_BF16 && d->group_rows == 0 && d->n_rows >= 1 && d->n_rows <= kSmallRows &&
           P.at == P.wt + sizeof(uint16_t) * (size_t)d->d_out * (size_t)d->d_in;
}

WsLayout ws_layout(const cwl_linear_desc* d, int32_t n_proj = 1) {
    WsLayout L;
    const size_t es = d->dt == CWL_F32 ? 4 : 2;
    const size_t n = (size_t)d->n_rows;
    const size_t R = (size_t)n_proj * (size_t)padded_rank(d->r_max);
    size_t off = 0;
    L.meta = off; off = align_up(off + sizeof(TokMeta) * (n + 1), 256);
    L.blk_r = off; off = align_up(off + sizeof(int32_t) * 4 * (n / 256 + 1), 256);   // four entries per 256 rows, padded
    L.r_eff = off; off = align_up(off + sizeof(int32_t) * (n + 1), 256);
    L.perm = off; off = align_up(off + sizeof(int32_t) * (n + 1), 256);
    L.uhat = off; off = align_up(off + es * (n + 1) * R, 256);
    L.partial = off;
    if (small_rows_path(d, packed_layout(d, n_proj))) {
        // (the one-row path keeps x A there, fp32, every adapter's padded directions: at most 8 KiB)
        const size_t pb = small_rows_plan(d, n_proj).partial_bytes;
        const size_t ub = sizeof(float) * (size_t)n_proj * (size_t)padded_rank(d->r_max);
        off = align_up(off + (pb > ub ? pb : ub), 256);
    }
    else if (n_proj == 1 && shrink_split_plan(d).splits >= 2) off = align_up(off + shrink_split_plan(d).partial_bytes, 256);
    L.total = off;
    return L;
}

cwl_status check_desc(const cwl_linear_desc* d) {
    if (!d) return CWL_ERR_NULL;
    if (d->dt != CWL_F32 && d->dt != CWL_BF16) return CWL_ERR_INVALID_ARG;
    if (d->n_rows < 0 || d->n_rows >= (int64_t)1 << 31) return CWL_ERR_INVALID_ARG;
    if (d->d_in < 1 || d->d_out < 1 || d->d_in >= (int64_t)1 << 31 || d->d_out >= (int64_t)1 << 31)
        return CWL_ERR_INVALID_ARG;
    if (d->r_max < 0 || d->r_max > CWL_MAX_RANK) return CWL_ERR_INVALID_ARG;
    if (d->K < 1 || d->K > CWL_MAX_LADDER) return CWL_ERR_INVALID_ARG;
    if (!d->ranks || !d->scales) return CWL_ERR_NULL;
    for (int32_t k = 0; k < d->K; ++k) {
        if (d->ranks[k] < 0 || d->ranks[k] > d->r_max) return CWL_ERR_INVALID_ARG;
        if (k > 0 && d->ranks[k] < d->ranks[k - 1]) return CWL_ERR_INVALID_ARG;
        if (d->scales[k] != d->scales[k]) return CWL_ERR_INVALID_ARG;
    }
    if (d->blend_w < 0) return CWL_ERR_INVALID_ARG;
    if (d->group_rows != 0 && d->group_rows != 1) return CWL_ERR_INVALID_ARG;
    if (d->ldx < d->d_in || d->ldy < d->d_out) return CWL_ERR_INVALID_ARG;
    if (d->dt == CWL_BF16) {
        if (d->d_in % 64 != 0 || d->d_out % 8 != 0 || d->ldx % 8 != 0 || d->ldy % 8 != 0)
            return CWL_ERR_UNSUPPORTED;
    }
    return CWL_OK;
}

cwl_status check_raw_weights(const cwl_linear_desc* d) {
    if (d->ldw < d->d_out || d->ldb < d->d_out) return CWL_ERR_INVALID_ARG;
    if (d->lda < (d->r_max > 0 ? d->r_max : 1)) return CWL_ERR_INVALID_ARG;
    return CWL_OK;
}

template <typename T>
cwl_status prepack_typed(const cwl_linear_desc* d, const PackedLayout& L, const void* W,
                         const void* A, const void* B, char* packed, hipStream_t st) {
    cwl_status s = transpose_pad<T>(W, d->d_in, d->d_out, d->ldw, packed + L.wt, d->d_out, d->d_in, st);
    if (s != CWL_OK) return s;
    s = transpose_pad<T>(A, d->d_in, d->r_max, d->lda, packed + L.at, L.R, d->d_in, st);
    if (s != CWL_OK) return s;
    return transpose_pad<T>(B, d->r_max, d->d_out, d->ldb, packed + L.bt, d->d_out, L.R, st);
}

// the weights of a group, projection by projection, into the rows of the shared W^T, A^T and B^T
template <typename T>
cwl_status prepack_group_typed(const cwl_linear_desc* d, const cwl_group* g, const PackedLayout& L,
                               char* packed, hipStream_t st) {
    int64_t col0 = 0;
    for (int32_t p = 0; p < g->n_proj; ++p) {
        const int64_t n = g->d_out[p];
        char* wt = packed + L.wt + sizeof(T) * (size_t)col0 * (size_t)d->d_in;
        char* at = packed + L.at + sizeof(T) * (size_t)p * (size_t)L.R * (size_t)d->d_in;
        char* bt = packed + L.bt + sizeof(T) * (size_t)col0 * (size_t)L.R;
        cwl_status s = transpose_pad<T>(g->W[p], d->d_in, n, n, wt, n, d->d_in, st);
        if (s != CWL_OK) return s;
        s = transpose_pad<T>(g->A[p], d->d_in, d->r_max, d->r_max > 0 ? d->r_max : 1, at, L.R, d->d_in, st);
        if (s != CWL_OK) return s;
        s = transpose_pad<T>(g->B[p], d->r_max, n, n, bt, n, L.R, st);
        if (s != CWL_OK) return s;
        col0 += n;
    }
    return CWL_OK;
}

// a group's shape: 1 .. CWL_MAX_GROUP projections whose columns add up to d->d_out; token order only
cwl_status check_group(const cwl_linear_desc* d, const cwl_group* g) {
    if (!g) return CWL_ERR_NULL;
    if (g->n_proj < 1 || g->n_proj > CWL_MAX_GROUP) return CWL_ERR_INVALID_ARG;
    int64_t sum = 0;
    for (int32_t p = 0; p < g->n_proj; ++p) {
        if (g->d_out[p] < 1 || g->d_out[p] > d->d_out) return CWL_ERR_INVALID_ARG;
        if (d->dt == CWL_BF16 && g->d_out[p] % 8 != 0) return CWL_ERR_UNSUPPORTED;
        sum += g->d_out[p];
    }
    if (sum != d->d_out) return CWL_ERR_INVALID_ARG;
    if (d->group_rows != 0) return CWL_ERR_UNSUPPORTED;
    return CWL_OK;
}

// Columns of the projections of a group, one after the other; a single projection is a group of one.
GroupCols group_cols(const cwl_linear_desc* d, const cwl_group* g) {
    GroupCols c = {};
    if (!g) {
        c.n_proj = 1;
        c.cols[0] = d->d_out;
        return c;
    }
    c.n_proj = g->n_proj;
    int64_t off = 0;
    for (int32_t p = 0; p < g->n_proj; ++p) {
        c.col0[p] = off;
        c.cols[p] = g->d_out[p];
        off += g->d_out[p];
    }
    return c;
}

// `gate`: per-row gate entries supplied by the caller (then the chunk table is not looked at), or
// NULL: the entries are derived from the chunk table.  `grp`: the projections that share x (their
// weights packed side by side); every projection has its own directions of uhat and its own B.
cwl_status run_packed(const cwl_linear_desc* d, const GroupCols& grp, const void* x, const char* packed,
                      const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
                      const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                      int32_t chunk_cap, const TokMeta* gate, void* y, char* ws, hipStream_t st) {
    const int32_t n_proj = grp.n_proj;
    const PackedLayout P = packed_layout(d, n_proj);
    const WsLayout L = ws_layout(d, n_proj);
    if (small_rows_path(d, P) && gemv_rows_serves(d))
        return run_gemv_rows(d, grp, x, packed + P.wt, packed + P.at, packed + P.bt, seq_offsets, n_seqs, chunk_offsets,
                             chunk_start, chunk_len, rank_idx, chunk_cap, gate, y,
                             reinterpret_cast<float*>(ws + L.partial), reinterpret_cast<TokMeta*>(ws + L.meta), st);
    if (small_rows_path(d, P))
        return run_small_rows(d, grp, x, packed + P.wt, packed + P.bt, seq_offsets, n_seqs, chunk_offsets,
                              chunk_start, chunk_len, rank_idx, chunk_cap, y,
                              reinterpret_cast<float*>(ws + L.partial),
                              reinterpret_cast<TokMeta*>(ws + L.meta), gate, st);
    const TokMeta* meta = gate ? gate : reinterpret_cast<TokMeta*>(ws + L.meta);
    int32_t* blk_r = reinterpret_cast<int32_t*>(ws + L.blk_r);
    int32_t* r_eff = reinterpret_cast<int32_t*>(ws + L.r_eff);
    int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
    char* uhat = ws + L.uhat;
    const size_t es = d->dt == CWL_F32 ? 4 : 2;
    const int64_t R_all = (int64_t)n_proj * P.R;        // directions of all adapters: leading dimension of uhat

    Ladder lad = {};
    lad.K = d->K;
    for (int32_t k = 0; k < d->K; ++k) {
        lad.ranks[k] = d->ranks[k];
        lad.scales[k] = d->scales[k];
    }
    const bool grouped = d->group_rows == 1;
    const unsigned meta_blocks = (unsigned)((d->n_rows + 255) / 256);
    // splits >= 2: split shrink (bf16, one projection)
    SmallPlan split = {};
    split.splits = 1;
    if (n_proj == 1) split = shrink_split_plan(d);
    // with the split shrink in token order the gate table comes with the partial products
    const bool table_with_products = !gate && split.splits >= 2 && !grouped;
    prof_begin(CWL_PROF_META, st);
    if (gate)
        block_rank_from_gate_kernel<<<dim3(meta_blocks), dim3(256), 0, st>>>(d->n_rows, gate, d->r_max, blk_r);
    else if (!table_with_products)
        token_meta_kernel<<<dim3(meta_blocks), dim3(256), 0, st>>>(
            d->n_rows, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap,
            lad, d->blend_w, reinterpret_cast<TokMeta*>(ws + L.meta), grouped ? nullptr : blk_r,
            grouped ? r_eff : nullptr);
    CWL_RETURN_IF_LAUNCH_FAILED();
    if (grouped) {
        const int64_t sort_blocks = (d->n_rows + kParSortRows - 1) / kParSortRows;
        if (sort_blocks > 1 && sort_blocks <= kParSortBlocks) {
            // (the counts live in uhat, which the shrink only writes later: 68 bytes per 2048 rows)
            int32_t* counts = reinterpret_cast<int32_t*>(uhat);
            sort_count_kernel<<<dim3((unsigned)sort_blocks), dim3(256), 0, st>>>(d->n_rows, r_eff, counts);
            CWL_RETURN_IF_LAUNCH_FAILED();
            sort_scatter_kernel<<<dim3((unsigned)sort_blocks), dim3(256), 0, st>>>(d->n_rows, r_eff, counts,
                                                                                  (int32_t)sort_blocks, perm);
        } else {
            group_rows_kernel<<<dim3(1), dim3(kSortThreads), 0, st>>>(d->n_rows, r_eff, perm);
        }
        CWL_RETURN_IF_LAUNCH_FAILED();
        block_rank_kernel<<<dim3(meta_blocks), dim3(256), 0, st>>>(d->n_rows, r_eff, perm, blk_r);
        CWL_RETURN_IF_LAUNCH_FAILED();
    }
    prof_end(CWL_PROF_META, st);

    GemmArgs sh = {};
    sh.A1 = x;            sh.lda1 = d->ldx;
    sh.B1 = packed + P.at; sh.ldb1 = d->d_in;
    sh.K1 = (int32_t)d->d_in;
    sh.M = d->n_rows;     sh.N = P.R;
    sh.C = uhat;          sh.ldc = R_all;
    sh.meta = meta;       sh.perm = grouped ? perm : nullptr;
    sh.gate_blk_r = blk_r;

    GemmArgs mn = {};
    mn.A1 = x;            mn.lda1 = d->ldx;
    mn.B1 = packed + P.wt; mn.ldb1 = d->d_in;
    mn.K1 = (int32_t)d->d_in;
    mn.A2 = uhat;         mn.lda2 = R_all;
    mn.B2 = packed + P.bt; mn.ldb2 = P.R;
    mn.blk_r = blk_r;
    mn.M = d->n_rows;     mn.N = d->d_out;
    mn.C = y;             mn.ldc = d->ldy;
    mn.meta = meta;       mn.perm = grouped ? perm : nullptr;

    cwl_status s = CWL_OK;
    prof_begin(CWL_PROF_SHRINK, st);
    if (split.splits >= 2) {
        float* partial = reinterpret_cast<float*>(ws + L.partial);
        GemmArgs pa = {};
        pa.A1 = x;             pa.lda1 = d->ldx;
        pa.B1 = packed + P.at; pa.ldb1 = d->d_in;
        pa.K1 = (int32_t)d->d_in;
        pa.M = d->n_rows;      pa.N = P.R;
        pa.N_tile = split.n_tile;
        pa.splits = split.splits;
        pa.ks_per_split = split.ks_per_split;
        pa.partial = partial;
        pa.ldp = split.ldp;
        pa.partial_stride = split.partial_stride;
        MetaJob job = {};
        job.seq_offsets = seq_offsets;
        job.chunk_offsets = chunk_offsets;
        job.chunk_start = chunk_start;
        job.chunk_len = chunk_len;
        job.rank_idx = rank_idx;
        job.n_seqs = n_seqs;
        job.chunk_cap = chunk_cap;
        job.blend_w = d->blend_w;
        job.lad = lad;
        job.meta = reinterpret_cast<TokMeta*>(ws + L.meta);
        job.blk_r = blk_r;
        job.n_blocks = table_with_products ? (int32_t)meta_blocks : 0;
        pa.perm = grouped ? perm : nullptr;
        s = launch_partial_bf16(pa, job, st);
        if (s == CWL_OK) {
            if (split.splits <= 4) s = launch_shrink_fixup<4>(d->n_rows, P.R, partial, split.splits, split.partial_stride, meta, pa.perm, uhat, st);
            else if (split.splits <= 8) s = launch_shrink_fixup<8>(d->n_rows, P.R, partial, split.splits, split.partial_stride, meta, pa.perm, uhat, st);
            else if (split.splits <= 16) s = launch_shrink_fixup<16>(d->n_rows, P.R, partial, split.splits, split.partial_stride, meta, pa.perm, uhat, st);
            else s = launch_shrink_fixup<32>(d->n_rows, P.R, partial, split.splits, split.partial_stride, meta, pa.perm, uhat, st);
        }
    } else if (n_proj == 1) {
        GemmArgs g1 = sh;
        g1.gate_period = P.R;                          // one adapter: the direction is the column
        if (d->dt == CWL_F32) s = launch_gemm_f32(sh, EPI_GATE, st);
        else if (shrink_wide_bf16_serves(g1)) s = launch_shrink_wide_bf16(g1, st);
        else s = launch_shrink_bf16(sh, st);
    } else {
        // one shrink over the concatenated adapters: x is read once for as many adapters as fit the
        // widest shrink tile (256 directions), their directions side by side in uhat
        // (from kShrinkTallRows rows up the bf16 shrink takes any number of 64-direction column tiles)
        const int32_t per_launch = (d->dt == CWL_F32 || d->n_rows >= kShrinkTallRows) ? n_proj
                                   : (256 / P.R > 0 ? 256 / P.R : 1);
        for (int32_t p0 = 0; p0 < n_proj && s == CWL_OK; p0 += per_launch) {
            const int32_t np = n_proj - p0 < per_launch ? n_proj - p0 : per_launch;
            GemmArgs g2 = sh;
            g2.B1 = packed + P.at + es * (size_t)p0 * (size_t)P.R * (size_t)d->d_in;
            g2.N = (int64_t)np * P.R;
            g2.C = uhat + es * (size_t)p0 * (size_t)P.R;
            g2.gate_period = P.R;
            if (d->dt == CWL_F32) s = launch_gemm_f32(g2, EPI_GATE, st);
            else if (shrink_wide_bf16_serves(g2)) s = launch_shrink_wide_bf16(g2, st);
            else s = launch_shrink_bf16(g2, st);
        }
    }
    prof_end(CWL_PROF_SHRINK, st);
    if (s != CWL_OK) return s;
    prof_begin(CWL_PROF_MAIN, st);
    for (int32_t p = 0; p < n_proj && s == CWL_OK; ++p) {
        GemmArgs g2 = mn;
        if (n_proj > 1) {
            g2.B1 = packed + P.wt + es * (size_t)grp.col0[p] * (size_t)d->d_in;
            g2.N = grp.cols[p];
            g2.C = static_cast<char*>(y) + es * (size_t)grp.col0[p];
            g2.A2 = uhat + es * (size_t)p * (size_t)P.R;
            g2.B2 = packed + P.bt + es * (size_t)grp.col0[p] * (size_t)P.R;
        }
        s = d->dt == CWL_F32 ? launch_gemm_f32(g2, EPI_STORE, st) : launch_main_bf16(g2, st);
    }
    prof_end(CWL_PROF_MAIN, st);
    return s;
}

cwl_status check_call(const cwl_linear_desc* d, const void* x, const int32_t* seq_offsets,
                      int32_t n_seqs, const int32_t* chunk_offsets, const int32_t* chunk_start,
                      const int32_t* chunk_len, const int32_t* rank_idx, int32_t chunk_cap,
                      const void* y, const void* ws, bool ws_given = true) {
    if (n_seqs < 0 || chunk_cap < 0) return CWL_ERR_INVALID_ARG;
    if (d->n_rows == 0) return CWL_OK;
    if (!x || !y || (ws_given && !ws)) return CWL_ERR_NULL;
    if (n_seqs > 0 && (!seq_offsets || !chunk_offsets)) return CWL_ERR_NULL;
    if (n_seqs > 0 && chunk_cap > 0 && (!chunk_start || !chunk_len || !rank_idx)) return CWL_ERR_NULL;
    if (ws_given && reinterpret_cast<uintptr_t>(ws) % 256) return CWL_ERR_INVALID_ARG;
    if (d->dt == CWL_BF16 &&
        (reinterpret_cast<uintptr_t>(x) % 16 || reinterpret_cast<uintptr_t>(y) % 16))
        return CWL_ERR_UNSUPPORTED;
    if (d->dt == CWL_F32 && (reinterpret_cast<uintptr_t>(x) % 4 || reinterpret_cast<uintptr_t>(y) % 4))
        return CWL_ERR_INVALID_ARG;
    return CWL_OK;
}

// ---- the two-phase call: x A first (no chunk table needed), gate + main GEMM later -----------------
// What the first phase leaves for the second: nothing up to kSmallRows rows (there the whole layer is
// one product and the second phase is the ordinary call), the fp32 slices of the split shrink below
// 16384 rows, else x A [n_rows, padded rank] in fp32.
size_t shrunk_bytes(const cwl_linear_desc* d) {
    if (small_rows_path(d, packed_layout(d))) return 256;
    const SmallPlan split = shrink_split_plan(d);
    if (split.splits >= 2) return align_up(split.partial_bytes, 256);
    return align_up(sizeof(float) * (size_t)d->n_rows * (size_t)padded_rank(d->r_max), 256);
}

cwl_status run_shrunk(const cwl_linear_desc* d, const void* x, const char* packed, const float* u,
                      const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
                      const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                      int32_t chunk_cap, void* y, char* ws, hipStream_t st) {
    const PackedLayout P = packed_layout(d);
    if (small_rows_path(d, P))
        return run_packed(d, group_cols(d, nullptr), x, packed, seq_offsets, n_seqs, chunk_offsets, chunk_start,
                          chunk_len, rank_idx, chunk_cap, nullptr, y, ws, st);
    const WsLayout L = ws_layout(d);
    int32_t* blk_r = reinterpret_cast<int32_t*>(ws + L.blk_r);
    char* uhat = ws + L.uhat;
    Ladder lad = {};
    lad.K = d->K;
    for (int32_t k = 0; k < d->K; ++k) {
        lad.ranks[k] = d->ranks[k];
        lad.scales[k] = d->scales[k];
    }
    SmallPlan split = shrink_split_plan(d);
    int32_t splits = split.splits >= 2 ? split.splits : 1;
    const int64_t pstride = split.splits >= 2 ? split.partial_stride : 0;
#define CWL_GATE_ARGS d, P.R, u, splits, pstride, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap, lad, uhat, blk_r, st
    cwl_status s;
    prof_begin(CWL_PROF_META, st);
    if (d->dt == CWL_F32) s = launch_gate_product<1, float>(CWL_GATE_ARGS);
    else if (splits <= 1) s = launch_gate_product<1, __bf16>(CWL_GATE_ARGS);
    else if (splits <= 4) s = launch_gate_product<4, __bf16>(CWL_GATE_ARGS);
    else if (splits <= 8) s = launch_gate_product<8, __bf16>(CWL_GATE_ARGS);
    else if (splits <= 16) s = launch_gate_product<16, __bf16>(CWL_GATE_ARGS);
    else s = launch_gate_product<32, __bf16>(CWL_GATE_ARGS);
#undef CWL_GATE_ARGS
    prof_end(CWL_PROF_META, st);
    if (s != CWL_OK) return s;
    GemmArgs mn = {};
    mn.A1 = x;             mn.lda1 = d->ldx;
    mn.B1 = packed + P.wt; mn.ldb1 = d->d_in;
    mn.K1 = (int32_t)d->d_in;
    mn.A2 = uhat;          mn.lda2 = P.R;
    mn.B2 = packed + P.bt; mn.ldb2 = P.R;
    mn.blk_r = blk_r;
    mn.M = d->n_rows;      mn.N = d->d_out;
    mn.C = y;              mn.ldc = d->ldy;
    prof_begin(CWL_PROF_MAIN, st);
    s = d->dt == CWL_F32 ? launch_gemm_f32(mn, EPI_STORE, st) : launch_main_bf16(mn, st);
    prof_end(CWL_PROF_MAIN, st);
    return s;
}

// Address of the static scratch array on the current device, looked up once per device (each GPU
// holds its own copy of the array at its own address).
void* g_scratch_ptr[kMaxDevices] = {};

cwl_status static_scratch(char** out) {
    const int dev = device_slot();
    if (dev < 0) return CWL_ERR_DEVICE;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return CWL_ERR_DEVICE;
        if (reinterpret_cast<uintptr_t>(p) % 256) return CWL_ERR_DEVICE;
        g_scratch_ptr[dev] = p;
    }
    *out = static_cast<char*>(g_scratch_ptr[dev]);
    return CWL_OK;
}

}  // namespace

// ---- the first phase as the chunker's call sees it (declared in partition_seq.h) ----
cwl_status check_shrink_phase(const cwl_linear_desc* d, const void* x, const void* packed, const void* u,
                              size_t u_bytes) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    if (d->group_rows != 0) return CWL_ERR_UNSUPPORTED;
    if (d->n_rows == 0) return CWL_OK;
    if (!x || !packed || !u) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256 || reinterpret_cast<uintptr_t>(u) % 256) return CWL_ERR_INVALID_ARG;
    if (d->dt == CWL_BF16 && reinterpret_cast<uintptr_t>(x) % 16) return CWL_ERR_UNSUPPORTED;
    if (d->dt == CWL_F32 && reinterpret_cast<uintptr_t>(x) % 4) return CWL_ERR_INVALID_ARG;
    if (u_bytes < shrunk_bytes(d)) return CWL_ERR_CAPACITY;
    return CWL_OK;
}

cwl_status run_shrink_phase(const cwl_linear_desc* d, const void* x, const char* packed, float* u, hipStream_t st) {
    const PackedLayout P = packed_layout(d);
    if (small_rows_path(d, P)) return CWL_OK;
    GemmArgs sh = {};
    sh.A1 = x;             sh.lda1 = d->ldx;
    sh.B1 = packed + P.at; sh.ldb1 = d->d_in;
    sh.K1 = (int32_t)d->d_in;
    sh.M = d->n_rows;      sh.N = P.R;
    cwl_status s = CWL_OK;
    prof_begin(CWL_PROF_SHRINK, st);
    const SmallPlan split = shrink_split_plan(d);
    if (d->dt == CWL_F32) {
        sh.C = u;          sh.ldc = P.R;
        s = launch_gemm_f32(sh, EPI_STORE, st);
    } else if (split.splits >= 2) {
        sh.N_tile = split.n_tile;
        sh.splits = split.splits;
        sh.ks_per_split = split.ks_per_split;
        sh.partial = u;
        sh.ldp = split.ldp;
        sh.partial_stride = split.partial_stride;
        MetaJob job = {};
        s = launch_partial_bf16(sh, job, st);
    } else {
        sh.partial = u;    sh.ldp = P.R;
        s = launch_shrink_raw_bf16(sh, st);
    }
    prof_end(CWL_PROF_SHRINK, st);
    return s;
}

// One launch for the short-sequence chunker and the product: only where the product is the one-pass
// kernel on 64-row tiles with a ring small enough for two workgroups per compute unit.
cwl_status launch_seq_with_shrink(const part::SeqJob& job, const cwl_linear_desc* d, const void* x,
                                  const char* packed, float* u, hipStream_t st) {
    const PackedLayout P = packed_layout(d);
    if (d->dt != CWL_BF16 || small_rows_path(d, P) || shrink_split_plan(d).splits >= 2 ||
        d->n_rows >= kShrinkTallRows || (P.R != 64 && P.R != 128))
        return CWL_ERR_UNSUPPORTED;
    GemmArgs sh = {};
    sh.A1 = x;             sh.lda1 = d->ldx;
    sh.B1 = packed + P.at; sh.ldb1 = d->d_in;
    sh.K1 = (int32_t)d->d_in;
    sh.M = d->n_rows;      sh.N = P.R;
    sh.partial = u;        sh.ldp = P.R;
    return launch_seq_shrink_raw_bf16(job, sh, st);
}

}  // namespace cwl

using namespace cwl;

extern "C" size_t cwl_packed_weights_bytes(const cwl_linear_desc* d) {
    if (check_desc(d) != CWL_OK) return 0;
    return packed_layout(d).total;
}

extern "C" cwl_status cwl_prepack_weights(const cwl_linear_desc* d, const void* W, const void* A,
                                          const void* B, void* packed, size_t packed_bytes,
                                          void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_raw_weights(d);
    if (s != CWL_OK) return s;
    if (!W || !packed) return CWL_ERR_NULL;
    if (d->r_max > 0 && (!A || !B)) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CWL_ERR_INVALID_ARG;
    const PackedLayout L = packed_layout(d);
    if (packed_bytes < L.total) return CWL_ERR_CAPACITY;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d->dt == CWL_F32) return prepack_typed<float>(d, L, W, A, B, static_cast<char*>(packed), st);
    return prepack_typed<uint16_t>(d, L, W, A, B, static_cast<char*>(packed), st);
}

extern "C" size_t cwl_linear_packed_workspace_bytes(const cwl_linear_desc* d) {
    if (check_desc(d) != CWL_OK) return 0;
    return ws_layout(d).total;
}

extern "C" size_t cwl_linear_workspace_bytes(const cwl_linear_desc* d) {
    if (check_desc(d) != CWL_OK) return 0;
    return ws_layout(d).total + packed_layout(d).total;
}

extern "C" cwl_status cwl_chunkwise_lora_linear_packed(
    const cwl_linear_desc* d, const void* x, const void* packed, const int32_t* seq_offsets,
    int32_t n_seqs, const int32_t* chunk_offsets, const int32_t* chunk_start,
    const int32_t* chunk_len, const int32_t* rank_idx, int32_t chunk_cap, void* y, void* workspace,
    size_t workspace_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_call(d, x, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                   chunk_cap, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CWL_ERR_INVALID_ARG;
    if (workspace_bytes < ws_layout(d).total) return CWL_ERR_CAPACITY;
    return run_packed(d, group_cols(d, nullptr), x, static_cast<const char*>(packed), seq_offsets, n_seqs,
                      chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap, nullptr, y,
                      static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

extern "C" cwl_status cwl_chunkwise_lora_linear_packed_static(
    const cwl_linear_desc* d, const void* x, const void* packed, const int32_t* seq_offsets,
    int32_t n_seqs, const int32_t* chunk_offsets, const int32_t* chunk_start,
    const int32_t* chunk_len, const int32_t* rank_idx, int32_t chunk_cap, void* y, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_call(d, x, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                   chunk_cap, y, nullptr, false);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CWL_ERR_INVALID_ARG;
    if (ws_layout(d).total > CWL_STATIC_SCRATCH_BYTES) return CWL_ERR_CAPACITY;
    char* ws = nullptr;
    s = static_scratch(&ws);
    if (s != CWL_OK) return s;
    return run_packed(d, group_cols(d, nullptr), x, static_cast<const char*>(packed), seq_offsets, n_seqs,
                      chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap, nullptr, y, ws,
                      static_cast<hipStream_t>(stream));
}

extern "C" size_t cwl_lora_shrink_bytes(const cwl_linear_desc* d) {
    if (check_desc(d) != CWL_OK || d->group_rows != 0) return 0;
    return shrunk_bytes(d);
}

extern "C" cwl_status cwl_lora_shrink_packed(const cwl_linear_desc* d, const void* x, const void* packed,
                                             void* u, size_t u_bytes, void* stream) {
    const cwl_status s = check_shrink_phase(d, x, packed, u, u_bytes);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    return run_shrink_phase(d, x, static_cast<const char*>(packed), static_cast<float*>(u),
                            static_cast<hipStream_t>(stream));
}

extern "C" cwl_status cwl_chunkwise_lora_linear_packed_shrunk(
    const cwl_linear_desc* d, const void* x, const void* packed, const void* u, size_t u_bytes,
    const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets, const int32_t* chunk_start,
    const int32_t* chunk_len, const int32_t* rank_idx, int32_t chunk_cap, void* y, void* workspace,
    size_t workspace_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    if (d->group_rows != 0) return CWL_ERR_UNSUPPORTED;
    s = check_call(d, x, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                   chunk_cap, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed || !u) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256 || reinterpret_cast<uintptr_t>(u) % 256) return CWL_ERR_INVALID_ARG;
    if (u_bytes < shrunk_bytes(d)) return CWL_ERR_CAPACITY;
    if (workspace_bytes < ws_layout(d).total) return CWL_ERR_CAPACITY;
    return run_shrunk(d, x, static_cast<const char*>(packed), static_cast<const float*>(u), seq_offsets, n_seqs,
                      chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap, y,
                      static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

extern "C" cwl_status cwl_chunkwise_lora_linear(
    const cwl_linear_desc* d, const void* x, const void* W, const void* A, const void* B,
    const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets,
    const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
    int32_t chunk_cap, void* y, void* workspace, size_t workspace_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_raw_weights(d);
    if (s != CWL_OK) return s;
    s = check_call(d, x, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                   chunk_cap, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!W) return CWL_ERR_NULL;
    if (d->r_max > 0 && (!A || !B)) return CWL_ERR_NULL;
    const size_t core = ws_layout(d).total;
    const PackedLayout L = packed_layout(d);
    if (workspace_bytes < core + L.total) return CWL_ERR_CAPACITY;
    char* ws = static_cast<char*>(workspace);
    char* packed = ws + core;
    hipStream_t st = static_cast<hipStream_t>(stream);
    s = d->dt == CWL_F32 ? prepack_typed<float>(d, L, W, A, B, packed, st)
                         : prepack_typed<uint16_t>(d, L, W, A, B, packed, st);
    if (s != CWL_OK) return s;
    return run_packed(d, group_cols(d, nullptr), x, packed, seq_offsets, n_seqs, chunk_offsets, chunk_start,
                      chunk_len, rank_idx, chunk_cap, nullptr, y, ws, st);
}

extern "C" cwl_status cwl_gated_lora_linear_packed(const cwl_linear_desc* d, const void* x,
                                                   const void* packed, const cwl_token_gate* gate,
                                                   void* y, void* workspace, size_t workspace_bytes,
                                                   void* stream) {
    static_assert(sizeof(cwl_token_gate) == sizeof(TokMeta), "a gate entry is a TokMeta");
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    if (d->group_rows != 0) return CWL_ERR_UNSUPPORTED;
    s = check_call(d, x, nullptr, 0, nullptr, nullptr, nullptr, nullptr, 0, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed || !gate) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256 || reinterpret_cast<uintptr_t>(gate) % 16)
        return CWL_ERR_INVALID_ARG;
    if (workspace_bytes < ws_layout(d).total) return CWL_ERR_CAPACITY;
    return run_packed(d, group_cols(d, nullptr), x, static_cast<const char*>(packed), nullptr, 0, nullptr,
                      nullptr, nullptr, nullptr, 0, reinterpret_cast<const TokMeta*>(gate), y,
                      static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

// ---- projections that share x -----------------------------------------------------------------
extern "C" size_t cwl_packed_weights_grouped_bytes(const cwl_linear_desc* d, const cwl_group* g) {
    if (check_desc(d) != CWL_OK || check_group(d, g) != CWL_OK) return 0;
    return packed_layout(d, g->n_proj).total;
}

extern "C" size_t cwl_linear_grouped_workspace_bytes(const cwl_linear_desc* d, const cwl_group* g) {
    if (check_desc(d) != CWL_OK || check_group(d, g) != CWL_OK) return 0;
    return ws_layout(d, g->n_proj).total;
}

extern "C" cwl_status cwl_prepack_weights_grouped(const cwl_linear_desc* d, const cwl_group* g, void* packed,
                                                  size_t packed_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_group(d, g);
    if (s != CWL_OK) return s;
    if (!packed) return CWL_ERR_NULL;
    for (int32_t p = 0; p < g->n_proj; ++p) {
        if (!g->W[p]) return CWL_ERR_NULL;
        if (d->r_max > 0 && (!g->A[p] || !g->B[p])) return CWL_ERR_NULL;
    }
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CWL_ERR_INVALID_ARG;
    const PackedLayout L = packed_layout(d, g->n_proj);
    if (packed_bytes < L.total) return CWL_ERR_CAPACITY;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (d->dt == CWL_F32) return prepack_group_typed<float>(d, g, L, static_cast<char*>(packed), st);
    return prepack_group_typed<uint16_t>(d, g, L, static_cast<char*>(packed), st);
}

extern "C" cwl_status cwl_chunkwise_lora_linear_grouped_packed(
    const cwl_linear_desc* d, const cwl_group* g, const void* x, const void* packed,
    const int32_t* seq_offsets, int32_t n_seqs, const int32_t* chunk_offsets, const int32_t* chunk_start,
    const int32_t* chunk_len, const int32_t* rank_idx, int32_t chunk_cap, void* y, void* workspace,
    size_t workspace_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_group(d, g);
    if (s != CWL_OK) return s;
    s = check_call(d, x, seq_offsets, n_seqs, chunk_offsets, chunk_start, chunk_len, rank_idx,
                   chunk_cap, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256) return CWL_ERR_INVALID_ARG;
    if (workspace_bytes < ws_layout(d, g->n_proj).total) return CWL_ERR_CAPACITY;
    return run_packed(d, group_cols(d, g), x, static_cast<const char*>(packed), seq_offsets, n_seqs,
                      chunk_offsets, chunk_start, chunk_len, rank_idx, chunk_cap, nullptr, y,
                      static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

extern "C" cwl_status cwl_gated_lora_linear_grouped_packed(const cwl_linear_desc* d, const cwl_group* g,
                                                           const void* x, const void* packed,
                                                           const cwl_token_gate* gate, void* y, void* workspace,
                                                           size_t workspace_bytes, void* stream) {
    cwl_status s = check_desc(d);
    if (s != CWL_OK) return s;
    s = check_group(d, g);
    if (s != CWL_OK) return s;
    s = check_call(d, x, nullptr, 0, nullptr, nullptr, nullptr, nullptr, 0, y, workspace);
    if (s != CWL_OK) return s;
    if (d->n_rows == 0) return CWL_OK;
    if (!packed || !gate) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(packed) % 256 || reinterpret_cast<uintptr_t>(gate) % 16)
        return CWL_ERR_INVALID_ARG;
    if (workspace_bytes < ws_layout(d, g->n_proj).total) return CWL_ERR_CAPACITY;
    return run_packed(d, group_cols(d, g), x, static_cast<const char*>(packed), nullptr, 0, nullptr, nullptr,
                      nullptr, nullptr, 0, reinterpret_cast<const TokMeta*>(gate), y,
                      static_cast<char*>(workspace), static_cast<hipStream_t>(stream));
}

extern "C" const char* cwl_status_string(cwl_status s) {
    switch (s) {
        case CWL_OK: return "ok";
        case CWL_ERR_NULL: return "null pointer";
        case CWL_ERR_INVALID_ARG: return "invalid argument";
        case CWL_ERR_INFEASIBLE: return "length bounds infeasible (l_max < 2*l_min - 1)";
        case CWL_ERR_CAPACITY: return "buffer or workspace too small";
        case CWL_ERR_UNSUPPORTED: return "unsupported shape, alignment or dtype";
        case CWL_ERR_DEVICE: return "HIP launch failed";
    }
    return "unknown status";
}

extern "C" int32_t cwl_abi_version(void) { return 1; }
