// cwl_select_ranks_budget, cwl_bucket_sequences and cwl_partition_chunks_aligned (gfx950 only): the
// budget of high-capacity regions per sequence (Sec. III-B of arxiv 2601.21109), the buckets of
// sequences by complexity percentile with the complexity-balanced micro-batches (Sec. III-G,
// Sec. IV-F), and the chunker whose boundaries are shared inside a bucket (Sec. III-G).
// include/cwl.h states the readings taken.  All of it is integer work on the quantised scores and
// on tables of a few thousand entries: short kernels whose cost is their launch.
//
// Aligned chunker, six launches:
//   plan    (one workgroup): members of every bucket, its longest member, and from those the rows
//           [v_off[b], v_off[b+1]) that the bucket's mean series takes in a scratch score array;
//   mean    (one thread per row of that array): floor-mean of the members' quantised scores,
//           written back as an fp32 score that quantises to exactly that integer;
//   chunker (the kernels of cwl_partition_chunks) on the mean series, one "sequence" per bucket;
//   offsets (one workgroup): chunks of each sequence = the bucket's chunk starts inside it
//           (a binary search), exclusive scan into chunk_offsets, status word;
//   emit    (one workgroup per sequence, one wavefront per chunk): start, length cut at the end of
//           the sequence, and the sum of the sequence's own quantised scores.
#include "common.h"

namespace cwl {
namespace {

constexpr int kMaxSeqs = 4096;      // what the single-workgroup ranking / planning kernels hold in LDS
constexpr int kMaxBuckets = 4096;
constexpr int kOne = 1024;          // threads of the single-workgroup kernels
constexpr int kPer = kMaxSeqs / kOne;

// exclusive prefix sum over the workgroup of one value per thread; *total = the sum
__device__ int64_t block_excl_scan(int64_t v, int64_t* wave_tot /*LDS[waves]*/, int64_t* total) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t incl = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int64_t t = shfl_up_i64(incl, off);
        if (lane >= off) incl += t;
    }
    __syncthreads();
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    int64_t pre = 0, tot = 0;
    for (int w = 0; w < (int)blockDim.x / 64; ++w) {
        if (w < wave) pre += wave_tot[w];
        tot += wave_tot[w];
    }
    *total = tot;
    return pre + incl - v;
}

// ---- rung selection under a budget: one wavefront per sequence ----
__global__ void __launch_bounds__(256)
select_budget_kernel(const int64_t* __restrict__ chunk_sum, const int32_t* __restrict__ chunk_len,
                     const int32_t* __restrict__ chunk_offsets, int32_t n_seqs, int32_t cap, TauTable th,
                     int32_t K, int32_t k_high, int32_t budget, int32_t* __restrict__ rank_idx,
                     int32_t* __restrict__ n_asked) {
    const int lane = threadIdx.x & 63;
    const int32_t s = (int32_t)blockIdx.x * 4 + (int32_t)(threadIdx.x >> 6);
    if (s >= n_seqs) return;
    int64_t c0 = chunk_offsets[s], c1 = chunk_offsets[s + 1];
    if (c0 < 0) c0 = 0;
    if (c1 > cap) c1 = cap;
    int32_t asked = 0;                                   // the same in every lane
    for (int64_t c = c0; c < c1; c += 64) {
        const int64_t i = c + lane;
        const bool in = i < c1;
        int32_t k = 0;
        if (in) {
            const int64_t sum = chunk_sum[i];
            const int64_t len = chunk_len[i];
            for (int32_t j = 0; j < K - 1; ++j) k += (sum >= th.tau_q[j] * len) ? 1 : 0;
        }
        const bool asks = in && k >= k_high;
        const unsigned long long m = __ballot(asks);
        const int32_t before = asked + __popcll(m & ((1ull << lane) - 1ull));
        if (asks && before >= budget) k = k_high - 1;
        if (in) rank_idx[i] = k;
        asked += __popcll(m);
    }
    if (lane == 0 && n_asked) n_asked[s] = asked;
}

// ---- sum of the quantised scores of each sequence: one workgroup per sequence ----
__global__ void __launch_bounds__(kOne)
seq_sum_kernel(const float* __restrict__ score, int64_t n_rows, const int32_t* __restrict__ seq_offsets,
               int64_t* __restrict__ seq_sum) {
    __shared__ int64_t wave_tot[kOne / 64];
    int64_t base, T;
    bool bad = false, nan = false;
    seq_extent(seq_offsets, (int32_t)blockIdx.x, n_rows, &base, &T, &bad);
    int64_t acc = 0;
    for (int64_t t = threadIdx.x; t < T; t += kOne) acc += quantise_score(score[base + t], &nan);
    acc = wave_sum_i64(acc);
    if ((threadIdx.x & 63) == 0) wave_tot[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t tot = 0;
        for (int w = 0; w < kOne / 64; ++w) tot += wave_tot[w];
        seq_sum[blockIdx.x] = tot;
    }
}

// ---- rank by mean score, buckets, micro-batches: one workgroup ----
__global__ void __launch_bounds__(kOne)
bucket_rank_kernel(const int64_t* __restrict__ seq_sum, const int32_t* __restrict__ seq_offsets, int64_t n_rows,
                   int32_t n_seqs, int32_t n_buckets, int32_t n_micro, int32_t* __restrict__ order,
                   int32_t* __restrict__ bucket, int32_t* __restrict__ micro) {
    __shared__ int32_t mean[kMaxSeqs];
    for (int32_t s = threadIdx.x; s < n_seqs; s += kOne) {
        int64_t base, T;
        bool bad = false;
        seq_extent(seq_offsets, s, n_rows, &base, &T, &bad);
        mean[s] = T > 0 ? (int32_t)(seq_sum[s] / T) : 0;      // at most 2^20
    }
    __syncthreads();
    for (int32_t s = threadIdx.x; s < n_seqs; s += kOne) {
        const int32_t mine = mean[s];
        int32_t rho = 0;
        for (int32_t u = 0; u < n_seqs; ++u) {
            const int32_t v = mean[u];
            rho += (v < mine || (v == mine && u < s)) ? 1 : 0;
        }
        order[rho] = s;
        bucket[s] = (int32_t)(((int64_t)rho * n_buckets) / n_seqs);
        if (micro) {
            const int32_t round = rho / n_micro, j = rho % n_micro;
            micro[s] = (round & 1) ? n_micro - 1 - j : j;
        }
    }
}

// ---- aligned chunker ----
struct AlignWs {
    int32_t* members;      // [n_seqs]       sequences grouped by bucket
    int32_t* member_off;   // [n_buckets+1]
    int32_t* v_off;        // [n_buckets+1]  rows of each bucket's mean series in vscore
    int32_t* flags;        // [1]            status bits met by the plan and mean kernels
    float* vscore;         // [n_rows]
    int32_t* v_co;         // [n_buckets+1]  chunk table of the mean series
    int32_t* v_start;      // [v_cap]
    int32_t* v_len;        // [v_cap]
    int64_t* v_sum;        // [v_cap]
    int32_t* v_status;     // [1]
    void* part;            // workspace of the chunker
    size_t part_bytes;
    int32_t v_cap;
};

size_t align_ws_layout(int64_t n_rows, int32_t n_seqs, int32_t n_buckets, const cwl_chunk_params* p, void* base,
                       AlignWs* ws) {
    const int64_t v_cap = n_rows / (p->l_min > 0 ? p->l_min : 1) + n_buckets + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = align_up(off + bytes, 256);
        return o;
    };
    const size_t part_bytes = cwl_partition_workspace_bytes(n_rows, n_buckets, p);
    const size_t o_sum = take(sizeof(int64_t) * (size_t)v_cap);
    const size_t o_mem = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    const size_t o_moff = take(sizeof(int32_t) * (size_t)(n_buckets + 1));
    const size_t o_voff = take(sizeof(int32_t) * (size_t)(n_buckets + 1));
    const size_t o_flags = take(sizeof(int32_t));
    const size_t o_vs = take(sizeof(float) * (size_t)(n_rows + 1));
    const size_t o_vco = take(sizeof(int32_t) * (size_t)(n_buckets + 1));
    const size_t o_start = take(sizeof(int32_t) * (size_t)v_cap);
    const size_t o_len = take(sizeof(int32_t) * (size_t)v_cap);
    const size_t o_stat = take(sizeof(int32_t));
    const size_t o_part = take(part_bytes);
    if (ws) {
        char* b = static_cast<char*>(base);
        ws->v_sum = reinterpret_cast<int64_t*>(b + o_sum);
        ws->members = reinterpret_cast<int32_t*>(b + o_mem);
        ws->member_off = reinterpret_cast<int32_t*>(b + o_moff);
        ws->v_off = reinterpret_cast<int32_t*>(b + o_voff);
        ws->flags = reinterpret_cast<int32_t*>(b + o_flags);
        ws->vscore = reinterpret_cast<float*>(b + o_vs);
        ws->v_co = reinterpret_cast<int32_t*>(b + o_vco);
        ws->v_start = reinterpret_cast<int32_t*>(b + o_start);
        ws->v_len = reinterpret_cast<int32_t*>(b + o_len);
        ws->v_status = reinterpret_cast<int32_t*>(b + o_stat);
        ws->part = b + o_part;
        ws->part_bytes = part_bytes;
        ws->v_cap = (int32_t)(v_cap > 0x7fffffff ? 0x7fffffff : v_cap);
    }
    return off;
}

__device__ __forceinline__ int32_t bucket_of(const int32_t* bucket, int32_t s, int32_t n_buckets, bool* bad) {
    int32_t b = bucket[s];
    if (b < 0) { *bad = true; b = 0; }
    if (b >= n_buckets) { *bad = true; b = n_buckets - 1; }
    return b;
}

// plan: members of every bucket and the rows of its mean series
__global__ void __launch_bounds__(kOne)
align_plan_kernel(int64_t n_rows, const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                  const int32_t* __restrict__ bucket, int32_t n_buckets, AlignWs ws) {
    __shared__ int32_t cnt[kMaxBuckets];       // members, then the write cursor of the bucket
    __shared__ int32_t tmax[kMaxBuckets];      // longest member
    __shared__ int64_t wave_tot[kOne / 64];
    const int tid = threadIdx.x;
    for (int32_t b = tid; b < n_buckets; b += kOne) { cnt[b] = 0; tmax[b] = 0; }
    __syncthreads();
    bool bad_seq = false, bad_bucket = false;
    if (tid == 0 && (int64_t)seq_offsets[n_seqs] != n_rows) bad_seq = true;
    for (int32_t s = tid; s < n_seqs; s += kOne) {
        int64_t base, T;
        seq_extent(seq_offsets, s, n_rows, &base, &T, &bad_seq);
        const int32_t b = bucket_of(bucket, s, n_buckets, &bad_bucket);
        atomicAdd(&cnt[b], 1);
        atomicMax(&tmax[b], (int32_t)T);
    }
    __syncthreads();
    // exclusive scans over the buckets, kPer consecutive buckets per thread
    int64_t c_loc[kPer], t_loc[kPer], c_sum = 0, t_sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int32_t b = tid * kPer + i;
        c_loc[i] = c_sum;
        t_loc[i] = t_sum;
        if (b < n_buckets) { c_sum += cnt[b]; t_sum += tmax[b]; }
    }
    int64_t c_tot, t_tot;
    const int64_t c_pre = block_excl_scan(c_sum, wave_tot, &c_tot);
    const int64_t t_pre = block_excl_scan(t_sum, wave_tot, &t_tot);
    __syncthreads();
    // well-formed offsets give t_tot <= n_rows; overlapping sequences could exceed the scratch rows
    bool clipped = false;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int32_t b = tid * kPer + i;
        if (b < n_buckets) {
            int64_t v = t_pre + t_loc[i];
            if (v > n_rows) { v = n_rows; clipped = true; }
            ws.v_off[b] = (int32_t)v;
            ws.member_off[b] = (int32_t)(c_pre + c_loc[i]);
            cnt[b] = (int32_t)(c_pre + c_loc[i]);
        }
    }
    if (tid == 0) {
        int64_t v = t_tot;
        if (v > n_rows) { v = n_rows; clipped = true; }
        ws.v_off[n_buckets] = (int32_t)v;
        ws.member_off[n_buckets] = (int32_t)c_tot;
    }
    __syncthreads();
    for (int32_t s = tid; s < n_seqs; s += kOne) {
        bool ignore = false;
        const int32_t b = bucket_of(bucket, s, n_buckets, &ignore);
        ws.members[atomicAdd(&cnt[b], 1)] = s;            // order inside a bucket does not matter: sums only
    }
    const int any_seq = __syncthreads_or((bad_seq || clipped) ? 1 : 0);
    const int any_bucket = __syncthreads_or(bad_bucket ? 1 : 0);
    if (tid == 0)
        *ws.flags = (any_seq ? (int32_t)CWL_STATUS_BAD_OFFSETS : 0) | (any_bucket ? (int32_t)CWL_STATUS_BAD_BUCKET : 0);
}

// mean series of every bucket: one thread per row of vscore
__global__ void __launch_bounds__(256)
align_mean_kernel(const float* __restrict__ score, int64_t n_rows, const int32_t* __restrict__ seq_offsets,
                  int32_t n_buckets, AlignWs ws) {
    const int64_t v = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (v >= ws.v_off[n_buckets]) return;
    // the bucket b with v_off[b] <= v < v_off[b+1]
    int32_t lo = 0, hi = n_buckets;
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if ((int64_t)ws.v_off[mid] <= v) lo = mid + 1; else hi = mid;
    }
    const int32_t b = lo - 1;
    const int64_t t = v - ws.v_off[b];
    int64_t acc = 0;
    int32_t alive = 0;
    bool nan = false, bad = false;
    const int32_t m1 = ws.member_off[b + 1];
    for (int32_t m = ws.member_off[b]; m < m1; ++m) {
        int64_t base, T;
        seq_extent(seq_offsets, ws.members[m], n_rows, &base, &T, &bad);
        if (t < T) {
            acc += quantise_score(score[base + t], &nan);
            ++alive;
        }
    }
    const int64_t mean = alive > 0 ? acc / alive : 0;
    ws.vscore[v] = (float)mean * (1.0f / 1024.0f);        // exact, and quantises back to `mean`
    if (nan) atomicOr(ws.flags, (int32_t)CWL_STATUS_NAN_SCORE);
}

// chunks of every sequence, CSR offsets, status word
__global__ void __launch_bounds__(kOne)
align_offsets_kernel(int64_t n_rows, const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                     const int32_t* __restrict__ bucket, int32_t n_buckets, AlignWs ws,
                     int32_t* __restrict__ chunk_offsets, int32_t cap, int32_t* __restrict__ status_word) {
    __shared__ int64_t wave_tot[kOne / 64];
    const int tid = threadIdx.x;
    int64_t loc[kPer], sum = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int32_t s = tid * kPer + i;
        loc[i] = sum;
        if (s < n_seqs) {
            int64_t base, T;
            bool bad = false;
            seq_extent(seq_offsets, s, n_rows, &base, &T, &bad);
            const int32_t b = bucket_of(bucket, s, n_buckets, &bad);
            int32_t c0 = ws.v_co[b], c1 = ws.v_co[b + 1];
            if (c1 > ws.v_cap) c1 = ws.v_cap;
            // chunk starts of the bucket are ascending: count those before the end of the sequence
            const int64_t end = (int64_t)ws.v_off[b] + T;
            int32_t lo = c0, hi = c1;
            while (lo < hi) {
                const int32_t mid = lo + (hi - lo) / 2;
                if ((int64_t)ws.v_start[mid] < end) lo = mid + 1; else hi = mid;
            }
            sum += lo > c0 ? lo - c0 : 0;
        }
    }
    int64_t total;
    const int64_t pre = block_excl_scan(sum, wave_tot, &total);
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        const int32_t s = tid * kPer + i;
        if (s < n_seqs) chunk_offsets[s] = (int32_t)(pre + loc[i]);
    }
    if (tid == 0) {
        chunk_offsets[n_seqs] = (int32_t)total;
        // of the mean series' own status only the capacity bit can mean anything: their offsets are
        // well-formed by construction but do not end at n_rows, which the chunker reports
        *status_word = *ws.flags | (*ws.v_status & (int32_t)CWL_STATUS_CAPACITY) |
                       (total > cap ? (int32_t)CWL_STATUS_CAPACITY : 0);
    }
}

// the chunk records of one sequence: one wavefront per chunk
__global__ void __launch_bounds__(256)
align_emit_kernel(const float* __restrict__ score, int64_t n_rows, const int32_t* __restrict__ seq_offsets,
                  const int32_t* __restrict__ bucket, int32_t n_buckets, AlignWs ws,
                  const int32_t* __restrict__ chunk_offsets, int32_t* __restrict__ chunk_start,
                  int32_t* __restrict__ chunk_len, int64_t* __restrict__ chunk_sum, int32_t cap) {
    const int32_t s = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int64_t base, T;
    bool bad = false, nan = false;
    seq_extent(seq_offsets, s, n_rows, &base, &T, &bad);
    const int32_t b = bucket_of(bucket, s, n_buckets, &bad);
    const int64_t first = chunk_offsets[s];
    const int64_t count = (int64_t)chunk_offsets[s + 1] - first;
    const int32_t c0 = ws.v_co[b];
    const int64_t v0 = ws.v_off[b];
    for (int64_t i = wave; i < count; i += 4) {
        const int64_t dst = first + i;
        if (dst >= cap) break;
        const int64_t rel = (int64_t)ws.v_start[c0 + i] - v0;
        int64_t len = ws.v_len[c0 + i];
        if (len > T - rel) len = T - rel;
        int64_t acc = 0;
        for (int64_t t = lane; t < len; t += 64) acc += quantise_score(score[base + rel + t], &nan);
        acc = wave_sum_i64(acc);
        if (lane == 0) {
            chunk_start[dst] = (int32_t)(base + rel);
            chunk_len[dst] = (int32_t)len;
            chunk_sum[dst] = acc;
        }
    }
}

}  // namespace
}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_select_ranks_budget(const int64_t* chunk_sum, const int32_t* chunk_len,
                                              const int32_t* chunk_offsets, int32_t n_seqs, int32_t cap,
                                              const float* thresholds, int32_t K, int32_t k_high,
                                              int32_t budget, int32_t* rank_idx, int32_t* n_asked,
                                              void* stream) {
    if (K < 1 || K > CWL_MAX_LADDER || n_seqs < 0 || cap < 0 || k_high < 1 || budget < 0) return CWL_ERR_INVALID_ARG;
    if (K > 1 && !thresholds) return CWL_ERR_NULL;
    TauTable th;
    if (fill_tau_table(thresholds, K, &th) != CWL_OK) return CWL_ERR_INVALID_ARG;
    if (n_seqs == 0) return CWL_OK;
    if (!chunk_offsets) return CWL_ERR_NULL;
    if (cap > 0 && (!chunk_sum || !chunk_len || !rank_idx)) return CWL_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    prof_begin(CWL_PROF_SELECT, s);
    select_budget_kernel<<<dim3((unsigned)((n_seqs + 3) / 4)), dim3(256), 0, s>>>(
        chunk_sum, chunk_len, chunk_offsets, n_seqs, cap, th, K, k_high, budget, rank_idx, n_asked);
    prof_end(CWL_PROF_SELECT, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

extern "C" cwl_status cwl_bucket_sequences(const float* score, int64_t n_rows, const int32_t* seq_offsets,
                                           int32_t n_seqs, int32_t n_buckets, int32_t n_micro,
                                           int64_t* seq_sum, int32_t* order, int32_t* bucket, int32_t* micro,
                                           void* stream) {
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0 || n_buckets < 1) return CWL_ERR_INVALID_ARG;
    if (micro && n_micro < 1) return CWL_ERR_INVALID_ARG;
    if (n_seqs > kMaxSeqs) return CWL_ERR_UNSUPPORTED;
    if (n_seqs == 0) return CWL_OK;
    if (!seq_offsets || !seq_sum || !order || !bucket) return CWL_ERR_NULL;
    if (n_rows > 0 && !score) return CWL_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    prof_begin(CWL_PROF_PARTITION, s);
    seq_sum_kernel<<<dim3((unsigned)n_seqs), dim3(kOne), 0, s>>>(score, n_rows, seq_offsets, seq_sum);
    CWL_RETURN_IF_LAUNCH_FAILED();
    bucket_rank_kernel<<<dim3(1), dim3(kOne), 0, s>>>(seq_sum, seq_offsets, n_rows, n_seqs, n_buckets,
                                                      micro ? n_micro : 1, order, bucket, micro);
    prof_end(CWL_PROF_PARTITION, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

extern "C" size_t cwl_aligned_workspace_bytes(int64_t n_rows, int32_t n_seqs, int32_t n_buckets,
                                              const cwl_chunk_params* p) {
    if (n_rows < 0 || n_seqs < 0 || n_buckets < 1 || check_chunk_params(p) != CWL_OK) return 0;
    return align_ws_layout(n_rows, n_seqs, n_buckets, p, nullptr, nullptr);
}

extern "C" cwl_status cwl_partition_chunks_aligned(const float* score, int64_t n_rows,
                                                   const int32_t* seq_offsets, int32_t n_seqs,
                                                   const int32_t* bucket, int32_t n_buckets,
                                                   const cwl_chunk_params* p, int32_t* chunk_offsets,
                                                   int32_t* chunk_start, int32_t* chunk_len,
                                                   int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                                   void* workspace, size_t workspace_bytes, void* stream) {
    cwl_status st = check_chunk_params(p);
    if (st != CWL_OK) return st;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0 || cap < 0 || n_buckets < 1) return CWL_ERR_INVALID_ARG;
    if (n_seqs > kMaxSeqs || n_buckets > kMaxBuckets) return CWL_ERR_UNSUPPORTED;
    if (!seq_offsets || !chunk_offsets || !status_word || !workspace) return CWL_ERR_NULL;
    if (n_seqs > 0 && !bucket) return CWL_ERR_NULL;
    if (n_rows > 0 && !score) return CWL_ERR_NULL;
    if (cap > 0 && (!chunk_start || !chunk_len || !chunk_sum)) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return CWL_ERR_INVALID_ARG;
    AlignWs ws;
    const size_t need = align_ws_layout(n_rows, n_seqs, n_buckets, p, workspace, &ws);
    if (workspace_bytes < need) return CWL_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    prof_begin(CWL_PROF_PARTITION, s);
    align_plan_kernel<<<dim3(1), dim3(kOne), 0, s>>>(n_rows, seq_offsets, n_seqs, bucket, n_buckets, ws);
    CWL_RETURN_IF_LAUNCH_FAILED();
    if (n_rows > 0) {
        align_mean_kernel<<<dim3((unsigned)((n_rows + 255) / 256)), dim3(256), 0, s>>>(score, n_rows, seq_offsets,
                                                                                      n_buckets, ws);
        CWL_RETURN_IF_LAUNCH_FAILED();
    }
    prof_end(CWL_PROF_PARTITION, s);
    // the mean series are as long as the bucket's longest member: about the average sequence
    st = partition_chunks_avg_len(ws.vscore, n_rows, ws.v_off, n_buckets, p, ws.v_co, ws.v_start, ws.v_len,
                                  ws.v_sum, ws.v_cap, ws.v_status, ws.part, ws.part_bytes, stream,
                                  n_seqs > 0 ? n_rows / n_seqs : 0);
    if (st != CWL_OK) return st;
    prof_begin(CWL_PROF_PARTITION, s);
    align_offsets_kernel<<<dim3(1), dim3(kOne), 0, s>>>(n_rows, seq_offsets, n_seqs, bucket, n_buckets, ws,
                                                        chunk_offsets, cap, status_word);
    CWL_RETURN_IF_LAUNCH_FAILED();
    if (n_seqs > 0 && cap > 0) {
        align_emit_kernel<<<dim3((unsigned)n_seqs), dim3(256), 0, s>>>(score, n_rows, seq_offsets, bucket, n_buckets,
                                                                       ws, chunk_offsets, chunk_start, chunk_len,
                                                                       chunk_sum, cap);
        CWL_RETURN_IF_LAUNCH_FAILED();
    }
    prof_end(CWL_PROF_PARTITION, s);
    return CWL_OK;
}
