// cwl_partition_chunks and cwl_select_ranks: the adaptive chunker and the rung selector
// (Sec. III-B / III-C and IV-B / IV-C of arxiv 2601.21109).  Integer work after the one fp32
// quantisation of the scores; latency bound.
//
// Kernel 1 (one workgroup per sequence): quantise the scores, block-scan them into a prefix
// array P, then wavefront 0 places the boundaries: its 64 lanes test 64 candidate ends at once
// and a ballot picks the first admissible end at which a test fires.  Chunks go to a staging
// area whose per-sequence offset is the worst-case chunk count of the preceding sequences.
// (Well-formed offsets never overflow the staging area; writes are bounds-checked all the same.)
// Kernel 2 (one workgroup per sequence): turns the per-sequence counts into CSR offsets, copies the
// staged chunks to their final place and writes the status word.
#include "common.h"

namespace {

using cwl::quantise_score;

constexpr int kThreads = 256;
constexpr int kItems = 8;   // tokens per thread per scan pass

struct PartWs {             // layout of the workspace
    int32_t* q;             // [n_rows]
    int64_t* P;             // [n_rows + n_seqs]   (T_b + 1 entries per sequence)
    int32_t* st_start;      // [stage_cap]
    int32_t* st_len;        // [stage_cap]
    int64_t* st_sum;        // [stage_cap]
    int32_t* seq_count;     // [n_seqs]
    int32_t* seq_stage;     // [n_seqs]
    int32_t* seq_status;    // [n_seqs] status bits met in each sequence
    int64_t stage_cap;
};

__host__ size_t part_ws_layout(int64_t n_rows, int32_t n_seqs, int32_t l_min, void* base, PartWs* ws,
                               int64_t* stage_cap_out) {
    const int64_t stage_cap = n_rows / (l_min > 0 ? l_min : 1) + n_seqs + 1;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        size_t o = off;
        off = cwl::align_up(off + bytes, 256);
        return o;
    };
    char* b = static_cast<char*>(base);
    size_t o_P = take(sizeof(int64_t) * (size_t)(n_rows + n_seqs + 1));
    size_t o_sum = take(sizeof(int64_t) * (size_t)stage_cap);
    size_t o_q = take(sizeof(int32_t) * (size_t)(n_rows + 1));
    size_t o_start = take(sizeof(int32_t) * (size_t)stage_cap);
    size_t o_len = take(sizeof(int32_t) * (size_t)stage_cap);
    size_t o_cnt = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    size_t o_stage = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    size_t o_status = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    if (ws) {
        ws->P = reinterpret_cast<int64_t*>(b + o_P);
        ws->st_sum = reinterpret_cast<int64_t*>(b + o_sum);
        ws->q = reinterpret_cast<int32_t*>(b + o_q);
        ws->st_start = reinterpret_cast<int32_t*>(b + o_start);
        ws->st_len = reinterpret_cast<int32_t*>(b + o_len);
        ws->seq_count = reinterpret_cast<int32_t*>(b + o_cnt);
        ws->seq_stage = reinterpret_cast<int32_t*>(b + o_stage);
        ws->seq_status = reinterpret_cast<int32_t*>(b + o_status);
        ws->stage_cap = stage_cap;
    }
    if (stage_cap_out) *stage_cap_out = stage_cap;
    return off;
}

__device__ __forceinline__ int64_t shfl_up_i64(int64_t v, int delta) {
    int lo = __shfl_up((int)(v & 0xffffffffll), delta);
    int hi = __shfl_up((int)(v >> 32), delta);
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

// sum over the block of one int64 per thread; every thread gets the result
__device__ int64_t block_sum_i64(int64_t v, int64_t* smem /*[4]*/) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) {
        int lo = __shfl_xor((int)(v & 0xffffffffll), off);
        int hi = __shfl_xor((int)(v >> 32), off);
        v += ((int64_t)hi << 32) | (uint32_t)lo;
    }
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    return smem[0] + smem[1] + smem[2] + smem[3];
}

// sequence b: validated (first row, length); a malformed entry yields length 0
__device__ __forceinline__ void seq_extent(const int32_t* seq_offsets, int32_t b, int64_t n_rows,
                                           int64_t* base, int64_t* T, bool* bad) {
    const int64_t s = seq_offsets[b], e = seq_offsets[b + 1];
    if (s < 0 || e < s || e > n_rows) {
        *bad = true;
        *base = 0;
        *T = 0;
    } else {
        *base = s;
        *T = e - s;
    }
}

__device__ __forceinline__ int64_t chunk_bound(int64_t T, int32_t l_min) {
    if (T <= 0) return 0;
    return T < l_min ? 1 : T / l_min;
}

__global__ void partition_init_kernel(int32_t* status_word) { *status_word = 0; }

constexpr int kLdsTokens = 8192;   // sequences up to this length keep q and P in LDS
constexpr size_t kLdsBytes = sizeof(int64_t) * (kLdsTokens + 1) + sizeof(int32_t) * kLdsTokens;

// Quantise the scores of one sequence and scan them: q[t], P[t+1] = q[0] + .. + q[t], P[0] = 0.
__device__ void quantise_and_scan(const float* __restrict__ h, int64_t T, int32_t* q, int64_t* P,
                                  int64_t* wave_tot /*LDS[4]*/, bool* saw_nan) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int64_t carry = 0;
    for (int64_t t0 = 0; t0 < T; t0 += kThreads * kItems) {
        const int64_t idx0 = t0 + (int64_t)tid * kItems;
        int64_t local[kItems];
        int64_t sum = 0;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t t = idx0 + i;
            int32_t qv = 0;
            if (t < T) {
                qv = quantise_score(h[t], saw_nan);
                q[t] = qv;
            }
            sum += qv;
            local[i] = sum;
        }
        int64_t incl = sum;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int64_t v = shfl_up_i64(incl, off);
            if (lane >= off) incl += v;
        }
        __syncthreads();
        if (lane == 63) wave_tot[wave] = incl;
        __syncthreads();
        int64_t wave_prefix = 0, total = 0;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w < wave) wave_prefix += wave_tot[w];
            total += wave_tot[w];
        }
        const int64_t excl = carry + wave_prefix + incl - sum;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t t = idx0 + i;
            if (t < T) P[t + 1] = excl + local[i];
        }
        carry += total;
    }
    if (tid == 0) P[0] = 0;
}

// Boundary placement for one sequence by one wavefront: 64 candidate ends per step, a ballot picks
// the first admissible end at which a test fires.  Returns the number of chunks.
__device__ int32_t place_boundaries(const int32_t* q, const int64_t* P, int64_t base, int64_t T,
                                    int32_t l_min, int32_t l_max, int64_t theta_q, int64_t delta_q,
                                    const PartWs& ws, int64_t stage_off) {
    const int lane = threadIdx.x & 63;
    int32_t n_chunks = 0;
    if (T > 0 && T < l_min) {
        if (lane == 0 && stage_off < ws.stage_cap) {
            ws.st_start[stage_off] = (int32_t)base;
            ws.st_len[stage_off] = (int32_t)T;
            ws.st_sum[stage_off] = P[T];
        }
        return 1;
    }
    int64_t p = 0;
    while (p < T) {
        const int64_t e_hi = (p + l_max < T) ? p + l_max : T;
        int64_t e_star = (T - p <= l_max) ? T : ((p + l_max < T - l_min) ? p + l_max : T - l_min);
        const int64_t Pp = P[p];
        for (int64_t e0 = p + l_min; e0 <= e_hi; e0 += 64) {
            const int64_t e = e0 + lane;
            bool fire = false;
            if (e <= e_hi && (e <= T - l_min || e == T)) {
                if (e == T) {
                    fire = true;
                } else {
                    const int64_t n = e - p;
                    const int64_t S = P[e] - Pp;
                    const int64_t qe = q[e];
                    int64_t d = qe * n - S;
                    if (d < 0) d = -d;
                    fire = (S >= theta_q * n) || (qe >= theta_q) || (d > delta_q * n);
                }
            }
            const unsigned long long mask = __ballot(fire);
            if (mask) {
                e_star = e0 + (__ffsll(mask) - 1);
                break;
            }
        }
        const int64_t slot = stage_off + n_chunks;
        if (lane == 0 && slot < ws.stage_cap) {
            ws.st_start[slot] = (int32_t)(base + p);
            ws.st_len[slot] = (int32_t)(e_star - p);
            ws.st_sum[slot] = P[e_star] - Pp;
        }
        ++n_chunks;
        p = e_star;
    }
    return n_chunks;
}

__global__ void __launch_bounds__(kThreads)
partition_seq_kernel(const float* __restrict__ entropy, int64_t n_rows,
                     const int32_t* __restrict__ seq_offsets, int32_t n_seqs, int32_t l_min,
                     int32_t l_max, int64_t theta_q, int64_t delta_q, PartWs ws) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __shared__ int64_t red[4];
    __shared__ int64_t wave_tot[4];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int32_t b = blockIdx.x;
    bool bad = false, saw_nan = false;
    int64_t base, T;
    seq_extent(seq_offsets, b, n_rows, &base, &T, &bad);
    if (b == n_seqs - 1 && (int64_t)seq_offsets[n_seqs] != n_rows) bad = true;

    // staging offset: worst-case chunk count of the sequences before this one
    int64_t mine = 0;
    for (int32_t bb = tid; bb < b; bb += kThreads) {
        int64_t s0, t0;
        bool ignore = false;
        seq_extent(seq_offsets, bb, n_rows, &s0, &t0, &ignore);
        mine += chunk_bound(t0, l_min);
    }
    const int64_t stage_off = block_sum_i64(mine, red);

    // q and P of this sequence live in LDS when they fit (the boundary placement is a chain of
    // dependent look-ups, so their latency is the run time), else in the workspace
    const bool in_lds = T <= kLdsTokens;
    int32_t n_chunks;
    if (in_lds) {
        int64_t* P = reinterpret_cast<int64_t*>(lds_raw);
        int32_t* q = reinterpret_cast<int32_t*>(lds_raw + sizeof(int64_t) * (kLdsTokens + 1));
        quantise_and_scan(entropy + base, T, q, P, wave_tot, &saw_nan);
        __syncthreads();
        n_chunks = wave == 0 ? place_boundaries(q, P, base, T, l_min, l_max, theta_q, delta_q, ws, stage_off) : 0;
    } else {
        int64_t* P = ws.P + base + b;
        int32_t* q = ws.q + base;
        quantise_and_scan(entropy + base, T, q, P, wave_tot, &saw_nan);
        __syncthreads();   // P and q of this sequence are visible to the whole workgroup
        n_chunks = wave == 0 ? place_boundaries(q, P, base, T, l_min, l_max, theta_q, delta_q, ws, stage_off) : 0;
    }
    // status bits met in this sequence, combined over sequences by the compact kernel
    const int32_t nan_any = __syncthreads_or(saw_nan ? 1 : 0);
    const int32_t bad_any = __syncthreads_or(bad ? 1 : 0);
    if (tid == 0) {
        ws.seq_count[b] = n_chunks;
        ws.seq_stage[b] = (int32_t)stage_off;
        ws.seq_status[b] = (nan_any ? (int32_t)CWL_STATUS_NAN_SCORE : 0) | (bad_any ? (int32_t)CWL_STATUS_BAD_OFFSETS : 0);
    }
}

__global__ void __launch_bounds__(kThreads)
partition_compact_kernel(int32_t n_seqs, PartWs ws, int32_t* __restrict__ chunk_offsets,
                         int32_t* __restrict__ chunk_start, int32_t* __restrict__ chunk_len,
                         int64_t* __restrict__ chunk_sum, int32_t cap, int32_t* status_word) {
    __shared__ int64_t red[4];
    const int tid = threadIdx.x;
    const int32_t b = blockIdx.x;
    int64_t mine = 0;
    for (int32_t bb = tid; bb < b; bb += kThreads) mine += ws.seq_count[bb];
    const int64_t first = block_sum_i64(mine, red);
    const int32_t count = ws.seq_count[b];
    const int32_t stage = ws.seq_stage[b];
    if (tid == 0) {
        chunk_offsets[b] = (int32_t)first;
        if (b == n_seqs - 1) chunk_offsets[n_seqs] = (int32_t)(first + count);
    }
    if (b == n_seqs - 1) {
        // the last workgroup knows the total: it writes the status word (no atomics, no pre-clear)
        int32_t bits = 0;
        for (int32_t bb = tid; bb < n_seqs; bb += kThreads) bits |= ws.seq_status[bb];
        // __syncthreads_or tells whether any thread's value is non-zero: combine bit by bit
        const int32_t nan_any = __syncthreads_or(bits & (int32_t)CWL_STATUS_NAN_SCORE);
        const int32_t bad_any = __syncthreads_or(bits & (int32_t)CWL_STATUS_BAD_OFFSETS);
        if (tid == 0) {
            int32_t w = (nan_any ? (int32_t)CWL_STATUS_NAN_SCORE : 0) | (bad_any ? (int32_t)CWL_STATUS_BAD_OFFSETS : 0);
            if (first + count > cap) w |= (int32_t)CWL_STATUS_CAPACITY;
            *status_word = w;
        }
    }
    for (int32_t i = tid; i < count; i += kThreads) {
        const int64_t dst = first + i;
        if (dst < cap && (int64_t)stage + i < ws.stage_cap) {
            chunk_start[dst] = ws.st_start[stage + i];
            chunk_len[dst] = ws.st_len[stage + i];
            chunk_sum[dst] = ws.st_sum[stage + i];
        }
    }
}

struct Thresholds {
    int64_t tau_q[CWL_MAX_LADDER];
};

__global__ void select_ranks_kernel(const int64_t* __restrict__ chunk_sum,
                                    const int32_t* __restrict__ chunk_len,
                                    const int32_t* __restrict__ chunk_offsets, int32_t n_seqs,
                                    int32_t cap, Thresholds th, int32_t K,
                                    int32_t* __restrict__ rank_idx) {
    const int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    int64_t n = chunk_offsets[n_seqs];
    if (n > cap) n = cap;
    if (c >= n) return;
    const int64_t s = chunk_sum[c];
    const int64_t len = chunk_len[c];
    int32_t k = 0;
    for (int32_t j = 0; j < K - 1; ++j) k += (s >= th.tau_q[j] * len) ? 1 : 0;
    rank_idx[c] = k;
}

cwl_status check_params(const cwl_chunk_params* p) {
    if (!p) return CWL_ERR_NULL;
    if (p->l_min < 1 || p->l_max < p->l_min) return CWL_ERR_INVALID_ARG;
    if ((int64_t)p->l_max < 2 * (int64_t)p->l_min - 1) return CWL_ERR_INFEASIBLE;
    return CWL_OK;
}

}  // namespace

extern "C" size_t cwl_partition_workspace_bytes(int64_t n_rows, int32_t n_seqs,
                                                const cwl_chunk_params* p) {
    if (n_rows < 0 || n_seqs < 0 || check_params(p) != CWL_OK) return 0;
    return part_ws_layout(n_rows, n_seqs, p->l_min, nullptr, nullptr, nullptr);
}

extern "C" cwl_status cwl_partition_chunks(const float* entropy, int64_t n_rows,
                                           const int32_t* seq_offsets, int32_t n_seqs,
                                           const cwl_chunk_params* p, int32_t* chunk_offsets,
                                           int32_t* chunk_start, int32_t* chunk_len,
                                           int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    cwl_status st = check_params(p);
    if (st != CWL_OK) return st;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0 || cap < 0) return CWL_ERR_INVALID_ARG;
    if (!seq_offsets || !chunk_offsets || !status_word) return CWL_ERR_NULL;
    if (n_rows > 0 && !entropy) return CWL_ERR_NULL;
    if (cap > 0 && (!chunk_start || !chunk_len || !chunk_sum)) return CWL_ERR_NULL;
    if (!workspace) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return CWL_ERR_INVALID_ARG;
    PartWs ws;
    const size_t need = part_ws_layout(n_rows, n_seqs, p->l_min, workspace, &ws, nullptr);
    if (workspace_bytes < need) return CWL_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t theta_q = cwl::quantise_threshold(p->theta_hard);
    const int64_t delta_q = cwl::quantise_threshold(p->delta_dev);
    if (n_seqs == 0) {
        // no sequences: status 0, chunk_offsets[0] = 0
        partition_init_kernel<<<1, 1, 0, s>>>(status_word);
        CWL_RETURN_IF_LAUNCH_FAILED();
        partition_init_kernel<<<1, 1, 0, s>>>(chunk_offsets);
        CWL_RETURN_IF_LAUNCH_FAILED();
        return CWL_OK;
    }
    static bool attr_set = false;
    if (!attr_set) {
        if (hipFuncSetAttribute(reinterpret_cast<const void*>(partition_seq_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsBytes) != hipSuccess)
            return CWL_ERR_DEVICE;
        attr_set = true;
    }
    cwl::prof_begin(CWL_PROF_PARTITION, s);
    partition_seq_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), kLdsBytes, s>>>(
        entropy, n_rows, seq_offsets, n_seqs, p->l_min, p->l_max, theta_q, delta_q, ws);
    CWL_RETURN_IF_LAUNCH_FAILED();
    partition_compact_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), 0, s>>>(
        n_seqs, ws, chunk_offsets, chunk_start, chunk_len, chunk_sum, cap, status_word);
    cwl::prof_end(CWL_PROF_PARTITION, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}

extern "C" cwl_status cwl_select_ranks(const int64_t* chunk_sum, const int32_t* chunk_len,
                                       const int32_t* chunk_offsets, int32_t n_seqs, int32_t cap,
                                       const float* thresholds, int32_t K, int32_t* rank_idx,
                                       void* stream) {
    if (K < 1 || K > CWL_MAX_LADDER || n_seqs < 0 || cap < 0) return CWL_ERR_INVALID_ARG;
    if (K > 1 && !thresholds) return CWL_ERR_NULL;
    Thresholds th = {};
    for (int32_t j = 0; j < K - 1; ++j) {
        if (thresholds[j] != thresholds[j]) return CWL_ERR_INVALID_ARG;
        if (j > 0 && thresholds[j] < thresholds[j - 1]) return CWL_ERR_INVALID_ARG;
        th.tau_q[j] = cwl::quantise_threshold(thresholds[j]);
    }
    if (cap == 0) return CWL_OK;
    if (!chunk_sum || !chunk_len || !chunk_offsets || !rank_idx) return CWL_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const unsigned blocks = (unsigned)((cap + 255) / 256);
    cwl::prof_begin(CWL_PROF_SELECT, s);
    select_ranks_kernel<<<dim3(blocks), dim3(256), 0, s>>>(chunk_sum, chunk_len, chunk_offsets,
                                                           n_seqs, cap, th, K, rank_idx);
    cwl::prof_end(CWL_PROF_SELECT, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
