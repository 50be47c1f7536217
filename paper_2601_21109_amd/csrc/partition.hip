// cwl_partition_chunks and cwl_select_ranks: the adaptive chunker and the rung selector
// (Sec. III-B / III-C and IV-B / IV-C of arxiv 2601.21109).  Integer work after the one fp32
// quantisation of the scores.
//
// The chunker is a greedy chain: a chunk starts where the previous one ended, and its end is the
// first admissible position at which a test fires (chunk_end below; one wavefront tests 64
// candidate ends per step).  Two paths produce the same staged chunks:
//
// Short sequences (batch average up to 4096 tokens): one kernel, one workgroup per sequence:
// scores quantised and scanned into LDS (the workspace beyond 8192 tokens), then wavefront 0 walks
// the chain, a few LDS look-ups per chunk.  A 2048-token sequence has ~30 chunks: ~20 us.
//
// Long sequences: the chain has hundreds of dependent steps and one wavefront per sequence leaves
// the chip idle.  The end e = next(p) is a pure function of the start p (given the quantised
// scores and their prefix sums), so the path is
//   1. scan    (one workgroup per sequence): quantise the scores, inclusive prefix sums;
//   2. next    (64 starts per workgroup, all tokens of the batch): next(p) for EVERY position p,
//              one wavefront per start testing 64 candidate ends per step out of an LDS copy of
//              the window of scores it can reach;
//   3. walk    (one workgroup per sequence): next[] of the sequence into LDS, one lane follows
//              the chain (an LDS look-up per chunk), all lanes then form lengths and sums;
//   4. compact (one workgroup per sequence): per-sequence counts into CSR offsets, staged chunks
//              to their final place, status word.
// Most of step 2 is wasted (one position in L-bar is a chunk start), but it is a few million
// integer tests spread over the whole chip, against a dependent chain of hundreds of look-ups
// (32768 tokens in one sequence: 460 us on the first path, ~140 us on this one).  Both paths end
// with the compact kernel.
// Chunks are staged at a per-sequence offset = the worst-case chunk count of the preceding
// sequences.  (Well-formed offsets never overflow the staging area; writes are bounds-checked.)
#include "partition_seq.h"

namespace {

using cwl::quantise_score;
using cwl::seq_extent;
using cwl::shfl_up_i64;
using cwl::wave_sum_i64;
using namespace cwl::part;       // the short-sequence chunker's device code and the workspace layout

constexpr int kBig = 1024;       // scan and walk kernels: one workgroup per sequence, so a wide one
constexpr int kStarts = 32;      // start positions per workgroup of the next kernel
constexpr int kWalkLds = 36864; // longest sequence whose next[] is walked out of LDS (144 KiB)

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
    size_t o_P = take(sizeof(int64_t) * (size_t)(n_rows + 1));
    size_t o_sum = take(sizeof(int64_t) * (size_t)stage_cap);
    size_t o_q = take(sizeof(int32_t) * (size_t)(n_rows + 1));
    size_t o_next = take(sizeof(int32_t) * (size_t)(n_rows + 1));
    size_t o_start = take(sizeof(int32_t) * (size_t)stage_cap);
    size_t o_len = take(sizeof(int32_t) * (size_t)stage_cap);
    size_t o_cnt = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    size_t o_stage = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    size_t o_status = take(sizeof(int32_t) * (size_t)(n_seqs + 1));
    if (ws) {
        ws->Pin = reinterpret_cast<int64_t*>(b + o_P);
        ws->st_sum = reinterpret_cast<int64_t*>(b + o_sum);
        ws->q = reinterpret_cast<int32_t*>(b + o_q);
        ws->next = reinterpret_cast<int32_t*>(b + o_next);
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

__global__ void partition_init_kernel(int32_t* status_word) { *status_word = 0; }

// ---- 1. scan ----
__global__ void __launch_bounds__(kBig)
partition_scan_kernel(const float* __restrict__ entropy, int64_t n_rows,
                      const int32_t* __restrict__ seq_offsets, int32_t n_seqs, int32_t l_min,
                      PartWs ws) {
    __shared__ int64_t red[kBig / 64];
    __shared__ int64_t wave_tot[kBig / 64];
    const int tid = threadIdx.x;
    const int32_t b = blockIdx.x;
    bool bad = false, saw_nan = false;
    int64_t base, T;
    seq_extent(seq_offsets, b, n_rows, &base, &T, &bad);
    if (b == n_seqs - 1 && (int64_t)seq_offsets[n_seqs] != n_rows) bad = true;

    // staging offset: worst-case chunk count of the sequences before this one
    int64_t mine = 0;
    for (int32_t bb = tid; bb < b; bb += kBig) {
        int64_t s0, t0;
        bool ignore = false;
        seq_extent(seq_offsets, bb, n_rows, &s0, &t0, &ignore);
        mine += chunk_bound(t0, l_min);
    }
    const int64_t stage_off = block_sum_i64(mine, red);

    quantise_and_scan(entropy + base, T, ws.q + base, ws.Pin + base, wave_tot, &saw_nan);

    // status bits met in this sequence, combined over sequences by the compact kernel
    const int32_t nan_any = __syncthreads_or(saw_nan ? 1 : 0);
    const int32_t bad_any = __syncthreads_or(bad ? 1 : 0);
    if (tid == 0) {
        ws.seq_stage[b] = (int32_t)stage_off;
        ws.seq_status[b] = (nan_any ? (int32_t)CWL_STATUS_NAN_SCORE : 0) | (bad_any ? (int32_t)CWL_STATUS_BAD_OFFSETS : 0);
    }
}

// ---- 2. next ----
// Workgroup g owns the global rows [32 g, 32 g + 32) as chunk starts, 8 per wavefront.  When the
// window of rows those starts can reach (32 + l_max + 1) fits the LDS given to the kernel, it is
// copied there first (the copy ignores sequence borders; a start only looks inside its own
// sequence).  Rows outside every well-formed sequence get no entry: the walk never reads them.
__global__ void __launch_bounds__(kThreads)
partition_next_kernel(int64_t n_rows, const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                      int32_t l_min, int32_t l_max, int64_t theta_q, int64_t delta_q, PartWs ws,
                      int32_t lds_rows) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    const int tid = threadIdx.x, wave = tid >> 6;
    const int64_t g0 = (int64_t)blockIdx.x * kStarts;
    int64_t win = (int64_t)kStarts + l_max + 1;
    if (g0 + win > n_rows) win = n_rows - g0;
    const bool in_lds = win <= lds_rows;
    int64_t* Pl = reinterpret_cast<int64_t*>(lds_raw);
    int32_t* ql = reinterpret_cast<int32_t*>(lds_raw + sizeof(int64_t) * (size_t)lds_rows);
    if (in_lds) {
        for (int64_t i = tid; i < win; i += kThreads) {
            Pl[i] = ws.Pin[g0 + i];
            ql[i] = ws.q[g0 + i];
        }
        __syncthreads();
    }
    // the sequence holding row g0: the last b with seq_offsets[b] <= g0 (offsets ascend when well
    // formed); all threads look, the largest hit wins
    __shared__ int32_t b0_sh;
    if (tid == 0) b0_sh = 0;
    __syncthreads();
    for (int32_t bb = tid; bb < n_seqs; bb += kThreads)
        if ((int64_t)seq_offsets[bb] <= g0) atomicMax(&b0_sh, bb);
    __syncthreads();
    int32_t b = b0_sh;
    for (int i = 0; i < kStarts / 4; ++i) {
        const int64_t t = g0 + wave * (kStarts / 4) + i;          // wave-uniform
        if (t >= n_rows) break;
        while (b + 1 < n_seqs && (int64_t)seq_offsets[b + 1] <= t) ++b;
        int64_t base, T;
        bool bad = false;
        seq_extent(seq_offsets, b, n_rows, &base, &T, &bad);
        if (bad || t < base || t >= base + T) continue;
        int64_t e;
        if (in_lds) e = chunk_end<int64_t>(ql, Pl, g0 - base, t - base, T, l_min, l_max, theta_q, delta_q);
        else e = chunk_end<int64_t>(ws.q + base, ws.Pin + base, (int64_t)0, t - base, T, l_min, l_max, theta_q, delta_q);
        if ((tid & 63) == 0) ws.next[t] = (int32_t)(base + e);
    }
}

// ---- 3. walk ----
__global__ void __launch_bounds__(kBig)
partition_walk_kernel(int64_t n_rows, const int32_t* __restrict__ seq_offsets, int32_t n_seqs, PartWs ws) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __shared__ int32_t n_sh;
    const int tid = threadIdx.x;
    const int32_t b = blockIdx.x;
    int64_t base, T;
    bool bad = false;
    seq_extent(seq_offsets, b, n_rows, &base, &T, &bad);
    const int64_t stage_off = ws.seq_stage[b];
    int32_t* nx = reinterpret_cast<int32_t*>(lds_raw);
    const bool in_lds = T <= kWalkLds;
    if (in_lds) {
#pragma unroll 4
        for (int64_t i = tid; i < T; i += kBig) nx[i] = ws.next[base + i];
    }
    __syncthreads();
    // One lane follows the chain.  In LDS the starts are written over the entries already passed
    // (the n-th chunk starts at local position >= n, and that entry has been read by then).
    if (tid == 0) {
        int32_t n = 0;
        int64_t p = base;
        const int64_t end = base + T;
        if (in_lds) {
            while (p < end) {
                const int64_t e = nx[p - base];
                nx[n++] = (int32_t)p;
                p = (e > p && e <= end) ? e : end;      // entries are in (p, end] by construction
            }
        } else {
            while (p < end) {
                const int64_t e = ws.next[p];
                if (stage_off + n < ws.stage_cap) ws.st_start[stage_off + n] = (int32_t)p;
                ++n;
                p = (e > p && e <= end) ? e : end;
            }
        }
        n_sh = n;
        ws.seq_count[b] = n;
    }
    __syncthreads();
    const int32_t n = n_sh;
    // lengths and score sums of the chunks, all lanes
    for (int32_t i = tid; i < n; i += kBig) {
        const int64_t slot = stage_off + i;
        if (slot >= ws.stage_cap) continue;
        int64_t s, e;
        if (in_lds) {
            s = nx[i];
            e = (i + 1 < n) ? nx[i + 1] : base + T;
        } else {
            // written by lane 0 of this workgroup before the barrier; read back past the vector cache
            s = __hip_atomic_load(&ws.st_start[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            e = (i + 1 < n) ? __hip_atomic_load(&ws.st_start[slot + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                            : base + T;
        }
        ws.st_start[slot] = (int32_t)s;
        ws.st_len[slot] = (int32_t)(e - s);
        ws.st_sum[slot] = ws.Pin[e - 1] - ws.Pin[s] + ws.q[s];
    }
}

// ---- short sequences: the body of partition_seq.h as a kernel of its own ----
__global__ void __launch_bounds__(kThreads) partition_seq_kernel(SeqJob job) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    partition_seq_body(job, (int32_t)blockIdx.x, lds_raw);
}

// ---- 4. compact (and, when rank_idx is given, the selector's rule on every chunk it places) ----
__global__ void __launch_bounds__(kThreads)
partition_compact_kernel(int32_t n_seqs, PartWs ws, int32_t* __restrict__ chunk_offsets,
                         int32_t* __restrict__ chunk_start, int32_t* __restrict__ chunk_len,
                         int64_t* __restrict__ chunk_sum, int32_t cap, int32_t* status_word,
                         cwl::TauTable th, int32_t K, int32_t* __restrict__ rank_idx /* may be NULL */) {
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
            const int64_t s = ws.st_sum[stage + i];
            const int32_t len = ws.st_len[stage + i];
            chunk_start[dst] = ws.st_start[stage + i];
            chunk_len[dst] = len;
            chunk_sum[dst] = s;
            if (rank_idx) {
                // Sec. III-C / IV-C: rung = number of thresholds the chunk's mean reaches (a mean on a
                // threshold goes up), as an integer test on the sum
                int32_t k = 0;
                for (int32_t j = 0; j < K - 1; ++j) k += (s >= th.tau_q[j] * (int64_t)len) ? 1 : 0;
                rank_idx[dst] = k;
            }
        }
    }
}

__global__ void select_ranks_kernel(const int64_t* __restrict__ chunk_sum,
                                    const int32_t* __restrict__ chunk_len,
                                    const int32_t* __restrict__ chunk_offsets, int32_t n_seqs,
                                    int32_t cap, cwl::TauTable th, int32_t K,
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

// What cwl_schedule_chunks adds to the chunker's call: the selector's table and the first phase of
// the two-phase layer (NULL descriptor: none).
struct ScheduleExtras {
    const cwl::TauTable* th;
    int32_t K;
    int32_t* rank_idx;
    const cwl_linear_desc* shrink;
    const void* x;
    const void* packed;
    void* u;
};

// avg_len: what the host knows of the sequence lengths (their average); it picks the path
cwl_status partition_impl(const float* entropy, int64_t n_rows, const int32_t* seq_offsets, int32_t n_seqs,
                          const cwl_chunk_params* p, int32_t* chunk_offsets, int32_t* chunk_start,
                          int32_t* chunk_len, int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                          void* workspace, size_t workspace_bytes, void* stream, int64_t avg_len,
                          const ScheduleExtras* ex) {
    cwl_status st = cwl::check_chunk_params(p);
    if (st != CWL_OK) return st;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0 || cap < 0) return CWL_ERR_INVALID_ARG;
    if (!seq_offsets || !chunk_offsets || !status_word) return CWL_ERR_NULL;
    if (n_rows > 0 && !entropy) return CWL_ERR_NULL;
    if (cap > 0 && (!chunk_start || !chunk_len || !chunk_sum)) return CWL_ERR_NULL;
    if (ex && cap > 0 && !ex->rank_idx) return CWL_ERR_NULL;
    if (!workspace) return CWL_ERR_NULL;
    if (reinterpret_cast<uintptr_t>(workspace) % 256) return CWL_ERR_INVALID_ARG;
    PartWs ws;
    const size_t need = part_ws_layout(n_rows, n_seqs, p->l_min, workspace, &ws, nullptr);
    if (workspace_bytes < need) return CWL_ERR_CAPACITY;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t theta_q = cwl::quantise_threshold(p->theta_hard);
    const int64_t delta_q = cwl::quantise_threshold(p->delta_dev);
    const bool with_shrink = ex && ex->shrink && ex->shrink->n_rows > 0;
    if (n_seqs == 0) {
        // no sequences: status 0, chunk_offsets[0] = 0
        partition_init_kernel<<<1, 1, 0, s>>>(status_word);
        CWL_RETURN_IF_LAUNCH_FAILED();
        partition_init_kernel<<<1, 1, 0, s>>>(chunk_offsets);
        CWL_RETURN_IF_LAUNCH_FAILED();
        if (with_shrink) return cwl::run_shrink_phase(ex->shrink, ex->x, static_cast<const char*>(ex->packed),
                                                      static_cast<float*>(ex->u), s);
        return CWL_OK;
    }
    // LDS of the next kernel: a window of kStarts + l_max + 1 rows (12 bytes each), if that fits a CU
    constexpr size_t kLdsMax = 144 * 1024;
    const int64_t win = (int64_t)kStarts + p->l_max + 1;
    const int32_t lds_rows = (win * 12 <= (int64_t)kLdsMax) ? (int32_t)win : 0;
    const size_t next_lds = (size_t)lds_rows * 12;
    const size_t walk_lds = (size_t)kWalkLds * sizeof(int32_t);
    static cwl::PerDeviceFlag next_set, walk_set, seq_set;
    if (cwl::ensure_dynamic_lds(reinterpret_cast<const void*>(partition_next_kernel), (int)kLdsMax, next_set) != CWL_OK ||
        cwl::ensure_dynamic_lds(reinterpret_cast<const void*>(partition_walk_kernel), (int)walk_lds, walk_set) != CWL_OK ||
        cwl::ensure_dynamic_lds(reinterpret_cast<const void*>(partition_seq_kernel), (int)kSeqLdsBytes, seq_set) != CWL_OK)
        return CWL_ERR_DEVICE;
    // which path: the host knows only the batch average of the sequence lengths
    const bool long_sequences = avg_len > 4096;
    SeqJob job = {};
    job.entropy = entropy;
    job.n_rows = n_rows;
    job.seq_offsets = seq_offsets;
    job.n_seqs = n_seqs;
    job.l_min = p->l_min;
    job.l_max = p->l_max;
    job.theta_q = theta_q;
    job.delta_q = delta_q;
    job.ws = ws;
    job.lds_tokens = kLdsTokens;
    bool shrink_done = false;
    cwl::prof_begin(CWL_PROF_PARTITION, s);
    if (!long_sequences) {
        // the chunk walk keeps one wavefront per sequence busy: the layer's first product, which needs
        // nothing from it and all of the chip's memory bandwidth, shares its launch where it can
        if (with_shrink) {
            const cwl_status fs = cwl::launch_seq_with_shrink(job, ex->shrink, ex->x, static_cast<const char*>(ex->packed),
                                                              static_cast<float*>(ex->u), s);
            if (fs == CWL_OK) shrink_done = true;
            else if (fs != CWL_ERR_UNSUPPORTED) return fs;
        }
        if (!shrink_done) {
            partition_seq_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), kSeqLdsBytes, s>>>(job);
            CWL_RETURN_IF_LAUNCH_FAILED();
        }
    } else {
        partition_scan_kernel<<<dim3((unsigned)n_seqs), dim3(kBig), 0, s>>>(
            entropy, n_rows, seq_offsets, n_seqs, p->l_min, ws);
        CWL_RETURN_IF_LAUNCH_FAILED();
        const unsigned blocks = (unsigned)((n_rows + kStarts - 1) / kStarts);
        partition_next_kernel<<<dim3(blocks), dim3(kThreads), next_lds, s>>>(
            n_rows, seq_offsets, n_seqs, p->l_min, p->l_max, theta_q, delta_q, ws, lds_rows);
        CWL_RETURN_IF_LAUNCH_FAILED();
        partition_walk_kernel<<<dim3((unsigned)n_seqs), dim3(kBig), walk_lds, s>>>(n_rows, seq_offsets, n_seqs, ws);
        CWL_RETURN_IF_LAUNCH_FAILED();
    }
    cwl::TauTable none = {};
    partition_compact_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), 0, s>>>(
        n_seqs, ws, chunk_offsets, chunk_start, chunk_len, chunk_sum, cap, status_word, ex ? *ex->th : none,
        ex ? ex->K : 0, ex ? ex->rank_idx : nullptr);
    cwl::prof_end(CWL_PROF_PARTITION, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    if (with_shrink && !shrink_done)
        return cwl::run_shrink_phase(ex->shrink, ex->x, static_cast<const char*>(ex->packed), static_cast<float*>(ex->u), s);
    return CWL_OK;
}

}  // namespace

extern "C" size_t cwl_partition_workspace_bytes(int64_t n_rows, int32_t n_seqs,
                                                const cwl_chunk_params* p) {
    if (n_rows < 0 || n_seqs < 0 || cwl::check_chunk_params(p) != CWL_OK) return 0;
    return part_ws_layout(n_rows, n_seqs, p->l_min, nullptr, nullptr, nullptr);
}

cwl_status cwl::partition_chunks_avg_len(const float* entropy, int64_t n_rows,
                                         const int32_t* seq_offsets, int32_t n_seqs,
                                         const cwl_chunk_params* p, int32_t* chunk_offsets,
                                         int32_t* chunk_start, int32_t* chunk_len,
                                         int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                         void* workspace, size_t workspace_bytes, void* stream,
                                         int64_t avg_len) {
    return partition_impl(entropy, n_rows, seq_offsets, n_seqs, p, chunk_offsets, chunk_start, chunk_len, chunk_sum,
                          cap, status_word, workspace, workspace_bytes, stream, avg_len, nullptr);
}

extern "C" cwl_status cwl_partition_chunks(const float* entropy, int64_t n_rows,
                                           const int32_t* seq_offsets, int32_t n_seqs,
                                           const cwl_chunk_params* p, int32_t* chunk_offsets,
                                           int32_t* chunk_start, int32_t* chunk_len,
                                           int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                           void* workspace, size_t workspace_bytes, void* stream) {
    return cwl::partition_chunks_avg_len(entropy, n_rows, seq_offsets, n_seqs, p, chunk_offsets, chunk_start,
                                         chunk_len, chunk_sum, cap, status_word, workspace, workspace_bytes,
                                         stream, n_seqs > 0 ? n_rows / n_seqs : 0);
}

extern "C" cwl_status cwl_schedule_chunks(const float* entropy, int64_t n_rows, const int32_t* seq_offsets,
                                          int32_t n_seqs, const cwl_chunk_params* p, const float* thresholds,
                                          int32_t K, int32_t* chunk_offsets, int32_t* chunk_start,
                                          int32_t* chunk_len, int64_t* chunk_sum, int32_t* rank_idx, int32_t cap,
                                          int32_t* status_word, void* workspace, size_t workspace_bytes,
                                          const cwl_linear_desc* shrink, const void* x, const void* packed,
                                          void* u, size_t u_bytes, void* stream) {
    if (K < 1 || K > CWL_MAX_LADDER) return CWL_ERR_INVALID_ARG;
    if (K > 1 && !thresholds) return CWL_ERR_NULL;
    cwl::TauTable th;
    if (cwl::fill_tau_table(thresholds, K, &th) != CWL_OK) return CWL_ERR_INVALID_ARG;
    if (shrink) {
        const cwl_status cs = cwl::check_shrink_phase(shrink, x, packed, u, u_bytes);
        if (cs != CWL_OK) return cs;
    }
    ScheduleExtras ex = {&th, K, rank_idx, shrink, x, packed, u};
    return partition_impl(entropy, n_rows, seq_offsets, n_seqs, p, chunk_offsets, chunk_start, chunk_len, chunk_sum,
                          cap, status_word, workspace, workspace_bytes, stream, n_seqs > 0 ? n_rows / n_seqs : 0, &ex);
}

extern "C" cwl_status cwl_select_ranks(const int64_t* chunk_sum, const int32_t* chunk_len,
                                       const int32_t* chunk_offsets, int32_t n_seqs, int32_t cap,
                                       const float* thresholds, int32_t K, int32_t* rank_idx,
                                       void* stream) {
    if (K < 1 || K > CWL_MAX_LADDER || n_seqs < 0 || cap < 0) return CWL_ERR_INVALID_ARG;
    if (K > 1 && !thresholds) return CWL_ERR_NULL;
    cwl::TauTable th;
    if (cwl::fill_tau_table(thresholds, K, &th) != CWL_OK) return CWL_ERR_INVALID_ARG;
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
