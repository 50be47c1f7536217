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
#include "common.h"

namespace {

using cwl::quantise_score;
using cwl::seq_extent;
using cwl::shfl_up_i64;
using cwl::wave_sum_i64;

constexpr int kThreads = 256;    // compact and next kernels
constexpr int kBig = 1024;       // scan and walk kernels: one workgroup per sequence, so a wide one
constexpr int kItems = 8;        // tokens per thread per scan pass
constexpr int kStarts = 32;      // start positions per workgroup of the next kernel
constexpr int kWalkLds = 36864; // longest sequence whose next[] is walked out of LDS (144 KiB)

struct PartWs {             // layout of the workspace
    int32_t* q;             // [n_rows]  quantised scores
    int64_t* Pin;           // [n_rows]  inclusive prefix sums of q inside each sequence
    int32_t* next;          // [n_rows]  end (global row index, exclusive) of a chunk starting at each row
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

// sum over the block of one int64 per thread; every thread gets the result
__device__ int64_t block_sum_i64(int64_t v, int64_t* smem /*[waves]*/) {
    v = wave_sum_i64(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) smem[threadIdx.x >> 6] = v;
    __syncthreads();
    int64_t tot = 0;
    for (unsigned w = 0; w < blockDim.x / 64; ++w) tot += smem[w];
    return tot;
}

__device__ __forceinline__ int64_t chunk_bound(int64_t T, int32_t l_min) {
    if (T <= 0) return 0;
    return T < l_min ? 1 : T / l_min;
}

__global__ void partition_init_kernel(int32_t* status_word) { *status_word = 0; }

// Quantise the scores of one sequence and scan them: q[t], Pin[t] = q[0] + .. + q[t].
__device__ __forceinline__ void quantise_and_scan(const float* __restrict__ h, int64_t T, int32_t* q, int64_t* Pin,
                                  int64_t* wave_tot /*LDS[waves]*/, bool* saw_nan) {
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_waves = (int)blockDim.x / 64;
    int64_t carry = 0;
    for (int64_t t0 = 0; t0 < T; t0 += (int64_t)blockDim.x * kItems) {
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
        for (int w = 0; w < n_waves; ++w) {
            if (w < wave) wave_prefix += wave_tot[w];
            total += wave_tot[w];
        }
        const int64_t excl = carry + wave_prefix + incl - sum;
#pragma unroll
        for (int i = 0; i < kItems; ++i) {
            const int64_t t = idx0 + i;
            if (t < T) Pin[t] = excl + local[i];
        }
        carry += total;
    }
}

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
// End of the chunk that would start at local position p of a sequence of length T (Sec. III-B):
// candidates e = p + l_min .. min(p + l_max, T) that leave either nothing or at least l_min tokens
// behind them; the first one at which the chunk's mean reaches theta, the token after it is hard,
// or that token deviates from the chunk mean by more than delta; else the longest admissible
// end.  q and Pin are indexed by local position (pointers already at the sequence, or at an LDS
// copy of a window of it shifted by `shift`).  One wavefront, 64 candidates per step.
// (IT: int64_t, or int32_t where positions are known to fit -- half the integer instructions in the
// chain walk, whose latency is the run time of the short-sequence kernel)
template <typename IT>
__device__ __forceinline__ IT chunk_end(const int32_t* q, const int64_t* Pin, IT shift, IT p, IT T,
                             int32_t l_min, int32_t l_max, int64_t theta_q, int64_t delta_q) {
    const int lane = threadIdx.x & 63;
    const int32_t theta32 = (int32_t)theta_q, delta32 = (int32_t)delta_q;
    const IT e_hi = (p + l_max < T) ? p + l_max : T;
    IT e_star = (T - p <= l_max) ? T : ((p + l_max < T - l_min) ? p + l_max : T - l_min);
    const int64_t Pex_p = Pin[p - shift] - q[p - shift];          // sum of the tokens before p
    for (IT e0 = p + l_min; e0 <= e_hi; e0 += 64) {
        const IT e = e0 + lane;
        bool fire = false;
        if (e <= e_hi && (e <= T - l_min || e == T)) {
            if (e == T) {
                fire = true;
            } else {
                // scores, thresholds (<= 2^21) and lengths fit 32 bits: 32 x 32 -> 64-bit products
                const int32_t n = (int32_t)(e - p);
                const int64_t S = Pin[e - 1 - shift] - Pex_p;
                const int32_t qe = q[e - shift];
                int64_t d = (int64_t)qe * n - S;
                if (d < 0) d = -d;
                fire = (S >= (int64_t)theta32 * n) || (qe >= theta32) || (d > (int64_t)delta32 * n);
            }
        }
        const unsigned long long mask = __ballot(fire);
        if (mask) {
            e_star = e0 + (__ffsll(mask) - 1);
            break;
        }
    }
    return e_star;
}

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

// ---- short sequences: scan and chain walk in one kernel ----
constexpr int kLdsTokens = 8192;   // sequences up to this length keep q and Pin in LDS
constexpr size_t kSeqLdsBytes = (sizeof(int64_t) + 2 * sizeof(int32_t)) * kLdsTokens;   // Pin, q, chunk starts

__global__ void __launch_bounds__(kThreads)
partition_seq_kernel(const float* __restrict__ entropy, int64_t n_rows,
                     const int32_t* __restrict__ seq_offsets, int32_t n_seqs, int32_t l_min,
                     int32_t l_max, int64_t theta_q, int64_t delta_q, PartWs ws) {
    extern __shared__ __attribute__((aligned(16))) char lds_raw[];
    __shared__ int64_t red[kThreads / 64];
    __shared__ int64_t wave_tot[kThreads / 64];
    __shared__ int32_t n_sh;
    const int tid = threadIdx.x, wave = tid >> 6;
    const int32_t b = blockIdx.x;
    bool bad = false, saw_nan = false;
    int64_t base, T;
    seq_extent(seq_offsets, b, n_rows, &base, &T, &bad);
    if (b == n_seqs - 1 && (int64_t)seq_offsets[n_seqs] != n_rows) bad = true;

    int64_t mine = 0;
    for (int32_t bb = tid; bb < b; bb += kThreads) {
        int64_t s0, t0;
        bool ignore = false;
        seq_extent(seq_offsets, bb, n_rows, &s0, &t0, &ignore);
        mine += chunk_bound(t0, l_min);
    }
    const int64_t stage_off = block_sum_i64(mine, red);

    // q and Pin of this sequence live in LDS when they fit (the chain walk is a series of dependent
    // look-ups, so their latency is the run time), else in the workspace.  Two instantiations, so
    // that the LDS one is compiled to LDS instructions rather than to generic-address ones.
    int32_t n_chunks = 0;
    // `starts`: LDS array for the chunk starts (then the chunk records are written by all threads after
    // the walk, and the walk itself issues no global stores), or NULL: lane 0 writes every record as it goes
    auto run = [&](auto it_tag, int32_t* q, int64_t* Pin, int32_t* starts) {
        using IT = decltype(it_tag);                        // position type of the walk
        quantise_and_scan(entropy + base, T, q, Pin, wave_tot, &saw_nan);
        __syncthreads();       // q and Pin of the sequence are visible to the whole workgroup
        if (wave == 0) {
            const IT Tw = (IT)T;
            // a chunk cannot be longer than the sequence: with l_max cut to T the 32-bit sums below cannot overflow
            const int32_t l_max_w = (int64_t)l_max > T ? (int32_t)T : l_max;
            IT p = 0;
            while (p < Tw) {
                const IT e = chunk_end<IT>(q, Pin, (IT)0, p, Tw, l_min, l_max_w, theta_q, delta_q);
                if ((tid & 63) == 0) {
                    if (starts) {
                        starts[n_chunks] = (int32_t)p;
                    } else {
                        const int64_t slot = stage_off + n_chunks;
                        if (slot < ws.stage_cap) {
                            ws.st_start[slot] = (int32_t)(base + p);
                            ws.st_len[slot] = (int32_t)(e - p);
                            ws.st_sum[slot] = Pin[e - 1] - Pin[p] + q[p];
                        }
                    }
                }
                ++n_chunks;
                p = e;
            }
            if (starts && (tid & 63) == 0) n_sh = n_chunks;
        }
        if (starts) {
            __syncthreads();
            const int32_t n = n_sh;
            for (int32_t c = tid; c < n; c += kThreads) {
                const int32_t p0 = starts[c];
                const int32_t e0 = (c + 1 < n) ? starts[c + 1] : (int32_t)T;
                const int64_t slot = stage_off + c;
                if (slot < ws.stage_cap) {
                    ws.st_start[slot] = (int32_t)(base + p0);
                    ws.st_len[slot] = e0 - p0;
                    ws.st_sum[slot] = Pin[e0 - 1] - Pin[p0] + q[p0];
                }
            }
            n_chunks = n;
        }
    };
    if (T <= kLdsTokens)
        run(int32_t{0}, reinterpret_cast<int32_t*>(lds_raw + sizeof(int64_t) * kLdsTokens),
            reinterpret_cast<int64_t*>(lds_raw),
            reinterpret_cast<int32_t*>(lds_raw + (sizeof(int64_t) + sizeof(int32_t)) * kLdsTokens));
    else
        run(int64_t{0}, ws.q + base, ws.Pin + base, nullptr);
    const int32_t nan_any = __syncthreads_or(saw_nan ? 1 : 0);
    const int32_t bad_any = __syncthreads_or(bad ? 1 : 0);
    if (tid == 0) {
        ws.seq_count[b] = n_chunks;
        ws.seq_stage[b] = (int32_t)stage_off;
        ws.seq_status[b] = (nan_any ? (int32_t)CWL_STATUS_NAN_SCORE : 0) | (bad_any ? (int32_t)CWL_STATUS_BAD_OFFSETS : 0);
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

// ---- 4. compact ----
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

}  // namespace

extern "C" size_t cwl_partition_workspace_bytes(int64_t n_rows, int32_t n_seqs,
                                                const cwl_chunk_params* p) {
    if (n_rows < 0 || n_seqs < 0 || cwl::check_chunk_params(p) != CWL_OK) return 0;
    return part_ws_layout(n_rows, n_seqs, p->l_min, nullptr, nullptr, nullptr);
}

// avg_len: what the host knows of the sequence lengths (their average); it picks the path
cwl_status cwl::partition_chunks_avg_len(const float* entropy, int64_t n_rows,
                                         const int32_t* seq_offsets, int32_t n_seqs,
                                         const cwl_chunk_params* p, int32_t* chunk_offsets,
                                         int32_t* chunk_start, int32_t* chunk_len,
                                         int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                         void* workspace, size_t workspace_bytes, void* stream,
                                         int64_t avg_len) {
    cwl_status st = cwl::check_chunk_params(p);
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
    // LDS of the next kernel: a window of kStarts + l_max + 1 rows (12 bytes each), if that fits a CU
    constexpr size_t kLdsMax = 144 * 1024;
    const int64_t win = (int64_t)kStarts + p->l_max + 1;
    const int32_t lds_rows = (win * 12 <= (int64_t)kLdsMax) ? (int32_t)win : 0;
    const size_t next_lds = (size_t)lds_rows * 12;
    const size_t walk_lds = (size_t)kWalkLds * sizeof(int32_t);
    static PerDeviceFlag next_set, walk_set, seq_set;
    if (ensure_dynamic_lds(reinterpret_cast<const void*>(partition_next_kernel), (int)kLdsMax, next_set) != CWL_OK ||
        ensure_dynamic_lds(reinterpret_cast<const void*>(partition_walk_kernel), (int)walk_lds, walk_set) != CWL_OK ||
        ensure_dynamic_lds(reinterpret_cast<const void*>(partition_seq_kernel), (int)kSeqLdsBytes, seq_set) != CWL_OK)
        return CWL_ERR_DEVICE;
    // which path: the host knows only the batch average of the sequence lengths
    const bool long_sequences = avg_len > 4096;
    cwl::prof_begin(CWL_PROF_PARTITION, s);
    if (!long_sequences) {
        partition_seq_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), kSeqLdsBytes, s>>>(
            entropy, n_rows, seq_offsets, n_seqs, p->l_min, p->l_max, theta_q, delta_q, ws);
        CWL_RETURN_IF_LAUNCH_FAILED();
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
    partition_compact_kernel<<<dim3((unsigned)n_seqs), dim3(kThreads), 0, s>>>(
        n_seqs, ws, chunk_offsets, chunk_start, chunk_len, chunk_sum, cap, status_word);
    cwl::prof_end(CWL_PROF_PARTITION, s);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
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
