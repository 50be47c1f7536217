// The short-sequence chunker as device code that more than one kernel can carry (gfx950 only): the
// workspace layout, the scan of the quantised scores, the test of 64 candidate chunk ends per step
// (Sec. III-B / IV-B of arxiv 2601.21109) and the body of the kernel that chunks one sequence per
// workgroup.  partition.hip launches that body on its own; the two-phase layer's first product can
// ride in the same launch (gemm_bf16.hip), because the chunk walk occupies one wavefront per sequence.
#pragma once
#include "common.h"

namespace cwl {
namespace part {

constexpr int kThreads = 256;    // workgroup of the sequence, compact and next kernels
constexpr int kItems = 8;        // tokens per thread per scan pass

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

// sum over the block of one int64 per thread; every thread gets the result
__device__ __forceinline__ int64_t block_sum_i64(int64_t v, int64_t* smem /*[waves]*/) {
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

// ---- short sequences: scan and chain walk in one kernel ----
constexpr int kLdsTokens = 8192;   // the chunker's own launch: sequences up to this length keep q and Pin in LDS
constexpr size_t kSeqLdsPerToken = sizeof(int64_t) + 2 * sizeof(int32_t);   // Pin, q, chunk starts
constexpr size_t kSeqLdsBytes = kSeqLdsPerToken * kLdsTokens;

// What the body needs besides its LDS: the kernel arguments of the short-sequence chunker.
struct SeqJob {
    const float* entropy;
    int64_t n_rows;
    const int32_t* seq_offsets;
    int32_t n_seqs, l_min, l_max;
    int64_t theta_q, delta_q;
    PartWs ws;
    int32_t lds_tokens;     // sequences up to this length keep q, Pin and the chunk starts in the 16 * lds_tokens
                            // bytes of dynamic LDS the launch provides; longer ones use the workspace
};

// Workgroup of kThreads threads, sequence b; lds_raw: 16-byte aligned, 16 * job.lds_tokens bytes.
__device__ __forceinline__ void partition_seq_body(const SeqJob& job, const int32_t b, char* lds_raw) {
    const float* __restrict__ entropy = job.entropy;
    const int64_t n_rows = job.n_rows;
    const int32_t* __restrict__ seq_offsets = job.seq_offsets;
    const int32_t n_seqs = job.n_seqs, l_min = job.l_min, l_max = job.l_max;
    const int64_t theta_q = job.theta_q, delta_q = job.delta_q;
    const PartWs& ws = job.ws;
    const int64_t lds_tokens = job.lds_tokens;
    __shared__ int64_t red[kThreads / 64];
    __shared__ int64_t wave_tot[kThreads / 64];
    __shared__ int32_t n_sh;
    const int tid = threadIdx.x, wave = tid >> 6;
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
    if (T <= lds_tokens)
        run(int32_t{0}, reinterpret_cast<int32_t*>(lds_raw + sizeof(int64_t) * lds_tokens),
            reinterpret_cast<int64_t*>(lds_raw),
            reinterpret_cast<int32_t*>(lds_raw + (sizeof(int64_t) + sizeof(int32_t)) * lds_tokens));
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

}  // namespace part

// The first phase of the two-phase layer (u = x A, fp32, no gate) as the chunker's call sees it
// (linear.hip): argument check, the launch on its own, and the launch that carries the chunker's
// workgroups in front of the product's (CWL_ERR_UNSUPPORTED where the shapes do not allow it:
// nothing was launched and the caller launches the two separately).
cwl_status check_shrink_phase(const cwl_linear_desc* d, const void* x, const void* packed, const void* u,
                              size_t u_bytes);
cwl_status run_shrink_phase(const cwl_linear_desc* d, const void* x, const char* packed, float* u, hipStream_t st);
cwl_status launch_seq_with_shrink(const part::SeqJob& job, const cwl_linear_desc* d, const void* x,
                                  const char* packed, float* u, hipStream_t st);

}  // namespace cwl
