// cwl_stream_step: the chunker, the selector and the cross-fade one token at a time (gfx950 only).
// Sec. III-A / III-B of arxiv 2601.21109 have the estimator and the chunker run while decoding and
// Sec. III-F keeps the scheduler's state between steps; the rules are those of
// cwl_partition_chunks / cwl_select_ranks / cwl_chunkwise_lora_linear applied to what is known when
// a token arrives (include/cwl.h states them).  One thread per sequence: a step touches 32 bytes
// of state per sequence and is pure launch latency.  cwl_stream_step_aligned adds what the batch
// controller of Sec. III-G / IV-F and the budget of Sec. III-B mean for a batch that is being decoded:
// one close decision per bucket, taken on the bucket's mean score, and a counter of high-capacity
// chunks per sequence.
#include "linear_common.h"

namespace cwl {
namespace {

static_assert(sizeof(cwl_stream_state) == 32, "layout of the cached state");
static_assert(sizeof(cwl_bucket_state) == 16, "layout of a bucket's open chunk");
static_assert(sizeof(cwl_token_gate) == sizeof(TokMeta), "a gate entry is a TokMeta");

__device__ __forceinline__ bool close_test(int64_t n, int64_t S, int64_t qe, int32_t l_min, int32_t l_max,
                                           int64_t theta_q, int64_t delta_q) {
    if (n < l_min) return false;
    int64_t d = qe * n - S;
    d = d < 0 ? -d : d;
    return n == l_max || S >= theta_q * n || qe >= theta_q || d > delta_q * n;
}

__device__ __forceinline__ int32_t rung_of(int64_t S, int64_t n, const TauTable& taus, int32_t K) {
    int32_t k = 0;
#pragma unroll
    for (int j = 0; j < CWL_MAX_LADDER - 1; ++j) k += (j < K - 1 && S >= taus.tau_q[j] * n) ? 1 : 0;
    return k;
}

// One sequence takes its new token.  shared_close < 0: the sequence decides on its own open chunk;
// otherwise the decision (0 / 1) was taken for its bucket.  n_high: counters of the budget, or NULL.
__device__ __forceinline__ void
step_sequence(int32_t b, int64_t qe, int shared_close, int32_t l_min, int32_t l_max, int64_t theta_q,
              int64_t delta_q, const TauTable& taus, const Ladder& lad, int32_t blend_w, int32_t k_high,
              int32_t budget, int32_t* __restrict__ n_high, cwl_stream_state* __restrict__ state,
              cwl_token_gate* __restrict__ gate, int32_t* __restrict__ closed_len,
              int64_t* __restrict__ closed_sum) {
    cwl_stream_state st = state[b];
    int32_t c_len = 0;
    int64_t c_sum = 0;
    const bool closes = shared_close < 0 ? close_test(st.n, st.sum, qe, l_min, l_max, theta_q, delta_q)
                                         : shared_close != 0;
    int32_t used = n_high ? n_high[b] : 0;
    if (closes && st.n > 0) {
        if (n_high && rung_of(st.sum, st.n, taus, lad.K) >= k_high) {
            used += 1;
            n_high[b] = used;
        }
        c_len = st.n;
        c_sum = st.sum;
        st.k_prev = st.k_cur;
        st.n_chunks += 1;
        st.n = 0;
        st.sum = 0;
    }
    st.n += 1;
    st.sum += qe;
    st.pos += 1;
    int32_t k = rung_of(st.sum, st.n, taus, lad.K);
    if (n_high && k >= k_high && used >= budget) k = k_high - 1;
    st.k_cur = k;
    // rank and scale of rungs k and k_prev (constant indices keep the ladder in scalar registers)
    int32_t r_c = 0, r_p = 0;
    float s_c = 0.0f, s_p = 0.0f;
#pragma unroll
    for (int j = 0; j < CWL_MAX_LADDER; ++j) {
        if (j == k) { r_c = lad.ranks[j]; s_c = lad.scales[j]; }
        if (j == st.k_prev) { r_p = lad.ranks[j]; s_p = lad.scales[j]; }
    }
    if (r_c <= 0) s_c = 0.0f;
    if (r_p <= 0) s_p = 0.0f;
    cwl_token_gate g = {r_c, 0, s_c, 0.0f};
    const int32_t j_off = st.n - 1;
    if (st.n_chunks > 0 && blend_w > 0 && j_off < blend_w) {
        const float lambda = (float)(j_off + 1) / (float)(blend_w + 1);
        g.g_cur = lambda * s_c;
        g.r_prev = r_p;
        g.g_prev = (1.0f - lambda) * s_p;
    }
    state[b] = st;
    gate[b] = g;
    if (closed_len) closed_len[b] = c_len;
    if (closed_sum) closed_sum[b] = c_sum;
}

__global__ void __launch_bounds__(256)
stream_step_kernel(const float* __restrict__ entropy, int32_t n_seqs, int32_t l_min, int32_t l_max,
                   int64_t theta_q, int64_t delta_q, TauTable taus, Ladder lad, int32_t blend_w,
                   int32_t k_high, int32_t budget, int32_t* __restrict__ n_high,
                   cwl_stream_state* __restrict__ state, cwl_token_gate* __restrict__ gate,
                   int32_t* __restrict__ closed_len, int64_t* __restrict__ closed_sum,
                   int32_t* __restrict__ status_word) {
    const int32_t b = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (b >= n_seqs) return;
    bool is_nan = false;
    const int64_t qe = quantise_score(entropy[b], &is_nan);
    if (is_nan) atomicOr(reinterpret_cast<unsigned int*>(status_word), CWL_STATUS_NAN_SCORE);
    step_sequence(b, qe, -1, l_min, l_max, theta_q, delta_q, taus, lad, blend_w, k_high, budget, n_high, state,
                  gate, closed_len, closed_sum);
}

// The step with the close decision shared inside each bucket: one workgroup.  The members' new scores
// are summed per bucket in LDS, one thread per bucket takes the decision on the bucket's open chunk
// (of the mean series), then every sequence takes its token.
constexpr int kAlignedThreads = 1024;
constexpr int kAlignedMax = 4096;     // sequences and buckets the one workgroup holds in LDS

__global__ void __launch_bounds__(kAlignedThreads)
stream_step_aligned_kernel(const float* __restrict__ entropy, int32_t n_seqs, int32_t l_min, int32_t l_max,
                           int64_t theta_q, int64_t delta_q, TauTable taus, Ladder lad, int32_t blend_w,
                           const int32_t* __restrict__ bucket, int32_t n_buckets,
                           cwl_bucket_state* __restrict__ bucket_state, int32_t k_high, int32_t budget,
                           int32_t* __restrict__ n_high, cwl_stream_state* __restrict__ state,
                           cwl_token_gate* __restrict__ gate, int32_t* __restrict__ closed_len,
                           int64_t* __restrict__ closed_sum, int32_t* __restrict__ status_word) {
    __shared__ unsigned long long tot[kAlignedMax];
    __shared__ int32_t cnt[kAlignedMax];          // members in the call, then the bucket's decision
    const int tid = threadIdx.x;
    for (int32_t b = tid; b < n_buckets; b += kAlignedThreads) { tot[b] = 0; cnt[b] = 0; }
    __syncthreads();
    uint32_t bits = 0;
    for (int32_t s = tid; s < n_seqs; s += kAlignedThreads) {
        bool is_nan = false;
        const int32_t q = quantise_score(entropy[s], &is_nan);
        if (is_nan) bits |= CWL_STATUS_NAN_SCORE;
        int32_t b = bucket[s];
        if (b < 0 || b >= n_buckets) {
            bits |= CWL_STATUS_BAD_BUCKET;
            b = b < 0 ? 0 : n_buckets - 1;
        }
        atomicAdd(&tot[b], (unsigned long long)q);
        atomicAdd(&cnt[b], 1);
    }
    if (bits) atomicOr(reinterpret_cast<unsigned int*>(status_word), bits);
    __syncthreads();
    for (int32_t b = tid; b < n_buckets; b += kAlignedThreads) {
        int32_t decision = 0;
        if (cnt[b] > 0) {
            const int64_t qm = (int64_t)(tot[b] / (unsigned long long)cnt[b]);
            cwl_bucket_state bs = bucket_state[b];
            if (close_test(bs.n, bs.sum, qm, l_min, l_max, theta_q, delta_q)) {
                decision = 1;
                bs.n = 0;
                bs.sum = 0;
            }
            bs.n += 1;
            bs.sum += qm;
            bucket_state[b] = bs;
        }
        cnt[b] = decision;
    }
    __syncthreads();
    for (int32_t s = tid; s < n_seqs; s += kAlignedThreads) {
        bool ignore = false;
        const int64_t qe = quantise_score(entropy[s], &ignore);
        int32_t b = bucket[s];
        b = b < 0 ? 0 : (b >= n_buckets ? n_buckets - 1 : b);
        step_sequence(s, qe, cnt[b], l_min, l_max, theta_q, delta_q, taus, lad, blend_w, k_high, budget, n_high,
                      state, gate, closed_len, closed_sum);
    }
}

}  // namespace
}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_stream_step(const float* entropy, int32_t n_seqs, const cwl_chunk_params* p,
                                      const float* thresholds, int32_t K, const int32_t* ranks,
                                      const float* scales, int32_t blend_w, cwl_stream_state* state,
                                      cwl_token_gate* gate, int32_t* closed_len, int64_t* closed_sum,
                                      int32_t* status_word, void* stream) {
    return cwl_stream_step_aligned(entropy, n_seqs, p, thresholds, K, ranks, scales, blend_w, nullptr, 0, nullptr,
                                   1, 0, nullptr, state, gate, closed_len, closed_sum, status_word, stream);
}

extern "C" cwl_status cwl_stream_step_aligned(const float* entropy, int32_t n_seqs, const cwl_chunk_params* p,
                                              const float* thresholds, int32_t K, const int32_t* ranks,
                                              const float* scales, int32_t blend_w, const int32_t* bucket,
                                              int32_t n_buckets, cwl_bucket_state* bucket_state, int32_t k_high,
                                              int32_t budget, int32_t* n_high, cwl_stream_state* state,
                                              cwl_token_gate* gate, int32_t* closed_len, int64_t* closed_sum,
                                              int32_t* status_word, void* stream) {
    if (!p) return CWL_ERR_NULL;
    if (cwl_status ps = check_chunk_params(p); ps != CWL_OK) return ps;
    if (K < 1 || K > CWL_MAX_LADDER || n_seqs < 0 || blend_w < 0) return CWL_ERR_INVALID_ARG;
    if (!ranks || !scales || (K > 1 && !thresholds)) return CWL_ERR_NULL;
    TauTable taus;
    if (fill_tau_table(thresholds, K, &taus) != CWL_OK) return CWL_ERR_INVALID_ARG;
    Ladder lad = {};
    lad.K = K;
    for (int32_t k = 0; k < K; ++k) {
        if (ranks[k] < 0 || ranks[k] > CWL_MAX_RANK || scales[k] != scales[k]) return CWL_ERR_INVALID_ARG;
        if (k > 0 && ranks[k] < ranks[k - 1]) return CWL_ERR_INVALID_ARG;
        lad.ranks[k] = ranks[k];
        lad.scales[k] = scales[k];
    }
    if (n_high && (k_high < 1 || budget < 0)) return CWL_ERR_INVALID_ARG;
    if (bucket) {
        if (n_buckets < 1) return CWL_ERR_INVALID_ARG;
        if (n_seqs > kAlignedMax || n_buckets > kAlignedMax) return CWL_ERR_UNSUPPORTED;
        if (!bucket_state) return CWL_ERR_NULL;
    }
    if (n_seqs == 0) return CWL_OK;
    if (!entropy || !state || !gate || !status_word) return CWL_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int64_t theta_q = quantise_threshold(p->theta_hard), delta_q = quantise_threshold(p->delta_dev);
    prof_begin(CWL_PROF_PARTITION, st);
    if (bucket) {
        stream_step_aligned_kernel<<<dim3(1), dim3(kAlignedThreads), 0, st>>>(
            entropy, n_seqs, p->l_min, p->l_max, theta_q, delta_q, taus, lad, blend_w, bucket, n_buckets,
            bucket_state, k_high, budget, n_high, state, gate, closed_len, closed_sum, status_word);
    } else {
        const unsigned blocks = (unsigned)((n_seqs + 255) / 256);
        stream_step_kernel<<<dim3(blocks), dim3(256), 0, st>>>(
            entropy, n_seqs, p->l_min, p->l_max, theta_q, delta_q, taus, lad, blend_w, k_high, budget, n_high,
            state, gate, closed_len, closed_sum, status_word);
    }
    prof_end(CWL_PROF_PARTITION, st);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
