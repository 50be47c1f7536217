// cwl_stream_step: the chunker, the selector and the cross-fade one token at a time (gfx950 only).
// Sec. III-A / III-B of arxiv 2601.21109 have the estimator and the chunker run while decoding and
// Sec. III-F keeps the scheduler's state between steps; the rules are those of
// cwl_partition_chunks / cwl_select_ranks / cwl_chunkwise_lora_linear applied to what is known when
// a token arrives (include/cwl.h states them).  One thread per sequence: a step touches 32 bytes
// of state per sequence and is pure launch latency.
#include "linear_common.h"

namespace cwl {
namespace {

struct StreamTaus {
    int64_t tau_q[CWL_MAX_LADDER];
};

static_assert(sizeof(cwl_stream_state) == 32, "layout of the cached state");
static_assert(sizeof(cwl_token_gate) == sizeof(TokMeta), "a gate entry is a TokMeta");

__global__ void __launch_bounds__(256)
stream_step_kernel(const float* __restrict__ entropy, int32_t n_seqs, int32_t l_min, int32_t l_max,
                   int64_t theta_q, int64_t delta_q, StreamTaus taus, Ladder lad, int32_t blend_w,
                   cwl_stream_state* __restrict__ state, cwl_token_gate* __restrict__ gate,
                   int32_t* __restrict__ closed_len, int64_t* __restrict__ closed_sum,
                   int32_t* __restrict__ status_word) {
    const int32_t b = (int32_t)(blockIdx.x * blockDim.x + threadIdx.x);
    if (b >= n_seqs) return;
    bool is_nan = false;
    const int64_t qe = quantise_score(entropy[b], &is_nan);
    if (is_nan) atomicOr(reinterpret_cast<unsigned int*>(status_word), CWL_STATUS_NAN_SCORE);
    cwl_stream_state st = state[b];
    int32_t c_len = 0;
    int64_t c_sum = 0;
    if (st.n >= l_min) {
        const int64_t n = st.n, S = st.sum;
        int64_t d = qe * n - S;
        d = d < 0 ? -d : d;
        if (st.n == l_max || S >= theta_q * n || qe >= theta_q || d > delta_q * n) {
            c_len = st.n;
            c_sum = S;
            st.k_prev = st.k_cur;
            st.n_chunks += 1;
            st.n = 0;
            st.sum = 0;
        }
    }
    st.n += 1;
    st.sum += qe;
    st.pos += 1;
    int32_t k = 0;
#pragma unroll
    for (int j = 0; j < CWL_MAX_LADDER - 1; ++j)
        k += (j < lad.K - 1 && st.sum >= taus.tau_q[j] * (int64_t)st.n) ? 1 : 0;
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

}  // namespace
}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_stream_step(const float* entropy, int32_t n_seqs, const cwl_chunk_params* p,
                                      const float* thresholds, int32_t K, const int32_t* ranks,
                                      const float* scales, int32_t blend_w, cwl_stream_state* state,
                                      cwl_token_gate* gate, int32_t* closed_len, int64_t* closed_sum,
                                      int32_t* status_word, void* stream) {
    if (!p) return CWL_ERR_NULL;
    if (p->l_min < 1 || p->l_max < p->l_min) return CWL_ERR_INVALID_ARG;
    if ((int64_t)p->l_max < 2 * (int64_t)p->l_min - 1) return CWL_ERR_INFEASIBLE;
    if (K < 1 || K > CWL_MAX_LADDER || n_seqs < 0 || blend_w < 0) return CWL_ERR_INVALID_ARG;
    if (!ranks || !scales || (K > 1 && !thresholds)) return CWL_ERR_NULL;
    StreamTaus taus = {};
    Ladder lad = {};
    lad.K = K;
    for (int32_t j = 0; j < K - 1; ++j) {
        if (thresholds[j] != thresholds[j]) return CWL_ERR_INVALID_ARG;
        if (j > 0 && thresholds[j] < thresholds[j - 1]) return CWL_ERR_INVALID_ARG;
        taus.tau_q[j] = quantise_threshold(thresholds[j]);
    }
    for (int32_t k = 0; k < K; ++k) {
        if (ranks[k] < 0 || ranks[k] > CWL_MAX_RANK || scales[k] != scales[k]) return CWL_ERR_INVALID_ARG;
        if (k > 0 && ranks[k] < ranks[k - 1]) return CWL_ERR_INVALID_ARG;
        lad.ranks[k] = ranks[k];
        lad.scales[k] = scales[k];
    }
    if (n_seqs == 0) return CWL_OK;
    if (!entropy || !state || !gate || !status_word) return CWL_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned blocks = (unsigned)((n_seqs + 255) / 256);
    prof_begin(CWL_PROF_PARTITION, st);
    stream_step_kernel<<<dim3(blocks), dim3(256), 0, st>>>(
        entropy, n_seqs, p->l_min, p->l_max, quantise_threshold(p->theta_hard),
        quantise_threshold(p->delta_dev), taus, lad, blend_w, state, gate, closed_len, closed_sum,
        status_word);
    prof_end(CWL_PROF_PARTITION, st);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
