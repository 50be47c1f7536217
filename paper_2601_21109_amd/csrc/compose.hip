// cwl_compose_scores: the composite difficulty score (gfx950 only).  Sec. III-A of arxiv 2601.21109
// lists, next to the entropy, an n-gram novelty signal against the recent context and a small
// positional prior; include/cwl.h states the reading taken.  A workgroup takes 64 tokens and first
// copies the token ids it can look back at (its own 64 plus window + n - 1 before them) into LDS.
// Four threads share a token: each tests every fourth earlier position of the window, eight
// positions per round with their LDS reads issued together (the n-gram's last id first, the rest
// only where that one matches), and the four answers are combined with two lane exchanges.  One
// thread per token walking its window position by position, each test waiting for the one
// before, took 47 us for 16384 tokens at window 256 on a quarter of the chip.
#include "common.h"

namespace cwl {
namespace {

constexpr int kCompThreads = 256;
constexpr int kCompParts = 4;                                // threads per token
constexpr int kCompTokens = kCompThreads / kCompParts;       // tokens per workgroup
constexpr int kCompRound = 8;                                // positions per thread and round
constexpr int kMaxWindow = 4096;
constexpr int kMaxN = 8;

__global__ void __launch_bounds__(kCompThreads)
compose_scores_kernel(const float* __restrict__ entropy, const int32_t* __restrict__ ids, int64_t n_rows,
                      const int32_t* __restrict__ seq_offsets, int32_t n_seqs, int32_t n, int32_t window,
                      float w_entropy, float w_novelty, float w_prior, float prior_len,
                      float* __restrict__ score, int32_t* __restrict__ novelty) {
    extern __shared__ int32_t ids_lds[];                     // ids[origin .. t0 + 63]
    const int64_t t0 = (int64_t)blockIdx.x * kCompTokens;
    int64_t origin = t0 - window - (n - 1);
    if (origin < 0) origin = 0;
    int64_t last = t0 + kCompTokens;
    if (last > n_rows) last = n_rows;
    for (int64_t i = origin + threadIdx.x; i < last; i += kCompThreads) ids_lds[i - origin] = ids[i];
    const int part = threadIdx.x % kCompParts;
    const int64_t t = t0 + threadIdx.x / kCompParts;
    const bool live = t < n_rows;                            // (every lane stays for the exchanges below)
    // (the entropy and the sequence search are asked for while the ids are on their way into LDS)
    const float h = (live && part == 0) ? entropy[t] : 0.0f;
    // sequence: last b with seq_offsets[b] <= t
    int32_t b = -1;
    if (live) {
        int32_t lo = 0, hi = n_seqs;
        while (lo < hi) {
            const int32_t mid = lo + (hi - lo) / 2;
            if ((int64_t)seq_offsets[mid] <= t) lo = mid + 1; else hi = mid;
        }
        b = lo - 1;
        if (b >= 0 && t >= (int64_t)seq_offsets[b + 1]) b = -1;
    }
    __syncthreads();
    int64_t j = 0;
    int32_t found = 0;
    if (b >= 0) {
        const int64_t base = seq_offsets[b];
        j = t - base;
        if (j >= n - 1) {
            int64_t jlo = j - window;
            if (jlo < n - 1) jlo = n - 1;
            const int32_t* cur = ids_lds + (t - origin);     // cur[-i] = id at position j - i
            const int32_t* seq0 = ids_lds + (base - origin); // seq0[jp] = id at position jp
            // the n-gram's last three ids (fewer for shorter n-grams) are compared without a branch, the rest
            // only where those match: with a small alphabet a test of the last id alone sent some lane of every
            // wavefront into the slow path at nearly every position
            const int32_t n_fast = n < 3 ? n : 3;
            const int32_t cur0 = cur[0], cur1 = n_fast > 1 ? cur[-1] : 0, cur2 = n_fast > 2 ? cur[-2] : 0;
            for (int64_t jp0 = jlo + part; jp0 < j && !found; jp0 += kCompParts * kCompRound) {
                int32_t id0[kCompRound], id1[kCompRound], id2[kCompRound];
#pragma unroll
                for (int u = 0; u < kCompRound; ++u) {
                    int64_t jp = jp0 + (int64_t)u * kCompParts;
                    if (jp > j - 1) jp = j - 1;               // in bounds; its answer is dropped below
                    id0[u] = seq0[jp];
                    id1[u] = n_fast > 1 ? seq0[jp - 1] : 0;
                    id2[u] = n_fast > 2 ? seq0[jp - 2] : 0;
                }
#pragma unroll
                for (int u = 0; u < kCompRound; ++u) {
                    const int64_t jp = jp0 + (int64_t)u * kCompParts;
                    if (jp < j && id0[u] == cur0 && id1[u] == cur1 && id2[u] == cur2) {
                        bool same = true;
                        for (int32_t i = 3; i < n; ++i)
                            if (seq0[jp - i] != cur[-i]) { same = false; break; }
                        if (same) found = 1;
                    }
                }
            }
        }
    }
    found |= __shfl_xor(found, 1);
    found |= __shfl_xor(found, 2);
    if (!live || part != 0) return;
    float s = w_entropy * h;
    int32_t is_new = 0;
    if (b >= 0) {
        is_new = found ? 0 : 1;
        float prior = 0.0f;
        if (prior_len > 0.0f) prior = fmaxf(1.0f - (float)j / prior_len, 0.0f);
        s = fmaf(w_prior, prior, fmaf(w_novelty, (float)is_new, s));
    }
    score[t] = s;
    if (novelty) novelty[t] = is_new;
}

}  // namespace
}  // namespace cwl

using namespace cwl;

extern "C" cwl_status cwl_compose_scores(const float* entropy, const int32_t* token_ids, int64_t n_rows,
                                         const int32_t* seq_offsets, int32_t n_seqs, const cwl_score_mix* m,
                                         float* score, int32_t* novelty, void* stream) {
    if (!m) return CWL_ERR_NULL;
    if (n_rows < 0 || n_rows >= (int64_t)1 << 31 || n_seqs < 0) return CWL_ERR_INVALID_ARG;
    if (m->n < 1 || m->window < 0) return CWL_ERR_INVALID_ARG;
    if (m->n > kMaxN || m->window > kMaxWindow) return CWL_ERR_UNSUPPORTED;
    if (m->w_entropy != m->w_entropy || m->w_novelty != m->w_novelty || m->w_prior != m->w_prior ||
        m->prior_len != m->prior_len)
        return CWL_ERR_INVALID_ARG;
    if (n_rows == 0) return CWL_OK;
    if (!entropy || !token_ids || !score) return CWL_ERR_NULL;
    if (n_seqs > 0 && !seq_offsets) return CWL_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const unsigned blocks = (unsigned)((n_rows + kCompTokens - 1) / kCompTokens);
    const size_t lds = sizeof(int32_t) * (size_t)(kCompTokens + m->window + m->n - 1);
    prof_begin(CWL_PROF_SCORE, st);
    compose_scores_kernel<<<dim3(blocks), dim3(kCompThreads), lds, st>>>(
        entropy, token_ids, n_rows, seq_offsets, n_seqs, m->n, m->window, m->w_entropy, m->w_novelty,
        m->w_prior, m->prior_len, score, novelty);
    prof_end(CWL_PROF_SCORE, st);
    CWL_RETURN_IF_LAUNCH_FAILED();
    return CWL_OK;
}
