// Token -> gate entry of cwl_chunkwise_lora_linear (gfx950 only): the token's sequence (binary
// search in seq_offsets), its chunk (binary search in that sequence's chunk_start range), then
// (r_cur, g_cur, r_prev, g_prev) with the cross-fade of Sec. III-D: inside the first blend_w tokens
// of a chunk that is not the first of its sequence, g_cur = lambda s_cur and
// g_prev = (1 - lambda) s_prev with lambda = (j + 1) / (blend_w + 1).  Tokens outside every chunk
// and out-of-range rungs get the zero entry (base product only).
#pragma once
#include "linear_common.h"

namespace cwl {

// lad_ranks / lad_scales: the ladder in memory that takes a per-thread index (LDS)
__device__ __forceinline__ TokMeta token_meta_of(int64_t t, const int32_t* __restrict__ seq_offsets, int32_t n_seqs,
                                                 const int32_t* __restrict__ chunk_offsets,
                                                 const int32_t* __restrict__ chunk_start,
                                                 const int32_t* __restrict__ chunk_len,
                                                 const int32_t* __restrict__ rank_idx, int32_t chunk_cap,
                                                 int32_t K, const int32_t* lad_ranks, const float* lad_scales,
                                                 int32_t blend_w) {
    TokMeta m = {0, 0, 0.0f, 0.0f};
    if (n_seqs <= 0) return m;
    // sequence: last b with seq_offsets[b] <= t
    int32_t lo = 0, hi = n_seqs;           // first index in [0, n_seqs] with offset > t
    while (lo < hi) {
        const int32_t mid = lo + (hi - lo) / 2;
        if ((int64_t)seq_offsets[mid] <= t) lo = mid + 1; else hi = mid;
    }
    const int32_t b = lo - 1;
    if (b < 0 || t >= (int64_t)seq_offsets[b + 1]) return m;
    int32_t c0 = chunk_offsets[b], c1 = chunk_offsets[b + 1];
    if (c1 > chunk_cap) c1 = chunk_cap;
    int32_t l2 = c0, h2 = c1;              // first chunk in [c0, c1) with start > t
    while (l2 < h2) {
        const int32_t mid = l2 + (h2 - l2) / 2;
        if ((int64_t)chunk_start[mid] <= t) l2 = mid + 1; else h2 = mid;
    }
    const int32_t c = l2 - 1;
    if (c < c0 || c0 < 0) return m;
    const int64_t j = t - chunk_start[c];
    if (j >= chunk_len[c]) return m;
    const int32_t k = rank_idx[c];
    const bool k_ok = k >= 0 && k < K;
    const int32_t r_cur = k_ok ? lad_ranks[k] : 0;
    const float s_cur = (k_ok && r_cur > 0) ? lad_scales[k] : 0.0f;
    if (c == c0 || blend_w == 0 || j >= blend_w) {
        m.r_cur = r_cur;
        m.g_cur = s_cur;
    } else {
        const int32_t kp = rank_idx[c - 1];
        const bool kp_ok = kp >= 0 && kp < K;
        const int32_t r_prev = kp_ok ? lad_ranks[kp] : 0;
        const float s_prev = (kp_ok && r_prev > 0) ? lad_scales[kp] : 0.0f;
        const float lambda = (float)(j + 1) / (float)(blend_w + 1);
        m.r_cur = r_cur;
        m.g_cur = lambda * s_cur;
        m.r_prev = r_prev;
        m.g_prev = (1.0f - lambda) * s_prev;
    }
    return m;
}

// the ladder, passed by value, into LDS arrays of CWL_MAX_LADDER entries (call from every thread
// of the block, then synchronise)
__device__ __forceinline__ void ladder_to_lds(const Ladder& lad, int32_t* lad_ranks, float* lad_scales) {
    if (threadIdx.x < CWL_MAX_LADDER) {
        int32_t r = 0;
        float sc = 0.0f;
#pragma unroll
        for (int k = 0; k < CWL_MAX_LADDER; ++k)
            if (k == (int)threadIdx.x) { r = lad.ranks[k]; sc = lad.scales[k]; }
        lad_ranks[threadIdx.x] = r;
        lad_scales[threadIdx.x] = sc;
    }
}

}  // namespace cwl
