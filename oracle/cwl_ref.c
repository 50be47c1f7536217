/*
 * cwl_ref.c -- plain CPU oracle for the ChunkWise LoRA hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct statement of what the
 * path computes.  It shares no code, header, table or helper with the HIP library; only the
 * tests, the smoke check and the bench's cpu_baseline leg may build or call it.
 *
 * All floating-point work is done in double, with one exception: the INT8 codes of the KV-cache
 * policy are decided in fp32, the precision the kernel decides them in.  Inputs are the exact fp32 values the device
 * sees (bf16 inputs are widened to fp32 by the caller, which is exact).
 *
 * Paper passages followed (arxiv 2601.21109):
 *   - Sec. III-A signal (i), Sec. IV-A: next-token entropy from the logits   -> cwl_ref_entropy
 *   - Sec. III-B, Sec. IV-B: online grouping into chunks under (L_min, L_max)
 *     and an average-complexity threshold                                     -> cwl_ref_partition
 *   - Sec. III-C, Sec. IV-C: chunk mean -> rung of the rank ladder            -> cwl_ref_select
 *   - Sec. III-C (sliced ladder), Sec. III-D (linear cross-fade at joins)     -> cwl_ref_linear
 *   - Sec. III-A/B (signals and grouping computed step by step while decoding), Sec. III-F
 *     (scheduler state kept between steps): the same rules one token at a time -> cwl_ref_stream_step
 *   - the layer for rows that bring their own gate (what a decode step feeds) -> cwl_ref_gated_linear
 *   - Sec. III-A signals (ii) n-gram novelty against the recent context and (iv) positional
 *     prior, mixed with the entropy into one score                             -> cwl_ref_compose_scores
 *   - Sec. III-B budget of high-capacity regions per sequence                   -> cwl_ref_limit_high
 *   - Sec. III-G buckets of sequences by complexity percentile, Sec. IV-F
 *     complexity-balanced micro-batches                                        -> cwl_ref_bucket_sequences
 *   - Sec. III-G chunk boundaries aligned inside a bucket                       -> cwl_ref_partition_aligned
 *   - the two above one token at a time, for a batch that is being decoded      -> cwl_ref_stream_step_aligned
 *   - Sec. III-E / IV-F chunk difficulty toggles the KV-cache policy per chunk: INT8 on easy
 *     chunks, full fidelity on hard ones                                        -> cwl_ref_kv_quantise
 *     (its inverse, kv_dequantise, in reference.py)
 *   - Sec. III-C the ladder itself, one SVD of the adapter update: in reference.py (build_ladder),
 *     a float64 library SVD of the product written out
 *
 * The paper gives no formulas for the chunk rule, the rung map or the cross-fade weights; the
 * readings taken are written out step by step in the comments of each function.
 *
 * Parity pins: every function here is pinned by tests that do not call back into this file's
 * own formulas (closed forms, library float64 routines, brute force, hand-worked examples).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define CWL_REF_OK 0
#define CWL_REF_ERR_INVALID 2
#define CWL_REF_ERR_INFEASIBLE 3
#define CWL_REF_ERR_CAPACITY 4

int cwl_ref_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void cwl_ref_set_num_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------------------------------
 * Entropy of softmax(z) in nats (Sec. III-A (i)):  H = -sum_v p_v ln p_v,  p = softmax(z).
 * With m = max z, S = sum exp(z-m), T = sum (z-m) exp(z-m):   H = ln S - T / S.
 * A logit of -inf has p = 0 and contributes nothing.  A row holding NaN or +inf, or made of
 * -inf only, has no defined distribution: the result is NaN.
 * ------------------------------------------------------------------------------------------ */
void cwl_ref_entropy(const float* logits, int64_t n_rows, int64_t vocab, int64_t row_stride,
                     double* H) {
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < n_rows; ++t) {
        const float* z = logits + t * row_stride;
        double m = -INFINITY;
        int bad = 0;
        for (int64_t v = 0; v < vocab; ++v) {
            double zv = (double)z[v];
            if (isnan(zv) || (isinf(zv) && zv > 0)) bad = 1;
            if (zv > m) m = zv;
        }
        if (bad || vocab <= 0 || isinf(m)) { H[t] = NAN; continue; }
        double S = 0.0, T = 0.0;
        for (int64_t v = 0; v < vocab; ++v) {
            double zv = (double)z[v];
            if (isinf(zv)) continue;            /* -inf: probability zero, skip (never 0*inf) */
            double d = zv - m;
            double e = exp(d);
            S += e;
            T += d * e;
        }
        H[t] = log(S) - T / S;
    }
}

/* ------------------------------------------------------------------------------------------
 * Score -> integer.  The chunk rule and the rung map must give the same answer whatever the
 * summation order of the entropy, so the fp32 score is turned into Q10 fixed-point nats once:
 *      q = floor(h * 1024 + 0.5)     evaluated in fp32
 * (h * 1024 is exact; the only rounding is the one add).  Negative, -0 and NaN map to 0 (NaN
 * also raises *nan_flag); the result is clamped to 2^20.  Thresholds go through the same
 * expression but are clamped to 2^21, so that a threshold of +inf can never be met.
 * ------------------------------------------------------------------------------------------ */
#define Q_MAX (1 << 20)
#define QT_MAX (1 << 21)

int32_t cwl_ref_quantise(float h, int32_t* nan_flag) {
    if (isnan(h)) { if (nan_flag) *nan_flag = 1; return 0; }
    if (!(h > 0.0f)) return 0;
    volatile float scaled = h * 1024.0f;           /* volatile: keep the two roundings apart */
    volatile float shifted = scaled + 0.5f;
    float f = floorf(shifted);
    if (f >= (float)Q_MAX) return Q_MAX;
    return (int32_t)f;
}

int64_t cwl_ref_quantise_threshold(float h) {
    if (isnan(h)) return QT_MAX;
    if (!(h > 0.0f)) return 0;
    volatile float scaled = h * 1024.0f;
    volatile float shifted = scaled + 0.5f;
    float f = floorf(shifted);
    if (f >= (float)QT_MAX) return QT_MAX;
    return (int64_t)f;
}

void cwl_ref_quantise_rows(const float* h, int64_t n, int32_t* q, int32_t* nan_flag) {
    for (int64_t i = 0; i < n; ++i) q[i] = cwl_ref_quantise(h[i], nan_flag);
}

/* ------------------------------------------------------------------------------------------
 * Adaptive chunker (Sec. III-B, Sec. IV-B: tokens are grouped as they arrive, under length bounds
 * and a threshold on the average complexity).  Reading: a chunk opened at p is extended one token at a time
 * and is closed at the first end e (chunk = [p, e)) in [p+L_min, p+L_max] at which
 *      hard :  the chunk's mean score has reached theta           S >= theta_q * n
 *      enter:  the token that would come next is itself hard      q[e] >= theta_q
 *      dev  :  the next token leaves the chunk's regime           |q[e]*n - S| > delta_q * n
 * where S = sum of q over [p, e), n = e - p.  An end is only admissible if it leaves either
 * nothing or at least L_min tokens behind it, so no tail shorter than L_min is ever stranded.
 * If nothing fires the chunk runs to the last admissible end.  A sequence shorter than L_min is
 * one chunk (the only exception to the bounds).  Hard spans are therefore cut every L_min
 * tokens and easy spans grow to L_max, which is the behaviour Sec. III-B describes.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_partition(const int32_t* q, const int32_t* seq_offsets, int32_t n_seqs,
                      int32_t l_min, int32_t l_max, int64_t theta_q, int64_t delta_q,
                      int32_t* chunk_offsets, int32_t* chunk_start, int32_t* chunk_len,
                      int64_t* chunk_sum, int32_t cap) {
    if (l_min < 1 || l_max < l_min) return CWL_REF_ERR_INVALID;
    if ((int64_t)l_max < 2 * (int64_t)l_min - 1) return CWL_REF_ERR_INFEASIBLE;
    int64_t n_chunks = 0;
    for (int32_t b = 0; b < n_seqs; ++b) {
        chunk_offsets[b] = (int32_t)n_chunks;
        const int64_t base = seq_offsets[b];
        const int64_t T = (int64_t)seq_offsets[b + 1] - base;
        if (T < 0) return CWL_REF_ERR_INVALID;
        if (T == 0) continue;
        const int32_t* qs = q + base;
        int64_t* P = (int64_t*)malloc((size_t)(T + 1) * sizeof(int64_t));
        P[0] = 0;
        for (int64_t i = 0; i < T; ++i) P[i + 1] = P[i] + qs[i];
        if (T < l_min) {
            if (n_chunks < cap) {
                chunk_start[n_chunks] = (int32_t)base;
                chunk_len[n_chunks] = (int32_t)T;
                chunk_sum[n_chunks] = P[T];
            }
            ++n_chunks;
            free(P);
            continue;
        }
        int64_t p = 0;
        while (p < T) {
            int64_t last;
            if (T - p <= l_max) last = T;
            else last = (p + l_max < T - l_min) ? p + l_max : T - l_min;
            int64_t e_star = last;
            int64_t e_hi = (p + l_max < T) ? p + l_max : T;
            for (int64_t e = p + l_min; e <= e_hi; ++e) {
                if (!(e <= T - l_min || e == T)) continue;
                if (e == T) { e_star = e; break; }
                const int64_t n = e - p;
                const int64_t S = P[e] - P[p];
                const int64_t qe = qs[e];
                const int hard = S >= theta_q * n;
                const int enter = qe >= theta_q;
                int64_t d = qe * n - S;
                if (d < 0) d = -d;
                const int dev = d > delta_q * n;
                if (hard || enter || dev) { e_star = e; break; }
            }
            if (n_chunks < cap) {
                chunk_start[n_chunks] = (int32_t)(base + p);
                chunk_len[n_chunks] = (int32_t)(e_star - p);
                chunk_sum[n_chunks] = P[e_star] - P[p];
            }
            ++n_chunks;
            p = e_star;
        }
        free(P);
    }
    chunk_offsets[n_seqs] = (int32_t)n_chunks;
    return n_chunks > cap ? CWL_REF_ERR_CAPACITY : CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Rung selection (Sec. III-C, Sec. IV-C: a rule that maps percentiles of the score to rungs): the caller's K-1
 * ascending thresholds are the percentile table; the rung is the number of thresholds the
 * chunk's mean score reaches,  k = #{ j : sum >= tau_q[j] * len }.  A mean exactly on a
 * threshold goes up.
 * ------------------------------------------------------------------------------------------ */
void cwl_ref_select(const int64_t* chunk_sum, const int32_t* chunk_len, int64_t n_chunks,
                    const int64_t* tau_q, int32_t K, int32_t* rank_idx) {
    for (int64_t c = 0; c < n_chunks; ++c) {
        int32_t k = 0;
        for (int32_t j = 0; j < K - 1; ++j)
            if (chunk_sum[c] >= tau_q[j] * (int64_t)chunk_len[c]) ++k;
        rank_idx[c] = k;
    }
}

/* ------------------------------------------------------------------------------------------
 * Chunk-segmented variable-rank LoRA linear with the boundary cross-fade.
 *   adapter of rung k on token t (Sec. III-C: first r_k directions of the stored factors):
 *        D_k(t) = s_k * sum_{i < r_k} (x_t . A[:, i]) * B[i, :]
 *   token t in chunk c at offset j = t - start_c (Sec. III-D: outgoing ramps down, incoming up):
 *        first chunk of its sequence, or j >= w, or w == 0:   y_t = x_t W + D_{k_c}(t)
 *        otherwise, lambda = (j + 1) / (w + 1):
 *              y_t = x_t W + (1 - lambda) * D_{k_{c-1}}(t) + lambda * D_{k_c}(t)
 * A rung of rank 0 contributes nothing whatever its scale.  A token that no chunk covers gets
 * the base product only.  Only the rows listed in `rows` are evaluated (all of them when rows
 * is NULL); y is [n_sel, d_out] in double, not rounded.  With x_compact != 0 the array x holds
 * just the listed rows, in the order of `rows` (x[i] is token rows[i]); the chunk table still
 * refers to the original token numbering.
 * ------------------------------------------------------------------------------------------ */
static void adapter_term(const double* u, const float* B, int64_t ldb, int64_t d_out,
                         int32_t r, double s, double weight, double* acc) {
    if (r <= 0 || weight == 0.0) return;
    for (int64_t j = 0; j < d_out; ++j) {
        double d = 0.0;
        for (int32_t i = 0; i < r; ++i) d += u[i] * (double)B[(int64_t)i * ldb + j];
        acc[j] += weight * (s * d);
    }
}

int cwl_ref_linear(const float* x, int64_t ldx, const float* W, int64_t ldw,
                   const float* A, int64_t lda, const float* B, int64_t ldb,
                   int64_t n_rows, int64_t d_in, int64_t d_out, int32_t r_max,
                   int32_t K, const int32_t* ranks, const float* scales, int32_t blend_w,
                   const int32_t* seq_offsets, int32_t n_seqs,
                   const int32_t* chunk_offsets, const int32_t* chunk_start,
                   const int32_t* chunk_len, const int32_t* rank_idx,
                   const int64_t* rows, int64_t n_sel, int32_t x_compact, double* y) {
    if (K < 1 || r_max < 0 || blend_w < 0) return CWL_REF_ERR_INVALID;
    for (int32_t k = 0; k < K; ++k)
        if (ranks[k] < 0 || ranks[k] > r_max) return CWL_REF_ERR_INVALID;
    /* token -> (chunk, is-first-chunk-of-its-sequence); -1 where no chunk covers the token */
    int32_t* tok_chunk = (int32_t*)malloc((size_t)(n_rows > 0 ? n_rows : 1) * sizeof(int32_t));
    char* tok_first = (char*)calloc((size_t)(n_rows > 0 ? n_rows : 1), 1);
    for (int64_t t = 0; t < n_rows; ++t) tok_chunk[t] = -1;
    for (int32_t b = 0; b < n_seqs; ++b) {
        for (int32_t c = chunk_offsets[b]; c < chunk_offsets[b + 1]; ++c) {
            for (int32_t j = 0; j < chunk_len[c]; ++j) {
                int64_t t = (int64_t)chunk_start[c] + j;
                if (t < 0 || t >= n_rows) continue;
                if (t < seq_offsets[b] || t >= seq_offsets[b + 1]) continue;
                tok_chunk[t] = c;
                tok_first[t] = (c == chunk_offsets[b]);
            }
        }
    }
    const int64_t count = rows ? n_sel : n_rows;
#pragma omp parallel
    {
        double* u = (double*)malloc((size_t)(r_max > 0 ? r_max : 1) * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t s_i = 0; s_i < count; ++s_i) {
            const int64_t t = rows ? rows[s_i] : s_i;
            double* yt = y + s_i * d_out;
            const float* xt = x + ((rows && x_compact) ? s_i : t) * ldx;
            for (int64_t j = 0; j < d_out; ++j) yt[j] = 0.0;
            for (int64_t k = 0; k < d_in; ++k) {            /* base product x_t W */
                const double xv = (double)xt[k];
                const float* wrow = W + k * ldw;
                for (int64_t j = 0; j < d_out; ++j) yt[j] += xv * (double)wrow[j];
            }
            const int32_t c = tok_chunk[t];
            if (c < 0) continue;
            for (int32_t i = 0; i < r_max; ++i) {           /* u = x_t A, all stored directions */
                double a = 0.0;
                for (int64_t k = 0; k < d_in; ++k) a += (double)xt[k] * (double)A[k * lda + i];
                u[i] = a;
            }
            const int32_t kc = rank_idx[c];
            const int64_t j_off = t - chunk_start[c];
            if (tok_first[t] || blend_w == 0 || j_off >= blend_w) {
                adapter_term(u, B, ldb, d_out, ranks[kc], (double)scales[kc], 1.0, yt);
            } else {
                const double lambda = (double)(j_off + 1) / (double)(blend_w + 1);
                const int32_t kp = rank_idx[c - 1];
                adapter_term(u, B, ldb, d_out, ranks[kp], (double)scales[kp], 1.0 - lambda, yt);
                adapter_term(u, B, ldb, d_out, ranks[kc], (double)scales[kc], lambda, yt);
            }
        }
        free(u);
    }
    free(tok_chunk);
    free(tok_first);
    return CWL_REF_OK;
}


/* ------------------------------------------------------------------------------------------
 * Decode-step form of the chunker, the selector and the cross-fade (Sec. III-A and III-B have the
 * estimator and the chunker run while decoding, Sec. III-F keeps the scheduler's state between steps).
 * One call consumes ONE new token per sequence.  Per sequence the cached state is the open
 * chunk (tokens n, score sum S), the rung in force at the previous token (k_cur), the rung the
 * previous chunk ended with (k_prev), the number of chunks closed and of tokens seen.
 *
 * Reading (the paper gives no online rule): the new token, with score qe, is tested against the
 * open chunk exactly as the batch chunker tests an end e = (position of the new token): if the
 * open chunk has n >= L_min tokens and (n == L_max, or hard, or enter, or dev -- the three tests
 * of cwl_ref_partition on S, n, qe) the chunk is closed in front of the token and the token opens
 * the next one; otherwise it joins the open chunk.  The end of the sequence is not known, so the
 * batch rule that keeps a tail of at least L_min has no counterpart here: both forms place the
 * same boundaries as long as the chunk starts at least L_min + L_max before the end.
 * The rung in force for a token is the selector's rule on the open chunk as far as it is known,
 * k = #{ j : S >= tau_q[j] * n } with the token itself included; at the last token of a chunk that
 * is the rung the batch form gives the whole chunk.  The first w tokens of a chunk that is not the
 * first of its sequence cross-fade from the rung the previous chunk ended with:
 *      lambda = (j + 1) / (w + 1),  j = offset of the token in its chunk,
 *      gate = (r_cur, lambda * s_cur, r_prev, (1 - lambda) * s_prev);   else (r_cur, s_cur, 0, 0).
 * closed_len / closed_sum report the chunk this token closed (0 when none).
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_stream_step(const int32_t* q_new, int32_t n_seqs, int32_t l_min, int32_t l_max,
                        int64_t theta_q, int64_t delta_q, const int64_t* tau_q, int32_t K,
                        const int32_t* ranks, const float* scales, int32_t blend_w,
                        int32_t* st_n, int64_t* st_sum, int32_t* st_k_cur, int32_t* st_k_prev,
                        int32_t* st_chunks, int64_t* st_pos,
                        int32_t* r_cur, double* g_cur, int32_t* r_prev, double* g_prev,
                        int32_t* closed_len, int64_t* closed_sum) {
    if (l_min < 1 || l_max < l_min || K < 1 || blend_w < 0) return CWL_REF_ERR_INVALID;
    if ((int64_t)l_max < 2 * (int64_t)l_min - 1) return CWL_REF_ERR_INFEASIBLE;
    for (int32_t b = 0; b < n_seqs; ++b) {
        const int64_t qe = q_new[b];
        closed_len[b] = 0;
        closed_sum[b] = 0;
        if (st_n[b] >= l_min) {
            const int64_t n = st_n[b], S = st_sum[b];
            const int hard = S >= theta_q * n;
            const int enter = qe >= theta_q;
            int64_t d = qe * n - S;
            if (d < 0) d = -d;
            const int dev = d > delta_q * n;
            if (n == l_max || hard || enter || dev) {
                closed_len[b] = (int32_t)n;
                closed_sum[b] = S;
                st_k_prev[b] = st_k_cur[b];
                st_chunks[b] += 1;
                st_n[b] = 0;
                st_sum[b] = 0;
            }
        }
        st_n[b] += 1;
        st_sum[b] += qe;
        st_pos[b] += 1;
        int32_t k = 0;
        for (int32_t j = 0; j < K - 1; ++j)
            if (st_sum[b] >= tau_q[j] * (int64_t)st_n[b]) ++k;
        st_k_cur[b] = k;
        const int32_t rc = ranks[k];
        const double sc = rc > 0 ? (double)scales[k] : 0.0;
        const int32_t j_off = st_n[b] - 1;
        if (st_chunks[b] == 0 || blend_w == 0 || j_off >= blend_w) {
            r_cur[b] = rc;  g_cur[b] = sc;
            r_prev[b] = 0;  g_prev[b] = 0.0;
        } else {
            const int32_t kp = st_k_prev[b];
            const int32_t rp = ranks[kp];
            const double sp = rp > 0 ? (double)scales[kp] : 0.0;
            const double lambda = (double)(j_off + 1) / (double)(blend_w + 1);
            r_cur[b] = rc;  g_cur[b] = lambda * sc;
            r_prev[b] = rp; g_prev[b] = (1.0 - lambda) * sp;
        }
    }
    return CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * The layer for rows that bring their own gate (Sec. III-C sliced ladder, Sec. III-D cross-fade,
 * with the weights already decided):
 *      y_t = x_t W + g_cur(t) * sum_{i < r_cur(t)} (x_t . A[:, i]) B[i, :]
 *                  + g_prev(t) * sum_{i < r_prev(t)} (x_t . A[:, i]) B[i, :]
 * y is [n_rows, d_out] in double, not rounded.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_gated_linear(const float* x, int64_t ldx, const float* W, int64_t ldw,
                         const float* A, int64_t lda, const float* B, int64_t ldb,
                         int64_t n_rows, int64_t d_in, int64_t d_out, int32_t r_max,
                         const int32_t* r_cur, const double* g_cur, const int32_t* r_prev,
                         const double* g_prev, double* y) {
    if (r_max < 0) return CWL_REF_ERR_INVALID;
    for (int64_t t = 0; t < n_rows; ++t)
        if (r_cur[t] < 0 || r_cur[t] > r_max || r_prev[t] < 0 || r_prev[t] > r_max) return CWL_REF_ERR_INVALID;
#pragma omp parallel
    {
        double* u = (double*)malloc((size_t)(r_max > 0 ? r_max : 1) * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (int64_t t = 0; t < n_rows; ++t) {
            double* yt = y + t * d_out;
            const float* xt = x + t * ldx;
            for (int64_t j = 0; j < d_out; ++j) yt[j] = 0.0;
            for (int64_t k = 0; k < d_in; ++k) {
                const double xv = (double)xt[k];
                const float* wrow = W + k * ldw;
                for (int64_t j = 0; j < d_out; ++j) yt[j] += xv * (double)wrow[j];
            }
            for (int32_t i = 0; i < r_max; ++i) {
                double a = 0.0;
                for (int64_t k = 0; k < d_in; ++k) a += (double)xt[k] * (double)A[k * lda + i];
                u[i] = a;
            }
            adapter_term(u, B, ldb, d_out, r_cur[t], 1.0, g_cur[t], yt);
            adapter_term(u, B, ldb, d_out, r_prev[t], 1.0, g_prev[t], yt);
        }
        free(u);
    }
    return CWL_REF_OK;
}


/* ------------------------------------------------------------------------------------------
 * Composite difficulty score (Sec. III-A lists, next to the entropy, an n-gram novelty signal
 * against the recent context and a small positional prior that favours early steps; the paper
 * gives neither formula nor weights).  Reading, per token t at position j of its sequence:
 *   novelty_t = 1 if the n-gram of token ids that ends at j, ids[j-n+1 .. j], ends at none of the
 *               positions j' with max(n-1, j-window) <= j' < j of the same sequence; tokens with
 *               j < n-1 (no complete n-gram yet) count as new;  else 0;
 *   prior_t   = max(0, 1 - j / prior_len)   (0 when prior_len <= 0): a linear ramp down over the
 *               first prior_len tokens;
 *   score_t   = w_entropy * H_t + w_novelty * novelty_t + w_prior * prior_t.
 * A token outside every sequence keeps score_t = w_entropy * H_t and novelty 0.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_compose_scores(const float* entropy, const int32_t* ids, int64_t n_rows,
                           const int32_t* seq_offsets, int32_t n_seqs, int32_t n, int32_t window,
                           double w_entropy, double w_novelty, double w_prior, double prior_len,
                           double* score, int32_t* novelty) {
    if (n < 1 || window < 0) return CWL_REF_ERR_INVALID;
    for (int64_t t = 0; t < n_rows; ++t) {
        score[t] = w_entropy * (double)entropy[t];
        novelty[t] = 0;
    }
    for (int32_t b = 0; b < n_seqs; ++b) {
        const int64_t base = seq_offsets[b];
        const int64_t T = (int64_t)seq_offsets[b + 1] - base;
        if (T < 0 || base < 0 || base + T > n_rows) return CWL_REF_ERR_INVALID;
        const int32_t* s_ids = ids + base;
        for (int64_t j = 0; j < T; ++j) {
            int is_new = 1;
            if (j >= n - 1) {
                int64_t lo = j - window;
                if (lo < n - 1) lo = n - 1;
                for (int64_t jp = lo; jp < j && is_new; ++jp) {
                    int same = 1;
                    for (int32_t i = 0; i < n; ++i)
                        if (s_ids[jp - i] != s_ids[j - i]) { same = 0; break; }
                    if (same) is_new = 0;
                }
            }
            double prior = 0.0;
            if (prior_len > 0.0) {
                prior = 1.0 - (double)j / prior_len;
                if (prior < 0.0) prior = 0.0;
            }
            novelty[base + j] = is_new;
            score[base + j] = w_entropy * (double)entropy[base + j] + w_novelty * (double)is_new + w_prior * prior;
        }
    }
    return CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Budget of high-capacity regions per sequence (Sec. III-B lists the budget among the chunker's
 * constraints; the paper gives no rule).  Reading: a chunk asks for high capacity when the rung
 * the selector gives it is at least k_high.  Chunks are met in sequence order, as the online
 * chunker meets them; the first `budget` chunks of a sequence that ask keep their rung, every
 * later one that asks is set to rung k_high - 1, the highest one that is not high capacity.
 * n_asked[s] (when not NULL) reports how many chunks of sequence s asked.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_limit_high(int32_t* rank_idx, const int32_t* chunk_offsets, int32_t n_seqs,
                       int32_t k_high, int32_t budget, int32_t* n_asked) {
    if (k_high < 1 || budget < 0) return CWL_REF_ERR_INVALID;
    for (int32_t s = 0; s < n_seqs; ++s) {
        int32_t asked = 0;
        for (int32_t c = chunk_offsets[s]; c < chunk_offsets[s + 1]; ++c) {
            if (rank_idx[c] >= k_high) {
                if (asked >= budget) rank_idx[c] = k_high - 1;
                ++asked;
            }
        }
        if (n_asked) n_asked[s] = asked;
    }
    return CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Buckets of sequences by complexity percentile, and complexity-balanced micro-batches
 * (Sec. III-G: sequences of a batch are bucketed by complexity percentiles so that their chunk
 * boundaries can be aligned; Sec. IV-F: a batch controller keeps micro-batches balanced in
 * complexity).  Reading: the complexity of a sequence is the mean of its quantised scores,
 * m_s = floor(sum_s / T_s) (0 for an empty sequence).  Sequences are ranked by (m_s, s) ascending,
 * rho_s being the rank; order[rho_s] = s.  With n_buckets equal-count percentile bins,
 *      bucket_s = floor(rho_s * n_buckets / n_seqs),
 * so bucket 0 holds the sequences below the (100 / n_buckets)-th percentile, and so on.
 * Micro-batches (when asked for) are dealt from the ranked order in alternating direction, round
 * by round:  round = floor(rho / n_micro), j = rho mod n_micro,
 *      micro_s = j for even rounds, n_micro - 1 - j for odd rounds,
 * which gives every micro-batch the same number of sequences (within one) and total complexities
 * that differ by no more than the spread of m over the batch.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_bucket_sequences(const int32_t* q, const int32_t* seq_offsets, int32_t n_seqs,
                             int32_t n_buckets, int32_t n_micro, int64_t* seq_sum,
                             int32_t* order, int32_t* bucket, int32_t* micro) {
    if (n_buckets < 1 || n_micro < 0) return CWL_REF_ERR_INVALID;
    int64_t* mean = (int64_t*)malloc((size_t)(n_seqs + 1) * sizeof(int64_t));
    for (int32_t s = 0; s < n_seqs; ++s) {
        const int64_t T = (int64_t)seq_offsets[s + 1] - seq_offsets[s];
        if (T < 0) { free(mean); return CWL_REF_ERR_INVALID; }
        int64_t sum = 0;
        for (int64_t t = 0; t < T; ++t) sum += q[seq_offsets[s] + t];
        seq_sum[s] = sum;
        mean[s] = T > 0 ? sum / T : 0;
    }
    /* rank by counting: rho_s = number of sequences that come before s in (mean, index) order */
    for (int32_t s = 0; s < n_seqs; ++s) {
        int32_t rho = 0;
        for (int32_t u = 0; u < n_seqs; ++u)
            if (mean[u] < mean[s] || (mean[u] == mean[s] && u < s)) ++rho;
        order[rho] = s;
        bucket[s] = (int32_t)(((int64_t)rho * n_buckets) / n_seqs);
        if (micro && n_micro > 0) {
            const int32_t round = rho / n_micro, j = rho % n_micro;
            micro[s] = (round % 2 == 0) ? j : n_micro - 1 - j;
        }
    }
    free(mean);
    return CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Chunker with boundaries aligned inside each bucket (Sec. III-G: chunk boundaries of the
 * sequences of a bucket are aligned, while every sequence keeps its own rank choices).
 * Reading: the sequences of a bucket share one set of boundaries, those the chunker of
 * cwl_ref_partition places on the bucket's mean score series
 *      m_b[t] = floor( sum over members s with T_s > t of q_s[t]  /  number of such members ),
 * t < max T_s over the members.  A member takes every boundary that falls inside it: its chunks
 * are [e_i, min(e_{i+1}, T_s)) for the bucket's chunk starts e_i < T_s, so only its last chunk
 * can be shorter than the bucket's (and shorter than L_min).  Chunk sums are the member's own
 * scores, so the selector still decides per sequence.  With one sequence per bucket this is
 * cwl_ref_partition.
 * ------------------------------------------------------------------------------------------ */
int cwl_ref_partition_aligned(const int32_t* q, const int32_t* seq_offsets, int32_t n_seqs,
                              const int32_t* bucket, int32_t n_buckets,
                              int32_t l_min, int32_t l_max, int64_t theta_q, int64_t delta_q,
                              int32_t* chunk_offsets, int32_t* chunk_start, int32_t* chunk_len,
                              int64_t* chunk_sum, int32_t cap) {
    if (n_buckets < 1) return CWL_REF_ERR_INVALID;
    if (l_min < 1 || l_max < l_min) return CWL_REF_ERR_INVALID;
    if ((int64_t)l_max < 2 * (int64_t)l_min - 1) return CWL_REF_ERR_INFEASIBLE;
    int64_t n_rows = 0;
    for (int32_t s = 0; s < n_seqs; ++s) {
        if (bucket[s] < 0 || bucket[s] >= n_buckets) return CWL_REF_ERR_INVALID;
        if (seq_offsets[s + 1] < seq_offsets[s]) return CWL_REF_ERR_INVALID;
        if (seq_offsets[s + 1] > n_rows) n_rows = seq_offsets[s + 1];
    }
    /* boundaries of every bucket: bstart[b] points at the bucket's ascending chunk starts */
    int32_t** bstart = (int32_t**)calloc((size_t)n_buckets, sizeof(int32_t*));
    int32_t* bcount = (int32_t*)calloc((size_t)n_buckets, sizeof(int32_t));
    int32_t* bend = (int32_t*)calloc((size_t)n_buckets, sizeof(int32_t));   /* bucket's longest member */
    int32_t* m = (int32_t*)malloc((size_t)(n_rows + 1) * sizeof(int32_t));
    for (int32_t b = 0; b < n_buckets; ++b) {
        int64_t Tmax = 0;
        for (int32_t s = 0; s < n_seqs; ++s)
            if (bucket[s] == b && (int64_t)seq_offsets[s + 1] - seq_offsets[s] > Tmax)
                Tmax = (int64_t)seq_offsets[s + 1] - seq_offsets[s];
        bend[b] = (int32_t)Tmax;
        for (int64_t t = 0; t < Tmax; ++t) {
            int64_t sum = 0, alive = 0;
            for (int32_t s = 0; s < n_seqs; ++s)
                if (bucket[s] == b && (int64_t)seq_offsets[s + 1] - seq_offsets[s] > t) {
                    sum += q[seq_offsets[s] + t];
                    ++alive;
                }
            m[t] = (int32_t)(sum / alive);
        }
        const int32_t vcap = (int32_t)Tmax + 1;
        int32_t voff[2] = {0, (int32_t)Tmax};
        int32_t vco[2];
        int32_t* vstart = (int32_t*)malloc((size_t)vcap * sizeof(int32_t));
        int32_t* vlen = (int32_t*)malloc((size_t)vcap * sizeof(int32_t));
        int64_t* vsum = (int64_t*)malloc((size_t)vcap * sizeof(int64_t));
        const int st = cwl_ref_partition(m, voff, 1, l_min, l_max, theta_q, delta_q, vco, vstart, vlen, vsum, vcap);
        free(vlen);
        free(vsum);
        if (st != CWL_REF_OK) { free(vstart); free(m); free(bstart); free(bcount); free(bend); return st; }
        bstart[b] = vstart;
        bcount[b] = vco[1];
    }
    int64_t n_chunks = 0;
    for (int32_t s = 0; s < n_seqs; ++s) {
        chunk_offsets[s] = (int32_t)n_chunks;
        const int64_t base = seq_offsets[s];
        const int64_t T = (int64_t)seq_offsets[s + 1] - base;
        const int32_t b = bucket[s];
        for (int32_t i = 0; i < bcount[b]; ++i) {
            const int64_t e0 = bstart[b][i];
            if (e0 >= T) break;
            int64_t e1 = (i + 1 < bcount[b]) ? bstart[b][i + 1] : bend[b];
            if (e1 > T) e1 = T;
            if (n_chunks < cap) {
                int64_t sum = 0;
                for (int64_t t = e0; t < e1; ++t) sum += q[base + t];
                chunk_start[n_chunks] = (int32_t)(base + e0);
                chunk_len[n_chunks] = (int32_t)(e1 - e0);
                chunk_sum[n_chunks] = sum;
            }
            ++n_chunks;
        }
    }
    chunk_offsets[n_seqs] = (int32_t)n_chunks;
    for (int32_t b = 0; b < n_buckets; ++b) free(bstart[b]);
    free(bstart); free(bcount); free(bend); free(m);
    return n_chunks > cap ? CWL_REF_ERR_CAPACITY : CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------
 * Decode step of a batch under the batch controller: boundaries aligned inside each bucket
 * (Sec. III-G speaks of batched decoding) and the budget of high-capacity chunks (Sec. III-B),
 * one new token per sequence.  It is cwl_ref_stream_step with two changes.
 *   Alignment (bucket != NULL): every bucket keeps one open chunk of its own on the bucket's mean
 * series, state (bn, bsum).  The mean of the step is qm = floor(sum of the members' new scores /
 * number of members in the call).  The close test of cwl_ref_stream_step is taken once per bucket
 * on (bn, bsum, qm); when it fires, every member closes its own open chunk (if it has one) in front
 * of its new token.  The bucket's chunk then takes qm as the members' chunks take their own score.
 * A bucket without members in the call keeps its state.  With bucket == NULL every sequence decides
 * on its own open chunk as in cwl_ref_stream_step.
 *   Budget (n_high != NULL): n_high[s] counts the closed chunks of sequence s whose last token had
 * a rung of at least k_high before any lowering, which is the chunk's rung in the batch form.  The
 * rung in force for a token is the selector's rule on the open chunk, lowered to k_high - 1 when it
 * is at least k_high and n_high[s] >= budget.  k_prev, the outgoing rung of the cross-fade, is the
 * rung in force at the previous chunk's last token, lowered or not.
 * Fed token by token to sequences of equal length, this places the boundaries of
 * cwl_ref_partition_aligned (where the end cannot matter) and ends every chunk on the rung that
 * cwl_ref_select followed by cwl_ref_limit_high gives it.
 * ------------------------------------------------------------------------------------------ */
static int32_t rung_of(int64_t S, int64_t n, const int64_t* tau_q, int32_t K) {
    int32_t k = 0;
    for (int32_t j = 0; j < K - 1; ++j)
        if (S >= tau_q[j] * n) ++k;
    return k;
}

static int close_test(int64_t n, int64_t S, int64_t qe, int32_t l_min, int32_t l_max,
                      int64_t theta_q, int64_t delta_q) {
    if (n < l_min) return 0;
    int64_t d = qe * n - S;
    if (d < 0) d = -d;
    return n == l_max || S >= theta_q * n || qe >= theta_q || d > delta_q * n;
}

int cwl_ref_stream_step_aligned(const int32_t* q_new, int32_t n_seqs, int32_t l_min, int32_t l_max,
                                int64_t theta_q, int64_t delta_q, const int64_t* tau_q, int32_t K,
                                const int32_t* ranks, const float* scales, int32_t blend_w,
                                const int32_t* bucket, int32_t n_buckets, int32_t* bk_n, int64_t* bk_sum,
                                int32_t k_high, int32_t budget, int32_t* n_high,
                                int32_t* st_n, int64_t* st_sum, int32_t* st_k_cur, int32_t* st_k_prev,
                                int32_t* st_chunks, int64_t* st_pos,
                                int32_t* r_cur, double* g_cur, int32_t* r_prev, double* g_prev,
                                int32_t* closed_len, int64_t* closed_sum) {
    if (l_min < 1 || l_max < l_min || K < 1 || blend_w < 0) return CWL_REF_ERR_INVALID;
    if ((int64_t)l_max < 2 * (int64_t)l_min - 1) return CWL_REF_ERR_INFEASIBLE;
    if (n_high && (k_high < 1 || budget < 0)) return CWL_REF_ERR_INVALID;
    int* bclose = NULL;
    if (bucket) {
        if (n_buckets < 1) return CWL_REF_ERR_INVALID;
        for (int32_t s = 0; s < n_seqs; ++s)
            if (bucket[s] < 0 || bucket[s] >= n_buckets) return CWL_REF_ERR_INVALID;
        bclose = (int*)calloc((size_t)n_buckets, sizeof(int));
        for (int32_t b = 0; b < n_buckets; ++b) {
            int64_t tot = 0, members = 0;
            for (int32_t s = 0; s < n_seqs; ++s)
                if (bucket[s] == b) { tot += q_new[s]; ++members; }
            if (members == 0) continue;
            const int64_t qm = tot / members;
            bclose[b] = close_test(bk_n[b], bk_sum[b], qm, l_min, l_max, theta_q, delta_q);
            if (bclose[b]) { bk_n[b] = 0; bk_sum[b] = 0; }
            bk_n[b] += 1;
            bk_sum[b] += qm;
        }
    }
    for (int32_t s = 0; s < n_seqs; ++s) {
        const int64_t qe = q_new[s];
        closed_len[s] = 0;
        closed_sum[s] = 0;
        const int closes = bucket ? bclose[bucket[s]]
                                  : close_test(st_n[s], st_sum[s], qe, l_min, l_max, theta_q, delta_q);
        if (closes && st_n[s] > 0) {
            if (n_high && rung_of(st_sum[s], st_n[s], tau_q, K) >= k_high) n_high[s] += 1;
            closed_len[s] = st_n[s];
            closed_sum[s] = st_sum[s];
            st_k_prev[s] = st_k_cur[s];
            st_chunks[s] += 1;
            st_n[s] = 0;
            st_sum[s] = 0;
        }
        st_n[s] += 1;
        st_sum[s] += qe;
        st_pos[s] += 1;
        int32_t k = rung_of(st_sum[s], st_n[s], tau_q, K);
        if (n_high && k >= k_high && n_high[s] >= budget) k = k_high - 1;
        st_k_cur[s] = k;
        const int32_t rc = ranks[k];
        const double sc = rc > 0 ? (double)scales[k] : 0.0;
        const int32_t j_off = st_n[s] - 1;
        if (st_chunks[s] == 0 || blend_w == 0 || j_off >= blend_w) {
            r_cur[s] = rc;  g_cur[s] = sc;
            r_prev[s] = 0;  g_prev[s] = 0.0;
        } else {
            const int32_t kp = st_k_prev[s];
            const int32_t rp = ranks[kp];
            const double sp = rp > 0 ? (double)scales[kp] : 0.0;
            const double lambda = (double)(j_off + 1) / (double)(blend_w + 1);
            r_cur[s] = rc;  g_cur[s] = lambda * sc;
            r_prev[s] = rp; g_prev[s] = (1.0 - lambda) * sp;
        }
    }
    free(bclose);
    return CWL_REF_OK;
}

/* ------------------------------------------------------------------------------------------------
 * KV-cache policy per chunk (Sec. III-E, the KV-cache policy controller; Sec. IV-F).  The paper
 * lets chunk difficulty drive the memory policy: on easy spans selected heads may be stored in
 * INT8, hard spans keep full fidelity, and the policy is toggled per chunk.  It gives no rule, no
 * granularity of the scales and no layout.  Reading taken:
 *   - a chunk is "easy" when its rung is below k_keep (0 <= rank_idx[c] < k_keep); a rung outside
 *     the ladder's index range below zero counts as hard;
 *   - every head of an easy chunk's rows is quantised (no head subset), symmetric, one scale per
 *     (row, head): amax = max |x| over the head (NaN ignored), scale = amax / 127,
 *     code = round-to-nearest-even(x * (127 / amax)) clamped to [-127, 127], all in fp32 (the
 *     precision the kernel decides the integer in); amax = 0 gives scale 0 and codes 0; a NaN
 *     element has code 0;
 *   - layout: two pools.  Rows of easy chunks, in table order and row order inside a chunk, take the
 *     next free row of the INT8 pool (codes [., H*D], scales [., H]); rows of the other chunks take
 *     the next free row of the full-fidelity pool, copied bit for bit.  slot[t] >= 0: row of the INT8
 *     pool; slot[t] <= -1: row -1 - slot[t] of the full pool; rows that no chunk covers are not
 *     cached (slot = INT32_MIN).
 * kv holds the exact bf16 values widened to fp32.  counts[0] / counts[1]: rows in the INT8 / full pool.
 * ------------------------------------------------------------------------------------------------ */
#define CWL_REF_SLOT_ABSENT INT32_MIN

int cwl_ref_kv_quantise(const float* kv, int64_t n_rows, int32_t n_heads, int32_t head_dim,
                        const int32_t* chunk_start, const int32_t* chunk_len, const int32_t* rank_idx,
                        int64_t n_chunks, int32_t k_keep, int32_t* slot, int8_t* codes, float* scale,
                        float* kept, int64_t* counts) {
    if (n_rows < 0 || n_heads < 1 || head_dim < 1 || n_chunks < 0) return CWL_REF_ERR_INVALID;
    const int64_t width = (int64_t)n_heads * head_dim;
    for (int64_t t = 0; t < n_rows; ++t) slot[t] = CWL_REF_SLOT_ABSENT;
    int64_t nq = 0, nf = 0;
    for (int64_t c = 0; c < n_chunks; ++c) {
        const int easy = rank_idx[c] >= 0 && rank_idx[c] < k_keep;
        for (int32_t j = 0; j < chunk_len[c]; ++j) {
            const int64_t t = (int64_t)chunk_start[c] + j;
            if (t < 0 || t >= n_rows) return CWL_REF_ERR_INVALID;
            const float* row = kv + t * width;
            if (!easy) {
                slot[t] = (int32_t)(-1 - nf);
                memcpy(kept + nf * width, row, sizeof(float) * (size_t)width);
                ++nf;
                continue;
            }
            slot[t] = (int32_t)nq;
            for (int32_t h = 0; h < n_heads; ++h) {
                const float* x = row + (int64_t)h * head_dim;
                float amax = 0.0f;
                for (int32_t i = 0; i < head_dim; ++i) {
                    const float a = fabsf(x[i]);
                    if (a > amax) amax = a;          /* a NaN compares false: ignored */
                }
                const float inv = amax > 0.0f ? 127.0f / amax : 0.0f;
                scale[nq * n_heads + h] = amax / 127.0f;
                for (int32_t i = 0; i < head_dim; ++i) {
                    const float v = x[i] * inv;
                    int32_t code = 0;
                    if (v == v) {
                        const float r = rintf(v);        /* default rounding mode: nearest, ties to even */
                        code = r > 127.0f ? 127 : (r < -127.0f ? -127 : (int32_t)r);
                    }
                    codes[nq * width + (int64_t)h * head_dim + i] = (int8_t)code;
                }
            }
            ++nq;
        }
    }
    counts[0] = nq;
    counts[1] = nf;
    return CWL_REF_OK;
}
