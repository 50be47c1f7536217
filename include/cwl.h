/*
 * cwl.h -- C ABI of the ChunkWise LoRA hot path for AMD MI355X (gfx950).
 *
 * The four calls follow the pipeline of arxiv 2601.21109, Sec. III (A: token complexity
 * estimator, B: adaptive chunker, C: per-chunk rank & scale selector, D: boundary-safe composer
 * on the LoRA projection):
 *
 *      cwl_score_tokens  ->  cwl_partition_chunks  ->  cwl_select_ranks  ->  cwl_chunkwise_lora_linear
 *
 * Around them: cwl_compose_scores (the other difficulty signals of Sec. III-A mixed into the score),
 * cwl_select_ranks_budget / cwl_bucket_sequences / cwl_partition_chunks_aligned (the chunker's budget
 * and the batch controller of Sec. III-G and IV-F), cwl_stream_step[_aligned] +
 * cwl_gated_lora_linear_packed (the same rules one token per sequence at a time, for decoding),
 * cwl_schedule_chunks + cwl_lora_shrink_packed + cwl_chunkwise_lora_linear_packed_shrunk (the same
 * pipeline in five launches: the part of the layer that needs no chunk table rides in the chunker's
 * launch), cwl_kv_quantise_chunks / cwl_kv_dequantise (the chunk-level KV-cache policy of Sec. III-E),
 * and the set-up calls cwl_prepack_weights and cwl_build_ladder (the ladder of Sec. III-C by one SVD).
 *
 * General rules
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - The caller owns every buffer.  The library never allocates, frees or synchronises; every
 *     call only enqueues kernels on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  Scratch memory comes in through the `workspace` arguments, sized by the matching
 *     *_workspace_bytes() query; workspaces must be 256-byte aligned.
 *   - All matrices are row-major.  Leading dimensions are in elements.
 *   - Argument errors are detected on the host before anything is launched and returned
 *     synchronously.  Data-dependent conditions are reported through a device status word.
 *   - Token rows, chunk indices and sequence offsets are 32-bit: n_rows < 2^31.
 *   - Results are deterministic: the same inputs give bitwise identical outputs.
 *   - Calls work on the current HIP device; pointers and `stream` must belong to it.  The library
 *     keeps a little set-once host state per device (kernel attributes, the number of compute
 *     units) without locking: the first call of an entry point on a device should not run
 *     concurrently with another host thread's first call on the same device.
 */
#ifndef CWL_H
#define CWL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    CWL_OK = 0,
    CWL_ERR_NULL = 1,          /* a required pointer is NULL                                  */
    CWL_ERR_INVALID_ARG = 2,   /* a size, stride, ladder or threshold is out of range         */
    CWL_ERR_INFEASIBLE = 3,    /* l_max < 2*l_min - 1: the length bounds cannot always be met */
    CWL_ERR_CAPACITY = 4,      /* a caller-provided buffer or workspace is too small          */
    CWL_ERR_UNSUPPORTED = 5,   /* shape / dtype combination the kernels do not cover          */
    CWL_ERR_DEVICE = 6         /* the HIP runtime refused a launch                            */
} cwl_status;

typedef enum { CWL_F32 = 0, CWL_BF16 = 1 } cwl_dtype;

/* Bits of the device status word written by cwl_partition_chunks(_aligned). */
#define CWL_STATUS_CAPACITY 1u     /* more chunks than `cap`; only the first cap were written  */
#define CWL_STATUS_NAN_SCORE 2u    /* a NaN score was met and scored as 0                      */
#define CWL_STATUS_BAD_OFFSETS 4u  /* seq_offsets not non-decreasing within [0, n_rows]        */
#define CWL_STATUS_BAD_BUCKET 8u   /* a bucket index outside [0, n_buckets) (taken as the nearest) */

#define CWL_MAX_LADDER 16          /* largest K (rungs of the rank ladder)                     */
#define CWL_MAX_RANK 256           /* largest r_max                                            */

const char* cwl_status_string(cwl_status s);   /* static string, never NULL */
int32_t cwl_abi_version(void);

/* ---------------------------------------------------------------------------------------------
 * cwl_score_tokens -- per-token difficulty score (Sec. III-A, signal (i); Sec. IV-A):
 * the entropy, in nats, of the next-token distribution softmax(logits[t, :]).
 *
 *   logits      [n_rows, vocab], element type `dt`, row t starts at logits + t*row_stride
 *   row_stride  in elements, >= vocab
 *   entropy     [n_rows] fp32, written
 *
 * Accumulation is fp32.  A logit of -inf has probability 0; a row holding NaN or +inf, or made
 * of -inf only, scores NaN.  n_rows == 0 is a no-op.  vocab must be >= 1.
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_score_tokens(const void* logits, cwl_dtype dt, int64_t n_rows, int64_t vocab,
                            int64_t row_stride, float* entropy, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_compose_scores -- composite difficulty score (Sec. III-A names, next to the entropy, an
 * n-gram novelty signal against the recent context and a small positional prior that favours
 * early steps; no formula or weight is given, this is the reading taken).  For token t at position
 * j of its sequence:
 *      novelty_t = 1 if the n-gram of token ids ending at j ends at none of the positions j' with
 *                  max(n-1, j-window) <= j' < j of the same sequence (tokens with j < n-1 count
 *                  as new), else 0
 *      prior_t   = max(0, 1 - j / prior_len)         (0 when prior_len <= 0)
 *      score_t   = w_entropy * entropy_t + w_novelty * novelty_t + w_prior * prior_t     (fp32)
 * A row outside every sequence gets w_entropy * entropy_t and novelty 0.  The result is a score in
 * the units of its weights; with the weights in nats it can be handed to cwl_partition_chunks in
 * place of the entropy.
 *
 *   entropy     [n_rows] fp32        token_ids   [n_rows] int32
 *   seq_offsets [n_seqs+1]           m           host; 1 <= n <= 8, 0 <= window <= 4096 (else
 *                                                CWL_ERR_UNSUPPORTED)
 *   score       [n_rows] fp32, written (may alias entropy)
 *   novelty     [n_rows] int32, written when not NULL
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t n, window;
    float w_entropy, w_novelty, w_prior;
    float prior_len;
} cwl_score_mix;

cwl_status cwl_compose_scores(const float* entropy, const int32_t* token_ids, int64_t n_rows,
                              const int32_t* seq_offsets, int32_t n_seqs, const cwl_score_mix* m /*host*/,
                              float* score, int32_t* novelty, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_partition_chunks -- adaptive chunker (Sec. III-B, Sec. IV-B).
 *
 * Scores are first turned into Q10 fixed-point integers q = floor(h*1024 + 0.5) (fp32; NaN and
 * negatives -> 0, clamped to 2^20) so that every later decision is an integer one.  Each
 * sequence is then cut greedily, left to right: a chunk opened at p closes at the first end e
 * (chunk = [p, e)), p+l_min <= e <= p+l_max, that leaves either no tail or a tail of at least
 * l_min tokens, and at which, with S = sum of q over the chunk and n = e-p,
 *      S >= theta_q*n          (the chunk's mean reached the average-complexity threshold), or
 *      q[e] >= theta_q         (the next token is itself hard and opens a new chunk), or
 *      |q[e]*n - S| > delta_q*n (the next token leaves the chunk's regime);
 * if none fires, at the last such end.  A sequence shorter than l_min becomes one chunk.  So
 * hard spans are cut every l_min tokens and easy spans grow to l_max.
 *
 *   entropy        [n_rows] fp32 scores
 *   seq_offsets    [n_seqs+1] first row of each sequence; seq_offsets[n_seqs] == n_rows
 *   p              host; 1 <= l_min <= l_max, l_max >= 2*l_min-1 (else CWL_ERR_INFEASIBLE);
 *                  theta_hard / delta_dev in nats, +INF disables the test
 *   chunk_offsets  [n_seqs+1] written: index of the first chunk of each sequence (CSR)
 *   chunk_start    [cap] written: first global row of the chunk
 *   chunk_len      [cap] written
 *   chunk_sum      [cap] written: sum of q over the chunk (int64)
 *   cap            capacity of the three chunk arrays; n_rows/l_min + n_seqs always suffices
 *   status_word    one int32, written: 0 or an OR of CWL_STATUS_* bits
 *   workspace      >= cwl_partition_workspace_bytes(n_rows, n_seqs, p) bytes
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int32_t l_min, l_max;
    float theta_hard;
    float delta_dev;
} cwl_chunk_params;

size_t cwl_partition_workspace_bytes(int64_t n_rows, int32_t n_seqs, const cwl_chunk_params* p);

cwl_status cwl_partition_chunks(const float* entropy, int64_t n_rows, const int32_t* seq_offsets,
                                int32_t n_seqs, const cwl_chunk_params* p /*host*/,
                                int32_t* chunk_offsets, int32_t* chunk_start, int32_t* chunk_len,
                                int64_t* chunk_sum, int32_t cap, int32_t* status_word,
                                void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_select_ranks -- per-chunk rung of the rank ladder (Sec. III-C; Sec. IV-C, a rule that maps
 * score percentiles to rungs): rank_idx[c] = #{ j : chunk_sum[c] >= tau_q[j] * chunk_len[c] }, where
 * tau_q[j] is thresholds[j] quantised like the scores.  A mean exactly on a threshold goes up.
 *
 *   chunk_sum, chunk_len, chunk_offsets   as written by cwl_partition_chunks
 *   cap          capacity of chunk_sum / chunk_len / rank_idx; chunks beyond it are ignored
 *   thresholds   host, [K-1], ascending, nats (the percentile table)
 *   K            rungs of the ladder, 1 <= K <= CWL_MAX_LADDER
 *   rank_idx     [cap] written for every existing chunk: 0 .. K-1
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_select_ranks(const int64_t* chunk_sum, const int32_t* chunk_len,
                            const int32_t* chunk_offsets, int32_t n_seqs, int32_t cap,
                            const float* thresholds /*host*/, int32_t K, int32_t* rank_idx,
                            void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_select_ranks_budget -- cwl_select_ranks under a budget of high-capacity regions per sequence
 * (Sec. III-B lists such a budget among the chunker's constraints).  A chunk asks for high capacity
 * when the rung cwl_select_ranks gives it is >= k_high.  The chunks of a sequence are taken in
 * order, as the online chunker meets them: the first `budget` that ask keep their rung, every later
 * one that asks gets rung k_high - 1.
 *
 *   k_high   >= 1 (k_high >= K: no chunk asks)        budget   >= 0
 *   n_asked  [n_seqs] written when not NULL: chunks of each sequence that asked
 *   the other arguments as for cwl_select_ranks
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_select_ranks_budget(const int64_t* chunk_sum, const int32_t* chunk_len,
                                   const int32_t* chunk_offsets, int32_t n_seqs, int32_t cap,
                                   const float* thresholds /*host*/, int32_t K, int32_t k_high,
                                   int32_t budget, int32_t* rank_idx, int32_t* n_asked, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_bucket_sequences -- buckets of the sequences of a batch by complexity percentile (Sec. III-G)
 * and complexity-balanced micro-batches (Sec. IV-F).  The complexity of a sequence is the mean of
 * its scores, quantised as in cwl_partition_chunks: m_s = floor(seq_sum[s] / T_s), 0 when empty.
 * Sequences are ranked by (m_s, s) ascending, order[rho] = the sequence of rank rho, and
 *      bucket[s] = floor(rho_s * n_buckets / n_seqs)          equal-count percentile bins,
 *      micro[s]  = j in even rounds, n_micro-1-j in odd ones,   round = rho_s / n_micro, j = rho_s % n_micro
 * (the ranked order dealt out in alternating direction: micro-batches of equal size within one
 * whose total complexities differ by no more than the spread of m over the batch).
 *
 *   score [n_rows] fp32     seq_offsets [n_seqs+1]     n_seqs <= 4096 (else CWL_ERR_UNSUPPORTED)
 *   n_buckets >= 1          n_micro >= 1 when micro is not NULL
 *   seq_sum [n_seqs] int64, order / bucket [n_seqs] int32: written;  micro [n_seqs] written when not NULL
 * A malformed seq_offsets entry counts as an empty sequence.
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_bucket_sequences(const float* score, int64_t n_rows, const int32_t* seq_offsets,
                                int32_t n_seqs, int32_t n_buckets, int32_t n_micro, int64_t* seq_sum,
                                int32_t* order, int32_t* bucket, int32_t* micro, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_partition_chunks_aligned -- the chunker with boundaries aligned inside each bucket
 * (Sec. III-G: boundaries are aligned by bucketing the sequences, each sequence keeps its own
 * rank choices).  The sequences of a bucket share the boundaries that the rule of
 * cwl_partition_chunks places on the bucket's mean series
 *      m_b[t] = floor( sum of q_s[t] over the members s with T_s > t  /  their number ),
 * t < the longest member.  A member takes every boundary inside it, its chunks are
 * [e_i, min(e_{i+1}, T_s)) for the bucket's chunk starts e_i < T_s, so only its last chunk can be
 * shorter than the bucket's (and than l_min); chunk_sum holds the member's own scores.  With one
 * sequence per bucket the result is that of cwl_partition_chunks.
 *
 *   bucket   [n_seqs] device, values in [0, n_buckets) (e.g. from cwl_bucket_sequences); a value
 *            outside is taken as the nearest bucket and sets CWL_STATUS_BAD_BUCKET
 *   n_seqs, n_buckets <= 4096 (else CWL_ERR_UNSUPPORTED)
 *   workspace >= cwl_aligned_workspace_bytes(n_rows, n_seqs, n_buckets, p) bytes
 *   the other arguments, the outputs and the status word as for cwl_partition_chunks
 * ------------------------------------------------------------------------------------------- */
size_t cwl_aligned_workspace_bytes(int64_t n_rows, int32_t n_seqs, int32_t n_buckets,
                                   const cwl_chunk_params* p);

cwl_status cwl_partition_chunks_aligned(const float* score, int64_t n_rows, const int32_t* seq_offsets,
                                        int32_t n_seqs, const int32_t* bucket, int32_t n_buckets,
                                        const cwl_chunk_params* p /*host*/, int32_t* chunk_offsets,
                                        int32_t* chunk_start, int32_t* chunk_len, int64_t* chunk_sum,
                                        int32_t cap, int32_t* status_word, void* workspace,
                                        size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_chunkwise_lora_linear -- the chunk-segmented, variable-rank LoRA projection with the
 * boundary cross-fade (Sec. III-C: slice the first r directions of the stored factors;
 * Sec. III-D: outgoing adapter ramps down linearly while the incoming one ramps up).
 *
 * For token t in chunk c (rung k = rank_idx[c], r = ranks[k], s = scales[k]) at offset
 * j = t - chunk_start[c]:
 *      D_k(t) = s_k * (x_t . A[:, :r_k]) . B[:r_k, :]
 *      y_t = x_t W + D_k(t)                                   first chunk of its sequence,
 *                                                             or j >= blend_w, or blend_w == 0
 *      y_t = x_t W + (1-l)*D_{k'}(t) + l*D_k(t),  l=(j+1)/(blend_w+1),  k' = rung of chunk c-1
 * A rung of rank 0 adds nothing.  A token no chunk covers, or whose rank_idx is outside
 * [0, K), gets the base product only.
 *
 *   x [n_rows, d_in] (ldx)    W [d_in, d_out] (ldw)    A [d_in, r_max] (lda)
 *   B [r_max, d_out] (ldb)    y [n_rows, d_out] (ldy), written; all of element type `dt`
 *   ranks   host [K], ascending, 0 <= ranks[k] <= r_max      scales  host [K]
 *   blend_w >= 0
 *   seq_offsets / chunk_offsets / chunk_start / chunk_len / rank_idx: the chunk table as written
 *   by cwl_partition_chunks and cwl_select_ranks; chunk_cap is the capacity of the three
 *   per-chunk arrays (chunks at or beyond it are treated as absent)
 *
 * CWL_F32 : fp32 FMA arithmetic.  CWL_BF16: bf16 operands on the matrix cores, fp32
 * accumulation, the gated shrink output is rounded to bf16 once, y is rounded to bf16 once.
 * CWL_BF16 needs d_in % 64 == 0 and d_out % 8 == 0, 16-byte aligned x / y and ldx % 8 == 0,
 * ldy % 8 == 0 (else CWL_ERR_UNSUPPORTED).
 *
 * The launch plan depends on the shape (up to 512 rows: the weights are streamed once by several
 * hundred workgroups, each over a slice of d_in, and a second kernel adds the slices in a fixed
 * order; otherwise output tiles of 128 x 128 to 256 x 256); the arithmetic stated above does not,
 * and a call gives the same bits every time.
 *
 * The static weights can be re-laid out once with cwl_prepack_weights (K-contiguous, padded
 * ladder) and then used through cwl_chunkwise_lora_linear_packed; the plain entry point does
 * the same re-layout into its workspace on every call.
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int64_t n_rows, d_in, d_out;
    int32_t r_max, K;
    const int32_t* ranks;    /* host [K] */
    const float* scales;     /* host [K] */
    int32_t blend_w;
    cwl_dtype dt;
    int64_t ldx, ldw, lda, ldb, ldy;
    int32_t group_rows;      /* 0: rows in token order; 1: group token rows by rank bucket so
                                that row tiles are rank-homogeneous (same result; from 65536
                                rows up the fp32 sums of x A run in another order, so the last
                                bit of a bf16 output may differ between the two settings)      */
} cwl_linear_desc;

size_t cwl_packed_weights_bytes(const cwl_linear_desc* d);
cwl_status cwl_prepack_weights(const cwl_linear_desc* d, const void* W, const void* A,
                               const void* B, void* packed, size_t packed_bytes, void* stream);

size_t cwl_linear_workspace_bytes(const cwl_linear_desc* d);          /* plain entry point  */
size_t cwl_linear_packed_workspace_bytes(const cwl_linear_desc* d);   /* packed entry point */

cwl_status cwl_chunkwise_lora_linear(const cwl_linear_desc* d, const void* x, const void* W,
                                     const void* A, const void* B, const int32_t* seq_offsets,
                                     int32_t n_seqs, const int32_t* chunk_offsets,
                                     const int32_t* chunk_start, const int32_t* chunk_len,
                                     const int32_t* rank_idx, int32_t chunk_cap, void* y,
                                     void* workspace, size_t workspace_bytes, void* stream);

cwl_status cwl_chunkwise_lora_linear_packed(const cwl_linear_desc* d, const void* x,
                                            const void* packed, const int32_t* seq_offsets,
                                            int32_t n_seqs, const int32_t* chunk_offsets,
                                            const int32_t* chunk_start, const int32_t* chunk_len,
                                            const int32_t* rank_idx, int32_t chunk_cap, void* y,
                                            void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * The layer in two phases (Sec. III-C: the rank slice is an index operation over the stored
 * factors, so the product with all stored directions does not depend on the scheduler's decisions).
 *
 *   cwl_lora_shrink_packed                    u = x A, every stored direction, fp32, no gate.  It
 *                                             reads x and the packed adapter only, NOT the chunk
 *                                             table: it may be enqueued before the scores exist, or
 *                                             on a second stream beside cwl_partition_chunks and
 *                                             cwl_select_ranks, which occupy a few compute units.
 *   cwl_chunkwise_lora_linear_packed_shrunk   the rest of cwl_chunkwise_lora_linear_packed: the
 *                                             gate of the chunk table applied to u (rounded to the
 *                                             element type once, as the one-call form rounds it),
 *                                             then y = x W + uhat B.
 *
 * Together they compute what cwl_chunkwise_lora_linear_packed computes, with the same kernels in the
 * same order of summation (bit for bit the same y; a direction that the one-call form skips because
 * no row of its block uses it is computed here and multiplied by a zero gate).  `u` is an opaque
 * device buffer of cwl_lora_shrink_bytes(d) bytes, 256-byte aligned, written by the first call and
 * read by the second; the caller orders the two (same stream, or an event) and must not change x in
 * between.  Both calls take the same descriptor.  group_rows must be 0 (CWL_ERR_UNSUPPORTED).
 * Up to 512 rows the whole layer is one product, the first call enqueues nothing and the second is
 * the one-call form.
 * ------------------------------------------------------------------------------------------- */
size_t cwl_lora_shrink_bytes(const cwl_linear_desc* d);      /* 0: descriptor rejected */

cwl_status cwl_lora_shrink_packed(const cwl_linear_desc* d, const void* x, const void* packed,
                                  void* u, size_t u_bytes, void* stream);

cwl_status cwl_chunkwise_lora_linear_packed_shrunk(const cwl_linear_desc* d, const void* x,
                                                   const void* packed, const void* u, size_t u_bytes,
                                                   const int32_t* seq_offsets, int32_t n_seqs,
                                                   const int32_t* chunk_offsets, const int32_t* chunk_start,
                                                   const int32_t* chunk_len, const int32_t* rank_idx,
                                                   int32_t chunk_cap, void* y, void* workspace,
                                                   size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_schedule_chunks -- the scheduler as one call: cwl_partition_chunks (Sec. III-B, IV-B) and
 * cwl_select_ranks (Sec. III-C, IV-C) with the same arguments and the same table and rungs, bit for
 * bit; a chunk's rung is decided by the kernel that writes its record.  When `shrink` is not NULL
 * the call also does what cwl_lora_shrink_packed(shrink, x, packed, u, u_bytes) does, and where the
 * shapes allow it (sequences of 4096 tokens or fewer on average, bf16, 16384 .. 65535 rows, r_max
 * <= 128) the product's workgroups ride in the chunker's launch: the chunk walk is a chain of
 * dependent look-ups that keeps one wavefront per sequence busy, the product streams x from HBM and
 * needs nothing the chunker writes, so the two cost little more than the longer of them.  Elsewhere
 * the product is launched behind the chunker; the results are the same either way.
 *
 *   the chunker's and the selector's arguments as in cwl_partition_chunks / cwl_select_ranks
 *   (rank_idx [cap] written);  shrink, x, packed, u, u_bytes as in cwl_lora_shrink_packed, or
 *   shrink == NULL: the scheduler alone.
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_schedule_chunks(const float* entropy, int64_t n_rows, const int32_t* seq_offsets,
                               int32_t n_seqs, const cwl_chunk_params* p /*host*/,
                               const float* thresholds /*host*/, int32_t K, int32_t* chunk_offsets,
                               int32_t* chunk_start, int32_t* chunk_len, int64_t* chunk_sum,
                               int32_t* rank_idx, int32_t cap, int32_t* status_word, void* workspace,
                               size_t workspace_bytes, const cwl_linear_desc* shrink /*host, may be NULL*/,
                               const void* x, const void* packed, void* u, size_t u_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_chunkwise_lora_linear_packed_static -- cwl_chunkwise_lora_linear_packed for callers that
 * cannot allocate device memory and have no workspace to hand over: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same
 * bits in y; the scratch memory is an array of CWL_STATIC_SCRATCH_BYTES that the library holds in
 * the device's memory from the moment it is loaded until the process ends (one copy per GPU).  The
 * call allocates and frees nothing; its first call on a device looks up the array's address there.
 *
 *   CWL_ERR_CAPACITY   the descriptor needs more than CWL_STATIC_SCRATCH_BYTES
 *                      (cwl_linear_packed_workspace_bytes(d) says how much); nothing is launched
 *
 * Every call on one GPU uses the same array: calls that may overlap on one GPU (two streams, two
 * host threads) race and must be ordered by the caller.  The array keeps the last call's contents;
 * nothing in it has to start at zero, every kernel reads only what the same call wrote.
 * ------------------------------------------------------------------------------------------- */
#define CWL_STATIC_SCRATCH_BYTES ((size_t)16 << 20)

cwl_status cwl_chunkwise_lora_linear_packed_static(const cwl_linear_desc* d, const void* x,
                                                   const void* packed, const int32_t* seq_offsets,
                                                   int32_t n_seqs, const int32_t* chunk_offsets,
                                                   const int32_t* chunk_start, const int32_t* chunk_len,
                                                   const int32_t* rank_idx, int32_t chunk_cap, void* y,
                                                   void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_stream_step -- the chunker, the selector and the cross-fade one token at a time (Sec. III-A
 * and III-B run the estimator and the chunker while decoding; Sec. III-F keeps the scheduler's state
 * between steps).  One call consumes ONE new token per sequence: its score, quantised as in
 * cwl_partition_chunks, is tested against the sequence's open chunk (n tokens, score sum S) exactly
 * as the batch chunker tests an end in front of that token: if n >= l_min and
 *      n == l_max,  or  S >= theta_q*n,  or  q >= theta_q,  or  |q*n - S| > delta_q*n
 * the chunk is closed and the token opens the next one, else the token joins the open chunk.  The
 * end of the sequence is unknown here, so the batch rule that never leaves a tail shorter than
 * l_min has no counterpart: both forms place the same boundaries for every chunk that starts at
 * least l_min + l_max tokens before the end.  The rung in force for the token is the selector's
 * rule on the open chunk with the token included, k = #{ j : S >= tau_q[j]*n }; at the last token
 * of a chunk that is the rung cwl_select_ranks gives the whole chunk.  Its gate entry is
 *      (r_cur, s_cur, 0, 0)                                       first chunk of the sequence,
 *                                                                 blend_w == 0, or offset j >= blend_w
 *      (r_cur, l*s_cur, r_prev, (1-l)*s_prev),  l = (j+1)/(blend_w+1)    otherwise,
 * r_prev / s_prev being those of the rung the previous chunk ended with; a rung of rank 0 has
 * scale 0.  cwl_gated_lora_linear_packed applies such entries.
 *
 *   entropy      [n_seqs] fp32: the score of each sequence's new token (e.g. from cwl_score_tokens)
 *   p, thresholds, K   as for cwl_partition_chunks / cwl_select_ranks (host)
 *   ranks, scales      host [K], as in cwl_linear_desc
 *   state        [n_seqs] in/out; all-zero bytes start a sequence
 *   gate         [n_seqs] written
 *   closed_len / closed_sum   [n_seqs] written when not NULL: length and score sum of the chunk
 *                this token closed, 0 when it closed none
 *   status_word  one int32, OR-ed with CWL_STATUS_NAN_SCORE when a score is NaN (scored as 0);
 *                the caller clears it
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int64_t sum;        /* score sum of the open chunk                          */
    int64_t pos;        /* tokens seen                                           */
    int32_t n;          /* tokens in the open chunk                              */
    int32_t n_chunks;   /* chunks closed                                         */
    int32_t k_cur;      /* rung in force at the latest token                     */
    int32_t k_prev;     /* rung the previous chunk ended with (once one closed)  */
} cwl_stream_state;

typedef struct {
    int32_t r_cur, r_prev;
    float g_cur, g_prev;
} cwl_token_gate;

cwl_status cwl_stream_step(const float* entropy, int32_t n_seqs, const cwl_chunk_params* p /*host*/,
                           const float* thresholds /*host*/, int32_t K, const int32_t* ranks /*host*/,
                           const float* scales /*host*/, int32_t blend_w, cwl_stream_state* state,
                           cwl_token_gate* gate, int32_t* closed_len, int64_t* closed_sum,
                           int32_t* status_word, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_stream_step_aligned -- cwl_stream_step for a batch under the batch controller: boundaries
 * aligned inside each bucket (Sec. III-G, which speaks of batched decoding) and the budget of
 * high-capacity chunks (Sec. III-B).  Two changes to cwl_stream_step:
 *   bucket != NULL: every bucket keeps an open chunk of its own on the bucket's mean series
 * (bucket_state: n tokens, sum).  With qm = floor(sum of the members' new quantised scores / number
 * of members in the call), the close test of cwl_stream_step is taken once per bucket on
 * (n, sum, qm); when it fires every member closes its own open chunk, if it has one, in front of
 * its new token; the bucket's chunk then takes qm.  A bucket with no member in the call keeps its
 * state.  Sequences of equal length fed token by token get the boundaries of
 * cwl_partition_chunks_aligned wherever the end cannot matter.
 *   n_high != NULL: n_high[s] counts the closed chunks of sequence s whose last token had a rung
 * >= k_high before any lowering (the chunk's rung in the batch form).  The rung in force for a
 * token is lowered to k_high - 1 when it is >= k_high and n_high[s] >= budget, so every chunk ends
 * on the rung cwl_select_ranks_budget gives it.
 * With bucket == NULL and n_high == NULL this is cwl_stream_step.
 *
 *   bucket        [n_seqs] device or NULL; values in [0, n_buckets), else the nearest bucket and
 *                 CWL_STATUS_BAD_BUCKET; needs n_seqs, n_buckets <= 4096 (else CWL_ERR_UNSUPPORTED)
 *   bucket_state  [n_buckets] in/out, all-zero bytes at the start
 *   k_high >= 1, budget >= 0 (read when n_high != NULL)     n_high  [n_seqs] in/out, zero at the start
 *   the other arguments as for cwl_stream_step
 * ------------------------------------------------------------------------------------------- */
typedef struct {
    int64_t sum;        /* sum of the mean series over the bucket's open chunk */
    int32_t n;          /* tokens in it                                        */
    int32_t reserved;
} cwl_bucket_state;

cwl_status cwl_stream_step_aligned(const float* entropy, int32_t n_seqs, const cwl_chunk_params* p /*host*/,
                                   const float* thresholds /*host*/, int32_t K, const int32_t* ranks /*host*/,
                                   const float* scales /*host*/, int32_t blend_w, const int32_t* bucket,
                                   int32_t n_buckets, cwl_bucket_state* bucket_state, int32_t k_high,
                                   int32_t budget, int32_t* n_high, cwl_stream_state* state,
                                   cwl_token_gate* gate, int32_t* closed_len, int64_t* closed_sum,
                                   int32_t* status_word, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_gated_lora_linear_packed -- the layer of cwl_chunkwise_lora_linear for rows that bring their
 * own gate entry (Sec. III-C sliced ladder, Sec. III-D cross-fade, weights already decided), e.g.
 * the one token per sequence of a decode step:
 *      y_t = x_t W + g_cur(t) (x_t . A[:, :r_cur(t)]) . B[:r_cur(t), :]
 *                  + g_prev(t) (x_t . A[:, :r_prev(t)]) . B[:r_prev(t), :]
 * Ranks outside [0, r_max] are clipped.  `d`, `packed`, the workspace size and the arithmetic are
 * those of cwl_chunkwise_lora_linear_packed; ranks, scales, K and blend_w of `d` must be valid
 * but are not used, group_rows must be 0.
 *
 *   gate   [n_rows] device
 * ------------------------------------------------------------------------------------------- */
cwl_status cwl_gated_lora_linear_packed(const cwl_linear_desc* d, const void* x, const void* packed,
                                        const cwl_token_gate* gate, void* y, void* workspace,
                                        size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Projections that share their input (Sec. III-C and III-F: every LoRA-carrying projection of a layer
 * slices its own ladder under the one chunk table; q/k/v read the same x, so do gate/up).  A group
 * is 1 .. CWL_MAX_GROUP projections p with the same d_in, r_max, ladder and element type, each with
 * its own W_p [d_in, d_out_p], A_p [d_in, r_max], B_p [r_max, d_out_p] (all contiguous, row-major).
 * The grouped calls give exactly the layer of cwl_chunkwise_lora_linear for every projection,
 *      y[:, c_p : c_p + d_out_p] = x W_p + (gated x A_p[:, :r]) B_p[:r, :],    c_p = d_out_0 + .. + d_out_{p-1},
 * every projection on the prefixes of ITS OWN factors, in one wide output y [n_rows, sum d_out_p]:
 * the gate table is made once, one shrink pass over x serves the adapters of all projections (below
 * 65536 rows as many as have 256 directions together per pass), and up to 512 rows the weights of all
 * projections are streamed by one launch.  In `d`: d_out = sum of d_out_p, ldw / lda / ldb are not used,
 * group_rows must be 0.  Sums may run in another order than in the single-projection calls.
 *
 *   cwl_group.W / A / B   device pointers, read by cwl_prepack_weights_grouped only
 *   packed     >= cwl_packed_weights_grouped_bytes(d, g) bytes, 256-byte aligned
 *   workspace  >= cwl_linear_grouped_workspace_bytes(d, g) bytes
 *   the other arguments as for cwl_chunkwise_lora_linear_packed / cwl_gated_lora_linear_packed
 * ------------------------------------------------------------------------------------------- */
#define CWL_MAX_GROUP 8

typedef struct {
    int32_t n_proj;
    int64_t d_out[CWL_MAX_GROUP];
    const void* W[CWL_MAX_GROUP];
    const void* A[CWL_MAX_GROUP];
    const void* B[CWL_MAX_GROUP];
} cwl_group;

size_t cwl_packed_weights_grouped_bytes(const cwl_linear_desc* d, const cwl_group* g /*host*/);
size_t cwl_linear_grouped_workspace_bytes(const cwl_linear_desc* d, const cwl_group* g /*host*/);

cwl_status cwl_prepack_weights_grouped(const cwl_linear_desc* d, const cwl_group* g /*host*/, void* packed,
                                       size_t packed_bytes, void* stream);

cwl_status cwl_chunkwise_lora_linear_grouped_packed(const cwl_linear_desc* d, const cwl_group* g /*host*/,
                                                    const void* x, const void* packed,
                                                    const int32_t* seq_offsets, int32_t n_seqs,
                                                    const int32_t* chunk_offsets, const int32_t* chunk_start,
                                                    const int32_t* chunk_len, const int32_t* rank_idx,
                                                    int32_t chunk_cap, void* y, void* workspace,
                                                    size_t workspace_bytes, void* stream);

cwl_status cwl_gated_lora_linear_grouped_packed(const cwl_linear_desc* d, const cwl_group* g /*host*/,
                                                const void* x, const void* packed, const cwl_token_gate* gate,
                                                void* y, void* workspace, size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_build_ladder -- the rank ladder of a trained adapter (Sec. III-C: obtained once by an SVD of
 * the adapter matrix; a rung then slices its first r directions).  With dW = A B = U diag(sigma) V^T,
 * sigma descending, the call writes
 *      A' = U[:, :r] diag(sqrt(sigma))        B' = diag(sqrt(sigma)) V^T[:r, :]
 * so that A' B' = dW and A'[:, :k] B'[:k, :] is the best rank-k approximation of dW for every k:
 * A' and B' are the factors cwl_chunkwise_lora_linear slices.  Directions whose singular value is
 * below 1e-12 of the largest carry nothing and come out as zero columns / rows with sigma = 0.
 * Singular vectors are fixed only up to sign (and rotation inside equal singular values); sigma and
 * the truncated products are unique.  Set-up work, run once per adapter; fp64 inside.
 *
 *   A [d_in, r] (lda)     B [r, d_out] (ldb)     element type `dt`, 1 <= r <= CWL_MAX_RANK
 *   A_out [d_in, r] (lda_out), B_out [r, d_out] (ldb_out): written, type `dt`; may be A and B
 *   sigma  [r] device, fp64, written
 *   workspace >= cwl_ladder_workspace_bytes(r) bytes, 256-byte aligned
 * ------------------------------------------------------------------------------------------- */
size_t cwl_ladder_workspace_bytes(int32_t r);

cwl_status cwl_build_ladder(cwl_dtype dt, const void* A, int64_t lda, const void* B, int64_t ldb,
                            int64_t d_in, int64_t d_out, int32_t r, void* A_out, int64_t lda_out,
                            void* B_out, int64_t ldb_out, double* sigma, void* workspace,
                            size_t workspace_bytes, void* stream);

/* ---------------------------------------------------------------------------------------------
 * cwl_kv_quantise_chunks / cwl_kv_dequantise -- the chunk-level KV-cache policy (Sec. III-E: chunk
 * difficulty drives the memory policy, easy spans may be stored in INT8, hard spans keep full
 * fidelity, the policy is toggled per chunk; Sec. IV-F).  The paper gives no rule, scale granularity
 * or layout; this call takes: a chunk is easy when its rung is below k_keep (0 <= rank_idx[c] <
 * k_keep); every head of an easy chunk's rows is quantised symmetrically with one fp32 scale per
 * (row, head): amax = max |x| over the head (a NaN element is ignored and gets code 0),
 *      scale = amax / 127,     code = round-to-nearest-even(x * (127 / amax)) in [-127, 127]
 * (fp32; amax == 0: scale 0, codes 0).  The cache is kept in two pools: rows of easy chunks take the
 * next rows of the INT8 pool, rows of the other chunks the next rows of the full pool, copied bit for
 * bit, both in table order and row order inside a chunk.  The sparsifying and windowing policies the
 * paper also names need attention weights and are not part of this library.
 *
 *   kv          bf16 [n_rows, n_heads * head_dim], leading dimension ld (elements); one of K or V
 *   chunk_offsets / chunk_start / chunk_len / rank_idx / chunk_cap   the chunk table as written by the
 *               chunker and the selector (chunk starts ascending); n_seqs sequences
 *   p           host: n_heads >= 1, head_dim in {32, 64, 128, 256, 512}, n_heads * head_dim <= 8192
 *               (else CWL_ERR_UNSUPPORTED), k_keep >= 0 (0: nothing is quantised)
 *   slot        [n_rows] written: >= 0 row of the INT8 pool; <= -1: row -1 - slot of the full pool;
 *               CWL_KV_SLOT_ABSENT: not cached (no chunk covers the row, or its pool is full)
 *   counts      [2] written: rows the INT8 pool / the full pool need for this table
 *   q_codes     int8 [cap_q, n_heads * head_dim], q_scale fp32 [cap_q, n_heads]: the INT8 pool
 *   f_pool      bf16 [cap_f, n_heads * head_dim]: the full pool; n_rows rows each always suffice
 *   status_word one int32, written: 0, or CWL_STATUS_CAPACITY when a pool was too small
 *   workspace   >= cwl_kv_workspace_bytes(chunk_cap) bytes, 256-byte aligned
 * 16-byte aligned kv / f_pool, 8-byte aligned q_codes, ld % 8 == 0 (else CWL_ERR_UNSUPPORTED).
 *
 * cwl_kv_dequantise reads the cache back as bf16 [n_rows, n_heads * head_dim] (ld_out): a full-pool
 * row as stored, an INT8 row as code * scale (fp32 product, rounded to bf16 once), an absent row as
 * zeros -- the form exact attention kernels take.
 * ------------------------------------------------------------------------------------------- */
#define CWL_KV_SLOT_ABSENT (-2147483647 - 1)

typedef struct {
    int32_t n_heads, head_dim;
    int32_t k_keep;
} cwl_kv_params;

size_t cwl_kv_workspace_bytes(int32_t chunk_cap);

cwl_status cwl_kv_quantise_chunks(const void* kv, int64_t ld, int64_t n_rows, const int32_t* chunk_offsets,
                                  int32_t n_seqs, const int32_t* chunk_start, const int32_t* chunk_len,
                                  const int32_t* rank_idx, int32_t chunk_cap, const cwl_kv_params* p /*host*/,
                                  int32_t* slot, int32_t* counts, int8_t* q_codes, float* q_scale,
                                  int64_t cap_q, void* f_pool, int64_t cap_f, int32_t* status_word,
                                  void* workspace, size_t workspace_bytes, void* stream);

cwl_status cwl_kv_dequantise(const int32_t* slot, int64_t n_rows, const int8_t* q_codes,
                             const float* q_scale, const void* f_pool, const cwl_kv_params* p /*host*/,
                             void* out, int64_t ld_out, void* stream);

/* ---------------------------------------------------------------------------------------------
 * Measurement aid (not part of the method): per-kernel durations from HIP events.
 * cwl_profile_enable(slot_mask), bit i standing for slot i, creates the events on first use (this
 * is the one place the library creates runtime objects), zeroes the counters and makes every
 * later launch of a kernel whose slot is in the mask record an event pair on its stream (an event
 * record leaves the stream idle for some microseconds, so enable only what is read);
 * cwl_profile_enable(0) stops that.  A mask with bits beyond the slots is CWL_ERR_INVALID_ARG.
 * cwl_profile_read waits
 * for the recorded launches of `slot` (the most recent 256 at most) and returns their summed
 * duration in milliseconds and their count.  Host-side, not thread-safe.
 * ------------------------------------------------------------------------------------------- */
#define CWL_PROF_SCORE 0      /* the entropy kernel of cwl_score_tokens; cwl_compose_scores */
#define CWL_PROF_PARTITION 1  /* all kernels of cwl_partition_chunks; cwl_stream_step     */
#define CWL_PROF_SELECT 2     /* the kernel of cwl_select_ranks                          */
#define CWL_PROF_META 3       /* gate table / grouping kernels of the linear; with at     
                                 most 512 rows: the fix-up kernel                        */
#define CWL_PROF_SHRINK 4     /* shrink GEMM (x A, gated)                                */
#define CWL_PROF_MAIN 5       /* main GEMM (x W + uhat B); with at most 512 rows: the     
                                 partial products x [W | A]                              */
#define CWL_PROF_KV 6         /* both kernels of cwl_kv_quantise_chunks                  */
#define CWL_PROF_SLOTS 7

cwl_status cwl_profile_enable(int32_t slot_mask);
cwl_status cwl_profile_read(int32_t slot, double* total_ms /*host*/, int64_t* launches /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* CWL_H */
