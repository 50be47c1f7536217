"""numpy-facing wrapper around the plain C oracle (``cwl_ref.c``) -- TEST INFRASTRUCTURE ONLY.

Argument marshalling only: every number is produced by the C file, in double.  The wrapper holds
no arithmetic of the method apart from ``bf16_round`` (round-to-nearest-even of a double to the
bf16 grid, used when a test wants the oracle's output on the device's storage grid).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cwl_ref.c")
_LIB = os.path.join(_HERE, "libcwl_ref.so")
_lib = None

OK, ERR_INVALID, ERR_INFEASIBLE, ERR_CAPACITY = 0, 2, 3, 4


def build(force=True):
    """Compile cwl_ref.c with gcc (-O2, OpenMP over token rows, no fast-math, no contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-Wall", "-Wextra", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is not None:
        return _lib
    build(force=False)
    lib = ctypes.CDLL(_LIB)
    i32, i64, f32 = ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    P = ctypes.c_void_p
    lib.cwl_ref_num_threads.restype = ctypes.c_int
    lib.cwl_ref_set_num_threads.argtypes = [ctypes.c_int]
    lib.cwl_ref_entropy.argtypes = [P, i64, i64, i64, P]
    lib.cwl_ref_entropy.restype = None
    lib.cwl_ref_quantise_rows.argtypes = [P, i64, P, P]
    lib.cwl_ref_quantise_rows.restype = None
    lib.cwl_ref_quantise_threshold.argtypes = [f32]
    lib.cwl_ref_quantise_threshold.restype = i64
    lib.cwl_ref_partition.argtypes = [P, P, i32, i32, i32, i64, i64, P, P, P, P, i32]
    lib.cwl_ref_partition.restype = ctypes.c_int
    lib.cwl_ref_select.argtypes = [P, P, i64, P, i32, P]
    lib.cwl_ref_select.restype = None
    lib.cwl_ref_linear.argtypes = [P, i64, P, i64, P, i64, P, i64, i64, i64, i64, i32,
                                   i32, P, P, i32, P, i32, P, P, P, P, P, i64, i32, P]
    lib.cwl_ref_linear.restype = ctypes.c_int
    lib.cwl_ref_stream_step.argtypes = [P, i32, i32, i32, i64, i64, P, i32, P, P, i32,
                                        P, P, P, P, P, P, P, P, P, P, P, P]
    lib.cwl_ref_stream_step.restype = ctypes.c_int
    lib.cwl_ref_gated_linear.argtypes = [P, i64, P, i64, P, i64, P, i64, i64, i64, i64, i32, P, P, P, P, P]
    lib.cwl_ref_gated_linear.restype = ctypes.c_int
    f64 = ctypes.c_double
    lib.cwl_ref_compose_scores.argtypes = [P, P, i64, P, i32, i32, i32, f64, f64, f64, f64, P, P]
    lib.cwl_ref_compose_scores.restype = ctypes.c_int
    lib.cwl_ref_limit_high.argtypes = [P, P, i32, i32, i32, P]
    lib.cwl_ref_limit_high.restype = ctypes.c_int
    lib.cwl_ref_bucket_sequences.argtypes = [P, P, i32, i32, i32, P, P, P, P]
    lib.cwl_ref_bucket_sequences.restype = ctypes.c_int
    lib.cwl_ref_partition_aligned.argtypes = [P, P, i32, P, i32, i32, i32, i64, i64, P, P, P, P, i32]
    lib.cwl_ref_partition_aligned.restype = ctypes.c_int
    lib.cwl_ref_stream_step_aligned.argtypes = [P, i32, i32, i32, i64, i64, P, i32, P, P, i32,
                                                P, i32, P, P, i32, i32, P,
                                                P, P, P, P, P, P, P, P, P, P, P, P]
    lib.cwl_ref_stream_step_aligned.restype = ctypes.c_int
    lib.cwl_ref_kv_quantise.argtypes = [P, i64, i32, i32, P, P, P, i64, i32, P, P, P, P, P]
    lib.cwl_ref_kv_quantise.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def _arr(a, dtype):
    return np.ascontiguousarray(np.asarray(a), dtype=dtype)


def num_threads():
    return int(_load().cwl_ref_num_threads())


def set_num_threads(n):
    _load().cwl_ref_set_num_threads(int(n))


def entropy(logits):
    """Row-wise softmax entropy in nats; ``logits`` is [N, V] float32 (exact device values)."""
    z = _arr(logits, np.float32)
    assert z.ndim == 2
    H = np.empty(z.shape[0], dtype=np.float64)
    _load().cwl_ref_entropy(_ptr(z), z.shape[0], z.shape[1], z.shape[1], _ptr(H))
    return H


def quantise(h):
    """fp32 scores -> Q10 integers.  Returns (q int32[N], nan_seen bool)."""
    h = _arr(h, np.float32).ravel()
    q = np.empty(h.shape[0], dtype=np.int32)
    flag = np.zeros(1, dtype=np.int32)
    _load().cwl_ref_quantise_rows(_ptr(h), h.shape[0], _ptr(q), _ptr(flag))
    return q, bool(flag[0])


def quantise_threshold(h):
    return int(_load().cwl_ref_quantise_threshold(ctypes.c_float(float(np.float32(h)))))


def partition(q, seq_offsets, l_min, l_max, theta_q, delta_q, cap=None):
    """Chunk table of the adaptive chunker.  Returns (status, dict of arrays)."""
    q = _arr(q, np.int32).ravel()
    so = _arr(seq_offsets, np.int32).ravel()
    n_seqs = so.shape[0] - 1
    if cap is None:
        cap = int(q.shape[0]) + n_seqs + 1
    off = np.zeros(n_seqs + 1, dtype=np.int32)
    start = np.zeros(max(cap, 1), dtype=np.int32)
    length = np.zeros(max(cap, 1), dtype=np.int32)
    csum = np.zeros(max(cap, 1), dtype=np.int64)
    st = _load().cwl_ref_partition(_ptr(q), _ptr(so), n_seqs, int(l_min), int(l_max),
                                   int(theta_q), int(delta_q), _ptr(off), _ptr(start),
                                   _ptr(length), _ptr(csum), int(cap))
    n = min(int(off[-1]), cap) if st in (OK, ERR_CAPACITY) else 0
    return st, {"chunk_offsets": off, "chunk_start": start[:n].copy(),
                "chunk_len": length[:n].copy(), "chunk_sum": csum[:n].copy()}


def select(chunk_sum, chunk_len, tau_q):
    cs = _arr(chunk_sum, np.int64).ravel()
    cl = _arr(chunk_len, np.int32).ravel()
    tq = _arr(tau_q, np.int64).ravel()
    out = np.empty(cs.shape[0], dtype=np.int32)
    _load().cwl_ref_select(_ptr(cs), _ptr(cl), cs.shape[0], _ptr(tq), tq.shape[0] + 1, _ptr(out))
    return out


def linear(x, W, A, B, ranks, scales, blend_w, seq_offsets, chunk_offsets, chunk_start,
           chunk_len, rank_idx, rows=None, x_compact=False):
    """y[rows] of the chunk-segmented LoRA linear, float64, unrounded.

    x [N, d_in], W [d_in, d_out], A [d_in, r_max], B [r_max, d_out]: float32 arrays holding the
    exact values the device sees.  With ``x_compact`` x holds only the listed rows (x[i] is token
    rows[i]) -- for large inputs of which only a row sample is brought to the host.
    """
    x, W, A, B = (_arr(a, np.float32) for a in (x, W, A, B))
    n_rows, d_in = x.shape
    if x_compact:
        assert rows is not None and len(rows) == n_rows
        n_rows = int(np.asarray(seq_offsets).ravel()[-1])
    d_out = W.shape[1]
    r_max = A.shape[1]
    assert W.shape[0] == d_in and A.shape[0] == d_in and B.shape == (r_max, d_out)
    ranks = _arr(ranks, np.int32).ravel()
    scales = _arr(scales, np.float32).ravel()
    K = ranks.shape[0]
    assert scales.shape[0] == K
    so = _arr(seq_offsets, np.int32).ravel()
    co = _arr(chunk_offsets, np.int32).ravel()
    cs = _arr(chunk_start, np.int32).ravel()
    cl = _arr(chunk_len, np.int32).ravel()
    ri = _arr(rank_idx, np.int32).ravel()
    n_seqs = so.shape[0] - 1
    assert co.shape[0] == n_seqs + 1 and cs.shape[0] >= co[-1] and ri.shape[0] >= co[-1]
    if co[-1] > 0:
        assert ri[:co[-1]].min() >= 0 and ri[:co[-1]].max() < K
    if rows is None:
        rows_arr, n_sel, rows_ptr = None, n_rows, ctypes.c_void_p(0)
    else:
        rows_arr = _arr(rows, np.int64).ravel()
        assert rows_arr.size == 0 or (rows_arr.min() >= 0 and rows_arr.max() < n_rows)
        n_sel, rows_ptr = rows_arr.shape[0], _ptr(rows_arr)
    y = np.empty((n_sel, d_out), dtype=np.float64)
    st = _load().cwl_ref_linear(_ptr(x), x.shape[1], _ptr(W), W.shape[1], _ptr(A), A.shape[1],
                                _ptr(B), B.shape[1], n_rows, d_in, d_out, r_max, K, _ptr(ranks),
                                _ptr(scales), int(blend_w), _ptr(so), n_seqs, _ptr(co), _ptr(cs),
                                _ptr(cl), _ptr(ri), rows_ptr, n_sel, 1 if x_compact else 0, _ptr(y))
    if st != OK:
        raise ValueError(f"cwl_ref_linear: status {st}")
    return y


class StreamState:
    """Cached scheduler state of the decode-step form, one entry per sequence (all zero at start,
    k_prev = -1)."""

    def __init__(self, n_seqs):
        self.n = np.zeros(n_seqs, np.int32)
        self.sum = np.zeros(n_seqs, np.int64)
        self.k_cur = np.zeros(n_seqs, np.int32)
        self.k_prev = np.full(n_seqs, -1, np.int32)
        self.chunks = np.zeros(n_seqs, np.int32)
        self.pos = np.zeros(n_seqs, np.int64)


def stream_step(state, q_new, l_min, l_max, theta_q, delta_q, tau_q, ranks, scales, blend_w):
    """One decode step: one new quantised score per sequence.  Updates ``state`` in place and returns
    (status, dict with r_cur, g_cur, r_prev, g_prev, closed_len, closed_sum)."""
    qn = _arr(q_new, np.int32).ravel()
    B = qn.shape[0]
    assert state.n.shape[0] == B
    tq = _arr(tau_q, np.int64).ravel()
    rk = _arr(ranks, np.int32).ravel()
    sc = _arr(scales, np.float32).ravel()
    assert rk.shape[0] == tq.shape[0] + 1 == sc.shape[0]
    out = {"r_cur": np.zeros(B, np.int32), "g_cur": np.zeros(B, np.float64),
           "r_prev": np.zeros(B, np.int32), "g_prev": np.zeros(B, np.float64),
           "closed_len": np.zeros(B, np.int32), "closed_sum": np.zeros(B, np.int64)}
    st = _load().cwl_ref_stream_step(_ptr(qn), B, int(l_min), int(l_max), int(theta_q), int(delta_q),
                                     _ptr(tq), rk.shape[0], _ptr(rk), _ptr(sc), int(blend_w),
                                     _ptr(state.n), _ptr(state.sum), _ptr(state.k_cur), _ptr(state.k_prev),
                                     _ptr(state.chunks), _ptr(state.pos),
                                     _ptr(out["r_cur"]), _ptr(out["g_cur"]), _ptr(out["r_prev"]),
                                     _ptr(out["g_prev"]), _ptr(out["closed_len"]), _ptr(out["closed_sum"]))
    return st, out


class BucketState:
    """Open chunk of every bucket's mean series (all zero at start)."""

    def __init__(self, n_buckets):
        self.n = np.zeros(n_buckets, np.int32)
        self.sum = np.zeros(n_buckets, np.int64)


def stream_step_aligned(state, q_new, l_min, l_max, theta_q, delta_q, tau_q, ranks, scales, blend_w,
                        bucket=None, bucket_state=None, k_high=1, budget=0, n_high=None):
    """One decode step of a batch with boundaries shared inside each bucket (``bucket`` + ``bucket_state``,
    both or neither) and a budget of high-capacity chunks (``n_high``: int32 counters, updated in place,
    or None for no budget).  Returns (status, dict) like stream_step."""
    qn = _arr(q_new, np.int32).ravel()
    B = qn.shape[0]
    assert state.n.shape[0] == B
    tq = _arr(tau_q, np.int64).ravel()
    rk = _arr(ranks, np.int32).ravel()
    sc = _arr(scales, np.float32).ravel()
    assert rk.shape[0] == tq.shape[0] + 1 == sc.shape[0]
    assert (bucket is None) == (bucket_state is None)
    null = ctypes.c_void_p(0)
    if bucket is not None:
        bk = _arr(bucket, np.int32).ravel()
        assert bk.shape[0] == B
        bk_args = (_ptr(bk), bucket_state.n.shape[0], _ptr(bucket_state.n), _ptr(bucket_state.sum))
    else:
        bk_args = (null, 0, null, null)
    if n_high is not None:
        assert n_high.dtype == np.int32 and n_high.shape[0] == B
    out = {"r_cur": np.zeros(B, np.int32), "g_cur": np.zeros(B, np.float64),
           "r_prev": np.zeros(B, np.int32), "g_prev": np.zeros(B, np.float64),
           "closed_len": np.zeros(B, np.int32), "closed_sum": np.zeros(B, np.int64)}
    st = _load().cwl_ref_stream_step_aligned(
        _ptr(qn), B, int(l_min), int(l_max), int(theta_q), int(delta_q), _ptr(tq), rk.shape[0], _ptr(rk), _ptr(sc),
        int(blend_w), *bk_args, int(k_high), int(budget), null if n_high is None else _ptr(n_high),
        _ptr(state.n), _ptr(state.sum), _ptr(state.k_cur), _ptr(state.k_prev), _ptr(state.chunks), _ptr(state.pos),
        _ptr(out["r_cur"]), _ptr(out["g_cur"]), _ptr(out["r_prev"]), _ptr(out["g_prev"]),
        _ptr(out["closed_len"]), _ptr(out["closed_sum"]))
    return st, out


def gated_linear(x, W, A, B, r_cur, g_cur, r_prev, g_prev):
    """y = x W + g_cur (x A[:, :r_cur]) B[:r_cur] + g_prev (x A[:, :r_prev]) B[:r_prev], per row, float64."""
    x, W, A, B = (_arr(a, np.float32) for a in (x, W, A, B))
    n_rows, d_in = x.shape
    d_out, r_max = W.shape[1], A.shape[1]
    assert W.shape[0] == d_in and A.shape[0] == d_in and B.shape == (r_max, d_out)
    rc, rp = _arr(r_cur, np.int32).ravel(), _arr(r_prev, np.int32).ravel()
    gc, gp = _arr(g_cur, np.float64).ravel(), _arr(g_prev, np.float64).ravel()
    assert rc.shape[0] == rp.shape[0] == gc.shape[0] == gp.shape[0] == n_rows
    y = np.empty((n_rows, d_out), dtype=np.float64)
    st = _load().cwl_ref_gated_linear(_ptr(x), x.shape[1], _ptr(W), W.shape[1], _ptr(A), A.shape[1],
                                      _ptr(B), B.shape[1], n_rows, d_in, d_out, r_max,
                                      _ptr(rc), _ptr(gc), _ptr(rp), _ptr(gp), _ptr(y))
    if st != OK:
        raise ValueError(f"cwl_ref_gated_linear: status {st}")
    return y


def compose_scores(entropy, token_ids, seq_offsets, n, window, w_entropy, w_novelty, w_prior, prior_len):
    """Composite score: w_entropy H + w_novelty [n-gram new within `window`] + w_prior max(0, 1 - j / prior_len).
    Returns (status, score float64[N], novelty int32[N])."""
    h = _arr(entropy, np.float32).ravel()
    ids = _arr(token_ids, np.int32).ravel()
    so = _arr(seq_offsets, np.int32).ravel()
    assert ids.shape[0] == h.shape[0]
    score = np.zeros(h.shape[0], np.float64)
    nov = np.zeros(h.shape[0], np.int32)
    st = _load().cwl_ref_compose_scores(_ptr(h), _ptr(ids), h.shape[0], _ptr(so), so.shape[0] - 1, int(n),
                                        int(window), float(w_entropy), float(w_novelty), float(w_prior),
                                        float(prior_len), _ptr(score), _ptr(nov))
    return st, score, nov


def limit_high(rank_idx, chunk_offsets, k_high, budget):
    """Budget of high-capacity chunks per sequence.  Returns (status, limited rank_idx, n_asked[n_seqs])."""
    ri = _arr(rank_idx, np.int32).ravel().copy()
    co = _arr(chunk_offsets, np.int32).ravel()
    assert ri.shape[0] >= co[-1]
    asked = np.zeros(co.shape[0] - 1, np.int32)
    st = _load().cwl_ref_limit_high(_ptr(ri), _ptr(co), co.shape[0] - 1, int(k_high), int(budget), _ptr(asked))
    return st, ri, asked


def bucket_sequences(q, seq_offsets, n_buckets, n_micro=0):
    """Percentile buckets and micro-batches of the sequences of a batch.
    Returns (status, dict with seq_sum, order, bucket, micro)."""
    q = _arr(q, np.int32).ravel()
    so = _arr(seq_offsets, np.int32).ravel()
    n = so.shape[0] - 1
    out = {"seq_sum": np.zeros(n, np.int64), "order": np.zeros(n, np.int32),
           "bucket": np.zeros(n, np.int32), "micro": np.zeros(n, np.int32)}
    st = _load().cwl_ref_bucket_sequences(_ptr(q), _ptr(so), n, int(n_buckets), int(n_micro), _ptr(out["seq_sum"]),
                                          _ptr(out["order"]), _ptr(out["bucket"]), _ptr(out["micro"]))
    return st, out


def partition_aligned(q, seq_offsets, bucket, n_buckets, l_min, l_max, theta_q, delta_q, cap=None):
    """Chunk table with the boundaries shared inside each bucket.  Returns (status, dict of arrays)."""
    q = _arr(q, np.int32).ravel()
    so = _arr(seq_offsets, np.int32).ravel()
    bk = _arr(bucket, np.int32).ravel()
    n_seqs = so.shape[0] - 1
    assert bk.shape[0] == n_seqs
    if cap is None:
        cap = int(q.shape[0]) + n_seqs + 1
    off = np.zeros(n_seqs + 1, dtype=np.int32)
    start = np.zeros(max(cap, 1), dtype=np.int32)
    length = np.zeros(max(cap, 1), dtype=np.int32)
    csum = np.zeros(max(cap, 1), dtype=np.int64)
    st = _load().cwl_ref_partition_aligned(_ptr(q), _ptr(so), n_seqs, _ptr(bk), int(n_buckets), int(l_min),
                                           int(l_max), int(theta_q), int(delta_q), _ptr(off), _ptr(start),
                                           _ptr(length), _ptr(csum), int(cap))
    n = min(int(off[-1]), cap) if st in (OK, ERR_CAPACITY) else 0
    return st, {"chunk_offsets": off, "chunk_start": start[:n].copy(),
                "chunk_len": length[:n].copy(), "chunk_sum": csum[:n].copy()}


def build_ladder(A, B):
    """Rank ladder of the adapter update by one SVD (Sec. III-C: the ladder is obtained once by an SVD of
    the adapter matrix, and a rung slices its first r directions).

    dW = A B = U diag(sigma) V^T with sigma descending (float64 library SVD of the product written out).
    Reading: the two factors share the singular values evenly, A' = U[:, :r] diag(sqrt(sigma)),
    B' = diag(sqrt(sigma)) V^T[:r, :], so that A'[:, :k] B'[:k, :] is the best rank-k approximation of
    dW for every k and A' B' = dW.  Directions whose sigma is below 1e-12 sigma_max carry nothing and
    are set to zero.  Singular vectors are fixed only up to sign (and rotation inside equal singular
    values); sigma and the truncated products are unique.  Returns (A' [d_in, r], B' [r, d_out],
    sigma [r]) in float64."""
    A64 = np.asarray(A, dtype=np.float32).astype(np.float64)
    B64 = np.asarray(B, dtype=np.float32).astype(np.float64)
    r = A64.shape[1]
    assert B64.shape[0] == r
    U, S, Vt = np.linalg.svd(A64 @ B64, full_matrices=False)
    n = min(r, S.shape[0])
    sigma = np.zeros(r)
    sigma[:n] = S[:n]
    A2 = np.zeros((A64.shape[0], r))
    B2 = np.zeros((r, B64.shape[1]))
    keep = sigma[:n] > 1e-12 * max(sigma[0], 1e-300)
    root = np.sqrt(sigma[:n]) * keep
    A2[:, :n] = U[:, :n] * root
    B2[:n, :] = root[:, None] * Vt[:n, :]
    sigma[:n] *= keep
    return A2, B2, sigma


SLOT_ABSENT = -2 ** 31


def kv_quantise(kv, n_heads, head_dim, chunk_start, chunk_len, rank_idx, k_keep):
    """Chunk-level KV-cache policy (Sec. III-E, IV-F): rows of chunks whose rung is below ``k_keep`` go to an
    INT8 pool (symmetric, one fp32 scale per row and head), the rows of the other chunks to a full-fidelity
    pool.  ``kv``: [N, n_heads * head_dim] float32 holding exact bf16 values.  Returns a dict: slot int32 [N],
    codes int8 [Nq, H*D], scale float32 [Nq, H], kept float32 [Nf, H*D]."""
    x = _arr(kv, np.float32)
    assert x.ndim == 2 and x.shape[1] == n_heads * head_dim
    cs = _arr(chunk_start, np.int32).ravel()
    cl = _arr(chunk_len, np.int32).ravel()
    rk = _arr(rank_idx, np.int32).ravel()
    n = x.shape[0]
    slot = np.empty(n, dtype=np.int32)
    codes = np.zeros((max(n, 1), x.shape[1]), dtype=np.int8)
    scale = np.zeros((max(n, 1), n_heads), dtype=np.float32)
    kept = np.zeros((max(n, 1), x.shape[1]), dtype=np.float32)
    counts = np.zeros(2, dtype=np.int64)
    st = _load().cwl_ref_kv_quantise(_ptr(x), n, int(n_heads), int(head_dim), _ptr(cs), _ptr(cl), _ptr(rk),
                                     cs.shape[0], int(k_keep), _ptr(slot), _ptr(codes), _ptr(scale), _ptr(kept),
                                     _ptr(counts))
    assert st == OK, st
    nq, nf = int(counts[0]), int(counts[1])
    return {"slot": slot, "codes": codes[:nq].copy(), "scale": scale[:nq].copy(), "kept": kept[:nf].copy()}


def kv_dequantise(slot, codes, scale, kept, n_heads, head_dim):
    """The cache read back as bf16 values (float32 array [N, H*D]): a kept row as it was stored, an INT8 row as
    code * scale formed in fp32 (the kernel's precision) and rounded to bf16 once, an absent row as zeros."""
    slot = np.asarray(slot, dtype=np.int64)
    out = np.zeros((slot.shape[0], n_heads * head_dim), dtype=np.float32)
    for t, s in enumerate(slot):
        if s == SLOT_ABSENT:
            continue
        if s < 0:
            out[t] = kept[-1 - s]
        else:
            with np.errstate(invalid="ignore"):          # code 0 times an infinite scale is NaN, as on the device
                prod = codes[s].astype(np.float32).reshape(n_heads, head_dim) * scale[s].astype(np.float32)[:, None]
            out[t] = bf16_round(prod.astype(np.float32).reshape(-1)).astype(np.float32)
    return out


def bf16_round(y):
    """Round float64 values to the bf16 grid (nearest, ties to even), returned as float64."""
    f = np.asarray(y, dtype=np.float64).astype(np.float32)   # fp32 first: bf16 is its top half
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> 16) & 1
    rounded = ((bits + 0x7FFF + lsb) >> 16) << 16
    out = rounded.astype(np.uint32).view(np.float32)
    return np.where(np.isfinite(f), out, f).astype(np.float64)
