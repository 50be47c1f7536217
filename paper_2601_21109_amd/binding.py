"""Thin ctypes binding of the C ABI in ``include/cwl.h``: argument marshalling only.

PyTorch supplies device memory (``torch.empty(device=...)``, ``data_ptr()``) and the current HIP
stream; every step of the path runs in the library's kernels.  The library is loaded on first
use; if it is missing the call raises -- there is no fallback of any kind.
"""
import ctypes
import math
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcwl.so")

OK, ERR_NULL, ERR_INVALID_ARG, ERR_INFEASIBLE, ERR_CAPACITY, ERR_UNSUPPORTED, ERR_DEVICE = range(7)
F32, BF16 = 0, 1
STATUS_CAPACITY, STATUS_NAN_SCORE, STATUS_BAD_OFFSETS, STATUS_BAD_BUCKET = 1, 2, 4, 8
MAX_LADDER, MAX_RANK = 16, 256
STATIC_SCRATCH_BYTES = 16 << 20
MAX_GROUP = 8

EXPORTS = ["cwl_status_string", "cwl_abi_version", "cwl_score_tokens", "cwl_compose_scores",
           "cwl_partition_workspace_bytes", "cwl_partition_chunks", "cwl_select_ranks",
           "cwl_select_ranks_budget", "cwl_bucket_sequences", "cwl_aligned_workspace_bytes",
           "cwl_partition_chunks_aligned",
           "cwl_packed_weights_bytes", "cwl_prepack_weights", "cwl_linear_workspace_bytes",
           "cwl_linear_packed_workspace_bytes", "cwl_chunkwise_lora_linear",
           "cwl_chunkwise_lora_linear_packed", "cwl_chunkwise_lora_linear_packed_static",
           "cwl_lora_shrink_bytes", "cwl_lora_shrink_packed", "cwl_chunkwise_lora_linear_packed_shrunk",
           "cwl_schedule_chunks", "cwl_kv_workspace_bytes", "cwl_kv_quantise_chunks", "cwl_kv_dequantise",
           "cwl_stream_step", "cwl_stream_step_aligned",
           "cwl_gated_lora_linear_packed", "cwl_packed_weights_grouped_bytes",
           "cwl_linear_grouped_workspace_bytes", "cwl_prepack_weights_grouped",
           "cwl_chunkwise_lora_linear_grouped_packed", "cwl_gated_lora_linear_grouped_packed",
           "cwl_ladder_workspace_bytes", "cwl_build_ladder",
           "cwl_profile_enable", "cwl_profile_read"]
PROF_SCORE, PROF_PARTITION, PROF_SELECT, PROF_META, PROF_SHRINK, PROF_MAIN, PROF_KV = range(7)
PROF_SLOTS = 7
KV_SLOT_ABSENT = -2 ** 31


class ChunkParams(ctypes.Structure):
    _fields_ = [("l_min", ctypes.c_int32), ("l_max", ctypes.c_int32),
                ("theta_hard", ctypes.c_float), ("delta_dev", ctypes.c_float)]


class ScoreMix(ctypes.Structure):
    _fields_ = [("n", ctypes.c_int32), ("window", ctypes.c_int32), ("w_entropy", ctypes.c_float),
                ("w_novelty", ctypes.c_float), ("w_prior", ctypes.c_float), ("prior_len", ctypes.c_float)]


class KvParams(ctypes.Structure):
    _fields_ = [("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("k_keep", ctypes.c_int32)]


class LinearDesc(ctypes.Structure):
    _fields_ = [("n_rows", ctypes.c_int64), ("d_in", ctypes.c_int64), ("d_out", ctypes.c_int64),
                ("r_max", ctypes.c_int32), ("K", ctypes.c_int32),
                ("ranks", ctypes.POINTER(ctypes.c_int32)), ("scales", ctypes.POINTER(ctypes.c_float)),
                ("blend_w", ctypes.c_int32), ("dt", ctypes.c_int),
                ("ldx", ctypes.c_int64), ("ldw", ctypes.c_int64), ("lda", ctypes.c_int64),
                ("ldb", ctypes.c_int64), ("ldy", ctypes.c_int64), ("group_rows", ctypes.c_int32)]


class Group(ctypes.Structure):
    _fields_ = [("n_proj", ctypes.c_int32), ("d_out", ctypes.c_int64 * MAX_GROUP),
                ("W", ctypes.c_void_p * MAX_GROUP), ("A", ctypes.c_void_p * MAX_GROUP),
                ("B", ctypes.c_void_p * MAX_GROUP)]


class CwlError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


_lib = None


def lib():
    """The loaded HIP library.  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                           "`python -m paper_2601_21109_amd.build` (there is no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    i32, i64, P, sz = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    L.cwl_status_string.argtypes = [ctypes.c_int]
    L.cwl_status_string.restype = ctypes.c_char_p
    L.cwl_abi_version.restype = i32
    L.cwl_score_tokens.argtypes = [P, ctypes.c_int, i64, i64, i64, P, P]
    L.cwl_compose_scores.argtypes = [P, P, i64, P, i32, ctypes.POINTER(ScoreMix), P, P, P]
    L.cwl_compose_scores.restype = ctypes.c_int
    L.cwl_partition_workspace_bytes.argtypes = [i64, i32, ctypes.POINTER(ChunkParams)]
    L.cwl_partition_workspace_bytes.restype = sz
    L.cwl_partition_chunks.argtypes = [P, i64, P, i32, ctypes.POINTER(ChunkParams), P, P, P, P,
                                       i32, P, P, sz, P]
    L.cwl_select_ranks.argtypes = [P, P, P, i32, i32, ctypes.POINTER(ctypes.c_float), i32, P, P]
    L.cwl_select_ranks_budget.argtypes = [P, P, P, i32, i32, ctypes.POINTER(ctypes.c_float), i32, i32, i32, P, P, P]
    L.cwl_bucket_sequences.argtypes = [P, i64, P, i32, i32, i32, P, P, P, P, P]
    L.cwl_aligned_workspace_bytes.argtypes = [i64, i32, i32, ctypes.POINTER(ChunkParams)]
    L.cwl_aligned_workspace_bytes.restype = sz
    L.cwl_partition_chunks_aligned.argtypes = [P, i64, P, i32, P, i32, ctypes.POINTER(ChunkParams), P, P, P, P,
                                               i32, P, P, sz, P]
    dp = ctypes.POINTER(LinearDesc)
    for name in ("cwl_packed_weights_bytes", "cwl_linear_workspace_bytes",
                 "cwl_linear_packed_workspace_bytes", "cwl_lora_shrink_bytes"):
        getattr(L, name).argtypes = [dp]
        getattr(L, name).restype = sz
    L.cwl_prepack_weights.argtypes = [dp, P, P, P, P, sz, P]
    L.cwl_chunkwise_lora_linear.argtypes = [dp, P, P, P, P, P, i32, P, P, P, P, i32, P, P, sz, P]
    L.cwl_chunkwise_lora_linear_packed.argtypes = [dp, P, P, P, i32, P, P, P, P, i32, P, P, sz, P]
    fp = ctypes.POINTER(ctypes.c_float)
    L.cwl_stream_step.argtypes = [P, i32, ctypes.POINTER(ChunkParams), fp, i32, ctypes.POINTER(i32), fp,
                                  i32, P, P, P, P, P, P]
    L.cwl_stream_step_aligned.argtypes = [P, i32, ctypes.POINTER(ChunkParams), ctypes.POINTER(ctypes.c_float), i32,
                                          ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_float), i32,
                                          P, i32, P, i32, i32, P, P, P, P, P, P, P]
    L.cwl_ladder_workspace_bytes.argtypes = [i32]
    L.cwl_ladder_workspace_bytes.restype = sz
    L.cwl_build_ladder.argtypes = [ctypes.c_int, P, i64, P, i64, i64, i64, i32, P, i64, P, i64, P, P, sz, P]
    L.cwl_gated_lora_linear_packed.argtypes = [dp, P, P, P, P, P, sz, P]
    L.cwl_profile_enable.argtypes = [i32]
    L.cwl_profile_read.argtypes = [i32, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(i64)]
    gp = ctypes.POINTER(Group)
    L.cwl_packed_weights_grouped_bytes.argtypes = [dp, gp]
    L.cwl_linear_grouped_workspace_bytes.argtypes = [dp, gp]
    L.cwl_prepack_weights_grouped.argtypes = [dp, gp, P, sz, P]
    L.cwl_chunkwise_lora_linear_grouped_packed.argtypes = [dp, gp, P, P, P, i32, P, P, P, P, i32, P, P, sz, P]
    L.cwl_gated_lora_linear_grouped_packed.argtypes = [dp, gp, P, P, P, P, P, sz, P]
    L.cwl_chunkwise_lora_linear_packed_static.argtypes = [dp, P, P, P, i32, P, P, P, P, i32, P, P]
    L.cwl_lora_shrink_packed.argtypes = [dp, P, P, P, sz, P]
    kp = ctypes.POINTER(KvParams)
    L.cwl_kv_workspace_bytes.argtypes = [i32]
    L.cwl_kv_quantise_chunks.argtypes = [P, i64, i64, P, i32, P, P, P, i32, kp, P, P, P, P, i64, P, i64, P, P, sz, P]
    L.cwl_kv_dequantise.argtypes = [P, i64, P, P, P, kp, P, i64, P]
    L.cwl_schedule_chunks.argtypes = [P, i64, P, i32, ctypes.POINTER(ChunkParams), ctypes.POINTER(ctypes.c_float), i32,
                                      P, P, P, P, P, i32, P, P, sz, dp, P, P, P, sz, P]
    L.cwl_chunkwise_lora_linear_packed_shrunk.argtypes = [dp, P, P, P, sz, P, i32, P, P, P, P, i32, P, P, sz, P]
    # return types: byte counts are size_t, everything else but the two informational calls a status
    for name in EXPORTS:
        if name.endswith("_bytes"):
            getattr(L, name).restype = sz
        elif name not in ("cwl_status_string", "cwl_abi_version"):
            getattr(L, name).restype = ctypes.c_int
    _lib = L
    return L


def status_string(status):
    return lib().cwl_status_string(int(status)).decode()


def _check(status, where):
    if status != OK:
        raise CwlError(status, where)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


def _dt(t):
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ws(nbytes, device):
    # torch's caching allocator hands out 512-byte aligned blocks
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# ------------------------------------------------------------------------------------------------
def score_tokens(logits, out=None):
    """entropy[t] (nats, fp32) of softmax(logits[t, :]).  logits: [N, V] fp32 or bf16, device."""
    assert logits.is_cuda and logits.dim() == 2 and logits.stride(1) == 1
    n, v = logits.shape
    if out is None:
        out = torch.empty(n, dtype=torch.float32, device=logits.device)
    _check(lib().cwl_score_tokens(_ptr(logits), _dt(logits), n, v, logits.stride(0) if n > 1 else v,
                                  _ptr(out), _stream()), "cwl_score_tokens")
    return out


def compose_scores(entropy, token_ids, seq_offsets, n, window, w_entropy=1.0, w_novelty=0.0, w_prior=0.0,
                   prior_len=0.0, out=None, novelty=None):
    """Composite difficulty score (entropy, n-gram novelty within `window`, positional prior).  Returns
    (score fp32 [N], novelty int32 [N])."""
    assert entropy.is_cuda and entropy.dtype == torch.float32 and entropy.is_contiguous()
    assert token_ids.is_cuda and token_ids.dtype == torch.int32 and token_ids.is_contiguous()
    assert token_ids.numel() == entropy.numel()
    n_rows, n_seqs = entropy.numel(), seq_offsets.numel() - 1
    if out is None:
        out = torch.empty_like(entropy)
    if novelty is None:
        novelty = torch.empty(n_rows, dtype=torch.int32, device=entropy.device)
    m = ScoreMix(int(n), int(window), float(w_entropy), float(w_novelty), float(w_prior), float(prior_len))
    _check(lib().cwl_compose_scores(_ptr(entropy), _ptr(token_ids), n_rows, _ptr(seq_offsets), n_seqs,
                                    ctypes.byref(m), _ptr(out), _ptr(novelty), _stream()), "cwl_compose_scores")
    return out, novelty


def partition_chunks(entropy, seq_offsets, l_min, l_max, theta_hard=math.inf, delta_dev=math.inf,
                     cap=None, out=None):
    """Chunk table of the adaptive chunker.  Returns a dict of device tensors
    (chunk_offsets, chunk_start, chunk_len, chunk_sum, status_word) plus 'cap'.  A dict returned
    by an earlier call of the same shape can be passed as `out` to reuse its buffers."""
    assert entropy.is_cuda and entropy.dtype == torch.float32 and entropy.is_contiguous()
    assert seq_offsets.is_cuda and seq_offsets.dtype == torch.int32
    dev = entropy.device
    n_rows, n_seqs = entropy.numel(), seq_offsets.numel() - 1
    p = ChunkParams(int(l_min), int(l_max), float(theta_hard), float(delta_dev))
    if out is not None:
        cap = out["cap"]
    elif cap is None:
        cap = n_rows // max(int(l_min), 1) + n_seqs + 1
    nbytes = lib().cwl_partition_workspace_bytes(n_rows, n_seqs, ctypes.byref(p))
    out = out if out is not None else {
        "chunk_offsets": torch.empty(n_seqs + 1, dtype=torch.int32, device=dev),
        "chunk_start": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_len": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_sum": torch.empty(max(cap, 1), dtype=torch.int64, device=dev),
        "status_word": torch.empty(1, dtype=torch.int32, device=dev),
        "cap": int(cap),
        "_workspace": _ws(nbytes, dev),
    }
    ws = out["_workspace"]
    _check(lib().cwl_partition_chunks(_ptr(entropy), n_rows, _ptr(seq_offsets), n_seqs,
                                      ctypes.byref(p), _ptr(out["chunk_offsets"]),
                                      _ptr(out["chunk_start"]), _ptr(out["chunk_len"]),
                                      _ptr(out["chunk_sum"]), int(cap), _ptr(out["status_word"]),
                                      _ptr(ws), ws.numel(), _stream()), "cwl_partition_chunks")
    return out


def select_ranks(table, thresholds, K, out=None):
    """rank_idx[c] (int32, device) for every chunk of `table` (from partition_chunks)."""
    dev = table["chunk_len"].device
    n_seqs = table["chunk_offsets"].numel() - 1
    cap = table["cap"]
    rank_idx = out if out is not None else torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
    th = (ctypes.c_float * max(K - 1, 1))(*[float(t) for t in thresholds])
    _check(lib().cwl_select_ranks(_ptr(table["chunk_sum"]), _ptr(table["chunk_len"]),
                                  _ptr(table["chunk_offsets"]), n_seqs, cap, th, int(K),
                                  _ptr(rank_idx), _stream()), "cwl_select_ranks")
    return rank_idx


def select_ranks_budget(table, thresholds, K, k_high, budget, out=None, n_asked=None):
    """select_ranks with at most `budget` chunks per sequence on a rung >= k_high.  Returns
    (rank_idx, n_asked), both int32 on the device."""
    dev = table["chunk_len"].device
    n_seqs = table["chunk_offsets"].numel() - 1
    cap = table["cap"]
    rank_idx = out if out is not None else torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
    n_asked = n_asked if n_asked is not None else torch.zeros(max(n_seqs, 1), dtype=torch.int32, device=dev)
    th = (ctypes.c_float * max(K - 1, 1))(*[float(t) for t in thresholds])
    _check(lib().cwl_select_ranks_budget(_ptr(table["chunk_sum"]), _ptr(table["chunk_len"]),
                                         _ptr(table["chunk_offsets"]), n_seqs, cap, th, int(K), int(k_high),
                                         int(budget), _ptr(rank_idx), _ptr(n_asked), _stream()),
           "cwl_select_ranks_budget")
    return rank_idx, n_asked


def bucket_sequences(score, seq_offsets, n_buckets, n_micro=0, out=None):
    """Percentile buckets (and micro-batches when n_micro > 0) of the sequences of a batch.  Returns a
    dict of device tensors: seq_sum (int64), order, bucket, micro (int32; micro absent when n_micro == 0)."""
    assert score.is_cuda and score.dtype == torch.float32 and score.is_contiguous()
    assert seq_offsets.is_cuda and seq_offsets.dtype == torch.int32
    dev = score.device
    n_rows, n_seqs = score.numel(), seq_offsets.numel() - 1
    if out is None:
        out = {"seq_sum": torch.zeros(max(n_seqs, 1), dtype=torch.int64, device=dev),
               "order": torch.zeros(max(n_seqs, 1), dtype=torch.int32, device=dev),
               "bucket": torch.zeros(max(n_seqs, 1), dtype=torch.int32, device=dev)}
        if n_micro > 0:
            out["micro"] = torch.zeros(max(n_seqs, 1), dtype=torch.int32, device=dev)
    _check(lib().cwl_bucket_sequences(_ptr(score), n_rows, _ptr(seq_offsets), n_seqs, int(n_buckets),
                                      int(n_micro), _ptr(out["seq_sum"]), _ptr(out["order"]), _ptr(out["bucket"]),
                                      _ptr(out.get("micro")), _stream()), "cwl_bucket_sequences")
    return out


def partition_chunks_aligned(score, seq_offsets, bucket, n_buckets, l_min, l_max, theta_hard=math.inf,
                             delta_dev=math.inf, cap=None, out=None):
    """Chunk table with the boundaries shared inside each bucket; same result layout as partition_chunks."""
    assert score.is_cuda and score.dtype == torch.float32 and score.is_contiguous()
    assert seq_offsets.is_cuda and seq_offsets.dtype == torch.int32
    assert bucket.is_cuda and bucket.dtype == torch.int32
    dev = score.device
    n_rows, n_seqs = score.numel(), seq_offsets.numel() - 1
    p = ChunkParams(int(l_min), int(l_max), float(theta_hard), float(delta_dev))
    if out is not None:
        cap = out["cap"]
    elif cap is None:
        cap = n_rows // max(int(l_min), 1) + n_seqs + 1
    nbytes = lib().cwl_aligned_workspace_bytes(n_rows, n_seqs, int(n_buckets), ctypes.byref(p))
    out = out if out is not None else {
        "chunk_offsets": torch.empty(n_seqs + 1, dtype=torch.int32, device=dev),
        "chunk_start": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_len": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_sum": torch.empty(max(cap, 1), dtype=torch.int64, device=dev),
        "status_word": torch.empty(1, dtype=torch.int32, device=dev),
        "cap": int(cap),
        "_workspace": _ws(nbytes, dev),
    }
    ws = out["_workspace"]
    _check(lib().cwl_partition_chunks_aligned(_ptr(score), n_rows, _ptr(seq_offsets), n_seqs, _ptr(bucket),
                                              int(n_buckets), ctypes.byref(p), _ptr(out["chunk_offsets"]),
                                              _ptr(out["chunk_start"]), _ptr(out["chunk_len"]),
                                              _ptr(out["chunk_sum"]), int(cap), _ptr(out["status_word"]),
                                              _ptr(ws), ws.numel(), _stream()), "cwl_partition_chunks_aligned")
    return out


class _Desc:
    """Owns the host arrays a cwl_linear_desc points to."""

    def __init__(self, n_rows, d_in, d_out, r_max, ranks, scales, blend_w, dt, ldx, ldw, lda, ldb,
                 ldy, group_rows):
        K = len(ranks)
        self.ranks = (ctypes.c_int32 * max(K, 1))(*[int(r) for r in ranks])
        self.scales = (ctypes.c_float * max(K, 1))(*[float(s) for s in scales])
        self.c = LinearDesc(n_rows, d_in, d_out, r_max, K, self.ranks, self.scales, int(blend_w), dt,
                            ldx, ldw, lda, ldb, ldy, int(group_rows))

    def ref(self):
        return ctypes.byref(self.c)


def _desc_for(x, d_out, r_max, ranks, scales, blend_w, y, W=None, A=None, B=None, group_rows=0):
    n_rows, d_in = x.shape
    ldx = x.stride(0) if n_rows > 1 else d_in
    ldy = y.stride(0) if n_rows > 1 else d_out
    ldw = W.stride(0) if W is not None and W.shape[0] > 1 else d_out
    lda = A.stride(0) if A is not None and A.shape[0] > 1 else max(r_max, 1)
    ldb = B.stride(0) if B is not None and B.shape[0] > 1 else d_out
    return _Desc(n_rows, d_in, d_out, r_max, ranks, scales, blend_w, _dt(x), ldx, ldw, lda, ldb, ldy,
                 group_rows)


class PackedWeights:
    """Static weights re-laid out once by cwl_prepack_weights."""

    def __init__(self, blob, d_in, d_out, r_max, dtype):
        self.blob, self.d_in, self.d_out, self.r_max, self.dtype = blob, d_in, d_out, r_max, dtype


def prepack_weights(W, A, B):
    """W [d_in, d_out], A [d_in, r_max], B [r_max, d_out] -> PackedWeights (device)."""
    assert W.is_cuda and W.dim() == 2 and W.stride(1) == 1
    d_in, d_out = W.shape
    r_max = A.shape[1]
    assert A.shape[0] == d_in and B.shape == (r_max, d_out)
    assert A.dtype == W.dtype and B.dtype == W.dtype
    dummy_x = torch.empty((1, d_in), dtype=W.dtype, device=W.device)
    dummy_y = torch.empty((1, d_out), dtype=W.dtype, device=W.device)
    d = _desc_for(dummy_x, d_out, r_max, [r_max], [1.0], 0, dummy_y, W, A, B)
    d.c.n_rows = 0
    nbytes = lib().cwl_packed_weights_bytes(d.ref())
    if nbytes == 0:
        raise CwlError(ERR_INVALID_ARG, "cwl_packed_weights_bytes")
    blob = _ws(nbytes, W.device)
    _check(lib().cwl_prepack_weights(d.ref(), _ptr(W), _ptr(A if r_max else None),
                                     _ptr(B if r_max else None), _ptr(blob), blob.numel(),
                                     _stream()), "cwl_prepack_weights")
    return PackedWeights(blob, d_in, d_out, r_max, W.dtype)


def chunkwise_lora_linear(x, W, A, B, ranks, scales, blend_w, seq_offsets, table, rank_idx,
                          out=None, group_rows=0, workspace=None):
    """y = x W + chunk-wise gated LoRA term with the boundary cross-fade (see include/cwl.h).

    `W` may be a raw [d_in, d_out] tensor (with A, B) or a PackedWeights (A = B = None)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1
    packed = isinstance(W, PackedWeights)
    d_out = W.d_out if packed else W.shape[1]
    r_max = W.r_max if packed else A.shape[1]
    n_rows = x.shape[0]
    if out is None:
        out = torch.empty((n_rows, d_out), dtype=x.dtype, device=x.device)
    n_seqs = seq_offsets.numel() - 1
    cap = table["cap"]
    L = lib()
    if packed:
        assert W.dtype == x.dtype and W.d_in == x.shape[1]
        d = _desc_for(x, d_out, r_max, ranks, scales, blend_w, out, group_rows=group_rows)
        need = L.cwl_linear_packed_workspace_bytes(d.ref())
    else:
        d = _desc_for(x, d_out, r_max, ranks, scales, blend_w, out, W, A, B, group_rows=group_rows)
        need = L.cwl_linear_workspace_bytes(d.ref())
    if need == 0:
        # the descriptor was rejected: let the call itself say why
        need = 256
    ws = workspace if workspace is not None else _ws(need, x.device)
    common = (_ptr(seq_offsets), n_seqs, _ptr(table["chunk_offsets"]), _ptr(table["chunk_start"]),
              _ptr(table["chunk_len"]), _ptr(rank_idx), cap, _ptr(out), _ptr(ws), ws.numel(),
              _stream())
    if packed:
        _check(L.cwl_chunkwise_lora_linear_packed(d.ref(), _ptr(x), _ptr(W.blob), *common),
               "cwl_chunkwise_lora_linear_packed")
    else:
        _check(L.cwl_chunkwise_lora_linear(d.ref(), _ptr(x), _ptr(W), _ptr(A if r_max else None),
                                           _ptr(B if r_max else None), *common),
               "cwl_chunkwise_lora_linear")
    return out


def chunkwise_lora_linear_static(x, packed, ranks, scales, blend_w, seq_offsets, table, rank_idx, out=None):
    """chunkwise_lora_linear on PackedWeights with the library's own static scratch array instead of a
    workspace: the call allocates nothing when `out` is given."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(packed, PackedWeights)
    assert packed.dtype == x.dtype and packed.d_in == x.shape[1]
    if out is None:
        out = torch.empty((x.shape[0], packed.d_out), dtype=x.dtype, device=x.device)
    d = _desc_for(x, packed.d_out, packed.r_max, ranks, scales, blend_w, out)
    _check(lib().cwl_chunkwise_lora_linear_packed_static(
        d.ref(), _ptr(x), _ptr(packed.blob), _ptr(seq_offsets), seq_offsets.numel() - 1,
        _ptr(table["chunk_offsets"]), _ptr(table["chunk_start"]), _ptr(table["chunk_len"]), _ptr(rank_idx),
        table["cap"], _ptr(out), _stream()), "cwl_chunkwise_lora_linear_packed_static")
    return out


def schedule_chunks(entropy, seq_offsets, l_min, l_max, theta_hard, delta_dev, thresholds, K, cap=None, out=None,
                    rank_idx=None, shrink=None):
    """partition_chunks and select_ranks as one call; returns (table, rank_idx).  `shrink`, when given, is
    (x, packed, ranks, scales, blend_w, u): the call then also does lora_shrink(x, packed, ..., out=u), in the
    chunker's own launch where the shapes allow it (u from an earlier lora_shrink of the same shapes, or a uint8
    tensor of cwl_lora_shrink_bytes bytes)."""
    assert entropy.is_cuda and entropy.dtype == torch.float32 and entropy.is_contiguous()
    assert seq_offsets.is_cuda and seq_offsets.dtype == torch.int32
    dev = entropy.device
    n_rows, n_seqs = entropy.numel(), seq_offsets.numel() - 1
    p = ChunkParams(int(l_min), int(l_max), float(theta_hard), float(delta_dev))
    if out is not None:
        cap = out["cap"]
    elif cap is None:
        cap = n_rows // max(int(l_min), 1) + n_seqs + 1
    nbytes = lib().cwl_partition_workspace_bytes(n_rows, n_seqs, ctypes.byref(p))
    out = out if out is not None else {
        "chunk_offsets": torch.empty(n_seqs + 1, dtype=torch.int32, device=dev),
        "chunk_start": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_len": torch.empty(max(cap, 1), dtype=torch.int32, device=dev),
        "chunk_sum": torch.empty(max(cap, 1), dtype=torch.int64, device=dev),
        "status_word": torch.empty(1, dtype=torch.int32, device=dev),
        "cap": int(cap),
        "_workspace": _ws(nbytes, dev),
    }
    if rank_idx is None:
        rank_idx = torch.zeros(max(cap, 1), dtype=torch.int32, device=dev)
    th = (ctypes.c_float * max(K - 1, 1))(*[float(t) for t in thresholds])
    ws = out["_workspace"]
    if shrink is not None:
        x, packed, ranks, scales, blend_w, u = shrink
        assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(packed, PackedWeights)
        dummy_y = torch.empty((0, packed.d_out), dtype=x.dtype, device=dev)
        d = _desc_for(x, packed.d_out, packed.r_max, ranks, scales, blend_w, dummy_y)
        d.c.ldy = packed.d_out
        tail = (d.ref(), _ptr(x), _ptr(packed.blob), _ptr(u), u.numel())
    else:
        tail = (None, None, None, None, 0)
    _check(lib().cwl_schedule_chunks(_ptr(entropy), n_rows, _ptr(seq_offsets), n_seqs, ctypes.byref(p), th, int(K),
                                     _ptr(out["chunk_offsets"]), _ptr(out["chunk_start"]), _ptr(out["chunk_len"]),
                                     _ptr(out["chunk_sum"]), _ptr(rank_idx), int(cap), _ptr(out["status_word"]),
                                     _ptr(ws), ws.numel(), *tail, _stream()), "cwl_schedule_chunks")
    return out, rank_idx


def lora_shrink(x, packed, ranks, scales, blend_w, out=None):
    """First phase of the two-phase layer: u = x A (every stored direction, fp32, no gate) into an opaque
    uint8 buffer, which chunkwise_lora_linear_shrunk takes.  Needs no chunk table."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(packed, PackedWeights)
    assert packed.dtype == x.dtype and packed.d_in == x.shape[1]
    dummy_y = torch.empty((0, packed.d_out), dtype=x.dtype, device=x.device)
    d = _desc_for(x, packed.d_out, packed.r_max, ranks, scales, blend_w, dummy_y)
    d.c.ldy = packed.d_out
    need = lib().cwl_lora_shrink_bytes(d.ref())
    if out is None:
        out = _ws(need, x.device)
    _check(lib().cwl_lora_shrink_packed(d.ref(), _ptr(x), _ptr(packed.blob), _ptr(out), out.numel(), _stream()),
           "cwl_lora_shrink_packed")
    return out


def chunkwise_lora_linear_shrunk(x, packed, u, ranks, scales, blend_w, seq_offsets, table, rank_idx, out=None,
                                 workspace=None):
    """Second phase: the chunk table's gate on `u` (from lora_shrink on the same x), then y = x W + uhat B."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(packed, PackedWeights)
    assert packed.dtype == x.dtype and packed.d_in == x.shape[1]
    if out is None:
        out = torch.empty((x.shape[0], packed.d_out), dtype=x.dtype, device=x.device)
    d = _desc_for(x, packed.d_out, packed.r_max, ranks, scales, blend_w, out)
    need = lib().cwl_linear_packed_workspace_bytes(d.ref())
    ws = workspace if workspace is not None else _ws(max(need, 256), x.device)
    _check(lib().cwl_chunkwise_lora_linear_packed_shrunk(
        d.ref(), _ptr(x), _ptr(packed.blob), _ptr(u), u.numel(), _ptr(seq_offsets), seq_offsets.numel() - 1,
        _ptr(table["chunk_offsets"]), _ptr(table["chunk_start"]), _ptr(table["chunk_len"]), _ptr(rank_idx),
        table["cap"], _ptr(out), _ptr(ws), ws.numel(), _stream()), "cwl_chunkwise_lora_linear_packed_shrunk")
    return out


def kv_quantise_chunks(kv, n_heads, head_dim, k_keep, table, rank_idx, cap_q=None, cap_f=None, out=None):
    """Chunk-level KV-cache policy: rows of chunks whose rung is below `k_keep` into an INT8 pool (one fp32 scale
    per row and head), the other chunks' rows into a full-fidelity pool.  kv: bf16 [N, n_heads * head_dim].
    Returns a dict of device tensors: slot, counts, q_codes, q_scale, f_pool, status_word (+ the shape)."""
    assert kv.is_cuda and kv.dim() == 2 and kv.stride(1) == 1 and kv.dtype == torch.bfloat16
    n, width = kv.shape
    assert width == n_heads * head_dim
    dev = kv.device
    cap_q = n if cap_q is None else int(cap_q)
    cap_f = n if cap_f is None else int(cap_f)
    p = KvParams(int(n_heads), int(head_dim), int(k_keep))
    if out is None:
        out = {"slot": torch.empty(max(n, 1), dtype=torch.int32, device=dev),
               "counts": torch.empty(2, dtype=torch.int32, device=dev),
               "q_codes": torch.empty((max(cap_q, 1), width), dtype=torch.int8, device=dev),
               "q_scale": torch.empty((max(cap_q, 1), n_heads), dtype=torch.float32, device=dev),
               "f_pool": torch.empty((max(cap_f, 1), width), dtype=torch.bfloat16, device=dev),
               "status_word": torch.empty(1, dtype=torch.int32, device=dev),
               "_workspace": _ws(lib().cwl_kv_workspace_bytes(table["cap"]), dev),
               "cap_q": cap_q, "cap_f": cap_f, "n_heads": int(n_heads), "head_dim": int(head_dim)}
    ws = out["_workspace"]
    n_seqs = table["chunk_offsets"].numel() - 1
    _check(lib().cwl_kv_quantise_chunks(
        _ptr(kv), kv.stride(0) if n > 1 else width, n, _ptr(table["chunk_offsets"]), n_seqs, _ptr(table["chunk_start"]),
        _ptr(table["chunk_len"]), _ptr(rank_idx), table["cap"], ctypes.byref(p), _ptr(out["slot"]), _ptr(out["counts"]),
        _ptr(out["q_codes"]), _ptr(out["q_scale"]), out["cap_q"], _ptr(out["f_pool"]), out["cap_f"],
        _ptr(out["status_word"]), _ptr(ws), ws.numel(), _stream()), "cwl_kv_quantise_chunks")
    return out


def kv_dequantise(cache, n_rows, out=None):
    """The cache written by kv_quantise_chunks read back as bf16 [n_rows, n_heads * head_dim]."""
    width = cache["n_heads"] * cache["head_dim"]
    dev = cache["slot"].device
    if out is None:
        out = torch.empty((n_rows, width), dtype=torch.bfloat16, device=dev)
    p = KvParams(cache["n_heads"], cache["head_dim"], 0)
    _check(lib().cwl_kv_dequantise(_ptr(cache["slot"]), int(n_rows), _ptr(cache["q_codes"]), _ptr(cache["q_scale"]),
                                   _ptr(cache["f_pool"]), ctypes.byref(p), _ptr(out),
                                   out.stride(0) if n_rows > 1 else width, _stream()), "cwl_kv_dequantise")
    return out


class PackedGroup:
    """Static weights of projections that share x, re-laid out side by side by cwl_prepack_weights_grouped."""

    def __init__(self, blob, d_in, d_outs, r_max, dtype):
        self.blob, self.d_in, self.d_outs, self.r_max, self.dtype = blob, d_in, list(d_outs), r_max, dtype
        self.d_out = sum(self.d_outs)

    def group(self, Ws=None, As=None, Bs=None):
        g = Group()
        g.n_proj = len(self.d_outs)
        for p, n in enumerate(self.d_outs):
            g.d_out[p] = n
            if Ws is not None:
                g.W[p], g.A[p], g.B[p] = Ws[p].data_ptr(), As[p].data_ptr(), Bs[p].data_ptr()
        return g

    def split(self, y):
        """Views of the wide output, one per projection."""
        outs, c = [], 0
        for n in self.d_outs:
            outs.append(y[:, c:c + n])
            c += n
        return outs


def _group_desc(x, pg, ranks, scales, blend_w, y):
    return _desc_for(x, pg.d_out, pg.r_max, ranks, scales, blend_w, y)


def prepack_weights_grouped(Ws, As, Bs):
    """Lists of W_p [d_in, d_out_p], A_p [d_in, r_max], B_p [r_max, d_out_p] (contiguous, same d_in, r_max and
    dtype) -> PackedGroup."""
    assert 1 <= len(Ws) <= MAX_GROUP and len(As) == len(Ws) and len(Bs) == len(Ws)
    d_in, r_max, dtype, dev = Ws[0].shape[0], As[0].shape[1], Ws[0].dtype, Ws[0].device
    for W, A, B in zip(Ws, As, Bs):
        assert W.is_cuda and W.is_contiguous() and A.is_contiguous() and B.is_contiguous()
        assert W.shape[0] == d_in and A.shape == (d_in, r_max) and B.shape == (r_max, W.shape[1])
        assert W.dtype == dtype and A.dtype == dtype and B.dtype == dtype
    pg = PackedGroup(None, d_in, [W.shape[1] for W in Ws], r_max, dtype)
    dummy_x = torch.empty((1, d_in), dtype=dtype, device=dev)
    dummy_y = torch.empty((1, pg.d_out), dtype=dtype, device=dev)
    d = _group_desc(dummy_x, pg, [r_max], [1.0], 0, dummy_y)
    d.c.n_rows = 0
    g = pg.group(Ws, As, Bs)
    nbytes = lib().cwl_packed_weights_grouped_bytes(d.ref(), ctypes.byref(g))
    if nbytes == 0:
        raise CwlError(ERR_INVALID_ARG, "cwl_packed_weights_grouped_bytes")
    pg.blob = _ws(nbytes, dev)
    _check(lib().cwl_prepack_weights_grouped(d.ref(), ctypes.byref(g), _ptr(pg.blob), pg.blob.numel(), _stream()),
           "cwl_prepack_weights_grouped")
    return pg


def grouped_workspace(n_rows, pg, ranks, scales, blend_w, device):
    x = torch.empty((1, pg.d_in), dtype=pg.dtype, device=device)
    y = torch.empty((1, pg.d_out), dtype=pg.dtype, device=device)
    d = _group_desc(x, pg, ranks, scales, blend_w, y)
    d.c.n_rows = n_rows
    d.c.ldx, d.c.ldy = pg.d_in, pg.d_out
    g = pg.group()
    return _ws(lib().cwl_linear_grouped_workspace_bytes(d.ref(), ctypes.byref(g)), device)


def chunkwise_lora_linear_grouped(x, pg, ranks, scales, blend_w, seq_offsets, table, rank_idx, out=None,
                                  workspace=None):
    """The layer for every projection of a PackedGroup at once; returns the wide output
    [n_rows, sum d_out_p] (PackedGroup.split gives the per-projection views)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(pg, PackedGroup)
    assert pg.dtype == x.dtype and pg.d_in == x.shape[1]
    if out is None:
        out = torch.empty((x.shape[0], pg.d_out), dtype=x.dtype, device=x.device)
    d = _group_desc(x, pg, ranks, scales, blend_w, out)
    g = pg.group()
    need = lib().cwl_linear_grouped_workspace_bytes(d.ref(), ctypes.byref(g)) or 256
    ws = workspace if workspace is not None else _ws(need, x.device)
    _check(lib().cwl_chunkwise_lora_linear_grouped_packed(
        d.ref(), ctypes.byref(g), _ptr(x), _ptr(pg.blob), _ptr(seq_offsets), seq_offsets.numel() - 1,
        _ptr(table["chunk_offsets"]), _ptr(table["chunk_start"]), _ptr(table["chunk_len"]), _ptr(rank_idx),
        table["cap"], _ptr(out), _ptr(ws), ws.numel(), _stream()), "cwl_chunkwise_lora_linear_grouped_packed")
    return out


def gated_lora_linear_grouped(x, pg, gate, ranks, scales, out=None, workspace=None):
    """gated_lora_linear for every projection of a PackedGroup at once (decode steps)."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(pg, PackedGroup)
    assert gate.is_cuda and gate.dtype == torch.int32 and gate.is_contiguous() and gate.shape == (x.shape[0], 4)
    if out is None:
        out = torch.empty((x.shape[0], pg.d_out), dtype=x.dtype, device=x.device)
    d = _group_desc(x, pg, ranks, scales, 0, out)
    g = pg.group()
    need = lib().cwl_linear_grouped_workspace_bytes(d.ref(), ctypes.byref(g)) or 256
    ws = workspace if workspace is not None else _ws(need, x.device)
    _check(lib().cwl_gated_lora_linear_grouped_packed(d.ref(), ctypes.byref(g), _ptr(x), _ptr(pg.blob), _ptr(gate),
                                                      _ptr(out), _ptr(ws), ws.numel(), _stream()),
           "cwl_gated_lora_linear_grouped_packed")
    return out


def stream_state(n_seqs, device):
    """Zeroed cached scheduler state for `n_seqs` sequences: int64 [n_seqs, 4], one cwl_stream_state
    per row (sum, pos, n | n_chunks << 32, k_cur | k_prev << 32)."""
    return torch.zeros((n_seqs, 4), dtype=torch.int64, device=device)


def stream_state_fields(state):
    """Host view of a state tensor as a dict of numpy arrays (sum, pos, n, n_chunks, k_cur, k_prev)."""
    h = state.cpu().numpy()
    lo = lambda v: (v & 0xffffffff).astype("int64").astype("int32")
    hi = lambda v: (v >> 32).astype("int32")
    return {"sum": h[:, 0].copy(), "pos": h[:, 1].copy(), "n": lo(h[:, 2]), "n_chunks": hi(h[:, 2]),
            "k_cur": lo(h[:, 3]), "k_prev": hi(h[:, 3])}


def stream_step(entropy, state, l_min, l_max, theta_hard, delta_dev, thresholds, ranks, scales, blend_w,
                out=None):
    """One decode step of the chunker / selector / cross-fade: entropy [B] fp32 (one new token per
    sequence), state from stream_state (updated in place).  Returns a dict of device tensors: gate
    (int32 [B, 4]: r_cur, r_prev and the bit patterns of the fp32 g_cur, g_prev), closed_len,
    closed_sum, status_word (OR-ed into; zeroed when this call allocates it)."""
    assert entropy.is_cuda and entropy.dtype == torch.float32 and entropy.is_contiguous()
    assert state.is_cuda and state.dtype == torch.int64 and state.is_contiguous()
    B, dev, K = entropy.numel(), entropy.device, len(ranks)
    assert state.shape == (B, 4)
    if out is None:
        out = {"gate": torch.empty((B, 4), dtype=torch.int32, device=dev),
               "closed_len": torch.empty(B, dtype=torch.int32, device=dev),
               "closed_sum": torch.empty(B, dtype=torch.int64, device=dev),
               "status_word": torch.zeros(1, dtype=torch.int32, device=dev)}
    p = ChunkParams(int(l_min), int(l_max), float(theta_hard), float(delta_dev))
    th = (ctypes.c_float * max(K - 1, 1))(*[float(t) for t in thresholds])
    rk = (ctypes.c_int32 * max(K, 1))(*[int(r) for r in ranks])
    sc = (ctypes.c_float * max(K, 1))(*[float(v) for v in scales])
    _check(lib().cwl_stream_step(_ptr(entropy), B, ctypes.byref(p), th, K, rk, sc, int(blend_w),
                                 _ptr(state), _ptr(out["gate"]), _ptr(out["closed_len"]),
                                 _ptr(out["closed_sum"]), _ptr(out["status_word"]), _stream()),
           "cwl_stream_step")
    return out


def bucket_state(n_buckets, device):
    """Zeroed open chunks of the buckets' mean series: int64 [n_buckets, 2], one cwl_bucket_state per row
    (sum, n in the low half of the second word)."""
    return torch.zeros((n_buckets, 2), dtype=torch.int64, device=device)


def stream_step_aligned(entropy, state, l_min, l_max, theta_hard, delta_dev, thresholds, ranks, scales, blend_w,
                        bucket=None, bucket_st=None, k_high=1, budget=0, n_high=None, out=None):
    """stream_step for a batch under the batch controller: `bucket` (int32 [B]) + `bucket_st` (from
    bucket_state) share the close decision inside each bucket; `n_high` (int32 [B], zero at the start,
    updated in place) applies a budget of `budget` chunks per sequence on rungs >= k_high."""
    assert entropy.is_cuda and entropy.dtype == torch.float32 and entropy.is_contiguous()
    assert state.is_cuda and state.dtype == torch.int64 and state.is_contiguous()
    B, dev, K = entropy.numel(), entropy.device, len(ranks)
    assert state.shape == (B, 4)
    n_buckets = 0
    if bucket is not None:
        assert bucket.is_cuda and bucket.dtype == torch.int32 and bucket.numel() == B
        assert bucket_st is not None and bucket_st.dtype == torch.int64 and bucket_st.is_contiguous()
        n_buckets = bucket_st.shape[0]
    if n_high is not None:
        assert n_high.is_cuda and n_high.dtype == torch.int32 and n_high.numel() == B
    if out is None:
        out = {"gate": torch.empty((B, 4), dtype=torch.int32, device=dev),
               "closed_len": torch.empty(B, dtype=torch.int32, device=dev),
               "closed_sum": torch.empty(B, dtype=torch.int64, device=dev),
               "status_word": torch.zeros(1, dtype=torch.int32, device=dev)}
    p = ChunkParams(int(l_min), int(l_max), float(theta_hard), float(delta_dev))
    th = (ctypes.c_float * max(K - 1, 1))(*[float(t) for t in thresholds])
    rk = (ctypes.c_int32 * max(K, 1))(*[int(r) for r in ranks])
    sc = (ctypes.c_float * max(K, 1))(*[float(v) for v in scales])
    _check(lib().cwl_stream_step_aligned(_ptr(entropy), B, ctypes.byref(p), th, K, rk, sc, int(blend_w),
                                         _ptr(bucket), n_buckets, _ptr(bucket_st), int(k_high), int(budget),
                                         _ptr(n_high), _ptr(state), _ptr(out["gate"]), _ptr(out["closed_len"]),
                                         _ptr(out["closed_sum"]), _ptr(out["status_word"]), _stream()),
           "cwl_stream_step_aligned")
    return out


def build_ladder(A, B):
    """Rank ladder of the adapter update A B by one SVD: returns (A', B', sigma) on the device, A' / B' in the
    dtype of A / B (fp32 or bf16), sigma float64 [r] descending."""
    assert A.is_cuda and B.is_cuda and A.dim() == 2 and B.dim() == 2 and A.dtype == B.dtype
    assert A.stride(1) == 1 and B.stride(1) == 1
    d_in, r = A.shape
    d_out = B.shape[1]
    assert B.shape[0] == r
    A2, B2 = torch.empty_like(A, memory_format=torch.contiguous_format), torch.empty_like(
        B, memory_format=torch.contiguous_format)
    sigma = torch.empty(r, dtype=torch.float64, device=A.device)
    nbytes = lib().cwl_ladder_workspace_bytes(int(r))
    if nbytes == 0:
        raise CwlError(ERR_INVALID_ARG, "cwl_ladder_workspace_bytes")
    ws = _ws(nbytes, A.device)
    lda = A.stride(0) if d_in > 1 else r
    ldb = B.stride(0) if r > 1 else d_out
    _check(lib().cwl_build_ladder(_dt(A), _ptr(A), lda, _ptr(B), ldb, d_in, d_out, r, _ptr(A2), r, _ptr(B2), d_out,
                                  _ptr(sigma), _ptr(ws), ws.numel(), _stream()), "cwl_build_ladder")
    return A2, B2, sigma


def gated_lora_linear(x, packed, gate, ranks, scales, out=None, workspace=None):
    """y = x W + per-row gated adapter terms; `gate` is int32 [n_rows, 4] as written by stream_step,
    `packed` a PackedWeights.  ranks / scales only fill the descriptor."""
    assert x.is_cuda and x.dim() == 2 and x.stride(1) == 1 and isinstance(packed, PackedWeights)
    assert gate.is_cuda and gate.dtype == torch.int32 and gate.is_contiguous() and gate.shape == (x.shape[0], 4)
    n_rows = x.shape[0]
    if out is None:
        out = torch.empty((n_rows, packed.d_out), dtype=x.dtype, device=x.device)
    d = _desc_for(x, packed.d_out, packed.r_max, ranks, scales, 0, out)
    need = lib().cwl_linear_packed_workspace_bytes(d.ref()) or 256
    ws = workspace if workspace is not None else _ws(need, x.device)
    _check(lib().cwl_gated_lora_linear_packed(d.ref(), _ptr(x), _ptr(packed.blob), _ptr(gate), _ptr(out),
                                              _ptr(ws), ws.numel(), _stream()),
           "cwl_gated_lora_linear_packed")
    return out


def linear_workspace(x_shape, dtype, d_out, r_max, ranks, scales, blend_w, device, packed=True):
    """Pre-allocate a workspace for repeated chunkwise_lora_linear calls of one shape."""
    x = torch.empty((1, x_shape[1]), dtype=dtype, device=device)
    y = torch.empty((1, d_out), dtype=dtype, device=device)
    d = _desc_for(x, d_out, r_max, ranks, scales, blend_w, y)
    d.c.n_rows = x_shape[0]
    d.c.ldx, d.c.ldy = x_shape[1], d_out
    L = lib()
    n = L.cwl_linear_packed_workspace_bytes(d.ref()) if packed else L.cwl_linear_workspace_bytes(d.ref())
    return _ws(n, device)


def table_from_host(seq_offsets, chunk_offsets, chunk_start, chunk_len, rank_idx, device):
    """Upload a host chunk table (numpy int arrays) in the form the calls above take."""
    import numpy as np

    def up(a, dt):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=dt)).to(device)

    n = max(len(chunk_start), 1)
    pad = lambda a, dt: up(np.concatenate([np.asarray(a, dtype=dt), np.zeros(n - len(a), dt)]), dt)
    table = {"chunk_offsets": up(chunk_offsets, np.int32), "chunk_start": pad(chunk_start, np.int32),
             "chunk_len": pad(chunk_len, np.int32), "cap": len(chunk_start)}
    return up(seq_offsets, np.int32), table, pad(rank_idx, np.int32)


def profile_enable(slots=True):
    """Turn per-kernel HIP-event timing on (and reset it) or off.  ``slots``: True (all), False
    (off) or an iterable of PROF_* slots to record."""
    if slots is True:
        mask = (1 << PROF_SLOTS) - 1
    elif not slots:
        mask = 0
    else:
        mask = 0
        for sl in slots:
            mask |= 1 << int(sl)
    _check(lib().cwl_profile_enable(mask), "cwl_profile_enable")


def profile_read(slot):
    """(total milliseconds, launches) of the recorded launches of one tracked kernel slot."""
    ms, n = ctypes.c_double(0.0), ctypes.c_int64(0)
    _check(lib().cwl_profile_read(int(slot), ctypes.byref(ms), ctypes.byref(n)), "cwl_profile_read")
    return ms.value, n.value
